// C-ABI layer: context, arena layout, weight loading, and the sequencing of kernel
// launches for prefill / draft / verify / accept (declared in include/swift.h).
#include "../../include/swift.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "swift_kernels.h"

using namespace swift;

// ------------------------------------------------------------------------------------------
// errors
// ------------------------------------------------------------------------------------------
static thread_local std::string g_err;

static int fail(int code, const std::string &msg) {
    g_err = msg;
    return code;
}

#define HIP_TRY(expr)                                                                                   \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess)                                                                           \
            return fail(SWIFT_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(e_));             \
    } while (0)

extern "C" const char *swift_last_error(void) { return g_err.c_str(); }

// ------------------------------------------------------------------------------------------
// host-only helpers
// ------------------------------------------------------------------------------------------
static inline uint64_t align_up(uint64_t v, uint64_t a = 256) { return (v + a - 1) / a * a; }
static inline int elem_bytes(int dtype) { return dtype == SWIFT_F32 ? 4 : 2; }

extern "C" int swift_check_config(const swift_model_config *c) {
    if (!c) return fail(SWIFT_EINVAL, "null config");
    if (c->n_layers <= 0 || c->hidden <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 ||
        c->ffn <= 0 || c->vocab <= 0 || c->max_seq <= 0)
        return fail(SWIFT_EINVAL, "sizes must be positive");
    if (c->dtype != SWIFT_F32 && c->dtype != SWIFT_BF16) return fail(SWIFT_EINVAL, "unknown dtype");
    const int d = c->head_dim;
    if (!(d == 16 || d == 32 || d == 64 || d == 128)) return fail(SWIFT_EINVAL, "head_dim must be 16, 32, 64 or 128");
    if (c->n_q_heads % c->n_kv_heads) return fail(SWIFT_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
    const int group = c->n_q_heads / c->n_kv_heads;
    if (!(group == 1 || group == 2 || group == 4 || group == 8))
        return fail(SWIFT_EINVAL, "query heads per key/value head must be 1, 2, 4 or 8");
    if (c->hidden % 8 || c->ffn % 8 || c->vocab % 2) return fail(SWIFT_EINVAL, "hidden, ffn must be multiples of 8; vocab even");
    if ((int64_t)c->ffn * 4 > 160 * 1024 - 1024 || (int64_t)c->hidden * 4 > 160 * 1024 - 1024 ||
        (int64_t)c->n_q_heads * d * 4 > 160 * 1024 - 1024)
        return fail(SWIFT_EINVAL, "an activation row must fit in LDS (<= 40704 fp32)");
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return fail(SWIFT_EINVAL, "rms_eps >= 0, rope_theta > 0");
    return SWIFT_OK;
}

namespace {

struct LayerOff {
    uint64_t attn_norm, wqkv, wo, mlp_norm, wgu, wd;
};

struct Layout {
    uint64_t embed, lm_head, final_norm;
    std::vector<LayerOff> layers;
    uint64_t cos, sin, kv;
    uint64_t kv_k_bytes, kv_v_bytes;  // one layer's key plane, value plane (the value plane follows the key plane)
    int nb32;                         // > 0: values transposed in blocks of 32 slots, nb32 blocks per kv head
    bool mfma_attn;                   // decode / draft / verify attention on the matrix cores (bf16, heads of 64 or 128)
    uint64_t q_s;  // queries as two bf16 terms (matrix-core attention)
    uint64_t x, q, att, h, logits, part_o, part_ml, out_tok, out_conf, out_topk;
    uint64_t samp_q, samp_p, samp_out;  // speculative sampling: draft and target distributions [16][V], results
    // tiled path: split activations (three bf16 terms, MFMA B layout), RMSNorm partials, split-K scratch
    uint64_t xs, as_, hs, pss, mv_part, mv_counters;
    // elements from one sub-block of a prompt macro block to the next, per activation buffer
    uint64_t sub_x, sub_q, sub_q_s, sub_xs, sub_as, sub_hs, sub_pss;
    int mv_part_capacity;
    uint64_t stage, stage_bytes;  // staging for host tensors that are re-tiled on the device
    uint64_t total;
    int n_split_max;
    // bf16 matrices whose activation row fits the MFMA kernel's LDS budget are stored tiled
    bool tiled_h, tiled_q, tiled_f;  // for K = hidden, K = n_q*d, K = ffn
    bool tiled;                      // all three: the whole model runs on the tiled MFMA kernels
};

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
// bytes of a tiled [rows][K] bf16 matrix whose row groups hold `rows_per_group` matrix rows... (16 tile rows)
inline uint64_t tiled_bytes(uint64_t n_rg, uint64_t K) { return n_rg * ceil_div(K, 32) * 1024; }

Layout make_layout(const swift_model_config &c) {
    Layout L;
    const uint64_t eb = elem_bytes(c.dtype);
    const uint64_t H = c.hidden, Q = (uint64_t)c.n_q_heads * c.head_dim, KV = (uint64_t)c.n_kv_heads * c.head_dim,
                   F = c.ffn, V = c.vocab;
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) {
        uint64_t o = off;
        off = align_up(off + bytes);
        return o;
    };
    const bool bf = c.dtype == SWIFT_BF16;
    // bf16 models run on the tiled MFMA kernels (a depth too large for the LDS-resident kernel goes
    // through the K-chunked block kernel, whatever the row count)
    L.tiled = bf;
    L.tiled_h = L.tiled_q = L.tiled_f = L.tiled;
    L.embed = take(V * H * eb);
    L.lm_head = take(L.tiled_h ? tiled_bytes(ceil_div(V, 16), H) : V * H * eb);
    L.final_norm = take(H * 4);
    L.layers.resize(c.n_layers);
    for (auto &y : L.layers) {
        y.attn_norm = take(H * 4);
        y.wqkv = take(L.tiled_h ? tiled_bytes((Q + 2 * KV) / 16, H) : (Q + 2 * KV) * H * eb);
        y.wo = take(L.tiled_q ? tiled_bytes(ceil_div(H, 16), Q) : H * Q * eb);
        y.mlp_norm = take(H * 4);
        y.wgu = take(L.tiled_h ? tiled_bytes(ceil_div(F, 8), H) : 2 * F * H * eb);
        y.wd = take(L.tiled_f ? tiled_bytes(ceil_div(H, 16), F) : H * F * eb);
    }
    L.cos = take((uint64_t)c.max_seq * (c.head_dim / 2) * 4);
    L.sin = take((uint64_t)c.max_seq * (c.head_dim / 2) * 4);
    L.mfma_attn = attn_mfma_applies(c.dtype, c.head_dim);
    L.nb32 = L.mfma_attn ? (c.max_seq + 31) / 32 : 0;
    L.kv_k_bytes = align_up(KV * c.max_seq * eb);
    L.kv_v_bytes = align_up(L.mfma_attn ? KV * (uint64_t)L.nb32 * 32 * eb : KV * c.max_seq * eb);
    L.kv = take((uint64_t)c.n_layers * (L.kv_k_bytes + L.kv_v_bytes));
    L.n_split_max = kAttnMaxSplit;
    // (tiled path: a prompt macro block holds kMacroSub sub-blocks of kMaxBlockRows rows, each with activation
    // buffers of its own; every other pass uses the first sub-block's)
    const uint64_t subs = L.tiled ? kMacroSub : 1;
    L.sub_x = kMaxBlockRows * H;
    L.sub_q = kMaxBlockRows * Q;
    L.sub_q_s = kMaxBlockRows * Q * 2;
    L.sub_xs = ceil_div(H, 32) * 4 * 3 * kMaxBlockRows * 8;
    L.sub_as = ceil_div(Q, 32) * 4 * 3 * kMaxBlockRows * 8;
    L.sub_hs = ceil_div(F, 32) * 4 * 3 * kMaxBlockRows * 8;
    L.sub_pss = ceil_div(H, 16) * kMaxBlockRows;
    L.x = take(subs * L.sub_x * 4);
    L.q = take(subs * L.sub_q * 4);
    L.att = take(kMaxBlockRows * Q * 4);
    L.q_s = take(subs * L.sub_q_s * 2);
    L.h = take(kMaxBlockRows * F * 4);
    L.logits = take(kMaxBlockRows * V * 4);
    L.part_o = take((uint64_t)kMaxRows * c.n_q_heads * L.n_split_max * c.head_dim * 4);
    L.part_ml = take((uint64_t)kMaxRows * c.n_q_heads * L.n_split_max * 2 * 4);
    L.out_tok = take(kMaxBlockRows * 4);
    L.out_conf = take(kMaxBlockRows * 4);
    L.out_topk = take(kMaxBlockRows * kTopK * 4);
    L.samp_q = take((uint64_t)kMaxRows * V * 4);
    L.samp_p = take((uint64_t)kMaxRows * V * 4);
    L.samp_out = take(256);
    L.xs = take(subs * L.sub_xs * 2);
    L.as_ = take(subs * L.sub_as * 2);
    L.hs = take(subs * L.sub_hs * 2);
    L.pss = take(subs * L.sub_pss * 4);
    L.mv_part_capacity = 8192;
    L.mv_part = take((uint64_t)L.mv_part_capacity * 16 * kMaxBlockRows * 4);
    L.mv_counters = take(4096 * 4);
    L.stage_bytes = bf ? std::max(std::max(V * H, F * H), std::max(Q * H, KV * H)) * eb : 0;
    L.stage = take(L.stage_bytes);
    L.total = off;
    return L;
}

}  // namespace

extern "C" int swift_device_bytes(const swift_model_config *cfg, uint64_t *bytes) {
    if (!bytes) return fail(SWIFT_EINVAL, "null output");
    int rc = swift_check_config(cfg);
    if (rc) return rc;
    *bytes = make_layout(*cfg).total;
    return SWIFT_OK;
}

extern "C" double swift_expected_speedup(double M, double alpha, double c) { return M * alpha / ((M - 1.0) * c + alpha); }

extern "C" int swift_match_prefix(const int32_t *draft, const int32_t *target, int k) {
    if (k <= 0 || !draft || !target) return 0;
    int m = 0;
    while (m < k && draft[m] == target[m]) ++m;
    return m;
}

namespace {
struct SubBytes {
    uint64_t attn_w, mlp_w, head_w, kv_slot;  // kv_slot: one slot of one layer (K and V)
};
SubBytes sub_bytes(const swift_model_config &c) {
    const uint64_t eb = elem_bytes(c.dtype);
    const uint64_t H = c.hidden, Q = (uint64_t)c.n_q_heads * c.head_dim, KV = (uint64_t)c.n_kv_heads * c.head_dim,
                   F = c.ffn, V = c.vocab;
    SubBytes b;
    b.attn_w = (Q + 2 * KV) * H * eb + H * Q * eb + H * 4;
    b.mlp_w = 3 * F * H * eb + H * 4;
    b.head_w = V * H * eb + H * 4;
    b.kv_slot = 2 * KV * eb;
    return b;
}
}  // namespace

extern "C" int swift_pass_bytes(const swift_model_config *cfg, const uint8_t *skip, int n_ctx, int rows,
                                uint64_t *bytes) {
    if (!bytes || n_ctx < 0 || rows < 1) return fail(SWIFT_EINVAL, "bad argument");
    int rc = swift_check_config(cfg);
    if (rc) return rc;
    const SubBytes b = sub_bytes(*cfg);
    uint64_t t = b.head_w + (uint64_t)rows * cfg->hidden * elem_bytes(cfg->dtype);
    for (int l = 0; l < cfg->n_layers; ++l) {
        if (!(skip && skip[2 * l])) t += b.attn_w + b.kv_slot * ((uint64_t)n_ctx + rows);
        if (!(skip && skip[2 * l + 1])) t += b.mlp_w;
    }
    *bytes = t;
    return SWIFT_OK;
}

// ------------------------------------------------------------------------------------------
// static scratch of the allocation-free entry point (swift_verify_static)
// ------------------------------------------------------------------------------------------
// Layout of the array: [arrival counters][split-K partial sums][attention partials: part_ml | part_o].
constexpr size_t kStaticCounterBytes = 4096 * 4;
constexpr int kStaticPartSlots = 8192;  // row-group-splits of kMaxRows rows, as the arena's area holds for such blocks
constexpr size_t kStaticPartBytes = (size_t)kStaticPartSlots * 16 * kMaxRows * 4;            // 16 MiB
constexpr size_t kStaticAttnBytes = SWIFT_STATIC_SCRATCH_BYTES - kStaticCounterBytes - kStaticPartBytes;
static __device__ __align__(256) unsigned char scratch[SWIFT_STATIC_SCRATCH_BYTES];
// The array's address on each device (every GPU holds its own copy at its own address); set once per device.
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];

namespace {
// Resolves the array's device address for the current device (first call on a device only).
int static_scratch(char **out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(SWIFT_EDEVICE, "device ordinal out of range");
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(SWIFT_EDEVICE, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = (char *)g_scratch_ptr[dev];
    return SWIFT_OK;
}
}  // namespace

// ------------------------------------------------------------------------------------------
// context
// ------------------------------------------------------------------------------------------
// Device memory the kernels use beyond their inputs and outputs: split-K partial sums and arrival
// counters of the block projection kernel, partial results of attention split over the cache length.
struct Scratch {
    float *mv_part;
    int *mv_counters;
    int mv_part_capacity;  // row-group-splits mv_part holds for a block of kMaxBlockRows rows (arena) / kMaxRows rows (static)
    float *part_o, *part_ml;
    size_t part_o_floats;  // capacity of part_o (part_ml holds 2 floats per head_dim floats of part_o)
};

struct ProfRec {
    hipEvent_t a, b;
    uint64_t bytes;
};

struct swift_ctx {
    swift_model_config c;
    Layout L;
    char *base;
    hipStream_t stream;
    int n_cu;
    Scratch arena_scr;  // the scratch buffers inside the arena
    Scratch scr;        // the ones the kernels of the current call use
    bool no_events;     // the current call must not create HIP events (allocation-free entry point)
    std::vector<bool> loaded;  // per tensor slot
    int n_loaded;
    // pinned host staging for results
    int32_t *h_tok;
    float *h_conf;
    // decoding state
    int n;            // cache length
    int32_t pending;  // -1 before prefill
    int k_verify;     // -1: no verify outstanding
    int32_t vtokens[SWIFT_MAX_BLOCK], targets[SWIFT_MAX_BLOCK];
    int tree_levels;  // -1: no tree verification outstanding
    int tree_width[SWIFT_MAX_BLOCK];
    int k_sampled;    // draft tokens of the last swift_draft_step_sample whose distributions are kept (-1: none)
    int32_t sampled[SWIFT_MAX_BLOCK];
    bool want_topk;   // the next pass with logits also keeps the top candidates of its rows
    int32_t *h_topk;  // pinned, [kTopK]
    swift_stats st;
    // launch-shape overrides per kernel class (0 = automatic); measurement hook
    int tune_ks[SWIFT_KC_COUNT], tune_wg[SWIFT_KC_COUNT];
    int prefill_sub, gemm_rgw;  // swift_debug_prefill
    // profiling
    int prof_class;
    std::vector<ProfRec> prof;
    std::vector<hipEvent_t> pool;
};

namespace {

template <typename T>
T *dptr(swift_ctx *x, uint64_t off) {
    return reinterpret_cast<T *>(x->base + off);
}

int n_tensors(const swift_model_config &c) { return 3 + 9 * c.n_layers; }

// kernel_events: the launch goes through launch_mv, which can attach the events to the dispatch
// itself; otherwise the launch is bracketed by two event records on the stream.
template <typename F>
hipError_t timed(swift_ctx *x, int kc, uint64_t bytes, F &&f, bool kernel_events = false) {
    if (x->prof_class != kc || x->no_events) return f();
    hipEvent_t ev[2];
    for (auto &e : ev) {
        if (!x->pool.empty()) {
            e = x->pool.back();
            x->pool.pop_back();
        } else {
            hipError_t r = hipEventCreate(&e);
            if (r != hipSuccess) return r;
        }
    }
    hipError_t r;
    if (kernel_events) {
        set_launch_events(ev[0], ev[1]);
        r = f();
        set_launch_events(nullptr, nullptr);
    } else {
        r = hipEventRecord(ev[0], x->stream);
        if (r != hipSuccess) return r;
        r = f();
        if (r != hipSuccess) return r;
        r = hipEventRecord(ev[1], x->stream);
    }
    x->prof.push_back({ev[0], ev[1], bytes});
    return r;
}

char *kv_base(swift_ctx *x, int layer, int which) {
    return x->base + x->L.kv + (uint64_t)layer * (x->L.kv_k_bytes + x->L.kv_v_bytes) + (which ? x->L.kv_k_bytes : 0);
}

// The rows of a token tree: level of each block row, block row of the first candidate of each level (the only
// one with children).
typedef TreeTab TreeRows;

// ---- storage-generic path: one token through the network at position `pos`; row = which row of
// the activation / logits buffers to use.  skip == nullptr: full model.  want_logits: run the LM
// head and the arg-max for this row.  tree: the row is block row `row` of a token tree whose first row
// sits in slot tree_base; `pos` is then the row's cache slot and it is rotated for its level's position.
int forward_row(swift_ctx *x, int32_t token, int pos, const uint8_t *skip, int row, bool want_logits,
                bool reuse_kv = false, const TreeRows *tree = nullptr, int tree_base = 0) {
    const swift_model_config &c = x->c;
    const Layout &L = x->L;
    const int H = c.hidden, d = c.head_dim, Q = c.n_q_heads * d, KV = c.n_kv_heads * d, F = c.ffn, V = c.vocab;
    const uint64_t eb = elem_bytes(c.dtype);
    hipStream_t s = x->stream;
    float *xr = dptr<float>(x, L.x) + (size_t)row * H;
    float *qr = dptr<float>(x, L.q) + (size_t)row * Q;
    float *ar = dptr<float>(x, L.att) + (size_t)row * Q;
    float *hr = dptr<float>(x, L.h) + (size_t)row * F;
    float *lr = dptr<float>(x, L.logits) + (size_t)row * V;

    auto linear = [&](int kc, int epi, uint64_t w_off, int O, int K, const float *xin, const float *gain, float *out,
                      int layer) -> int {
        GemvArgs g{};
        g.W = x->base + w_off;
        g.O = O;
        g.K = K;
        g.xin = xin;
        g.gain = gain;
        g.eps = c.rms_eps;
        g.out = out;
        if (epi == EPI_QKV) {
            g.kcache = kv_base(x, layer, 0);
            g.vcache = kv_base(x, layer, 1);
            const int rope_pos = tree ? tree_base + tree->depth[row] : pos;
            g.cos_row = dptr<float>(x, L.cos) + (size_t)rope_pos * (d / 2);
            g.sin_row = dptr<float>(x, L.sin) + (size_t)rope_pos * (d / 2);
        }
        g.pos = pos;
        g.max_seq = c.max_seq;
        g.head_dim = d;
        g.n_q_heads = c.n_q_heads;
        g.n_kv_heads = c.n_kv_heads;
        HIP_TRY(timed(x, kc, (uint64_t)O * K * eb, [&] { return launch_gemv(c.dtype, epi, g, x->n_cu, s); }));
        return SWIFT_OK;
    };
    int rc;
    EmbedArgs ea{x->base + L.embed, H, token, xr};
    HIP_TRY(timed(x, SWIFT_KC_OTHER, H * eb, [&] { return launch_embed(c.dtype, ea, s); }));
    for (int l = 0; l < c.n_layers; ++l) {
        const LayerOff &y = L.layers[l];
        if (!(skip && skip[2 * l])) {
            // (reuse_kv: only the query rows of the fused matrix; the cache slot keeps what it holds)
            if ((rc = linear(SWIFT_KC_QKV, EPI_QKV, y.wqkv, reuse_kv ? Q : Q + 2 * KV, H, xr, dptr<float>(x, y.attn_norm), qr,
                             l)))
                return rc;
            AttnArgs a{};
            a.q = qr;
            a.kcache = kv_base(x, l, 0);
            a.vcache = kv_base(x, l, 1);
            a.n_ctx = pos + 1;
            a.rows = 1;
            a.max_seq = c.max_seq;
            a.head_dim = d;
            a.n_q_heads = c.n_q_heads;
            a.n_kv_heads = c.n_kv_heads;
            a.part_o = x->scr.part_o;
            a.part_ml = x->scr.part_ml;
            a.max_split = L.n_split_max;
            a.out = ar;
            a.out_s = nullptr;
            if (tree) {
                a.tree = 1;
                a.n_base = tree_base;
                a.row_base = row;
                a.tt = *tree;
            }
            HIP_TRY(timed(x, SWIFT_KC_ATTN, (uint64_t)2 * KV * eb * (pos + 1),
                          [&] { return launch_attn_decode(c.dtype, a, x->n_cu, s); }));
            if ((rc = linear(SWIFT_KC_OPROJ, EPI_RESID, y.wo, H, Q, ar, nullptr, xr, l))) return rc;
        }
        if (!(skip && skip[2 * l + 1])) {
            if ((rc = linear(SWIFT_KC_GATEUP, EPI_SWIGLU, y.wgu, 2 * F, H, xr, dptr<float>(x, y.mlp_norm), hr, l))) return rc;
            if ((rc = linear(SWIFT_KC_DOWN, EPI_RESID, y.wd, H, F, hr, nullptr, xr, l))) return rc;
        }
    }
    if (want_logits) {
        if ((rc = linear(SWIFT_KC_LMHEAD, EPI_LOGITS, L.lm_head, V, H, xr, dptr<float>(x, L.final_norm), lr, 0))) return rc;
        ArgmaxArgs m{lr, V, 1, dptr<int32_t>(x, L.out_tok) + row, dptr<float>(x, L.out_conf) + row,
                     x->want_topk ? dptr<int32_t>(x, L.out_topk) + (size_t)row * kTopK : nullptr, kTopK};
        HIP_TRY(timed(x, SWIFT_KC_OTHER, (uint64_t)V * 4, [&] { return launch_argmax_conf(m, s); }));
    }
    return SWIFT_OK;
}

// Attention of a block of a.rows chain or tree rows whose first row attends a.n_ctx slots; RLC: layout code of the
// block a.out_s belongs to.  The kernel is chosen from the configuration and the block's kind alone.
int block_attention(swift_ctx *x, const AttnArgs &at, int RLC) {
    const swift_model_config &c = x->c;
    const Layout &L = x->L;
    hipStream_t s = x->stream;
    const int R = at.rows, Q = c.n_q_heads * c.head_dim, KV = c.n_kv_heads * c.head_dim, ctx0 = at.n_ctx - 1;
    if (attn_block_applies(c.dtype, at)) {
        AttnArgs a = at;
        a.out_rows = RLC;
        HIP_TRY(timed(x, SWIFT_KC_ATTN, (uint64_t)2 * KV * 2 * (ctx0 + R), [&] { return launch_attn_block(a, x->n_cu, s); }));
    } else if (L.mfma_attn) {
        AttnArgs a = at;
        a.out_rows = RLC;
        HIP_TRY(timed(x, SWIFT_KC_ATTN, (uint64_t)2 * KV * 2 * (ctx0 + R), [&] { return launch_attn_mfma(a, x->n_cu, s); }));
    } else {
        // a launch of the split kernel covers up to kMaxRows rows of the block (its partial buffers)
        const int per_launch = attn_uses_head_kernel(c.max_seq, c.n_kv_heads) ? R : kMaxRows;
        for (int row0 = 0; row0 < R; row0 += per_launch) {
            AttnArgs a = at;
            a.q += (size_t)row0 * Q;
            a.n_ctx += row0;
            a.row_base = row0;  // (a tree has at most kMaxRows rows: one part)
            a.rows = std::min(per_launch, R - row0);
            a.out_s += 8 * block_terms(RLC) * row0;  // first of this part's term columns
            a.out_rows = RLC;
            HIP_TRY(timed(x, SWIFT_KC_ATTN, (uint64_t)2 * KV * 2 * (ctx0 + row0 + a.rows),
                          [&] { return launch_attn_decode(c.dtype, a, x->n_cu, s); }));
        }
    }
    return SWIFT_OK;
}

// ---- tiled bf16 path: a block of R rows (tokens[0..R) at positions pos0..pos0+R-1) through the
// network in one sweep over the weights.  Row r attends cache slots [0, pos0 + r].
// tree: the rows are those of a token tree (R <= 16): row r goes to slot pos0 + r, is rotated for position
// pos0 + its level, and attends the committed slots and the rows on its path from the root.
// exact: the block's rows must come out as they would from any other block size (draft, verify and tree
// passes: the exact layouts, up to kMaxRows rows); otherwise blocks of more than 16 rows take the bulk layouts.
//
// n_sub > 0: a prompt macro block instead: n_sub sub-blocks of kMaxBlockRows rows, the last one with R rows, at
// positions pos0 .. (tokens holds all their rows).  Every projection is one launch of the blocked matrix product
// over all sub-blocks; attention, the embedding and the LM head (last sub-block only: results land in rows
// [0, R)) go sub-block by sub-block.  Bulk layouts; no tree.  With reuse_kv (a candidate-evaluation window of more
// than one sub-block) the caller asks for every sub-block's predictions afterwards (macro_sub_logits).
int forward_block_tiled(swift_ctx *x, const int32_t *tokens, int R, int pos0, const uint8_t *skip, bool want_logits,
                        bool reuse_kv, const TreeRows *tree, bool exact, int n_sub = 0) {
    if (n_sub > 0 && (tree || exact || n_sub > kMacroSub)) return fail(SWIFT_EINVAL, "bad macro block");
    // layout code of every split activation of this pass
    const int RLC = n_sub > 0 ? (kMaxBlockRows | kBulkLayout) : block_row_layout(R, exact);
    const swift_model_config &c = x->c;
    const Layout &L = x->L;
    const int H = c.hidden, d = c.head_dim, Q = c.n_q_heads * d, KV = c.n_kv_heads * d, F = c.ffn, V = c.vocab;
    hipStream_t s = x->stream;
    float *xf = dptr<float>(x, L.x);
    float *qf = dptr<float>(x, L.q);
    uint16_t *xs = dptr<uint16_t>(x, L.xs), *as_ = dptr<uint16_t>(x, L.as_), *hs = dptr<uint16_t>(x, L.hs);
    float *pss = dptr<float>(x, L.pss);
    const int n_pss = (H + 15) / 16;

    // non-skipped sublayers in order; the kernel that updates the residual stream pre-multiplies
    // its split output with the RMSNorm gain of whichever sublayer (or the final norm) reads it next
    struct Stage { int layer, kind; };
    std::vector<Stage> stages;
    stages.reserve(2 * c.n_layers);
    for (int l = 0; l < c.n_layers; ++l) {
        if (!(skip && skip[2 * l])) stages.push_back({l, 0});
        if (!(skip && skip[2 * l + 1])) stages.push_back({l, 1});
    }
    auto gain_of = [&](size_t i) -> const float * {
        if (i >= stages.size()) return dptr<float>(x, L.final_norm);
        const LayerOff &y = L.layers[stages[i].layer];
        return dptr<float>(x, stages[i].kind == 0 ? y.attn_norm : y.mlp_norm);
    };
    auto base_args = [&](uint64_t w_off, int O, int K, int n_rg) {
        MvArgs m{};
        m.Wt = x->base + w_off;
        m.O = O;
        m.K = K;
        m.T = (K + 31) / 32;
        m.n_rg = n_rg;
        m.R = R;
        m.RL = RLC;
        m.rp = n_sub > 0 ? kMaxBlockRows : block_row_pitch(R);
        m.eps = c.rms_eps;
        m.norm_dim = H;
        m.pos0 = pos0;
        m.max_seq = c.max_seq;
        m.head_dim = d;
        m.n_q_heads = c.n_q_heads;
        m.n_kv_heads = c.n_kv_heads;
        m.cos_tab = dptr<float>(x, L.cos);
        m.sin_tab = dptr<float>(x, L.sin);
        m.part = x->scr.mv_part;
        m.counters = x->scr.mv_counters;
        m.part_capacity = L.mv_part_capacity;  // (decides the K split, hence the summation order: one value everywhere)
        return m;
    };
    // ---- the pass as a list of launches
    struct Launch {
        int kc;       // kernel class (profiling, launch-shape overrides)
        int epi;      // projections: Epilogue; attention: -1
        MvArgs mv;
        AttnArgs at;
    };
    std::vector<Launch> list;
    list.reserve(5 * stages.size() + 1);
    auto push_mv = [&](int kc, int epi, const MvArgs &m) {
        Launch st{};
        st.kc = kc;
        st.epi = epi;
        st.mv = m;
        list.push_back(st);
    };
    for (size_t i = 0; i < stages.size(); ++i) {
        const int l = stages[i].layer;
        const LayerOff &y = L.layers[l];
        const float *gnext = gain_of(i + 1);
        if (stages[i].kind == 0) {
            // (reuse_kv: the query heads' row groups only; they come first in the fused matrix)
            MvArgs m = reuse_kv ? base_args(y.wqkv, Q, H, Q / 16) : base_args(y.wqkv, Q + 2 * KV, H, (Q + 2 * KV) / 16);
            m.in_s = xs;
            m.pss = pss;
            m.n_pss = n_pss;
            m.out_f32 = qf;
            m.ld_out = Q;
            m.kcache = kv_base(x, l, 0);
            m.vcache = kv_base(x, l, 1);
            m.nb32 = L.nb32;
            // (the two-term copy of the queries is the operand of the matrix-core attention of blocks of up to 32 rows;
            // a macro block's attention takes the fp32 queries)
            m.q_s = L.mfma_attn && n_sub == 0 ? dptr<uint16_t>(x, L.q_s) : nullptr;
            if (tree) {
                m.tree = 1;
                memcpy(m.depth, tree->depth, sizeof(m.depth));
            }
            // the committed keys/values the attention launch will read: warmed into L2 by spare workgroups of
            // this launch (one-workgroup-per-head attention only: its workgroup-to-head mapping is what the
            // warm-up relies on)
            if (!reuse_kv && attn_uses_head_kernel(c.max_seq, c.n_kv_heads)) {
                m.pf_heads = c.n_kv_heads;
                m.pf_rows = pos0;
            }
            push_mv(SWIFT_KC_QKV, EPI_QKV, m);

            Launch at{};
            at.kc = SWIFT_KC_ATTN;
            at.epi = -1;
            AttnArgs &a = at.at;
            a.q = qf;
            a.kcache = kv_base(x, l, 0);
            a.vcache = kv_base(x, l, 1);
            a.n_ctx = pos0 + 1;
            a.rows = R;
            a.max_seq = c.max_seq;
            a.head_dim = d;
            a.n_q_heads = c.n_q_heads;
            a.n_kv_heads = c.n_kv_heads;
            a.part_o = x->scr.part_o;
            a.part_ml = x->scr.part_ml;
            a.max_split = L.n_split_max;
            a.nb32 = L.nb32;
            a.q_s = dptr<uint16_t>(x, L.q_s);
            a.out = nullptr;
            a.out_s = as_;
            if (tree) {
                a.tree = 1;
                a.n_base = pos0;
                a.row_base = 0;
                a.tt = *tree;
            }
            list.push_back(at);

            MvArgs o = base_args(y.wo, H, Q, (H + 15) / 16);
            o.in_s = as_;
            o.out_f32 = xf;
            o.ld_out = H;
            o.out_s = xs;
            o.gain_next = gnext;
            o.pss_out = pss;
            push_mv(SWIFT_KC_OPROJ, EPI_RESID, o);
        } else {
            MvArgs m = base_args(y.wgu, 2 * F, H, (F + 7) / 8);
            m.in_s = xs;
            m.pss = pss;
            m.n_pss = n_pss;
            m.out_s = hs;
            push_mv(SWIFT_KC_GATEUP, EPI_SWIGLU, m);
            MvArgs w = base_args(y.wd, H, F, (H + 15) / 16);
            w.in_s = hs;
            w.out_f32 = xf;
            w.ld_out = H;
            w.out_s = xs;
            w.gain_next = gnext;
            w.pss_out = pss;
            push_mv(SWIFT_KC_DOWN, EPI_RESID, w);
        }
    }
    // (macro block: the LM head reads the last sub-block's buffers)
    const int last = n_sub > 0 ? n_sub - 1 : 0;
    if (want_logits) {
        MvArgs m = base_args(L.lm_head, V, H, (V + 15) / 16);
        m.in_s = xs + last * L.sub_xs;
        m.pss = pss + last * L.sub_pss;
        m.n_pss = n_pss;
        m.out_f32 = dptr<float>(x, L.logits);
        m.ld_out = V;
        push_mv(SWIFT_KC_LMHEAD, EPI_LOGITS, m);
    }

    MacroArgs ma{};
    ma.S = n_sub;
    ma.rows_last = R;
    auto sub_rows = [&](int sb) { return sb == last ? R : kMaxBlockRows; };
    for (int sb = 0; sb <= last; ++sb) {
        EmbedRowsArgs ea{};
        ea.E = dptr<uint16_t>(x, L.embed);
        ea.H = H;
        ea.R = sub_rows(sb);
        for (int r = 0; r < ea.R; ++r) ea.tokens[r] = tokens[sb * kMaxBlockRows + r];
        ea.x = xf + sb * L.sub_x;
        ea.xs = xs + sb * L.sub_xs;
        ea.gain_next = gain_of(0);
        ea.pss = pss + sb * L.sub_pss;
        ea.rp = n_sub > 0 ? kMaxBlockRows : block_row_pitch(R);
        ea.RL = RLC;
        HIP_TRY(timed(x, SWIFT_KC_OTHER, (uint64_t)ea.R * H * 2, [&] { return launch_embed_rows(ea, s); }));
    }

    // ---- one launch per stage
    for (size_t i = 0; i < list.size(); ++i) {
        const int kc = list[i].kc;
        if (list[i].epi < 0 && n_sub > 0 && L.mfma_attn) {
            // (the block attention kernel takes the whole macro block in one launch)
            AttnArgs a = list[i].at;
            a.rows = last * kMaxBlockRows + R;
            a.sub_rows = kMaxBlockRows;
            a.sub_q = L.sub_q;
            a.sub_out_s = L.sub_as;
            a.out_rows = RLC;
            HIP_TRY(timed(x, SWIFT_KC_ATTN, (uint64_t)2 * KV * 2 * (pos0 + a.rows), [&] { return launch_attn_block(a, x->n_cu, s); }));
        } else if (list[i].epi < 0) {
            for (int sb = 0; sb <= last; ++sb) {
                AttnArgs a = list[i].at;
                a.rows = sub_rows(sb);
                a.n_ctx += sb * kMaxBlockRows;
                a.q += sb * L.sub_q;
                a.q_s += sb * L.sub_q_s;
                a.out_s += sb * L.sub_as;
                int rc = block_attention(x, a, RLC);
                if (rc) return rc;
            }
        } else if (n_sub > 0 && list[i].epi != EPI_LOGITS) {
            // (sub-block strides: which buffers a launch reads and writes follows from its epilogue)
            const MvArgs &m = list[i].mv;
            const int epi = list[i].epi;
            ma.in_s = kc == SWIFT_KC_OPROJ ? L.sub_as : kc == SWIFT_KC_DOWN ? L.sub_hs : L.sub_xs;
            ma.pss = L.sub_pss;
            ma.out_f32 = epi == EPI_QKV ? L.sub_q : L.sub_x;
            ma.out_s = epi == EPI_SWIGLU ? L.sub_hs : L.sub_xs;
            ma.pss_out = L.sub_pss;
            ma.q_s = L.sub_q_s;
            HIP_TRY(timed(x, kc, (uint64_t)m.O * m.K * 2, [&] { return launch_gemm(epi, m, ma, x->n_cu, x->gemm_rgw, s); }));
        } else {
            const MvArgs &m = list[i].mv;
            const int epi = list[i].epi;
            HIP_TRY(timed(x, kc, (uint64_t)m.O * m.K * 2,
                          [&] { return launch_mv(epi, m, x->n_cu, x->tune_ks[kc], x->tune_wg[kc], s); }, true));
        }
    }
    if (want_logits) {
        ArgmaxArgs am{dptr<float>(x, L.logits), V, R, dptr<int32_t>(x, L.out_tok), dptr<float>(x, L.out_conf),
                      x->want_topk ? dptr<int32_t>(x, L.out_topk) : nullptr, kTopK};
        HIP_TRY(timed(x, SWIFT_KC_OTHER, (uint64_t)R * V * 4, [&] { return launch_argmax_conf(am, s); }));
    }
    return SWIFT_OK;
}

// After a macro block pass: LM head and arg-max over the `rows` rows of sub-block sb, whose final residual stream the
// pass left in that sub-block's buffers; results land in rows [0, rows).
int macro_sub_logits(swift_ctx *x, int sb, int rows) {
    const swift_model_config &c = x->c;
    const Layout &L = x->L;
    if (!L.tiled || sb < 0 || sb >= kMacroSub || rows < 1 || rows > kMaxBlockRows) return fail(SWIFT_EINVAL, "bad sub-block");
    hipStream_t s = x->stream;
    MvArgs m{};
    m.Wt = x->base + L.lm_head;
    m.O = c.vocab;
    m.K = c.hidden;
    m.T = (c.hidden + 31) / 32;
    m.n_rg = (c.vocab + 15) / 16;
    m.R = rows;
    m.RL = kMaxBlockRows | kBulkLayout;
    m.rp = kMaxBlockRows;
    m.eps = c.rms_eps;
    m.norm_dim = c.hidden;
    m.max_seq = c.max_seq;
    m.head_dim = c.head_dim;
    m.n_q_heads = c.n_q_heads;
    m.n_kv_heads = c.n_kv_heads;
    m.part = x->scr.mv_part;
    m.counters = x->scr.mv_counters;
    m.part_capacity = L.mv_part_capacity;
    m.in_s = dptr<uint16_t>(x, L.xs) + sb * L.sub_xs;
    m.pss = dptr<float>(x, L.pss) + sb * L.sub_pss;
    m.n_pss = (c.hidden + 15) / 16;
    m.out_f32 = dptr<float>(x, L.logits);
    m.ld_out = c.vocab;
    HIP_TRY(timed(x, SWIFT_KC_LMHEAD, (uint64_t)m.O * m.K * 2,
                  [&] { return launch_mv(EPI_LOGITS, m, x->n_cu, x->tune_ks[SWIFT_KC_LMHEAD], x->tune_wg[SWIFT_KC_LMHEAD], s); }, true));
    ArgmaxArgs am{dptr<float>(x, L.logits), c.vocab, rows, dptr<int32_t>(x, L.out_tok), dptr<float>(x, L.out_conf),
                  x->want_topk ? dptr<int32_t>(x, L.out_topk) : nullptr, kTopK};
    HIP_TRY(timed(x, SWIFT_KC_OTHER, (uint64_t)rows * c.vocab * 4, [&] { return launch_argmax_conf(am, s); }));
    return SWIFT_OK;
}

// R rows through the network; results (token, confidence, logits) land in rows [0, R).
// reuse_kv: the rows' keys and values are not computed; every row attends what the cache already holds
// for slots up to its own position (candidate evaluation).
int forward_block(swift_ctx *x, const int32_t *tokens, int R, int pos0, const uint8_t *skip, bool want_logits,
                  bool reuse_kv = false, const TreeRows *tree = nullptr, bool exact = true) {
    if (tree && R > kMaxRows) return fail(SWIFT_EINVAL, "a token tree has at most SWIFT_MAX_BLOCK rows");
    if (exact && R > kMaxRows) return fail(SWIFT_EINVAL, "a verify block has at most SWIFT_MAX_BLOCK rows");
    if (x->L.tiled) return forward_block_tiled(x, tokens, R, pos0, skip, want_logits, reuse_kv, tree, exact);
    for (int r = 0; r < R; ++r) {
        int rc = forward_row(x, tokens[r], pos0 + r, skip, r, want_logits, reuse_kv, tree, pos0);
        if (rc) return rc;
    }
    return SWIFT_OK;
}

// Copies rows [0, rows) of the token / confidence results to the pinned staging area and waits.
int read_results(swift_ctx *x, int rows) {
    // (tokens and confidences lie kMaxBlockRows words apart on the device and in the staging area alike: one copy)
    if (x->L.out_conf != x->L.out_tok + kMaxBlockRows * 4 || (char *)x->h_conf != (char *)x->h_tok + kMaxBlockRows * 4)
        return fail(SWIFT_EINVAL, "result areas are not adjacent");
    HIP_TRY(hipMemcpyAsync(x->h_tok, dptr<int32_t>(x, x->L.out_tok), (kMaxBlockRows + rows) * 4, hipMemcpyDeviceToHost, x->stream));
    HIP_TRY(hipStreamSynchronize(x->stream));
    // a token id is fed back as an embedding row index: never pass on one outside the vocabulary
    for (int i = 0; i < rows; ++i)
        if (x->h_tok[i] < 0 || x->h_tok[i] >= x->c.vocab)
            return fail(SWIFT_EDEVICE, "the arg-max kernel returned a token id outside the vocabulary");
    return SWIFT_OK;
}

// tensor slot index for a name, plus where and how it is stored
struct Slot {
    int index;
    uint64_t off;       // destination offset in the arena
    int64_t n;          // expected element count
    bool is_gain;
    int rows, cols;     // matrix shape [rows][cols] as given by the caller
    uint64_t dst_pitch; // row-major destination: bytes between consecutive rows (0 = contiguous)
    bool tiled;         // destination is in the tiled MFMA layout
    int tile_mode, part;
    int n_rg;           // row groups this tensor fills
};

bool find_slot(swift_ctx *x, const char *name, Slot *out) {
    const swift_model_config &c = x->c;
    const Layout &L = x->L;
    const uint64_t eb = elem_bytes(c.dtype);
    const int H = c.hidden, d = c.head_dim, Q = c.n_q_heads * d, KV = c.n_kv_heads * d, F = c.ffn, V = c.vocab;
    auto mat = [&](int idx, uint64_t off, int r, int k, uint64_t pitch = 0) {
        *out = Slot{idx, off, (int64_t)r * k, false, r, k, pitch, false, 0, 0, 0};
        return true;
    };
    auto tiled = [&](int idx, uint64_t off, int r, int k, int mode, int part, int n_rg) {
        *out = Slot{idx, off, (int64_t)r * k, false, r, k, 0, true, mode, part, n_rg};
        return true;
    };
    auto gain = [&](int idx, uint64_t off) {
        *out = Slot{idx, off, H, true, 1, H, 0, false, 0, 0, 0};
        return true;
    };
    const uint64_t TH = (uint64_t)((H + 31) / 32) * 1024;  // bytes of one row group with K = hidden
    if (!strcmp(name, "embed")) return mat(0, L.embed, V, H);
    if (!strcmp(name, "lm_head"))
        return L.tiled_h ? tiled(1, L.lm_head, V, H, TILE_PLAIN, 0, (V + 15) / 16) : mat(1, L.lm_head, V, H);
    if (!strcmp(name, "final_norm")) return gain(2, L.final_norm);
    if (name[0] != 'l') return false;
    char *end;
    long l = strtol(name + 1, &end, 10);
    if (end == name + 1 || *end != '.' || l < 0 || l >= c.n_layers) return false;
    const char *f = end + 1;
    const LayerOff &y = L.layers[l];
    const int b = 3 + 9 * (int)l;
    if (!strcmp(f, "attn_norm")) return gain(b + 0, y.attn_norm);
    if (L.tiled_h) {
        // fused q|k|v, rotary pairs in one row group; d/16 row groups per head
        if (!strcmp(f, "wq")) return tiled(b + 1, y.wqkv, Q, H, TILE_PAIR, 0, Q / 16);
        if (!strcmp(f, "wk")) return tiled(b + 2, y.wqkv + (uint64_t)(Q / 16) * TH, KV, H, TILE_PAIR, 0, KV / 16);
        if (!strcmp(f, "wv"))
            return tiled(b + 3, y.wqkv + (uint64_t)((Q + KV) / 16) * TH, KV, H, TILE_PAIR, 0, KV / 16);
        if (!strcmp(f, "wg")) return tiled(b + 6, y.wgu, F, H, TILE_GATEUP, 0, (F + 7) / 8);
        if (!strcmp(f, "wu")) return tiled(b + 7, y.wgu, F, H, TILE_GATEUP, 1, (F + 7) / 8);
    } else {
        if (!strcmp(f, "wq")) return mat(b + 1, y.wqkv, Q, H);
        if (!strcmp(f, "wk")) return mat(b + 2, y.wqkv + (uint64_t)Q * H * eb, KV, H);
        if (!strcmp(f, "wv")) return mat(b + 3, y.wqkv + (uint64_t)(Q + KV) * H * eb, KV, H);
        // gate and up rows are interleaved: row 2f = gate f, row 2f+1 = up f
        if (!strcmp(f, "wg")) return mat(b + 6, y.wgu, F, H, 2 * (uint64_t)H * eb);
        if (!strcmp(f, "wu")) return mat(b + 7, y.wgu + (uint64_t)H * eb, F, H, 2 * (uint64_t)H * eb);
    }
    if (!strcmp(f, "wo")) return L.tiled_q ? tiled(b + 4, y.wo, H, Q, TILE_PLAIN, 0, (H + 15) / 16) : mat(b + 4, y.wo, H, Q);
    if (!strcmp(f, "mlp_norm")) return gain(b + 5, y.mlp_norm);
    if (!strcmp(f, "wd")) return L.tiled_f ? tiled(b + 8, y.wd, H, F, TILE_PLAIN, 0, (H + 15) / 16) : mat(b + 8, y.wd, H, F);
    return false;
}

}  // namespace

extern "C" int swift_create(const swift_model_config *cfg, void *device_mem, uint64_t device_bytes, void *hip_stream,
                            swift_ctx **out) {
    if (!out) return fail(SWIFT_EINVAL, "null output");
    *out = nullptr;
    int rc = swift_check_config(cfg);
    if (rc) return rc;
    if (!device_mem || ((uintptr_t)device_mem & 255)) return fail(SWIFT_EINVAL, "device_mem must be non-null, 256-byte aligned");
    Layout L = make_layout(*cfg);
    if (device_bytes < L.total) return fail(SWIFT_ECAPACITY, "device arena smaller than swift_device_bytes");
    int dev = 0, n_cu = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    // the static scratch array's address on this device (needed by swift_verify_static only; resolved here
    // so that that call has nothing left to set up)
    char *static_base = nullptr;
    rc = static_scratch(&static_base);
    if (rc) return rc;
    swift_ctx *x = new swift_ctx();
    x->c = *cfg;
    x->L = L;
    x->base = (char *)device_mem;
    x->stream = (hipStream_t)hip_stream;
    x->n_cu = n_cu > 0 ? n_cu : 256;
    x->loaded.assign(n_tensors(*cfg), false);
    x->n_loaded = 0;
    x->n = 0;
    x->pending = -1;
    x->k_verify = -1;
    x->tree_levels = -1;
    x->k_sampled = -1;
    x->want_topk = false;
    x->h_topk = nullptr;
    memset(&x->st, 0, sizeof(x->st));
    x->arena_scr = Scratch{dptr<float>(x, L.mv_part), dptr<int>(x, L.mv_counters), L.mv_part_capacity, dptr<float>(x, L.part_o),
                           dptr<float>(x, L.part_ml), (size_t)kMaxRows * cfg->n_q_heads * L.n_split_max * cfg->head_dim};
    x->scr = x->arena_scr;
    x->no_events = false;
    x->prof_class = -1;
    memset(x->tune_ks, 0, sizeof(x->tune_ks));
    memset(x->tune_wg, 0, sizeof(x->tune_wg));
    x->prefill_sub = 0;
    x->gemm_rgw = 0;
    x->h_tok = nullptr;
    x->h_conf = nullptr;
    hipError_t e = hipHostMalloc((void **)&x->h_tok, (2 * kMaxBlockRows + 4 + kTopK) * 4, hipHostMallocDefault);
    if (e != hipSuccess) {
        delete x;
        return fail(SWIFT_EDEVICE, std::string("hipHostMalloc: ") + hipGetErrorString(e));
    }
    x->h_conf = (float *)(x->h_tok + kMaxBlockRows);
    x->h_topk = x->h_tok + 2 * kMaxBlockRows + 4;

    // rotary tables: angle = pos * theta^(-2i/d) in fp64, cos/sin rounded to fp32
    const int half = cfg->head_dim / 2;
    std::vector<float> ct((size_t)cfg->max_seq * half), stb((size_t)cfg->max_seq * half);
    for (int i = 0; i < half; ++i) {
        const double freq = std::pow((double)cfg->rope_theta, -2.0 * (double)i / (double)cfg->head_dim);
        for (int p = 0; p < cfg->max_seq; ++p) {
            const double ang = (double)p * freq;
            ct[(size_t)p * half + i] = (float)std::cos(ang);
            stb[(size_t)p * half + i] = (float)std::sin(ang);
        }
    }
    e = hipMemsetAsync(x->base + L.mv_counters, 0, 4096 * 4, x->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(x->base + L.cos, ct.data(), ct.size() * 4, hipMemcpyHostToDevice, x->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(x->base + L.sin, stb.data(), stb.size() * 4, hipMemcpyHostToDevice, x->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(x->stream);
    if (e != hipSuccess) {
        (void)hipHostFree(x->h_tok);
        delete x;
        return fail(SWIFT_EDEVICE, std::string("rotary table upload: ") + hipGetErrorString(e));
    }
    *out = x;
    return SWIFT_OK;
}

extern "C" int swift_destroy(swift_ctx *x) {
    if (!x) return fail(SWIFT_EINVAL, "null context");
    (void)hipStreamSynchronize(x->stream);
    for (auto &r : x->prof) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    for (auto &e : x->pool) (void)hipEventDestroy(e);
    if (x->h_tok) (void)hipHostFree(x->h_tok);
    delete x;
    return SWIFT_OK;
}

extern "C" int swift_load_tensor(swift_ctx *x, const char *name, const void *data, int dtype, int64_t n_elems) {
    if (!x || !name || !data) return fail(SWIFT_EINVAL, "null argument");
    Slot sl;
    if (!find_slot(x, name, &sl)) return fail(SWIFT_EINVAL, std::string("unknown tensor name: ") + name);
    if (n_elems != sl.n) return fail(SWIFT_EINVAL, std::string("wrong element count for ") + name);
    const int want = sl.is_gain ? SWIFT_F32 : x->c.dtype;
    if (dtype != want) return fail(SWIFT_EINVAL, std::string("wrong dtype for ") + name);
    const uint64_t eb = elem_bytes(want);
    if (sl.tiled) {
        // re-tile on the device; a host tensor goes through the staging area first
        hipPointerAttribute_t pa;
        const void *src = data;
        hipError_t pe = hipPointerGetAttributes(&pa, data);
        const bool on_device = pe == hipSuccess && pa.type == hipMemoryTypeDevice;
        if (pe != hipSuccess) (void)hipGetLastError();  // plain host memory is reported as an error by some runtimes
        if (!on_device) {
            if ((uint64_t)sl.n * eb > x->L.stage_bytes) return fail(SWIFT_ECAPACITY, "staging area too small");
            HIP_TRY(hipMemcpyAsync(x->base + x->L.stage, data, (uint64_t)sl.n * eb, hipMemcpyHostToDevice, x->stream));
            src = x->base + x->L.stage;
        }
        TileArgs t{};
        t.src = src;
        t.src_rows = sl.rows;
        t.K = sl.cols;
        t.dst = x->base + sl.off;
        t.T = (sl.cols + 31) / 32;
        t.n_rg = sl.n_rg;
        t.mode = sl.tile_mode;
        t.head_dim = x->c.head_dim;
        t.part = sl.part;
        HIP_TRY(launch_tile_weights(t, x->stream));
    } else if (sl.dst_pitch == 0) {
        HIP_TRY(hipMemcpyAsync(x->base + sl.off, data, (uint64_t)sl.n * eb, hipMemcpyDefault, x->stream));
    } else {
        HIP_TRY(hipMemcpy2DAsync(x->base + sl.off, sl.dst_pitch, data, (uint64_t)sl.cols * eb, (uint64_t)sl.cols * eb,
                                 sl.rows, hipMemcpyDefault, x->stream));
    }
    HIP_TRY(hipStreamSynchronize(x->stream));
    if (!x->loaded[sl.index]) {
        x->loaded[sl.index] = true;
        x->n_loaded++;
    }
    return SWIFT_OK;
}

// ------------------------------------------------------------------------------------------
// decoding path
// ------------------------------------------------------------------------------------------
extern "C" int swift_prefill(swift_ctx *x, const int32_t *prompt, int n_prompt, int32_t *first_token) {
    if (!x || !prompt || !first_token) return fail(SWIFT_EINVAL, "null argument");
    if (n_prompt < 1) return fail(SWIFT_EINVAL, "empty prompt");
    if (n_prompt >= x->c.max_seq) return fail(SWIFT_ECAPACITY, "prompt does not leave room in the cache");
    if (x->n_loaded != n_tensors(x->c)) return fail(SWIFT_ESTATE, "not all tensors are loaded");
    for (int i = 0; i < n_prompt; ++i)
        if (prompt[i] < 0 || prompt[i] >= x->c.vocab) return fail(SWIFT_EINVAL, "token id out of range");
    int last_rows = 0;
    if (x->L.tiled) {
        // bf16 models: macro blocks of up to kMacroSub sub-blocks of 64 rows share one sweep over the weights (a
        // blocked matrix product per projection); what is left at the end, if it fits one sub-block, goes through
        // the block kernels
        const int subs = x->prefill_sub > 0 ? x->prefill_sub : kMacroSub;
        for (int i = 0; i < n_prompt;) {
            const int rows = std::min(subs * kMaxBlockRows, n_prompt - i);
            const bool macro = x->prefill_sub >= 0 && rows > kMaxBlockRows;
            const int n_blk = std::min(rows, kMaxBlockRows * (macro ? subs : 1));
            const int n_sub = macro ? (n_blk + kMaxBlockRows - 1) / kMaxBlockRows : 0;
            last_rows = macro ? n_blk - (n_sub - 1) * kMaxBlockRows : n_blk;
            int rc = forward_block_tiled(x, prompt + i, last_rows, i, nullptr, i + n_blk == n_prompt, false, nullptr, false, n_sub);
            if (rc) return rc;
            i += n_blk;
        }
    } else {
        for (int i = 0; i < n_prompt; i += kMaxRows) {
            last_rows = std::min((int)kMaxRows, n_prompt - i);
            int rc = forward_block(x, prompt + i, last_rows, i, nullptr, i + last_rows == n_prompt, false, nullptr, false);
            if (rc) return rc;
        }
    }
    int rc = read_results(x, last_rows);
    if (rc) return rc;
    x->n = n_prompt;
    x->pending = x->h_tok[last_rows - 1];
    x->k_verify = -1;
    x->tree_levels = -1;
    x->k_sampled = -1;
    memset(&x->st, 0, sizeof(x->st));
    x->st.emitted_total = 1;
    *first_token = x->pending;
    return SWIFT_OK;
}

extern "C" int swift_eval_mask(swift_ctx *x, const uint8_t *skip_mask, const int32_t *window, int gamma,
                               int32_t *predicted, int *n_match) {
    if (!x || !skip_mask || !window || !n_match) return fail(SWIFT_EINVAL, "null argument");
    if (gamma < 1 || gamma > SWIFT_MAX_WINDOW) return fail(SWIFT_EINVAL, "gamma out of range (1..128)");
    if (x->pending < 0) return fail(SWIFT_ESTATE, "candidate evaluation before prefill");
    if (gamma > x->n) return fail(SWIFT_ESTATE, "window longer than the cache");
    for (int i = 0; i <= gamma; ++i)
        if (window[i] < 0 || window[i] >= x->c.vocab) return fail(SWIFT_EINVAL, "token id out of range");
    int m = 0;
    if (x->L.tiled && x->prefill_sub >= 0 && gamma > kMaxBlockRows) {
        // bf16 models: a window of more than one 64-row block is one macro block (one sweep over the weights of
        // the candidate's sublayers for all its rows), then the LM head and the arg-max sub-block by sub-block
        const int n_sub = (gamma + kMaxBlockRows - 1) / kMaxBlockRows;
        int rc = forward_block_tiled(x, window, gamma - (n_sub - 1) * kMaxBlockRows, x->n - gamma, skip_mask, false, true,
                                     nullptr, false, n_sub);
        if (rc) return rc;
        for (int sb = 0; sb < n_sub; ++sb) {
            const int r0 = sb * kMaxBlockRows, rows = std::min(kMaxBlockRows, gamma - r0);
            if ((rc = macro_sub_logits(x, sb, rows))) return rc;
            if ((rc = read_results(x, rows))) return rc;
            for (int i = 0; i < rows; ++i) {
                if (predicted) predicted[r0 + i] = x->h_tok[i];
                if (x->h_tok[i] == window[r0 + i + 1]) ++m;
            }
        }
        *n_match = m;
        return SWIFT_OK;
    }
    // Rows read the target's cache and write nothing, so a longer window can also be evaluated block by block
    // (fp32 models; bf16 models when macro blocks are switched off).
    for (int r0 = 0; r0 < gamma; r0 += kMaxBlockRows) {
        const int rows = std::min(kMaxBlockRows, gamma - r0);
        int rc = forward_block(x, window + r0, rows, x->n - gamma + r0, skip_mask, true, true, nullptr, false);
        if (rc) return rc;
        rc = read_results(x, rows);
        if (rc) return rc;
        for (int i = 0; i < rows; ++i) {
            if (predicted) predicted[r0 + i] = x->h_tok[i];
            if (x->h_tok[i] == window[r0 + i + 1]) ++m;
        }
    }
    *n_match = m;
    return SWIFT_OK;
}

extern "C" int swift_draft_step(swift_ctx *x, const uint8_t *skip_mask, int max_k, float conf_threshold,
                                int32_t *draft_tokens, float *draft_conf, int *k_out) {
    if (!x || !skip_mask || !k_out) return fail(SWIFT_EINVAL, "null argument");
    if (max_k < 0 || max_k > SWIFT_MAX_BLOCK - 1) return fail(SWIFT_EINVAL, "max_k out of range");
    if (max_k > 0 && (!draft_tokens || !draft_conf)) return fail(SWIFT_EINVAL, "null output array");
    if (x->pending < 0) return fail(SWIFT_ESTATE, "draft before prefill");
    if (x->n + max_k + 1 > x->c.max_seq) return fail(SWIFT_ECAPACITY, "draft would run past the cache capacity");
    int32_t prev = x->pending;
    int k = 0;
    x->k_verify = -1;     // the draft overwrites slots an outstanding verification wrote: its accept must fail
    x->tree_levels = -1;
    x->k_sampled = -1;
    for (int j = 1; j <= max_k; ++j) {
        int rc = forward_block(x, &prev, 1, x->n + j - 1, skip_mask, true);
        if (rc) return rc;
        rc = read_results(x, 1);
        if (rc) return rc;
        draft_tokens[k] = x->h_tok[0];
        draft_conf[k] = x->h_conf[0];
        prev = x->h_tok[0];
        ++k;
        x->st.draft_passes++;
        if (x->h_conf[0] < conf_threshold) break;
    }
    *k_out = k;
    return SWIFT_OK;
}

namespace {
int verify_impl(swift_ctx *x, const int32_t *tokens, int k, int32_t *target_tokens, float *logits_out) {
    int rc = forward_block(x, tokens, k + 1, x->n, nullptr, true);
    if (rc) return rc;
    rc = read_results(x, k + 1);
    if (rc) return rc;
    if (logits_out) {
        HIP_TRY(hipMemcpyAsync(logits_out, dptr<float>(x, x->L.logits), (size_t)(k + 1) * x->c.vocab * 4,
                               hipMemcpyDeviceToHost, x->stream));
        HIP_TRY(hipStreamSynchronize(x->stream));
    }
    for (int i = 0; i <= k; ++i) {
        x->vtokens[i] = tokens[i];
        x->targets[i] = x->h_tok[i];
        target_tokens[i] = x->h_tok[i];
    }
    x->k_verify = k;
    x->tree_levels = -1;
    x->k_sampled = -1;
    x->st.verify_passes++;
    return SWIFT_OK;
}

int check_verify_args(swift_ctx *x, const int32_t *tokens, int k, int32_t *target_tokens) {
    if (!x || !tokens || !target_tokens) return fail(SWIFT_EINVAL, "null argument");
    if (k < 0 || k > SWIFT_MAX_BLOCK - 1) return fail(SWIFT_EINVAL, "k out of range");
    if (x->pending < 0) return fail(SWIFT_ESTATE, "verify before prefill");
    if (tokens[0] != x->pending) return fail(SWIFT_EINVAL, "tokens[0] must be the pending token");
    for (int i = 0; i <= k; ++i)
        if (tokens[i] < 0 || tokens[i] >= x->c.vocab) return fail(SWIFT_EINVAL, "token id out of range");
    if (x->n + k + 1 > x->c.max_seq) return fail(SWIFT_ECAPACITY, "block would run past the cache capacity");
    return SWIFT_OK;
}
}  // namespace

extern "C" int swift_verify(swift_ctx *x, const int32_t *tokens, int k, int32_t *target_tokens, float *logits_out) {
    int rc = check_verify_args(x, tokens, k, target_tokens);
    if (rc) return rc;
    return verify_impl(x, tokens, k, target_tokens, logits_out);
}

// ------------------------------------------------------------------------------------------
// verification without any allocation: the kernels' scratch in a file-scope device array
// ------------------------------------------------------------------------------------------
extern "C" int swift_verify_static(swift_ctx *x, const int32_t *tokens, int k, int32_t *target_tokens, float *logits_out) {
    int rc = check_verify_args(x, tokens, k, target_tokens);
    if (rc) return rc;
    const swift_model_config &c = x->c;
    const int R = k + 1, d = c.head_dim, H = c.hidden, Q = c.n_q_heads * d, KV = c.n_kv_heads * d, F = c.ffn, V = c.vocab;
    // ---- what this block needs of the array, checked before anything is launched
    size_t attn_floats = 0;
    {
        AttnArgs a{};
        a.rows = R;
        a.n_ctx = x->n + 1;
        a.max_seq = c.max_seq;
        a.head_dim = d;
        a.n_q_heads = c.n_q_heads;
        a.n_kv_heads = c.n_kv_heads;
        a.max_split = x->L.n_split_max;
        a.nb32 = x->L.nb32;
        attn_floats = x->L.mfma_attn ? attn_mfma_partial_floats(a, x->n_cu) : attn_partial_floats(c.dtype, a, x->n_cu);
    }
    // part_o then holds attn_floats floats and part_ml two per head_dim of them
    const size_t ml_bytes = align_up(attn_floats / d * 2 * 4);
    if (ml_bytes + attn_floats * 4 > kStaticAttnBytes)
        return fail(SWIFT_ECAPACITY, "swift_verify_static: the attention partials of a block of " + std::to_string(R) +
                                         " rows of this model need " + std::to_string(ml_bytes + attn_floats * 4) +
                                         " bytes, the static scratch holds " + std::to_string(kStaticAttnBytes) +
                                         "; use swift_verify");
    if (x->L.tiled) {
        const struct { int O, K, n_rg; } mats[5] = {{Q + 2 * KV, H, (Q + 2 * KV) / 16}, {H, Q, (H + 15) / 16},
                                                    {2 * F, H, (F + 7) / 8},             {H, F, (H + 15) / 16},
                                                    {V, H, (V + 15) / 16}};
        for (const auto &mt : mats) {
            MvArgs m{};
            m.O = mt.O;
            m.K = mt.K;
            m.T = (mt.K + 31) / 32;
            m.n_rg = mt.n_rg;
            m.R = R;
            m.RL = block_row_layout(R, true);
            m.head_dim = d;
            m.part_capacity = x->L.mv_part_capacity;
            const int slots = mv_split_slots(m, x->n_cu);
            if (slots > kStaticPartSlots || (mt.n_rg + 7) / 8 > (int)(kStaticCounterBytes / 4))
                return fail(SWIFT_ECAPACITY, "swift_verify_static: a projection of this model needs more split-K scratch "
                                             "than the static array holds; use swift_verify");
        }
    }
    char *base = nullptr;
    rc = static_scratch(&base);
    if (rc) return rc;
    Scratch st{};
    st.mv_counters = (int *)base;
    st.mv_part = (float *)(base + kStaticCounterBytes);
    st.mv_part_capacity = kStaticPartSlots;
    st.part_ml = (float *)(base + kStaticCounterBytes + kStaticPartBytes);
    st.part_o = (float *)(base + kStaticCounterBytes + kStaticPartBytes + ml_bytes);
    st.part_o_floats = attn_floats;
    // The array keeps what the last call left (of any context on this device): the arrival counters must
    // start at zero.  A fill kernel, not a memset: the caller may be capturing the stream into a graph.
    HIP_TRY(launch_fill_u32(st.mv_counters, 0u, (int64_t)(kStaticCounterBytes / 4), x->stream));
    x->scr = st;
    x->no_events = true;
    rc = verify_impl(x, tokens, k, target_tokens, logits_out);
    x->scr = x->arena_scr;
    x->no_events = false;
    return rc;
}

extern "C" int swift_accept(swift_ctx *x, int32_t *emitted, int *n_emitted) {
    if (!x || !emitted || !n_emitted) return fail(SWIFT_EINVAL, "null argument");
    if (x->k_verify < 0) return fail(SWIFT_ESTATE, "accept without a preceding verify");
    const int k = x->k_verify;
    const int m = swift_match_prefix(x->vtokens + 1, x->targets, k);
    for (int i = 0; i < m; ++i) emitted[i] = x->vtokens[1 + i];
    emitted[m] = x->targets[m];
    *n_emitted = m + 1;
    x->n += m + 1;
    x->pending = x->targets[m];
    x->k_verify = -1;
    x->st.accepted += m;
    x->st.emitted_by_verify += m + 1;
    x->st.emitted_total += m + 1;
    return SWIFT_OK;
}

// ------------------------------------------------------------------------------------------
// dynamic verification (Section 4.2, second strategy): top-k candidates per draft position, verified as a
// token tree
// ------------------------------------------------------------------------------------------
extern "C" int swift_topk_width(float p) { return p <= 0.5f ? 10 : p <= 0.8f ? 5 : p <= 0.95f ? 3 : 1; }

extern "C" int swift_draft_step_topk(swift_ctx *x, const uint8_t *skip_mask, int max_k, float conf_threshold, int max_width,
                                     int32_t *tokens, float *draft_conf, int *width, int *k_out) {
    if (!x || !skip_mask || !k_out) return fail(SWIFT_EINVAL, "null argument");
    if (max_k < 0 || max_k > SWIFT_MAX_BLOCK - 1) return fail(SWIFT_EINVAL, "max_k out of range");
    if (max_width < 1) return fail(SWIFT_EINVAL, "max_width must be at least 1");
    if (max_k > 0 && (!tokens || !draft_conf || !width)) return fail(SWIFT_EINVAL, "null output array");
    if (x->pending < 0) return fail(SWIFT_ESTATE, "draft before prefill");
    // every row of the block needs a cache slot of its own
    const int cap_rows = std::min(SWIFT_MAX_BLOCK, x->c.max_seq - x->n);
    if (cap_rows < 1) return fail(SWIFT_ECAPACITY, "no cache slot left for the pending token");
    int32_t prev = x->pending;
    int k = 0, rows = 1;
    x->k_verify = -1;     // the draft overwrites slots an outstanding verification wrote: its accept must fail
    x->tree_levels = -1;
    x->k_sampled = -1;
    for (int j = 1; j <= max_k && rows < cap_rows; ++j) {
        x->want_topk = true;
        int rc = forward_block(x, &prev, 1, x->n + j - 1, skip_mask, true);
        x->want_topk = false;
        if (rc) return rc;
        HIP_TRY(hipMemcpyAsync(x->h_topk, dptr<int32_t>(x, x->L.out_topk), kTopK * 4, hipMemcpyDeviceToHost, x->stream));
        rc = read_results(x, 1);
        if (rc) return rc;
        const float p = x->h_conf[0];
        int w = swift_topk_width(p);
        w = std::min(w, max_width);
        w = std::min(w, cap_rows - rows);
        w = std::min(w, x->c.vocab);
        for (int i = 0; i < w; ++i) tokens[(size_t)k * SWIFT_TOPK + i] = x->h_topk[i];
        width[k] = w;
        draft_conf[k] = p;
        prev = x->h_tok[0];
        rows += w;
        ++k;
        x->st.draft_passes++;
        if (p < conf_threshold) break;
    }
    *k_out = k;
    return SWIFT_OK;
}

extern "C" int swift_verify_tree(swift_ctx *x, const int32_t *tokens, const int *width, int levels, int32_t *target_tokens,
                                 float *logits_out) {
    if (!x || !tokens || !target_tokens) return fail(SWIFT_EINVAL, "null argument");
    if (levels < 0 || levels > SWIFT_MAX_BLOCK - 1 || (levels > 0 && !width)) return fail(SWIFT_EINVAL, "levels out of range");
    if (x->pending < 0) return fail(SWIFT_ESTATE, "verify before prefill");
    if (tokens[0] != x->pending) return fail(SWIFT_EINVAL, "tokens[0] must be the pending token");
    TreeRows t{};
    int rows = 1;
    for (int j = 1; j <= levels; ++j) {
        const int w = width[j - 1];
        if (w < 1 || w > SWIFT_TOPK) return fail(SWIFT_EINVAL, "level width out of range (1..10)");
        if (rows + w > SWIFT_MAX_BLOCK) return fail(SWIFT_EINVAL, "more than SWIFT_MAX_BLOCK rows in the tree");
        t.spine[j] = (uint8_t)rows;
        for (int i = 0; i < w; ++i) t.depth[rows++] = (uint8_t)j;
    }
    for (int r = 0; r < rows; ++r)
        if (tokens[r] < 0 || tokens[r] >= x->c.vocab) return fail(SWIFT_EINVAL, "token id out of range");
    if (x->n + rows > x->c.max_seq) return fail(SWIFT_ECAPACITY, "block would run past the cache capacity");
    int rc = forward_block(x, tokens, rows, x->n, nullptr, true, false, &t);
    if (rc) return rc;
    rc = read_results(x, rows);
    if (rc) return rc;
    if (logits_out) {
        HIP_TRY(hipMemcpyAsync(logits_out, dptr<float>(x, x->L.logits), (size_t)rows * x->c.vocab * 4, hipMemcpyDeviceToHost,
                               x->stream));
        HIP_TRY(hipStreamSynchronize(x->stream));
    }
    for (int r = 0; r < rows; ++r) {
        x->vtokens[r] = tokens[r];
        x->targets[r] = x->h_tok[r];
        target_tokens[r] = x->h_tok[r];
    }
    x->tree_levels = levels;
    for (int j = 0; j < levels; ++j) x->tree_width[j] = width[j];
    x->k_verify = -1;
    x->k_sampled = -1;
    x->st.verify_passes++;
    return SWIFT_OK;
}

extern "C" int swift_accept_tree(swift_ctx *x, int32_t *emitted, int *n_emitted) {
    if (!x || !emitted || !n_emitted) return fail(SWIFT_EINVAL, "null argument");
    if (x->tree_levels < 0) return fail(SWIFT_ESTATE, "accept without a preceding tree verification");
    const swift_model_config &c = x->c;
    KvMoveArgs mv{};
    int32_t cur = x->targets[0];
    int acc = 0, start = 1;
    for (int j = 1; j <= x->tree_levels; ++j) {
        const int w = x->tree_width[j - 1];
        int hit = -1;
        for (int i = 0; i < w && hit < 0; ++i)
            if (x->vtokens[start + i] == cur) hit = i;
        if (hit < 0) break;
        const int row = start + hit;
        emitted[acc++] = cur;
        if (row != acc) {  // the accepted row's keys/values to slot n + acc
            mv.src[mv.n_moves] = x->n + row;
            mv.dst[mv.n_moves] = x->n + acc;
            ++mv.n_moves;
        }
        cur = x->targets[row];
        if (hit != 0) break;  // a candidate beside the first has no children
        start += w;
    }
    if (mv.n_moves > 0) {
        mv.kv = x->base + x->L.kv;
        mv.layer_elems = (int64_t)((x->L.kv_k_bytes + x->L.kv_v_bytes) / elem_bytes(c.dtype));
        mv.v_offset = (int64_t)(x->L.kv_k_bytes / elem_bytes(c.dtype));
        mv.n_layers = c.n_layers;
        mv.nb32 = x->L.nb32;
        mv.n_kv_heads = c.n_kv_heads;
        mv.max_seq = c.max_seq;
        mv.head_dim = c.head_dim;
        HIP_TRY(launch_kv_move(c.dtype, mv, x->stream));
    }
    emitted[acc] = cur;
    *n_emitted = acc + 1;
    x->n += acc + 1;
    x->pending = cur;
    x->tree_levels = -1;
    x->st.accepted += acc;
    x->st.emitted_by_verify += acc + 1;
    x->st.emitted_total += acc + 1;
    return SWIFT_OK;
}

// ------------------------------------------------------------------------------------------
// speculative sampling (Section 5.1, Appendix B.2)
// ------------------------------------------------------------------------------------------
namespace {
int check_sampling(float temperature, float top_p) {
    if (!(temperature > 0.f) || !(top_p > 0.f)) return fail(SWIFT_EINVAL, "temperature and top_p must be positive");
    return SWIFT_OK;
}
bool is_uniform(float u) { return u >= 0.f && u < 1.f; }
// probs row `dst_row` of buffer `dst` <- warped logits rows [row0, row0 + rows)
int warp_rows(swift_ctx *x, int row0, int rows, float temperature, float top_p, uint64_t dst, int dst_row) {
    WarpArgs w{};
    w.logits = dptr<float>(x, x->L.logits) + (size_t)row0 * x->c.vocab;
    w.ld_logits = x->c.vocab;
    w.V = x->c.vocab;
    w.rows = rows;
    w.temperature = temperature;
    w.top_p = top_p;
    w.probs = dptr<float>(x, dst) + (size_t)dst_row * x->c.vocab;
    HIP_TRY(timed(x, SWIFT_KC_OTHER, (uint64_t)rows * x->c.vocab * 8, [&] { return launch_warp(w, x->stream); }));
    return SWIFT_OK;
}
}  // namespace

extern "C" int swift_prefill_sample(swift_ctx *x, const int32_t *prompt, int n_prompt, float temperature, float top_p,
                                    float u, int32_t *first_token) {
    if (!first_token) return fail(SWIFT_EINVAL, "null argument");
    int rc = check_sampling(temperature, top_p);
    if (rc) return rc;
    if (!is_uniform(u)) return fail(SWIFT_EINVAL, "uniforms must lie in [0, 1)");
    int32_t greedy;
    rc = swift_prefill(x, prompt, n_prompt, &greedy);
    if (rc) return rc;
    // the last prompt row's logits are still in place
    const int block = x->L.tiled ? kMaxBlockRows : kMaxRows;
    const int last_row = (n_prompt - 1) % block;
    rc = warp_rows(x, last_row, 1, temperature, top_p, x->L.samp_p, 0);
    if (rc) return rc;
    HIP_TRY(launch_draw(dptr<float>(x, x->L.samp_p), x->c.vocab, u, dptr<int32_t>(x, x->L.samp_out), x->stream));
    HIP_TRY(hipMemcpyAsync(x->h_topk, dptr<int32_t>(x, x->L.samp_out), 4, hipMemcpyDeviceToHost, x->stream));
    HIP_TRY(hipStreamSynchronize(x->stream));
    x->pending = x->h_topk[0];
    *first_token = x->pending;
    return SWIFT_OK;
}

extern "C" int swift_draft_step_sample(swift_ctx *x, const uint8_t *skip_mask, int max_k, float conf_threshold,
                                       float temperature, float top_p, const float *u, int32_t *draft_tokens,
                                       float *draft_conf, int *k_out) {
    if (!x || !skip_mask || !k_out) return fail(SWIFT_EINVAL, "null argument");
    if (max_k < 0 || max_k > SWIFT_MAX_BLOCK - 1) return fail(SWIFT_EINVAL, "max_k out of range");
    if (max_k > 0 && (!draft_tokens || !draft_conf || !u)) return fail(SWIFT_EINVAL, "null array");
    int rc = check_sampling(temperature, top_p);
    if (rc) return rc;
    for (int j = 0; j < max_k; ++j)
        if (!is_uniform(u[j])) return fail(SWIFT_EINVAL, "uniforms must lie in [0, 1)");
    if (x->pending < 0) return fail(SWIFT_ESTATE, "draft before prefill");
    if (x->n + max_k + 1 > x->c.max_seq) return fail(SWIFT_ECAPACITY, "draft would run past the cache capacity");
    int32_t prev = x->pending;
    int k = 0;
    x->k_verify = -1;     // the draft overwrites slots an outstanding verification wrote: its accept must fail
    x->tree_levels = -1;
    x->k_sampled = -1;
    for (int j = 1; j <= max_k; ++j) {
        rc = forward_block(x, &prev, 1, x->n + j - 1, skip_mask, true);
        if (rc) return rc;
        rc = warp_rows(x, 0, 1, temperature, top_p, x->L.samp_q, k);
        if (rc) return rc;
        HIP_TRY(launch_draw(dptr<float>(x, x->L.samp_q) + (size_t)k * x->c.vocab, x->c.vocab, u[j - 1],
                            dptr<int32_t>(x, x->L.samp_out), x->stream));
        HIP_TRY(hipMemcpyAsync(x->h_topk, dptr<int32_t>(x, x->L.samp_out), 4, hipMemcpyDeviceToHost, x->stream));
        rc = read_results(x, 1);
        if (rc) return rc;
        prev = x->h_topk[0];
        draft_tokens[k] = prev;
        draft_conf[k] = x->h_conf[0];
        x->sampled[k] = prev;
        ++k;
        x->st.draft_passes++;
        if (x->h_conf[0] < conf_threshold) break;
    }
    x->k_sampled = k;
    *k_out = k;
    return SWIFT_OK;
}

extern "C" int swift_verify_sample(swift_ctx *x, const int32_t *tokens, int k, float temperature, float top_p,
                                   const float *u_accept, float u_final, int32_t *emitted, int *n_emitted,
                                   float *probs_out) {
    if (!x || !tokens || !emitted || !n_emitted) return fail(SWIFT_EINVAL, "null argument");
    if (k < 0 || k > SWIFT_MAX_BLOCK - 1) return fail(SWIFT_EINVAL, "k out of range");
    if (k > 0 && !u_accept) return fail(SWIFT_EINVAL, "null array");
    int rc = check_sampling(temperature, top_p);
    if (rc) return rc;
    if (!is_uniform(u_final)) return fail(SWIFT_EINVAL, "uniforms must lie in [0, 1)");
    for (int i = 0; i < k; ++i)
        if (!is_uniform(u_accept[i])) return fail(SWIFT_EINVAL, "uniforms must lie in [0, 1)");
    if (x->pending < 0) return fail(SWIFT_ESTATE, "verify before prefill");
    if (tokens[0] != x->pending) return fail(SWIFT_EINVAL, "tokens[0] must be the pending token");
    if (k > 0 && x->k_sampled < k) return fail(SWIFT_ESTATE, "no draft distributions for these tokens (swift_draft_step_sample first)");
    for (int i = 0; i < k; ++i)
        if (tokens[1 + i] != x->sampled[i]) return fail(SWIFT_EINVAL, "tokens differ from the last sampled draft");
    if (x->n + k + 1 > x->c.max_seq) return fail(SWIFT_ECAPACITY, "block would run past the cache capacity");
    rc = forward_block(x, tokens, k + 1, x->n, nullptr, true);
    if (rc) return rc;
    rc = warp_rows(x, 0, k + 1, temperature, top_p, x->L.samp_p, 0);
    if (rc) return rc;
    SpecAcceptArgs sa{};
    sa.p = dptr<float>(x, x->L.samp_p);
    sa.q = dptr<float>(x, x->L.samp_q);
    sa.V = x->c.vocab;
    sa.k = k;
    for (int i = 0; i < k; ++i) {
        sa.x[i] = tokens[1 + i];
        sa.u_accept[i] = u_accept[i];
    }
    sa.u_final = u_final;
    sa.out = dptr<int32_t>(x, x->L.samp_out);
    HIP_TRY(timed(x, SWIFT_KC_OTHER, (uint64_t)x->c.vocab * 8, [&] { return launch_spec_accept(sa, x->stream); }));
    HIP_TRY(hipMemcpyAsync(x->h_topk, dptr<int32_t>(x, x->L.samp_out), 8, hipMemcpyDeviceToHost, x->stream));
    rc = read_results(x, k + 1);
    if (rc) return rc;
    if (probs_out) {
        HIP_TRY(hipMemcpyAsync(probs_out, dptr<float>(x, x->L.samp_p), (size_t)(k + 1) * x->c.vocab * 4, hipMemcpyDeviceToHost,
                               x->stream));
        HIP_TRY(hipStreamSynchronize(x->stream));
    }
    const int m = x->h_topk[0];
    if (m < 0 || m > k) return fail(SWIFT_EDEVICE, "acceptance kernel returned an impossible count");
    for (int i = 0; i < m; ++i) emitted[i] = tokens[1 + i];
    emitted[m] = x->h_topk[1];
    *n_emitted = m + 1;
    x->n += m + 1;
    x->pending = x->h_topk[1];
    x->k_verify = -1;
    x->tree_levels = -1;
    x->k_sampled = -1;
    x->st.verify_passes++;
    x->st.accepted += m;
    x->st.emitted_by_verify += m + 1;
    x->st.emitted_total += m + 1;
    return SWIFT_OK;
}

extern "C" int swift_rollback(swift_ctx *x, int new_cache_len, int32_t pending_token) {
    if (!x) return fail(SWIFT_EINVAL, "null context");
    if (x->pending < 0) return fail(SWIFT_ESTATE, "rollback before prefill");
    if (new_cache_len < 0 || new_cache_len > x->n) return fail(SWIFT_EINVAL, "new length must be in [0, cache length]");
    if (pending_token < 0 || pending_token >= x->c.vocab) return fail(SWIFT_EINVAL, "token id out of range");
    x->n = new_cache_len;
    x->pending = pending_token;
    x->k_verify = -1;
    x->tree_levels = -1;
    x->k_sampled = -1;
    return SWIFT_OK;
}

extern "C" int swift_get_state(swift_ctx *x, int *cache_len, int32_t *pending_token) {
    if (!x) return fail(SWIFT_EINVAL, "null context");
    if (cache_len) *cache_len = x->n;
    if (pending_token) *pending_token = x->pending;
    return SWIFT_OK;
}

extern "C" int swift_get_config(swift_ctx *x, swift_model_config *out) {
    if (!x || !out) return fail(SWIFT_EINVAL, "null argument");
    *out = x->c;
    return SWIFT_OK;
}

extern "C" int swift_get_stats(swift_ctx *x, swift_stats *out) {
    if (!x || !out) return fail(SWIFT_EINVAL, "null argument");
    *out = x->st;
    return SWIFT_OK;
}

// ------------------------------------------------------------------------------------------
// test and measurement hooks
// ------------------------------------------------------------------------------------------
extern "C" int swift_debug_poison_kv(swift_ctx *x) {
    if (!x) return fail(SWIFT_EINVAL, "null context");
    const swift_model_config &c = x->c;
    const uint64_t eb = elem_bytes(c.dtype);
    const int64_t tail = (int64_t)(c.max_seq - x->n) * c.head_dim;
    for (int l = 0; l < c.n_layers; ++l)
        for (int w = 0; w < 2; ++w) {
            if (w == 1 && x->L.nb32 > 0) {
                HIP_TRY(launch_vt_poison(kv_base(x, l, 1), c.n_kv_heads, x->L.nb32, c.head_dim, x->n, x->stream));
                continue;
            }
            for (int g = 0; g < c.n_kv_heads; ++g) {
                char *p = kv_base(x, l, w) + ((uint64_t)g * c.max_seq + x->n) * c.head_dim * eb;
                HIP_TRY(launch_fill_nan(c.dtype, p, tail, x->stream));
            }
        }
    HIP_TRY(hipStreamSynchronize(x->stream));
    return SWIFT_OK;
}

extern "C" int swift_debug_read_logits(swift_ctx *x, int row, float *out) {
    if (!x || !out || row < 0 || row >= kMaxBlockRows) return fail(SWIFT_EINVAL, "bad argument");
    HIP_TRY(hipMemcpyAsync(out, dptr<float>(x, x->L.logits) + (size_t)row * x->c.vocab, (size_t)x->c.vocab * 4,
                           hipMemcpyDeviceToHost, x->stream));
    HIP_TRY(hipStreamSynchronize(x->stream));
    return SWIFT_OK;
}

extern "C" int swift_debug_read_kv(swift_ctx *x, int layer, int pos, float *k_out, float *v_out) {
    if (!x || !k_out || !v_out || layer < 0 || layer >= x->c.n_layers || pos < 0 || pos >= x->c.max_seq)
        return fail(SWIFT_EINVAL, "bad argument");
    const swift_model_config &c = x->c;
    const uint64_t eb = elem_bytes(c.dtype);
    // stage through the attention output buffer (fp32, >= n_q*d elements, idle between passes)
    float *tmp = dptr<float>(x, x->L.att);
    for (int w = 0; w < 2; ++w) {
        if (w == 1 && x->L.nb32 > 0) {
            HIP_TRY(launch_vt_read(kv_base(x, layer, 1), c.n_kv_heads, x->L.nb32, c.head_dim, pos, tmp, x->stream));
        } else {
            for (int g = 0; g < c.n_kv_heads; ++g) {
                const char *src = kv_base(x, layer, w) + ((uint64_t)g * c.max_seq + pos) * c.head_dim * eb;
                HIP_TRY(launch_to_f32(c.dtype, src, tmp + (size_t)g * c.head_dim, c.head_dim, x->stream));
            }
        }
        HIP_TRY(hipMemcpyAsync(w == 0 ? k_out : v_out, tmp, (size_t)c.n_kv_heads * c.head_dim * 4, hipMemcpyDeviceToHost,
                               x->stream));
        HIP_TRY(hipStreamSynchronize(x->stream));
    }
    return SWIFT_OK;
}

extern "C" int swift_debug_attn_path(swift_ctx *x, int rows, int tree, char *out, int capacity) {
    if (!x || !out || capacity < 1 || rows < 1 || rows > kMaxBlockRows || (tree && rows > kMaxRows))
        return fail(SWIFT_EINVAL, "bad argument");
    const swift_model_config &c = x->c;
    AttnArgs a{};
    a.n_ctx = x->n + 1;
    a.rows = rows;
    a.max_seq = c.max_seq;
    a.head_dim = c.head_dim;
    a.n_q_heads = c.n_q_heads;
    a.n_kv_heads = c.n_kv_heads;
    a.max_split = x->L.n_split_max;
    a.tree = tree ? 1 : 0;
    a.n_base = x->n;
    a.nb32 = x->L.nb32;
    if (tree)  // (a chain of `rows` levels: the deepest tree of that many rows)
        for (int r = 0; r < rows; ++r) a.tt.depth[r] = a.tt.spine[r] = (uint8_t)r;
    if (x->L.tiled && attn_block_applies(c.dtype, a))
        snprintf(out, (size_t)capacity, "block<bf16, d %d>", c.head_dim);
    else if (x->L.mfma_attn)
        attn_mfma_path_name(a, x->n_cu, out, capacity);
    else
        attn_path_name(c.dtype, a, x->n_cu, out, capacity);
    return SWIFT_OK;
}

extern "C" int swift_debug_tune(swift_ctx *x, int kernel_class, int waves_per_row_group, int workgroups) {
    if (!x || kernel_class < 0 || kernel_class >= SWIFT_KC_COUNT) return fail(SWIFT_EINVAL, "bad argument");
    if (!(waves_per_row_group == 0 || waves_per_row_group == 1 || waves_per_row_group == 2 ||
          waves_per_row_group == 4 || waves_per_row_group == 8 || waves_per_row_group == 16) || workgroups < 0 ||
        workgroups > 65535)
        return fail(SWIFT_EINVAL, "bad argument");
    x->tune_ks[kernel_class] = waves_per_row_group;
    x->tune_wg[kernel_class] = workgroups;
    return SWIFT_OK;
}

extern "C" int swift_debug_prefill(swift_ctx *x, int sub_blocks, int tiling) {
    if (!x || sub_blocks < -1 || sub_blocks > kMacroSub || tiling < 0 || tiling > 6)
        return fail(SWIFT_EINVAL, "bad argument");
    x->prefill_sub = sub_blocks;
    x->gemm_rgw = tiling;
    return SWIFT_OK;
}

extern "C" int swift_profile_class(swift_ctx *x, int kernel_class) {
    if (!x || kernel_class < -1 || kernel_class >= SWIFT_KC_COUNT) return fail(SWIFT_EINVAL, "bad argument");
    x->prof_class = kernel_class;
    return SWIFT_OK;
}

extern "C" int swift_profile_read(swift_ctx *x, int64_t *launches, double *total_ms, uint64_t *total_bytes) {
    if (!x || !launches || !total_ms || !total_bytes) return fail(SWIFT_EINVAL, "null argument");
    HIP_TRY(hipStreamSynchronize(x->stream));
    double ms = 0.0;
    uint64_t bytes = 0;
    for (auto &r : x->prof) {
        float t = 0.f;
        HIP_TRY(hipEventElapsedTime(&t, r.a, r.b));
        ms += t;
        bytes += r.bytes;
        x->pool.push_back(r.a);
        x->pool.push_back(r.b);
    }
    *launches = (int64_t)x->prof.size();
    *total_ms = ms;
    *total_bytes = bytes;
    x->prof.clear();
    return SWIFT_OK;
}
