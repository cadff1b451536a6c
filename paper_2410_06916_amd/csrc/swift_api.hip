// C-ABI layer: context, arena layout, weight loading, and the sequencing of kernel
// launches for prefill / draft / verify / accept (declared in include/swift.h).
#include "../../include/swift.h"

#include <hip/hip_runtime.h>

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
    uint64_t x, q, att, h, logits, part_o, part_ml, out_tok, out_conf;
    uint64_t total;
    int n_split_max;
};

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
    L.embed = take(V * H * eb);
    L.lm_head = take(V * H * eb);
    L.final_norm = take(H * 4);
    L.layers.resize(c.n_layers);
    for (auto &y : L.layers) {
        y.attn_norm = take(H * 4);
        y.wqkv = take((Q + 2 * KV) * H * eb);
        y.wo = take(H * Q * eb);
        y.mlp_norm = take(H * 4);
        y.wgu = take(2 * F * H * eb);
        y.wd = take(H * F * eb);
    }
    L.cos = take((uint64_t)c.max_seq * (c.head_dim / 2) * 4);
    L.sin = take((uint64_t)c.max_seq * (c.head_dim / 2) * 4);
    L.kv = take((uint64_t)c.n_layers * 2 * KV * c.max_seq * eb);
    L.n_split_max = (c.max_seq + kAttnChunk - 1) / kAttnChunk;
    L.x = take(kMaxRows * H * 4);
    L.q = take(kMaxRows * Q * 4);
    L.att = take(kMaxRows * Q * 4);
    L.h = take(kMaxRows * F * 4);
    L.logits = take(kMaxRows * V * 4);
    L.part_o = take((uint64_t)kMaxRows * c.n_q_heads * L.n_split_max * c.head_dim * 4);
    L.part_ml = take((uint64_t)kMaxRows * c.n_q_heads * L.n_split_max * 2 * 4);
    L.out_tok = take(kMaxRows * 4);
    L.out_conf = take(kMaxRows * 4);
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
// context
// ------------------------------------------------------------------------------------------
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
    swift_stats st;
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

template <typename F>
hipError_t timed(swift_ctx *x, int kc, uint64_t bytes, F &&f) {
    if (x->prof_class != kc) return f();
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
    hipError_t r = hipEventRecord(ev[0], x->stream);
    if (r != hipSuccess) return r;
    r = f();
    if (r != hipSuccess) return r;
    r = hipEventRecord(ev[1], x->stream);
    x->prof.push_back({ev[0], ev[1], bytes});
    return r;
}

char *kv_base(swift_ctx *x, int layer, int which) {
    const uint64_t eb = elem_bytes(x->c.dtype);
    const uint64_t per = (uint64_t)x->c.n_kv_heads * x->c.max_seq * x->c.head_dim * eb;
    return x->base + x->L.kv + ((uint64_t)layer * 2 + which) * per;
}

// One token through the network at position `pos`; row = which row of the activation /
// logits buffers to use.  skip == nullptr: full model.  want_logits: run the LM head and
// the arg-max for this row.
int forward_row(swift_ctx *x, int32_t token, int pos, const uint8_t *skip, int row, bool want_logits) {
    const swift_model_config &c = x->c;
    const int H = c.hidden, d = c.head_dim, Q = c.n_q_heads * d, KV = c.n_kv_heads * d, F = c.ffn, V = c.vocab;
    const uint64_t eb = elem_bytes(c.dtype);
    hipStream_t s = x->stream;
    float *xr = dptr<float>(x, x->L.x) + (size_t)row * H;
    float *qr = dptr<float>(x, x->L.q) + (size_t)row * Q;
    float *ar = dptr<float>(x, x->L.att) + (size_t)row * Q;
    float *hr = dptr<float>(x, x->L.h) + (size_t)row * F;
    float *lr = dptr<float>(x, x->L.logits) + (size_t)row * V;

    EmbedArgs ea{x->base + x->L.embed, H, token, xr};
    HIP_TRY(timed(x, SWIFT_KC_OTHER, H * eb, [&] { return launch_embed(c.dtype, ea, s); }));

    for (int l = 0; l < c.n_layers; ++l) {
        const LayerOff &y = x->L.layers[l];
        if (!(skip && skip[2 * l])) {
            GemvArgs g{};
            g.W = x->base + y.wqkv;
            g.O = Q + 2 * KV;
            g.K = H;
            g.xin = xr;
            g.gain = dptr<float>(x, y.attn_norm);
            g.eps = c.rms_eps;
            g.out = qr;
            g.kcache = kv_base(x, l, 0);
            g.vcache = kv_base(x, l, 1);
            g.cos_row = dptr<float>(x, x->L.cos) + (size_t)pos * (d / 2);
            g.sin_row = dptr<float>(x, x->L.sin) + (size_t)pos * (d / 2);
            g.pos = pos;
            g.max_seq = c.max_seq;
            g.head_dim = d;
            g.n_q_heads = c.n_q_heads;
            g.n_kv_heads = c.n_kv_heads;
            HIP_TRY(timed(x, SWIFT_KC_QKV, (uint64_t)g.O * g.K * eb,
                          [&] { return launch_gemv(c.dtype, EPI_QKV, g, x->n_cu, s); }));

            AttnArgs a{};
            a.q = qr;
            a.kcache = kv_base(x, l, 0);
            a.vcache = kv_base(x, l, 1);
            a.n_ctx = pos + 1;
            a.max_seq = c.max_seq;
            a.head_dim = d;
            a.n_q_heads = c.n_q_heads;
            a.n_kv_heads = c.n_kv_heads;
            a.part_o = dptr<float>(x, x->L.part_o);
            a.part_ml = dptr<float>(x, x->L.part_ml);
            a.out = ar;
            HIP_TRY(timed(x, SWIFT_KC_ATTN, (uint64_t)2 * KV * eb * (pos + 1),
                          [&] { return launch_attn_decode(c.dtype, a, s); }));

            GemvArgs o{};
            o.W = x->base + y.wo;
            o.O = H;
            o.K = Q;
            o.xin = ar;
            o.gain = nullptr;
            o.out = xr;
            o.head_dim = d;
            HIP_TRY(timed(x, SWIFT_KC_OPROJ, (uint64_t)o.O * o.K * eb,
                          [&] { return launch_gemv(c.dtype, EPI_RESID, o, x->n_cu, s); }));
        }
        if (!(skip && skip[2 * l + 1])) {
            GemvArgs g{};
            g.W = x->base + y.wgu;
            g.O = 2 * F;
            g.K = H;
            g.xin = xr;
            g.gain = dptr<float>(x, y.mlp_norm);
            g.eps = c.rms_eps;
            g.out = hr;
            g.head_dim = d;
            HIP_TRY(timed(x, SWIFT_KC_GATEUP, (uint64_t)g.O * g.K * eb,
                          [&] { return launch_gemv(c.dtype, EPI_SWIGLU, g, x->n_cu, s); }));
            GemvArgs w{};
            w.W = x->base + y.wd;
            w.O = H;
            w.K = F;
            w.xin = hr;
            w.gain = nullptr;
            w.out = xr;
            w.head_dim = d;
            HIP_TRY(timed(x, SWIFT_KC_DOWN, (uint64_t)w.O * w.K * eb,
                          [&] { return launch_gemv(c.dtype, EPI_RESID, w, x->n_cu, s); }));
        }
    }
    if (want_logits) {
        GemvArgs g{};
        g.W = x->base + x->L.lm_head;
        g.O = V;
        g.K = H;
        g.xin = xr;
        g.gain = dptr<float>(x, x->L.final_norm);
        g.eps = c.rms_eps;
        g.out = lr;
        g.head_dim = d;
        HIP_TRY(timed(x, SWIFT_KC_LMHEAD, (uint64_t)g.O * g.K * eb,
                      [&] { return launch_gemv(c.dtype, EPI_LOGITS, g, x->n_cu, s); }));
        ArgmaxArgs m{lr, V, 1, dptr<int32_t>(x, x->L.out_tok) + row, dptr<float>(x, x->L.out_conf) + row};
        HIP_TRY(timed(x, SWIFT_KC_OTHER, (uint64_t)V * 4, [&] { return launch_argmax_conf(m, s); }));
    }
    return SWIFT_OK;
}

// Copies rows [0, rows) of the token / confidence results to the pinned staging area and waits.
int read_results(swift_ctx *x, int rows) {
    HIP_TRY(hipMemcpyAsync(x->h_tok, dptr<int32_t>(x, x->L.out_tok), rows * 4, hipMemcpyDeviceToHost, x->stream));
    HIP_TRY(hipMemcpyAsync(x->h_conf, dptr<float>(x, x->L.out_conf), rows * 4, hipMemcpyDeviceToHost, x->stream));
    HIP_TRY(hipStreamSynchronize(x->stream));
    return SWIFT_OK;
}

// tensor slot index for a name, plus where and how it is stored
struct Slot {
    int index;
    uint64_t off;       // destination offset in the arena
    int64_t n;          // expected element count
    bool is_gain;
    int rows, cols;     // matrix shape [rows][cols] as given by the caller
    uint64_t dst_pitch; // bytes between consecutive destination rows (0 = contiguous)
};

bool find_slot(swift_ctx *x, const char *name, Slot *out) {
    const swift_model_config &c = x->c;
    const uint64_t eb = elem_bytes(c.dtype);
    const int H = c.hidden, Q = c.n_q_heads * c.head_dim, KV = c.n_kv_heads * c.head_dim, F = c.ffn, V = c.vocab;
    auto mat = [&](int idx, uint64_t off, int r, int k, uint64_t pitch = 0) {
        *out = Slot{idx, off, (int64_t)r * k, false, r, k, pitch};
        return true;
    };
    auto gain = [&](int idx, uint64_t off) {
        *out = Slot{idx, off, H, true, 1, H, 0};
        return true;
    };
    if (!strcmp(name, "embed")) return mat(0, x->L.embed, V, H);
    if (!strcmp(name, "lm_head")) return mat(1, x->L.lm_head, V, H);
    if (!strcmp(name, "final_norm")) return gain(2, x->L.final_norm);
    if (name[0] != 'l') return false;
    char *end;
    long l = strtol(name + 1, &end, 10);
    if (end == name + 1 || *end != '.' || l < 0 || l >= c.n_layers) return false;
    const char *f = end + 1;
    const LayerOff &y = x->L.layers[l];
    const int b = 3 + 9 * (int)l;
    if (!strcmp(f, "attn_norm")) return gain(b + 0, y.attn_norm);
    if (!strcmp(f, "wq")) return mat(b + 1, y.wqkv, Q, H);
    if (!strcmp(f, "wk")) return mat(b + 2, y.wqkv + (uint64_t)Q * H * eb, KV, H);
    if (!strcmp(f, "wv")) return mat(b + 3, y.wqkv + (uint64_t)(Q + KV) * H * eb, KV, H);
    if (!strcmp(f, "wo")) return mat(b + 4, y.wo, H, Q);
    if (!strcmp(f, "mlp_norm")) return gain(b + 5, y.mlp_norm);
    // gate and up rows are interleaved: row 2f = gate f, row 2f+1 = up f
    if (!strcmp(f, "wg")) return mat(b + 6, y.wgu, F, H, 2 * (uint64_t)H * eb);
    if (!strcmp(f, "wu")) return mat(b + 7, y.wgu + (uint64_t)H * eb, F, H, 2 * (uint64_t)H * eb);
    if (!strcmp(f, "wd")) return mat(b + 8, y.wd, H, F);
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
    memset(&x->st, 0, sizeof(x->st));
    x->prof_class = -1;
    x->h_tok = nullptr;
    x->h_conf = nullptr;
    hipError_t e = hipHostMalloc((void **)&x->h_tok, 2 * kMaxRows * 4, hipHostMallocDefault);
    if (e != hipSuccess) {
        delete x;
        return fail(SWIFT_EDEVICE, std::string("hipHostMalloc: ") + hipGetErrorString(e));
    }
    x->h_conf = (float *)(x->h_tok + kMaxRows);

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
    e = hipMemcpyAsync(x->base + L.cos, ct.data(), ct.size() * 4, hipMemcpyHostToDevice, x->stream);
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
    if (sl.dst_pitch == 0) {
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
    for (int i = 0; i < n_prompt; ++i) {
        int rc = forward_row(x, prompt[i], i, nullptr, 0, i == n_prompt - 1);
        if (rc) return rc;
    }
    int rc = read_results(x, 1);
    if (rc) return rc;
    x->n = n_prompt;
    x->pending = x->h_tok[0];
    x->k_verify = -1;
    memset(&x->st, 0, sizeof(x->st));
    x->st.emitted_total = 1;
    *first_token = x->pending;
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
    for (int j = 1; j <= max_k; ++j) {
        int rc = forward_row(x, prev, x->n + j - 1, skip_mask, 0, true);
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

extern "C" int swift_verify(swift_ctx *x, const int32_t *tokens, int k, int32_t *target_tokens, float *logits_out) {
    if (!x || !tokens || !target_tokens) return fail(SWIFT_EINVAL, "null argument");
    if (k < 0 || k > SWIFT_MAX_BLOCK - 1) return fail(SWIFT_EINVAL, "k out of range");
    if (x->pending < 0) return fail(SWIFT_ESTATE, "verify before prefill");
    if (tokens[0] != x->pending) return fail(SWIFT_EINVAL, "tokens[0] must be the pending token");
    for (int i = 0; i <= k; ++i)
        if (tokens[i] < 0 || tokens[i] >= x->c.vocab) return fail(SWIFT_EINVAL, "token id out of range");
    if (x->n + k + 1 > x->c.max_seq) return fail(SWIFT_ECAPACITY, "block would run past the cache capacity");
    for (int i = 0; i <= k; ++i) {
        int rc = forward_row(x, tokens[i], x->n + i, nullptr, i, true);
        if (rc) return rc;
    }
    int rc = read_results(x, k + 1);
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
    x->st.verify_passes++;
    return SWIFT_OK;
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

extern "C" int swift_rollback(swift_ctx *x, int new_cache_len, int32_t pending_token) {
    if (!x) return fail(SWIFT_EINVAL, "null context");
    if (x->pending < 0) return fail(SWIFT_ESTATE, "rollback before prefill");
    if (new_cache_len < 0 || new_cache_len > x->n) return fail(SWIFT_EINVAL, "new length must be in [0, cache length]");
    if (pending_token < 0 || pending_token >= x->c.vocab) return fail(SWIFT_EINVAL, "token id out of range");
    x->n = new_cache_len;
    x->pending = pending_token;
    x->k_verify = -1;
    return SWIFT_OK;
}

extern "C" int swift_get_state(swift_ctx *x, int *cache_len, int32_t *pending_token) {
    if (!x) return fail(SWIFT_EINVAL, "null context");
    if (cache_len) *cache_len = x->n;
    if (pending_token) *pending_token = x->pending;
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
        for (int w = 0; w < 2; ++w)
            for (int g = 0; g < c.n_kv_heads; ++g) {
                char *p = kv_base(x, l, w) + ((uint64_t)g * c.max_seq + x->n) * c.head_dim * eb;
                HIP_TRY(launch_fill_nan(c.dtype, p, tail, x->stream));
            }
    HIP_TRY(hipStreamSynchronize(x->stream));
    return SWIFT_OK;
}

extern "C" int swift_debug_read_logits(swift_ctx *x, int row, float *out) {
    if (!x || !out || row < 0 || row >= kMaxRows) return fail(SWIFT_EINVAL, "bad argument");
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
        for (int g = 0; g < c.n_kv_heads; ++g) {
            const char *src = kv_base(x, layer, w) + ((uint64_t)g * c.max_seq + pos) * c.head_dim * eb;
            HIP_TRY(launch_to_f32(c.dtype, src, tmp + (size_t)g * c.head_dim, c.head_dim, x->stream));
        }
        HIP_TRY(hipMemcpyAsync(w == 0 ? k_out : v_out, tmp, (size_t)c.n_kv_heads * c.head_dim * 4, hipMemcpyDeviceToHost,
                               x->stream));
        HIP_TRY(hipStreamSynchronize(x->stream));
    }
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
