// Launch interface between the C-ABI layer (swift_api.hip) and the gfx950 kernels
// (swift_kernels.hip: storage-generic single-row path; swift_tiled.hip: bf16 tiled MFMA path).
// Plain structs and functions; every launcher enqueues on the given stream and returns the
// hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swift {

constexpr int kMaxRows = 32;       // rows of one verify block or token tree (SWIFT_MAX_BLOCK)
constexpr int kMaxBlockRows = 64;  // rows of one prefill block
// How the split activations of a block are laid out: a code that holds the rows the layout is pitched for and
// how many bf16 terms an fp32 activation is split into.
//  * exact layouts (draft, verify and tree blocks of up to kMaxRows rows; any block of up to 16 rows): pitched for
//    the block's own row count, three terms (hi + mid + lo is the value exactly) and one fixed summation order,
//    so that a row's result does not depend on the rows it shares a pass with;
//  * bulk layouts (prefill blocks and candidate evaluation windows of more than 16 rows): pitched for 32 or 64
//    rows, the first two terms only (relative error 2^-17 per element): a third less to stage, read and
//    multiply, and no promise about the order.
// Term t of row r is column terms * r + t.
constexpr int kBulkLayout = 0x100;
__host__ __device__ inline int layout_rows(int RL) { return RL & 0xff; }
__host__ __device__ inline int block_terms(int RL) { return (RL & kBulkLayout) ? 2 : 3; }
inline int block_row_layout(int R, bool exact) { return (exact || R <= 16) ? R : ((R <= 32 ? 32 : kMaxBlockRows) | kBulkLayout); }
// Row pitch of the per-row-group partial sums of squares (pss): 16 for blocks of up to 16 rows, else 64.
inline int block_row_pitch(int R) { return R <= 16 ? 16 : kMaxBlockRows; }
// The rows of a token tree (block rows 0 .. rows-1): level of each row; block row of the first candidate of each
// level (the only one with children; spine[0] = 0, the block's first row).
struct TreeTab {
    uint8_t depth[kMaxRows], spine[kMaxRows];
};
constexpr int kAttnMaxSplit = 64;  // most cache-length splits of one (row, kv head)
constexpr int kGemvThreads = 256;  // 4 wavefronts of 64

enum Dtype : int { F32 = 0, BF16 = 1 };

// Which computation follows the row dot products of a weight-streaming pass.
enum Epilogue : int {
    EPI_QKV = 0,     // rotate q,k at the row's position; q -> fp32 buffer; k,v -> cache slot
    EPI_RESID = 1,   // x += y                                (o_proj, down_proj)
    EPI_SWIGLU = 2,  // h = silu(gate) * up
    EPI_LOGITS = 3,  // logits = y                            (LM head)
};

// ------------------------------------------------------------------------------------------
// storage-generic path (fp32 or bf16 row-major weights, one activation row)
// ------------------------------------------------------------------------------------------
struct GemvArgs {
    const void *W;      // [O][K] in the model's storage dtype, row-major
    int O, K;
    const float *xin;   // [K] fp32
    const float *gain;  // [K] fp32 RMSNorm gain, or nullptr: no normalisation
    float eps;
    float *out;
    // EPI_QKV only
    void *kcache, *vcache;           // this layer's [n_kv][max_seq][d]
    const float *cos_row, *sin_row;  // rotary table rows for `pos`: [d/2] each
    int pos, max_seq, head_dim, n_q_heads, n_kv_heads;  // pos: the cache slot the keys/values go to
};
hipError_t launch_gemv(int dtype, int epilogue, const GemvArgs &a, int n_cu, hipStream_t s);

struct EmbedArgs {
    const void *E;  // [V][H]
    int H;
    int32_t token;
    float *x;  // [H]
};
hipError_t launch_embed(int dtype, const EmbedArgs &a, hipStream_t s);

struct AttnArgs {
    const float *q;               // [rows][n_q][d] fp32 (already rotated)
    const void *kcache, *vcache;  // this layer's [n_kv][max_seq][d]
    int n_ctx;                    // row r attends slots [0, n_ctx + r)
    int rows;
    int max_seq, head_dim, n_q_heads, n_kv_heads;
    float *part_o;                // [rows][n_q][n_split][d]   unnormalised partial outputs
    float *part_ml;               // [rows][n_q][n_split][2]   running max, running sum
    int max_split;                // splits the partial buffers can hold
    float *out;                   // fp32 [rows][n_q][d], or nullptr
    uint16_t *out_s;              // bf16 term split [n_q*d/8][terms * layout rows][8], or nullptr
    int out_rows;                 // layout code (block_row_layout) of the block out_s belongs to (0: an exact layout
                                  // of `rows` rows); a launch may cover a part of a larger block: out_s then points
                                  // at its first column
    // Token tree instead of a chain (tree != 0; at most kMaxRows block rows).  Launch row r is block row
    // row_base + r and sits at level tt.depth[row] of the tree; the block's keys/values sit in slots
    // n_base + block row.  The row attends, in this order, the committed slots [0, n_base), then for level
    // i = 0 .. depth-1 the slot of block row tt.spine[i], then its own slot: the same sequence of keys/values, batched
    // the same way, as a chain row at position n_base + depth, so the result is the chain's bit for bit.
    int tree, n_base, row_base;
    TreeTab tt;
    // Matrix-core attention (bf16 cache, heads of 64 or 128; attn_mfma_applies): the values are stored in
    // groups of eight slots (see kv_vt_index), nb32 chunks of 32 slots per kv head.
    int nb32;
    const uint16_t *q_s;          // matrix-core attention: the query rows as two bf16 terms, [rows][n_q][2][d]
    // Prompt macro block (block attention kernel only): the rows come in sub-blocks of sub_rows rows (0: one block),
    // sub-block z with buffers of its own at q + z * sub_q and out_s + z * sub_out_s (elements); row r of the macro
    // block is row r % sub_rows of sub-block r / sub_rows and attends n_ctx + r slots as in any chain block.
    int sub_rows;
    int64_t sub_q, sub_out_s;
};
// ------------------------------------------------------------------------------------------
// key/value cache layouts
// ------------------------------------------------------------------------------------------
// Keys: [kv head][slot][d].  Values: the same, except for bf16 caches with heads of 64 or 128, whose
// attention runs on the matrix cores and wants eight consecutive slots of one value element in one 16-byte
// load: there the values are stored in groups of eight slots, [kv head][slot / 8][element][slot % 8], with
// 4 * nb32 groups per head (nb32 = ceil(max_seq / 32): whole 32-slot chunks).  A token's values then land 16
// bytes apart inside one 16 * d byte region, and the 32 slots of a chunk are one contiguous 64 * d bytes.
inline bool attn_mfma_applies(int dtype, int head_dim) { return dtype == 1 /* BF16 */ && (head_dim == 64 || head_dim == 128); }
__host__ __device__ inline size_t kv_vt_index(int kv_head, int nb32, int d, int slot, int elem) {
    return (((size_t)kv_head * nb32 * 4 + (slot >> 3)) * d + elem) * 8 + (slot & 7);
}
// Rows one launch of the matrix-core attention kernel takes (two tiles of 16 members for one kv head per
// workgroup; more members go to further workgroups)
constexpr int kAttnMfmaMaxRows = 32;
hipError_t launch_attn_mfma(const AttnArgs &a, int n_cu, hipStream_t s);
int attn_mfma_path_name(const AttnArgs &a, int n_cu, char *out, int capacity);
size_t attn_mfma_partial_floats(const AttnArgs &a, int n_cu);
// True when the attention of a block runs on the one-workgroup-per-(kv head, row) kernel (no partial
// buffers: one launch may then cover any number of rows); false: the split kernel, at most kMaxRows
// rows per launch.  Depends on the cache capacity and the head count only.
inline bool attn_uses_head_kernel(int max_seq, int n_kv_heads) { return max_seq <= 1600 && n_kv_heads >= 24; }
hipError_t launch_attn_decode(int dtype, const AttnArgs &a, int n_cu, hipStream_t s);
// Writes the name of the kernel instance launch_attn_decode would take for `a` (e.g. "split<bf16, group 1,
// rows 3>") into out; returns the length snprintf reports.  Host only.
int attn_path_name(int dtype, const AttnArgs &a, int n_cu, char *out, int capacity);
// Floats of part_o the attention launches of a block described by `a` may write at any cache length up to
// max_seq (part_ml: 2 floats per head_dim floats of part_o); 0: the kernel keeps everything on chip.
size_t attn_partial_floats(int dtype, const AttnArgs &a, int n_cu);
// Merges the partial results of n_split cache ranges of `chunk` slots, per (row, query head), in range order.
hipError_t launch_attn_combine(const AttnArgs &a, int chunk, int n_split, hipStream_t s);
// Blocks of 17..64 chain rows over a bf16 cache with head_dim 64 or 128: the whole block in one launch on the
// matrix cores (all rows share every key/value load).  `a` describes the whole block (rows, out_rows), or a prompt
// macro block of up to kMacroSub such blocks (sub_rows = 64).
bool attn_block_applies(int dtype, const AttnArgs &a);
hipError_t launch_attn_block(const AttnArgs &a, int n_cu, hipStream_t s);

constexpr int kTopK = 10;  // candidates kept per row (SWIFT_TOPK)
struct ArgmaxArgs {
    const float *logits;  // [rows][V]
    int V, rows;
    int32_t *tokens;      // [rows]
    float *conf;          // [rows]
    int32_t *topk;        // nullptr, or [rows][kTopK]: the n_topk largest logits' indices, largest first,
    int n_topk;           //   equal values in index order (topk[0] is the arg-max)
};
hipError_t launch_argmax_conf(const ArgmaxArgs &a, hipStream_t s);

// ------------------------------------------------------------------------------------------
// speculative sampling
// ------------------------------------------------------------------------------------------
// probs[r] = softmax(logits[r] / temperature) restricted to its nucleus (top_p) and renormalised
struct WarpArgs {
    const float *logits;  // [rows][ld_logits]
    int ld_logits, V, rows;
    float temperature, top_p;
    float *probs;         // [rows][V]
};
hipError_t launch_warp(const WarpArgs &a, hipStream_t s);
// out[0] = the first token j with probs[0] + .. + probs[j] > u * (sum of probs), 0 <= u < 1
hipError_t launch_draw(const float *probs, int V, float u, int32_t *out, hipStream_t s);
// Keep / replace rule over a verified block of k draft tokens x[i] drawn from q[i] (rows of [.][V]), target
// distributions p[0..k]: out[0] = number of tokens kept, out[1] = the token that follows them.
struct SpecAcceptArgs {
    const float *p, *q;
    int V, k;
    int32_t x[kMaxRows];
    float u_accept[kMaxRows];
    float u_final;
    int32_t *out;
};
hipError_t launch_spec_accept(const SpecAcceptArgs &a, hipStream_t s);

// Copies cache slots src[i] -> dst[i], i = 0 .. n_moves-1 in this order, for every kv head of the key plane and
// the value plane of every layer.  Layer l's keys start at kv + l * layer_elems ([n_kv][max_seq][d]), its values
// v_offset elements later ([n_kv][max_seq][d], or transposed in blocks with nb32 > 0: kv_vt_index).
struct KvMoveArgs {
    void *kv;
    int64_t layer_elems, v_offset;
    int n_layers, n_kv_heads, max_seq, head_dim, nb32;
    int n_moves;
    int src[32], dst[32];
};
hipError_t launch_kv_move(int dtype, const KvMoveArgs &a, hipStream_t s);

hipError_t launch_vt_poison(void *plane, int n_kv, int nb32, int d, int first_slot, hipStream_t s);
hipError_t launch_vt_read(const void *plane, int n_kv, int nb32, int d, int slot, float *dst, hipStream_t s);
hipError_t launch_fill_nan(int dtype, void *p, int64_t n_elems, hipStream_t s);
// p[i] = v for n 32-bit words (a kernel rather than a memset, so that the call may be captured into a graph)
hipError_t launch_fill_u32(void *p, uint32_t v, int64_t n, hipStream_t s);

// dst[i] (fp32) = src[i] (dtype)
hipError_t launch_to_f32(int dtype, const void *src, float *dst, int64_t n, hipStream_t s);

// ------------------------------------------------------------------------------------------
// tiled bf16 path
// ------------------------------------------------------------------------------------------
// Weights.  A bf16 matrix [O][K] is stored as 1 KB tiles of 16 rows x 32 k, tile (rg, t) at
// element offset ((rg * T) + t) * 512 with T = ceil(K/32); inside a tile lane l of a wavefront
// owns the 8 consecutive k values 32t + 8(l>>4) .. +7 of tile row (l & 15), i.e. exactly the A
// operand of v_mfma_f32_16x16x32_bf16, so one 128-bit load per lane feeds one MFMA.  Rows beyond
// O and k beyond K are zero.  Which matrix row sits in tile row j of row group rg:
enum TileMode : int {
    TILE_PLAIN = 0,   // row = 16 rg + j
    TILE_PAIR = 1,    // rotary pairs together: head = rg / (d/16), g = rg % (d/16);
                      //   j < 8: row = head*d + 8g + j ;  j >= 8: row = head*d + d/2 + 8g + (j-8)
    TILE_GATEUP = 2,  // j < 8: gate row 8 rg + j ;  j >= 8: up row 8 rg + (j-8)
};

struct TileArgs {
    const void *src;  // row-major [src_rows][K] bf16 (device)
    int src_rows, K;
    void *dst;        // tiled destination (start of the first row group written)
    int T, n_rg;      // k-tiles per row group, row groups to write
    int mode, head_dim;
    int part;         // TILE_GATEUP: 0 = src holds the gate rows, 1 = the up rows
};
hipError_t launch_tile_weights(const TileArgs &a, hipStream_t s);

// Activations between the tiled kernels.  An fp32 activation vector of R rows (tokens) that
// feeds a projection is kept as three bf16 terms per value (value = hi + mid + lo exactly), laid
// out as the MFMA B operand: [K/8 chunks][NC = 3R columns][8 k] bf16, column 3r + term (bulk
// layouts: the first two terms, NC = 2 x 32 or 2 x 64 columns, column 2r + term; block_terms).  The
// residual stream itself stays fp32 [R][H]; the kernel that updates it also writes the split of
// (x * gain of the next consumer) and, per 16-row group, the partial sums of squares of x, so the
// consumer only adds up the partials (fixed order) to get the RMSNorm scale 1/sqrt(mean x^2 + eps)
// and applies it to its results (W.(x*g) * scale == W.(x*scale*g) up to fp32 rounding).
struct MvArgs {
    const void *Wt;        // tiled weights
    int O, K, T, n_rg;     // real rows / depth, k-tiles, row groups
    int R;                 // activation rows, 1..64
    int RL;                // layout code of the split layouts (in_s, out_s): block_row_layout
                           // (columns of rows that do not exist hold garbage that no result depends on)
    const uint16_t *in_s;  // split input [K/8][3 RL][8]
    const float *pss;      // [n_pss][rp] partial sums of squares of the producer, or nullptr: no norm
    int n_pss, norm_dim;
    int rp;                // row pitch of pss and pss_out: 16 for blocks of up to 16 rows, else 64
    float eps;
    float *out_f32;        // QKV: q [R][ld_out]; LOGITS: logits [R][ld_out]; RESID: x [R][ld_out] (in/out)
    int ld_out;
    uint16_t *out_s;       // SWIGLU: split h [F/8][3 RL][8]; RESID: split of x*gain_next [O/8][3 RL][8]
    const float *gain_next;  // RESID: [O]
    float *pss_out;        // RESID: [n_rg][rp]
    void *kcache, *vcache;   // QKV: this layer's [n_kv][max_seq][d]
    const float *cos_tab, *sin_tab;  // QKV: [max_seq][d/2]
    int pos0, max_seq, head_dim, n_q_heads, n_kv_heads;
    // QKV: row r's keys/values go to slot pos0 + r; it is rotated for position pos0 + r, or, for the rows
    // of a token tree (tree != 0, R <= kMaxRows), for position pos0 + depth[r] (the row's level)
    int tree;
    uint8_t depth[kMaxRows];
    int nb32;              // QKV: > 0: the values go to the grouped layout (kv_vt_index), nb32 32-slot chunks per head
    uint16_t *q_s;         // QKV: nullptr, or [R][n_q][2][d]: the rotated queries once more, as two bf16 terms (hi, then
                           // what is left of the fp32 value after hi), the operand form of the matrix-core attention
    // multi-row kernel only: split-K scratch
    float *part;           // [k splits][row group][R][16] fp32 partial results
    int *counters;         // one per 8-row-group block, zero between launches
    int part_capacity;     // row-group-splits the scratch can hold
    int S;                 // set by the launcher
    int kgroup;            // set by the launcher: K slices whose sums are added first (see mv_slice_group)
    // QKV, LDS-resident kernel only: cache lines to pull into the L2 of the die that will run the attention of
    // kv head g right after this launch (rows [0, pf_rows) of head g's keys and values); pf_heads = 0: none.
    // n_wg: workgroups that do the projection; pf_first, pf_wgs: first warm-up workgroup and how many (all set by
    // the launcher)
    int pf_rows, pf_heads, n_wg, pf_first, pf_wgs;
};
// position block row r of a QKV pass is rotated for
__host__ __device__ inline int mv_rope_pos(const MvArgs &a, int r) {
    return a.pos0 + (a.tree ? (int)a.depth[r & (kMaxRows - 1)] : r);
}
constexpr size_t kMvMaxLds = 150 * 1024;
// Rows the LDS-resident kernel takes (3R term columns must fit one MFMA column block)
constexpr int kMvSmallRows = 5;
// LDS bytes of the LDS-resident kernel for depth K and R rows
inline size_t mv1_lds_bytes(int K, int R, int head_dim) {
    const size_t NC = 3 * (size_t)R;
    return 16 + (size_t)((K + 31) / 32) * 64 * NC + 2 * 8 * 16 * NC * 4 + 64 + 2048 + (size_t)R * head_dim * 4 + 64;
}
// Kernel-precise timing: the next launch_mv on this thread records `start` when its kernel begins
// and `stop` when it ends (timestamps of the dispatch itself, no extra packets on the stream).
void set_launch_events(hipEvent_t start, hipEvent_t stop);
// ks_override / wg_override: 0 = choose automatically (LDS-resident kernel only).
hipError_t launch_mv(int epilogue, MvArgs a, int n_cu, int ks_override, int wg_override, hipStream_t s);
// Row-group-splits of `part` (16 * R floats each) that launch_mv writes for a block of up to 16 rows
// described by `a` (0: the launch splits K inside workgroups only and uses neither `part` nor `counters`).
int mv_split_slots(const MvArgs &a, int n_cu);

// Prompt macro blocks: up to kMacroSub consecutive sub-blocks of 64 rows (the last one may hold fewer) go through a
// projection in one launch.  Each sub-block has buffers of its own, laid out as for a 64-row block in the bulk
// layout; sub-block s is found at the given element strides from sub-block 0's pointers in MvArgs, its rows sit at
// positions pos0 + 64 s ..
constexpr int kMacroSub = 8;
struct MacroArgs {
    int S;          // sub-blocks, 1..kMacroSub
    int rows_last;  // rows of the last one, 1..64 (the others hold 64)
    int64_t in_s, pss, out_f32, out_s, pss_out, q_s;  // strides, in elements of the respective buffer
};
// epilogue: EPI_QKV, EPI_RESID or EPI_SWIGLU; a.R is ignored, a.RL must be the 64-row bulk layout, a.rp = 64, a.K a
// multiple of 8.  tiling_override: 0 = automatic, else the tile shape (tuning runs): 1..4 = that many row groups per
// wavefront on two sub-blocks side by side, 5 / 6 = one / two row groups per wavefront on one sub-block.
hipError_t launch_gemm(int epilogue, const MvArgs &a, const MacroArgs &ma, int n_cu, int tiling_override, hipStream_t s);

// x[r] = E[token r] (fp32), split of x * gain_next, partial sums of squares per 16 elements.
struct EmbedRowsArgs {
    const uint16_t *E;  // [V][H] bf16 row-major
    int H, R;
    int RL;             // layout code of xs: block_row_layout
    int32_t tokens[kMaxBlockRows];
    float *x;           // [R][H]
    uint16_t *xs;       // [H/8][3 RL][8]
    const float *gain_next;
    float *pss;         // [ceil(H/16)][rp]
    int rp;             // row pitch of pss (16 or 64)
};
hipError_t launch_embed_rows(const EmbedRowsArgs &a, hipStream_t s);

}  // namespace swift
