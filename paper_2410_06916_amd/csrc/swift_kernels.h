// Launch interface between the C-ABI layer (swift_api.hip) and the gfx950 kernels
// (swift_kernels.hip).  Plain structs and functions; every launcher enqueues on the
// given stream and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swift {

constexpr int kMaxRows = 16;       // rows of one block pass (SWIFT_MAX_BLOCK)
constexpr int kAttnChunk = 128;    // cache slots handled by one attention workgroup
constexpr int kGemvThreads = 256;  // 4 wavefronts of 64

enum Dtype : int { F32 = 0, BF16 = 1 };

// Which computation precedes / follows the row dot products of a weight-streaming pass.
enum Epilogue : int {
    EPI_QKV = 0,     // rotate q,k at `pos`; q -> out (fp32); k,v -> cache slot `pos`
    EPI_RESID = 1,   // out[o] += y[o]                       (o_proj, down_proj)
    EPI_SWIGLU = 2,  // out[f] = silu(y[2f]) * y[2f+1]        (gate/up rows interleaved)
    EPI_LOGITS = 3,  // out[o] = y[o]                         (LM head)
};

struct GemvArgs {
    const void *W;      // [O][K] in the model's storage dtype, row-major
    int O, K;
    const float *xin;   // [K] fp32
    const float *gain;  // [K] fp32 RMSNorm gain, or nullptr: no normalisation
    float eps;
    float *out;
    // EPI_QKV only
    void *kcache, *vcache;        // this layer's [n_kv][max_seq][d]
    const float *cos_row, *sin_row;  // rotary table rows for `pos`: [d/2] each
    int pos, max_seq, head_dim, n_q_heads, n_kv_heads;
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
    const float *q;               // [n_q][d] fp32 (already rotated)
    const void *kcache, *vcache;  // this layer's [n_kv][max_seq][d]
    int n_ctx;                    // slots [0, n_ctx) are attended
    int max_seq, head_dim, n_q_heads, n_kv_heads;
    float *part_o;                // [n_q][n_split][d]   unnormalised partial outputs
    float *part_ml;               // [n_q][n_split][2]   running max, running sum
    float *out;                   // [n_q][d]
};
hipError_t launch_attn_decode(int dtype, const AttnArgs &a, hipStream_t s);

struct ArgmaxArgs {
    const float *logits;  // [rows][V]
    int V, rows;
    int32_t *tokens;      // [rows]
    float *conf;          // [rows]
};
hipError_t launch_argmax_conf(const ArgmaxArgs &a, hipStream_t s);

hipError_t launch_fill_nan(int dtype, void *p, int64_t n_elems, hipStream_t s);

// dst[i] (fp32) = src[i] (dtype)
hipError_t launch_to_f32(int dtype, const void *src, float *dst, int64_t n, hipStream_t s);

// ---- tiled bf16 weights -------------------------------------------------------------------
// A bf16 matrix [O][K] is stored as 1 KB tiles of 16 rows x 32 k, tile (rg, t) at element offset
// ((rg * T) + t) * 512 with T = ceil(K/32); inside a tile lane l of a wavefront owns the 8
// consecutive k values 32t + 8(l>>4) .. +7 of tile row (l & 15), i.e. exactly the A operand of
// v_mfma_f32_16x16x32_bf16, so one 128-bit load per lane feeds one MFMA.  Rows beyond O and k
// beyond K are zero.  Which matrix row sits in tile row j of row group rg depends on the mode:
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

// One activation row against a tiled matrix (MFMA, fp32 activation split into three bf16 terms).
struct MvArgs {
    const void *Wt;
    int O, K, T, n_rg;
    const float *xin;   // [K] fp32
    const float *gain;  // [K] fp32 or nullptr
    float eps;
    float *out;
    void *kcache, *vcache;
    const float *cos_row, *sin_row;
    int pos, max_seq, head_dim, n_q_heads, n_kv_heads;
    int S;              // row-group rounds per workgroup (set by the launcher)
};
// LDS bytes the kernel needs for a K-wide activation; the launcher refuses more than kMvMaxLds.
constexpr size_t kMvMaxLds = 150 * 1024;
inline size_t mv_lds_bytes(int K) { return (size_t)((K + 31) / 32) * 192 + 1024 + 16 + 512; }
// ks_override / wg_override: 0 = choose automatically.
hipError_t launch_mv1(int epilogue, MvArgs a, int n_cu, int ks_override, int wg_override, hipStream_t s);

}  // namespace swift
