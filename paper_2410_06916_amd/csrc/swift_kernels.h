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

}  // namespace swift
