// Speculative sampling on the device (paper Section 5.1 and Appendix B.2: speculative sampling as the
// acceptance rule; temperature and top-p for the sampled runs): the distribution tokens are drawn from,
// inverse-CDF draws from caller-supplied uniforms, and the keep / replace rule over a verified block.
// Every sum below is taken in a fixed order, so a call gives the same token on every run.
#include <math.h>

#include "swift_device.h"
#include "swift_kernels.h"

namespace swift {

namespace {

constexpr int kThreads = 1024;  // one workgroup of 16 wavefronts per row

// Sum over the workgroup, the same value in every thread.  sh: 16 floats; two barriers.
__device__ inline float block_sum(float v, float *sh) {
    v = wave_sum(v);
    __syncthreads();  // earlier readers of sh are done
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) t += sh[w];
    return t;
}
__device__ inline float block_max(float v, float *sh) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = sh[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) t = fmaxf(t, sh[w]);
    return t;
}

// Inverse-CDF draw in token-id order from the non-negative weights w(j), j < V: the first j with
// w(0) + .. + w(j) > u * total.  Thread t owns the contiguous ids [t*C, (t+1)*C); a running sum is the
// thread's base (the chunks before it, added up by a fixed scan) plus the sum of its own ids so far.
// Returns the token (the same in every thread); *total_out = the total.  sh: 16 floats, shi: 16 ints.
template <typename W>
__device__ inline int block_draw(W w, int V, float u, float *sh, int *shi, float *total_out) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int C = (V + kThreads - 1) / kThreads;
    const int j0 = tid * C, j1 = min(V, j0 + C);
    float s = 0.f;
    int last_pos = -1;  // last id of the chunk with a positive weight
    for (int j = j0; j < j1; ++j) {
        const float x = w(j);
        s += x;
        if (x > 0.f) last_pos = j;
    }
    // exclusive scan over the threads: inside the wavefront lane by lane (Hillis-Steele), then the
    // wavefronts' totals in order
    float inc = s;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float o = __shfl_up(inc, off, 64);
        if (lane >= off) inc += o;
    }
    __syncthreads();
    if (lane == 63) sh[wave] = inc;
    __syncthreads();
    float wbase = 0.f, total = 0.f;
#pragma unroll
    for (int k = 0; k < kThreads / 64; ++k) {
        if (k == wave) wbase = total;
        total += sh[k];
    }
    const float base = wbase + (inc - s);
    const float thr = u * total;
    int cand = 0x7fffffff;
    if (base + s > thr) {  // the running sum at the end of the chunk: this chunk holds a candidate
        float local = 0.f;
        for (int j = j0; j < j1; ++j) {
            const float x = w(j);
            local += x;
            if (base + local > thr && x > 0.f) {
                cand = j;
                break;
            }
        }
    }
    // the smallest candidate wins; if rounding left none, the last id with a positive weight
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        cand = min(cand, __shfl_xor(cand, off, 64));
        last_pos = max(last_pos, __shfl_xor(last_pos, off, 64));
    }
    __syncthreads();
    if (lane == 0) {
        shi[wave] = cand;
        shi[16 + wave] = last_pos;
    }
    __syncthreads();
    int best = 0x7fffffff, lastp = -1;
#pragma unroll
    for (int k = 0; k < kThreads / 64; ++k) {
        best = min(best, shi[k]);
        lastp = max(lastp, shi[16 + k]);
    }
    if (total_out) *total_out = total;
    return best != 0x7fffffff ? best : (lastp >= 0 ? lastp : 0);
}

// Workgroup r: probs[r] = softmax(logits[r] / temperature) cut to its nucleus and renormalised.
// Nucleus: every token whose probability is at least t*, the largest probability value t for which the
// tokens with probability >= t together reach top_p (so tokens as probable as the last one needed all
// stay).  t* is found by bisection over the bit patterns of the probabilities (for positive floats the
// order of the values is the order of their bits), one workgroup-wide sum per step.
// REGS: the row fits 32 values per thread and stays in registers between the steps; otherwise it lives in the
// output row (each thread re-reads only what it wrote itself).
#define SWIFT_EACH(body)                                         \
    if constexpr (REGS) {                                        \
        _Pragma("unroll") for (int k = 0; k < PT; ++k) {         \
            const int i = tid + kThreads * k;                    \
            const bool ok = i < V;                               \
            (void)ok;                                            \
            float &x = v[k];                                     \
            body                                                 \
        }                                                        \
    } else {                                                     \
        for (int i = tid; i < V; i += kThreads) {                \
            const bool ok = true;                                \
            (void)ok;                                            \
            float &x = pr[i];                                    \
            body                                                 \
        }                                                        \
    }
template <bool REGS>
__global__ __launch_bounds__(kThreads) void k_warp(WarpArgs a) {
    constexpr int PT = 32;
    const float *lg = a.logits + (size_t)blockIdx.x * a.ld_logits;
    float *pr = a.probs + (size_t)blockIdx.x * a.V;
    const int tid = threadIdx.x, V = a.V;
    __shared__ float sh[16];
    float v[REGS ? PT : 1];
    float mx = -INFINITY;
    SWIFT_EACH(x = ok ? lg[i] : -INFINITY; mx = fmaxf(mx, x);)
    mx = block_max(mx, sh);
    const float inv_t = 1.0f / a.temperature;
    float z = 0.f;
    SWIFT_EACH(x = ok ? expf((x - mx) * inv_t) : 0.f; z += x;)
    z = block_sum(z, sh);
    float pmax = 0.f;
    SWIFT_EACH(x = x / z; pmax = fmaxf(pmax, x);)
    pmax = block_max(pmax, sh);
    uint32_t lo = 0;
    if (a.top_p < 1.0f) {
        uint32_t hi = __float_as_uint(pmax);
        while (lo < hi) {
            const uint32_t mid = lo + (hi - lo + 1) / 2;
            float s = 0.f;
            SWIFT_EACH(s += __float_as_uint(x) >= mid ? x : 0.f;)
            s = block_sum(s, sh);
            if (s >= a.top_p)
                lo = mid;
            else
                hi = mid - 1;
        }
    }
    float kept = 0.f;
    SWIFT_EACH(kept += __float_as_uint(x) >= lo ? x : 0.f;)
    kept = block_sum(kept, sh);
    SWIFT_EACH(if (ok) pr[i] = __float_as_uint(x) >= lo ? x / kept : 0.f;)
}
#undef SWIFT_EACH

// out[0] = a draw from probs (one row) with the uniform u
__global__ __launch_bounds__(kThreads) void k_draw(const float *probs, int V, float u, int32_t *out) {
    __shared__ float sh[16];
    __shared__ int shi[32];
    const int tok = block_draw([&](int j) { return probs[j]; }, V, u, sh, shi, nullptr);
    if (threadIdx.x == 0) out[0] = tok;
}

// The keep / replace rule over a verified block: draft token x_i (drawn from q_i) is kept iff
// u_i * q_i(x_i) < p_i(x_i); the first token that is not kept is replaced by a draw from
// max(0, p_i - q_i) (from p_i if that is zero everywhere) and ends the block; if all k are kept one more
// token is drawn from p_{k+1}.  out[0] = tokens kept, out[1] = the final token.
__global__ __launch_bounds__(kThreads) void k_spec_accept(SpecAcceptArgs a) {
    __shared__ float sh[16];
    __shared__ int shi[32];
    const int V = a.V;
    int m = 0;
    for (; m < a.k; ++m) {
        const int x = a.x[m];
        const float px = a.p[(size_t)m * V + x], qx = a.q[(size_t)m * V + x];
        if (!(a.u_accept[m] * qx < px)) break;
    }
    const float *p = a.p + (size_t)m * V;
    int tok;
    if (m < a.k) {
        const float *q = a.q + (size_t)m * V;
        float total;
        tok = block_draw([&](int j) { return fmaxf(p[j] - q[j], 0.f); }, V, a.u_final, sh, shi, &total);
        if (!(total > 0.f)) tok = block_draw([&](int j) { return p[j]; }, V, a.u_final, sh, shi, nullptr);
    } else {
        tok = block_draw([&](int j) { return p[j]; }, V, a.u_final, sh, shi, nullptr);
    }
    if (threadIdx.x == 0) {
        a.out[0] = m;
        a.out[1] = tok;
    }
}

}  // namespace

hipError_t launch_warp(const WarpArgs &a, hipStream_t s) {
    if (a.rows < 1 || a.V < 1 || !(a.temperature > 0.f) || !(a.top_p > 0.f)) return hipErrorInvalidValue;
    if (a.V <= 32 * kThreads)
        hipLaunchKernelGGL(k_warp<true>, dim3(a.rows), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL(k_warp<false>, dim3(a.rows), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_draw(const float *probs, int V, float u, int32_t *out, hipStream_t s) {
    if (V < 1 || !(u >= 0.f && u < 1.f)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_draw, dim3(1), dim3(kThreads), 0, s, probs, V, u, out);
    return hipGetLastError();
}

hipError_t launch_spec_accept(const SpecAcceptArgs &a, hipStream_t s) {
    if (a.k < 0 || a.k > kMaxRows - 1 || a.V < 1 || !(a.u_final >= 0.f && a.u_final < 1.f)) return hipErrorInvalidValue;
    for (int i = 0; i < a.k; ++i)
        if (a.x[i] < 0 || a.x[i] >= a.V) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_spec_accept, dim3(1), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace swift
