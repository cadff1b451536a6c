// gfx950 kernels of the draft / verify forward pass (single-row path).
//
// Every projection of the decoder is a weight-streaming pass: the weight matrix is read
// from HBM exactly once with 128-bit loads, the activation vector lives in LDS, and the
// operation that follows the projection (rotation + cache append, SwiGLU, residual add)
// runs in the same kernel on the finished dot products.  Wavefronts are 64 lanes wide;
// one wavefront owns two output rows at a time so that the rows an epilogue needs
// together (a rotary pair, a gate/up pair) are produced by the same wavefront.
#include "swift_kernels.h"

#include <math.h>

namespace swift {

// ------------------------------------------------------------------------------------------
// storage types
// ------------------------------------------------------------------------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 128-bit load

struct F32T {
    static constexpr int VEC = 4;  // elements per 16-byte load
    using elem = float;
    __device__ static void unpack(const u32x4 &v, float *f) {
        f[0] = __uint_as_float(v.x);
        f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z);
        f[3] = __uint_as_float(v.w);
    }
    __device__ static float load1(const elem *p) { return *p; }
    __device__ static void store1(elem *p, float f) { *p = f; }
};

__device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

struct BF16T {
    static constexpr int VEC = 8;
    using elem = uint16_t;
    __device__ static void unpack(const u32x4 &v, float *f) {
        f[0] = __uint_as_float(v.x << 16);
        f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16);
        f[3] = __uint_as_float(v.y & 0xffff0000u);
        f[4] = __uint_as_float(v.z << 16);
        f[5] = __uint_as_float(v.z & 0xffff0000u);
        f[6] = __uint_as_float(v.w << 16);
        f[7] = __uint_as_float(v.w & 0xffff0000u);
    }
    __device__ static float load1(const elem *p) { return __uint_as_float((uint32_t)(*p) << 16); }
    __device__ static void store1(elem *p, float f) { *p = f32_to_bf16_rne(f); }
};

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Sum over the whole workgroup (blockDim.x = 256); every thread gets the result.
// The order of additions is fixed, so every workgroup computes the same bits.
__device__ inline float block_sum_256(float v, float *red /* >= 4 floats of LDS */) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// ------------------------------------------------------------------------------------------
// weight-streaming pass, one activation row
// ------------------------------------------------------------------------------------------
template <typename T, int EPI>
__global__ __launch_bounds__(kGemvThreads) void k_gemv(GemvArgs a) {
    extern __shared__ __align__(16) float xs[];  // [K] activation (normalised if gain != null)
    __shared__ float red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int K = a.K;

    // ---- prologue: stage the activation row in LDS, RMS-normalised when a gain is given
    if (a.gain) {
        float ss = 0.f;
        for (int i = tid; i < K; i += kGemvThreads) {
            float v = a.xin[i];
            xs[i] = v;
            ss += v * v;
        }
        ss = block_sum_256(ss, red);
        const float r = 1.0f / sqrtf(ss / (float)K + a.eps);
        for (int i = tid; i < K; i += kGemvThreads) xs[i] = xs[i] * r * a.gain[i];
    } else {
        for (int i = tid; i < K; i += kGemvThreads) xs[i] = a.xin[i];
    }
    __syncthreads();

    // ---- units of two output rows
    const int d = a.head_dim, half = d >> 1;
    const int n_units = a.O >> 1;
    const int chunks = K / T::VEC;
    const typename T::elem *W = (const typename T::elem *)a.W;
    const int waves_total = gridDim.x * (kGemvThreads / 64);

    for (int u = blockIdx.x * (kGemvThreads / 64) + wave; u < n_units; u += waves_total) {
        int ra, rb;
        if (EPI == EPI_QKV) {
            const int hh = u / half, i = u - hh * half;  // head (q heads, then k heads, then v heads)
            ra = hh * d + i;
            rb = ra + half;
        } else {
            ra = 2 * u;
            rb = ra + 1;
        }
        const u32x4 *wa = (const u32x4 *)(W + (size_t)ra * K);
        const u32x4 *wb = (const u32x4 *)(W + (size_t)rb * K);
        float acc_a = 0.f, acc_b = 0.f;
#pragma unroll 4
        for (int c = lane; c < chunks; c += 64) {
            const u32x4 va = __builtin_nontemporal_load(wa + c);
            const u32x4 vb = __builtin_nontemporal_load(wb + c);
            float fa[T::VEC], fb[T::VEC];
            T::unpack(va, fa);
            T::unpack(vb, fb);
            const float *xp = xs + c * T::VEC;
#pragma unroll
            for (int j = 0; j < T::VEC; ++j) {
                acc_a = fmaf(fa[j], xp[j], acc_a);
                acc_b = fmaf(fb[j], xp[j], acc_b);
            }
        }
        acc_a = wave_sum(acc_a);
        acc_b = wave_sum(acc_b);
        if (lane != 0) continue;

        if (EPI == EPI_QKV) {
            const int hh = u / half, i = u - hh * half;
            const int nq = a.n_q_heads, nkv = a.n_kv_heads;
            if (hh < nq + nkv) {  // rotary pair (i, i + d/2)
                const float c = a.cos_row[i], s = a.sin_row[i];
                const float ya = acc_a * c - acc_b * s;
                const float yb = acc_b * c + acc_a * s;
                if (hh < nq) {
                    a.out[hh * d + i] = ya;
                    a.out[hh * d + i + half] = yb;
                } else {
                    typename T::elem *kc =
                        (typename T::elem *)a.kcache + ((size_t)(hh - nq) * a.max_seq + a.pos) * d;
                    T::store1(kc + i, ya);
                    T::store1(kc + i + half, yb);
                }
            } else {
                typename T::elem *vc =
                    (typename T::elem *)a.vcache + ((size_t)(hh - nq - nkv) * a.max_seq + a.pos) * d;
                T::store1(vc + i, acc_a);
                T::store1(vc + i + half, acc_b);
            }
        } else if (EPI == EPI_RESID) {
            a.out[ra] += acc_a;
            a.out[rb] += acc_b;
        } else if (EPI == EPI_SWIGLU) {
            a.out[u] = acc_a / (1.0f + expf(-acc_a)) * acc_b;
        } else {
            a.out[ra] = acc_a;
            a.out[rb] = acc_b;
        }
    }
}

template <typename T, int EPI>
static hipError_t launch_gemv_t(const GemvArgs &a, int n_cu, hipStream_t s) {
    const size_t lds = (size_t)a.K * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemv<T, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           160 * 1024 - 64);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int n_units = a.O / 2;
    const int wg_needed = (n_units + 3) / 4;
    // a few workgroups per compute unit; each one stages the activation row once
    int occupancy = lds > 48 * 1024 ? (lds > 76 * 1024 ? 1 : 2) : 4;
    int grid = n_cu * occupancy;
    if (grid > wg_needed) grid = wg_needed;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL((k_gemv<T, EPI>), dim3(grid), dim3(kGemvThreads), lds, s, a);
    return hipGetLastError();
}

hipError_t launch_gemv(int dtype, int epi, const GemvArgs &a, int n_cu, hipStream_t s) {
#define SWIFT_CASE(E)                                                      \
    case E:                                                                \
        return dtype == F32 ? launch_gemv_t<F32T, E>(a, n_cu, s) : launch_gemv_t<BF16T, E>(a, n_cu, s);
    switch (epi) {
        SWIFT_CASE(EPI_QKV)
        SWIFT_CASE(EPI_RESID)
        SWIFT_CASE(EPI_SWIGLU)
        SWIFT_CASE(EPI_LOGITS)
    }
#undef SWIFT_CASE
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------------
// embedding gather
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_embed(EmbedArgs a) {
    const typename T::elem *row = (const typename T::elem *)a.E + (size_t)a.token * a.H;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.H; i += gridDim.x * blockDim.x)
        a.x[i] = T::load1(row + i);
}

hipError_t launch_embed(int dtype, const EmbedArgs &a, hipStream_t s) {
    const int grid = (a.H + 255) / 256;
    if (dtype == F32)
        hipLaunchKernelGGL(k_embed<F32T>, dim3(grid), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(k_embed<BF16T>, dim3(grid), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// decode attention: one query row, all heads, split over the cache length
// ------------------------------------------------------------------------------------------
// Workgroup (kv head g, split s) handles cache slots [s*kAttnChunk, ...) for the query heads
// that share kv head g.  A group of LPP = d / VEC lanes owns one cache slot at a time; lane j
// of the group holds elements [j*VEC, (j+1)*VEC) of that slot's key and value.  Each lane
// group keeps a running (max, sum, weighted value) per query head (online softmax); groups,
// then wavefronts, are merged at the end and the workgroup writes one partial per head.
template <typename T, int GROUP>
__global__ __launch_bounds__(256) void k_attn_decode(AttnArgs a) {
    constexpr int VEC = T::VEC;
    const int d = a.head_dim;
    const int LPP = d / VEC;        // lanes per cache slot (power of two, <= 32)
    const int SPW = 64 / LPP;       // slots per wavefront step
    const int n_split = gridDim.y;
    const int g = blockIdx.x, sp = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lj = lane & (LPP - 1), lg = lane / LPP;
    const int lo = sp * kAttnChunk;
    const int hi = min(a.n_ctx, lo + kAttnChunk);
    const float scale = 1.0f / sqrtf((float)d);

    float q[GROUP][VEC];
#pragma unroll
    for (int h = 0; h < GROUP; ++h)
#pragma unroll
        for (int j = 0; j < VEC; ++j) q[h][j] = a.q[(size_t)(g * GROUP + h) * d + lj * VEC + j];

    float m[GROUP], l[GROUP], o[GROUP][VEC];
#pragma unroll
    for (int h = 0; h < GROUP; ++h) {
        m[h] = -INFINITY;
        l[h] = 0.f;
#pragma unroll
        for (int j = 0; j < VEC; ++j) o[h][j] = 0.f;
    }

    const typename T::elem *kc = (const typename T::elem *)a.kcache + (size_t)g * a.max_seq * d;
    const typename T::elem *vc = (const typename T::elem *)a.vcache + (size_t)g * a.max_seq * d;

    for (int p0 = lo + wave * SPW; p0 < hi; p0 += 4 * SPW) {
        const int p = p0 + lg;
        const bool live = p < hi;
        const int pc = live ? p : hi - 1;  // clamp: dead lane groups recompute a live slot and discard it
        const u32x4 kv = *(const u32x4 *)(kc + (size_t)pc * d + lj * VEC);
        const u32x4 vv = *(const u32x4 *)(vc + (size_t)pc * d + lj * VEC);
        float kf[VEC], vf[VEC];
        T::unpack(kv, kf);
        T::unpack(vv, vf);
#pragma unroll
        for (int h = 0; h < GROUP; ++h) {
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < VEC; ++j) s = fmaf(q[h][j], kf[j], s);
            for (int off = LPP >> 1; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
            s *= scale;
            if (live) {
                const float mn = fmaxf(m[h], s);
                const float corr = expf(m[h] - mn);  // exp(-inf) = 0 on the first slot
                const float pr = expf(s - mn);
                l[h] = l[h] * corr + pr;
#pragma unroll
                for (int j = 0; j < VEC; ++j) o[h][j] = o[h][j] * corr + pr * vf[j];
                m[h] = mn;
            }
        }
    }

    // merge lane groups of one wavefront (butterfly over the lane bits above LPP)
#pragma unroll
    for (int h = 0; h < GROUP; ++h) {
        for (int off = LPP; off < 64; off <<= 1) {
            const float m2 = __shfl_xor(m[h], off, 64);
            const float l2 = __shfl_xor(l[h], off, 64);
            const float mn = fmaxf(m[h], m2);
            const float c1 = (m[h] == -INFINITY) ? 0.f : expf(m[h] - mn);
            const float c2 = (m2 == -INFINITY) ? 0.f : expf(m2 - mn);
            l[h] = l[h] * c1 + l2 * c2;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const float o2 = __shfl_xor(o[h][j], off, 64);
                o[h][j] = o[h][j] * c1 + o2 * c2;
            }
            m[h] = mn;
        }
    }

    // merge the four wavefronts through LDS
    __shared__ float sm[4][GROUP], sl[4][GROUP];
    __shared__ float so[4][GROUP][256];
    if (lg == 0) {
#pragma unroll
        for (int h = 0; h < GROUP; ++h) {
            if (lj == 0) {
                sm[wave][h] = m[h];
                sl[wave][h] = l[h];
            }
#pragma unroll
            for (int j = 0; j < VEC; ++j) so[wave][h][lj * VEC + j] = o[h][j];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < GROUP * d; idx += 256) {
        const int h = idx / d, j = idx - h * d;
        float mn = fmaxf(fmaxf(sm[0][h], sm[1][h]), fmaxf(sm[2][h], sm[3][h]));
        float ls = 0.f, os = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float c = (sm[w][h] == -INFINITY) ? 0.f : expf(sm[w][h] - mn);
            ls += sl[w][h] * c;
            os += so[w][h][j] * c;
        }
        const int head = g * GROUP + h;
        a.part_o[((size_t)head * n_split + sp) * d + j] = os;
        if (j == 0) {
            a.part_ml[((size_t)head * n_split + sp) * 2 + 0] = mn;
            a.part_ml[((size_t)head * n_split + sp) * 2 + 1] = ls;
        }
    }
}

// out[head][j] = sum_s o_s[j] e^{m_s - M} / sum_s l_s e^{m_s - M}
__global__ void k_attn_combine(const float *part_o, const float *part_ml, int n_split, int d, float *out) {
    const int head = blockIdx.x;
    float M = -INFINITY;
    for (int s = 0; s < n_split; ++s) M = fmaxf(M, part_ml[((size_t)head * n_split + s) * 2]);
    for (int j = threadIdx.x; j < d; j += blockDim.x) {
        float L = 0.f, O = 0.f;
        for (int s = 0; s < n_split; ++s) {
            const float c = expf(part_ml[((size_t)head * n_split + s) * 2] - M);
            L += part_ml[((size_t)head * n_split + s) * 2 + 1] * c;
            O += part_o[((size_t)head * n_split + s) * d + j] * c;
        }
        out[(size_t)head * d + j] = O / L;
    }
}

template <typename T>
static hipError_t launch_attn_t(const AttnArgs &a, hipStream_t s) {
    const int group = a.n_q_heads / a.n_kv_heads;
    const int n_split = (a.n_ctx + kAttnChunk - 1) / kAttnChunk;
    dim3 grid(a.n_kv_heads, n_split), block(256);
    switch (group) {
        case 1: hipLaunchKernelGGL((k_attn_decode<T, 1>), grid, block, 0, s, a); break;
        case 2: hipLaunchKernelGGL((k_attn_decode<T, 2>), grid, block, 0, s, a); break;
        case 4: hipLaunchKernelGGL((k_attn_decode<T, 4>), grid, block, 0, s, a); break;
        case 8: hipLaunchKernelGGL((k_attn_decode<T, 8>), grid, block, 0, s, a); break;
        default: return hipErrorInvalidValue;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_attn_combine, dim3(a.n_q_heads), dim3(a.head_dim < 64 ? 64 : a.head_dim), 0, s, a.part_o,
                       a.part_ml, n_split, a.head_dim, a.out);
    return hipGetLastError();
}

hipError_t launch_attn_decode(int dtype, const AttnArgs &a, hipStream_t s) {
    return dtype == F32 ? launch_attn_t<F32T>(a, s) : launch_attn_t<BF16T>(a, s);
}

// ------------------------------------------------------------------------------------------
// greedy choice + confidence:  token = first arg-max, conf = 1 / sum exp(l - max)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_argmax_conf(ArgmaxArgs a) {
    const float *lg = a.logits + (size_t)blockIdx.x * a.V;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ float smax[16];
    __shared__ int sidx[16];
    __shared__ float ssum[16];
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = tid; i < a.V; i += 1024) {
        const float v = lg[i];
        if (v > best) {  // i increases per thread, so the first maximum is kept
            best = v;
            bi = i;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(best, off, 64);
        const int oi = __shfl_xor(bi, off, 64);
        if (ov > best || (ov == best && oi < bi)) {
            best = ov;
            bi = oi;
        }
    }
    if (lane == 0) {
        smax[wave] = best;
        sidx[wave] = bi;
    }
    __syncthreads();
    best = smax[0];
    bi = sidx[0];
    for (int w = 1; w < 16; ++w)
        if (smax[w] > best || (smax[w] == best && sidx[w] < bi)) {
            best = smax[w];
            bi = sidx[w];
        }
    float sum = 0.f;
    for (int i = tid; i < a.V; i += 1024) sum += expf(lg[i] - best);
    sum = wave_sum(sum);
    if (lane == 0) ssum[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int w = 0; w < 16; ++w) t += ssum[w];
        a.tokens[blockIdx.x] = bi;
        a.conf[blockIdx.x] = 1.0f / t;
    }
}

hipError_t launch_argmax_conf(const ArgmaxArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(k_argmax_conf, dim3(a.rows), dim3(1024), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// utilities
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_fill_nan(typename T::elem *p, int64_t n) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        T::store1(p + i, __uint_as_float(0x7fc00000u));
}

hipError_t launch_fill_nan(int dtype, void *p, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    int grid = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    if (dtype == F32)
        hipLaunchKernelGGL(k_fill_nan<F32T>, dim3(grid), dim3(256), 0, s, (float *)p, n);
    else
        hipLaunchKernelGGL(k_fill_nan<BF16T>, dim3(grid), dim3(256), 0, s, (uint16_t *)p, n);
    return hipGetLastError();
}

template <typename T>
__global__ void k_to_f32(const typename T::elem *src, float *dst, int64_t n) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        dst[i] = T::load1(src + i);
}

hipError_t launch_to_f32(int dtype, const void *src, float *dst, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    int grid = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    if (dtype == F32)
        hipLaunchKernelGGL(k_to_f32<F32T>, dim3(grid), dim3(256), 0, s, (const float *)src, dst, n);
    else
        hipLaunchKernelGGL(k_to_f32<BF16T>, dim3(grid), dim3(256), 0, s, (const uint16_t *)src, dst, n);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// tiled bf16 weights: layout conversion
// ------------------------------------------------------------------------------------------
__global__ void k_tile_weights(TileArgs a) {
    // one thread per 16-byte chunk of the destination
    const int64_t n_chunks = (int64_t)a.n_rg * a.T * 64;
    const uint16_t *src = (const uint16_t *)a.src;
    u32x4 *dst = (u32x4 *)a.dst;
    const int d = a.head_dim, half = d >> 1, gph = half >> 3;  // row groups per head (TILE_PAIR)
    for (int64_t c = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c < n_chunks;
         c += (int64_t)gridDim.x * blockDim.x) {
        const int l = (int)(c & 63);
        const int64_t tile = c >> 6;
        const int t = (int)(tile % a.T);
        const int rg = (int)(tile / a.T);
        const int j = l & 15, k0 = 32 * t + 8 * (l >> 4);
        int row;
        if (a.mode == TILE_PLAIN) {
            row = 16 * rg + j;
        } else if (a.mode == TILE_PAIR) {
            const int head = rg / gph, g = rg - head * gph;
            row = head * d + 8 * g + (j & 7) + (j >= 8 ? half : 0);
        } else {
            if ((j >= 8) != (a.part == 1)) continue;  // the other half of the tile comes from the other tensor
            row = 8 * rg + (j & 7);
        }
        u32x4 v = {0u, 0u, 0u, 0u};
        if (row < a.src_rows) {
            if (k0 + 8 <= a.K) {
                v = *(const u32x4 *)(src + (size_t)row * a.K + k0);
            } else {
                uint16_t e[8];
                for (int i = 0; i < 8; ++i) e[i] = (k0 + i < a.K) ? src[(size_t)row * a.K + k0 + i] : (uint16_t)0;
                v.x = e[0] | ((uint32_t)e[1] << 16);
                v.y = e[2] | ((uint32_t)e[3] << 16);
                v.z = e[4] | ((uint32_t)e[5] << 16);
                v.w = e[6] | ((uint32_t)e[7] << 16);
            }
        }
        dst[c] = v;
    }
}

hipError_t launch_tile_weights(const TileArgs &a, hipStream_t s) {
    const int64_t n_chunks = (int64_t)a.n_rg * a.T * 64;
    if (n_chunks <= 0) return hipSuccess;
    int64_t grid = (n_chunks + 255) / 256;
    if (grid > 65536) grid = 65536;
    hipLaunchKernelGGL(k_tile_weights, dim3((unsigned)grid), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// weight-streaming pass over a tiled matrix, one activation row, MFMA
// ------------------------------------------------------------------------------------------
// y = W . xhat with xhat kept in fp32 precision: xhat = hi + mid + lo, three bf16 terms that go
// into columns 0..2 of the MFMA B operand (the other 13 columns are zero); y is the sum of the
// three result columns.  A workgroup has 8 wavefronts; KS of them share one row group (each takes
// a contiguous slice of its k-tiles), so a workgroup works on G = 8/KS row groups at a time and the
// slices are added in LDS in a fixed order.  Every wavefront keeps two batches of eight 1 KB tile
// loads in flight, and the first batch is issued before the activation is staged.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int EPI, int KS>
__global__ __launch_bounds__(512) void k_mv1(MvArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    // LDS: [16 B of zeros][4T chunks x 3 terms x 8 bf16][2 x 8 wavefronts x 16 rows fp32][cos|sin row]
    uint16_t *Bs = (uint16_t *)(smem + 16);
    float *red = (float *)(smem + 16 + (size_t)a.T * 192);
    float *rot = red + 256;  // [d/2] cos then [d/2] sin (q|k|v epilogue only)
    __shared__ float ssum[8];
    constexpr int G = 8 / KS;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform from here on
    const int g = wave / KS, ks = wave - g * KS;
    const int T = a.T;
    const int n = (T + KS - 1) / KS;           // k-tiles per wavefront and row group
    const int t0 = min(ks * n, T - 1);
    const int nv = max(0, min(n, T - ks * n)); // ... of which exist
    const int nvm1 = max(nv - 1, 0);
    const u32x4 *Wt = (const u32x4 *)a.Wt;
    const int W = gridDim.x;
    const int last_rg = a.n_rg - 1;
    const int col = lane & 15, kg = lane >> 4;
    // byte address of this lane's B chunk for tile t: boff + t * bstride; lanes of columns >= 3
    // (and tiles past the wavefront's slice) read the zero chunk at address 0
    const int boff = col < 3 ? 16 + (kg * 3 + col) * 16 : 0;
    const int bstride = col < 3 ? 192 : 0;

    // Rolling window of 16 tile loads (16 KB) per wavefront: slot u of the next batch is issued as
    // soon as slot u of the current batch has been consumed.  Loads are unconditional: a slot past
    // the slice is clamped to the slice's last tile and multiplied by the zero chunk.
    u32x4 buf[16];
    const u32x4 *base = nullptr;
    auto load_slot = [&](int i) { return __builtin_nontemporal_load(base + (size_t)min(i, nvm1) * 64); };
    auto mma_slot = [&](int i, const u32x4 &av, f32x4 &acc, int live_mask) {
        const int m = (i < nv) ? live_mask : 0;              // all ones or zero, wavefront-uniform
        const int addr = (boff + (t0 + i) * bstride) & m;
        const u32x4 bv = *(const u32x4 *)(smem + addr);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv),
                                                      acc, 0, 0, 0);
    };
    auto prime = [&](int seg) {
        const int rg = min((seg * W + (int)blockIdx.x) * G + g, last_rg);
        base = Wt + ((size_t)rg * T + t0) * 64 + lane;
#pragma unroll
        for (int u = 0; u < 16; ++u) buf[u] = load_slot(u);
    };

    // ---- stage the activation: optional RMSNorm, then the three-term bf16 split.  The activation
    // loads are issued before the first weight loads so that they return first; the weight loads
    // are then in flight while the norm and the split run.
    auto split_store = [&](int i, float v) {
        const uint16_t hi = f32_to_bf16_rne(v);
        const float r1 = v - __uint_as_float((uint32_t)hi << 16);
        const uint16_t mid = f32_to_bf16_rne(r1);
        const float r2 = r1 - __uint_as_float((uint32_t)mid << 16);
        const uint16_t lo = f32_to_bf16_rne(r2);
        uint16_t *p = Bs + (size_t)(i >> 3) * 24 + (i & 7);
        p[0] = hi;
        p[8] = mid;
        p[16] = lo;
    };
    if (tid < 4) ((uint32_t *)smem)[tid] = 0u;
    const int Kp = T * 32;
    if (a.gain && Kp <= 16 * 512) {
        float xv[16], gv[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int i = tid + 512 * e;
            xv[e] = (i < a.K) ? a.xin[i] : 0.f;
            gv[e] = (i < a.K) ? a.gain[i] : 0.f;
        }
        prime(0);
        if (EPI == EPI_QKV) {
            const int half = a.head_dim >> 1;
            if (tid < half) {
                rot[tid] = a.cos_row[tid];
                rot[half + tid] = a.sin_row[tid];
            }
        }
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) ss += xv[e] * xv[e];
        ss = wave_sum(ss);
        if (lane == 0) ssum[wave] = ss;
        __syncthreads();
        ss = ((ssum[0] + ssum[1]) + (ssum[2] + ssum[3])) + ((ssum[4] + ssum[5]) + (ssum[6] + ssum[7]));
        const float r = 1.0f / sqrtf(ss / (float)a.K + a.eps);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int i = tid + 512 * e;
            if (i < Kp) split_store(i, xv[e] * r * gv[e]);
        }
    } else {
        prime(0);
        float r = 1.0f;
        if (a.gain) {
            float ss = 0.f;
            for (int i = tid; i < a.K; i += 512) {
                const float v = a.xin[i];
                ss += v * v;
            }
            ss = wave_sum(ss);
            if (lane == 0) ssum[wave] = ss;
            __syncthreads();
            ss = ((ssum[0] + ssum[1]) + (ssum[2] + ssum[3])) + ((ssum[4] + ssum[5]) + (ssum[6] + ssum[7]));
            r = 1.0f / sqrtf(ss / (float)a.K + a.eps);
        }
        if (EPI == EPI_QKV) {
            const int half = a.head_dim >> 1;
            if (tid < half) {
                rot[tid] = a.cos_row[tid];
                rot[half + tid] = a.sin_row[tid];
            }
        }
        for (int i0 = 0; i0 < Kp; i0 += 8 * 512) {
            float xv[8], gv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int i = i0 + tid + 512 * e;
                xv[e] = (i < a.K) ? a.xin[i] : 0.f;
                gv[e] = (a.gain && i < a.K) ? a.gain[i] : 1.f;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int i = i0 + tid + 512 * e;
                if (i < Kp) split_store(i, a.gain ? xv[e] * r * gv[e] : xv[e]);
            }
        }
    }
    __syncthreads();

    for (int seg = 0; seg < a.S; ++seg) {
        if (seg > 0) prime(seg);
        const int rg = (seg * W + (int)blockIdx.x) * G + g;
        const bool live = rg <= last_rg;
        const int live_mask = live ? -1 : 0;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};

        const int nb16 = (n + 15) >> 4;
        for (int b = 0; b + 1 < nb16; ++b) {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                mma_slot(b * 16 + u, buf[u], acc, live_mask);
                buf[u] = load_slot((b + 1) * 16 + u);
            }
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) mma_slot((nb16 - 1) * 16 + u, buf[u], acc, live_mask);

        // ---- end of the row group: add the three term columns, then the KS slices, then the epilogue
        float *rp = red + (size_t)(seg & 1) * 128;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float c1 = __shfl_down(acc[r], 1, 64), c2 = __shfl_down(acc[r], 2, 64);
            const float y = (acc[r] + c1) + c2;
            if (col == 0) rp[wave * 16 + 4 * kg + r] = y;
        }
        __syncthreads();
        if (!live || ks != 0 || lane >= 16) continue;
        float ya = 0.f, yb = 0.f;
        const bool paired = (EPI == EPI_QKV || EPI == EPI_SWIGLU);
#pragma unroll
        for (int k2 = 0; k2 < KS; ++k2) {
            ya += rp[(g * KS + k2) * 16 + (paired ? (lane & 7) : lane)];
            if (paired) yb += rp[(g * KS + k2) * 16 + (lane & 7) + 8];
        }
        if (EPI == EPI_RESID) {
            // x[row] += y as a fire-and-forget atomic: one add per element per launch, so the
            // result is the plain sum, and no load sits in the weight stream's wait counter
            const int row = 16 * rg + lane;
            if (row < a.O) atomicAdd(a.out + row, ya);
        } else if (EPI == EPI_LOGITS) {
            const int row = 16 * rg + lane;
            if (row < a.O) a.out[row] = ya;
        } else if (EPI == EPI_SWIGLU) {
            const int f = 8 * rg + lane;
            if (lane < 8 && 2 * f < a.O) a.out[f] = ya / (1.0f + expf(-ya)) * yb;
        } else {
            if (lane < 8) {
                const int d = a.head_dim, half = d >> 1, gph = half >> 3;
                const int hh = rg / gph, i = 8 * (rg - hh * gph) + lane;
                const int nq = a.n_q_heads, nkv = a.n_kv_heads;
                if (hh < nq + nkv) {
                    const float c = rot[i], s = rot[half + i];
                    const float qa = ya * c - yb * s, qb = yb * c + ya * s;
                    if (hh < nq) {
                        a.out[hh * d + i] = qa;
                        a.out[hh * d + i + half] = qb;
                    } else {
                        uint16_t *kc = (uint16_t *)a.kcache + ((size_t)(hh - nq) * a.max_seq + a.pos) * d;
                        kc[i] = f32_to_bf16_rne(qa);
                        kc[i + half] = f32_to_bf16_rne(qb);
                    }
                } else {
                    uint16_t *vc = (uint16_t *)a.vcache + ((size_t)(hh - nq - nkv) * a.max_seq + a.pos) * d;
                    vc[i] = f32_to_bf16_rne(ya);
                    vc[i + half] = f32_to_bf16_rne(yb);
                }
            }
        }
    }
}

template <int EPI, int KS>
static hipError_t launch_mv1_t(const MvArgs &a, int grid, size_t lds, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_mv1<EPI, KS>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)kMvMaxLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((k_mv1<EPI, KS>), dim3(grid), dim3(512), lds, s, a);
    return hipGetLastError();
}

hipError_t launch_mv1(int epi, MvArgs a, int n_cu, int ks_override, int wg_override, hipStream_t s) {
    const size_t lds = mv_lds_bytes(a.K);
    if (lds > kMvMaxLds) return hipErrorInvalidValue;
    // Work split: KS wavefronts per row group, W workgroups, S rounds, chosen so that every
    // workgroup gets the same number of row groups (a weight stream is only as fast as its
    // slowest wavefront) with 6..16 wavefronts per compute unit and >= 8 k-tiles per wavefront.
    int occ = (int)((160 * 1024) / (lds + 512));
    if (occ > 2) occ = 2;  // 16 wavefronts per compute unit at most
    if (occ < 1) occ = 1;
    const int max_wg = n_cu * occ;
    int best_ks = 8, best_w = 1, best_s = 1;
    double best_score = 1e30;
    for (int ks = 8; ks >= 1; ks /= 2) {
        if (ks_override && ks != ks_override) continue;
        const int G = 8 / ks;
        const int n = (a.T + ks - 1) / ks;
        // many short slices beat few long ones (measured: 16 tiles per wavefront is the sweet spot),
        // as long as a slice still fills most of the 16-deep load window
        if (n < 12 && ks > 1 && !ks_override) continue;
        for (int S = 1; S <= 8; ++S) {
            int W = (a.n_rg + G * S - 1) / (G * S);
            if (W > max_wg) continue;
            const double waste = (double)W * G * S / a.n_rg;           // >= 1
            const double fill = (double)W / max_wg;                     // fraction of resident slots used
            const double score = waste + (fill < 0.5 ? (0.5 - fill) : 0.0) + 0.002 * S + 0.01 * (8 / ks - 1);
            if (score < best_score) {
                best_score = score;
                best_ks = ks;
                best_w = W;
                best_s = S;
            }
        }
    }
    if (wg_override > 0) {
        const int G = 8 / best_ks;
        best_w = wg_override;
        best_s = (a.n_rg + G * best_w - 1) / (G * best_w);
    }
    a.S = best_s;
#define SWIFT_MV_CASE(E)                                                                   \
    case E:                                                                                \
        switch (best_ks) {                                                                 \
            case 1: return launch_mv1_t<E, 1>(a, best_w, lds, s);                          \
            case 2: return launch_mv1_t<E, 2>(a, best_w, lds, s);                          \
            case 4: return launch_mv1_t<E, 4>(a, best_w, lds, s);                          \
            default: return launch_mv1_t<E, 8>(a, best_w, lds, s);                         \
        }
    switch (epi) {
        SWIFT_MV_CASE(EPI_QKV)
        SWIFT_MV_CASE(EPI_RESID)
        SWIFT_MV_CASE(EPI_SWIGLU)
        SWIFT_MV_CASE(EPI_LOGITS)
    }
#undef SWIFT_MV_CASE
    return hipErrorInvalidValue;
}

}  // namespace swift
