// gfx950 kernels of the bf16 path: tiled weights streamed once from HBM into MFMA, activations
// kept in fp32 precision as three bf16 terms (two in blocks of more than 16 rows).  k_mv1 handles blocks of 1-5 activation rows whose
// activation fits in LDS (draft pass, plain decoding, short verify blocks), k_mvN blocks of up to
// 64 rows (longer verify blocks, prefill, candidate evaluation).
#include <math.h>

#include <algorithm>

#include <hip/hip_ext.h>

#include "swift_device.h"
#include "swift_kernels.h"
#include "swift_mv.h"

namespace swift {

// Events for the next projection launch (see set_launch_events in swift_kernels.h).
static thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;
void set_launch_events(hipEvent_t start, hipEvent_t stop) {
    g_ev_start = start;
    g_ev_stop = stop;
}
template <typename K, typename... Args>
static hipError_t launch_maybe_timed(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t s, Args... args) {
    if (g_ev_start) {
        hipEvent_t a = g_ev_start, b = g_ev_stop;
        g_ev_start = g_ev_stop = nullptr;
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, s, a, b, 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// weight layout conversion
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
// embedding gather for R rows: fp32 residual, split of x * gain_next, partial sums of squares
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_embed_rows(EmbedRowsArgs a) {
    // one thread per (row r, element i); 16 consecutive lanes share a 16-element group
    const int NT = block_terms(a.RL), NC = NT * layout_rows(a.RL);
    const int Hp = (a.H + 15) & ~15;
    const int total = a.R * Hp;
    for (int idx0 = blockIdx.x * 256; idx0 < total; idx0 += gridDim.x * 256) {
        const int idx = idx0 + threadIdx.x;
        const int r = idx / Hp, i = idx - r * Hp;
        float v = 0.f;
        const bool ok = idx < total && i < a.H;
        if (ok) {
            v = __uint_as_float((uint32_t)a.E[(size_t)a.tokens[r] * a.H + i] << 16);
            a.x[(size_t)r * a.H + i] = v;
            uint16_t hi, mid, lo;
            split3(v * a.gain_next[i], hi, mid, lo);
            uint16_t *p = a.xs + ((size_t)(i >> 3) * NC + NT * r) * 8 + (i & 7);
            p[0] = hi;
            p[8] = mid;
            if (NT == 3) p[16] = lo;
        }
        float ss = v * v;
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
        if (idx < total && (i & 15) == 0) a.pss[(size_t)(i >> 4) * a.rp + r] = ss;
    }
}

hipError_t launch_embed_rows(const EmbedRowsArgs &a, hipStream_t s) {
    const int Hp = (a.H + 15) & ~15;
    const int grid = (a.R * Hp + 255) / 256;
    hipLaunchKernelGGL(k_embed_rows, dim3(grid), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// shared pieces of the projection kernels
// ------------------------------------------------------------------------------------------
// RMSNorm scale per block row from the producer's partial sums of squares [n_pss][16].  All 512
// threads load (thread = (partial p mod 32, row r)); mv_norm_load issues the first eight loads per
// thread (enough for 256 partials, hidden <= 4096) so that the caller can put them ahead of the
// weight loads; mv_norm_finish adds the rest, then 16 threads add the 32 per-lane sums in order:
// the summation order is fixed.  One barrier, before the final sums.  (Full barriers: LDS-only ones, which would leave the
// caller's first weight loads in flight, measured 0.3 us slower per launch.)
struct NormPart {
    float v[8];
};
__device__ inline NormPart mv_norm_load(const MvArgs &a) {
    NormPart np;
    const int tid = threadIdx.x, r = tid & 15, q = tid >> 4;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int p = q + 32 * u;
        np.v[u] = (a.pss && p < a.n_pss) ? a.pss[(size_t)p * a.rp + r] : 0.f;
    }
    return np;
}
template <bool LDS_ONLY = false>
__device__ inline void mv_norm_finish(const MvArgs &a, const NormPart &np, float *rs /* LDS [16] */,
                                      float *scratch /* LDS [512] */) {
    const int tid = threadIdx.x, r = tid & 15, q = tid >> 4;
    if (a.pss) {
        float ss = 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) ss += np.v[u];
        for (int p0 = 256; p0 < a.n_pss; p0 += 256) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = p0 + q + 32 * u;
                v[u] = p < a.n_pss ? a.pss[(size_t)p * a.rp + r] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) ss += v[u];
        }
        scratch[q * 16 + r] = ss;
    }
    if (LDS_ONLY)
        lds_barrier();
    else
        __syncthreads();
    if (tid < 16) {
        float ss = 0.f;
        if (a.pss)
            for (int q2 = 0; q2 < 32; ++q2) ss += scratch[q2 * 16 + tid];
        rs[tid] = a.pss ? 1.0f / sqrtf(ss / (float)a.norm_dim + a.eps) : 1.0f;
    }
    // (no barrier here: the scales are read by the epilogue only, and every caller has a barrier between
    // this point and its epilogue)
}

// The same for blocks of up to 64 rows (row pitch 64): thread = (partial p mod 8, row r), then 64
// threads add the 8 per-thread sums in order.  One barrier, before the final sums.  scratch: LDS [512].
__device__ inline void mv_norm_rows64(const MvArgs &a, float *rs /* LDS [64] */, float *scratch) {
    const int tid = threadIdx.x, r = tid & 63, q = tid >> 6;
    if (a.pss) {
        float ss = 0.f;
        for (int p0 = 0; p0 < a.n_pss; p0 += 64) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = p0 + q + 8 * u;
                v[u] = p < a.n_pss ? a.pss[(size_t)p * a.rp + r] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) ss += v[u];
        }
        scratch[q * 64 + r] = ss;
    }
    __syncthreads();
    if (tid < 64) {
        float ss = 0.f;
        if (a.pss)
            for (int q2 = 0; q2 < 8; ++q2) ss += scratch[q2 * 64 + tid];
        rs[tid] = a.pss ? 1.0f / sqrtf(ss / (float)a.norm_dim + a.eps) : 1.0f;
    }
    // (no barrier here: the scales are read by the epilogue only, and every caller has a barrier between
    // this point and its epilogue)
}

// The same for exact layouts of 17..32 rows (row pitch 64), in the summation order of mv_norm_load /
// mv_norm_finish -- a row's scale must not depend on the rows it shares a pass with: thread (row r, q) adds
// the partials q + 32 u and q + 16 + 32 u, u = 0, 1, .., as two sums; then 32 threads add the 32 sums in
// order.  One barrier, before the final sums.  scratch: LDS [1024].
__device__ inline void mv_norm_rows32(const MvArgs &a, float *rs /* LDS [64] */, float *scratch) {
    const int tid = threadIdx.x, r = tid & 31, q0 = tid >> 5;
    if (a.pss) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int q = q0 + 16 * half;
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = q + 32 * u;
                v[u] = p < a.n_pss ? a.pss[(size_t)p * a.rp + r] : 0.f;
            }
            float ss = 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) ss += v[u];
            for (int p0 = 256; p0 < a.n_pss; p0 += 256) {
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int p = p0 + q + 32 * u;
                    v[u] = p < a.n_pss ? a.pss[(size_t)p * a.rp + r] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) ss += v[u];
            }
            scratch[q * 32 + r] = ss;
        }
    }
    __syncthreads();
    if (tid < 32) {
        float ss = 0.f;
        if (a.pss)
            for (int q2 = 0; q2 < 32; ++q2) ss += scratch[q2 * 32 + tid];
        rs[tid] = a.pss ? 1.0f / sqrtf(ss / (float)a.norm_dim + a.eps) : 1.0f;
    }
}

// Slices (of the 8 K slices of a row group) whose sums are added first, in slice order, before the
// group sums are added in group order: 8, 4, 2 or 1.  It is the number of slices one workgroup of
// the block kernel covers when that kernel splits K over workgroups to fill the chip, and it
// depends on the matrix (and the device) only, so that every kernel adds a row's slice sums in the
// same order whatever the number of rows in the pass.
static int mv_slice_group(const MvArgs &a, int n_cu) {
    const int n_rb = (a.n_rg + 7) / 8;
    int ksp = n_cu / n_rb;
    if (ksp < 1) ksp = 1;
    if (ksp > 8) ksp = 8;
    int p2 = 1;
    while (p2 * 2 <= ksp) p2 *= 2;
    ksp = p2;
    const int n_c = (a.T + 7) / 8;
    // (a workgroup's K range holds at least 8 tiles; the partial sums fit the scratch)
    while (ksp > 1 && (n_c * (8 / ksp) < 8 || (int64_t)ksp * a.n_rg > a.part_capacity)) ksp /= 2;
    return 8 / ksp;
}

// ------------------------------------------------------------------------------------------
// 1..5 activation rows: Y = W . X, MFMA, whole activation in LDS, K split over wavefronts
// ------------------------------------------------------------------------------------------
// The NC = 3R term columns of X (R <= 5, so NC <= 15) fit one MFMA column block; lanes of columns
// >= NC read a zero chunk.  A workgroup has 8 wavefronts; KS of them share one 16-row group of W,
// each taking a contiguous slice of its k-tiles, so a workgroup works on G = 8/KS row groups at a
// time and the slices (and the three terms) are added in LDS in a fixed order.  Every wavefront
// keeps a rolling window of NS (10..16) 1 KB tile loads in flight, walked in blocks of NS slots (the
// launcher picks the depth that cuts the slice with the fewest unused slots); the first window is
// issued before the activation is staged, and the window rolls on from one round into the next.
template <int EPI, int KS, int NS>
__global__ __launch_bounds__(512, 4) void k_mv1(MvArgs a) {  // 4 wavefronts per SIMD: <= 128 VGPRs, two workgroups per CU
    extern __shared__ __align__(16) unsigned char smem[];
    const int R = a.R, NC = 3 * R;
    // LDS: [16 B zeros][4T chunks x NC x 8 bf16][2 x 8 wavefronts x NC x 16 fp32][16 scales][512 scratch][R x d rotary]
    float *red = (float *)(smem + 16 + (size_t)a.T * 64 * NC);
    float *rs = red + 2 * 8 * 16 * NC;
    float *nscratch = rs + 16;
    float *rot = nscratch + 512;  // per block row: [d/2 cos | d/2 sin] at that row's position
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
    const int W = a.n_wg;
    if (EPI == EPI_QKV && (int)blockIdx.x >= W) {
        // Cache warm-up for the attention launch that follows: warm-up workgroup p reads the committed keys
        // and values of the kv heads congruent to p.  Workgroups go to the dies round-robin by index, and the
        // attention kernel's workgroup for head g has index g (+ a multiple of 8 per further row), so with
        // pf_first and the number of warm-up workgroups multiples of 8 the lines land in the L2
        // that kernel's loads will ask.  No result; no barrier.
        // (pf_wgs warm-up workgroups, a multiple of 8: workgroup p takes the heads congruent to p modulo pf_wgs)
        const int p = (int)blockIdx.x - a.pf_first;
        if (p < 0) return;
        const size_t head_units = (size_t)a.max_seq * a.head_dim / 8;  // 16-byte units of one head
        const int n_units = a.pf_rows * a.head_dim / 8;
        // (values in groups of eight slots: the groups that hold rows [0, pf_rows) are contiguous too)
        const size_t v_head_units = a.nb32 > 0 ? (size_t)a.nb32 * 32 * a.head_dim / 8 : head_units;
        const int v_units = a.nb32 > 0 ? (a.pf_rows + 31) / 32 * 32 * a.head_dim / 8 : n_units;
        u32x4 x = {0u, 0u, 0u, 0u};
        for (int gh = p; gh < a.pf_heads; gh += a.pf_wgs) {
            const u32x4 *kp = (const u32x4 *)a.kcache + (size_t)gh * head_units;
            const u32x4 *vp = (const u32x4 *)a.vcache + (size_t)gh * v_head_units;
            // (eight steps' loads requested together: one step at a time, the loop is a chain of memory latencies)
            for (int i0 = tid; i0 < v_units; i0 += 8 * 512) {  // (v_units >= n_units)
                u32x4 t[16];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int i = i0 + 512 * u;
                    t[2 * u] = i < n_units ? kp[i] : u32x4{0u, 0u, 0u, 0u};  // (plain loads: the lines are meant to stay in L2)
                    t[2 * u + 1] = i < v_units ? vp[i] : u32x4{0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) x ^= t[u];
            }
        }
        // (keeps the loads alive; the flag word is never all ones)
        if ((x.x & x.y & x.z & x.w) == 0xffffffffu && a.pf_rows < 0) ((volatile uint32_t *)smem)[0] = x.x;
        return;
    }
    const int last_rg = a.n_rg - 1;
    const int col = lane & 15, kg = lane >> 4;
    // byte address of this lane's B chunk for tile t: boff + t * bstride; lanes of columns >= NC
    // (and slots past the wavefront's slice) read the zero chunk at address 0
    const int boff = col < NC ? 16 + (kg * NC + col) * 16 : 0;
    const int bstride = col < NC ? 64 * NC : 0;

    u32x4 buf[NS];
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
        for (int u = 0; u < NS; ++u) buf[u] = load_slot(u);
    };

    // ---- stage the split activation (a plain copy: the producer kernel already wrote it in B
    // layout).  Its loads, and those of the norm partials, go out ahead of the weight loads so
    // that they return first; the first weight window is in flight while LDS is filled.
    {
        const u32x4 *src = (const u32x4 *)a.in_s;
        u32x4 *dst = (u32x4 *)(smem + 16);
        const int n_units = T * 4 * NC, real_units = (a.K >> 3) * NC;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        // The residual projections read their norm partials ahead of the weight window and wait for them
        // with an LDS-only barrier, so that the MFMAs start on the first tiles while the rest of the window
        // is still on its way (o_proj 10.7 -> 10.4 us, down_proj 19.0 -> 18.2 us); the other epilogues measured
        // slower that way (q|k|v by 2.7 us) and keep the full barrier.
        constexpr bool kEarlyNorm = EPI == EPI_RESID;
        NormPart np;
        auto side_loads = [&]() {
            if (tid < 4) ((uint32_t *)smem)[tid] = 0u;
            if (EPI == EPI_QKV) {
                // the lines the epilogues of this workgroup's rounds will write values into (wavefront s: round s)
                if (wave < a.S)
                    for (int gg = 0; gg < G; ++gg) mv_touch_value_lines(a, min((wave * W + (int)blockIdx.x) * G + gg, last_rg), lane);
                const int d = a.head_dim, half = d >> 1;
                for (int i = tid; i < R * half; i += 512) {
                    const int r = i / half, e = i - r * half;
                    rot[r * d + e] = a.cos_tab[(size_t)mv_rope_pos(a, r) * half + e];
                    rot[r * d + half + e] = a.sin_tab[(size_t)mv_rope_pos(a, r) * half + e];
                }
            }
        };
        if (n_units <= 4 * 512) {  // depth <= 5461 for one row: four loads per thread cover it
            u32x4 tmp[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int i = tid + 512 * q;
                tmp[q] = i < real_units ? src[i] : zero;
            }
            if (kEarlyNorm) np = mv_norm_load(a);
            prime(0);
            side_loads();
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int i = tid + 512 * q;
                if (i < n_units) dst[i] = tmp[q];
            }
        } else {
            u32x4 tmp[9];
#pragma unroll
            for (int q = 0; q < 9; ++q) {
                const int i = tid + 512 * q;
                tmp[q] = i < real_units ? src[i] : zero;
            }
            if (kEarlyNorm) np = mv_norm_load(a);
            prime(0);
            side_loads();
#pragma unroll
            for (int q = 0; q < 9; ++q) {
                const int i = tid + 512 * q;
                if (i < n_units) dst[i] = tmp[q];
            }
            for (int i0 = 9 * 512; i0 < n_units; i0 += 4 * 512) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int i = i0 + tid + 512 * q;
                    tmp[q] = i < real_units ? src[i] : zero;
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int i = i0 + tid + 512 * q;
                    if (i < n_units) dst[i] = tmp[q];
                }
            }
        }
        if (!kEarlyNorm) np = mv_norm_load(a);
        mv_norm_finish<kEarlyNorm>(a, np, rs, nscratch);
    }

    for (int seg = 0; seg < a.S; ++seg) {
        const int rg = (seg * W + (int)blockIdx.x) * G + g;
        const bool live = rg <= last_rg;
        const int live_mask = live ? -1 : 0;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};

        const int nb16 = (n + NS - 1) / NS;
        // (As compiled, the NS reloads of a block go out together behind its last MFMA.  Pinning each
        // reload behind the MFMA that frees its slot with scheduling barriers measured the same.)
        for (int b = 0; b + 1 < nb16; ++b) {
#pragma unroll
            for (int u = 0; u < NS; ++u) {
                mma_slot(b * NS + u, buf[u], acc, live_mask);
                buf[u] = load_slot((b + 1) * NS + u);
            }
        }
        if (seg + 1 < a.S) {
            // the window rolls on into the next round's row group: the stream never drains
            const int rgn = min(((seg + 1) * W + (int)blockIdx.x) * G + g, last_rg);
            base = Wt + ((size_t)rgn * T + t0) * 64 + lane;
#pragma unroll
            for (int u = 0; u < NS; ++u) {
                mma_slot((nb16 - 1) * NS + u, buf[u], acc, live_mask);
                buf[u] = load_slot(u);
            }
        } else {
#pragma unroll
            for (int u = 0; u < NS; ++u) mma_slot((nb16 - 1) * NS + u, buf[u], acc, live_mask);
        }

        // ---- end of the row group: every wavefront parks its NC result columns in LDS; one
        // wavefront per row group adds terms and K slices and runs the epilogue
        float *rp = red + (size_t)(seg & 1) * (8 * 16 * NC);
        if (col < NC) {
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) rp[(wave * NC + col) * 16 + 4 * kg + r4] = acc[r4];
        }
        lds_barrier();  // (the next round's tile loads stay in flight)
        if (!live || ks != 0) continue;
        mv_epilogue<EPI>(a, rg, lane, rs, EPI == EPI_QKV ? rot : nullptr, [&](int r, int j) {
            // Slice sums are added per term in groups of kgroup slices (slice order), the three
            // terms of a group are combined, and the groups are added in order.  (Rolled loops: this
            // runs in one wavefront per row group while the load window stays in registers.)
            const int kgroup = a.kgroup;
            const float *w = rp + (g * KS * NC + 3 * r) * 16 + j;
            const int ss = NC * 16;  // from one slice to the next
            float y = 0.f;
#pragma unroll 1
            for (int k0 = 0; k0 < KS; k0 += kgroup) {
                float hi = w[0], mid = w[16], lo = w[32];
                w += ss;
#pragma unroll 1
                for (int k2 = 1; k2 < kgroup; ++k2) {
                    hi += w[0];
                    mid += w[16];
                    lo += w[32];
                    w += ss;
                }
                const float gs = (hi + mid) + lo;
                y = k0 == 0 ? gs : y + gs;
            }
            return y;
        });
    }
}

template <int EPI, int KS, int NS>
static hipError_t launch_mv1_t(const MvArgs &a, int grid, size_t lds, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_mv1<EPI, KS, NS>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)kMvMaxLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    return launch_maybe_timed(k_mv1<EPI, KS, NS>, dim3(grid), dim3(512), lds, s, a);
}

static hipError_t launch_mv1(int epi, MvArgs a, int n_cu, int ks_override, int wg_override, hipStream_t s) {
    const size_t lds = mv1_lds_bytes(a.K, a.R, a.head_dim);
    if (lds > kMvMaxLds) return hipErrorInvalidValue;
    // Work split: KS wavefronts per row group, W workgroups, S rounds, chosen so that every
    // workgroup gets the same number of row groups (a weight stream is only as fast as its
    // slowest wavefront) with at most 16 wavefronts per compute unit.
    int occ = (int)((160 * 1024) / (lds + 512));
    if (occ > 2) occ = 2;
    if (occ < 1) occ = 1;
    const int max_wg = n_cu * occ;
    int best_ks = 8, best_w = 1, best_s = 1;
    double best_score = 1e30;
    // Always 8 K slices per row group (unless a tuning run overrides it): the slice boundaries and
    // the order in which slice sums are added define a row's result bit for bit, and the block kernel
    // for 6-16 rows uses the same ones, so that a token's logits do not depend on how many rows
    // share its pass (speculative output == plain greedy output exactly, not just up to rounding).
    for (int ks = 8; ks >= 1; ks /= 2) {
        if (ks != (ks_override ? ks_override : 8)) continue;
        const int G = 8 / ks;
        for (int S = 1; S <= 64; ++S) {
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
    a.n_wg = best_w;
    int grid = best_w;
    // (the warm-up workgroups only pay while they run beside the projection: they take free slots only)
    a.pf_first = (best_w + 7) / 8 * 8;
    a.pf_wgs = std::min((max_wg - a.pf_first) / 8 * 8, (a.pf_heads + 7) / 8 * 8);
    // Only with one workgroup per head, the compute units clearly under-filled (measured with 480 of 512 slots
    // taken: the extra workgroups slow the projection down by more than the attention gains), and a context
    // short enough for a workgroup to read its whole head well before the projection ends: one compute unit
    // takes in about 37 GB/s and the weights stream at about 5 TB/s, so a head may hold 0.6 of what can be
    // read in that time (7B shape: up to about 860 slots; warming only part of a longer head measured worse
    // than not warming at all).
    const double t_us = (double)a.n_rg * a.T * 1024.0 / 5.0e6;
    const double head_bytes = (double)a.pf_rows * a.head_dim * 4.0;  // keys and values, bf16
    if (epi == EPI_QKV && a.pf_heads > 0 && a.pf_rows > 0 && a.pf_wgs >= a.pf_heads &&
        a.pf_first + a.pf_wgs <= max_wg * 85 / 100 && head_bytes <= 0.6 * 37.0e3 * t_us) {
        grid = a.pf_first + a.pf_wgs;
    } else {
        a.pf_heads = 0;
        a.pf_wgs = 0;
    }
    a.kgroup = best_ks == 8 ? mv_slice_group(a, n_cu) : best_ks;
    // Slots per block of the load window (= loads in flight per wavefront): 16 unless another depth
    // cuts a slice of n tiles with fewer wasted slots (n = 43: 3 x 15 instead of 3 x 16; n = 20:
    // 2 x 10 instead of 2 x 16).  Only for the 8-way split, which is what the big shapes use.
    int ns = 16;
    if (best_ks == 8) {
        const int n = (a.T + 7) / 8;
        int best_waste = (n + 15) / 16 * 16 - n;
        for (int c = 15; c >= 10; --c) {
            const int waste = (n + c - 1) / c * c - n;
            if (waste < best_waste && (n + c - 1) / c <= (n + 15) / 16 + 1) {
                best_waste = waste;
                ns = c;
            }
        }
    }
#define SWIFT_MV_CASE(E)                                                                   \
    case E:                                                                                \
        switch (best_ks) {                                                                 \
            case 1: return launch_mv1_t<E, 1, 16>(a, grid, lds, s);                      \
            case 2: return launch_mv1_t<E, 2, 16>(a, grid, lds, s);                      \
            case 4: return launch_mv1_t<E, 4, 16>(a, grid, lds, s);                      \
            default:                                                                       \
                switch (ns) {                                                              \
                    case 10: return launch_mv1_t<E, 8, 10>(a, grid, lds, s);             \
                    case 11: return launch_mv1_t<E, 8, 11>(a, grid, lds, s);             \
                    case 12: return launch_mv1_t<E, 8, 12>(a, grid, lds, s);             \
                    case 13: return launch_mv1_t<E, 8, 13>(a, grid, lds, s);             \
                    case 14: return launch_mv1_t<E, 8, 14>(a, grid, lds, s);             \
                    case 15: return launch_mv1_t<E, 8, 15>(a, grid, lds, s);             \
                    default: return launch_mv1_t<E, 8, 16>(a, grid, lds, s);             \
                }                                                                          \
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

// ------------------------------------------------------------------------------------------
// a block of 2..64 activation rows: Y = W . X, MFMA, K chunked through LDS, optional split-K
// ------------------------------------------------------------------------------------------
// Each of the 8 wavefronts of a workgroup owns RG 16-row groups of W; the workgroup walks its K
// range in chunks of CT tiles.  The B operand of a chunk (4 CT k-chunks x NC = 3R columns x 16 B,
// already in B layout in global memory) is copied into one of two LDS buffers while the MFMAs of
// the previous chunk run; the A tiles of the next chunk are loaded into a second register set at
// the same time.  NCB = ceil(NC/16) column blocks; a B operand read from LDS feeds RG MFMAs (with
// RG = 2 the LDS traffic per MFMA halves, which is what bounds the 64-row case).  With
// gridDim.y > 1 the K range is split over workgroups: each writes its partial results, and the
// workgroup that arrives last at a counter adds the partials in split order (so the result does
// not depend on arrival order) and runs the epilogue.
//
// CANON (exact layouts: verify blocks of up to 32 rows, 1-6 column blocks) reproduces the LDS-resident kernel
// bit for bit: the K range of a row group is cut into the same 8 slices of ceil(T/8) tiles, a slice is
// accumulated from zero tile by tile, a workgroup covers a group of 8, 4, 2 or 1 whole slices (mv_slice_group: a
// function of the matrix alone, not of the row count) and adds their sums per term in slice order, combines
// the three terms, and the last workgroup adds the group results in order.  The LDS-resident kernel adds its 8
// slice sums in the same grouping.  The bulk variants (NCB = 4 / 8: layouts of 32 / 64 rows, two-term columns)
// keep their own fixed order.
template <int EPI, int NCB, int CT, int RG, bool DMA, bool CANON>
__global__ __launch_bounds__(512) void k_mvN(MvArgs a, int TS, int rpw) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int R = a.R, NT = block_terms(a.RL), NC = NT * layout_rows(a.RL);  // NC: columns of the split input as laid out
    const int buf_bytes = 4 * CT * NC * 16;
    // the result dump (NCB * 8 KB) reuses the B buffers, so the region is at least that large
    const int main_bytes = max(2 * buf_bytes, NCB * 8192);
    float *rs = (float *)(smem + 16 + (size_t)main_bytes);
    int *flag = (int *)(rs + 64);
    float *nscratch = rs + 80;  // [1024]
    float *dump = (float *)(smem + 16);  // reuses the B buffers after the last MFMA
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T = a.T;
    // rpw <= 8 wavefronts of a workgroup own row groups (the launcher's choice: as many as spread the matrix
    // evenly over the compute units); the others only help with the copies and the barriers
    const bool active = wave < rpw;
    const int rg0 = ((int)blockIdx.x * rpw + min(wave, rpw - 1)) * RG;  // first row group of this wavefront
    const int tb = (int)blockIdx.y * TS;
    const int nt = min(T, tb + TS) - tb;  // >= 1 (launcher)
    const int col = lane & 15, kg = lane >> 4;
    constexpr bool kCanon = CANON;  // exact layouts (verify blocks); the bulk variants keep their own order
    // A slice is walked in chunks of CT tiles that do not run over its end (the last chunk of a slice
    // may be partial), so that slices end between chunks.  The prefill variant has one "slice": its
    // whole K range.
    const int n_c = kCanon ? (T + 7) >> 3 : nt;   // tiles of a slice
    const int nchs = (n_c + CT - 1) / CT;         // chunks of a slice
    const int nch = ((nt + n_c - 1) / n_c - 1) * nchs + ((nt - 1) % n_c) / CT + 1;  // chunks of this workgroup
    const int KSP = gridDim.y;
    // first tile (relative to tb) of chunk c, and the tiles of it that exist
    auto chunk_t0 = [&](int c) { return (c / nchs) * n_c + (c % nchs) * CT; };
    auto chunk_nt = [&](int c) { return min(min(CT, n_c - (c % nchs) * CT), nt - chunk_t0(c)); };
    const u32x4 *base[RG];
#pragma unroll
    for (int g = 0; g < RG; ++g)  // row groups past the end repeat the last one; their results are dropped
        base[g] = (const u32x4 *)a.Wt + ((size_t)min(rg0 + g, a.n_rg - 1) * T + tb) * 64 + lane;
    if (EPI == EPI_QKV && active) {  // the lines this wavefront's epilogue will write values into
#pragma unroll
        for (int g = 0; g < RG; ++g) mv_touch_value_lines(a, min(rg0 + g, a.n_rg - 1), lane);
    }
    const u32x4 *bsrc = (const u32x4 *)a.in_s;
    const int real_units = (a.K >> 3) * NC;
    const int chunk_units = 4 * CT * NC;  // 16-byte units of one B chunk (<= 512 NQ)
    constexpr int NQ = (4 * CT * NCB * 16 + 511) / 512;  // ... per thread

    // per-lane B addressing: byte offset inside a buffer for tile u, column block cb:
    //   ((4u + kg) * NC + 16 cb + col) * 16 = boff0 + u * tstride + 256 cb.
    // Columns that do not exist (col >= NC in the last block, rows >= R of a 64-row layout) read
    // whatever lies there: they only produce result columns that nobody reads.
    const int boff0 = 16 + (kg * NC + col) * 16;
    const int tstride = 4 * NC * 16;

    f32x4 acc[RG][NCB];
    // The sums of this workgroup's slices are added in slice order as the slices are completed.
    f32x4 ssum[kCanon ? NCB : 1];
#pragma unroll
    for (int g = 0; g < RG; ++g)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) acc[g][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cb = 0; cb < (kCanon ? NCB : 1); ++cb) ssum[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto slice_end = [&]() {
#pragma unroll
        for (int cb = 0; cb < (kCanon ? NCB : 1); ++cb) {
            ssum[cb] += acc[0][cb];
            acc[0][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };
    auto loadA = [&](int c, u32x4(&A)[RG][CT]) {
        const int t0 = chunk_t0(c);
#pragma unroll
        for (int g = 0; g < RG; ++g)
#pragma unroll
            for (int u = 0; u < CT; ++u)
                A[g][u] = active ? __builtin_nontemporal_load(base[g] + (size_t)min(t0 + u, nt - 1) * 64)
                                 : u32x4{0u, 0u, 0u, 0u};
    };
    auto loadB = [&](int c, u32x4(&tmp)[NQ]) {
        const int gu0 = 4 * (tb + chunk_t0(c)) * NC;
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int i = tid + 512 * q;
            tmp[q] = (i < chunk_units && gu0 + i < real_units) ? bsrc[gu0 + i] : zero;
        }
    };
    auto storeB = [&](int bi, const u32x4(&tmp)[NQ]) {
        u32x4 *dst = (u32x4 *)(smem + 16 + (size_t)bi * buf_bytes);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int i = tid + 512 * q;
            if (i < chunk_units) dst[i] = tmp[q];
        }
    };
    // DMA variants: B chunk c -> LDS buffer bi straight from global memory (no registers, no LDS write
    // instructions: the data lands while the wavefronts run MFMAs).  A wavefront's 64 lanes fill 64
    // consecutive 16-byte units from a wavefront-uniform base; lanes past the chunk take no part.  Units
    // past the real K range (a ragged last tile) are zeroed with ordinary writes.
    auto dmaB = [&](int c, int bi) {
        const int gu0 = 4 * (tb + chunk_t0(c)) * NC;
        u32x4 *dst = (u32x4 *)(smem + 16 + (size_t)bi * buf_bytes);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int i = tid + 512 * q;
            if (i < chunk_units) {
                if (gu0 + i < real_units)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(bsrc + gu0 + i),
                                                     (__attribute__((address_space(3))) void *)(dst + 512 * q + 64 * wave), 16, 0, 0);
                else
                    dst[i] = u32x4{0u, 0u, 0u, 0u};
            }
        }
    };
    // The B operands of a tile (NCB LDS reads) are requested one tile ahead of the MFMAs that use
    // them.  Slots past the chunk's tiles multiply a zero A operand.
    auto mfmas = [&](int c, const u32x4(&A)[RG][CT], int bi) {
        const int ntc = chunk_nt(c);
        const unsigned char *bp = smem + boff0 + bi * buf_bytes;
        u32x4 bq[2][NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) bq[0][cb] = *(const u32x4 *)(bp + 256 * cb);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < CT; ++u) {
            if (u + 1 < CT) {
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
                    bq[(u + 1) & 1][cb] = *(const u32x4 *)(bp + (u + 1) * tstride + 256 * cb);
            }
            // (keep the reads above the MFMAs: left alone, the scheduler sinks each read to just
            // before its use to save registers, and every MFMA then waits out the LDS latency)
            __builtin_amdgcn_sched_barrier(0);
            const bool ok = u < ntc;  // wavefront-uniform
#pragma unroll
            for (int g = 0; g < RG; ++g) {
                const u32x4 zero = {0u, 0u, 0u, 0u};
                const u32x4 av = ok ? A[g][u] : zero;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
                    acc[g][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av),
                                                                         __builtin_bit_cast(bf16x8, bq[u & 1][cb]),
                                                                         acc[g][cb], 0, 0, 0);
            }
        }
        if (kCanon && ((c + 1) % nchs == 0 || c + 1 == nch)) slice_end();
    };

    u32x4 A0[RG][CT], A1[RG][CT];
    if constexpr (DMA) {
        // Pipeline: while the MFMAs of chunk c run, the B operand and the A tiles of chunk c + 1 are on their
        // way, the former straight into the other LDS buffer.  Per step: wait for this wavefront's own loads
        // of chunk c, then one barrier (everybody's part of B(c) has landed; nobody reads the other buffer).
        if (tid < 4) ((uint32_t *)smem)[tid] = 0u;
        dmaB(0, 0);
        loadA(0, A0);
        if (a.rp == 16)
            mv_norm_finish(a, mv_norm_load(a), rs, nscratch);
        else if (CANON)
            mv_norm_rows32(a, rs, nscratch);
        else
            mv_norm_rows64(a, rs, nscratch);
        auto step = [&](int c, const u32x4(&Ac)[RG][CT], int bc, u32x4(&An)[RG][CT], int bn) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            lds_barrier();
            if (c + 1 < nch) {
                dmaB(c + 1, bn);
                loadA(c + 1, An);
            }
            mfmas(c, Ac, bc);
        };
        for (int c = 0; c < nch; c += 2) {
            step(c, A0, 0, A1, 1);
            if (c + 1 < nch) step(c + 1, A1, 1, A0, 0);
        }
    } else {
        // Pipeline: while the MFMAs of chunk c run, the A tiles of chunk c + 1 and the B operand of
        // chunk c + 2 are on their way from memory, and the B operand of chunk c + 1 (loaded during
        // the previous step) is copied into the other LDS buffer.  One LDS-only barrier per step: it
        // does not wait for the loads in flight.
        u32x4 tmp[NQ];
        loadB(0, tmp);
        loadA(0, A0);
        if (tid < 4) ((uint32_t *)smem)[tid] = 0u;
        storeB(0, tmp);
        if (nch > 1) loadB(1, tmp);
        if (a.rp == 16)
            mv_norm_finish(a, mv_norm_load(a), rs, nscratch);
        else if (CANON)
            mv_norm_rows32(a, rs, nscratch);
        else
            mv_norm_rows64(a, rs, nscratch);

        auto step = [&](int c, const u32x4(&Ac)[RG][CT], int bc, u32x4(&An)[RG][CT], int bn) {
            lds_barrier();  // chunk c's B is visible; nobody reads buffer bn any more
            if (c + 1 < nch) {
                storeB(bn, tmp);
                if (c + 2 < nch) loadB(c + 2, tmp);
                loadA(c + 1, An);
            }
            mfmas(c, Ac, bc);
        };
        for (int c = 0; c < nch; c += 2) {
            step(c, A0, 0, A1, 1);
            if (c + 1 < nch) step(c + 1, A1, 1, A0, 0);
        }
    }

    // ---- per row group of the wavefront: results to LDS (dump[wave][column][tile row]), then the
    // epilogue, or with split K the partial
    float *dw = dump + (size_t)wave * (NCB * 256);
    auto y_local = [&](int r, int j) {
        const float y2 = dw[(NT * r) * 16 + j] + dw[(NT * r + 1) * 16 + j];
        return NT == 3 ? y2 + dw[(3 * r + 2) * 16 + j] : y2;
    };
    auto dump_regs = [&](const f32x4(&v)[NCB]) {
        __syncthreads();  // the B buffers / the previous dump are no longer read
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) dw[(16 * cb + col) * 16 + 4 * kg + r4] = v[cb][r4];
        __syncthreads();
    };
#pragma unroll
    for (int g = 0; g < RG; ++g) {
        const int rg = rg0 + g;
        const bool live = active && rg < a.n_rg;
        if constexpr (kCanon)
            dump_regs(ssum);  // (RG = 1) the sum of this workgroup's slices, per term
        else
            dump_regs(acc[g]);
        if (KSP == 1) {
            if (live) mv_epilogue<EPI>(a, rg, lane, rs, nullptr, y_local);
        } else if (live) {
            // publish the partial, terms combined (device-scope atomic stores write through, so the
            // release below has nothing to flush)
            float *pp = a.part + ((size_t)blockIdx.y * a.n_rg + rg) * (16 * R);
            for (int idx = lane; idx < 16 * R; idx += 64)
                __hip_atomic_store(pp + idx, y_local(idx >> 4, idx & 15), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (KSP == 1) return;
    // ---- split-K: the last workgroup of this row block to arrive reduces.
    // One release/acquire per workgroup: the barrier orders every wavefront's partial stores before
    // thread 0's device-scope read-modify-write on the counter, which publishes them (release) and,
    // in the workgroup that arrives last, makes the other workgroups' partials visible (acquire).
    // Separate fences around a relaxed atomic cost 10+ us more per launch on this multi-die part.
    __syncthreads();
    if (tid == 0) {
        const int old = __hip_atomic_fetch_add(a.counters + blockIdx.x, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        *flag = (old == KSP - 1) ? 1 : 0;
    }
    __syncthreads();
    if (*flag == 0) return;
    // (plain loads below: ordered after thread 0's acquire by the barrier)
#pragma unroll
    for (int g = 0; g < RG; ++g) {
        const int rg = rg0 + g;
        if (!active || rg >= a.n_rg) continue;
        const float *p0 = a.part + (size_t)rg * (16 * R);
        const size_t sstride = (size_t)a.n_rg * (16 * R);
        mv_epilogue<EPI>(a, rg, lane, rs, nullptr, [&](int r, int j) {
            float v[8];
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2) v[s2] = s2 < KSP ? p0[s2 * sstride + r * 16 + j] : 0.f;
            float y = v[0];
#pragma unroll
            for (int s2 = 1; s2 < 8; ++s2) y += v[s2];
            return y;
        });
    }
    if (tid == 0) a.counters[blockIdx.x] = 0;
}

template <int EPI, int NCB, int CT, int RG, bool DMA, bool CANON>
static hipError_t launch_mvN_t(const MvArgs &a, int n_cu, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_mvN<EPI, NCB, CT, RG, DMA, CANON>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMvMaxLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int NC = block_terms(a.RL) * layout_rows(a.RL);
    const size_t buf2 = 2 * (size_t)4 * CT * NC * 16;
    const size_t lds = 16 + (buf2 > (size_t)NCB * 8192 ? buf2 : (size_t)NCB * 8192) + 320 + 4096;
    const int n_rb = (a.n_rg + 8 * RG - 1) / (8 * RG);
    // split K over workgroups until about one workgroup per compute unit exists
    // (never more workgroups than compute units: one workgroup fills a compute unit's registers,
    // so a partial second round would double the kernel's duration)
    int ksp = n_cu / n_rb;
    if (ksp < 1) ksp = 1;
    if (ksp > 8) ksp = 8;
    int TS;
    if (CANON) {
        TS = ((a.T + 7) / 8) * mv_slice_group(a, n_cu);
    } else {
        while (ksp > 1 && ((a.T + ksp - 1) / ksp < 8 || (int64_t)a.n_rg * ksp > a.part_capacity)) --ksp;
        TS = (a.T + ksp - 1) / ksp;
    }
    ksp = (a.T + TS - 1) / TS;  // workgroups whose K range holds tiles
    // With fewer workgroups than compute units, a workgroup takes fewer row groups, so that every compute unit
    // gets about the same share: what bounds these launches is what ONE compute unit can take in (weights plus
    // its copy of the activation), not the chip's HBM rate.
    int rpw = 8, grid_x = n_rb;
    if (n_rb * ksp < n_cu) {
        rpw = (a.n_rg * ksp + RG * n_cu - 1) / (RG * n_cu);
        if (rpw < 4) rpw = 4;
        if (rpw > 8) rpw = 8;
        grid_x = (a.n_rg + rpw * RG - 1) / (rpw * RG);
    }
    return launch_maybe_timed(k_mvN<EPI, NCB, CT, RG, DMA, CANON>, dim3(grid_x, ksp), dim3(512), lds, s, a, TS, rpw);
}

int mv_split_slots(const MvArgs &a, int n_cu) {
    if (a.RL & kBulkLayout) return a.part_capacity;  // (bulk layouts: not needed by callers)
    if (a.R <= kMvSmallRows && mv1_lds_bytes(a.K, a.R, a.head_dim) <= kMvMaxLds) return 0;  // LDS-resident kernel
    const int TS = ((a.T + 7) / 8) * mv_slice_group(a, n_cu);
    const int ksp = (a.T + TS - 1) / TS;
    return ksp > 1 ? ksp * a.n_rg : 0;
}

hipError_t launch_mv(int epi, MvArgs a, int n_cu, int ks_override, int wg_override, hipStream_t s) {
    const bool bulk = (a.RL & kBulkLayout) != 0;
    const int lrows = layout_rows(a.RL);
    if (a.R < 1 || a.R > kMaxBlockRows || (a.rp != 16 && a.rp != 64) || a.R > a.rp || a.R > lrows ||
        (bulk ? (lrows != 32 && lrows != 64) : (lrows != a.R || lrows > kMaxRows)))
        return hipErrorInvalidValue;
    // small blocks (in their own exact layout) whose whole activation fits in LDS take the single-pass kernel
    if (!bulk && a.R <= kMvSmallRows && ks_override != 16 && mv1_lds_bytes(a.K, a.R, a.head_dim) <= kMvMaxLds)
        return launch_mv1(epi, a, n_cu, ks_override, wg_override, s);
    // exact layouts (up to 32 rows): 1-6 column blocks of three-term columns, K chunks of 8 tiles, the fixed
    // summation order; bulk layouts of 32 / 64 rows (prefill, candidate evaluation): 4 / 8 column blocks of
    // two-term columns
    const int ncb = (block_terms(a.RL) * lrows + 15) / 16;
#define SWIFT_MVN_CASE(E)                                                                \
    case E:                                                                              \
        if (bulk) switch (ncb) {                                                         \
                case 4: return launch_mvN_t<E, 4, 8, 1, true, false>(a, n_cu, s);        \
                case 8: return launch_mvN_t<E, 8, 8, 1, true, false>(a, n_cu, s);        \
                default: return hipErrorInvalidValue;                                    \
            }                                                                            \
        switch (ncb) {                                                                   \
            case 1: return launch_mvN_t<E, 1, 8, 1, false, true>(a, n_cu, s);            \
            case 2: return launch_mvN_t<E, 2, 8, 1, false, true>(a, n_cu, s);            \
            case 3: return launch_mvN_t<E, 3, 8, 1, false, true>(a, n_cu, s);            \
            case 4: return launch_mvN_t<E, 4, 8, 1, false, true>(a, n_cu, s);            \
            case 5: return launch_mvN_t<E, 5, 8, 1, false, true>(a, n_cu, s);            \
            case 6: return launch_mvN_t<E, 6, 8, 1, false, true>(a, n_cu, s);            \
            default: return hipErrorInvalidValue;                                        \
        }
    switch (epi) {
        SWIFT_MVN_CASE(EPI_QKV)
        SWIFT_MVN_CASE(EPI_RESID)
        SWIFT_MVN_CASE(EPI_SWIGLU)
        SWIFT_MVN_CASE(EPI_LOGITS)
    }
#undef SWIFT_MVN_CASE
    return hipErrorInvalidValue;
}

}  // namespace swift
