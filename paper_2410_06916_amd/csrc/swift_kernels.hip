// gfx950 kernels of the draft / verify forward pass: storage-generic single-row projections,
// attention over the cache, arg-max/confidence, utilities.
//
// Every projection of the decoder is a weight-streaming pass: the weight matrix is read
// from HBM exactly once with 128-bit loads, the activation vector lives in LDS, and the
// operation that follows the projection (rotation + cache append, SwiGLU, residual add)
// runs in the same kernel on the finished dot products.  Wavefronts are 64 lanes wide;
// one wavefront owns two output rows at a time so that the rows an epilogue needs
// together (a rotary pair, a gate/up pair) are produced by the same wavefront.
#include "swift_kernels.h"
#include "swift_attn.h"

#include <math.h>
#include <stdio.h>

#include "swift_device.h"

namespace swift {

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
// attention over the cache for a block of query rows, split over the cache length
// ------------------------------------------------------------------------------------------
// Workgroup (kv head g, split sp, row block rb) handles `chunk` cache slots for the query heads
// that share kv head g and for RB consecutive block rows, which share every key/value load; row r
// attends slots [0, n_ctx + r).  A group of LPP = d / VEC lanes owns one cache slot at a time (lane j
// of the group holds elements [j*VEC, (j+1)*VEC) of that slot's key and value); step s of wavefront w
// covers slots lo + (4 s + w) * SPW .., so the four wavefronts read consecutive slots, and the loads
// of NB steps are issued together.  Each lane group keeps a running (max, sum, weighted value) per
// (row, query head) (online softmax); groups, then wavefronts, are merged.  A row whose range ends in
// the first chunk is normalised and written directly; otherwise the workgroup writes the row's partial
// and k_attn_combine merges the partials in split order.  What a row's result is does not depend on
// which other rows share its workgroup: slots beyond a row's range leave its running values untouched.
// TREE: the rows are those of a token tree (attn_row_ctx, attn_phys_slot); each row then has a slot of its
// own inside its range, so rows do not share loads (RB = 1).
template <typename T, int GROUP, int RB, bool TREE = false>
__global__ __launch_bounds__(256) void k_attn_split(AttnArgs a, int chunk) {
    static_assert(!TREE || RB == 1, "tree rows do not share key/value loads");
    constexpr int VEC = T::VEC;
    constexpr int NB = GROUP <= 2 ? 4 : 1;
    constexpr int M = GROUP * RB;  // members: (row rr, head h) -> rr * GROUP + h
    const int d = a.head_dim;
    const int LPP = d / VEC;   // lanes per cache slot (power of two, <= 32)
    const int SPW = 64 / LPP;  // slots per wavefront step
    const int n_split = gridDim.y;
    const int g = blockIdx.x, sp = blockIdx.y, row0 = blockIdx.z * RB;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lj = lane & (LPP - 1), lg = lane / LPP;
    const int lo = sp * chunk;
    const int n_rows = min(RB, a.rows - row0);
    // end of the longest row's range here
    const int hi_max = min(TREE ? attn_row_ctx<TREE>(a, row0) : a.n_ctx + row0 + n_rows - 1, lo + chunk);
    if (hi_max <= lo) return;  // no row of this block reaches this chunk
    const float scale = 1.0f / sqrtf((float)d);
    const int nq = a.n_q_heads;

    float q[M][VEC];
    int lim[M];
#pragma unroll
    for (int mm = 0; mm < M; ++mm) {
        const int rr = mm / GROUP, h = mm - rr * GROUP;
        const int row = min(row0 + rr, a.rows - 1);
        // block row r sees the cache up to its own slot; rows past the block take part in nothing
        lim[mm] = rr < n_rows ? min(attn_row_ctx<TREE>(a, row0 + rr), lo + chunk) : 0;
#pragma unroll
        for (int j = 0; j < VEC; ++j) q[mm][j] = a.q[((size_t)row * nq + g * GROUP + h) * d + lj * VEC + j];
    }

    float m[M], l[M], o[M][VEC];
#pragma unroll
    for (int mm = 0; mm < M; ++mm) {
        m[mm] = -INFINITY;
        l[mm] = 0.f;
#pragma unroll
        for (int j = 0; j < VEC; ++j) o[mm][j] = 0.f;
    }

    const typename T::elem *kc = (const typename T::elem *)a.kcache + (size_t)g * a.max_seq * d;
    const typename T::elem *vc = (const typename T::elem *)a.vcache + (size_t)g * a.max_seq * d;
    const int steps = (hi_max - lo + 4 * SPW - 1) / (4 * SPW);

    for (int s0 = 0; s0 < steps; s0 += NB) {
        u32x4 kv[NB], vv[NB];
        int pos[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int p = lo + ((s0 + b) * 4 + wave) * SPW + lg;
            // clamp: slots past the range are loaded and discarded
            const int pc = attn_phys_slot<TREE>(a, row0, min(p, hi_max - 1));
            pos[b] = p;
            kv[b] = *(const u32x4 *)(kc + (size_t)pc * d + lj * VEC);
            vv[b] = *(const u32x4 *)(vc + (size_t)pc * d + lj * VEC);
        }
        attn_batch<T, M, NB>(kv, vv, pos, lim, q, scale, LPP, m, l, o);
    }

    // merge lane groups of one wavefront (butterfly over the lane bits above LPP)
#pragma unroll
    for (int mm = 0; mm < M; ++mm) {
        for (int off = LPP; off < 64; off <<= 1) {
            const float m2 = __shfl_xor(m[mm], off, 64);
            const float l2 = __shfl_xor(l[mm], off, 64);
            const float mn = fmaxf(m[mm], m2);
            const float c1 = (m[mm] == -INFINITY) ? 0.f : __expf(m[mm] - mn);
            const float c2 = (m2 == -INFINITY) ? 0.f : __expf(m2 - mn);
            l[mm] = l[mm] * c1 + l2 * c2;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const float o2 = __shfl_xor(o[mm][j], off, 64);
                o[mm][j] = o[mm][j] * c1 + o2 * c2;
            }
            m[mm] = mn;
        }
    }

    // merge the four wavefronts through LDS
    __shared__ float sm[4][M], sl[4][M];
    __shared__ float so[4][M][128];
    if (lg == 0) {
#pragma unroll
        for (int mm = 0; mm < M; ++mm) {
            if (lj == 0) {
                sm[wave][mm] = m[mm];
                sl[wave][mm] = l[mm];
            }
#pragma unroll
            for (int j = 0; j < VEC; ++j) so[wave][mm][lj * VEC + j] = o[mm][j];
        }
    }
    __syncthreads();

    const int ocode = a.out_rows ? a.out_rows : a.rows, orows = layout_rows(ocode);
    for (int idx = tid; idx < M * d; idx += 256) {
        const int mm = idx / d, j = idx - mm * d;
        const int rr = mm / GROUP, h = mm - rr * GROUP;
        const int row = row0 + rr;
        if (rr >= n_rows) continue;                      // no such row
        const int n_ctx = attn_row_ctx<TREE>(a, row);
        if (lo >= n_ctx) continue;                       // the row ends before this chunk
        const int ns_row = (n_ctx + chunk - 1) / chunk;  // splits this row really has
        const float mn = fmaxf(fmaxf(sm[0][mm], sm[1][mm]), fmaxf(sm[2][mm], sm[3][mm]));
        float ls = 0.f, os = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float c = (sm[w][mm] == -INFINITY) ? 0.f : __expf(sm[w][mm] - mn);
            ls += sl[w][mm] * c;
            os += so[w][mm][j] * c;
        }
        if (ns_row == 1) {
            const float y = os / ls;
            const int e = (g * GROUP + h) * d + j;
            if (a.out) a.out[(size_t)row * nq * d + e] = y;
            if (a.out_s) {
                uint16_t hi16, mid16, lo16;
                split3(y, hi16, mid16, lo16);
                const int nt = block_terms(ocode);
                uint16_t *p = a.out_s + ((size_t)(e >> 3) * (nt * orows) + nt * row) * 8 + (e & 7);
                p[0] = hi16;
                p[8] = mid16;
                if (nt == 3) p[16] = lo16;
            }
        } else {
            const size_t slot = ((size_t)row * nq + g * GROUP + h) * n_split + sp;
            a.part_o[slot * d + j] = os;
            if (j == 0) {
                a.part_ml[slot * 2 + 0] = mn;
                a.part_ml[slot * 2 + 1] = ls;
            }
        }
    }
}

// Merges the split partials of every (row, head) in split order and writes the result.  A second
// launch rather than a last-arriver merge inside k_attn_split: publishing the partials device-wide
// from inside the kernel measured slower than this launch on this multi-die part (by 5 us per layer
// at 7600 cache slots).
__global__ void k_attn_combine(AttnArgs a, int chunk, int n_split) {
    const int head = blockIdx.x, row = blockIdx.y, d = a.head_dim;
    const int ns = ((a.tree ? attn_row_ctx<true>(a, row) : attn_row_ctx<false>(a, row)) + chunk - 1) / chunk;
    if (ns == 1) return;  // written directly by the split kernel
    const size_t base = ((size_t)row * a.n_q_heads + head) * n_split;
    float M = -INFINITY;
    for (int s = 0; s < ns; ++s) M = fmaxf(M, a.part_ml[(base + s) * 2]);
    for (int j = threadIdx.x; j < d; j += blockDim.x) {
        float L = 0.f, O = 0.f;
        for (int s = 0; s < ns; ++s) {
            const float c = __expf(a.part_ml[(base + s) * 2] - M);
            L += a.part_ml[(base + s) * 2 + 1] * c;
            O += a.part_o[(base + s) * d + j] * c;
        }
        const float y = O / L;
        const int e = head * d + j;
        if (a.out) a.out[(size_t)row * a.n_q_heads * d + e] = y;
        if (a.out_s) {
            uint16_t hi, mid, lo;
            split3(y, hi, mid, lo);
            const int ocode = a.out_rows ? a.out_rows : a.rows, orows = layout_rows(ocode), nt = block_terms(ocode);
            // (a prompt macro block: the row's sub-block has an output buffer of its own)
            const int z = a.sub_rows ? row / a.sub_rows : 0, r = row - z * a.sub_rows;
            uint16_t *p = a.out_s + (size_t)z * a.sub_out_s + ((size_t)(e >> 3) * (nt * orows) + nt * r) * 8 + (e & 7);
            p[0] = hi;
            p[8] = mid;
            if (nt == 3) p[16] = lo;
        }
    }
}

// Short contexts: one workgroup of kAttnHeadWaves wavefronts per (kv head, block row) walks the whole cache
// range (attn_head_unit), so nothing goes through global memory and one launch suffices.
constexpr int kAttnHeadWaves = 8;  // wavefronts of a one-workgroup-per-head attention workgroup
template <typename T, int GROUP, bool TREE, int RB>
__global__ __launch_bounds__(64 * kAttnHeadWaves) void k_attn_head(AttnArgs a) {
    extern __shared__ __align__(16) float sh[];
    attn_head_unit<T, GROUP, TREE, RB, kAttnHeadWaves>(a, blockIdx.x, blockIdx.y * RB, sh);
}

template <typename T, int GROUP, bool TREE, int RB>
static hipError_t launch_attn_head_tt(const AttnArgs &a, hipStream_t s) {
    constexpr int M = GROUP * RB;
    const size_t lds = (size_t)(2 * kAttnHeadWaves * M + kAttnHeadWaves * M * a.head_dim) * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_attn_head<T, GROUP, TREE, RB>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((k_attn_head<T, GROUP, TREE, RB>), dim3(a.n_kv_heads, (a.rows + RB - 1) / RB),
                       dim3(64 * kAttnHeadWaves), lds, s, a);
    return hipGetLastError();
}
// Which attention kernel instance a launch takes.  Which kernel runs, and where the cache range is cut,
// depends on the cache capacity and the head count only, never on the current length; the number of block
// rows only decides how many rows share a workgroup's key/value loads, which changes no row's result.
struct AttnPlan {
    bool head;     // one workgroup per (kv head, row block) over the whole range; else split over the cache length
    int group;     // query heads per kv head
    int rb;        // block rows that share a workgroup's loads
    int chunk;     // split kernel: cache slots per workgroup
    int n_split;   // split kernel: ranges the longest row reaches
};
template <typename T>
static AttnPlan attn_plan(const AttnArgs &a, int n_cu) {
    AttnPlan p{};
    p.group = a.n_q_heads / a.n_kv_heads;
    // The one-workgroup-per-head kernel needs enough kv heads to occupy the chip with a single row.
    p.head = attn_uses_head_kernel(a.max_seq, a.n_kv_heads);
    if (p.head) {
        // Blocks with more (head, row) pairs than compute units: two rows share every key/value load where the
        // registers allow it, so that a compute unit does not read a head's cache twice (7B, 9 rows: 19 -> 15 us
        // per layer; with fewer pairs the one-row workgroups are faster: 13 against 15.5 us at 4 rows).
        p.rb = (!a.tree && p.group == 1 && a.rows * a.n_kv_heads > n_cu) ? 2 : 1;
        return p;
    }
    // longest row of the block (a tree: an upper bound; workgroups beyond a row's range leave at once)
    const int ctx = a.tree ? a.n_base + a.row_base + a.rows : a.n_ctx + a.rows - 1;
    const int d = a.head_dim, VEC = T::VEC, SPW = 64 / (d / VEC);
    const int gran = 4 * SPW;  // slots one workgroup step covers
    // chunk length: a full cache cut into enough pieces for about two workgroups per compute unit with one row
    int want = (2 * n_cu + a.n_kv_heads - 1) / a.n_kv_heads;
    if (want > a.max_split) want = a.max_split;
    if (want < 1) want = 1;
    p.chunk = (a.max_seq + want - 1) / want;
    p.chunk = (p.chunk + gran - 1) / gran * gran;
    p.n_split = (ctx + p.chunk - 1) / p.chunk;  // <= want <= max_split
    // Block rows that share their key/value loads in one workgroup (the more, the less cache traffic; bounded
    // by registers: members = heads per kv head x rows).  One to three rows take the instance with as many
    // members: the same arithmetic per row without the idle members' share of the vector arithmetic.
    if (a.tree)
        p.rb = 1;
    else if (p.group == 1)
        p.rb = a.rows < 4 ? a.rows : 4;
    else if (p.group == 2)
        p.rb = a.rows == 1 ? 1 : 2;
    else
        p.rb = 1;
    return p;
}

template <typename T>
static hipError_t launch_attn_t(const AttnArgs &a, int n_cu, hipStream_t s) {
    if (a.tree && (a.row_base < 0 || a.row_base + a.rows > kMaxRows)) return hipErrorInvalidValue;
    const AttnPlan p = attn_plan<T>(a, n_cu);
    if (p.head) {
#define SWIFT_HEAD_CASE(G)                                                            \
    case G:                                                                           \
        if (a.tree) return launch_attn_head_tt<T, G, true, 1>(a, s);                  \
        if (G == 1 && p.rb == 2) return launch_attn_head_tt<T, 1, false, 2>(a, s);    \
        return launch_attn_head_tt<T, G, false, 1>(a, s);
        switch (p.group) {
            SWIFT_HEAD_CASE(1)
            SWIFT_HEAD_CASE(2)
            SWIFT_HEAD_CASE(4)
            SWIFT_HEAD_CASE(8)
            default: return hipErrorInvalidValue;
        }
#undef SWIFT_HEAD_CASE
    }
    const int chunk = p.chunk, n_split = p.n_split;
    dim3 grid(a.n_kv_heads, n_split, (a.rows + p.rb - 1) / p.rb), block(256);
#define SWIFT_SPLIT(G, RB, TREE) hipLaunchKernelGGL((k_attn_split<T, G, RB, TREE>), grid, block, 0, s, a, chunk)
    const int key = p.group * 100 + p.rb * 10 + (a.tree ? 1 : 0);
    switch (key) {
        case 111: SWIFT_SPLIT(1, 1, true); break;
        case 211: SWIFT_SPLIT(2, 1, true); break;
        case 411: SWIFT_SPLIT(4, 1, true); break;
        case 811: SWIFT_SPLIT(8, 1, true); break;
        case 110: SWIFT_SPLIT(1, 1, false); break;
        case 120: SWIFT_SPLIT(1, 2, false); break;
        case 130: SWIFT_SPLIT(1, 3, false); break;
        case 140: SWIFT_SPLIT(1, 4, false); break;
        case 210: SWIFT_SPLIT(2, 1, false); break;
        case 220: SWIFT_SPLIT(2, 2, false); break;
        case 410: SWIFT_SPLIT(4, 1, false); break;
        case 810: SWIFT_SPLIT(8, 1, false); break;
        default: return hipErrorInvalidValue;
    }
#undef SWIFT_SPLIT
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_split == 1) return e;
    hipLaunchKernelGGL(k_attn_combine, dim3(a.n_q_heads, a.rows), dim3(a.head_dim < 64 ? 64 : a.head_dim), 0, s, a, chunk,
                       n_split);
    return hipGetLastError();
}

size_t attn_partial_floats(int dtype, const AttnArgs &a, int n_cu) {
    const AttnPlan p = dtype == F32 ? attn_plan<F32T>(a, n_cu) : attn_plan<BF16T>(a, n_cu);
    if (p.head) return 0;
    const int max_splits = (a.max_seq + p.chunk - 1) / p.chunk;
    return (size_t)a.rows * a.n_q_heads * max_splits * a.head_dim;
}

int attn_path_name(int dtype, const AttnArgs &a, int n_cu, char *out, int capacity) {
    const AttnPlan p = dtype == F32 ? attn_plan<F32T>(a, n_cu) : attn_plan<BF16T>(a, n_cu);
    return snprintf(out, (size_t)capacity, "%s<%s, group %d, rows %d%s>", p.head ? "head" : "split",
                    dtype == F32 ? "f32" : "bf16", p.group, p.rb, a.tree ? ", tree" : "");
}

hipError_t launch_attn_combine(const AttnArgs &a, int chunk, int n_split, hipStream_t s) {
    hipLaunchKernelGGL(k_attn_combine, dim3(a.n_q_heads, a.rows), dim3(a.head_dim < 64 ? 64 : a.head_dim), 0, s, a, chunk,
                       n_split);
    return hipGetLastError();
}

hipError_t launch_attn_decode(int dtype, const AttnArgs &a, int n_cu, hipStream_t s) {
    return dtype == F32 ? launch_attn_t<F32T>(a, n_cu, s) : launch_attn_t<BF16T>(a, n_cu, s);
}

// ------------------------------------------------------------------------------------------
// greedy choice + confidence:  token = first arg-max, conf = 1 / sum exp(l - max)
// ------------------------------------------------------------------------------------------
template <bool TOPK>
__global__ __launch_bounds__(1024) void k_argmax_conf(ArgmaxArgs a) {
    const float *lg = a.logits + (size_t)blockIdx.x * a.V;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ float smax[16];
    __shared__ int sidx[16];
    __shared__ float ssum[16];
    float best = -INFINITY;
    int bi = 0x7fffffff;
    // up to 32 logits per thread stay in registers (one round of loads, all in flight together)
    constexpr int PT = 32;
    const bool in_regs = a.V <= 1024 * PT;
    float v[PT];
    if (in_regs) {
#pragma unroll
        for (int k = 0; k < PT; ++k) {
            const int i = tid + 1024 * k;
            v[k] = i < a.V ? lg[i] : -INFINITY;
        }
#pragma unroll
        for (int k = 0; k < PT; ++k)
            if (v[k] > best) {  // i increases with k, so the first maximum is kept
                best = v[k];
                bi = tid + 1024 * k;
            }
    } else {
        for (int i = tid; i < a.V; i += 1024) {
            const float x = lg[i];
            if (x > best) {  // i increases per thread, so the first maximum is kept
                best = x;
                bi = i;
            }
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
    // nothing compared greater than -inf (a row of NaN or -inf only): token 0, like a scan that starts
    // from index 0 and moves on strict improvement only
    if (bi == 0x7fffffff) bi = 0;
    float sum = 0.f;
    if (in_regs) {
#pragma unroll
        for (int k = 0; k < PT; ++k)
            if (tid + 1024 * k < a.V) sum += expf(v[k] - best);
    } else {
        for (int i = tid; i < a.V; i += 1024) sum += expf(lg[i] - best);
    }
    sum = wave_sum(sum);
    if (lane == 0) ssum[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int w = 0; w < 16; ++w) t += ssum[w];
        a.tokens[blockIdx.x] = bi;
        a.conf[blockIdx.x] = 1.0f / t;
    }
    if (!TOPK) return;
    // the next largest logits, one per round: strike the last winner out, find the first maximum again
    __shared__ int taken[kTopK];
    if (tid == 0) {
        taken[0] = bi;
        a.topk[(size_t)blockIdx.x * kTopK] = bi;
    }
    for (int j = 1; j < a.n_topk; ++j) {
        __syncthreads();  // taken[j-1] is written; the previous round's reads of smax/sidx are done
        best = -INFINITY;
        bi = 0x7fffffff;
        if (in_regs) {
            const int last = taken[j - 1];
#pragma unroll
            for (int k = 0; k < PT; ++k) {
                if (tid + 1024 * k == last) v[k] = -INFINITY;
                if (v[k] > best) {
                    best = v[k];
                    bi = tid + 1024 * k;
                }
            }
            // (a struck-out logit and a real -inf logit look alike: real ones are told apart below)
        } else {
            for (int i = tid; i < a.V; i += 1024) {
                bool free_ = true;
                for (int t = 0; t < j; ++t) free_ &= taken[t] != i;
                const float x = lg[i];
                if (free_ && x > best) {
                    best = x;
                    bi = i;
                }
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
        if (bi == 0x7fffffff) {
            // only -inf logits are left: the lowest index not taken yet
            int i = 0;
            for (bool again = true; again;) {
                again = false;
                for (int t = 0; t < j; ++t)
                    if (taken[t] == i) {
                        ++i;
                        again = true;
                    }
            }
            bi = i;
        }
        if (tid == 0) {
            taken[j] = bi;
            a.topk[(size_t)blockIdx.x * kTopK + j] = bi;
        }
    }
}

hipError_t launch_argmax_conf(const ArgmaxArgs &a, hipStream_t s) {
    if (a.topk) {
        if (a.n_topk < 1 || a.n_topk > kTopK) return hipErrorInvalidValue;
        hipLaunchKernelGGL(k_argmax_conf<true>, dim3(a.rows), dim3(1024), 0, s, a);
    } else {
        hipLaunchKernelGGL(k_argmax_conf<false>, dim3(a.rows), dim3(1024), 0, s, a);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// cache compaction after acceptance on a token tree
// ------------------------------------------------------------------------------------------
// Workgroup (kv head, plane) carries out the moves in order; element e of every move is handled by the
// same thread, so a move that overwrites the source of an earlier one comes after that one's read.
template <typename T>
__global__ void k_kv_move(KvMoveArgs a) {
    const int layer = blockIdx.y >> 1, is_v = blockIdx.y & 1, d = a.head_dim;
    typename T::elem *plane = (typename T::elem *)a.kv + (size_t)layer * a.layer_elems + (is_v ? a.v_offset : 0);
    if (is_v && a.nb32 > 0) {
        for (int i = 0; i < a.n_moves; ++i)
            for (int e = threadIdx.x; e < d; e += blockDim.x)
                plane[kv_vt_index(blockIdx.x, a.nb32, d, a.dst[i], e)] = plane[kv_vt_index(blockIdx.x, a.nb32, d, a.src[i], e)];
        return;
    }
    typename T::elem *p = plane + (size_t)blockIdx.x * a.max_seq * d;
    for (int i = 0; i < a.n_moves; ++i) {
        const typename T::elem *src = p + (size_t)a.src[i] * d;
        typename T::elem *dst = p + (size_t)a.dst[i] * d;
        for (int e = threadIdx.x; e < d; e += blockDim.x) dst[e] = src[e];
    }
}

hipError_t launch_kv_move(int dtype, const KvMoveArgs &a, hipStream_t s) {
    if (a.n_moves <= 0) return hipSuccess;
    if (a.n_moves > 32) return hipErrorInvalidValue;
    for (int i = 0; i < a.n_moves; ++i)
        if (a.src[i] < 0 || a.src[i] >= a.max_seq || a.dst[i] < 0 || a.dst[i] >= a.max_seq) return hipErrorInvalidValue;
    dim3 grid(a.n_kv_heads, 2 * a.n_layers), block(a.head_dim < 64 ? 64 : a.head_dim > 256 ? 256 : a.head_dim);
    if (dtype == F32)
        hipLaunchKernelGGL(k_kv_move<F32T>, grid, block, 0, s, a);
    else
        hipLaunchKernelGGL(k_kv_move<BF16T>, grid, block, 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// the transposed value layout (bf16; kv_vt_index): test and debug helpers
// ------------------------------------------------------------------------------------------
// NaN-fills every value of slots >= first_slot of every kv head of one layer's value plane.
__global__ void k_vt_poison(uint16_t *plane, int n_kv, int nb32, int d, int first_slot) {
    const int64_t per_head = (int64_t)nb32 * 32 * d;
    const int64_t first = (int64_t)(first_slot >> 3) * d * 8;  // groups below hold committed slots only
    const int64_t n = (int64_t)n_kv * (per_head - first);
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t h = i / (per_head - first), r = first + i % (per_head - first);
        const int slot = (int)(r / ((int64_t)d * 8)) * 8 + (int)(r & 7);
        if (slot >= first_slot) plane[h * per_head + r] = 0x7fc0;
    }
}
hipError_t launch_vt_poison(void *plane, int n_kv, int nb32, int d, int first_slot, hipStream_t s) {
    hipLaunchKernelGGL(k_vt_poison, dim3(1024), dim3(256), 0, s, (uint16_t *)plane, n_kv, nb32, d, first_slot);
    return hipGetLastError();
}
// dst[h * d + e] = value element e of slot `slot` of kv head h
__global__ void k_vt_read(const uint16_t *plane, int n_kv, int nb32, int d, int slot, float *dst) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_kv * d) dst[i] = __uint_as_float((uint32_t)plane[kv_vt_index(i / d, nb32, d, slot, i % d)] << 16);
}
hipError_t launch_vt_read(const void *plane, int n_kv, int nb32, int d, int slot, float *dst, hipStream_t s) {
    hipLaunchKernelGGL(k_vt_read, dim3((n_kv * d + 255) / 256), dim3(256), 0, s, (const uint16_t *)plane, n_kv, nb32, d, slot, dst);
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

__global__ void k_fill_u32(uint32_t *p, uint32_t v, int64_t n) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

hipError_t launch_fill_u32(void *p, uint32_t v, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    int grid = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    hipLaunchKernelGGL(k_fill_u32, dim3(grid), dim3(256), 0, s, (uint32_t *)p, v, n);
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

}  // namespace swift
