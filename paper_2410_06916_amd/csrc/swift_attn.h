// Attention device code of the row-at-a-time attention kernels.
#pragma once
#include <math.h>

#include "swift_device.h"
#include "swift_kernels.h"

namespace swift {

// ------------------------------------------------------------------------------------------
// attention: shared inner step
// ------------------------------------------------------------------------------------------
// Sum over the lanes that share one cache slot.  Sixteen lanes are one DPP row: butterfly inside
// quads, then half-row and row mirrors (every lane ends with the total), four single instructions.
__device__ inline float slot_sum(float v, int lpp) {
    if (lpp == 16) {
        v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
        v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
        v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));  // row_half_mirror
        v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));  // row_mirror
        return v;
    }
    for (int off = lpp >> 1; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// One batch of NB cache slots per lane group against GROUP query heads: scores, one running-max
// update for the whole batch, probabilities, weighted values (online softmax).
// Member h (a query head, or a (row, query head) pair when several block rows share the loads) takes
// part in slot pos[b] iff pos[b] < lim[h].
template <typename T, int GROUP, int NB>
__device__ inline void attn_batch(const u32x4 (&kv)[NB], const u32x4 (&vv)[NB], const int (&pos)[NB],
                                  const int (&lim)[GROUP], const float (&q)[GROUP][T::VEC], float scale, int lpp,
                                  float (&m)[GROUP], float (&l)[GROUP], float (&o)[GROUP][T::VEC]) {
    constexpr int VEC = T::VEC;
    float vf[NB][VEC];
#pragma unroll
    for (int b = 0; b < NB; ++b) T::unpack(vv[b], vf[b]);
    float sc[GROUP][NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        float kf[VEC];
        T::unpack(kv[b], kf);
#pragma unroll
        for (int h = 0; h < GROUP; ++h) {
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < VEC; ++j) s = fmaf(q[h][j], kf[j], s);
            s = slot_sum(s, lpp) * scale;
            sc[h][b] = pos[b] < lim[h] ? s : -INFINITY;
        }
    }
#pragma unroll
    for (int h = 0; h < GROUP; ++h) {
        float mn = m[h];
#pragma unroll
        for (int b = 0; b < NB; ++b) mn = fmaxf(mn, sc[h][b]);
        if (mn == -INFINITY) continue;  // nothing live yet
        const float corr = __expf(m[h] - mn);  // exp(-inf) = 0 on the first live batch
        float pr[NB], ps = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            pr[b] = __expf(sc[h][b] - mn);
            ps += pr[b];
        }
        l[h] = l[h] * corr + ps;
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            float acc = o[h][j] * corr;
#pragma unroll
            for (int b = 0; b < NB; ++b) acc = fmaf(pr[b], vf[b][j], acc);
            o[h][j] = acc;
        }
        m[h] = mn;
    }
}

// Cache slots launch row `row` attends (it walks logical slots [0, this value)).
template <bool TREE>
__device__ inline int attn_row_ctx(const AttnArgs &a, int row) {
    if constexpr (TREE)
        return a.n_base + (int)a.tt.depth[(a.row_base + row) & (kMaxRows - 1)] + 1;
    else
        return a.n_ctx + row;
}
// Where logical slot p of launch row `row` lives in the cache (p < attn_row_ctx).  A chain row's logical
// slots are the physical ones; a tree row's slots beyond the committed prefix are those of the rows on
// its path from the root.
template <bool TREE>
__device__ inline int attn_phys_slot(const AttnArgs &a, int row, int p) {
    if constexpr (TREE) {
        const int lvl = p - a.n_base;
        if (lvl < 0) return p;
        const int depth = (int)a.tt.depth[(a.row_base + row) & (kMaxRows - 1)];
        return a.n_base + (lvl < depth ? (int)a.tt.spine[lvl & (kMaxRows - 1)] : a.row_base + row);
    } else {
        return p;
    }
}

// One workgroup of NW wavefronts (64 NW threads, all of them call this) computes the attention of
// block row `row` for the GROUP query heads that share kv head g over the row's whole range of
// attn_row_ctx slots.  Step s of wavefront w covers slots (NW s + w) * SPW ..; the loads of NB steps
// are issued together.  sh: LDS, [NW*M] max, [NW*M] sum, [NW*M*d] weighted values (M members).
template <typename T, int GROUP, bool TREE = false, int RB = 1, int NW = 16>
__device__ inline void attn_head_unit(const AttnArgs &a, int g, int row0, float *sh) {
    // RB consecutive block rows share every key/value load (chain rows only: a tree row has a slot of its
    // own inside its range).  Members: (row rr, head h) -> rr * GROUP + h.  What a row's result is does not
    // depend on the rows that share its workgroup: slots beyond a row's range leave its running values
    // untouched.
    static_assert(!TREE || RB == 1, "tree rows do not share key/value loads");
    constexpr int VEC = T::VEC;
    constexpr int M = GROUP * RB;
    constexpr int NB = M <= 2 ? 4 : 1;
    const int d = a.head_dim;
    const int LPP = d / VEC, SPW = 64 / LPP;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lj = lane & (LPP - 1), lg = lane / LPP;
    const int n_rows = min(RB, a.rows - row0);
    const int n_ctx = attn_row_ctx<TREE>(a, row0 + n_rows - 1);  // the longest row's range
    const float scale = 1.0f / sqrtf((float)d);
    const int nq = a.n_q_heads;
    float *sm = sh, *sl = sh + NW * M, *so = sh + 2 * NW * M;

    float q[M][VEC];
    int lim[M];
#pragma unroll
    for (int mm = 0; mm < M; ++mm) {
        const int rr = mm / GROUP, h = mm - rr * GROUP;
        const int row = min(row0 + rr, a.rows - 1);
        lim[mm] = rr < n_rows ? attn_row_ctx<TREE>(a, row0 + rr) : 0;  // rows past the block take part in nothing
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
    const int steps = (n_ctx + NW * SPW - 1) / (NW * SPW);

    for (int s0 = 0; s0 < steps; s0 += NB) {
        u32x4 kv[NB], vv[NB];
        int pos[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int p = ((s0 + b) * NW + wave) * SPW + lg;
            const int pc = attn_phys_slot<TREE>(a, row0, min(p, n_ctx - 1));
            pos[b] = p;
            kv[b] = *(const u32x4 *)(kc + (size_t)pc * d + lj * VEC);
            vv[b] = *(const u32x4 *)(vc + (size_t)pc * d + lj * VEC);
        }
        attn_batch<T, M, NB>(kv, vv, pos, lim, q, scale, LPP, m, l, o);
    }
    // merge the lane groups of a wavefront
#pragma unroll
    for (int h = 0; h < M; ++h) {
        for (int off = LPP; off < 64; off <<= 1) {
            const float m2 = __shfl_xor(m[h], off, 64);
            const float l2 = __shfl_xor(l[h], off, 64);
            const float mn = fmaxf(m[h], m2);
            const float c1 = (m[h] == -INFINITY) ? 0.f : __expf(m[h] - mn);
            const float c2 = (m2 == -INFINITY) ? 0.f : __expf(m2 - mn);
            l[h] = l[h] * c1 + l2 * c2;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const float o2 = __shfl_xor(o[h][j], off, 64);
                o[h][j] = o[h][j] * c1 + o2 * c2;
            }
            m[h] = mn;
        }
    }
    if (lg == 0) {
#pragma unroll
        for (int h = 0; h < M; ++h) {
            if (lj == 0) {
                sm[wave * M + h] = m[h];
                sl[wave * M + h] = l[h];
            }
#pragma unroll
            for (int j = 0; j < VEC; ++j) so[((size_t)wave * M + h) * d + lj * VEC + j] = o[h][j];
        }
    }
    __syncthreads();
    // merge the wavefronts, normalise, write
    for (int idx = tid; idx < M * d; idx += 64 * NW) {
        const int mm = idx / d, j = idx - mm * d;
        const int rr = mm / GROUP, h = mm - rr * GROUP;
        if (rr >= n_rows) continue;
        const int row = row0 + rr;
        float mn = -INFINITY;
        for (int w = 0; w < NW; ++w) mn = fmaxf(mn, sm[w * M + mm]);
        float ls = 0.f, os = 0.f;
        for (int w = 0; w < NW; ++w) {
            const float mw = sm[w * M + mm];
            const float c = (mw == -INFINITY) ? 0.f : __expf(mw - mn);
            ls += sl[w * M + mm] * c;
            os += so[((size_t)w * M + mm) * d + j] * c;
        }
        const float y = os / ls;
        const int e = (g * GROUP + h) * d + j;
        if (a.out) a.out[(size_t)row * nq * d + e] = y;
        if (a.out_s) {
            uint16_t hi, mid, lo;
            split3(y, hi, mid, lo);
            const int ocode = a.out_rows ? a.out_rows : a.rows, orows = layout_rows(ocode), nt = block_terms(ocode);
            uint16_t *p = a.out_s + ((size_t)(e >> 3) * (nt * orows) + nt * row) * 8 + (e & 7);
            p[0] = hi;
            p[8] = mid;
            if (nt == 3) p[16] = lo;
        }
    }
}

}  // namespace swift
