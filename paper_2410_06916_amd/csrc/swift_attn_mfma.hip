// Attention of decode, draft and verify rows over a bf16 cache with heads of 64 or 128 on the matrix
// cores (paper Sections 3.1 and 4.2: a draft or plain decoding pass has one row, a verify pass the pending
// token and its k drafts as one causal block, dynamic verification the rows of a token tree).
//
// All rows of a block and all query heads of a kv head's group are the columns ("members") of one MFMA
// tile, so a workgroup reads every key/value chunk of its cache range once for up to 16 members -- once
// per block for a block of up to 16 rows on one kv head per query head.  The operands come straight from
// global memory in MFMA layout with 128-bit loads: the keys as stored, the values from a cache that holds
// eight slots of an element together (kv_vt_index), so nothing is transposed or staged on the way.
//
// What a row computes (the same for a row decoded alone, a row of a chain block and a row of a tree, bit for
// bit, because every step below is per member and its order does not depend on the other members):
//  * the row's prefix -- logical slots [0, P), P = its position -- is walked in chunks of 32 slots.  A
//    workgroup owns a range of the cache capacity fixed by the configuration alone; its wavefronts take the
//    range's chunks round-robin, each folding its chunks in order into a running (max, sum, weighted values)
//    with S^T = K Q^T and O^T += V^T P^T (queries and probabilities as two bf16 terms each: relative error
//    2^-17 against the 2^-9 of the bf16 keys and values; fp32 sums); the wavefronts' results are merged in
//    wavefront order, the ranges' in range order (k_attn_mfma_combine);
//  * the row's own slot (its key and value, written to the cache by the projection kernel of the same pass)
//    is merged last, in fp32 vector arithmetic.  For a tree row the prefix beyond the committed slots is
//    the first candidates of the levels above it: one mapping for all rows, so tree rows share the loads
//    too, and only the own slot differs from row to row.
#include <math.h>
#include <stdio.h>

#include <algorithm>

#include "swift_device.h"
#include "swift_kernels.h"

namespace swift {

namespace {

constexpr int kAmPad = 4;  // floats of padding per member row of the merge area

__device__ inline bf16x8 am_pack(const uint16_t (&v)[8]) {
    u32x4 u;
    u.x = (uint32_t)v[0] | ((uint32_t)v[1] << 16);
    u.y = (uint32_t)v[2] | ((uint32_t)v[3] << 16);
    u.z = (uint32_t)v[4] | ((uint32_t)v[5] << 16);
    u.w = (uint32_t)v[6] | ((uint32_t)v[7] << 16);
    return __builtin_bit_cast(bf16x8, u);
}

// Logical slots [0, this) are launch row r's prefix; its own slot holds the row's key and value.
template <bool TREE>
__device__ inline int am_prefix_end(const AttnArgs &a, int r) {
    return TREE ? a.n_base + (int)a.tt.depth[(a.row_base + r) & (kMaxRows - 1)] : a.n_ctx - 1 + r;
}
template <bool TREE>
__device__ inline int am_own_slot(const AttnArgs &a, int r) {
    return TREE ? a.n_base + a.row_base + r : a.n_ctx - 1 + r;
}
// Cache slot of logical prefix slot p.  Tree rows: beyond the committed slots the prefix is the block's
// first row, then the first candidates of the levels in between.
template <bool TREE>
__device__ inline int am_phys(const AttnArgs &a, int p) {
    if (TREE && p >= a.n_base) return a.n_base + (int)a.tt.spine[(p - a.n_base) & (kMaxRows - 1)];
    return p;
}

__device__ inline float am_bf(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// q . k of a row's own slot, by one wavefront: lane l takes elements 2l, 2l+1 (+128 ...), then a butterfly.
__device__ inline float am_own_score(const float *q, const uint16_t *k, int d, int lane, float scale) {
    float s = 0.f;
    for (int e = 2 * lane; e < d; e += 128) {
        s = fmaf(q[e], am_bf(k[e]), s);
        s = fmaf(q[e + 1], am_bf(k[e + 1]), s);
    }
    return wave_sum(s) * scale;
}

// Merges the own slot (score s_own, value v_own) into the prefix's (max mn, sum ls, weighted value os) and
// normalises.  An empty prefix has mn = -inf, ls = os = 0.
__device__ inline float am_finish(float mn, float ls, float os, float s_own, float v_own) {
    const float m2 = fmaxf(mn, s_own);
    const float c1 = mn == -INFINITY ? 0.f : __expf(mn - m2);
    const float c2 = __expf(s_own - m2);
    return (os * c1 + c2 * v_own) / (ls * c1 + c2);
}

__device__ inline void am_write(const AttnArgs &a, int row, int e, float y) {
    if (a.out) a.out[(size_t)row * a.n_q_heads * a.head_dim + e] = y;
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

// Lane layout of v_mfma_f32_16x16x32_bf16 (C = A B): lane = 16 g + col.
//   A (16 x 32): row col,    k = 8 g .. 8 g + 7        B (32 x 16): column col, k = 8 g .. 8 g + 7
//   C (16 x 16): column col, rows 4 g .. 4 g + 3
// Scores of a 32-slot chunk are two tiles tt = 0, 1; tile row 4 g + i is slot 8 g + 4 tt + i of the chunk, so
// that a lane's eight probabilities are slots 8 g .. 8 g + 7: the k range of its B operand in O^T = V^T P^T.
//
// Workgroup (kv head, cache range sp, member tile z), blockDim.x / 64 wavefronts.  range: slots per workgroup, a
// multiple of 32.  hi_all: end of the longest prefix of the block.
template <int D, bool TREE>
__global__ __launch_bounds__(512) void k_attn_mfma(AttnArgs a, int range, int hi_all) {
    constexpr int DC = D / 32;      // k steps of a score tile
    constexpr int DT = D / 16;      // 16-row tiles of O^T
    constexpr int MP = D + kAmPad;  // pitch of a member's values in the merge area
    extern __shared__ __align__(16) float am_sh[];
    const int kvh = blockIdx.x, sp = blockIdx.y, n_split = gridDim.y;
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int NW = blockDim.x >> 6;
    const int nq = a.n_q_heads, group = nq / a.n_kv_heads;
    const int M_total = a.rows * group;
    const int m0 = 16 * blockIdx.z;  // first member of this workgroup's tile; member m = (row m / group, head m % group)
    const int lo = sp * range, hi = min(hi_all, lo + range);
    const float scale = 1.0f / sqrtf((float)D);
    const uint16_t *kc = (const uint16_t *)a.kcache + (size_t)kvh * a.max_seq * D;
    const uint16_t *vt = (const uint16_t *)a.vcache + (size_t)kvh * a.nb32 * D * 32;

    // ---- this lane's member (column col of the tile)
    const int mem = m0 + col;
    const bool mem_ok = mem < M_total;
    const int mrow = mem_ok ? mem / group : 0, mhead = mem_ok ? mem - mrow * group : 0;
    const int lim = mem_ok ? min(am_prefix_end<TREE>(a, mrow), lo + range) : 0;  // the prefix slots it sees here
    // ---- operands of a chunk, straight from the cache in MFMA A layout
    // Chunks that lie below safe_end hold 32 prefix slots that sit where their numbers say: keys as stored,
    // values one 16-byte load per eight slots.  In the chunk in which the longest prefix ends, the keys of the
    // slots past it are replaced by its last slot's and their values by zeros (an unwritten slot may hold
    // anything, and 0 x NaN is NaN in an MFMA); a tree's chunks beyond the committed slots go slot by slot
    // through the mapping.
    const int safe_end = TREE ? min(a.n_base, hi_all) : hi_all;
    auto load_keys = [&](int c, u32x4(&kA)[2][DC]) {
        const bool plain = 32 * (c + 1) <= safe_end;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const int slot = 32 * c + 8 * (col >> 2) + 4 * tt + (col & 3);
            const int ps = plain ? slot : am_phys<TREE>(a, min(slot, hi_all - 1));
            const uint16_t *kp = kc + (size_t)ps * D + 8 * g;
#pragma unroll
            for (int cc = 0; cc < DC; ++cc) kA[tt][cc] = *(const u32x4 *)(kp + 32 * cc);
        }
    };
    auto load_values = [&](int c, u32x4(&vA)[DT]) {
        const bool plain = 32 * (c + 1) <= safe_end;
        if (!TREE || plain) {
            const uint16_t *vp = vt + ((size_t)(4 * c + g) * D + col) * 8;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) vA[dt] = *(const u32x4 *)(vp + dt * (16 * 8));
            if (!plain) {
                // the chunk in which the longest prefix ends: the slots past it are zeroed in the registers
                const int n_ok = hi_all - (32 * c + 8 * g);  // slots of this lane's eight that belong to the prefix
                const uint32_t m0 = n_ok >= 2 ? 0xffffffffu : n_ok == 1 ? 0x0000ffffu : 0u;
                const uint32_t m1 = n_ok >= 4 ? 0xffffffffu : n_ok == 3 ? 0x0000ffffu : 0u;
                const uint32_t m2 = n_ok >= 6 ? 0xffffffffu : n_ok == 5 ? 0x0000ffffu : 0u;
                const uint32_t m3 = n_ok >= 8 ? 0xffffffffu : n_ok == 7 ? 0x0000ffffu : 0u;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    vA[dt].x &= m0;
                    vA[dt].y &= m1;
                    vA[dt].z &= m2;
                    vA[dt].w &= m3;
                }
            }
        } else {
            // a tree's chunks beyond the committed slots: slot by slot through the mapping
            int ps[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) ps[j] = am_phys<TREE>(a, min(32 * c + 8 * g + j, hi_all - 1));
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                uint16_t e[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) e[j] = vt[((size_t)(ps[j] >> 3) * D + 16 * dt + col) * 8 + (ps[j] & 7)];
                vA[dt] = __builtin_bit_cast(u32x4, am_pack(e));
            }
        }
    };

    float m_run = -INFINITY, l_run = 0.f;
    f32x4 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int c_end = (hi + 31) >> 5;
    u32x4 kA[2][DC], kB[2][DC], vA[DT];
    int c = (lo >> 5) + wave;
    // the first chunk's operands are requested before anything else, so that the set-up below (query operands,
    // own slots) runs while they are on their way
    if (c < c_end) {
        load_keys(c, kA);
        load_values(c, vA);
    }

    // query operands: two bf16 terms per value (relative error 2^-17; the keys they meet are bf16), written in
    // this form by the projection kernel
    bf16x8 qop[DC][2];
    {
        const uint16_t *qp = a.q_s + ((size_t)(mrow * nq + kvh * group + mhead) * 2) * D + 8 * g;
#pragma unroll
        for (int c = 0; c < DC; ++c)
#pragma unroll
            for (int t = 0; t < 2; ++t) qop[c][t] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(qp + t * D + 32 * c));
    }
    // ---- the own slots of the rows that are finished here (prefix inside the first range), requested before
    // the prefix is walked so that their latency is not paid at the end: scores by whole wavefronts into LDS,
    // the value elements each thread will need in the last phase into registers
    constexpr int kOwnMax = 16 * D / 256;  // elements per thread in the last phase with four wavefronts
    float *s_own = am_sh + (size_t)NW * (16 * (MP + 2));
    float v_own[kOwnMax];
    if (sp == 0) {
        // (member mm by wavefront NW - 1 - mm % NW: the last wavefronts have the fewest chunks to walk)
        for (int mm = NW - 1 - wave; mm < 16; mm += NW) {
            const int m = m0 + mm;
            if (m >= M_total) continue;
            const int row = m / group, head = m - row * group;
            if (am_prefix_end<TREE>(a, row) > range) continue;  // finished by the combine kernel
            const float sc = am_own_score(a.q + ((size_t)row * nq + kvh * group + head) * D,
                                          kc + (size_t)am_own_slot<TREE>(a, row) * D, D, lane, scale);
            if (lane == 0) s_own[mm] = sc;
        }
#pragma unroll
        for (int u = 0; u < kOwnMax; ++u) {
            const int idx = tid + u * (int)blockDim.x, mm = idx / D, dd = idx - mm * D, m = m0 + mm;
            v_own[u] = 0.f;
            if (idx < 16 * D && m < M_total && am_prefix_end<TREE>(a, m / group) <= range) {
                const int own = am_own_slot<TREE>(a, m / group);
                v_own[u] = am_bf(vt[((size_t)(own >> 3) * D + dd) * 8 + (own & 7)]);
            }
        }
    }

    // ---- this wavefront's chunks: every NW-th of the range, folded in order.  The keys of the next chunk are
    // requested before the current chunk's scores are computed (two sets of key registers, used in turn); the
    // value operands are dead once they are multiplied, so the next chunk's values are requested right after
    // the second product, into the same registers.
    auto step = [&](int c, const u32x4(&kCur)[2][DC], u32x4(&kNxt)[2][DC]) {
        const bool more = c + NW < c_end;  // wavefront-uniform
        if (more) load_keys(c + NW, kNxt);
        float s[8];
        float mx = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int cc = 0; cc < DC; ++cc)
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kCur[tt][cc]), qop[cc][t], acc, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int slot = 32 * c + 8 * g + 4 * tt + i;
                const float v = slot < lim ? acc[i] * scale : -INFINITY;
                s[4 * tt + i] = v;
                mx = fmaxf(mx, v);
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float mn = fmaxf(m_run, mx);
        const float ms = mn == -INFINITY ? 0.f : mn;  // nothing live yet: every exponential below is 0
        const float corr = __expf(m_run - ms);
        float ps = 0.f;
        uint16_t ph[8], pl[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float p = __expf(s[j] - ms);
            ps += p;
            const uint32_t hb = f32_to_bf16_rne_finite(p);
            ph[j] = (uint16_t)hb;
            pl[j] = (uint16_t)f32_to_bf16_rne_finite(p - __uint_as_float(hb << 16));
        }
        const bf16x8 phi = am_pack(ph), plo = am_pack(pl);
        l_run = l_run * corr + ps;
        m_run = mn;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            o[dt] *= corr;
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vA[dt]), phi, o[dt], 0, 0, 0);
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vA[dt]), plo, o[dt], 0, 0, 0);
        }
        if (more) load_values(c + NW, vA);
    };
    for (; c < c_end; c += 2 * NW) {
        step(c, kA, kB);
        if (c + NW < c_end) step(c + NW, kB, kA);
    }

    // ---- merge the wavefronts (in wavefront order), then finish the rows whose prefix ends in the first
    // range with their own slot, or leave the range's partial result for k_attn_mfma_combine
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    float *wbase = am_sh + (size_t)wave * (16 * (MP + 2));
    if (g == 0) {
        wbase[col] = m_run;
        wbase[16 + col] = l_run;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i) wbase[32 + col * MP + 16 * dt + 4 * g + i] = o[dt][i];
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kOwnMax; ++u) {
        const int idx = tid + u * (int)blockDim.x;
        if (idx >= 16 * D) break;
        const int mm = idx / D, dd = idx - mm * D;
        const int m = m0 + mm;
        if (m >= M_total) continue;
        const int row = m / group, head = m - row * group;
        const int pe = am_prefix_end<TREE>(a, row);
        const int nsr = (pe + range - 1) / range;  // ranges the row's prefix reaches (0: an empty prefix)
        if (sp >= max(nsr, 1)) continue;
        float mn = -INFINITY;
        for (int w = 0; w < NW; ++w) mn = fmaxf(mn, am_sh[(size_t)w * (16 * (MP + 2)) + mm]);
        float ls = 0.f, os = 0.f;
        for (int w = 0; w < NW; ++w) {
            const float *wb = am_sh + (size_t)w * (16 * (MP + 2));
            const float mw = wb[mm];
            const float cw = mw == -INFINITY ? 0.f : __expf(mw - mn);
            ls += wb[16 + mm] * cw;
            os += wb[32 + mm * MP + dd] * cw;
        }
        const int qh = kvh * group + head;
        if (nsr <= 1) {
            am_write(a, row, qh * D + dd, am_finish(mn, ls, os, s_own[mm], v_own[u]));
        } else {
            const size_t slot = ((size_t)row * nq + qh) * n_split + sp;
            a.part_o[slot * D + dd] = os;
            if (dd == 0) {
                a.part_ml[slot * 2] = mn;
                a.part_ml[slot * 2 + 1] = ls;
            }
        }
    }
}

// Rows whose prefix spans several ranges: merges the ranges' partial results in range order, then the own
// slot.  One workgroup of two wavefronts per (query head, row): thread t owns value element t; the first
// wavefront also computes the own slot's score.
template <bool TREE>
__global__ __launch_bounds__(128) void k_attn_mfma_combine(AttnArgs a, int range, int n_split) {
    __shared__ float sh_own;
    const int head = blockIdx.x, row = blockIdx.y, tid = threadIdx.x, d = a.head_dim;
    const int pe = am_prefix_end<TREE>(a, row);
    const int nsr = (pe + range - 1) / range;
    if (nsr <= 1) return;  // finished by the attention kernel itself
    const int kvh = head / (a.n_q_heads / a.n_kv_heads);
    const uint16_t *kc = (const uint16_t *)a.kcache + (size_t)kvh * a.max_seq * d;
    const uint16_t *vt = (const uint16_t *)a.vcache + (size_t)kvh * a.nb32 * d * 32;
    const int own = am_own_slot<TREE>(a, row);
    const size_t base = ((size_t)row * a.n_q_heads + head) * n_split;
    const float *__restrict__ ml = a.part_ml + base * 2;
    const float *__restrict__ po = a.part_o + base * d + tid;
    // everything this thread needs, requested together: the ranges' (max, sum) pairs and its element of their
    // weighted values, eight ranges at a time
    const bool live = tid < d;
    const float v_own = live ? am_bf(vt[((size_t)(own >> 3) * d + tid) * 8 + (own & 7)]) : 0.f;
    float mn = -INFINITY, ls = 0.f, os = 0.f;
    for (int s0 = 0; s0 < nsr; s0 += 8) {
        float m8[8], l8[8], o8[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int sidx = min(s0 + u, nsr - 1);
            m8[u] = ml[2 * sidx];
            l8[u] = ml[2 * sidx + 1];
            o8[u] = live ? po[(size_t)sidx * d] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (s0 + u >= nsr) break;
            // running merge in range order (a range's maximum is -inf only if its rows see nothing there)
            const float m2 = fmaxf(mn, m8[u]);
            const float c1 = mn == -INFINITY ? 0.f : __expf(mn - m2);
            const float c2 = m8[u] == -INFINITY ? 0.f : __expf(m8[u] - m2);
            ls = ls * c1 + l8[u] * c2;
            os = os * c1 + o8[u] * c2;
            mn = m2;
        }
    }
    if (tid < 64) {
        const float sc = am_own_score(a.q + ((size_t)row * a.n_q_heads + head) * d, kc + (size_t)own * d, d, tid,
                                      1.0f / sqrtf((float)d));
        if (tid == 0) sh_own = sc;
    }
    __syncthreads();
    if (live) am_write(a, row, head * d + tid, am_finish(mn, ls, os, sh_own, v_own));
}

// The launch shape.  Everything that shapes a row's arithmetic (wavefronts per workgroup, slots per range)
// follows from the cache capacity and the head count alone.
struct AmPlan {
    int nw;        // wavefronts per workgroup
    int range;     // cache slots per workgroup
    int hi_all;    // end of the longest prefix of the block
    int n_split;   // ranges that prefix reaches
    int n_tiles;   // member tiles (16 members each) = workgroups per (kv head, range)
};
AmPlan am_plan(const AttnArgs &a, int n_cu) {
    AmPlan p{};
    // Short caches of many-headed models: one workgroup per kv head walks the whole prefix (no partial results,
    // no second launch), with eight wavefronts to have enough loads in flight; otherwise the capacity is cut
    // into enough ranges for about two workgroups per compute unit with one member tile.
    const bool single = attn_uses_head_kernel(a.max_seq, a.n_kv_heads);
    p.nw = single ? 8 : 4;
    int want = single ? 1 : (2 * n_cu + a.n_kv_heads - 1) / a.n_kv_heads;
    if (want > a.max_split) want = a.max_split;
    if (want < 1) want = 1;
    // (whole chunks; a range need not hold the same number of chunks for every wavefront)
    p.range = std::max(32 * p.nw, ((a.max_seq + want - 1) / want + 31) / 32 * 32);
    if (a.tree) {
        int deepest = 0;
        for (int r = 0; r < a.rows; ++r) deepest = std::max(deepest, (int)a.tt.depth[(a.row_base + r) & (kMaxRows - 1)]);
        p.hi_all = a.n_base + deepest;
    } else {
        p.hi_all = a.n_ctx - 1 + a.rows - 1;
    }
    p.n_split = std::max(1, (p.hi_all + p.range - 1) / p.range);
    p.n_tiles = (a.rows * (a.n_q_heads / a.n_kv_heads) + 15) / 16;
    return p;
}

}  // namespace

size_t attn_mfma_partial_floats(const AttnArgs &a, int n_cu) {
    const AmPlan p = am_plan(a, n_cu);
    const int max_splits = (a.max_seq + p.range - 1) / p.range;
    return max_splits > 1 ? (size_t)a.rows * a.n_q_heads * max_splits * a.head_dim : 0;
}

int attn_mfma_path_name(const AttnArgs &a, int n_cu, char *out, int capacity) {
    const AmPlan p = am_plan(a, n_cu);
    return snprintf(out, (size_t)capacity, "mfma<d %d, group %d, %d wavefronts, range %d, tiles %d%s>", a.head_dim,
                    a.n_q_heads / a.n_kv_heads, p.nw, p.range, p.n_tiles, a.tree ? ", tree" : "");
}

hipError_t launch_attn_mfma(const AttnArgs &a, int n_cu, hipStream_t s) {
    if ((a.head_dim != 64 && a.head_dim != 128) || a.rows < 1 || a.rows > kAttnMfmaMaxRows || a.nb32 < (a.max_seq + 31) / 32 ||
        a.n_kv_heads < 1 || a.n_q_heads % a.n_kv_heads != 0 || !a.q || !a.q_s || !a.kcache || !a.vcache || (!a.out && !a.out_s) ||
        !a.part_o || !a.part_ml)
        return hipErrorInvalidValue;
    if (a.tree ? (a.row_base < 0 || a.row_base + a.rows > kMaxRows || a.n_base < 0 || a.n_base + a.row_base + a.rows > a.max_seq)
               : (a.n_ctx < 1 || a.n_ctx - 1 + a.rows > a.max_seq))
        return hipErrorInvalidValue;
    const AmPlan p = am_plan(a, n_cu);
    if (p.n_split > a.max_split) return hipErrorInvalidValue;
    const int D = a.head_dim;
    const size_t lds = ((size_t)p.nw * 16 * (D + kAmPad + 2) + 16) * sizeof(float);
    const dim3 grid(a.n_kv_heads, p.n_split, p.n_tiles), block(64 * p.nw);
#define SWIFT_AM(DD, TR)                                                                                        \
    do {                                                                                                        \
        static bool attr_set = false;                                                                           \
        if (!attr_set) {                                                                                        \
            hipError_t e = hipFuncSetAttribute((const void *)k_attn_mfma<DD, TR>,                               \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);          \
            if (e != hipSuccess) return e;                                                                      \
            attr_set = true;                                                                                    \
        }                                                                                                       \
        hipLaunchKernelGGL((k_attn_mfma<DD, TR>), grid, block, lds, s, a, p.range, p.hi_all);                   \
    } while (0)
    if (D == 128) {
        if (a.tree) SWIFT_AM(128, true); else SWIFT_AM(128, false);
    } else {
        if (a.tree) SWIFT_AM(64, true); else SWIFT_AM(64, false);
    }
#undef SWIFT_AM
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.n_split == 1) return e;
    const dim3 cgrid(a.n_q_heads, a.rows);
    if (a.tree)
        hipLaunchKernelGGL(k_attn_mfma_combine<true>, cgrid, dim3(128), 0, s, a, p.range, p.n_split);
    else
        hipLaunchKernelGGL(k_attn_mfma_combine<false>, cgrid, dim3(128), 0, s, a, p.range, p.n_split);
    return hipGetLastError();
}

}  // namespace swift
