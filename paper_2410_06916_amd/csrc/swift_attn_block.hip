// Causal attention of a block of 17..64 rows over a bf16 cache on the matrix cores (prefill blocks and
// the blocks of candidate evaluation; paper Section 3.1: the verify / prefill pass processes its rows as
// one causal block).  One workgroup per (query head, range of cache slots): its four wavefronts take 16
// block rows each and share every 64-slot chunk of keys and values through LDS, so a chunk is read once
// for all 64 rows instead of once per group of rows.  The values come from a cache that stores eight slots of
// an element together, so they reach LDS as V^T with plain 16-byte copies.
//
// Arithmetic.  Scores: S^T = K Q^T with the fp32 query rows as three bf16 terms (the products are
// exact, the sums fp32).  The transposed form leaves a row's scores in one lane column, so its
// probabilities are, without any data movement, the B operand of O^T = V^T P^T, and the online-softmax
// rescale of O^T is per lane.  Probabilities enter that product as two bf16 terms (relative error
// 2^-17; the values they weight are bf16).  Rows of up to 16-row blocks never come here: their results
// must not depend on how many rows share a pass, and they keep the one fp32 code path that guarantees it.
#include <math.h>

#include "swift_device.h"
#include "swift_kernels.h"

namespace swift {

namespace {

__device__ inline bf16x8 pack_bf16x8(const uint16_t (&v)[8]) {
    u32x4 u;
    u.x = (uint32_t)v[0] | ((uint32_t)v[1] << 16);
    u.y = (uint32_t)v[2] | ((uint32_t)v[3] << 16);
    u.z = (uint32_t)v[4] | ((uint32_t)v[5] << 16);
    u.w = (uint32_t)v[6] | ((uint32_t)v[7] << 16);
    return __builtin_bit_cast(bf16x8, u);
}

// Lane layout of v_mfma_f32_16x16x32_bf16 (C = A B): lane = 16 g + col.
//   A (16 x 32): row col,    k = 8 g .. 8 g + 7        B (32 x 16): column col, k = 8 g .. 8 g + 7
//   C (16 x 16): column col, rows 4 g .. 4 g + 3
// Scores of one half chunk (32 slots) are two MFMA tiles tt = 0, 1; tile row 4 g + i is slot
// 8 g + 4 tt + i of the half, so that a lane's eight probabilities of the half are slots 8 g .. 8 g + 7:
// the k range of its B operand in the second product.
// A prompt macro block (a.sub_rows = 64) is one launch too: blockIdx.z is the sub-block, which is treated as a block
// of its own whose partial results sit at the macro block's row numbers.
template <int D>
__global__ __launch_bounds__(256) void k_attn_block(AttnArgs am, int chunk) {
    constexpr int DC = D / 32;   // k steps of a score tile
    constexpr int DT = D / 16;   // 16-row tiles of O^T
    constexpr int PPR = D / 8;   // 16-byte pieces per cache row
    constexpr int NPC = PPR / 4; // pieces per thread, per chunk and matrix (64 slots, 256 threads)
    constexpr int KP = D + 8;    // LDS pitch of a key row (elements)
    constexpr int VP = 64 + 8;   // LDS pitch of a row of V^T
    __shared__ __align__(16) uint16_t Ks[64 * KP];
    __shared__ __align__(16) uint16_t Vt[D * VP];

    AttnArgs a = am;
    const int row_base = (int)blockIdx.z * 64;  // first row of this sub-block in the macro block
    if (am.sub_rows) {
        a.rows = min(64, am.rows - row_base);
        a.n_ctx = am.n_ctx + row_base;
        a.q = am.q + (size_t)blockIdx.z * am.sub_q;
        if (am.out_s) a.out_s = am.out_s + (size_t)blockIdx.z * am.sub_out_s;
    }
    const int head = blockIdx.x, sp = blockIdx.y, n_split = gridDim.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 15, g = lane >> 4;
    const int nq = a.n_q_heads, kvh = head / (nq / a.n_kv_heads);
    const int lo = sp * chunk;
    const int hi_all = min(a.n_ctx + a.rows - 1, lo + chunk);  // end of the longest row's range here
    if (hi_all <= lo) return;
    const uint16_t *kc = (const uint16_t *)a.kcache + (size_t)kvh * a.max_seq * D;
    const uint16_t *vt = (const uint16_t *)a.vcache + (size_t)kvh * a.nb32 * D * 32;
    const int row = 16 * wave + col;
    const int lim = row < a.rows ? a.n_ctx + row : 0;  // rows past the block take part in nothing
    const int tile_lim = a.n_ctx + min(16 * wave + 15, a.rows - 1);
    const bool tile_live = 16 * wave < a.rows;

    bf16x8 qop[DC][3];
    {
        const float *qp = a.q + ((size_t)min(row, a.rows - 1) * nq + head) * D + 8 * g;
#pragma unroll
        for (int c = 0; c < DC; ++c) {
            uint16_t h[8], m[8], l[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) split3(qp[32 * c + j], h[j], m[j], l[j]);
            qop[c][0] = pack_bf16x8(h);
            qop[c][1] = pack_bf16x8(m);
            qop[c][2] = pack_bf16x8(l);
        }
    }

    u32x4 kr[NPC], vr[NPC];
    // Keys: piece p = (slot p / PPR, 8 elements).  Slots past the longest row's range are replaced by its last
    // slot (an unwritten slot may hold anything).  Values come from the cache that groups eight slots per element
    // (kv_vt_index): piece p = (8-slot group p / D of the chunk, element p % D); slots past the range are zeroed in the
    // registers (0 x NaN is NaN in the second product).
    auto load_chunk = [&](int k0) {
#pragma unroll
        for (int u = 0; u < NPC; ++u) {
            const int p = tid + 256 * u, key = p / PPR, dj = p - key * PPR;
            kr[u] = *(const u32x4 *)(kc + (size_t)min(k0 + key, hi_all - 1) * D + 8 * dj);
            const int sg = p / D, dd = p - sg * D;
            const int grp = min((k0 >> 3) + sg, 4 * a.nb32 - 1);
            u32x4 v = *(const u32x4 *)(vt + ((size_t)grp * D + dd) * 8);
            const int n_ok = hi_all - (k0 + 8 * sg);  // slots of this piece inside the range
            if (n_ok < 8) {
                uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (j >= n_ok) w[j >> 1] &= (j & 1) ? 0x0000ffffu : 0xffff0000u;
                v = u32x4{w[0], w[1], w[2], w[3]};
            }
            vr[u] = v;
        }
    };
    // V^T in LDS: element (dd, key) at row dd, column 8 ((key / 8) ^ (dd / 8 & 7)) + key % 8
    auto store_chunk = [&]() {
#pragma unroll
        for (int u = 0; u < NPC; ++u) {
            const int p = tid + 256 * u, key = p / PPR, dj = p - key * PPR;
            *(u32x4 *)(Ks + key * KP + 8 * dj) = kr[u];
            const int sg = p / D, dd = p - sg * D;
            *(u32x4 *)(Vt + dd * VP + 8 * (sg ^ ((dd >> 3) & 7))) = vr[u];
        }
    };

    const float scale = 1.0f / sqrtf((float)D);
    float m_run = -INFINITY, l_run = 0.f;
    f32x4 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    load_chunk(lo);
    for (int k0 = lo; k0 < hi_all; k0 += 64) {
        store_chunk();
        __syncthreads();
        if (k0 + 64 < hi_all) load_chunk(k0 + 64);
        if (tile_live && k0 < tile_lim) {  // wavefront-uniform: some row of the tile reaches this chunk
            float s[2][2][4];
            float mx = -INFINITY;
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                    const uint16_t *kp = Ks + (32 * hf + 8 * (col >> 2) + 4 * tt + (col & 3)) * KP + 8 * g;
#pragma unroll
                    for (int c = 0; c < DC; ++c) {
                        const bf16x8 av = __builtin_bit_cast(bf16x8, *(const u32x4 *)(kp + 32 * c));
#pragma unroll
                        for (int t = 0; t < 3; ++t)
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, qop[c][t], acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int key = k0 + 32 * hf + 8 * g + 4 * tt + i;
                        const float v = key < lim ? acc[i] * scale : -INFINITY;
                        s[hf][tt][i] = v;
                        mx = fmaxf(mx, v);
                    }
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float mn = fmaxf(m_run, mx);
            const float ms = mn == -INFINITY ? 0.f : mn;  // nothing live yet: every exponential below is 0
            const float corr = __expf(m_run - ms);
            float ps = 0.f;
            bf16x8 phi[2], plo[2];
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                uint16_t h[8], l[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float p = __expf(s[hf][j >> 2][j & 3] - ms);
                    ps += p;
                    const uint32_t hb = f32_to_bf16_rne_finite(p);
                    h[j] = (uint16_t)hb;
                    l[j] = (uint16_t)f32_to_bf16_rne_finite(p - __uint_as_float(hb << 16));
                }
                phi[hf] = pack_bf16x8(h);
                plo[hf] = pack_bf16x8(l);
            }
            l_run = l_run * corr + ps;
            m_run = mn;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                o[dt] *= corr;
                const int dd = 16 * dt + col;
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const bf16x8 av = __builtin_bit_cast(
                        bf16x8, *(const u32x4 *)(Vt + dd * VP + 8 * ((4 * hf + g) ^ ((dd >> 3) & 7))));
                    o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, phi[hf], o[dt], 0, 0, 0);
                    o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, plo[hf], o[dt], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }
    // a row's sum is spread over its four lanes (the running maximum is common to them)
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (row >= a.rows) return;
    const int ns_row = (a.n_ctx + row + chunk - 1) / chunk;  // ranges this row reaches
    if (sp >= ns_row) return;
    if (ns_row == 1) {  // the row ends in the first range: normalise and write
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const int e = head * D + 16 * dt + 4 * g;
            uint16_t hi[4], mid[4], lw[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float y = o[dt][i] * inv;
                if (a.out) a.out[(size_t)row * nq * D + e + i] = y;
                split3(y, hi[i], mid[i], lw[i]);
            }
            if (a.out_s) {
                const int ocode = a.out_rows ? a.out_rows : a.rows, orows = layout_rows(ocode), nt = block_terms(ocode);
                uint16_t *p = a.out_s + ((size_t)(e >> 3) * (nt * orows) + nt * row) * 8 + (e & 7);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    p[i] = hi[i];
                    p[8 + i] = mid[i];
                    if (nt == 3) p[16 + i] = lw[i];
                }
            }
        }
    } else {  // partial result of this range; k_attn_combine merges the ranges in order
        const size_t base = ((size_t)(row_base + row) * nq + head) * n_split + sp;
        if (g == 0) {
            a.part_ml[base * 2] = m_run;
            a.part_ml[base * 2 + 1] = l_run;
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 4; ++i) a.part_o[base * D + 16 * dt + 4 * g + i] = o[dt][i];
    }
}

}  // namespace

bool attn_block_applies(int dtype, const AttnArgs &a) {
    return dtype == BF16 && !a.tree && a.rows > kMaxRows && a.rows <= 64 && (a.head_dim == 64 || a.head_dim == 128);
}

hipError_t launch_attn_block(const AttnArgs &a, int n_cu, hipStream_t s) {
    const int n_sub = a.sub_rows ? (a.rows + 63) / 64 : 1;
    if (a.tree || a.rows < 1 || a.rows > 64 * n_sub || (a.sub_rows != 0 && a.sub_rows != 64) || n_sub > kMacroSub ||
        (a.sub_rows && a.out) || (a.head_dim != 64 && a.head_dim != 128) || a.n_ctx < 1 ||
        a.n_kv_heads < 1 || a.n_q_heads % a.n_kv_heads != 0 || a.n_ctx + a.rows - 1 > a.max_seq || (!a.out && !a.out_s) ||
        a.nb32 < (a.max_seq + 31) / 32 ||
        !a.part_o || !a.part_ml)
        return hipErrorInvalidValue;
    const int ctx = a.n_ctx + a.rows - 1;
    // ranges: about two workgroups per compute unit, at least two chunks each, and no more partial results
    // than the buffers hold (they are sized for kMaxRows rows times max_split ranges)
    int want = (2 * n_cu + a.n_q_heads * n_sub - 1) / (a.n_q_heads * n_sub);
    const int cap = kMaxRows * a.max_split / a.rows;
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    int chunk = ((ctx + want - 1) / want + 63) / 64 * 64;
    if (chunk < 128) chunk = 128;
    const int n_split = (ctx + chunk - 1) / chunk;
    if ((int64_t)n_split * a.rows > (int64_t)kMaxRows * a.max_split) return hipErrorInvalidValue;
    const dim3 grid(a.n_q_heads, n_split, n_sub), block(256);
    if (a.head_dim == 128)
        hipLaunchKernelGGL(k_attn_block<128>, grid, block, 0, s, a, chunk);
    else
        hipLaunchKernelGGL(k_attn_block<64>, grid, block, 0, s, a, chunk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_split == 1) return e;
    return launch_attn_combine(a, chunk, n_split, s);
}

}  // namespace swift
