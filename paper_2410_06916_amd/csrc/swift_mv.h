// Epilogue of the tiled projection kernels.
#pragma once
#include <math.h>

#include "swift_device.h"
#include "swift_kernels.h"

namespace swift {

// Values in the grouped layout (kv_vt_index) are written two bytes at a time into 128-byte lines that the
// pass fills only partly, and such a store completes only once the rest of the line has been fetched.  The
// projection kernel therefore touches the lines its epilogue will write while the weights stream: lane
// (block row r, half) of the calling wavefront reads one word of the line that holds elements 8 g .. 8 g + 7
// (+ d/2) of row r's slot; rg is a row group of the value part of the fused q|k|v matrix (else nothing
// happens).  The loaded word is only kept alive, never used.
__device__ inline void mv_touch_value_lines(const MvArgs &a, int rg, int lane) {
    const int d = a.head_dim, half = d >> 1, gph = half >> 3;
    const int hh = rg / gph, head = hh - a.n_q_heads - a.n_kv_heads;
    const int r = lane >> 1;
    if (a.nb32 <= 0 || head < 0 || head >= a.n_kv_heads || r >= a.R) return;
    const int i = 8 * (rg - hh * gph) + (lane & 1) * half;
    const uint32_t w = *(const volatile uint32_t *)((const uint16_t *)a.vcache + (kv_vt_index(head, a.nb32, d, a.pos0 + r, i) & ~(size_t)1));
    asm volatile("" ::"v"(w));
}

// What follows the dot products of one 16-row group, run by one whole wavefront.
// Y(r, j): finished dot product of block row r and tile row j (before the norm scale).
// rot: optional LDS copy of the rotary rows, [R][d/2 cos | d/2 sin]; nullptr = read the tables.
// ONE_PASS: the caller guarantees R <= 4, so that one pass of the wavefront covers the row group
// (no loop around the loads and stores below).
template <int EPI, bool ONE_PASS = false, typename YF>
__device__ inline void mv_epilogue(const MvArgs &a, int rg, int lane, const float *rs, const float *rot, YF Y) {
    const int R = a.R, NT = block_terms(a.RL), NC = NT * layout_rows(a.RL);  // NC: column pitch of the split outputs
    if (EPI == EPI_RESID || EPI == EPI_LOGITS) {
        const int iters = ONE_PASS ? 1 : (16 * R + 63) >> 6;
        for (int it = 0; it < iters; ++it) {
            const int idx = it * 64 + lane;
            const int r = idx >> 4, j = idx & 15;
            const int row = 16 * rg + j;
            const bool ok = r < R && row < a.O;
            if (EPI == EPI_LOGITS) {
                if (ok) a.out_f32[(size_t)r * a.ld_out + row] = Y(r, j) * rs[r];
            } else {
                float xn = 0.f;
                if (ok) {
                    float *xp = a.out_f32 + (size_t)r * a.ld_out + row;
                    xn = *xp + Y(r, j);
                    *xp = xn;
                    uint16_t hi, mid, lo;
                    split3(xn * a.gain_next[row], hi, mid, lo);
                    uint16_t *p = a.out_s + ((size_t)(row >> 3) * NC + NT * r) * 8 + (row & 7);
                    p[0] = hi;
                    p[8] = mid;
                    if (NT == 3) p[16] = lo;
                }
                float ss = xn * xn;
#pragma unroll
                for (int off = 8; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
                if (r < R && j == 0) a.pss_out[(size_t)rg * a.rp + r] = ss;
            }
        }
    } else {
        const int iters = ONE_PASS ? 1 : (8 * R + 63) >> 6;
        for (int it = 0; it < iters; ++it) {
            const int idx = it * 64 + lane;
            const int r = idx >> 3, j = idx & 7;
            if (r >= R) continue;
            const float sc = rs[r];
            const float ya = Y(r, j) * sc, yb = Y(r, j + 8) * sc;
            if (EPI == EPI_SWIGLU) {
                if (2 * (8 * rg + j) < a.O) {
                    uint16_t hi, mid, lo;
                    split3(ya / (1.0f + expf(-ya)) * yb, hi, mid, lo);
                    uint16_t *p = a.out_s + ((size_t)rg * NC + NT * r) * 8 + j;
                    p[0] = hi;
                    p[8] = mid;
                    if (NT == 3) p[16] = lo;
                }
            } else {
                const int d = a.head_dim, half = d >> 1, gph = half >> 3;
                const int hh = rg / gph, i = 8 * (rg - hh * gph) + j;
                const int nq = a.n_q_heads, nkv = a.n_kv_heads, pos = a.pos0 + r, rpos = mv_rope_pos(a, r);
                if (hh < nq + nkv) {
                    const float c = rot ? rot[r * d + i] : a.cos_tab[(size_t)rpos * half + i];
                    const float s = rot ? rot[r * d + half + i] : a.sin_tab[(size_t)rpos * half + i];
                    const float qa = ya * c - yb * s, qb = yb * c + ya * s;
                    if (hh < nq) {
                        float *qp = a.out_f32 + (size_t)r * a.ld_out + hh * d + i;
                        qp[0] = qa;
                        qp[half] = qb;
                        if (a.q_s) {
                            uint16_t *qs = a.q_s + ((size_t)(r * nq + hh) * 2) * d + i;
                            const uint32_t ha = f32_to_bf16_rne_finite(qa), hb = f32_to_bf16_rne_finite(qb);
                            qs[0] = (uint16_t)ha;
                            qs[half] = (uint16_t)hb;
                            qs[d] = (uint16_t)f32_to_bf16_rne_finite(qa - __uint_as_float(ha << 16));
                            qs[d + half] = (uint16_t)f32_to_bf16_rne_finite(qb - __uint_as_float(hb << 16));
                        }
                    } else {
                        uint16_t *kc = (uint16_t *)a.kcache + ((size_t)(hh - nq) * a.max_seq + pos) * d + i;
                        kc[0] = f32_to_bf16_rne(qa);
                        kc[half] = f32_to_bf16_rne(qb);
                    }
                } else if (a.nb32 > 0) {  // values in groups of eight slots
                    uint16_t *vc = (uint16_t *)a.vcache + kv_vt_index(hh - nq - nkv, a.nb32, d, pos, i);
                    vc[0] = f32_to_bf16_rne(ya);
                    vc[half * 8] = f32_to_bf16_rne(yb);
                } else {
                    uint16_t *vc = (uint16_t *)a.vcache + ((size_t)(hh - nq - nkv) * a.max_seq + pos) * d + i;
                    vc[0] = f32_to_bf16_rne(ya);
                    vc[half] = f32_to_bf16_rne(yb);
                }
            }
        }
    }
}

}  // namespace swift
