// gfx950 persistent kernel of the bf16 tiled path: the whole decoder stack (and the LM head) of a
// block of up to four rows in ONE launch.  OFF by default (swift_debug_persistent turns it on): it is
// correct, and measured slower than one launch per stage on this part.
//
// Idea: a weight-streaming projection of a 7B-shaped model lasts 8-30 us, of which about 5 us are
// fixed cost (launch, first-load latency, tail).  Here one workgroup of 16 wavefronts sits on every
// compute unit for the whole pass; a stage (projection or attention) ends with a grid-wide barrier
// on a counter in device memory, and every wavefront's window of sixteen 1 KB weight-tile loads
// rolls on across the stage boundary: the tiles of the next projection are requested while the
// current one finishes, the barrier completes and the next activation is staged.
//
// Measured (7B shape, one row, 512 cached tokens): 9.2 ms per pass against 2.9 ms launch per stage.
// A compute unit returns vector-memory data in request order, so everything the synchronisation
// needs from memory (the epilogue's stores being acknowledged, the arrival, every poll of the
// counter, the staged activation) queues behind the 256 KB of weight tiles that the compute unit
// has in flight: the barrier takes ~40 us instead of the 4-8 us it takes on an idle memory system.
// Polling through the scalar cache path instead reads stale L2 lines for even longer.  Without
// the deep window across the boundary the barrier costs what a launch boundary costs.
#include <math.h>

#include "swift_attn.h"
#include "swift_device.h"
#include "swift_kernels.h"
#include "swift_mv.h"

namespace swift {

namespace {

constexpr int NW = 16;  // wavefronts per workgroup

// Stage descriptors are read from memory with vector loads; everything in them is the same for
// all lanes, so the values are moved to scalar registers (the vector registers are needed for the
// weight window).
template <typename P>
__device__ inline P *uni(P *p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (P *)(((uint64_t)hi << 32) | lo);
}
__device__ inline int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline float uni(float v) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v))); }

__device__ inline MvArgs uni(const MvArgs &g) {
    MvArgs m;
    m.Wt = uni(g.Wt);
    m.O = uni(g.O);
    m.K = uni(g.K);
    m.T = uni(g.T);
    m.n_rg = uni(g.n_rg);
    m.R = uni(g.R);
    m.RL = uni(g.RL);
    m.in_s = uni(g.in_s);
    m.pss = uni(g.pss);
    m.n_pss = uni(g.n_pss);
    m.norm_dim = uni(g.norm_dim);
    m.rp = uni(g.rp);
    m.eps = uni(g.eps);
    m.out_f32 = uni(g.out_f32);
    m.ld_out = uni(g.ld_out);
    m.out_s = uni(g.out_s);
    m.gain_next = uni(g.gain_next);
    m.pss_out = uni(g.pss_out);
    m.kcache = uni(g.kcache);
    m.vcache = uni(g.vcache);
    m.cos_tab = uni(g.cos_tab);
    m.sin_tab = uni(g.sin_tab);
    m.pos0 = uni(g.pos0);
    m.max_seq = uni(g.max_seq);
    m.head_dim = uni(g.head_dim);
    m.n_q_heads = uni(g.n_q_heads);
    m.n_kv_heads = uni(g.n_kv_heads);
    m.tree = 0;  // token trees do not run on this kernel
    m.depth4 = 0;
    m.pf_rows = m.pf_heads = m.n_wg = m.pf_first = m.pf_wgs = 0;
    m.part = nullptr;
    m.counters = nullptr;
    m.part_capacity = 0;
    m.S = 0;
    return m;
}
__device__ inline AttnArgs uni(const AttnArgs &g) {
    AttnArgs t;
    t.q = uni(g.q);
    t.kcache = uni(g.kcache);
    t.vcache = uni(g.vcache);
    t.n_ctx = uni(g.n_ctx);
    t.rows = uni(g.rows);
    t.max_seq = uni(g.max_seq);
    t.head_dim = uni(g.head_dim);
    t.n_q_heads = uni(g.n_q_heads);
    t.n_kv_heads = uni(g.n_kv_heads);
    t.part_o = nullptr;
    t.part_ml = nullptr;
    t.max_split = 0;
    t.out = uni(g.out);
    t.out_s = uni(g.out_s);
    t.out_rows = uni(g.out_rows);
    t.tree = 0;
    t.n_base = 0;
    t.row_base = 0;
    t.depth4 = 0;
    t.spine4 = 0;
    return t;
}

// A wavefront's share of one projection stage.  The k-tiles of a row group are cut into NW slices
// (wavefront w takes slice w); a workgroup takes row groups wgi, wgi + nwg, ... one per round; a
// slice is walked in chunks of 8 tiles.  All fields are wavefront-uniform.
struct Slice {
    const u32x4 *Wt;
    int T, n_rg;
    int t0, nv, nvm1;  // first k-tile of the slice, tiles that exist, max(nv - 1, 0)
    int nch;           // chunks per round
    int nwg, wgi;      // workgroups that share the stage, this workgroup's index among them
    int total;         // chunks of this wavefront in the stage (rounds * nch)
    int total_pad;     // ... rounded up to even (chunks alternate between the two register buffers)
};

// What the load cursor needs to know about a stage; a copy of these fields sits in LDS so that
// looking at the stages ahead costs no global loads (which would queue up behind the weight window).
struct StageLite {
    const u32x4 *Wt;
    int T, n_rg;
    int wg_first;
    int n_units;  // attention stage: pairs (> 0); projection stage: 0
    int pad[2];
};

__device__ inline void slice_init(Slice &w, const StageLite *st, int wave, int wg, int n_wg) {
    w.Wt = st->Wt;
    w.T = st->T;
    w.n_rg = st->n_rg;
    const int n = (w.T + NW - 1) / NW;
    w.t0 = min(wave * n, w.T - 1);
    w.nv = max(0, min(n, w.T - wave * n));
    w.nvm1 = max(w.nv - 1, 0);
    w.nch = (n + 7) >> 3;
    w.nwg = n_wg - st->wg_first;
    w.wgi = wg - st->wg_first;
    const int rounds = (w.wgi >= 0 && w.wgi < w.n_rg) ? (w.n_rg - w.wgi + w.nwg - 1) / w.nwg : 0;
    w.total = rounds * w.nch;
    w.total_pad = (w.total + 1) & ~1;
}

// Where the next chunk of weight tiles comes from: runs two chunks ahead of the arithmetic,
// through the rounds of a stage and on into the next projection stage this workgroup works on.
struct LoadCursor {
    int s;         // stage of the next chunk; n_stages: nothing left
    int q;         // chunk number inside the stage
    int round, chunk;
    bool blocked;  // parked in front of an attention stage that this workgroup computes
    Slice w;
    const u32x4 *base;  // per lane: tile 0 of the slice in the current round's row group
};

__device__ inline void lc_set_base(LoadCursor &c, int lane) {
    const int rg = min(c.round * c.w.nwg + c.w.wgi, c.w.n_rg - 1);
    c.base = c.w.Wt + ((size_t)rg * c.w.T + c.w.t0) * 64 + lane;
}

// Moves to the first projection stage at or after c.s in which this workgroup has work.
__device__ inline void lc_seek(LoadCursor &c, const StageLite *stages, int n_stages, int wave, int wg, int n_wg,
                                int lane) {
    c.blocked = false;
    while (c.s < n_stages) {
        const StageLite *st = stages + c.s;
        if (st->n_units > 0) {
            if (wg < st->n_units) {
                c.blocked = true;  // the attention code needs the registers of the window
                return;
            }
        } else {
            Slice w;
            slice_init(w, st, wave, wg, n_wg);
            if (w.total_pad > 0) {
                c.w = w;
                c.q = 0;
                c.round = 0;
                c.chunk = 0;
                lc_set_base(c, lane);
                return;
            }
        }
        ++c.s;
    }
}

__device__ inline void lc_advance(LoadCursor &c, const StageLite *stages, int n_stages, int wave, int wg, int n_wg,
                                   int lane) {
    if (c.blocked || c.s >= n_stages) return;
    ++c.q;
    if (c.q >= c.w.total_pad) {
        ++c.s;
        lc_seek(c, stages, n_stages, wave, wg, n_wg, lane);
        return;
    }
    if (c.q < c.w.total) {
        if (++c.chunk == c.w.nch) {
            c.chunk = 0;
            ++c.round;
            lc_set_base(c, lane);
        }
    }
    // else: the padding chunk of an odd stage repeats the last chunk's (clamped) loads
}

// Loads past the end of a slice repeat its last tile (a cache hit); nothing is ever read from
// outside the matrix the cursor last pointed into.
// (The pointer comes out of a descriptor in memory, so the compiler cannot tell that it is a global
// address; said explicitly, the load is a global_load, which does not tie up the LDS counter.)
typedef __attribute__((address_space(1))) const u32x4 global_u32x4;
__device__ inline u32x4 lc_load(const LoadCursor &c, int u) {
    const global_u32x4 *p = (const global_u32x4 *)(c.base + (size_t)min(c.chunk * 8 + u, c.w.nvm1) * 64);
    return __builtin_nontemporal_load(p);
}

// Grid-wide barrier k of this launch is complete when the counter has reached
// barrier_base + (k + 1) * gridDim.x.  A workgroup arrives once per stage with ONE acquire-release
// read-modify-write, done by a wavefront whose own stores are complete and at a point where all
// stores of the workgroup for that stage are complete; waiting polls with a bound.
__device__ inline void grid_arrive_one(const StackArgs &a) {
    __hip_atomic_fetch_add(a.barrier, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline bool grid_wait(const StackArgs &a, unsigned target, int *flag /* LDS */) {
    if (threadIdx.x == 0) {
        int spins = 0, ok = 1;
        while ((int)(__hip_atomic_load(a.barrier, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
            if (++spins > a.spin_limit) {
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(2);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if (!ok) __hip_atomic_store(a.error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = ok;
    }
    lds_barrier();
    return *flag != 0;
}

}  // namespace

template <int GROUP>
__global__ __launch_bounds__(1024) void k_stack(StackArgs a) {
    const StackStage *stages = a.stages;
    const int n_stages = a.n_stages;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wg = blockIdx.x, n_wg = gridDim.x;
    const int col = lane & 15, kg = lane >> 4;
    // LDS: [16 B zeros][activation | attention scratch: act_bytes][2 x NW x NC x 16 fp32][16 scales]
    //      [1024 scratch][R x d rotary][flag][n_stages x StageLite]
    const int R = a.R, NC = 3 * R;
    if (tid < 4) ((uint32_t *)smem)[tid] = 0u;
    float *red = (float *)(smem + 16 + (size_t)a.act_bytes);
    float *rs = red + 2 * NW * 16 * NC;
    float *nscratch = rs + 16;
    float *rot = nscratch + 1024;
    int *flag = (int *)(rot + R * a.head_dim);
    float *att_sh = (float *)(smem + 16);
    StageLite *lite = (StageLite *)(flag + 4);
    for (int i = tid; i < n_stages; i += 1024) {
        const StackStage *st = stages + i;
        StageLite l;
        l.Wt = (const u32x4 *)st->mv.Wt;
        l.T = st->mv.T;
        l.n_rg = st->mv.n_rg;
        l.wg_first = st->wg_first;
        l.n_units = st->type == ST_ATTN ? st->n_units : 0;
        l.pad[0] = l.pad[1] = 0;
        lite[i] = l;
    }
    __syncthreads();

    u32x4 bufA[8], bufB[8];
    LoadCursor lc;
    lc.s = 0;
    lc.q = lc.round = lc.chunk = 0;
    lc.base = nullptr;
    lc_seek(lc, lite, n_stages, wave, wg, n_wg, lane);
    auto prime = [&]() {
        if (lc.blocked || lc.s >= n_stages) return;
#pragma unroll
        for (int u = 0; u < 8; ++u) bufA[u] = lc_load(lc, u);
        lc_advance(lc, lite, n_stages, wave, wg, n_wg, lane);
#pragma unroll
        for (int u = 0; u < 8; ++u) bufB[u] = lc_load(lc, u);
        lc_advance(lc, lite, n_stages, wave, wg, n_wg, lane);
    };
    prime();

    for (int s = 0; s < n_stages; ++s) {
        const StackStage *st = stages + s;
        if (s > 0) {
            if (!grid_wait(a, a.barrier_base + (unsigned)s * (unsigned)n_wg, flag)) return;
        }
        const bool traced = a.trace && tid == 0 && (wg == 0 || wg == n_wg - 1);
        uint64_t *trace = a.trace + ((size_t)(wg == 0 ? 0 : 1) * n_stages + s) * 2;
        if (traced) trace[0] = wall_clock64();
        bool worked = false;  // a projection stage in which this workgroup arrives from its last epilogue
        if (lite[s].n_units > 0) {
            if (wg < lite[s].n_units) {
                AttnArgs at = uni(st->at);
                at.n_ctx = a.pos0 + 1;
                attn_head_unit<BF16T, GROUP>(at, wg % at.n_kv_heads, wg / at.n_kv_heads, att_sh);
                // the window was not kept over the attention: start it again behind this stage
                lc.s = s + 1;
                lc_seek(lc, lite, n_stages, wave, wg, n_wg, lane);
                prime();
            }
        } else {
            Slice w;
            slice_init(w, lite + s, wave, wg, n_wg);
            if (w.total_pad > 0) {
                worked = true;
                MvArgs m = uni(st->mv);
                m.pos0 = a.pos0;
                const int epi = uni(st->epi);
                // ---- stage the split activation, the norm scale and the rotary rows
                {
                    const u32x4 *src = (const u32x4 *)m.in_s;
                    u32x4 *dst = (u32x4 *)(smem + 16);
                    const int n_units = m.T * 4 * NC, real_units = (m.K >> 3) * NC;
                    const u32x4 zero = {0u, 0u, 0u, 0u};
                    for (int i0 = 0; i0 < n_units; i0 += 4 * 1024) {
                        u32x4 tmp[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int i = i0 + tid + 1024 * q;
                            tmp[q] = i < real_units ? src[i] : zero;
                        }
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int i = i0 + tid + 1024 * q;
                            if (i < n_units) dst[i] = tmp[q];
                        }
                    }
                    if (epi == EPI_QKV) {
                        const int d = m.head_dim, half = d >> 1;
                        for (int i = tid; i < R * half; i += 1024) {
                            const int r = i / half, e = i - r * half;
                            rot[r * d + e] = m.cos_tab[(size_t)(m.pos0 + r) * half + e];
                            rot[r * d + half + e] = m.sin_tab[(size_t)(m.pos0 + r) * half + e];
                        }
                    }
                    // RMSNorm scale per row from the producer's partial sums of squares, fixed order
                    const int r = tid & 15, qg = tid >> 4;
                    if (m.pss) {
                        float ss = 0.f;
                        for (int p0 = 0; p0 < m.n_pss; p0 += 256) {
                            float v[4];
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                const int p = p0 + qg + 64 * u;
                                v[u] = p < m.n_pss ? m.pss[(size_t)p * m.rp + r] : 0.f;
                            }
#pragma unroll
                            for (int u = 0; u < 4; ++u) ss += v[u];
                        }
                        nscratch[qg * 16 + r] = ss;
                    }
                    __syncthreads();
                    if (tid < 16) {
                        float ss = 0.f;
                        if (m.pss)
                            for (int q2 = 0; q2 < 64; ++q2) ss += nscratch[q2 * 16 + tid];
                        rs[tid] = m.pss ? 1.0f / sqrtf(ss / (float)m.norm_dim + m.eps) : 1.0f;
                    }
                    __syncthreads();
                }

                // byte address of this lane's B chunk for tile t: boff + t * bstride; lanes of
                // columns >= NC (and masked slots) read the zero chunk at address 0
                const int boff = col < NC ? 16 + (kg * NC + col) * 16 : 0;
                const int bstride = col < NC ? 64 * NC : 0;
                int round = 0, chunk = 0;
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};

                auto round_end = [&]() {
                    const int rg = round * w.nwg + w.wgi;
                    float *rp = red + (size_t)(round & 1) * (NW * 16 * NC);
                    // (the lane number is made opaque here so that the per-lane addresses of this
                    // rarely executed code are computed on the spot instead of being kept in
                    // registers, or spilled, across the streaming loop)
                    int lane_l = lane;
                    asm volatile("" : "+v"(lane_l));
                    const int col_l = lane_l & 15, kg_l = lane_l >> 4;
                    if (col_l < NC) {
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) rp[(wave * NC + col_l) * 16 + 4 * kg_l + r4] = acc[r4];
                    }
                    lds_barrier();
                    if (wave == (round & (NW - 1))) {
                        auto Y = [&](int r, int j) {
                            float y = 0.f;
#pragma unroll 1
                            for (int k2 = 0; k2 < NW; ++k2) {
                                const float *wv = rp + (k2 * NC + 3 * r) * 16 + j;
                                y += (wv[0] + wv[16]) + wv[32];
                            }
                            return y;
                        };
                        switch (epi) {
                            case EPI_QKV: mv_epilogue<EPI_QKV, true>(m, rg, lane_l, rs, rot, Y); break;
                            case EPI_RESID: mv_epilogue<EPI_RESID, true>(m, rg, lane_l, rs, nullptr, Y); break;
                            case EPI_SWIGLU: mv_epilogue<EPI_SWIGLU, true>(m, rg, lane_l, rs, nullptr, Y); break;
                            default: mv_epilogue<EPI_LOGITS, true>(m, rg, lane_l, rs, nullptr, Y); break;
                        }
                        // Results are in the cache hierarchy before this wavefront goes on to a
                        // barrier.  After the last round it also arrives for the workgroup: every
                        // earlier round's epilogue wavefront passed this point before the barrier
                        // above, so all of the workgroup's stores of this stage are complete.
                        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                        if ((round + 1) * w.nch == w.total && s + 1 < n_stages && lane_l == 0) grid_arrive_one(a);
                    }
                    chunk = 0;
                    ++round;
                    acc = f32x4{0.f, 0.f, 0.f, 0.f};
                };
                auto step = [&](u32x4(&buf)[8], int qq) {
                    const int vm = qq < w.total ? -1 : 0;  // padding chunk: arithmetic on zeros
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int i = chunk * 8 + u;
                        const int msk = (i < w.nv) ? vm : 0;
                        const int addr = (boff + (w.t0 + i) * bstride) & msk;
                        const u32x4 bv = *(const u32x4 *)(smem + addr);
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, buf[u]),
                                                                      __builtin_bit_cast(bf16x8, bv), acc, 0, 0, 0);
                        buf[u] = lc_load(lc, u);
                    }
                    lc_advance(lc, lite, n_stages, wave, wg, n_wg, lane);
                    if (vm) {
                        if (++chunk == w.nch) round_end();
                    }
                };
                for (int qq = 0; qq < w.total_pad; qq += 2) {
                    step(bufA, qq);
                    step(bufB, qq + 1);
                }
            }
        }
        if (traced) trace[1] = wall_clock64();
        if (s + 1 < n_stages && !worked) {
            // nothing of this stage's projection here (or attention: all stores waited for below)
            __syncthreads();
            if (tid == 0) grid_arrive_one(a);
        }
    }
}

hipError_t launch_stack(const StackArgs &a, int group, size_t lds, int n_wg, hipStream_t s) {
    if (lds > kStackMaxLds || n_wg < 1 || a.n_stages < 1) return hipErrorInvalidValue;
#define SWIFT_STACK_CASE(G)                                                                              \
    case G: {                                                                                            \
        static bool attr_set = false;                                                                    \
        if (!attr_set) {                                                                                 \
            hipError_t e = hipFuncSetAttribute((const void *)k_stack<G>,                                 \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStackMaxLds); \
            if (e != hipSuccess) return e;                                                               \
            attr_set = true;                                                                             \
        }                                                                                                \
        hipLaunchKernelGGL(k_stack<G>, dim3(n_wg), dim3(kStackThreads), lds, s, a);                      \
        return hipGetLastError();                                                                        \
    }
    switch (group) {
        SWIFT_STACK_CASE(1)
        SWIFT_STACK_CASE(2)
        SWIFT_STACK_CASE(4)
        SWIFT_STACK_CASE(8)
    }
#undef SWIFT_STACK_CASE
    return hipErrorInvalidValue;
}

}  // namespace swift
