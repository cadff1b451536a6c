// Projections of a prompt macro block: up to kMacroSub sub-blocks of 64 rows through one weight matrix in
// one launch, as a blocked matrix product on the matrix cores (paper Section 4.2: the pass over the input
// that fills the cache before drafting starts; Section 3.1: the rows of a block are independent given the
// cache, so any number of them may share one sweep over the weights).
//
// A workgroup of 8 wavefronts owns a tile of WM RGW 16-row groups of W times WN sub-blocks (WN x 64 rows x 2
// bf16 terms = 128 WN columns; WM WN = 8, WN = 2 or 1).  Wavefront (wm, wn) = (w % WM, w / WM) owns RGW row groups
// times the 128 columns of sub-block wn: 8 RGW accumulator tiles.  Both operands reach LDS straight from global
// memory (no registers in between) through a ring of NST stages of one 32-deep k tile each: WM RGW weight tiles
// of 1 KB (already in A-operand order) and the sub-blocks' 8 KB of split activations each (already in B-operand
// order).  In step t the operands of stage t + 1 are read from LDS and stage t is multiplied while stages
// t + 2 .. t + NST - 1 are on their way and stage t + NST is requested: what a compute unit can take in is
// bounded by the bytes it keeps in flight, and the ring is what keeps most of LDS in flight.  One barrier per
// stage.
//
// The workgroups that share a weight tile (the other column tiles of the macro block) and those that
// share activations (the other row tiles) are given consecutive positions on one die, so that what one of
// them pulls from memory the others find in that die's L2.
//
// The epilogue is the block kernel's (mv_epilogue), run per (row group, sub-block) on that sub-block's
// buffers: every sub-block ends up exactly as laid out for a 64-row block of the bulk layout.
//
// Where the tiles alone would leave compute units idle -- a matrix of few rows (o_proj, down_proj) under a macro
// block of two to four sub-blocks: a prompt of 65-256 tokens, a candidate-evaluation window of more than 64 -- the
// depth is split over two or four workgroups per tile as well (gridDim.y): each publishes its results, the
// workgroup that arrives last at the tile's counter adds them in part order and runs the epilogue.
#include <math.h>

#include <type_traits>

#include "swift_device.h"
#include "swift_kernels.h"
#include "swift_mv.h"

namespace swift {

namespace {

constexpr int kRingBytes = 144 * 1024;   // most of LDS: what is in flight bounds what a compute unit takes in
constexpr int kNormFloats = 2 * 16 * 64;  // scratch of gemm_norm_scales

// RMSNorm scales of the workgroup's two sub-blocks: rs[64 wn + r].  Thread (wn, q, r4) adds the partials q, q + 16,
// .. of rows 4 r4 .. 4 r4 + 3 of sub-block wn (16 loads of 16 bytes in flight at a time); then one thread per row
// adds the sixteen sums in order.
__device__ inline void gemm_norm_scales(const MvArgs &a, const MacroArgs &ma, int sub0, float *rs, float *scratch) {
    const int tid = threadIdx.x, r4 = tid & 15, q = (tid >> 4) & 15, wn = tid >> 8;
    const int sub = min(sub0 + wn, ma.S - 1);
    if (a.pss) {
        const float *p = a.pss + (size_t)sub * ma.pss + 4 * r4;
        f32x4 ss = {0.f, 0.f, 0.f, 0.f};
        for (int p0 = 0; p0 < a.n_pss; p0 += 256) {
            f32x4 v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int i = p0 + q + 16 * u;
                v[u] = i < a.n_pss ? *(const f32x4 *)(p + (size_t)i * a.rp) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) ss += v[u];
        }
        *(f32x4 *)(scratch + (wn * 16 + q) * 64 + 4 * r4) = ss;
    }
    __syncthreads();
    if (tid < 128) {
        const int w2 = tid >> 6, r2 = tid & 63;
        float ss = 0.f;
        if (a.pss)
            for (int q2 = 0; q2 < 16; ++q2) ss += scratch[(w2 * 16 + q2) * 64 + r2];
        rs[tid] = a.pss ? 1.0f / sqrtf(ss / (float)a.norm_dim + a.eps) : 1.0f;
    }
}

template <int RGW>
struct GemmOperands {
    u32x4 av[RGW], bv[8];
};

template <int EPI, int WN, int RGW>
__global__ __launch_bounds__(512) void k_gemm(MvArgs a, MacroArgs ma, int MT, int NN, int TS) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int WM = 8 / WN;                    // wavefronts along the rows; WN sub-blocks side by side
    constexpr int TRG = WM * RGW;                 // row groups of the workgroup's tile
    constexpr int A_BYTES = TRG * 1024;
    constexpr int ST_BYTES = A_BYTES + WN * 8192;
    constexpr int NST = kRingBytes / ST_BYTES;   // stages of the ring
    constexpr int NP = TRG + 8 * WN;              // 1 KB pieces of a stage
    constexpr int PW = (NP + 7) / 8;              // pieces a wavefront copies per stage (PW - 1 past the remainder)
    static_assert(NST >= 3 && NST * PW < 64, "ring depth against the load counter");
    unsigned char *ring = smem;
    float *rs = (float *)(smem + kRingBytes);     // [2][64]
    float *nscratch = rs + 128;                   // [kNormFloats]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    // workgroup -> tile: the NN column tiles of a row tile sit next to each other on one die (consecutive
    // workgroup ids go round the 8 dies)
    const int id = blockIdx.x, die = id & 7, qd = id >> 3;
    const int nt = qd % NN, mt = (qd / NN) * 8 + die;
    if (mt >= MT) return;
    const int sub0 = WN * nt;
    const int T = a.T;
    const int col = lane & 15, kg = lane >> 4;
    // gridDim.y > 1: the depth is split over workgroups, TS k tiles each (matrices of few rows under a macro block of
    // few sub-blocks would otherwise leave most compute units idle); the parts' results are added at the end
    const int KSP = gridDim.y, kz = blockIdx.y;
    const int t_lo = kz * TS, t_hi = min(T, t_lo + TS);  // (every part holds tiles: the launcher)

    // ---- what this wavefront copies per stage: pieces p = wave + 8 i, each 64 lanes x 16 bytes from a
    // wavefront-uniform address
    const unsigned char *src[PW];   // tile 0 of the piece (wavefront-uniform)
    int stride[PW];                 // bytes from one k tile to the next
    int seg64[PW];                  // B pieces: first 16-byte unit of the piece inside its tile (A pieces: -1)
    uint32_t voff[PW];              // this lane's byte offset from src[i] in the next stage to be issued
#pragma unroll
    for (int i = 0; i < PW; ++i) {
        const int p = wave + 8 * i;
        if (p < TRG) {
            const int rg = min(mt * TRG + p, a.n_rg - 1);  // row groups past the end repeat the last one
            src[i] = (const unsigned char *)a.Wt + (size_t)rg * T * 1024;
            stride[i] = 1024;
            seg64[i] = -1;
        } else {
            const int q = min(p, NP - 1) - TRG, sb = min(sub0 + (q >> 3), ma.S - 1), seg = q & 7;
            src[i] = (const unsigned char *)(a.in_s + (size_t)sb * ma.in_s) + seg * 1024;
            stride[i] = 8192;
            seg64[i] = seg * 64;
        }
        voff[i] = lane * 16 + t_lo * stride[i];
    }
    const bool full_share = (NP % 8 == 0) || wave < NP % 8;  // this wavefront copies PW pieces (else PW - 1)
    // FULL: whether this wavefront copies PW pieces (a compile-time copy of full_share)
    auto issue = [&](int slot_bytes, auto FULL) {
        unsigned char *dst = ring + slot_bytes + wave * 1024;
#pragma unroll
        for (int i = 0; i < PW; ++i) {
            if (i < PW - 1 || decltype(FULL)::value)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[i] + (size_t)voff[i]),
                                                 (__attribute__((address_space(3))) void *)(dst + i * 8192), 16, 0, 0);
            voff[i] += stride[i];
        }
    };
    // waits until at most N stages' worth of this wavefront's loads are in flight (loads complete in order; every
    // stage is the same number of loads per lane)
    auto wait_all_but = [&](auto N, auto FULL) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(decltype(N)::value * (decltype(FULL)::value ? PW : PW - 1)) : "memory");
    };
    // (the wait as a builtin: the compiler follows it, unlike one inside inline assembly, and so does not add a
    // wait of its own for the operand reads of the previous step in front of the matrix instructions)
    auto lds_sync = [&]() {
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wavefront's LDS reads and writes are done
        asm volatile("s_barrier" ::: "memory");
    };

    f32x4 acc[RGW][8];
#pragma unroll
    for (int g = 0; g < RGW; ++g)
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) acc[g][cb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // A ragged last k tile (depth not a multiple of 32) is not part of the pipeline: it is handled at the end (by
    // the part that holds it).  TF: full tiles of this workgroup's part; TR: the ragged tile's number, if it is here.
    const bool ragged = (a.K & 31) != 0 && t_hi == T;
    const int TF = t_hi - t_lo - (ragged ? 1 : 0), TR = T - 1;
    const unsigned char *a_base = ring + (wm * RGW) * 1024 + lane * 16;
    const unsigned char *b_base = ring + A_BYTES + wn * 8192 + (kg * 128 + col) * 16;
    // (wavefronts without a sub-block -- an odd sub-block count leaves half of the last column tile empty -- go
    // through the motions on the last sub-block's data; their results are dropped)
    auto read_operands = [&](int slot_bytes, GemmOperands<RGW> &o) {
#pragma unroll
        for (int g = 0; g < RGW; ++g) o.av[g] = *(const u32x4 *)(a_base + slot_bytes + g * 1024);
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) o.bv[cb] = *(const u32x4 *)(b_base + slot_bytes + cb * 256);
    };
    auto multiply = [&](const GemmOperands<RGW> &o) {
#pragma unroll
        for (int g = 0; g < RGW; ++g)
#pragma unroll
            for (int cb = 0; cb < 8; ++cb)
                acc[g][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, o.av[g]),
                                                                     __builtin_bit_cast(bf16x8, o.bv[cb]), acc[g][cb], 0, 0, 0);
    };

    // The pipeline.  Step t: the operands of stage t are in registers (read during step t - 1).  Once stage t + 1
    // has landed for everybody -- and everybody's reads of stage t have completed: the barrier waits for them --
    // stage t + NST is requested into the slot stage t leaves, the operands of stage t + 1 are read into the other
    // register set, and the matrix cores work on stage t meanwhile.  `slot`: byte offset of stage t's ring slot.
    // The loop body is kept free of conditions: a wavefront issues at most one scalar instruction every few cycles,
    // and whatever the loop needs beyond the matrix instructions is paid for in full.
    auto pipeline = [&](auto FULL) {
        constexpr auto ALL = std::integral_constant<int, 0>();
        constexpr auto AHEAD = std::integral_constant<int, NST - 2>();  // stages t + 2 .. t + NST - 1 may stay in flight
#pragma unroll
        for (int t = 0; t < NST; ++t)
            if (t < TF) issue(t * ST_BYTES, FULL);
        gemm_norm_scales(a, ma, sub0, rs, nscratch);
        if (TF == 0) return;
        GemmOperands<RGW> o0, o1;
        wait_all_but(ALL, FULL);
        lds_sync();
        read_operands(0, o0);
        int t = 0, slot = 0;
        auto next_slot = [&](int sl) { return sl + ST_BYTES == NST * ST_BYTES ? 0 : sl + ST_BYTES; };
        auto steady = [&](const GemmOperands<RGW> &cur, GemmOperands<RGW> &nxt) {
            const int nslot = next_slot(slot);
            wait_all_but(AHEAD, FULL);
            lds_sync();
            issue(slot, FULL);
            read_operands(nslot, nxt);
            // (the reads stay in front of the matrix instructions: left alone, the scheduler sinks them behind to
            // save registers, and LDS and the matrix cores then take turns instead of working side by side)
            __builtin_amdgcn_sched_barrier(0);
            multiply(cur);
            slot = nslot;
        };
        // (the last step reads a slot nobody needs: no harm)
        auto drain = [&](const GemmOperands<RGW> &cur, GemmOperands<RGW> &nxt) {
            const int nslot = next_slot(slot);
            wait_all_but(ALL, FULL);
            lds_sync();
            read_operands(nslot, nxt);
            __builtin_amdgcn_sched_barrier(0);
            multiply(cur);
            slot = nslot;
        };
        for (; t + NST + 1 < TF; t += 2) {  // both steps issue a stage
            steady(o0, o1);
            steady(o1, o0);
        }
        if (t + NST < TF) {  // an odd number of issuing steps: one more, then the operands sit in the other set
            steady(o0, o1);
            drain(o1, o0);
            t += 2;
        }
        for (; t < TF; t += 2) {
            drain(o0, o1);
            if (t + 1 < TF) drain(o1, o0);
        }
    };
    if (full_share)
        pipeline(std::true_type());
    else
        pipeline(std::false_type());
    if (ragged) {
        // the ragged tile: copied with ordinary loads, zeros past the real depth (a piece lies wholly inside or
        // wholly outside it), into the first ring slot
        const int real_units = (a.K >> 3) * 128;  // 16-byte units of a sub-block's split activation
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PW; ++i) {
            if (i < PW - 1 || full_share) {
                const bool past = seg64[i] >= 0 && seg64[i] + TR * 512 >= real_units;
                const unsigned char *sp = src[i] + (size_t)TR * stride[i];
                const u32x4 v = past ? u32x4{0u, 0u, 0u, 0u} : *(const u32x4 *)(sp + lane * 16);
                *(u32x4 *)(ring + wave * 1024 + i * 8192 + lane * 16) = v;
            }
        }
        __syncthreads();
        GemmOperands<RGW> o;
        read_operands(0, o);
        multiply(o);
    }

    // ---- epilogue per row group: results to LDS (dump[wave][column][tile row]), then the block kernel's epilogue
    // on the sub-block's own buffers
    const int sub = min(sub0 + wn, ma.S - 1);
    MvArgs as = a;
    as.R = sub == ma.S - 1 ? ma.rows_last : 64;
    as.pos0 = a.pos0 + 64 * sub;
    as.in_s = a.in_s + (size_t)sub * ma.in_s;
    if (a.out_f32) as.out_f32 = a.out_f32 + (size_t)sub * ma.out_f32;
    if (a.out_s) as.out_s = a.out_s + (size_t)sub * ma.out_s;
    if (a.pss_out) as.pss_out = a.pss_out + (size_t)sub * ma.pss_out;
    if (a.q_s) as.q_s = a.q_s + (size_t)sub * ma.q_s;
    float *dw = (float *)ring + (size_t)wave * 2048;
    const bool wave_live = sub0 + wn < ma.S;
    const float *rsw = rs + 64 * wn;
    auto dump = [&](int g) {
        __syncthreads();  // the ring / the previous dump is no longer read
#pragma unroll
        for (int cb = 0; cb < 8; ++cb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) dw[(16 * cb + col) * 16 + 4 * kg + r4] = acc[g][cb][r4];
        __syncthreads();
    };
    if (KSP == 1) {
#pragma unroll
        for (int g = 0; g < RGW; ++g) {
            const int rg = (mt * WM + wm) * RGW + g;
            dump(g);
            if (wave_live && rg < a.n_rg)
                mv_epilogue<EPI>(as, rg, lane, rsw, nullptr,
                                 [&](int r, int j) { return dw[(2 * r) * 16 + j] + dw[(2 * r + 1) * 16 + j]; });
        }
        return;
    }
    // ---- depth split over workgroups: every part publishes its results, the two terms combined, as
    // part[(kz n_rg + rg) S + sub][row][tile row]; the workgroup that arrives last at the tile's counter adds the
    // parts in part order (so the result does not depend on who is last) and runs the epilogue.
    // (device-scope atomic stores write through, so thread 0's release has nothing to flush; the barrier orders every
    // wavefront's stores before it)
    const size_t pslot = 1024;
#pragma unroll
    for (int g = 0; g < RGW; ++g) {
        const int rg = (mt * WM + wm) * RGW + g;
        dump(g);
        if (wave_live && rg < a.n_rg) {
            float *pp = a.part + (((size_t)kz * a.n_rg + rg) * ma.S + sub) * pslot;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int idx = lane + 64 * i, r = idx >> 4, j = idx & 15;
                __hip_atomic_store(pp + idx, dw[(2 * r) * 16 + j] + dw[(2 * r + 1) * 16 + j], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    int *flag = (int *)nscratch;
    __syncthreads();
    if (tid == 0) {
        const int old = __hip_atomic_fetch_add(a.counters + mt * NN + nt, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        *flag = (old == KSP - 1) ? 1 : 0;
    }
    __syncthreads();
    if (*flag == 0) return;
    // (plain loads below: ordered after thread 0's acquire by the barrier)
#pragma unroll
    for (int g = 0; g < RGW; ++g) {
        const int rg = (mt * WM + wm) * RGW + g;
        const bool live = wave_live && rg < a.n_rg;
        __syncthreads();  // the previous dump is no longer read
        if (live) {
            const float *p0 = a.part + ((size_t)rg * ma.S + sub) * pslot + lane * 4;
            const size_t kstride = (size_t)a.n_rg * ma.S * pslot;
            f32x4 sum[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) sum[q] = *(const f32x4 *)(p0 + 256 * q);
            for (int k2 = 1; k2 < KSP; ++k2) {
                f32x4 v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) v[q] = *(const f32x4 *)(p0 + k2 * kstride + 256 * q);
#pragma unroll
                for (int q = 0; q < 4; ++q) sum[q] += v[q];
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) *(f32x4 *)(dw + lane * 4 + 256 * q) = sum[q];
        }
        __syncthreads();
        if (live) mv_epilogue<EPI>(as, rg, lane, rsw, nullptr, [&](int r, int j) { return dw[r * 16 + j]; });
    }
    if (tid == 0) a.counters[mt * NN + nt] = 0;
}

template <int EPI, int WN, int RGW>
hipError_t launch_gemm_t(const MvArgs &a, const MacroArgs &ma, int ksp, hipStream_t s) {
    static bool attr_set = false;
    const size_t lds = kRingBytes + 128 * 4 + kNormFloats * 4;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm<EPI, WN, RGW>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    constexpr int TRG = (8 / WN) * RGW;
    const int MT = (a.n_rg + TRG - 1) / TRG, NN = (ma.S + WN - 1) / WN;
    const int grid = ((MT + 7) / 8) * 8 * NN;
    const int TS = (a.T + ksp - 1) / ksp;
    ksp = (a.T + TS - 1) / TS;  // parts that hold tiles
    if (ksp > 1 && (!a.part || !a.counters || (int64_t)ksp * a.n_rg * ma.S > a.part_capacity || MT * NN > 4096))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL((k_gemm<EPI, WN, RGW>), dim3(grid, ksp), dim3(512), lds, s, a, ma, MT, NN, TS);
    return hipGetLastError();
}

// Tilings: code 1..4 = two sub-blocks side by side (workgroup tile 64 RGW rows x 256 columns, RGW = the code),
// 5, 6 = one sub-block (tile 128 or 256 rows x 128 columns: for matrices with few rows, where the narrower tile
// gives as many workgroups with fewer bytes to copy per product).
struct GemmTiling {
    int wn, rgw;
};
constexpr GemmTiling kGemmTilings[7] = {{0, 0}, {2, 1}, {2, 2}, {2, 3}, {2, 4}, {1, 1}, {1, 2}};

// Depth parts for a tiling: 1 unless the tiles leave compute units idle; then the largest of 2, 4 that still gives
// at most one workgroup per compute unit, parts of at least 16 k tiles, and partial results that fit the scratch.
// Only for macro blocks of up to four sub-blocks: with more, the parts' results are too many bytes (measured at
// eight sub-blocks, same machine: down_proj 128-131 us with four parts against 113 us unsplit).
int gemm_depth_parts(const MvArgs &a, const MacroArgs &ma, int n_cu, int code) {
    const int wn = kGemmTilings[code].wn, rgw = kGemmTilings[code].rgw, trg = (8 / wn) * rgw;
    const int MT = (a.n_rg + trg - 1) / trg, NN = (ma.S + wn - 1) / wn;
    int ksp = 1;
    while (ma.S <= 4 && ksp < 4 && MT * NN * ksp * 2 <= n_cu && a.T / (ksp * 2) >= 16 && a.part && a.counters &&
           (int64_t)ksp * 2 * a.n_rg * ma.S <= a.part_capacity && MT * NN <= 4096)
        ksp *= 2;
    return ksp;
}

int gemm_tiling(const MvArgs &a, const MacroArgs &ma, int n_cu) {
    // The one that finishes first by a simple count: rounds of workgroups (one per compute unit) times the k tiles
    // of a workgroup times the longer of a stage's multiply time and the time to take its bytes in (about 21 bytes
    // per cycle and compute unit when the units of a die stream the same data: measured), plus, with the depth
    // split, what publishing and adding the parts costs (measured: about 20 us, and the parts' bytes written and read
    // at about 3 TB/s).
    int best = 1;
    double best_t = 1e30;
    for (int code = 1; code <= 6; ++code) {
        const int wn = kGemmTilings[code].wn, rgw = kGemmTilings[code].rgw, trg = (8 / wn) * rgw;
        const int MT = (a.n_rg + trg - 1) / trg, NN = (ma.S + wn - 1) / wn;
        const int ksp = gemm_depth_parts(a, ma, n_cu, code);
        const int rounds = (MT * NN * ksp + n_cu - 1) / n_cu;
        const double mfma = 256.0 * rgw, intake = (trg + 8.0 * wn) * 1024.0 / 21.0;  // cycles per stage
        const double parts = ksp > 1 ? 45000.0 + 2.0 * ksp * a.n_rg * ma.S * 4096.0 * 0.0007 : 0.0;
        const double t = rounds * ((a.T + ksp - 1) / ksp) * (mfma > intake ? mfma : intake) + parts;
        if (t < best_t) {
            best_t = t;
            best = code;
        }
    }
    return best;
}

}  // namespace

hipError_t launch_gemm(int epi, const MvArgs &a, const MacroArgs &ma, int n_cu, int tiling_override, hipStream_t s) {
    if (ma.S < 1 || ma.S > kMacroSub || ma.rows_last < 1 || ma.rows_last > 64 || a.RL != (64 | kBulkLayout) || a.rp != 64 ||
        (a.K & 7) != 0 || a.T != (a.K + 31) / 32 || a.n_rg < 1 || !a.Wt || !a.in_s || a.tree)
        return hipErrorInvalidValue;
    const int code = (tiling_override >= 1 && tiling_override <= 6) ? tiling_override : gemm_tiling(a, ma, n_cu);
    const int ksp = gemm_depth_parts(a, ma, n_cu, code);
#define SWIFT_GEMM_CASE(E)                                                \
    case E:                                                               \
        switch (code) {                                                   \
            case 1: return launch_gemm_t<E, 2, 1>(a, ma, ksp, s);         \
            case 2: return launch_gemm_t<E, 2, 2>(a, ma, ksp, s);         \
            case 3: return launch_gemm_t<E, 2, 3>(a, ma, ksp, s);         \
            case 4: return launch_gemm_t<E, 2, 4>(a, ma, ksp, s);         \
            case 5: return launch_gemm_t<E, 1, 1>(a, ma, ksp, s);         \
            default: return launch_gemm_t<E, 1, 2>(a, ma, ksp, s);        \
        }
    switch (epi) {
        SWIFT_GEMM_CASE(EPI_QKV)
        SWIFT_GEMM_CASE(EPI_RESID)
        SWIFT_GEMM_CASE(EPI_SWIGLU)
    }
#undef SWIFT_GEMM_CASE
    return hipErrorInvalidValue;
}

}  // namespace swift
