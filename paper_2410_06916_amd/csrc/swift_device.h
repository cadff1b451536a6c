// Device-side helpers shared by the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swift {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 128-bit load
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// fp32 -> bf16 bits, round to nearest even (NaN stays NaN)
__device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
// same for finite inputs only (no NaN test)
__device__ inline uint32_t f32_to_bf16_rne_finite(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// v = hi + mid + lo exactly (three bf16 terms carry the 24-bit significand of an fp32 value)
__device__ inline void split3(float v, uint16_t &hi, uint16_t &mid, uint16_t &lo) {
    const uint32_t h = f32_to_bf16_rne_finite(v);
    const float r1 = v - __uint_as_float(h << 16);
    const uint32_t m = f32_to_bf16_rne_finite(r1);
    const float r2 = r1 - __uint_as_float(m << 16);
    hi = (uint16_t)h;
    mid = (uint16_t)m;
    lo = (uint16_t)f32_to_bf16_rne_finite(r2);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// load and store of the wavefront (its release fence covers global memory), which would drain a
// window of weight loads that is deliberately kept in flight across the barrier.
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

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

}  // namespace swift
