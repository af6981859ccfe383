// Shared device helpers of the dynadiag kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dd {

constexpr int kWave = 64;

// Storage-type traits: fp32 or bfloat16 in memory, fp32 in registers.
struct F32 {
    using storage = float;
    static __device__ __forceinline__ float load(const storage *p) { return *p; }
    static __device__ __forceinline__ void store(storage *p, float v) { *p = v; }
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }

// Round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
    u += 0x7fffu + ((u >> 16) & 1u);
    return uint16_t(u >> 16);
}

struct BF16 {
    using storage = uint16_t;
    static __device__ __forceinline__ float load(const storage *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(storage *p, float v) { *p = f32_to_bf16(v); }
};

// off mod D into [0, D) for any int32 off.
__device__ __forceinline__ int canonical_offset(int off, int D)
{
    int r = off % D;
    return r < 0 ? r + D : r;
}

}  // namespace dd
