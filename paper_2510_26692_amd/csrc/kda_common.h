// Shared device/host helpers for the KDA kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "kda.h"

namespace kda {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;      // CDNA wavefront width
constexpr int kChunk = 64;     // C of Section 3.1
constexpr float kLog2e = 1.4426950408889634f;

// bf16 bit pattern -> fp32 (exact).
__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16)
{
    return __uint_as_float(bits16 << 16);
}

// Two packed bf16 (little endian: element 0 in the low half) -> two floats.
__device__ __forceinline__ void unpack_bf16x2(uint32_t w, float &lo, float &hi)
{
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xffff0000u);
}

// Two floats -> two packed bf16, round to nearest even (element 0 in the low half).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Scalar element loads, widened to fp32, for the two supported input dtypes.
template <typename T> __device__ __forceinline__ float load_as_float(const T *p);
template <> __device__ __forceinline__ float load_as_float<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float load_as_float<__hip_bfloat16>(const __hip_bfloat16 *p)
{
    return bf16_bits_to_float(*reinterpret_cast<const uint16_t *>(p));
}

// 2^x through the hardware exponential (v_exp_f32).  Arguments here are always
// <= ~0 or bounded, so no range fix-up is wanted; denormal results flush to 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Error reporting shared by the entry points (defined in kda_api.hip).
kda_status fail(kda_status code, const char *fmt, ...);

}  // namespace kda
