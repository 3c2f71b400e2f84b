// Internal helpers shared by the HIP sources of the C2R library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/c2r.h"

#define C2R_WAVE 64
#define C2R_MAX_E 64
#define C2R_CANON_CHUNK 256

namespace c2r {

static inline int launch_status() {
    return hipPeekAtLastError() == hipSuccess ? C2R_OK : C2R_ERR_LAUNCH;
}

static inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

static inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// bf16 <-> fp32 on raw bits. Storage is uint16_t; conversion to fp32 is exact.
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (C2R_WAVE - 1); }

}  // namespace c2r
