// Internal helpers shared by the HIP sources of the C2R library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/c2r.h"

#define C2R_WAVE 64
#define C2R_MAX_E 64
#define C2R_CANON_CHUNK 256

namespace c2r {

// An error that the caller's own earlier HIP work left behind in this thread must not be blamed
// on this library's launches: every entry point reads (and thereby clears) it before it
// launches anything, and launch_status() then reports only what its own launches raised.
static inline void drop_stale_error() { (void)hipGetLastError(); }

static inline int launch_status() {
    return hipGetLastError() == hipSuccess ? C2R_OK : C2R_ERR_LAUNCH;
}

static inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

static inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// bf16 <-> fp32 on raw bits. Storage is uint16_t; conversion to fp32 is exact.
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// fp32 -> bf16, round to nearest even, NaN stays NaN: the hardware conversion
// (v_cvt_pk_bf16_f32), one instruction for two values and no branch on NaN.
typedef __bf16 c2r_bf16x2 __attribute__((ext_vector_type(2)));
typedef float c2r_f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const c2r_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, c2r_bf16x2));
}

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.0f) & 0xffffu; }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (C2R_WAVE - 1); }

}  // namespace c2r
