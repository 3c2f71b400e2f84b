// Benchmark equipment, NOT part of the C2R library or its ABI: built into its own shared
// object (libc2r_benchaid.so) that only bench.py loads.
// Measured ceiling of the matrix pipe on this chip: a loop of independent
// v_mfma_f32_16x16x32_bf16 on register operands, nothing else.  The benchmark reports it
// next to the vendor peak (on random operands the chip is power limited well below it).
//   operands : 1024 x 16 bytes of bf16 in DEVICE memory (zeros reach the clock-limited peak,
//              random values are power limited)
//   iters    : loop trips; every wave issues 8 matrix instructions per trip
//   blocks   : workgroups of 512 threads (1..65536)
//   out      : float[blocks * 512] in DEVICE memory (sums, so the loop is not removed)
//   flops    : HOST pointer or NULL; receives the floating-point operations of the launch
//   clocks   : uint64[2] in DEVICE memory or NULL; receives, from one thread of the first
//              workgroup, the shader cycles and the ticks of the constant 100 MHz clock that
//              the loop took: cycles / (ticks / 1e8) is the clock the chip really ran at
// Returns 0, or -1 for a bad argument, -4 if the launch was refused.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace benchaid {

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_THREADS = 512, PROBE_ACC = 8;

__global__ __launch_bounds__(PROBE_THREADS) void probe_mfma_kernel(const probe_bf16x8 *__restrict__ operands,
                                                                  int iters, float *__restrict__ out,
                                                                  unsigned long long *__restrict__ clocks) {
    const probe_bf16x8 a = operands[threadIdx.x], b = operands[threadIdx.x + PROBE_THREADS];
    probe_f32x4 acc[PROBE_ACC];
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[i][v] = 0.0f;
    // one thread stamps the shader-cycle counter and the constant 100 MHz clock around the loop:
    // their ratio is the clock the loop really ran at (the chip lowers it at its power limit)
    const bool stamp = clocks && blockIdx.x == 0 && threadIdx.x == 0;
    unsigned long long c0 = 0, w0 = 0;
    if (stamp) {
        c0 = clock64();
        w0 = wall_clock64();
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_ACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
    }
    if (stamp) {
        clocks[0] = clock64() - c0;
        clocks[1] = wall_clock64() - w0;
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) s += acc[i][v];
    out[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

}  // namespace benchaid

using namespace benchaid;

extern "C" int benchaid_probe_mfma_bf16(const void *operands, int iters, int blocks, float *out, double *flops,
                                   uint64_t *clocks, void *stream) {
    if (!operands || !out || iters < 1 || blocks < 1 || blocks > 65536) return -1;
    if (reinterpret_cast<uintptr_t>(operands) % 16 || reinterpret_cast<uintptr_t>(clocks) % 8) return -1;
    probe_mfma_kernel<<<dim3((unsigned)blocks), dim3(PROBE_THREADS), 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const probe_bf16x8 *>(operands), iters, out, reinterpret_cast<unsigned long long *>(clocks));
    if (flops) *flops = (double)blocks * (PROBE_THREADS / 64) * (double)iters * PROBE_ACC * (2.0 * 16 * 16 * 32);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
