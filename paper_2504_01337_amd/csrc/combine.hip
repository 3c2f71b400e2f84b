// Un-permute and gate-weighted sum (last sentence of Sec. 3.1): every thread owns
// one 16-byte vector of an output row, gathers the matching vector of each of the
// token's K expert rows, accumulates in fp32 in slot order and rounds once.
#include "c2r_internal.h"

namespace c2r {

template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4 *__restrict__ y_perm,
                                                      const float *__restrict__ gates,
                                                      const int32_t *__restrict__ inv_perm, int64_t T,
                                                      int row_vecs, int K,
                                                      const uint4 *__restrict__ y_shared,
                                                      uint4 *__restrict__ y) {
    constexpr int N = BF16 ? 8 : 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= T * row_vecs) return;
    const int64_t t = i / row_vecs;
    const int v = (int)(i - t * row_vecs);
    float acc[N];
#pragma unroll
    for (int j = 0; j < N; ++j) acc[j] = 0.0f;
    auto add = [&](const uint4 q, float g) {
        if constexpr (BF16) {
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[2 * j] = __builtin_fmaf(g, __uint_as_float(w[j] << 16), acc[2 * j]);
                acc[2 * j + 1] = __builtin_fmaf(g, __uint_as_float(w[j] & 0xffff0000u), acc[2 * j + 1]);
            }
        } else {
            acc[0] = __builtin_fmaf(g, __uint_as_float(q.x), acc[0]);
            acc[1] = __builtin_fmaf(g, __uint_as_float(q.y), acc[1]);
            acc[2] = __builtin_fmaf(g, __uint_as_float(q.z), acc[2]);
            acc[3] = __builtin_fmaf(g, __uint_as_float(q.w), acc[3]);
        }
    };
    for (int s = 0; s < K; ++s) {
        const int32_t p = inv_perm[t * K + s];
        if (p < 0) continue;
        add(y_perm[(int64_t)p * row_vecs + v], gates[t * K + s]);
    }
    if (y_shared) add(y_shared[i], 1.0f);
    uint4 out;
    if constexpr (BF16) {
        out.x = pack_bf16x2(acc[0], acc[1]);
        out.y = pack_bf16x2(acc[2], acc[3]);
        out.z = pack_bf16x2(acc[4], acc[5]);
        out.w = pack_bf16x2(acc[6], acc[7]);
    } else {
        out.x = __float_as_uint(acc[0]);
        out.y = __float_as_uint(acc[1]);
        out.z = __float_as_uint(acc[2]);
        out.w = __float_as_uint(acc[3]);
    }
    y[i] = out;
}

}  // namespace c2r

using namespace c2r;

extern "C" int c2r_combine(const void *y_perm, c2r_dtype dt, const float *gates,
                           const int32_t *inv_perm, int64_t T, int d, int K, const void *y_shared,
                           void *y, void *stream) {
    drop_stale_error();
    if (T < 0 || d < 1 || K < 1) return C2R_ERR_INVALID_ARG;
    if (dt != C2R_F32 && dt != C2R_BF16) return C2R_ERR_INVALID_ARG;
    if (T == 0) return C2R_OK;
    if (!y_perm || !gates || !inv_perm || !y) return C2R_ERR_INVALID_ARG;
    if (d % 8 != 0) return C2R_ERR_UNSUPPORTED;
    if (!aligned(y_perm, 16) || !aligned(y, 16) || (y_shared && !aligned(y_shared, 16)))
        return C2R_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int row_vecs = d * (dt == C2R_BF16 ? 2 : 4) / 16;
    const int64_t n = T * row_vecs;
    const int64_t nblk = (n + 255) / 256;
    if (nblk >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    if (dt == C2R_BF16)
        combine_kernel<true><<<dim3((unsigned)nblk), dim3(256), 0, st>>>(
            static_cast<const uint4 *>(y_perm), gates, inv_perm, T, row_vecs, K,
            static_cast<const uint4 *>(y_shared), static_cast<uint4 *>(y));
    else
        combine_kernel<false><<<dim3((unsigned)nblk), dim3(256), 0, st>>>(
            static_cast<const uint4 *>(y_perm), gates, inv_perm, T, row_vecs, K,
            static_cast<const uint4 *>(y_shared), static_cast<uint4 *>(y));
    return launch_status();
}
