// Routing statistics of Sec. 3.2 and Sec. 4.1, computed where the indices and the
// co-activation matrix already are (device memory):
//
//  collaboration_degree_kernel  Eq. 3: the entropy of each expert's co-activation
//                               frequencies with the other experts (fp64)
//  distinct_devices_kernel      per token, the number of distinct devices that host its
//                               selected experts, for up to MAX_MAPS expert -> device maps in
//                               one pass over the indices; the totals give the token
//                               redundancy 1 - total / (T*K) of Sec. 4.1 for every
//                               expert-parallel degree at once
#include "c2r_internal.h"

namespace c2r {

constexpr int MAX_MAPS = 8;

// One wave per expert i, lane j holds C[i][j].  The diagonal takes part neither in the
// normalisation nor in the sum; terms with a zero count are zero.  Natural logarithm.
__global__ __launch_bounds__(64) void collaboration_degree_kernel(const int32_t *__restrict__ C, int E,
                                                                  double *__restrict__ P) {
    const int i = blockIdx.x, j = threadIdx.x;
    int64_t c = 0;
    if (j < E && j != i) {
        c = C[(size_t)i * E + j];
        if (c < 0) c = 0;
    }
    int64_t s = c;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    double term = 0.0;
    if (c > 0) {
        const double p = (double)c / (double)s;
        term = -p * log(p);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) term += __shfl_xor(term, off);
    if (j == 0) P[i] = term;
}

__global__ __launch_bounds__(64) void zero_totals_kernel(unsigned long long *__restrict__ totals, int n) {
    if ((int)threadIdx.x < n) totals[threadIdx.x] = 0ull;
}

// One thread per token.  The maps sit in LDS; a token's devices under map m are the bits of
// one 64-bit word.  The per-wave sums go to the totals with one integer atomic per map, so
// the result does not depend on the order of the waves.
__global__ __launch_bounds__(256) void distinct_devices_kernel(
    const int32_t *__restrict__ topk_idx, int64_t T, int K, int E, const int32_t *__restrict__ maps,
    int n_maps, int n_dev, int32_t *__restrict__ per_token, unsigned long long *__restrict__ totals) {
    __shared__ int32_t dev_of[MAX_MAPS][C2R_MAX_E];
    for (int q = threadIdx.x; q < n_maps * E; q += blockDim.x) {
        const int v = maps[q];
        dev_of[q / E][q % E] = (v >= 0 && v < n_dev) ? v : -1;
    }
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t seen[MAX_MAPS];
#pragma unroll
    for (int m = 0; m < MAX_MAPS; ++m) seen[m] = 0;
    if (t < T) {
        for (int s = 0; s < K; ++s) {
            const int e = topk_idx[t * K + s];
            if (e < 0 || e >= E) continue;
#pragma unroll
            for (int m = 0; m < MAX_MAPS; ++m) {
                if (m < n_maps) {
                    const int g = dev_of[m][e];
                    if (g >= 0) seen[m] |= 1ull << g;
                }
            }
        }
    }
#pragma unroll
    for (int m = 0; m < MAX_MAPS; ++m) {
        if (m < n_maps) {  // uniform over the grid
            int n = __popcll((unsigned long long)seen[m]);
            if (per_token && t < T) per_token[(size_t)m * T + t] = n;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) n += __shfl_xor(n, off);
            if (lane_id() == 0 && n > 0) atomicAdd(&totals[m], (unsigned long long)n);
        }
    }
}

}  // namespace c2r

using namespace c2r;

extern "C" int c2r_collaboration_degree(const int32_t *C, int E, double *P, void *stream) {
    drop_stale_error();
    if (E < 1) return C2R_ERR_INVALID_ARG;
    if (E > C2R_MAX_E) return C2R_ERR_UNSUPPORTED;
    if (!C || !P) return C2R_ERR_INVALID_ARG;
    collaboration_degree_kernel<<<dim3(E), dim3(64), 0, static_cast<hipStream_t>(stream)>>>(C, E, P);
    return launch_status();
}

extern "C" int c2r_distinct_devices(const int32_t *topk_idx, int64_t T, int K, int E,
                                    const int32_t *expert_device, int n_maps, int n_dev,
                                    int32_t *per_token, int64_t *totals, void *stream) {
    drop_stale_error();
    if (T < 0 || K < 1 || E < 1 || n_maps < 1 || n_dev < 1) return C2R_ERR_INVALID_ARG;
    if (E > C2R_MAX_E || n_dev > C2R_MAX_E || n_maps > MAX_MAPS) return C2R_ERR_UNSUPPORTED;
    if (!totals || !expert_device || (T > 0 && !topk_idx)) return C2R_ERR_INVALID_ARG;
    if (!aligned(totals, 8)) return C2R_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned long long *tot = reinterpret_cast<unsigned long long *>(totals);
    zero_totals_kernel<<<dim3(1), dim3(64), 0, st>>>(tot, n_maps);
    if (T > 0) {
        const int64_t nblk = (T + 255) / 256;
        if (nblk >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
        distinct_devices_kernel<<<dim3((unsigned)nblk), dim3(256), 0, st>>>(topk_idx, T, K, E, expert_device,
                                                                           n_maps, n_dev, per_token, tot);
    }
    return launch_status();
}
