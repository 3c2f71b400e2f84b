// Expert collaboration matrix (Eq. 2) and collaborator lists (Eq. 4).
//
// Co-activation is a histogram over expert pairs kept in LDS: a thread takes a token, forms
// the 64-bit set of its experts (duplicates and out-of-range entries drop out) and adds 1 to
// red[a][b] for every pair a <= b of the set, the diagonal included - K (K + 1) / 2 LDS
// atomics per token, 10 for K = 4.  Only the upper triangle is counted (the matrix is
// symmetric); the workgroup's histogram then goes to C with one integer atomic per entry,
// C[i][j] += red[min(i,j)][max(i,j)].  Integer adds commute, so the result is exact and
// reproducible.  LDS atomics of lanes that hit the same pair serialise, one per cycle: with
// every token on one pair that is 64 cycles per instruction, still a fraction of what a
// conflict-free formulation through ballots and popcounts costs (it was measured: 64 ballots
// to transpose the wave's bit matrix and 64 x (2 readlane + 2 popcount) per 64 tokens are
// ~700 instructions of 4 cycles each, 38 us for 2^20 tokens, where this is ~150 and 10).
#include "c2r_internal.h"

namespace c2r {

template <int NW>
__global__ __launch_bounds__(NW * 64) void coactivation_kernel(const int32_t *__restrict__ topk_idx,
                                                              int64_t T, int K, int E,
                                                              int32_t *__restrict__ C) {
    __shared__ int32_t red[C2R_MAX_E * C2R_MAX_E];  // red[a * 64 + b], a <= b
    for (int i = threadIdx.x; i < C2R_MAX_E * C2R_MAX_E; i += NW * 64) red[i] = 0;
    __syncthreads();

    constexpr int UN = 4;  // tokens per thread and trip: their index loads are in flight together
    const int64_t stride = (int64_t)gridDim.x * NW * 64;
    for (int64_t t0 = (int64_t)blockIdx.x * NW * 64 + threadIdx.x; t0 < T; t0 += UN * stride) {
        uint64_t m[UN];
        if (K == 4) {
            int4 q[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int64_t t = t0 + u * stride;
                q[u] = *reinterpret_cast<const int4 *>(topk_idx + (t < T ? t : t0) * 4);
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int v[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
                m[u] = 0;
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    if (v[s] >= 0 && v[s] < E) m[u] |= 1ull << v[s];
                if (t0 + u * stride >= T) m[u] = 0;
            }
        } else {
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int64_t t = t0 + u * stride;
                m[u] = 0;
                if (t < T)
                    for (int s = 0; s < K; ++s) {
                        const int v = topk_idx[t * K + s];
                        if (v >= 0 && v < E) m[u] |= 1ull << v;
                    }
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            uint64_t ma = m[u];
            while (ma) {  // a: the set's experts in ascending order
                const int a = __ffsll((unsigned long long)ma) - 1;
                uint64_t mb = ma;  // b >= a: a itself (the diagonal) and the higher ones
                ma &= ma - 1;
                while (mb) {
                    const int b = __ffsll((unsigned long long)mb) - 1;
                    mb &= mb - 1;
                    atomicAdd(&red[a * C2R_MAX_E + b], 1);
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < E * E; i += NW * 64) {
        const int r = i / E, c = i - r * E;
        const int32_t v = red[(r < c ? r : c) * C2R_MAX_E + (r < c ? c : r)];
        if (v) atomicAdd(&C[i], v);
    }
}

// One wave per expert row: rank of (count desc, index asc) by comparing against
// every other entry of the row, broadcast lane by lane.
__global__ __launch_bounds__(64) void collaborators_kernel(const int32_t *__restrict__ C, int E, int n,
                                                           int32_t *__restrict__ collab_idx,
                                                           uint64_t *__restrict__ collab_mask) {
    const int i = blockIdx.x, j = threadIdx.x;
    const bool valid = j < E && j != i;
    const int32_t c = valid ? C[(size_t)i * E + j] : 0;
    int rank = 0;
    for (int q = 0; q < E; ++q) {
        const int32_t cq = __shfl(c, q);
        if (q != i && (cq > c || (cq == c && q < j))) ++rank;
    }
    const bool in_list = valid && rank < n;
    if (in_list && collab_idx) collab_idx[(size_t)i * n + rank] = j;
    const uint64_t bal = __ballot(in_list);
    if (collab_mask && j == 0) collab_mask[i] = bal;
}

// Greedy co-location of collaborating experts (Sec. 3.4), one wave, lane = expert.  Devices
// are filled in order with ceil(E / n_dev) experts each: a device starts with the unplaced
// expert whose row of C (diagonal left out) sums highest and then keeps taking the unplaced
// expert with the largest total co-activation with its members; ties go to the lower index.
// C sits in LDS; each step adds the new member's column entry to a running sum per lane and takes
// a wave-wide arg max.
__global__ __launch_bounds__(64) void place_experts_kernel(const int32_t *__restrict__ C, int E, int n_dev,
                                                           int32_t *__restrict__ expert_device) {
    __shared__ int32_t Cl[C2R_MAX_E][C2R_MAX_E + 1];
    const int e = threadIdx.x;
    for (int i = e; i < E * E; i += 64) Cl[i / E][i % E] = C[i];
    __syncthreads();
    const int cap = (E + n_dev - 1) / n_dev;
    uint64_t placed = 0;  // wave-uniform
    int mine = -1;
    long long row_sum = 0;  // this expert's row of C without the diagonal: its score for an empty device
    if (e < E)
        for (int j = 0; j < E; ++j)
            if (j != e) row_sum += Cl[e][j];
    for (int g = 0; g < n_dev; ++g) {
        uint64_t members = 0;
        long long with_members = 0;  // co-activation with the device's members, kept up as they join
        for (int m = 0; m < cap; ++m) {
            const bool free_lane = e < E && !((placed >> e) & 1ull);
            const long long score = members == 0 ? row_sum : with_members;
            // arg max over the free lanes, lower index on ties: the largest score first ...
            long long best = free_lane ? score : -1;  // scores are sums of counts, never negative
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const long long o = __shfl_xor(best, off);
                best = o > best ? o : best;
            }
            const uint64_t cand = __ballot(free_lane && score == best);
            if (cand == 0) break;  // everything is placed
            const int pick = __ffsll((unsigned long long)cand) - 1;
            if (e == pick) mine = g;
            placed |= 1ull << pick;
            members |= 1ull << pick;
            if (e < E && e != pick) with_members += Cl[e][pick];
        }
    }
    if (e < E) expert_device[e] = mine;
}

}  // namespace c2r

using namespace c2r;

extern "C" int c2r_place_experts(const int32_t *C, int E, int n_dev, int32_t *expert_device, void *stream) {
    drop_stale_error();
    if (E < 1 || n_dev < 1) return C2R_ERR_INVALID_ARG;
    if (E > C2R_MAX_E || n_dev > C2R_MAX_E) return C2R_ERR_UNSUPPORTED;
    if (!C || !expert_device) return C2R_ERR_INVALID_ARG;
    place_experts_kernel<<<dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream)>>>(C, E, n_dev, expert_device);
    return launch_status();
}

extern "C" int c2r_build_coactivation(const int32_t *topk_idx, int64_t T, int K, int E, int32_t *C,
                                      void *stream) {
    drop_stale_error();
    if (T < 0 || K < 1 || E < 1) return C2R_ERR_INVALID_ARG;
    if (E > C2R_MAX_E) return C2R_ERR_UNSUPPORTED;
    if (T == 0) return C2R_OK;
    if (!topk_idx || !C) return C2R_ERR_INVALID_ARG;
    if (!aligned(topk_idx, 16) || !aligned(C, 4)) return C2R_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t nbatch = (T + 63) / 64;
    // Every workgroup ends with one integer atomic per entry of C, all workgroups on the same
    // E*E addresses, so a long stream runs as few, large workgroups (16 waves, four tokens per
    // thread and trip), a short one as 4-wave workgroups that still spread over the chip.
    const bool big = T >= (1 << 18);
    const int nw = big ? 16 : 4;
    int64_t nblk = (T + nw * 64 * 4 - 1) / (nw * 64 * 4);
    const int64_t cap = 256;  // one workgroup per CU (measured on 2^20 tokens: 128 -> 16.4 us, 256 -> 15.4, 512 -> 15.2)
    if (nblk > cap) nblk = cap;
    const dim3 grid((unsigned)nblk), block(nw * 64);
    if (big)
        coactivation_kernel<16><<<grid, block, 0, st>>>(topk_idx, T, K, E, C);
    else
        coactivation_kernel<4><<<grid, block, 0, st>>>(topk_idx, T, K, E, C);
    return launch_status();
}

extern "C" int c2r_collaborators(const int32_t *C, int E, int Tc, int32_t *collab_idx,
                                 uint64_t *collab_mask, void *stream) {
    drop_stale_error();
    if (E < 1 || Tc < 0) return C2R_ERR_INVALID_ARG;
    if (E > C2R_MAX_E) return C2R_ERR_UNSUPPORTED;
    if (!C || (!collab_idx && !collab_mask)) return C2R_ERR_INVALID_ARG;
    const int n = Tc < E - 1 ? Tc : E - 1;
    if (n == 0 && !collab_mask) return C2R_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    collaborators_kernel<<<dim3(E), dim3(64), 0, st>>>(C, E, n, collab_idx, collab_mask);
    return launch_status();
}
