// Expert collaboration matrix (Eq. 2) and collaborator lists (Eq. 4).
//
// Co-activation without a single contended atomic in the token loop: a wave
// takes 64 tokens, each lane builds the 64-bit set of its token's experts, and
// E wave ballots transpose that 64x64 bit matrix so that lane i holds
// B_i = {tokens of this batch that selected expert i}.  Then
//     C[i, j] += popcount(B_i & B_j)
// with B_j broadcast from lane j; lane i keeps row i of the wave's partial
// matrix in registers across all its batches.  The cost per batch does not
// depend on how skewed the expert load is.  Partial matrices are reduced through
// LDS per workgroup and added to C with one integer atomic per entry per
// workgroup (integer adds commute, so the result is exact and reproducible).
#include "c2r_internal.h"

namespace c2r {

template <int EP>
__global__ __launch_bounds__(256) void coactivation_kernel(const int32_t *__restrict__ topk_idx,
                                                           int64_t T, int K, int E,
                                                           int32_t *__restrict__ C) {
    __shared__ int32_t red[EP * EP];
    for (int i = threadIdx.x; i < EP * EP; i += 256) red[i] = 0;
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int64_t nbatch = (T + 63) / 64;

    int32_t acc[EP];
#pragma unroll
    for (int j = 0; j < EP; ++j) acc[j] = 0;

    for (int64_t b = wave; b < nbatch; b += nwaves) {
        const int64_t t = b * 64 + lane;
        uint64_t m = 0;
        if (t < T) {
            if (K == 4) {
                const int4 q = *reinterpret_cast<const int4 *>(topk_idx + t * 4);
                const int v[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    if (v[s] >= 0 && v[s] < E) m |= 1ull << v[s];
            } else {
                for (int s = 0; s < K; ++s) {
                    const int v = topk_idx[t * K + s];
                    if (v >= 0 && v < E) m |= 1ull << v;
                }
            }
        }
        const uint32_t mlo = (uint32_t)m, mhi = (uint32_t)(m >> 32);
        // bit-matrix transpose through ballots: lane i <- B_i
        uint32_t blo = 0, bhi = 0;
#pragma unroll
        for (int i = 0; i < EP; ++i) {
            const bool bit = (((i < 32) ? (mlo >> (i & 31)) : (mhi >> (i & 31))) & 1u) != 0;
            const uint64_t bal = __ballot(bit);
            blo = lane == i ? (uint32_t)bal : blo;
            bhi = lane == i ? (uint32_t)(bal >> 32) : bhi;
        }
#pragma unroll
        for (int j = 0; j < EP; ++j) {
            const uint32_t jlo = __builtin_amdgcn_readlane(blo, j);
            const uint32_t jhi = __builtin_amdgcn_readlane(bhi, j);
            acc[j] += __popc(blo & jlo) + __popc(bhi & jhi);
        }
    }

    if (lane < EP) {
#pragma unroll
        for (int j = 0; j < EP; ++j)
            if (acc[j]) atomicAdd(&red[lane * EP + j], acc[j]);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < EP * EP; i += 256) {
        const int r = i / EP, c = i % EP;
        const int32_t v = red[i];
        if (v && r < E && c < E) atomicAdd(&C[(size_t)r * E + c], v);
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
    int64_t nblk = (nbatch + 3) / 4;
    if (nblk > 1024) nblk = 1024;  // ~4 workgroups per CU; each wave loops over its batches
    const dim3 grid((unsigned)nblk), block(256);
    if (E <= 8)
        coactivation_kernel<8><<<grid, block, 0, st>>>(topk_idx, T, K, E, C);
    else if (E <= 16)
        coactivation_kernel<16><<<grid, block, 0, st>>>(topk_idx, T, K, E, C);
    else if (E <= 32)
        coactivation_kernel<32><<<grid, block, 0, st>>>(topk_idx, T, K, E, C);
    else
        coactivation_kernel<64><<<grid, block, 0, st>>>(topk_idx, T, K, E, C);
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
