// Token dispatch on one device: stable counting sort of the assignments
// a = t*K + s by local expert slot, then a coalesced row scatter.
//
//  1. permute_hist_kernel   per-block LDS histogram of local slots
//  2. permute_scan_kernel   counts, exclusive offsets, and the start position of
//                           every (block, slot) run (folded into step 3 when there are
//                           few blocks: each block sums the histograms it needs itself)
//  3. permute_rank_kernel   stable rank inside the block: each wave step ranks
//                           its 64 assignments with ballots (equal keys keep
//                           lane order), an LDS prefix over the block's wave
//                           steps orders the steps; writes perm / inv_perm
//  4. permute_rows_kernel   one wave per token: the row of x is read once and
//                           written to each of its (up to K) sorted positions
//                           with 16-byte accesses
// Everything is deterministic: no atomically assigned slots.
#include "c2r_internal.h"

namespace c2r {

constexpr int PB_THREADS = 256;
constexpr int PB_ITEMS = 4;                        // assignments per thread
constexpr int PB_SPAN = PB_THREADS * PB_ITEMS;     // assignments per block
constexpr int PB_STEPS = PB_SPAN / C2R_WAVE;       // wave steps per block (16)

__device__ __forceinline__ int slot_of(int e, int E, const int32_t *__restrict__ local_slot,
                                       int E_local) {
    if (e < 0 || e >= E) return -1;
    const int s = local_slot ? local_slot[e] : e;
    return (s >= 0 && s < E_local) ? s : -1;
}

__global__ __launch_bounds__(PB_THREADS) void permute_hist_kernel(
    const int32_t *__restrict__ topk_idx, int64_t A, int E, const int32_t *__restrict__ local_slot,
    int E_local, int32_t *__restrict__ block_counts) {
    __shared__ int32_t hist[C2R_MAX_E];
    if (threadIdx.x < C2R_MAX_E) hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * PB_SPAN;
#pragma unroll
    for (int i = 0; i < PB_ITEMS; ++i) {
        const int64_t a = base + i * PB_THREADS + threadIdx.x;
        if (a < A) {
            const int s = slot_of(topk_idx[a], E, local_slot, E_local);
            if (s >= 0) atomicAdd(&hist[s], 1);
        }
    }
    __syncthreads();
    if (threadIdx.x < E_local) block_counts[(size_t)blockIdx.x * E_local + threadIdx.x] = hist[threadIdx.x];
}

// One block of 64 threads; thread s walks the blocks for slot s.
__global__ __launch_bounds__(64) void permute_scan_kernel(const int32_t *__restrict__ block_counts,
                                                          int nblocks, int E_local,
                                                          int32_t *__restrict__ block_base,
                                                          int32_t *__restrict__ counts,
                                                          int32_t *__restrict__ offsets) {
    const int s = threadIdx.x;
    int32_t total = 0;
    if (s < E_local)
        for (int b = 0; b < nblocks; ++b) total += block_counts[(size_t)b * E_local + s];
    // exclusive scan over slots (64 lanes)
    int32_t incl = total;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int32_t v = __shfl_up(incl, off);
        if (s >= off) incl += v;
    }
    const int32_t excl = incl - total;
    if (s < E_local) {
        counts[s] = total;
        offsets[s] = excl;
        if (s == E_local - 1) offsets[E_local] = incl;
        int32_t run = excl;
        for (int b = 0; b < nblocks; ++b) {
            block_base[(size_t)b * E_local + s] = run;
            run += block_counts[(size_t)b * E_local + s];
        }
    }
}

// FUSED: there are few blocks, so every block derives the run starts itself from the block
// histograms (and block 0 also writes counts / offsets) instead of a separate scan launch.
template <bool FUSED>
__global__ __launch_bounds__(PB_THREADS) void permute_rank_kernel(
    const int32_t *__restrict__ topk_idx, int64_t A, int E, const int32_t *__restrict__ local_slot,
    int E_local, const int32_t *__restrict__ block_base, const int32_t *__restrict__ block_counts,
    int nblocks, int32_t *__restrict__ counts, int32_t *__restrict__ offsets,
    int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm) {
    __shared__ int32_t step_cnt[PB_STEPS][C2R_MAX_E];
    __shared__ int32_t part_tot[PB_THREADS / 64][C2R_MAX_E], part_pre[PB_THREADS / 64][C2R_MAX_E];
    __shared__ int32_t run_base[C2R_MAX_E];
    if (FUSED) {
        const int e = threadIdx.x & 63, part = threadIdx.x >> 6;
        int32_t tot = 0, pre = 0;
        if (e < E_local) {
            for (int b = part; b < nblocks; b += PB_THREADS / 64) {
                const int32_t v = block_counts[(size_t)b * E_local + e];
                tot += v;
                if (b < (int)blockIdx.x) pre += v;
            }
        }
        part_tot[part][e] = tot;
        part_pre[part][e] = pre;
        __syncthreads();
        if (threadIdx.x < 64) {
            int32_t total = 0, before = 0;
#pragma unroll
            for (int q = 0; q < PB_THREADS / 64; ++q) {
                total += part_tot[q][e];
                before += part_pre[q][e];
            }
            int32_t incl = total;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int32_t v = __shfl_up(incl, off);
                if (e >= off) incl += v;
            }
            run_base[e] = incl - total + before;
            if (blockIdx.x == 0 && e < E_local) {
                counts[e] = total;
                offsets[e] = incl - total;
                if (e == E_local - 1) offsets[E_local] = incl;
            }
        }
    }
    for (int i = threadIdx.x; i < PB_STEPS * C2R_MAX_E; i += PB_THREADS) (&step_cnt[0][0])[i] = 0;
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t base = (int64_t)blockIdx.x * PB_SPAN;
    const uint64_t lt = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    int slot[PB_ITEMS], rank[PB_ITEMS];
#pragma unroll
    for (int i = 0; i < PB_ITEMS; ++i) {
        const int64_t a = base + i * PB_THREADS + threadIdx.x;  // wave step q = i*4 + wave covers
        const int q = i * (PB_THREADS / 64) + wave;             // 64 consecutive assignments
        const int s = a < A ? slot_of(topk_idx[a], E, local_slot, E_local) : -1;
        int r = 0;
        uint64_t todo = __ballot(s >= 0);
        while (todo) {
            const int leader = __ffsll((unsigned long long)todo) - 1;
            const int sl = __shfl(s, leader);
            const uint64_t grp = __ballot(s == sl);
            if (s == sl) {
                r = __popcll(grp & lt);
                if (r == 0) step_cnt[q][sl] = __popcll(grp);
            }
            todo &= ~grp;
        }
        slot[i] = s;
        rank[i] = r;
    }
    __syncthreads();
    // exclusive prefix over the block's wave steps, per slot, seeded with the block's start
    if (threadIdx.x < E_local) {
        int32_t run = FUSED ? run_base[threadIdx.x] : block_base[(size_t)blockIdx.x * E_local + threadIdx.x];
#pragma unroll
        for (int q = 0; q < PB_STEPS; ++q) {
            const int32_t c = step_cnt[q][threadIdx.x];
            step_cnt[q][threadIdx.x] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PB_ITEMS; ++i) {
        const int64_t a = base + i * PB_THREADS + threadIdx.x;
        const int q = i * (PB_THREADS / 64) + wave;
        if (a < A) {
            if (slot[i] >= 0) {
                const int32_t p = step_cnt[q][slot[i]] + rank[i];
                perm[p] = (int32_t)a;
                inv_perm[a] = p;
            } else {
                inv_perm[a] = -1;
            }
        }
    }
}

// One wave per token; row bytes must be a multiple of 16.
__global__ __launch_bounds__(256) void permute_rows_kernel(const uint4 *__restrict__ x, int64_t T, int K,
                                                           int row_vecs,
                                                           const int32_t *__restrict__ inv_perm,
                                                           uint4 *__restrict__ x_perm) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    bool any = false;
    for (int s = 0; s < K; ++s) any |= inv_perm[t * K + s] >= 0;
    if (!any) return;
    const uint4 *src = x + t * row_vecs;
    for (int v0 = 0; v0 < row_vecs; v0 += 256) {
        uint4 r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = v0 + i * 64 + lane;
            if (v < row_vecs) r[i] = src[v];
        }
        for (int s = 0; s < K; ++s) {
            const int32_t p = inv_perm[t * K + s];
            if (p < 0) continue;
            uint4 *dst = x_perm + (int64_t)p * row_vecs;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int v = v0 + i * 64 + lane;
                if (v < row_vecs) dst[v] = r[i];
            }
        }
    }
}

size_t permute_workspace_bytes(int64_t T, int E, int K) {
    if (T <= 0 || K <= 0 || E <= 0) return 0;
    const int64_t A = T * K;
    const int64_t nblocks = (A + PB_SPAN - 1) / PB_SPAN;
    return 2 * round_up((size_t)nblocks * (size_t)(E < C2R_MAX_E ? E : C2R_MAX_E) * sizeof(int32_t), 256);
}

}  // namespace c2r

using namespace c2r;

extern "C" int c2r_permute(const void *x, c2r_dtype dt, const int32_t *topk_idx, int64_t T, int d,
                           int E, int K, const int32_t *local_slot, int E_local, int32_t *counts,
                           int32_t *offsets, int32_t *perm, int32_t *inv_perm, void *x_perm,
                           void *ws, size_t ws_bytes, void *stream) {
    if (T < 0 || E < 1 || K < 1 || E_local < 1 || E_local > E) return C2R_ERR_INVALID_ARG;
    if (!local_slot && E_local != E) return C2R_ERR_INVALID_ARG;
    if (dt != C2R_F32 && dt != C2R_BF16) return C2R_ERR_INVALID_ARG;
    if (E > C2R_MAX_E) return C2R_ERR_UNSUPPORTED;
    if (T * (int64_t)K >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    if (!counts || !offsets) return C2R_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t A = T * K;
    if ((A > 0) && (!topk_idx || !perm || !inv_perm)) return C2R_ERR_INVALID_ARG;
    if (x_perm && A > 0) {
        if (!x || d < 1) return C2R_ERR_INVALID_ARG;
        if (d % 8 != 0) return C2R_ERR_UNSUPPORTED;
        if (!aligned(x, 16) || !aligned(x_perm, 16)) return C2R_ERR_INVALID_ARG;
    }
    const int64_t nblocks = (A + PB_SPAN - 1) / PB_SPAN;
    const size_t half = round_up((size_t)nblocks * E_local * sizeof(int32_t), 256);
    if (nblocks > 0 && (!ws || ws_bytes < 2 * half || !aligned(ws, 256))) return C2R_ERR_WORKSPACE;
    int32_t *block_counts = static_cast<int32_t *>(ws);
    int32_t *block_base = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + half);
    if (nblocks > 0)
        permute_hist_kernel<<<dim3((unsigned)nblocks), dim3(PB_THREADS), 0, st>>>(
            topk_idx, A, E, local_slot, E_local, block_counts);
    const bool fused = nblocks > 0 && nblocks <= 256;  // each block re-reads nblocks*E_local counts
    if (!fused)
        permute_scan_kernel<<<dim3(1), dim3(64), 0, st>>>(block_counts, (int)nblocks, E_local, block_base,
                                                          counts, offsets);
    if (nblocks > 0) {
        if (fused)
            permute_rank_kernel<true><<<dim3((unsigned)nblocks), dim3(PB_THREADS), 0, st>>>(
                topk_idx, A, E, local_slot, E_local, block_base, block_counts, (int)nblocks, counts, offsets,
                perm, inv_perm);
        else
            permute_rank_kernel<false><<<dim3((unsigned)nblocks), dim3(PB_THREADS), 0, st>>>(
                topk_idx, A, E, local_slot, E_local, block_base, block_counts, (int)nblocks, counts, offsets,
                perm, inv_perm);
        if (x_perm) {
            const int row_vecs = d * (dt == C2R_BF16 ? 2 : 4) / 16;
            permute_rows_kernel<<<dim3((unsigned)((T + 3) / 4)), dim3(256), 0, st>>>(
                static_cast<const uint4 *>(x), T, K, row_vecs, inv_perm, static_cast<uint4 *>(x_perm));
        }
    }
    return launch_status();
}
