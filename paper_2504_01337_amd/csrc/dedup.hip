// Zero-redundancy dispatch (Sec. 3.4): a token is sent ONCE to every device that hosts at
// least one of its selected experts and replicated there.  On one GPU this builds the
// index of that exchange and runs the two-level combine that goes with it:
//
//   dedup_count_kernel / dedup_rank_kernel : the list of (device, token) copies, ordered by
//       device then token (a stable counting sort of per-token device SETS: a wave ranks
//       its 64 tokens for device g with one ballot of "token has an expert on g"), and for
//       every assignment the row of the copy it uses;
//   combine_partial_kernel : what each expert device returns - one row per copy, the
//       gate-weighted fp32 sum of the outputs of ITS experts for that token, rounded once;
//   combine_copies_kernel  : what the token's home device does - add the partial rows of the
//       token's copies (+ the shared expert) in fp32, round once.
#include "c2r_internal.h"

namespace c2r {

constexpr int DB_THREADS = 256;
constexpr int DB_ITEMS = 4;                     // tokens per thread
constexpr int DB_SPAN = DB_THREADS * DB_ITEMS;  // tokens per block
constexpr int DB_STEPS = DB_SPAN / C2R_WAVE;    // wave steps per block

__device__ __forceinline__ int device_of(int e, int E, const int32_t *__restrict__ expert_device, int n_dev) {
    if (e < 0 || e >= E) return -1;
    const int g = expert_device[e];
    return (g >= 0 && g < n_dev) ? g : -1;
}

// The expert -> device map of the call, checked once per workgroup into LDS (-1: no device).
__device__ __forceinline__ void load_device_table(int32_t *tab, int E, const int32_t *__restrict__ expert_device,
                                                  int n_dev) {
    if (threadIdx.x < C2R_MAX_E) {
        const int e = threadIdx.x;
        tab[e] = e < E ? device_of(e, E, expert_device, n_dev) : -1;
    }
    __syncthreads();
}

// Devices of a token's K experts.  The K indices are loaded together (independent loads); for
// K <= 8 the devices are also returned packed, one byte per slot (device + 1, 0: none), so that
// the caller need not load the indices again.
__device__ __forceinline__ uint64_t device_set(const int32_t *__restrict__ topk_idx, int64_t t, int64_t T, int K,
                                               int E, const int32_t *tab, uint64_t *packed = nullptr) {
    uint64_t m = 0, pk = 0;
    if (t < T) {
        if (K <= 8) {
            int32_t e[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) e[s] = topk_idx[t * K + (s < K ? s : K - 1)];  // (no load behind a branch)
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int g = (s < K && e[s] >= 0 && e[s] < E) ? tab[e[s]] : -1;
                if (g >= 0) {
                    m |= 1ull << g;
                    pk |= (uint64_t)(g + 1) << (8 * s);
                }
            }
        } else {
            for (int s = 0; s < K; ++s) {
                const int32_t e = topk_idx[t * K + s];
                const int g = (e >= 0 && e < E) ? tab[e] : -1;
                if (g >= 0) m |= 1ull << g;
            }
        }
    }
    if (packed) *packed = pk;
    return m;
}

__global__ __launch_bounds__(DB_THREADS) void dedup_count_kernel(
    const int32_t *__restrict__ topk_idx, int64_t T, int K, int E, const int32_t *__restrict__ expert_device,
    int n_dev, int32_t *__restrict__ block_counts) {
    __shared__ int32_t hist[C2R_MAX_E], dev_tab[C2R_MAX_E];
    if (threadIdx.x < C2R_MAX_E) hist[threadIdx.x] = 0;
    load_device_table(dev_tab, E, expert_device, n_dev);
    const int lane = threadIdx.x & 63;
    const int64_t base = (int64_t)blockIdx.x * DB_SPAN;
    uint64_t sets[DB_ITEMS];
#pragma unroll
    for (int i = 0; i < DB_ITEMS; ++i)
        sets[i] = device_set(topk_idx, base + i * DB_THREADS + threadIdx.x, T, K, E, dev_tab);
#pragma unroll
    for (int i = 0; i < DB_ITEMS; ++i) {
        const uint64_t m = sets[i];
        for (int g = 0; g < n_dev; ++g) {
            const int c = __popcll(__ballot((m >> g) & 1ull));
            if (lane == 0 && c) atomicAdd(&hist[g], c);
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < n_dev) block_counts[(size_t)blockIdx.x * n_dev + threadIdx.x] = hist[threadIdx.x];
}

// Every block derives the start of its (block, device) runs itself from the block
// histograms; block 0 also writes the counts and offsets.
__global__ __launch_bounds__(DB_THREADS) void dedup_rank_kernel(
    const int32_t *__restrict__ topk_idx, int64_t T, int K, int E, const int32_t *__restrict__ expert_device,
    int n_dev, const int32_t *__restrict__ block_counts, int nblocks, int32_t *__restrict__ send_counts,
    int32_t *__restrict__ send_offsets, int32_t *__restrict__ send_token, int32_t *__restrict__ send_row) {
    __shared__ int32_t step_cnt[DB_STEPS][C2R_MAX_E];
    __shared__ int32_t part_tot[DB_THREADS / 64][C2R_MAX_E], part_pre[DB_THREADS / 64][C2R_MAX_E];
    __shared__ int32_t run_base[C2R_MAX_E], dev_tab[C2R_MAX_E];
    load_device_table(dev_tab, E, expert_device, n_dev);
    {
        const int g = threadIdx.x & 63, part = threadIdx.x >> 6;
        int32_t tot = 0, pre = 0;
        if (g < n_dev)
#pragma unroll 8
            for (int b = part; b < nblocks; b += DB_THREADS / 64) {
                const int32_t v = block_counts[(size_t)b * n_dev + g];
                tot += v;
                if (b < (int)blockIdx.x) pre += v;
            }
        part_tot[part][g] = tot;
        part_pre[part][g] = pre;
        __syncthreads();
        if (threadIdx.x < 64) {
            int32_t total = 0, before = 0;
#pragma unroll
            for (int q = 0; q < DB_THREADS / 64; ++q) {
                total += part_tot[q][g];
                before += part_pre[q][g];
            }
            int32_t incl = total;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int32_t v = __shfl_up(incl, off);
                if (g >= off) incl += v;
            }
            run_base[g] = incl - total + before;
            if (blockIdx.x == 0 && g < n_dev) {
                send_counts[g] = total;
                send_offsets[g] = incl - total;
                if (g == n_dev - 1) send_offsets[n_dev] = incl;
            }
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t base = (int64_t)blockIdx.x * DB_SPAN;
    const uint64_t lt = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    uint64_t sets[DB_ITEMS], packed[DB_ITEMS];
#pragma unroll
    for (int i = 0; i < DB_ITEMS; ++i)
        sets[i] = device_set(topk_idx, base + i * DB_THREADS + threadIdx.x, T, K, E, dev_tab, &packed[i]);
#pragma unroll
    for (int i = 0; i < DB_ITEMS; ++i) {
        const int q = i * (DB_THREADS / 64) + wave;  // wave step q covers 64 consecutive tokens
        for (int g = 0; g < n_dev; ++g) {
            const int c = __popcll(__ballot((sets[i] >> g) & 1ull));
            if (lane == 0) step_cnt[q][g] = c;
        }
    }
    __syncthreads();
    // exclusive prefix over the block's wave steps, per device, seeded with the block's start
    if ((int)threadIdx.x < n_dev) {
        int32_t run = run_base[threadIdx.x];
#pragma unroll
        for (int q = 0; q < DB_STEPS; ++q) {
            const int32_t c = step_cnt[q][threadIdx.x];
            step_cnt[q][threadIdx.x] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < DB_ITEMS; ++i) {
        const int64_t t = base + i * DB_THREADS + threadIdx.x;
        const int q = i * (DB_THREADS / 64) + wave;
        for (int g = 0; g < n_dev; ++g) {
            const bool mine = (sets[i] >> g) & 1ull;
            const uint64_t bal = __ballot(mine);
            if (mine) {
                const int32_t pos = step_cnt[q][g] + __popcll(bal & lt);
                send_token[pos] = (int32_t)t;
                if (K <= 8) {
#pragma unroll
                    for (int s = 0; s < 8; ++s)
                        if (s < K && (int)((packed[i] >> (8 * s)) & 0xff) == g + 1) send_row[t * K + s] = pos;
                } else {
                    for (int s = 0; s < K; ++s) {
                        const int32_t e = topk_idx[t * K + s];
                        if (e >= 0 && e < E && dev_tab[e] == g) send_row[t * K + s] = pos;
                    }
                }
            }
        }
        if (t < T) {
            if (K <= 8) {
#pragma unroll
                for (int s = 0; s < 8; ++s)
                    if (s < K && ((packed[i] >> (8 * s)) & 0xff) == 0) send_row[t * K + s] = -1;
            } else {
                for (int s = 0; s < K; ++s) {
                    const int32_t e = topk_idx[t * K + s];
                    if (!(e >= 0 && e < E && dev_tab[e] >= 0)) send_row[t * K + s] = -1;
                }
            }
        }
    }
}

template <bool BF16>
struct VecAcc {
    static constexpr int N = BF16 ? 8 : 4;
    float acc[N];
    __device__ __forceinline__ VecAcc() {
#pragma unroll
        for (int j = 0; j < N; ++j) acc[j] = 0.0f;
    }
    __device__ __forceinline__ void add(const uint4 q, float g) {
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
    }
    __device__ __forceinline__ uint4 rounded() const {
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
        return out;
    }
};

// One thread per 16-byte vector of a copy's partial row.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_partial_kernel(
    const uint4 *__restrict__ y_perm, const float *__restrict__ gates, const int32_t *__restrict__ inv_perm,
    const int32_t *__restrict__ send_token, const int32_t *__restrict__ send_row,
    const int32_t *__restrict__ n_send_ptr, int64_t T, int64_t cap_rows, int row_vecs, int K,
    uint4 *__restrict__ y_part) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t n_send = *n_send_ptr;
    n_send = n_send < 0 ? 0 : (n_send > cap_rows ? cap_rows : n_send);
    if (i >= n_send * row_vecs) return;
    const int64_t r = i / row_vecs;
    const int v = (int)(i - r * row_vecs);
    const int64_t t = send_token[r];
    VecAcc<BF16> a;
    if (t >= 0 && t < T)
        for (int s = 0; s < K; ++s) {
            const int32_t p = inv_perm[t * K + s];
            if (send_row[t * K + s] != (int32_t)r || p < 0) continue;
            a.add(y_perm[(int64_t)p * row_vecs + v], gates[t * K + s]);
        }
    y_part[i] = a.rounded();
}

// One thread per 16-byte vector of an output row: the token's copies in order of first use.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_copies_kernel(
    const uint4 *__restrict__ y_part, const int32_t *__restrict__ send_row, int64_t T, int64_t cap_rows,
    int row_vecs, int K, const uint4 *__restrict__ y_shared, uint4 *__restrict__ y) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= T * row_vecs) return;
    const int64_t t = i / row_vecs;
    const int v = (int)(i - t * row_vecs);
    VecAcc<BF16> a;
    for (int s = 0; s < K; ++s) {
        const int32_t r = send_row[t * K + s];
        bool seen = r < 0 || r >= cap_rows;
        for (int b = 0; b < s && !seen; ++b) seen = send_row[t * K + b] == r;
        if (!seen) a.add(y_part[(int64_t)r * row_vecs + v], 1.0f);
    }
    if (y_shared) a.add(y_shared[i], 1.0f);
    y[i] = a.rounded();
}

size_t dedup_workspace_bytes(int64_t T, int n_dev) {
    if (T <= 0 || n_dev <= 0) return 0;
    const int64_t nblocks = (T + DB_SPAN - 1) / DB_SPAN;
    return round_up((size_t)nblocks * n_dev * sizeof(int32_t), 256);
}

}  // namespace c2r

using namespace c2r;

extern "C" int c2r_dedup_dispatch(const int32_t *topk_idx, int64_t T, int K, int E, const int32_t *expert_device,
                                  int n_dev, int32_t *send_counts, int32_t *send_offsets, int32_t *send_token,
                                  int32_t *send_row, void *ws, size_t ws_bytes, void *stream) {
    drop_stale_error();
    if (T < 0 || K < 1 || E < 1 || n_dev < 1) return C2R_ERR_INVALID_ARG;
    if (E > C2R_MAX_E || n_dev > C2R_MAX_E) return C2R_ERR_UNSUPPORTED;
    if (T * (int64_t)K >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    if (!expert_device || !send_counts || !send_offsets) return C2R_ERR_INVALID_ARG;
    if (T > 0 && (!topk_idx || !send_token || !send_row)) return C2R_ERR_INVALID_ARG;
    const size_t need = dedup_workspace_bytes(T > 0 ? T : 1, n_dev);
    if (!ws || ws_bytes < need || !aligned(ws, 256)) return C2R_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t nblocks = T > 0 ? (T + DB_SPAN - 1) / DB_SPAN : 1;
    if (nblocks >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    int32_t *block_counts = static_cast<int32_t *>(ws);
    dedup_count_kernel<<<dim3((unsigned)nblocks), dim3(DB_THREADS), 0, st>>>(topk_idx, T, K, E, expert_device, n_dev,
                                                                           block_counts);
    dedup_rank_kernel<<<dim3((unsigned)nblocks), dim3(DB_THREADS), 0, st>>>(
        topk_idx, T, K, E, expert_device, n_dev, block_counts, (int)nblocks, send_counts, send_offsets, send_token,
        send_row);
    return launch_status();
}

extern "C" int c2r_combine_partial(const void *y_perm, c2r_dtype dt, const float *gates, const int32_t *inv_perm,
                                   const int32_t *send_token, const int32_t *send_row, const int32_t *n_send,
                                   int64_t T, int64_t cap_rows, int d, int K, void *y_part, void *stream) {
    drop_stale_error();
    if (T < 0 || cap_rows < 0 || d < 1 || K < 1) return C2R_ERR_INVALID_ARG;
    if (dt != C2R_F32 && dt != C2R_BF16) return C2R_ERR_INVALID_ARG;
    if (T == 0 || cap_rows == 0) return C2R_OK;
    if (!y_perm || !gates || !inv_perm || !send_token || !send_row || !n_send || !y_part) return C2R_ERR_INVALID_ARG;
    if (d % 8 != 0) return C2R_ERR_UNSUPPORTED;
    if (!aligned(y_perm, 16) || !aligned(y_part, 16)) return C2R_ERR_INVALID_ARG;
    const int row_vecs = d * (dt == C2R_BF16 ? 2 : 4) / 16;
    const int64_t nblk = (cap_rows * row_vecs + 255) / 256;
    if (nblk >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == C2R_BF16)
        combine_partial_kernel<true><<<dim3((unsigned)nblk), dim3(256), 0, st>>>(
            static_cast<const uint4 *>(y_perm), gates, inv_perm, send_token, send_row, n_send, T, cap_rows, row_vecs, K,
            static_cast<uint4 *>(y_part));
    else
        combine_partial_kernel<false><<<dim3((unsigned)nblk), dim3(256), 0, st>>>(
            static_cast<const uint4 *>(y_perm), gates, inv_perm, send_token, send_row, n_send, T, cap_rows, row_vecs, K,
            static_cast<uint4 *>(y_part));
    return launch_status();
}

extern "C" int c2r_combine_copies(const void *y_part, c2r_dtype dt, const int32_t *send_row, int64_t T,
                                  int64_t cap_rows, int d, int K, const void *y_shared, void *y, void *stream) {
    drop_stale_error();
    if (T < 0 || cap_rows < 0 || d < 1 || K < 1) return C2R_ERR_INVALID_ARG;
    if (dt != C2R_F32 && dt != C2R_BF16) return C2R_ERR_INVALID_ARG;
    if (T == 0) return C2R_OK;
    if (!y_part || !send_row || !y) return C2R_ERR_INVALID_ARG;
    if (d % 8 != 0) return C2R_ERR_UNSUPPORTED;
    if (!aligned(y_part, 16) || !aligned(y, 16) || (y_shared && !aligned(y_shared, 16))) return C2R_ERR_INVALID_ARG;
    const int row_vecs = d * (dt == C2R_BF16 ? 2 : 4) / 16;
    const int64_t nblk = (T * row_vecs + 255) / 256;
    if (nblk >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == C2R_BF16)
        combine_copies_kernel<true><<<dim3((unsigned)nblk), dim3(256), 0, st>>>(
            static_cast<const uint4 *>(y_part), send_row, T, cap_rows, row_vecs, K, static_cast<const uint4 *>(y_shared),
            static_cast<uint4 *>(y));
    else
        combine_copies_kernel<false><<<dim3((unsigned)nblk), dim3(256), 0, st>>>(
            static_cast<const uint4 *>(y_part), send_row, T, cap_rows, row_vecs, K, static_cast<const uint4 *>(y_shared),
            static_cast<uint4 *>(y));
    return launch_status();
}
