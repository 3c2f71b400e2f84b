// Token dispatch on one device: stable counting sort of the assignments
// a = t*K + s by local expert slot, then a coalesced row scatter.
//
//  1. permute_hist_kernel   per-block LDS histogram of local slots
//  2. permute_scan_kernel   counts, exclusive offsets, and the start position of
//                           every (block, slot) run
//  3. permute_rank_kernel   stable rank inside the block: each wave step ranks
//                           its 64 assignments with ballots (equal keys keep
//                           lane order), an LDS prefix over the block's wave
//                           steps orders the steps; writes perm / inv_perm
//  4. permute_rows_kernel   one wave per token: the row of x is read once and
//                           written to each of its (up to K) sorted positions
//                           with 16-byte accesses
// Up to 49152 assignments, steps 1-3 are one launch instead (permute_by_slot_kernel: 11 us at
// 32768 assignments and linear in their number; the three launches take 16-24 us from 65536 to
// 262144 assignments).
// Everything is deterministic: no atomically assigned slots.
#include <mutex>

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

// One workgroup of SCAN_WAVES waves; lane s works for slot s, wave w for a contiguous share of
// the blocks (loads of a share are independent of one another, so they are in flight together;
// one thread walking all the blocks of a large batch would wait for them one by one).
constexpr int SCAN_WAVES = 16;

__global__ __launch_bounds__(SCAN_WAVES * 64) void permute_scan_kernel(const int32_t *__restrict__ block_counts,
                                                                      int nblocks, int E_local,
                                                                      int32_t *__restrict__ block_base,
                                                                      int32_t *__restrict__ counts,
                                                                      int32_t *__restrict__ offsets) {
    __shared__ int32_t share_total[SCAN_WAVES][64];
    const int s = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int per = (nblocks + SCAN_WAVES - 1) / SCAN_WAVES;
    const int b0 = min(w * per, nblocks), b1 = min(b0 + per, nblocks);
    int32_t mine = 0;
    if (s < E_local) {
#pragma unroll 8
        for (int b = b0; b < b1; ++b) mine += block_counts[(size_t)b * E_local + s];
    }
    share_total[w][s] = mine;
    __syncthreads();
    int32_t total = 0, before = 0;  // the slot's count; its count in the shares of lower waves
#pragma unroll
    for (int v = 0; v < SCAN_WAVES; ++v) {
        const int32_t t = share_total[v][s];
        before += v < w ? t : 0;
        total += t;
    }
    // exclusive scan over slots (64 lanes)
    int32_t incl = total;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int32_t v = __shfl_up(incl, off);
        if (s >= off) incl += v;
    }
    const int32_t excl = incl - total;
    if (s < E_local) {
        if (w == 0) {
            counts[s] = total;
            offsets[s] = excl;
            if (s == E_local - 1) offsets[E_local] = incl;
        }
        int32_t run = excl + before;
#pragma unroll 8
        for (int b = b0; b < b1; ++b) {
            block_base[(size_t)b * E_local + s] = run;
            run += block_counts[(size_t)b * E_local + s];
        }
    }
}

__global__ __launch_bounds__(PB_THREADS) void permute_rank_kernel(
    const int32_t *__restrict__ topk_idx, int64_t A, int E, const int32_t *__restrict__ local_slot,
    int E_local, const int32_t *__restrict__ block_base, int32_t *__restrict__ perm,
    int32_t *__restrict__ inv_perm) {
    __shared__ int32_t step_cnt[PB_STEPS][C2R_MAX_E];
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
        int32_t run = block_base[(size_t)blockIdx.x * E_local + threadIdx.x];
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

// Small batches (the whole index array is a few hundred KB and sits in L2): one launch, one
// workgroup per local expert slot.  The workgroup's 16 waves each own a contiguous
// sixteenth of the assignments; a first sweep counts, per wave, the assignments of this
// slot and of all lower slots, a second sweep hands out the positions in order (ballot +
// prefix inside a 64-assignment step, running count across steps, wave totals across
// waves), which is the same stable order as the counting sort above.  Workgroup 0 also
// marks the assignments that belong to no local slot.
constexpr int PE_WAVES = 16;
constexpr int64_t BY_SLOT_MAX = 3 << 14;  // assignments up to which the one-launch form is the faster one
constexpr int PE_STEPS = 32;  // 64-assignment steps a wave holds in registers at a time

__global__ __launch_bounds__(PE_WAVES * 64) void permute_by_slot_kernel(
    const int32_t *__restrict__ topk_idx, int A, int E, const int32_t *__restrict__ local_slot, int E_local,
    int32_t *__restrict__ counts, int32_t *__restrict__ offsets, int32_t *__restrict__ perm,
    int32_t *__restrict__ inv_perm) {
    __shared__ int32_t w_mine[PE_WAVES], w_less[PE_WAVES];
    const int e = blockIdx.x, lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int seg = ((A + PE_WAVES - 1) / PE_WAVES + 63) / 64 * 64;  // assignments per wave, whole steps
    const int a_begin = wave * seg, a_end = min(A, a_begin + seg);
    // Up to 2048 assignments per wave (A <= 32768) the slots are loaded once, all loads in
    // flight together, and stay in registers for both sweeps; longer segments go in pieces
    // of that size and are read again by the second sweep.
    const bool single = seg <= PE_STEPS * 64;
    int sl[PE_STEPS];
    // (every load is unconditional, on a clamped index, so that all of them are in flight at
    // once: guarded loads end up one branch and one memory round trip each)
    auto load = [&](int c0) {
#pragma unroll
        for (int u = 0; u < PE_STEPS; ++u) sl[u] = topk_idx[min(c0 + u * 64 + lane, A - 1)];
        if (local_slot) {
            int ex[PE_STEPS];
#pragma unroll
            for (int u = 0; u < PE_STEPS; ++u) ex[u] = sl[u];
#pragma unroll
            for (int u = 0; u < PE_STEPS; ++u) sl[u] = local_slot[min(max(ex[u], 0), E - 1)];
#pragma unroll
            for (int u = 0; u < PE_STEPS; ++u) sl[u] = (ex[u] >= 0 && ex[u] < E) ? sl[u] : -1;
        } else {
#pragma unroll
            for (int u = 0; u < PE_STEPS; ++u) sl[u] = sl[u] < E ? sl[u] : -1;
        }
#pragma unroll
        for (int u = 0; u < PE_STEPS; ++u) {
            const bool slot_ok = sl[u] >= 0 && sl[u] < E_local;
            sl[u] = c0 + u * 64 + lane < a_end ? (slot_ok ? sl[u] : -1) : -2;  // -2: past the end
        }
    };
    int mine = 0, less = 0;
    for (int c0 = a_begin; c0 < a_end; c0 += PE_STEPS * 64) {
        load(c0);
#pragma unroll
        for (int u = 0; u < PE_STEPS; ++u) {
            mine += sl[u] == e;
            less += sl[u] >= 0 && sl[u] < e;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        mine += __shfl_xor(mine, off);
        less += __shfl_xor(less, off);
    }
    if (lane == 0) {
        w_mine[wave] = mine;
        w_less[wave] = less;
    }
    __syncthreads();
    int start = 0, total = 0;  // this slot's first position; its count
#pragma unroll
    for (int w = 0; w < PE_WAVES; ++w) {
        start += w_less[w];
        total += w_mine[w];
    }
    int run = start;
#pragma unroll
    for (int w = 0; w < PE_WAVES; ++w) run += w < wave ? w_mine[w] : 0;
    if (threadIdx.x == 0) {
        counts[e] = total;
        offsets[e] = start;
        if (e == E_local - 1) offsets[E_local] = start + total;
    }
    const uint64_t lt = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    for (int c0 = a_begin; c0 < a_end; c0 += PE_STEPS * 64) {
        if (!single) load(c0);
#pragma unroll
        for (int u = 0; u < PE_STEPS; ++u) {
            const int a = c0 + u * 64 + lane;
            const uint64_t m = __ballot(sl[u] == e);
            if (sl[u] == e) {
                const int p = run + __popcll(m & lt);
                perm[p] = a;
                inv_perm[a] = p;
            } else if (e == 0 && sl[u] == -1) {
                inv_perm[a] = -1;
            }
            run += __popcll(m);
        }
    }
}

// One wave per token; row bytes must be a multiple of 16.  The token's K positions are fetched
// first, all at once (they are one 16-byte vector for K = 4), then the row is read in pieces of
// 4 KB - four loads per lane in flight together, unconditional on clamped indices when the piece is
// whole - and every piece goes out to the K positions with stores that bypass the caches' keep
// policy (each output row is written once and read by another kernel).
__global__ __launch_bounds__(256) void permute_rows_kernel(const uint4 *__restrict__ x, int64_t T, int K,
                                                           int row_vecs,
                                                           const int32_t *__restrict__ inv_perm,
                                                           uint4 *__restrict__ x_perm) {
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const u32x4 *src = reinterpret_cast<const u32x4 *>(x) + t * row_vecs;
    u32x4 *out = reinterpret_cast<u32x4 *>(x_perm);
    if (K == 4 && (reinterpret_cast<uintptr_t>(inv_perm) & 15) == 0) {
        const i32x4 pos = *reinterpret_cast<const i32x4 *>(inv_perm + t * 4);
        if ((pos[0] & pos[1] & pos[2] & pos[3]) < 0) return;  // (all four negative: the token goes nowhere)
        for (int v0 = 0; v0 < row_vecs; v0 += 256) {
            u32x4 r[4];
            const bool whole = v0 + 256 <= row_vecs;  // (uniform)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int v = v0 + i * 64 + lane;
                r[i] = __builtin_nontemporal_load(src + (whole || v < row_vecs ? v : 0));
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                if (pos[s] < 0) continue;
                u32x4 *dst = out + (int64_t)pos[s] * row_vecs;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int v = v0 + i * 64 + lane;
                    if (whole || v < row_vecs) __builtin_nontemporal_store(r[i], dst + v);
                }
            }
        }
        return;
    }
    bool any = false;
    for (int s = 0; s < K; ++s) any |= inv_perm[t * K + s] >= 0;
    if (!any) return;
    for (int v0 = 0; v0 < row_vecs; v0 += 256) {
        u32x4 r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = v0 + i * 64 + lane;
            r[i] = src[v < row_vecs ? v : 0];
        }
        for (int s = 0; s < K; ++s) {
            const int32_t p = inv_perm[t * K + s];
            if (p < 0) continue;
            u32x4 *dst = out + (int64_t)p * row_vecs;
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

static int permute_impl(const void *x, c2r_dtype dt, const int32_t *topk_idx, int64_t T, int d,
                        int E, int K, const int32_t *local_slot, int E_local, int32_t *counts,
                        int32_t *offsets, int32_t *perm, int32_t *inv_perm, void *x_perm,
                        void *ws, size_t ws_bytes, void *stream) {
    drop_stale_error();
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
    if (A > 0 && A <= BY_SLOT_MAX) {
        // the index array is swept once per slot out of L2, in one launch
        permute_by_slot_kernel<<<dim3((unsigned)E_local), dim3(PE_WAVES * 64), 0, st>>>(
            topk_idx, (int)A, E, local_slot, E_local, counts, offsets, perm, inv_perm);
    } else {
        if (nblocks > 0)
            permute_hist_kernel<<<dim3((unsigned)nblocks), dim3(PB_THREADS), 0, st>>>(
                topk_idx, A, E, local_slot, E_local, block_counts);
        permute_scan_kernel<<<dim3(1), dim3(SCAN_WAVES * 64), 0, st>>>(block_counts, (int)nblocks, E_local,
                                                                      block_base, counts, offsets);
        if (nblocks > 0)
            permute_rank_kernel<<<dim3((unsigned)nblocks), dim3(PB_THREADS), 0, st>>>(
                topk_idx, A, E, local_slot, E_local, block_base, perm, inv_perm);
    }
    if (nblocks > 0) {
        if (x_perm) {
            const int row_vecs = d * (dt == C2R_BF16 ? 2 : 4) / 16;
            permute_rows_kernel<<<dim3((unsigned)((T + 3) / 4)), dim3(256), 0, st>>>(
                static_cast<const uint4 *>(x), T, K, row_vecs, inv_perm, static_cast<uint4 *>(x_perm));
        }
    }
    return launch_status();
}

extern "C" int c2r_permute(const void *x, c2r_dtype dt, const int32_t *topk_idx, int64_t T, int d,
                           int E, int K, const int32_t *local_slot, int E_local, int32_t *counts,
                           int32_t *offsets, int32_t *perm, int32_t *inv_perm, void *x_perm,
                           void *ws, size_t ws_bytes, void *stream) {
    return permute_impl(x, dt, topk_idx, T, d, E, K, local_slot, E_local, counts, offsets, perm, inv_perm, x_perm,
                        ws, ws_bytes, stream);
}

// ---- c2r_permute for callers that cannot allocate: the block histograms live in a static
//      device array instead of a caller-provided workspace ----
namespace c2r {
constexpr int64_t NOALLOC_MAX_ASSIGNMENTS = 1ll << 22;
constexpr size_t NOALLOC_SCRATCH_BYTES =
    2 * (size_t)(NOALLOC_MAX_ASSIGNMENTS / PB_SPAN) * C2R_MAX_E * sizeof(int32_t);  // 2 MiB
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];
constexpr int NOALLOC_MAX_DEVICES = 64;
static void *scratch_ptr[NOALLOC_MAX_DEVICES];  // per device: every GPU holds its own copy of the array
static std::mutex scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up once per device: in host
// code the array's name is only a handle for this query, never an address a kernel may use).
static int noalloc_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= NOALLOC_MAX_DEVICES) return C2R_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return C2R_ERR_LAUNCH;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return C2R_OK;
}
}  // namespace c2r

extern "C" int c2r_permute_noalloc(const void *x, c2r_dtype dt, const int32_t *topk_idx, int64_t T, int d,
                                   int E, int K, const int32_t *local_slot, int E_local, int32_t *counts,
                                   int32_t *offsets, int32_t *perm, int32_t *inv_perm, void *x_perm,
                                   void *stream) {
    if (T < 0 || K < 1) return C2R_ERR_INVALID_ARG;
    if (T > NOALLOC_MAX_ASSIGNMENTS || T * (int64_t)K > NOALLOC_MAX_ASSIGNMENTS) return C2R_ERR_UNSUPPORTED;
    void *ws = nullptr;
    const int rc = noalloc_scratch(&ws);
    if (rc != C2R_OK) return rc;
    return permute_impl(x, dt, topk_idx, T, d, E, K, local_slot, E_local, counts, offsets, perm, inv_perm, x_perm,
                        ws, NOALLOC_SCRATCH_BYTES, stream);
}
