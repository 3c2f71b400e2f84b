// Ragged-group tile lookup shared by the expert-FFN kernels.
#pragma once
#include "c2r_internal.h"

namespace c2r {

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves (no
// LDS round trips): shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the row totals
// are passed on with the two row broadcasts.  Every lane must be active.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
#if defined(__HIP_DEVICE_COMPILE__)
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);  // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);  // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);  // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);  // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2, 3
#endif
    return v;
}

struct GroupTile {
    int expert;        // local expert slot, -1: no such tile
    int row_begin;     // first row of the tile in x_perm
    int row_end;       // one past the expert's last row
};

// Per-wave map from M-tile number to expert group, held one expert per lane.  M-tiles are
// numbered expert after expert in slot order (measured: numbering the big experts first, or
// dealing tile groups round-robin to the XCDs, costs more in lost L2 locality than the
// better balance returns).
struct GroupMap {
    int lo, hi;        // this lane's expert: row range (clamped to [0, A_cap])
    int tiles;         // its number of M-tiles
    int first;         // its first M-tile number
    int total_mtiles;  // M-tiles over all experts
};

// Every wave calls this with all 64 lanes active; E_local <= 64.  Offsets are clamped so
// that a corrupt array cannot send a load out of bounds.
template <int BM>
__device__ __forceinline__ GroupMap build_group_map(const int32_t *__restrict__ offsets, int E_local,
                                                     int A_cap) {
    const int lane = lane_id();
    GroupMap m;
    m.lo = m.hi = 0;
    if (lane < E_local) {
        int lo = offsets[lane], hi = offsets[lane + 1];
        lo = lo < 0 ? 0 : (lo > A_cap ? A_cap : lo);
        hi = hi < lo ? lo : (hi > A_cap ? A_cap : hi);
        m.lo = lo;
        m.hi = hi;
    }
    const int cnt = m.hi - m.lo;
    m.tiles = (cnt + BM - 1) / BM;
    const int incl = wave_inclusive_scan(m.tiles);
    m.first = incl - m.tiles;
    m.total_mtiles = __shfl(incl, 63);
    return m;
}

__device__ __forceinline__ GroupTile locate_group_tile(const GroupMap &m, int mt, int BM) {
    GroupTile g;
    const uint64_t hit = __ballot(mt >= m.first && mt < m.first + m.tiles);
    if (hit == 0) {
        g.expert = -1;
        g.row_begin = g.row_end = 0;
        return g;
    }
    const int e = __ffsll((unsigned long long)hit) - 1;
    g.expert = e;
    g.row_begin = __shfl(m.lo, e) + (mt - __shfl(m.first, e)) * BM;
    g.row_end = __shfl(m.hi, e);
    return g;
}

// silu(g) * u with the hardware reciprocal (1 ulp): the result is rounded to bf16 anyway
__device__ __forceinline__ float silu_mul(float g, float u) {
    return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// XOR key of the 16-byte chunk position inside a 128-byte tile row.  Chosen so that
// any 8 consecutive rows AND the even (or odd) rows of any 16 consecutive rows get 8
// distinct keys: a ds_read_b128 of one chunk column over consecutive rows is then
// conflict free whether the LDS serves 8 or 16 lanes per cycle.
__device__ __forceinline__ int swz_key(int row) { return ((row >> 1) & 7) ^ ((row & 1) << 2); }

struct TileId {
    int mt, nt;
    int sub, nsub;  // the tile's rows are cut into nsub equal parts and this workgroup owns part sub
    bool valid;
};

// Workgroup -> tile.  Tiles are numbered so that consecutive numbers walk GM M-tiles
// (fastest) by all N-tiles: the ~32 workgroups running together on one XCD then cover a
// near-square block of tiles and re-use each other's A and B k-slices out of that XCD's
// L2.  Each XCD (workgroup id mod 8) gets one contiguous range of tile numbers, so an
// expert's weights are mostly streamed by one XCD.
//
// With SPLIT_TAIL, the tiles an XCD has left after its last full round of 32 (one per CU)
// are cut along M into 2 or 4 row parts, each its own workgroup, so that the last round
// occupies the CUs that would idle; the parts are dispatched last because workgroups are
// handed out in id order.
constexpr int TILE_GM = 4;
constexpr int CUS_PER_XCD = 32;

template <bool SPLIT_TAIL>
__device__ __forceinline__ TileId xcd_grouped_tile(int total_mtiles, int ntn) {
    TileId t;
    t.valid = false;
    t.mt = t.nt = t.sub = 0;
    t.nsub = 1;
    const int total = total_mtiles * ntn;
    const int per_xcd = (total + 7) / 8;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int first = xcd * per_xcd;
    int cnt = total - first;
    cnt = cnt > per_xcd ? per_xcd : cnt;
    if (cnt <= 0) return t;
    int idx = slot;
    if (SPLIT_TAIL) {
        const int full = cnt / CUS_PER_XCD * CUS_PER_XCD, r = cnt - full;
        const int s = r == 0 ? 1 : (r * 4 <= CUS_PER_XCD ? 4 : (r * 2 <= CUS_PER_XCD ? 2 : 1));
        if (slot >= full) {
            const int q = slot - full;
            if (q >= r * s) return t;
            idx = full + q / s;
            t.sub = q % s;
            t.nsub = s;
        }
    } else if (slot >= cnt) {
        return t;
    }
    const int tile = first + idx;
    const int grp = tile / (TILE_GM * ntn);
    const int first_m = grp * TILE_GM;
    const int gsz = total_mtiles - first_m < TILE_GM ? total_mtiles - first_m : TILE_GM;
    const int rem = tile - grp * TILE_GM * ntn;
    t.mt = first_m + rem % gsz;
    t.nt = rem / gsz;
    t.valid = true;
    return t;
}

// Host side: workgroups to launch (a multiple of 8 that covers every tile, plus room for a
// split last round: at most CUS_PER_XCD workgroups per XCD replace its r < 32 tail tiles).
static inline int64_t xcd_grouped_grid(int64_t mtiles_bound, int ntn, bool split_tail) {
    const int64_t per_xcd = (mtiles_bound * ntn + 7) / 8;
    return (per_xcd + (split_tail ? CUS_PER_XCD : 0)) * 8;
}

// ---- Ragged tile map of the fast bf16 kernel --------------------------------------------
// M-tiles of BM rows are cut expert after expert; they fall into two classes.  FULL tiles hold
// more than BM/2 rows and are bound by the matrix pipe; a SHORT tile (at most BM/2 rows: only
// an expert's last one can be) is bound by streaming its expert's weights and takes about two
// thirds of a full tile's time however few rows it holds.  The classes are numbered apart:
//   class A  full tiles, expert after expert; inside an expert in chunks of TILE_GM M-tiles,
//            inside a chunk N-tile after N-tile with the chunk's M-tiles fastest, so that the
//            ~32 workgroups that run together on an XCD form a block of ONE expert's tiles
//            and share its k-slices in that XCD's L2 (a chunk never spans two experts);
//   class B  short tiles, expert after expert, N-tile after N-tile.
// Every XCD gets an equal COUNT of each class (a contiguous range of its numbers): tiles of a
// class cost the same, so the XCDs' loads are equal without a cost model, and the short tiles
// run LAST: an XCD hands its list out to whichever CU is free, so what decides the idle tail
// at the end of a launch is the length of the last items, and these are the shortest.
// (Before: one numbering with ranges of equal estimated cost, short tiles where their expert
// stood.  Measured at the Qwen-MoE shape: the XCDs finished 20-50 us apart and the CUs of an
// XCD idled 22 us at the end of each routed pass.)
struct RaggedMap {
    int lo, hi;            // this lane's expert: row range (clamped to [0, A_cap])
    int full, shortt;      // its full M-tiles; 1 if its last M-tile is a short one
    int firstA, firstB;    // exclusive prefixes of the two over the experts
    int totalA, totalB;    // wave-uniform totals
};

// From the expert's row range held by each lane (lo, hi: as build_group_map clamps them; lanes
// past E_local hold an empty range).  Every wave calls this with all 64 lanes active.
template <int BM>
__device__ __forceinline__ RaggedMap ragged_map_of(int lo, int hi) {
    RaggedMap m;
    m.lo = lo;
    m.hi = hi;
    const int cnt = hi - lo;
    const int tiles = (cnt + BM - 1) / BM;
    m.shortt = (tiles > 0 && cnt - (tiles - 1) * BM <= BM / 2) ? 1 : 0;
    m.full = tiles - m.shortt;
    // one scan for both: the short-tile count rides in the high byte (at most 64 of them)
    const int incl = wave_inclusive_scan(m.full | (m.shortt << 24));
    const int excl = incl - (m.full | (m.shortt << 24));
    m.firstA = excl & 0xffffff;
    m.firstB = excl >> 24;
    const int tot = __builtin_amdgcn_readlane(incl, 63);
    m.totalA = tot & 0xffffff;
    m.totalB = tot >> 24;
    return m;
}

// This lane's expert's row range, clamped so that a corrupt array cannot send a load out of bounds.
__device__ __forceinline__ void load_group_range(const int32_t *__restrict__ offsets, int E_local, int A_cap, int &lo,
                                                 int &hi) {
    lo = hi = 0;
    const int lane = lane_id();
    if (lane < E_local) {
        lo = offsets[lane];
        hi = offsets[lane + 1];
        lo = lo < 0 ? 0 : (lo > A_cap ? A_cap : lo);
        hi = hi < lo ? lo : (hi > A_cap ? A_cap : hi);
    }
}

struct RaggedTile {
    int expert, row_begin, row_end;  // row_begin: first row of the tile; row_end: the expert's end
    int nt;
    bool valid;
};

// Class A tile number -> tile.
template <int BM>
__device__ __forceinline__ RaggedTile ragged_full_tile_at(const RaggedMap &m, int ntn, int tile) {
    RaggedTile t;
    t.valid = false;
    t.expert = -1;
    t.row_begin = t.row_end = t.nt = 0;
    const int tlo = m.firstA * ntn;
    const uint64_t hit = __ballot(m.full > 0 && tile >= tlo && tile < tlo + m.full * ntn);
    if (hit == 0) return t;
    const int e = __ffsll((unsigned long long)hit) - 1;
    const int tiles = __builtin_amdgcn_readlane(m.full, e), first = __builtin_amdgcn_readlane(m.firstA, e);
    const int tp = tile - first * ntn;
    const int c = tp / (TILE_GM * ntn);
    const int gsz = tiles - c * TILE_GM < TILE_GM ? tiles - c * TILE_GM : TILE_GM;
    const int rem = tp - c * TILE_GM * ntn;
    const int mloc = c * TILE_GM + rem % gsz;
    t.nt = rem / gsz;
    t.expert = e;
    t.row_begin = __builtin_amdgcn_readlane(m.lo, e) + mloc * BM;
    t.row_end = __builtin_amdgcn_readlane(m.hi, e);
    t.valid = true;
    return t;
}

// Class B tile number -> tile.
template <int BM>
__device__ __forceinline__ RaggedTile ragged_short_tile_at(const RaggedMap &m, int ntn, int tile) {
    RaggedTile t;
    t.valid = false;
    t.expert = -1;
    t.row_begin = t.row_end = t.nt = 0;
    const int tlo = m.firstB * ntn;
    const uint64_t hit = __ballot(m.shortt > 0 && tile >= tlo && tile < tlo + ntn);
    if (hit == 0) return t;
    const int e = __ffsll((unsigned long long)hit) - 1;
    t.nt = tile - __builtin_amdgcn_readlane(m.firstB, e) * ntn;
    t.expert = e;
    t.row_begin = __builtin_amdgcn_readlane(m.lo, e) + __builtin_amdgcn_readlane(m.full, e) * BM;
    t.row_end = __builtin_amdgcn_readlane(m.hi, e);
    t.valid = true;
    return t;
}

// ---- An XCD's list.  A launch carries one problem or TWO (the routed groups and an always-on
// shared expert, a single group).  The list of an XCD is: its share of the single group's
// tiles (the longest items first: at the Qwen-MoE shape a tile of the shared expert's down
// pass runs 88 k-slices, a routed one 22), then its share of the ragged problem's full tiles,
// then its share of the short tiles; the last round of the COMBINED list is cut into row
// parts. ----
struct XcdRange {
    int first, cnt;  // first tile number and number of tiles of one XCD
};

__device__ __forceinline__ void single_group_tile_at(int total_mtiles, int ntn, int tile, int &mt, int &nt) {
    const int grp = tile / (TILE_GM * ntn);
    const int first_m = grp * TILE_GM;
    const int gsz = total_mtiles - first_m < TILE_GM ? total_mtiles - first_m : TILE_GM;
    const int rem = tile - grp * TILE_GM * ntn;
    mt = first_m + rem % gsz;
    nt = rem / gsz;
}

// An equal share of n numbered tiles for each of the 8 XCDs (contiguous ranges).
__device__ __forceinline__ XcdRange equal_range(int n, int xcd) {
    XcdRange r;
    const int per_xcd = (n + 7) / 8;
    r.first = xcd * per_xcd;
    int cnt = n - r.first;
    cnt = cnt > per_xcd ? per_xcd : cnt;
    r.cnt = cnt > 0 ? cnt : 0;
    return r;
}

// Slot of an XCD's list of cnt tiles -> tile index in the list and row part.  The tiles left
// after the last full round of CUS_PER_XCD are cut along M into 2 or 4 parts, each a workgroup
// of its own (at most CUS_PER_XCD of them), so that the last round occupies the CUs that
// would idle; the parts are dispatched last.
struct TailSplit {
    int idx, sub, nsub;
    bool valid;
};

__device__ __forceinline__ TailSplit split_last_round(int cnt, int slot) {
    TailSplit t;
    t.idx = slot;
    t.sub = 0;
    t.nsub = 1;
    t.valid = false;
    if (cnt <= 0) return t;
    const int full = cnt / CUS_PER_XCD * CUS_PER_XCD, r = cnt - full;
    const int s = r == 0 ? 1 : (r * 4 <= CUS_PER_XCD ? 4 : (r * 2 <= CUS_PER_XCD ? 2 : 1));
    if (slot >= full) {
        const int q = slot - full;
        if (q >= r * s) return t;
        t.idx = full + q / s;
        t.sub = q % s;
        t.nsub = s;
    }
    t.valid = true;
    return t;
}

// Host side: bound on the tiles one XCD may get from a ragged problem (its share of the full
// tiles plus its share of at most one short tile per expert) / from a single group.
static inline int64_t ragged_per_xcd_bound(int64_t mtiles_bound, int E_local, int ntn) {
    return (mtiles_bound * ntn + 7) / 8 + ((int64_t)E_local * ntn + 7) / 8;
}
static inline int64_t single_per_xcd_bound(int64_t mtiles_bound, int ntn) { return (mtiles_bound * ntn + 7) / 8; }

// One problem of a fast bf16 FFN launch (see ffn_bf16_dma.hip); a launch carries one or two.
struct FfnProblem {
    const uint16_t *A;        // activations [rows, lda] (or, with gather, the un-permuted [T, lda])
    const int32_t *offsets;   // DEVICE int32[E_local + 1]; nullptr: one group, rows [row_lo, row_hi)
    const uint16_t *B0, *B1;  // weights [E_local, N, Kdim] (B1: the up projection of pass 0)
    uint16_t *out;            // [rows, ldo]
    const int32_t *gather;    // row p of the sorted order is A[gather[p] / gather_div], or nullptr
    int lda, E_local, A_cap, N, Kdim, ldo, ntn, zero_to, gather_div, gather_rows, row_lo, row_hi;
};
struct FfnLaunch {
    FfnProblem p[2];            // p[0]: the ragged problem (several groups), p[1]: the single group
    int has_ragged, has_single;  // which of the two the launch carries (at least one)
};

}  // namespace c2r
