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
// Tiles are numbered expert after expert; inside an expert in chunks of TILE_GM M-tiles, and
// inside a chunk N-tile after N-tile with the chunk's M-tiles fastest.  A chunk never spans
// two experts, so the ~32 workgroups that run together on an XCD stream each expert's
// weight k-slices once per chunk (with chunks of consecutive M-tiles regardless of expert,
// a chunk held 2-3 small experts and streamed all of their weights: measured 2.2 x the
// weight bytes at the Qwen-MoE shape).  Each XCD gets a contiguous range of tile numbers of
// equal estimated COST, not equal count: an M-tile of at most BM/2 rows (only an expert's
// last one can be) runs the short path, which is bound by streaming the expert's weights and
// counted as two thirds of a full tile (weights 3 : 2 measured 0.5-1 % faster per pass than
// 2 : 1, 3 : 1 and 1 : 1), and ranges of equal count were measured 6 % apart in cost on
// Zipf-sized experts.  A boundary moves at
// most 1/64 of the tiles away from its equal-count position, which bounds the workgroups a
// launch needs (ragged_grid) without knowing the group sizes on the host.
// estimated cost of an M-tile: full, and an expert's last one if it has at most BM/2 rows
#define C2R_COST_FULL 3
#define C2R_COST_SHORT 2
struct RaggedMap {
    int lo, hi;        // this lane's expert: row range (clamped to [0, A_cap])
    int tiles, first;  // its M-tiles and its first M-tile number
    int cost, pcost;   // C2R_COST_FULL per M-tile, C2R_COST_SHORT for a short last one; exclusive prefix over experts
    int total_mtiles, total_cost;  // wave-uniform
};

template <int BM>
__device__ __forceinline__ RaggedMap build_ragged_map(const int32_t *__restrict__ offsets, int E_local, int A_cap) {
    const GroupMap gm = build_group_map<BM>(offsets, E_local, A_cap);
    RaggedMap m;
    m.lo = gm.lo;
    m.hi = gm.hi;
    m.tiles = gm.tiles;
    m.first = gm.first;
    m.total_mtiles = gm.total_mtiles;
    const int cnt = gm.hi - gm.lo;
    const bool short_last = gm.tiles > 0 && cnt - (gm.tiles - 1) * BM <= BM / 2;
    m.cost = C2R_COST_FULL * gm.tiles - (short_last ? C2R_COST_FULL - C2R_COST_SHORT : 0);
    const int incl = wave_inclusive_scan(m.cost);
    m.pcost = incl - m.cost;
    m.total_cost = __builtin_amdgcn_readfirstlane(__shfl(incl, 63));
    return m;
}

// First tile number of XCD x's range (x = 8: one past the last tile).  Same result in every
// wave of the launch: integer arithmetic on the same map.
__device__ __forceinline__ int ragged_boundary(const RaggedMap &m, int ntn, int x) {
    const int total = m.total_mtiles * ntn;
    if (x <= 0) return 0;
    if (x >= 8) return total;
    const int even = (int)((uint64_t)(uint32_t)total * (uint32_t)x / 8u), win = total / 64;
    const uint64_t G = (uint64_t)(uint32_t)ntn * (uint32_t)m.total_cost;  // < 2^32 (launcher check)
    const uint32_t g = (uint32_t)(G * (uint32_t)x / 8u);
    const uint32_t clo = (uint32_t)ntn * (uint32_t)m.pcost, chi = clo + (uint32_t)ntn * (uint32_t)m.cost;
    const uint64_t hit = __ballot(m.cost > 0 && g >= clo && g < chi);
    if (hit == 0) return even;
    const int e = __ffsll((unsigned long long)hit) - 1;
    const int tiles = __builtin_amdgcn_readlane(m.tiles, e), first = __builtin_amdgcn_readlane(m.first, e);
    const int cost = __builtin_amdgcn_readlane(m.cost, e), pc = __builtin_amdgcn_readlane(m.pcost, e);
    const uint32_t r = g - (uint32_t)ntn * (uint32_t)pc;  // cost offset inside the expert
    const int sh = C2R_COST_FULL * tiles - cost;           // > 0: the last M-tile is short (full - short cost)
    const int gl = tiles - TILE_GM * ((tiles - 1) / TILE_GM);  // M-tiles of the last chunk
    const uint32_t R = (uint32_t)C2R_COST_FULL * (uint32_t)(tiles - gl) * (uint32_t)ntn;  // cost of the full chunks
    uint32_t t;
    if (r < R)
        t = r / (uint32_t)C2R_COST_FULL;
    else  // the last chunk's tiles cost (2 gl - sh) / gl on average (its M-tiles alternate)
        t = (uint32_t)(tiles - gl) * (uint32_t)ntn + (r - R) * (uint32_t)gl / (uint32_t)(C2R_COST_FULL * gl - sh);
    const int b = first * ntn + (int)t;
    return b < even - win ? even - win : (b > even + win ? even + win : b);
}

struct RaggedTile {
    int expert, row_begin, row_end;  // row_begin: first row of the tile (part); row_end: the expert's end
    int nt;
    int sub, nsub;  // the tile's rows are cut into nsub equal parts and this workgroup owns part sub
    bool valid;
};

// Workgroup (XCD, slot) -> tile.  The tiles an XCD has left after its last full round of
// CUS_PER_XCD are cut along M into 2 or 4 row parts, each its own workgroup, so that the
// last round occupies the CUs that would idle; the parts are dispatched last.
template <int BM>
__device__ __forceinline__ RaggedTile ragged_tile(const RaggedMap &m, int ntn, int xcd, int slot) {
    RaggedTile t;
    t.valid = false;
    t.expert = -1;
    t.row_begin = t.row_end = t.nt = t.sub = 0;
    t.nsub = 1;
    const int b0 = ragged_boundary(m, ntn, xcd), b1 = ragged_boundary(m, ntn, xcd + 1);
    const int cnt = b1 - b0;
    if (cnt <= 0) return t;
    int idx = slot;
    const int full = cnt / CUS_PER_XCD * CUS_PER_XCD, r = cnt - full;
    const int s = r == 0 ? 1 : (r * 4 <= CUS_PER_XCD ? 4 : (r * 2 <= CUS_PER_XCD ? 2 : 1));
    if (slot >= full) {
        const int q = slot - full;
        if (q >= r * s) return t;
        idx = full + q / s;
        t.sub = q % s;
        t.nsub = s;
    }
    const int tile = b0 + idx;
    const int tlo = m.first * ntn;
    const uint64_t hit = __ballot(m.tiles > 0 && tile >= tlo && tile < tlo + m.tiles * ntn);
    if (hit == 0) return t;
    const int e = __ffsll((unsigned long long)hit) - 1;
    const int tiles = __builtin_amdgcn_readlane(m.tiles, e), first = __builtin_amdgcn_readlane(m.first, e);
    const int tp = tile - first * ntn;
    const int c = tp / (TILE_GM * ntn);
    const int gsz = tiles - c * TILE_GM < TILE_GM ? tiles - c * TILE_GM : TILE_GM;
    const int rem = tp - c * TILE_GM * ntn;
    const int mloc = c * TILE_GM + rem % gsz;
    t.nt = rem / gsz;
    t.expert = e;
    t.row_begin = __builtin_amdgcn_readlane(m.lo, e) + mloc * BM + t.sub * (BM / t.nsub);
    t.row_end = __builtin_amdgcn_readlane(m.hi, e);
    t.valid = true;
    return t;
}

// Host side: workgroups to launch for the ragged map: a range holds at most 1/8 + 2/64 of
// the tiles (+1 for rounding), plus the split last round.
static inline int64_t ragged_grid(int64_t mtiles_bound, int ntn) {
    const int64_t total = mtiles_bound * ntn;
    const int64_t per_xcd = (total + 7) / 8 + 2 * (total / 64) + 2;
    return (per_xcd + CUS_PER_XCD) * 8;
}

}  // namespace c2r
