// Ragged-group tile lookup shared by the expert-FFN kernels.
#pragma once
#include "c2r_internal.h"

namespace c2r {

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
    int incl = m.tiles;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
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

}  // namespace c2r
