// Ragged-group tile lookup shared by the expert-FFN kernels.
#pragma once
#include "c2r_internal.h"

namespace c2r {

struct GroupTile {
    int expert;       // local expert slot, -1: this workgroup has no tile
    int row_begin;    // first row of the tile in x_perm
    int row_end;      // one past the expert's last row
    int total_mtiles; // M-tiles over all experts
};

// Every wave calls this with all 64 lanes active.  Lane e sizes expert e's row
// range (offsets are clamped to [0, A_cap] so a corrupt array cannot send a load
// out of bounds), a wave scan turns tile counts into tile ranges, and the M-tile
// number mt is located with a ballot.  E_local <= 64.
template <int BM>
__device__ __forceinline__ GroupTile find_group_tile(const int32_t *__restrict__ offsets, int E_local,
                                                      int A_cap, int mt) {
    const int lane = lane_id();
    int lo = 0, hi = 0;
    if (lane < E_local) {
        lo = offsets[lane];
        hi = offsets[lane + 1];
        lo = lo < 0 ? 0 : (lo > A_cap ? A_cap : lo);
        hi = hi < lo ? lo : (hi > A_cap ? A_cap : hi);
    }
    const int tiles = (hi - lo + BM - 1) / BM;
    int incl = tiles;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    GroupTile g;
    g.total_mtiles = __shfl(incl, 63);
    const uint64_t hit = __ballot(incl > mt);
    if (mt < 0 || hit == 0) {
        g.expert = -1;
        g.row_begin = g.row_end = 0;
        return g;
    }
    const int e = __ffsll((unsigned long long)hit) - 1;
    const int excl_e = __shfl(incl - tiles, e);
    g.expert = e;
    g.row_begin = __shfl(lo, e) + (mt - excl_e) * BM;
    g.row_end = __shfl(hi, e);
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
    int mt, nt, total_mtiles;
    bool valid;
};

// Workgroup -> tile.  Tiles are numbered so that consecutive numbers walk GM M-tiles
// (fastest) by all N-tiles: the ~32 workgroups running together on one XCD then cover a
// near-square block of tiles and re-use each other's A and B k-slices out of that XCD's
// L2.  Each XCD (workgroup id mod 8) gets one contiguous range of tile numbers.
__device__ __forceinline__ TileId xcd_grouped_tile(int total_mtiles, int ntn) {
    constexpr int GM = 4;
    TileId t;
    t.total_mtiles = total_mtiles;
    t.valid = false;
    t.mt = t.nt = 0;
    const int total = total_mtiles * ntn;
    const int per_xcd = (total + 7) / 8;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int tile = xcd * per_xcd + slot;
    if (slot >= per_xcd || tile >= total) return t;
    const int grp = tile / (GM * ntn);
    const int first_m = grp * GM;
    const int gsz = total_mtiles - first_m < GM ? total_mtiles - first_m : GM;
    const int rem = tile - grp * GM * ntn;
    t.mt = first_m + rem % gsz;
    t.nt = rem / gsz;
    t.valid = true;
    return t;
}

}  // namespace c2r
