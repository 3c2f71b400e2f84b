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

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

}  // namespace c2r
