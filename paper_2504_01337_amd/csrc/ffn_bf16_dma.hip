// Grouped SwiGLU expert FFN in bf16, fast path: global -> LDS copies that bypass the
// register file (global_load_lds_dwordx4), 8 waves per workgroup, 256 x 256 output tiles,
// 64-wide k-slices in LDS (two stages of the activation tile, a ring of three of the weight
// tile: 160 KB), v_mfma_f32_16x16x32_bf16 (measured 4-8 % faster
// here than the 32x32x16 form at equal LDS traffic: a quarter of the accumulator registers
// move per instruction, and under this chip's power limit that buys clock).
//
// Same two passes, tile numbering and epilogue as the generic kernel in ffn_bf16.hip;
// what differs is how a k-slice reaches LDS.  One wave-level copy instruction moves
// 64 x 16 bytes = 8 tile rows of 128 bytes, i.e. whole cache lines (measured: 128-byte
// rows copy at ~25 TB/s chip-wide, 64-byte rows at ~16 TB/s).  Lane l lands at byte 16*l of the 1 KB run, i.e. row l/8, chunk
// position l%8, so the lane fetches the global chunk (l%8) ^ swz_key(row) and the
// swizzled layout falls out without any LDS write instruction.  The copies are
// asynchronous and overlap the MFMAs: the A tile of slice k+2 goes out when the stage of
// slice k is handed over, the B tile of slice k+2 a little earlier into the ring slot of
// slice k-1 (weights stream from HBM and take longest); one "my copies of the next slice
// landed, my reads returned" wait + bare barrier per slice, placed before the slice's last
// k-step, hands the stages over (see slice_step).
//
// Contract (checked by the launcher): the contraction length seen by A is padded to a
// multiple of 64 with zeros (lda >= 64 * ceil(K/64)); a B chunk past K is re-read from
// chunk 0 of the same row and multiplied by those zeros.
#include <atomic>
#include <type_traits>

#include "ffn_common.h"

namespace c2r {

// 16 bytes per lane, global -> LDS, without passing through registers.  `lds` is the
// wave-uniform start of the 1024-byte run; lane l's data lands at lds + 16*l.
// Written as inline assembly on purpose: when the compiler sees the copy as an LDS write
// it guards later LDS reads with vmcnt(0) whenever its alias bookkeeping loses track
// (it does across this kernel's unrolled ring), which serialises the pipeline.  Hidden
// from it, the only waits on copies are the ones this file states (wait_copies_but).
// The source is a wave-uniform base (scalar registers) plus a 32-bit byte offset per lane:
// no 64-bit address arithmetic per copy, and half the address bits to send.
__device__ __forceinline__ void copy16_to_lds(const unsigned char *base, uint32_t off, unsigned char *lds) {
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
    asm volatile(
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, %1"
        :
        : "v"(off), "s"(base), "s"(lds_addr)
        : "memory", "m0");
#endif
}

// A pointer the compiler may keep in scalar registers (the value is the same in every lane).
__device__ __forceinline__ const unsigned char *uniform_ptr(const unsigned char *p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const unsigned char *>(((uint64_t)hi << 32) | lo);
}

// Wait until at most N of this wave's copies are still in flight (they complete in order);
// the other counters are left alone.
template <int N>
__device__ __forceinline__ void wait_copies_but() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
#endif
}

// vmcnt(0) and lgkmcnt(0): this wave's copies have landed and its LDS reads have returned.
__device__ __forceinline__ void wait_copies_and_lds() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0x0070);
#endif
}

// lgkmcnt(0) alone: this wave's LDS reads have returned and its LDS writes are done; whatever
// it has in flight to or from memory (the epilogue's stores) stays in flight.
__device__ __forceinline__ void wait_lds_only() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0xC07F);
#endif
}

// Same, and this wave's LDS reads have returned (lgkmcnt(0)).
template <int N>
__device__ __forceinline__ void wait_copies_but_and_lds() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
#endif
}

// Bare workgroup barrier.  __syncthreads() (and any workgroup fence) also drains every
// outstanding copy (vmcnt(0)), which would serialise the slices in flight; here the
// caller states exactly which copies must have landed (wait_copies_but) and the
// scheduling fences keep the compiler from moving LDS reads across the barrier.
__device__ __forceinline__ void lds_barrier() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#endif
}

// The launch arguments as the tile function reads them: through the constant address space
// (scalar loads from the kernel-argument segment).
typedef const __attribute__((address_space(4))) FfnLaunch FfnLaunchConst;
typedef const __attribute__((address_space(4))) FfnProblem FfnProblemConst;
typedef FfnLaunchConst *FfnLaunchArgs;

// Shapes shared by the per-tile function and the kernel around it.
template <int WM, int WN>
struct FfnShape {
    static constexpr int BM = 256, BN = 256, BK = 64, NW = WM * WN, ROWB = BK * 2;
    static constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    static constexpr int LONG_BYTES = 2 * A_BYTES + 3 * B_BYTES;         // 2 A stages + a ring of 3 B stages
    static constexpr int SHORT_BYTES = 3 * (128 + BN) * ROWB;            // ring of 3 x (128 A rows + B tile)
    static constexpr int SMEM_BYTES = LONG_BYTES > SHORT_BYTES ? LONG_BYTES : SHORT_BYTES;
};

// Length of XCD x's list (tiles, with the last round cut into parts): what its queue hands out.
__device__ __forceinline__ int xcd_list_slots(int n_tiles) {
    if (n_tiles <= 0) return 0;
    const int full = n_tiles / CUS_PER_XCD * CUS_PER_XCD, r = n_tiles - full;
    const int s = r == 0 ? 1 : (r * 4 <= CUS_PER_XCD ? 4 : (r * 2 <= CUS_PER_XCD ? 2 : 1));
    return full + r * s;
}

// One output tile: position `slot` of XCD `xcd`'s list.  Every wave of the workgroup calls it
// with the same arguments; it returns early (all waves alike) when the position holds nothing.
// grp_lo, grp_hi: the row range of this lane's expert of the ragged problem (load_group_range);
// sg_lo, sg_hi: the row range of the single group (clamped), the same in every lane.
// before_epilogue(): called once by every wave after the tile's last k-step (the kernel draws
// the next ticket there, so that the trip to the counter overlaps the epilogue); not called on
// the early returns.
template <int MODE, int WM, int WN, class BeforeEpilogue>
__device__ __forceinline__ void ffn_tile(const FfnLaunchArgs Lp, unsigned char *smem, const int xcd, const int slot,
                                         const int grp_lo, const int grp_hi, const int sg_lo, const int sg_hi,
                                         BeforeEpilogue &&before_epilogue) {
    const FfnLaunchConst &L = *Lp;
    constexpr int BM = 256, BN = 256, BK = 64;
    constexpr int NW = WM * WN;                // waves
    constexpr int TM = BM / WM, TN = BN / WN;  // wave tile
    constexpr int ROWB = BK * 2;               // 128 bytes per tile row: whole cache lines per copy
    constexpr int GA = BM / 8 / NW, GB = BN / 8 / NW;  // 8-row copy groups per wave
    constexpr int A_BYTES = BM * ROWB, STAGE_BYTES = (BM + BN) * ROWB;
    constexpr int BNF = MODE == 0 ? BN / 2 : BN;
    static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "copy groups divide evenly");
    // Short tiles (<= LM rows, i.e. small experts) are bound by streaming their expert's
    // weights from HBM, not by the MFMAs: they use the same LDS as a three-stage ring of
    // (LM A rows + BN B rows), two slices in flight instead of one.
    constexpr int LM = 128, L_A_BYTES = LM * ROWB, L_STAGE_BYTES = (LM + BN) * ROWB, L_NSTAGE = 3;
    constexpr int L_GA = LM / 8 / NW;  // A copy groups per wave on the short path
    // Long path: two stages of A (rows of the activations: shared through L2 by the workgroups of
    // a tile row, short latency) and a ring of THREE stages of B (rows of the weights: streamed
    // from HBM, long latency), so that a B slice is copied two slices ahead of its use.
    constexpr int B_BYTES = BN * ROWB, B_NSTAGE = 3;
    constexpr int LONG_BYTES = 2 * A_BYTES + B_NSTAGE * B_BYTES;
    // Tiles of at most TM_T rows (experts with a handful of tokens: most of the short tiles) need
    // even less room for A and get a ring of four stages, three slices in flight: what such a
    // tile takes is the latency of its weight slices divided by the slices in flight.
    constexpr int TM_T = 64, T_A_BYTES = TM_T * ROWB, T_STAGE_BYTES = (TM_T + BN) * ROWB, T_NSTAGE = 4;
    static_assert(TM_T / 8 == NW, "one A copy group per wave on the tiny path");
    constexpr int SMEM_BYTES = LONG_BYTES > L_NSTAGE * L_STAGE_BYTES ? LONG_BYTES : L_NSTAGE * L_STAGE_BYTES;
    static_assert(T_NSTAGE * T_STAGE_BYTES <= SMEM_BYTES, "the tiny ring fits");
    static_assert(SMEM_BYTES == FfnShape<WM, WN>::SMEM_BYTES, "the kernel allocates what the tile function lays out");
    static_assert(LM == TM && (LM / 8) % NW == 0, "the short path is the first wave row's M range");
    unsigned char *const st0 = smem, *const st1 = smem + A_BYTES;  // the two A stages
    // B ring slot q lives at smem + 2*A_BYTES + q*B_BYTES.  Copies and fragment reads address B
    // as "stage + A_BYTES + ...", so a B slot is handed to them as the pointer A_BYTES below it.
    unsigned char *bcur = smem + A_BYTES, *bnxt = bcur + B_BYTES, *bwr = bnxt + B_BYTES;

    // (the thread index is made opaque per tile: what is derived from it - copy offsets, fragment
    // addresses - is then recomputed per tile instead of being hoisted out of the kernel's tile
    // loop and held in registers across it)
    int tid_opaque = threadIdx.x;
    asm volatile("" : "+v"(tid_opaque));
    const int tid = tid_opaque, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // Tile of this workgroup.  The launch carries one problem, or two (the routed groups and an
    // always-on shared expert).  An XCD's list: its share of the single group's tiles, then of
    // the ragged problem's full tiles, then of its short tiles (ffn_common.h).  One group (a
    // shared expert, a plain GEMM) needs no map: its bounds are two scalars.
    // (the launcher puts the ragged problem, if any, in p[0] and the single group in p[1])
    const bool ragged0 = L.has_ragged != 0, have_sg = L.has_single != 0;
    const int slo = sg_lo, shi = sg_hi;
    int smt = 0;
    XcdRange rs, ra, rb;
    rs.first = rs.cnt = ra.first = ra.cnt = rb.first = rb.cnt = 0;
    if (have_sg) {
        smt = (shi - slo + BM - 1) / BM;
        rs = equal_range(smt * L.p[1].ntn, xcd);
    }
    RaggedMap rmap;
    if (ragged0) {
        rmap = ragged_map_of<BM>(grp_lo, grp_hi);
        ra = equal_range(rmap.totalA * L.p[0].ntn, xcd);
        rb = equal_range(rmap.totalB * L.p[0].ntn, xcd);
    }
    TailSplit ts = split_last_round(rs.cnt + ra.cnt + rb.cnt, slot);
    if (!ts.valid) return;
    // (the same in every lane, but derived from cross-lane moves: say so, so that everything
    // picked by them - the problem's arguments above all - stays in scalar registers)
    ts.idx = __builtin_amdgcn_readfirstlane(ts.idx);
    ts.sub = __builtin_amdgcn_readfirstlane(ts.sub);
    ts.nsub = __builtin_amdgcn_readfirstlane(ts.nsub);
    const int n_s = __builtin_amdgcn_readfirstlane(rs.cnt), n_a = __builtin_amdgcn_readfirstlane(ra.cnt);
    // Position in the XCD's list -> item.  The short tiles are SPREAD evenly through the list
    // (a short tile streams its expert's weights from HBM at what one CU can pull, ~44 GB/s,
    // with the matrix pipe nearly idle: side by side with compute-bound tiles on the other CUs
    // that costs nothing but the CU; all of them together at the end or at the start of the
    // launch is a phase in which the whole chip waits for HBM - measured 36 us per short tile
    // instead of 28).  The other items keep their order: single group first, then full tiles.
    // ... except that the LAST few short tiles of the range close the list: the CUs that run out
    // of full tiles first take them while the others finish their last full tile, which fills
    // part of the idle tail of the launch with work that would otherwise sit in the middle of
    // it (few enough of them that they do not have to share HBM: FILL_TAIL per XCD).
    constexpr int FILL_TAIL = 12;
    const int n_b = __builtin_amdgcn_readfirstlane(rb.cnt);
    const int n_tail = n_b < FILL_TAIL ? n_b : FILL_TAIL, n_bi = n_b - n_tail, n_main = n_s + n_a + n_bi;
    const bool in_tail = ts.idx >= n_main;
    const int b_before = in_tail ? n_bi + (ts.idx - n_main)
                                 : (int)((uint32_t)ts.idx * (uint32_t)n_bi / (uint32_t)(n_main > 0 ? n_main : 1));
    const bool is_b = in_tail || (int)(((uint32_t)ts.idx + 1u) * (uint32_t)n_bi / (uint32_t)(n_main > 0 ? n_main : 1)) > b_before;
    const int o_rank = ts.idx - b_before;  // rank among the other items
    const bool second = !is_b && o_rank < n_s;  // workgroup-uniform: this tile is the single group's (p[1])
    GroupTile g;
    int tile_nt;
    const int tile_nsub = ts.nsub;
    if (second) {
        int mt;
        single_group_tile_at(smt, L.p[1].ntn, rs.first + o_rank, mt, tile_nt);
        g.expert = 0;
        g.row_begin = slo + mt * BM + ts.sub * (BM / ts.nsub);  // of this workgroup's part of the tile
        g.row_end = shi;
    } else {
        const RaggedTile tr = is_b ? ragged_short_tile_at<BM>(rmap, L.p[0].ntn, rb.first + b_before)
                                   : ragged_full_tile_at<BM>(rmap, L.p[0].ntn, ra.first + o_rank - n_s);
        if (!tr.valid) return;
        g.expert = tr.expert;
        g.row_begin = tr.row_begin + ts.sub * (BM / ts.nsub);
        g.row_end = tr.row_end;
        tile_nt = tr.nt;
    }
    // the problem's arguments, uniform over the workgroup from here on
    const FfnProblemConst &P = L.p[second ? 1 : 0];  // (a scalar address: the fields are scalar loads)
    const uint16_t *__restrict__ A = P.A;
    const uint16_t *__restrict__ B0 = P.B0;
    const uint16_t *__restrict__ B1 = P.B1;
    uint16_t *__restrict__ out = P.out;
    const int32_t *__restrict__ gather = P.gather;
    const int lda = P.lda, N = P.N, Kdim = P.Kdim, ldo = P.ldo;
    const int zero_to = P.zero_to, gather_div = P.gather_div, gather_rows = P.gather_rows;
    const int n0 = tile_nt * BNF;
    int rows = g.row_end - g.row_begin;  // may exceed the tile (clamped by the row guards below)
    if (rows <= 0) return;
    if (tile_nsub > 1 && rows > BM / tile_nsub) rows = BM / tile_nsub;
    const bool short_tile = rows <= LM;        // workgroup-uniform
    const bool tiny_tile = rows <= TM_T;

    // ---- copy roles: one copy instruction fills 8 tile rows (1024 bytes); lane l lands on
    //      row l/8, chunk position l%8 and therefore fetches chunk (l%8) ^ key(row) ----
    const int lrow = lane >> 3, lpos = lane & 7;
    int chunkc[2];  // for even / odd 8-row groups (the key depends on row bits 0..3)
#pragma unroll
    for (int par = 0; par < 2; ++par) chunkc[par] = lpos ^ swz_key(par * 8 + lrow);
    // With `gather`, A is the un-permuted activation matrix and row p of the sorted order is
    // A[gather[p] / gather_div] (the dispatch gather folded into the copy addresses).
    const unsigned char *baseA =
        uniform_ptr(reinterpret_cast<const unsigned char *>(gather ? A : A + (size_t)g.row_begin * lda));
    const unsigned char *baseB0 = uniform_ptr(reinterpret_cast<const unsigned char *>(B0 + (size_t)g.expert * N * Kdim));
    const unsigned char *baseB1 =
        MODE == 0 ? uniform_ptr(reinterpret_cast<const unsigned char *>(B1 + (size_t)g.expert * N * Kdim)) : baseB0;
    uint32_t offA[GA], offB[GB], rowB[GB];
    int rowA[GA];
#pragma unroll
    for (int i = 0; i < GA; ++i) {
        const int rg = tiny_tile ? wave : short_tile ? wave * L_GA + (i < L_GA ? i : 0) : wave * GA + i;
        const int r = rg * 8 + lrow;
        rowA[i] = r < rows ? r : rows - 1;
    }
    if (gather) {
#pragma unroll
        for (int i = 0; i < GA; ++i) rowA[i] = gather[g.row_begin + rowA[i]];  // the index loads fly together
#pragma unroll
        for (int i = 0; i < GA; ++i) {
            const int r = rowA[i] > 0 ? (int)((uint32_t)rowA[i] / (uint32_t)gather_div) : 0;
            rowA[i] = r < gather_rows ? r : gather_rows - 1;  // an out-of-range entry cannot leave A
        }
    }
#pragma unroll
    for (int i = 0; i < GA; ++i) {
        const int rg = tiny_tile ? wave : short_tile ? wave * L_GA + (i < L_GA ? i : 0) : wave * GA + i;
        offA[i] = (uint32_t)rowA[i] * (uint32_t)lda * 2u + (uint32_t)chunkc[rg & 1] * 16u;
    }
#pragma unroll
    for (int i = 0; i < GB; ++i) {
        const int rg = wave * GB + i;
        int r = rg * 8 + lrow;
        if (MODE == 0 && r >= BN / 2) r -= BN / 2;
        int c = n0 + r;
        c = c < N ? c : N - 1;
        rowB[i] = (uint32_t)c * (uint32_t)Kdim * 2u;
        offB[i] = rowB[i] + (uint32_t)chunkc[rg & 1] * 16u;
    }
    // GB*8 rows per wave divide BN/2, so a wave's B rows are all gate rows or all up rows
    const unsigned char *baseB = (MODE == 0 && wave * GB * 8 >= BN / 2) ? baseB1 : baseB0;

    const int nk = (Kdim + BK - 1) / BK;
    const bool ktail = (Kdim % BK) != 0;
    // Piece p of a slice's copy: p < GA are this wave's A row groups, the rest its B groups.
    // Copies are issued one at a time between MFMAs (see slice_step): the texture-address
    // unit takes one 64-lane x 16-byte request per ~16 cycles, so a burst of all of a
    // workgroup's copies would hold every wave at its copy instructions for ~1000 cycles
    // with the matrix pipe idle.
    // `inner`: kt is known not to be the last slice (no k tail to clamp).
    auto copy_piece = [&](int kt, unsigned char *stage, int p, bool inner = false) {
        const uint32_t kb = (uint32_t)kt * ROWB;  // the slice's byte offset goes into the scalar base
        if (p < GA) {
            copy16_to_lds(baseA + kb, offA[p], stage + (wave * GA + p) * 1024);
        } else if (inner) {
            const int i = p - GA, rg = wave * GB + i;
            copy16_to_lds(baseB + kb, offB[i], stage + A_BYTES + rg * 1024);
        } else {  // a B chunk past K is taken from chunk 0: it meets A's zero padding
            const int i = p - GA, rg = wave * GB + i;
            const bool clampB = ktail && kt == nk - 1 && kt * BK + chunkc[rg & 1] * 8 >= Kdim;
            copy16_to_lds(baseB, clampB ? rowB[i] : offB[i] + kb, stage + A_BYTES + rg * 1024);
        }
    };
    constexpr int NPIECE = GA + GB;

    // v_mfma_f32_16x16x32_bf16: 16 x 16 output fragments, 32 k per instruction.  A wave owns
    // 8 x 4 of them (128 x 64 outputs); a k-step is one 32-wide k range x one 64-row half.
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr int FM16 = TM / 16, FN16 = TN / 16;
    static_assert(FM16 == 8 && FN16 == 4, "k-step macros below");
    f32x4 acc[FM16][FN16];
#pragma unroll
    for (int i = 0; i < FM16; ++i)
#pragma unroll
        for (int j = 0; j < FN16; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;

    const int fr = lane & 15, fq = lane >> 4;
    uint32_t rdA[FM16], rdB[FN16];
#pragma unroll
    for (int i = 0; i < FM16; ++i) rdA[i] = (uint32_t)(wm * TM + i * 16 + fr) * ROWB;
#pragma unroll
    for (int j = 0; j < FN16; ++j) {
        int r;
        if (MODE == 0)
            r = (j < FN16 / 2) ? wn * (TN / 2) + j * 16 : BN / 2 + wn * (TN / 2) + (j - FN16 / 2) * 16;
        else
            r = wn * TN + j * 16;
        rdB[j] = (uint32_t)(tiny_tile ? T_A_BYTES : short_tile ? L_A_BYTES : A_BYTES) + (uint32_t)(r + fr) * ROWB;
    }
    const int sw = swz_key(fr);
    // waves whose whole M range lies past the group's end, or whose output columns all lie past N (the
    // last N-tile of a width that is not a multiple of the tile: 688 = 5 x 128 + 48), only help with
    // the copies: their results would be thrown away, and under the chip's power limit matrix
    // instructions on padding cost the other waves clock
    const bool cols_exist = n0 + (MODE == 0 ? wn * (TN / 2) : wn * TN) < N;  // (uniform per wave)
    const bool active = __builtin_amdgcn_readfirstlane(rows - wm * TM) > 0 && cols_exist;

    bf16x8 aset[2][4], bset[2][4];
    // A fragments of k range kq (0, 1) and 64-row half `half` into set `set`
    auto read_a = [&](const unsigned char *stage, int kq, int half, int set) {
        const uint32_t ch = (uint32_t)(((kq * 4 + fq) ^ sw) * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) aset[set][i] = *reinterpret_cast<const bf16x8 *>(stage + rdA[half * 4 + i] + ch);
    };
    // the first n (wave-uniform, 1..4) of them only
    auto read_a_first = [&](const unsigned char *stage, int kq, int half, int set, int n) {
        const uint32_t ch = (uint32_t)(((kq * 4 + fq) ^ sw) * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i < n) aset[set][i] = *reinterpret_cast<const bf16x8 *>(stage + rdA[half * 4 + i] + ch);
    };
    auto read_b = [&](const unsigned char *stage, int kq, int set) {
        const uint32_t ch = (uint32_t)(((kq * 4 + fq) ^ sw) * 16);
#pragma unroll
        for (int j = 0; j < 4; ++j) bset[set][j] = *reinterpret_cast<const bf16x8 *>(stage + rdB[j] + ch);
    };
    static_assert(NPIECE == 8, "copy schedule below: the A pieces in one k-step, the B pieces in another");
    // MFMAs of one k-step (operands swapped: the lane's 4 results lie along n) with up to
    // eight copy pieces P0.. of slice CKT slipped in after every second MFMA.  Macros, so that
    // every fragment and piece index is a literal and the arrays stay in registers.
#define C2R_MFMA(AS, BS, H, I, J)                                                                 \
    acc[(H) * 4 + (I)][J] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bset[BS][J], aset[AS][I],     \
                                                                    acc[(H) * 4 + (I)][J], 0, 0, 0)
#define C2R_MFMA_ROW(AS, BS, H, I) \
    C2R_MFMA(AS, BS, H, I, 0);     \
    C2R_MFMA(AS, BS, H, I, 1);     \
    C2R_MFMA(AS, BS, H, I, 2);     \
    C2R_MFMA(AS, BS, H, I, 3)
#define C2R_COPY_IF(Q, NCP, CKT, CST, P0)           \
    if ((Q) < (NCP)) {                              \
        __builtin_amdgcn_sched_barrier(0);          \
        copy_piece(CKT, CST, (P0) + (Q), STEADY);   \
        __builtin_amdgcn_sched_barrier(0);          \
    }
#define C2R_MFMA_HALF(AS, BS, H, I, J0) \
    C2R_MFMA(AS, BS, H, I, (J0));         \
    C2R_MFMA(AS, BS, H, I, (J0) + 1)
#define C2R_KSTEP(AS, BS, H, CKT, CST, P0, NCP, EARLY) \
    do {                                            \
        __builtin_amdgcn_sched_barrier(0);          \
        C2R_MFMA_HALF(AS, BS, H, 0, 0);             \
        __builtin_amdgcn_sched_barrier(0);          \
        EARLY;                                      \
        __builtin_amdgcn_sched_barrier(0);          \
        C2R_COPY_IF(0, NCP, CKT, CST, P0)           \
        C2R_MFMA_HALF(AS, BS, H, 0, 2);             \
        C2R_COPY_IF(1, NCP, CKT, CST, P0)           \
        C2R_MFMA_HALF(AS, BS, H, 1, 0);             \
        C2R_COPY_IF(2, NCP, CKT, CST, P0)           \
        C2R_MFMA_HALF(AS, BS, H, 1, 2);             \
        C2R_COPY_IF(3, NCP, CKT, CST, P0)           \
        C2R_MFMA_HALF(AS, BS, H, 2, 0);             \
        C2R_COPY_IF(4, NCP, CKT, CST, P0)           \
        C2R_MFMA_HALF(AS, BS, H, 2, 2);             \
        C2R_COPY_IF(5, NCP, CKT, CST, P0)           \
        C2R_MFMA_HALF(AS, BS, H, 3, 0);             \
        C2R_COPY_IF(6, NCP, CKT, CST, P0)           \
        C2R_MFMA_HALF(AS, BS, H, 3, 2);             \
        C2R_COPY_IF(7, NCP, CKT, CST, P0)           \
        __builtin_amdgcn_sched_barrier(0);          \
    } while (0)

    // One 64-wide slice = four k-steps.  The hand-over barrier sits before the LAST k-step:
    // by then the copy of the next slice has landed and every wave has finished reading this
    // slice's stages.  After it, the A tile of the slice after next starts going into the A
    // stage just handed over (the wave's 4 A pieces in the last k-step, one after every second
    // MFMA: as early as the stage allows, they have one slice to land in), and the first
    // fragments of the next slice are read while the last k-step's MFMAs run, so the MFMA
    // stream never starts a slice by waiting on LDS.  The B tile of the slice after next goes
    // into the ring slot that the slice BEFORE this one used, free since the previous
    // hand-over (the wave's 4 B pieces in one of the first three k-steps).
    // `steady` (a compile-time flag): kt + 3 < nk, i.e. both following slices exist and neither
    // is the last, so every copy is unconditional and unclamped: the instruction stream
    // between the MFMAs is what limits a wave that has a SIMD nearly to itself.
    auto slice_step = [&](int kt, unsigned char *cur, unsigned char *nxt, auto steady) {
        constexpr bool STEADY = decltype(steady)::value;
        static_assert(GA == 4 && GB == 4, "pieces 0..3 are the wave's A groups, 4..7 its B groups");
        const bool c1 = STEADY || kt + 1 < nk;
        const int nb = STEADY || kt + 2 < nk ? GB : 0;  // B pieces of slice kt+2, before the hand-over
        const int na = nb ? GA : 0;                      // A pieces of slice kt+2, after the hand-over
        if (active) {
            // (the first reads of a slice go out after its first two MFMAs: the compiler's wait
            // at the top of the loop body covers every LDS read in flight, and there the only
            // ones in flight should be those the first MFMAs need anyway)
            // (the B pieces have two slices to land in, so their place is free: measured, the
            // down pass likes them in the third k-step - away from the A pieces, which follow
            // the hand-over - by 2-3 %, the gate/up pass in the first by 1 %)
            constexpr int BSTEP = MODE == 1 ? 2 : 0;
            C2R_KSTEP(0, 0, 0, kt + 2, bwr, GA, (BSTEP == 0 ? nb : 0), read_a(cur, 0, 1, 1));
            read_a(cur, 1, 0, 0);
            read_b(bcur, 1, 1);
            C2R_KSTEP(1, 0, 1, kt + 2, bwr, GA, (BSTEP == 1 ? nb : 0), (void)0);
            read_a(cur, 1, 1, 1);
            C2R_KSTEP(0, 1, 0, kt + 2, bwr, GA, (BSTEP == 2 ? nb : 0), (void)0);
        } else if (nb) {
            copy_piece(kt + 2, bwr, 4, STEADY);
            copy_piece(kt + 2, bwr, 5, STEADY);
            copy_piece(kt + 2, bwr, 6, STEADY);
            copy_piece(kt + 2, bwr, 7, STEADY);
        }
        // my copies of slice kt+1 (A: issued after the previous hand-over, B: a slice earlier
        // still) have landed once at most the B pieces of slice kt+2 are outstanding; my reads of
        // this slice's stages have returned
        if (nb)
            wait_copies_but_and_lds<GB>();
        else
            wait_copies_and_lds();
        lds_barrier();
        if (active) {
            if (c1) {
                read_a(nxt, 0, 0, 0);
                read_b(bnxt, 0, 0);
            }
            C2R_KSTEP(1, 1, 1, kt + 2, cur, 0, na, (void)0);
        } else if (na) {
            copy_piece(kt + 2, cur, 0, STEADY);
            copy_piece(kt + 2, cur, 1, STEADY);
            copy_piece(kt + 2, cur, 2, STEADY);
            copy_piece(kt + 2, cur, 3, STEADY);
        }
        unsigned char *const freed = bcur;  // every wave has read it: the slot of slice kt+3
        bcur = bnxt;
        bnxt = bwr;
        bwr = freed;
    };

    if (tiny_tile) {
        // ---- tiny tile: four-stage ring, three slices in flight, one barrier per slice ----
        static_assert(GB == 4, "five copies per wave per slice below");
        auto tiny_copy = [&](int kt) {
            unsigned char *stage = smem + (kt & (T_NSTAGE - 1)) * T_STAGE_BYTES;
            const uint32_t kb = (uint32_t)kt * ROWB;
            copy16_to_lds(baseA + kb, offA[0], stage + wave * 1024);
            const bool last = ktail && kt == nk - 1;
            const bool clamp0 = last && kt * BK + chunkc[0] * 8 >= Kdim, clamp1 = last && kt * BK + chunkc[1] * 8 >= Kdim;
            unsigned char *sb = stage + T_A_BYTES + wave * GB * 1024;
            copy16_to_lds(baseB, clamp0 ? rowB[0] : offB[0] + kb, sb);
            copy16_to_lds(baseB, clamp1 ? rowB[1] : offB[1] + kb, sb + 1024);
            copy16_to_lds(baseB, clamp0 ? rowB[2] : offB[2] + kb, sb + 2048);
            copy16_to_lds(baseB, clamp1 ? rowB[3] : offB[3] + kb, sb + 3072);
        };
        const int nf = (rows + 15) >> 4;  // 1..4 fragments of 16 rows hold rows of the group
        tiny_copy(0);
        if (nk > 1) tiny_copy(1);
        if (nk > 2) tiny_copy(2);
        for (int kt = 0; kt < nk; ++kt) {
            // slice kt has landed once at most the copies of slices kt+1 and kt+2 are outstanding
            if (kt + 2 < nk)
                wait_copies_but_and_lds<10>();
            else if (kt + 1 < nk)
                wait_copies_but_and_lds<5>();
            else
                wait_copies_but_and_lds<0>();
            lds_barrier();  // every wave's reads of slice kt-1 have returned: its stage is free
            if (kt + 3 < nk) tiny_copy(kt + 3);
            if (wm == 0 && cols_exist) {
                const unsigned char *stage = smem + (kt & (T_NSTAGE - 1)) * T_STAGE_BYTES;
#pragma unroll
                for (int kq = 0; kq < 2; ++kq) {
                    read_b(stage, kq, 0);
                    read_a_first(stage, kq, 0, 0, nf);
                    C2R_MFMA_ROW(0, 0, 0, 0);
                    if (nf > 1) { C2R_MFMA_ROW(0, 0, 0, 1); }
                    if (nf > 2) { C2R_MFMA_ROW(0, 0, 0, 2); }
                    if (nf > 3) { C2R_MFMA_ROW(0, 0, 0, 3); }
                }
            }
        }
    } else if (short_tile) {
        // ---- short tile: three-stage ring, two slices in flight, one barrier per slice ----
        static_assert(L_GA == 2 && GB == 4, "six copies per wave per slice below");
        auto short_copy = [&](int kt) {
            unsigned char *stage = smem + (kt % L_NSTAGE) * L_STAGE_BYTES;
            const uint32_t kb = (uint32_t)kt * ROWB;
            copy16_to_lds(baseA + kb, offA[0], stage + (wave * L_GA + 0) * 1024);
            copy16_to_lds(baseA + kb, offA[1], stage + (wave * L_GA + 1) * 1024);
            const bool last = ktail && kt == nk - 1;
            const bool clamp0 = last && kt * BK + chunkc[0] * 8 >= Kdim, clamp1 = last && kt * BK + chunkc[1] * 8 >= Kdim;
            unsigned char *sb = stage + L_A_BYTES + wave * GB * 1024;  // wave * GB is even: groups alternate parity
            copy16_to_lds(baseB, clamp0 ? rowB[0] : offB[0] + kb, sb);
            copy16_to_lds(baseB, clamp1 ? rowB[1] : offB[1] + kb, sb + 1024);
            copy16_to_lds(baseB, clamp0 ? rowB[2] : offB[2] + kb, sb + 2048);
            copy16_to_lds(baseB, clamp1 ? rowB[3] : offB[3] + kb, sb + 3072);
        };
        // Only the 16-row fragments that hold rows of the group are computed: most short tiles
        // belong to experts with a handful of tokens, the chip is power limited, and matrix
        // instructions on padding rows cost the other workgroups clock.
        const int nf = (rows + 15) >> 4;  // 1..8, workgroup-uniform
        short_copy(0);
        if (nk > 1) short_copy(1);
        for (int kt = 0; kt < nk; ++kt) {
            // slice kt has landed once at most the copies of slice kt+1 are outstanding; every
            // wave's reads of slice kt-1 have returned, so its stage may be refilled
            if (kt + 1 < nk)
                wait_copies_but_and_lds<6>();
            else
                wait_copies_but_and_lds<0>();
            lds_barrier();
            if (kt + 2 < nk) short_copy(kt + 2);
            if (wm == 0 && cols_exist) {
                const unsigned char *stage = smem + (kt % L_NSTAGE) * L_STAGE_BYTES;
#pragma unroll
                for (int kq = 0; kq < 2; ++kq) {
                    read_b(stage, kq, 0);
                    read_a_first(stage, kq, 0, 0, nf);
                    C2R_MFMA_ROW(0, 0, 0, 0);
                    if (nf > 1) { C2R_MFMA_ROW(0, 0, 0, 1); }
                    if (nf > 2) { C2R_MFMA_ROW(0, 0, 0, 2); }
                    if (nf > 3) { C2R_MFMA_ROW(0, 0, 0, 3); }
                    if (nf > 4) {
                        read_a_first(stage, kq, 1, 1, nf - 4);
                        C2R_MFMA_ROW(1, 0, 1, 0);
                        if (nf > 5) { C2R_MFMA_ROW(1, 0, 1, 1); }
                        if (nf > 6) { C2R_MFMA_ROW(1, 0, 1, 2); }
                        if (nf > 7) { C2R_MFMA_ROW(1, 0, 1, 3); }
                    }
                }
            }
        }
    } else {
        copy_piece(0, st0, 0);
        copy_piece(0, st0, 1);
        copy_piece(0, st0, 2);
        copy_piece(0, st0, 3);
        copy_piece(0, bcur, 4);
        copy_piece(0, bcur, 5);
        copy_piece(0, bcur, 6);
        copy_piece(0, bcur, 7);
        // every stage is free at the start of a tile: slice 1 goes out right behind slice 0
        if (nk > 1) {
            copy_piece(1, st1, 0);
            copy_piece(1, st1, 1);
            copy_piece(1, st1, 2);
            copy_piece(1, st1, 3);
            copy_piece(1, bnxt, 4);
            copy_piece(1, bnxt, 5);
            copy_piece(1, bnxt, 6);
            copy_piece(1, bnxt, 7);
            wait_copies_but<8>();  // slice 0 has landed
        } else {
            wait_copies_but<0>();
        }
        lds_barrier();
        if (active) {
            read_a(st0, 0, 0, 0);
            read_b(bcur, 0, 0);
        }
        int kt = 0;
        for (; kt + 4 < nk; kt += 2) {  // both slices of the pair are followed by two inner slices
            slice_step(kt, st0, st1, std::true_type{});
            slice_step(kt + 1, st1, st0, std::true_type{});
        }
        for (; kt < nk; kt += 2) {
            slice_step(kt, st0, st1, std::false_type{});
            if (kt + 1 >= nk) break;
            slice_step(kt + 1, st1, st0, std::false_type{});
        }
        wait_copies_but<0>();
    }
#undef C2R_KSTEP
#undef C2R_COPY_IF
#undef C2R_MFMA_ROW
#undef C2R_MFMA

    before_epilogue();
    // ---- epilogue.  Fragment (i, j) holds C^T: lane (fr, fq), register v is
    //      row m = i*16 + fr, column n = j*16 + 4*fq + v.  Every wave of the workgroup is
    //      here at once with the matrix pipe idle, so the common case (all of the tile's
    //      columns exist) is kept short: hardware bf16 conversion, no per-element guards, and
    //      whole rows per store instruction (measured: routed down pass 227 -> 210 us against
    //      8-byte stores straight from the fragments). ----
    constexpr int FJ = MODE == 0 ? FN16 / 2 : FN16;
    const int col0 = n0 + (MODE == 0 ? wn * (TN / 2) : wn * TN);
    if (n0 + BNF <= N) {
        // The wave's 128 x (FJ*16) results go through a private piece of the (now idle) stage
        // memory so that they leave as whole rows: a lane's 8-byte fragment pieces would be
        // 16 separate 32-byte requests per store instruction, the rows read back are 8 (or
        // 4) lanes x 16 bytes = one contiguous 128 (64) bytes each.
        constexpr int ROW_BYTES = FJ * 16 * 2, PITCH = ROW_BYTES + 16;
        constexpr int LPR = ROW_BYTES / 16, RPI = 64 / LPR;  // lanes per row, rows per store instruction
        static_assert(NW * TM * PITCH <= SMEM_BYTES, "staging fits the stage memory");
        if (short_tile) {  // the ring may still be read by a slower wave
            wait_copies_but_and_lds<0>();
            lds_barrier();
        }
        unsigned char *stg = smem + wave * (TM * PITCH);
        const int rlim = rows - wm * TM;  // rows of this wave's M range that exist
#pragma unroll
        for (int i = 0; i < FM16; ++i) {
            if (i * 16 < rlim) {  // wave-uniform: skip fragment rows wholly past the end
#pragma unroll
                for (int j = 0; j < FJ; ++j) {
                    float v4[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        v4[u] = MODE == 0 ? silu_mul(acc[i][j][u], acc[i][j + FN16 / 2][u]) : acc[i][j][u];
                    *reinterpret_cast<uint2 *>(stg + (i * 16 + fr) * PITCH + (j * 16 + fq * 4) * 2) =
                        make_uint2(pack_bf16x2(v4[0], v4[1]), pack_bf16x2(v4[2], v4[3]));
                }
            }
        }
        const int srow = lane / LPR, chunk = lane % LPR;
        uint16_t *o = out + ((size_t)g.row_begin + wm * TM + srow) * ldo + col0 + chunk * 8;
#pragma unroll
        for (int r0 = 0; r0 < TM; r0 += RPI) {
            if (r0 + srow < rlim)
                *reinterpret_cast<uint4 *>(o) = *reinterpret_cast<const uint4 *>(stg + (r0 + srow) * PITCH + chunk * 16);
            o += (size_t)RPI * ldo;
        }
        return;
    }
    uint16_t *outb = out + (size_t)g.row_begin * ldo;
#pragma unroll
    for (int i = 0; i < FM16; ++i) {
        const int r = wm * TM + i * 16 + fr;
        if (r >= rows) continue;
#pragma unroll
        for (int j = 0; j < FJ; ++j) {
            const int col = col0 + j * 16 + fq * 4;
            uint2 pk = make_uint2(0, 0);
            if (col >= N) {
                // pass 0 keeps the padding columns of h at zero for pass 1's k tail
                if (col < zero_to) *reinterpret_cast<uint2 *>(outb + (size_t)r * ldo + col) = pk;
                continue;
            }
            float v4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v4[u] = MODE == 0 ? silu_mul(acc[i][j][u], acc[i][j + FN16 / 2][u]) : acc[i][j][u];
            pk.x = pack_bf16x2(v4[0], v4[1]);
            pk.y = pack_bf16x2(v4[2], v4[3]);
            *reinterpret_cast<uint2 *>(outb + (size_t)r * ldo + col) = pk;
        }
    }
}

// Work queues of the launches in flight: per launch one set of 8 ticket counters (one per XCD)
// and a count of the workgroups that have left.  All zero between launches: the last workgroup
// to leave a launch clears the set it used.  The host hands the sets out round-robin, so up to
// FFN_QUEUE_SETS launches of this kernel may be in flight on a GPU at once (on any streams).
constexpr int FFN_QUEUE_SETS = 64, FFN_QUEUE_INTS = 16;
__device__ int ffn_queues[FFN_QUEUE_SETS * FFN_QUEUE_INTS];

// The kernel: one workgroup per CU, each pulling tiles until none are left.  The hardware hands
// workgroups out strictly in order, the k-th of an XCD to shader engine k mod 4 - measured: a CU
// freed early by a short tile stayed empty for 100 us behind a workgroup that waited for a CU
// of ANOTHER engine - so with one workgroup per tile every tile shorter than its neighbours
// left a bubble, and the ragged groups' tiles differ by a factor of six.  Here the list of an
// XCD (ffn_common.h) is a queue: a ticket counter in device memory that the workgroups of that
// XCD draw from (the L2 locality of the list is kept), and a workgroup whose own XCD has
// nothing left draws from the others'.
template <int MODE, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64) void ffn_bf16_dma_kernel(const FfnLaunch L, int *__restrict__ queues) {
    typedef FfnShape<WM, WN> S;
    static_assert(S::SMEM_BYTES <= 160 * 1024, "one workgroup per CU owns all of its LDS");
    __shared__ __attribute__((aligned(1024))) unsigned char smem[S::SMEM_BYTES];
    // The claimed position (XCD of the list, slot; -1: nothing left) is handed to the waves in
    // the last bytes of the stage memory, which is all of the CU's LDS: every layout of a tile
    // writes them only after its first hand-over barrier (the third weight stage of a full
    // tile, the fourth ring stage of a tiny one; a short tile never does), and no wave gets
    // there before every wave has read the claim.
    int *const claim = reinterpret_cast<int *>(smem + S::SMEM_BYTES - 64);
    const int tid = threadIdx.x, lane = tid & 63;
    const int home = (int)(blockIdx.x & 7);
    // every wave keeps the row range of "its lane's" expert of the ragged problem (the tile
    // lookup is wave-wide arithmetic on them; they do not change during the launch)
    int grp_lo = 0, grp_hi = 0;
    if (L.has_ragged) load_group_range(L.p[0].offsets, L.p[0].E_local, L.p[0].A_cap, grp_lo, grp_hi);
    // ... and the single group's row range (two scalars)
    int sg_lo = 0, sg_hi = 0;
    if (L.has_single) {
        sg_lo = L.p[1].offsets ? L.p[1].offsets[0] : L.p[1].row_lo;
        sg_hi = L.p[1].offsets ? L.p[1].offsets[1] : L.p[1].row_hi;
        sg_lo = sg_lo < 0 ? 0 : (sg_lo > L.p[1].A_cap ? L.p[1].A_cap : sg_lo);
        sg_hi = sg_hi < sg_lo ? sg_lo : (sg_hi > L.p[1].A_cap ? L.p[1].A_cap : sg_hi);
        sg_lo = __builtin_amdgcn_readfirstlane(sg_lo);
        sg_hi = __builtin_amdgcn_readfirstlane(sg_hi);
    }
    // the first wave works the queues; its lane x < 8 keeps the number of slots of XCD x's list
    int my_len = 0;
    if (tid < 64) {
        const int n_s = (sg_hi - sg_lo + S::BM - 1) / S::BM * (L.has_single ? L.p[1].ntn : 0);
        int totA = 0, totB = 0;
        if (L.has_ragged) {
            const RaggedMap m = ragged_map_of<S::BM>(grp_lo, grp_hi);
            totA = m.totalA * L.p[0].ntn;
            totB = m.totalB * L.p[0].ntn;
        }
        const int x = lane & 7;
        my_len = xcd_list_slots(equal_range(n_s, x).cnt + equal_range(totA, x).cnt + equal_range(totB, x).cnt);
    }
    int q = home;        // the queue this workgroup draws from: its own XCD's until that is empty
    // The first position of every workgroup is its own number in its XCD (no trip to the counter
    // before the first tile); the counters hand out what lies beyond those.
    int ticket = (int)(blockIdx.x >> 3);  // (lane 0 of the first wave) a ticket of queue q drawn ahead
    bool drawn = true;                    // such a ticket is at hand
    for (;;) {
        if (tid < 64) {
            // Every trip ends by checking the ticket it holds, so no valid ticket is ever dropped.
            // A ticket that comes back past the end of its list (another workgroup was faster) makes
            // that list look empty from then on, so at most one draw per list fails: 9 trips at most.
            int t = -1;
            bool have = drawn;  // the ticket drawn during the last epilogue, or the static first one
            drawn = false;
            for (int tries = 0; tries < 16; ++tries) {
                if (!have) {
                    // Look before drawing: one coherent read of the eight counters tells which lists
                    // still hold something (counters only grow, so "empty" is final), and a workgroup
                    // that finds them all empty leaves at once - drawing from eight empty queues one
                    // after the other cost 15 us at the end of every launch.
                    const int x = lane & 7;
                    const int seen = __hip_atomic_load(&queues[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) +
                                     (((int)gridDim.x - x + 7) >> 3);
                    const uint32_t avail = (uint32_t)__ballot(lane < 8 && seen < my_len) & 0xffu;
                    if (avail == 0) break;  // (t is -1)
                    // own XCD's list first, then the next one (cyclically) that holds something
                    const uint32_t rot = ((avail >> q) | (avail << (8 - q))) & 0xffu;
                    q = (q + __builtin_ctz(rot)) & 7;
                    if (lane == 0) ticket = atomicAdd(&queues[q], 1) + (((int)gridDim.x - q + 7) >> 3);
                }
                have = false;
                t = __builtin_amdgcn_readfirstlane(ticket);
                if (t < __builtin_amdgcn_readlane(my_len, q)) break;
                t = -1;
            }
            if (lane == 0) {
                claim[0] = q;
                claim[1] = t;
            }
        }
        wait_lds_only();
        lds_barrier();  // the claim is visible
        q = __builtin_amdgcn_readfirstlane(claim[0]);
        const int slot = __builtin_amdgcn_readfirstlane(claim[1]);
        if (slot < 0) break;  // every queue is empty
        // The launch arguments are re-read per tile through a pointer the compiler cannot see
        // through: held in registers across the tile they are ~50 scalars too many.
        // (L is the kernel's first argument: it sits at the start of the kernel-argument segment)
        FfnLaunchArgs Lp = (FfnLaunchArgs)__builtin_amdgcn_kernarg_segment_ptr();
        asm volatile("" : "+s"(Lp));
        drawn = false;
        ffn_tile<MODE, WM, WN>(Lp, smem, q, slot, grp_lo, grp_hi, sg_lo, sg_hi, [&]() {
            // the next ticket of the same queue, drawn while the epilogue runs
            if (tid == 0) ticket = atomicAdd(&queues[q], 1) + (((int)gridDim.x - q + 7) >> 3);
            drawn = true;
        });
        // This wave's LDS reads have returned; then every wave's: the next claim and the next tile's
        // copies may overwrite the stages.  The epilogue's stores are NOT waited for (a workgroup
        // that ends does not wait for its stores either): they drain while the next tile is looked
        // up and its first slices are requested.  The copy waits of the next tile stay correct with
        // stores in flight: they ask for "at most N operations outstanding", copies complete in
        // order among themselves, so older stores still in flight only make a wait longer.
        wait_lds_only();
        lds_barrier();
    }
    // the last workgroup to leave clears the set for the launch that gets it next
    // (this workgroup's draws have all returned - their values were used - so they precede the
    // count below; no fence: a device-scope release would write the XCD's whole L2 back)
    if (tid == 0) {
        if (atomicAdd(&queues[8], 1) == (int)gridDim.x - 1) {
            for (int i = 0; i < 9; ++i) atomicExch(&queues[i], 0);
        }
    }
}

// One problem of a pass.  pass 0: a = x_perm [A_cap, d] (d % 64 == 0) or, with gather, x [T, d];
// out = h with row pitch ldo >= F, columns [F, ldo) zeroed.  pass 1: a = h (pitch lda, zero
// padded to 64), out = y_perm.  offsets == nullptr: one group, rows [0, A_cap).
FfnProblem ffn_bf16_dma_problem(int pass, const uint16_t *a, int lda, const int32_t *offsets, int E_local,
                                int64_t A_cap, int d, int F, const uint16_t *b0, const uint16_t *b1, uint16_t *out,
                                int ldo, const int32_t *gather, int gather_div, int gather_rows) {
    constexpr int BN = 256;
    FfnProblem P;
    P.A = a;
    P.offsets = offsets;
    P.B0 = b0;
    P.B1 = pass == 0 ? b1 : nullptr;
    P.out = out;
    P.gather = pass == 0 ? gather : nullptr;
    P.lda = lda;
    P.E_local = E_local;
    P.A_cap = (int)A_cap;
    P.N = pass == 0 ? F : d;
    P.Kdim = pass == 0 ? d : F;
    P.ldo = ldo;
    P.ntn = pass == 0 ? (ldo + BN / 2 - 1) / (BN / 2) : (d + BN - 1) / BN;
    P.zero_to = pass == 0 ? ldo : 0;
    P.gather_div = pass == 0 ? gather_div : 1;
    P.gather_rows = pass == 0 ? gather_rows : 1;
    P.row_lo = 0;
    P.row_hi = (int)A_cap;
    return P;
}

// Launches one pass over one problem (second == nullptr) or over two in ONE grid: the second
// must be a single group (E_local == 1).
int launch_ffn_bf16_dma(int pass, const FfnProblem &first, const FfnProblem *second, hipStream_t st) {
    drop_stale_error();
    constexpr int BM = 256, WM = 2, WN = 4;
    if (second && second->E_local != 1) return C2R_ERR_INVALID_ARG;
    // the kernel expects the ragged problem (more than one group) in p[0], a single group in p[1]
    FfnLaunch L;
    const FfnProblem *single = second ? second : (first.E_local == 1 ? &first : nullptr);
    const FfnProblem *ragged = first.E_local != 1 ? &first : nullptr;
    if (second && !ragged) return C2R_ERR_INVALID_ARG;  // (two single groups: launch them one by one)
    L.p[0] = ragged ? *ragged : *single;
    L.p[1] = single ? *single : *ragged;
    L.has_ragged = ragged ? 1 : 0;
    L.has_single = single ? 1 : 0;
    // one workgroup per CU (fewer if the bound on the tiles is smaller), whatever the number of tiles
    int64_t tiles = 0;
    if (ragged)
        tiles += 8 * ragged_per_xcd_bound(((int64_t)ragged->A_cap + BM - 1) / BM + ragged->E_local, ragged->E_local,
                                          ragged->ntn);
    if (single) tiles += 8 * single_per_xcd_bound(((int64_t)single->A_cap + BM - 1) / BM + 1, single->ntn);
    tiles += 8 * CUS_PER_XCD;  // (row parts of the last rounds)
    const int64_t grid = tiles < 8 * CUS_PER_XCD ? tiles : 8 * CUS_PER_XCD;
    static std::atomic<unsigned> next_set{0};
    static std::atomic<int *> queue_base[64];  // per device: the address of that device's copy of ffn_queues
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return C2R_ERR_LAUNCH;
    int *base = queue_base[dev].load();
    if (!base) {  // (in host code the array's name is only a handle for this query)
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(ffn_queues)) != hipSuccess || !p) return C2R_ERR_LAUNCH;
        base = static_cast<int *>(p);
        queue_base[dev].store(base);
    }
    int *queues = base + (next_set.fetch_add(1) % FFN_QUEUE_SETS) * FFN_QUEUE_INTS;
    const dim3 g((unsigned)grid), b(WM * WN * 64);
    if (pass == 0)
        ffn_bf16_dma_kernel<0, WM, WN><<<g, b, 0, st>>>(L, queues);
    else
        ffn_bf16_dma_kernel<1, WM, WN><<<g, b, 0, st>>>(L, queues);
    return launch_status();
}

int launch_ffn_bf16_dma_pass(int pass, const uint16_t *a, int lda, const int32_t *offsets, int E_local,
                             int64_t A_cap, int d, int F, const uint16_t *b0, const uint16_t *b1,
                             uint16_t *out, int ldo, const int32_t *gather, int gather_div, int gather_rows,
                             hipStream_t st) {
    const FfnProblem P = ffn_bf16_dma_problem(pass, a, lda, offsets, E_local, A_cap, d, F, b0, b1, out, ldo, gather,
                                              gather_div, gather_rows);
    return launch_ffn_bf16_dma(pass, P, nullptr, st);
}

}  // namespace c2r
