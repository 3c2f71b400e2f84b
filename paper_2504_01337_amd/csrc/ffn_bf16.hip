// Grouped SwiGLU expert FFN in bf16 on the CDNA4 matrix cores.
//
// Two GEMM passes over the ragged expert groups, both "NT" (A and B rows are
// contiguous along the contraction index, which is what the MFMA operand
// layout wants: each lane supplies 8 consecutive k of one row):
//   pass 0: h[r, f] = silu(x[r,:] . w_gate[e,f,:]) * (x[r,:] . w_up[e,f,:])   K = d
//   pass 1: y[r, j] = h[r,:] . w_down[e,j,:]                                    K = F
// In pass 0 a workgroup's B tile holds BN/2 gate rows followed by the BN/2 up rows
// of the same f range, and every wave owns matching gate / up fragments, so the
// SwiGLU product is formed in registers and only h (bf16) is written.
//
// Tiling: WM x WN waves per workgroup (two per SIMD, so one wave's loads and address
// arithmetic overlap the other's MFMAs); v_mfma_f32_32x32x16_bf16; a BM x BN x BK
// tile per step, double buffered in LDS with 16-byte chunks XOR-swizzled by row so
// that both the staging writes and the fragment reads are bank-conflict free.
// Global loads for step k+1 are issued before the MFMAs of step k.
// Workgroup -> tile: M-tiles are enumerated over the non-empty experts from the
// device-side offsets (no host sync); tile numbers are dealt to the 8 XCDs in
// contiguous ranges so that workgroups sharing an A or B panel share an L2.
#include "ffn_common.h"

namespace c2r {

template <int MODE, int BM, int BN, int BK, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64) void ffn_bf16_kernel(const uint16_t *__restrict__ A, int lda,
                                                       const int32_t *__restrict__ offsets,
                                                       int E_local, int A_cap, int N, int Kdim,
                                                       const uint16_t *__restrict__ B0,
                                                       const uint16_t *__restrict__ B1,
                                                       uint16_t *__restrict__ out, int ldo, int ntn) {
    constexpr int NT = WM * WN * 64;  // threads per workgroup
    constexpr int TM = BM / WM, TN = BN / WN;  // wave tile
    constexpr int FM = TM / 32, FN = TN / 32;  // 32x32 fragments per wave
    constexpr int CPR = BK / 8;                // 16-byte chunks per tile row
    constexpr int ROWB = BK * 2;               // bytes per tile row
    constexpr int NA = BM * CPR / NT, NB = BN * CPR / NT;
    constexpr int RSTEP = NT / CPR;            // tile rows covered by one pass of the loader
    static_assert(CPR == 8 && RSTEP % 16 == 0, "swizzle key uses row bits 0..3");
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    constexpr int BNF = MODE == 0 ? BN / 2 : BN;  // output columns per tile
    static_assert(MODE == 1 || FN % 2 == 0, "gate/up fragments pair up");
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * (A_BYTES + B_BYTES)];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- which tile ----
    const GroupMap gmap = build_group_map<BM>(offsets, E_local, A_cap);
    const TileId tl = xcd_grouped_tile<false>(gmap.total_mtiles, ntn);
    if (!tl.valid) return;
    const int nt = tl.nt;
    const GroupTile g = locate_group_tile(gmap, tl.mt, BM);
    if (g.expert < 0) return;
    const int n0 = nt * BNF;
    const int rows = g.row_end - g.row_begin;  // >= 1; may exceed BM

    // ---- loader roles ----
    const int lc = tid % CPR, lr = tid / CPR;
    const unsigned char *baseA = reinterpret_cast<const unsigned char *>(A + (size_t)g.row_begin * lda);
    const unsigned char *baseB0 = reinterpret_cast<const unsigned char *>(B0 + (size_t)g.expert * N * Kdim);
    const unsigned char *baseB1 = MODE == 0 ? reinterpret_cast<const unsigned char *>(B1 + (size_t)g.expert * N * Kdim) : nullptr;
    uint32_t offA[NA], offB[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        int r = lr + RSTEP * i;
        r = r < rows ? r : rows - 1;
        offA[i] = (uint32_t)r * (uint32_t)lda * 2u + lc * 16u;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        int r = lr + RSTEP * i;
        if (MODE == 0 && r >= BN / 2) r -= BN / 2;
        int c = n0 + r;
        c = c < N ? c : N - 1;
        offB[i] = (uint32_t)c * (uint32_t)Kdim * 2u + lc * 16u;
    }
    const uint32_t lds_w = (uint32_t)lr * ROWB + ((lc ^ swz_key(lr)) * 16u);

    uint4 ra[NA], rb[NB];
    auto gload = [&](int k0) {
        const bool in = k0 + lc * 8 < Kdim;
#pragma unroll
        for (int i = 0; i < NA; ++i)
            ra[i] = in ? *reinterpret_cast<const uint4 *>(baseA + offA[i] + (size_t)k0 * 2) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const unsigned char *bb = (MODE == 0 && lr + RSTEP * i >= BN / 2) ? baseB1 : baseB0;
            rb[i] = in ? *reinterpret_cast<const uint4 *>(bb + offB[i] + (size_t)k0 * 2) : make_uint4(0, 0, 0, 0);
        }
    };
    auto lstore = [&](int s) {
        unsigned char *sa = smem + s * (A_BYTES + B_BYTES);
        unsigned char *sb = sa + A_BYTES;
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<uint4 *>(sa + lds_w + i * RSTEP * ROWB) = ra[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) *reinterpret_cast<uint4 *>(sb + lds_w + i * RSTEP * ROWB) = rb[i];
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // fragment read addresses (row part); rows are multiples of 32 plus lane%32, so the key is the lane's
    const int fr = lane & 31, fh = lane >> 5;
    uint32_t rdA[FM], rdB[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) rdA[i] = (uint32_t)(wm * TM + i * 32 + fr) * ROWB;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        int r;
        if (MODE == 0)
            r = (j < FN / 2) ? wn * (TN / 2) + j * 32 : BN / 2 + wn * (TN / 2) + (j - FN / 2) * 32;
        else
            r = wn * TN + j * 32;
        rdB[j] = (uint32_t)(r + fr) * ROWB;
    }
    const int sw = swz_key(fr);
    // rows of this wave's M range that exist (wave-uniform): fragments past the group's
    // end are never multiplied
    const int wrows = __builtin_amdgcn_readfirstlane(rows - wm * TM);

    constexpr int NKK = BK / 16;
    bf16x8 af[2][FM], bfr[2][FN];
    auto read_frags = [&](const unsigned char *sa, const unsigned char *sb, int kk, int set) {
        const uint32_t ch = (uint32_t)(((kk * 2 + fh) ^ sw) * 16);
#pragma unroll
        for (int i = 0; i < FM; ++i) af[set][i] = *reinterpret_cast<const bf16x8 *>(sa + rdA[i] + ch);
#pragma unroll
        for (int j = 0; j < FN; ++j) bfr[set][j] = *reinterpret_cast<const bf16x8 *>(sb + rdB[j] + ch);
    };

    const int nk = (Kdim + BK - 1) / BK;
    gload(0);
    lstore(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const unsigned char *sa = smem + cur * (A_BYTES + B_BYTES);
        const unsigned char *sb = sa + A_BYTES;
        read_frags(sa, sb, 0, 0);
        if (kt + 1 < nk) gload((kt + 1) * BK);
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            // fetch the next k-slice's fragments before this slice's MFMAs are issued
            if (kk + 1 < NKK) read_frags(sa, sb, kk + 1, (kk + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                if (i * 32 < wrows) {
#pragma unroll
                    for (int j = 0; j < FN; ++j)  // operands swapped: the lane's 4-element runs lie along n
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i],
                                                                            acc[i][j], 0, 0, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (kt + 1 < nk) lstore(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue.  Fragment (i, j) holds C^T: lane (fr, fh), register v is
    //      row m = i*32 + fr, column n = j*32 + 8*(v/4) + 4*fh + v%4  -> 8-byte stores ----
    uint16_t *outb = out + (size_t)g.row_begin * ldo;
    constexpr int FJ = MODE == 0 ? FN / 2 : FN;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int r = wm * TM + i * 32 + fr;
        if (r >= rows) continue;
#pragma unroll
        for (int j = 0; j < FJ; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = n0 + (MODE == 0 ? wn * (TN / 2) : wn * TN) + j * 32 + q * 8 + fh * 4;
                if (col >= N) continue;  // N and col are multiples of 4
                float v4[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (MODE == 0)
                        v4[u] = silu_mul(acc[i][j][q * 4 + u], acc[i][j + FN / 2][q * 4 + u]);
                    else
                        v4[u] = acc[i][j][q * 4 + u];
                }
                uint2 pk;
                pk.x = pack_bf16x2(v4[0], v4[1]);
                pk.y = pack_bf16x2(v4[2], v4[3]);
                *reinterpret_cast<uint2 *>(outb + (size_t)r * ldo + col) = pk;
            }
        }
    }
}

template <int BM, int BN, int BK, int WM, int WN>
static int launch_cfg(int pass, const uint16_t *a, const int32_t *offsets, int E_local, int64_t A_cap, int d,
                      int F, const uint16_t *b0, const uint16_t *b1, uint16_t *out, hipStream_t st) {
    drop_stale_error();
    const int64_t mtiles = (A_cap + BM - 1) / BM + E_local;
    const int ntn = pass == 0 ? (F + BN / 2 - 1) / (BN / 2) : (d + BN - 1) / BN;
    const int64_t grid = xcd_grouped_grid(mtiles, ntn, false);
    if (grid >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    if (pass == 0)
        ffn_bf16_kernel<0, BM, BN, BK, WM, WN><<<dim3((unsigned)grid), dim3(WM * WN * 64), 0, st>>>(
            a, d, offsets, E_local, (int)A_cap, F, d, b0, b1, out, F, ntn);
    else
        ffn_bf16_kernel<1, BM, BN, BK, WM, WN><<<dim3((unsigned)grid), dim3(WM * WN * 64), 0, st>>>(
            a, F, offsets, E_local, (int)A_cap, d, F, b0, nullptr, out, d, ntn);
    return launch_status();
}

int launch_ffn_bf16_pass(int pass, const uint16_t *a, const int32_t *offsets, int E_local, int64_t A_cap, int d,
                         int F, const uint16_t *b0, const uint16_t *b1, uint16_t *out, hipStream_t st) {
    return launch_cfg<256, 256, 64, 2, 4>(pass, a, offsets, E_local, A_cap, d, F, b0, b1, out, st);
}

}  // namespace c2r
