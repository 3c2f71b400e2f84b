// Grouped SwiGLU expert FFN in fp32 (vector FMA, LDS tiled): the small-shape /
// full-precision path.  Same ragged-group tiling as the bf16 MFMA path.
//   mode 0: h[r, f]  = silu(x[r,:] . w_gate[e,f,:]) * (x[r,:] . w_up[e,f,:])
//   mode 1: y[r, j]  = h[r,:] . w_down[e,j,:]
#include "ffn_common.h"

namespace c2r {

constexpr int F32_BM = 64, F32_BN = 64, F32_BK = 16;

template <int MODE>
__global__ __launch_bounds__(256) void ffn_f32_kernel(const float *__restrict__ A, int lda,
                                                      const int32_t *__restrict__ offsets, int E_local,
                                                      int A_cap, int N, int Kdim,
                                                      const float *__restrict__ B0,
                                                      const float *__restrict__ B1,
                                                      float *__restrict__ out, int ldo) {
    __shared__ float As[F32_BK][F32_BM + 4];
    __shared__ float Bs[MODE == 0 ? 2 : 1][F32_BK][F32_BN + 4];
    const int ntn = (N + F32_BN - 1) / F32_BN;
    const int mt = blockIdx.x / ntn, nt = blockIdx.x % ntn;
    const GroupMap gmap = build_group_map<F32_BM>(offsets, E_local, A_cap);
    const GroupTile g = locate_group_tile(gmap, mt, F32_BM);
    if (g.expert < 0) return;
    const int n0 = nt * F32_BN;
    const float *Bg = B0 + (size_t)g.expert * N * Kdim;
    const float *Bu = MODE == 0 ? B1 + (size_t)g.expert * N * Kdim : nullptr;

    const int tid = threadIdx.x;
    const int lr = tid >> 2, lk = (tid & 3) * 4;  // loader: row lr, k offset lk
    int arow = g.row_begin + lr;
    arow = arow < g.row_end ? arow : g.row_end - 1;
    int brow = n0 + lr;
    brow = brow < N ? brow : N - 1;
    const int ty = tid >> 4, tx = tid & 15;  // 16 x 16 threads, 4 x 4 outputs each

    float accg[4][4] = {}, accu[4][4] = {};
    for (int k0 = 0; k0 < Kdim; k0 += F32_BK) {
        float4 a = make_float4(0, 0, 0, 0), b0 = a, b1 = a;
        if (k0 + lk < Kdim) {  // Kdim is a multiple of 4
            a = *reinterpret_cast<const float4 *>(A + (size_t)arow * lda + k0 + lk);
            b0 = *reinterpret_cast<const float4 *>(Bg + (size_t)brow * Kdim + k0 + lk);
            if (MODE == 0) b1 = *reinterpret_cast<const float4 *>(Bu + (size_t)brow * Kdim + k0 + lk);
        }
        __syncthreads();
        As[lk + 0][lr] = a.x; As[lk + 1][lr] = a.y; As[lk + 2][lr] = a.z; As[lk + 3][lr] = a.w;
        Bs[0][lk + 0][lr] = b0.x; Bs[0][lk + 1][lr] = b0.y; Bs[0][lk + 2][lr] = b0.z; Bs[0][lk + 3][lr] = b0.w;
        if (MODE == 0) {
            Bs[MODE == 0 ? 1 : 0][lk + 0][lr] = b1.x; Bs[MODE == 0 ? 1 : 0][lk + 1][lr] = b1.y;
            Bs[MODE == 0 ? 1 : 0][lk + 2][lr] = b1.z; Bs[MODE == 0 ? 1 : 0][lk + 3][lr] = b1.w;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < F32_BK; ++k) {
            const float4 av = *reinterpret_cast<const float4 *>(&As[k][ty * 4]);
            const float4 gv = *reinterpret_cast<const float4 *>(&Bs[0][k][tx * 4]);
            const float ar[4] = {av.x, av.y, av.z, av.w};
            const float gr[4] = {gv.x, gv.y, gv.z, gv.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) accg[i][j] = __builtin_fmaf(ar[i], gr[j], accg[i][j]);
            if (MODE == 0) {
                const float4 uv = *reinterpret_cast<const float4 *>(&Bs[MODE == 0 ? 1 : 0][k][tx * 4]);
                const float ur[4] = {uv.x, uv.y, uv.z, uv.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) accu[i][j] = __builtin_fmaf(ar[i], ur[j], accu[i][j]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = g.row_begin + ty * 4 + i;
        if (r >= g.row_end) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = n0 + tx * 4 + j;
            if (c >= N) continue;
            float v = accg[i][j];
            if (MODE == 0) {
                const float gq = accg[i][j];
                v = gq / (1.0f + expf(-gq)) * accu[i][j];
            }
            out[(size_t)r * ldo + c] = v;
        }
    }
}

int launch_ffn_f32_pass(int pass, const float *a, const int32_t *offsets, int E_local, int64_t A_cap, int d,
                        int F, const float *b0, const float *b1, float *out, hipStream_t st) {
    drop_stale_error();
    const int64_t mtiles = (A_cap + F32_BM - 1) / F32_BM + E_local;
    const int N = pass == 0 ? F : d;
    const int64_t grid = mtiles * ((N + F32_BN - 1) / F32_BN);
    if (grid >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    if (pass == 0)
        ffn_f32_kernel<0><<<dim3((unsigned)grid), dim3(256), 0, st>>>(a, d, offsets, E_local, (int)A_cap, F, d, b0,
                                                                     b1, out, F);
    else
        ffn_f32_kernel<1><<<dim3((unsigned)grid), dim3(256), 0, st>>>(a, F, offsets, E_local, (int)A_cap, d, F, b0,
                                                                     nullptr, out, d);
    return launch_status();
}

}  // namespace c2r
