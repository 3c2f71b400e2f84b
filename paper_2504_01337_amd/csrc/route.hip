// Router logits (Eq. 1) and collaboration-constrained selection (Sec. 3.3, step 2).
//
// Two kernels.
//  route_partial_kernel: lane = token.  One wave owns 64 tokens and one 256-long
//    k-chunk; it stages x through LDS (coalesced 16-byte loads, conflict-free
//    per-lane row reads) and keeps one fp32 accumulator per expert in VGPRs.
//    The W_g row for the current k is wave-uniform, so it is fetched with scalar
//    loads and used as the SGPR operand of v_fma_f32.  The accumulation order
//    inside a chunk is exactly the ABI's declared order (one fma per k,
//    ascending).  Chunk results go to scratch as part[tile][chunk][expert][64]
//    (token fastest: coalesced both here and in the reader, and one tile's
//    partials are one contiguous run).  When there are few token tiles the
//    experts are also split over several waves so that every SIMD has work.
//  route_select_kernel: lane = token.  Adds the chunk results left to right,
//    adds the bias, then does arg max / masked top-(K-1) entirely in registers
//    with one 64-bit collaborator mask per expert held in LDS.
#include "c2r_internal.h"

namespace c2r {

// Wp[s][k][j] = W_g[k][s*epw + j] (zero past E): each expert split gets its own dense
// [d, epw] matrix, so a wave streams its W rows as one contiguous run of scalar loads.
__global__ __launch_bounds__(256) void pack_router_kernel(const float *__restrict__ Wg, int d, int E,
                                                          int epw, int esplit, float *__restrict__ Wp) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)d * epw * esplit) return;
    const int j = (int)(i % epw);
    const int k = (int)((i / epw) % d);
    const int s = (int)(i / ((int64_t)epw * d));
    const int e = s * epw + j;
    Wp[i] = e < E ? Wg[(int64_t)k * E + e] : 0.0f;
}

template <bool BF16, int EP>  // EP: experts handled by one wave
__global__ __launch_bounds__(64) void route_partial_kernel(const void *__restrict__ x,
                                                           const float *__restrict__ W,
                                                           int64_t T, int d, int nchunk, int esplit,
                                                           int ep_total, int64_t ntiles,
                                                           float *__restrict__ part) {
    constexpr int VEC = BF16 ? 8 : 4;  // elements per 16-byte vector
    constexpr int KSUB = 8 * VEC;      // elements per staged row segment (128 bytes)
    constexpr int PITCH = 128 + 16;    // LDS row pitch in bytes: odd multiple of 16 -> no conflicts
    constexpr int ESZ = BF16 ? 2 : 4;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][64 * PITCH];

    const int lane = threadIdx.x;
    // token tile fastest: the workgroups dispatched together share one (chunk, split), i.e. the
    // same W rows, which then stay hot in the scalar cache and L2
    const int64_t tile = blockIdx.x % ntiles;
    const int cs = (int)(blockIdx.x / ntiles);
    const int split = cs % esplit, chunk = cs / esplit;
    W += (size_t)split * d * EP;  // this split's dense [d, EP] matrix
    const int k_begin = chunk * C2R_CANON_CHUNK;
    const int k_end = min(d, k_begin + C2R_CANON_CHUNK);
    const int64_t t0 = tile * 64;
    const int lrow = lane >> 3, lc = lane & 7;
    const unsigned char *xb = static_cast<const unsigned char *>(x);

    uint4 stage[8];
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int64_t t = t0 + lrow + 8 * i;
            t = t < T ? t : T - 1;  // rows past the end re-read the last token; never stored
            int kc = k0 + lc * VEC;
            if (kc < k_end)
                stage[i] = *reinterpret_cast<const uint4 *>(xb + ((size_t)t * d + kc) * ESZ);
            else
                stage[i] = make_uint4(0, 0, 0, 0);
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<uint4 *>(&lds[buf][(lrow + 8 * i) * PITCH + lc * 16]) = stage[i];
    };

    float acc[EP];
#pragma unroll
    for (int e = 0; e < EP; ++e) acc[e] = 0.0f;

    gload(k_begin);
    lstore(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = k_begin; k0 < k_end; k0 += KSUB) {
        const int knext = k0 + KSUB;
        if (knext < k_end) gload(knext);
        const int nvec = min(KSUB, k_end - k0) / VEC;
        for (int v = 0; v < nvec; ++v) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(&lds[buf][lane * PITCH + v * 16]);
            float xv[VEC];
            if constexpr (BF16) {
                xv[0] = __uint_as_float(raw.x << 16);
                xv[1] = __uint_as_float(raw.x & 0xffff0000u);
                xv[2] = __uint_as_float(raw.y << 16);
                xv[3] = __uint_as_float(raw.y & 0xffff0000u);
                xv[4] = __uint_as_float(raw.z << 16);
                xv[5] = __uint_as_float(raw.z & 0xffff0000u);
                xv[6] = __uint_as_float(raw.w << 16);
                xv[7] = __uint_as_float(raw.w & 0xffff0000u);
            } else {
                xv[0] = __uint_as_float(raw.x);
                xv[1] = __uint_as_float(raw.y);
                xv[2] = __uint_as_float(raw.z);
                xv[3] = __uint_as_float(raw.w);
            }
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const float *__restrict__ wrow = W + (size_t)(k0 + v * VEC + j) * EP;
#pragma unroll
                for (int e = 0; e < EP; ++e) acc[e] = __builtin_fmaf(xv[j], wrow[e], acc[e]);
            }
        }
        if (knext < k_end) lstore(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    float *dst = part + (((size_t)tile * nchunk + chunk) * ep_total + split * EP) * 64 + lane;
#pragma unroll
    for (int e = 0; e < EP; ++e) dst[e * 64] = acc[e];
}

// Among experts whose bit is set in m: the largest logit, first one standing
// unless a later one is strictly larger (so ties and NaNs go to the lower index).
template <int EP>
__device__ __forceinline__ void pick(const float (&l)[EP], uint64_t m, int &bi, float &bv) {
    bi = -1;
    bv = 0.0f;
    const uint32_t lo = (uint32_t)m, hi = (uint32_t)(m >> 32);
#pragma unroll
    for (int e = 0; e < EP; ++e) {
        const bool ok = (((e < 32) ? (lo >> (e & 31)) : (hi >> (e & 31))) & 1u) != 0;
        const bool take = ok && (bi < 0 || l[e] > bv);
        bv = take ? l[e] : bv;
        bi = take ? e : bi;
    }
}

template <int EP, bool ROWMAJOR>
__global__ __launch_bounds__(64) void route_select_kernel(
    const float *__restrict__ src, int nchunk, const float *__restrict__ bias,
    int64_t T, int E, int K, const int32_t *__restrict__ collab_idx, int Tc,
    int32_t *__restrict__ topk_idx, float *__restrict__ gates, float *__restrict__ logits_out) {
    __shared__ uint64_t mask_tab[C2R_MAX_E];
    constexpr int LP = EP + 1;  // odd pitch: per-lane row reads hit distinct banks
    __shared__ float tile[ROWMAJOR ? 64 * LP : 1];

    const uint64_t all = E >= 64 ? ~0ull : ((1ull << E) - 1ull);
    if (threadIdx.x < C2R_MAX_E) {
        const int e = threadIdx.x;
        uint64_t m = 0;
        if (e < E) {
            if (collab_idx) {
                for (int j = 0; j < Tc; ++j) {
                    int v = collab_idx[(size_t)e * Tc + j];
                    if (v >= 0 && v < E && v != e) m |= 1ull << v;
                }
            } else {
                m = all & ~(1ull << e);
            }
        }
        mask_tab[e] = m;
    }

    const int64_t t = (int64_t)blockIdx.x * 64 + threadIdx.x;
    const int lane = threadIdx.x;
    float l[EP];
    if constexpr (ROWMAJOR) {
        // wave-private transpose: 64 consecutive rows of E floats are one contiguous run
        float *tl = tile;
        const int64_t tw = (int64_t)blockIdx.x * 64;
        const int64_t rows = T - tw < 64 ? T - tw : 64;  // may be <= 0
        const int64_t nflt = rows > 0 ? rows * E : 0;
        const float *base = src + tw * E;
        const uint32_t rcp = (uint32_t)((0x100000000ull + E - 1) / E);
        for (int64_t i = (int64_t)lane * 4; i < nflt; i += 256) {
            float v[4];
            if (i + 4 <= nflt) {
                const float4 q = *reinterpret_cast<const float4 *>(base + i);
                v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = i + j < nflt ? base[i + j] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t f = (uint32_t)i + j;
                if (f < nflt) {
                    const uint32_t r = __umulhi(f, rcp);  // f / E, exact for f < 4096
                    tl[r * LP + (f - r * E)] = v[j];
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < EP; ++e) l[e] = (e < E && lane < rows) ? tl[lane * LP + e] : 0.0f;
    } else {
        const float *p = src + (size_t)blockIdx.x * nchunk * EP * 64 + lane;
#pragma unroll
        for (int e = 0; e < EP; ++e) l[e] = p[e * 64];
        for (int c = 1; c < nchunk; ++c) {
            p += EP * 64;
#pragma unroll
            for (int e = 0; e < EP; ++e) l[e] = l[e] + p[e * 64];
        }
        if (bias) {
#pragma unroll
            for (int e = 0; e < EP; ++e)
                if (e < E) l[e] = l[e] + bias[e];
        }
        __syncthreads();
    }
    if (t >= T) return;

    if (logits_out) {
#pragma unroll
        for (int e = 0; e < EP; ++e)
            if (e < E) logits_out[(size_t)t * E + e] = l[e];
    }

    int e0;
    float v0;
    pick<EP>(l, all, e0, v0);
    uint64_t m = mask_tab[e0];
    topk_idx[(size_t)t * K] = e0;
    gates[(size_t)t * K] = 1.0f;
    float den = 1.0f;
    for (int s = 1; s < K; ++s) {
        int e;
        float v;
        pick<EP>(l, m, e, v);
        float g = 0.0f;
        if (e >= 0) {
            m &= ~(1ull << e);
            g = expf(v - v0);
        }
        den += g;
        topk_idx[(size_t)t * K + s] = e;
        gates[(size_t)t * K + s] = g;
    }
    for (int s = 0; s < K; ++s) gates[(size_t)t * K + s] = gates[(size_t)t * K + s] / den;
}

static int check_route_args(int64_t T, int E, int K, const int32_t *collab_idx, int Tc) {
    if (T < 0 || E < 1 || K < 1 || K > E) return C2R_ERR_INVALID_ARG;
    if (collab_idx && Tc < K - 1) return C2R_ERR_INVALID_ARG;
    if (E > C2R_MAX_E) return C2R_ERR_UNSUPPORTED;
    if (T * (int64_t)K >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    return C2R_OK;
}

static inline int ep_of(int E) { return (E + 3) / 4 * 4; }

struct RouteLayout {
    int EP, nchunk, esplit;
    int64_t Tpad;
    size_t part_bytes, wpad_bytes;
};

static RouteLayout route_layout(int64_t T, int d, int E) {
    RouteLayout L;
    L.EP = ep_of(E);
    L.nchunk = (d + C2R_CANON_CHUNK - 1) / C2R_CANON_CHUNK;
    if (L.nchunk < 1) L.nchunk = 1;
    L.Tpad = (T + 63) / 64 * 64;
    // split the experts over `esplit` waves (each a multiple of 4 experts, at least 8) until
    // there are about two waves per SIMD (256 CUs x 4 SIMDs)
    L.esplit = 1;
    const int64_t base_waves = L.Tpad / 64 * L.nchunk;
    for (int s = 1; s <= L.EP / 4; ++s) {
        if ((L.EP / 4) % s != 0) continue;
        if (L.EP / s < 8 && s > 1) break;
        L.esplit = s;
        if (base_waves * s >= 2048) break;
    }
    L.part_bytes = round_up((size_t)L.nchunk * L.EP * (size_t)L.Tpad * sizeof(float), 256);
    L.wpad_bytes = (E % 4 || L.esplit > 1) ? round_up((size_t)d * L.EP * sizeof(float), 256) : 0;
    return L;
}

size_t route_workspace_bytes(int64_t T, int d, int E) {
    if (T <= 0 || d <= 0 || E <= 0) return 0;
    RouteLayout L = route_layout(T, d, E);
    return L.part_bytes + L.wpad_bytes;
}

#define C2R_EP_SWITCH(EPV, ...) \
    switch (EPV) {               \
        case 4: { constexpr int EP = 4; __VA_ARGS__; } break;   \
        case 8: { constexpr int EP = 8; __VA_ARGS__; } break;   \
        case 12: { constexpr int EP = 12; __VA_ARGS__; } break; \
        case 16: { constexpr int EP = 16; __VA_ARGS__; } break; \
        case 20: { constexpr int EP = 20; __VA_ARGS__; } break; \
        case 24: { constexpr int EP = 24; __VA_ARGS__; } break; \
        case 28: { constexpr int EP = 28; __VA_ARGS__; } break; \
        case 32: { constexpr int EP = 32; __VA_ARGS__; } break; \
        case 36: { constexpr int EP = 36; __VA_ARGS__; } break; \
        case 40: { constexpr int EP = 40; __VA_ARGS__; } break; \
        case 44: { constexpr int EP = 44; __VA_ARGS__; } break; \
        case 48: { constexpr int EP = 48; __VA_ARGS__; } break; \
        case 52: { constexpr int EP = 52; __VA_ARGS__; } break; \
        case 56: { constexpr int EP = 56; __VA_ARGS__; } break; \
        case 60: { constexpr int EP = 60; __VA_ARGS__; } break; \
        case 64: { constexpr int EP = 64; __VA_ARGS__; } break; \
        default: return C2R_ERR_UNSUPPORTED;             \
    }

}  // namespace c2r

using namespace c2r;

extern "C" int c2r_route_chunk(void) { return C2R_CANON_CHUNK; }

extern "C" int c2r_route(const void *x, c2r_dtype x_dt, const float *Wg, const float *bias,
                         int64_t T, int d, int E, int K, const int32_t *collab_idx, int Tc,
                         int32_t *topk_idx, float *gates, float *logits_out, void *ws,
                         size_t ws_bytes, void *stream) {
    int rc = check_route_args(T, E, K, collab_idx, Tc);
    if (rc != C2R_OK) return rc;
    if (d < 1 || (x_dt != C2R_F32 && x_dt != C2R_BF16)) return C2R_ERR_INVALID_ARG;
    if (T == 0) return C2R_OK;
    if (!x || !Wg || !topk_idx || !gates) return C2R_ERR_INVALID_ARG;
    if (d % 8 != 0) return C2R_ERR_UNSUPPORTED;
    if (!aligned(x, 16) || !aligned(Wg, 4)) return C2R_ERR_INVALID_ARG;
    const RouteLayout L = route_layout(T, d, E);
    if (!ws || ws_bytes < L.part_bytes + L.wpad_bytes || !aligned(ws, 256)) return C2R_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *part = static_cast<float *>(ws);
    const float *W = Wg;
    const int EPW = L.EP / L.esplit;
    if (L.wpad_bytes) {
        float *Wp = reinterpret_cast<float *>(static_cast<char *>(ws) + L.part_bytes);
        const int64_t n = (int64_t)d * L.EP;
        pack_router_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(Wg, d, E, EPW, L.esplit, Wp);
        W = Wp;
    }
    const int64_t ntiles = L.Tpad / 64;
    const int64_t nblk = ntiles * L.nchunk * L.esplit;
    if (nblk >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    if (x_dt == C2R_BF16) {
        C2R_EP_SWITCH(EPW, route_partial_kernel<true, EP><<<dim3((unsigned)nblk), dim3(64), 0, st>>>(
                               x, W, T, d, L.nchunk, L.esplit, L.EP, ntiles, part));
    } else {
        C2R_EP_SWITCH(EPW, route_partial_kernel<false, EP><<<dim3((unsigned)nblk), dim3(64), 0, st>>>(
                               x, W, T, d, L.nchunk, L.esplit, L.EP, ntiles, part));
    }
    C2R_EP_SWITCH(L.EP, route_select_kernel<EP, false><<<dim3((unsigned)ntiles), dim3(64), 0, st>>>(
                            part, L.nchunk, bias, T, E, K, collab_idx, Tc, topk_idx, gates, logits_out));
    return launch_status();
}

extern "C" int c2r_route_from_logits(const float *logits, int64_t T, int E, int K,
                                     const int32_t *collab_idx, int Tc, int32_t *topk_idx,
                                     float *gates, void *stream) {
    int rc = check_route_args(T, E, K, collab_idx, Tc);
    if (rc != C2R_OK) return rc;
    if (T == 0) return C2R_OK;
    if (!logits || !topk_idx || !gates) return C2R_ERR_INVALID_ARG;
    if (!aligned(logits, 16)) return C2R_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t nsel = (T + 63) / 64;
    if (nsel >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    const int EPV = ep_of(E);
    C2R_EP_SWITCH(EPV, route_select_kernel<EP, true><<<dim3((unsigned)nsel), dim3(64), 0, st>>>(
                           logits, 1, (const float *)nullptr, T, E, K, collab_idx, Tc, topk_idx, gates,
                           (float *)nullptr));
    return launch_status();
}
