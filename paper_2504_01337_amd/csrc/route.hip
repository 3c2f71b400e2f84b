// Router logits (Eq. 1) and collaboration-constrained selection (Sec. 3.3, step 2).
//
// Two kernels.
//  route_partial_kernel: an fp32 GEMM over one 256-long k-chunk in which every (token,
//    expert) sum is built with one fused multiply-add per k in ascending k - exactly the
//    ABI's declared order - either by one thread on the vector pipe (up to 8 experts) or by
//    a chain of v_mfma_f32_32x32x2_f32 on the matrix pipe, whose two products per
//    instruction are added in that same order.  Chunk results go to scratch as
//    part[tile][chunk][expert][64] (token fastest, one tile's partials contiguous).
//  route_select_kernel: adds the chunk results left to right (four tokens per lane), adds the
//    bias, then does arg max / masked top-(K-1) in registers with one 64-bit collaborator
//    mask per expert held in LDS: four lanes per token over a quarter of the experts each
//    (chunk partials), or one lane per token over all of them (stored logits).
#include "c2r_internal.h"

#include <type_traits>

namespace c2r {

// Wp[k][j] = W_g[k][j] zero-padded to a row length that is a multiple of 4 (only needed when
// E is not one), so that W rows can be fetched with 16-byte loads.
__global__ __launch_bounds__(256) void pack_router_kernel(const float *__restrict__ Wg, int d, int E,
                                                          int ep, float *__restrict__ Wp) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)d * ep) return;
    const int j = (int)(i % ep), k = (int)(i / ep);
    Wp[i] = j < E ? Wg[(int64_t)k * E + j] : 0.0f;
}

// Partial logits of one 256-long k-chunk for NWV token tiles of 8*TQ tokens (one per wave), all
// experts.  A register-tiled fp32 GEMM: lane = (token lane tl, expert lane el) on an 8 x 8 grid; the
// thread owns tokens tl + 8q (q < TQ) and experts el*TE + j (j < TE), i.e. TQ*TE accumulators,
// and walks k upward one fused multiply-add at a time, which is the declared order.  Both
// operands come from LDS (x as stored, 16 bytes = 8 bf16 or 4 fp32 per token per read; W
// rows as fp32), staged in 32-wide k sub-tiles that are double buffered against global
// loads held in registers; the W sub-tile is shared by the workgroup's waves.
// TQ = 4 halves a wave's tile: twice the waves for batches that would otherwise leave one wave
// per SIMD with nothing to hide its LDS latency behind.
//
// MFMA = true does the same sums on the matrix pipe: one v_mfma_f32_32x32x2_f32 adds, to each of
// 32 experts x 32 tokens, the products of k and k+1 - as two fused multiply-adds, k first,
// then k+1, each rounded to nearest even (checked on the chip against chains of fmaf: bit
// identical, denormal and overflow ranges included), so a chain of them over ascending k IS
// the declared order, at twice the rate the vector pipe reaches without packed instructions.
// Lanes 0-31 feed k, lanes 32-63 k+1: one W value and one x value per lane and instruction.
// With 32-token wave tiles a whole chunk is software-pipelined (see PIPE below): operands of
// sub-tile i in registers, sub-tile i+1 in a ring of three LDS buffers, i+2 on its way from
// staging registers into LDS, i+3 to i+5 in flight from memory.
// ALLCHUNKS (matrix pipe only): the workgroup walks ALL the chunks of its tokens and adds the
// chunk results up in registers, left to right - the declared order - so that scratch holds one
// 64-expert vector per token (256 bytes) instead of one per chunk (2 KB at d = 2048, written
// here and read back by the selection).  For batches with at least one wave tile per SIMD of
// the chip; smaller batches need the chunks as separate workgroups to fill it.
template <bool BF16, int TE, int NWV, int TQ, bool MFMA, bool ALLCHUNKS = false>
__global__ __launch_bounds__(NWV * 64, (MFMA && TQ == 4) ? 2 : 1) void route_partial_kernel(const void *__restrict__ x,
                                                                const float *__restrict__ W, int ldw,
                                                                int ep, int64_t T, int d, int nchunk,
                                                                int64_t ntiles,
                                                                float *__restrict__ part) {
    constexpr int EPAD = 8 * TE;         // experts covered by a wave
    constexpr int TOK = 8 * TQ;          // tokens covered by a wave
    constexpr int KS = 32;               // k per staged sub-tile
    constexpr int VEC = BF16 ? 8 : 4;    // elements per 16-byte vector of x
    constexpr int ESZ = BF16 ? 2 : 4;
    constexpr int XV = KS / VEC;         // 16-byte vectors per token per sub-tile
    constexpr int XPITCH = KS * ESZ + 16;  // bytes; token rows 8 apart land on distinct bank groups
    constexpr int XLOADS = TOK * XV / 64;  // vectors per lane per sub-tile
    static_assert(XLOADS >= 1 && 64 % TOK == 0, "a wave loads whole vectors; wave tiles divide the 64-token tile");
    constexpr int WF4 = KS * EPAD / 4;     // float4 per W sub-tile
    constexpr int WLOADS = (WF4 + NWV * 64 - 1) / (NWV * 64);
    // One wave's matrix instructions of a sub-tile overlap its own operand reads of the next one
    // (PIPE): that takes a third LDS buffer and two operand register sets, which fit 32-token
    // wave tiles only.
    constexpr bool PIPE = MFMA && TOK == 32;
    constexpr int NBUF = PIPE ? 3 : 2;
    // (Counted on the matrix-pipe form at E = 60: SQ_LDS_BANK_CONFLICT = 128 cycles per wave task of
    // 8 sub-tiles, i.e. 16 per sub-tile - one per x operand read: 32 token rows 80 bytes apart fall
    // on 16 banks, a 2-way conflict that any row pitch that keeps the 16-byte staging stores
    // aligned has.  Against the 2048 matrix-pipe cycles of a sub-tile that is under 1 %; padding
    // the W rows instead, 32 floats per 64-wide row, changed neither the counter nor the time.)
    constexpr int WPITCH = EPAD;
    __shared__ __attribute__((aligned(16))) float Wl[NBUF][KS][WPITCH];
    __shared__ __attribute__((aligned(16))) unsigned char Xl[NBUF][NWV][TOK * XPITCH];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tl = lane & 7, el = lane >> 3;
    const int64_t nwt = ntiles * (64 / TOK);       // wave tiles
    const int64_t ngroups = (nwt + NWV - 1) / NWV;
    const int64_t tgroup = blockIdx.x % ngroups;  // token tiles fastest: neighbours share W rows in L2
    const int chunk_first = ALLCHUNKS ? 0 : (int)(blockIdx.x / ngroups);
    const int chunk_last = ALLCHUNKS ? nchunk - 1 : chunk_first;
    const int64_t wt = tgroup * NWV + wave;        // may be >= nwt: such a wave only helps load W
    const bool live = wt < nwt;
    int chunk = chunk_first, k_begin = chunk * C2R_CANON_CHUNK;
    int k_end = min(d, k_begin + C2R_CANON_CHUNK);
    const int64_t t0 = wt * TOK;
    const unsigned char *xb = static_cast<const unsigned char *>(x);

    // global loads of a sub-tile are held in registers until its LDS buffer is free; several sets
    // (two in the plain loop, three in the pipelined one), so that a sub-tile is fetched two or
    // three sub-tiles ahead (on the matrix pipe one sub-tile of compute is shorter than the
    // memory latency)
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    struct Staged {
        f32x4 w[WLOADS];
        u32x4 x[XLOADS];
    };
    // Every load is issued, out-of-range ones on a clamped address: with no branch around a
    // load the compiler counts the loads in flight and waits only for the older set.  What a
    // clamped load brings is never used: k past the end of the chunk is left out by the
    // compute loops, experts >= ep and tokens >= T are accumulated and never stored or read.
    auto gload = [&](Staged &r, int k0) __attribute__((always_inline)) {
        f32x4 (&wreg)[WLOADS] = r.w;
        u32x4 (&xreg)[XLOADS] = r.x;
#pragma unroll
        for (int i = 0; i < WLOADS; ++i) {
            const int idx = tid + i * NWV * 64;
            const int k = idx / (EPAD / 4), c = idx % (EPAD / 4);
            const int kk = min(k0 + k, k_end - 1), cc = c * 4 < ep ? c : 0;
            wreg[i] = *reinterpret_cast<const f32x4 *>(W + (size_t)kk * ldw + cc * 4);
        }
#pragma unroll
        for (int i = 0; i < XLOADS; ++i) {
            const int idx = lane + i * 64;
            const int tok = idx / XV, c = idx % XV;
            int64_t t = t0 + tok;
            t = t < T ? t : T - 1;  // rows past the end (and dead waves) re-read a valid token
            t = t < 0 ? 0 : t;
            const int kc = min(k0 + c * VEC, k_end - VEC);
            xreg[i] = *reinterpret_cast<const u32x4 *>(xb + ((size_t)t * d + kc) * ESZ);
        }
    };
    // The same loads of a whole sub-tile (nothing to clamp in k): a uniform base per sub-tile
    // plus a 32-bit lane offset that is the same for every sub-tile.
    uint32_t woff[WLOADS], xoff[XLOADS];
#pragma unroll
    for (int i = 0; i < WLOADS; ++i) {
        const int idx = tid + i * NWV * 64;
        const int k = min(idx / (EPAD / 4), KS - 1), c = idx % (EPAD / 4);
        woff[i] = (uint32_t)((k * ldw + (c * 4 < ep ? c * 4 : 0)) * 4);
    }
    const int64_t tb = t0 < T ? t0 : T - 1;  // wave-uniform; dead waves re-read valid tokens
#pragma unroll
    for (int i = 0; i < XLOADS; ++i) {
        const int idx = lane + i * 64;
        const int64_t room = T - 1 - tb, tok = idx / XV < room ? idx / XV : room;
        xoff[i] = (uint32_t)((tok * d + (idx % XV) * VEC) * ESZ);
    }
    auto gload_whole = [&](Staged &r, int k0) __attribute__((always_inline)) {
        const unsigned char *wb = reinterpret_cast<const unsigned char *>(W + (size_t)k0 * ldw);
        const unsigned char *xs = xb + ((size_t)tb * d + k0) * ESZ;
#pragma unroll
        for (int i = 0; i < WLOADS; ++i) r.w[i] = *reinterpret_cast<const f32x4 *>(wb + woff[i]);
#pragma unroll
        for (int i = 0; i < XLOADS; ++i) r.x[i] = *reinterpret_cast<const u32x4 *>(xs + xoff[i]);
    };
    auto lstore = [&](const Staged &r, int buf) __attribute__((always_inline)) {
        const f32x4 (&wreg)[WLOADS] = r.w;
        const u32x4 (&xreg)[XLOADS] = r.x;
#pragma unroll
        for (int i = 0; i < WLOADS; ++i) {
            const int idx = tid + i * NWV * 64;
            if (WF4 % (NWV * 64) == 0 || idx < WF4) *reinterpret_cast<f32x4 *>(&Wl[buf][idx / (EPAD / 4)][(idx % (EPAD / 4)) * 4]) = wreg[i];
        }
#pragma unroll
        for (int i = 0; i < XLOADS; ++i) {
            const int idx = lane + i * 64;
            *reinterpret_cast<u32x4 *>(&Xl[buf][wave][(idx / XV) * XPITCH + (idx % XV) * 16]) = xreg[i];
        }
    };

    typedef float f32x16 __attribute__((ext_vector_type(16)));
    constexpr int NEB = MFMA ? EPAD / 32 : 1, NTB = MFMA ? TOK / 32 : 1;  // 32-expert / 32-token blocks
    static_assert(!MFMA || (EPAD % 32 == 0 && TOK % 32 == 0), "whole 32 x 32 blocks");
    f32x16 macc[NEB][NTB];
#pragma unroll
    for (int a = 0; a < NEB; ++a)
#pragma unroll
        for (int b = 0; b < NTB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) macc[a][b][i] = 0.0f;
    f32x16 mtot[ALLCHUNKS ? NEB : 1][ALLCHUNKS ? NTB : 1];  // sum of the chunks done so far
    const int mh = lane >> 5, mc = lane & 31;  // k parity and block column fed by this lane
    float acc[TQ][TE];
#pragma unroll
    for (int q = 0; q < TQ; ++q)
#pragma unroll
        for (int j = 0; j < TE; ++j) acc[q][j] = 0.0f;

    auto compute = [&](int buf, int k0) __attribute__((always_inline)) {
        const int nvec = min(KS, k_end - k0) / VEC;  // workgroup-uniform
        if constexpr (MFMA) {
            auto pair = [&](int kp) __attribute__((always_inline)) {
                float wv[NEB], xv[NTB];
#pragma unroll
                for (int a = 0; a < NEB; ++a) wv[a] = Wl[buf][2 * kp + mh][a * 32 + mc];
#pragma unroll
                for (int b = 0; b < NTB; ++b) {
                    const unsigned char *row = &Xl[buf][wave][(b * 32 + mc) * XPITCH];
                    if (BF16) {  // one word holds x[k] (low half) and x[k+1] (high half)
                        const uint32_t word = *reinterpret_cast<const uint32_t *>(row + kp * 4);
                        xv[b] = __uint_as_float(mh ? (word & 0xffff0000u) : (word << 16));
                    } else {
                        xv[b] = *reinterpret_cast<const float *>(row + (2 * kp + mh) * 4);
                    }
                }
#pragma unroll
                for (int a = 0; a < NEB; ++a)
#pragma unroll
                    for (int b = 0; b < NTB; ++b)
                        macc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(wv[a], xv[b], macc[a][b], 0, 0, 0);
            };
            const int npair = nvec * VEC / 2;
            if (npair == KS / 2) {
                // a whole sub-tile: every operand is read first, into registers of its own, so that
                // the matrix instructions never wait for a read issued just before them
                float wv[KS / 2][NEB], xv[KS / 2][NTB];
#pragma unroll
                for (int kp = 0; kp < KS / 2; ++kp)
#pragma unroll
                    for (int a = 0; a < NEB; ++a) wv[kp][a] = Wl[buf][2 * kp + mh][a * 32 + mc];
#pragma unroll
                for (int b = 0; b < NTB; ++b) {
                    const unsigned char *row = &Xl[buf][wave][(b * 32 + mc) * XPITCH];
#pragma unroll
                    for (int kp = 0; kp < KS / 2; ++kp) {
                        if (BF16) {
                            const uint32_t word = *reinterpret_cast<const uint32_t *>(row + kp * 4);
                            xv[kp][b] = __uint_as_float(mh ? (word & 0xffff0000u) : (word << 16));
                        } else {
                            xv[kp][b] = *reinterpret_cast<const float *>(row + (2 * kp + mh) * 4);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);  // (the scheduler would sink each read to its use)
#pragma unroll
                for (int kp = 0; kp < KS / 2; ++kp)
#pragma unroll
                    for (int a = 0; a < NEB; ++a)
#pragma unroll
                        for (int b = 0; b < NTB; ++b)
                            macc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(wv[kp][a], xv[kp][b], macc[a][b], 0, 0, 0);
            } else {
                for (int kp = 0; kp < npair; ++kp) pair(kp);
            }
        } else
        for (int v = 0; v < nvec; ++v) {
            uint4 xp[TQ];
#pragma unroll
            for (int q = 0; q < TQ; ++q)
                xp[q] = *reinterpret_cast<const uint4 *>(&Xl[buf][wave][(tl + 8 * q) * XPITCH + v * 16]);
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                float wv[TE];
#pragma unroll
                for (int j = 0; j < TE; ++j) wv[j] = Wl[buf][v * VEC + u][el * TE + j];
#pragma unroll
                for (int q = 0; q < TQ; ++q) {
                    const uint32_t word = BF16 ? (u < 2 ? xp[q].x : u < 4 ? xp[q].y : u < 6 ? xp[q].z : xp[q].w)
                                               : (u == 0 ? xp[q].x : u == 1 ? xp[q].y : u == 2 ? xp[q].z : xp[q].w);
                    const float xv = BF16 ? __uint_as_float((u & 1) ? (word & 0xffff0000u) : (word << 16))
                                          : __uint_as_float(word);
#pragma unroll
                    for (int j = 0; j < TE; ++j) acc[q][j] = __builtin_fmaf(xv, wv[j], acc[q][j]);
                }
            }
        }
    };
    for (;; ++chunk) {  // one trip unless ALLCHUNKS
    if constexpr (ALLCHUNKS) {
        k_begin = chunk * C2R_CANON_CHUNK;
        k_end = min(d, k_begin + C2R_CANON_CHUNK);
    }
    bool piped = false;
    if constexpr (PIPE) {
        // Sub-tile i: operands in registers (set i % 2); sub-tile i+1: in LDS buffer (i+1) % 3;
        // sub-tile i+2: on its way from the staging registers into buffer (i+2) % 3; sub-tiles
        // i+3 and i+4: global loads in flight.  The chain of every accumulator still takes k in
        // ascending order, two per instruction.
        struct Ops {
            float w[KS / 2][NEB];
            uint32_t x[KS / 2][NTB];
        };
        auto read_ops = [&](Ops &o, int buf) __attribute__((always_inline)) {
#pragma unroll
            for (int kp = 0; kp < KS / 2; ++kp)
#pragma unroll
                for (int a = 0; a < NEB; ++a) o.w[kp][a] = Wl[buf][2 * kp + mh][a * 32 + mc];
#pragma unroll
            for (int b = 0; b < NTB; ++b) {
                const unsigned char *row = &Xl[buf][wave][(b * 32 + mc) * XPITCH];
#pragma unroll
                for (int kp = 0; kp < KS / 2; ++kp)  // bf16: the word holds x[k] (low) and x[k+1] (high)
                    o.x[kp][b] = *reinterpret_cast<const uint32_t *>(row + (BF16 ? kp : 2 * kp + mh) * 4);
            }
        };
        const int sh = mh ? 0 : 16;
        auto mma = [&](const Ops &o) __attribute__((always_inline)) {
#pragma unroll
            for (int kp = 0; kp < KS / 2; ++kp)
#pragma unroll
                for (int b = 0; b < NTB; ++b) {
                    const float xv = __uint_as_float(BF16 ? (o.x[kp][b] << sh) & 0xffff0000u : o.x[kp][b]);
#pragma unroll
                    for (int a = 0; a < NEB; ++a)
                        macc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.w[kp][a], xv, macc[a][b], 0, 0, 0);
                }
        };
        // Whole chunks only, and the sub-tile loop unrolled into straight-line code: only there
        // does the compiler count the loads in flight exactly, so that a wait for the older
        // staging set leaves the younger one in flight.  (A ragged last chunk takes the loop below.)
        constexpr int NSUB = C2R_CANON_CHUNK / KS;
        static_assert(NSUB >= 5, "the prologue fetches sub-tiles 0 to 4");
        if (k_end - k_begin == C2R_CANON_CHUNK) {
            // sub-tile j waits in staging set j % 3; the first three are requested together
            Staged R[3];
            Ops O[2];
            gload_whole(R[0], k_begin);
            gload_whole(R[1], k_begin + KS);
            gload_whole(R[2], k_begin + 2 * KS);
            lstore(R[0], 0);
            gload_whole(R[0], k_begin + 3 * KS);
            __syncthreads();
            read_ops(O[0], 0);
            lstore(R[1], 1);
            gload_whole(R[1], k_begin + 4 * KS);
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NSUB; ++i) {
                if (i + 1 < NSUB) read_ops(O[(i + 1) & 1], (i + 1) % 3);
                if (i + 2 < NSUB) lstore(R[(i + 2) % 3], (i + 2) % 3);
                if (i + 5 < NSUB) gload_whole(R[(i + 2) % 3], k_begin + (i + 5) * KS);
                mma(O[i & 1]);
                // the step's memory instructions go between its matrix instructions, one each:
                // the wave issues them while the matrix pipe works
#pragma unroll
                for (int m = 0; m < NEB * NTB * KS / 2; ++m) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // a matrix instruction
                    if (m < 20) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);       // an LDS read
                    else if (m < 24) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // an LDS write
                    else if (m < 28) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // a global load
                }
                __builtin_amdgcn_sched_barrier(0);
                if (i + 1 < NSUB) __syncthreads();
            }
            piped = true;
        }
    }
    if (!piped) {
    Staged r0, r1;
    gload(r0, k_begin);
    lstore(r0, 0);
    gload(r1, k_begin + KS);  // (past the end of the chunk: clamped loads, never stored)
    gload(r0, k_begin + 2 * KS);
    __syncthreads();
    for (int k0 = k_begin; k0 < k_end; k0 += 2 * KS) {
        compute(0, k0);
        if (k0 + KS < k_end) lstore(r1, 1);
        gload(r1, k0 + 3 * KS);
        __syncthreads();
        if (k0 + KS >= k_end) break;
        compute(1, k0 + KS);
        if (k0 + 2 * KS < k_end) lstore(r0, 0);
        gload(r0, k0 + 4 * KS);
        __syncthreads();
    }
    }
    if constexpr (ALLCHUNKS) {
        // chunk results are added left to right (plain fp32 adds, as the selection kernel does
        // when it reads them from scratch), and the next chunk starts again from +0
#pragma unroll
        for (int a = 0; a < NEB; ++a)
#pragma unroll
            for (int b = 0; b < NTB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    mtot[a][b][i] = chunk == 0 ? macc[a][b][i] : mtot[a][b][i] + macc[a][b][i];
                    macc[a][b][i] = 0.0f;
                }
        __syncthreads();  // every wave is done with the LDS buffers before the next chunk refills them
    }
    if (chunk >= chunk_last) break;
    }
    if (!live) return;
    const int64_t tile = wt / (64 / TOK);           // the 64-token tile and this wave's part of it
    float *dst = part + (((size_t)tile * (ALLCHUNKS ? 1 : nchunk) + (ALLCHUNKS ? 0 : chunk)) * ep) * 64 +
                 (wt % (64 / TOK)) * TOK;
    if constexpr (MFMA) {
        // register i of a 32 x 32 block: expert (i/4)*8 + 4*(lane/32) + i%4, token lane%32
#pragma unroll
        for (int a = 0; a < NEB; ++a)
#pragma unroll
            for (int b = 0; b < NTB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int e = a * 32 + (i / 4) * 8 + mh * 4 + i % 4;
                    if (e < ep) dst[(size_t)e * 64 + b * 32 + mc] = ALLCHUNKS ? mtot[a][b][i] : macc[a][b][i];
                }
        return;
    }
#pragma unroll
    for (int j = 0; j < TE; ++j) {
        const int e = el * TE + j;
        if (e < ep) {
#pragma unroll
            for (int q = 0; q < TQ; ++q) dst[(size_t)e * 64 + tl + 8 * q] = acc[q][j];
        }
    }
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

// ROWMAJOR (stored logits [T, E]): one wave per 64 tokens.  Otherwise (chunk partials):
// SEL_WAVES waves per 64 tokens; each sums the chunks of a quarter of the experts (the
// loads of one wave alone cover the memory latency four times worse) and leaves its
// logits in LDS, then the first wave selects.
constexpr int SEL_WAVES = 4;

template <int EP, bool ROWMAJOR>
__global__ __launch_bounds__(ROWMAJOR ? 64 : SEL_WAVES * 64) void route_select_kernel(
    const float *__restrict__ src, int nchunk, const float *__restrict__ bias,
    int64_t T, int E, int K, const int32_t *__restrict__ collab_idx, int Tc,
    int32_t *__restrict__ topk_idx, float *__restrict__ gates, float *__restrict__ logits_out) {
    __shared__ uint64_t mask_tab[C2R_MAX_E];
    constexpr int LP = EP + 1;  // odd pitch: per-lane row reads hit distinct banks
    __shared__ float tile[64 * LP];

    const uint64_t all = E >= 64 ? ~0ull : ((1ull << E) - 1ull);
    // one 64-bit collaborator mask per expert; the list entries are spread over all the threads
    // (one thread walking a whole list would wait for Tc loads one after another)
    if (threadIdx.x < C2R_MAX_E)
        mask_tab[threadIdx.x] = (!collab_idx && (int)threadIdx.x < E) ? all & ~(1ull << threadIdx.x) : 0ull;
    if (collab_idx) {
        __syncthreads();
        const int n = E * Tc;
#pragma unroll 4
        for (int i = threadIdx.x; i < n; i += blockDim.x) {
            const int v = collab_idx[i], e = i / Tc;
            if (v >= 0 && v < E && v != e)
                atomicOr(reinterpret_cast<unsigned long long *>(&mask_tab[e]), 1ull << v);
        }
    }

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t t = (int64_t)blockIdx.x * 64 + lane;
    float l[EP];
    if constexpr (ROWMAJOR) {
        // wave-private transpose: 64 consecutive rows of E floats are one contiguous run
        float *tl = tile;
        const int64_t tw = (int64_t)blockIdx.x * 64;
        const int64_t rows = T - tw < 64 ? T - tw : 64;  // may be <= 0
        const int64_t nflt = rows > 0 ? rows * E : 0;
        const float *base = src + tw * E;
        const uint32_t rcp = (uint32_t)((0x100000000ull + E - 1) / E);
        auto scatter = [&](uint32_t f, float v) __attribute__((always_inline)) {
            // f / E, exact for f < 4096 (the 32-bit reciprocal of 1 does not exist)
            const uint32_t r = E == 1 ? f : __umulhi(f, rcp);
            tl[r * LP + (f - r * E)] = v;
        };
        if (rows == 64) {
            // a whole tile: 64 E floats (a multiple of 4), fetched with every load in flight at once -
            // unconditional, out-of-range ones on a clamped address - and only then spread over LDS:
            // what this kernel does is stream the logits, and a wave that waits for one 1 KB load
            // at a time (the loop below) leaves the memory pipe a fifth full
            typedef float f32x4 __attribute__((ext_vector_type(4)));
            constexpr int NV = EP / 4;
            f32x4 q[NV];
#pragma unroll
            for (int u = 0; u < NV; ++u) {
                const uint32_t i = (uint32_t)lane * 4 + u * 256;
                q[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(base + (i < nflt ? i : 0)));
            }
#pragma unroll
            for (int u = 0; u < NV; ++u) {
                const uint32_t i = (uint32_t)lane * 4 + u * 256;
                if (i < nflt) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) scatter(i + j, q[u][j]);
                }
            }
        } else
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
                if (f < nflt) scatter(f, v[j]);
            }
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < EP; ++e) l[e] = (e < E && lane < rows) ? tl[lane * LP + e] : 0.0f;
    } else {
        static_assert(EP % SEL_WAVES == 0, "experts divide over the waves");
        constexpr int EW = EP / SEL_WAVES;   // experts of this wave
        constexpr int ES = (EW + 3) / 4;     // in steps of four
        // A lane adds up four tokens (16-byte loads) of one expert per step: lane = (token quad,
        // expert within the step).  Chunk results are added left to right; eight chunks x ES
        // loads are in flight together (the partial sums were written by other XCDs a moment
        // ago, so every batch costs a trip to memory), all of them unconditional on clamped
        // indices.
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        constexpr int CU = 8;
        const int tq4 = lane & 15, es = lane >> 4;
        const float *p = src + ((size_t)blockIdx.x * nchunk * EP + (size_t)wave * EW) * 64 + 4 * tq4;
        f32x4 sum[ES];
        for (int c0 = 0; c0 < nchunk; c0 += CU) {
            f32x4 v[CU][ES];
#pragma unroll
            for (int u = 0; u < CU; ++u) {
                const int cc = min(c0 + u, nchunk - 1);
#pragma unroll
                for (int j = 0; j < ES; ++j) {
                    const int el = min(4 * j + es, EW - 1);
                    v[u][j] = *reinterpret_cast<const f32x4 *>(p + ((size_t)cc * EP + el) * 64);
                }
            }
#pragma unroll
            for (int u = 0; u < CU; ++u) {
                const bool have = c0 + u < nchunk;  // wave-uniform
#pragma unroll
                for (int j = 0; j < ES; ++j) sum[j] = !have ? sum[j] : (c0 + u == 0) ? v[u][j] : sum[j] + v[u][j];
            }
        }
#pragma unroll
        for (int j = 0; j < ES; ++j) {
            const int el = 4 * j + es, e = wave * EW + el;
            if (el < EW) {
                if (bias && e < E) sum[j] = sum[j] + bias[e];
#pragma unroll
                for (int i = 0; i < 4; ++i) tile[(4 * tq4 + i) * LP + e] = sum[j][i];
            }
        }
        __syncthreads();
        // Selection by all the waves: four lanes per token, each over a quarter of the experts.
        constexpr int EQ = EP / 4;
        const int tl = wave * (64 / SEL_WAVES) + (lane >> 2), sub = lane & 3;
        const int64_t tq = (int64_t)blockIdx.x * 64 + tl;
        if (tq >= T) return;  // (the four lanes of a token leave together)
        float lq[EQ];
#pragma unroll
        for (int j = 0; j < EQ; ++j) lq[j] = tile[tl * LP + sub * EQ + j];
        if (logits_out) {
#pragma unroll
            for (int j = 0; j < EQ; ++j)
                if (sub * EQ + j < E) logits_out[(size_t)tq * E + sub * EQ + j] = lq[j];
        }
        // The scan "first one standing unless a later one is strictly larger" over all experts,
        // taken apart: the largest value that is not a NaN (ties to the lower index) of each
        // quarter, the quarters merged in index order, and at the end the one case in which the
        // scan differs from that: its first allowed expert holds a NaN, which then stands.
        auto pick4 = [&](uint64_t m, int &bi, float &bv) __attribute__((always_inline)) {
            const uint32_t mloc = (uint32_t)(m >> (sub * EQ));
            bi = -1;
            bv = 0.0f;
#pragma unroll
            for (int j = 0; j < EQ; ++j) {
                const bool ok = ((mloc >> j) & 1u) != 0;
                const bool take = ok && (lq[j] > bv || (bi < 0 && lq[j] == lq[j]));
                bv = take ? lq[j] : bv;
                bi = take ? sub * EQ + j : bi;
            }
#pragma unroll
            for (int xr = 1; xr <= 2; xr <<= 1) {
                const int obi = __shfl_xor(bi, xr);
                const float obv = __shfl_xor(bv, xr);
                const bool first = (sub & xr) == 0;  // this lane's part holds the lower indices
                const int abi = first ? bi : obi, bbi = first ? obi : bi;
                const float abv = first ? bv : obv, bbv = first ? obv : bv;
                const bool later = abi < 0 || (bbi >= 0 && bbv > abv);
                bi = later ? bbi : abi;
                bv = later ? bbv : abv;
            }
            if (m != 0) {
                const int f = __ffsll((unsigned long long)m) - 1;
                const float lf = tile[tl * LP + f];
                if (lf != lf) {
                    bi = f;
                    bv = lf;
                }
            }
        };
        int e0;
        float v0;
        pick4(all, e0, v0);
        uint64_t m = mask_tab[e0];
        const float g0 = expf(v0 - v0);  // 1, or NaN when the largest logit is infinite or a NaN
        float den = g0;
        if (sub == 0) {
            topk_idx[(size_t)tq * K] = e0;
            gates[(size_t)tq * K] = g0;
        }
        for (int s = 1; s < K; ++s) {
            int e;
            float v;
            pick4(m, e, v);
            float g = 0.0f;
            if (e >= 0) {
                m &= ~(1ull << e);
                g = expf(v - v0);
            }
            den += g;
            if (sub == 0) {
                topk_idx[(size_t)tq * K + s] = e;
                gates[(size_t)tq * K + s] = g;
            }
        }
        if (sub == 0)
            for (int s = 0; s < K; ++s) gates[(size_t)tq * K + s] = gates[(size_t)tq * K + s] / den;
        return;
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
    const float g0 = expf(v0 - v0);  // 1, or NaN when the largest logit is infinite or a NaN
    float den = g0;
    if (K <= 8) {
        // the usual case: the token's slots stay in registers and leave as 16-byte stores
        int es[8];
        float gs[8];
        es[0] = e0;
        gs[0] = g0;
#pragma unroll
        for (int s = 1; s < 8; ++s) {
            es[s] = -1;
            gs[s] = 0.0f;
            if (s < K) {
                int e;
                float v;
                pick<EP>(l, m, e, v);
                if (e >= 0) {
                    m &= ~(1ull << e);
                    gs[s] = expf(v - v0);
                }
                es[s] = e;
                den += gs[s];
            }
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) gs[s] = gs[s] / den;
        if (K == 4 && ((reinterpret_cast<uintptr_t>(topk_idx) | reinterpret_cast<uintptr_t>(gates)) & 15) == 0) {
            typedef int i32x4 __attribute__((ext_vector_type(4)));
            typedef float f32x4 __attribute__((ext_vector_type(4)));
            const i32x4 ev = {es[0], es[1], es[2], es[3]};
            const f32x4 gv = {gs[0], gs[1], gs[2], gs[3]};
            __builtin_nontemporal_store(ev, reinterpret_cast<i32x4 *>(topk_idx + (size_t)t * 4));
            __builtin_nontemporal_store(gv, reinterpret_cast<f32x4 *>(gates + (size_t)t * 4));
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s)
                if (s < K) {
                    topk_idx[(size_t)t * K + s] = es[s];
                    gates[(size_t)t * K + s] = gs[s];
                }
        }
        return;
    }
    topk_idx[(size_t)t * K] = e0;
    gates[(size_t)t * K] = g0;
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

// Selection from stored logits [T, E] (the profiling pass of Sec. 3.2 routes 2^20 tokens of stored
// router outputs), for E a multiple of 4 and K <= 4.  What the kernel has to do is stream the
// logits, so the arithmetic per token is kept small:
//  * phase 1: a quad of lanes fetches a token's row, lane `sub` the 16-byte pieces at columns
//    16 i + 4 sub (64 contiguous bytes per quad and load, every load of a 64-token group in flight
//    at once), and the values go to LDS transposed, [column][token], the token position XOR-ed with
//    16 sub so that neither these writes nor the reads of phase 2 meet on a bank.
//  * phase 2, one lane per token.  A logit becomes an order-preserving integer (-0 counted as +0)
//    whose low 6 bits are replaced by 63 - column: the largest few of these keys - a chain of one
//    max and a few med3 per value, no index bookkeeping - are the largest logits WITH their
//    columns, ties to the lower column, provided the keys' upper 26 bits differ among the ones
//    kept and the next one below them (then the replaced bits decided nothing).  Without lists the
//    chain keeps five keys of the E columns: the token's K experts and the guard.  With lists it
//    keeps two (top-1 and guard), then walks the top-1's collaborator list ONLY (built once per
//    workgroup from the 64-bit masks, ascending: duplicates, the expert itself and out-of-range
//    entries are gone) keeping four: Tc visits instead of (K - 1) E.
//  * A token that fails the proviso, or has a NaN or an infinity among its logits, takes the
//    literal scan (first one standing unless a later one is strictly larger) for every slot.
// COUNT: the token's expert pairs are added to the co-activation matrix (Eq. 2) on the spot - an LDS
// histogram per workgroup as in coact.hip, one integer atomic per entry at the end - and either
// output may be left out (null): the profiling pass wants the counts, not the selections.
template <int NV, bool LISTS, bool COUNT>
__global__ __launch_bounds__(256) void route_select_rows_kernel(const float *__restrict__ logits, int64_t T, int E, int K,
                                                                const int32_t *__restrict__ collab_idx, int Tc,
                                                                int32_t *__restrict__ topk_idx,
                                                                float *__restrict__ gates, int32_t *__restrict__ Cmat,
                                                                int64_t ngroups) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    // per wave: [column][token ^ 4 * (column >> 2)] floats for 16 NV columns; a power of two, so that
    // offsets inside a tile may be combined with XOR
    constexpr int TILE_BYTES = NV == 1 ? 4096 : NV == 2 ? 8192 : 16384;
    __shared__ __attribute__((aligned(1024))) unsigned char tile_mem[4 * TILE_BYTES];
    __shared__ uint64_t mask_tab[LISTS ? C2R_MAX_E : 1];
    // clist[e][k]: the k-th collaborator c of e (ascending) as the byte offset of its column in a
    // wave's tile, swizzle term included: c * 256 + 64 * ((c >> 2) & 3)
    __shared__ __attribute__((aligned(16))) uint16_t clist[LISTS ? C2R_MAX_E * 64 : 4];
    __shared__ int cnt[LISTS ? C2R_MAX_E : 1];
    __shared__ int maxcnt;
    __shared__ int32_t red[COUNT ? C2R_MAX_E * C2R_MAX_E : 1];  // co-activation counts of this workgroup, red[a][b], a <= b

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint64_t all = E >= 64 ? ~0ull : ((1ull << E) - 1ull);
    auto code_of = [](int c) __attribute__((always_inline)) { return (uint32_t)(c * 256 + ((c >> 2) << 4)); };
    int nmax = 0;
    if constexpr (COUNT) {
        for (int i = tid; i < C2R_MAX_E * C2R_MAX_E; i += 256) red[i] = 0;
        if constexpr (!LISTS) __syncthreads();
    }
    if constexpr (LISTS) {
        if (tid < C2R_MAX_E) mask_tab[tid] = 0ull;
        if (tid == 0) maxcnt = 0;
        for (int i = tid; i < C2R_MAX_E * 64 / 2; i += 256) reinterpret_cast<uint32_t *>(clist)[i] = 0u;
        __syncthreads();
        const int n = E * Tc;
#pragma unroll 4
        for (int i = tid; i < n; i += 256) {
            const int v = collab_idx[i], e = i / Tc;
            if (v >= 0 && v < E && v != e) atomicOr(reinterpret_cast<unsigned long long *>(&mask_tab[e]), 1ull << v);
        }
        __syncthreads();
        if (tid < C2R_MAX_E) {
            uint64_t m = mask_tab[tid];
            int n2 = 0;
            while (m) {
                clist[tid * 64 + n2++] = (uint16_t)code_of(__ffsll((unsigned long long)m) - 1);
                m &= m - 1;
            }
            cnt[tid] = n2;
            atomicMax(&maxcnt, n2);
        }
        __syncthreads();
        nmax = __builtin_amdgcn_readfirstlane(maxcnt);
    }

    constexpr int EMPTY = (int)0x80000000;  // below every key
    // A 64-token group is one contiguous run of 64 E floats = E / 4 wave-wide 16-byte loads; lane l's
    // piece of load u holds columns col .. col + 3 of token tok, the same in every group.  Byte offsets
    // into tile_mem: of that piece's first float (the others follow 256 bytes apart), and of this
    // lane's token for the reads of phase 2.
    const int NU = E / 4;  // <= 4 NV
    uint32_t wr_off[4 * NV];
#pragma unroll
    for (int u = 0; u < 4 * NV; ++u) {
        const int f = u * 256 + lane * 4, tok = (f / E) & 63, col = f - (f / E) * E;
        wr_off[u] = (uint32_t)(wave * TILE_BYTES) + (((uint32_t)(tok * 4)) ^ code_of(col));
    }
    const uint32_t lanebase = (uint32_t)(wave * TILE_BYTES + lane * 4);
    auto lds_f = [&](uint32_t off) __attribute__((always_inline)) -> float & {
        return *reinterpret_cast<float *>(tile_mem + off);
    };
    // this token's logit of column c (any c, per lane)
    auto logit_of = [&](int c) __attribute__((always_inline)) { return lds_f(lanebase ^ code_of(c)); };
    auto key_of = [](float v, int c) __attribute__((always_inline)) {
        const int b = __float_as_int(v);
        return ((b ^ ((b >> 31) & 0x7fffffff)) & ~63) | (63 - c);
    };
    auto med3 = [](int a, int b, int c) __attribute__((always_inline)) {
        int d;
        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
        return d;
    };

    // all loads of a 64-token group go out together (a piece past the end of the logits re-reads the start)
    f32x4 q[4 * NV];
    auto request = [&](int64_t g) __attribute__((always_inline)) {
        const int64_t left = T - g * 64;
        const int nflt = (int)(left < 64 ? left : 64) * E;
        const float *base = logits + g * 64 * E;
#pragma unroll
        for (int u = 0; u < 4 * NV; ++u) {
            const int f = u * 256 + lane * 4;
            if (u < 4 * NV - 3 || u < NU)  // (uniform)
                q[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(base + (f < nflt ? f : 0)));
        }
    };
    const int64_t gstep = (int64_t)gridDim.x * 4;
    int64_t g = (int64_t)blockIdx.x * 4 + wave;
    if (g < ngroups) request(g);
    for (; g < ngroups; g += gstep) {
        // ---- phase 1: the group's logits into LDS, transposed (-0 stored as +0)
#pragma unroll
        for (int u = 0; u < 4 * NV; ++u)
            if (u < 4 * NV - 3 || u < NU) {
#pragma unroll
                for (int j = 0; j < 4; ++j) lds_f(wr_off[u] + j * 256) = q[u][j] + 0.0f;
            }
        // ... and the next group's go out and fly while phase 2 runs (two groups of a wave in flight,
        // with a second register set and the loop body twice, measured slower: 72 against 65 us)
        if (g + gstep < ngroups) request(g + gstep);
        // (the wave's own LDS writes, read back by other lanes of the same wave: LDS operations of a
        // wave complete in order; the fences keep the compiler from moving them)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- phase 2: one lane per token
        const int64_t t = g * 64 + lane;
        constexpr int NKEEP = LISTS ? 2 : 5;
        int k[NKEEP];
#pragma unroll
        for (int u = 0; u < NKEEP; ++u) k[u] = EMPTY;
        float chk = 0.0f;
#pragma unroll
        for (int c = 0; c < NV * 16; ++c) {
            if (c < (NV - 1) * 16 || c < E) {  // (uniform)
                const float v = lds_f((lanebase ^ (uint32_t)((c >> 2) << 4)) + c * 256);
                chk = __builtin_fmaf(v, 0.0f, chk);  // NaN once a NaN or an infinity went in
                const int kk = key_of(v, c);
                int nk[NKEEP];
                nk[0] = max(k[0], kk);
#pragma unroll
                for (int u = 1; u < NKEEP; ++u) nk[u] = med3(k[u - 1], k[u], kk);  // (k[0] >= k[1] >= ... throughout)
#pragma unroll
                for (int u = 0; u < NKEEP; ++u) k[u] = nk[u];
            }
        }
        bool literal = chk != chk;
#pragma unroll
        for (int u = 0; u + 1 < NKEEP; ++u) literal = literal || !((k[u] >> 6) > (k[u + 1] >> 6) || k[u] == EMPTY);
        int es[4] = {-1, -1, -1, -1};
        float vs[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        es[0] = 63 - (k[0] & 63);
        if constexpr (LISTS) {
            // the top-1's list: four keys kept, the three slots and the guard
            const int n = cnt[es[0]];
            const uint16_t *lst = clist + es[0] * 64;
            int m[4] = {EMPTY, EMPTY, EMPTY, EMPTY};
            for (int kq = 0; kq < nmax; kq += 4) {
                const uint2 w = *reinterpret_cast<const uint2 *>(lst + kq);
                uint32_t code[4] = {w.x & 0xffffu, w.x >> 16, w.y & 0xffffu, w.y >> 16};
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = lds_f(lanebase ^ code[j]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int kk = kq + j < n ? key_of(v[j], (int)(code[j] >> 8)) : EMPTY;
                    const int n0 = max(m[0], kk), n1 = med3(m[0], m[1], kk), n2 = med3(m[1], m[2], kk),
                              n3 = med3(m[2], m[3], kk);
                    m[0] = n0;
                    m[1] = n1;
                    m[2] = n2;
                    m[3] = n3;
                }
            }
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                literal = literal || !((m[u] >> 6) > (m[u + 1] >> 6) || m[u] == EMPTY);
                es[u + 1] = m[u] == EMPTY ? -1 : 63 - (m[u] & 63);
            }
        } else {
#pragma unroll
            for (int u = 1; u < 4; ++u) es[u] = k[u] == EMPTY ? -1 : 63 - (k[u] & 63);
        }
        float gs[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        float den = 1.0f;
        if (literal) {
            // the literal scan, slot by slot (a NaN stands if it is the first allowed expert)
            auto pick_row = [&](uint64_t mm, int &bi, float &bv) {
                bi = -1;
                bv = 0.0f;
                for (int e = 0; e < E; ++e) {
                    const float v = logit_of(e);
                    const bool take = ((mm >> e) & 1ull) != 0 && (bi < 0 || v > bv);
                    bv = take ? v : bv;
                    bi = take ? e : bi;
                }
            };
            int e0;
            float v0;
            pick_row(all, e0, v0);
            uint64_t mm = all & ~(1ull << e0);
            if constexpr (LISTS) mm = mask_tab[e0];
            es[0] = e0;
            gs[0] = expf(v0 - v0);
            den = gs[0];
#pragma unroll
            for (int s2 = 1; s2 < 4; ++s2) {
                es[s2] = -1;
                if (s2 < K) {
                    int e;
                    float v;
                    pick_row(mm, e, v);
                    if (e >= 0) {
                        mm &= ~(1ull << e);
                        gs[s2] = expf(v - v0);
                    }
                    es[s2] = e;
                    den += gs[s2];
                }
            }
        } else {
#pragma unroll
            for (int s2 = 1; s2 < 4; ++s2)
                if (s2 >= K) es[s2] = -1;
            if (gates) {  // (uniform)
#pragma unroll
                for (int s2 = 0; s2 < 4; ++s2) vs[s2] = logit_of(es[s2] < 0 ? 0 : es[s2]);
                gs[0] = expf(vs[0] - vs[0]);
                den = gs[0];
#pragma unroll
                for (int s2 = 1; s2 < 4; ++s2)
                    if (s2 < K) {
                        if (es[s2] >= 0) gs[s2] = expf(vs[s2] - vs[0]);
                        den += gs[s2];
                    }
            }
        }
        if (t < T) {
            const bool vec = K == 4 && ((reinterpret_cast<uintptr_t>(topk_idx) | reinterpret_cast<uintptr_t>(gates)) & 15) == 0;
            if (topk_idx) {
                if (vec) {
                    const i32x4 ev = {es[0], es[1], es[2], es[3]};
                    __builtin_nontemporal_store(ev, reinterpret_cast<i32x4 *>(topk_idx + (size_t)t * 4));
                } else {
#pragma unroll
                    for (int s2 = 0; s2 < 4; ++s2)
                        if (s2 < K) topk_idx[(size_t)t * K + s2] = es[s2];
                }
            }
            if (gates) {
#pragma unroll
                for (int s2 = 0; s2 < 4; ++s2) gs[s2] = gs[s2] / den;
                if (vec) {
                    const f32x4 gv = {gs[0], gs[1], gs[2], gs[3]};
                    __builtin_nontemporal_store(gv, reinterpret_cast<f32x4 *>(gates + (size_t)t * 4));
                } else {
#pragma unroll
                    for (int s2 = 0; s2 < 4; ++s2)
                        if (s2 < K) gates[(size_t)t * K + s2] = gs[s2];
                }
            }
            if constexpr (COUNT) {
                // Eq. 2: one count for every pair a <= b of the token's experts, the diagonal included,
                // into the workgroup's histogram (upper triangle)
                uint64_t ma = 0;
#pragma unroll
                for (int s2 = 0; s2 < 4; ++s2)
                    if (es[s2] >= 0) ma |= 1ull << es[s2];
                while (ma) {
                    const int ea = __ffsll((unsigned long long)ma) - 1;
                    uint64_t mb = ma;
                    ma &= ma - 1;
                    while (mb) {
                        const int eb = __ffsll((unsigned long long)mb) - 1;
                        mb &= mb - 1;
                        atomicAdd(&red[ea * C2R_MAX_E + eb], 1);
                    }
                }
            }
        }
        // the next group's logits overwrite the tile: every lane's reads of it come first
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    if constexpr (COUNT) {
        __syncthreads();
        for (int i = tid; i < E * E; i += 256) {
            const int r = i / E, c = i - r * E;
            const int32_t v = red[(r < c ? r : c) * C2R_MAX_E + (r < c ? c : r)];
            if (v) atomicAdd(&Cmat[i], v);
        }
    }
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
    int EP, nchunk;
    int64_t Tpad;
    size_t part_bytes, wpad_bytes;
};

static RouteLayout route_layout(int64_t T, int d, int E) {
    RouteLayout L;
    L.EP = ep_of(E);
    L.nchunk = (d + C2R_CANON_CHUNK - 1) / C2R_CANON_CHUNK;
    if (L.nchunk < 1) L.nchunk = 1;
    L.Tpad = (T + 63) / 64 * 64;
    L.part_bytes = round_up((size_t)L.nchunk * L.EP * (size_t)L.Tpad * sizeof(float), 256);
    L.wpad_bytes = (E % 4) ? round_up((size_t)d * L.EP * sizeof(float), 256) : 0;
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
    drop_stale_error();
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
    int ldw = E;
    if (L.wpad_bytes) {
        float *Wp = reinterpret_cast<float *>(static_cast<char *>(ws) + L.part_bytes);
        const int64_t n = (int64_t)d * L.EP;
        pack_router_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(Wg, d, E, L.EP, Wp);
        W = Wp;
        ldw = L.EP;
    } else if (!aligned(Wg, 16)) {
        return C2R_ERR_INVALID_ARG;
    }
    const int64_t ntiles = L.Tpad / 64;
    // Four waves per workgroup share the W sub-tiles.  On the matrix pipe a wave tile is always
    // 32 tokens (the pipelined form of the kernel; at E = 60, d = 2048 it beats 64-token tiles
    // at every batch size: 191 vs 238 us for the stage at T = 65536).  On the vector pipe a batch
    // with fewer than two 64-token wave tiles per SIMD of the chip uses half-size wave tiles:
    // with one wave per SIMD nothing hides its latencies.
    const int te = L.EP > 32 ? 8 : L.EP > 16 ? 4 : L.EP > 8 ? 2 : 1;
    const bool wide = ntiles * L.nchunk >= 2048 && te == 1;
    constexpr int NWV = 4;
    const int64_t nwt = wide ? ntiles : ntiles * 2;
    // With at least one 32-token wave tile per SIMD of the chip (1024), a workgroup on the matrix
    // pipe walks all the chunks of its tokens and keeps the running sum in registers: scratch then
    // holds ONE vector per token instead of one per chunk.  Smaller batches need the chunks as
    // separate workgroups to fill the chip.
    const bool all_chunks = !wide && te > 1 && nwt >= 1024 && L.nchunk > 1;
    const int nchunk_out = all_chunks ? 1 : L.nchunk;
    const int64_t nblk = (nwt + NWV - 1) / NWV * nchunk_out;
    if (nblk >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    // more than 8 experts: the matrix pipe, a wave covering 32 or 64 experts (columns past the packed
    // expert count re-read column 0; their sums are never stored)
#define C2R_ROUTE_LAUNCH(BF, TE, NWV, TQ, MF)                                                     \
    route_partial_kernel<BF, TE, NWV, TQ, MF><<<dim3((unsigned)nblk), dim3(NWV * 64), 0, st>>>(    \
        x, W, ldw, L.EP, T, d, L.nchunk, ntiles, part)
#define C2R_ROUTE_LAUNCH_ALL(BF, TE, NWV, TQ)                                                          \
    route_partial_kernel<BF, TE, NWV, TQ, true, true><<<dim3((unsigned)nblk), dim3(NWV * 64), 0, st>>>(  \
        x, W, ldw, L.EP, T, d, L.nchunk, ntiles, part)
#define C2R_ROUTE_TE(BF, NWV, TQ)                                     \
    if (all_chunks) {                                                 \
        if (te == 8) { C2R_ROUTE_LAUNCH_ALL(BF, 8, NWV, TQ); }        \
        else { C2R_ROUTE_LAUNCH_ALL(BF, 4, NWV, TQ); }                \
    } else                                                            \
    switch (te) {                                                     \
        case 8: C2R_ROUTE_LAUNCH(BF, 8, NWV, TQ, true); break;        \
        case 4: C2R_ROUTE_LAUNCH(BF, 4, NWV, TQ, true); break;        \
        case 2: C2R_ROUTE_LAUNCH(BF, 4, NWV, TQ, true); break;        \
        default: C2R_ROUTE_LAUNCH(BF, 1, NWV, TQ, false); break;      \
    }
    if (x_dt == C2R_BF16) {
        if (wide) { C2R_ROUTE_LAUNCH(true, 1, NWV, 8, false); } else { C2R_ROUTE_TE(true, NWV, 4) }
    } else {
        if (wide) { C2R_ROUTE_LAUNCH(false, 1, NWV, 8, false); } else { C2R_ROUTE_TE(false, NWV, 4) }
    }
#undef C2R_ROUTE_TE
#undef C2R_ROUTE_LAUNCH_ALL
#undef C2R_ROUTE_LAUNCH
    C2R_EP_SWITCH(L.EP, route_select_kernel<EP, false><<<dim3((unsigned)ntiles), dim3(SEL_WAVES * 64), 0, st>>>(
                            part, nchunk_out, bias, T, E, K, collab_idx, Tc, topk_idx, gates, logits_out));
    return launch_status();
}

// Selection from stored logits; with Cmat the tokens' expert pairs are counted as well (then topk_idx
// and gates may be null where the fused kernel runs: E a multiple of 4, K <= 4).
static int route_from_logits_impl(const float *logits, int64_t T, int E, int K, const int32_t *collab_idx, int Tc,
                                  int32_t *topk_idx, float *gates, int32_t *Cmat, hipStream_t st) {
    const int64_t nsel = (T + 63) / 64;
    if (nsel >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    if (E % 4 == 0 && K <= 4) {
        // few, long-lived workgroups: each builds the collaborator lists once and then walks its groups
        // (as many as fit a CU's LDS at once: two with 64-column tiles, four with 32 columns or fewer)
        const int64_t cap = E <= 32 ? 1024 : 512;
        const int64_t nblk = (nsel + 3) / 4 < cap ? (nsel + 3) / 4 : cap;
        const dim3 grid((unsigned)nblk), block(256);
#define C2R_ROWS_ARGS logits, T, E, K, collab_idx, Tc, topk_idx, gates, Cmat, nsel
#define C2R_ROWS_LAUNCH(NVV)                                                               \
    if (Cmat) {                                                                            \
        if (collab_idx)                                                                    \
            route_select_rows_kernel<NVV, true, true><<<grid, block, 0, st>>>(C2R_ROWS_ARGS);   \
        else                                                                               \
            route_select_rows_kernel<NVV, false, true><<<grid, block, 0, st>>>(C2R_ROWS_ARGS);  \
    } else if (collab_idx)                                                                 \
        route_select_rows_kernel<NVV, true, false><<<grid, block, 0, st>>>(C2R_ROWS_ARGS);      \
    else                                                                                   \
        route_select_rows_kernel<NVV, false, false><<<grid, block, 0, st>>>(C2R_ROWS_ARGS)
        switch ((E + 15) / 16) {
            case 1: C2R_ROWS_LAUNCH(1); break;
            case 2: C2R_ROWS_LAUNCH(2); break;
            case 3: C2R_ROWS_LAUNCH(3); break;
            default: C2R_ROWS_LAUNCH(4); break;
        }
#undef C2R_ROWS_LAUNCH
#undef C2R_ROWS_ARGS
        return launch_status();
    }
    if (!topk_idx || !gates) return C2R_ERR_UNSUPPORTED;
    const int EPV = ep_of(E);
    C2R_EP_SWITCH(EPV, route_select_kernel<EP, true><<<dim3((unsigned)nsel), dim3(64), 0, st>>>(
                           logits, 1, (const float *)nullptr, T, E, K, collab_idx, Tc, topk_idx, gates,
                           (float *)nullptr));
    const int rc = launch_status();
    if (rc != C2R_OK || !Cmat) return rc;
    return c2r_build_coactivation(topk_idx, T, K, E, Cmat, st);
}

extern "C" int c2r_route_from_logits(const float *logits, int64_t T, int E, int K,
                                     const int32_t *collab_idx, int Tc, int32_t *topk_idx,
                                     float *gates, void *stream) {
    drop_stale_error();
    int rc = check_route_args(T, E, K, collab_idx, Tc);
    if (rc != C2R_OK) return rc;
    if (T == 0) return C2R_OK;
    if (!logits || !topk_idx || !gates) return C2R_ERR_INVALID_ARG;
    if (!aligned(logits, 16)) return C2R_ERR_INVALID_ARG;
    return route_from_logits_impl(logits, T, E, K, collab_idx, Tc, topk_idx, gates, nullptr,
                                  static_cast<hipStream_t>(stream));
}

extern "C" int c2r_profile_from_logits(const float *logits, int64_t T, int E, int K,
                                       const int32_t *collab_idx, int Tc, int32_t *topk_idx,
                                       float *gates, int32_t *C, void *stream) {
    drop_stale_error();
    int rc = check_route_args(T, E, K, collab_idx, Tc);
    if (rc != C2R_OK) return rc;
    if (T == 0) return C2R_OK;
    if (!logits || !C) return C2R_ERR_INVALID_ARG;
    if (!aligned(logits, 16) || !aligned(C, 4)) return C2R_ERR_INVALID_ARG;
    if (topk_idx && !aligned(topk_idx, 4)) return C2R_ERR_INVALID_ARG;
    return route_from_logits_impl(logits, T, E, K, collab_idx, Tc, topk_idx, gates, C,
                                  static_cast<hipStream_t>(stream));
}
