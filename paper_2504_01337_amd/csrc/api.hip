// Host entry points that do not belong to a single kernel file: version,
// workspace query, and the expert-FFN dispatcher (fp32 vector path / bf16 MFMA path).
#include "c2r_internal.h"

namespace c2r {
size_t route_workspace_bytes(int64_t T, int d, int E);
size_t permute_workspace_bytes(int64_t T, int E, int K);
size_t dedup_workspace_bytes(int64_t T, int n_dev);
int launch_ffn_f32_pass(int pass, const float *a, const int32_t *offsets, int E_local, int64_t A_cap, int d,
                        int F, const float *b0, const float *b1, float *out, hipStream_t st);
int launch_ffn_bf16_pass(int pass, const uint16_t *a, const int32_t *offsets, int E_local, int64_t A_cap, int d,
                         int F, const uint16_t *b0, const uint16_t *b1, uint16_t *out, hipStream_t st);
int launch_ffn_bf16_dma_pass(int pass, const uint16_t *a, int lda, const int32_t *offsets, int E_local,
                             int64_t A_cap, int d, int F, const uint16_t *b0, const uint16_t *b1,
                             uint16_t *out, int ldo, const int32_t *gather, int gather_div, int gather_rows,
                             hipStream_t st);
struct FfnProblem;
}  // namespace c2r
#include "ffn_common.h"
namespace c2r {
FfnProblem ffn_bf16_dma_problem(int pass, const uint16_t *a, int lda, const int32_t *offsets, int E_local,
                                int64_t A_cap, int d, int F, const uint16_t *b0, const uint16_t *b1, uint16_t *out,
                                int ldo, const int32_t *gather, int gather_div, int gather_rows);
int launch_ffn_bf16_dma(int pass, const FfnProblem &first, const FfnProblem *second, hipStream_t st);
}  // namespace c2r

using namespace c2r;

// Row pitch of the hidden activation h inside the library's own workspace: padded to the
// k-slice of the fast bf16 path (the padding is kept at zero by the first pass).
static bool fast_bf16(c2r_dtype dt, int d, int F) {
    // the copy-engine kernel: bf16 and a model width of whole 64-element k-slices (F is
    // padded to such slices inside the workspace)
    (void)F;
    return dt == C2R_BF16 && d % 64 == 0;
}

static int h_pitch(c2r_dtype dt, int d, int F) { return fast_bf16(dt, d, F) ? (F + 63) / 64 * 64 : F; }

extern "C" int c2r_version(void) { return 100; }

extern "C" size_t c2r_workspace_bytes(int stage, int64_t T, int d, int E, int K, int F, c2r_dtype dt) {
    switch (stage) {
        case C2R_STAGE_COACTIVATION:
            return 0;
        case C2R_STAGE_ROUTE:
            return route_workspace_bytes(T, d, E);
        case C2R_STAGE_PERMUTE:
            return permute_workspace_bytes(T, E, K);
        case C2R_STAGE_EXPERT_FFN: {
            if (T <= 0 || F <= 0) return 0;
            const size_t sz = dt == C2R_BF16 ? 2 : 4;
            return round_up((size_t)T * (size_t)(K > 0 ? K : 1) * (size_t)h_pitch(dt, d, F) * sz, 256);
        }
        case C2R_STAGE_DEDUP_DISPATCH:
            return dedup_workspace_bytes(T, E);  // E: number of devices
        default:
            return 0;
    }
}

static int check_ffn(c2r_dtype dt, int E_local, int64_t A_cap, int d, int F) {
    if (E_local < 1 || A_cap < 0 || d < 1 || F < 1) return C2R_ERR_INVALID_ARG;
    if (dt != C2R_F32 && dt != C2R_BF16) return C2R_ERR_INVALID_ARG;
    if (E_local > C2R_MAX_E) return C2R_ERR_UNSUPPORTED;
    if (A_cap >= (1ll << 31)) return C2R_ERR_UNSUPPORTED;
    if (d % 8 != 0 || F % 8 != 0) return C2R_ERR_UNSUPPORTED;
    const size_t sz = dt == C2R_BF16 ? 2 : 4;
    // 32-bit byte offsets are used inside one tile's rows and inside one expert's weights
    if ((size_t)d * F * sz >= (1ull << 32) || 256ull * (d > F ? d : F) * sz >= (1ull << 32))
        return C2R_ERR_UNSUPPORTED;
    return C2R_OK;
}

// ldh: pitch of h (output of pass 0, input of pass 1).  The copy-engine path needs the
// contraction rows of A padded to a multiple of 64 elements.
static int ffn_pass(int pass, c2r_dtype dt, const void *a, const int32_t *offsets, int E_local, int64_t A_cap,
                    int d, int F, int ldh, const void *b0, const void *b1, void *out, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (fast_bf16(dt, d, F) && ldh % 64 == 0)
        return launch_ffn_bf16_dma_pass(pass, static_cast<const uint16_t *>(a), pass == 0 ? d : ldh, offsets,
                                        E_local, A_cap, d, F, static_cast<const uint16_t *>(b0),
                                        static_cast<const uint16_t *>(b1), static_cast<uint16_t *>(out),
                                        pass == 0 ? ldh : d, nullptr, 1, 1, st);
    if (ldh != F) return C2R_ERR_UNSUPPORTED;
    if (dt == C2R_BF16)
        return launch_ffn_bf16_pass(pass, static_cast<const uint16_t *>(a), offsets, E_local, A_cap, d, F,
                                    static_cast<const uint16_t *>(b0), static_cast<const uint16_t *>(b1),
                                    static_cast<uint16_t *>(out), st);
    return launch_ffn_f32_pass(pass, static_cast<const float *>(a), offsets, E_local, A_cap, d, F,
                               static_cast<const float *>(b0), static_cast<const float *>(b1),
                               static_cast<float *>(out), st);
}

extern "C" int c2r_expert_ffn_gate_up(const void *x_perm, c2r_dtype dt, const int32_t *offsets, int E_local,
                                      int64_t A_cap, int d, int F, const void *w_gate, const void *w_up,
                                      void *h, void *stream) {
    const int rc = check_ffn(dt, E_local, A_cap, d, F);
    if (rc != C2R_OK) return rc;
    if (A_cap == 0) return C2R_OK;
    if (!x_perm || !offsets || !w_gate || !w_up || !h) return C2R_ERR_INVALID_ARG;
    if (!aligned(x_perm, 16) || !aligned(w_gate, 16) || !aligned(w_up, 16) || !aligned(h, 16))
        return C2R_ERR_INVALID_ARG;
    return ffn_pass(0, dt, x_perm, offsets, E_local, A_cap, d, F, F, w_gate, w_up, h, stream);
}

extern "C" int c2r_expert_ffn_gate_up_gather(const void *x, c2r_dtype dt, const int32_t *perm, int64_t T, int K,
                                             const int32_t *offsets, int E_local, int64_t A_cap, int d, int F,
                                             const void *w_gate, const void *w_up, void *h, void *stream) {
    const int rc = check_ffn(dt, E_local, A_cap, d, F);
    if (rc != C2R_OK) return rc;
    if (T < 1 || K < 1) return C2R_ERR_INVALID_ARG;
    if (A_cap == 0) return C2R_OK;
    if (!x || !perm || !offsets || !w_gate || !w_up || !h) return C2R_ERR_INVALID_ARG;
    if (!aligned(x, 16) || !aligned(w_gate, 16) || !aligned(w_up, 16) || !aligned(h, 16))
        return C2R_ERR_INVALID_ARG;
    // only the copy-engine kernel folds the gather into its addresses (32-bit row offsets into x)
    if (!fast_bf16(dt, d, F) || F % 64 != 0 || (uint64_t)T * d * 2 >= (1ull << 32)) return C2R_ERR_UNSUPPORTED;
    return launch_ffn_bf16_dma_pass(0, static_cast<const uint16_t *>(x), d, offsets, E_local, A_cap, d, F,
                                    static_cast<const uint16_t *>(w_gate), static_cast<const uint16_t *>(w_up),
                                    static_cast<uint16_t *>(h), F, perm, K, (int)T, static_cast<hipStream_t>(stream));
}

extern "C" int c2r_expert_ffn_down(const void *h, c2r_dtype dt, const int32_t *offsets, int E_local,
                                   int64_t A_cap, int d, int F, const void *w_down, void *y_perm,
                                   void *stream) {
    const int rc = check_ffn(dt, E_local, A_cap, d, F);
    if (rc != C2R_OK) return rc;
    if (A_cap == 0) return C2R_OK;
    if (!h || !offsets || !w_down || !y_perm) return C2R_ERR_INVALID_ARG;
    if (!aligned(h, 16) || !aligned(w_down, 16) || !aligned(y_perm, 16)) return C2R_ERR_INVALID_ARG;
    return ffn_pass(1, dt, h, offsets, E_local, A_cap, d, F, F, w_down, nullptr, y_perm, stream);
}

extern "C" int c2r_expert_ffn(const void *x_perm, c2r_dtype dt, const int32_t *offsets, int E_local,
                              int64_t A_cap, int d, int F, const void *w_gate, const void *w_up,
                              const void *w_down, void *y_perm, void *ws, size_t ws_bytes,
                              void *stream) {
    int rc = check_ffn(dt, E_local, A_cap, d, F);
    if (rc != C2R_OK) return rc;
    if (A_cap == 0) return C2R_OK;
    if (!x_perm || !offsets || !w_gate || !w_up || !w_down || !y_perm) return C2R_ERR_INVALID_ARG;
    if (!aligned(x_perm, 16) || !aligned(w_gate, 16) || !aligned(w_up, 16) || !aligned(w_down, 16) ||
        !aligned(y_perm, 16))
        return C2R_ERR_INVALID_ARG;
    const int ldh = h_pitch(dt, d, F);
    const size_t need = round_up((size_t)A_cap * ldh * (dt == C2R_BF16 ? 2 : 4), 256);
    if (!ws || ws_bytes < need || !aligned(ws, 256)) return C2R_ERR_WORKSPACE;
    rc = ffn_pass(0, dt, x_perm, offsets, E_local, A_cap, d, F, ldh, w_gate, w_up, ws, stream);
    if (rc != C2R_OK) return rc;
    return ffn_pass(1, dt, ws, offsets, E_local, A_cap, d, F, ldh, w_down, nullptr, y_perm, stream);
}

extern "C" int c2r_expert_ffn_gather(const void *x, c2r_dtype dt, const int32_t *perm, int64_t T, int K,
                                     const int32_t *offsets, int E_local, int64_t A_cap, int d, int F,
                                     const void *w_gate, const void *w_up, const void *w_down, void *y_perm,
                                     void *ws, size_t ws_bytes, void *stream) {
    int rc = check_ffn(dt, E_local, A_cap, d, F);
    if (rc != C2R_OK) return rc;
    if (T < 1 || K < 1) return C2R_ERR_INVALID_ARG;
    if (A_cap == 0) return C2R_OK;
    if (!x || !perm || !offsets || !w_gate || !w_up || !w_down || !y_perm) return C2R_ERR_INVALID_ARG;
    if (!aligned(x, 16) || !aligned(w_gate, 16) || !aligned(w_up, 16) || !aligned(w_down, 16) || !aligned(y_perm, 16))
        return C2R_ERR_INVALID_ARG;
    // only the copy-engine kernel folds the gather into its addresses (32-bit row offsets into x)
    if (!fast_bf16(dt, d, F) || (uint64_t)T * d * 2 >= (1ull << 32)) return C2R_ERR_UNSUPPORTED;
    const int ldh = h_pitch(dt, d, F);
    const size_t need = round_up((size_t)A_cap * ldh * 2, 256);
    if (!ws || ws_bytes < need || !aligned(ws, 256)) return C2R_ERR_WORKSPACE;
    rc = launch_ffn_bf16_dma_pass(0, static_cast<const uint16_t *>(x), d, offsets, E_local, A_cap, d, F,
                                  static_cast<const uint16_t *>(w_gate), static_cast<const uint16_t *>(w_up),
                                  static_cast<uint16_t *>(ws), ldh, perm, K, (int)T, static_cast<hipStream_t>(stream));
    if (rc != C2R_OK) return rc;
    return ffn_pass(1, dt, ws, offsets, E_local, A_cap, d, F, ldh, w_down, nullptr, y_perm, stream);
}

// ---- routed groups and an always-on shared expert in ONE launch per pass ----
static int check_with_shared(c2r_dtype dt, int64_t T, int E_local, int64_t A_cap, int d, int F, int F_shared) {
    int rc = check_ffn(dt, E_local, A_cap, d, F);
    if (rc != C2R_OK) return rc;
    if (T < 1 || F_shared < 1) return C2R_ERR_INVALID_ARG;
    rc = check_ffn(dt, 1, T, d, F_shared);
    if (rc != C2R_OK) return rc;
    if (dt != C2R_BF16 || d % 64 != 0 || F % 64 != 0 || F_shared % 64 != 0) return C2R_ERR_UNSUPPORTED;
    if ((uint64_t)T * d * 2 >= (1ull << 32)) return C2R_ERR_UNSUPPORTED;
    return C2R_OK;
}

extern "C" int c2r_expert_ffn_gate_up_with_shared(const void *x, c2r_dtype dt, const int32_t *perm, int64_t T, int K,
                                                  const int32_t *offsets, int E_local, int64_t A_cap, int d, int F,
                                                  const void *w_gate, const void *w_up, void *h, int F_shared,
                                                  const void *ws_gate, const void *ws_up, void *h_shared,
                                                  void *stream) {
    const int rc = check_with_shared(dt, T, E_local, A_cap, d, F, F_shared);
    if (rc != C2R_OK) return rc;
    if (K < 1) return C2R_ERR_INVALID_ARG;
    if (!x || !ws_gate || !ws_up || !h_shared) return C2R_ERR_INVALID_ARG;
    if (A_cap > 0 && (!perm || !offsets || !w_gate || !w_up || !h)) return C2R_ERR_INVALID_ARG;
    if (!aligned(x, 16) || !aligned(w_gate, 16) || !aligned(w_up, 16) || !aligned(h, 16) || !aligned(ws_gate, 16) ||
        !aligned(ws_up, 16) || !aligned(h_shared, 16))
        return C2R_ERR_INVALID_ARG;
    const uint16_t *xs = static_cast<const uint16_t *>(x);
    const FfnProblem shared = ffn_bf16_dma_problem(0, xs, d, nullptr, 1, T, d, F_shared,
                                                   static_cast<const uint16_t *>(ws_gate),
                                                   static_cast<const uint16_t *>(ws_up),
                                                   static_cast<uint16_t *>(h_shared), F_shared, nullptr, 1, 1);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (A_cap == 0) return launch_ffn_bf16_dma(0, shared, nullptr, st);
    const FfnProblem routed = ffn_bf16_dma_problem(0, xs, d, offsets, E_local, A_cap, d, F,
                                                   static_cast<const uint16_t *>(w_gate),
                                                   static_cast<const uint16_t *>(w_up), static_cast<uint16_t *>(h), F,
                                                   perm, K, (int)T);
    return launch_ffn_bf16_dma(0, routed, &shared, st);
}

extern "C" int c2r_expert_ffn_down_with_shared(const void *h, c2r_dtype dt, const int32_t *offsets, int E_local,
                                               int64_t A_cap, int d, int F, const void *w_down, void *y_perm,
                                               int64_t T, int F_shared, const void *h_shared, const void *ws_down,
                                               void *y_shared, void *stream) {
    const int rc = check_with_shared(dt, T, E_local, A_cap, d, F, F_shared);
    if (rc != C2R_OK) return rc;
    if (!h_shared || !ws_down || !y_shared) return C2R_ERR_INVALID_ARG;
    if (A_cap > 0 && (!h || !offsets || !w_down || !y_perm)) return C2R_ERR_INVALID_ARG;
    if (!aligned(h, 16) || !aligned(w_down, 16) || !aligned(y_perm, 16) || !aligned(h_shared, 16) ||
        !aligned(ws_down, 16) || !aligned(y_shared, 16))
        return C2R_ERR_INVALID_ARG;
    const FfnProblem shared = ffn_bf16_dma_problem(1, static_cast<const uint16_t *>(h_shared), F_shared, nullptr, 1, T, d,
                                                   F_shared, static_cast<const uint16_t *>(ws_down), nullptr,
                                                   static_cast<uint16_t *>(y_shared), d, nullptr, 1, 1);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (A_cap == 0) return launch_ffn_bf16_dma(1, shared, nullptr, st);
    const FfnProblem routed = ffn_bf16_dma_problem(1, static_cast<const uint16_t *>(h), F, offsets, E_local, A_cap, d, F,
                                                   static_cast<const uint16_t *>(w_down), nullptr,
                                                   static_cast<uint16_t *>(y_perm), d, nullptr, 1, 1);
    return launch_ffn_bf16_dma(1, routed, &shared, st);
}
