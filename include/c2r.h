/*
 * c2r.h - C ABI of the MI355X (gfx950) hot path of a collaboration-constrained
 * routing (C2R) Mixture-of-Experts layer, after arXiv 2504.01337.
 *
 * Notation follows the paper where it has one: x is a token's hidden state,
 * W_g the router weight (Eq. 1), N (here E) the number of experts, K the
 * experts per token, C the expert collaboration matrix (Eq. 2), T (here Tc)
 * the length of the collaborator list Top-T(E_i) (Eq. 4).
 *
 * Conventions shared by every call
 *  - Every pointer is a DEVICE pointer owned by the caller unless it says
 *    "host".  The library never allocates, frees or keeps a pointer.
 *  - Row-major everywhere.  Indices are int32; token counts are int64.
 *  - `stream` is a hipStream_t passed as void*.  All work is enqueued on it and
 *    the call returns without synchronising; stages enqueued on one stream run
 *    in order, so a layer needs no host synchronisation between stages.
 *  - Scratch memory comes from the caller: ask c2r_workspace_bytes() for the
 *    stage and pass at least that many bytes, 256-byte aligned.
 *  - Return value: C2R_OK or a negative c2r_status.  Arguments are checked on
 *    the host before anything is launched; on error nothing was enqueued.
 *    Expert indices and group offsets that live in device memory are range
 *    checked inside the kernels (out-of-range experts are skipped, offsets are
 *    clamped to the stated capacity).  inv_perm entries are trusted to be < the
 *    number of rows of y_perm, as c2r_permute writes them.
 *  - Implemented limits: E <= 64, K <= E, T*K < 2^31, and row sizes (d, F) that
 *    are multiples of 8 elements.  Outside them: C2R_ERR_UNSUPPORTED.
 */
#ifndef C2R_H
#define C2R_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { C2R_F32 = 0, C2R_BF16 = 1 } c2r_dtype;

typedef enum {
    C2R_OK = 0,
    C2R_ERR_INVALID_ARG = -1, /* null pointer, K < 1, K > E, Tc < K-1, misaligned pointer ... */
    C2R_ERR_UNSUPPORTED = -2, /* outside the implemented limits listed above */
    C2R_ERR_WORKSPACE = -3,   /* workspace missing or smaller than c2r_workspace_bytes() */
    C2R_ERR_LAUNCH = -4       /* the HIP runtime refused a launch (hipGetLastError kept) */
} c2r_status;

typedef enum {
    C2R_STAGE_COACTIVATION = 0,
    C2R_STAGE_ROUTE = 1,
    C2R_STAGE_PERMUTE = 2,
    C2R_STAGE_EXPERT_FFN = 3,
    C2R_STAGE_DEDUP_DISPATCH = 4 /* pass the number of devices as E */
} c2r_stage;

/* Library version (major*10000 + minor*100 + patch). */
int c2r_version(void);

/*
 * Length of the k-chunks of the router's summation order, a fixed constant of
 * the ABI (256).  c2r_route computes every logit of Eq. 1 in fp32 as follows:
 * k = 0..d-1 is cut into consecutive chunks of this length; inside a chunk one
 * fused multiply-add per element, acc = fma(x[t,k], W_g[k,e], acc), ascending k,
 * starting from +0; the chunk results are added left to right; the bias, if
 * any, is added last.  An implementation of this order on another machine
 * reproduces the logits, hence the selections, bit for bit.
 */
int c2r_route_chunk(void);

/*
 * Bytes of caller-provided scratch a stage needs for the given sizes (0 when it
 * needs none).  T tokens, d model width, E experts, K experts per token, F
 * expert intermediate width (only for C2R_STAGE_EXPERT_FFN), dt the activation
 * type.  Host call, no GPU work.
 */
size_t c2r_workspace_bytes(int stage, int64_t T, int d, int E, int K, int F, c2r_dtype dt);

/*
 * Expert collaboration matrix, Eq. 2 (Sec. 3.2): for every token t and every
 * ordered pair (i, j) of its selected experts, i = j included,
 *     C[i, j] += 1.
 * topk_idx : int32[T, K]  selected experts per token (entries outside [0, E)
 *            are ignored, so a token padded with -1 counts for fewer experts)
 * C        : int32[E, E]  in/out.  ACCUMULATES, so a corpus can be profiled
 *            batch by batch; the caller zeroes it before the first batch.
 * Result is exact and independent of scheduling (integer adds) as long as no
 * entry passes 2^31 - 1: the adds wrap, they do not saturate.  The largest entry
 * is a diagonal one (tokens that selected that expert), so a corpus of fewer
 * than 2^31 tokens cannot overflow; beyond that, fold C into a wider host-side
 * matrix between batches.
 */
int c2r_build_coactivation(const int32_t *topk_idx, int64_t T, int K, int E, int32_t *C,
                           void *stream);

/*
 * Collaborator lists, Eq. 4 (Sec. 3.3, step 1): for every expert i the
 * n = min(Tc, E-1) other experts j != i with the largest C[i, j], in
 * descending order of count, equal counts to the lower index.  The expert
 * itself is never in its own list (with Tc >= E-1 the constraint vanishes, as
 * Fig. 3's caption notes for N = 8, T = 7).
 * C           : int32[E, E]
 * collab_idx  : int32[E, n]  out
 * collab_mask : uint64[E] out or NULL; bit j of word i set iff j is in i's list
 */
int c2r_collaborators(const int32_t *C, int E, int Tc, int32_t *collab_idx, uint64_t *collab_mask,
                      void *stream);

/*
 * Router of Eq. 1 followed by the C2R selection of Sec. 3.3 (step 2).
 *   logits l[t, e] = sum_k x[t, k] W_g[k, e] (+ bias[e]), fp32, in the order
 *   stated at c2r_route_chunk().
 *   slot 0      = arg max_e l[t, e] over ALL experts (ties: lower index);
 *   slots 1..K-1 = the K-1 largest logits among the collaborator list of the
 *                 slot-0 expert, descending (ties: lower index);
 *   gates[t, s] = softmax over the K kept logits (they sum to 1), as
 *                 exp(l - l_slot0) / sum: a token whose largest logit is infinite
 *                 or a NaN gets NaN gates.
 * collab_idx == NULL selects the conventional top-K of Eq. 1 (used to profile
 * the pre-trained router, Sec. 3.2).
 * x          : [T, d] of x_dt (fp32 or bf16)
 * Wg         : fp32[d, E]   (the layout of "x . W_g")
 * bias       : fp32[E] or NULL (per-expert logit offset; not in the paper,
 *              used by synthetic load-skewed workloads)
 * collab_idx : int32[E, Tc] or NULL; entries outside [0, E) or equal to the
 *              row's own expert are ignored
 * topk_idx   : int32[T, K] out; a slot the list cannot fill gets -1 and gate 0
 * gates      : fp32[T, K] out
 * logits_out : fp32[T, E] out or NULL
 * ws         : c2r_workspace_bytes(C2R_STAGE_ROUTE, T, d, E, K, 0, x_dt)
 * Errors: Tc < K-1 with a list given, K > E -> C2R_ERR_INVALID_ARG.
 */
int c2r_route(const void *x, c2r_dtype x_dt, const float *Wg, const float *bias, int64_t T, int d,
              int E, int K, const int32_t *collab_idx, int Tc, int32_t *topk_idx, float *gates,
              float *logits_out, void *ws, size_t ws_bytes, void *stream);

/*
 * The selection and gates of c2r_route applied to logits that already exist
 * (profiling a stored logit stream, Sec. 3.2).  logits: fp32[T, E].  No scratch.
 */
int c2r_route_from_logits(const float *logits, int64_t T, int E, int K, const int32_t *collab_idx,
                          int Tc, int32_t *topk_idx, float *gates, void *stream);

/*
 * The profiling pass of Sec. 3.2 in one launch: c2r_route_from_logits followed by
 * c2r_build_coactivation (Eq. 2) on its selections, i.e. C[i, j] += the number of these T
 * tokens whose selected experts include both i and j (diagonal included).  Exact integer counts,
 * independent of the order of execution; the same results as the two calls in a row.
 * logits   : fp32[T, E], 16-byte aligned
 * topk_idx : int32[T, K] out, or NULL
 * gates    : fp32[T, K] out, or NULL   (a pass that only wants the counts passes NULL for both:
 *            they may be NULL when E is a multiple of 4 and K <= 4, the shapes the fused kernel
 *            covers; other shapes run the two kernels one after the other and need both
 *            arrays: C2R_ERR_UNSUPPORTED without them)
 * C        : int32[E, E], accumulated into (the caller zeroes it before the first batch); the
 *            int32 ceiling of c2r_build_coactivation applies
 * Errors as c2r_route_from_logits; C == NULL -> C2R_ERR_INVALID_ARG.
 */
int c2r_profile_from_logits(const float *logits, int64_t T, int E, int K, const int32_t *collab_idx,
                            int Tc, int32_t *topk_idx, float *gates, int32_t *C, void *stream);

/*
 * Token dispatch on one device (the step the paper inherits from dropless MoE
 * frameworks, Sec. 2 / Sec. 3.1): a stable sort of the assignments
 * a = t*K + s by local expert slot, and the gather of their rows.
 * local_slot : int32[E] or NULL.  local_slot[e] = position of expert e among
 *              this device's E_local experts, or -1 if it lives elsewhere;
 *              NULL means all E experts are local (then E_local must equal E).
 * counts     : int32[E_local] out   rows per local expert
 * offsets    : int32[E_local+1] out exclusive prefix sum of counts
 * perm       : int32[T*K] out; perm[p] = a for sorted position p < offsets[E_local];
 *              inside an expert's range a is ascending; the rest is untouched
 * inv_perm   : int32[T*K] out; inv_perm[a] = p, or -1 if a's expert is not local
 * x_perm     : [T*K, d] of dt out, row p = x[perm[p] / K]; may be NULL to get
 *              the index arrays only
 * ws         : c2r_workspace_bytes(C2R_STAGE_PERMUTE, T, d, E, K, 0, dt)
 */
int c2r_permute(const void *x, c2r_dtype dt, const int32_t *topk_idx, int64_t T, int d, int E,
                int K, const int32_t *local_slot, int E_local, int32_t *counts, int32_t *offsets,
                int32_t *perm, int32_t *inv_perm, void *x_perm, void *ws, size_t ws_bytes,
                void *stream);

/*
 * c2r_permute for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments, results and errors,
 * but no workspace argument - the block histograms live in a 2 MiB static device array that
 * the library holds on every GPU it runs on until the process ends.  The call allocates
 * nothing and frees nothing.
 * Limit: T*K <= 4194304 assignments; beyond it C2R_ERR_UNSUPPORTED (use c2r_permute).
 * Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two
 * streams, two host threads) race on it and must be serialised by the caller; calls on one
 * stream, or on different GPUs, are safe.  Nothing in the array needs clearing between calls
 * (each call overwrites the part it reads).
 */
int c2r_permute_noalloc(const void *x, c2r_dtype dt, const int32_t *topk_idx, int64_t T, int d, int E,
                        int K, const int32_t *local_slot, int E_local, int32_t *counts,
                        int32_t *offsets, int32_t *perm, int32_t *inv_perm, void *x_perm,
                        void *stream);

/*
 * Grouped expert FFN (Sec. 3.1: every token is processed by each expert selected for it):
 * for each local expert e and each row r in [offsets[e], offsets[e+1]):
 *     y_perm[r] = W_down,e ( silu(W_gate,e x_perm[r]) * (W_up,e x_perm[r]) )
 * with silu(z) = z / (1 + exp(-z)), no biases, un-weighted by the gate.
 * bf16: products accumulate in fp32; the hidden activation is rounded to bf16
 * once, y_perm once.  fp32: fp32 throughout.
 * offsets : int32[E_local+1] in DEVICE memory (as written by c2r_permute)
 * A_cap   : rows allocated in x_perm / y_perm (>= offsets[E_local], e.g. T*K)
 * w_gate, w_up : [E_local, F, d] of dt;  w_down : [E_local, d, F] of dt
 * y_perm  : [A_cap, d] of dt out; rows beyond offsets[E_local] are untouched
 * ws      : c2r_workspace_bytes(C2R_STAGE_EXPERT_FFN, A_cap, d, E_local, 1, F, dt)
 * A shared always-on expert is this call with E_local = 1, offsets = {0, T}
 * and x itself as x_perm.
 * Concurrency (this and every other c2r_expert_ffn_* call, bf16 shapes of the fast kernel): a
 * launch hands its tiles out through a set of counters in a static device array; the library
 * holds 64 sets per GPU and gives them to launches in turn, and a set is all zero again when its
 * launch ends.  Two launches that were given the same set (every 64th call) must not RUN at the
 * same time: on one stream they never do, however many are queued; a caller that spreads these
 * calls over several streams keeps fewer than 64 of them outstanding (enqueued and not finished)
 * per GPU.  A launch recorded into a HIP graph keeps the set it was given at capture: replays of
 * that graph must not overlap each other.
 */
int c2r_expert_ffn(const void *x_perm, c2r_dtype dt, const int32_t *offsets, int E_local,
                   int64_t A_cap, int d, int F, const void *w_gate, const void *w_up,
                   const void *w_down, void *y_perm, void *ws, size_t ws_bytes, void *stream);

/*
 * The two passes of c2r_expert_ffn (the expert computation of Sec. 3.1, shapes of Sec. 4.1) as
 * calls of their own (same arguments and limits), for callers that time them or put other work
 * between them:
 *   gate_up : h[r, f]      = silu(W_gate,e[f,:] . x_perm[r]) * (W_up,e[f,:] . x_perm[r])
 *   down    : y_perm[r, j] = W_down,e[j,:] . h[r]
 * h : [A_cap, F] of dt, caller-owned (what c2r_expert_ffn keeps in its workspace).
 */
int c2r_expert_ffn_gate_up(const void *x_perm, c2r_dtype dt, const int32_t *offsets, int E_local,
                           int64_t A_cap, int d, int F, const void *w_gate, const void *w_up,
                           void *h, void *stream);
int c2r_expert_ffn_down(const void *h, c2r_dtype dt, const int32_t *offsets, int E_local,
                        int64_t A_cap, int d, int F, const void *w_down, void *y_perm, void *stream);

/*
 * c2r_expert_ffn_gate_up with the row gather of the dispatch (Sec. 3.1) folded in: row p of
 * the sorted order is read as x[perm[p] / K] instead of x_perm[p], so c2r_permute can be
 * called with x_perm == NULL and the [T*K, d] copy is never written.  Same result bit for
 * bit.  x: [T, d] of dt; perm: int32[A_cap] as written by c2r_permute (entries at
 * positions >= offsets[E_local] are never read).  Limits: bf16, d and F multiples of 64,
 * T*d*2 < 2^32; otherwise C2R_ERR_UNSUPPORTED (use c2r_permute's x_perm instead).
 */
int c2r_expert_ffn_gate_up_gather(const void *x, c2r_dtype dt, const int32_t *perm, int64_t T, int K,
                                  const int32_t *offsets, int E_local, int64_t A_cap, int d, int F,
                                  const void *w_gate, const void *w_up, void *h, void *stream);

/*
 * c2r_expert_ffn (both passes, h in the workspace) with the row gather of the dispatch
 * (Sec. 3.1) folded into the first pass, as in c2r_expert_ffn_gate_up_gather: x [T, d] is
 * read through perm and x_perm is never needed.  Unlike the split entry points it takes any
 * F that c2r_expert_ffn takes (h is padded inside the workspace), e.g. F = 688 or 1376.
 * Same result as c2r_expert_ffn on the x_perm of c2r_permute, bit for bit.
 * ws: c2r_workspace_bytes(C2R_STAGE_EXPERT_FFN, A_cap, d, E_local, 1, F, dt) bytes, 256-aligned.
 * Limits: bf16, d a multiple of 64, T*d*2 < 2^32; otherwise C2R_ERR_UNSUPPORTED.
 */
int c2r_expert_ffn_gather(const void *x, c2r_dtype dt, const int32_t *perm, int64_t T, int K,
                          const int32_t *offsets, int E_local, int64_t A_cap, int d, int F,
                          const void *w_gate, const void *w_up, const void *w_down, void *y_perm,
                          void *ws, size_t ws_bytes, void *stream);

/*
 * The two FFN passes for a layer that also has an always-on shared expert (the Qwen1.5-MoE
 * setting of Sec. 4.1: routed experts plus one shared expert that every token runs through,
 * Sec. 3.1 for the routed part): the routed groups AND the shared expert in ONE launch per
 * pass, so that the shared expert's uniform tiles fill the compute units that the ragged
 * groups' last tiles leave idle.  Results are bit-identical to
 * c2r_expert_ffn_gate_up_gather / c2r_expert_ffn_down on the routed groups plus
 * c2r_expert_ffn_gate_up / c2r_expert_ffn_down with E_local = 1, offsets = {0, T} on x.
 *   gate_up : h[r, f]        = silu(W_gate,e[f,:] . x[perm[r] / K]) * (W_up,e[f,:] . x[perm[r] / K])
 *             h_shared[t, f] = silu(Ws_gate[f,:] . x[t]) * (Ws_up[f,:] . x[t])
 *   down    : y_perm[r, j]   = W_down,e[j,:] . h[r];   y_shared[t, j] = Ws_down[j,:] . h_shared[t]
 * x : [T, d];  perm, offsets : as written by c2r_permute;  h : [A_cap, F];  y_perm : [A_cap, d]
 * ws_gate, ws_up : [F_shared, d];  ws_down : [d, F_shared];  h_shared : [T, F_shared];
 * y_shared : [T, d].  A_cap == 0 runs the shared expert alone.
 * Limits: bf16; d, F and F_shared multiples of 64; T*d*2 < 2^32; else C2R_ERR_UNSUPPORTED.
 */
int c2r_expert_ffn_gate_up_with_shared(const void *x, c2r_dtype dt, const int32_t *perm, int64_t T, int K,
                                       const int32_t *offsets, int E_local, int64_t A_cap, int d, int F,
                                       const void *w_gate, const void *w_up, void *h, int F_shared,
                                       const void *ws_gate, const void *ws_up, void *h_shared, void *stream);
int c2r_expert_ffn_down_with_shared(const void *h, c2r_dtype dt, const int32_t *offsets, int E_local,
                                    int64_t A_cap, int d, int F, const void *w_down, void *y_perm, int64_t T,
                                    int F_shared, const void *h_shared, const void *ws_down, void *y_shared,
                                    void *stream);

/*
 * Un-permute and gate-weighted sum (Sec. 3.1, last sentence):
 *     y[t] = sum_{s<K, inv_perm[t*K+s] >= 0} gates[t,s] * y_perm[inv_perm[t*K+s]]  (+ y_shared[t])
 * summed in fp32 in slot order and rounded once to dt.
 * y_shared : [T, d] of dt or NULL (output of an always-on shared expert, weight 1)
 * y        : [T, d] of dt out
 */
int c2r_combine(const void *y_perm, c2r_dtype dt, const float *gates, const int32_t *inv_perm,
                int64_t T, int d, int K, const void *y_shared, void *y, void *stream);

/*
 * Zero-redundancy dispatch index (Sec. 3.4: a token whose experts share a device travels
 * there once and is replicated on arrival), built on one GPU.  For a
 * map expert -> device, every token gets ONE copy per device that hosts at least one of its
 * selected experts.  The copies are listed device after device, tokens ascending:
 *   send_counts[g], send_offsets[g]   : copies for device g (send_offsets has n_dev+1 entries,
 *                                       the last one the total n_send = sum over tokens of
 *                                       the number of distinct devices of their experts)
 *   send_token[send_offsets[g] + i]   : the i-th token device g receives
 *   send_row[t*K + s]                 : the position in send_token of the copy that slot s of
 *                                       token t uses on its expert's device; -1 if the slot
 *                                       is empty (topk_idx < 0 or >= E) or its expert has no
 *                                       device (expert_device outside [0, n_dev))
 * 1 - n_send / (T*K) is the token redundancy of Sec. 4.1.
 * topk_idx : int32[T,K]; expert_device : int32[E]; n_dev <= 64
 * send_counts int32[n_dev], send_offsets int32[n_dev+1], send_token int32[T*K] (capacity;
 * entries past n_send untouched), send_row int32[T*K]: all DEVICE memory, all out.
 * ws : c2r_workspace_bytes(C2R_STAGE_DEDUP_DISPATCH, T, 0, n_dev, K, 0, C2R_F32)
 * Deterministic (no atomically assigned positions), integer results exact.
 */
int c2r_dedup_dispatch(const int32_t *topk_idx, int64_t T, int K, int E, const int32_t *expert_device,
                       int n_dev, int32_t *send_counts, int32_t *send_offsets, int32_t *send_token,
                       int32_t *send_row, void *ws, size_t ws_bytes, void *stream);

/*
 * Expert -> device map that co-locates collaborating experts (Sec. 3.4 proposes placing
 * experts that collaborate closely on one device; the paper names the goal
 * and gives no procedure - this is a greedy fill).  Devices 0..n_dev-1 are filled in order
 * with ceil(E / n_dev) experts each (the last ones with what is left): a device starts with
 * the unplaced expert whose row of C, diagonal left out, sums highest, and then keeps taking
 * the unplaced expert with the largest total co-activation with the experts already on it;
 * ties go to the lower index.  Co-activation counts are non-negative (Eq. 2).
 * C : int32[E,E] (DEVICE, as c2r_build_coactivation leaves it); expert_device : int32[E] out.
 */
int c2r_place_experts(const int32_t *C, int E, int n_dev, int32_t *expert_device, void *stream);

/*
 * The combine that goes with it (Sec. 3.4, Sec. 3.1 last sentence), in two levels.
 * c2r_combine_partial is what an expert device returns: one row per token copy r,
 *     y_part[r] = sum_{s : send_row[t*K+s] == r, inv_perm[t*K+s] >= 0} gates[t,s] * y_perm[inv_perm[t*K+s]]
 * with t = send_token[r], summed in fp32 in slot order and rounded once to dt.
 * c2r_combine_copies is what the token's home device does:
 *     y[t] = sum over the distinct rows r among send_row[t*K + 0..K-1], in order of first
 *            appearance, of y_part[r]  (+ y_shared[t]),  fp32, rounded once to dt.
 * Against c2r_combine the result differs only by the extra rounding of the partial rows.
 * n_send   : DEVICE pointer to the number of copies (&send_offsets[n_dev])
 * cap_rows : rows allocated in y_part (>= *n_send, e.g. T*K); rows >= *n_send untouched
 * y_part   : [cap_rows, d] of dt;  y_shared : [T, d] of dt or NULL;  y : [T, d] of dt out
 */
int c2r_combine_partial(const void *y_perm, c2r_dtype dt, const float *gates, const int32_t *inv_perm,
                        const int32_t *send_token, const int32_t *send_row, const int32_t *n_send,
                        int64_t T, int64_t cap_rows, int d, int K, void *y_part, void *stream);
int c2r_combine_copies(const void *y_part, c2r_dtype dt, const int32_t *send_row, int64_t T,
                       int64_t cap_rows, int d, int K, const void *y_shared, void *y, void *stream);

/*
 * Collaboration degree of every expert (Eq. 3): the entropy of the frequencies with which
 * expert i is co-activated with each OTHER expert,
 *     p_ij = C[i,j] / sum_{j' != i} C[i,j'],    P[i] = - sum_{j != i, C[i,j] > 0} p_ij ln p_ij
 * (the equation's limits are printed inconsistently; the reading taken leaves the diagonal
 * out of the sum and of the normalisation and uses the natural logarithm).  A row without
 * co-activations gives 0.  Computed in fp64.
 * C : int32[E,E] (DEVICE, as c2r_build_coactivation leaves it; negative entries count as 0)
 * P : double[E] out (DEVICE).  E <= 64.
 */
int c2r_collaboration_degree(const int32_t *C, int E, double *P, void *stream);

/*
 * Distinct destination devices per token, for several expert -> device maps in one pass
 * over the indices (Sec. 4.1: the token redundancy of an expert-parallel degree is the
 * share of (token, expert) copies that a zero-redundancy dispatch does not send,
 * 1 - totals[m] / (T*K); Table 3 lists it for degrees 2..6).
 * topk_idx      : int32[T,K] (entries outside [0,E) are skipped)
 * expert_device : int32[n_maps, E]; entries outside [0, n_dev) mean "no device" and are
 *                 skipped.  n_maps <= 8, n_dev <= 64, E <= 64.
 * per_token     : int32[n_maps, T] out or NULL - the count for every token and map
 * totals        : int64[n_maps] out (8-byte aligned) - the sum over the tokens; equals the
 *                 n_send that c2r_dedup_dispatch reports for the same map.  Exact.
 * All pointers are DEVICE memory.
 */
int c2r_distinct_devices(const int32_t *topk_idx, int64_t T, int K, int E, const int32_t *expert_device,
                         int n_maps, int n_dev, int32_t *per_token, int64_t *totals, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* C2R_H */
