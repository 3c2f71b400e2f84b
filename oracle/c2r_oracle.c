/*
 * CPU oracle for the collaboration-constrained routing (C2R) MoE layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, step-by-step statement
 * of what the layer computes, written from the paper (arXiv 2504.01337) and
 * independent of the HIP library: it shares no code, header, table or helper
 * with it.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it; the product path never does.
 *
 * Floating point is fp64 throughout, with two stated exceptions:
 *   - orc_logits_canon_f32 reproduces the router's *declared* fp32 summation
 *     order so that selections can be compared bit for bit (the paper is silent
 *     on precision; the reading is "router in fp32, ties to the lower index");
 *   - selections are decided on fp32 logits (the precision the router works in).
 *
 * Parity pins (tests/test_oracle_*.py): C = M^T M against an integer matmul,
 * brute-force subset enumeration for the constrained selection, the T >= N-1
 * degeneracy of Fig. 3's caption, a dense SwiGLU MLP via a library fp64 matmul,
 * exact-arithmetic logits, permutation bijection / stability properties, and the
 * speed-up products printed in Table 3.  The values of the expert FFN on Gaussian
 * inputs have no printed example in the paper: they are pinned by the dense-MLP
 * special case and the definition only.
 *
 * Loops run over tokens with OpenMP where tokens are independent; nothing is
 * blocked, fused or reordered beyond that.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- Eq. 1: router logits  l[t,e] = sum_k x[t,k] W_g[k,e] (+ b[e]) ---- */

/* fp64 accumulation of the exactly representable inputs: the numerical reference. */
void orc_logits_f64(const float *x, const float *Wg, const float *bias, int64_t T, int d, int E,
                    double *logits) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            double s = 0.0;
            for (int k = 0; k < d; ++k) s += (double)x[t * d + k] * (double)Wg[(int64_t)k * E + e];
            if (bias) s += (double)bias[e];
            logits[t * E + e] = s;
        }
    }
}

/*
 * fp32 logits in the library's declared order: k is cut into consecutive chunks
 * of `chunk` elements; inside a chunk one fused multiply-add per element,
 * ascending k, starting from +0; chunk results are added left to right in fp32;
 * the bias, if any, is added last.
 */
void orc_logits_canon_f32(const float *x, const float *Wg, const float *bias, int64_t T, int d,
                          int E, int chunk, float *logits) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            float total = 0.0f;
            for (int k0 = 0; k0 < d; k0 += chunk) {
                int k1 = k0 + chunk < d ? k0 + chunk : d;
                float part = 0.0f;
                for (int k = k0; k < k1; ++k)
                    part = __builtin_fmaf(x[t * d + k], Wg[(int64_t)k * E + e], part);
                total = (k0 == 0) ? part : total + part;
            }
            if (bias) total = total + bias[e];
            logits[t * E + e] = total;
        }
    }
}

/* ---- Sec. 3.3 (2): selection.  "a beats b" = larger logit, else lower index. ---- */

/* Pick, among experts with allowed[e] != 0, the one with the largest logit; the
 * first allowed expert stands unless a later one is strictly larger. */
static int pick_best(const float *l, const unsigned char *allowed, int E) {
    int best = -1;
    for (int e = 0; e < E; ++e) {
        if (!allowed[e]) continue;
        if (best < 0 || l[e] > l[best]) best = e;
    }
    return best;
}

/*
 * For every token: slot 0 = arg max over all experts.  The remaining K-1 slots
 * are taken, best first, from the collaborator list of the slot-0 expert
 * (collab_idx[e0, 0..Tc)); with collab_idx == NULL every other expert is a
 * candidate, which is the conventional top-K of Eq. 1.  Gates are the softmax
 * over the K kept logits (Eq. 1), in fp64.
 * Returns 0, or -1 if a list cannot supply K-1 distinct experts.
 */
int orc_route(const float *logits, int64_t T, int E, int K, const int32_t *collab_idx, int Tc,
              int32_t *topk_idx, double *gates) {
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const float *l = logits + t * E;
        unsigned char *allowed = (unsigned char *)malloc((size_t)E);
        memset(allowed, 1, (size_t)E);
        int e0 = pick_best(l, allowed, E);
        topk_idx[t * K] = e0;
        if (collab_idx) {
            memset(allowed, 0, (size_t)E);
            for (int j = 0; j < Tc; ++j) allowed[collab_idx[(int64_t)e0 * Tc + j]] = 1;
        }
        allowed[e0] = 0;
        for (int s = 1; s < K; ++s) {
            int e = pick_best(l, allowed, E);
            if (e < 0) {
#pragma omp atomic write
                bad = 1;
                topk_idx[t * K + s] = -1;
                continue;
            }
            allowed[e] = 0;
            topk_idx[t * K + s] = e;
        }
        free(allowed);
        if (gates) {
            double den = 0.0;
            for (int s = 0; s < K; ++s) {
                int e = topk_idx[t * K + s];
                double v = e < 0 ? 0.0 : exp((double)l[e] - (double)l[e0]);
                gates[t * K + s] = v;
                den += v;
            }
            for (int s = 0; s < K; ++s) gates[t * K + s] /= den;
        }
    }
    return bad ? -1 : 0;
}

/* ---- Eq. 2: C[i,j] += #tokens that select both i and j (i = j included). ---- */
void orc_coactivation(const int32_t *topk_idx, int64_t T, int K, int E, int64_t *C) {
    for (int64_t t = 0; t < T; ++t)
        for (int a = 0; a < K; ++a)
            for (int b = 0; b < K; ++b) {
                int i = topk_idx[t * K + a], j = topk_idx[t * K + b];
                if (i >= 0 && j >= 0) C[(int64_t)i * E + j] += 1;
            }
}

/* ---- Eq. 4: per row i, the Tc other experts with the largest C[i,j];
 *      equal counts go to the lower index; the expert itself is left out. ---- */
void orc_collaborators(const int64_t *C, int E, int Tc, int32_t *collab_idx) {
    int n = Tc < E - 1 ? Tc : E - 1;
    int *order = (int *)malloc(sizeof(int) * (size_t)E);
    for (int i = 0; i < E; ++i) {
        int m = 0;
        for (int j = 0; j < E; ++j)
            if (j != i) order[m++] = j;
        /* insertion sort by (count descending, index ascending) */
        for (int a = 1; a < m; ++a) {
            int v = order[a], b = a - 1;
            while (b >= 0 && (C[(int64_t)i * E + order[b]] < C[(int64_t)i * E + v] ||
                              (C[(int64_t)i * E + order[b]] == C[(int64_t)i * E + v] &&
                               order[b] > v))) {
                order[b + 1] = order[b];
                --b;
            }
            order[b + 1] = v;
        }
        for (int j = 0; j < n; ++j) collab_idx[(int64_t)i * n + j] = order[j];
    }
    free(order);
}

/* ---- Dispatch: stable sort of assignments a = t*K + s by local expert slot. ---- */
void orc_permute(const int32_t *topk_idx, int64_t T, int K, int E, const int32_t *local_slot,
                 int E_local, int32_t *counts, int32_t *offsets, int32_t *perm,
                 int32_t *inv_perm) {
    int64_t A = T * K;
    for (int e = 0; e < E_local; ++e) counts[e] = 0;
    for (int64_t a = 0; a < A; ++a) {
        int e = topk_idx[a];
        int ls = (e < 0 || e >= E) ? -1 : (local_slot ? local_slot[e] : e);
        if (ls >= 0) counts[ls] += 1;
    }
    offsets[0] = 0;
    for (int e = 0; e < E_local; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(E_local + 1));
    memcpy(cursor, offsets, sizeof(int32_t) * (size_t)(E_local + 1));
    for (int64_t a = 0; a < A; ++a) {
        int e = topk_idx[a];
        int ls = (e < 0 || e >= E) ? -1 : (local_slot ? local_slot[e] : e);
        if (ls < 0) {
            inv_perm[a] = -1;
            continue;
        }
        int32_t p = cursor[ls]++;
        perm[p] = (int32_t)a;
        inv_perm[a] = p;
    }
    free(cursor);
}

/* ---- Expert: E_e(x) = W_down ( silu(W_gate x) * (W_up x) ), fp64, no rounding. ---- */
static void expert_row(const float *x, const float *wg, const float *wu, const float *wd, int d,
                       int F, double *h, double *y) {
    for (int f = 0; f < F; ++f) {
        double g = 0.0, u = 0.0;
        for (int k = 0; k < d; ++k) {
            g += (double)wg[(int64_t)f * d + k] * (double)x[k];
            u += (double)wu[(int64_t)f * d + k] * (double)x[k];
        }
        h[f] = g / (1.0 + exp(-g)) * u;
    }
    for (int j = 0; j < d; ++j) {
        double s = 0.0;
        for (int f = 0; f < F; ++f) s += (double)wd[(int64_t)j * F + f] * h[f];
        y[j] = s;
    }
}

/* Rows of x_rows[n,d], row r handled by expert expert_of_row[r]; y_rows[n,d] fp64. */
void orc_expert_ffn_rows(const float *x_rows, const int32_t *expert_of_row, int64_t n, int d, int F,
                         const float *w_gate, const float *w_up, const float *w_down,
                         double *y_rows) {
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)F);
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < n; ++r) {
            int64_t e = expert_of_row[r];
            expert_row(x_rows + r * d, w_gate + e * F * d, w_up + e * F * d, w_down + e * d * F, d,
                       F, h, y_rows + r * d);
        }
        free(h);
    }
}

/*
 * Whole layer for a list of tokens: y[t] = sum_s g[t,s] E_{e_s}(x[t]) (+ shared
 * expert, coefficient 1).  Experts with local_slot < 0 contribute nothing (they
 * live on another device).  tokens[n] indexes x, topk_idx and gates; y is [n,d].
 */
void orc_layer_tokens(const float *x, const int64_t *tokens, int64_t n, int d, int E, int K, int F,
                      const int32_t *topk_idx, const double *gates, const int32_t *local_slot,
                      const float *w_gate, const float *w_up, const float *w_down, int F_shared,
                      const float *ws_gate, const float *ws_up, const float *ws_down, double *y) {
    int Fm = F > F_shared ? F : F_shared;
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)Fm);
        double *ye = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < n; ++i) {
            int64_t t = tokens[i];
            double *yt = y + i * d;
            for (int j = 0; j < d; ++j) yt[j] = 0.0;
            for (int s = 0; s < K; ++s) {
                int e = topk_idx[t * K + s];
                if (e < 0 || e >= E) continue;
                int64_t ls = local_slot ? local_slot[e] : e;
                if (ls < 0) continue;
                expert_row(x + t * d, w_gate + ls * F * d, w_up + ls * F * d, w_down + ls * d * F,
                           d, F, h, ye);
                for (int j = 0; j < d; ++j) yt[j] += gates[t * K + s] * ye[j];
            }
            if (F_shared > 0) {
                expert_row(x + t * d, ws_gate, ws_up, ws_down, d, F_shared, h, ye);
                for (int j = 0; j < d; ++j) yt[j] += ye[j];
            }
        }
        free(h);
        free(ye);
    }
}

/* Gate-weighted sum over already computed expert rows (un-permute + combine). */
void orc_combine(const double *y_perm, const double *gates, const int32_t *inv_perm, int64_t T,
                 int d, int K, const double *y_shared, double *y) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int j = 0; j < d; ++j) {
            double s = 0.0;
            for (int q = 0; q < K; ++q) {
                int32_t p = inv_perm[t * K + q];
                if (p >= 0) s += gates[t * K + q] * y_perm[(int64_t)p * d + j];
            }
            if (y_shared) s += y_shared[t * d + j];
            y[t * d + j] = s;
        }
    }
}

/* ---- Sec. 3.4: number of distinct devices a token's K experts live on. ---- */
void orc_distinct_devices(const int32_t *topk_idx, int64_t T, int K, const int32_t *dev_of_expert,
                          int32_t *distinct) {
    for (int64_t t = 0; t < T; ++t) {
        int n = 0;
        for (int a = 0; a < K; ++a) {
            int da = dev_of_expert[topk_idx[t * K + a]], seen = 0;
            for (int b = 0; b < a; ++b)
                if (dev_of_expert[topk_idx[t * K + b]] == da) seen = 1;
            if (!seen) ++n;
        }
        distinct[t] = n;
    }
}

/* ---- Sec. 3.4: zero-redundancy dispatch.  A token goes ONCE to every device that hosts at
 * least one of its selected experts and is replicated there.  The send list is ordered by
 * device, then by token; send_row[t*K+s] is the position in that list of the copy that slot
 * s of token t uses (-1: empty slot or expert without a device).  send_offsets has n_dev+1
 * entries.  Returns the number of copies sent. ---- */
int64_t orc_dedup_dispatch(const int32_t *topk_idx, int64_t T, int K, int E, const int32_t *dev_of_expert,
                           int n_dev, int32_t *send_counts, int32_t *send_offsets, int32_t *send_token,
                           int32_t *send_row) {
    int64_t n = 0;
    for (int64_t a = 0; a < T * K; ++a) send_row[a] = -1;
    for (int g = 0; g < n_dev; ++g) {
        send_offsets[g] = (int32_t)n;
        for (int64_t t = 0; t < T; ++t) {
            int hit = 0;
            for (int s = 0; s < K; ++s) {
                int32_t e = topk_idx[t * K + s];
                if (e >= 0 && e < E && dev_of_expert[e] == g) {
                    hit = 1;
                    send_row[t * K + s] = (int32_t)n;
                }
            }
            if (hit) send_token[n++] = (int32_t)t;
        }
        send_counts[g] = (int32_t)n - send_offsets[g];
    }
    send_offsets[n_dev] = (int32_t)n;
    return n;
}

/* The combine that goes with it: every device first adds up, gate-weighted, the outputs of
 * its own experts for each token copy it received (one partial row per copy, y_part), and
 * the token's home device adds the partial rows of its copies (+ the shared expert). */
void orc_combine_partial(const double *y_perm, const double *gates, const int32_t *inv_perm,
                         const int32_t *send_row, int64_t T, int d, int K, int64_t n_send, double *y_part) {
    memset(y_part, 0, sizeof(double) * (size_t)n_send * d);
    for (int64_t t = 0; t < T; ++t)
        for (int s = 0; s < K; ++s) {
            int32_t r = send_row[t * K + s], p = inv_perm[t * K + s];
            if (r < 0 || p < 0) continue;
            for (int j = 0; j < d; ++j) y_part[(int64_t)r * d + j] += gates[t * K + s] * y_perm[(int64_t)p * d + j];
        }
}

void orc_combine_copies(const double *y_part, const int32_t *send_row, int64_t T, int d, int K,
                        const double *y_shared, double *y) {
    for (int64_t t = 0; t < T; ++t)
        for (int j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int s = 0; s < K; ++s) {
                int32_t r = send_row[t * K + s];
                int seen = r < 0;
                for (int b = 0; b < s && !seen; ++b) seen = send_row[t * K + b] == r;
                if (!seen) acc += y_part[(int64_t)r * d + j];
            }
            if (y_shared) acc += y_shared[t * d + j];
            y[t * d + j] = acc;
        }
}

/* ---- Sec. 3.4 proposes placing experts that collaborate closely on one device.
 * The paper names the goal and gives no procedure; the reading taken is a greedy fill.
 * Devices 0..n_dev-1 are filled one after the other, each with cap = ceil(E / n_dev) experts
 * (the last ones with what is left).  A device starts with the unplaced expert whose
 * co-activation with all other experts (its row of C without the diagonal) is largest, and
 * then repeatedly takes the unplaced expert with the largest total co-activation with the
 * experts already on the device.  Ties go to the lower index. ---- */
void orc_place_experts(const int64_t *C, int E, int n_dev, int32_t *expert_device) {
    int cap = (E + n_dev - 1) / n_dev;
    for (int e = 0; e < E; ++e) expert_device[e] = -1;
    for (int g = 0; g < n_dev; ++g) {
        int members = 0;
        while (members < cap) {
            int best = -1;
            int64_t best_score = 0;
            for (int e = 0; e < E; ++e) {
                if (expert_device[e] >= 0) continue;
                int64_t score = 0;
                for (int j = 0; j < E; ++j) {
                    if (j == e) continue;
                    if (members == 0 || expert_device[j] == g) score += C[(int64_t)e * E + j];
                }
                if (best < 0 || score > best_score) {
                    best = e;
                    best_score = score;
                }
            }
            if (best < 0) break; /* everything is placed */
            expert_device[best] = g;
            ++members;
        }
    }
}
