/*
 * CPU oracle for the Mixture-of-Experts layer forward.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, by-the-definition implementation used to check the GPU path.
 * Nothing in the product path may call it; only the tests, the smoke check and
 * the benchmark's reported CPU-baseline leg do.  It shares no code with the GPU
 * path: no headers, tables, helpers or pre/post-processing.
 *
 * What the paper fixes (Section 2.1, "MoE Architecture & Inference"): the layer is a
 * gating network plus several experts; the gate scores every expert with a
 * softmax and activates the top-k; each expert is an FFN; the layer output of a
 * token is the weighted sum of its selected experts' outputs.  Section 5 adds
 * that the expert layer is evaluated expert by expert over the tokens of all
 * batches of a batch group, hot experts first; that only changes the order of
 * work, never the result, so the oracle evaluates token by token.
 *
 * Readings where the paper is silent (each is listed in the design notes):
 *  - expert FFN = bias-free SwiGLU: W2 * (silu(W1 x) .* (W3 x));
 *  - routing weights are renormalised over the k winners (= softmax over the k
 *    winning logits); a flag keeps the un-renormalised full-softmax variant;
 *  - selection is on logits, ties go to the lower expert index;
 *  - the fp32 gate logits use one fixed summation order (ko_gate_logits_f32)
 *    so that "the k largest" is a well-defined, reproducible set;
 *  - experts are ordered for execution by (batches touching it desc, tokens
 *    desc, index asc);
 *  - shared experts (always on, weight 1) are added after the routed slots.
 *
 * Arithmetic: gate logits in fp32 with the stated order (they decide integers);
 * everything else in fp64 with no intermediate rounding.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KO_LANES 64

#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the token loop of ko_moe_forward will use (reported beside timings). */
int ko_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- storage helpers ---------------------------------------------------- */

/* bfloat16 bit pattern -> double (exact: bf16 is the top half of an fp32). */
static double bf16_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* wtype: 0 = float32 array, 1 = bfloat16 bit patterns (uint16), 2 = float64 array. */
static double weight_at(const void *w, int wtype, size_t i) {
    if (wtype == 0) return (double)((const float *)w)[i];
    if (wtype == 2) return ((const double *)w)[i];
    return bf16_to_double(((const uint16_t *)w)[i]);
}

/* ---- gate (Section 2.1: gating network scores the experts) --------------- */

/*
 * fp32 gate logits, logits[t,e] = sum_i X[t,i] * Wg[e,i], in the fixed order:
 * the d elements are cut into vectors of V consecutive elements; vector c
 * belongs to lane (c mod 64); each lane accumulates its elements in increasing
 * i with a fused multiply-add starting from 0; the 64 lane sums are then
 * combined by a butterfly, step m = 32,16,8,4,2,1: every lane l replaces its
 * value by value[l] + value[l xor m].  After the last step all lanes hold the
 * same number, which is the logit.
 */
void ko_gate_logits_f32(const float *X, const float *Wg, int N, int d, int E, int V,
                        float *logits) {
    for (int t = 0; t < N; ++t) {
        for (int e = 0; e < E; ++e) {
            float lane[KO_LANES], next[KO_LANES];
            for (int l = 0; l < KO_LANES; ++l) lane[l] = 0.0f;
            for (int i = 0; i < d; ++i) {
                int l = (i / V) % KO_LANES;
                lane[l] = fmaf(X[(size_t)t * d + i], Wg[(size_t)e * d + i], lane[l]);
            }
            for (int m = KO_LANES / 2; m >= 1; m >>= 1) {
                for (int l = 0; l < KO_LANES; ++l) next[l] = lane[l] + lane[l ^ m];
                memcpy(lane, next, sizeof lane);
            }
            logits[(size_t)t * E + e] = lane[0];
        }
    }
}

/* The same logits in fp64 with a plain left-to-right sum (diagnostic). */
void ko_gate_logits_f64(const float *X, const float *Wg, int N, int d, int E, double *logits) {
    for (int t = 0; t < N; ++t)
        for (int e = 0; e < E; ++e) {
            double s = 0.0;
            for (int i = 0; i < d; ++i)
                s += (double)X[(size_t)t * d + i] * (double)Wg[(size_t)e * d + i];
            logits[(size_t)t * E + e] = s;
        }
}

/*
 * Top-k activation: idx[t,0..k-1] = the k experts with the largest logits,
 * listed by (logit descending, expert index ascending).
 */
void ko_topk(const float *logits, int N, int E, int k, int32_t *idx) {
    char *taken = (char *)malloc((size_t)E);
    for (int t = 0; t < N; ++t) {
        const float *row = logits + (size_t)t * E;
        memset(taken, 0, (size_t)E);
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || row[e] > row[best]) best = e; /* strict: lower index wins ties */
            }
            taken[best] = 1;
            idx[(size_t)t * k + j] = best;
        }
    }
    free(taken);
}

/*
 * Routing weights of the selected experts.
 * renorm != 0: w[t,j] = exp(l_j - m) / sum_{j'<k} exp(l_j' - m), m = l_0 (the
 *              largest), i.e. the softmax over all experts renormalised over
 *              the winners.
 * renorm == 0: w[t,j] = softmax over all E experts, taken at the winners.
 */
void ko_gate_weights(const float *logits, const int32_t *idx, int N, int E, int k, int renorm,
                     double *w) {
    for (int t = 0; t < N; ++t) {
        const float *row = logits + (size_t)t * E;
        const int32_t *sel = idx + (size_t)t * k;
        double m = (double)row[sel[0]];
        double den = 0.0;
        if (renorm) {
            for (int j = 0; j < k; ++j) den += exp((double)row[sel[j]] - m);
        } else {
            for (int e = 0; e < E; ++e) den += exp((double)row[e] - m);
        }
        for (int j = 0; j < k; ++j) w[(size_t)t * k + j] = exp((double)row[sel[j]] - m) / den;
    }
}

/* ---- dispatch (Section 5: the expert layer is divided by experts) ------- */

/*
 * Assignment a = t*k + j sends token t to expert idx[a].
 * counts[e]   = number of assignments to e
 * offsets     = exclusive prefix sum of counts over e = 0..E-1 (E+1 entries)
 * inv_perm[a] = offsets[idx[a]] + number of earlier assignments a' < a to the
 *               same expert (stable grouping); perm is its inverse
 * nbatch[e]   = number of batches of the group with at least one token on e
 * exec_order  = experts with counts > 0 by (nbatch desc, counts desc, e asc);
 *               entries past *n_active are set to -1
 */
void ko_dispatch(const int32_t *idx, int N, int k, int E, const int32_t *batch_offsets, int B,
                 int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                 int32_t *nbatch, int32_t *exec_order, int32_t *n_active) {
    int A = N * k;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int a = 0; a < A; ++a) counts[idx[a]]++;
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t *seen = (int32_t *)calloc((size_t)(E > 0 ? E : 1), sizeof(int32_t));
    for (int a = 0; a < A; ++a) {
        int e = idx[a];
        inv_perm[a] = offsets[e] + seen[e];
        seen[e]++;
    }
    for (int a = 0; a < A; ++a) perm[inv_perm[a]] = a;
    for (int e = 0; e < E; ++e) nbatch[e] = 0;
    for (int b = 0; b < B; ++b) {
        for (int e = 0; e < E; ++e) seen[e] = 0;
        for (int t = batch_offsets[b]; t < batch_offsets[b + 1]; ++t)
            for (int j = 0; j < k; ++j) seen[idx[(size_t)t * k + j]] = 1;
        for (int e = 0; e < E; ++e) nbatch[e] += seen[e];
    }
    free(seen);
    int n = 0;
    for (int e = 0; e < E; ++e)
        if (counts[e] > 0) exec_order[n++] = e;
    for (int i = 1; i < n; ++i) { /* insertion sort, keys are distinct through e */
        int e = exec_order[i], p = i;
        while (p > 0) {
            int q = exec_order[p - 1];
            int q_first = nbatch[q] > nbatch[e] ||
                          (nbatch[q] == nbatch[e] &&
                           (counts[q] > counts[e] || (counts[q] == counts[e] && q < e)));
            if (q_first) break;
            exec_order[p] = q;
            --p;
        }
        exec_order[p] = e;
    }
    for (int i = n; i < E; ++i) exec_order[i] = -1;
    *n_active = n;
}

/* ---- experts and the weighted sum (Section 2.1) ------------------------- */

static double silu(double z) { return z / (1.0 + exp(-z)); }

/* One expert on one token: out = W2 * (silu(W1 x) .* (W3 x)); W1,W3 [f,d], W2 [d,f]. */
static void expert_swiglu(const double *x, const void *w1, const void *w3, const void *w2,
                          int wtype, int d, int f, double *h, double *out) {
    for (int n = 0; n < f; ++n) {
        double g = 0.0, u = 0.0;
        for (int i = 0; i < d; ++i) {
            g += weight_at(w1, wtype, (size_t)n * d + i) * x[i];
            u += weight_at(w3, wtype, (size_t)n * d + i) * x[i];
        }
        h[n] = silu(g) * u;
    }
    for (int m = 0; m < d; ++m) {
        double s = 0.0;
        for (int n = 0; n < f; ++n) s += weight_at(w2, wtype, (size_t)m * f + n) * h[n];
        out[m] = s;
    }
}

/* Exposed for tests: a single expert applied to a single token. */
void ko_expert_ffn(const double *x, const void *w1, const void *w3, const void *w2, int wtype,
                   int d, int f, double *out) {
    double *h = (double *)malloc(sizeof(double) * (size_t)f);
    expert_swiglu(x, w1, w3, w2, wtype, d, f, h, out);
    free(h);
}

/*
 * Layer output for the tokens listed in sel[0..n_sel-1] (sel == NULL: tokens
 * 0..n_sel-1):
 *   Y[t] = sum_{j<k} w[t,j] * FFN_{idx[t,j]}(X[t]) + sum_{s<S} FFN_{E+s}(X[t])
 * slots in order j = 0..k-1, then shared experts s = 0..S-1.
 * w1/w3/w2 are arrays of E+S pointers.  expert_kind 0 = SwiGLU FFN, 1 = identity
 * expert (FFN_e(x) = x, used to check the combine alone).
 * Y is [n_sel, d] in fp64.
 */
void ko_moe_forward(const float *X, const int32_t *idx, const double *w, int d, int f, int E,
                    int k, int S, const void *const *w1, const void *const *w3,
                    const void *const *w2, int wtype, int expert_kind, const int32_t *sel,
                    int n_sel, double *Y) {
    (void)E;
#pragma omp parallel
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)d);
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
        double *h = (double *)malloc(sizeof(double) * (size_t)(f > 0 ? f : 1));
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_sel; ++r) {
            int t = sel ? sel[r] : r;
            double *y = Y + (size_t)r * d;
            for (int i = 0; i < d; ++i) {
                x[i] = (double)X[(size_t)t * d + i];
                y[i] = 0.0;
            }
            for (int j = 0; j < k + S; ++j) {
                int e = j < k ? idx[(size_t)t * k + j] : E + (j - k);
                double wt = j < k ? w[(size_t)t * k + j] : 1.0;
                if (expert_kind == 1) {
                    for (int i = 0; i < d; ++i) o[i] = x[i];
                } else {
                    expert_swiglu(x, w1[e], w3[e], w2[e], wtype, d, f, h, o);
                }
                for (int i = 0; i < d; ++i) y[i] += wt * o[i];
            }
        }
        free(x);
        free(o);
        free(h);
    }
}

/* ------------------------------------------------------------------------------------------
 * Expert correlation table, path length l = 1 (paper Section 6.2).
 *
 * table[p][e] counts how often a token that activated expert p in the previous expert layer
 * activated expert e in this one; every (previous slot, current slot) pair of a token counts
 * once.  Plain loops over tokens and slot pairs.
 */
void ko_corr_update(const int32_t *idx_prev, const int32_t *idx_cur, int N, int k, int E,
                    int64_t *table) {
    for (int t = 0; t < N; ++t)
        for (int a = 0; a < k; ++a)
            for (int b = 0; b < k; ++b)
                table[(size_t)idx_prev[(size_t)t * k + a] * E + idx_cur[(size_t)t * k + b]] += 1;
}

/* Tendency of the batch group towards the experts of this layer, and the K experts to prefetch.
 * A token that activated p in the previous layer tends to e with the recorded frequency
 * table[p][e] / sum_e' table[p][e']; the tendencies of all tokens of all batches are added up
 * (tokens enter only through counts_prev[p], the number of assignments to p), in fp64, previous
 * experts in increasing index.  Rows never observed contribute nothing.  The K best by
 * (score desc, index asc) with a positive score are returned; *n_out <= K.
 */
void ko_corr_predict(const int64_t *table, const int32_t *counts_prev, int E, int K,
                     double *score, int32_t *experts, int32_t *n_out) {
    for (int e = 0; e < E; ++e) score[e] = 0.0;
    for (int p = 0; p < E; ++p) {
        if (counts_prev[p] <= 0) continue;
        int64_t row = 0;
        for (int e = 0; e < E; ++e) row += table[(size_t)p * E + e];
        if (row <= 0) continue;
        for (int e = 0; e < E; ++e) {
            const double freq = (double)table[(size_t)p * E + e] / (double)row;
            score[e] = score[e] + (double)counts_prev[p] * freq;
        }
    }
    int n = 0;
    for (int r = 0; r < K && r < E; ++r) {
        int best = -1;
        for (int e = 0; e < E; ++e) {
            int taken = 0;
            for (int q = 0; q < n; ++q) taken |= (experts[q] == e);
            if (taken || !(score[e] > 0.0)) continue;
            if (best < 0 || score[e] > score[best]) best = e; /* first index wins ties */
        }
        if (best < 0) break;
        experts[n++] = best;
    }
    *n_out = n;
}

/* ------------------------------------------------------------------------------------------
 * 4-bit group quantisation of expert weights (paper Section 7, "Quantization", Eq. 8).
 *
 * A row of `cols` weights is cut into groups of `group` consecutive weights; group g of row r
 * has a scale s and a zero point z (bf16-valued, real: the zero point is not an integer), and
 * every weight is a 4-bit code q in 0..15:
 *     W_q = round(W / s + z)            (ko_quant_q4, clamped to the 4-bit range)
 *     W   = s * (W_q - z)               (ko_dequant_q4)
 * Codes are stored two per byte, the even column in the low nibble.  Dequantisation is done in
 * fp64 from the exact values of s and z.  The paper converts the tensors back to their original
 * precision before computing with them: with to_bf16 != 0 the dequantised weight is rounded to
 * bfloat16 (nearest, ties to even), which is what the expert then multiplies with.
 */
/* x rounded to bfloat16 (8 significant bits), nearest-even, directly from fp64. */
static double round_to_bf16(double x) {
    if (x == 0.0 || !isfinite(x)) return x;
    int e;
    frexp(x, &e);              /* |x| = m * 2^e, 0.5 <= m < 1  ->  leading bit at 2^(e-1) */
    int qe = e - 8;            /* unit in the last place of 8 significant bits */
    if (qe < -133) qe = -133;  /* bfloat16 subnormals */
    const double q = ldexp(1.0, qe);
    return rint(x / q) * q;    /* both scalings by a power of two are exact */
}

double ko_round_bf16(double x) { return round_to_bf16(x); }

void ko_dequant_q4(const uint8_t *q, const uint16_t *s_bf16, const uint16_t *z_bf16, int rows,
                   int cols, int group, int to_bf16, double *out) {
    const int ng = cols / group;
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < cols; ++c) {
            const uint8_t byte = q[(size_t)r * (cols / 2) + c / 2];
            const int code = (c & 1) ? (byte >> 4) : (byte & 15);
            const double s = bf16_to_double(s_bf16[(size_t)r * ng + c / group]);
            const double z = bf16_to_double(z_bf16[(size_t)r * ng + c / group]);
            const double v = s * ((double)code - z);
            out[(size_t)r * cols + c] = to_bf16 ? round_to_bf16(v) : v;
        }
}

/* Eq. 8 forward for given s and z (how they are chosen is not part of it): round to nearest,
 * ties to even (rint under the default rounding mode), then clamp to 0..15. */
void ko_quant_q4(const double *w, const uint16_t *s_bf16, const uint16_t *z_bf16, int rows, int cols,
                 int group, uint8_t *q) {
    const int ng = cols / group;
    memset(q, 0, (size_t)rows * (cols / 2));
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < cols; ++c) {
            const double s = bf16_to_double(s_bf16[(size_t)r * ng + c / group]);
            const double z = bf16_to_double(z_bf16[(size_t)r * ng + c / group]);
            double v = rint(w[(size_t)r * cols + c] / s + z);
            if (v < 0.0) v = 0.0;
            if (v > 15.0) v = 15.0;
            const uint8_t code = (uint8_t)v;
            q[(size_t)r * (cols / 2) + c / 2] |= (c & 1) ? (uint8_t)(code << 4) : code;
        }
}

/* ------------------------------------------------------------------------------------------
 * Constraint-sensitive planner, stage "constraint solving" (paper Section 7, inequality group).
 *
 * n batches per batch group are enough when the compute of n batches covers the transfers that
 * must have landed at four points of the pipeline (the arrows I-IV of the pipeline figure):
 *   I    n * t_c_A                                   >= t_io_G
 *   II   n * (t_c_A + t_c_G)                         >= t_io_G + K * t_io_E
 *   III  n * (t_c_A + t_c_G) + t_c_hotE              >= t_io_G + (K + 1) * t_io_E
 *   IV   n * (t_c_A + t_c_G) + t_c_hotE + sum_Q t_c_E >= t_io_G + (K + len(Q)) * t_io_E + t_io_A
 * (K = prefetched hot experts, Q = queue of activated experts that are not hot).  The answer is
 * the smallest positive integer n that satisfies the group.  Readings: the legend's t_c_topk-E is
 * the formulas' t_c_hot-E; with an empty queue nothing cold is computed or moved, so III and IV
 * do not apply (the paper's best case).
 *
 * Written as the search the text describes: n = 1, 2, 3, ... until all inequalities hold, each
 * evaluated as printed.  Returns -1 when no n up to n_max does (e.g. no compute to hide I/O behind).
 */
int64_t ko_plan_batches(double t_c_A, double t_c_G, double t_c_hotE, const double *t_c_E, int len_q,
                        double t_io_A, double t_io_G, double t_io_E, int K, int64_t n_max) {
    double sum_q = 0.0;
    for (int i = 0; i < len_q; ++i) sum_q += t_c_E[i];
    for (int64_t n = 1; n <= n_max; ++n) {
        const double dn = (double)n;
        if (!(dn * t_c_A >= t_io_G)) continue;
        if (!(dn * (t_c_A + t_c_G) >= t_io_G + K * t_io_E)) continue;
        if (len_q > 0) {
            if (!(dn * (t_c_A + t_c_G) + t_c_hotE >= t_io_G + (K + 1) * t_io_E)) continue;
            if (!(dn * (t_c_A + t_c_G) + t_c_hotE + sum_q >= t_io_G + (K + len_q) * t_io_E + t_io_A)) continue;
        }
        return n;
    }
    return -1;
}
