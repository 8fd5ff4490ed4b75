/* CPU oracle of the non-expert (attention) layer of the multi-batch pipeline.
 * TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it; the product path never does.
 *
 * The paper's MoE block (Section 2.1) is an attention layer and an MoE layer, each with its
 * normalisation layer folded in (Section 4); Algorithm 1 runs the non-expert layer batch by
 * batch, each batch bringing its hidden state h and its key-value cache c.  The paper takes the
 * attention arithmetic from the models it evaluates (Mixtral family, Section 9.1); what is
 * written out here is the textbook definition of that layer for one decoding step:
 *
 *   xn = x / sqrt(mean(x^2) + eps) * g                         (RMS normalisation)
 *   q = Wq xn, k = Wk xn, v = Wv xn                             (projections)
 *   q, k rotated by position (rotary embedding, half-split pairs (i, i + hd/2),
 *       angle = pos * theta^(-2i/hd))
 *   cache[pos] = (k, v) in the cache's storage type (bf16)
 *   o_h = softmax_p(q_h . K_g[p] / sqrt(hd)) V_g[p],  p = 0..pos, g = h / (Hq/Hkv)
 *   y = x + Wo concat_h(o_h)
 *
 * All arithmetic is fp64; the only roundings are the ones a storage format forces (the new
 * cache rows are bf16, and attention reads them back from the cache).
 *
 * Cache layout: [n_seq][Hkv][max_len][hd] bf16 bit patterns.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_bits_to_double(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* nearest bf16, ties to even; finite inputs inside the bf16 range */
static uint16_t double_to_bf16_bits(double x) {
    if (x == 0.0 || isnan(x) || isinf(x)) {
        float f = (float)x;
        uint32_t u;
        memcpy(&u, &f, sizeof u);
        return (uint16_t)(u >> 16);
    }
    int ex;
    (void)frexp(fabs(x), &ex);      /* |x| = m 2^ex, m in [0.5, 1) */
    int e = ex - 1;                 /* |x| in [2^e, 2^(e+1)) */
    if (e < -126) e = -126;         /* subnormal spacing */
    const double ulp = ldexp(1.0, e - 7);
    const double r = nearbyint(x / ulp) * ulp; /* default rounding mode: ties to even */
    float f = (float)r;                         /* exact: r has at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

uint16_t ka_bf16_bits(double x) { return double_to_bf16_bits(x); }

static double wat(const void *w, int wtype, size_t i) {
    if (wtype == 0) return (double)((const float *)w)[i];
    if (wtype == 2) return ((const double *)w)[i];
    return bf16_bits_to_double(((const uint16_t *)w)[i]);
}

/* RMS normalisation of one row. */
void ka_rmsnorm(const double *x, const void *g, int wtype, int d, double eps, double *out) {
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += x[i] * x[i];
    const double r = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; ++i) out[i] = x[i] * r * wat(g, wtype, i);
}

/* Rotary embedding of one head vector (hd even) at integer position pos, in place. */
void ka_rope(double *v, int hd, int pos, double theta) {
    const int half = hd / 2;
    for (int i = 0; i < half; ++i) {
        const double ang = (double)pos * pow(theta, -2.0 * i / hd);
        const double c = cos(ang), s = sin(ang);
        const double a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

/* y = W x, W [rows, cols] row-major */
static void matvec(const void *w, int wtype, int rows, int cols, const double *x, double *y) {
    for (int r = 0; r < rows; ++r) {
        double acc = 0.0;
        for (int c = 0; c < cols; ++c) acc += wat(w, wtype, (size_t)r * cols + c) * x[c];
        y[r] = acc;
    }
}

/* One decoding step of the attention layer for a batch of n_seq sequences that all hold pos
 * cached positions.  kc / vc are updated in place at index pos.  y [n_seq, d] fp64. */
void ka_attn_decode(const float *x, int n_seq, int d, int Hq, int Hkv, int hd, const void *g,
                    const void *wq, const void *wk, const void *wv, const void *wo, int wtype,
                    uint16_t *kc, uint16_t *vc, int max_len, int pos, double theta, double eps,
                    double *y) {
    const int dq = Hq * hd, dkv = Hkv * hd, group = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < n_seq; ++s) {
        double *xd = malloc(sizeof(double) * d), *xn = malloc(sizeof(double) * d);
        double *q = malloc(sizeof(double) * dq), *k = malloc(sizeof(double) * dkv);
        double *v = malloc(sizeof(double) * dkv), *o = malloc(sizeof(double) * dq);
        double *p = malloc(sizeof(double) * (pos + 1)), *out = malloc(sizeof(double) * d);
        for (int i = 0; i < d; ++i) xd[i] = (double)x[(size_t)s * d + i];
        ka_rmsnorm(xd, g, wtype, d, eps, xn);
        matvec(wq, wtype, dq, d, xn, q);
        matvec(wk, wtype, dkv, d, xn, k);
        matvec(wv, wtype, dkv, d, xn, v);
        for (int h = 0; h < Hq; ++h) ka_rope(q + (size_t)h * hd, hd, pos, theta);
        for (int h = 0; h < Hkv; ++h) ka_rope(k + (size_t)h * hd, hd, pos, theta);
        for (int h = 0; h < Hkv; ++h) {
            uint16_t *krow = kc + (((size_t)s * Hkv + h) * max_len + pos) * hd;
            uint16_t *vrow = vc + (((size_t)s * Hkv + h) * max_len + pos) * hd;
            for (int i = 0; i < hd; ++i) {
                krow[i] = double_to_bf16_bits(k[(size_t)h * hd + i]);
                vrow[i] = double_to_bf16_bits(v[(size_t)h * hd + i]);
            }
        }
        for (int h = 0; h < Hq; ++h) {
            const int gk = h / group;
            const uint16_t *K = kc + ((size_t)s * Hkv + gk) * max_len * hd;
            const uint16_t *V = vc + ((size_t)s * Hkv + gk) * max_len * hd;
            double mx = -INFINITY;
            for (int t = 0; t <= pos; ++t) {
                double acc = 0.0;
                for (int i = 0; i < hd; ++i) acc += q[(size_t)h * hd + i] * bf16_bits_to_double(K[(size_t)t * hd + i]);
                p[t] = acc / sqrt((double)hd);
                if (p[t] > mx) mx = p[t];
            }
            double den = 0.0;
            for (int t = 0; t <= pos; ++t) {
                p[t] = exp(p[t] - mx);
                den += p[t];
            }
            for (int i = 0; i < hd; ++i) {
                double acc = 0.0;
                for (int t = 0; t <= pos; ++t) acc += p[t] * bf16_bits_to_double(V[(size_t)t * hd + i]);
                o[(size_t)h * hd + i] = acc / den;
            }
        }
        matvec(wo, wtype, d, dq, o, out);
        for (int i = 0; i < d; ++i) y[(size_t)s * d + i] = xd[i] + out[i];
        free(xd); free(xn); free(q); free(k); free(v); free(o); free(p); free(out);
    }
}
