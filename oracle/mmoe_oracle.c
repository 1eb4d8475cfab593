/*
 * CPU oracle for the forward pass of one multi-model MoE layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the
 * GPU library is checked against.  It shares no code with the GPU path and the
 * product never calls it; only tests, the smoke check and the benchmark's
 * reported CPU baseline do.
 *
 * What the layer computes (paper, Algorithm 2, the per-layer body, and the
 * description of the gate in section 3.2): the requested model's gate scores
 * the activations and the top experts are selected with weighted-averaging
 * coefficients; each selected (layer, expert) location is looked up in the
 * expert map; the expert that is resident for that location is applied, which
 * may belong to another model when the location is consolidated and is the
 * requested model's own otherwise (Figure 3); the experts' outputs are combined
 * with the gate's coefficients.  Here one batch mixes tokens of several
 * variants, so each token carries its variant id, the map is the table
 * M[v][e] -> pool slot, and the pool holds every resident expert once.
 *
 * Readings where the paper gives no formula:
 *   - router logit: fp32 dot product in a fixed summation order (below), plus
 *     an optional fp32 bias added last;
 *   - selection: k times the largest remaining logit, ties to the lower index;
 *     picks are listed in selection order;
 *   - coefficients, two readings of "the gate network generates weighted
 *     averaging coefficients for each expert, and ... the top experts are
 *     selected" (section 3.2).  Gate mode 0: softmax over the k selected logits
 *     (they sum to 1; k = 1 gives exactly 1), the Mixtral-style gate.  Gate
 *     mode 1: softmax over all E logits, each selected expert keeping its own
 *     probability with no renormalisation (they sum to less than 1 unless
 *     k = E), the Switch-style gate of the family the paper uses for its
 *     scalability experiment (section 4.3);
 *   - SwiGLU expert: (silu(x W1) * (x W3)) W2, silu(a) = a / (1 + exp(-a));
 *     ReLU expert: relu(x W1) W2; GELU expert: gelu(x W1) W2 with
 *     gelu(a) = a * Phi(a) = a/2 * (1 + erf(a / sqrt 2)); no biases; an expert
 *     is 3*d*f (resp. 2*d*f) parameters, matching the 176.16 M the paper states
 *     for Mixtral;
 *   - bf16 storage: every stored tensor is bf16; sums are carried in fp64 here;
 *     the activation H is rounded to bf16 before the second product.
 *
 * Summation order of the router dot product (part of the written contract
 * because it decides integer outputs): element i belongs to lane
 * (i div 4) mod 64; each lane accumulates its elements in ascending i with one
 * fused multiply-add per element, in fp32, starting from +0; the 64 partial
 * sums are then combined by a butterfly: for off = 32,16,8,4,2,1 every lane l
 * replaces its value by p[l] + p[l xor off].  All lanes end with the same
 * value, which is the logit.
 *
 * Dtype codes: 0 = fp32, 1 = bf16 (raw 16-bit patterns).  Weight layout is the
 * plain one: W1, W3 [S, d, f]; W2 [S, f, d]; Wr [V, E, d]; all row-major.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_RELU = 0, ORC_SWIGLU = 1, ORC_GELU = 2 };
enum { ORC_GATE_SELECTED = 0, ORC_GATE_ALL = 1 };

int mmoe_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline float bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* stored element -> exact fp32 value */
static inline float load_elem(const void *base, int dtype, size_t i)
{
    return dtype == ORC_BF16 ? bf16_to_f32(((const uint16_t *)base)[i]) : ((const float *)base)[i];
}

/* round a double to the nearest bf16 (ties to even), returned as a double */
static double round_to_bf16(double x)
{
    if (x == 0.0 || !isfinite(x))
        return x;
    int e;
    double m = frexp(x, &e);          /* x = m * 2^e, 0.5 <= |m| < 1       */
    if (e < -125) e = -125;           /* subnormal range: fixed quantum   */
    double q = ldexp(1.0, e - 8);     /* bf16 keeps 8 significant bits    */
    (void)m;
    return nearbyint(x / q) * q;      /* default rounding mode: to even   */
}

/* ---- step R: router logits, top-k, coefficients ------------------------------ */

static float canonical_dot(const void *x, size_t xoff, const void *w, size_t woff, int d, int dtype)
{
    float p[64], q[64];
    for (int l = 0; l < 64; ++l)
        p[l] = 0.0f;
    for (int i = 0; i < d; ++i) {
        int lane = (i / 4) % 64;
        p[lane] = fmaf(load_elem(x, dtype, xoff + i), load_elem(w, dtype, woff + i), p[lane]);
    }
    for (int off = 32; off >= 1; off >>= 1) {
        for (int l = 0; l < 64; ++l)
            q[l] = p[l] + p[l ^ off];
        memcpy(p, q, sizeof p);
    }
    return p[0];
}

/*
 * topk_idx [T,k] int32, topk_w [T,k] double, logits [T,E] float (may be NULL).
 */
void mmoe_oracle_route(int T, int d, int V, int E, int k, int dtype, int gate, const void *X,
                       const int32_t *vid, const void *Wr, const float *br,
                       int32_t *topk_idx, double *topk_w, float *logits)
{
    (void)V;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        int v = vid[t];
        float *lg = (float *)malloc(sizeof(float) * E);
        char *taken = (char *)calloc(E, 1);
        for (int e = 0; e < E; ++e) {
            float s = canonical_dot(X, (size_t)t * d, Wr, ((size_t)v * E + e) * d, d, dtype);
            if (br)
                s = s + br[(size_t)v * E + e];
            lg[e] = s;
            if (logits)
                logits[(size_t)t * E + e] = s;
        }
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e])
                    continue;
                if (best < 0 || lg[e] > lg[best]) /* strict: equal keeps the lower index */
                    best = e;
            }
            taken[best] = 1;
            topk_idx[(size_t)t * k + j] = best;
        }
        double m = (double)lg[topk_idx[(size_t)t * k]];
        double z = 0.0;
        for (int j = 0; j < k; ++j) {
            double ej = exp((double)lg[topk_idx[(size_t)t * k + j]] - m);
            topk_w[(size_t)t * k + j] = ej;
            z += ej;
        }
        if (gate == ORC_GATE_ALL) { /* the normaliser runs over every expert, selected or not */
            z = 0.0;
            for (int e = 0; e < E; ++e)
                z += exp((double)lg[e] - m);
        }
        for (int j = 0; j < k; ++j)
            topk_w[(size_t)t * k + j] /= z;
        free(lg);
        free(taken);
    }
}

/* ---- steps M and G: table lookup, histogram, stable grouping ----------------- */

void mmoe_oracle_remap_group(int T, int k, int E, int S, const int32_t *vid,
                             const int32_t *topk_idx, const int32_t *M, int32_t *slot,
                             int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm)
{
    int P = T * k;
    for (int s = 0; s < S; ++s)
        counts[s] = 0;
    for (int p = 0; p < P; ++p) {
        int t = p / k;
        slot[p] = M[(size_t)vid[t] * E + topk_idx[p]];
        counts[slot[p]] += 1;
    }
    offsets[0] = 0;
    for (int s = 0; s < S; ++s)
        offsets[s + 1] = offsets[s] + counts[s];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (S > 0 ? S : 1));
    for (int s = 0; s < S; ++s)
        cursor[s] = offsets[s];
    for (int p = 0; p < P; ++p) { /* ascending p: stable */
        int r = cursor[slot[p]]++;
        perm[r] = p;
        inv_perm[p] = r;
    }
    free(cursor);
}

/* Xg[r,:] = X[perm[r] / k, :]  (a copy of stored elements) */
void mmoe_oracle_gather(int P, int d, int k, int dtype, const void *X, const int32_t *perm, void *Xg)
{
    size_t es = dtype == ORC_BF16 ? 2 : 4;
    for (int r = 0; r < P; ++r)
        memcpy((char *)Xg + (size_t)r * d * es, (const char *)X + (size_t)(perm[r] / k) * d * es,
               (size_t)d * es);
}

/* ---- step F: one expert applied to one row ------------------------------------ */

static void ffn_row(int d, int f, int dtype, int act, const void *Xsrc, size_t xrow, const void *W1,
                    const void *W3, const void *W2, int s, double *g, double *u, double *y)
{
    size_t w13 = (size_t)s * d * f, w2 = (size_t)s * f * d;
    for (int n = 0; n < f; ++n) {
        g[n] = 0.0;
        u[n] = 0.0;
    }
    for (int i = 0; i < d; ++i) {
        double xi = (double)load_elem(Xsrc, dtype, xrow * d + i);
        size_t row = w13 + (size_t)i * f;
        for (int n = 0; n < f; ++n)
            g[n] += xi * (double)load_elem(W1, dtype, row + n);
        if (act == ORC_SWIGLU)
            for (int n = 0; n < f; ++n)
                u[n] += xi * (double)load_elem(W3, dtype, row + n);
    }
    for (int n = 0; n < f; ++n) {
        double h;
        if (act == ORC_SWIGLU)
            h = g[n] / (1.0 + exp(-g[n])) * u[n];
        else if (act == ORC_GELU)
            h = 0.5 * g[n] * (1.0 + erf(g[n] / sqrt(2.0)));
        else
            h = g[n] > 0.0 ? g[n] : 0.0;
        g[n] = dtype == ORC_BF16 ? round_to_bf16(h) : h;
    }
    for (int c = 0; c < d; ++c)
        y[c] = 0.0;
    for (int n = 0; n < f; ++n) {
        double hn = g[n];
        size_t row = w2 + (size_t)n * d;
        for (int c = 0; c < d; ++c)
            y[c] += hn * (double)load_elem(W2, dtype, row + c);
    }
}

/*
 * Apply slot rslot[i]'s expert to row xrow[i] of Xsrc, for i in [0, n).
 * out [n, d] double.  The grouped stage is the case xrow[r] = r over Xg with
 * rslot[r] = the slot whose [offsets[s], offsets[s+1]) contains r.
 */
void mmoe_oracle_ffn_rows(int n, const int32_t *xrow, const int32_t *rslot, int d, int f, int dtype,
                          int act, const void *Xsrc, const void *W1, const void *W3, const void *W2,
                          double *out)
{
#pragma omp parallel
    {
        double *g = (double *)malloc(sizeof(double) * f);
        double *u = (double *)malloc(sizeof(double) * f);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n; ++i)
            ffn_row(d, f, dtype, act, Xsrc, (size_t)xrow[i], W1, W3, W2, rslot[i], g, u,
                    out + (size_t)i * d);
        free(g);
        free(u);
    }
}

/* ---- step C: Y[t,:] = sum_j w[t,j] * Yg[inv_perm[t k + j], :], ascending j ------ */

void mmoe_oracle_combine(int T, int d, int k, const double *Yg, const int32_t *inv_perm,
                         const double *topk_w, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double *y = Y + (size_t)t * d;
        for (int c = 0; c < d; ++c)
            y[c] = 0.0;
        for (int j = 0; j < k; ++j) {
            const double *src = Yg + (size_t)inv_perm[(size_t)t * k + j] * d;
            double w = topk_w[(size_t)t * k + j];
            for (int c = 0; c < d; ++c)
                y[c] += w * src[c];
        }
    }
}

/* ---- Algorithm 1 (initial expert loader): degree of similarity of one expert location ------- */

/*
 * The paper flattens an expert block into one vector and takes the L2 distance between the
 * experts that two models hold at the same (layer, expert) location; with more than two models the
 * degree of similarity of the location is the sum over all model-to-model combinations
 * (section 3.1).  Here: V models, the location's flattened expert of model v at ptrs[v]
 * (n stored elements); returns  sum_{i<j} sqrt( sum_t (a_i[t] - a_j[t])^2 )  in double.
 * The listing sums over ordered pairs, which doubles every location's value and ranks them
 * the same.  Fixed partition into runs of 2^20 elements, partial sums added in ascending order:
 * the result does not depend on the number of threads.
 */
double mmoe_oracle_location_distance(int V, size_t n, int dtype, const void *const *ptrs)
{
    const size_t run = (size_t)1 << 20;
    const size_t nrun = (n + run - 1) / run;
    double total = 0.0;
    for (int i = 0; i < V; ++i)
        for (int j = i + 1; j < V; ++j) {
            double *part = (double *)malloc(sizeof(double) * (nrun ? nrun : 1));
#pragma omp parallel for schedule(static)
            for (size_t r = 0; r < nrun; ++r) {
                size_t lo = r * run, hi = lo + run < n ? lo + run : n;
                double acc = 0.0;
                for (size_t t = lo; t < hi; ++t) {
                    double df = (double)load_elem(ptrs[i], dtype, t) - (double)load_elem(ptrs[j], dtype, t);
                    acc += df * df;
                }
                part[r] = acc;
            }
            double sq = 0.0;
            for (size_t r = 0; r < nrun; ++r)
                sq += part[r];
            free(part);
            total += sqrt(sq);
        }
    return total;
}
