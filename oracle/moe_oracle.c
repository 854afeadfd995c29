/*
 * CPU oracle for the MoE draft / verify layer of MoE-SpeQ (arXiv 2511.14102).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU library is
 * checked against.  It shares no code, header, table or helper with the GPU path and the
 * product never calls it.  Everything is fp64, plain loops, no blocking, no reordering.
 * Inputs are the *logical* layouts: bf16 / fp16 values arrive as their 16-bit patterns and
 * are widened exactly here; int4 codes arrive one per byte.
 *
 * What it computes (paper section 2.1: a router produces a distribution over the experts,
 * the top-k are selected per token, their FFN outputs are combined weighted by the router
 * scores; section 3.4.2: gate and shared experts stay 16-bit, all other expert weights are
 * 4-bit in the draft; section 4.1.3: 4-bit groups along the input dimension;
 * section 3.4.4: tokens are regrouped so that each expert's tokens are contiguous;
 * section 2.3: verification needs the union of the experts of all tokens of the window):
 *
 *   l[t,e]   = sum_h x[t,h] * Wr[e,h] + b[e]
 *   ids[t,:] = the k largest l[t,:], descending, equal values -> lower index first
 *   p        = softmax(l[t,:]);  conf[t,j] = p[ids[t,j]]
 *   w[t,j]   = conf[t,j] / sum_j conf[t,j]   (renormalise)   or   conf[t,j]
 *   FFN_e(x) = Wd_e * ( silu(Wg_e x) (.) (Wu_e x) ),  silu(a) = a / (1 + exp(-a))
 *   y[t]     = sum_j w[t,j] FFN_{ids[t,j]}(x[t]) + sum_s FFN_shared_s(x[t])
 *   draft:  W = (q - z) * s per group of g input columns;   verify:  W = bf16 value
 *
 * Every function has at least one pin in tests/test_oracle_pins.py that does not go
 * through this file (brute force, closed forms, scipy / numpy routines, invariants).
 * The paper prints no worked numeric example of this path, so there is no golden value
 * from the paper itself.
 *
 * The only concession to run time is `#pragma omp parallel for` over the independent
 * output rows of a matrix-vector product; each row is still one sequential fp64 sum.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- exact widening of the 16-bit formats ------------------------------------------- */

/* bf16 is the upper half of an IEEE binary32. */
double orc_bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double orc_fp16_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int ex = (h >> 10) & 0x1f;
    int fr = h & 0x3ff;
    double v;
    if (ex == 0)
        v = ldexp((double)fr, -24);                 /* zero and subnormals */
    else if (ex == 31)
        v = fr ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + fr), ex - 25);    /* (1 + fr/1024) * 2^(ex-15) */
    return sign ? -v : v;
}

/* ---- router: logits, top-k, softmax weights (section 2.1) ---------------------------- */

/*
 * x [T,H] bf16 bits, wr [E,H] bf16 bits, bias [E] fp32 or NULL.
 * Outputs: ids [T,k]; w, conf [T,k]; logits [T,E] (may be NULL).
 */
void orc_route(const uint16_t *x, const uint16_t *wr, const float *bias,
               int T, int H, int E, int k, int renormalize,
               int32_t *ids, double *w, double *conf, double *logits)
{
    double *l = (double *)malloc(sizeof(double) * (size_t)E);
    char *taken = (char *)malloc((size_t)E);
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h)
                acc += orc_bf16_to_f64(x[(size_t)t * H + h]) * orc_bf16_to_f64(wr[(size_t)e * H + h]);
            l[e] = acc + (bias ? (double)bias[e] : 0.0);
            if (logits) logits[(size_t)t * E + e] = l[e];
        }
        /* k rounds of "largest remaining"; strict > keeps the lowest index among equals */
        memset(taken, 0, (size_t)E);
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || l[e] > l[best]) best = e;
            }
            taken[best] = 1;
            ids[(size_t)t * k + j] = best;
        }
        /* softmax over all E logits, shifted by the row maximum */
        double mx = l[0];
        for (int e = 1; e < E; ++e) if (l[e] > mx) mx = l[e];
        double den = 0.0;
        for (int e = 0; e < E; ++e) den += exp(l[e] - mx);
        double sel = 0.0;
        for (int j = 0; j < k; ++j) {
            double p = exp(l[ids[(size_t)t * k + j]] - mx) / den;
            conf[(size_t)t * k + j] = p;
            sel += p;
        }
        for (int j = 0; j < k; ++j)
            w[(size_t)t * k + j] = renormalize ? conf[(size_t)t * k + j] / sel
                                               : conf[(size_t)t * k + j];
    }
    free(l);
    free(taken);
}

/* ---- token -> expert histogram and stable permutation (section 3.4.4) ---------------- */

/*
 * ids [n] (n = T*k assignments, index a = t*k + j).  count [E], off [E+1] exclusive scan,
 * perm [n]: assignment indices ordered by expert, ascending a within one expert.
 */
void orc_perm(const int32_t *ids, int n, int E, int32_t *count, int32_t *off, int32_t *perm)
{
    for (int e = 0; e < E; ++e) count[e] = 0;
    for (int a = 0; a < n; ++a) count[ids[a]]++;
    off[0] = 0;
    for (int e = 0; e < E; ++e) off[e + 1] = off[e] + count[e];
    int pos = 0;
    for (int e = 0; e < E; ++e)
        for (int a = 0; a < n; ++a)
            if (ids[a] == e) perm[pos++] = a;
}

/* ---- union of the experts of a window (section 2.3; |E_new| of section 3.2.2) -------- */

/*
 * ids [n] any order, values in [0,E).  slot_of_expert [E] (-1 = not resident) or NULL.
 * mask [(E+63)/64]; list [E] ascending unique ids, *n_list; missing [E] = listed experts
 * whose slot is -1 (ascending), *n_missing (0 when slot_of_expert is NULL).
 */
void orc_union(const int32_t *ids, int n, int E, const int32_t *slot_of_expert,
               uint64_t *mask, int32_t *list, int32_t *n_list,
               int32_t *missing, int32_t *n_missing)
{
    int words = (E + 63) / 64;
    for (int i = 0; i < words; ++i) mask[i] = 0;
    for (int a = 0; a < n; ++a) mask[ids[a] / 64] |= (uint64_t)1 << (ids[a] % 64);
    int nl = 0, nm = 0;
    for (int e = 0; e < E; ++e) {
        if (!((mask[e / 64] >> (e % 64)) & 1)) continue;
        list[nl++] = e;
        if (slot_of_expert && slot_of_expert[e] < 0) missing[nm++] = e;
    }
    *n_list = nl;
    *n_missing = nm;
}

/* ---- expert FFN ---------------------------------------------------------------------- */

static double silu(double a) { return a / (1.0 + exp(-a)); }

/* out[r] = sum_c W[r,c] v[c], W bf16 bits row-major [R,C] */
static void matvec_bf16(const uint16_t *W, int R, int C, const double *v, double *out)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < R; ++r) {
        double acc = 0.0;
        for (int c = 0; c < C; ++c)
            acc += orc_bf16_to_f64(W[(size_t)r * C + c]) * v[c];
        out[r] = acc;
    }
}

/*
 * out[r] = sum_c (q[r,c] - z[r,c/g]) * s[r,c/g] * v[c]
 * q one code per byte [R,C]; s, z fp16 bits [R, C/g]  (section 4.1.3: 4-bit, group size g)
 */
static void matvec_int4(const uint8_t *q, const uint16_t *s, const uint16_t *z,
                        int R, int C, int g, const double *v, double *out)
{
    int G = C / g;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < R; ++r) {
        double acc = 0.0;
        for (int c = 0; c < C; ++c) {
            double sc = orc_fp16_to_f64(s[(size_t)r * G + c / g]);
            double zp = orc_fp16_to_f64(z[(size_t)r * G + c / g]);
            acc += ((double)q[(size_t)r * C + c] - zp) * sc * v[c];
        }
        out[r] = acc;
    }
}

/* Dequantised weight values, for tests of the closed form: out[r,c] = (q - z) * s. */
void orc_dequant(const uint8_t *q, const uint16_t *s, const uint16_t *z,
                 int R, int C, int g, double *out)
{
    int G = C / g;
    for (int r = 0; r < R; ++r)
        for (int c = 0; c < C; ++c)
            out[(size_t)r * C + c] = ((double)q[(size_t)r * C + c]
                                      - orc_fp16_to_f64(z[(size_t)r * G + c / g]))
                                     * orc_fp16_to_f64(s[(size_t)r * G + c / g]);
}

/* One 16-bit expert on one token: out[H] = Wd ( silu(Wg x) (.) (Wu x) ).  Wg, Wu [I,H]; Wd [H,I]. */
void orc_ffn_bf16(const uint16_t *wg, const uint16_t *wu, const uint16_t *wd,
                  int H, int I, const double *x, double *out)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)I);
    double *b = (double *)malloc(sizeof(double) * (size_t)I);
    matvec_bf16(wg, I, H, x, a);
    matvec_bf16(wu, I, H, x, b);
    for (int i = 0; i < I; ++i) a[i] = silu(a[i]) * b[i];
    matvec_bf16(wd, H, I, a, out);
    free(a);
    free(b);
}

/* One 4-bit expert on one token. */
void orc_ffn_int4(const uint8_t *qg, const uint16_t *sg, const uint16_t *zg,
                  const uint8_t *qu, const uint16_t *su, const uint16_t *zu,
                  const uint8_t *qd, const uint16_t *sd, const uint16_t *zd,
                  int H, int I, int g, const double *x, double *out)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)I);
    double *b = (double *)malloc(sizeof(double) * (size_t)I);
    matvec_int4(qg, sg, zg, I, H, g, x, a);
    matvec_int4(qu, su, zu, I, H, g, x, b);
    for (int i = 0; i < I; ++i) a[i] = silu(a[i]) * b[i];
    matvec_int4(qd, sd, zd, H, I, g, a, out);
    free(a);
    free(b);
}

/* ---- the layer ----------------------------------------------------------------------- */

/*
 * Verify pass (16-bit experts).  wg, wu [E+S, I, H]; wd [E+S, H, I]; shared experts are the
 * last S.  ids, w [T,k] from orc_route.  present [E] (0 = expert not resident: its term is
 * left out, which is what a non-strict verify call does before the caller loads it) or NULL.
 * y [T,H] fp64.
 */
void orc_layer_bf16(const uint16_t *x, const uint16_t *wg, const uint16_t *wu,
                    const uint16_t *wd, int T, int H, int I, int E, int S, int k,
                    const int32_t *ids, const double *w, const uint8_t *present, double *y)
{
    size_t mat = (size_t)H * I;
    double *xv = (double *)malloc(sizeof(double) * (size_t)H);
    double *o = (double *)malloc(sizeof(double) * (size_t)H);
    for (int t = 0; t < T; ++t) {
        for (int h = 0; h < H; ++h) {
            xv[h] = orc_bf16_to_f64(x[(size_t)t * H + h]);
            y[(size_t)t * H + h] = 0.0;
        }
        for (int j = 0; j < k; ++j) {
            int e = ids[(size_t)t * k + j];
            if (present && !present[e]) continue;
            orc_ffn_bf16(wg + e * mat, wu + e * mat, wd + e * mat, H, I, xv, o);
            for (int h = 0; h < H; ++h) y[(size_t)t * H + h] += w[(size_t)t * k + j] * o[h];
        }
        for (int s = 0; s < S; ++s) {
            size_t e = (size_t)E + s;
            orc_ffn_bf16(wg + e * mat, wu + e * mat, wd + e * mat, H, I, xv, o);
            for (int h = 0; h < H; ++h) y[(size_t)t * H + h] += o[h];
        }
    }
    free(xv);
    free(o);
}

/*
 * Draft pass (4-bit routed experts, 16-bit shared experts).  q* [E, rows, cols] one code per
 * byte; s*, z* [E, rows, cols/g] fp16 bits.  Shared experts: swg, swu [S,I,H], swd [S,H,I]
 * bf16 bits (NULL when S == 0).  y [T,H] fp64.
 */
void orc_layer_int4(const uint16_t *x,
                    const uint8_t *qg, const uint16_t *sg, const uint16_t *zg,
                    const uint8_t *qu, const uint16_t *su, const uint16_t *zu,
                    const uint8_t *qd, const uint16_t *sd, const uint16_t *zd,
                    const uint16_t *swg, const uint16_t *swu, const uint16_t *swd,
                    int T, int H, int I, int E, int S, int k, int g,
                    const int32_t *ids, const double *w, double *y)
{
    (void)E;
    size_t mat = (size_t)H * I;
    size_t gu_sz = (size_t)I * (H / g), d_sz = (size_t)H * (I / g);
    double *xv = (double *)malloc(sizeof(double) * (size_t)H);
    double *o = (double *)malloc(sizeof(double) * (size_t)H);
    for (int t = 0; t < T; ++t) {
        for (int h = 0; h < H; ++h) {
            xv[h] = orc_bf16_to_f64(x[(size_t)t * H + h]);
            y[(size_t)t * H + h] = 0.0;
        }
        for (int j = 0; j < k; ++j) {
            size_t e = (size_t)ids[(size_t)t * k + j];
            orc_ffn_int4(qg + e * mat, sg + e * gu_sz, zg + e * gu_sz,
                         qu + e * mat, su + e * gu_sz, zu + e * gu_sz,
                         qd + e * mat, sd + e * d_sz, zd + e * d_sz, H, I, g, xv, o);
            for (int h = 0; h < H; ++h) y[(size_t)t * H + h] += w[(size_t)t * k + j] * o[h];
        }
        for (int s = 0; s < S; ++s) {
            orc_ffn_bf16(swg + s * mat, swu + s * mat, swd + s * mat, H, I, xv, o);
            for (int h = 0; h < H; ++h) y[(size_t)t * H + h] += o[h];
        }
    }
    free(xv);
    free(o);
}
