/*
 * psf_oracle.c -- float64 CPU oracle for causal polynomial-sketch attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is compared against.  It shares no code, header, table or
 * helper with the HIP path and must never be called from the product path;
 * only tests, the smoke check and the bench's cpu_baseline leg use it.
 *
 * Everything is float64, row-major, plain loops (no BLAS, no blocking beyond
 * what the paper's block algorithm itself states).  One call handles one
 * (batch, head) unit; the *_batch drivers at the bottom only loop over units
 * (OpenMP over units, nothing inside a unit is parallel).
 *
 * What each function follows in the paper (PolySketchFormer, arXiv 2310.01655):
 *   oracle_pswn              Algorithm 1, PolySketchWithNegativity (literal recursion)
 *   psf_oracle_sketch        Algorithm 1, the M = PolySketchWithNegativity(A, r, p/2)
 *                            step of PolySketchNonNegative
 *   psf_oracle_self_tensor   Algorithm 1, M^{(x)2}; Kronecker index order of Section 1.2
 *   psf_oracle_power_tensor  Section 2.2, exact feature map x^{(x)p}
 *   psf_oracle_attn_def      Section 3 (causal Polysketch attention, 1 + sum in the
 *                            denominator), Section 3.2 (exact weights inside a block),
 *                            Section 2.2 (<x,y>^p = <x^{(x)p}, y^{(x)p}>)
 *   psf_oracle_attn_noncausal  Section 2.2, Polysketch attention without a mask
 *   psf_oracle_attn_block    Section 3.1 block lower-triangular multiplication
 *                            (H_l, Z_l, P_l, row = p + a_i^T Z_l), Section 3.2 for P_l
 *   oracle_lpswn,            Algorithm 2 (learnable sketches, Appendix D): the recursion of
 *   psf_oracle_sketch_learned  Algorithm 1 with each projection M G replaced by a dense network
 *                            f(M) and sqrt(r) tanh(sqrt(1/r) .) around the Hadamard product
 *   oracle_lpswn_bwd,        gradient of Algorithm 2 with respect to the input rows and to the
 *   oracle_learned_net_bwd   networks' parameters (chain rule through layer norm, gelu, tanh)
 *   oracle_pswn_bwd,         gradient of the same definition (Section 3 with the weights of
 *   psf_oracle_attn_bwd      Sections 3.1/3.2, sketch of Algorithm 1) with respect to Q, K, V:
 *                            the chain rule written out pair by pair; the paper trains
 *                            through this function but prints no formula for it
 *
 * Pins (tests/test_oracle_*.py): brute-force masked polynomial attention written
 * in numpy, block-size invariance, definition == block algorithm, p = 2 base
 * case, closed forms for row 0 and V == 1, Monte-Carlo moments of the sketch,
 * non-negativity and the convex-hull bound; the gradient functions against central
 * finite differences of the forward functions above, automatic differentiation of an
 * independently written forward, and closed forms (tests/test_oracle_bwd_pins.py).
 * No function here is unpinned.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

enum { FEAT_SKETCH = 0, FEAT_EXACT = 1 };
enum { LOCAL_EXACT = 0, LOCAL_SKETCH = 1 };

static int is_pow2(long v) { return v > 0 && (v & (v - 1)) == 0; }

static double ipow(double x, long p)
{
    double y = 1.0;
    for (long e = 0; e < p; ++e) y *= x;
    return y;
}

static double dot(const double *x, const double *y, long m)
{
    double s = 0.0;
    for (long c = 0; c < m; ++c) s += x[c] * y[c];
    return s;
}

/* ---- Algorithm 1: PolySketchWithNegativity(A in R^{k x m}, r, deg) ----------------
 * Returns a freshly malloc'ed k x cols matrix, cols = m when deg == 1, else r.
 * The Gaussian matrices are not sampled here: they are inputs.  Those with m rows
 * are taken from g_first, those with r rows from g_inner, each list consumed in the
 * order the recursion reaches its "sample G1, G2" line: left subtree, right subtree,
 * then the node itself. */
static double *oracle_pswn(const double *A, long k, long m, long r, long deg,
                           const double **g_first, const double **g_inner)
{
    if (deg == 1) {
        double *out = (double *)malloc(sizeof(double) * (size_t)k * (size_t)m);
        if (out) memcpy(out, A, sizeof(double) * (size_t)k * (size_t)m);
        return out;
    }
    double *M1 = oracle_pswn(A, k, m, r, deg / 2, g_first, g_inner);
    double *M2 = oracle_pswn(A, k, m, r, deg / 2, g_first, g_inner);
    long rows = (deg / 2 == 1) ? m : r;          /* columns of M1 and M2 */
    const double *G1, *G2;
    if (deg / 2 == 1) {             /* M1 = M2 = A: matrices with m rows */
        G1 = *g_first;  G2 = G1 + rows * r;  *g_first = G2 + rows * r;
    } else {
        G1 = *g_inner;  G2 = G1 + rows * r;  *g_inner = G2 + rows * r;
    }
    double *out = (double *)malloc(sizeof(double) * (size_t)k * (size_t)r);
    if (!M1 || !M2 || !out) { free(M1); free(M2); free(out); return NULL; }
    double scale = sqrt(1.0 / (double)r);
    for (long i = 0; i < k; ++i) {
        for (long c = 0; c < r; ++c) {
            double u = 0.0, v = 0.0;
            for (long e = 0; e < rows; ++e) {
                u += M1[i * rows + e] * G1[e * r + c];
                v += M2[i * rows + e] * G2[e * r + c];
            }
            out[i * r + c] = scale * (u * v);
        }
    }
    free(M1);
    free(M2);
    return out;
}

/* Number of Gaussian matrices the degree-p feature map uses (Theorem 1.1, item 3). */
long psf_oracle_num_g_first(long p) { return p / 2 >= 2 ? p / 2 : 0; }
long psf_oracle_num_g_inner(long p) { return p / 2 >= 4 ? p / 2 - 2 : 0; }

/* M = PolySketchWithNegativity(X, r, p/2); X is k x d.  G holds the d x r matrices
 * first, then the r x r ones.  M_out is k x r, or k x d when p == 2 (base case). */
int psf_oracle_sketch(const double *X, long k, long d, long r, long p,
                      const double *G, double *M_out)
{
    if (!is_pow2(p) || p < 2 || k < 0 || d <= 0 || r <= 0) return 1;
    const double *gf = G;
    const double *gi = G ? G + psf_oracle_num_g_first(p) * d * r : NULL;
    double *M = oracle_pswn(X, k, d, r, p / 2, &gf, &gi);
    if (!M) return 2;
    long cols = (p == 2) ? d : r;
    memcpy(M_out, M, sizeof(double) * (size_t)k * (size_t)cols);
    free(M);
    return 0;
}

/* ---- Algorithm 2: learnable sketches (Appendix D) -----------------------------------
 * One network f: R^win -> R^r, applied to every row (the reading of Appendix D taken here):
 *   u  = LayerNorm(a; g1, b1)                  layer normalisation "before the input"
 *   h1 = gelu(u W1)          W1: win x 8r      first hidden layer, size 8r
 *   v  = LayerNorm(h1; g2, b2)                 "and [before] the second hidden layer"
 *   h2 = v W2                W2: 8r x r        second hidden layer, size r, no activation
 *   h3 = gelu(h2 W3)         W3: r x 8r        third hidden layer, size 8r
 *   f  = h3 W4               W4: 8r x r        output, dimension r
 * Dense layers carry no bias (the appendix counts 8 h r + 24 r^2 parameters per network, which
 * is exactly the four matrices); layer normalisation has a learnable scale and bias and uses
 * the biased variance with eps = 1e-6; gelu is the tanh form
 * 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))).  Parameters of one network are stored as
 * [g1, b1, W1, g2, b2, W2, W3, W4], matrices row-major (input index first). */
static long learned_net_len(long win, long r)
{
    return 2 * win + win * 8 * r + 2 * 8 * r + 8 * r * r + r * 8 * r + 8 * r * r;
}

static double gelu_tanh(double x)
{
    return 0.5 * x * (1.0 + tanh(0.7978845608028654 * (x + 0.044715 * x * x * x)));
}

static void layer_norm(const double *x, long m, const double *g, const double *b, double *out)
{
    double mean = 0.0, var = 0.0;
    for (long e = 0; e < m; ++e) mean += x[e];
    mean /= (double)m;
    for (long e = 0; e < m; ++e) var += (x[e] - mean) * (x[e] - mean);
    var /= (double)m;
    double inv = 1.0 / sqrt(var + 1e-6);
    for (long e = 0; e < m; ++e) out[e] = (x[e] - mean) * inv * g[e] + b[e];
}

static double *oracle_learned_net(const double *A, long k, long win, long r, const double **params)
{
    const double *g1 = *params, *b1 = g1 + win, *W1 = b1 + win;
    const double *g2 = W1 + win * 8 * r, *b2 = g2 + 8 * r, *W2 = b2 + 8 * r;
    const double *W3 = W2 + 8 * r * r, *W4 = W3 + r * 8 * r;
    *params = W4 + 8 * r * r;
    long hid = 8 * r;
    double *out = (double *)malloc(sizeof(double) * (size_t)k * (size_t)r);
    double *u = (double *)malloc(sizeof(double) * (size_t)(win > hid ? win : hid));
    double *h = (double *)malloc(sizeof(double) * (size_t)hid);
    double *h2 = (double *)malloc(sizeof(double) * (size_t)r);
    if (!out || !u || !h || !h2) { free(out); free(u); free(h); free(h2); return NULL; }
    for (long i = 0; i < k; ++i) {
        layer_norm(A + i * win, win, g1, b1, u);
        for (long c = 0; c < hid; ++c) {
            double s = 0.0;
            for (long e = 0; e < win; ++e) s += u[e] * W1[e * hid + c];
            h[c] = gelu_tanh(s);
        }
        layer_norm(h, hid, g2, b2, u);
        for (long c = 0; c < r; ++c) {
            double s = 0.0;
            for (long e = 0; e < hid; ++e) s += u[e] * W2[e * r + c];
            h2[c] = s;
        }
        for (long c = 0; c < hid; ++c) {
            double s = 0.0;
            for (long e = 0; e < r; ++e) s += h2[e] * W3[e * hid + c];
            h[c] = gelu_tanh(s);
        }
        for (long c = 0; c < r; ++c) {
            double s = 0.0;
            for (long e = 0; e < hid; ++e) s += h[e] * W4[e * r + c];
            out[i * r + c] = s;
        }
    }
    free(u); free(h); free(h2);
    return out;
}

/* LearnablePolysketchWithNegativity(A, r, deg): as oracle_pswn, with f1(M1) * f2(M2) inside
 * sqrt(r) tanh(sqrt(1/r) .).  Networks are consumed from *params in the order the recursion
 * reaches them: left subtree, right subtree, then f1, f2 of the node. */
static double *oracle_lpswn(const double *A, long k, long m, long r, long deg, const double **params)
{
    if (deg == 1) {
        double *out = (double *)malloc(sizeof(double) * (size_t)k * (size_t)m);
        if (out) memcpy(out, A, sizeof(double) * (size_t)k * (size_t)m);
        return out;
    }
    double *M1 = oracle_lpswn(A, k, m, r, deg / 2, params);
    double *M2 = oracle_lpswn(A, k, m, r, deg / 2, params);
    long win = (deg / 2 == 1) ? m : r;
    double *F1 = M1 ? oracle_learned_net(M1, k, win, r, params) : NULL;
    double *F2 = M2 ? oracle_learned_net(M2, k, win, r, params) : NULL;
    double *out = (double *)malloc(sizeof(double) * (size_t)k * (size_t)r);
    if (!F1 || !F2 || !out) { free(M1); free(M2); free(F1); free(F2); free(out); return NULL; }
    double sr = sqrt((double)r);
    for (long i = 0; i < k * r; ++i) out[i] = sr * tanh(F1[i] * F2[i] / sr);
    free(M1); free(M2); free(F1); free(F2);
    return out;
}

/* Number of parameters of the learned degree-p sketch: p - 2 networks (Appendix D), the
 * p/2 first-level ones with input width d, the others with input width r. */
long psf_oracle_learned_len(long d, long r, long p)
{
    if (p < 4) return 0;
    return (p / 2) * learned_net_len(d, r) + (p / 2 - 2) * learned_net_len(r, r);
}

/* M = LearnablePolysketchWithNegativity(X, r, p/2); M_out is k x r (k x d when p == 2). */
int psf_oracle_sketch_learned(const double *X, long k, long d, long r, long p,
                              const double *params, double *M_out)
{
    if (!is_pow2(p) || p < 2 || k < 0 || d <= 0 || r <= 0) return 1;
    const double *pp = params;
    double *M = oracle_lpswn(X, k, d, r, p / 2, &pp);
    if (!M) return 2;
    memcpy(M_out, M, sizeof(double) * (size_t)k * (size_t)((p == 2) ? d : r));
    free(M);
    return 0;
}

/* Phi[i, a*m + b] = M[i,a] * M[i,b]  (a (x) b lists a_1 b_1, a_1 b_2, ...). */
void psf_oracle_self_tensor(const double *M, long k, long m, double *Phi)
{
    for (long i = 0; i < k; ++i)
        for (long a = 0; a < m; ++a)
            for (long b = 0; b < m; ++b)
                Phi[(i * m + a) * m + b] = M[i * m + a] * M[i * m + b];
}

/* Phi = X^{(x)p}: x^{(x)p} = x (x) x^{(x)(p-1)}, x^{(x)1} = x.  Phi is k x d^p. */
int psf_oracle_power_tensor(const double *X, long k, long d, long p, double *Phi)
{
    long F = 1;
    for (long e = 0; e < p; ++e) F *= d;
    double *prev = (double *)malloc(sizeof(double) * (size_t)F);
    if (!prev) return 2;
    for (long i = 0; i < k; ++i) {
        const double *x = X + i * d;
        double *out = Phi + i * F;
        long len = d;
        memcpy(out, x, sizeof(double) * (size_t)d);
        for (long e = 2; e <= p; ++e) {
            memcpy(prev, out, sizeof(double) * (size_t)len);
            for (long a = 0; a < d; ++a)
                for (long t = 0; t < len; ++t) out[a * len + t] = x[a] * prev[t];
            len *= d;
        }
    }
    free(prev);
    return 0;
}

/* ---- the definition: rows of causal Polysketch attention -------------------------
 * For the listed rows i (0-based; rows == NULL means all n rows):
 *   o_i = sum_{j<=i} w_ij v_j / (1 + sum_{j<=i} w_ij)
 *   w_ij = <q_i,k_j>^p                    if feat == EXACT, or (local == EXACT and
 *                                         i, j fall in the same block of b rows)
 *        = <phi'(q_i), phi'(k_j)>         otherwise, phi'(x) = m(x) (x) m(x)
 * MQ, MK are the n x mcols sketches m(q_i), m(k_j) (unused when feat == EXACT).
 * explicit_features != 0 evaluates <phi',phi'> as the r^2-term sum; otherwise as
 * <m,m>^2, which Section 3.1 states is the same number.  W_out (nrows x n, may be
 * NULL) receives the weights, zero above the diagonal. */
int psf_oracle_attn_def(const double *Q, const double *K, const double *V,
                        const double *MQ, const double *MK,
                        long n, long d, long dv, long mcols, long p, long b,
                        int feat, int local, int explicit_features,
                        const long *rows, long nrows, double *O_out, double *W_out)
{
    if (n <= 0 || b <= 0 || n % b != 0) return 1;
    if (!rows) nrows = n;
    double *acc = (double *)malloc(sizeof(double) * (size_t)dv);
    if (!acc) return 2;
    for (long t = 0; t < nrows; ++t) {
        long i = rows ? rows[t] : t;
        if (i < 0 || i >= n) { free(acc); return 1; }
        double den = 1.0;
        for (long c = 0; c < dv; ++c) acc[c] = 0.0;
        if (W_out) for (long j = 0; j < n; ++j) W_out[t * n + j] = 0.0;
        for (long j = 0; j <= i; ++j) {
            double w;
            int same_block = (i / b) == (j / b);
            if (feat == FEAT_EXACT || (local == LOCAL_EXACT && same_block)) {
                w = ipow(dot(Q + i * d, K + j * d, d), p);
            } else if (explicit_features) {
                w = 0.0;
                for (long a = 0; a < mcols; ++a)
                    for (long e = 0; e < mcols; ++e)
                        w += (MQ[i * mcols + a] * MQ[i * mcols + e]) *
                             (MK[j * mcols + a] * MK[j * mcols + e]);
            } else {
                double s = dot(MQ + i * mcols, MK + j * mcols, mcols);
                w = s * s;
            }
            den += w;
            for (long c = 0; c < dv; ++c) acc[c] += w * V[j * dv + c];
            if (W_out) W_out[t * n + j] = w;
        }
        for (long c = 0; c < dv; ++c) O_out[t * dv + c] = acc[c] / den;
    }
    free(acc);
    return 0;
}

/* ---- non-causal Polysketch attention (Section 2.2) -------------------------------------
 * Attn = D^-1 phi'(Q) phi'(K)^T V with D = diag(1 + phi'(Q) phi'(K)^T 1): every query sees all
 * nk keys, there is no mask and no block structure,
 *   o_i = sum_j w_ij v_j / (1 + sum_j w_ij),   w_ij = <phi'(q_i), phi'(k_j)> = <m(q_i), m(k_j)>^2
 * (feat == EXACT: w_ij = <q_i, k_j>^p, the polynomial attention the sketch approximates).
 * explicit_features != 0 evaluates the weight as the r^2-term sum over phi' = m (x) m.
 * Q, MQ have nq rows; K, V, MK have nk rows. */
int psf_oracle_attn_noncausal(const double *Q, const double *K, const double *V,
                              const double *MQ, const double *MK, long nq, long nk, long d, long dv,
                              long mcols, long p, int feat, int explicit_features, double *O_out)
{
    if (nq <= 0 || nk <= 0) return 1;
    double *acc = (double *)malloc(sizeof(double) * (size_t)dv);
    if (!acc) return 2;
    for (long i = 0; i < nq; ++i) {
        double den = 1.0;
        for (long c = 0; c < dv; ++c) acc[c] = 0.0;
        for (long j = 0; j < nk; ++j) {
            double w;
            if (feat == FEAT_EXACT) {
                w = ipow(dot(Q + i * d, K + j * d, d), p);
            } else if (explicit_features) {
                w = 0.0;
                for (long a = 0; a < mcols; ++a)
                    for (long e = 0; e < mcols; ++e)
                        w += (MQ[i * mcols + a] * MQ[i * mcols + e]) *
                             (MK[j * mcols + a] * MK[j * mcols + e]);
            } else {
                double u = dot(MQ + i * mcols, MK + j * mcols, mcols);
                w = u * u;
            }
            den += w;
            for (long c = 0; c < dv; ++c) acc[c] += w * V[j * dv + c];
        }
        for (long c = 0; c < dv; ++c) O_out[i * dv + c] = acc[c] / den;
    }
    free(acc);
    return 0;
}

/* ---- the paper's block algorithm, step by step -----------------------------------
 * A = PhiQ, B = PhiK (n x F explicit features), C = [V | 1] (n x (dv+1)).
 *   H_l = sum_{i in B_l} b_i c_i^T          Z_l = sum_{j<l} H_j   (sequential)
 *   P_l = lt(A_l B_l^T) C_l                 or lt((Q_l K_l^T)^p) C_l   (local exact)
 *   row i of lt(A B^T) C = row i' of P_l + a_i^T Z_l
 * then the last column is the denominator: o_i = row[0:dv] / (1 + row[dv]). */
int psf_oracle_attn_block(const double *Q, const double *K, const double *V,
                          const double *PhiQ, const double *PhiK,
                          long n, long d, long dv, long F, long p, long b,
                          int local_exact, double *O_out)
{
    if (n <= 0 || b <= 0 || n % b != 0) return 1;
    long t = n / b, kc = dv + 1;
    double *C = (double *)malloc(sizeof(double) * (size_t)n * (size_t)kc);
    double *Z = (double *)calloc((size_t)F * (size_t)kc, sizeof(double));
    double *H = (double *)malloc(sizeof(double) * (size_t)F * (size_t)kc);
    double *P = (double *)malloc(sizeof(double) * (size_t)b * (size_t)kc);
    double *S = (double *)malloc(sizeof(double) * (size_t)b * (size_t)b);
    if (!C || !Z || !H || !P || !S) { free(C); free(Z); free(H); free(P); free(S); return 2; }
    for (long i = 0; i < n; ++i) {
        for (long c = 0; c < dv; ++c) C[i * kc + c] = V[i * dv + c];
        C[i * kc + dv] = 1.0;
    }
    for (long l = 0; l < t; ++l) {
        long r0 = l * b;
        /* S = lt(A_l B_l^T), or lt((Q_l K_l^T)^p) when exact weights are used locally */
        for (long x = 0; x < b; ++x)
            for (long y = 0; y < b; ++y) {
                double s = 0.0;
                if (y <= x) {
                    if (local_exact) s = ipow(dot(Q + (r0 + x) * d, K + (r0 + y) * d, d), p);
                    else s = dot(PhiQ + (r0 + x) * F, PhiK + (r0 + y) * F, F);
                }
                S[x * b + y] = s;
            }
        /* P_l = S C_l */
        for (long x = 0; x < b; ++x)
            for (long c = 0; c < kc; ++c) {
                double s = 0.0;
                for (long y = 0; y < b; ++y) s += S[x * b + y] * C[(r0 + y) * kc + c];
                P[x * kc + c] = s;
            }
        /* rows of this block: P_l + A_l Z_l   (Z holds Z_l = sum_{j<l} H_j here) */
        for (long x = 0; x < b; ++x) {
            const double *a = PhiQ + (r0 + x) * F;
            double den = 1.0 + P[x * kc + dv];
            for (long f = 0; f < F; ++f) den += a[f] * Z[f * kc + dv];
            for (long c = 0; c < dv; ++c) {
                double num = P[x * kc + c];
                for (long f = 0; f < F; ++f) num += a[f] * Z[f * kc + c];
                O_out[(r0 + x) * dv + c] = num / den;
            }
        }
        /* H_l = B_l^T C_l, then Z_{l+1} = Z_l + H_l */
        for (long f = 0; f < F; ++f)
            for (long c = 0; c < kc; ++c) H[f * kc + c] = 0.0;
        for (long x = 0; x < b; ++x) {
            const double *bf = PhiK + (r0 + x) * F;
            for (long f = 0; f < F; ++f)
                for (long c = 0; c < kc; ++c) H[f * kc + c] += bf[f] * C[(r0 + x) * kc + c];
        }
        for (long f = 0; f < F; ++f)
            for (long c = 0; c < kc; ++c) Z[f * kc + c] += H[f * kc + c];
    }
    free(C); free(Z); free(H); free(P); free(S);
    return 0;
}

/* ---- gradient of Algorithm 1 -------------------------------------------------------
 * Given dOut = dL/d PolySketchWithNegativity(A, r, deg) (k x cols), adds dL/dA (k x m) into
 * dA.  Mirrors oracle_pswn: the node's output is sqrt(1/r) (M1 G1) * (M2 G2), so with
 * U = M1 G1, W = M2 G2:  dU = sqrt(1/r) dOut * W,  dW = sqrt(1/r) dOut * U,
 * dM1 = dU G1^T,  dM2 = dW G2^T, and the two subtrees are differentiated in turn with the
 * matrices they consumed in the forward recursion (left subtree first, then right, then
 * the node). */
static int oracle_pswn_bwd(const double *A, long k, long m, long r, long deg,
                           const double **g_first, const double **g_inner,
                           const double *dOut, double *dA)
{
    if (deg == 1) {
        for (long i = 0; i < k * m; ++i) dA[i] += dOut[i];
        return 0;
    }
    const double *gf0 = *g_first, *gi0 = *g_inner;            /* where the left subtree starts */
    double *M1 = oracle_pswn(A, k, m, r, deg / 2, g_first, g_inner);
    const double *gf1 = *g_first, *gi1 = *g_inner;            /* where the right subtree starts */
    double *M2 = oracle_pswn(A, k, m, r, deg / 2, g_first, g_inner);
    long rows = (deg / 2 == 1) ? m : r;
    const double *G1, *G2;
    if (deg / 2 == 1) { G1 = *g_first;  G2 = G1 + rows * r;  *g_first = G2 + rows * r; }
    else              { G1 = *g_inner;  G2 = G1 + rows * r;  *g_inner = G2 + rows * r; }
    double *dM1 = (double *)calloc((size_t)k * (size_t)rows, sizeof(double));
    double *dM2 = (double *)calloc((size_t)k * (size_t)rows, sizeof(double));
    if (!M1 || !M2 || !dM1 || !dM2) { free(M1); free(M2); free(dM1); free(dM2); return 2; }
    double scale = sqrt(1.0 / (double)r);
    for (long i = 0; i < k; ++i) {
        for (long c = 0; c < r; ++c) {
            double u = 0.0, w = 0.0;
            for (long e = 0; e < rows; ++e) {
                u += M1[i * rows + e] * G1[e * r + c];
                w += M2[i * rows + e] * G2[e * r + c];
            }
            double du = scale * dOut[i * r + c] * w, dw = scale * dOut[i * r + c] * u;
            for (long e = 0; e < rows; ++e) {
                dM1[i * rows + e] += du * G1[e * r + c];
                dM2[i * rows + e] += dw * G2[e * r + c];
            }
        }
    }
    const double *a = gf0, *b = gi0;
    int e1 = oracle_pswn_bwd(A, k, m, r, deg / 2, &a, &b, dM1, dA);
    a = gf1; b = gi1;
    int e2 = oracle_pswn_bwd(A, k, m, r, deg / 2, &a, &b, dM2, dA);
    free(M1); free(M2); free(dM1); free(dM2);
    return e1 ? e1 : e2;
}

/* dX (k x d, overwritten) = (d m(x) / d x)^T dM for every row, m = PolySketchWithNegativity
 * (x, r, p/2) as in psf_oracle_sketch. */
int psf_oracle_sketch_bwd(const double *X, long k, long d, long r, long p,
                          const double *G, const double *dM, double *dX)
{
    if (!is_pow2(p) || p < 2 || k < 0 || d <= 0 || r <= 0) return 1;
    const double *gf = G;
    const double *gi = G ? G + psf_oracle_num_g_first(p) * d * r : NULL;
    for (long i = 0; i < k * d; ++i) dX[i] = 0.0;
    return oracle_pswn_bwd(X, k, d, r, p / 2, &gf, &gi, dM, dX);
}

/* ---- gradient of Algorithm 2 --------------------------------------------------------
 * The learned sketch is trained, so both gradients are needed: with respect to the input rows
 * and with respect to the parameters of the networks.  Everything below is the chain rule
 * through oracle_learned_net / oracle_lpswn, row by row.
 *
 * d gelu(x) / dx for the tanh form: with c = sqrt(2/pi), t = tanh(c (x + 0.044715 x^3)):
 * 0.5 (1 + t) + 0.5 x (1 - t^2) c (1 + 3 * 0.044715 x^2). */
static double gelu_tanh_grad(double x)
{
    const double c = 0.7978845608028654;
    double t = tanh(c * (x + 0.044715 * x * x * x));
    return 0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * c * (1.0 + 3.0 * 0.044715 * x * x);
}

/* y = (x - mean) inv g + b with inv = 1 / sqrt(var + eps), biased variance.  Given dy: adds
 * dg += dy * xhat, db += dy, and writes dx = inv (dxh - mean(dxh) - xhat mean(dxh * xhat)) with
 * dxh = dy * g (the eps sits inside the square root, so the formula is exact for it too). */
static void layer_norm_bwd(const double *x, long m, const double *g, const double *dy,
                           double *dg, double *db, double *dx)
{
    double mean = 0.0, var = 0.0;
    for (long e = 0; e < m; ++e) mean += x[e];
    mean /= (double)m;
    for (long e = 0; e < m; ++e) var += (x[e] - mean) * (x[e] - mean);
    var /= (double)m;
    double inv = 1.0 / sqrt(var + 1e-6);
    double s1 = 0.0, s2 = 0.0;
    for (long e = 0; e < m; ++e) {
        double xh = (x[e] - mean) * inv, dxh = dy[e] * g[e];
        s1 += dxh;
        s2 += dxh * xh;
        dg[e] += dy[e] * xh;
        db[e] += dy[e];
    }
    s1 /= (double)m;
    s2 /= (double)m;
    for (long e = 0; e < m; ++e) {
        double xh = (x[e] - mean) * inv;
        dx[e] = inv * (dy[e] * g[e] - s1 - xh * s2);
    }
}

/* One network f (see oracle_learned_net): given dF = dL/df (k x r), adds dL/dA into dA (k x win)
 * and dL/dparams into dP, which has the layout of the network's own parameter block
 * [g1, b1, W1, g2, b2, W2, W3, W4].  The forward values of a row are recomputed first. */
static int oracle_learned_net_bwd(const double *A, long k, long win, long r, const double *P,
                                  const double *dF, double *dA, double *dP)
{
    long hid = 8 * r;
    const double *g1 = P, *b1 = g1 + win, *W1 = b1 + win;
    const double *g2 = W1 + win * hid, *b2 = g2 + hid, *W2 = b2 + hid;
    const double *W3 = W2 + hid * r, *W4 = W3 + r * hid;
    double *dg1 = dP, *db1 = dg1 + win, *dW1 = db1 + win;
    double *dg2 = dW1 + win * hid, *db2 = dg2 + hid, *dW2 = db2 + hid;
    double *dW3 = dW2 + hid * r, *dW4 = dW3 + r * hid;
    long big = win > hid ? win : hid;
    double *buf = (double *)malloc(sizeof(double) * (size_t)(2 * win + 8 * hid + 2 * r + 2 * big));
    if (!buf) return 2;
    double *u0 = buf, *du0 = u0 + win, *s1 = du0 + win, *h1 = s1 + hid, *v = h1 + hid, *s3 = v + hid,
           *h3 = s3 + hid, *dh = h3 + hid, *dv = dh + hid, *ds = dv + hid, *h2 = ds + hid, *dh2 = h2 + r,
           *da = dh2 + r;
    (void)big;
    for (long i = 0; i < k; ++i) {
        const double *a = A + i * win, *df = dF + i * r;
        /* forward, keeping what the reverse pass needs */
        layer_norm(a, win, g1, b1, u0);
        for (long c = 0; c < hid; ++c) {
            double t = 0.0;
            for (long e = 0; e < win; ++e) t += u0[e] * W1[e * hid + c];
            s1[c] = t;
            h1[c] = gelu_tanh(t);
        }
        layer_norm(h1, hid, g2, b2, v);
        for (long c = 0; c < r; ++c) {
            double t = 0.0;
            for (long e = 0; e < hid; ++e) t += v[e] * W2[e * r + c];
            h2[c] = t;
        }
        for (long c = 0; c < hid; ++c) {
            double t = 0.0;
            for (long e = 0; e < r; ++e) t += h2[e] * W3[e * hid + c];
            s3[c] = t;
            h3[c] = gelu_tanh(t);
        }
        /* f = h3 W4 */
        for (long e = 0; e < hid; ++e) {
            double t = 0.0;
            for (long c = 0; c < r; ++c) {
                t += df[c] * W4[e * r + c];
                dW4[e * r + c] += h3[e] * df[c];
            }
            ds[e] = t * gelu_tanh_grad(s3[e]);            /* dL/ds3 */
        }
        /* s3 = h2 W3 */
        for (long e = 0; e < r; ++e) {
            double t = 0.0;
            for (long c = 0; c < hid; ++c) {
                t += ds[c] * W3[e * hid + c];
                dW3[e * hid + c] += h2[e] * ds[c];
            }
            dh2[e] = t;
        }
        /* h2 = v W2 */
        for (long e = 0; e < hid; ++e) {
            double t = 0.0;
            for (long c = 0; c < r; ++c) {
                t += dh2[c] * W2[e * r + c];
                dW2[e * r + c] += v[e] * dh2[c];
            }
            dv[e] = t;
        }
        /* v = LayerNorm(h1) */
        layer_norm_bwd(h1, hid, g2, dv, dg2, db2, dh);
        /* h1 = gelu(s1), s1 = u0 W1 */
        for (long c = 0; c < hid; ++c) ds[c] = dh[c] * gelu_tanh_grad(s1[c]);
        for (long e = 0; e < win; ++e) {
            double t = 0.0;
            for (long c = 0; c < hid; ++c) {
                t += ds[c] * W1[e * hid + c];
                dW1[e * hid + c] += u0[e] * ds[c];
            }
            du0[e] = t;
        }
        /* u0 = LayerNorm(a) */
        layer_norm_bwd(a, win, g1, du0, dg1, db1, da);
        for (long e = 0; e < win; ++e) dA[i * win + e] += da[e];
    }
    free(buf);
    return 0;
}

/* Reverse of oracle_lpswn.  The node's output is sqrt(r) tanh(F1 * F2 / sqrt(r)), so with
 * t = tanh(F1 F2 / sqrt(r)):  dF1 = dOut (1 - t^2) F2,  dF2 = dOut (1 - t^2) F1 (the two
 * sqrt(r) cancel); each network is then differentiated with respect to its input M1 / M2 and
 * its parameters, and the subtrees in turn.  *params walks the parameter blob exactly as in
 * the forward recursion; dP0 is the gradient blob (same layout), P0 the start of the blob. */
static int oracle_lpswn_bwd(const double *A, long k, long m, long r, long deg, const double **params,
                            const double *P0, double *dP0, const double *dOut, double *dA)
{
    if (deg == 1) {
        for (long i = 0; i < k * m; ++i) dA[i] += dOut[i];
        return 0;
    }
    const double *p_left = *params;
    double *M1 = oracle_lpswn(A, k, m, r, deg / 2, params);
    const double *p_right = *params;
    double *M2 = oracle_lpswn(A, k, m, r, deg / 2, params);
    long win = (deg / 2 == 1) ? m : r;
    const double *p_f1 = *params;
    double *F1 = M1 ? oracle_learned_net(M1, k, win, r, params) : NULL;
    const double *p_f2 = *params;
    double *F2 = M2 ? oracle_learned_net(M2, k, win, r, params) : NULL;
    double *dF1 = (double *)malloc(sizeof(double) * (size_t)k * (size_t)r);
    double *dF2 = (double *)malloc(sizeof(double) * (size_t)k * (size_t)r);
    double *dM1 = (double *)calloc((size_t)k * (size_t)win, sizeof(double));
    double *dM2 = (double *)calloc((size_t)k * (size_t)win, sizeof(double));
    int err = (!M1 || !M2 || !F1 || !F2 || !dF1 || !dF2 || !dM1 || !dM2) ? 2 : 0;
    if (!err) {
        double sr = sqrt((double)r);
        for (long i = 0; i < k * r; ++i) {
            double t = tanh(F1[i] * F2[i] / sr);
            double dz = dOut[i] * (1.0 - t * t);
            dF1[i] = dz * F2[i];
            dF2[i] = dz * F1[i];
        }
        err = oracle_learned_net_bwd(M1, k, win, r, p_f1, dF1, dM1, dP0 + (p_f1 - P0));
        if (!err) err = oracle_learned_net_bwd(M2, k, win, r, p_f2, dF2, dM2, dP0 + (p_f2 - P0));
        const double *pp = p_left;
        if (!err) err = oracle_lpswn_bwd(A, k, m, r, deg / 2, &pp, P0, dP0, dM1, dA);
        pp = p_right;
        if (!err) err = oracle_lpswn_bwd(A, k, m, r, deg / 2, &pp, P0, dP0, dM2, dA);
    }
    free(M1); free(M2); free(F1); free(F2); free(dF1); free(dF2); free(dM1); free(dM2);
    return err;
}

/* dX (k x d, overwritten) = (d m / d x)^T dM and, added into dParams (psf_oracle_learned_len
 * entries, NOT cleared here so that several calls can accumulate), (d m / d params)^T dM, for
 * m = LearnablePolysketchWithNegativity(x, r, p/2) as in psf_oracle_sketch_learned. */
int psf_oracle_sketch_learned_bwd(const double *X, long k, long d, long r, long p,
                                  const double *params, const double *dM, double *dX, double *dParams)
{
    if (!is_pow2(p) || p < 2 || k < 0 || d <= 0 || r <= 0) return 1;
    for (long i = 0; i < k * d; ++i) dX[i] = 0.0;
    const double *pp = params;
    return oracle_lpswn_bwd(X, k, d, r, p / 2, &pp, params, dParams, dM, dX);
}

/* ---- gradient of the definition -----------------------------------------------------
 * L is any scalar with dL/dO = dO (n x dv).  With N_i = sum_{j<=i} w_ij v_j,
 * D_i = 1 + sum_{j<=i} w_ij, o_i = N_i / D_i:
 *   g_i = dO_i / D_i,  c_i = -<dO_i, o_i> / D_i,  dL/dw_ij = <g_i, v_j> + c_i,
 *   dV_j = sum_{i>=j} w_ij g_i,
 *   w = <q,k>^p   (exact pair):    ds = p <q,k>^{p-1} dw,  dq_i += ds k_j,  dk_j += ds q_i
 *   w = <m(q),m(k)>^2 (sketched):  du = 2 <m(q),m(k)> dw,  dm(q_i) += du m(k_j), and v.v.,
 * then dQ += J_m(Q)^T dm(Q), dK += J_m(K)^T dm(K) through oracle_pswn_bwd.  The sketch
 * matrices G are constants.  One unit; dQ, dK (n x d) and dV (n x dv) are overwritten. */
static int oracle_attn_bwd_rows(const double *Q, const double *K, const double *V, const double *G,
                                const double *dO, long n, long d, long dv, long r, long p, long b,
                                int feat, int local, const long *rows, long nrows,
                                double *dQ, double *dK, double *dV, int learned, double *dP)
{
    if (n <= 0 || b <= 0 || n % b != 0 || !is_pow2(p) || p < 2) return 1;
    long mcols = (p == 2) ? d : r;
    int sketch = feat == FEAT_SKETCH;
    double *mq = NULL, *mk = NULL, *dmq = NULL, *dmk = NULL;
    double *w = (double *)malloc(sizeof(double) * (size_t)n);
    double *num = (double *)malloc(sizeof(double) * (size_t)dv);
    double *tmp = (double *)malloc(sizeof(double) * (size_t)n * (size_t)d);
    int err = (!w || !num || !tmp) ? 2 : 0;
    if (sketch && !err) {
        mq = (double *)malloc(sizeof(double) * (size_t)n * (size_t)mcols);
        mk = (double *)malloc(sizeof(double) * (size_t)n * (size_t)mcols);
        dmq = (double *)calloc((size_t)n * (size_t)mcols, sizeof(double));
        dmk = (double *)calloc((size_t)n * (size_t)mcols, sizeof(double));
        if (!mq || !mk || !dmq || !dmk) err = 2;
        if (!err) err = learned ? psf_oracle_sketch_learned(Q, n, d, r, p, G, mq) : psf_oracle_sketch(Q, n, d, r, p, G, mq);
        if (!err) err = learned ? psf_oracle_sketch_learned(K, n, d, r, p, G, mk) : psf_oracle_sketch(K, n, d, r, p, G, mk);
    }
    if (!err) {
        for (long i = 0; i < n * d; ++i) dQ[i] = dK[i] = 0.0;
        for (long i = 0; i < n * dv; ++i) dV[i] = 0.0;
        for (long ri = 0; ri < (rows ? nrows : n); ++ri) {
            long i = rows ? rows[ri] : ri;
            if (i < 0 || i >= n) { err = 1; break; }
            double den = 1.0;
            for (long c = 0; c < dv; ++c) num[c] = 0.0;
            for (long j = 0; j <= i; ++j) {
                int exact = feat == FEAT_EXACT || (local == LOCAL_EXACT && (i / b) == (j / b));
                if (exact) w[j] = ipow(dot(Q + i * d, K + j * d, d), p);
                else { double u = dot(mq + i * mcols, mk + j * mcols, mcols); w[j] = u * u; }
                den += w[j];
                for (long c = 0; c < dv; ++c) num[c] += w[j] * V[j * dv + c];
            }
            double ci = 0.0;                       /* c_i = -<dO_i, o_i> / D_i */
            for (long c = 0; c < dv; ++c) ci -= dO[i * dv + c] * (num[c] / den);
            ci /= den;
            for (long j = 0; j <= i; ++j) {
                double dw = ci;
                for (long c = 0; c < dv; ++c) {
                    double g = dO[i * dv + c] / den;
                    dw += g * V[j * dv + c];
                    dV[j * dv + c] += w[j] * g;
                }
                int exact = feat == FEAT_EXACT || (local == LOCAL_EXACT && (i / b) == (j / b));
                if (exact) {
                    double s = dot(Q + i * d, K + j * d, d);
                    double ds = (double)p * ipow(s, p - 1) * dw;
                    for (long e = 0; e < d; ++e) {
                        dQ[i * d + e] += ds * K[j * d + e];
                        dK[j * d + e] += ds * Q[i * d + e];
                    }
                } else {
                    double u = dot(mq + i * mcols, mk + j * mcols, mcols);
                    double du = 2.0 * u * dw;
                    for (long e = 0; e < mcols; ++e) {
                        dmq[i * mcols + e] += du * mk[j * mcols + e];
                        dmk[j * mcols + e] += du * mq[i * mcols + e];
                    }
                }
            }
        }
        if (sketch && !err) {
            /* learned sketches: the same networks serve the query and the key rows, so their
             * parameter gradients add up */
            err = learned ? psf_oracle_sketch_learned_bwd(Q, n, d, r, p, G, dmq, tmp, dP)
                          : psf_oracle_sketch_bwd(Q, n, d, r, p, G, dmq, tmp);
            for (long i = 0; i < n * d && !err; ++i) dQ[i] += tmp[i];
            if (!err) err = learned ? psf_oracle_sketch_learned_bwd(K, n, d, r, p, G, dmk, tmp, dP)
                                    : psf_oracle_sketch_bwd(K, n, d, r, p, G, dmk, tmp);
            for (long i = 0; i < n * d && !err; ++i) dK[i] += tmp[i];
        }
    }
    free(w); free(num); free(tmp); free(mq); free(mk); free(dmq); free(dmk);
    return err;
}

int psf_oracle_attn_bwd(const double *Q, const double *K, const double *V, const double *G,
                        const double *dO, long n, long d, long dv, long r, long p, long b,
                        int feat, int local, double *dQ, double *dK, double *dV)
{
    return oracle_attn_bwd_rows(Q, K, V, G, dO, n, d, dv, r, p, b, feat, local, NULL, 0, dQ, dK, dV, 0, NULL);
}

/* The same gradient with learned sketches (Algorithm 2) in place of Algorithm 1: params holds
 * the networks' parameters (psf_oracle_learned_len entries); dParams (same length, overwritten)
 * receives dL/dparams, the sum of the query-side and key-side contributions.  Sketch features
 * only; p in {2, 4, 8, 16} (p = 2: no networks, dParams untouched). */
int psf_oracle_attn_bwd_learned(const double *Q, const double *K, const double *V, const double *params,
                                const double *dO, long n, long d, long dv, long r, long p, long b,
                                int local, double *dQ, double *dK, double *dV, double *dParams)
{
    long len = psf_oracle_learned_len(d, r, p);
    for (long i = 0; i < len; ++i) dParams[i] = 0.0;
    return oracle_attn_bwd_rows(Q, K, V, params, dO, n, d, dv, r, p, b, FEAT_SKETCH, local, NULL, 0,
                                dQ, dK, dV, 1, dParams);
}

/* The same sums restricted to the listed query rows i (each listed once): row i of dQ is complete
 * for every listed i; row j of dK and dV is complete when every i >= j is listed (list a whole
 * tail of the sequence for that); all other rows hold partial sums and are to be ignored.  For
 * sequences too long for the full O(n^2) loop. */
int psf_oracle_attn_bwd_rows(const double *Q, const double *K, const double *V, const double *G,
                             const double *dO, long n, long d, long dv, long r, long p, long b,
                             int feat, int local, const long *rows, long nrows,
                             double *dQ, double *dK, double *dV)
{
    if (!rows || nrows < 0) return 1;
    return oracle_attn_bwd_rows(Q, K, V, G, dO, n, d, dv, r, p, b, feat, local, rows, nrows, dQ, dK, dV, 0, NULL);
}

/* ---- drivers over (batch, head) units ---------------------------------------------
 * Q, K, V are [units, n, d|dv]; G is [g_sets, g_len] with unit u using set
 * (u % heads) when g_sets == heads, set 0 when g_sets == 1.  Rows are shared by all
 * units.  OpenMP splits the unit loop only.  Returns the number of threads used,
 * or a negative error code. */
#ifdef _OPENMP
#include <omp.h>
#endif

int psf_oracle_attn_def_batch(const double *Q, const double *K, const double *V,
                              const double *G, long g_sets, long heads,
                              long units, long n, long d, long dv, long p, long r, long b,
                              int feat, int local,
                              const long *rows, long nrows, double *O_out, int max_threads)
{
    if (!is_pow2(p) || p < 2) return -1;
    long mcols = (p == 2) ? d : r;
    long g_len = psf_oracle_num_g_first(p) * d * r + psf_oracle_num_g_inner(p) * r * r;
    long orows = rows ? nrows : n;
    int err = 0, used = 1;
#ifdef _OPENMP
    if (max_threads > 0) omp_set_num_threads(max_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (long u = 0; u < units; ++u) {
        const double *q = Q + u * n * d, *k = K + u * n * d, *v = V + u * n * dv;
        double *mq = NULL, *mk = NULL;
        int e = 0;
        if (feat == FEAT_SKETCH) {
            const double *g = G + ((g_sets == 1) ? 0 : (u % heads)) * g_len;
            mq = (double *)malloc(sizeof(double) * (size_t)n * (size_t)mcols);
            mk = (double *)malloc(sizeof(double) * (size_t)n * (size_t)mcols);
            if (!mq || !mk) e = 2;
            if (!e) e = psf_oracle_sketch(q, n, d, r, p, g, mq);
            if (!e) e = psf_oracle_sketch(k, n, d, r, p, g, mk);
        }
        if (!e)
            e = psf_oracle_attn_def(q, k, v, mq, mk, n, d, dv, mcols, p, b, feat, local, 0,
                                    rows, nrows, O_out + u * orows * dv, NULL);
        free(mq);
        free(mk);
        if (e) {
#ifdef _OPENMP
#pragma omp critical
#endif
            err = e;
        }
    }
    return err ? -err : used;
}

/* Same driver for the gradient: dO is [units, n, dv]; dQ, dK [units, n, d], dV [units, n, dv]. */
int psf_oracle_attn_bwd_batch(const double *Q, const double *K, const double *V,
                              const double *G, long g_sets, long heads, const double *dO,
                              long units, long n, long d, long dv, long p, long r, long b,
                              int feat, int local, double *dQ, double *dK, double *dV,
                              int max_threads)
{
    if (!is_pow2(p) || p < 2) return -1;
    long g_len = psf_oracle_num_g_first(p) * d * r + psf_oracle_num_g_inner(p) * r * r;
    int err = 0, used = 1;
#ifdef _OPENMP
    if (max_threads > 0) omp_set_num_threads(max_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (long u = 0; u < units; ++u) {
        const double *g = G ? G + ((g_sets == 1) ? 0 : (u % heads)) * g_len : NULL;
        int e = psf_oracle_attn_bwd(Q + u * n * d, K + u * n * d, V + u * n * dv, g,
                                    dO + u * n * dv, n, d, dv, r, p, b, feat, local,
                                    dQ + u * n * d, dK + u * n * d, dV + u * n * dv);
        if (e) {
#ifdef _OPENMP
#pragma omp critical
#endif
            err = e;
        }
    }
    return err ? -err : used;
}
