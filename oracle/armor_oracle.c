/*
 * CPU oracle for the ARMOR per-layer factorization (W-bar ~= A * (W' (.) M) * B).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64-accumulating
 * restatement of the paper's algorithm, used only by tests, by the smoke check and by the
 * CPU-baseline leg of the benchmark.  It shares no code with the HIP library and must never be
 * called from the product path.
 *
 * What it follows, step by step, in the paper's notation:
 *   - normalisation of W ............................ Sec. 3.2 (definition of W-bar, r(1), r(2))
 *   - proxy loss .................................... Sec. 3.2, Eq. 2 (weights are diag(X X^T) only)
 *   - initialisation ................................ Sec. 3.3, Eq. 3
 *   - continuous update (sequential GD, 1/beta) ..... Sec. 3.3.1, Alg. 2, Lemma 1, App. D (Eq. 9-11)
 *   - continuous update (joint Adam, as run in practice) Sec. 3.3.1, App. F
 *   - sparse-core update ............................ Sec. 3.3.2, App. B.1 (Eq. 5-8), Alg. 3
 *   - outer loop .................................... Alg. 1
 *   - N:M generalisation, unstructured mode ......... Sec. 4.5
 *   - denormalisation ............................... Sec. 3.2, last paragraph
 *   - the factorized layer applied to activations ... Sec. 3.1 (y = A (S (B x))), Sec. 4.4
 *
 * Conventions: all matrices row-major; W[i*d_in + j] couples output i with input j; the sparse
 * axis is d_in (groups of M consecutive columns in a row).  A is stored [d_out/b][b][b], B is
 * stored [d_in/b][b][b] (Sec. 3.1).  The optimiser state (A, B, core C = W' (.) M) is kept in
 * fp32 between sub-steps; every sum is accumulated in fp64.  Quantities that decide an integer
 * (importance scores, selection keys, per-pattern gains) are rounded to fp32 before comparing.
 *
 * Readings of points the paper leaves open (each also listed in the design notes):
 *   - each of the three gradients of Alg. 2 is evaluated at the already-updated parameters
 *     (Lemma 1), and beta is recomputed each time;
 *   - the B-gradient and beta_B use S'^T S' (the derivation in App. D.2; the printed S'^T S is a typo);
 *   - the selection score is the L1 norm over the M entries of a group of the UNMASKED core
 *     gradient -2 A^T (R D) B^T (Sec. 3.3.2);
 *   - "select with probability p" is an exponential race over a counter-based hash:
 *     key = -ln(u)/g, smallest key wins, ties to the lower group index;
 *   - the pseudo-inverse of Eq. 7/8 is the Moore-Penrose inverse, eigenvalues below
 *     1e-12 * lambda_max dropped;
 *   - ties in top-N go to the lower index; zero norms in the normalisation are replaced by 1.
 *
 * Parity status: every function here is pinned by a CPU test against something other than
 * itself (closed forms, numpy dense algebra, finite differences, brute-force least squares,
 * invariants from Thm. 1 / Lemma 1 / Lemma 2).  The absolute values of A, S, B after n
 * iterations are "parity unpinned" by the paper (it prints no worked example).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int64_t d_out, d_in, b, nbi, nbj;
} dims_t;

static dims_t mk_dims(int64_t d_out, int64_t d_in, int64_t b) {
    dims_t d = {d_out, d_in, b, d_out / b, d_in / b};
    return d;
}

static double *dalloc(int64_t n) { return (double *)calloc((size_t)(n > 0 ? n : 1), sizeof(double)); }

static double *to_double(const float *x, int64_t n) {
    double *y = dalloc(n);
    for (int64_t k = 0; k < n; ++k) y[k] = (double)x[k];
    return y;
}

/* ------------------------------------------------------------------------------------------
 * Counter-based uniform generator shared BY SPECIFICATION (not by code) with the HIP library:
 * 64-bit counter -> splitmix64 finaliser -> top 24 bits -> u in (0, 1].
 * counter = ((t * n_blocks + blk) * groups_per_block + kappa) + 1,  t = 1..n_iters.
 * ------------------------------------------------------------------------------------------ */
static uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

float oracle_uniform(uint64_t seed, int64_t t, int64_t n_blocks, int64_t blk,
                     int64_t groups_per_block, int64_t kappa) {
    uint64_t ctr = (uint64_t)((t * n_blocks + blk) * groups_per_block + kappa) + 1ULL;
    uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ULL * ctr);
    return (float)((z >> 40) + 1ULL) * (1.0f / 16777216.0f);
}

/* ------------------------------------------------------------------------------------------
 * Gram matrix of the calibration data (Sec. 2 / Eq. 2): X is [n x d] row-major (one token per
 * row, i.e. the paper's X^T); H = sum_t x_t x_t^T; the loss only uses D = diag(H).
 * ------------------------------------------------------------------------------------------ */
void oracle_gram(const float *X, int64_t n, int64_t d, double *H) {
#pragma omp parallel for schedule(static)
    for (int64_t a = 0; a < d; ++a) {
        for (int64_t c = 0; c < d; ++c) H[a * d + c] = 0.0;
        for (int64_t t = 0; t < n; ++t) {
            double xa = (double)X[t * d + a];
            for (int64_t c = 0; c < d; ++c) H[a * d + c] += xa * (double)X[t * d + c];
        }
    }
}

static float bf16_to_float(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Selected entries H[rows[e]][cols[e]] one by one; X given as fp32 or as raw bf16 bit patterns. */
void oracle_gram_entries(const float *X, int64_t n, int64_t d, const int64_t *rows,
                         const int64_t *cols, int64_t cnt, double *out) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < cnt; ++e) {
        double s = 0.0;
        for (int64_t t = 0; t < n; ++t) s += (double)X[t * d + rows[e]] * (double)X[t * d + cols[e]];
        out[e] = s;
    }
}

void oracle_gram_entries_bf16(const uint16_t *X, int64_t n, int64_t d, const int64_t *rows,
                              const int64_t *cols, int64_t cnt, double *out) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < cnt; ++e) {
        double s = 0.0;
        for (int64_t t = 0; t < n; ++t)
            s += (double)bf16_to_float(X[t * d + rows[e]]) * (double)bf16_to_float(X[t * d + cols[e]]);
        out[e] = s;
    }
}

/* ------------------------------------------------------------------------------------------
 * Normalisation (Sec. 3.2): r1_j = ||W[:,j]||, W1 = W / r1 (columns), r2_i = ||W1[i,:]||,
 * W-bar = W1 / r2 (rows).
 * ------------------------------------------------------------------------------------------ */
void oracle_normalize(const float *W, int64_t d_out, int64_t d_in, float *Wbar, float *r1, float *r2) {
    for (int64_t j = 0; j < d_in; ++j) {
        double s = 0.0;
        for (int64_t i = 0; i < d_out; ++i) s += (double)W[i * d_in + j] * (double)W[i * d_in + j];
        double r = sqrt(s);
        r1[j] = (float)(r > 0.0 ? r : 1.0);
    }
    for (int64_t i = 0; i < d_out; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < d_in; ++j) {
            double w1 = (double)W[i * d_in + j] / (double)r1[j];
            s += w1 * w1;
        }
        double r = sqrt(s);
        r2[i] = (float)(r > 0.0 ? r : 1.0);
    }
    for (int64_t i = 0; i < d_out; ++i)
        for (int64_t j = 0; j < d_in; ++j)
            Wbar[i * d_in + j] = (float)(((double)W[i * d_in + j] / (double)r1[j]) / (double)r2[i]);
}

/* ------------------------------------------------------------------------------------------
 * Initialisation (Eq. 3): A = B = I, W' = W-bar, M = top-N of every group of M consecutive
 * columns by the importance I_ij = W-bar_ij^2 * D_j.  The score is formed in fp32 as (w*w)*d.
 * mask holds one byte (0/1) per matrix entry; C = W-bar (.) M.
 * ------------------------------------------------------------------------------------------ */
static float importance(float w, float d) {
    volatile float ww = w * w; /* volatile: keep the two roundings, no contraction */
    return ww * d;
}

void oracle_init_nm(const float *Wbar, const float *D, int64_t d_out, int64_t d_in, int N, int M,
                    float *C, uint8_t *mask) {
    for (int64_t i = 0; i < d_out; ++i)
        for (int64_t g = 0; g < d_in / M; ++g) {
            float s[64];
            for (int p = 0; p < M; ++p) s[p] = importance(Wbar[i * d_in + g * M + p], D[g * M + p]);
            for (int p = 0; p < M; ++p) {
                int rank = 0; /* entries that beat p: larger score, or equal score and lower index */
                for (int q = 0; q < M; ++q)
                    if (s[q] > s[p] || (s[q] == s[p] && q < p)) ++rank;
                int keep = rank < N;
                mask[i * d_in + g * M + p] = (uint8_t)keep;
                C[i * d_in + g * M + p] = keep ? Wbar[i * d_in + g * M + p] : 0.0f;
            }
        }
}

void oracle_init_identity(float *A, int64_t nblk, int64_t b) {
    memset(A, 0, sizeof(float) * (size_t)(nblk * b * b));
    for (int64_t i = 0; i < nblk; ++i)
        for (int64_t p = 0; p < b; ++p) A[i * b * b + p * b + p] = 1.0f;
}

/* Unstructured variant (Sec. 4.5; the count-budget optimum of Eq. 2 for the naive core):
 * keep the `keep` largest importances over the whole matrix, ties to the lower linear index. */
typedef struct { float s; int64_t idx; } scored_t;
static int cmp_scored(const void *a, const void *b) {
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->idx < y->idx) ? -1 : (x->idx > y->idx);
}
void oracle_init_unstructured(const float *Wbar, const float *D, int64_t d_out, int64_t d_in,
                              int64_t keep, float *C, uint8_t *mask) {
    int64_t P = d_out * d_in;
    scored_t *v = (scored_t *)malloc(sizeof(scored_t) * (size_t)(P > 0 ? P : 1));
    for (int64_t e = 0; e < P; ++e) { v[e].s = importance(Wbar[e], D[e % d_in]); v[e].idx = e; }
    qsort(v, (size_t)P, sizeof(scored_t), cmp_scored);
    for (int64_t e = 0; e < P; ++e) { mask[e] = 0; C[e] = 0.0f; }
    for (int64_t e = 0; e < keep && e < P; ++e) { mask[v[e].idx] = 1; C[v[e].idx] = Wbar[v[e].idx]; }
    free(v);
}

/* ------------------------------------------------------------------------------------------
 * Block-diagonal products (Sec. 3.1 notation).  X, Y are d_out x d_in in fp64.
 *   right_mul: Y^(i,j) = X^(i,j) * op(B^j)       left_mul: Y^(i,j) = op(A^i) * X^(i,j)
 * ------------------------------------------------------------------------------------------ */
static void right_mul(const double *X, const double *Bd, int trans, dims_t d, double *Y) {
    int64_t b = d.b;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < d.d_out; ++r)
        for (int64_t j = 0; j < d.nbj; ++j) {
            const double *Bj = Bd + j * b * b;
            double *y = Y + r * d.d_in + j * b;
            const double *x = X + r * d.d_in + j * b;
            for (int64_t q = 0; q < b; ++q) y[q] = 0.0;
            for (int64_t p = 0; p < b; ++p) {
                double xv = x[p];
                if (!trans) for (int64_t q = 0; q < b; ++q) y[q] += xv * Bj[p * b + q];
                else        for (int64_t q = 0; q < b; ++q) y[q] += xv * Bj[q * b + p];
            }
        }
}

static void left_mul(const double *Ad, int trans, const double *X, dims_t d, double *Y) {
    int64_t b = d.b;
#pragma omp parallel for schedule(static)
    for (int64_t row = 0; row < d.d_out; ++row) {
        int64_t i = row / b, p = row % b;
        const double *Ai = Ad + i * b * b;
        double *y = Y + row * d.d_in;
        for (int64_t c = 0; c < d.d_in; ++c) y[c] = 0.0;
        for (int64_t k = 0; k < b; ++k) {
            double a = trans ? Ai[k * b + p] : Ai[p * b + k];
            const double *x = X + (i * b + k) * d.d_in;
            for (int64_t c = 0; c < d.d_in; ++c) y[c] += a * x[c];
        }
    }
}

/* residual R = W-bar - A * C * B  (Eq. 1), computed as A * (C * B) */
static void residual(const double *Wb, const double *Ad, const double *Cd, const double *Bd,
                     dims_t d, double *R) {
    int64_t P = d.d_out * d.d_in;
    double *S = dalloc(P);
    right_mul(Cd, Bd, 0, d, S);
    left_mul(Ad, 0, S, d, R);
    for (int64_t e = 0; e < P; ++e) R[e] = Wb[e] - R[e];
    free(S);
}

static double weighted_sq(const double *R, const double *Dd, dims_t d) {
    double L = 0.0;
    for (int64_t i = 0; i < d.d_out; ++i)
        for (int64_t j = 0; j < d.d_in; ++j) L += R[i * d.d_in + j] * R[i * d.d_in + j] * Dd[j];
    return L;
}

/* Proxy loss (Eq. 2): L = sum_ij (W-bar_ij - (A C B)_ij)^2 D_j. */
double oracle_proxy_loss(const float *Wbar, const float *A, const float *C, const float *B,
                         const float *D, int64_t d_out, int64_t d_in, int64_t b) {
    dims_t d = mk_dims(d_out, d_in, b);
    int64_t P = d_out * d_in;
    double *Wb = to_double(Wbar, P), *Cd = to_double(C, P), *Ad = to_double(A, d.nbi * b * b),
           *Bd = to_double(B, d.nbj * b * b), *Dd = to_double(D, d_in), *R = dalloc(P);
    residual(Wb, Ad, Cd, Bd, d, R);
    double L = weighted_sq(R, Dd, d);
    free(Wb); free(Cd); free(Ad); free(Bd); free(Dd); free(R);
    return L;
}

/* Dense reconstruction A*C*B for tests of the denormalisation identity. */
void oracle_reconstruct(const float *A, const float *C, const float *B, int64_t d_out, int64_t d_in,
                        int64_t b, double *What) {
    dims_t d = mk_dims(d_out, d_in, b);
    int64_t P = d_out * d_in;
    double *Cd = to_double(C, P), *Ad = to_double(A, d.nbi * b * b), *Bd = to_double(B, d.nbj * b * b),
           *S = dalloc(P);
    right_mul(Cd, Bd, 0, d, S);
    left_mul(Ad, 0, S, d, What);
    free(Cd); free(Ad); free(Bd); free(S);
}

/* ------------------------------------------------------------------------------------------
 * Gradients and smoothness constants (App. D).
 * ------------------------------------------------------------------------------------------ */
/* grad_A^(i) = sum_j [ 2 A^i S^ij D^j S^ij^T - 2 W-bar^ij D^j S^ij^T ] = -2 sum_j (R D)^ij S^ij^T,
 * S = C B (App. D.1).  beta_A = 2 sum_ij || S^ij D^j S^ij^T ||_F (Eq. 9). */
static void grad_beta_A(const double *Wb, const double *Ad, const double *Cd, const double *Bd,
                        const double *Dd, dims_t d, double *gA, double *beta) {
    int64_t P = d.d_out * d.d_in, b = d.b;
    double *S = dalloc(P), *R = dalloc(P);
    right_mul(Cd, Bd, 0, d, S);
    left_mul(Ad, 0, S, d, R);
    for (int64_t e = 0; e < P; ++e) R[e] = Wb[e] - R[e];
    if (gA) {
#pragma omp parallel for schedule(static)
        for (int64_t row = 0; row < d.d_out; ++row) {
            int64_t i = row / b, p = row % b;
            for (int64_t q = 0; q < b; ++q) {
                double s = 0.0;
                const double *r = R + row * d.d_in, *sq = S + (i * b + q) * d.d_in;
                for (int64_t c = 0; c < d.d_in; ++c) s += r[c] * Dd[c] * sq[c];
                gA[i * b * b + p * b + q] = -2.0 * s;
            }
        }
    }
    if (beta) {
        double tot = 0.0, *term = dalloc(d.nbi * d.nbj); /* summed in block order below: reruns agree bit for bit */
#pragma omp parallel for schedule(static)
        for (int64_t blk = 0; blk < d.nbi * d.nbj; ++blk) {
            int64_t i = blk / d.nbj, j = blk % d.nbj;
            double f2 = 0.0;
            for (int64_t p = 0; p < b; ++p)
                for (int64_t q = 0; q < b; ++q) {
                    double s = 0.0;
                    const double *sp = S + (i * b + p) * d.d_in + j * b, *sq = S + (i * b + q) * d.d_in + j * b;
                    for (int64_t c = 0; c < b; ++c) s += sp[c] * Dd[j * b + c] * sq[c];
                    f2 += s * s;
                }
            term[blk] = sqrt(f2);
        }
        for (int64_t blk = 0; blk < d.nbi * d.nbj; ++blk) tot += term[blk];
        free(term);
        *beta = 2.0 * tot;
    }
    free(S); free(R);
}

/* grad_B^(j) = sum_i [ 2 S'^ij^T S'^ij B^j D^j - 2 S'^ij^T W-bar^ij D^j ] = -2 sum_i S'^ij^T (R D)^ij,
 * S' = A C (App. D.2).  beta_B = 2 sum_ij || S'^ij^T S'^ij ||_F ||D^j||_F (Eq. 10). */
static void grad_beta_B(const double *Wb, const double *Ad, const double *Cd, const double *Bd,
                        const double *Dd, dims_t d, double *gB, double *beta) {
    int64_t P = d.d_out * d.d_in, b = d.b;
    double *Sp = dalloc(P), *R = dalloc(P);
    left_mul(Ad, 0, Cd, d, Sp);
    right_mul(Sp, Bd, 0, d, R);
    for (int64_t e = 0; e < P; ++e) R[e] = Wb[e] - R[e];
    if (gB) {
#pragma omp parallel for schedule(static)
        for (int64_t col = 0; col < d.d_in; ++col) { /* col = j*b + p indexes the row p of B^j */
            int64_t j = col / b, p = col % b;
            for (int64_t q = 0; q < b; ++q) {
                double s = 0.0;
                for (int64_t row = 0; row < d.d_out; ++row)
                    s += Sp[row * d.d_in + col] * R[row * d.d_in + j * b + q];
                gB[j * b * b + p * b + q] = -2.0 * s * Dd[j * b + q];
            }
        }
    }
    if (beta) {
        double tot = 0.0, *term = dalloc(d.nbi * d.nbj);
#pragma omp parallel for schedule(static)
        for (int64_t blk = 0; blk < d.nbi * d.nbj; ++blk) {
            int64_t i = blk / d.nbj, j = blk % d.nbj;
            double f2 = 0.0, dn = 0.0;
            for (int64_t p = 0; p < b; ++p)
                for (int64_t q = 0; q < b; ++q) {
                    double s = 0.0;
                    for (int64_t r = 0; r < b; ++r)
                        s += Sp[(i * b + r) * d.d_in + j * b + p] * Sp[(i * b + r) * d.d_in + j * b + q];
                    f2 += s * s;
                }
            for (int64_t c = 0; c < b; ++c) dn += Dd[j * b + c] * Dd[j * b + c];
            term[blk] = sqrt(f2) * sqrt(dn);
        }
        for (int64_t blk = 0; blk < d.nbi * d.nbj; ++blk) tot += term[blk];
        free(term);
        *beta = 2.0 * tot;
    }
    free(Sp); free(R);
}

/* Unmasked core gradient  Gfull = 2 A^T A C B D B^T - 2 A^T W-bar D B^T = -2 A^T (R D) B^T
 * (App. D.3 before the mask is applied). */
static void core_gradient(const double *Wb, const double *Ad, const double *Cd, const double *Bd,
                          const double *Dd, dims_t d, double *G, double *R_out) {
    int64_t P = d.d_out * d.d_in;
    double *R = dalloc(P), *T = dalloc(P);
    residual(Wb, Ad, Cd, Bd, d, R);
    if (R_out) memcpy(R_out, R, sizeof(double) * (size_t)P);
    for (int64_t i = 0; i < d.d_out; ++i)
        for (int64_t j = 0; j < d.d_in; ++j) R[i * d.d_in + j] *= Dd[j];
    left_mul(Ad, 1, R, d, T);
    right_mul(T, Bd, 1, d, G);
    for (int64_t e = 0; e < P; ++e) G[e] *= -2.0;
    free(R); free(T);
}

/* beta_W' = 2 ||A^T A||_F ||B D B^T||_F (Eq. 11); both matrices are block diagonal. */
static double beta_W(const double *Ad, const double *Bd, const double *Dd, dims_t d) {
    int64_t b = d.b;
    double fa = 0.0, fb = 0.0;
    for (int64_t i = 0; i < d.nbi; ++i)
        for (int64_t p = 0; p < b; ++p)
            for (int64_t q = 0; q < b; ++q) {
                double s = 0.0;
                for (int64_t k = 0; k < b; ++k) s += Ad[i * b * b + k * b + p] * Ad[i * b * b + k * b + q];
                fa += s * s;
            }
    for (int64_t j = 0; j < d.nbj; ++j)
        for (int64_t p = 0; p < b; ++p)
            for (int64_t q = 0; q < b; ++q) {
                double s = 0.0;
                for (int64_t k = 0; k < b; ++k)
                    s += Bd[j * b * b + p * b + k] * Dd[j * b + k] * Bd[j * b * b + q * b + k];
                fb += s * s;
            }
    return 2.0 * sqrt(fa) * sqrt(fb);
}

/* Exposed pieces (for the finite-difference, smoothness and brute-force pins). */
void oracle_grad_A(const float *Wbar, const float *A, const float *C, const float *B, const float *D,
                   int64_t d_out, int64_t d_in, int64_t b, double *gA, double *beta) {
    dims_t d = mk_dims(d_out, d_in, b);
    int64_t P = d_out * d_in;
    double *Wb = to_double(Wbar, P), *Cd = to_double(C, P), *Ad = to_double(A, d.nbi * b * b),
           *Bd = to_double(B, d.nbj * b * b), *Dd = to_double(D, d_in);
    grad_beta_A(Wb, Ad, Cd, Bd, Dd, d, gA, beta);
    free(Wb); free(Cd); free(Ad); free(Bd); free(Dd);
}
void oracle_grad_B(const float *Wbar, const float *A, const float *C, const float *B, const float *D,
                   int64_t d_out, int64_t d_in, int64_t b, double *gB, double *beta) {
    dims_t d = mk_dims(d_out, d_in, b);
    int64_t P = d_out * d_in;
    double *Wb = to_double(Wbar, P), *Cd = to_double(C, P), *Ad = to_double(A, d.nbi * b * b),
           *Bd = to_double(B, d.nbj * b * b), *Dd = to_double(D, d_in);
    grad_beta_B(Wb, Ad, Cd, Bd, Dd, d, gB, beta);
    free(Wb); free(Cd); free(Ad); free(Bd); free(Dd);
}
/* Gfull (unmasked, includes the factor -2... sign: this IS the gradient w.r.t. the core) and beta_W'.
 * The W' gradient of App. D.3 is Gfull (.) M. */
void oracle_grad_core(const float *Wbar, const float *A, const float *C, const float *B, const float *D,
                      int64_t d_out, int64_t d_in, int64_t b, double *Gfull, double *beta) {
    dims_t d = mk_dims(d_out, d_in, b);
    int64_t P = d_out * d_in;
    double *Wb = to_double(Wbar, P), *Cd = to_double(C, P), *Ad = to_double(A, d.nbi * b * b),
           *Bd = to_double(B, d.nbj * b * b), *Dd = to_double(D, d_in);
    if (Gfull) core_gradient(Wb, Ad, Cd, Bd, Dd, d, Gfull, NULL);
    if (beta) *beta = beta_W(Ad, Bd, Dd, d);
    free(Wb); free(Cd); free(Ad); free(Bd); free(Dd);
}

/* ------------------------------------------------------------------------------------------
 * Continuous update (Alg. 2 with the evaluation points of Lemma 1):
 *   A <- A - grad_A(A,B,C)/beta_A ;  B <- B - grad_B(A_new,B,C)/beta_B ;
 *   C <- C - (grad_core(A_new,B_new,C) (.) M)/beta_W'.
 * A zero beta (an all-zero operand) leaves that parameter unchanged.
 * ------------------------------------------------------------------------------------------ */
void oracle_continuous_update(const float *Wbar, const float *D, const uint8_t *mask, int64_t d_out,
                              int64_t d_in, int64_t b, float *A, float *C, float *B, double *etas) {
    dims_t d = mk_dims(d_out, d_in, b);
    int64_t P = d_out * d_in, na = d.nbi * b * b, nb = d.nbj * b * b;
    double *Wb = to_double(Wbar, P), *Dd = to_double(D, d_in);
    double beta;
    { /* A step */
        double *Cd = to_double(C, P), *Ad = to_double(A, na), *Bd = to_double(B, nb), *g = dalloc(na);
        grad_beta_A(Wb, Ad, Cd, Bd, Dd, d, g, &beta);
        if (beta > 0.0) for (int64_t e = 0; e < na; ++e) A[e] = (float)(Ad[e] - g[e] / beta);
        if (etas) etas[0] = beta > 0.0 ? 1.0 / beta : 0.0;
        free(Cd); free(Ad); free(Bd); free(g);
    }
    { /* B step at the new A */
        double *Cd = to_double(C, P), *Ad = to_double(A, na), *Bd = to_double(B, nb), *g = dalloc(nb);
        grad_beta_B(Wb, Ad, Cd, Bd, Dd, d, g, &beta);
        if (beta > 0.0) for (int64_t e = 0; e < nb; ++e) B[e] = (float)(Bd[e] - g[e] / beta);
        if (etas) etas[1] = beta > 0.0 ? 1.0 / beta : 0.0;
        free(Cd); free(Ad); free(Bd); free(g);
    }
    { /* W' step at the new A, B; only kept entries move */
        double *Cd = to_double(C, P), *Ad = to_double(A, na), *Bd = to_double(B, nb), *G = dalloc(P);
        core_gradient(Wb, Ad, Cd, Bd, Dd, d, G, NULL);
        beta = beta_W(Ad, Bd, Dd, d);
        if (beta > 0.0)
            for (int64_t e = 0; e < P; ++e)
                if (mask[e]) C[e] = (float)(Cd[e] - G[e] / beta);
        if (etas) etas[2] = beta > 0.0 ? 1.0 / beta : 0.0;
        free(Cd); free(Ad); free(Bd); free(G);
    }
    free(Wb); free(Dd);
}

/* ------------------------------------------------------------------------------------------
 * Symmetric eigen-decomposition by cyclic Jacobi rotations (textbook), for the N x N
 * pseudo-inverse of Eq. 7 / Eq. 8.  G is overwritten by its diagonalised form; V gets the
 * eigenvectors in its columns.
 * ------------------------------------------------------------------------------------------ */
static void jacobi_eig(int n, double *G, double *V) {
    for (int p = 0; p < n; ++p)
        for (int q = 0; q < n; ++q) V[p * n + q] = (p == q) ? 1.0 : 0.0;
    for (int sweep = 0; sweep < 60; ++sweep) {
        double off = 0.0, diag = 0.0;
        for (int p = 0; p < n; ++p)
            for (int q = 0; q < n; ++q) {
                if (p != q) off += G[p * n + q] * G[p * n + q];
                else diag += G[p * n + q] * G[p * n + q];
            }
        if (off <= 1e-30 * diag || off == 0.0) break;
        for (int p = 0; p < n - 1; ++p)
            for (int q = p + 1; q < n; ++q) {
                double apq = G[p * n + q];
                if (apq == 0.0) continue;
                double theta = (G[q * n + q] - G[p * n + p]) / (2.0 * apq);
                double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                double c = 1.0 / sqrt(t * t + 1.0), s = t * c;
                for (int k = 0; k < n; ++k) { /* columns p, q of G */
                    double gkp = G[k * n + p], gkq = G[k * n + q];
                    G[k * n + p] = c * gkp - s * gkq;
                    G[k * n + q] = s * gkp + c * gkq;
                }
                for (int k = 0; k < n; ++k) { /* rows p, q of G */
                    double gpk = G[p * n + k], gqk = G[q * n + k];
                    G[p * n + k] = c * gpk - s * gqk;
                    G[q * n + k] = s * gpk + c * gqk;
                }
                for (int k = 0; k < n; ++k) {
                    double vkp = V[k * n + p], vkq = V[k * n + q];
                    V[k * n + p] = c * vkp - s * vkq;
                    V[k * n + q] = s * vkp + c * vkq;
                }
            }
    }
}

/* w = G^+ q for a symmetric PSD G; returns q^T G^+ q. */
static double pinv_solve(int n, const double *Gin, const double *q, double *w) {
    double G[64], V[64];
    memcpy(G, Gin, sizeof(double) * (size_t)(n * n));
    jacobi_eig(n, G, V);
    double lmax = 0.0;
    for (int k = 0; k < n; ++k) if (G[k * n + k] > lmax) lmax = G[k * n + k];
    for (int p = 0; p < n; ++p) w[p] = 0.0;
    double gain = 0.0;
    if (lmax <= 0.0) return 0.0;
    for (int k = 0; k < n; ++k) {
        double lam = G[k * n + k];
        if (lam <= 1e-12 * lmax) continue;
        double proj = 0.0;
        for (int p = 0; p < n; ++p) proj += V[p * n + k] * q[p];
        for (int p = 0; p < n; ++p) w[p] += V[p * n + k] * proj / lam;
        gain += proj * proj / lam;
    }
    return gain;
}

/* next N-subset of {0..M-1} in lexicographic order; returns 0 when exhausted */
static int next_subset(int *s, int N, int M) {
    int p = N - 1;
    while (p >= 0 && s[p] == M - N + p) --p;
    if (p < 0) return 0;
    ++s[p];
    for (int q = p + 1; q < N; ++q) s[q] = s[q - 1] + 1;
    return 1;
}

/* ------------------------------------------------------------------------------------------
 * Sparse-core update (Alg. 3, App. B.1).  For every block (i,j): score all groups, draw one,
 * sweep the C(M,N) masks by Eq. 7, write Eq. 8's weights.
 * selection: 0 = L1-weighted random (the paper's default), 1 = L1 greedy (argmax),
 *            2 = L2-weighted random, 3 = uniform random   (App. E.1).
 * chosen_kappa / chosen_pattern (optional, one per block): the drawn group index
 * kappa = i' * (b/M) + k and the winning pattern as an M-bit mask (bit p = column p kept);
 * -1 / 0 for a skipped block (||a|| = 0).
 * ------------------------------------------------------------------------------------------ */
void oracle_sparse_core_update(const float *Wbar, const float *A, const float *B, const float *D,
                               int64_t d_out, int64_t d_in, int64_t b, int N, int M, uint64_t seed,
                               int64_t t, int selection, float *C, uint8_t *mask,
                               int32_t *chosen_kappa, int32_t *chosen_pattern) {
    dims_t d = mk_dims(d_out, d_in, b);
    int64_t P = d_out * d_in, na = d.nbi * b * b, nb = d.nbj * b * b;
    double *Wb = to_double(Wbar, P), *Cd = to_double(C, P), *Ad = to_double(A, na), *Bd = to_double(B, nb),
           *Dd = to_double(D, d_in), *G = dalloc(P), *R = dalloc(P);
    core_gradient(Wb, Ad, Cd, Bd, Dd, d, G, R);
    int64_t gpr = b / M, gpb = b * gpr, nblocks = d.nbi * d.nbj;

#pragma omp parallel for schedule(static)
    for (int64_t blk = 0; blk < nblocks; ++blk) {
        int64_t i = blk / d.nbj, j = blk % d.nbj;
        /* --- selection --- */
        int64_t best_k = 0;
        float best_key = INFINITY, best_g = -1.0f;
        for (int64_t kap = 0; kap < gpb; ++kap) {
            int64_t ip = kap / gpr, k = kap % gpr;
            const double *g = G + (i * b + ip) * d_in + j * b + k * M;
            double acc = 0.0;
            for (int p = 0; p < M; ++p) acc += (selection == 2) ? g[p] * g[p] : fabs(g[p]);
            float score = (selection == 2) ? (float)sqrt(acc) : (float)acc;
            if (selection == 3) score = 1.0f;
            if (selection == 1) {
                if (score > best_g) { best_g = score; best_k = kap; }
            } else {
                float u = oracle_uniform(seed, t, nblocks, blk, gpb, kap);
                float key = (score > 0.0f) ? (float)(-log((double)u)) / score : INFINITY;
                if (key < best_key) { best_key = key; best_k = kap; }
            }
        }
        int64_t ip = best_k / gpr, k0 = (best_k % gpr) * M;
        if (chosen_kappa) chosen_kappa[blk] = (int32_t)best_k;
        if (chosen_pattern) chosen_pattern[blk] = 0;
        /* --- Eq. 6: DeltaW = W-bar^ij - A^i W''^ij B^j = R^ij + a (c^T Bg), formed explicitly --- */
        const double *Ai = Ad + i * b * b, *Bj = Bd + j * b * b;
        double *a = dalloc(b), *dW = dalloc(b * b), *v = dalloc(b);
        double a2 = 0.0;
        for (int64_t r = 0; r < b; ++r) { a[r] = Ai[r * b + ip]; a2 += a[r] * a[r]; }
        if (a2 > 0.0) {
            double c[64];
            for (int p = 0; p < M; ++p) c[p] = Cd[(i * b + ip) * d_in + j * b + k0 + p];
            for (int64_t r = 0; r < b; ++r)
                for (int64_t q = 0; q < b; ++q) {
                    double cb = 0.0;
                    for (int p = 0; p < M; ++p) cb += c[p] * Bj[(k0 + p) * b + q];
                    dW[r * b + q] = R[(i * b + r) * d_in + j * b + q] + a[r] * cb;
                }
            /* v = DeltaW^T a  (length b), so that q_s = B' D v */
            for (int64_t q = 0; q < b; ++q) {
                double s = 0.0;
                for (int64_t r = 0; r < b; ++r) s += dW[r * b + q] * a[r];
                v[q] = s;
            }
            int s[64];
            for (int p = 0; p < N; ++p) s[p] = p;
            float best_gain = -INFINITY;
            int best_s[64];
            double best_w[64];
            do {
                double Gs[64], qs[64], w[64];
                for (int x = 0; x < N; ++x) {
                    double acc = 0.0;
                    for (int64_t q = 0; q < b; ++q) acc += Bj[(k0 + s[x]) * b + q] * Dd[j * b + q] * v[q];
                    qs[x] = acc;
                    for (int y = 0; y < N; ++y) {
                        double gg = 0.0;
                        for (int64_t q = 0; q < b; ++q)
                            gg += Bj[(k0 + s[x]) * b + q] * Dd[j * b + q] * Bj[(k0 + s[y]) * b + q];
                        Gs[x * N + y] = gg;
                    }
                }
                double gain = pinv_solve(N, Gs, qs, w) / a2; /* Eq. 7, second term */
                if ((float)gain > best_gain) {
                    best_gain = (float)gain;
                    for (int x = 0; x < N; ++x) { best_s[x] = s[x]; best_w[x] = w[x] / a2; } /* Eq. 8 */
                }
            } while (next_subset(s, N, M));
            int pat = 0;
            for (int p = 0; p < M; ++p) {
                C[(i * b + ip) * d_in + j * b + k0 + p] = 0.0f;
                mask[(i * b + ip) * d_in + j * b + k0 + p] = 0;
            }
            for (int x = 0; x < N; ++x) {
                C[(i * b + ip) * d_in + j * b + k0 + best_s[x]] = (float)best_w[x];
                mask[(i * b + ip) * d_in + j * b + k0 + best_s[x]] = 1;
                pat |= 1 << best_s[x];
            }
            if (chosen_pattern) chosen_pattern[blk] = pat;
        } else if (chosen_kappa) {
            chosen_kappa[blk] = -1;
        }
        free(a); free(dW); free(v);
    }
    free(Wb); free(Cd); free(Ad); free(Bd); free(Dd); free(G); free(R);
}

/* ------------------------------------------------------------------------------------------
 * Outer loop (Alg. 1).  sparsity: 0 = N:M (both steps), 1 = unstructured (continuous step only,
 * Sec. 4.5; `keep` entries kept).  loss_trace[0..n_iters] = L(theta_t); loss_cont_trace[t-1]
 * (optional, n_iters entries) = loss after the continuous step of iteration t.
 * Outputs stay in the normalised space; r1, r2 are returned for the denormalisation.
 *
 * Extended form (diagnostics and restart; no arithmetic of its own):
 *   init_from   0: theta_0 by Eq. 3.  1: theta_0 = the caller's (A, C, B, mask) (normalised space;
 *               C must be zero where mask is 0): Alg. 1 takes theta_0 as an input, so any feasible
 *               point is a legitimate start, and a run cut in two pieces is the same run.
 *   iter_offset iterations already done: iteration t of this call draws its groups with the
 *               counter of iteration iter_offset + t.
 *   etas        optional [n_iters][3]: the step sizes eta_A, eta_B, eta_W' = 1/beta of Eq. 9-11 that
 *               iteration t used (0 when beta = 0).
 *   mask_changes optional [n_iters]: groups whose kept set the sparse-core step changed.
 * ------------------------------------------------------------------------------------------ */
static int64_t count_changed_groups(const uint8_t *before, const uint8_t *after, int64_t P, int M) {
    int64_t n = 0;
    for (int64_t g = 0; g < P / M; ++g) {
        int differs = 0;
        for (int p = 0; p < M; ++p) differs |= before[g * M + p] != after[g * M + p];
        n += differs;
    }
    return n;
}

void oracle_factorize_layer_ex(const float *W, const float *D, int64_t d_out, int64_t d_in, int64_t b,
                               int N, int M, int n_iters, uint64_t seed, int selection, int sparsity,
                               int64_t keep, int init_from, int64_t iter_offset, float *A, float *C,
                               float *B, uint8_t *mask, float *Wbar, float *r1, float *r2,
                               double *loss_trace, double *loss_cont_trace, double *etas,
                               int64_t *mask_changes, double tol, int *iters_done) {
    /* tol: the tolerance input of Alg. 1, which the listing declares and never uses.  Reading: the loop ends
     * after the first iteration t whose decrease is within it, L_{t-1} - L_t <= tol * L_0 (tol = 0: all n_iters
     * iterations run, also when the loss stops moving); iters_done receives that t, entries of the traces
     * after it are left untouched. */
    dims_t d = mk_dims(d_out, d_in, b);
    int64_t P = d_out * d_in;
    uint8_t *before = mask_changes ? (uint8_t *)malloc((size_t)P) : NULL;
    oracle_normalize(W, d_out, d_in, Wbar, r1, r2);
    if (!init_from) {
        oracle_init_identity(A, d.nbi, b);
        oracle_init_identity(B, d.nbj, b);
        if (sparsity == 0) oracle_init_nm(Wbar, D, d_out, d_in, N, M, C, mask);
        else oracle_init_unstructured(Wbar, D, d_out, d_in, keep, C, mask);
    }
    loss_trace[0] = oracle_proxy_loss(Wbar, A, C, B, D, d_out, d_in, b);
    if (iters_done) *iters_done = 0;
    for (int t = 1; t <= n_iters; ++t) {
        oracle_continuous_update(Wbar, D, mask, d_out, d_in, b, A, C, B, etas ? etas + 3 * (t - 1) : NULL);
        if (loss_cont_trace) loss_cont_trace[t - 1] = oracle_proxy_loss(Wbar, A, C, B, D, d_out, d_in, b);
        if (before) memcpy(before, mask, (size_t)P);
        if (sparsity == 0)
            oracle_sparse_core_update(Wbar, A, B, D, d_out, d_in, b, N, M, seed, iter_offset + t, selection, C,
                                      mask, NULL, NULL);
        if (mask_changes) mask_changes[t - 1] = sparsity == 0 ? count_changed_groups(before, mask, P, M) : 0;
        loss_trace[t] = oracle_proxy_loss(Wbar, A, C, B, D, d_out, d_in, b);
        if (iters_done) *iters_done = t;
        if (tol > 0.0 && loss_trace[t - 1] - loss_trace[t] <= tol * loss_trace[0]) break;
    }
    free(before);
}

void oracle_factorize_layer(const float *W, const float *D, int64_t d_out, int64_t d_in, int64_t b,
                            int N, int M, int n_iters, uint64_t seed, int selection, int sparsity,
                            int64_t keep, float *A, float *C, float *B, uint8_t *mask, float *Wbar,
                            float *r1, float *r2, double *loss_trace, double *loss_cont_trace) {
    oracle_factorize_layer_ex(W, D, d_out, d_in, b, N, M, n_iters, seed, selection, sparsity, keep, 0, 0, A, C, B,
                              mask, Wbar, r1, r2, loss_trace, loss_cont_trace, NULL, NULL, 0.0, NULL);
}

/* ------------------------------------------------------------------------------------------
 * Joint Adam continuous step (Sec. 3.3.1: what the authors run in practice; App. F gives the
 * learning rate 1e-4).  One gradient evaluation at the current point for A, B and W' together,
 * then the published Adam update (Kingma & Ba, Alg. 1, with bias correction) on each parameter:
 *     m <- b1 m + (1-b1) g ;  v <- b2 v + (1-b2) g^2 ;
 *     theta <- theta - lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)
 * Readings (the paper gives only the learning rate): b1 = 0.9, b2 = 0.999, eps = 1e-8 (the
 * optimiser's published defaults); the moments of W' are kept per entry and never reset; a pruned
 * entry sees a zero gradient, so its moments only decay, and its value stays exactly zero (it does
 * not enter A (W' . M) B; a re-admitted entry is overwritten by Eq. 8).  Moments are fp32 state,
 * arithmetic in fp64.  t is the 1-based iteration.  No monotonicity guarantee (Sec. 3.3.1).
 * ------------------------------------------------------------------------------------------ */
static void adam_apply(float *theta, float *m, float *v, const double *g, const uint8_t *mask, int64_t n,
                       double lr, double b1, double b2, double eps, int64_t t) {
    double c1 = 1.0 - pow(b1, (double)t), c2 = 1.0 - pow(b2, (double)t);
    for (int64_t e = 0; e < n; ++e) {
        double ge = (mask == NULL || mask[e]) ? g[e] : 0.0;
        double me = b1 * (double)m[e] + (1.0 - b1) * ge;
        double ve = b2 * (double)v[e] + (1.0 - b2) * ge * ge;
        m[e] = (float)me;
        v[e] = (float)ve;
        if (mask == NULL || mask[e])
            theta[e] = (float)((double)theta[e] - lr * (me / c1) / (sqrt(ve / c2) + eps));
    }
}

void oracle_adam_update(const float *Wbar, const float *D, const uint8_t *mask, int64_t d_out, int64_t d_in,
                        int64_t b, float *A, float *C, float *B, float *mA, float *vA, float *mB, float *vB,
                        float *mC, float *vC, double lr, double b1, double b2, double eps, int64_t t) {
    dims_t d = mk_dims(d_out, d_in, b);
    int64_t P = d_out * d_in, na = d.nbi * b * b, nb = d.nbj * b * b;
    double *Wb = to_double(Wbar, P), *Dd = to_double(D, d_in), *Cd = to_double(C, P), *Ad = to_double(A, na),
           *Bd = to_double(B, nb), *gA = dalloc(na), *gB = dalloc(nb), *G = dalloc(P);
    grad_beta_A(Wb, Ad, Cd, Bd, Dd, d, gA, NULL);          /* all three at the same point */
    grad_beta_B(Wb, Ad, Cd, Bd, Dd, d, gB, NULL);
    core_gradient(Wb, Ad, Cd, Bd, Dd, d, G, NULL);
    adam_apply(A, mA, vA, gA, NULL, na, lr, b1, b2, eps, t);
    adam_apply(B, mB, vB, gB, NULL, nb, lr, b1, b2, eps, t);
    adam_apply(C, mC, vC, G, mask, P, lr, b1, b2, eps, t);
    free(Wb); free(Dd); free(Cd); free(Ad); free(Bd); free(gA); free(gB); free(G);
}

/* Alg. 1 with the joint Adam continuous step.  Same outputs as oracle_factorize_layer; init_from,
 * iter_offset and mask_changes as in oracle_factorize_layer_ex (a start from a given point begins
 * with zero moments and step count 1: the moments are not part of theta). */
void oracle_factorize_layer_adam_ex(const float *W, const float *D, int64_t d_out, int64_t d_in, int64_t b, int N,
                                    int M, int n_iters, uint64_t seed, int selection, int sparsity, int64_t keep,
                                    double lr, double b1, double b2, double eps, int init_from, int64_t iter_offset,
                                    float *A, float *C, float *B, uint8_t *mask, float *Wbar, float *r1, float *r2,
                                    double *loss_trace, double *loss_cont_trace, int64_t *mask_changes) {
    dims_t d = mk_dims(d_out, d_in, b);
    int64_t P = d_out * d_in, na = d.nbi * b * b, nb = d.nbj * b * b;
    float *mA = (float *)calloc((size_t)na, 4), *vA = (float *)calloc((size_t)na, 4),
          *mB = (float *)calloc((size_t)nb, 4), *vB = (float *)calloc((size_t)nb, 4),
          *mC = (float *)calloc((size_t)P, 4), *vC = (float *)calloc((size_t)P, 4);
    uint8_t *before = mask_changes ? (uint8_t *)malloc((size_t)P) : NULL;
    oracle_normalize(W, d_out, d_in, Wbar, r1, r2);
    if (!init_from) {
        oracle_init_identity(A, d.nbi, b);
        oracle_init_identity(B, d.nbj, b);
        if (sparsity == 0) oracle_init_nm(Wbar, D, d_out, d_in, N, M, C, mask);
        else oracle_init_unstructured(Wbar, D, d_out, d_in, keep, C, mask);
    }
    loss_trace[0] = oracle_proxy_loss(Wbar, A, C, B, D, d_out, d_in, b);
    for (int t = 1; t <= n_iters; ++t) {
        oracle_adam_update(Wbar, D, mask, d_out, d_in, b, A, C, B, mA, vA, mB, vB, mC, vC, lr, b1, b2, eps, t);
        if (loss_cont_trace) loss_cont_trace[t - 1] = oracle_proxy_loss(Wbar, A, C, B, D, d_out, d_in, b);
        if (before) memcpy(before, mask, (size_t)P);
        if (sparsity == 0)
            oracle_sparse_core_update(Wbar, A, B, D, d_out, d_in, b, N, M, seed, iter_offset + t, selection, C, mask,
                                      NULL, NULL);
        if (mask_changes) mask_changes[t - 1] = sparsity == 0 ? count_changed_groups(before, mask, P, M) : 0;
        loss_trace[t] = oracle_proxy_loss(Wbar, A, C, B, D, d_out, d_in, b);
    }
    free(before);
    free(mA); free(vA); free(mB); free(vB); free(mC); free(vC);
}

void oracle_factorize_layer_adam(const float *W, const float *D, int64_t d_out, int64_t d_in, int64_t b, int N,
                                 int M, int n_iters, uint64_t seed, int selection, int sparsity, int64_t keep,
                                 double lr, double b1, double b2, double eps, float *A, float *C, float *B,
                                 uint8_t *mask, float *Wbar, float *r1, float *r2, double *loss_trace,
                                 double *loss_cont_trace) {
    oracle_factorize_layer_adam_ex(W, D, d_out, d_in, b, N, M, n_iters, seed, selection, sparsity, keep, lr, b1, b2,
                                   eps, 0, 0, A, C, B, mask, Wbar, r1, r2, loss_trace, loss_cont_trace, NULL);
}

/* ------------------------------------------------------------------------------------------
 * Denormalisation (Sec. 3.2, last paragraph): W ~= diag(r2) (A C B) diag(r1), so row p of block
 * i of A is scaled by r2[i*b+p] and column q of block j of B by r1[j*b+q].
 * ------------------------------------------------------------------------------------------ */
void oracle_denormalize(float *A, float *B, const float *r1, const float *r2, int64_t d_out,
                        int64_t d_in, int64_t b) {
    for (int64_t i = 0; i < d_out / b; ++i)
        for (int64_t p = 0; p < b; ++p)
            for (int64_t q = 0; q < b; ++q)
                A[i * b * b + p * b + q] = (float)((double)A[i * b * b + p * b + q] * (double)r2[i * b + p]);
    for (int64_t j = 0; j < d_in / b; ++j)
        for (int64_t p = 0; p < b; ++p)
            for (int64_t q = 0; q < b; ++q)
                B[j * b * b + p * b + q] = (float)((double)B[j * b * b + p * b + q] * (double)r1[j * b + q]);
}

/* ------------------------------------------------------------------------------------------
 * Compressed N:M storage: for each row and group, the N kept values in increasing column order
 * and their in-group column indices: one byte each from oracle_pack_nm, the compact bit
 * fields from oracle_pack_index_bits.
 * ------------------------------------------------------------------------------------------ */
void oracle_pack_nm(const float *C, const uint8_t *mask, int64_t d_out, int64_t d_in, int N, int M,
                    float *values, uint8_t *index) {
    for (int64_t i = 0; i < d_out; ++i)
        for (int64_t g = 0; g < d_in / M; ++g) {
            int x = 0;
            for (int p = 0; p < M; ++p)
                if (mask[i * d_in + g * M + p] && x < N) {
                    values[(i * (d_in / M) + g) * N + x] = C[i * d_in + g * M + p];
                    index[(i * (d_in / M) + g) * N + x] = (uint8_t)p;
                    ++x;
                }
        }
}

/* The index stream in its compact form: entry e of a row (e counts kept entries left to right) occupies
 * field_bits bits (1, 2 or 4 for M = 2, 4, 8) starting at bit e*field_bits of the row, bit 0 being the
 * least significant bit of the row's first byte.  row_bytes = ceil(entries*field_bits / 8). */
void oracle_pack_index_bits(const uint8_t *index, int64_t d_out, int64_t entries, int field_bits,
                            uint8_t *packed, int64_t row_bytes) {
    for (int64_t i = 0; i < d_out; ++i) {
        for (int64_t q = 0; q < row_bytes; ++q) packed[i * row_bytes + q] = 0;
        for (int64_t e = 0; e < entries; ++e)
            for (int t = 0; t < field_bits; ++t) {
                int64_t pos = e * field_bits + t;
                if ((index[i * entries + e] >> t) & 1) packed[i * row_bytes + pos / 8] |= (uint8_t)(1u << (pos % 8));
            }
    }
}

/* ------------------------------------------------------------------------------------------
 * The factorized layer applied to a batch of activations (Sec. 3.1: the wrappers are applied as
 * batched block products around the N:M core; Sec. 4.4 times exactly this on a batch of tokens):
 *     u = B x   (block j of u from block j of x),   v = S u,   y = A v   (block i of y from block i of v)
 * X is [n][d_in] (one token per row), Y is [n][d_out].  S comes in its compressed form: per row
 * and group the N kept values in increasing column order and their in-group columns (one byte
 * each, as oracle_pack_nm writes them).  All sums in fp64.  With round_bf16 != 0 the two
 * intermediates u and v are rounded to bfloat16 (round to nearest even) before the next product,
 * which is what a bf16 pipeline with fp32 accumulators does; with 0 nothing is rounded and the
 * result is the exact product X (A S B)^T.
 * ------------------------------------------------------------------------------------------ */
static double round_to_bf16(double x) {
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return x; /* NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

void oracle_apply_packed(const float *X, int64_t n, const float *A, const float *values, const uint8_t *index,
                         const float *B, int64_t d_out, int64_t d_in, int64_t b, int N, int M, int round_bf16,
                         double *Y) {
    int64_t gpr = d_in / M;
    double *u = dalloc(d_in), *v = dalloc(d_out);
    for (int64_t t = 0; t < n; ++t) {
        const float *x = X + t * d_in;
        for (int64_t j = 0; j < d_in / b; ++j)
            for (int64_t p = 0; p < b; ++p) {
                double acc = 0.0;
                for (int64_t q = 0; q < b; ++q) acc += (double)B[(j * b + p) * b + q] * (double)x[j * b + q];
                u[j * b + p] = round_bf16 ? round_to_bf16(acc) : acc;
            }
        for (int64_t o = 0; o < d_out; ++o) {
            double acc = 0.0;
            for (int64_t g = 0; g < gpr; ++g)
                for (int e = 0; e < N; ++e) {
                    int64_t at = (o * gpr + g) * N + e;
                    acc += (double)values[at] * u[g * M + index[at]];
                }
            v[o] = round_bf16 ? round_to_bf16(acc) : acc;
        }
        for (int64_t i = 0; i < d_out / b; ++i)
            for (int64_t p = 0; p < b; ++p) {
                double acc = 0.0;
                for (int64_t q = 0; q < b; ++q) acc += (double)A[(i * b + p) * b + q] * v[i * b + q];
                Y[t * d_out + i * b + p] = acc;
            }
    }
    free(u);
    free(v);
}
