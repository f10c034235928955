/*
 * RotateK CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of what the RotateK hot path computes,
 * written from the paper's definitions (Sec. 3.2 "Overview of RotateK",
 * Eq. 1-3, "Query-Weighted PCA", Eq. 4, Alg. 1, Alg. 2, App. C).  It shares no
 * code with the HIP path and is never called by the product: only the tests,
 * the smoke check and the benchmark's cpu_baseline leg load it.
 *
 * Where the method has a plain definition the oracle is that definition:
 *   - centered scatter by the two-pass formula         (Alg. 1 steps 1-3)
 *   - Hadamard re-weighting by sigma sigma^T           (Alg. 1 step 5, Eq. 4)
 *   - full symmetric eigendecomposition, eigenvectors ordered by decreasing
 *     eigenvalue (the definition of R in "Query-Weighted PCA"); computed by
 *     textbook cyclic Jacobi so that no library is trusted blindly -- the
 *     tests pin it against LAPACK, closed forms and brute force
 *   - K~ = K R_k, delta_mu = mu - R_k R_k^T mu        (Alg. 1 steps 14-15)
 *   - q~ = q R_k, b = q . delta_mu,
 *     softmax((q~ K~^T + b)/sqrt(d)) V by the one-pass
 *     max-subtracted definition                        (Alg. 2 steps 1-3, 6)
 * No blocking, fusion or reordering beyond those statements.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py.
 *
 * All matrices are row-major double.  Index conventions:
 *   K [N,d], C [d,d], R [d,d] (column j = j-th eigenvector), Rr [d,r],
 *   Kt [L,r] (packed rotated keys), V [L,d].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Alg. 1 steps 1-3: per-channel mean, centered keys, centered scatter.
 * tok (optional): row indices into K, taken in list order; n = rows used.
 * center = 0 gives the literal uncentered K^T K of Sec. 3.3's first line
 * (mu is still returned as the mean).                                        */
void orc_mean_scatter(const double* K, int64_t n, int d, const int32_t* tok,
                      int center, double* mu, double* C)
{
    for (int j = 0; j < d; ++j) mu[j] = 0.0;
    for (int64_t t = 0; t < n; ++t) {
        const double* row = K + (tok ? (int64_t)tok[t] : t) * d;
        for (int j = 0; j < d; ++j) mu[j] += row[j];
    }
    if (n > 0) for (int j = 0; j < d; ++j) mu[j] /= (double)n;

    for (int i = 0; i < d * d; ++i) C[i] = 0.0;
    double* x = (double*)malloc(sizeof(double) * (size_t)d);
    for (int64_t t = 0; t < n; ++t) {
        const double* row = K + (tok ? (int64_t)tok[t] : t) * d;
        for (int j = 0; j < d; ++j) x[j] = center ? row[j] - mu[j] : row[j];
        for (int i = 0; i < d; ++i) {
            double xi = x[i];
            double* Ci = C + (size_t)i * d;
            for (int j = 0; j < d; ++j) Ci[j] += xi * x[j];
        }
    }
    free(x);
}

/* Alg. 1 step 5 / Eq. 4: C_q[i][j] = sigma_i sigma_j C[i][j].  sigma NULL = ones. */
void orc_weight(const double* C, const double* sigma, int d, double* Cq)
{
    for (int i = 0; i < d; ++i)
        for (int j = 0; j < d; ++j)
            Cq[i * d + j] = sigma ? sigma[i] * sigma[j] * C[i * d + j] : C[i * d + j];
}

/* ------------------------------------------------------------------------ */
/* Full symmetric eigendecomposition by cyclic (row-by-row) Jacobi.
 * Each rotation J = [[c, s], [-s, c]] in the (p,q) plane is chosen so that
 * (J^T A J)[p][q] = 0; A <- J^T A J, V <- V J.  Stops when the off-diagonal
 * Frobenius norm is <= tol * ||A||_F.  On return column j of R is the
 * eigenvector of lam[j]; pairs are sorted by decreasing eigenvalue (ties: the
 * pair that sat in the lower column first), and every eigenvector's sign is
 * fixed so that its largest-magnitude entry (lowest index on ties) is > 0.
 * Returns the number of sweeps used, or -1 if max_sweeps was not enough.     */
int orc_jacobi_eigh(const double* A_in, int d, double tol, int max_sweeps,
                    double* R, double* lam)
{
    size_t nn = (size_t)d * d;
    double* A = (double*)malloc(sizeof(double) * nn);
    double* V = (double*)malloc(sizeof(double) * nn);
    memcpy(A, A_in, sizeof(double) * nn);
    /* symmetrise defensively: the definition is for a symmetric matrix */
    for (int i = 0; i < d; ++i)
        for (int j = i + 1; j < d; ++j) {
            double m = 0.5 * (A[i * d + j] + A[j * d + i]);
            A[i * d + j] = m; A[j * d + i] = m;
        }
    for (size_t i = 0; i < nn; ++i) V[i] = 0.0;
    for (int i = 0; i < d; ++i) V[i * d + i] = 1.0;

    double normF = 0.0;
    for (size_t i = 0; i < nn; ++i) normF += A[i] * A[i];
    normF = sqrt(normF);

    int sweeps = -1;
    for (int sweep = 0; sweep <= max_sweeps; ++sweep) {
        double off = 0.0;
        for (int i = 0; i < d; ++i)
            for (int j = 0; j < d; ++j)
                if (i != j) off += A[i * d + j] * A[i * d + j];
        off = sqrt(off);
        if (off <= tol * normF) { sweeps = sweep; break; }
        if (sweep == max_sweeps) break;
        for (int p = 0; p < d - 1; ++p) {
            for (int q = p + 1; q < d; ++q) {
                double apq = A[p * d + q];
                if (apq == 0.0) continue;
                double tau = (A[q * d + q] - A[p * d + p]) / (2.0 * apq);
                double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(tau * tau + 1.0));
                double c = 1.0 / sqrt(t * t + 1.0);
                double s = t * c;
                for (int k = 0; k < d; ++k) {           /* A <- A J (columns p,q) */
                    double akp = A[k * d + p], akq = A[k * d + q];
                    A[k * d + p] = c * akp - s * akq;
                    A[k * d + q] = s * akp + c * akq;
                }
                for (int k = 0; k < d; ++k) {           /* A <- J^T A (rows p,q) */
                    double apk = A[p * d + k], aqk = A[q * d + k];
                    A[p * d + k] = c * apk - s * aqk;
                    A[q * d + k] = s * apk + c * aqk;
                }
                for (int k = 0; k < d; ++k) {           /* V <- V J */
                    double vkp = V[k * d + p], vkq = V[k * d + q];
                    V[k * d + p] = c * vkp - s * vkq;
                    V[k * d + q] = s * vkp + c * vkq;
                }
            }
        }
    }

    /* order: decreasing eigenvalue, ties by original column (insertion sort) */
    int* ord = (int*)malloc(sizeof(int) * (size_t)d);
    for (int j = 0; j < d; ++j) ord[j] = j;
    for (int a = 1; a < d; ++a) {
        int oj = ord[a];
        double lj = A[oj * d + oj];
        int b = a - 1;
        while (b >= 0 && A[ord[b] * d + ord[b]] < lj) { ord[b + 1] = ord[b]; --b; }
        ord[b + 1] = oj;
    }
    for (int j = 0; j < d; ++j) {
        int src = ord[j];
        lam[j] = A[src * d + src];
        int arg = 0; double best = -1.0;
        for (int i = 0; i < d; ++i) {
            double a = fabs(V[i * d + src]);
            if (a > best) { best = a; arg = i; }
        }
        double sg = V[arg * d + src] < 0.0 ? -1.0 : 1.0;
        for (int i = 0; i < d; ++i) R[i * d + j] = sg * V[i * d + src];
    }
    free(ord); free(A); free(V);
    return sweeps;
}

/* ------------------------------------------------------------------------ */
/* Head-wise keep-mask in the rotated basis ("the first k columns" of the
 * eigenvalue-ordered R, Sec. 3.2).  Works on eigenvalues given in ANY column
 * order: rank(c) = #{i : lam[i] > lam[c]  or  (lam[i] == lam[c] and i < c)};
 * keep_idx[j] = the column whose rank is j (j < r); mask[c] = rank(c) < r.   */
void orc_select(const double* lam, int d, int r, uint8_t* mask, int32_t* keep_idx)
{
    for (int c = 0; c < d; ++c) {
        int rank = 0;
        for (int i = 0; i < d; ++i)
            if (lam[i] > lam[c] || (lam[i] == lam[c] && i < c)) ++rank;
        mask[c] = (uint8_t)(rank < r);
        if (rank < r) keep_idx[rank] = c;
    }
}

/* R_k = the kept columns of R, in keep_idx order: Rr[c][j] = R[c][keep_idx[j]] */
void orc_gather_rotation(const double* R, const int32_t* keep_idx, int d, int r, double* Rr)
{
    for (int c = 0; c < d; ++c)
        for (int j = 0; j < r; ++j)
            Rr[c * r + j] = R[c * d + keep_idx[j]];
}

/* Alg. 1 step 15: delta_mu = mu - R_k R_k^T mu */
void orc_delta_mu(const double* mu, const double* Rr, int d, int r, double* dmu)
{
    double* w = (double*)malloc(sizeof(double) * (size_t)r);
    for (int j = 0; j < r; ++j) {
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += Rr[c * r + j] * mu[c];
        w[j] = s;
    }
    for (int c = 0; c < d; ++c) {
        double s = 0.0;
        for (int j = 0; j < r; ++j) s += Rr[c * r + j] * w[j];
        dmu[c] = mu[c] - s;
    }
    free(w);
}

/* ------------------------------------------------------------------------ */
/* Storage rounding of the packed cache: one round-to-nearest-even of the
 * exact value to bfloat16 (8 significant bits, fp32 exponent range).         */
double orc_round_bf16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);                 /* |x| = m 2^e, m in [0.5,1) */
    int q = e - 8;                      /* quantum exponent for 8 significant bits */
    if (q < -133) q = -133;             /* bf16 subnormal spacing 2^-133 */
    double y = ldexp(nearbyint(ldexp(x, -q)), q);   /* nearbyint: ties-to-even */
    if (fabs(y) > 3.3895313892515355e38) y = (x < 0 ? -INFINITY : INFINITY);
    return y;
}

double orc_round_f32(double x) { return (double)(float)x; }

/* Alg. 1 step 14: K~ = K R_k, then one rounding to the cache dtype.
 * tok (optional): rows of K taken in list order.
 * rounding: 0 none, 1 fp32, 2 bf16.                                          */
void orc_compress(const double* K, int64_t n, int d, const int32_t* tok,
                  const double* Rr, int r, int rounding, double* Kt)
{
    for (int64_t t = 0; t < n; ++t) {
        const double* row = K + (tok ? (int64_t)tok[t] : t) * d;
        for (int j = 0; j < r; ++j) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += row[c] * Rr[c * r + j];
            if (rounding == 1) s = orc_round_f32(s);
            else if (rounding == 2) s = orc_round_bf16(s);
            Kt[t * r + j] = s;
        }
    }
}

/* Alg. 1 step 4 / Sec. 3.2: sigma_j = || (Q_W)_{:,j} ||_2 over the rows of the query
 * window.  Qw [rows, d]; under grouped-query attention the caller stacks the windows
 * of the G query heads that share the KV head (rows = G * W).                    */
void orc_sigma_window(const double* Qw, int64_t rows, int d, double* sigma)
{
    for (int j = 0; j < d; ++j) {
        double a = 0.0;
        for (int64_t w = 0; w < rows; ++w) a += Qw[w * d + j] * Qw[w * d + j];
        sigma[j] = sqrt(a);
    }
}

/* ------------------------------------------------------------------------ */
/* Alg. 1 steps 6-13 / App. E: subspace iteration with shifted Cholesky-QR.
 * V [d,k] starts as V0 (the caller's N(0,1) draw); T times:
 *   V <- Cq V;  G <- V^T V;  rho <- eps * tr(G) / k;  L <- chol(G + rho I)
 *   (lower triangular, L L^T = G + rho I);  V <- V L^{-T}.
 * The Cholesky factor is the textbook one (row by row); V L^{-T} is a forward
 * substitution per row of V: x L^T = v, i.e. x_j = (v_j - sum_{m<j} x_m L[j][m]) / L[j][j].
 * Returns 0, or t+1 if iteration t met a non-positive pivot (V is then left as
 * it was before that iteration's orthonormalisation).                          */
int orc_subspace_iter(const double* Cq, int d, int k, const double* V0, int T, double eps, double* V)
{
    double* W = (double*)malloc(sizeof(double) * (size_t)d * k);
    double* G = (double*)malloc(sizeof(double) * (size_t)k * k);
    double* L = (double*)calloc((size_t)k * k, sizeof(double));
    int status = 0;
    for (int i = 0; i < d * k; ++i) V[i] = V0[i];
    for (int t = 0; t < T && status == 0; ++t) {
        for (int i = 0; i < d; ++i)
            for (int j = 0; j < k; ++j) {
                double a = 0.0;
                for (int m = 0; m < d; ++m) a += Cq[i * d + m] * V[m * k + j];
                W[i * k + j] = a;
            }
        double tr = 0.0;
        for (int a = 0; a < k; ++a)
            for (int b = 0; b < k; ++b) {
                double g = 0.0;
                for (int i = 0; i < d; ++i) g += W[i * k + a] * W[i * k + b];
                G[a * k + b] = g;
                if (a == b) tr += g;
            }
        double rho = eps * tr / (double)k;
        for (int a = 0; a < k; ++a) G[a * k + a] += rho;
        for (int a = 0; a < k && status == 0; ++a)
            for (int b = 0; b <= a; ++b) {
                double sum = G[a * k + b];
                for (int m = 0; m < b; ++m) sum -= L[a * k + m] * L[b * k + m];
                if (a == b) {
                    if (!(sum > 0.0)) { status = t + 1; break; }
                    L[a * k + a] = sqrt(sum);
                } else {
                    L[a * k + b] = sum / L[b * k + b];
                }
            }
        if (status) break;
        for (int i = 0; i < d; ++i)
            for (int j = 0; j < k; ++j) {
                double x = W[i * k + j];
                for (int m = 0; m < j; ++m) x -= V[i * k + m] * L[j * k + m];
                V[i * k + j] = x / L[j * k + j];
            }
    }
    free(W); free(G); free(L);
    return status;
}

/* ------------------------------------------------------------------------ */
/* Alg. 2 steps 1-3 and 6 for one query head over the packed cache:
 * q~ = q R_k; b = q . delta_mu (0 if dmu NULL); s_n = (q~ . K~_n + b) * scale
 * with scale = 1/sqrt(d) (the ORIGINAL head dim) unless scale_override > 0;
 * p = softmax(s) by the plain max-subtracted definition; out = sum_n p_n V_n.
 * L = 0 gives zeros.  If lse_out is given it receives (max, sum exp(s-max)).  */
void orc_decode_head(const double* q, const double* Kt, const double* V,
                     const double* Rr, const double* dmu, int64_t L, int d, int r,
                     double scale_override, double* out, double* lse_out)
{
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    if (lse_out) { lse_out[0] = -INFINITY; lse_out[1] = 0.0; }
    if (L <= 0) return;
    double scale = scale_override > 0.0 ? scale_override : 1.0 / sqrt((double)d);
    double* qt = (double*)malloc(sizeof(double) * (size_t)r);
    double* s = (double*)malloc(sizeof(double) * (size_t)L);
    for (int j = 0; j < r; ++j) {
        double a = 0.0;
        for (int c = 0; c < d; ++c) a += q[c] * Rr[c * r + j];
        qt[j] = a;
    }
    double b = 0.0;
    if (dmu) for (int c = 0; c < d; ++c) b += q[c] * dmu[c];
    double M = -INFINITY;
    for (int64_t n = 0; n < L; ++n) {
        double a = 0.0;
        for (int j = 0; j < r; ++j) a += qt[j] * Kt[n * r + j];
        s[n] = (a + b) * scale;
        if (s[n] > M) M = s[n];
    }
    double Z = 0.0;
    for (int64_t n = 0; n < L; ++n) { s[n] = exp(s[n] - M); Z += s[n]; }
    for (int64_t n = 0; n < L; ++n) {
        double p = s[n] / Z;
        const double* v = V + n * d;
        for (int c = 0; c < d; ++c) out[c] += p * v[c];
    }
    if (lse_out) { lse_out[0] = M; lse_out[1] = Z; }
    free(qt); free(s);
}

/* Alg. 2 in full for one query head: the visual segment is scored in the rotated
 * basis with the mean-correction bias (steps 1-3), the prompt/text segment with
 * its unrotated full-width Keys and no bias (step 4); the two score vectors are
 * concatenated (step 5) and ONE softmax over all N + M tokens weights the
 * concatenated Values [V_vis; V_pt] (step 6).  N = 0 and/or M = 0 allowed;
 * N + M = 0 gives zeros.                                                      */
void orc_decode_dual_head(const double* q, const double* Kt, const double* Vvis, int64_t N,
                          const double* Kpt, const double* Vpt, int64_t M,
                          const double* Rr, const double* dmu, int d, int r,
                          double scale_override, double* out)
{
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    if (N + M <= 0) return;
    double scale = scale_override > 0.0 ? scale_override : 1.0 / sqrt((double)d);
    double* qt = (double*)malloc(sizeof(double) * (size_t)r);
    double* s = (double*)malloc(sizeof(double) * (size_t)(N + M));
    for (int j = 0; j < r; ++j) {
        double a = 0.0;
        for (int c = 0; c < d; ++c) a += q[c] * Rr[c * r + j];
        qt[j] = a;
    }
    double b = 0.0;
    if (dmu) for (int c = 0; c < d; ++c) b += q[c] * dmu[c];
    for (int64_t n = 0; n < N; ++n) {
        double a = 0.0;
        for (int j = 0; j < r; ++j) a += qt[j] * Kt[n * r + j];
        s[n] = (a + b) * scale;
    }
    for (int64_t m = 0; m < M; ++m) {
        double a = 0.0;
        for (int c = 0; c < d; ++c) a += q[c] * Kpt[m * d + c];
        s[N + m] = a * scale;
    }
    double mx = -INFINITY;
    for (int64_t n = 0; n < N + M; ++n) if (s[n] > mx) mx = s[n];
    double Z = 0.0;
    for (int64_t n = 0; n < N + M; ++n) { s[n] = exp(s[n] - mx); Z += s[n]; }
    for (int64_t n = 0; n < N + M; ++n) {
        double p = s[n] / Z;
        const double* v = n < N ? Vvis + n * d : Vpt + (n - N) * d;
        for (int c = 0; c < d; ++c) out[c] += p * v[c];
    }
    free(qt); free(s);
}

/* Plain full attention softmax(q K^T / sqrt(d)) V on unrotated keys (the
 * left-hand side of Eq. 1); used by the self-checks.                          */
void orc_full_attn_head(const double* q, const double* K, const double* V,
                        int64_t L, int d, double scale_override, double* out)
{
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    if (L <= 0) return;
    double scale = scale_override > 0.0 ? scale_override : 1.0 / sqrt((double)d);
    double* s = (double*)malloc(sizeof(double) * (size_t)L);
    double M = -INFINITY;
    for (int64_t n = 0; n < L; ++n) {
        double a = 0.0;
        for (int c = 0; c < d; ++c) a += q[c] * K[n * d + c];
        s[n] = a * scale;
        if (s[n] > M) M = s[n];
    }
    double Z = 0.0;
    for (int64_t n = 0; n < L; ++n) { s[n] = exp(s[n] - M); Z += s[n]; }
    for (int64_t n = 0; n < L; ++n) {
        double p = s[n] / Z;
        for (int c = 0; c < d; ++c) out[c] += p * V[n * d + c];
    }
    free(s);
}

/* ------------------------------------------------------------------------ */
/* Batched drivers: the same functions looped over (batch item, KV head)
 * units, one unit per OpenMP thread.  Nothing is restructured.               */

/* K [U,N,d]; lens[u] rows used (NULL: N).  sigma [U,d] or NULL.
 * outputs mu [U,d], C [U,d,d] (un-weighted centered scatter), R [U,d,d],
 * lam [U,d], mask [U,d], keep_idx [U,r], Rr [U,d,r], dmu [U,d].
 * Returns the largest sweep count, or -1 if any unit failed to converge.     */
int orc_fit_batch(const double* K, int U, int64_t N, int d, const int32_t* lens,
                  const double* sigma, int center, int r,
                  double* mu, double* C, double* R, double* lam,
                  uint8_t* mask, int32_t* keep_idx, double* Rr, double* dmu)
{
    int worst = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < U; ++u) {
        int64_t n = lens ? lens[u] : N;
        size_t dd = (size_t)d * d;
        double* Cq = (double*)malloc(sizeof(double) * dd);
        orc_mean_scatter(K + (size_t)u * N * d, n, d, NULL, center, mu + (size_t)u * d, C + u * dd);
        orc_weight(C + u * dd, sigma ? sigma + (size_t)u * d : NULL, d, Cq);
        int sw = orc_jacobi_eigh(Cq, d, 1e-14, 60, R + u * dd, lam + (size_t)u * d);
        orc_select(lam + (size_t)u * d, d, r, mask + (size_t)u * d, keep_idx + (size_t)u * r);
        orc_gather_rotation(R + u * dd, keep_idx + (size_t)u * r, d, r, Rr + (size_t)u * d * r);
        orc_delta_mu(mu + (size_t)u * d, Rr + (size_t)u * d * r, d, r, dmu + (size_t)u * d);
        free(Cq);
#pragma omp critical
        { if (sw < 0) worst = -1; else if (worst >= 0 && sw > worst) worst = sw; }
    }
    return worst;
}

/* K [U,N,d], Rr [U,d,r] -> Kt [U,N,r] */
void orc_compress_batch(const double* K, int U, int64_t N, int d, const int32_t* lens,
                        const double* Rr, int r, int rounding, double* Kt)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < U; ++u)
        orc_compress(K + (size_t)u * N * d, lens ? lens[u] : N, d, NULL,
                     Rr + (size_t)u * d * r, r, rounding, Kt + (size_t)u * N * r);
}

/* q [B,Hq,d]; Kt [B,Hkv,cap,r]; V [B,Hkv,cap,d]; Rr [B,Hkv,d,r]; dmu [B,Hkv,d] or
 * NULL; lens [B] or NULL (cap); out [B,Hq,d].  Query head h reads KV head
 * h / (Hq/Hkv) (App. C: R is indexed by the KV head).                        */
void orc_decode_batch(const double* q, const double* Kt, const double* V,
                      const double* Rr, const double* dmu, const int32_t* lens,
                      int B, int Hq, int Hkv, int64_t cap, int d, int r,
                      double scale_override, double* out)
{
    int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < B * Hq; ++u) {
        int b = u / Hq, h = u % Hq, hk = h / G;
        size_t kv = (size_t)b * Hkv + hk;
        orc_decode_head(q + (size_t)u * d, Kt + kv * cap * r, V + kv * cap * d,
                        Rr + kv * d * r, dmu ? dmu + kv * d : NULL,
                        lens ? lens[b] : cap, d, r, scale_override,
                        out + (size_t)u * d, NULL);
    }
}

/* Alg. 2 in full for a batch: as orc_decode_batch plus the prompt/text segment
 * Kpt, Vpt [B,Hkv,cap_t,d] with lengths lens_t [B] (NULL: cap_t).             */
void orc_decode_dual_batch(const double* q, const double* Kt, const double* V,
                           const double* Kpt, const double* Vpt,
                           const double* Rr, const double* dmu, const int32_t* lens,
                           const int32_t* lens_t, int B, int Hq, int Hkv, int64_t cap,
                           int64_t cap_t, int d, int r, double scale_override, double* out)
{
    int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < B * Hq; ++u) {
        int b = u / Hq, h = u % Hq, hk = h / G;
        size_t kv = (size_t)b * Hkv + hk;
        orc_decode_dual_head(q + (size_t)u * d, Kt + kv * cap * r, V + kv * cap * d,
                             lens ? lens[b] : cap, Kpt + kv * cap_t * d, Vpt + kv * cap_t * d,
                             lens_t ? lens_t[b] : cap_t, Rr + kv * d * r,
                             dmu ? dmu + kv * d : NULL, d, r, scale_override,
                             out + (size_t)u * d);
    }
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
