/* Every function of the C oracle on small inputs held in heap blocks of exactly the stated size
 * (full, ragged, empty and token-list cases), for a build with -fsanitize=address,undefined: an
 * index past a stated shape, a use after free or an undefined operation ends the run.  A few values
 * with closed forms are checked on the way.  Built and run by tests/test_sanitizers.py. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void orc_mean_scatter(const double* K, int64_t n, int d, const int32_t* tok, int center, double* mu, double* C);
void orc_weight(const double* C, const double* sigma, int d, double* Cq);
int orc_jacobi_eigh(const double* A_in, int d, double tol, int max_sweeps, double* R, double* lam);
void orc_select(const double* lam, int d, int r, uint8_t* mask, int32_t* keep_idx);
void orc_gather_rotation(const double* R, const int32_t* keep_idx, int d, int r, double* Rr);
void orc_delta_mu(const double* mu, const double* Rr, int d, int r, double* dmu);
double orc_round_bf16(double x);
double orc_round_f32(double x);
void orc_compress(const double* K, int64_t n, int d, const int32_t* tok, const double* Rr, int r, int rounding, double* Kt);
void orc_sigma_window(const double* Qw, int64_t rows, int d, double* sigma);
int orc_subspace_iter(const double* Cq, int d, int k, const double* V0, int T, double eps, double* V);
void orc_decode_head(const double* q, const double* Kt, const double* V, const double* Rr, const double* dmu, int64_t L,
                     int d, int r, double scale_override, double* out, double* lse_out);
void orc_decode_dual_head(const double* q, const double* Kt, const double* Vvis, int64_t N, const double* Kpt,
                          const double* Vpt, int64_t M, const double* Rr, const double* dmu, int d, int r,
                          double scale_override, double* out);
void orc_full_attn_head(const double* q, const double* K, const double* V, int64_t L, int d, double scale_override, double* out);
int orc_fit_batch(const double* K, int U, int64_t N, int d, const int32_t* lens, const double* sigma, int center, int r,
                  double* mu, double* C, double* R, double* lam, uint8_t* mask, int32_t* keep_idx, double* Rr, double* dmu);
void orc_compress_batch(const double* K, int U, int64_t N, int d, const int32_t* lens, const double* Rr, int r, int rounding, double* Kt);
void orc_decode_batch(const double* q, const double* Kt, const double* V, const double* Rr, const double* dmu,
                      const int32_t* lens, int B, int Hq, int Hkv, int64_t cap, int d, int r, double scale_override, double* out);
void orc_decode_dual_batch(const double* q, const double* Kt, const double* V, const double* Kpt, const double* Vpt,
                           const double* Rr, const double* dmu, const int32_t* lens, const int32_t* lens_t, int B, int Hq,
                           int Hkv, int64_t cap, int64_t cap_t, int d, int r, double scale_override, double* out);
int orc_num_threads(void);

static uint64_t state = 0x9e3779b97f4a7c15ull;
static double rnd(void)                      /* uniform in (-1, 1), a fixed sequence */
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(int64_t)(state >> 11) / 4503599627370496.0 - 1.0;
}
static double* block(size_t n)
{
    double* p = (double*)malloc(sizeof(double) * (n ? n : 1));
    size_t i;
    if (!p) exit(99);
    for (i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
#define CHECK(c) do { if (!(c)) { printf("failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main(void)
{
    enum { d = 12, r = 5, N = 23, U = 3, B = 2, Hq = 4, Hkv = 2, cap = 9, capt = 4 };
    double *K = block(N * d), *mu = block(d), *C = block(d * d), *Cq = block(d * d), *R = block(d * d), *lam = block(d);
    double *Rr = block(d * r), *dmu = block(d), *Kt = block(N * r), *sig = block(d), *V0 = block(d * r), *Vs = block(d * r);
    uint8_t* mask = (uint8_t*)malloc(d);
    int32_t keep[r], tok[7] = {22, 0, 5, 5, 17, 3, 9};
    int i, j, sw;
    double tr = 0.0, sl = 0.0, chk = 0.0;

    /* covariance: full, token list, one row, no row */
    orc_mean_scatter(K, N, d, NULL, 1, mu, C);
    for (i = 0; i < d; ++i) tr += C[i * d + i];
    orc_mean_scatter(K, 7, d, tok, 0, mu, Cq);
    orc_mean_scatter(K, 1, d, NULL, 1, mu, Cq);
    for (i = 0; i < d * d; ++i) CHECK(fabs(Cq[i]) < 1e-12);          /* one centred row: nothing left */
    orc_mean_scatter(K, 0, d, NULL, 1, mu, Cq);
    for (i = 0; i < d; ++i) sig[i] = fabs(sig[i]) + 0.5;
    orc_weight(C, NULL, d, Cq);
    CHECK(memcmp(C, Cq, sizeof(double) * d * d) == 0);
    orc_weight(C, sig, d, Cq);
    /* eigensolver: trace and orthogonality */
    orc_weight(C, NULL, d, Cq);
    sw = orc_jacobi_eigh(Cq, d, 1e-14, 60, R, lam);
    CHECK(sw >= 1);
    for (i = 0; i < d; ++i) sl += lam[i];
    CHECK(fabs(sl - tr) <= 1e-10 * fabs(tr));
    for (i = 0; i < d; ++i)
        for (j = 0; j < d; ++j) {
            double s = 0.0;
            int c;
            for (c = 0; c < d; ++c) s += R[c * d + i] * R[c * d + j];
            CHECK(fabs(s - (i == j)) <= 1e-10);
        }
    orc_select(lam, d, r, mask, keep);
    {
        int32_t* all = (int32_t*)malloc(sizeof(int32_t) * d);
        orc_select(lam, d, d, mask, all);                 /* r = d: every column kept */
        for (i = 0; i < d; ++i) CHECK(mask[i] == 1);
        free(all);
    }
    orc_select(lam, d, r, mask, keep);
    for (i = 0, j = 0; i < d; ++i) j += mask[i];
    CHECK(j == r);
    orc_gather_rotation(R, keep, d, r, Rr);
    orc_mean_scatter(K, N, d, NULL, 1, mu, C);
    orc_delta_mu(mu, Rr, d, r, dmu);
    /* rounding: bf16 ties to even, specials */
    CHECK(orc_round_bf16(1.0 + 1.0 / 256.0) == 1.0 && orc_round_bf16(1.0 + 3.0 / 256.0) == 1.0 + 1.0 / 64.0);
    CHECK(orc_round_bf16(0.0) == 0.0 && isinf(orc_round_bf16(INFINITY)) && isnan(orc_round_bf16(NAN)));
    CHECK(orc_round_bf16(1e-45) == 0.0 || orc_round_bf16(1e-45) > 0.0);
    CHECK(orc_round_f32(0.1) == (double)0.1f);
    /* compress: three roundings, token list, nothing */
    for (i = 0; i < 3; ++i) orc_compress(K, N, d, NULL, Rr, r, i, Kt);
    orc_compress(K, 7, d, tok, Rr, r, 1, Kt);
    orc_compress(K, 0, d, NULL, Rr, r, 0, Kt);
    orc_sigma_window(K, N, d, sig);
    orc_sigma_window(K, 0, d, sig);
    /* subspace iteration from a random start; a rank-deficient matrix must report, not crash */
    orc_weight(C, NULL, d, Cq);
    CHECK(orc_subspace_iter(Cq, d, r, V0, 5, 1e-6, Vs) == 0);
    memset(Cq, 0, sizeof(double) * d * d);
    (void)orc_subspace_iter(Cq, d, r, V0, 2, 0.0, Vs);
    /* decode: empty, one row, full; with r = d and no pruning the packed path equals plain attention */
    {
        double *q = block(d), *V = block(N * d), *out = block(d), *ref = block(d), *Rd = block(d * d), *Kd = block(N * d), lse[2];
        orc_compress(K, N, d, NULL, Rr, r, 0, Kt);
        orc_decode_head(q, Kt, V, Rr, dmu, 0, d, r, 0.0, out, lse);
        for (i = 0; i < d; ++i) CHECK(out[i] == 0.0);
        orc_decode_head(q, Kt, V, Rr, dmu, 1, d, r, 0.0, out, NULL);
        for (i = 0; i < d; ++i) CHECK(fabs(out[i] - V[i]) < 1e-12);
        orc_decode_head(q, Kt, V, Rr, NULL, N, d, r, 0.3, out, lse);
        for (i = 0; i < d; ++i) for (j = 0; j < d; ++j) Rd[i * d + j] = R[i * d + j];
        orc_compress(K, N, d, NULL, Rd, d, 0, Kd);
        orc_decode_head(q, Kd, V, Rd, NULL, N, d, d, 0.0, out, NULL);
        orc_full_attn_head(q, K, V, N, d, 0.0, ref);
        for (i = 0; i < d; ++i) CHECK(fabs(out[i] - ref[i]) <= 1e-10);
        orc_full_attn_head(q, K, V, 0, d, 0.0, ref);
        orc_decode_dual_head(q, Kt, V, N, K, V, 6, Rr, dmu, d, r, 0.0, out);
        orc_decode_dual_head(q, Kt, V, 0, K, V, 6, Rr, dmu, d, r, 0.0, out);
        orc_decode_dual_head(q, Kt, V, N, K, V, 0, Rr, NULL, d, r, 0.0, out);
        orc_decode_dual_head(q, Kt, V, 0, K, V, 0, Rr, NULL, d, r, 0.0, out);
        for (i = 0; i < d; ++i) chk += out[i];
        free(q); free(V); free(out); free(ref); free(Rd); free(Kd);
    }
    /* batch forms: ragged lengths including an empty sequence */
    {
        const int32_t lens[U] = {N, 0, 7}, lb[B] = {cap, 0}, lt[B] = {0, capt};
        double *Kb = block((size_t)U * N * d), *mub = block(U * d), *Cb = block((size_t)U * d * d), *Rb = block((size_t)U * d * d);
        double *lamb = block(U * d), *Rrb = block((size_t)U * d * r), *dmub = block(U * d), *Ktb = block((size_t)U * N * r);
        double *sgb = block(U * d);
        uint8_t* mb = (uint8_t*)malloc(U * d);
        int32_t* kb = (int32_t*)malloc(sizeof(int32_t) * U * r);
        for (i = 0; i < U * d; ++i) sgb[i] = fabs(sgb[i]) + 0.5;
        CHECK(orc_fit_batch(Kb, U, N, d, lens, sgb, 1, r, mub, Cb, Rb, lamb, mb, kb, Rrb, dmub) >= 0);
        CHECK(orc_fit_batch(Kb, U, N, d, NULL, NULL, 0, r, mub, Cb, Rb, lamb, mb, kb, Rrb, dmub) >= 1);
        orc_compress_batch(Kb, U, N, d, lens, Rrb, r, 1, Ktb);
        orc_compress_batch(Kb, U, N, d, NULL, Rrb, r, 0, Ktb);
        {
            double *q = block(B * Hq * d), *Ktc = block((size_t)B * Hkv * cap * r), *Vc = block((size_t)B * Hkv * cap * d);
            double *Rrc = block((size_t)B * Hkv * d * r), *dmc = block(B * Hkv * d), *out = block(B * Hq * d);
            double *Kp = block((size_t)B * Hkv * capt * d), *Vp = block((size_t)B * Hkv * capt * d);
            orc_decode_batch(q, Ktc, Vc, Rrc, dmc, lb, B, Hq, Hkv, cap, d, r, 0.0, out);
            for (i = 0; i < Hq * d; ++i) CHECK(out[Hq * d + i] == 0.0);        /* the empty sequence */
            orc_decode_batch(q, Ktc, Vc, Rrc, NULL, NULL, B, Hq, Hkv, cap, d, r, 0.7, out);
            orc_decode_dual_batch(q, Ktc, Vc, Kp, Vp, Rrc, dmc, lb, lt, B, Hq, Hkv, cap, capt, d, r, 0.0, out);
            orc_decode_dual_batch(q, Ktc, Vc, Kp, Vp, Rrc, NULL, NULL, NULL, B, Hq, Hkv, cap, capt, d, r, 0.0, out);
            for (i = 0; i < B * Hq * d; ++i) chk += out[i];
            free(q); free(Ktc); free(Vc); free(Rrc); free(dmc); free(out); free(Kp); free(Vp);
        }
        free(Kb); free(mub); free(Cb); free(Rb); free(lamb); free(Rrb); free(dmub); free(Ktb); free(sgb); free(mb); free(kb);
    }
    CHECK(orc_num_threads() >= 1);
    CHECK(isfinite(chk));
    printf("oracle functions ran clean, checksum %.6f\n", chk);
    free(K); free(mu); free(C); free(Cq); free(R); free(lam); free(Rr); free(dmu); free(Kt); free(sig); free(V0); free(Vs); free(mask);
    return 0;
}
