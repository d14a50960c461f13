/*
 * Host-side sanitizer run of the CPU oracle (test infrastructure only): a small driver that takes every entry point
 * of sage_oracle.c through a seeded stream -- both SVD routes, several shrink cycles, basis (plain and weighted),
 * set_basis, scoring of fp32 and bf16 rows, selection, the stand-alone routines -- and checks a few of the invariants
 * the pins check (Method, FD paragraph: 0 <= sum(delta) <= ||A||_F^2 / l; Algorithm 1, Phase II: |alpha| <= 1). It is
 * compiled together with sage_oracle.c under -fsanitize=address,undefined by tests/test_oracle_pins.py; any invalid
 * access, leak or undefined operation makes it exit non-zero.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct orc_ctx orc_ctx;
orc_ctx *orc_create(int ell, int64_t D, int mode);
void orc_destroy(orc_ctx *c);
int orc_update_f32(orc_ctx *c, const float *G, int64_t rows);
int orc_update_bf16(orc_ctx *c, const uint16_t *G, int64_t rows);
int orc_basis(orc_ctx *c, int k);
int orc_basis_weighted(orc_ctx *c, int k);
int orc_set_basis(orc_ctx *c, const double *Vt, int k);
int orc_score_f32(orc_ctx *c, const float *G, int64_t rows);
int orc_score_bf16(orc_ctx *c, const uint16_t *G, int64_t rows);
int orc_select(orc_ctx *c, double keep_rate, int64_t *out_idx, int64_t cap, int64_t *out_m);
int orc_topm_f32(const float *alpha, int64_t N, int64_t m, int64_t *out_idx);
int orc_hestenes_rows(double *A, int n, int64_t D, double *sig2);
int orc_sym_jacobi(double *C, int n, double *Y, double *lam);
double orc_row_dot(const double *a, const double *b, int64_t D);
const double *orc_alpha(orc_ctx *c);
const double *orc_V(orc_ctx *c);
double orc_sum_delta(orc_ctx *c);
double orc_frob2(orc_ctx *c);
int orc_fill(orc_ctx *c);
int orc_n_shrinks(orc_ctx *c);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double rnd(void) { /* xorshift64*, uniform in (-1, 1) */
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return (double)((rng_state * 0x2545F4914F6CDD1Dull) >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static uint16_t to_bf16(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16); }

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "sanitize_check: %s failed at line %d\n", #cond, __LINE__); return 1; } } while (0)

int main(void) {
    const int ell = 6, k = 3;
    const int64_t D = 37, N = 83;
    float *G = (float *)malloc(sizeof(float) * N * D);
    uint16_t *H = (uint16_t *)malloc(sizeof(uint16_t) * N * D);
    for (int64_t i = 0; i < N; ++i)
        for (int64_t d = 0; d < D; ++d) {
            double v = rnd() * (1.0 + (double)(d % 5)) + (i % 7 == 0 ? 3.0 : 0.0) * (d % 3 == 0);
            G[i * D + d] = (float)v;
            H[i * D + d] = to_bf16((float)v);
        }
    for (int mode = 0; mode < 2; ++mode) {
        orc_ctx *c = orc_create(ell, D, mode);
        CHECK(c != NULL);
        CHECK(orc_update_f32(c, G, 5) == 0);           /* ragged cuts, single rows, a cut on a full buffer */
        CHECK(orc_update_f32(c, G + 5 * D, 2 * ell - 5) == 0);
        CHECK(orc_update_f32(c, G + 2 * ell * D, 1) == 0);
        CHECK(orc_update_f32(c, G + (2 * ell + 1) * D, N - 2 * ell - 1) == 0);
        CHECK(orc_n_shrinks(c) == (int)((N - 2 * ell) / ell + 1) && orc_fill(c) == (int)(N - ell * orc_n_shrinks(c)));
        CHECK(orc_sum_delta(c) >= 0.0 && orc_sum_delta(c) <= orc_frob2(c) / ell);
        int64_t idx[128], m = 0;
        for (int weighted = 0; weighted < 2; ++weighted) {
            CHECK((weighted ? orc_basis_weighted(c, k) : orc_basis(c, k)) == 0);
            CHECK(orc_score_f32(c, G, N) == 0);
            CHECK(orc_select(c, 0.25, idx, 128, &m) == 0 && m == 21);
            const double *al = orc_alpha(c);
            for (int64_t i = 0; i < N; ++i) CHECK(al[i] >= -1.0 && al[i] <= 1.0);
            for (int64_t i = 1; i < m; ++i) CHECK(idx[i] > idx[i - 1]);
            CHECK(orc_select(c, 0.0, idx, 0, &m) == 0 && m == 0);
            CHECK(orc_select(c, 1.0, idx, 2, &m) == -3 && m == N);   /* output array too small */
        }
        CHECK(orc_basis(c, ell) != 0 && orc_basis(c, 0) != 0);       /* k out of range */
        double *Vt = (double *)calloc((size_t)k * D, sizeof(double));
        for (int j = 0; j < k; ++j) Vt[j * D + j] = 1.0;
        CHECK(orc_set_basis(c, Vt, k) == 0);
        CHECK(orc_score_f32(c, G, 0) == 0);                           /* empty batch */
        CHECK(orc_select(c, 0.5, idx, 128, &m) == 0 && m == 0);
        free(Vt);
        orc_destroy(c);
    }
    {   /* bf16 rows, more rows than the first capacity of the score store (1024) */
        orc_ctx *c = orc_create(ell, D, 1);
        CHECK(orc_score_bf16(c, H, 1) == -2);                         /* score before basis */
        CHECK(orc_update_bf16(c, H, N) == 0);
        CHECK(orc_basis(c, k) == 0);
        for (int rep = 0; rep < 14; ++rep) CHECK(orc_score_bf16(c, H, N) == 0);
        int64_t *idx = (int64_t *)malloc(sizeof(int64_t) * 14 * N), m = 0;
        CHECK(orc_select(c, 0.1, idx, 14 * N, &m) == 0 && m == 116);
        free(idx);
        orc_destroy(c);
    }
    {   /* the stand-alone routines */
        enum { n = 9 };
        double A[n * 11], s2[n], C[n * n], Y[n * n], lam[n];
        for (int e = 0; e < n * 11; ++e) A[e] = rnd();
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) C[i * n + j] = orc_row_dot(A + i * 11, A + j * 11, 11);
        double tr = 0;
        for (int i = 0; i < n; ++i) tr += C[i * n + i];
        CHECK(orc_sym_jacobi(C, n, Y, lam) > 0);
        CHECK(orc_hestenes_rows(A, n, 11, s2) > 0);
        double sl = 0, ss = 0;
        for (int i = 0; i < n; ++i) { sl += lam[i]; ss += s2[i]; CHECK(fabs(lam[i] - s2[i]) <= 1e-10 * tr); }
        CHECK(fabs(sl - tr) <= 1e-10 * tr && fabs(ss - tr) <= 1e-10 * tr);
        float a[7] = {0.5f, -0.0f, 0.5f, 1.0f, 0.0f, -1.0f, 0.5f};
        int64_t out[7];
        CHECK(orc_topm_f32(a, 7, 3, out) == 0 && out[0] == 0 && out[1] == 2 && out[2] == 3);
        CHECK(orc_topm_f32(a, 7, 0, out) == 0 && orc_topm_f32(a, 7, 8, out) != 0 && orc_topm_f32(a, 0, 0, out) == 0);
        orc_destroy(NULL);
        CHECK(orc_create(1, 5, 0) == NULL && orc_create(4, 0, 0) == NULL && orc_create(4, 5, 2) == NULL);
    }
    free(G); free(H);
    printf("sanitize_check ok\n");
    return 0;
}
