/*
 * CPU oracle for the SAGE hot path: Frequent Directions sketch + agreement scoring + top-m selection.
 *
 * TEST INFRASTRUCTURE ONLY. Plain, slow, fp64, obviously-correct code used to check the HIP library.
 * It shares no source, header, table or helper with the HIP path, and nothing in the product imports it.
 *
 * What it follows (paper = arxiv 2510.02470):
 *   - Method section, FD paragraph + Algorithm 1 Phase I: rows are placed in a buffer; when the buffer is
 *     full take the SVD, delta = sigma_ell^2, Sigma'_jj = sqrt(max(sigma_j^2 - delta, 0)), S <- Sigma' V^T.
 *     Reading taken where the printed pseudo-code cannot be followed literally: the buffer holds n = 2*ell
 *     rows (Liberty's variant), new rows go only into rows that are zero, delta is the ell-th largest
 *     squared singular value, so a shrink happens every ell rows after the first fill and at least
 *     ell+1 rows are zero after it.
 *   - "Two-pass scoring" paragraph + Algorithm 1 Phase II: z = projection of g, zhat = z/||z|| (0 if z = 0),
 *     zbar = mean of zhat, u = zbar/||zbar|| (0 if zbar = 0), alpha_i = <zhat_i, u>.
 *     Reading: the projection is onto the top-k right singular vectors of the frozen sketch
 *     (z = V_k^T g), not the sigma-weighted rows of S.
 *   - Algorithm 1, "Select top-k by alpha": the m largest alpha; ties go to the lower index; the set is
 *     returned in ascending index order; m = floor(keep_rate*N + 0.5).
 *
 * Two SVD routes, both textbook Jacobi, both pinned against numpy.linalg.svd in the tests:
 *   mode 0: one-sided (Hestenes) Jacobi on the rows of B           -- the definition
 *   mode 1: fp64 Gram B B^T + cyclic two-sided Jacobi, rows rebuilt -- same result, cheaper when D is large
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int ell, n, mode;
    int64_t D;
    double *B;       /* n x D row-major */
    double *W;       /* work copy n x D (basis, gram-route rebuild) */
    int fill;
    double sum_delta, frob2, last_delta;
    int64_t rows_seen;
    int n_shrinks, last_sweeps;
    /* scoring */
    int k;
    double *V;       /* k x D, rows are v_j^T */
    double *sig2;    /* n, squared singular values found by the last decomposition, descending */
    double *zhat;    /* N x k, grows */
    int64_t n_scored, cap_scored;
    double *s;       /* k, sum of zhat */
    double *alpha;   /* N after select */
    double u[1024];
} orc_ctx;

static double bf16_to_double(uint16_t h) {
    uint32_t w = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &w, 4);
    return (double)f;
}

int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Round-robin ("chess tournament") pairing of n (even) players: step t in [0, n-1), slot i in [0, n/2). */
static void rr_pair(int n, int t, int i, int *p, int *q) {
    int m = n - 1; /* player m stays put and meets player t; the others pair up around t */
    int a = (i == 0) ? m : (t + i) % m;
    int b = (i == 0) ? t % m : (t + m - i) % m;
    if (a < b) { *p = a; *q = b; } else { *p = b; *q = a; }
}

/*
 * One-sided Jacobi (Hestenes) on the ROWS of A (n x D): plane rotations of row pairs until every pair is
 * orthogonal. On return the rows are sigma_j * v_j^T, sorted by norm descending; sig2[j] = sigma_j^2.
 * Returns the number of sweeps used. (Method section, "thin SVD"; the paper names no algorithm.)
 */
int orc_hestenes_rows(double *A, int n, int64_t D, double *sig2) {
    const double tol = 8.0 * 2.220446049250313e-16 * sqrt((double)D);
    int ne = n + (n & 1);  /* pad to even; the phantom row index n is skipped */
    int sweeps = 0;
    /* rows whose squared norm is below rounding level of the whole matrix are numerically zero: leave them */
    double fro = 0;
    for (int64_t e = 0; e < (int64_t)n * D; ++e) fro += A[e] * A[e];
    const double tiny = 2.220446049250313e-16 * 2.220446049250313e-16 * fro * (double)n;
    for (int sweep = 0; sweep < 60; ++sweep) {
        int rotated = 0;
        for (int t = 0; t < ne - 1; ++t) {
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : rotated)
            for (int i = 0; i < ne / 2; ++i) {
                int p, q;
                rr_pair(ne, t, i, &p, &q);
                if (q >= n) continue;
                double *ap = A + (int64_t)p * D, *aq = A + (int64_t)q * D;
                double pp = 0, qq = 0, pq = 0;
                for (int64_t d = 0; d < D; ++d) {
                    pp += ap[d] * ap[d];
                    qq += aq[d] * aq[d];
                    pq += ap[d] * aq[d];
                }
                if (pp <= tiny || qq <= tiny) continue;
                if (fabs(pq) <= tol * sqrt(pp) * sqrt(qq)) continue;
                /* rotation that zeroes <a_p, a_q> */
                double zeta = (qq - pp) / (2.0 * pq);
                double tt = (zeta >= 0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                double c = 1.0 / sqrt(1.0 + tt * tt), s = c * tt;
                for (int64_t d = 0; d < D; ++d) {
                    double x = ap[d], y = aq[d];
                    ap[d] = c * x - s * y;
                    aq[d] = s * x + c * y;
                }
                rotated += 1;
            }
        }
        sweeps = sweep + 1;
        if (!rotated) break;
    }
    /* norms, then selection sort of rows by norm descending (stable on ties) */
    double *nrm = (double *)malloc(sizeof(double) * n);
    for (int j = 0; j < n; ++j) {
        double a = 0;
        const double *r = A + (int64_t)j * D;
        for (int64_t d = 0; d < D; ++d) a += r[d] * r[d];
        nrm[j] = a;
    }
    int *ord = (int *)malloc(sizeof(int) * n);
    for (int j = 0; j < n; ++j) ord[j] = j;
    for (int a = 1; a < n; ++a) { /* insertion sort: stable */
        int v = ord[a];
        int b = a - 1;
        while (b >= 0 && nrm[ord[b]] < nrm[v]) { ord[b + 1] = ord[b]; --b; }
        ord[b + 1] = v;
    }
    double *tmp = (double *)malloc(sizeof(double) * (size_t)n * D);
    for (int j = 0; j < n; ++j) {
        memcpy(tmp + (int64_t)j * D, A + (int64_t)ord[j] * D, sizeof(double) * D);
        sig2[j] = nrm[ord[j]];
    }
    memcpy(A, tmp, sizeof(double) * (size_t)n * D);
    free(tmp); free(ord); free(nrm);
    return sweeps;
}

/*
 * Cyclic two-sided Jacobi for a symmetric n x n matrix C (row-major, destroyed): C = Y diag(lam) Y^T.
 * Y is n x n row-major with eigenvectors in COLUMNS; lam and the columns of Y are sorted descending.
 */
int orc_sym_jacobi(double *C, int n, double *Y, double *lam) {
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) Y[(int64_t)i * n + j] = (i == j) ? 1.0 : 0.0;
    int sweeps = 0;
    for (int sweep = 0; sweep < 60; ++sweep) {
        int rotated = 0;
        for (int p = 0; p < n - 1; ++p) {
            for (int q = p + 1; q < n; ++q) {
                double apq = C[(int64_t)p * n + q];
                double app = C[(int64_t)p * n + p], aqq = C[(int64_t)q * n + q];
                if (apq == 0.0) continue;
                if (fabs(apq) <= 1e-16 * sqrt(fabs(app)) * sqrt(fabs(aqq))) continue;
                double zeta = (aqq - app) / (2.0 * apq);
                double t = (zeta >= 0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
                /* C <- J^T C J with J = [[c, s], [-s, c]] acting on (p, q) */
                for (int r = 0; r < n; ++r) { /* columns p, q */
                    double x = C[(int64_t)r * n + p], y = C[(int64_t)r * n + q];
                    C[(int64_t)r * n + p] = c * x - s * y;
                    C[(int64_t)r * n + q] = s * x + c * y;
                }
                for (int r = 0; r < n; ++r) { /* rows p, q */
                    double x = C[(int64_t)p * n + r], y = C[(int64_t)q * n + r];
                    C[(int64_t)p * n + r] = c * x - s * y;
                    C[(int64_t)q * n + r] = s * x + c * y;
                }
                C[(int64_t)p * n + q] = 0.0;
                C[(int64_t)q * n + p] = 0.0;
                for (int r = 0; r < n; ++r) {
                    double x = Y[(int64_t)r * n + p], y = Y[(int64_t)r * n + q];
                    Y[(int64_t)r * n + p] = c * x - s * y;
                    Y[(int64_t)r * n + q] = s * x + c * y;
                }
                rotated += 1;
            }
        }
        sweeps = sweep + 1;
        if (!rotated) break;
    }
    int *ord = (int *)malloc(sizeof(int) * n);
    for (int j = 0; j < n; ++j) ord[j] = j;
    for (int a = 1; a < n; ++a) {
        int v = ord[a];
        int b = a - 1;
        while (b >= 0 && C[(int64_t)ord[b] * n + ord[b]] < C[(int64_t)v * n + v]) { ord[b + 1] = ord[b]; --b; }
        ord[b + 1] = v;
    }
    double *Yt = (double *)malloc(sizeof(double) * (size_t)n * n);
    for (int j = 0; j < n; ++j) {
        double l = C[(int64_t)ord[j] * n + ord[j]];
        lam[j] = l > 0 ? l : 0.0;
        for (int r = 0; r < n; ++r) Yt[(int64_t)r * n + j] = Y[(int64_t)r * n + ord[j]];
    }
    memcpy(Y, Yt, sizeof(double) * (size_t)n * n);
    free(Yt); free(ord);
    return sweeps;
}

/* One entry of the Gram matrix B B^T: the plain dot product of two rows, summed in index order. */
double orc_row_dot(const double *a, const double *b, int64_t D) {
    double acc = 0;
    for (int64_t d = 0; d < D; ++d) acc += a[d] * b[d];
    return acc;
}

/* Gram route: decompose the n x D matrix A. On return W (n x D) holds sigma_j v_j^T (descending), sig2 the
 * squared singular values. A is left untouched. */
static int gram_route(const double *A, int n, int64_t D, double *W, double *sig2) {
    double *C = (double *)malloc(sizeof(double) * (size_t)n * n);
    double *Y = (double *)malloc(sizeof(double) * (size_t)n * n);
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        for (int j = 0; j <= i; ++j) {
            double acc = orc_row_dot(A + (int64_t)i * D, A + (int64_t)j * D, D);
            C[(int64_t)i * n + j] = acc;
            C[(int64_t)j * n + i] = acc;
        }
    }
    int sweeps = orc_sym_jacobi(C, n, Y, sig2);
    /* sigma_j v_j^T = y_j^T A  (since A = U Sigma V^T and y_j = u_j) */
#pragma omp parallel for schedule(dynamic, 1)
    for (int j = 0; j < n; ++j) {
        double *w = W + (int64_t)j * D;
        for (int64_t d = 0; d < D; ++d) w[d] = 0.0;
        for (int i = 0; i < n; ++i) {
            double y = Y[(int64_t)i * n + j];
            if (y == 0.0) continue;
            const double *a = A + (int64_t)i * D;
            for (int64_t d = 0; d < D; ++d) w[d] += y * a[d];
        }
    }
    free(C); free(Y);
    return sweeps;
}

orc_ctx *orc_create(int ell, int64_t D, int mode) {
    if (ell < 2 || D < 1 || (mode != 0 && mode != 1)) return NULL;
    orc_ctx *c = (orc_ctx *)calloc(1, sizeof(orc_ctx));
    c->ell = ell; c->n = 2 * ell; c->D = D; c->mode = mode;
    c->B = (double *)calloc((size_t)c->n * D, sizeof(double));
    c->W = (double *)calloc((size_t)c->n * D, sizeof(double));
    c->sig2 = (double *)calloc(c->n, sizeof(double));
    return c;
}

void orc_destroy(orc_ctx *c) {
    if (!c) return;
    free(c->B); free(c->W); free(c->sig2); free(c->V); free(c->zhat); free(c->s); free(c->alpha);
    free(c);
}

/* decompose the current buffer into c->W = sigma_j v_j^T (descending) and c->sig2 */
static void decompose(orc_ctx *c) {
    size_t bytes = sizeof(double) * (size_t)c->n * c->D;
    if (c->mode == 0) {
        memcpy(c->W, c->B, bytes);
        c->last_sweeps = orc_hestenes_rows(c->W, c->n, c->D, c->sig2);
    } else {
        c->last_sweeps = gram_route(c->B, c->n, c->D, c->W, c->sig2);
    }
}

/* FD shrink (Method section; Algorithm 1 Phase I, the two lines after "if r mod ell = 0") */
static void shrink(orc_ctx *c) {
    decompose(c);
    double delta = c->sig2[c->ell - 1];
    for (int j = 0; j < c->n; ++j) {
        double *b = c->B + (int64_t)j * c->D;
        const double *w = c->W + (int64_t)j * c->D;
        double s2 = c->sig2[j];
        double keep = s2 - delta;
        if (j >= c->ell - 1 || keep <= 0.0 || s2 <= 0.0) {
            for (int64_t d = 0; d < c->D; ++d) b[d] = 0.0;
        } else {
            double f = sqrt(keep / s2); /* sqrt(sigma^2 - delta) / sigma */
            for (int64_t d = 0; d < c->D; ++d) b[d] = f * w[d];
        }
    }
    c->sum_delta += delta;
    c->last_delta = delta;
    c->n_shrinks += 1;
    c->fill = c->ell;
}

static void push_row_done(orc_ctx *c) {
    c->fill += 1;
    c->rows_seen += 1;
    if (c->fill == c->n) shrink(c);
}

int orc_update_f32(orc_ctx *c, const float *G, int64_t rows) {
    for (int64_t i = 0; i < rows; ++i) {
        double *b = c->B + (int64_t)c->fill * c->D;
        const float *g = G + i * c->D;
        double a = 0;
        for (int64_t d = 0; d < c->D; ++d) { b[d] = (double)g[d]; a += b[d] * b[d]; }
        c->frob2 += a;
        push_row_done(c);
    }
    return 0;
}

int orc_update_bf16(orc_ctx *c, const uint16_t *G, int64_t rows) {
    for (int64_t i = 0; i < rows; ++i) {
        double *b = c->B + (int64_t)c->fill * c->D;
        const uint16_t *g = G + i * c->D;
        double a = 0;
        for (int64_t d = 0; d < c->D; ++d) { b[d] = bf16_to_double(g[d]); a += b[d] * b[d]; }
        c->frob2 += a;
        push_row_done(c);
    }
    return 0;
}

/* Freeze: top-k right singular vectors of the buffer as it stands; no shrink; B unchanged.
 * weighted = 0: rows v_j^T (the reading used by default, see the header).
 * weighted = 1: rows sqrt(max(sigma_j^2 - delta, 0)) v_j^T with delta = sigma_ell^2, i.e. the first k rows of the
 *   sketch S = Sigma' V^T that a shrink of the buffer would write -- the paper's own projection z = S g ("Two-pass
 *   scoring"; Algorithm 1, Phase II), restricted to k rows. Right after a shrink these are the sketch rows themselves. */
static int basis_common(orc_ctx *c, int k, int weighted) {
    if (k < 1 || k > c->ell - 1 || k > 1024) return -1;
    decompose(c);
    free(c->V); free(c->s); free(c->zhat); free(c->alpha);
    c->V = (double *)calloc((size_t)k * c->D, sizeof(double));
    c->s = (double *)calloc(k, sizeof(double));
    c->zhat = NULL; c->alpha = NULL; c->n_scored = 0; c->cap_scored = 0;
    c->k = k;
    double thr = (double)c->n * 1.1920928955078125e-07 * c->sig2[0]; /* n * 2^-23 * sigma_1^2 */
    double delta = c->sig2[c->ell - 1];
    for (int j = 0; j < k; ++j) {
        double s2 = c->sig2[j];
        if (s2 <= thr || s2 <= 0.0) continue; /* rank-deficient: v_j := 0 */
        double f = 1.0 / sqrt(s2);            /* W holds sigma_j v_j^T */
        if (weighted) {
            double keep = s2 - delta;
            f = keep > 0.0 ? sqrt(keep / s2) : 0.0;
        }
        const double *w = c->W + (int64_t)j * c->D;
        double *v = c->V + (int64_t)j * c->D;
        for (int64_t d = 0; d < c->D; ++d) v[d] = w[d] * f;
    }
    return 0;
}

int orc_basis(orc_ctx *c, int k) { return basis_common(c, k, 0); }
int orc_basis_weighted(orc_ctx *c, int k) { return basis_common(c, k, 1); }

/* test hook: take a basis given by the caller (k x D, rows v_j^T) */
int orc_set_basis(orc_ctx *c, const double *Vt, int k) {
    if (k < 1 || k > 1024) return -1;
    free(c->V); free(c->s); free(c->zhat); free(c->alpha);
    c->V = (double *)malloc(sizeof(double) * (size_t)k * c->D);
    memcpy(c->V, Vt, sizeof(double) * (size_t)k * c->D);
    c->s = (double *)calloc(k, sizeof(double));
    c->zhat = NULL; c->alpha = NULL; c->n_scored = 0; c->cap_scored = 0;
    c->k = k;
    return 0;
}

static void score_row(orc_ctx *c, const double *g) {
    if (c->n_scored == c->cap_scored) {
        c->cap_scored = c->cap_scored ? 2 * c->cap_scored : 1024;
        c->zhat = (double *)realloc(c->zhat, sizeof(double) * (size_t)c->cap_scored * c->k);
    }
    double *z = c->zhat + c->n_scored * c->k;
    double q2 = 0;
    for (int j = 0; j < c->k; ++j) {
        const double *v = c->V + (int64_t)j * c->D;
        double a = 0;
        for (int64_t d = 0; d < c->D; ++d) a += v[d] * g[d];
        z[j] = a;
        q2 += a * a;
    }
    double q = sqrt(q2);
    for (int j = 0; j < c->k; ++j) {
        z[j] = (q > 0.0) ? z[j] / q : 0.0;
        c->s[j] += z[j];
    }
    c->n_scored += 1;
}

int orc_score_f32(orc_ctx *c, const float *G, int64_t rows) {
    if (!c->V) return -2;
    double *g = (double *)malloc(sizeof(double) * c->D);
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t d = 0; d < c->D; ++d) g[d] = (double)G[i * c->D + d];
        score_row(c, g);
    }
    free(g);
    return 0;
}

int orc_score_bf16(orc_ctx *c, const uint16_t *G, int64_t rows) {
    if (!c->V) return -2;
    double *g = (double *)malloc(sizeof(double) * c->D);
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t d = 0; d < c->D; ++d) g[d] = bf16_to_double(G[i * c->D + d]);
        score_row(c, g);
    }
    free(g);
    return 0;
}

/*
 * Top-m of a score vector in the kernel's precision (fp32): greatest under (alpha descending, index
 * ascending); written in ascending index order. Plain definition: a full stable sort.
 */
int orc_topm_f32(const float *alpha, int64_t N, int64_t m, int64_t *out_idx) {
    if (m < 0 || m > N) return -1;
    int64_t *ord = (int64_t *)malloc(sizeof(int64_t) * (N > 0 ? N : 1));
    int64_t *tmp = (int64_t *)malloc(sizeof(int64_t) * (N > 0 ? N : 1));
    for (int64_t i = 0; i < N; ++i) ord[i] = i;
    /* bottom-up merge sort, stable: key = alpha descending */
    for (int64_t w = 1; w < N; w *= 2) {
        for (int64_t lo = 0; lo < N; lo += 2 * w) {
            int64_t mid = lo + w < N ? lo + w : N, hi = lo + 2 * w < N ? lo + 2 * w : N;
            int64_t a = lo, b = mid, o = lo;
            while (a < mid && b < hi) {
                if (alpha[ord[b]] > alpha[ord[a]]) tmp[o++] = ord[b++];
                else tmp[o++] = ord[a++];
            }
            while (a < mid) tmp[o++] = ord[a++];
            while (b < hi) tmp[o++] = ord[b++];
        }
        memcpy(ord, tmp, sizeof(int64_t) * N);
    }
    /* the first m entries are the selection; emit ascending by index */
    char *in = (char *)calloc(N > 0 ? N : 1, 1);
    for (int64_t i = 0; i < m; ++i) in[ord[i]] = 1;
    int64_t o = 0;
    for (int64_t i = 0; i < N; ++i) if (in[i]) out_idx[o++] = i;
    free(in); free(ord); free(tmp);
    return 0;
}

int64_t orc_keep_count(double keep_rate, int64_t N) {
    double x = floor(keep_rate * (double)N + 0.5);
    int64_t m = (int64_t)x;
    if (m < 0) m = 0;
    if (m > N) m = N;
    return m;
}

/* consensus, scores, selection. out_idx needs room for m entries (cap). */
int orc_select(orc_ctx *c, double keep_rate, int64_t *out_idx, int64_t cap, int64_t *out_m) {
    if (!c->V) return -2;
    int64_t N = c->n_scored;
    double nn = 0;
    for (int j = 0; j < c->k; ++j) nn += c->s[j] * c->s[j];
    nn = sqrt(nn);
    for (int j = 0; j < c->k; ++j) c->u[j] = (nn > 0.0) ? c->s[j] / nn : 0.0;
    free(c->alpha);
    c->alpha = (double *)malloc(sizeof(double) * (N > 0 ? N : 1));
    float *a32 = (float *)malloc(sizeof(float) * (N > 0 ? N : 1));
    for (int64_t i = 0; i < N; ++i) {
        const double *z = c->zhat + i * c->k;
        double a = 0;
        for (int j = 0; j < c->k; ++j) a += z[j] * c->u[j];
        if (a > 1.0) a = 1.0;
        if (a < -1.0) a = -1.0;
        if (a == 0.0) a = 0.0; /* -0 -> +0 */
        c->alpha[i] = a;
        a32[i] = (float)a;
        if (a32[i] == 0.0f) a32[i] = 0.0f;
    }
    int64_t m = orc_keep_count(keep_rate, N);
    *out_m = m;
    int rc = 0;
    if (m > cap) rc = -3;
    else rc = orc_topm_f32(a32, N, m, out_idx);
    free(a32);
    return rc;
}

/* getters */
const double *orc_B(orc_ctx *c) { return c->B; }
const double *orc_V(orc_ctx *c) { return c->V; }
const double *orc_sig2(orc_ctx *c) { return c->sig2; }
const double *orc_alpha(orc_ctx *c) { return c->alpha; }
const double *orc_zhat(orc_ctx *c) { return c->zhat; }
const double *orc_u(orc_ctx *c) { return c->u; }
const double *orc_ssum(orc_ctx *c) { return c->s; }
int orc_fill(orc_ctx *c) { return c->fill; }
int64_t orc_n_scored(orc_ctx *c) { return c->n_scored; }
double orc_sum_delta(orc_ctx *c) { return c->sum_delta; }
double orc_last_delta(orc_ctx *c) { return c->last_delta; }
double orc_frob2(orc_ctx *c) { return c->frob2; }
int orc_n_shrinks(orc_ctx *c) { return c->n_shrinks; }
int orc_last_sweeps(orc_ctx *c) { return c->last_sweeps; }
int64_t orc_rows_seen(orc_ctx *c) { return c->rows_seen; }
