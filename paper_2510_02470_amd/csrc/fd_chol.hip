// Preconditioning of the Jacobi eigensolve of the Gram matrix by one Cholesky step.
//
// The shrink step needs the eigen-decomposition of the positive semi-definite C = B B^T (Method, FD paragraph). Two-sided
// Jacobi needs 7 sweeps on C itself at n = 512; on C' = L^T L, where P (C + eps I) P^T = L L^T is the Cholesky
// factorisation with the diagonal sorted in descending order, it needs 5 (C' is the matrix one step of the Cholesky LR
// iteration makes of C: it has the eigenvalues of C shifted by eps and is far closer to diagonal). With
// C' = W (Lambda + eps I) W^T the eigenvectors of C are the columns of P^T L W (Lambda + eps I)^{-1/2}. The shift eps
// (1e-6 trace) only keeps the factorisation away from the zero and slightly negative pivots a rank-deficient Gram
// matrix with fp32 rounding has; it shifts every eigenvalue by exactly eps and is taken off again. Columns whose
// eigenvalue is ~0 come out badly conditioned; the shrink gives them weight 0 (only lambda_j > lambda_ell counts).
//
// All in fp64; the 64x64x64 products run on the fp64 matrix cores. Blocked right-looking factorisation, 64 columns per
// step: `panel` (every work-group, a single wave, factors the 64x64 diagonal block in registers for itself, then solves
// its own 64 rows of the panel) and `syrk` (trailing update), then C' = L^T L, the unchanged Jacobi solve, and the back-transformation.
#include "sage_internal.h"

namespace sage {

typedef double cf64x4 __attribute__((ext_vector_type(4)));
constexpr int CLD = 68;  // leading dimension of a 64x64 LDS tile read as the row operand    (lane -> row l%16, k l/16)
constexpr int CLU = 72;  // leading dimension of a 64x64 LDS tile read as the column operand (lane -> k l/16, col l%16)

// acc(16x16) += a(16x4) b(4x16): lane l supplies a[l%16][l/16] and b[l/16][l%16]; acc element v of lane l is row
// 4v + l/16, column l%16.
__device__ __forceinline__ cf64x4 cmfma64(double a, double b, cf64x4 acc) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
}

// 64x64 global tile (row stride NP) -> LDS. transpose: dst[c][r] = src[r][c]. lower: entries above the diagonal read
// as zero (a diagonal block of L: the factorisation leaves the old upper triangle in place).
__device__ __forceinline__ void load_tile(double* dst, int ld, const double* __restrict__ src, int NP, bool transpose,
                                          bool lower, int tid) {
    double v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int e = u * 256 + tid, r = e >> 6, c = e & 63;
        v[u] = src[(int64_t)r * NP + c];
        if (lower && c > r) v[u] = 0.0;
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int e = u * 256 + tid, r = e >> 6, c = e & 63;
        dst[transpose ? c * ld + r : r * ld + c] = v[u];
    }
}

// acc[jt] (rows 16*wave .. +16, columns 16*jt .. +16) += As (64x64, [r][k], ld CLD) * Bs (64x64, [k][c], ld CLU)
__device__ __forceinline__ void tile_mma(const double* As, const double* Bs, cf64x4 (&acc)[4], int wave, int lane) {
    const int l16 = lane & 15, lk = lane >> 4;
    for (int k0 = 0; k0 < 64; k0 += 4) {
        const double a = As[(16 * wave + l16) * CLD + k0 + lk];
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) acc[jt] = cmfma64(a, Bs[(k0 + lk) * CLU + jt * 16 + l16], acc[jt]);
    }
}

// perm[rank] = index of the rank-th largest diagonal entry (ties: lower index first); diag0 = diagonal as given;
// scal[0] = eps = ridge_rel * trace (1 if the matrix is zero). One work-group of 512 threads, NP <= 512.
__global__ __launch_bounds__(512) void chol_prepare_kernel(const double* __restrict__ C, int NP, double ridge_rel,
                                                           int* __restrict__ perm, double* __restrict__ diag0,
                                                           double* __restrict__ scal) {
    __shared__ double l[512];
    __shared__ double red[512];
    const int j = threadIdx.x;
    double v = 0.0;
    if (j < NP) {
        v = C[(int64_t)j * NP + j];
        diag0[j] = v;
    }
    l[j] = v;
    red[j] = v > 0.0 ? v : 0.0;
    __syncthreads();
    for (int w = 256; w >= 1; w >>= 1) {  // fixed-shape tree
        if (j < w) red[j] += red[j + w];
        __syncthreads();
    }
    if (j < NP) {
        int rank = 0;
        for (int i = 0; i < NP; ++i) {
            const double x = l[i];
            rank += (x > v || (x == v && i < j)) ? 1 : 0;
        }
        perm[rank] = j;
    }
    if (j == 0) {
        const double tr = red[0];
        scal[0] = tr > 0.0 ? ridge_rel * tr : 1.0;
    }
}

// A[i][j] = C[perm[i]][perm[j]] + eps * (i == j)
__global__ __launch_bounds__(256) void chol_gather_kernel(const double* __restrict__ C, const int* __restrict__ perm,
                                                          const double* __restrict__ scal, double* __restrict__ A, int NP) {
    const int i = blockIdx.x;
    const int pi = perm[i];
    const double eps = scal[0];
    for (int j = threadIdx.x; j < NP; j += 256) {
        double v = C[(int64_t)pi * NP + perm[j]];
        if (i == j) v += eps;
        A[(int64_t)i * NP + j] = v;
    }
}

// Step kb of the factorisation, work-group b = 0 .. nbk-kb-1, one wave each. Lane i holds row i of the 64x64 diagonal
// block A_kk in registers and the wave factors it (right-looking: column j is scaled and every lane updates the rest of
// its row, the other lanes' entries of column j coming through v_readlane; all register indices are static, the loops
// are unrolled). b = 0 stores L_kk; b > 0 then solves X L_kk^T = A_{kb+b,kb}, lane r holding row r of X in registers
// and row j of L being read from lane j, and stores X. LDS only turns the tiles between memory order and lane order.
__device__ __forceinline__ double bcast_lane(double v, int src) {
    const long long u = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)u, src), hi = __builtin_amdgcn_readlane((int)(u >> 32), src);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

__global__ __launch_bounds__(64) void chol_panel_kernel(double* __restrict__ A, int NP, int kb,
                                                        const double* __restrict__ scal, double* __restrict__ Ld) {
    extern __shared__ double tr[];  // 64 x 65: global tiles are read and written row by row (coalesced) and turned here
    const int lane = threadIdx.x;
    const double floor_piv = scal[0] * 1e-6;  // pivots are >= eps in exact arithmetic
    // lane i <- row i of the 64x64 tile at T
    auto load_rows = [&](const double* T, int ldt, double (&v)[64]) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 64; ++r) v[r] = T[(int64_t)r * ldt + lane];  // element (r, lane): one 512-byte row per load
#pragma unroll
        for (int r = 0; r < 64; ++r) tr[r * 65 + lane] = v[r];
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 64; ++c) v[c] = tr[lane * 65 + c];
        __syncthreads();
    };
    auto store_rows = [&](double* T, int ldt, const double (&v)[64]) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < 64; ++c) tr[lane * 65 + c] = v[c];
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 64; ++r) T[(int64_t)r * ldt + lane] = tr[r * 65 + lane];
        __syncthreads();
    };
    double a[64];
    load_rows(A + ((int64_t)kb * 64) * NP + kb * 64, NP, a);
#pragma unroll
    for (int j = 0; j < 64; ++j) {
        const double d = sqrt(fmax(bcast_lane(a[j], j), floor_piv));
        double l = a[j] / d;
        if (lane == j) l = d;
        a[j] = l;  // lanes < j hold values nobody uses
#pragma unroll
        for (int k = j + 1; k < 64; ++k) a[k] -= l * bcast_lane(l, k);  // l_ij l_kj; lanes >= k hold entries of L there
    }
    const int b = blockIdx.x;
    if (b == 0) {
        double o[64];
#pragma unroll
        for (int c = 0; c < 64; ++c) o[c] = c <= lane ? a[c] : 0.0;
        // not into A_kk itself: the other work-groups of this launch may still be reading it
        store_rows(Ld + (int64_t)kb * 4096, 64, o);
        return;
    }
    double x[64];
    double* Xt = A + ((int64_t)(kb + b) * 64) * NP + kb * 64;
    load_rows(Xt, NP, x);
#pragma unroll
    for (int j = 0; j < 64; ++j) {  // x_j = (x_j - sum_{m<j} x_m L[j][m]) / L[j][j]; row j of L sits in lane j
        double s0 = x[j], s1 = 0.0;
#pragma unroll
        for (int m = 0; m + 1 < j; m += 2) {
            s0 -= x[m] * bcast_lane(a[m], j);
            s1 -= x[m + 1] * bcast_lane(a[m + 1], j);
        }
        if (j & 1) s0 -= x[j - 1] * bcast_lane(a[j - 1], j);
        x[j] = (s0 + s1) / bcast_lane(a[j], j);
    }
    store_rows(Xt, NP, x);
}

// The diagonal blocks of L, kept aside by the panel steps, go into the matrix.
__global__ __launch_bounds__(256) void chol_place_kernel(double* __restrict__ A, const double* __restrict__ Ld, int NP) {
    const int kb = blockIdx.x;
    for (int e = threadIdx.x; e < 4096; e += 256)
        A[((int64_t)kb * 64 + (e >> 6)) * NP + kb * 64 + (e & 63)] = Ld[(int64_t)kb * 4096 + e];
}

// Trailing update after step kb: A_ij -= L_ik L_jk^T for kb < j <= i < nbk; one work-group per tile.
__global__ __launch_bounds__(256) void chol_syrk_kernel(double* __restrict__ A, int NP, int kb) {
    extern __shared__ double sm[];
    double* As = sm;             // 64 x CLD
    double* Bs = sm + 64 * CLD;  // 64 x CLU
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    int t = blockIdx.x, i = 0;  // t = i (i + 1) / 2 + j over the T x T lower triangle, T = nbk - kb - 1
    while ((i + 1) * (i + 2) / 2 <= t) ++i;
    const int j = t - i * (i + 1) / 2;
    const int bi = kb + 1 + i, bj = kb + 1 + j;
    load_tile(As, CLD, A + ((int64_t)bi * 64) * NP + kb * 64, NP, false, false, tid);  // [r][k] = L_ik[r][k]
    load_tile(Bs, CLU, A + ((int64_t)bj * 64) * NP + kb * 64, NP, true, false, tid);   // [k][c] = L_jk[c][k]
    __syncthreads();
    cf64x4 acc[4];
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) acc[jt] = cf64x4{0.0, 0.0, 0.0, 0.0};
    tile_mma(As, Bs, acc, wave, lane);
    const int l16 = lane & 15, lk = lane >> 4;
    double* Aij = A + ((int64_t)bi * 64) * NP + bj * 64;
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            const int r = 16 * wave + 4 * v + lk, c = jt * 16 + l16;
            Aij[(int64_t)r * NP + c] -= acc[jt][v];
        }
}

// C' = L^T L: tile (i, j), i >= j: sum over m >= i of L_mi^T L_mj; written to both triangles.
__global__ __launch_bounds__(256) void chol_ltl_kernel(const double* __restrict__ L, double* __restrict__ Cout, int NP) {
    extern __shared__ double sm[];
    double* As = sm;
    double* Bs = sm + 64 * CLD;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nbk = NP / 64;
    int t = blockIdx.x, i = 0;
    while ((i + 1) * (i + 2) / 2 <= t) ++i;
    const int j = t - i * (i + 1) / 2;
    cf64x4 acc[4];
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) acc[jt] = cf64x4{0.0, 0.0, 0.0, 0.0};
    for (int m = i; m < nbk; ++m) {
        load_tile(As, CLD, L + ((int64_t)m * 64) * NP + i * 64, NP, true, m == i, tid);   // [r][k] = L_mi[k][r]
        load_tile(Bs, CLU, L + ((int64_t)m * 64) * NP + j * 64, NP, false, m == j, tid);  // [k][c] = L_mj[k][c]
        __syncthreads();
        tile_mma(As, Bs, acc, wave, lane);
        __syncthreads();
    }
    const int l16 = lane & 15, lk = lane >> 4;
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            const int r = i * 64 + 16 * wave + 4 * v + lk, c = j * 64 + jt * 16 + l16;
            Cout[(int64_t)r * NP + c] = acc[jt][v];
            Cout[(int64_t)c * NP + r] = acc[jt][v];
        }
}

// Yout[perm[r]][c] = (L W)[r][c] / sqrt(lambda'_c), lambda'_c = Cd[c][c] (the diagonal the Jacobi solve left, shift
// included; columns with lambda' <= 0 become 0). Tile (rb, cb): sum over kb <= rb of L_{rb,kb} W_{kb,cb}.
__global__ __launch_bounds__(256) void chol_back_kernel(const double* __restrict__ L, const double* __restrict__ W,
                                                        const double* __restrict__ Cd, const int* __restrict__ perm,
                                                        double* __restrict__ Yout, int NP) {
    extern __shared__ double sm[];
    double* As = sm;
    double* Bs = sm + 64 * CLD;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nbk = NP / 64;
    const int rb = blockIdx.x / nbk, cb = blockIdx.x % nbk;
    cf64x4 acc[4];
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) acc[jt] = cf64x4{0.0, 0.0, 0.0, 0.0};
    for (int kb = 0; kb <= rb; ++kb) {
        load_tile(As, CLD, L + ((int64_t)rb * 64) * NP + kb * 64, NP, false, kb == rb, tid);
        load_tile(Bs, CLU, W + ((int64_t)kb * 64) * NP + cb * 64, NP, false, false, tid);
        __syncthreads();
        tile_mma(As, Bs, acc, wave, lane);
        __syncthreads();
    }
    const int l16 = lane & 15, lk = lane >> 4;
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
        const int c = cb * 64 + jt * 16 + l16;
        const double lam = Cd[(int64_t)c * NP + c];
        const double sc = lam > 0.0 ? 1.0 / sqrt(lam) : 0.0;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = rb * 64 + 16 * wave + 4 * v + lk;
            Yout[(int64_t)perm[r] * NP + c] = acc[jt][v] * sc;
        }
    }
}

// Y <- Y2 (the back-transformed eigenvectors) and the shift comes off the eigenvalues: C[c][c] -= eps.
__global__ __launch_bounds__(256) void chol_finish_kernel(double* __restrict__ C, double* __restrict__ Y,
                                                          const double* __restrict__ Y2, const double* __restrict__ scal,
                                                          int NP) {
    const int row = blockIdx.x;
    for (int c = threadIdx.x; c < NP; c += 256) Y[(int64_t)row * NP + c] = Y2[(int64_t)row * NP + c];
    if (threadIdx.x == 0) C[(int64_t)row * NP + row] -= scal[0];
}

static const size_t CHOL_LDS = (size_t)(64 * CLD + 64 * CLU) * sizeof(double);
// The panel kernel uses 33 KB of LDS; it asks for 100 KB so that its single wave never shares a CU with a Gram work-group of
// the side stream (the same reason as for the Jacobi pivot kernel).
static const size_t CHOL_PANEL_LDS = 100 * 1024;

// Same contract as launch_eig: on return the diagonal of w.C holds the eigenvalues, the columns of w.Y the
// eigenvectors (rows in the order of the matrix given), w.diag0 the diagonal as given, w.stat the sweep records.
// The matrix must be positive semi-definite up to rounding. Needs w.L (NP x NP), w.Ld (NP x 64), w.perm (NP), w.scal.
hipError_t launch_eig_precond(const EigWork& w, int NP, double tol, int max_sweeps, hipStream_t st) {
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute((const void*)chol_panel_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)CHOL_PANEL_LDS);
        (void)hipFuncSetAttribute((const void*)chol_syrk_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)CHOL_LDS);
        (void)hipFuncSetAttribute((const void*)chol_ltl_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)CHOL_LDS);
        (void)hipFuncSetAttribute((const void*)chol_back_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)CHOL_LDS);
        attr = true;
    }
    const int nbk = NP / 64;
    hipLaunchKernelGGL(chol_prepare_kernel, dim3(1), dim3(512), 0, st, w.C, NP, 1e-6, w.perm, w.diag0, w.scal);
    hipLaunchKernelGGL(chol_gather_kernel, dim3(NP), dim3(256), 0, st, w.C, w.perm, w.scal, w.L, NP);
    for (int kb = 0; kb < nbk; ++kb) {
        hipLaunchKernelGGL(chol_panel_kernel, dim3(nbk - kb), dim3(64), CHOL_PANEL_LDS, st, w.L, NP, kb, w.scal, w.Ld);
        const int T = nbk - kb - 1;
        if (T > 0) hipLaunchKernelGGL(chol_syrk_kernel, dim3(T * (T + 1) / 2), dim3(256), CHOL_LDS, st, w.L, NP, kb);
    }
    hipLaunchKernelGGL(chol_place_kernel, dim3(nbk), dim3(256), 0, st, w.L, w.Ld, NP);
    hipLaunchKernelGGL(chol_ltl_kernel, dim3(nbk * (nbk + 1) / 2), dim3(256), CHOL_LDS, st, w.L, w.C, NP);
    EigWork w2 = w;
    w2.diag0 = w.lam;  // the solve records the diagonal it is given there; w.lam is rewritten by the sort afterwards
    hipError_t e = launch_eig(w2, NP, tol, max_sweeps, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(chol_back_kernel, dim3(nbk * nbk), dim3(256), CHOL_LDS, st, w.L, w.Y, w.C, w.perm, w.Y2, NP);
    hipLaunchKernelGGL(chol_finish_kernel, dim3(NP), dim3(256), 0, st, w.C, w.Y, w.Y2, w.scal, NP);
    return hipGetLastError();
}

}  // namespace sage
