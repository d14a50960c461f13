// Blocked two-sided Jacobi eigensolve of the (padded) Gram matrix, C = Y Lambda Y^T, in fp64, staged through
// LDS, and the coefficient matrices built from it.
//
// The shrink step (Method, FD paragraph) needs sigma_j^2 = lambda_j and, for the rebuild, the left singular
// vectors y_j of the buffer:  sigma_j v_j^T = y_j^T B.  The matrix is cut into 32x32 blocks. One sweep is:
//   step 0        every work-group takes two diagonal blocks and annihilates all pairs inside each block,
//   step 1..nb-1  round-robin over block pairs (I, J): annihilate every pair (p in I, q in J),
// so each off-diagonal element is rotated exactly once per sweep. A step is two kernels: `solve` runs the
// rotations of each 64x64 pivot sub-matrix in LDS and emits its accumulated 64x64 rotation Q_w; `apply`
// updates C <- Q^T C Q and Y <- Y Q with Q = blockdiag(Q_w) as small LDS-tiled products.
#include "sage_internal.h"

namespace sage {

constexpr double JACOBI_TOL = 1e-11;  // sweep converged when every |c_pq| it met was <= TOL * trace(C)
constexpr int LDA = 65;               // padded leading dimension of the 64x64 LDS matrices (doubles)

// round-robin pairing of n (even) players, step t in [0, n-1), slot i in [0, n/2): player n-1 stays put
__device__ __forceinline__ void rr_pair(int n, int t, int i, int& p, int& q) {
    int m = n - 1;
    int a = (i == 0) ? m : (t + i) % m;
    int b = (i == 0) ? (t % m) : (t + m - i) % m;
    p = a < b ? a : b;
    q = a < b ? b : a;
}

// block pair (I, J) of work-group w at step `st` of a sweep over nb blocks
__device__ __forceinline__ void block_pair(int nb, int st, int w, int& I, int& J) {
    if (st == 0) {
        I = 2 * w;
        J = 2 * w + 1;
    } else {
        rr_pair(nb, st - 1, w, I, J);
    }
}

__device__ __forceinline__ bool sweep_done(const double* stat, int sweep) {
    return sweep > 0 && stat[1 + sweep - 1] <= JACOBI_TOL;
}

__device__ __forceinline__ void atomic_max_pos_double(double* addr, double v) {
    // non-negative doubles order like their bit patterns
    atomicMax(reinterpret_cast<unsigned long long*>(addr), (unsigned long long)__double_as_longlong(v));
}

// Y = I, diag0 = diag(C), stat[0] = trace(C), stat[1..] = 0. grid = NP blocks of 256.
__global__ __launch_bounds__(256) void jac_init_kernel(const double* __restrict__ C, double* __restrict__ Y,
                                                       double* __restrict__ diag0, double* __restrict__ stat, int NP) {
    int row = blockIdx.x;
    for (int c = threadIdx.x; c < NP; c += 256) Y[(int64_t)row * NP + c] = (c == row) ? 1.0 : 0.0;
    if (row == 0) {
        __shared__ double red[512];
        for (int c = threadIdx.x; c < 512; c += 256) {
            double v = (c < NP) ? C[(int64_t)c * NP + c] : 0.0;
            red[c] = v;
            if (c < NP) diag0[c] = v;
        }
        __syncthreads();
        for (int w = 256; w >= 1; w >>= 1) {  // fixed-shape tree: deterministic
            if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            double tr = red[0];
            stat[0] = tr > 0.0 ? tr : 0.0;
        }
        if (threadIdx.x >= 1 && threadIdx.x <= MAX_SWEEPS + 1) stat[threadIdx.x] = 0.0;
    }
}

// One work-group per block pair: rotations of the 64x64 pivot sub-matrix, Q_w written to Qout[w].
__global__ __launch_bounds__(256) void jac_solve_kernel(const double* __restrict__ C, double* __restrict__ Qout,
                                                        double* __restrict__ stat, int NP, int sweep, int st) {
    if (sweep_done(stat, sweep)) return;
    extern __shared__ double sm[];
    double* A = sm;             // 64 x LDA
    double* Qm = sm + 64 * LDA; // 64 x LDA
    double* cs = Qm + 64 * LDA; // 32 x 2
    const int tid = threadIdx.x;
    const int nb = NP / 32;
    int I, J;
    block_pair(nb, st, blockIdx.x, I, J);
    const bool diag_mode = (st == 0);

    for (int e = tid; e < 64 * 64; e += 256) {
        int r = e >> 6, c = e & 63;
        int gr = (r < 32 ? I * 32 + r : J * 32 + r - 32);
        int gc = (c < 32 ? I * 32 + c : J * 32 + c - 32);
        A[r * LDA + c] = C[(int64_t)gr * NP + gc];
        Qm[r * LDA + c] = (r == c) ? 1.0 : 0.0;
    }
    __syncthreads();

    // largest element this step is about to annihilate, relative to the trace
    {
        double mx = 0.0;
        for (int e = tid; e < 64 * 64; e += 256) {
            int r = e >> 6, c = e & 63;
            bool mine = diag_mode ? ((r < 32) == (c < 32) && r != c) : ((r < 32) != (c < 32));
            if (mine) mx = fmax(mx, fabs(A[r * LDA + c]));
        }
        for (int o = 32; o >= 1; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o));
        double tr = stat[0];
        if ((tid & 63) == 0 && tr > 0.0) atomic_max_pos_double(&stat[1 + sweep], mx / tr);
    }

    const int nsteps = diag_mode ? 31 : 32;
    for (int t = 0; t < nsteps; ++t) {
        if (tid < 32) {
            int p, q;
            if (diag_mode) {
                rr_pair(32, t, tid & 15, p, q);
                if (tid >= 16) { p += 32; q += 32; }
            } else {
                p = tid;
                q = 32 + ((tid + t) & 31);
            }
            double apq = A[p * LDA + q];
            double c = 1.0, s = 0.0;
            if (apq != 0.0) {
                double app = A[p * LDA + p], aqq = A[q * LDA + q];
                double zeta = (aqq - app) / (2.0 * apq);
                double az = fabs(zeta);
                double tt = 1.0 / (az + sqrt(1.0 + az * az));
                if (zeta < 0.0) tt = -tt;
                c = 1.0 / sqrt(1.0 + tt * tt);
                s = c * tt;
            }
            cs[2 * tid] = c;
            cs[2 * tid + 1] = s;
        }
        __syncthreads();
        // 2x2 blocks: X <- R_i^T X R_j,  R = [[c, s], [-s, c]]
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            int b = it * 256 + tid;
            int i = b >> 5, j = b & 31;
            int pi, qi, pj, qj;
            if (diag_mode) {
                rr_pair(32, t, i & 15, pi, qi);
                if (i >= 16) { pi += 32; qi += 32; }
                rr_pair(32, t, j & 15, pj, qj);
                if (j >= 16) { pj += 32; qj += 32; }
            } else {
                pi = i; qi = 32 + ((i + t) & 31);
                pj = j; qj = 32 + ((j + t) & 31);
            }
            double ci = cs[2 * i], si = cs[2 * i + 1], cj = cs[2 * j], sj = cs[2 * j + 1];
            double x00 = A[pi * LDA + pj], x01 = A[pi * LDA + qj], x10 = A[qi * LDA + pj], x11 = A[qi * LDA + qj];
            double y00 = ci * x00 - si * x10, y01 = ci * x01 - si * x11;
            double y10 = si * x00 + ci * x10, y11 = si * x01 + ci * x11;
            double z00 = cj * y00 - sj * y01, z01 = sj * y00 + cj * y01;
            double z10 = cj * y10 - sj * y11, z11 = sj * y10 + cj * y11;
            if (i == j && si != 0.0) { z01 = 0.0; z10 = 0.0; }
            A[pi * LDA + pj] = z00; A[pi * LDA + qj] = z01;
            A[qi * LDA + pj] = z10; A[qi * LDA + qj] = z11;
        }
        // Q <- Q R_j
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            int b = it * 256 + tid;
            int r = b >> 5, j = b & 31;
            int pj, qj;
            if (diag_mode) {
                rr_pair(32, t, j & 15, pj, qj);
                if (j >= 16) { pj += 32; qj += 32; }
            } else {
                pj = j; qj = 32 + ((j + t) & 31);
            }
            double cj = cs[2 * j], sj = cs[2 * j + 1];
            double a = Qm[r * LDA + pj], bq = Qm[r * LDA + qj];
            Qm[r * LDA + pj] = cj * a - sj * bq;
            Qm[r * LDA + qj] = sj * a + cj * bq;
        }
        __syncthreads();
    }
    double* Qo = Qout + (int64_t)blockIdx.x * 4096;
    for (int e = tid; e < 4096; e += 256) Qo[e] = Qm[(e >> 6) * LDA + (e & 63)];
}

// 64x64x64 product in LDS by 256 threads, 4x4 micro-tile each: out(r0.., c0..) = sum_e L(e, r or r, e) * R(e, c).
// TRANS_L: left operand is read transposed (L^T R), else (L R).
template <bool TRANS_L>
__device__ __forceinline__ void mm64(const double* L, const double* R, double (&o)[4][4], int r0, int c0) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) o[u][v] = 0.0;
    for (int e = 0; e < 64; ++e) {
        double a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) a[u] = TRANS_L ? L[e * LDA + r0 + u] : L[(r0 + u) * LDA + e];
#pragma unroll
        for (int v = 0; v < 4; ++v) b[v] = R[e * LDA + c0 + v];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) o[u][v] = fma(a[u], b[v], o[u][v]);
    }
}

// grid = 2 * np^2 (np = NP/64 pairs): blocks [0, np^2) update C tile (a, b) <- Q_a^T C Q_b, the rest update
// Y tile (row chunk rc, b) <- Y Q_b. Every tile is read and written by exactly one work-group (in place).
__global__ __launch_bounds__(256) void jac_apply_kernel(double* __restrict__ C, double* __restrict__ Y,
                                                        const double* __restrict__ Q, const double* __restrict__ stat,
                                                        int NP, int sweep, int st) {
    if (sweep_done(stat, sweep)) return;
    extern __shared__ double sm[];
    double* X = sm;               // 64 x LDA
    double* Qb = sm + 64 * LDA;   // 64 x LDA
    double* Qa = Qb + 64 * LDA;   // 64 x LDA
    const int tid = threadIdx.x;
    const int np = NP / 64, nb = NP / 32;
    int bid = blockIdx.x;
    const bool isY = bid >= np * np;
    if (isY) bid -= np * np;
    const int a = bid / np, b = bid % np;
    int Ia, Ja, Ib, Jb;
    block_pair(nb, st, a, Ia, Ja);
    block_pair(nb, st, b, Ib, Jb);
    double* M = isY ? Y : C;

    for (int e = tid; e < 4096; e += 256) {
        int r = e >> 6, c = e & 63;
        int gr = isY ? (a * 64 + r) : (r < 32 ? Ia * 32 + r : Ja * 32 + r - 32);
        int gc = (c < 32 ? Ib * 32 + c : Jb * 32 + c - 32);
        X[r * LDA + c] = M[(int64_t)gr * NP + gc];
        Qb[r * LDA + c] = Q[(int64_t)b * 4096 + e];
        if (!isY) Qa[r * LDA + c] = Q[(int64_t)a * 4096 + e];
    }
    __syncthreads();
    const int r0 = (tid >> 4) * 4, c0 = (tid & 15) * 4;
    double o[4][4];
    mm64<false>(X, Qb, o, r0, c0);  // T = X Q_b
    if (!isY) {
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) X[(r0 + u) * LDA + c0 + v] = o[u][v];
        __syncthreads();
        mm64<true>(Qa, X, o, r0, c0);  // Q_a^T T
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        int r = r0 + u;
        int gr = isY ? (a * 64 + r) : (r < 32 ? Ia * 32 + r : Ja * 32 + r - 32);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            int c = c0 + v;
            int gc = (c < 32 ? Ib * 32 + c : Jb * 32 + c - 32);
            M[(int64_t)gr * NP + gc] = o[u][v];
        }
    }
}

// Eigenvalues = diagonal of the rotated C, clamped at 0; rank by counting (ties: lower column first).
// One work-group of 512 threads. Also records the sweeps that were needed in acc[3].
__global__ __launch_bounds__(512) void eig_sort_kernel(const double* __restrict__ C, const double* __restrict__ stat,
                                                       int* __restrict__ pos, double* __restrict__ lam, int NP,
                                                       double* __restrict__ acc) {
    __shared__ double l[512];
    int j = threadIdx.x;
    double v = 0.0;
    if (j < NP) {
        v = C[(int64_t)j * NP + j];
        if (!(v > 0.0)) v = 0.0;
    }
    l[j] = v;
    __syncthreads();
    if (j < NP) {
        int rank = 0;
        for (int i = 0; i < NP; ++i) {
            double x = l[i];
            rank += (x > v || (x == v && i < j)) ? 1 : 0;
        }
        pos[rank] = j;
        lam[rank] = v;
    }
    if (j == 0) {
        int used = MAX_SWEEPS;
        for (int s = 0; s < MAX_SWEEPS; ++s)
            if (stat[1 + s] <= JACOBI_TOL) { used = s + 1; break; }
        acc[3] = (double)used;
    }
}

// Shrink coefficients (Method, FD paragraph: delta = sigma_ell^2, Sigma'_jj = sqrt(max(sigma_j^2 - delta, 0))):
// new row m = w_m * y_m^T B with w_m = sqrt(max(lambda_m - delta, 0) / lambda_m); stored transposed, Mt[i][m].
__global__ __launch_bounds__(256) void shrink_coeffs_kernel(const double* __restrict__ Y, const int* __restrict__ pos,
                                                            const double* __restrict__ lam,
                                                            const double* __restrict__ diag0, int NP, int LP, int ell,
                                                            int frob_r0, int frob_r1, float* __restrict__ Mt,
                                                            double* __restrict__ acc) {
    int e = blockIdx.x * 256 + threadIdx.x;
    const double delta = lam[ell - 1];
    if (e < NP * LP) {
        int i = e / LP, m = e % LP;
        double lm = lam[m];
        double keep = lm - delta;
        double w = (keep > 0.0 && lm > 0.0) ? sqrt(keep / lm) : 0.0;
        Mt[e] = (w > 0.0) ? (float)(w * Y[(int64_t)i * NP + pos[m]]) : 0.f;
    }
    if (e == 0) {
        acc[0] += delta;
        acc[2] = delta;
        double f = 0.0;
        for (int r = frob_r0; r < frob_r1; ++r) f += diag0[r];
        acc[1] += f;
    }
}

// Basis coefficients: v_m^T = y_m^T B / sqrt(lambda_m) for m < k, or 0 when lambda_m <= n 2^-23 lambda_1.
__global__ __launch_bounds__(256) void basis_coeffs_kernel(const double* __restrict__ Y, const int* __restrict__ pos,
                                                           const double* __restrict__ lam,
                                                           const double* __restrict__ diag0, int NP, int KP, int k, int n,
                                                           int frob_r0, int frob_r1, float* __restrict__ Mt,
                                                           double* __restrict__ acc) {
    int e = blockIdx.x * 256 + threadIdx.x;
    const double thr = (double)n * 1.1920928955078125e-07 * lam[0];
    if (e < NP * KP) {
        int i = e / KP, m = e % KP;
        float out = 0.f;
        if (m < k) {
            double lm = lam[m];
            if (lm > thr && lm > 0.0) out = (float)(Y[(int64_t)i * NP + pos[m]] / sqrt(lm));
        }
        Mt[e] = out;
    }
    if (e == 0) {
        double f = 0.0;
        for (int r = frob_r0; r < frob_r1; ++r) f += diag0[r];
        acc[1] += f;
    }
}

static const size_t SOLVE_LDS = (size_t)(2 * 64 * LDA + 64) * sizeof(double);
static const size_t APPLY_LDS = (size_t)(3 * 64 * LDA) * sizeof(double);

hipError_t launch_eig(const EigWork& w, int NP, hipStream_t st) {
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute((const void*)jac_solve_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SOLVE_LDS);
        (void)hipFuncSetAttribute((const void*)jac_apply_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)APPLY_LDS);
        attr = true;
    }
    hipLaunchKernelGGL(jac_init_kernel, dim3(NP), dim3(256), 0, st, w.C, w.Y, w.diag0, w.stat, NP);
    const int np = NP / 64, nb = NP / 32;
    for (int sweep = 0; sweep < MAX_SWEEPS; ++sweep) {
        for (int s = 0; s < nb; ++s) {
            hipLaunchKernelGGL(jac_solve_kernel, dim3(np), dim3(256), SOLVE_LDS, st, w.C, w.Q, w.stat, NP, sweep, s);
            hipLaunchKernelGGL(jac_apply_kernel, dim3(2 * np * np), dim3(256), APPLY_LDS, st, w.C, w.Y, w.Q, w.stat, NP,
                               sweep, s);
        }
    }
    return hipGetLastError();
}

hipError_t launch_shrink_coeffs(const EigWork& w, int NP, int LP, int ell, int frob_r0, int frob_r1, float* Mt,
                                double* acc, hipStream_t st) {
    hipLaunchKernelGGL(eig_sort_kernel, dim3(1), dim3(512), 0, st, w.C, w.stat, w.pos, w.lam, NP, acc);
    hipLaunchKernelGGL(shrink_coeffs_kernel, dim3((NP * LP + 255) / 256), dim3(256), 0, st, w.Y, w.pos, w.lam, w.diag0,
                       NP, LP, ell, frob_r0, frob_r1, Mt, acc);
    return hipGetLastError();
}

hipError_t launch_basis_coeffs(const EigWork& w, int NP, int KP, int k, int n, int frob_r0, int frob_r1, float* Mt,
                               double* acc, hipStream_t st) {
    hipLaunchKernelGGL(eig_sort_kernel, dim3(1), dim3(512), 0, st, w.C, w.stat, w.pos, w.lam, NP, acc);
    hipLaunchKernelGGL(basis_coeffs_kernel, dim3((NP * KP + 255) / 256), dim3(256), 0, st, w.Y, w.pos, w.lam, w.diag0,
                       NP, KP, k, n, frob_r0, frob_r1, Mt, acc);
    return hipGetLastError();
}

}  // namespace sage
