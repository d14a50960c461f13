// Blocked two-sided Jacobi eigensolve of the (padded) Gram matrix, C = Y Lambda Y^T, in fp64, staged through
// LDS, and the coefficient matrices built from it.
//
// The shrink step (Method, FD paragraph) needs sigma_j^2 = lambda_j and, for the rebuild, the left singular
// vectors y_j of the buffer:  sigma_j v_j^T = y_j^T B.  The matrix is cut into 32x32 blocks. One sweep is:
//   step 0        every work-group takes two diagonal blocks and annihilates all pairs inside each block,
//   step 1..nb-1  round-robin over block pairs (I, J): annihilate every pair (p in I, q in J),
// so each off-diagonal element is rotated exactly once per sweep. A step is two kernels: a solve kernel runs the
// rotations of each 64x64 pivot sub-matrix in LDS and emits its accumulated 64x64 rotation Q_w; `apply`
// updates C <- Q^T C Q and Y <- Y Q with Q = blockdiag(Q_w) as 64x64x64 products on the fp64 matrix cores.
#include "sage_internal.h"

namespace sage {

constexpr int LDA = 65;  // padded leading dimension of the 64x64 LDS matrix of the solve kernels (doubles)

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

// stat[1 + s] = largest off-diagonal |c_pq| / trace(C) measured (jac_measure_kernel) just before sweep s. The solve
// is finished, and sweep s and all later ones do nothing, once that is <= tol.
__device__ __forceinline__ bool sweep_done(const double* stat, int sweep, double tol) {
    return stat[1 + sweep] <= tol;
}

__device__ __forceinline__ void atomic_max_pos_double(double* addr, double v) {
    // non-negative doubles order like their bit patterns
    atomicMax(reinterpret_cast<unsigned long long*>(addr), (unsigned long long)__double_as_longlong(v));
}

// Rotation [[c, s], [-s, c]] that annihilates a_pq of the symmetric 2x2 [[app, apq], [apq, aqq]] (the one of
// smaller angle): t = sign(a) apq / (|a| + sqrt(a^2 + apq^2)), a = (aqq - app)/2, c = 1/sqrt(1 + t^2), s = c t.
__device__ __forceinline__ void rot_params(double app, double aqq, double apq, double& c, double& s) {
    c = 1.0;
    s = 0.0;
    if (apq == 0.0) return;
    double a = 0.5 * (aqq - app);
    double den = fabs(a) + sqrt(a * a + apq * apq);
    if (!(den > 0.0)) return;
    double t = apq / den;
    if (a < 0.0) t = -t;
    c = 1.0 / sqrt(1.0 + t * t);
    s = c * t;
}

// Same rotation from the hardware reciprocal / reciprocal-square-root approximations, each polished by two Newton
// steps (the serial chain of a round starts here, so the IEEE division and square root are avoided). Also returns
// t = s/c, which gives the rotated diagonal in closed form: a_pp - t a_pq and a_qq + t a_pq.
__device__ __forceinline__ double rsqrt_newton(double x) {
    double y = __builtin_amdgcn_rsq(x);
    y = y * (1.5 - 0.5 * x * y * y);
    y = y * (1.5 - 0.5 * x * y * y);
    return y;
}
__device__ __forceinline__ void rot_params_fast(double app, double aqq, double apq, double& c, double& s, double& t) {
    c = 1.0;
    s = 0.0;
    t = 0.0;
    double a = 0.5 * (aqq - app);
    double h = a * a + apq * apq;
    if (apq == 0.0 || !(h > 1e-280) || !(h < 1e280)) return;  // nothing to rotate, or outside the safe range
    double den = fabs(a) + h * rsqrt_newton(h);
    double inv = __builtin_amdgcn_rcp(den);
    inv = inv * (2.0 - den * inv);
    inv = inv * (2.0 - den * inv);
    t = apq * inv;
    if (a < 0.0) t = -t;
    c = rsqrt_newton(1.0 + t * t);
    s = c * t;
}

// Y = I, diag0 = diag(C), stat[0] = trace(C), stat[1..] = 0. grid = NP blocks of 256.
__global__ __launch_bounds__(256) void jac_init_kernel(const double* __restrict__ C, double* __restrict__ Y,
                                                       double* __restrict__ diag0, double* __restrict__ stat, int NP,
                                                       int max_sweeps) {
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
        if (threadIdx.x == MAX_SWEEPS + 3) stat[MAX_SWEEPS + 3] = (double)max_sweeps;
    }
}

// all 16 global loads of a thread are issued before the first LDS store, so their latencies overlap
__device__ __forceinline__ void load_pivot(const double* __restrict__ C, int NP, int I, int J, double* A, int tid) {
    double v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        int e = u * 256 + tid;
        int r = e >> 6, c = e & 63;
        int gr = (r < 32 ? I * 32 + r : J * 32 + r - 32);
        int gc = (c < 32 ? I * 32 + c : J * 32 + c - 32);
        v[u] = C[(int64_t)gr * NP + gc];
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        int e = u * 256 + tid;
        A[(e >> 6) * LDA + (e & 63)] = v[u];
    }
}

// Before sweep `sweep`: stat[1 + sweep] = max off-diagonal |c_pq| / trace. One block per 16 matrix rows.
// Once a measurement is <= tol the later ones simply repeat it (the matrix no longer changes).
__global__ __launch_bounds__(256) void jac_measure_kernel(const double* __restrict__ C, double* __restrict__ stat, int NP,
                                                          int sweep, double tol) {
    if (sweep > 0 && stat[sweep] <= tol) return;  // stat[1 + sweep] stays 0 <= tol
    __shared__ double red[4];
    double mx = 0.0;
    for (int rr = 0; rr < 16; ++rr) {
        const int row = blockIdx.x * 16 + rr;
        for (int c = threadIdx.x; c < NP; c += 256)
            if (c != row) mx = fmax(mx, fabs(C[(int64_t)row * NP + c]));
    }
    for (int o = 32; o >= 1; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    double tr = stat[0];
    if (threadIdx.x == 0 && tr > 0.0) {
        mx = fmax(fmax(red[0], red[1]), fmax(red[2], red[3]));
        if (mx > 0.0) atomic_max_pos_double(&stat[1 + sweep], mx / tr);
    }
}

// Step 0 of a sweep: work-group w holds diagonal blocks 2w and 2w+1 as one 64x64 matrix and annihilates every pair
// inside each block (31 rounds of 16 + 16 disjoint rotations, round-robin inside a block). Q accumulates in LDS.
__global__ __launch_bounds__(256) void jac_diag_kernel(const double* __restrict__ C, double* __restrict__ Qout,
                                                       double* __restrict__ stat, int NP, int sweep, double tol) {
    if (sweep_done(stat, sweep, tol)) return;
    extern __shared__ double sm[];
    double* A = sm;              // 64 x LDA
    double* Qm = sm + 64 * LDA;  // 64 x LDA
    double* cs = Qm + 64 * LDA;  // 32 x 2
    const int tid = threadIdx.x;
    const int I = 2 * blockIdx.x, J = 2 * blockIdx.x + 1;
    load_pivot(C, NP, I, J, A, tid);
    for (int e = tid; e < 64 * 64; e += 256) Qm[(e >> 6) * LDA + (e & 63)] = ((e >> 6) == (e & 63)) ? 1.0 : 0.0;
    __syncthreads();

    for (int t = 0; t < 31; ++t) {
        if (tid < 32) {
            int p, q;
            rr_pair(32, t, tid & 15, p, q);
            if (tid >= 16) { p += 32; q += 32; }
            double c, s;
            rot_params(A[p * LDA + p], A[q * LDA + q], A[p * LDA + q], c, s);
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
            rr_pair(32, t, i & 15, pi, qi);
            if (i >= 16) { pi += 32; qi += 32; }
            rr_pair(32, t, j & 15, pj, qj);
            if (j >= 16) { pj += 32; qj += 32; }
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
            rr_pair(32, t, j & 15, pj, qj);
            if (j >= 16) { pj += 32; qj += 32; }
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

// Steps 1..nb-1: work-group w holds blocks (I, J) as one 64x64 matrix and annihilates every pair (p in I, q in J) in
// 32 rounds of 32 disjoint rotations. Index i = 4a + l of the first half (a < 8, l < 4) meets, in round
// (sigma, tau), index 4((a + tau) % 8) + (l + sigma) % 4 of the second half: a Latin square, so every pair is met
// once. A lives in LDS. Q lives in registers: a quad of lanes owns one row of Q, lane l of the quad holding the
// first-half columns {4a + l} and the second-half columns {32 + 4a' + (l + sigma) % 4}; with this schedule a round
// only rotates register pairs of one lane (static indices), and a change of sigma is a one-lane shift in the quad.
__global__ __launch_bounds__(256) void jac_cross_kernel(const double* __restrict__ C, double* __restrict__ Qout,
                                                        double* __restrict__ stat, int NP, int sweep, int st,
                                                        double tol) {
    if (sweep_done(stat, sweep, tol)) return;
    __shared__ double A[64 * LDA];
    __shared__ double cs[2][64];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nb = NP / 32;
    int I, J;
    block_pair(nb, st, blockIdx.x, I, J);
    load_pivot(C, NP, I, J, A, tid);

    const int qrow = wave * 16 + (lane >> 2), lq = lane & 3;
    double qa[8], qb[8];
#pragma unroll
    for (int a = 0; a < 8; ++a) {
        qa[a] = (qrow == 4 * a + lq) ? 1.0 : 0.0;
        qb[a] = (qrow == 32 + 4 * a + lq) ? 1.0 : 0.0;
    }
    __syncthreads();

    // the 496 pair-of-pairs (i < j) a round has to update are split statically: thread -> e = tid and e = 256 + tid
    int bi[2], bj[2];
    const bool second = (256 + tid) < 496;  // 16 threads have no second block
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        int e = u * 256 + tid, i = 0;
        if (e >= 496) e = 0;
        while (e >= 31 - i) { e -= 31 - i; ++i; }
        bi[u] = i;
        bj[u] = i + 1 + e;
    }

    for (int sigma = 0; sigma < 4; ++sigma) {
#pragma unroll
        for (int tau = 0; tau < 8; ++tau) {
            const int par = tau & 1;
            if (tid < 32) {
                // rotation of pair `tid`; its own 2x2 block has a closed form and nobody else touches it
                int p = tid;
                int q = 32 + ((((tid >> 2) + tau) & 7) << 2) + (((tid & 3) + sigma) & 3);
                double app = A[p * LDA + p], aqq = A[q * LDA + q], apq = A[p * LDA + q];
                double c, s, t;
                rot_params_fast(app, aqq, apq, c, s, t);
                cs[par][2 * tid] = c;
                cs[par][2 * tid + 1] = s;
                if (s != 0.0) {
                    A[p * LDA + p] = app - t * apq;
                    A[q * LDA + q] = aqq + t * apq;
                    A[p * LDA + q] = 0.0;
                    A[q * LDA + p] = 0.0;
                }
            }
            __syncthreads();
            // 2x2 blocks of A for pairs i < j: X <- R_i^T X R_j, written to (i, j) and mirrored to (j, i)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if (u == 1 && !second) continue;
                const int i = bi[u], j = bj[u];
                int pi = i, qi = 32 + ((((i >> 2) + tau) & 7) << 2) + (((i & 3) + sigma) & 3);
                int pj = j, qj = 32 + ((((j >> 2) + tau) & 7) << 2) + (((j & 3) + sigma) & 3);
                double ci = cs[par][2 * i], si = cs[par][2 * i + 1], cj = cs[par][2 * j], sj = cs[par][2 * j + 1];
                // only the upper triangle is kept current: (qi, pj) lives at (pj, qi), (qi, qj) at (min, max)
                const int o00 = pi * LDA + pj, o01 = pi * LDA + qj, o10 = pj * LDA + qi;
                const int o11 = qi < qj ? qi * LDA + qj : qj * LDA + qi;
                double x00 = A[o00], x01 = A[o01], x10 = A[o10], x11 = A[o11];
                double y00 = ci * x00 - si * x10, y01 = ci * x01 - si * x11;
                double y10 = si * x00 + ci * x10, y11 = si * x01 + ci * x11;
                A[o00] = cj * y00 - sj * y01;
                A[o01] = sj * y00 + cj * y01;
                A[o10] = cj * y10 - sj * y11;
                A[o11] = sj * y10 + cj * y11;
            }
            // Q <- Q R: register pairs (qa[a], qb[(a + tau) % 8]) of pair index i = 4a + lq
#pragma unroll
            for (int a = 0; a < 8; ++a) {
                const int i = 4 * a + lq;
                double c = cs[par][2 * i], s = cs[par][2 * i + 1];
                double x = qa[a], y = qb[(a + tau) & 7];
                qa[a] = c * x - s * y;
                qb[(a + tau) & 7] = s * x + c * y;
            }
            __syncthreads();
        }
        if (sigma < 3) {
            const int src = (lane & ~3) | ((lane + 1) & 3);
#pragma unroll
            for (int a = 0; a < 8; ++a) qb[a] = __shfl(qb[a], src);
        }
    }
    double* Qo = Qout + (int64_t)blockIdx.x * 4096 + qrow * 64;
#pragma unroll
    for (int a = 0; a < 8; ++a) {
        Qo[4 * a + lq] = qa[a];
        Qo[32 + 4 * a + ((lq + 3) & 3)] = qb[a];
    }
}

typedef double f64x4 __attribute__((ext_vector_type(4)));
constexpr int LDX = 68;  // leading dimension of an LDS matrix read as the row operand   (lane -> row l%16, k l/16)
constexpr int LDQ = 72;  // leading dimension of an LDS matrix read as the column operand (lane -> k l/16, col l%16)
constexpr int LDQB = 40; // the same for the 32-column half of Q_b (keeps the kernel's LDS under 96 KB, so that it fits
                         // on a CU beside one work-group of the Gram kernel running on the side stream)

// fp64 matrix-core step acc(16x16) += a(16x4) b(4x16): lane l supplies a[l%16][l/16] and b[l/16][l%16];
// acc element v of lane l is row 4v + l/16, column l%16.
__device__ __forceinline__ f64x4 mfma64(double a, double b, f64x4 acc) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
}

// grid = 4 * np^2 (np = NP/64 pairs): block -> (kind, tile (a, b), column half h). C tiles: out(a, b)[:, h] =
// Q_a^T (C(a, b) Q_b[:, h]); Y tiles: out(a, b)[:, h] = Y(a, b) Q_b[:, h]. Reads `in`, writes `out` (ping-pong), so
// the two halves of a tile never race. A wave owns 16 rows of the 64x32 result (2 accumulator tiles).
__global__ __launch_bounds__(256) void jac_apply_kernel(const double* __restrict__ Cin, double* __restrict__ Cout,
                                                        const double* __restrict__ Yin, double* __restrict__ Yout,
                                                        const double* __restrict__ Q, const double* __restrict__ stat,
                                                        int NP, int sweep, int st, double tol) {
    if (sweep_done(stat, sweep, tol)) return;
    extern __shared__ double sm[];
    double* X = sm;                // 64 x LDX
    double* Qb = sm + 64 * LDX;    // 64 x LDQB (32 columns), later T = X Q_b[:, h]
    double* Qa = Qb + 64 * LDQB;   // 64 x LDQ
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int np = NP / 64, nb = NP / 32;
    const int half = blockIdx.x & 1;
    int bid = blockIdx.x >> 1;
    const bool isY = bid >= np * np;
    if (isY) bid -= np * np;
    const int a = bid / np, b = bid % np;
    int Ia, Ja, Ib, Jb;
    block_pair(nb, st, a, Ia, Ja);
    block_pair(nb, st, b, Ib, Jb);
    const double* Min = isY ? Yin : Cin;
    double* Mout = isY ? Yout : Cout;

    {   // issue every global load before the first LDS store
        double vx[16], va[16], vb[8];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            int e = u * 256 + tid;
            int r = e >> 6, c = e & 63;
            int gr = isY ? (a * 64 + r) : (r < 32 ? Ia * 32 + r : Ja * 32 + r - 32);
            int gc = (c < 32 ? Ib * 32 + c : Jb * 32 + c - 32);
            vx[u] = Min[(int64_t)gr * NP + gc];
            va[u] = isY ? 0.0 : Q[(int64_t)a * 4096 + e];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            int e = u * 256 + tid;
            vb[u] = Q[(int64_t)b * 4096 + (e >> 5) * 64 + half * 32 + (e & 31)];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            int e = u * 256 + tid;
            X[(e >> 6) * LDX + (e & 63)] = vx[u];
            if (!isY) Qa[(e >> 6) * LDQ + (e & 63)] = va[u];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            int e = u * 256 + tid;
            Qb[(e >> 5) * LDQB + (e & 31)] = vb[u];
        }
    }
    __syncthreads();
    const int l16 = lane & 15, lk = lane >> 4, i0 = wave * 16;
    f64x4 acc[2];
#pragma unroll
    for (int jt = 0; jt < 2; ++jt) acc[jt] = f64x4{0.0, 0.0, 0.0, 0.0};
    for (int k0 = 0; k0 < 64; k0 += 4) {  // T = X Q_b[:, h]
        double av = X[(i0 + l16) * LDX + k0 + lk];
#pragma unroll
        for (int jt = 0; jt < 2; ++jt) acc[jt] = mfma64(av, Qb[(k0 + lk) * LDQB + jt * 16 + l16], acc[jt]);
    }
    if (!isY) {
        __syncthreads();  // everyone is done reading Q_b
#pragma unroll
        for (int jt = 0; jt < 2; ++jt)
#pragma unroll
            for (int v = 0; v < 4; ++v) Qb[(i0 + 4 * v + lk) * LDQB + jt * 16 + l16] = acc[jt][v];
        __syncthreads();
#pragma unroll
        for (int jt = 0; jt < 2; ++jt) acc[jt] = f64x4{0.0, 0.0, 0.0, 0.0};
        for (int k0 = 0; k0 < 64; k0 += 4) {  // Q_a^T T
            double av = Qa[(k0 + lk) * LDQ + i0 + l16];
#pragma unroll
            for (int jt = 0; jt < 2; ++jt) acc[jt] = mfma64(av, Qb[(k0 + lk) * LDQB + jt * 16 + l16], acc[jt]);
        }
    }
    const int gcb = (half == 0 ? Ib : Jb) * 32;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        int r = i0 + 4 * v + lk;
        int gr = isY ? (a * 64 + r) : (r < 32 ? Ia * 32 + r : Ja * 32 + r - 32);
#pragma unroll
        for (int jt = 0; jt < 2; ++jt) Mout[(int64_t)gr * NP + gcb + jt * 16 + l16] = acc[jt][v];
    }
}

// Eigenvalues = diagonal of the rotated C, clamped at 0; rank by counting (ties: lower column first).
// One work-group of 512 threads. Also records the sweeps that were needed in acc[3].
__global__ __launch_bounds__(512) void eig_sort_kernel(const double* __restrict__ C, const double* __restrict__ stat,
                                                       int* __restrict__ pos, double* __restrict__ lam, int NP,
                                                       double* __restrict__ acc, double tol) {
    // stat[17] holds the number of sweeps that were launched (written by jac_init_kernel)
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
        const int launched = (int)stat[MAX_SWEEPS + 3];
        int used = launched + SWEEPS_NOT_CONVERGED;  // the measurement after the last launched sweep was still > tol
        for (int s = 0; s <= launched && s <= MAX_SWEEPS; ++s)
            if (stat[1 + s] <= tol) { used = s; break; }
        acc[3] = (double)used;
    }
}

// Shrink coefficients (Method, FD paragraph: delta = sigma_ell^2, Sigma'_jj = sqrt(max(sigma_j^2 - delta, 0))):
// new row m = w_m * y_m^T B with w_m = sqrt(max(lambda_m - delta, 0) / lambda_m); stored in coeff_offset order.
__global__ __launch_bounds__(256) void shrink_coeffs_kernel(const double* __restrict__ Y, const int* __restrict__ pos,
                                                            const double* __restrict__ lam,
                                                            const double* __restrict__ diag0, int NP, int LP, int ell,
                                                            int ra0, int ra1, int rb0, int rb1,
                                                            float* __restrict__ Mt, double* __restrict__ acc,
                                                            double* __restrict__ known) {
    int e = blockIdx.x * 256 + threadIdx.x;
    const double delta = lam[ell - 1];
    if (e < NP) {  // squared norm of new row e: w_e^2 lambda_e
        double keep = e < ell ? lam[e] - delta : 0.0;
        known[e] = keep > 0.0 ? keep : 0.0;
    }
    if (e < NP * LP) {
        int i = e / LP, m = e % LP;
        double lm = lam[m];
        double keep = lm - delta;
        double w = (keep > 0.0 && lm > 0.0) ? sqrt(keep / lm) : 0.0;
        Mt[coeff_offset(i, m, LP)] = (w > 0.0) ? (float)(w * Y[(int64_t)i * NP + pos[m]]) : 0.f;
    }
    if (e == 0) {
        acc[0] += delta;
        acc[2] = delta;
        double f = 0.0;
        for (int r = ra0; r < ra1; ++r) f += diag0[r];
        for (int r = rb0; r < rb1; ++r) f += diag0[r];
        acc[1] += f;
    }
}

// Basis coefficients: v_m^T = y_m^T B / sqrt(lambda_m) for m < k, or 0 when lambda_m <= n 2^-23 lambda_1.
// weighted: the row is scaled by sqrt(max(lambda_m - delta, 0)) with delta = lambda_ell, which makes it the m-th row of
// the sketch a shrink of the buffer would write (the paper's own projection z = S g, "Two-pass scoring").
__global__ __launch_bounds__(256) void basis_coeffs_kernel(const double* __restrict__ Y, const int* __restrict__ pos,
                                                           const double* __restrict__ lam,
                                                           const double* __restrict__ diag0, int NP, int KP, int k, int n,
                                                           int ell, int weighted, int ra0, int ra1, int rb0, int rb1,
                                                           float* __restrict__ Mt, double* __restrict__ acc) {
    int e = blockIdx.x * 256 + threadIdx.x;
    const double thr = (double)n * 1.1920928955078125e-07 * lam[0];
    const double delta = lam[ell - 1];
    if (e < NP * KP) {
        int i = e / KP, m = e % KP;
        float out = 0.f;
        if (m < k) {
            double lm = lam[m];
            if (lm > thr && lm > 0.0) {
                double f = 1.0 / sqrt(lm);
                if (weighted) f = lm - delta > 0.0 ? sqrt((lm - delta) / lm) : 0.0;
                out = (float)(Y[(int64_t)i * NP + pos[m]] * f);
            }
        }
        Mt[coeff_offset(i, m, KP)] = out;
    }
    if (e == 0) {
        double f = 0.0;
        for (int r = ra0; r < ra1; ++r) f += diag0[r];
        for (int r = rb0; r < rb1; ++r) f += diag0[r];
        acc[1] += f;
    }
}

static const size_t DIAG_LDS = (size_t)(2 * 64 * LDA + 64) * sizeof(double);
static const size_t APPLY_LDS = (size_t)(64 * LDX + 64 * LDQB + 64 * LDQ) * sizeof(double);

hipError_t launch_eig(const EigWork& w, int NP, double tol, int max_sweeps, hipStream_t st) {
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute((const void*)jac_diag_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)DIAG_LDS);
        (void)hipFuncSetAttribute((const void*)jac_apply_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)APPLY_LDS);
        attr = true;
    }
    if (max_sweeps > MAX_SWEEPS) max_sweeps = MAX_SWEEPS;
    if (max_sweeps < 1) max_sweeps = 1;
    hipLaunchKernelGGL(jac_init_kernel, dim3(NP), dim3(256), 0, st, w.C, w.Y, w.diag0, w.stat, NP, max_sweeps);
    const int np = NP / 64, nb = NP / 32;
    // nb is even, so every sweep starts and ends on buffer 0: that is where the result is, whenever it converged
    double* Cb[2] = {w.C, w.C2};
    double* Yb[2] = {w.Y, w.Y2};
    for (int sweep = 0; sweep < max_sweeps; ++sweep) {
        hipLaunchKernelGGL(jac_measure_kernel, dim3(NP / 16), dim3(256), 0, st, w.C, w.stat, NP, sweep, tol);
        for (int s = 0; s < nb; ++s) {
            const int cur = s & 1;
            if (s == 0)
                hipLaunchKernelGGL(jac_diag_kernel, dim3(np), dim3(256), DIAG_LDS, st, Cb[cur], w.Q, w.stat, NP, sweep, tol);
            else
                hipLaunchKernelGGL(jac_cross_kernel, dim3(np), dim3(256), 0, st, Cb[cur], w.Q, w.stat, NP, sweep, s, tol);
            hipLaunchKernelGGL(jac_apply_kernel, dim3(4 * np * np), dim3(256), APPLY_LDS, st, Cb[cur], Cb[cur ^ 1], Yb[cur],
                               Yb[cur ^ 1], w.Q, w.stat, NP, sweep, s, tol);
        }
    }
    // what the last launched sweep left: eig_sort_kernel tells a converged solve from one that ran out of sweeps
    hipLaunchKernelGGL(jac_measure_kernel, dim3(NP / 16), dim3(256), 0, st, w.C, w.stat, NP, max_sweeps, tol);
    return hipGetLastError();
}

hipError_t launch_shrink_coeffs(const EigWork& w, int NP, int LP, int ell, int ra0, int ra1, int rb0, int rb1, float* Mt,
                                double* acc, double tol, hipStream_t st) {
    hipLaunchKernelGGL(eig_sort_kernel, dim3(1), dim3(512), 0, st, w.C, w.stat, w.pos, w.lam, NP, acc, tol);
    hipLaunchKernelGGL(shrink_coeffs_kernel, dim3((NP * LP + 255) / 256), dim3(256), 0, st, w.Y, w.pos, w.lam, w.diag0,
                       NP, LP, ell, ra0, ra1, rb0, rb1, Mt, acc, w.known);
    return hipGetLastError();
}

hipError_t launch_basis_coeffs(const EigWork& w, int NP, int KP, int k, int n, int ell, bool weighted, int ra0, int ra1,
                               int rb0, int rb1, float* Mt, double* acc, double tol, hipStream_t st) {
    hipLaunchKernelGGL(eig_sort_kernel, dim3(1), dim3(512), 0, st, w.C, w.stat, w.pos, w.lam, NP, acc, tol);
    hipLaunchKernelGGL(basis_coeffs_kernel, dim3((NP * KP + 255) / 256), dim3(256), 0, st, w.Y, w.pos, w.lam, w.diag0,
                       NP, KP, k, n, ell, weighted ? 1 : 0, ra0, ra1, rb0, rb1, Mt, acc);
    return hipGetLastError();
}

}  // namespace sage
