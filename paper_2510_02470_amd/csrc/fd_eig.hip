// Blocked two-sided Jacobi eigensolve of the (padded) Gram matrix, C = Y Lambda Y^T, in fp64, staged through
// LDS, and the coefficient matrices built from it.
//
// The shrink step (Method, FD paragraph) needs sigma_j^2 = lambda_j and, for the rebuild, the left singular
// vectors y_j of the buffer:  sigma_j v_j^T = y_j^T B.  The matrix is cut into 32x32 blocks. One sweep is nb - 1 steps;
// step st pairs the blocks round-robin (I, J) and annihilates every pair (p in I, q in J); step 1, whose pairs cover
// every block once, first annihilates the pairs inside I and inside J. So each off-diagonal element is rotated
// exactly once per sweep. A step is two kernels: `pivot` runs the rotations of each 64x64 pivot sub-matrix in LDS
// and emits its accumulated 64x64 rotation Q_w; `apply` updates C <- Q^T C Q and Y <- Y Q with Q = blockdiag(Q_w) as
// 64x64x64 products on the fp64 matrix cores (ping-pong between two copies of C and Y).
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
    rr_pair(nb, st - 1, w, I, J);  // st = 1 .. nb - 1
}

// stat[1 + s] = largest off-diagonal |c_pq| / trace(C) of the matrix sweep s starts from (written by
// jac_measure_kernel for s = 0, by the last jac_apply_kernel of sweep s - 1 otherwise). The solve is finished, and
// sweep s and all later ones do nothing, once that is <= tol.
__device__ __forceinline__ bool sweep_done(const double* stat, int sweep, double tol) {
    return stat[1 + sweep] <= tol;
}

__device__ __forceinline__ void atomic_max_pos_double(double* addr, double v) {
    // non-negative doubles order like their bit patterns
    atomicMax(reinterpret_cast<unsigned long long*>(addr), (unsigned long long)__double_as_longlong(v));
}

// Rotation [[c, s], [-s, c]] that annihilates a_pq of the symmetric 2x2 [[app, apq], [apq, aqq]] (the one of
// smaller angle): t = sign(a) apq / (|a| + sqrt(a^2 + apq^2)), a = (aqq - app)/2, c = 1/sqrt(1 + t^2), s = c t.
// The angle is taken in single precision and the normalisation in double precision. The pivot solve only has to
// produce an orthogonal Q that makes the pivot block nearly diagonal: the matrix itself is updated from Q in fp64 by
// jac_apply_kernel, so an angle that is good to ~2^-22 leaves a pivot element that is ~1e-7 of what it was (instead
// of 0), which the next sweep removes; c^2 + s^2 = 1 holds to fp64 rounding because c = 1/sqrt(1 + t^2) is polished
// by two Newton steps in fp64 and s = c t. The inputs are first scaled by 2^-e with 2^e >= trace(C) >= every |c_pq|,
// so they fit single precision; what underflows there is below 1e-19 trace and no longer matters (such a rotation
// is still orthogonal, it just need not annihilate anything). Branch-free, so that the scheduler can fill the waits
// of this serial chain with other work of the same wave. t is returned for the closed forms a_pp - t a_pq and
// a_qq + t a_pq.
__device__ __forceinline__ void rot_params_mixed(double app, double aqq, double apq, int e, double& c, double& s,
                                                 double& t) {
    const double a = 0.5 * (aqq - app);
    const float af = (float)__builtin_amdgcn_ldexp(a, -e), pf = (float)__builtin_amdgcn_ldexp(apq, -e);
    const float den = fabsf(af) + __builtin_amdgcn_sqrtf(af * af + pf * pf) + 1e-30f;
    float tf = pf * __builtin_amdgcn_rcpf(den);  // pf = 0 (nothing to rotate, or negligible): the identity
    if (a < 0.0) tf = -tf;
    t = (double)tf;
    const double x = __builtin_fma(t, t, 1.0);
    double y = (double)__builtin_amdgcn_rsqf((float)x);
    y = y * (1.5 - 0.5 * x * y * y);
    y = y * (1.5 - 0.5 * x * y * y);
    c = y;
    s = y * t;
}
// exponent for rot_params_mixed from trace(C) = stat[0]
__device__ __forceinline__ int scale_exponent(double trace) {
    return (trace > 1e-280 && trace < 1e280) ? __builtin_amdgcn_frexp_exp(trace) : 0;
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

// stat[1] = max off-diagonal |c_pq| / trace of the matrix as given (the record before sweep 0; the later records are
// written by the last jac_apply_kernel of each sweep). One block per 16 matrix rows.
__global__ __launch_bounds__(256) void jac_measure_kernel(const double* __restrict__ C, double* __restrict__ stat, int NP) {
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
        if (mx > 0.0) atomic_max_pos_double(&stat[1], mx / tr);
    }
}

// After the last sweep: a sweep is nb - 1 steps, an odd number, so after an odd number of executed sweeps the result
// sits in the second copies of C and Y; bring it to the first. The number of executed sweeps is the first record
// <= tol, or all that were launched.
__global__ __launch_bounds__(256) void jac_finish_kernel(double* __restrict__ C, const double* __restrict__ C2,
                                                         double* __restrict__ Y, const double* __restrict__ Y2,
                                                         const double* __restrict__ stat, int NP, double tol) {
    const int launched = (int)stat[MAX_SWEEPS + 3];
    int executed = launched;
    for (int s = 0; s < launched; ++s)
        if (stat[1 + s] <= tol) { executed = s; break; }
    if (!(executed & 1)) return;
    const int row = blockIdx.x;
    for (int c = threadIdx.x; c < NP; c += 256) {
        C[(int64_t)row * NP + c] = C2[(int64_t)row * NP + c];
        Y[(int64_t)row * NP + c] = Y2[(int64_t)row * NP + c];
    }
}

// Steps 1..nb-1: work-group w holds blocks (I, J) as one 64x64 matrix A (LDS, upper triangle kept current) and
// annihilates every pair (p in I, q in J) in 32 rounds of 32 disjoint rotations. Rotation iota = 16 b + x keeps
// p = iota and meets, in round r = 16 beta + rho, q = 32 + 16 (b ^ beta) + (x + rho) % 16: a Latin square, so every
// pair is met once.
//
// A round updates, for every two rotations i < j, the 2x2 block rows {p_i, q_i} x columns {p_j, q_j}: 496 blocks,
// one per thread of the 512. The block of rotations (iota, iota') with iota' = 16 b + (x + 1) % 16 holds the
// element (p_iota, q_iota') that rotation iota annihilates in the next round, so the thread that has just updated it
// goes on to compute the next rotation (the diagonal after this round's rotation is known in closed form) and
// publishes it for the next round: one barrier per round. Those 32 blocks, and the 32 that play this part at the
// change of beta, belong to wave 0, which has nothing else to do: the round's serial chain is one LDS round trip,
// a block update and a rotation. The other 432 blocks are dealt in row-major order to waves 1..7, so that
// consecutive lanes hold one i and consecutive j: their LDS accesses are rows or columns of A with distinct banks
// (LDA is odd), and (c_i, s_i) is a broadcast.
//
// Q lives in registers: a thread owns 4 rows of column p_iota and of the column q that iota currently meets. A round
// rotates those 4 register pairs with one (c, s); then the q columns move one lane down inside their 16 lanes (a
// DPP row rotation), plus a swap of the two 16-lane halves at the change of beta.
constexpr int cross_q(int iota, int r) { return 32 + ((((iota >> 4) ^ (r >> 4)) & 1) << 4) + ((iota + r) & 15); }

struct CrossTable {
    unsigned short e[512];  // [thread]: i | j << 5 | kind << 10 | valid << 12
};
// kind 1: the block's element (p_i, q_j) is the next pivot of rotation i; kind 2: (p_j, q_i) is that of rotation j
constexpr CrossTable make_cross_table() {
    CrossTable t{};
    bool special[32][32] = {};
    for (int half = 0; half < 2; ++half)  // half 0: ordinary rounds; half 1: the round before beta changes
        for (int iota = 0; iota < 32; ++iota) {
            const int b = iota >> 4, x = iota & 15;
            const int other = ((half ? b ^ 1 : b) << 4) + ((x + 1) & 15);
            const int i = iota < other ? iota : other, j = iota < other ? other : iota;
            const int kind = iota < other ? 1 : 2;
            t.e[32 * half + iota] = (unsigned short)(i | j << 5 | kind << 10 | 1 << 12);
            special[i][j] = true;
        }
    int k = 64;
    for (int i = 0; i < 32; ++i)
        for (int j = i + 1; j < 32; ++j)
            if (!special[i][j]) t.e[k++] = (unsigned short)(i | j << 5 | 1 << 12);
    return t;  // k == 496: the last 16 threads have no block
}
__device__ const CrossTable cross_table = make_cross_table();

__device__ __forceinline__ double dpp_row_ror15(double v) {  // lane l of a 16-lane row receives lane (l + 1) % 16
    const long long u = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_mov_dpp((int)u, 0x12F, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_mov_dpp((int)(u >> 32), 0x12F, 0xF, 0xF, false);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

__global__ __launch_bounds__(512) void jac_pivot_kernel(const double* __restrict__ C, double* __restrict__ Qout,
                                                        double* __restrict__ stat, int NP, int sweep, int st,
                                                        double tol) {
    extern __shared__ double dyn[];  // two copies of the pivot matrix, 64 x LDA each (the launch asks for more: see launch_eig)
    __shared__ __attribute__((aligned(16))) double cs[2][64];
    double* const A = dyn;             // the pair phase works in place here
    double* const A1 = dyn + 64 * LDA; // the within-block phase goes back and forth between A1 and A
    const bool within = st == 1;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nb = NP / 32;
    int I, J;
    block_pair(nb, st, blockIdx.x, I, J);
    // the pivot block is requested before the convergence record is looked at: one memory round trip, not two
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int e = u * 512 + tid;
        const int r = e >> 6, c = e & 63;
        const int gr = (r < 32 ? I * 32 + r : J * 32 + r - 32);
        const int gc = (c < 32 ? I * 32 + c : J * 32 + c - 32);
        v[u] = C[(int64_t)gr * NP + gc];
    }
    const unsigned ent = cross_table.e[tid];
    const double trace = stat[0];
    if (sweep_done(stat, sweep, tol)) return;
    const int sexp = scale_exponent(trace);
    {
        double* const Ain = within ? A1 : A;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int e = u * 512 + tid;
            Ain[(e >> 6) * LDA + (e & 63)] = v[u];
        }
    }
    const int i = ent & 31, j = (ent >> 5) & 31, kind = (ent >> 10) & 3;
    const bool valid = ((ent >> 12) & 1) != 0;

    const int iota = tid & 31, row0 = 4 * (tid >> 5);
    double qp[4], qq[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        qp[k] = (row0 + k == iota) ? 1.0 : 0.0;
        qq[k] = (row0 + k == 32 + iota) ? 1.0 : 0.0;
    }
    __syncthreads();

    if (within) {
        // ---- pairs inside block I and inside block J: 31 rounds, round t pairs index x with x ^ t (same block).
        // Rotation rho = 16 * block + r: its p is r with a zero inserted at the top bit of t, q = p ^ t. The same
        // 496 blocks of rotation pairs as below, one per thread, but read from one copy of the matrix and written
        // to the other, so that lane rho of wave 0 can, in the same round, work out the element its rotation
        // annihilates next (it recomputes that one element of whatever block holds it), the rotation, and the
        // diagonal after it. Lane rho also writes this round's pivot (0 once rotated) and the two diagonal entries:
        // every entry of the upper triangle is written exactly once per round. Q columns stay with their lanes:
        // lane iota owns columns iota and 32 + iota and fetches the partner columns from lane iota ^ t.
        if (tid < 32) {  // rotations of round 1
            const int p = 32 * (tid >> 4) + 2 * (tid & 15), q = p + 1;
            const double app = A1[p * LDA + p], aqq = A1[q * LDA + q], apq = A1[p * LDA + q];
            double c, s, t;
            rot_params_mixed(app, aqq, apq, sexp, c, s, t);
            cs[1][2 * tid] = c;
            cs[1][2 * tid + 1] = s;
            A1[p * LDA + p] = app - t * apq;
            A1[q * LDA + q] = aqq + t * apq;
        }
        __syncthreads();
        for (int t = 1; t < 32; ++t) {
            const int par = t & 1;
            const double* const R = par ? A1 : A;
            double* const W = par ? A : A1;
            const int hb = 31 - __builtin_clz(t);
            const int lowm = (1 << hb) - 1;
            auto p_of = [&](int rho) { return 32 * (rho >> 4) + ((((rho & 15) >> hb) << (hb + 1)) | (rho & lowm)); };
            auto up = [&](int r, int c) { return r < c ? r * LDA + c : c * LDA + r; };
            if (tid < 32) {
                const int rho = tid;
                const int p = p_of(rho), q = p ^ t;
                const double s_cur = cs[par][2 * rho + 1];
                const double piv = R[p * LDA + q];
                if (t < 31) {
                    const int t2 = t + 1, hb2 = 31 - __builtin_clz(t2);
                    const int p2 = 32 * (rho >> 4) + ((((rho & 15) >> hb2) << (hb2 + 1)) | (rho & ((1 << hb2) - 1)));
                    const int q2 = p2 ^ t2;
                    // rotations of this round that hold p2 and q2
                    auto rot_of = [&](int x) {
                        const int y = x & 31, m = y < (y ^ t) ? y : (y ^ t);
                        return 16 * (x >> 5) + (((m >> (hb + 1)) << hb) | (m & lowm));
                    };
                    const int ri = rot_of(p2), rj = rot_of(q2);
                    const int Pi = p_of(ri), Qi = Pi ^ t, Pj = p_of(rj), Qj = Pj ^ t;
                    const double ci = cs[par][2 * ri], si = cs[par][2 * ri + 1];
                    const double cj = cs[par][2 * rj], sj = cs[par][2 * rj + 1];
                    const double x00 = R[up(Pi, Pj)], x01 = R[up(Pi, Qj)], x10 = R[up(Qi, Pj)], x11 = R[up(Qi, Qj)];
                    const double app = R[p2 * LDA + p2], aqq = R[q2 * LDA + q2];
                    const bool urow = p2 != Pi, vcol = q2 != Pj;
                    const double y0 = urow ? si * x00 + ci * x10 : ci * x00 - si * x10;
                    const double y1 = urow ? si * x01 + ci * x11 : ci * x01 - si * x11;
                    const double z = vcol ? sj * y0 + cj * y1 : cj * y0 - sj * y1;
                    double c, s, tt;
                    rot_params_mixed(app, aqq, z, sexp, c, s, tt);
                    cs[par ^ 1][2 * rho] = c;
                    cs[par ^ 1][2 * rho + 1] = s;
                    W[p2 * LDA + p2] = app - tt * z;
                    W[q2 * LDA + q2] = aqq + tt * z;
                } else {
                    W[p * LDA + p] = R[p * LDA + p];
                    W[q * LDA + q] = R[q * LDA + q];
                }
                W[p * LDA + q] = s_cur != 0.0 ? 0.0 : piv;
            }
            {   // this thread's block of rotations (i, j)
                const int Pi = p_of(i), Qi = Pi ^ t, Pj = p_of(j), Qj = Pj ^ t;
                const int o00 = up(Pi, Pj), o01 = up(Pi, Qj), o10 = up(Qi, Pj), o11 = up(Qi, Qj);
                const double ci = cs[par][2 * i], si = cs[par][2 * i + 1], cj = cs[par][2 * j], sj = cs[par][2 * j + 1];
                const double x00 = R[o00], x01 = R[o01], x10 = R[o10], x11 = R[o11];
                const double y00 = ci * x00 - si * x10, y01 = ci * x01 - si * x11;
                const double y10 = si * x00 + ci * x10, y11 = si * x01 + ci * x11;
                if (valid) {
                    W[o00] = cj * y00 - sj * y01;
                    W[o01] = sj * y00 + cj * y01;
                    W[o10] = cj * y10 - sj * y11;
                    W[o11] = sj * y10 + cj * y11;
                }
            }
            {   // Q: columns iota (block I) and 32 + iota (block J) against those of lane iota ^ t
                const int mate = iota ^ t, m = iota < mate ? iota : mate;
                const int rr = ((m >> (hb + 1)) << hb) | (m & lowm);
                const double c0 = cs[par][2 * rr], s0 = cs[par][2 * rr + 1];
                const double c1 = cs[par][2 * (16 + rr)], s1 = cs[par][2 * (16 + rr) + 1];
                const bool first = iota < mate;  // this lane holds the pair's p
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const double op = __shfl_xor(qp[k], t), oq = __shfl_xor(qq[k], t);
                    qp[k] = first ? c0 * qp[k] - s0 * op : s0 * op + c0 * qp[k];
                    qq[k] = first ? c1 * qq[k] - s1 * oq : s1 * oq + c1 * qq[k];
                }
            }
            __syncthreads();
        }
        // 31 rounds from A1 end in A
    }

    // ---- pairs (p in I, q in J)
    if (tid < 32) {  // rotations of round 0: p = tid meets q = 32 + tid
        const int p = tid, q = 32 + tid;
        const double app = A[p * LDA + p], aqq = A[q * LDA + q], apq = A[p * LDA + q];
        double c, s, t;
        rot_params_mixed(app, aqq, apq, sexp, c, s, t);
        cs[0][2 * tid] = c;
        cs[0][2 * tid + 1] = s;
        if (s != 0.0) {
            A[p * LDA + p] = app - t * apq;
            A[q * LDA + q] = aqq + t * apq;
            A[p * LDA + q] = 0.0;
        }
    }
    // LDS offsets of this thread's block in round r; they are worked out before the barrier that opens the round
    const int o00 = i * LDA + j;
    int o01, o10, o11, od0, od1;
    auto offsets = [&](int r) {
        const int qi = cross_q(i, r), qj = cross_q(j, r);
        o01 = i * LDA + qj;
        o10 = j * LDA + qi;
        o11 = qi < qj ? qi * LDA + qj : qj * LDA + qi;
        const int rot = kind == 1 ? i : j, qn = kind == 1 ? qj : qi;  // wave 0: next round's rotation rot meets qn
        od0 = rot * (LDA + 1);
        od1 = qn * (LDA + 1);
    };
    offsets(0);
    const int csn = 2 * (kind == 1 ? i : j);
    __syncthreads();

    // Q <- Q R for this thread's column pair, then the q columns move on to the rotation that meets them next
    auto q_update = [&](int r, double qc, double qs) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const double x = qp[k], y = qq[k];
            qp[k] = qc * x - qs * y;
            qq[k] = qs * x + qc * y;
        }
        if (r < 31) {
#pragma unroll
            for (int k = 0; k < 4; ++k) qq[k] = dpp_row_ror15(qq[k]);
            if (r == 15) {
#pragma unroll
                for (int k = 0; k < 4; ++k) qq[k] = __shfl_xor(qq[k], 16);
            }
        }
    };

    for (int r = 0; r < 32; ++r) {
        const int par = r & 1;
        if (wave == 0) {
            // the serial chain of the round: block update, then next round's rotation from the fresh pivot
            const double ci = cs[par][2 * i], si = cs[par][2 * i + 1], cj = cs[par][2 * j], sj = cs[par][2 * j + 1];
            const double x00 = A[o00], x01 = A[o01], x10 = A[o10], x11 = A[o11];
            const double app = A[od0], aqq = A[od1];
            const double qc = cs[par][2 * iota], qs = cs[par][2 * iota + 1];
            const double y00 = ci * x00 - si * x10, y01 = ci * x01 - si * x11;
            const double y10 = si * x00 + ci * x10, y11 = si * x01 + ci * x11;
            double z01 = sj * y00 + cj * y01, z10 = cj * y10 - sj * y11;
            const double z00 = cj * y00 - sj * y01, z11 = sj * y10 + cj * y11;
            const bool act = r != 31 && ((r == 15) == (lane >= 32));  // lanes 0..31: ordinary rounds; 32..63: beta changes
            const double apq = kind == 1 ? z01 : z10;
            double c, s, t;
            rot_params_mixed(app, aqq, apq, sexp, c, s, t);
            if (act) {
                cs[par ^ 1][csn] = c;
                cs[par ^ 1][csn + 1] = s;
                if (s != 0.0) {
                    A[od0] = app - t * apq;
                    A[od1] = aqq + t * apq;
                    if (kind == 1) z01 = 0.0;
                    else z10 = 0.0;
                }
            }
            A[o00] = z00;
            A[o01] = z01;
            A[o10] = z10;
            A[o11] = z11;
            q_update(r, qc, qs);
        } else {
            // the other waves have time to spare: their Q work goes first, which keeps their LDS traffic out of the
            // way of wave 0's reads right after the barrier
            const double qc = cs[par][2 * iota], qs = cs[par][2 * iota + 1];
            q_update(r, qc, qs);
            __builtin_amdgcn_sched_barrier(0);
            const double ci = cs[par][2 * i], si = cs[par][2 * i + 1], cj = cs[par][2 * j], sj = cs[par][2 * j + 1];
            const double x00 = A[o00], x01 = A[o01], x10 = A[o10], x11 = A[o11];
            const double y00 = ci * x00 - si * x10, y01 = ci * x01 - si * x11;
            const double y10 = si * x00 + ci * x10, y11 = si * x01 + ci * x11;
            if (valid) {
                A[o00] = cj * y00 - sj * y01;
                A[o01] = sj * y00 + cj * y01;
                A[o10] = cj * y10 - sj * y11;
                A[o11] = sj * y10 + cj * y11;
            }
        }
        offsets(r + 1 < 32 ? r + 1 : 31);
        __syncthreads();
    }
    double* Qo = Qout + (int64_t)blockIdx.x * 4096 + row0 * 64;
    const int qlast = cross_q(iota, 31);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        Qo[k * 64 + iota] = qp[k];
        Qo[k * 64 + qlast] = qq[k];
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
                                                        const double* __restrict__ Q, double* __restrict__ stat,
                                                        int NP, int sweep, int st, double tol) {
    if (sweep_done(stat, sweep, tol)) return;
    __builtin_amdgcn_s_setprio(3);  // short and on the critical path: goes before the Gram waves it shares SIMDs with
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
    double mx = 0.0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        int r = i0 + 4 * v + lk;
        int gr = isY ? (a * 64 + r) : (r < 32 ? Ia * 32 + r : Ja * 32 + r - 32);
#pragma unroll
        for (int jt = 0; jt < 2; ++jt) {
            const int gc = gcb + jt * 16 + l16;
            Mout[(int64_t)gr * NP + gc] = acc[jt][v];
            if (gr != gc) mx = fmax(mx, fabs(acc[jt][v]));
        }
    }
    // The last step of a sweep leaves the matrix the next sweep starts from: its largest off-diagonal entry is the
    // record that sweep (and eig_sort_kernel, after the last one) looks at.
    if (!isY && st == nb - 1) {
        for (int o = 32; o >= 1; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o));
        const double tr = stat[0];
        if (lane == 0 && tr > 0.0 && mx > 0.0) atomic_max_pos_double(&stat[2 + sweep], mx / tr);
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
        int last = launched <= MAX_SWEEPS ? launched : MAX_SWEEPS;
        for (int s = 0; s <= launched && s <= MAX_SWEEPS; ++s)
            if (stat[1 + s] <= tol) { used = s; last = s; break; }
        acc[3] = (double)used;
        if (used >= SWEEPS_NOT_CONVERGED) acc[4] += 1.0;  // sticky: solves that ended above their tolerance
        acc[5] = stat[1 + last];                          // largest |off-diagonal| / trace the solve left
    }
}

// Shrink coefficients (Method, FD paragraph: delta = sigma_ell^2, Sigma'_jj = sqrt(max(sigma_j^2 - delta, 0))):
// new row m = w_m * y_m^T B with w_m = sqrt(max(lambda_m - delta, 0) / lambda_m); stored in coeff_offset order.
// Also records the Gram matrix of the rows the rebuild is about to write, diag(w) (Y^T C Y) diag(w), from the rotated
// matrix Crot the eigensolve left: the next cycle takes that block as known instead of recomputing it. Its diagonal
// is max(lambda_j - delta, 0); its off-diagonal entries are what the solve did not annihilate (at most its tolerance,
// more if it ran out of sweeps), so that the next Gram matrix is right whether or not the rows came out orthogonal.
__global__ __launch_bounds__(256) void shrink_coeffs_kernel(const double* __restrict__ Y, const int* __restrict__ pos,
                                                            const double* __restrict__ lam,
                                                            const double* __restrict__ diag0,
                                                            const double* __restrict__ Crot, int NP, int LP, int ell,
                                                            int ra0, int ra1, int rb0, int rb1,
                                                            float* __restrict__ Mt, double* __restrict__ acc,
                                                            double* __restrict__ known) {
    int e = blockIdx.x * 256 + threadIdx.x;
    const double delta = lam[ell - 1];
    if (e < LP * LP) {
        const int i = e / LP, j = e % LP;
        double v = 0.0;
        if (i < ell && j < ell) {
            const double li = lam[i], lj = lam[j];
            const double ki = li - delta, kj = lj - delta;
            if (i == j) v = ki > 0.0 ? ki : 0.0;
            else if (ki > 0.0 && kj > 0.0) v = sqrt(ki / li) * sqrt(kj / lj) * Crot[(int64_t)pos[i] * NP + pos[j]];
        }
        known[e] = v;
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

// The pivot kernel uses 66.5 KB of this (two copies of the pivot matrix); the rest is there so that a work-group does
// not fit on a CU that already holds a work-group of the Gram kernel running on the side stream (64 KB), so it goes
// to one of the CUs that launch leaves free. Sharing a SIMD with matrix-core waves stretched single pivot solves
// several times over.
static const size_t CROSS_PAD_LDS = 100 * 1024;
static const size_t APPLY_LDS = (size_t)(64 * LDX + 64 * LDQB + 64 * LDQ) * sizeof(double);

hipError_t launch_eig(const EigWork& w, int NP, double tol, int max_sweeps, hipStream_t st) {
    hipError_t ea = ensure_dynamic_lds((const void*)jac_apply_kernel, (int)APPLY_LDS);
    if (ea == hipSuccess) ea = ensure_dynamic_lds((const void*)jac_pivot_kernel, (int)CROSS_PAD_LDS);
    if (ea != hipSuccess) return ea;
    if (max_sweeps > MAX_SWEEPS) max_sweeps = MAX_SWEEPS;
    if (max_sweeps < 1) max_sweeps = 1;
    hipLaunchKernelGGL(jac_init_kernel, dim3(NP), dim3(256), 0, st, w.C, w.Y, w.diag0, w.stat, NP, max_sweeps);
    hipLaunchKernelGGL(jac_measure_kernel, dim3(NP / 16), dim3(256), 0, st, w.C, w.stat, NP);
    const int np = NP / 64, nb = NP / 32;
    // Executed sweeps are the first ones, so sweep number `sweep` starts on copy (sweep * (nb - 1)) & 1 = sweep & 1
    double* Cb[2] = {w.C, w.C2};
    double* Yb[2] = {w.Y, w.Y2};
    int cur = 0;
    for (int sweep = 0; sweep < max_sweeps; ++sweep) {
        for (int s = 1; s < nb; ++s) {
            hipLaunchKernelGGL(jac_pivot_kernel, dim3(np), dim3(512), CROSS_PAD_LDS, st, Cb[cur], w.Q, w.stat, NP, sweep, s, tol);
            hipLaunchKernelGGL(jac_apply_kernel, dim3(4 * np * np), dim3(256), APPLY_LDS, st, Cb[cur], Cb[cur ^ 1], Yb[cur],
                               Yb[cur ^ 1], w.Q, w.stat, NP, sweep, s, tol);
            cur ^= 1;
        }
    }
    hipLaunchKernelGGL(jac_finish_kernel, dim3(NP), dim3(256), 0, st, w.C, w.C2, w.Y, w.Y2, w.stat, NP, tol);
    return hipGetLastError();
}

hipError_t launch_shrink_coeffs(const EigWork& w, int NP, int LP, int ell, int ra0, int ra1, int rb0, int rb1, float* Mt,
                                double* acc, double tol, hipStream_t st) {
    hipLaunchKernelGGL(eig_sort_kernel, dim3(1), dim3(512), 0, st, w.C, w.stat, w.pos, w.lam, NP, acc, tol);
    hipLaunchKernelGGL(shrink_coeffs_kernel, dim3((NP * LP + 255) / 256), dim3(256), 0, st, w.Y, w.pos, w.lam, w.diag0,
                       w.C, NP, LP, ell, ra0, ra1, rb0, rb1, Mt, acc, w.known);
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
