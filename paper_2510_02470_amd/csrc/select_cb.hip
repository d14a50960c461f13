// Class-balanced selection (Algorithm 1, "if class balance required"; "Agreement Scoring and Selection", CB-SAGE):
// per class c the unit centroid u_c of the normalised projections of its rows, alpha_i = <zhat_i, u_c(i)>, and the
// top k_c rows of every class. The k_c share out the budget m = floor(keep * N + 0.5) of the plain selection in
// proportion to the class sizes (largest-remainder rule, see cb_quota_kernel), so that sum_c k_c = m as Algorithm 1
// requires.
//
// Everything that decides the result is integer work, so the outcome does not depend on timing:
//   * class sums are accumulated in 64-bit fixed point (zhat * 2^40, |zhat| <= 1, up to 2^23 rows per class) with
//     integer atomics -- addition of integers is associative, unlike floating point;
//   * the k_c-th largest score of every class comes from one radix select run for all classes at once (a 256-bin
//     histogram per class and byte, four passes over order-preserving 32-bit keys);
//   * ties at a class threshold go to the lowest row indices: a second radix select, over the row index, among the
//     rows that sit exactly on their class threshold;
//   * the selected rows are compacted in ascending row order (per-block counts, scan, emit).
#include "sage_internal.h"

namespace sage {

constexpr double CB_SCALE = 1099511627776.0;  // 2^40

__device__ __forceinline__ uint32_t cb_key(float a) {  // larger alpha <-> larger key; -0 and +0 share a key
    uint32_t b = __float_as_uint(a);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__global__ __launch_bounds__(256) void cb_zero_kernel(uint32_t* __restrict__ counts, long long* __restrict__ sums,
                                                      uint32_t* __restrict__ hist, uint32_t* __restrict__ misc, int C) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < C) counts[i] = 0;
    if (i < (int64_t)C * 128) sums[i] = 0;
    if (i < (int64_t)C * 256) hist[i] = 0;
    if (i < 4) misc[i] = 0;  // [0] total kept, [1] a label was out of range
}

// one wave per row: count the row for its class and add its zhat to the class sum (fixed point)
__global__ __launch_bounds__(256) void cb_accumulate_kernel(const float* __restrict__ zhat, const int* __restrict__ labels,
                                                            int64_t N, int k, int C, uint32_t* __restrict__ counts,
                                                            long long* __restrict__ sums, uint32_t* __restrict__ misc) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int64_t r = (int64_t)blockIdx.x * 4 + wave; r < N; r += (int64_t)gridDim.x * 4) {
        const int c = labels[r];
        if (c < 0 || c >= C) {
            if (lane == 0) misc[1] = 1;
            continue;
        }
        if (lane == 0) atomicAdd(&counts[c], 1u);
        const float* z = zhat + r * k;
        unsigned long long* s = reinterpret_cast<unsigned long long*>(sums + (int64_t)c * 128);
        if (lane < k) atomicAdd(&s[lane], (unsigned long long)__double2ll_rn((double)z[lane] * CB_SCALE));
        if (lane + 64 < k) atomicAdd(&s[lane + 64], (unsigned long long)__double2ll_rn((double)z[lane + 64] * CB_SCALE));
    }
}

// one work-group per class: u_c = S_c / ||S_c|| (0 if S_c = 0)
__global__ __launch_bounds__(128) void cb_unit_kernel(const long long* __restrict__ sums, int k,
                                                      double* __restrict__ ucls) {
    __shared__ double red[128];
    const int c = blockIdx.x, j = threadIdx.x;
    const double s = j < k ? (double)sums[(int64_t)c * 128 + j] / CB_SCALE : 0.0;
    red[j] = s * s;
    __syncthreads();
    for (int w = 64; w >= 1; w >>= 1) {  // fixed-shape tree
        if (j < w) red[j] += red[j + w];
        __syncthreads();
    }
    const double nrm = sqrt(red[0]);
    ucls[(int64_t)c * 128 + j] = nrm > 0.0 ? s / nrm : 0.0;
}

// The class budgets (Algorithm 1, class-balanced branch: sum_c k_c = k). With N_c rows in class c and N in all,
// m = floor(keep * N + 0.5) as in the plain selection, quota q_c = keep * N_c (fp64), k_c = floor(q_c), and the
// m - sum_c floor(q_c) rows still to hand out go one each to the classes with the largest fractional part
// q_c - floor(q_c) (equal parts: the lower class first) among those with k_c < N_c. All of it is exact integer or
// correctly rounded fp64 work, so the host-side definition gives the same numbers. One work-group of 1024 threads;
// also sets the start state of the selects (prefix 0, remain k_c) and misc[0] = sum_c k_c.
__global__ __launch_bounds__(1024) void cb_quota_kernel(const uint32_t* __restrict__ counts, int C, double keep,
                                                        uint32_t* __restrict__ kc, uint32_t* __restrict__ prefix,
                                                        uint32_t* __restrict__ remain, uint32_t* __restrict__ misc) {
#pragma clang fp contract(off)
    __shared__ unsigned long long red[1024];
    __shared__ uint32_t hist[256];
    __shared__ unsigned long long s_pre;
    __shared__ uint32_t s_rem;
    const int t = threadIdx.x;
    auto block_sum = [&](unsigned long long v) {
        red[t] = v;
        __syncthreads();
        for (int w = 512; w >= 1; w >>= 1) {
            if (t < w) red[t] += red[t + w];
            __syncthreads();
        }
        const unsigned long long r = red[0];
        __syncthreads();
        return r;
    };
    // The product keep * N_c must be rounded before floor() is subtracted from it. Contracted into a fused
    // multiply-add (the compiler's default, and __dmul_rn does not stop it) the difference comes from the unrounded
    // product: other bits than the host-side definition, even a negative "fraction" when keep * N_c rounds up to an
    // integer.
    auto quota = [&](uint32_t n) {
#pragma clang fp contract(off)
        return keep * (double)n;
    };
    auto frac_key = [&](uint32_t n) {  // order-preserving bits of the fractional part (a double in [0, 1))
#pragma clang fp contract(off)
        const double q = keep * (double)n;
        const double f = q - floor(q);
        return (unsigned long long)__double_as_longlong(f);
    };
    unsigned long long nsum = 0, bsum = 0, cand = 0;
    for (int c = t; c < C; c += 1024) {
        const uint32_t n = counts[c];
        const double f = floor(quota(n));
        const uint32_t b = f <= 0.0 ? 0u : (f >= (double)n ? n : (uint32_t)f);
        kc[c] = b;
        nsum += n;
        bsum += b;
        cand += b < n;
    }
    const unsigned long long N = block_sum(nsum), base = block_sum(bsum), ncand = block_sum(cand);
    double x;
    {
#pragma clang fp contract(off)
        const double kn = keep * (double)N;
        x = floor(kn + 0.5);
    }
    const unsigned long long m = x <= 0.0 ? 0ull : (x >= (double)N ? N : (unsigned long long)x);
    unsigned long long rem = m > base ? m - base : 0ull;
    if (rem > ncand) rem = ncand;
    if (rem > 0) {
        // radix select of the rem-th largest key among the candidates, a byte at a time from the top
        if (t == 0) { s_pre = 0ull; s_rem = (uint32_t)rem; }
        for (int shift = 56; shift >= 0; shift -= 8) {
            if (t < 256) hist[t] = 0;
            __syncthreads();
            const unsigned long long pre = s_pre;
            for (int c = t; c < C; c += 1024) {
                if (kc[c] >= counts[c]) continue;
                const unsigned long long key = frac_key(counts[c]);
                if (shift == 56 || (key >> (shift + 8)) == pre) atomicAdd(&hist[(key >> shift) & 255ull], 1u);
            }
            __syncthreads();
            if (t == 0) {
                uint32_t want = s_rem, cum = 0;
                int chosen = 0;
                for (int b = 255; b >= 0; --b) {
                    if (cum + hist[b] >= want) { chosen = b; break; }
                    cum += hist[b];
                }
                s_pre = (pre << 8) | (unsigned long long)chosen;
                s_rem = want - cum;
            }
            __syncthreads();
        }
        const unsigned long long T = s_pre;
        const uint32_t take = s_rem;  // classes exactly on the threshold that still get a row, lowest class first
        // ordered count of the threshold classes: every thread owns a contiguous run of classes
        const int chunk = (C + 1023) / 1024;
        const int c0 = t * chunk, c1 = c0 + chunk < C ? c0 + chunk : C;
        unsigned long long eq = 0;
        for (int c = c0; c < c1; ++c) eq += (kc[c] < counts[c] && frac_key(counts[c]) == T);
        red[t] = eq;
        __syncthreads();
        for (int o = 1; o < 1024; o <<= 1) {  // Hillis-Steele inclusive scan
            const unsigned long long a = t >= o ? red[t - o] : 0ull;
            __syncthreads();
            red[t] += a;
            __syncthreads();
        }
        unsigned long long before = red[t] - eq;
        __syncthreads();
        for (int c = c0; c < c1; ++c) {
            if (kc[c] >= counts[c]) continue;
            const unsigned long long key = frac_key(counts[c]);
            if (key > T) kc[c] += 1;
            else if (key == T) {
                if (before < take) kc[c] += 1;
                before += 1;
            }
        }
        __syncthreads();
    }
    unsigned long long tot = 0;
    for (int c = t; c < C; c += 1024) {
        prefix[c] = 0;
        remain[c] = kc[c];
        tot += kc[c];
    }
    tot = block_sum(tot);
    if (t == 0) misc[0] = (uint32_t)tot;
}

// The other budget rule: equal budgets. The m = floor(keep * N + 0.5) rows are dealt one at a time to the classes in
// turn, lowest class first, a full class being passed over. In closed form: with q the largest level for which
// sum_c min(N_c, q) <= m, class c gets min(N_c, q), and the m - sum_c min(N_c, q) rows left (fewer than there are
// classes larger than q) go one each to the lowest-numbered classes with N_c > q. Integer work throughout. One
// work-group of 1024 threads; also sets the start state of the selects and misc[0] = sum_c k_c, like cb_quota_kernel.
__global__ __launch_bounds__(1024) void cb_quota_equal_kernel(const uint32_t* __restrict__ counts, int C, double keep,
                                                              uint32_t* __restrict__ kc, uint32_t* __restrict__ prefix,
                                                              uint32_t* __restrict__ remain, uint32_t* __restrict__ misc) {
#pragma clang fp contract(off)
    __shared__ unsigned long long red[1024];
    const int t = threadIdx.x;
    auto block_sum = [&](unsigned long long v) {
        red[t] = v;
        __syncthreads();
        for (int w = 512; w >= 1; w >>= 1) {
            if (t < w) red[t] += red[t + w];
            __syncthreads();
        }
        const unsigned long long r = red[0];
        __syncthreads();
        return r;
    };
    auto block_max = [&](unsigned long long v) {
        red[t] = v;
        __syncthreads();
        for (int w = 512; w >= 1; w >>= 1) {
            if (t < w) red[t] = red[t] > red[t + w] ? red[t] : red[t + w];
            __syncthreads();
        }
        const unsigned long long r = red[0];
        __syncthreads();
        return r;
    };
    unsigned long long nsum = 0, nmax = 0;
    for (int c = t; c < C; c += 1024) {
        const unsigned long long n = counts[c];
        nsum += n;
        nmax = n > nmax ? n : nmax;
    }
    const unsigned long long N = block_sum(nsum), top = block_max(nmax);
    double x;
    {
#pragma clang fp contract(off)
        const double kn = keep * (double)N;
        x = floor(kn + 0.5);
    }
    const unsigned long long m = x <= 0.0 ? 0ull : (x >= (double)N ? N : (unsigned long long)x);
    auto dealt = [&](unsigned long long q) {  // sum_c min(N_c, q)
        unsigned long long s = 0;
        for (int c = t; c < C; c += 1024) {
            const unsigned long long n = counts[c];
            s += n < q ? n : q;
        }
        return block_sum(s);
    };
    unsigned long long lo = 0, hi = top;  // dealt(lo) <= m always (dealt(0) = 0); the answer is in [lo, hi]
    while (lo < hi) {                     // (every thread sees the same sums, so the loop is uniform)
        const unsigned long long mid = lo + (hi - lo + 1) / 2;
        if (dealt(mid) <= m) lo = mid;
        else hi = mid - 1;
    }
    const unsigned long long q = lo;
    const unsigned long long spare = m - dealt(q);  // < number of classes with N_c > q
    // ordered count of the classes that can take a spare row: every thread owns a contiguous run of classes
    const int chunk = (C + 1023) / 1024;
    const int c0 = t * chunk, c1 = c0 + chunk < C ? c0 + chunk : C;
    unsigned long long open = 0;
    for (int c = c0; c < c1; ++c) open += counts[c] > q;
    red[t] = open;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {  // Hillis-Steele inclusive scan
        const unsigned long long a = t >= o ? red[t - o] : 0ull;
        __syncthreads();
        red[t] += a;
        __syncthreads();
    }
    unsigned long long before = red[t] - open;
    __syncthreads();
    unsigned long long tot = 0;
    for (int c = c0; c < c1; ++c) {
        const unsigned long long n = counts[c];
        unsigned long long b = n < q ? n : q;
        if (n > q) {
            if (before < spare) b += 1;
            before += 1;
        }
        kc[c] = (uint32_t)b;
        prefix[c] = 0;
        remain[c] = (uint32_t)b;
        tot += b;
    }
    tot = block_sum(tot);
    if (t == 0) misc[0] = (uint32_t)tot;
}

// alpha_i = clamp(<zhat_i, u_c(i)>, -1, 1), -0 stored as +0; one wave per row
__global__ __launch_bounds__(256) void cb_cosine_kernel(const float* __restrict__ zhat, const int* __restrict__ labels,
                                                        int64_t N, int k, int C, const double* __restrict__ ucls,
                                                        float* __restrict__ alpha) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int64_t r = (int64_t)blockIdx.x * 4 + wave; r < N; r += (int64_t)gridDim.x * 4) {
        int c = labels[r];
        if (c < 0 || c >= C) c = 0;  // reported by cb_accumulate_kernel; keep the reads in bounds
        const float* z = zhat + r * k;
        const double* u = ucls + (int64_t)c * 128;
        double a = 0.0;
        if (lane < k) a = (double)z[lane] * u[lane];
        if (lane + 64 < k) a += (double)z[lane + 64] * u[lane + 64];
        for (int o = 32; o >= 1; o >>= 1) a += __shfl_xor(a, o);
        if (lane == 0) {
            if (a > 1.0) a = 1.0;
            if (a < -1.0) a = -1.0;
            float f = (float)a;
            if (f == 0.f) f = 0.f;
            alpha[r] = f;
        }
    }
}

// phase 0: histogram of byte shift/8 of the score keys whose higher bytes equal their class prefix
// phase 1: the same over the row index, among the rows whose score key equals their class threshold
__global__ __launch_bounds__(256) void cb_hist_kernel(const float* __restrict__ alpha, const int* __restrict__ labels,
                                                      int64_t N, int C, int phase, int shift,
                                                      const uint32_t* __restrict__ kc, const uint32_t* __restrict__ thr,
                                                      const uint32_t* __restrict__ prefix, uint32_t* __restrict__ hist) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < N; i += (int64_t)gridDim.x * 256) {
        const int c = labels[i];
        if (c < 0 || c >= C || kc[c] == 0) continue;
        uint32_t key = cb_key(alpha[i]);
        if (phase == 1) {
            if (key != thr[c]) continue;
            key = (uint32_t)i;
        }
        const bool match = shift == 24 ? true : ((key >> (shift + 8)) == prefix[c]);
        if (match) atomicAdd(&hist[(int64_t)c * 256 + ((key >> shift) & 255u)], 1u);
    }
}

// one thread per class: walk the class's bins (from the top in phase 0: k-th largest score; from the bottom in phase 1:
// k-th smallest index) until the remaining count is covered, extend the prefix, clear the bins
__global__ __launch_bounds__(256) void cb_pick_kernel(uint32_t* __restrict__ hist, int C, int phase,
                                                      const uint32_t* __restrict__ kc, uint32_t* __restrict__ prefix,
                                                      uint32_t* __restrict__ remain) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    uint32_t* h = hist + (int64_t)c * 256;
    if (kc[c]) {
        const uint32_t want = remain[c];
        uint32_t cum = 0;
        int chosen = phase == 0 ? 0 : 255;
        for (int t = 0; t < 256; ++t) {
            const int b = phase == 0 ? 255 - t : t;
            const uint32_t n = h[b];
            if (cum + n >= want) { chosen = b; break; }
            cum += n;
        }
        prefix[c] = (prefix[c] << 8) | (uint32_t)chosen;
        remain[c] = want - cum;
    }
    for (int b = 0; b < 256; ++b) h[b] = 0;
}

// between the phases: the score prefix is the class threshold; the index select starts with `remain` ties to take
__global__ __launch_bounds__(256) void cb_phase_kernel(int C, uint32_t* __restrict__ thr, uint32_t* __restrict__ prefix) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    thr[c] = prefix[c];
    prefix[c] = 0;
}

// row i is kept when its class keeps anything and its key is above the class threshold, or on it with an index not
// above the class's index threshold; per block of SELECT_BLOCK rows the number kept
__global__ __launch_bounds__(256) void cb_count_kernel(const float* __restrict__ alpha, const int* __restrict__ labels,
                                                       int64_t N, int C, const uint32_t* __restrict__ kc,
                                                       const uint32_t* __restrict__ thr, const uint32_t* __restrict__ tidx,
                                                       uint8_t* __restrict__ sel, uint32_t* __restrict__ blk) {
    __shared__ uint32_t sg[256];
    const int64_t base = (int64_t)blockIdx.x * SELECT_BLOCK + (int64_t)threadIdx.x * 8;
    uint32_t g = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int64_t i = base + q;
        if (i < N) {
            const int c = labels[i];
            bool keepit = false;
            if (c >= 0 && c < C && kc[c]) {
                const uint32_t key = cb_key(alpha[i]);
                keepit = key > thr[c] || (key == thr[c] && (uint32_t)i <= tidx[c]);
            }
            sel[i] = keepit ? 1 : 0;
            g += keepit;
        }
    }
    sg[threadIdx.x] = g;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) sg[threadIdx.x] += sg[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) blk[blockIdx.x] = sg[0];
}

// exclusive scan of the per-block counts, in place (single work-group, sequential over chunks of 256 blocks)
__global__ __launch_bounds__(256) void cb_scan_kernel(uint32_t* __restrict__ blk, int nblk) {
    __shared__ uint32_t sg[256];
    uint32_t carry = 0;
    for (int base = 0; base < nblk; base += 256) {
        const int i = base + threadIdx.x;
        const uint32_t g = i < nblk ? blk[i] : 0;
        sg[threadIdx.x] = g;
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {  // Hillis-Steele inclusive scan
            uint32_t ag = 0;
            if ((int)threadIdx.x >= o) ag = sg[threadIdx.x - o];
            __syncthreads();
            sg[threadIdx.x] += ag;
            __syncthreads();
        }
        if (i < nblk) blk[i] = carry + sg[threadIdx.x] - g;
        const uint32_t t = sg[255];
        __syncthreads();
        carry += t;
    }
}

__global__ __launch_bounds__(256) void cb_emit_kernel(const uint8_t* __restrict__ sel, int64_t N,
                                                      const uint32_t* __restrict__ blk, int64_t* __restrict__ out_idx) {
    __shared__ uint32_t sg[256];
    const int64_t base = (int64_t)blockIdx.x * SELECT_BLOCK + (int64_t)threadIdx.x * 8;
    uint8_t f[8];
    uint32_t g = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int64_t i = base + q;
        f[q] = i < N ? sel[i] : 0;
        g += f[q];
    }
    sg[threadIdx.x] = g;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
        uint32_t ag = 0;
        if ((int)threadIdx.x >= o) ag = sg[threadIdx.x - o];
        __syncthreads();
        sg[threadIdx.x] += ag;
        __syncthreads();
    }
    uint32_t slot = blk[blockIdx.x] + sg[threadIdx.x] - g;
#pragma unroll
    for (int q = 0; q < 8; ++q)
        if (f[q]) out_idx[slot++] = base + q;
}

size_t cb_work_bytes(int C, int64_t N) {
    const int64_t nblk = (N + SELECT_BLOCK - 1) / SELECT_BLOCK;
    size_t b = 0;
    b += (size_t)C * 4 * 6;             // counts, kc, prefix, remain, thr, (spare)
    b += (size_t)C * 128 * 8 * 2;       // sums, ucls
    b += (size_t)C * 256 * 4;           // hist
    b += 64;                            // misc
    b += (size_t)(nblk > 0 ? nblk : 1) * 4;  // blk
    b += (size_t)(N > 0 ? N : 1);       // sel
    return b + 4096;                    // alignment slack
}

CbWork cb_work_layout(void* base, int C, int64_t N) {
    CbWork w{};
    char* p = (char*)base;
    auto take = [&](size_t bytes) {
        char* q = p;
        p += (bytes + 255) / 256 * 256;
        return q;
    };
    w.sums = (long long*)take((size_t)C * 128 * 8);
    w.ucls = (double*)take((size_t)C * 128 * 8);
    w.counts = (uint32_t*)take((size_t)C * 4);
    w.kc = (uint32_t*)take((size_t)C * 4);
    w.prefix = (uint32_t*)take((size_t)C * 4);
    w.remain = (uint32_t*)take((size_t)C * 4);
    w.thr = (uint32_t*)take((size_t)C * 4);
    w.hist = (uint32_t*)take((size_t)C * 256 * 4);
    w.misc = (uint32_t*)take(64);
    const int64_t nblk = (N + SELECT_BLOCK - 1) / SELECT_BLOCK;
    w.blk = (uint32_t*)take((size_t)(nblk > 0 ? nblk : 1) * 4);
    w.sel = (uint8_t*)take((size_t)(N > 0 ? N : 1));
    return w;
}

// Stage 1: class counts, sums, centroids, k_c, scores. Afterwards misc[0] = total kept, misc[1] = bad label seen.
hipError_t launch_cb_scores(const float* zhat, const int* labels, int64_t N, int k, int C, double keep, int rule,
                            float* alpha, const CbWork& w, hipStream_t st) {
    const int64_t zi = (int64_t)C * 256;
    hipLaunchKernelGGL(cb_zero_kernel, dim3((unsigned)((zi + 255) / 256)), dim3(256), 0, st, w.counts, w.sums, w.hist,
                       w.misc, C);
    if (N > 0) {
        int64_t blocks = (N + 3) / 4;
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(cb_accumulate_kernel, dim3((unsigned)blocks), dim3(256), 0, st, zhat, labels, N, k, C, w.counts,
                           w.sums, w.misc);
    }
    hipLaunchKernelGGL(cb_unit_kernel, dim3(C), dim3(128), 0, st, w.sums, k, w.ucls);
    if (rule == SAGE_CB_EQUAL)
        hipLaunchKernelGGL(cb_quota_equal_kernel, dim3(1), dim3(1024), 0, st, w.counts, C, keep, w.kc, w.prefix, w.remain,
                           w.misc);
    else
        hipLaunchKernelGGL(cb_quota_kernel, dim3(1), dim3(1024), 0, st, w.counts, C, keep, w.kc, w.prefix, w.remain, w.misc);
    if (N > 0) {
        int64_t blocks = (N + 3) / 4;
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(cb_cosine_kernel, dim3((unsigned)blocks), dim3(256), 0, st, zhat, labels, N, k, C, w.ucls, alpha);
    }
    return hipGetLastError();
}

// Stage 2: thresholds per class, flags, compaction. out_idx receives misc[0] indices, ascending.
hipError_t launch_cb_select(const float* alpha, const int* labels, int64_t N, int C, int64_t* out_idx, const CbWork& w,
                            hipStream_t st) {
    if (N <= 0) return hipSuccess;
    int64_t hb = (N + 255) / 256;
    if (hb > 2048) hb = 2048;
    const unsigned cb = (unsigned)((C + 255) / 256);
    for (int phase = 0; phase < 2; ++phase) {
        for (int shift = 24; shift >= 0; shift -= 8) {
            hipLaunchKernelGGL(cb_hist_kernel, dim3((unsigned)hb), dim3(256), 0, st, alpha, labels, N, C, phase, shift, w.kc,
                               w.thr, w.prefix, w.hist);
            hipLaunchKernelGGL(cb_pick_kernel, dim3(cb), dim3(256), 0, st, w.hist, C, phase, w.kc, w.prefix, w.remain);
        }
        if (phase == 0) hipLaunchKernelGGL(cb_phase_kernel, dim3(cb), dim3(256), 0, st, C, w.thr, w.prefix);
    }
    const int64_t nblk = (N + SELECT_BLOCK - 1) / SELECT_BLOCK;
    // after phase 1 `prefix` is the index threshold of every class
    hipLaunchKernelGGL(cb_count_kernel, dim3((unsigned)nblk), dim3(256), 0, st, alpha, labels, N, C, w.kc, w.thr, w.prefix,
                       w.sel, w.blk);
    hipLaunchKernelGGL(cb_scan_kernel, dim3(1), dim3(256), 0, st, w.blk, (int)nblk);
    hipLaunchKernelGGL(cb_emit_kernel, dim3((unsigned)nblk), dim3(256), 0, st, w.sel, N, w.blk, out_idx);
    return hipGetLastError();
}

}  // namespace sage
