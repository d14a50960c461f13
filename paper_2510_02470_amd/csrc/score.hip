// Scoring pass, first half (Algorithm 1, Phase II, first line; Method, "Two-pass scoring"):
//   z_i = V_k^T g_i  (fp32 matrix cores, split over D),  zhat_i = z_i / ||z_i||_2 (0 if z_i = 0),
//   consensus sum  s += sum_i zhat_i  (fixed-order reductions, fp64).
#include "sage_internal.h"

namespace sage {

// load one 16-byte-wide piece (4 columns) of a batch row, widened to fp32; columns >= D read as 0
template <typename T, bool VEC>
__device__ __forceinline__ f32x4 load_piece(const T* __restrict__ row, int64_t d0, int64_t D) {
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if constexpr (VEC) {
        if (d0 < D) {  // D % 4 == 0 on this path
            if constexpr (sizeof(T) == 4) {
                v = *reinterpret_cast<const f32x4*>(row + d0);
            } else {
                uint2 u = *reinterpret_cast<const uint2*>(row + d0);
                v[0] = __uint_as_float(u.x << 16);
                v[1] = __uint_as_float(u.x & 0xffff0000u);
                v[2] = __uint_as_float(u.y << 16);
                v[3] = __uint_as_float(u.y & 0xffff0000u);
            }
        }
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float x = 0.f;
            if (d0 + c < D) {
                if constexpr (sizeof(T) == 4) x = row[d0 + c];
                else x = bf16_to_f32(row[d0 + c]);
            }
            v[c] = x;
        }
    }
    return v;
}

// Work-group tile: 128 batch rows x KP basis columns, a wave owns 32 rows. Split-K over D: block id ->
// (row tile, split) with the row tiles of one split adjacent on one XCD so that they share the basis slabs in L2.
// partial[split][row][KP] receives the fp32 partial projections.
template <int NT, typename T, bool VEC>  // NT = KP / 32
__global__ __launch_bounds__(256) void project_kernel(const T* __restrict__ G, int64_t R, const float* __restrict__ Vblk,
                                                      float* __restrict__ partial, int row_tiles, int64_t D,
                                                      int64_t slabs_total, int64_t slabs_per_split) {
    constexpr int KP = NT * 32;
    constexpr int GP = 128 * 4;       // batch pieces per stage
    constexpr int VP = KP * 4;        // basis pieces per stage
    constexpr int STAGE = GP + VP;
    constexpr int VPER = (VP + 255) / 256;
    __shared__ f32x4 lds[2 * STAGE];

    const int id = blockIdx.x;
    const int xcd = id & 7, y = id >> 3;
    const int rt = y % row_tiles;
    const int split = (y / row_tiles) * 8 + xcd;
    int64_t s0 = (int64_t)split * slabs_per_split;
    int64_t s1 = s0 + slabs_per_split;
    if (s1 > slabs_total) s1 = slabs_total;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, h = lane >> 5;
    const int64_t row_base = (int64_t)rt * 128;

    f32x16 acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;

    // staging slots: batch piece slot ps -> (row ps/4, logical piece (ps%4)^((row/4)%4)); same for the basis
    int grow[2], gp[2];
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        int ps = it * 256 + tid;
        grow[it] = ps >> 2;
        gp[it] = (ps & 3) ^ ((grow[it] >> 2) & 3);
    }
    int vsrc[VPER];
#pragma unroll
    for (int it = 0; it < VPER; ++it) {
        int ps = it * 256 + tid;
        int row = ps >> 2;
        vsrc[it] = row * 4 + ((ps & 3) ^ ((row >> 2) & 3));
    }
    const f32x4* Vv = reinterpret_cast<const f32x4*>(Vblk);
    f32x4 gpre[2], vpre[VPER];

    auto fetch = [&](int64_t s) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            int64_t r = row_base + grow[it];
            gpre[it] = (r < R) ? load_piece<T, VEC>(G + r * D, s * DC + gp[it] * 4, D) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int it = 0; it < VPER; ++it)
            if (it * 256 + tid < VP) vpre[it] = Vv[s * VP + vsrc[it]];
    };
    auto stash = [&](int buf) {
        f32x4* dst = lds + buf * STAGE;
#pragma unroll
        for (int it = 0; it < 2; ++it) dst[it * 256 + tid] = gpre[it];
#pragma unroll
        for (int it = 0; it < VPER; ++it)
            if (it * 256 + tid < VP) dst[GP + it * 256 + tid] = vpre[it];
    };

    if (s0 < s1) {
        fetch(s0);
        stash(0);
    }
    __syncthreads();
    for (int64_t s = s0; s < s1; ++s) {
        const int cur = (int)((s - s0) & 1);
        const bool more = s + 1 < s1;
        if (more) fetch(s + 1);
        const f32x4* gs = lds + cur * STAGE;
        const f32x4* vs = gs + GP;
        f32x4 a[2];
        {
            int r = wave * 32 + l32;
#pragma unroll
            for (int j = 0; j < 2; ++j) a[j] = gs[r * 4 + ((2 * j + h) ^ ((r >> 2) & 3))];
        }
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            int r = n * 32 + l32;
            f32x4 b[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = vs[r * 4 + ((2 * j + h) ^ ((r >> 2) & 3))];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    acc[n] = mfma32(a[j][c], b[j][c], acc[n]);
        }
        if (more) stash(cur ^ 1);
        __syncthreads();
    }

    float* out = partial + (int64_t)split * R * KP;
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            int64_t r = row_base + wave * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
            if (r < R) out[r * KP + n * 32 + l32] = acc[n][i];
        }
}

// Sum of the split-K partial projections, normalisation and consensus partial sums.
// A work-group of 1024 threads takes 4 rows, four waves per row: wave (row, quarter) adds a quarter of the splits
// in order, lane j holding coordinates 2j and 2j + 1, with all its loads (up to 32 at a time) in flight together;
// the quarter sums are added in quarter order by the row's first wave, which normalises. Writes zhat (R x k, fp32)
// and cons_partial[block][128] (fp64 sums of the block's zhat, the four rows added in row order). All in fp64, fixed
// order: the result does not depend on timing.
constexpr int FIN_ROWS = 4;
// mode 0: as above. mode 1: consensus partial sums only, zhat is not kept (first scoring pass of a run that does not
// store zhat). mode 2: the second such pass: alpha_i = clamp(<zhat_i, u>, -1, 1) straight from the recomputed zhat_i,
// with u = ssum / ||ssum|| rebuilt by every work-group and the arithmetic of cosine_kernel (same lanes, same order),
// so that the scores are bit-equal to those of the run that stores zhat.
__global__ __launch_bounds__(1024) void score_finalize_kernel(const float* __restrict__ partial, int64_t R, int KP, int k,
                                                              int splits, float* __restrict__ zhat,
                                                              double* __restrict__ cons_partial, int mode,
                                                              const double* __restrict__ ssum,
                                                              float* __restrict__ alpha) {
    __shared__ double red[FIN_ROWS][4][128];
    __shared__ double cs[FIN_ROWS][128];
    __shared__ double u[128];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (mode == 2) {  // work-group uniform
        double* tree = &red[0][0][0];
        if (tid < 128) {
            const double sv = tid < k ? ssum[tid] : 0.0;
            u[tid] = sv;
            tree[tid] = sv * sv;
        }
        __syncthreads();
        for (int w = 64; w >= 1; w >>= 1) {  // fixed-shape tree, as in cosine_kernel
            if (tid < w) tree[tid] += tree[tid + w];
            __syncthreads();
        }
        const double nrm = sqrt(tree[0]);
        __syncthreads();
        if (tid < 128) u[tid] = nrm > 0.0 ? u[tid] / nrm : 0.0;
        __syncthreads();
    }
    const int rr = wave >> 2, quarter = wave & 3;
    const int64_t r = (int64_t)blockIdx.x * FIN_ROWS + rr;
    const bool on = 2 * lane < KP;  // KP is a multiple of 32
    double z0 = 0.0, z1 = 0.0;
    if (r < R && on) {
        const int per = (splits + 3) / 4;
        const int sa = quarter * per, sb = sa + per < splits ? sa + per : splits;
        const float2* p0 = reinterpret_cast<const float2*>(partial + r * KP) + lane;
        const int64_t sstride = R * KP / 2;  // in float2
        for (int s = sa; s < sb; s += 32) {
            float2 v[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                const int ss = s + u < sb ? s + u : sb - 1;  // repeats are not added
                v[u] = p0[ss * sstride];
            }
#pragma unroll
            for (int u = 0; u < 32; ++u)
                if (s + u < sb) {
                    z0 += (double)v[u].x;
                    z1 += (double)v[u].y;
                }
        }
    }
    red[rr][quarter][2 * lane] = z0;
    red[rr][quarter][2 * lane + 1] = z1;
    __syncthreads();
    if (quarter == 0) {
        float h0 = 0.f, h1 = 0.f;
        if (r < R) {
            // lane j now holds coordinates j and j + 64
            double a0 = ((red[rr][0][lane] + red[rr][1][lane]) + red[rr][2][lane]) + red[rr][3][lane];
            double a1 = ((red[rr][0][lane + 64] + red[rr][1][lane + 64]) + red[rr][2][lane + 64]) + red[rr][3][lane + 64];
            if (lane >= k) a0 = 0.0;
            if (lane + 64 >= k) a1 = 0.0;
            double q2 = a0 * a0 + a1 * a1;
            for (int o = 32; o >= 1; o >>= 1) q2 += __shfl_xor(q2, o);
            const double nrm = sqrt(q2);
            if (nrm > 0.0) {
                h0 = (float)(a0 / nrm);
                h1 = (float)(a1 / nrm);
            }
            if (mode == 0) {
                if (lane < k) zhat[r * k + lane] = h0;
                if (lane + 64 < k) zhat[r * k + lane + 64] = h1;
            } else if (mode == 2) {
                double a = 0.0;
                if (lane < k) a = (double)h0 * u[lane];
                if (lane + 64 < k) a += (double)h1 * u[lane + 64];
                for (int o = 32; o >= 1; o >>= 1) a += __shfl_xor(a, o);
                if (lane == 0) {
                    if (a > 1.0) a = 1.0;
                    if (a < -1.0) a = -1.0;
                    float f = (float)a;
                    if (f == 0.f) f = 0.f;  // -0 -> +0
                    alpha[r] = f;
                }
            }
        }
        cs[rr][lane] = (double)h0;
        cs[rr][lane + 64] = (double)h1;
    }
    __syncthreads();
    if (mode != 2 && tid < 128)
        cons_partial[(int64_t)blockIdx.x * 128 + tid] = ((cs[0][tid] + cs[1][tid]) + cs[2][tid]) + cs[3][tid];
}

// ssum[j] += sum over blocks of cons_partial[block][j]: thread (group g = tid / 128, coordinate j = tid % 128) adds
// blocks g, g + 8, ... in order, the 8 group sums are then added in group order.
__global__ __launch_bounds__(1024) void consensus_add_kernel(const double* __restrict__ cons_partial, int nblocks, int k,
                                                             double* __restrict__ ssum) {
    __shared__ double red[8][128];
    const int j = threadIdx.x & 127, g = threadIdx.x >> 7;
    double s = 0.0;
    for (int b = g; b < nblocks; b += 32) {
        double v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = (b + 8 * u < nblocks) ? cons_partial[(int64_t)(b + 8 * u) * 128 + j] : 0.0;
#pragma unroll
        for (int u = 0; u < 4; ++u) s += v[u];
    }
    red[g][j] = s;
    __syncthreads();
    if (g == 0 && j < k) {
        double t = 0.0;
#pragma unroll
        for (int u = 0; u < 8; ++u) t += red[u][j];
        ssum[j] += t;
    }
}

ScorePlan score_plan(int64_t R, const Dims& d, int num_cu) {
    ScorePlan p;
    p.row_tiles = (int)((R + 127) / 128);
    int64_t want = ((int64_t)num_cu * 2 + p.row_tiles - 1) / p.row_tiles;
    int64_t s = (want + 7) / 8 * 8;
    int64_t smax = ((d.S + 3) / 4 + 7) / 8 * 8;  // at least ~4 slabs per split
    if (s > smax) s = smax;
    if (s < 8) s = 8;
    if (s > 512) s = 512;
    p.splits = (int)s;
    p.slabs_per_split = (d.S + s - 1) / s;
    return p;
}

template <int NT>
static hipError_t launch_project_nt(const void* G, int dtype, bool vec, int64_t R, const float* Vblk, float* partial,
                                    const ScorePlan& p, const Dims& d, hipStream_t st) {
    dim3 grid((unsigned)(p.row_tiles * p.splits));
#define SAGE_PROJ(TT, VV)                                                                                          \
    hipLaunchKernelGGL((project_kernel<NT, TT, VV>), grid, dim3(256), 0, st, (const TT*)G, R, Vblk, partial,       \
                       p.row_tiles, d.D, d.S, p.slabs_per_split)
    if (dtype == SAGE_BF16) {
        if (vec) SAGE_PROJ(uint16_t, true); else SAGE_PROJ(uint16_t, false);
    } else {
        if (vec) SAGE_PROJ(float, true); else SAGE_PROJ(float, false);
    }
#undef SAGE_PROJ
    return hipGetLastError();
}

hipError_t launch_project(const void* G, int dtype, int64_t R, const float* Vblk, int KP, float* partial,
                          const ScorePlan& p, const Dims& d, hipStream_t st) {
    size_t esz = dtype == SAGE_BF16 ? 2 : 4;
    bool vec = (d.D % 4 == 0) && (((uintptr_t)G) % (4 * esz) == 0);
    switch (KP / 32) {
        case 1: return launch_project_nt<1>(G, dtype, vec, R, Vblk, partial, p, d, st);
        case 2: return launch_project_nt<2>(G, dtype, vec, R, Vblk, partial, p, d, st);
        case 4: return launch_project_nt<4>(G, dtype, vec, R, Vblk, partial, p, d, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_score_finalize(const float* partial, int64_t R, int KP, int k, int splits, float* zhat_out,
                                 double* cons_partial, double* ssum, int mode, float* alpha_out, hipStream_t st) {
    int nblocks = (int)((R + FIN_ROWS - 1) / FIN_ROWS);
    hipLaunchKernelGGL(score_finalize_kernel, dim3(nblocks), dim3(1024), 0, st, partial, R, KP, k, splits, zhat_out,
                       cons_partial, mode, ssum, alpha_out);
    if (mode != 2) hipLaunchKernelGGL(consensus_add_kernel, dim3(1), dim3(1024), 0, st, cons_partial, nblocks, k, ssum);
    return hipGetLastError();
}

}  // namespace sage
