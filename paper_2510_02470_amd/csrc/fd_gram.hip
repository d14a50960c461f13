// Gram matrix of the sketch buffer, C = B B^T, on the fp32 matrix cores.
//
// The shrink step needs the SVD of the buffer (Method, FD paragraph: "compute a thin SVD S = U Sigma V^T");
// it is taken through the eigen-decomposition of this Gram matrix. Only the lower triangle is computed, in
// 64x64 tiles. The long dimension (D) is split over work-group "groups"; each group writes fp32 partial tiles
// that gram_reduce adds in a fixed order in fp64.
#include "sage_internal.h"

namespace sage {

__device__ __forceinline__ void tile_coords(int t, int& ti, int& tj) {
    // row-major enumeration of the lower triangle: t = ti*(ti+1)/2 + tj, tj <= ti
    int i = 0;
    while ((i + 1) * (i + 2) / 2 <= t) ++i;
    ti = i;
    tj = t - i * (i + 1) / 2;
}

// P = NP / 64 row panels. 256 threads = 4 waves; a wave owns up to 3 tiles (12 accumulators of 32x32).
// Dynamic LDS: 2 stages x NP rows x 64 B, 16-byte pieces XOR-swizzled by (row/4)%4 so that the 16 rows read
// by a quarter wave fall in distinct banks.
template <int P>
__global__ __launch_bounds__(256) void gram_kernel(const float* __restrict__ B, float* __restrict__ partial, int tiles,
                                                   int wg_per_group, int64_t slabs_total, int64_t slabs_per_group) {
    constexpr int NP = P * 64;
    constexpr int STAGE = NP * 4;  // float4 pieces per stage
    extern __shared__ f32x4 lds[];

    const int id = blockIdx.x;
    const int xcd = id & 7;  // consecutive block ids go to consecutive XCDs: keep a group on one XCD (shared L2)
    const int y = id >> 3;
    const int w = y % wg_per_group;
    const int group = (y / wg_per_group) * 8 + xcd;
    int64_t s0 = (int64_t)group * slabs_per_group;
    int64_t s1 = s0 + slabs_per_group;
    if (s1 > slabs_total) s1 = slabs_total;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, h = lane >> 5;

    int ti[3], tj[3];
    bool on[3];
    const int tbase = (w * 4 + wave) * 3;
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        int t = tbase + q;
        on[q] = t < tiles;
        ti[q] = 0;
        tj[q] = 0;
        if (on[q]) tile_coords(t, ti[q], tj[q]);
    }

    f32x16 acc[3][2][2];
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[q][a][b][i] = 0.f;

    // staging map: slot ps = it*256 + tid holds (row = ps/4, logical piece = (ps%4) ^ ((row/4)%4))
    int src[P];
#pragma unroll
    for (int it = 0; it < P; ++it) {
        int ps = it * 256 + tid;
        int row = ps >> 2;
        int p = (ps & 3) ^ ((row >> 2) & 3);
        src[it] = row * 4 + p;
    }
    const f32x4* Bv = reinterpret_cast<const f32x4*>(B);
    f32x4 pre[P];

    if (s0 < s1) {
        const f32x4* slab = Bv + s0 * STAGE;
#pragma unroll
        for (int it = 0; it < P; ++it) pre[it] = slab[src[it]];
#pragma unroll
        for (int it = 0; it < P; ++it) lds[it * 256 + tid] = pre[it];
    }
    __syncthreads();

    for (int64_t s = s0; s < s1; ++s) {
        const int cur = (int)((s - s0) & 1);
        const bool more = (s + 1 < s1);
        if (more) {
            const f32x4* slab = Bv + (s + 1) * STAGE;
#pragma unroll
            for (int it = 0; it < P; ++it) pre[it] = slab[src[it]];
        }
        const f32x4* st = lds + cur * STAGE;
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            if (on[q]) {
                f32x4 a[2][2], b[2][2];
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    int ra = ti[q] * 64 + rb * 32 + l32;
                    int rbw = tj[q] * 64 + rb * 32 + l32;
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        int p = 2 * j + h;
                        a[rb][j] = st[ra * 4 + (p ^ ((ra >> 2) & 3))];
                        b[rb][j] = st[rbw * 4 + (p ^ ((rbw >> 2) & 3))];
                    }
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
#pragma unroll
                        for (int rb = 0; rb < 2; ++rb) {
                            float av = a[rb][j][c];
#pragma unroll
                            for (int cb = 0; cb < 2; ++cb) {
                                float bv = b[cb][j][c];
                                acc[q][rb][cb] = mfma32(av, bv, acc[q][rb][cb]);
                            }
                        }
                    }
                }
            }
        }
        if (more) {
            f32x4* nx = lds + (cur ^ 1) * STAGE;
#pragma unroll
            for (int it = 0; it < P; ++it) nx[it * 256 + tid] = pre[it];
        }
        __syncthreads();
    }

    // partial[group][tile][64 x 64]
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        if (!on[q]) continue;
        float* out = partial + ((int64_t)group * tiles + (tbase + q)) * 4096;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    int r = rb * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
                    int c = cb * 32 + l32;
                    out[r * 64 + c] = acc[q][rb][cb][i];
                }
    }
}

// C (NP x NP, fp64, both triangles) = sum over groups of the partial tiles, in group order.
__global__ __launch_bounds__(256) void gram_reduce_kernel(const float* __restrict__ partial, double* __restrict__ C,
                                                          int NP, int tiles, int groups) {
    int t = blockIdx.x;
    int e = blockIdx.y * 256 + threadIdx.x;  // 0..4095
    int ti, tj;
    tile_coords(t, ti, tj);
    int r = e >> 6, c = e & 63;
    if (ti == tj && c > r) return;  // the diagonal tiles hold both triangles; keep one
    double s = 0.0;
    for (int g = 0; g < groups; ++g) s += (double)partial[((int64_t)g * tiles + t) * 4096 + e];
    int gr = ti * 64 + r, gc = tj * 64 + c;
    C[(int64_t)gr * NP + gc] = s;
    C[(int64_t)gc * NP + gr] = s;
}

GramPlan gram_plan(const Dims& d, int num_cu) {
    GramPlan p;
    int P = d.NP / 64;
    p.tiles = P * (P + 1) / 2;
    p.wg_per_group = (p.tiles + 11) / 12;
    int g = (num_cu / p.wg_per_group) / 8 * 8;
    if (g < 8) g = 8;
    // keep at least 4 slabs per group so that tiny problems do not drown in partial tiles
    int64_t gmax = ((d.S + 3) / 4 + 7) / 8 * 8;
    if (gmax < 8) gmax = 8;
    if (g > gmax) g = (int)gmax;
    p.groups = g;
    p.slabs_per_group = (d.S + g - 1) / g;
    p.partial_floats = (size_t)g * p.tiles * 4096;
    return p;
}

hipError_t launch_gram(const float* B, float* partial, const GramPlan& p, const Dims& d, hipStream_t st) {
    dim3 grid((unsigned)(p.groups * p.wg_per_group));
    size_t lds = (size_t)2 * d.NP * 64;
    switch (d.NP / 64) {
#define SAGE_GRAM_CASE(PP)                                                                                          \
    case PP: {                                                                                                      \
        static bool attr_set = false;                                                                               \
        if (!attr_set) {                                                                                            \
            (void)hipFuncSetAttribute((const void*)gram_kernel<PP>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536);   \
            attr_set = true;                                                                                        \
        }                                                                                                           \
        hipLaunchKernelGGL(gram_kernel<PP>, grid, dim3(256), lds, st, B, partial, p.tiles, p.wg_per_group, d.S,     \
                           p.slabs_per_group);                                                                      \
    } break;
        SAGE_GRAM_CASE(1)
        SAGE_GRAM_CASE(2)
        SAGE_GRAM_CASE(4)
        SAGE_GRAM_CASE(8)
#undef SAGE_GRAM_CASE
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_gram_reduce(const float* partial, double* C, const GramPlan& p, const Dims& d, hipStream_t st) {
    hipLaunchKernelGGL(gram_reduce_kernel, dim3(p.tiles, 16), dim3(256), 0, st, partial, C, d.NP, p.tiles, p.groups);
    return hipGetLastError();
}

}  // namespace sage
