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

// P = NP / 64 row panels. 256 threads = 4 waves; the unit of work is half a tile (32 rows x 64 columns, two
// 32x32 accumulators); a wave owns up to 3 units, a work-group 12 (6 tiles), and two work-groups share a CU so
// that one's LDS reads and barrier waits hide under the other's matrix-core work.
// Dynamic LDS: 2 stages x NP rows x 64 B, 16-byte pieces XOR-swizzled by (row/4)%4 so that the 16 rows read
// by a quarter wave fall in distinct banks.
template <int P>
__global__ __launch_bounds__(256, 2) void gram_kernel(const float* __restrict__ B, float* __restrict__ partial, int tiles,
                                                      int wg_per_group, int64_t slabs_total, int64_t slabs_per_group) {
    constexpr int NP = P * 64;
    constexpr int STAGE = NP * 4;  // 16-byte pieces per stage
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

    // unit u = 2 * tile + row half
    int arow[3], brow[3];
    bool on[3];
    const int ubase = (w * 4 + wave) * 3;
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        int u = ubase + q;
        on[q] = u < 2 * tiles;
        int ti = 0, tj = 0;
        if (on[q]) tile_coords(u >> 1, ti, tj);
        arow[q] = ti * 64 + (u & 1) * 32 + l32;
        brow[q] = tj * 64 + l32;
    }

    f32x16 acc[3][2];
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[q][b][i] = 0.f;

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
        // operands of the whole stage are fetched up front, first the pieces of k-half 0 for every unit, then those of
        // k-half 1, which land while the matrix cores work on half 0 (units that are switched off read rows that
        // exist and are simply not written back, so the stage is one straight-line block)
        f32x4 a[2][3], b[2][3][2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int p = 2 * j + h;
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const int ra = arow[q];
                a[j][q] = st[ra * 4 + (p ^ ((ra >> 2) & 3))];
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    const int rb = brow[q] + cb * 32;
                    b[j][q][cb] = st[rb * 4 + (p ^ ((rb >> 2) & 3))];
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads above: the scheduler would sink each next to its use
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int q = 0; q < 3; ++q)
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb) acc[q][cb] = mfma32(a[j][q][c], b[j][q][cb][c], acc[q][cb]);
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
            f32x4* nx = lds + (cur ^ 1) * STAGE;
#pragma unroll
            for (int it = 0; it < P; ++it) nx[it * 256 + tid] = pre[it];
        }
        __syncthreads();
    }

    // partial[group][tile][64 x 64]; unit u covers rows (u & 1) * 32 .. + 32 of tile u / 2
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        if (!on[q]) continue;
        const int u = ubase + q;
        float* out = partial + ((int64_t)group * tiles + (u >> 1)) * 4096 + (u & 1) * 2048;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int r = 8 * (i >> 2) + 4 * h + (i & 3);
                int c = cb * 32 + l32;
                out[r * 64 + c] = acc[q][cb][i];
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
    p.wg_per_group = (p.tiles + 5) / 6;
    int g = (2 * num_cu / p.wg_per_group) / 8 * 8;  // two work-groups per CU
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
