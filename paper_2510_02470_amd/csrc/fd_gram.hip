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

// P = NP / 64 row panels. Tiles t0 .. t0 + tiles - 1 of the row-major lower-triangle enumeration are computed (t0 > 0
// leaves out the leading panels whose Gram block the caller already knows). 256 threads = 4 waves; the unit of work is half a tile (32 rows x 64 columns, two
// 32x32 accumulators); a wave owns up to 3 units, a work-group 12 (6 tiles), and two work-groups share a CU so
// that one's LDS reads and barrier waits hide under the other's matrix-core work.
// Dynamic LDS: 2 stages x NP rows x 64 B, 16-byte pieces XOR-swizzled by (row/4)%4 so that the 16 rows read
// by a quarter wave fall in distinct banks.
// The buffer is two half buffers of LP = NP/2 rows each (same slab layout): `top` holds matrix rows 0 .. LP-1, `nw`
// matrix rows LP .. NP-1, of which only the first nfill hold data (the rest are taken as zero, whatever they hold).
// mode 0: tiles t0 .. t0+tiles-1 of the triangle; mode 1: the rectangle (new rows) x (top rows), tiles row-major;
// mode 2: the triangle of (new rows) x (new rows).
__device__ __forceinline__ void gram_tile(int mode, int P, int t0, int idx, int& ti, int& tj) {
    const int q = P >> 1;
    if (mode == 0) {
        tile_coords(t0 + idx, ti, tj);
    } else if (mode == 1) {
        ti = q + idx / q;
        tj = idx % q;
    } else {
        tile_coords(idx, ti, tj);
        ti += q;
        tj += q;
    }
}

template <int P>
__global__ __launch_bounds__(256, 2) void gram_kernel(const float* __restrict__ top, const float* __restrict__ nw,
                                                      int nfill, float* __restrict__ partial, int mode, int t0,
                                                      int tiles, int wg_per_group, int64_t slabs_total,
                                                      int64_t slabs_per_group) {
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
        if (on[q]) gram_tile(mode, P, t0, u >> 1, ti, tj);
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

    // staging map: slot ps = it*256 + tid holds (row = ps/4, logical piece = (ps%4) ^ ((row/4)%4)); the row comes from
    // the top half, the new half, or is zero
    constexpr int LP = NP / 2;
    constexpr int HALF4 = LP * 4;  // 16-byte pieces of one half buffer per slab
    int src[P];                    // piece index inside the half's slab, -1: zero row
    bool isnew[P];
#pragma unroll
    for (int it = 0; it < P; ++it) {
        int ps = it * 256 + tid;
        int row = ps >> 2;
        int p = (ps & 3) ^ ((row >> 2) & 3);
        isnew[it] = row >= LP;
        int hr = isnew[it] ? row - LP : row;
        src[it] = ((isnew[it] && hr >= nfill) || (mode == 2 && !isnew[it])) ? -1 : hr * 4 + p;  // mode 2 never reads top rows
    }
    const f32x4* Tv = reinterpret_cast<const f32x4*>(top);
    const f32x4* Nv = reinterpret_cast<const f32x4*>(nw);
    f32x4 pre[P];
    auto fetch = [&](int64_t sl) {
#pragma unroll
        for (int it = 0; it < P; ++it) {
            const f32x4* base = (isnew[it] ? Nv : Tv) + sl * HALF4;
            pre[it] = src[it] >= 0 ? base[src[it]] : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };

    if (s0 < s1) {
        fetch(s0);
#pragma unroll
        for (int it = 0; it < P; ++it) lds[it * 256 + tid] = pre[it];
    }
    __syncthreads();

    for (int64_t s = s0; s < s1; ++s) {
        const int cur = (int)((s - s0) & 1);
        const bool more = (s + 1 < s1);
        if (more) fetch(s + 1);
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

    // partial[group][tile - t0][64 x 64]; unit u covers rows (u & 1) * 32 .. + 32 of tile t0 + u / 2
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

// The (new rows) x (top rows) rectangle for NP = 512, with wider wave tiles than gram_kernel's: a wave owns 128 new rows
// x 64 top rows (8 accumulator tiles), so the 256 x 256 rectangle is exactly 8 wave tiles = 2 work-groups per column
// range -- no idle wave slots, a third less staging traffic than 3 work-groups, and 12 operand reads per 64
// matrix-core instructions instead of 18 per 48. Same staging, LDS layout and partial-tile output as gram_kernel
// in mode 1 (tile index (ti - 4) * 4 + tj).
__global__ __launch_bounds__(256, 2) void gram_cross8_kernel(const float* __restrict__ top, const float* __restrict__ nw,
                                                             int nfill, float* __restrict__ partial,
                                                             int64_t slabs_total, int64_t slabs_per_group) {
    constexpr int P = 8, NP = 512, LP = 256;
    constexpr int STAGE = NP * 4;
    constexpr int HALF4 = LP * 4;
    extern __shared__ f32x4 lds[];

    const int id = blockIdx.x;
    const int xcd = id & 7;
    const int y = id >> 3;
    const int w = y & 1;  // 2 work-groups per group
    const int group = (y >> 1) * 8 + xcd;
    int64_t s0 = (int64_t)group * slabs_per_group;
    int64_t s1 = s0 + slabs_per_group;
    if (s1 > slabs_total) s1 = slabs_total;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, h = lane >> 5;
    const int wt = w * 4 + wave;          // wave tile 0..7
    const int ag = wt >> 2, bg = wt & 3;  // new rows 128*ag .. + 128, top rows 64*bg .. + 64
    const int arow = LP + ag * 128 + l32; // + 32 * i, i < 4 (matrix row index: new half starts at LP)
    const int brow = bg * 64 + l32;       // + 32 * cb

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][b][e] = 0.f;

    int src[P];
#pragma unroll
    for (int it = 0; it < P; ++it) {
        int ps = it * 256 + tid;
        int row = ps >> 2;
        int p = (ps & 3) ^ ((row >> 2) & 3);
        int hr = row >= LP ? row - LP : row;
        src[it] = (row >= LP && hr >= nfill) ? -1 : hr * 4 + p;
    }
    const f32x4* Tv = reinterpret_cast<const f32x4*>(top);
    const f32x4* Nv = reinterpret_cast<const f32x4*>(nw);
    f32x4 pre[P];
    auto fetch = [&](int64_t sl) {
#pragma unroll
        for (int it = 0; it < P; ++it) {
            const f32x4* base = (it >= P / 2 ? Nv : Tv) + sl * HALF4;  // rows it*64 .. : the new half from it = 4 on
            pre[it] = src[it] >= 0 ? base[src[it]] : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };
    if (s0 < s1) {
        fetch(s0);
#pragma unroll
        for (int it = 0; it < P; ++it) lds[it * 256 + tid] = pre[it];
    }
    __syncthreads();

    for (int64_t s = s0; s < s1; ++s) {
        const int cur = (int)((s - s0) & 1);
        const bool more = (s + 1 < s1);
        if (more) fetch(s + 1);
        const f32x4* st = lds + cur * STAGE;
        f32x4 a[2][4], b[2][2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int p = 2 * j + h;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int ra = arow + 32 * i;
                a[j][i] = st[ra * 4 + (p ^ ((ra >> 2) & 3))];
            }
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const int rb = brow + 32 * cb;
                b[j][cb] = st[rb * 4 + (p ^ ((rb >> 2) & 3))];
            }
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads above: the scheduler would sink each next to its use
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb) acc[i][cb] = mfma32(a[j][i][c], b[j][cb][c], acc[i][cb]);
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
            f32x4* nx = lds + (cur ^ 1) * STAGE;
#pragma unroll
            for (int it = 0; it < P; ++it) nx[it * 256 + tid] = pre[it];
        }
        __syncthreads();
    }

    // tiles (ti - 4, tj) = (2*ag + i/2, bg); rows (i & 1) * 32 .. + 32 of the tile
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int tidx = (2 * ag + (i >> 1)) * 4 + bg;
        float* out = partial + ((int64_t)group * 16 + tidx) * 4096 + (i & 1) * 2048;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                int r = 8 * (e >> 2) + 4 * h + (e & 3);
                int c = cb * 32 + l32;
                out[r * 64 + c] = acc[i][cb][e];
            }
    }
}

// The same rectangle on the bf16 matrix cores: every fp32 value is written as three bf16 parts (24 significant bits)
// and the six products that matter (hi*hi, hi*mid, mid*hi, hi*lo, lo*hi, mid*mid) are accumulated in fp32 -- the
// fp32 result to a few 2^-24 per term, 6 x 32 cycles per 32 x 32 x 16 block instead of 8 x 64 on the fp32 matrix
// cores. One slab (16 columns) is exactly one k-step. The values are split when they are staged, once per
// work-group, so one work-group of 8 waves owns all 8 wave tiles of a column range (staging traffic is half of
// gram_cross8_kernel's, where two work-groups stage the same slabs). LDS holds a slab as [part][k-half][row] pieces
// of 16 bytes (8 bf16: the k-half of a row), 48 KB, double buffered; the 32 rows a matrix-core operand reads are
// 512 contiguous bytes. The next slab is split and stored piece by piece between the six groups of matrix-core
// instructions (all waves of a work-group run in step: conversions done in one block would leave the matrix cores
// idle), from registers that were loaded a stage earlier and are reloaded, for the slab after next, as soon as they
// have been consumed.
// NEW1: every new row in use is a bf16 value stored as fp32 (rows of a bf16 stream): its mid and lo parts are zero, so
// only its hi part is staged and only the three products with it are issued. The three left out would add exact
// zeros: the result has the same bits either way.
template <bool NEW1>
__global__ __launch_bounds__(512, 1) void gram_cross8_split_kernel(const float* __restrict__ top,
                                                                   const float* __restrict__ nw, int nfill,
                                                                   float* __restrict__ partial, int64_t slabs_total,
                                                                   int64_t slabs_per_group) {
    constexpr int NP = 512, LP = 256;
    constexpr int HALF4 = LP * 4;        // 16-byte pieces of a half buffer per slab
    constexpr int HREG = NP + 8;         // pieces per k-half region: the rows plus 128 bytes, so that the two regions a
                                         // staging store touches fall on different banks
    constexpr int PART16 = 2 * HREG;     // pieces per part: [k-half][row]
    constexpr int STAGE16 = 3 * PART16;  // 48.4 KB
    extern __shared__ u32x4 ldsx[];      // 2 * STAGE16

    const int id = blockIdx.x;
    const int xcd = id & 7;
    const int group = (id >> 3) * 8 + xcd;
    const int64_t s0 = (int64_t)group * slabs_per_group;
    int64_t s1 = s0 + slabs_per_group;
    if (s1 > slabs_total) s1 = slabs_total;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, h = lane >> 5;
    const int ag = wave >> 2, bg = wave & 3;  // new rows 128*ag .. + 128, top rows 64*bg .. + 64
    const int arow = LP + ag * 128 + l32;     // + 32 * i, i < 4
    const int brow = bg * 64 + l32;           // + 32 * cb

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][b][e] = 0.f;

    // staging: piece ps = it * 512 + tid is columns 4p .. 4p+3 of row ps >> 2 (rows >= LP: the new half)
    const f32x4* Tv = reinterpret_cast<const f32x4*>(top);
    const f32x4* Nv = reinterpret_cast<const f32x4*>(nw);
    int src[4], dst8[4];  // source piece in the half buffer (-1: a new row not in use), LDS offset in 8-byte units
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int ps = it * 512 + tid, row = ps >> 2, p = ps & 3;
        const int hr = row >= LP ? row - LP : row;
        src[it] = (row >= LP && hr >= nfill) ? -1 : hr * 4 + p;
        dst8[it] = (((p >> 1) * HREG + row) << 1) + (p & 1);
    }
    f32x4 pre[4];
    auto fetch1 = [&](int it, int64_t sl) __attribute__((always_inline)) {
        const int64_t sc = sl < s1 ? sl : s1 - 1;  // beyond the end: repeat (never used)
        const f32x4* base = (it >= 2 ? Nv : Tv) + sc * HALF4;
        pre[it] = src[it] >= 0 ? base[src[it]] : f32x4{0.f, 0.f, 0.f, 0.f};
    };
    auto store1 = [&](int it, int buf) __attribute__((always_inline)) {
        uint2* d = reinterpret_cast<uint2*>(ldsx + buf * STAGE16) + dst8[it];
        if (NEW1 && it >= 2) {  // new rows (pieces 1024 ..)
            d[0] = make_uint2(hi_bf16(pre[it][0], pre[it][1]), hi_bf16(pre[it][2], pre[it][3]));
            return;
        }
        unsigned a0, a1, a2, b0, b1, b2;
        split3_bf16(pre[it][0], pre[it][1], a0, a1, a2);
        split3_bf16(pre[it][2], pre[it][3], b0, b1, b2);
        d[0] = make_uint2(a0, b0);
        d[2 * PART16] = make_uint2(a1, b1);
        d[4 * PART16] = make_uint2(a2, b2);
    };
    if (s0 < s1) {
#pragma unroll
        for (int it = 0; it < 4; ++it) fetch1(it, s0);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            store1(it, 0);
            fetch1(it, s0 + 1);
        }
    }
    __syncthreads();

    constexpr int AP = NEW1 ? 1 : 3;  // parts of a new row
    constexpr int NQ = NEW1 ? 3 : 6;  // products
    for (int64_t s = s0; s < s1; ++s) {
        const int cur = (int)((s - s0) & 1);
        const u32x4* st = ldsx + cur * STAGE16 + h * HREG;
        u32x4 a[4][AP], b[2][3];
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            if (p < AP) {
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i][p] = st[p * PART16 + arow + 32 * i];
            }
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) b[cb][p] = st[p * PART16 + brow + 32 * cb];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {  // in the order the parts were read: the first group needs the hi parts only
            constexpr int PA[6] = {0, 0, 1, 1, 0, 2}, PB[6] = {0, 1, 0, 1, 2, 0};
            const int pa = NEW1 ? 0 : PA[q], pb = NEW1 ? q : PB[q];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) acc[i][cb] = mfma_bf16(a[i][pa], b[cb][pb], acc[i][cb]);
            // slab s + 1 into the other buffer, slab s + 2 on its way
            if (!NEW1 && q < 4) {
                store1(q, cur ^ 1);
                fetch1(q, s + 2);
            }
            if (NEW1) {
                store1(q, cur ^ 1);
                fetch1(q, s + 2);
                if (q == 2) {
                    store1(3, cur ^ 1);
                    fetch1(3, s + 2);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // the LDS stores above must be visible, the reads of this stage are consumed; the loads for slab s + 2 stay
        // in flight (a bare barrier: __syncthreads() would wait for them)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }

    // tiles (ti - 4, tj) = (2*ag + i/2, bg); rows (i & 1) * 32 .. + 32 of the tile
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int tidx = (2 * ag + (i >> 1)) * 4 + bg;
        float* out = partial + ((int64_t)group * 16 + tidx) * 4096 + (i & 1) * 2048;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                int r = 8 * (e >> 2) + 4 * h + (e & 3);
                int c = cb * 32 + l32;
                out[r * 64 + c] = acc[i][cb][e];
            }
    }
}

// The (new rows) x (new rows) triangle for NP = 512: 256 rows, i.e. 8 row blocks of 32 and 36 blocks (bi >= bj) of
// 32 x 32. Only the new rows are staged (16 KB per slab). The 36 blocks are dealt to the 4 waves, 9 each, so that a
// wave needs at most 6 operand rows-blocks per k-step: three 3 x 3 rectangles
//   rows {5,6,7} x {0,1,2},   rows {5,6,7} x {3,4,5},   rows {2,3,4} x {0,1,2},
// and the three 2 x 2 triangles on the diagonal that are left, {0,1}, {3,4}, {6,7} (on a diagonal block both
// operands are the same registers). No idle accumulators, 12 LDS reads per 72 matrix-core instructions. One
// work-group per column range; partial tiles in the layout of gram_kernel's mode 2 (the upper 32 x 32 block of a
// diagonal tile is not written and never read).
template <int W>
struct New8Map;
template <>
struct New8Map<0> {
    static constexpr int rows[6] = {5, 6, 7, 0, 1, 2};
    static constexpr int pa[9] = {0, 0, 0, 1, 1, 1, 2, 2, 2}, pb[9] = {3, 4, 5, 3, 4, 5, 3, 4, 5};
};
template <>
struct New8Map<1> {
    static constexpr int rows[6] = {5, 6, 7, 3, 4, 4};
    static constexpr int pa[9] = {0, 0, 0, 1, 1, 1, 2, 2, 2}, pb[9] = {3, 4, 0, 3, 4, 0, 3, 4, 0};
};
template <>
struct New8Map<2> {
    static constexpr int rows[6] = {2, 3, 4, 0, 1, 1};
    static constexpr int pa[9] = {0, 0, 0, 1, 1, 1, 2, 2, 2}, pb[9] = {3, 4, 0, 3, 4, 0, 3, 4, 0};
};
template <>
struct New8Map<3> {
    static constexpr int rows[6] = {0, 1, 3, 4, 6, 7};
    static constexpr int pa[9] = {0, 1, 1, 2, 3, 3, 4, 5, 5}, pb[9] = {0, 0, 1, 2, 2, 3, 4, 4, 5};
};

template <int W>
__device__ __forceinline__ void gram_new8_wave(const f32x4* __restrict__ Nv, int nfill, float* __restrict__ partial,
                                               int group, int64_t s0, int64_t s1, int64_t trips, f32x4* lds) {
    using M = New8Map<W>;
    constexpr int LP = 256, STAGE = LP * 4;
    const int tid = threadIdx.x & 255, lane = tid & 63;
    const int l32 = lane & 31, h = lane >> 5;

    f32x16 acc[9];
#pragma unroll
    for (int q = 0; q < 9; ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;

    int src[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int ps = it * 256 + tid;
        const int row = ps >> 2;
        const int p = (ps & 3) ^ ((row >> 2) & 3);
        src[it] = row >= nfill ? -1 : row * 4 + p;
    }
    f32x4 pre[4];
    auto fetch = [&](int64_t sl) {  // a slab beyond the range reads as zero
        const f32x4* base = Nv + sl * STAGE;
#pragma unroll
        for (int it = 0; it < 4; ++it) pre[it] = (src[it] >= 0 && sl < s1) ? base[src[it]] : f32x4{0.f, 0.f, 0.f, 0.f};
    };
    fetch(s0);
#pragma unroll
    for (int it = 0; it < 4; ++it) lds[it * 256 + tid] = pre[it];
    __syncthreads();

    for (int64_t t = 0; t < trips; ++t) {
        const int cur = (int)(t & 1);
        const bool more = (t + 1 < trips);
        if (more) fetch(s0 + t + 1);
        const f32x4* st = lds + cur * STAGE;
        f32x4 op[2][6];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int p = 2 * j + h;
#pragma unroll
            for (int o = 0; o < 6; ++o) {
                const int r = M::rows[o] * 32 + l32;
                op[j][o] = st[r * 4 + (p ^ ((r >> 2) & 3))];
            }
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads above: the scheduler would sink each next to its use
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int q = 0; q < 9; ++q) acc[q] = mfma32(op[j][M::pa[q]][c], op[j][M::pb[q]][c], acc[q]);
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
            f32x4* nx = lds + (cur ^ 1) * STAGE;
#pragma unroll
            for (int it = 0; it < 4; ++it) nx[it * 256 + tid] = pre[it];
        }
        __syncthreads();
    }

#pragma unroll
    for (int q = 0; q < 9; ++q) {
        const int bi = M::rows[M::pa[q]], bj = M::rows[M::pb[q]];
        const int ti = bi >> 1, tj = bj >> 1;
        float* out = partial + ((int64_t)group * 10 + ti * (ti + 1) / 2 + tj) * 4096 + (bi & 1) * 2048 + (bj & 1) * 32;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int r = 8 * (e >> 2) + 4 * h + (e & 3);
            out[r * 64 + l32] = acc[q][e];
        }
    }
}

// One work-group (4 waves, 32 KB of LDS) per column range, two per CU. Used when the launch has the chip to itself.
__global__ __launch_bounds__(256, 2) void gram_new8_kernel(const float* __restrict__ nw, int nfill,
                                                           float* __restrict__ partial, int64_t slabs_total,
                                                           int64_t slabs_per_group) {
    extern __shared__ f32x4 lds[];
    const int group = blockIdx.x;
    int64_t s0 = (int64_t)group * slabs_per_group;
    int64_t s1 = s0 + slabs_per_group;
    if (s1 > slabs_total) s1 = slabs_total;
    if (s0 > s1) s0 = s1;
    const f32x4* Nv = reinterpret_cast<const f32x4*>(nw);
    switch (threadIdx.x >> 6) {  // wave-uniform
        case 0: gram_new8_wave<0>(Nv, nfill, partial, group, s0, s1, s1 - s0, lds); break;
        case 1: gram_new8_wave<1>(Nv, nfill, partial, group, s0, s1, s1 - s0, lds); break;
        case 2: gram_new8_wave<2>(Nv, nfill, partial, group, s0, s1, s1 - s0, lds); break;
        default: gram_new8_wave<3>(Nv, nfill, partial, group, s0, s1, s1 - s0, lds); break;
    }
}

// The same triangle on the bf16 matrix cores with three-way split values (see gram_cross8_split_kernel): the new rows
// of a slab are split when they are staged ([part][k-half][row] pieces, 24 KB per stage), a wave's six operand row
// blocks are 18 LDS reads per 54 matrix-core instructions, and the next slab is split and stored between the six
// groups of matrix-core instructions. NEW1 (see gram_cross8_split_kernel): one part, one product.
template <int W, bool NEW1>
__device__ __forceinline__ void gram_new8_split_wave(const f32x4* __restrict__ Nv, int nfill, float* __restrict__ partial,
                                                     int group, int64_t s0, int64_t s1, u32x4* lds) {
    using M = New8Map<W>;
    constexpr int LP = 256, HALF4 = LP * 4;
    constexpr int HREG = LP + 8;         // pieces per k-half region (padded, see gram_cross8_split_kernel)
    constexpr int PART16 = 2 * HREG;     // pieces per part: [k-half][row]
    constexpr int STAGE16 = 3 * PART16;  // 24.4 KB
    const int tid = threadIdx.x & 255, lane = tid & 63;
    const int l32 = lane & 31, h = lane >> 5;

    f32x16 acc[9];
#pragma unroll
    for (int q = 0; q < 9; ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;

    int src[4], dst8[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int ps = it * 256 + tid, row = ps >> 2, p = ps & 3;
        src[it] = row >= nfill ? -1 : row * 4 + p;
        dst8[it] = (((p >> 1) * HREG + row) << 1) + (p & 1);
    }
    f32x4 pre[4];
    auto fetch1 = [&](int it, int64_t sl) __attribute__((always_inline)) {
        const int64_t sc = sl < s1 ? sl : s1 - 1;  // beyond the end: repeat (never used)
        pre[it] = src[it] >= 0 ? Nv[sc * HALF4 + src[it]] : f32x4{0.f, 0.f, 0.f, 0.f};
    };
    auto store1 = [&](int it, int buf) __attribute__((always_inline)) {
        uint2* d = reinterpret_cast<uint2*>(lds + buf * STAGE16) + dst8[it];
        if (NEW1) {
            d[0] = make_uint2(hi_bf16(pre[it][0], pre[it][1]), hi_bf16(pre[it][2], pre[it][3]));
            return;
        }
        unsigned a0, a1, a2, b0, b1, b2;
        split3_bf16(pre[it][0], pre[it][1], a0, a1, a2);
        split3_bf16(pre[it][2], pre[it][3], b0, b1, b2);
        d[0] = make_uint2(a0, b0);
        d[2 * PART16] = make_uint2(a1, b1);
        d[4 * PART16] = make_uint2(a2, b2);
    };
    if (s0 < s1) {
#pragma unroll
        for (int it = 0; it < 4; ++it) fetch1(it, s0);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            store1(it, 0);
            fetch1(it, s0 + 1);
        }
    }
    __syncthreads();

    for (int64_t s = s0; s < s1; ++s) {
        const int cur = (int)((s - s0) & 1);
        const u32x4* st = lds + cur * STAGE16 + h * HREG + l32;
        constexpr int NP3 = NEW1 ? 1 : 3, NQ = NEW1 ? 1 : 6;
        u32x4 op[6][NP3];
#pragma unroll
        for (int p = 0; p < NP3; ++p)
#pragma unroll
            for (int o = 0; o < 6; ++o) op[o][p] = st[p * PART16 + M::rows[o] * 32];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < NQ; ++k) {  // in the order the parts were read
            constexpr int PA[6] = {0, 0, 1, 1, 0, 2}, PB[6] = {0, 1, 0, 1, 2, 0};
#pragma unroll
            for (int q = 0; q < 9; ++q) acc[q] = mfma_bf16(op[M::pa[q]][PA[k]], op[M::pb[q]][PB[k]], acc[q]);
            if (NEW1) {
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    store1(it, cur ^ 1);
                    fetch1(it, s + 2);
                }
            } else if (k < 4) {
                store1(k, cur ^ 1);
                fetch1(k, s + 2);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the LDS stores; the loads for slab s + 2 stay in flight
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }

#pragma unroll
    for (int q = 0; q < 9; ++q) {
        const int bi = M::rows[M::pa[q]], bj = M::rows[M::pb[q]];
        const int ti = bi >> 1, tj = bj >> 1;
        float* out = partial + ((int64_t)group * 10 + ti * (ti + 1) / 2 + tj) * 4096 + (bi & 1) * 2048 + (bj & 1) * 32;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int r = 8 * (e >> 2) + 4 * h + (e & 3);
            out[r * 64 + l32] = acc[q][e];
        }
    }
}

template <bool NEW1>
__global__ __launch_bounds__(256, 2) void gram_new8_split_kernel(const float* __restrict__ nw, int nfill,
                                                                 float* __restrict__ partial, int64_t slabs_total,
                                                                 int64_t slabs_per_group) {
    extern __shared__ u32x4 ldsn[];
    const int group = blockIdx.x;
    int64_t s0 = (int64_t)group * slabs_per_group;
    int64_t s1 = s0 + slabs_per_group;
    if (s1 > slabs_total) s1 = slabs_total;
    if (s0 > s1) s0 = s1;
    const f32x4* Nv = reinterpret_cast<const f32x4*>(nw);
    switch (threadIdx.x >> 6) {  // wave-uniform
        case 0: gram_new8_split_wave<0, NEW1>(Nv, nfill, partial, group, s0, s1, ldsn); break;
        case 1: gram_new8_split_wave<1, NEW1>(Nv, nfill, partial, group, s0, s1, ldsn); break;
        case 2: gram_new8_split_wave<2, NEW1>(Nv, nfill, partial, group, s0, s1, ldsn); break;
        default: gram_new8_split_wave<3, NEW1>(Nv, nfill, partial, group, s0, s1, ldsn); break;
    }
}

// C (NP x NP, fp64, both triangles) = sum over groups of the partial tiles, in group order. With q = P/2:
// known_top: tiles with ti < q are not summed, their block is `known` (the top rows are the rows the last shrink
// wrote, whose Gram matrix it recorded: diagonal up to the tolerance of its eigensolve). Otherwise tile (ti, tj) comes from source A when its mode
// covers it, else from source B (mode-1 and mode-2 launches write separate partial buffers).
struct GramSrc {
    const float* partial;
    int mode, t0, tiles, groups;
};
__device__ __forceinline__ int gram_src_index(const GramSrc& g, int P, int t, int ti, int tj) {
    const int q = P >> 1;
    if (g.mode == 0) return (t >= g.t0 && t < g.t0 + g.tiles) ? t - g.t0 : -1;
    if (g.mode == 1) return (ti >= q && tj < q) ? (ti - q) * q + tj : -1;
    return (ti >= q && tj >= q) ? (ti - q) * (ti - q + 1) / 2 + (tj - q) : -1;
}
__global__ __launch_bounds__(256) void gram_reduce_kernel(GramSrc a, GramSrc b, double* __restrict__ C, int NP,
                                                          int known_top, const double* __restrict__ known) {
    const int P = NP / 64;
    int t = blockIdx.x;
    int e = blockIdx.y * 256 + threadIdx.x;  // 0..4095
    int ti, tj;
    tile_coords(t, ti, tj);
    int r = e >> 6, c = e & 63;
    if (ti == tj && c > r) return;  // the diagonal tiles hold both triangles; keep one
    int gr = ti * 64 + r, gc = tj * 64 + c;
    double s = 0.0;
    if (known_top && ti < (P >> 1)) {
        s = known[(int64_t)gr * (NP >> 1) + gc];
    } else {
        int ia = gram_src_index(a, P, t, ti, tj);
        const GramSrc& g = ia >= 0 ? a : b;
        int idx = ia >= 0 ? ia : gram_src_index(b, P, t, ti, tj);
        if (idx >= 0) {
            const float* p0 = g.partial + (int64_t)idx * 4096 + e;
            const int64_t gstride = (int64_t)g.tiles * 4096;
            int k = 0;
            for (; k + 8 <= g.groups; k += 8) {  // eight loads in flight, added in group order
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = p0[(k + u) * gstride];
#pragma unroll
                for (int u = 0; u < 8; ++u) s += (double)v[u];
            }
            for (; k < g.groups; ++k) s += (double)p0[k * gstride];
        }
    }
    C[(int64_t)gr * NP + gc] = s;
    C[(int64_t)gc * NP + gr] = s;
}

// wg_per_cu = 2 fills the chip. wg_per_cu = 1 is for the launch that shares the chip with the eigensolve (side
// stream): it also leaves 16 CUs (two per XCD) without any of its work-groups, because the eigensolve's pivot
// kernel needs more registers than remain on a CU that holds one of them.
GramPlan gram_plan(const Dims& d, int num_cu, int mode, bool skip_top, int wg_per_cu) {
    GramPlan p;
    const bool side = wg_per_cu == 1;
    const int P = d.NP / 64, q = P / 2;
    p.mode = mode;
    p.t0 = 0;
    if (mode == 0) {
        p.t0 = skip_top ? q * (q + 1) / 2 : 0;
        p.tiles = P * (P + 1) / 2 - p.t0;
    } else if (mode == 1) {
        p.tiles = (P - q) * q;
    } else {
        p.tiles = (P - q) * (P - q + 1) / 2;
    }
    p.wg_per_group = (p.tiles + 5) / 6;
    if (mode == 1 && P == 8) p.wg_per_group = 2;  // gram_cross8_kernel: 8 wave tiles of 128 x 64
    // gram_new8_kernel (the whole triangle in one work-group) when the launch has the chip to itself. Beside the
    // eigensolve the slower gram_kernel is the better neighbour: measured on one box, the eigensolve lost more time to
    // the denser kernel than the side stream gained (21.7 k rows/s against 22.8 k for the whole update at config 5).
    if (mode == 2 && P == 8 && !side) p.wg_per_group = 1;
    const int cus = side && num_cu > 32 ? num_cu - 16 : num_cu;
    int g = (wg_per_cu * cus / p.wg_per_group) / 8 * 8;
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

GramPlan gram_plan_split(const GramPlan& base, const Dims& d, int groups) {
    GramPlan p = base;
    const bool ok = d.NP == 512 && ((base.mode == 1 && base.tiles == 16) || (base.mode == 2 && base.tiles == 10));
    if (!ok) {
        p.tiles = 0;  // not available
        return p;
    }
    p.wg_per_group = 1;
    p.split = true;
    if (groups > 0) {
        int64_t gmax = ((d.S + 3) / 4 + 7) / 8 * 8;
        if (gmax < 8) gmax = 8;
        p.groups = groups > gmax ? (int)gmax : groups;
        p.slabs_per_group = (d.S + p.groups - 1) / p.groups;
        p.partial_floats = (size_t)p.groups * p.tiles * 4096;
    }
    return p;
}

hipError_t launch_gram(const float* top, const float* nw, int nfill, float* partial, const GramPlan& p, const Dims& d,
                       hipStream_t st, bool new_one) {
    if (p.tiles <= 0) return hipSuccess;
    dim3 grid((unsigned)(p.groups * p.wg_per_group));
    size_t lds = (size_t)2 * d.NP * 64;
    if (p.mode == 1 && d.NP == 512 && p.split) {
        constexpr int LDS_SPLIT = 2 * 3 * 2 * (512 + 8) * 16;  // two stages of [part][k-half][row + pad] pieces
        const void* kern = new_one ? (const void*)gram_cross8_split_kernel<true> : (const void*)gram_cross8_split_kernel<false>;
        if (hipError_t ea = ensure_dynamic_lds(kern, LDS_SPLIT); ea != hipSuccess) return ea;
        if (new_one)
            hipLaunchKernelGGL(gram_cross8_split_kernel<true>, grid, dim3(512), LDS_SPLIT, st, top, nw, nfill, partial, d.S,
                               p.slabs_per_group);
        else
            hipLaunchKernelGGL(gram_cross8_split_kernel<false>, grid, dim3(512), LDS_SPLIT, st, top, nw, nfill, partial,
                               d.S, p.slabs_per_group);
        return hipGetLastError();
    }
    if (p.mode == 1 && d.NP == 512) {
        if (hipError_t ea = ensure_dynamic_lds((const void*)gram_cross8_kernel, 65536); ea != hipSuccess) return ea;
        hipLaunchKernelGGL(gram_cross8_kernel, grid, dim3(256), lds, st, top, nw, nfill, partial, d.S, p.slabs_per_group);
        return hipGetLastError();
    }
    if (p.mode == 2 && d.NP == 512 && p.split) {
        // 49.5 KB are used; 64 KB are asked for, so that the eigensolve's pivot kernel (which asks for 100 KB for this
        // purpose) never shares a CU with one of these work-groups when the launch runs beside it
        constexpr int LDS_SPLIT = 65536;
        static_assert(2 * 3 * 2 * (256 + 8) * 16 <= LDS_SPLIT, "two stages must fit");
        if (new_one)
            hipLaunchKernelGGL(gram_new8_split_kernel<true>, grid, dim3(256), LDS_SPLIT, st, nw, nfill, partial, d.S,
                               p.slabs_per_group);
        else
            hipLaunchKernelGGL(gram_new8_split_kernel<false>, grid, dim3(256), LDS_SPLIT, st, nw, nfill, partial, d.S,
                               p.slabs_per_group);
        return hipGetLastError();
    }
    if (p.mode == 2 && d.NP == 512 && p.wg_per_group == 1) {
        if (hipError_t ea = ensure_dynamic_lds((const void*)gram_new8_kernel, 65536); ea != hipSuccess) return ea;
        hipLaunchKernelGGL(gram_new8_kernel, grid, dim3(256), 32768, st, nw, nfill, partial, d.S, p.slabs_per_group);
        return hipGetLastError();
    }
    switch (d.NP / 64) {
#define SAGE_GRAM_CASE(PP)                                                                                          \
    case PP: {                                                                                                      \
        if (hipError_t ea = ensure_dynamic_lds((const void*)gram_kernel<PP>, 65536); ea != hipSuccess) return ea;   \
        hipLaunchKernelGGL(gram_kernel<PP>, grid, dim3(256), lds, st, top, nw, nfill, partial, p.mode, p.t0, p.tiles,    \
                           p.wg_per_group, d.S, p.slabs_per_group);                                                 \
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

// a, b: the launches whose partial tiles make up C (b may be null); known: LP x LP doubles, read when known_top
hipError_t launch_gram_reduce(const float* partial_a, const GramPlan& a, const float* partial_b, const GramPlan* b,
                              double* C, bool known_top, const double* known, const Dims& d, hipStream_t st) {
    const int P = d.NP / 64;
    GramSrc sa{partial_a, a.mode, a.t0, a.tiles, a.groups};
    GramSrc sb{partial_b, b ? b->mode : 0, b ? b->t0 : 0, b ? b->tiles : 0, b ? b->groups : 0};
    hipLaunchKernelGGL(gram_reduce_kernel, dim3(P * (P + 1) / 2, 16), dim3(256), 0, st, sa, sb, C, d.NP, known_top ? 1 : 0,
                       known);
    return hipGetLastError();
}

}  // namespace sage
