// Scoring pass projection on the bf16 matrix cores with a split basis (Algorithm 1, Phase II, first line:
// z_i = V_k^T g_i; Method, "Two-pass scoring").
//
// At k = 128 the projection does 2k/e = 64..128 flop per byte of input row, far above what the fp32 matrix
// cores sustain per byte of HBM traffic, so the fp32 kernel in score.hip is compute-bound at a small fraction of
// the memory bandwidth. Here every fp32 basis entry is written as v = hi + lo with hi = bf16(v), lo = bf16(v - hi)
// (|v - hi - lo| <= 2^-17 |v|), bf16 rows are used as they are (exact), fp32 rows are split the same way in
// registers, and the products g*hi, g*lo (and glo*hi for fp32 rows) are accumulated in fp32 by
// v_mfma_f32_32x32x16_bf16. The error against an fp32 product is a few 2^-17 relative per term, below the fp32
// accumulation error over D ~ 1e6 terms.
//
// Work-group = 256 threads = 4 waves, two work-groups per CU. A wave owns 64 batch rows x KP basis columns
// (2 x KP/32 accumulator tiles). Its row operand comes straight from global memory into registers (nobody else
// needs those rows; a lane reads 16-byte pieces and over one chunk consumes whole 128-byte lines); the basis
// operand is shared by the 4 waves and is streamed through LDS with direct global->LDS loads, double buffered.
// The basis is kept in HBM as "images": for each chunk of KC columns exactly the bytes LDS will hold, so staging
// is a linear copy.
#include "sage_internal.h"

namespace sage {

// ---- basis images -----------------------------------------------------------------------------------------
// Chunk c covers columns c*KC .. c*KC + KC - 1 (KC = 64 for bf16 rows, 32 for fp32 rows: 128 bytes of a row).
// Its image has 2*KP rows of KC bf16: image row cc < KP is hi(v_cc), image row KP + cc is lo(v_cc). A row is cut
// into 16-byte pieces (8 columns); piece p of image row cc is stored at position swz(cc, p) of that row so that the
// lanes of a matrix-core operand read (32 consecutive image rows, one piece each) spread over all LDS banks. A
// 16-byte read is served 16 lanes at a time from 64 banks of 4 bytes (256 bytes), so the 16 pieces that 16
// consecutive image rows ask for must fall on 16 different 16-byte columns modulo 256 bytes:
//   KC = 64 (8 pieces, 128 B rows: even and odd rows are 128 bytes apart): swz = p ^ ((cc >> 1) & 7);
//   KC = 32 (4 pieces,  64 B rows: four rows span 256 bytes):              swz = p ^ ((cc >> 2) & 3).
// (With swz = p ^ (cc & 7), conflict-free for 8 lanes over 32 banks, the hardware counters showed one conflict
// cycle for every useful cycle of the operand reads.)
template <int KC>
__device__ __forceinline__ int img_piece(int cc, int p) {
    if constexpr (KC == 64) return cc * 8 + (p ^ ((cc >> 1) & 7));
    else return cc * 4 + (p ^ ((cc >> 2) & 3));
}

// One thread writes one 16-byte piece. Vblk is the fp32 column-slab basis (KP rows); columns >= D are zero there and
// columns >= Dp are written as zero here.
template <int KC>
__global__ __launch_bounds__(256) void basis_split_kernel(const float* __restrict__ Vblk, int KP, int64_t Dp,
                                                          int64_t chunks, u32x4* __restrict__ img) {
    constexpr int PPR = KC / 8;
    const int64_t per_chunk = (int64_t)2 * KP * PPR;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= chunks * per_chunk) return;
    const int64_t c = i / per_chunk;
    const int rem = (int)(i % per_chunk);
    const int cc = rem / PPR, p = rem % PPR;
    const int row = cc < KP ? cc : cc - KP;
    const int64_t d0 = c * KC + p * 8;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = 0.f;
    if (d0 < Dp) {  // 8 | DC: the piece lies inside one slab
        const float* src = Vblk + blk_off(d0, row, KP);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = src[e];
    }
    u32x4 out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float x = v[2 * e], y = v[2 * e + 1];
        unsigned hi = pack_bf16(x, y);
        if (cc < KP) {
            out[e] = hi;
        } else {
            float rx = x - __uint_as_float(hi << 16), ry = y - __uint_as_float(hi & 0xffff0000u);
            out[e] = pack_bf16(rx, ry);
        }
    }
    img[c * per_chunk + img_piece<KC>(cc, p)] = out;
}

hipError_t launch_basis_split(const float* Vblk, int KP, int dtype, void* img, const Dims& d, hipStream_t st) {
    const int KC = dtype == SAGE_BF16 ? 64 : 32;
    const int64_t chunks = (d.D + KC - 1) / KC;
    const int64_t total = chunks * 2 * KP * (KC / 8);
    dim3 grid((unsigned)((total + 255) / 256));
    if (KC == 64)
        hipLaunchKernelGGL(basis_split_kernel<64>, grid, dim3(256), 0, st, Vblk, KP, d.Dp, chunks, (u32x4*)img);
    else
        hipLaunchKernelGGL(basis_split_kernel<32>, grid, dim3(256), 0, st, Vblk, KP, d.Dp, chunks, (u32x4*)img);
    return hipGetLastError();
}

size_t basis_image_bytes(int KP, int dtype, const Dims& d) {
    const int KC = dtype == SAGE_BF16 ? 64 : 32;
    const int64_t chunks = (d.D + KC - 1) / KC;
    return (size_t)chunks * 2 * KP * KC * 2;
}

// ---- projection -------------------------------------------------------------------------------------------
// fp32 pieces (8 values in two u32x4) -> bf16 hi and lo operands
__device__ __forceinline__ void split8(const u32x4& x0, const u32x4& x1, u32x4& hi, u32x4& lo) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const u32x4& s = e < 2 ? x0 : x1;
        float x = __uint_as_float(s[(2 * e) & 3]), y = __uint_as_float(s[(2 * e + 1) & 3]);
        unsigned hh = pack_bf16(x, y);
        hi[e] = hh;
        lo[e] = pack_bf16(x - __uint_as_float(hh << 16), y - __uint_as_float(hh & 0xffff0000u));
    }
}

// Rows of a batch are D * sizeof(T) bytes apart, which in general is not a multiple of the 128-byte memory line, so a
// row's k-th 128 bytes straddle two lines and a kernel that walks every row in steps of 128 bytes from the row
// start fetches most lines twice. Here a wave only holds rows whose start addresses are congruent modulo 128 (rows
// w, w + 8, w + 16, ... of the work-group's 512: 8 * pitch is a multiple of 128 because the pitch is a multiple of 16)
// and walks them in line-aligned windows: with phi = (row address mod 128) / (bytes of 8 columns), window m of the
// wave is the 128 bytes that start 8*phi columns before column m*KC. Its basis operand is then the last phi pieces
// of image m-1 followed by the first PPR-phi pieces of image m, so LDS keeps a ring of four images: m-1 and m in
// use, m+1 and m+2 on their way in (an image requested only one window ahead arrived late: with the memory system
// saturated a load takes about two windows). The first and the last window of a split reach into the neighbouring
// splits; those pieces of the row operand are zeroed.
//
// Work-group = 512 threads = 8 waves (two per SIMD), one per CU, 512 batch rows x KP basis columns; a wave owns 64
// rows (2 accumulator row tiles) x KP columns. Row operands go straight from global memory to registers, the pieces
// of window m+2 being requested at the start of window m; images are streamed with direct global->LDS loads, also
// two windows ahead.
template <typename T>
struct RowOp {
    u32x4 v[4];  // bf16 rows: v[j] = k-step j; fp32 rows: v[2j], v[2j+1] = k-step j
};

template <int NT, typename T>  // NT = KP / 32
__global__ __launch_bounds__(512, 1) void project_split_kernel(const T* __restrict__ G, int64_t R,
                                                               const u32x4* __restrict__ img,
                                                               float* __restrict__ partial, int row_tiles, int64_t D,
                                                               int64_t chunks_total, int64_t chunks_per_split) {
    constexpr int KP = NT * 32;
    constexpr int KC = 128 / (int)sizeof(T);
    constexpr int PPR = KC / 8;        // pieces (8 columns) per window
    constexpr int PB = 8 * (int)sizeof(T);  // bytes of a piece in a row: 16 or 32
    constexpr int IMG = 2 * KP * PPR;  // 16-byte pieces per image
    constexpr int KS = KC / 16;        // matrix-core k-steps per window
    extern __shared__ u32x4 lds[];     // 4 * IMG

    const int id = blockIdx.x;
    const int xcd = id & 7, y = id >> 3;
    const int rt = y % row_tiles;
    const int split = (y / row_tiles) * 8 + xcd;
    const int64_t c0 = (int64_t)split * chunks_per_split;
    int64_t c1 = c0 + chunks_per_split;
    if (c1 > chunks_total) c1 = chunks_total;
    const int64_t nc = c1 - c0;
    const int64_t nv = nc > 0 ? nc + 1 : 0;  // windows c0 .. c1

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int64_t S = D * (int64_t)sizeof(T);  // row pitch in bytes
    const int64_t row0 = (int64_t)rt * 512;
    // phase of this wave's rows, in pieces
    const int phi = (int)(((reinterpret_cast<uintptr_t>(G) + (uintptr_t)((row0 + wave) * S)) & 127) / PB);

    // Lane offsets are taken from gbase = (first row of the work-group) - 128 bytes, so that they are never negative;
    // every offset is clamped to its own row, so no lane reads outside the batch (pieces outside the row meet zeros
    // of the image or are zeroed below). Rows >= R repeat row R-1; their results are not written.
    const char* gbase = reinterpret_cast<const char*>(G) + row0 * S - 128;
    unsigned lbase[2];
    const unsigned back = (unsigned)(PB * phi) - (unsigned)(PB * h);  // lbase - back = offset of the row's first byte
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        int64_t r = row0 + wave + 8 * (t * 32 + n);
        if (r > R - 1) r = R - 1;
        lbase[t] = (unsigned)((r - row0) * S) + 128u - back;
    }
    // piece x of window m for row tile t
    auto load_piece = [&](RowOp<T>& a, int t, int64_t m, int x) __attribute__((always_inline)) {
        const int xoff = sizeof(T) == 2 ? 32 * x : 64 * (x >> 1) + 16 * (x & 1);
        const unsigned lo = lbase[t] + back, hi = lo + (unsigned)S - 16u;
        unsigned o = lbase[t] + (unsigned)(m * 128) + (unsigned)xoff;
        o = o < lo ? lo : o;
        o = o > hi ? hi : o;
        a.v[x] = *reinterpret_cast<const u32x4*>(gbase + o);
    };
    // LDS piece index (inside one image, column tile 0) of this lane's basis operand for k-step j, and whether it
    // lies in the previous image
    int boff[KS];
    bool prev[KS];
#pragma unroll
    for (int j = 0; j < KS; ++j) {
        const int q = 2 * j + h;
        prev[j] = q < phi;
        boff[j] = img_piece<KC>(n, (q - phi) & (PPR - 1));
    }

    f32x16 acc[2][NT];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][ct][i] = 0.f;

    auto image_of = [&](int64_t c) {  // images outside the matrix repeat the nearest one (finite data, never counted)
        return c < 0 ? (int64_t)0 : (c > chunks_total - 1 ? chunks_total - 1 : c);
    };
    auto stage = [&](int64_t c, int slot) __attribute__((always_inline)) {
        const u32x4* src = img + image_of(c) * IMG + tid;
#pragma unroll
        for (int q = 0; q < IMG / 512; ++q)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + q * 512),
                                             (__attribute__((address_space(3))) void*)(lds + slot * IMG + q * 512 + wave * 64),
                                             16, 0, 0);
        if constexpr (IMG % 512 != 0) {  // IMG = 256 (KP = 32, fp32 rows): half a round; waves 4..7 repeat it, so that
                                         // every wave has the same number of loads in flight (the wait below counts)
            const u32x4* src2 = img + image_of(c) * IMG + (tid & 255);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src2),
                                             (__attribute__((address_space(3))) void*)(lds + slot * IMG + (wave & 3) * 64), 16,
                                             0, 0);
        }
    };
    constexpr int VL = (IMG + 511) / 512;  // image loads per wave and window

    // One window. Step s = (k-step j, column tile ct) in order; the basis operand of step s + 1 is fetched from LDS
    // before the matrix-core instructions of step s are issued, and the scheduler may not move anything across a
    // step (left alone it hoists a whole window of LDS reads and spills). The ring has four slots, image c in slot
    // c mod 4: m-1 and m are read, m+1 has landed or is landing, m+2 is requested now. a: row operand of this window;
    // afar: buffer that receives window m+2.
    auto visit = [&](RowOp<T> (&a)[2], RowOp<T> (&afar)[2], int64_t m) __attribute__((always_inline)) {
        const int sp = (int)((m - 1) & 3), sc = (int)(m & 3);
        stage(m + 2, (int)((m + 2) & 3));
        // The row loads of window m+2 go out in two bursts, row tile 0 now and row tile 1 half way through the window
        // (measured: 12% faster than one burst of 8). Within a burst the four pieces of a line are asked for back to
        // back, while the line is still on its way or fresh in the vector cache.
        const int64_t m2 = m + 2 > c1 ? c1 : m + 2;  // beyond the last window: repeat it (never used)
#pragma unroll
        for (int x = 0; x < 4; ++x) load_piece(afar[0], 0, m2, x);
        if (m == c0 || m == c1) {
            const bool first = m == c0, last = m == c1;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int q = 2 * (sizeof(T) == 2 ? x : (x >> 1)) + h;
                    if ((first && q < phi) || (last && q >= phi)) a[t].v[x] = u32x4{0u, 0u, 0u, 0u};
                }
        }
        int baddr[KS];
#pragma unroll
        for (int j = 0; j < KS; ++j) baddr[j] = boff[j] + (prev[j] ? sp : sc) * IMG;
        constexpr int STEPS = KS * 2 * NT;
        u32x4 b[2];
        b[0] = lds[baddr[0]];
        u32x4 ahi[2], alo[2];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const int j = s / (2 * NT), ct = s % (2 * NT);
            if (ct == 0) {
                if constexpr (sizeof(T) == 2) {
                    ahi[0] = a[0].v[j];
                    ahi[1] = a[1].v[j];
                } else {
                    split8(a[0].v[2 * j], a[0].v[2 * j + 1], ahi[0], alo[0]);
                    split8(a[1].v[2 * j], a[1].v[2 * j + 1], ahi[1], alo[1]);
                }
            }
            if (s + 1 < STEPS) {
                const int j2 = (s + 1) / (2 * NT), ct2 = (s + 1) % (2 * NT);
                b[(s + 1) % 2] = lds[baddr[j2] + ct2 * 32 * PPR];
            }
            if (s == STEPS / 2) {
#pragma unroll
                for (int x = 0; x < 4; ++x) load_piece(afar[1], 1, m2, x);
            }
            const u32x4 bb = b[s % 2];
#pragma unroll
            for (int t = 0; t < 2; ++t) acc[t][ct % NT] = mfma_bf16(ahi[t], bb, acc[t][ct % NT]);
            if constexpr (sizeof(T) == 4) {
                if (ct < NT) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) acc[t][ct] = mfma_bf16(alo[t], bb, acc[t][ct]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // This window requested VL image loads (image m+2) and 8 row loads (window m+2): once at most 8 + VL loads are
        // outstanding, image m+1 and the rows of window m+1 (and every older load) have landed; both were requested a
        // whole window earlier. A bare barrier: __syncthreads() carries a release fence, which on this target drains
        // every outstanding load and would throw the prefetch distance away. The LDS reads of this window have all
        // been consumed by matrix-core instructions above.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0x0F70 | (8 + VL));  // vmcnt(8 + VL); expcnt, lgkmcnt not waited for
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };

    // The windows of a split are walked from a start that differs from split to split and wrap around: work-groups
    // that all start at the first window of their split march over memory in lock step, a regular pattern that left
    // some memory channels idle (5.1 TB/s for the row stream alone against 6.2 TB/s with rotated starts). The two row
    // tiles of a split keep the same start, so that they still share the basis images through L2. A run of
    // consecutive windows needs the ring primed with the images around its first window, so the walk is two runs.
    RowOp<T> a0[2], a1[2], a2[2];
    // (always_inline: called twice, the compiler otherwise makes the fp32-row instance a real function with the
    // accumulators in scratch memory)
    auto run = [&](int64_t ms, int64_t len) __attribute__((always_inline)) {
        stage(ms - 1, (int)((ms - 1) & 3));
        stage(ms, (int)(ms & 3));
        stage(ms + 1, (int)((ms + 1) & 3));
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                load_piece(a0[t], t, ms, x);
                load_piece(a1[t], t, ms + 1, x);
            }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        // three windows per trip: the row buffers return to their roles
        int64_t i = 0;
        for (; i + 2 < len; i += 3) {
            visit(a0, a2, ms + i);
            visit(a1, a0, ms + i + 1);
            visit(a2, a1, ms + i + 2);
        }
        if (i < len) visit(a0, a2, ms + i);
        if (i + 1 < len) visit(a1, a0, ms + i + 1);
    };
    if (nv > 0) {
        const int64_t rot = nv >= 8 ? (int64_t)(((unsigned)split * 37u) % (unsigned)(nv - 4)) + 2 : 0;  // 2 .. nv - 3
        run(c0 + rot, nv - rot);
        if (rot > 0) run(c0, rot);
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing on its way to LDS when the work-group ends
    }

    float* out = partial + (int64_t)split * R * KP;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t r = row0 + wave + 8 * (t * 32 + 8 * (i >> 2) + 4 * h + (i & 3));
                if (r < R) out[r * KP + ct * 32 + n] = acc[t][ct][i];
            }
}

// Every row must start on a multiple of the bytes of 8 columns (16 for bf16, 32 for fp32 rows), hold at least one
// chunk, and 512 rows plus a line must span < 4 GiB (lane offsets are 32-bit).
bool split_path_ok(const void* G, int dtype, const Dims& d) {
    const int64_t esz = dtype == SAGE_BF16 ? 2 : 4;
    const int64_t KC = 128 / esz;
    return d.D % 8 == 0 && d.D >= KC && d.D * esz * 513 + 256 < ((int64_t)1 << 32) && ((uintptr_t)G) % (8 * esz) == 0;
}

ScorePlan score_split_plan(int64_t R, int dtype, const Dims& d, int num_cu) {
    ScorePlan p;
    const int KC = dtype == SAGE_BF16 ? 64 : 32;
    const int64_t chunks = (d.D + KC - 1) / KC;
    p.row_tiles = (int)((R + 511) / 512);
    int64_t want = ((int64_t)num_cu + p.row_tiles - 1) / p.row_tiles;  // one work-group per CU
    int64_t s = (want + 7) / 8 * 8;
    int64_t smax = ((chunks + 7) / 8 + 7) / 8 * 8;  // at least ~8 chunks per split
    if (s > smax) s = smax;
    if (s < 8) s = 8;
    if (s > 512) s = 512;
    p.splits = (int)s;
    p.slabs_per_split = (chunks + s - 1) / s;  // chunks per split on this path
    return p;
}

template <int NT, typename T>
static hipError_t launch_split_t(const T* G, int64_t R, const void* img, float* partial, const ScorePlan& p,
                                 const Dims& d, hipStream_t st) {
    constexpr int KC = 128 / (int)sizeof(T);
    constexpr size_t LDS = (size_t)4 * 2 * NT * 32 * (KC / 8) * 16;
    if (hipError_t ea = ensure_dynamic_lds((const void*)project_split_kernel<NT, T>, (int)LDS); ea != hipSuccess) return ea;
    const int64_t chunks = (d.D + KC - 1) / KC;
    dim3 grid((unsigned)(p.row_tiles * p.splits));
    hipLaunchKernelGGL((project_split_kernel<NT, T>), grid, dim3(512), LDS, st, G, R, (const u32x4*)img, partial,
                       p.row_tiles, d.D, chunks, p.slabs_per_split);
    return hipGetLastError();
}

template <int NT>
static hipError_t launch_split_nt(const void* G, int dtype, int64_t R, const void* img, float* partial,
                                  const ScorePlan& p, const Dims& d, hipStream_t st) {
    if (dtype == SAGE_BF16) return launch_split_t<NT, uint16_t>((const uint16_t*)G, R, img, partial, p, d, st);
    return launch_split_t<NT, float>((const float*)G, R, img, partial, p, d, st);
}

hipError_t launch_project_split(const void* G, int dtype, int64_t R, const void* img, int KP, float* partial,
                                const ScorePlan& p, const Dims& d, hipStream_t st) {
    switch (KP / 32) {
        case 1: return launch_split_nt<1>(G, dtype, R, img, partial, p, d, st);
        case 2: return launch_split_nt<2>(G, dtype, R, img, partial, p, d, st);
        case 4: return launch_split_nt<4>(G, dtype, R, img, partial, p, d, st);
        default: return hipErrorInvalidValue;
    }
}


// ---- projection of factored rows ----------------------------------------------------------------------------
// A per-example gradient of a linear last layer (weights C x dh, bias C) under a loss on the logits is the outer
// product of the logit error e_i (C values) with [h_i; 1] (dh features and a one): column c*dh + t of row i is
// e_ic * h_it, column C*dh + c is e_ic (Method, definition of g_i, for that layer). The row is never stored: the
// kernel below forms the row operand of a window (KC columns of class c starting at feature tw*KC) from 128 bytes of
// h_i and the value e_ic, rounds it as a stored row of the context's type would have been rounded (bf16: nearest
// even; fp32: the fp32 product, then split as above) and multiplies it with the same basis images. The C bias
// columns are added by project_bias_kernel into a partial slot of their own.
//
// A split is a block of classes x feature windows and is walked feature window by feature window, classes inside:
// the 128 bytes of h_i stay in registers for all classes of the split, and per window only the image and one value of
// e per row are fetched (e comes from a transposed copy, so that the 32 rows of a tile read 32 neighbouring values).
// From HBM the kernel reads little more than the images, once. (Walking the columns in their order instead re-reads
// the feature rows for every class; they do not stay in L2 beside the image stream, and that variant ran at the
// speed of the row-major kernel.)
//
// Work-group and wave shapes as in project_split_kernel (512 threads, 512 rows; a wave owns rows 64w .. 64w+63).
// Every window is a whole image, so the ring has three slots: the window's image in use, the next landed or landing,
// the one after requested.
struct OuterGeom {
    int C, dh;
    int class_groups, classes_per_group;  // split -> (class group, window group): split % class_groups, split / ...
    int window_groups, windows_per_group;
    int64_t et_pitch;                     // elements between classes in the transposed error matrix
};

template <int NT, typename T>
__global__ __launch_bounds__(512, 1) void project_outer_kernel(const T* __restrict__ Et, const T* __restrict__ H,
                                                               int64_t R, OuterGeom g, const u32x4* __restrict__ img,
                                                               float* __restrict__ partial, int row_tiles) {
    constexpr int KP = NT * 32;
    constexpr int KC = 128 / (int)sizeof(T);
    constexpr int PPR = KC / 8;
    constexpr int PB = 8 * (int)sizeof(T);
    constexpr int IMG = 2 * KP * PPR;
    constexpr int KS = KC / 16;
    extern __shared__ u32x4 lds[];  // 3 * IMG

    const int id = blockIdx.x;
    const int xcd = id & 7, y = id >> 3;
    const int rt = y % row_tiles;
    const int split = (y / row_tiles) * 8 + xcd;
    const int cpc = g.dh / KC;  // windows per class
    const int kg = split % g.class_groups, tg = split / g.class_groups;
    const int k0 = kg * g.classes_per_group;
    int k1 = k0 + g.classes_per_group;
    if (k1 > g.C) k1 = g.C;
    int t0 = tg * g.windows_per_group, t1 = t0 + g.windows_per_group;
    if (t1 > cpc) t1 = cpc;
    if (tg >= g.window_groups) t1 = t0;  // padding splits: nothing to do, their slot is zero
    const int nk = k1 > k0 ? k1 - k0 : 0;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int64_t row0 = (int64_t)rt * 512;
    // Rows >= R repeat row R-1 for the features; the transposed errors are padded to whole row tiles. Results of such
    // rows are not written.
    const char* hrow[2];
    const T* ecol[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int64_t rr = row0 + wave * 64 + t * 32 + n;
        const int64_t r = rr > R - 1 ? R - 1 : rr;
        hrow[t] = reinterpret_cast<const char*>(H + r * g.dh) + PB * h;
        ecol[t] = Et + rr;
    }
    int boff[KS];
#pragma unroll
    for (int j = 0; j < KS; ++j) boff[j] = img_piece<KC>(n, (2 * j + h) & (PPR - 1));

    f32x16 acc[2][NT];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][ct][i] = 0.f;

    const int64_t n_img = (int64_t)g.C * cpc;
    auto stage = [&](int cls, int tw, int slot) __attribute__((always_inline)) {
        int64_t ci = (int64_t)cls * cpc + tw;
        if (ci > n_img - 1) ci = n_img - 1;  // beyond the end: repeat (never used)
        const u32x4* src = img + ci * IMG + tid;
#pragma unroll
        for (int q = 0; q < IMG / 512; ++q)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + q * 512),
                                             (__attribute__((address_space(3))) void*)(lds + slot * IMG + q * 512 + wave * 64),
                                             16, 0, 0);
        if constexpr (IMG % 512 != 0) {  // IMG = 256: waves 4..7 repeat the half round (equal load counts per wave)
            const u32x4* src2 = img + ci * IMG + (tid & 255);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src2),
                                             (__attribute__((address_space(3))) void*)(lds + slot * IMG + (wave & 3) * 64), 16,
                                             0, 0);
        }
    };
    constexpr int VL = (IMG + 511) / 512;

    u32x4 hv[2][4];  // this lane's pieces of the feature rows, current feature window
    // the row operand of k-step j: e * h, rounded to the row type
    auto operand = [&](int t, T eraw, int j, u32x4& hi, u32x4& lo) __attribute__((always_inline)) {
        if constexpr (sizeof(T) == 2) {
            const float e = bf16_to_f32(eraw);
            const u32x4 raw = hv[t][j];
#pragma unroll
            for (int w = 0; w < 4; ++w)
                hi[w] = pack_bf16(__uint_as_float(raw[w] << 16) * e, __uint_as_float(raw[w] & 0xffff0000u) * e);
        } else {
            u32x4 x0, x1;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                x0[w] = __float_as_uint(__uint_as_float(hv[t][2 * j][w]) * eraw);
                x1[w] = __float_as_uint(__uint_as_float(hv[t][2 * j + 1][w]) * eraw);
            }
            split8(x0, x1, hi, lo);
        }
    };
    auto load_e = [&](T (&e)[2], int cls) __attribute__((always_inline)) {
        const int cc = cls > g.C - 1 ? g.C - 1 : cls;
#pragma unroll
        for (int t = 0; t < 2; ++t) e[t] = ecol[t][(int64_t)cc * g.et_pitch];
    };

    // One window: class cls of feature window tw, its image in slot sc; the image and the errors of class cls + 2 are
    // requested.
    auto visit = [&](const T (&e)[2], T (&efar)[2], int cls, int tw, int sc) __attribute__((always_inline)) {
        stage(cls + 2, tw, sc == 0 ? 2 : sc - 1);
        load_e(efar, cls + 2);
        int baddr[KS];
#pragma unroll
        for (int j = 0; j < KS; ++j) baddr[j] = boff[j] + sc * IMG;
        constexpr int STEPS = KS * 2 * NT;
        u32x4 b[2];
        b[0] = lds[baddr[0]];
        u32x4 ahi[2], alo[2];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const int j = s / (2 * NT), ct = s % (2 * NT);
            if (ct == 0) {
                operand(0, e[0], j, ahi[0], alo[0]);
                operand(1, e[1], j, ahi[1], alo[1]);
            }
            if (s + 1 < STEPS) {
                const int j2 = (s + 1) / (2 * NT), ct2 = (s + 1) % (2 * NT);
                b[(s + 1) % 2] = lds[baddr[j2] + ct2 * 32 * PPR];
            }
            const u32x4 bb = b[s % 2];
#pragma unroll
            for (int t = 0; t < 2; ++t) acc[t][ct % NT] = mfma_bf16(ahi[t], bb, acc[t][ct % NT]);
            if constexpr (sizeof(T) == 4) {
                if (ct < NT) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) acc[t][ct] = mfma_bf16(alo[t], bb, acc[t][ct]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // This window issued VL image loads and 2 error loads, all for class cls + 2: with at most that many
        // outstanding, the image and the errors of class cls + 1 have landed. Bare barrier as above.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0x0F70 | (2 + VL));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };

    T e0[2], e1[2], e2[2];
    if (nk > 0) {
        for (int tw = t0; tw < t1; ++tw) {
            stage(k0, tw, 0);
            stage(k0 + 1, tw, 1);
            load_e(e0, k0);
            load_e(e1, k0 + 1);
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int xoff = sizeof(T) == 2 ? 32 * x : 64 * (x >> 1) + 16 * (x & 1);
                    hv[t][x] = *reinterpret_cast<const u32x4*>(hrow[t] + tw * 128 + xoff);
                }
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            int i = 0;
            for (; i + 2 < nk; i += 3) {
                visit(e0, e2, k0 + i, tw, 0);
                visit(e1, e0, k0 + i + 1, tw, 1);
                visit(e2, e1, k0 + i + 2, tw, 2);
            }
            if (i < nk) visit(e0, e2, k0 + i, tw, 0);
            if (i + 1 < nk) visit(e1, e0, k0 + i + 1, tw, 1);
            // every wave has passed the last window's barrier: the ring may be primed again
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing on its way to LDS when the work-group ends
    }

    float* out = partial + (int64_t)split * R * KP;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t r = row0 + wave * 64 + t * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
                if (r < R) out[r * KP + ct * 32 + n] = acc[t][ct][i];
            }
}

// Et[c][r] = E[min(r, R-1)][c] for r < Rp (Rp: R rounded up to whole row tiles). 64 x 64 tiles through LDS.
template <typename T>
__global__ __launch_bounds__(256) void transpose_errors_kernel(const T* __restrict__ E, int64_t R, int C, int64_t Rp,
                                                               T* __restrict__ Et) {
    __shared__ T tile[64][65];
    const int64_t r0 = (int64_t)blockIdx.x * 64;
    const int c0 = blockIdx.y * 64;
    const int a = threadIdx.x & 63, b = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int rr = b + 4 * i;
        int64_t r = r0 + rr;
        if (r > R - 1) r = R - 1;
        tile[rr][a] = c0 + a < C ? E[r * C + c0 + a] : (T)0;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int cc = b + 4 * i;
        if (c0 + cc < C && r0 + a < Rp) Et[(int64_t)(c0 + cc) * Rp + r0 + a] = tile[a][cc];
    }
}

// The bias columns: out[r][j] = sum_c e_rc * V[j][C*dh + c] in fp32 (e is a stored value of the row type, so no
// rounding is involved). 256 threads, 8 rows x KP outputs per work-group, 16 columns of the basis at a time in LDS;
// blockIdx.y takes the classes [y * cps, (y + 1) * cps) and writes partial slot y (cps a multiple of 16).
template <typename T>
__global__ __launch_bounds__(256) void project_bias_kernel(const T* __restrict__ E, int64_t R, int C, int cps,
                                                           int64_t col0, const float* __restrict__ Vblk, int KP,
                                                           float* __restrict__ out) {
    __shared__ float Vs[128][17];
    __shared__ float Es[8][16];
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.x * 8;
    const int per = KP / 32;  // outputs per thread: (8 * KP) / 256
    const int cb0 = blockIdx.y * cps;
    int cb1 = cb0 + cps;
    if (cb1 > C) cb1 = C;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int cb = cb0; cb < cb1; cb += 16) {
        for (int i = tid; i < KP * 16; i += 256) {
            const int j = i >> 4, cc = i & 15;
            Vs[j][cc] = cb + cc < cb1 ? Vblk[blk_off(col0 + cb + cc, j, KP)] : 0.f;
        }
        if (tid < 128) {
            const int rr = tid >> 4, cc = tid & 15;
            const int64_t r = r0 + rr;
            float e = 0.f;
            if (r < R && cb + cc < cb1) {
                if constexpr (sizeof(T) == 2) e = bf16_to_f32(E[r * C + cb + cc]);
                else e = E[r * C + cb + cc];
            }
            Es[rr][cc] = e;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (q < per) {
                const int o = tid + 256 * q, rr = o / KP, j = o % KP;
#pragma unroll
                for (int cc = 0; cc < 16; ++cc) acc[q] = fmaf(Es[rr][cc], Vs[j][cc], acc[q]);
            }
        }
        __syncthreads();
    }
    float* dst = out + (int64_t)blockIdx.y * R * KP;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (q < per) {
            const int o = tid + 256 * q, rr = o / KP, j = o % KP;
            if (r0 + rr < R) dst[(r0 + rr) * KP + j] = acc[q];
        }
    }
}

// Work space of launch_project_outer: the transposed errors, C x (row tiles * 512) values.
size_t outer_work_bytes(int64_t R, int dtype, int64_t C) {
    return (size_t)C * (size_t)((R + 511) / 512 * 512) * (dtype == SAGE_BF16 ? 2 : 4);
}

// The factored projection needs whole windows inside a class and 16-byte aligned feature rows.
bool outer_path_ok(const void* E, const void* H, int dtype, int64_t C, int64_t dh) {
    const int64_t esz = dtype == SAGE_BF16 ? 2 : 4;
    const int64_t KC = 128 / esz;
    return dh >= KC && dh % KC == 0 && C < ((int64_t)1 << 24) && dh < ((int64_t)1 << 24) && ((uintptr_t)H) % 16 == 0 &&
           ((uintptr_t)E) % esz == 0;
}

// splits counts the slots of the main columns (a grid of class groups x window groups, padded to a multiple of 8);
// the bias columns go to the bias_slots slots after them, classes_per_bias_slot classes each. Window groups are kept as small as the split count
// allows, classes per split as many: the feature rows are read once per window of a split.
ScorePlan score_outer_plan(int64_t R, int dtype, int64_t C, int64_t dh, int num_cu) {
    ScorePlan p;
    const int KC = dtype == SAGE_BF16 ? 64 : 32;
    const int64_t cpc = dh / KC;
    p.row_tiles = (int)((R + 511) / 512);
    int64_t target = (((int64_t)num_cu + p.row_tiles - 1) / p.row_tiles + 7) / 8 * 8;
    if (target < 8) target = 8;
    if (target > 512) target = 512;
    int64_t wg = cpc < target ? cpc : target;
    int64_t cg = target / wg;
    if (cg < 1) cg = 1;
    if (cg > C) cg = C;
    p.windows_per_group = (int)((cpc + wg - 1) / wg);
    p.window_groups = (int)((cpc + p.windows_per_group - 1) / p.windows_per_group);
    p.classes_per_group = (int)((C + cg - 1) / cg);
    p.class_groups = (int)((C + p.classes_per_group - 1) / p.classes_per_group);
    p.splits = (p.class_groups * p.window_groups + 7) / 8 * 8;
    p.slabs_per_split = (int64_t)p.classes_per_group * p.windows_per_group;
    p.classes_per_bias_slot = (int)(((C + 7) / 8 + 15) / 16 * 16);  // up to 8 slots
    p.bias_slots = (int)((C + p.classes_per_bias_slot - 1) / p.classes_per_bias_slot);
    return p;
}

template <int NT, typename T>
static hipError_t launch_outer_t(const T* E, const T* H, int64_t R, int64_t C, int64_t dh, void* work, const void* img,
                                 const float* Vblk, float* partial, const ScorePlan& p, hipStream_t st) {
    constexpr int KC = 128 / (int)sizeof(T);
    constexpr size_t LDS = (size_t)3 * 2 * NT * 32 * (KC / 8) * 16;
    if (hipError_t ea = ensure_dynamic_lds((const void*)project_outer_kernel<NT, T>, (int)LDS); ea != hipSuccess) return ea;
    const int64_t Rp = (int64_t)p.row_tiles * 512;
    hipLaunchKernelGGL(transpose_errors_kernel<T>, dim3((unsigned)(Rp / 64), (unsigned)((C + 63) / 64)), dim3(256), 0, st, E,
                       R, (int)C, Rp, (T*)work);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    OuterGeom g;
    g.C = (int)C;
    g.dh = (int)dh;
    g.class_groups = p.class_groups;
    g.classes_per_group = p.classes_per_group;
    g.window_groups = p.window_groups;
    g.windows_per_group = p.windows_per_group;
    g.et_pitch = Rp;
    dim3 grid((unsigned)(p.row_tiles * p.splits));
    hipLaunchKernelGGL((project_outer_kernel<NT, T>), grid, dim3(512), LDS, st, (const T*)work, H, R, g, (const u32x4*)img,
                       partial, p.row_tiles);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(project_bias_kernel<T>, dim3((unsigned)((R + 7) / 8), (unsigned)p.bias_slots), dim3(256), 0, st, E, R,
                       (int)C, p.classes_per_bias_slot, C * dh, Vblk, NT * 32, partial + (size_t)p.splits * R * (NT * 32));
    return hipGetLastError();
}

template <int NT>
static hipError_t launch_outer_nt(const void* E, const void* H, int dtype, int64_t R, int64_t C, int64_t dh, void* work,
                                  const void* img, const float* Vblk, float* partial, const ScorePlan& p, hipStream_t st) {
    if (dtype == SAGE_BF16)
        return launch_outer_t<NT, uint16_t>((const uint16_t*)E, (const uint16_t*)H, R, C, dh, work, img, Vblk, partial, p,
                                            st);
    return launch_outer_t<NT, float>((const float*)E, (const float*)H, R, C, dh, work, img, Vblk, partial, p, st);
}

hipError_t launch_project_outer(const void* E, const void* H, int dtype, int64_t R, int64_t C, int64_t dh, void* work,
                                const void* img, const float* Vblk, int KP, float* partial, const ScorePlan& p,
                                hipStream_t st) {
    switch (KP / 32) {
        case 1: return launch_outer_nt<1>(E, H, dtype, R, C, dh, work, img, Vblk, partial, p, st);
        case 2: return launch_outer_nt<2>(E, H, dtype, R, C, dh, work, img, Vblk, partial, p, st);
        case 4: return launch_outer_nt<4>(E, H, dtype, R, C, dh, work, img, Vblk, partial, p, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sage
