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

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// v_mfma_f32_32x32x16_bf16: acc(32x32) += a(32x16) b(16x32). Lane l supplies a[l%32][8*(l/32) .. +8] and
// b[8*(l/32) .. +8][l%32]; acc element i of lane l is row 8*(i/4) + 4*(l/32) + i%4, column l%32.
__device__ __forceinline__ f32x16 mfma_bf16(u32x4 a, u32x4 b, f32x16 acc) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0,
                                                   0, 0);
}

__device__ __forceinline__ unsigned pack_bf16(float x, float y) {
    bf16x2 h = {(__bf16)x, (__bf16)y};  // round to nearest even (v_cvt_pk_bf16_f32)
    return __builtin_bit_cast(unsigned, h);
}

// ---- basis images -----------------------------------------------------------------------------------------
// Chunk c covers columns c*KC .. c*KC + KC - 1 (KC = 64 for bf16 rows, 32 for fp32 rows: 128 bytes of a row).
// Its image has 2*KP rows of KC bf16: image row cc < KP is hi(v_cc), image row KP + cc is lo(v_cc). A row is cut
// into 16-byte pieces (8 columns); piece p of image row cc is stored at position swz(cc, p) of that row so that the
// lanes of a matrix-core operand read (32 consecutive image rows, one piece each) spread over all LDS banks:
//   KC = 64 (8 pieces, 128 B rows): swz = p ^ (cc & 7);  KC = 32 (4 pieces, 64 B rows): swz = p ^ ((cc >> 1) & 3).
template <int KC>
__device__ __forceinline__ int img_piece(int cc, int p) {
    if constexpr (KC == 64) return cc * 8 + (p ^ (cc & 7));
    else return cc * 4 + (p ^ ((cc >> 1) & 3));
}

// First column of chunk c: c*KC, except that the last chunk is moved back to end exactly at column D (so that a
// lane never reads beyond its row); the columns it then shares with the chunk before are zero in its image.
__host__ __device__ inline int64_t chunk_start(int64_t c, int KC, int64_t D) {
    int64_t s = c * KC;
    return s + KC > D ? D - KC : s;
}

// One thread writes one 16-byte piece. Vblk is the fp32 column-slab basis (KP rows). Needs D >= KC.
template <int KC>
__global__ __launch_bounds__(256) void basis_split_kernel(const float* __restrict__ Vblk, int KP, int64_t D,
                                                          int64_t chunks, u32x4* __restrict__ img) {
    constexpr int PPR = KC / 8;
    const int64_t per_chunk = (int64_t)2 * KP * PPR;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= chunks * per_chunk) return;
    const int64_t c = i / per_chunk;
    const int rem = (int)(i % per_chunk);
    const int cc = rem / PPR, p = rem % PPR;
    const int row = cc < KP ? cc : cc - KP;
    const int64_t d0 = chunk_start(c, KC, D) + p * 8;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int64_t d = d0 + e;
        v[e] = (d >= c * KC) ? Vblk[blk_off(d, row, KP)] : 0.f;  // d < D always
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
        hipLaunchKernelGGL(basis_split_kernel<64>, grid, dim3(256), 0, st, Vblk, KP, d.D, chunks, (u32x4*)img);
    else
        hipLaunchKernelGGL(basis_split_kernel<32>, grid, dim3(256), 0, st, Vblk, KP, d.D, chunks, (u32x4*)img);
    return hipGetLastError();
}

size_t basis_image_bytes(int KP, int dtype, const Dims& d) {
    const int KC = dtype == SAGE_BF16 ? 64 : 32;
    const int64_t chunks = (d.D + KC - 1) / KC;
    return (size_t)chunks * 2 * KP * KC * 2;
}

// ---- projection -------------------------------------------------------------------------------------------
// Row operand of one chunk for one 32-row tile: 4 pieces of 16 bytes per lane.
//   bf16 rows: piece j (k-step j) = columns 16 j + 8 h .. + 8 of the chunk.
//   fp32 rows: pieces 2j, 2j + 1   = columns 16 j + 8 h .. + 8 of the chunk (two k-steps per chunk).
// The address is (wave-uniform chunk base) + (32-bit lane offset) + (compile-time piece offset), which lets the
// loads use the scalar-base addressing form: one offset register per row tile.
template <typename T>
struct RowOp {
    u32x4 v[4];
};

template <typename T>
__device__ __forceinline__ void load_piece(RowOp<T>& a, const char* __restrict__ chunk_base, unsigned lane_off, int q) {
    int off;
    if constexpr (sizeof(T) == 2) off = 32 * q;
    else off = 64 * (q >> 1) + 16 * (q & 1);
    a.v[q] = *reinterpret_cast<const u32x4*>(chunk_base + lane_off + off);
}

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

template <int NT, typename T>  // NT = KP / 32
__global__ __launch_bounds__(256, 2) void project_split_kernel(const T* __restrict__ G, int64_t R,
                                                               const u32x4* __restrict__ img,
                                                               float* __restrict__ partial, int row_tiles, int64_t D,
                                                               int64_t chunks_total, int64_t chunks_per_split) {
    constexpr int KP = NT * 32;
    constexpr int KC = 128 / (int)sizeof(T);
    constexpr int PPR = KC / 8;
    constexpr int IMG = 2 * KP * PPR;  // 16-byte pieces per image
    constexpr int ROUNDS = IMG / 256;  // staging rounds of the work-group (IMG is a multiple of 256)
    constexpr int KS = KC / 16;        // matrix-core k-steps per chunk
    __shared__ u32x4 lds[2 * IMG];

    const int id = blockIdx.x;
    const int xcd = id & 7, y = id >> 3;
    const int rt = y % row_tiles;
    const int split = (y / row_tiles) * 8 + xcd;
    const int64_t c0 = (int64_t)split * chunks_per_split;
    int64_t c1 = c0 + chunks_per_split;
    if (c1 > chunks_total) c1 = chunks_total;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int64_t row_base = (int64_t)rt * 256 + wave * 64;

    // byte offset of this lane's first piece from the first row of the work-group's row tile; rows >= R repeat row R-1
    const char* gwg = reinterpret_cast<const char*>(G) + (int64_t)rt * 256 * D * (int64_t)sizeof(T);
    unsigned loff[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        int64_t r = row_base + t * 32 + n;
        if (r > R - 1) r = R - 1;
        loff[t] = (unsigned)((r - (int64_t)rt * 256) * D * (int64_t)sizeof(T)) + (unsigned)(h * (sizeof(T) == 2 ? 16 : 32));
    }
    auto chunk_ptr = [&](int64_t c) { return gwg + chunk_start(c, KC, D) * (int64_t)sizeof(T); };
    // LDS piece index of this lane's basis operand for k-step j, column tile 0 (tile ct adds ct * 32 * PPR)
    int boff[KS];
#pragma unroll
    for (int j = 0; j < KS; ++j) boff[j] = img_piece<KC>(n, 2 * j + h);

    f32x16 acc[2][NT];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][ct][i] = 0.f;

    auto stage = [&](int64_t c, int buf) {
        const u32x4* src = img + c * IMG + tid;
#pragma unroll
        for (int q = 0; q < ROUNDS; ++q)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + q * 256),
                                             (__attribute__((address_space(3))) void*)(lds + buf * IMG + q * 256 + wave * 64),
                                             16, 0, 0);
    };
    // The split's chunks are visited in rotated order (start = a multiple of the split index): with a power-of-two
    // row pitch all work-groups would otherwise walk the same low address bits, i.e. the same memory channels, in
    // lock step. The work-groups of one split (different row tiles) keep the same order and share the images in L2.
    // Visits beyond the last repeat the last chunk (prefetches whose data is never used).
    const int64_t nc = c1 - c0;
    const int64_t phase = nc > 0 ? ((int64_t)split * 37) % nc : 0;
    auto chunk_of = [&](int64_t i) {
        int64_t c = c0 + (i < nc ? i : nc - 1) + phase;
        return c >= c1 ? c - nc : c;
    };
    // One visit. Step s = (k-step j, column tile ct) in order; the basis operand of step s + 2 is fetched from LDS
    // before the matrix-core instructions of step s are issued, and the scheduler may not move anything across a
    // step (left alone it hoists a whole chunk of LDS reads and spills). As soon as k-step j is done its row
    // registers are reloaded with the same pieces of the visit after next, so a row load has two visits to land.
    auto visit = [&](RowOp<T> (&a)[2], int64_t i, int buf) {
        stage(chunk_of(i + 1), buf ^ 1);
        const char* gnext = chunk_ptr(chunk_of(i + 2));
        const u32x4* vs = lds + buf * IMG;
        constexpr int STEPS = KS * 2 * NT;
        u32x4 b[3];
        b[0] = vs[boff[0]];
        b[1] = vs[boff[0] + 32 * PPR];
        u32x4 ahi[2], alo[2];
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
            if (s + 2 < STEPS) {
                const int j2 = (s + 2) / (2 * NT), ct2 = (s + 2) % (2 * NT);
                b[(s + 2) % 3] = vs[boff[j2] + ct2 * 32 * PPR];
            }
            const u32x4 bb = b[s % 3];
#pragma unroll
            for (int t = 0; t < 2; ++t) acc[t][ct % NT] = mfma_bf16(ahi[t], bb, acc[t][ct % NT]);
            if constexpr (sizeof(T) == 4) {
                if (ct < NT) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) acc[t][ct] = mfma_bf16(alo[t], bb, acc[t][ct]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (ct == 2 * NT - 1) {
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    if constexpr (sizeof(T) == 2) {
                        load_piece<T>(a[t], gnext, loff[t], j);
                    } else {
                        load_piece<T>(a[t], gnext, loff[t], 2 * j);
                        load_piece<T>(a[t], gnext, loff[t], 2 * j + 1);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // 8 row loads were issued after this visit's image loads: once at most 8 loads are outstanding the image of
        // the next visit (and every older load) has landed. vmcnt(8), expcnt and lgkmcnt not waited for.
        // A bare barrier: __syncthreads() carries a release fence, which on this target drains every outstanding
        // load (vmcnt(0)) and would throw the prefetch distance away. The LDS reads of this visit have all been
        // consumed by matrix-core instructions above, so there is nothing else to wait for.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0x0F78);
        __builtin_amdgcn_s_barrier();  // every wave has the image, and every wave is done reading this visit's image
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };

    RowOp<T> a[2], an[2];
    if (nc > 0) {
        stage(chunk_of(0), 0);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                load_piece<T>(a[t], chunk_ptr(chunk_of(0)), loff[t], q);
                load_piece<T>(an[t], chunk_ptr(chunk_of(1)), loff[t], q);
            }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        int64_t i = 0;
        for (; i + 1 < nc; i += 2) {
            visit(a, i, 0);
            visit(an, i + 1, 1);
        }
        if (i < nc) visit(a, i, 0);
    }

    float* out = partial + (int64_t)split * R * KP;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int64_t r = row_base + t * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
                if (r < R) out[r * KP + ct * 32 + n] = acc[t][ct][i];
            }
}

// Every row must start on a 16-byte boundary, hold at least one chunk, and 256 rows must span < 4 GiB (lane offsets
// are 32-bit).
bool split_path_ok(const void* G, int dtype, const Dims& d) {
    const int64_t esz = dtype == SAGE_BF16 ? 2 : 4;
    const int64_t KC = 128 / esz;
    return (d.D * esz) % 16 == 0 && d.D >= KC && d.D * esz * 256 < ((int64_t)1 << 32) && ((uintptr_t)G) % 16 == 0;
}

ScorePlan score_split_plan(int64_t R, int dtype, const Dims& d, int num_cu) {
    ScorePlan p;
    const int KC = dtype == SAGE_BF16 ? 64 : 32;
    const int64_t chunks = (d.D + KC - 1) / KC;
    p.row_tiles = (int)((R + 255) / 256);
    int64_t want = ((int64_t)num_cu * 2 + p.row_tiles - 1) / p.row_tiles;
    int64_t s = (want + 7) / 8 * 8;
    int64_t smax = ((chunks + 7) / 8 + 7) / 8 * 8;  // at least ~8 chunks per split
    if (s > smax) s = smax;
    if (s < 8) s = 8;
    if (s > 512) s = 512;
    p.splits = (int)s;
    p.slabs_per_split = (chunks + s - 1) / s;  // chunks per split on this path
    return p;
}

template <int NT>
static hipError_t launch_split_nt(const void* G, int dtype, int64_t R, const void* img, float* partial,
                                  const ScorePlan& p, const Dims& d, hipStream_t st) {
    dim3 grid((unsigned)(p.row_tiles * p.splits));
    if (dtype == SAGE_BF16) {
        const int64_t chunks = (d.D + 63) / 64;
        hipLaunchKernelGGL((project_split_kernel<NT, uint16_t>), grid, dim3(256), 0, st, (const uint16_t*)G, R,
                           (const u32x4*)img, partial, p.row_tiles, d.D, chunks, p.slabs_per_split);
    } else {
        const int64_t chunks = (d.D + 31) / 32;
        hipLaunchKernelGGL((project_split_kernel<NT, float>), grid, dim3(256), 0, st, (const float*)G, R,
                           (const u32x4*)img, partial, p.row_tiles, d.D, chunks, p.slabs_per_split);
    }
    return hipGetLastError();
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

}  // namespace sage
