// out[0:MP] = M * B on the fp32 matrix cores, column slab by column slab.
//
// Used twice: the rebuild of the shrink step, S <- Sigma' V^T = diag(w) Y^T B (Method, FD paragraph; Algorithm 1,
// Phase I, "S <- Sigma' V^T"), in place on the sketch, and the scoring basis V_k^T = diag(1/sigma) Y_k^T B
// (Algorithm 1, "Freeze S for scoring"), written to its own buffer.
//
// The buffer is two half buffers of LP = NP/2 rows (same slab layout): `top` = matrix rows 0 .. LP-1, `nw` = matrix rows
// LP .. NP-1 of which the first nfill hold data (the others count as zero, whatever they hold).
// A wave owns 32 columns for the whole product: it reads all NP buffer rows of those columns (its B operand comes
// straight from global memory, one 128 B line per row pair), keeps the MP x 32 result in accumulators, and only
// then writes. Nobody else touches those columns, so the update is safely in place (out == top, which is why neither
// pointer is declared restrict). The coefficient matrix
// streams through LDS in chunks of 16 buffer rows shared by the 4 waves of the work-group; it is stored in the
// order the matrix cores consume it (see coeff_offset), so a lane fetches the 8 coefficients of a chunk with two
// 16-byte LDS reads.
#include <type_traits>

#include "sage_internal.h"

namespace sage {

template <int MT>  // MT = MP / 32 accumulator tiles per wave
__global__ __launch_bounds__(256, 2) void rebuild_kernel(const float* top, const float* __restrict__ nw, int nfill,
                                                         const float* __restrict__ Mc, float* out, int NP, int out_NP,
                                                         int64_t Dp) {
    constexpr int MP = MT * 32;
    constexpr int CHUNK4 = 16 * MP / 4;  // 16-byte pieces per stage (16 buffer rows x MP coefficients)
    constexpr int PER = CHUNK4 / 256;    // pieces per thread per stage (MT / 2 ... at least 1)
    static_assert(CHUNK4 % 256 == 0 || CHUNK4 < 256, "chunk must tile the work-group");
    constexpr int PERC = PER > 0 ? PER : 1;
    __shared__ f32x4 Ms[3][CHUNK4];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = lane & 31, h = lane >> 5;
    const int64_t d = ((int64_t)blockIdx.x * 4 + wave) * 32 + c;  // this lane's column
    const bool live = d < Dp;  // Dp is a multiple of 16: the last 32-column group may overhang by 16
    const int64_t dc = live ? d : Dp - 1;
    const int LP = NP >> 1;
    const int64_t coff = ((dc / DC) * LP) * (int64_t)DC + (dc % DC) + (int64_t)h * DC;  // row h of this column, either half
    // lanes beyond the last column compute nothing that is stored; they read the new half only, which this kernel never
    // writes (out may be top: top and out are the same memory then, hence not declared restrict)
    const float* tcol = (live ? top : nw) + coff;
    const float* ncol = nw + coff;
    // rows 16*stg + 2*s + h of the matrix: stage stg lies in the top half when stg < LP/16. Rows of the new half are
    // always loaded (they exist); those not in use are zeroed when the stage consumes them (use_b), not here, so
    // that nothing waits for a load right after issuing it.
    auto fetch_b = [&](int stg, float (&b)[8]) {
        const int r0 = stg * 16;
        const float* bn = r0 >= LP ? ncol + (int64_t)(r0 - LP) * DC : tcol + (int64_t)r0 * DC;
#pragma unroll
        for (int s = 0; s < 8; ++s) b[s] = bn[(int64_t)(2 * s) * DC];
    };
    auto use_b = [&](int stg, const float (&b)[8], float (&o)[8]) {
        const int r0 = stg * 16;
        const int limit = r0 >= LP ? nfill - (r0 - LP) - h : 0x7fffffff;  // 2*s < limit: row in use
#pragma unroll
        for (int s = 0; s < 8; ++s) o[s] = 2 * s < limit ? b[s] : 0.f;
    };

    f32x16 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[m][i] = 0.f;

    const f32x4* Mv = reinterpret_cast<const f32x4*>(Mc);
    float bpre[8];
    f32x4 mpre[PERC];
    // prologue: coefficients of stages 0 and 1 into LDS, row operand of stage 0 on its way
    const int nstage = NP / 16;
    fetch_b(0, bpre);
#pragma unroll
    for (int u = 0; u < PERC; ++u)
        if (u * 256 + tid < CHUNK4) {
            Ms[0][u * 256 + tid] = Mv[u * 256 + tid];
            if (nstage > 1) Ms[1][u * 256 + tid] = Mv[(int64_t)CHUNK4 + u * 256 + tid];
        }
    __syncthreads();

    // LDS piece of (half h, coefficient row m, logical piece p): ((h * MP + m) * 2 + (p ^ ((m >> 3) & 1))).
    // The coefficient pieces are read from LDS while the matrix cores work: those of the second k-half of a stage
    // during its first half, those of the first k-half of the next stage during its second half (one read per four
    // matrix-core instructions, pinned by scheduling barriers). Three LDS buffers: stage s reads buffers s and s+1 and
    // fills buffer s+2 (mod 3), which was last read in stage s-1.
    const int x = (c >> 3) & 1;
    int lbase[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) lbase[m] = (h * MP + m * 32 + c) * 2;
    f32x4 a0[MT], a1[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) a0[m] = Ms[0][lbase[m] + x];
    int cur = 0;
    for (int stg = 0; stg < nstage; ++stg) {
        const int nxt = cur == 2 ? 0 : cur + 1, far = nxt == 2 ? 0 : nxt + 1;
        float bcur[8];
        use_b(stg, bpre, bcur);
        const bool more = stg + 1 < nstage, more2 = stg + 2 < nstage;
        // the coefficient loads first: waiting for them (to put them in LDS) then leaves the row loads in flight
        if (more2) {
#pragma unroll
            for (int u = 0; u < PERC; ++u)
                if (u * 256 + tid < CHUNK4) mpre[u] = Mv[(int64_t)(stg + 2) * CHUNK4 + u * 256 + tid];
        }
        if (more) fetch_b(stg + 1, bpre);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < MT; ++i) {  // first k-half; fetch a1[i]
            a1[i] = Ms[cur][lbase[i] + (x ^ 1)];
#pragma unroll
            for (int j = 4 * i; j < 4 * i + 4; ++j) acc[j % MT] = mfma32(a0[j % MT][j / MT], bcur[j / MT], acc[j % MT]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < MT; ++i) {  // second k-half; fetch the next stage's a0[i] (its last use was above)
            if (more) a0[i] = Ms[nxt][lbase[i] + x];
#pragma unroll
            for (int j = 4 * i; j < 4 * i + 4; ++j) acc[j % MT] = mfma32(a1[j % MT][j / MT], bcur[4 + j / MT], acc[j % MT]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more2) {
#pragma unroll
            for (int u = 0; u < PERC; ++u)
                if (u * 256 + tid < CHUNK4) Ms[far][u * 256 + tid] = mpre[u];
        }
        // A bare barrier after the LDS traffic: __syncthreads() would also wait for the row loads still in flight.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): vmcnt and expcnt not waited for
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        cur = nxt;
    }

    if (!live) return;
    const int64_t out_base = ((d / DC) * out_NP) * (int64_t)DC + (d % DC);
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            int r = m * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
            out[out_base + (int64_t)r * DC] = acc[m][i];
        }
}

hipError_t launch_rebuild(const float* top, const float* nw, int nfill, const float* Mc, float* out, int out_NP, int MP,
                          const Dims& d, hipStream_t st) {
    dim3 grid((unsigned)((d.Dp + 127) / 128));
#define SAGE_RB(MT)                                                                                                  \
    hipLaunchKernelGGL(rebuild_kernel<MT>, grid, dim3(256), 0, st, top, nw, nfill, Mc, out, d.NP, out_NP, d.Dp)
    switch (MP / 32) {
        case 1: SAGE_RB(1); break;
        case 2: SAGE_RB(2); break;
        case 4: SAGE_RB(4); break;
        case 8: SAGE_RB(8); break;
        default: return hipErrorInvalidValue;
    }
#undef SAGE_RB
    return hipGetLastError();
}


// ---- the same product on the bf16 matrix cores, three-way split ---------------------------------------------
// An fp32 matrix-core instruction (32x32x2) takes 64 cycles for 4096 flop, a bf16 one (32x32x16) 32 cycles for 32768.
// With x = hi + mid + lo (three bf16 parts, 24 significant bits) for both factors and the six products whose weight
// is at least 2^-16 of the leading one (hi*hi, hi*mid, mid*hi, hi*lo, lo*hi, mid*mid; the others are below 2^-24),
// 16 buffer rows cost 6 x 32 cycles per tile instead of 8 x 64: the fp32 result to within a few 2^-24 per term at
// 2.7 times the rate. Accumulation is fp32 in both cases.
//
// Same decomposition as rebuild_kernel: a wave owns 32 columns for the whole product, its column operand comes from
// global memory (8 rows of its k-half per stage of 16 buffer rows; k-slot (h, s) is buffer row 16*stage + 2s + h,
// the order coeff_offset groups the coefficients in) and is split in registers; the coefficients are split once per
// launch by coeff_split_kernel into the order LDS holds them, [stage][part][h][m][8 k-slots], and streamed through a
// ring of three LDS buffers with direct global->LDS loads two stages ahead. The column operand is requested two
// stages ahead as well.
template <int MT>
__global__ __launch_bounds__(256) void coeff_split_kernel(const float* __restrict__ Mc, int NP, u32x4* __restrict__ Mc3) {
    constexpr int MP = MT * 32;
    const int i = blockIdx.x * 256 + threadIdx.x;  // (stage, h, m)
    if (i >= (NP / 16) * 2 * MP) return;
    const int m = i % MP, h = (i / MP) & 1, stg = i / (2 * MP);
    float v[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) v[s] = Mc[coeff_offset(stg * 16 + 2 * s + h, m, MP)];
    u32x4 hi, mid, lo;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        unsigned a, b, c;
        split3_bf16(v[2 * e], v[2 * e + 1], a, b, c);
        hi[e] = a;
        mid[e] = b;
        lo[e] = c;
    }
    u32x4* dst = Mc3 + (int64_t)stg * (3 * 2 * MP) + h * MP + m;
    dst[0] = hi;
    dst[2 * MP] = mid;
    dst[4 * MP] = lo;
}

// NPT > 0: the buffer has NPT rows and the new rows in use hold bf16 values; their stages take the hi part alone and
// three products (the other three would add exact zeros). NPT = 0: any buffer, all parts.
template <int MT, int NPT>
__global__ __launch_bounds__(256, 2) void rebuild_split_kernel(const float* top, const float* __restrict__ nw, int nfill,
                                                               const u32x4* __restrict__ Mc3, float* out, int NP,
                                                               int out_NP, int64_t Dp) {
    constexpr int MP = MT * 32;
    constexpr int STAGE16 = 3 * 2 * MP;   // 16-byte pieces of coefficients per stage
    constexpr int ML = STAGE16 / 256;     // direct-to-LDS loads per thread and stage
    static_assert(STAGE16 % 256 == 0, "a stage must tile the work-group");
    extern __shared__ u32x4 Ms[];         // 3 * STAGE16

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31, h = lane >> 5;
    const int64_t d = ((int64_t)blockIdx.x * 4 + wave) * 32 + c;  // this lane's column
    const bool live = d < Dp;  // Dp is a multiple of 16: the last 32-column group may overhang by 16
    const int64_t dc = live ? d : Dp - 1;
    const int LP = NP >> 1;
    const int64_t coff = ((dc / DC) * LP) * (int64_t)DC + (dc % DC) + (int64_t)h * DC;  // row h of this column, either half
    // lanes beyond the last column compute nothing that is stored; they read the new half only, which this kernel never
    // writes (out may be top: top and out are the same memory then, hence not declared restrict)
    const float* tcol = (live ? top : nw) + coff;
    const float* ncol = nw + coff;
    const int nstage = NP / 16;
    auto fetch_b = [&](int stg, float (&b)[8]) __attribute__((always_inline)) {
        const int sg = stg < nstage ? stg : nstage - 1;  // beyond the end: repeat (never used)
        const int r0 = sg * 16;
        const float* bn = r0 >= LP ? ncol + (int64_t)(r0 - LP) * DC : tcol + (int64_t)r0 * DC;
#pragma unroll
        for (int s = 0; s < 8; ++s) b[s] = bn[(int64_t)(2 * s) * DC];
    };
    auto fetch_m = [&](int stg, int buf) __attribute__((always_inline)) {
        const int sg = stg < nstage ? stg : nstage - 1;
        const u32x4* src = Mc3 + (int64_t)sg * STAGE16 + tid;
#pragma unroll
        for (int q = 0; q < ML; ++q)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + q * 256),
                                             (__attribute__((address_space(3))) void*)(Ms + buf * STAGE16 + q * 256 + wave * 64),
                                             16, 0, 0);
    };

    f32x16 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[m][i] = 0.f;

    // One stage: 16 buffer rows. b: its column operand (requested two stages ago); bfar receives that of stage + 2.
    auto stage = [&](auto one_c, const float (&b)[8], float (&bfar)[8], int stg, int cur) __attribute__((always_inline)) {
        constexpr bool one = decltype(one_c)::value;  // a stage of new rows with one part
        const u32x4* A = Ms + cur * STAGE16 + h * MP + c;  // + part * 2 * MP + tile * 32
        u32x4 a[2][2][3];  // [buffer][tile of the pair][part]
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int p = 0; p < 3; ++p) a[0][t][p] = A[p * 2 * MP + t * 32];
        // rows of the new half that are not in use count as zero, whatever they hold
        const int r0 = stg * 16;
        const int limit = r0 >= LP ? nfill - (r0 - LP) - h : 0x7fffffff;  // 2*s < limit: row in use
        u32x4 bh, bm, bl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x = 4 * e < limit ? b[2 * e] : 0.f, y = 4 * e + 2 < limit ? b[2 * e + 1] : 0.f;
            if constexpr (one) {
                bh[e] = hi_bf16(x, y);
                bm[e] = 0u;
                bl[e] = 0u;
            } else {
                unsigned p0, p1, p2;
                split3_bf16(x, y, p0, p1, p2);
                bh[e] = p0;
                bm[e] = p1;
                bl[e] = p2;
            }
        }
        fetch_m(stg + 2, cur == 0 ? 2 : cur - 1);
        fetch_b(stg + 2, bfar);
        __builtin_amdgcn_sched_barrier(0);
        // two tiles at a time, their instructions alternating (an instruction never waits for the one just issued)
#pragma unroll
        for (int i = 0; i < MT; i += 2) {
            if (i + 2 < MT) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int p = 0; p < 3; ++p) a[((i >> 1) + 1) & 1][t][p] = A[p * 2 * MP + (i + 2 + t) * 32];
            }
            __builtin_amdgcn_sched_barrier(0);  // the reads go out before this pair's matrix-core instructions, not after
            const int bsel = (i >> 1) & 1;
            if constexpr (one) {
#pragma unroll
                for (int q = 2; q >= 0; --q)  // smallest terms first
#pragma unroll
                    for (int t = 0; t < 2; ++t) acc[i + t] = mfma_bf16(a[bsel][t][q], bh, acc[i + t]);
            } else {
#pragma unroll
                for (int q = 0; q < 6; ++q) {  // smallest terms first
                    constexpr int PA[6] = {2, 0, 1, 1, 0, 0};  // part of the coefficient
                    constexpr int PB[6] = {0, 2, 1, 0, 1, 0};  // part of the column operand
                    const u32x4 bb = PB[q] == 0 ? bh : (PB[q] == 1 ? bm : bl);
#pragma unroll
                    for (int t = 0; t < 2; ++t) acc[i + t] = mfma_bf16(a[bsel][t][PA[q]], bb, acc[i + t]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // Before the barrier: everything this wave asked for before this stage has landed, i.e. its share of the next
        // stage's coefficients and the next stage's column operand (at most the ML + 8 loads of this stage stay in
        // flight; loads return in order). The LDS reads above are consumed. A bare barrier (no fence: it would drain
        // the loads in flight) then makes the next stage's coefficients visible to all waves and frees this stage's
        // buffer.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0x0F70 | (8 + ML));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };

    // Stage s uses LDS buffer and row registers s mod 3 (+ a fixed offset, below).
    float b0[8], b1[8], b2[8];
    constexpr std::false_type all_parts{};
    constexpr std::true_type one_part{};
    auto triples = [&](auto one_c, int s, int end) __attribute__((always_inline)) {  // from ring position 0
        for (; s + 2 < end; s += 3) {
            stage(one_c, b0, b2, s, 0);
            stage(one_c, b1, b0, s + 1, 1);
            stage(one_c, b2, b1, s + 2, 2);
        }
        if (s < end) stage(one_c, b0, b2, s, 0);
        if (s + 1 < end) stage(one_c, b1, b0, s + 1, 1);
    };
    if constexpr (NPT == 0) {
        fetch_m(0, 0);
        fetch_m(1, 1);
        fetch_b(0, b0);
        fetch_b(1, b1);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        triples(all_parts, 0, nstage);
    } else {
        // The top half's NPT / 32 stages start at the ring position that lets the new half's start at position 0.
        constexpr int S1 = NPT / 32, R = S1 % 3;
        static_assert(R == 1 || R == 2, "buffers of 256 or 512 rows");
        if constexpr (R == 1) {
            fetch_m(0, 2);
            fetch_m(1, 0);
            fetch_b(0, b2);
            fetch_b(1, b0);
        } else {
            fetch_m(0, 1);
            fetch_m(1, 2);
            fetch_b(0, b1);
            fetch_b(1, b2);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if constexpr (R == 1) {
            stage(all_parts, b2, b1, 0, 2);
        } else {
            stage(all_parts, b1, b0, 0, 1);
            stage(all_parts, b2, b1, 1, 2);
        }
        triples(all_parts, R, S1);
        triples(one_part, S1, 2 * S1);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing on its way to LDS when the work-group ends

    if (!live) return;
    const int64_t out_base = ((d / DC) * out_NP) * (int64_t)DC + (d % DC);
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            int r = m * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
            out[out_base + (int64_t)r * DC] = acc[m][i];
        }
}

bool rebuild_split_ok(int MP) { return MP == 128 || MP == 256; }

size_t rebuild_split_bytes(const Dims& d, int MP) { return (size_t)(d.NP / 16) * 3 * 2 * MP * 16; }

template <int MT, int NPT>
static hipError_t launch_rebuild_split_t(const float* top, const float* nw, int nfill, const float* Mc, void* Mc3,
                                         float* out, int out_NP, const Dims& d, hipStream_t st) {
    constexpr int MP = MT * 32;
    constexpr size_t LDS = (size_t)3 * 3 * 2 * MP * 16;
    if (hipError_t ea = ensure_dynamic_lds((const void*)rebuild_split_kernel<MT, NPT>, (int)LDS); ea != hipSuccess)
        return ea;
    const int n = (d.NP / 16) * 2 * MP;
    hipLaunchKernelGGL(coeff_split_kernel<MT>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, Mc, d.NP, (u32x4*)Mc3);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((d.Dp + 127) / 128));
    hipLaunchKernelGGL((rebuild_split_kernel<MT, NPT>), grid, dim3(256), LDS, st, top, nw, nfill, (const u32x4*)Mc3, out,
                       d.NP, out_NP, d.Dp);
    return hipGetLastError();
}

hipError_t launch_rebuild_split(const float* top, const float* nw, int nfill, const float* Mc, void* Mc3, float* out,
                                int out_NP, int MP, const Dims& d, hipStream_t st, bool new_one) {
    if (MP == 256 && new_one && d.NP == 512) return launch_rebuild_split_t<8, 512>(top, nw, nfill, Mc, Mc3, out, out_NP, d, st);
    if (MP == 256) return launch_rebuild_split_t<8, 0>(top, nw, nfill, Mc, Mc3, out, out_NP, d, st);
    if (MP == 128 && new_one && d.NP == 512) return launch_rebuild_split_t<4, 512>(top, nw, nfill, Mc, Mc3, out, out_NP, d, st);
    if (MP == 128 && new_one && d.NP == 256) return launch_rebuild_split_t<4, 256>(top, nw, nfill, Mc, Mc3, out, out_NP, d, st);
    if (MP == 128) return launch_rebuild_split_t<4, 0>(top, nw, nfill, Mc, Mc3, out, out_NP, d, st);
    return hipErrorInvalidValue;
}

}  // namespace sage
