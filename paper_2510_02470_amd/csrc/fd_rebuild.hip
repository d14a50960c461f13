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
// then writes. Nobody else touches those columns, so the update is safely in place (out == top). The coefficient matrix
// streams through LDS in chunks of 16 buffer rows shared by the 4 waves of the work-group; it is stored in the
// order the matrix cores consume it (see coeff_offset), so a lane fetches the 8 coefficients of a chunk with two
// 16-byte LDS reads.
#include "sage_internal.h"

namespace sage {

template <int MT>  // MT = MP / 32 accumulator tiles per wave
__global__ __launch_bounds__(256, 2) void rebuild_kernel(const float* __restrict__ top, const float* __restrict__ nw,
                                                         int nfill, const float* __restrict__ Mc,
                                                         float* __restrict__ out, int NP, int out_NP, int64_t Dp) {
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
    const float* tcol = top + coff;
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

}  // namespace sage
