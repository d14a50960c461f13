// out[0:MP] = M * B on the fp32 matrix cores, column slab by column slab.
//
// Used twice: the rebuild of the shrink step, S <- Sigma' V^T = diag(w) Y^T B (Method, FD paragraph; Algorithm 1,
// Phase I, "S <- Sigma' V^T"), in place on the sketch, and the scoring basis V_k^T = diag(1/sigma) Y_k^T B
// (Algorithm 1, "Freeze S for scoring"), written to its own buffer.
//
// A wave owns 32 columns for the whole product: it reads all NP buffer rows of those columns (its B operand comes
// straight from global memory, one 128 B line per row pair), keeps the MP x 32 result in accumulators, and only
// then writes. Nobody else touches those columns, so the update is safely in place. The coefficient matrix
// streams through LDS in chunks of 16 buffer rows shared by the 4 waves of the work-group; it is stored in the
// order the matrix cores consume it (see coeff_offset), so a lane fetches the 8 coefficients of a chunk with two
// 16-byte LDS reads.
#include "sage_internal.h"

namespace sage {

template <int MT>  // MT = MP / 32 accumulator tiles per wave
__global__ __launch_bounds__(256, 2) void rebuild_kernel(const float* __restrict__ B, const float* __restrict__ Mc,
                                                         float* __restrict__ out, int NP, int out_NP, int zero_tail,
                                                         int64_t Dp) {
    constexpr int MP = MT * 32;
    constexpr int CHUNK4 = 16 * MP / 4;  // 16-byte pieces per stage (16 buffer rows x MP coefficients)
    constexpr int PER = CHUNK4 / 256;    // pieces per thread per stage (MT / 2 ... at least 1)
    static_assert(CHUNK4 % 256 == 0 || CHUNK4 < 256, "chunk must tile the work-group");
    constexpr int PERC = PER > 0 ? PER : 1;
    __shared__ f32x4 Ms[2][CHUNK4];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = lane & 31, h = lane >> 5;
    const int64_t d = ((int64_t)blockIdx.x * 4 + wave) * 32 + c;  // this lane's column
    const bool live = d < Dp;  // Dp is a multiple of 16: the last 32-column group may overhang by 16
    const int64_t dc = live ? d : Dp - 1;
    const float* bcol = B + ((dc / DC) * NP) * (int64_t)DC + (dc % DC) + (int64_t)h * DC;  // row h of this column

    f32x16 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[m][i] = 0.f;

    const f32x4* Mv = reinterpret_cast<const f32x4*>(Mc);
    float bpre[8];
    f32x4 mpre[PERC];
    // prologue: stage 0
#pragma unroll
    for (int s = 0; s < 8; ++s) bpre[s] = bcol[(int64_t)(2 * s) * DC];
#pragma unroll
    for (int u = 0; u < PERC; ++u)
        if (u * 256 + tid < CHUNK4) Ms[0][u * 256 + tid] = Mv[u * 256 + tid];
    __syncthreads();

    // LDS piece of (half h, coefficient row m, logical piece p): ((h * MP + m) * 2 + (p ^ ((m >> 3) & 1)))
    const int x = (c >> 3) & 1;
    const int nstage = NP / 16;
    for (int stg = 0; stg < nstage; ++stg) {
        const int cur = stg & 1;
        float bcur[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) bcur[s] = bpre[s];
        const bool more = stg + 1 < nstage;
        if (more) {
            const float* bn = bcol + (int64_t)(stg + 1) * 16 * DC;
#pragma unroll
            for (int s = 0; s < 8; ++s) bpre[s] = bn[(int64_t)(2 * s) * DC];
#pragma unroll
            for (int u = 0; u < PERC; ++u)
                if (u * 256 + tid < CHUNK4) mpre[u] = Mv[(int64_t)(stg + 1) * CHUNK4 + u * 256 + tid];
        }
        f32x4 a[MT][2];
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const int base = (h * MP + m * 32 + c) * 2;
            a[m][0] = Ms[cur][base + x];
            a[m][1] = Ms[cur][base + (x ^ 1)];
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads ahead of the matrix-core block
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int m = 0; m < MT; ++m) acc[m] = mfma32(a[m][p][e], bcur[4 * p + e], acc[m]);
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
#pragma unroll
            for (int u = 0; u < PERC; ++u)
                if (u * 256 + tid < CHUNK4) Ms[cur ^ 1][u * 256 + tid] = mpre[u];
        }
        __syncthreads();
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
    if (zero_tail) {
        for (int r = MP + h; r < out_NP; r += 2) out[out_base + (int64_t)r * DC] = 0.f;
    }
}

hipError_t launch_rebuild(const float* B, const float* Mc, float* out, int out_NP, int MP, bool zero_tail,
                          const Dims& d, hipStream_t st) {
    dim3 grid((unsigned)((d.Dp + 127) / 128));
    int zt = zero_tail ? 1 : 0;
    switch (MP / 32) {
        case 1: hipLaunchKernelGGL(rebuild_kernel<1>, grid, dim3(256), 0, st, B, Mc, out, d.NP, out_NP, zt, d.Dp); break;
        case 2: hipLaunchKernelGGL(rebuild_kernel<2>, grid, dim3(256), 0, st, B, Mc, out, d.NP, out_NP, zt, d.Dp); break;
        case 4: hipLaunchKernelGGL(rebuild_kernel<4>, grid, dim3(256), 0, st, B, Mc, out, d.NP, out_NP, zt, d.Dp); break;
        case 8: hipLaunchKernelGGL(rebuild_kernel<8>, grid, dim3(256), 0, st, B, Mc, out, d.NP, out_NP, zt, d.Dp); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace sage
