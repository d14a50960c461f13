// out[0:MP] = M * B on the fp32 matrix cores, column slab by column slab.
//
// Used twice: the rebuild of the shrink step, S <- Sigma' V^T = diag(w) Y^T B (Method, FD paragraph; Algorithm 1,
// Phase I, "S <- Sigma' V^T"), in place on the sketch, and the scoring basis V_k^T = diag(1/sigma) Y_k^T B
// (Algorithm 1, "Freeze S for scoring"), written to its own buffer.
//
// A wave owns 32 columns for the whole product: it reads all NP buffer rows of those columns (its B operand comes
// straight from global memory, one 128 B line per row pair), keeps the MP x 32 result in accumulators, and only
// then writes. Nobody else touches those columns, so the update is safely in place. The coefficient matrix
// (transposed, NP x MP) streams through LDS in chunks of 16 buffer rows shared by the 4 waves of the work-group.
#include "sage_internal.h"

namespace sage {

template <int MT>  // MT = MP / 32 accumulator tiles per wave
__global__ __launch_bounds__(256) void rebuild_kernel(const float* __restrict__ B, const float* __restrict__ Mt,
                                                      float* __restrict__ out, int NP, int out_NP, int zero_tail,
                                                      int64_t Dp) {
    constexpr int MP = MT * 32;
    constexpr int KC = 16;               // buffer rows per LDS stage
    constexpr int CHUNK = KC * MP;       // floats per stage
    constexpr int PER = CHUNK / 256;     // floats per thread per stage (2, 4, 8, 16)
    __shared__ float Ms[2][CHUNK];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = lane & 31, h = lane >> 5;
    const int64_t d = ((int64_t)blockIdx.x * 4 + wave) * 32 + c;  // this lane's column
    const bool live = d < Dp;  // Dp is a multiple of 16 and 32-column groups may overhang by 16
    const int64_t col_base = live ? ((d / DC) * NP) * (int64_t)DC + (d % DC) : 0;

    f32x16 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[m][i] = 0.f;

    float bpre[8];
    float mpre[PER];
    // prologue: stage 0
#pragma unroll
    for (int s = 0; s < 8; ++s) bpre[s] = live ? B[col_base + (int64_t)(2 * s + h) * DC] : 0.f;
#pragma unroll
    for (int u = 0; u < PER; ++u) Ms[0][u * 256 + tid] = Mt[u * 256 + tid];
    __syncthreads();

    const int nstage = NP / KC;
    for (int stg = 0; stg < nstage; ++stg) {
        const int cur = stg & 1;
        float bcur[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) bcur[s] = bpre[s];
        const bool more = stg + 1 < nstage;
        if (more) {
            const int k0 = (stg + 1) * KC;
#pragma unroll
            for (int s = 0; s < 8; ++s) bpre[s] = live ? B[col_base + (int64_t)(k0 + 2 * s + h) * DC] : 0.f;
#pragma unroll
            for (int u = 0; u < PER; ++u) mpre[u] = Mt[(int64_t)k0 * MP + u * 256 + tid];
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const float* mrow = &Ms[cur][(2 * s + h) * MP + c];
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[m] = mfma32(mrow[m * 32], bcur[s], acc[m]);
        }
        if (more) {
#pragma unroll
            for (int u = 0; u < PER; ++u) Ms[cur ^ 1][u * 256 + tid] = mpre[u];
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

hipError_t launch_rebuild(const float* B, const float* Mt, float* out, int out_NP, int MP, bool zero_tail,
                          const Dims& d, hipStream_t st) {
    dim3 grid((unsigned)((d.Dp + 127) / 128));
    int zt = zero_tail ? 1 : 0;
    switch (MP / 32) {
        case 1: hipLaunchKernelGGL(rebuild_kernel<1>, grid, dim3(256), 0, st, B, Mt, out, d.NP, out_NP, zt, d.Dp); break;
        case 2: hipLaunchKernelGGL(rebuild_kernel<2>, grid, dim3(256), 0, st, B, Mt, out, d.NP, out_NP, zt, d.Dp); break;
        case 4: hipLaunchKernelGGL(rebuild_kernel<4>, grid, dim3(256), 0, st, B, Mt, out, d.NP, out_NP, zt, d.Dp); break;
        case 8: hipLaunchKernelGGL(rebuild_kernel<8>, grid, dim3(256), 0, st, B, Mt, out, d.NP, out_NP, zt, d.Dp); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace sage
