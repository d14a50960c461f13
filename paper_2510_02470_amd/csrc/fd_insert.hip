// Row movement between the caller's row-major batches and the library's column-slab layout.
// Algorithm 1, Phase I, "S[r mod ell, :] <- g": a row is placed into a free (zero) buffer row.
#include "sage_internal.h"

namespace sage {

// One thread moves one 16-byte piece (4 columns) of one row. grid = (ceil(4*S / 256), rows).
// Columns >= D are written as zero so that padding never carries data.
template <typename T>
__global__ __launch_bounds__(256) void insert_kernel(const T* __restrict__ G, int row0, float* __restrict__ B,
                                                     int NP, int64_t D, int64_t S) {
    int64_t piece = (int64_t)blockIdx.x * 256 + threadIdx.x;  // piece index along the row
    if (piece >= S * 4) return;
    int64_t r = blockIdx.y;
    int64_t d0 = piece * 4;
    const T* g = G + r * D + d0;
    float v[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        float x = 0.f;
        if (d0 + c < D) {
            if constexpr (sizeof(T) == 2) x = bf16_to_f32(g[c]);
            else x = g[c];
        }
        v[c] = x;
    }
    float4* dst = reinterpret_cast<float4*>(B + blk_off(d0, row0 + (int)r, NP));
    *dst = make_float4(v[0], v[1], v[2], v[3]);
}

hipError_t launch_insert(const void* G, int dtype, int64_t rows, int row0, float* half, int half_rows, const Dims& d,
                         hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    dim3 grid((unsigned)((d.S * 4 + 255) / 256), (unsigned)rows);
    if (dtype == SAGE_BF16)
        hipLaunchKernelGGL(insert_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)G, row0, half, half_rows, d.D,
                           d.S);
    else
        hipLaunchKernelGGL(insert_kernel<float>, grid, dim3(256), 0, st, (const float*)G, row0, half, half_rows, d.D, d.S);
    return hipGetLastError();
}

// Factored rows (a linear last layer: column c*dh + t of row r is e_rc * h_rt, column C*dh + c is e_rc; Method,
// definition of g_i). The value a caller would have stored in a row of type T: the fp32 product, for bf16 rows
// rounded to nearest even (the product of two bf16 values is exact in fp32).
template <typename T>
__device__ __forceinline__ float outer_value(const T* __restrict__ e, const T* __restrict__ h, int64_t col, int64_t main,
                                             int64_t dh, int64_t D) {
    if (col >= D) return 0.f;
    if constexpr (sizeof(T) == 2) {
        if (col >= main) return bf16_to_f32(e[col - main]);
        const float x = bf16_to_f32(e[col / dh]) * bf16_to_f32(h[col % dh]);
        return (float)(__bf16)x;
    } else {
        if (col >= main) return e[col - main];
        return e[col / dh] * h[col % dh];
    }
}

// Same grid as insert_kernel: one thread writes 4 columns of one row into the slab layout.
template <typename T>
__global__ __launch_bounds__(256) void insert_outer_kernel(const T* __restrict__ E, const T* __restrict__ H, int64_t C,
                                                           int64_t dh, int row0, float* __restrict__ B, int NP, int64_t D,
                                                           int64_t S) {
    int64_t piece = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (piece >= S * 4) return;
    const int64_t r = blockIdx.y, d0 = piece * 4, main = C * dh;
    const T* e = E + r * C;
    const T* h = H + r * dh;
    float v[4];
    if (d0 + 3 < main) {  // one division per thread: the class and feature of column d0, then step with wrap-around
        int64_t cls = d0 / dh, t = d0 - cls * dh;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if constexpr (sizeof(T) == 2) v[c] = (float)(__bf16)(bf16_to_f32(e[cls]) * bf16_to_f32(h[t]));
            else v[c] = e[cls] * h[t];
            if (++t == dh) {
                t = 0;
                ++cls;
            }
        }
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = outer_value(e, h, d0 + c, main, dh, D);
    }
    float4* dst = reinterpret_cast<float4*>(B + blk_off(d0, row0 + (int)r, NP));
    *dst = make_float4(v[0], v[1], v[2], v[3]);
}

hipError_t launch_insert_outer(const void* E, const void* H, int dtype, int64_t C, int64_t dh, int64_t rows, int row0,
                               float* half, int half_rows, const Dims& d, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    dim3 grid((unsigned)((d.S * 4 + 255) / 256), (unsigned)rows);
    if (dtype == SAGE_BF16)
        hipLaunchKernelGGL(insert_outer_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)E, (const uint16_t*)H, C,
                           dh, row0, half, half_rows, d.D, d.S);
    else
        hipLaunchKernelGGL(insert_outer_kernel<float>, grid, dim3(256), 0, st, (const float*)E, (const float*)H, C, dh, row0,
                           half, half_rows, d.D, d.S);
    return hipGetLastError();
}

// The same rows written out row-major in their own type (for shapes the factored projection does not take).
template <typename T>
__global__ __launch_bounds__(256) void expand_outer_kernel(const T* __restrict__ E, const T* __restrict__ H, int64_t C,
                                                           int64_t dh, T* __restrict__ out, int64_t D) {
    const int64_t col = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (col >= D) return;
    const int64_t r = blockIdx.y;
    const float x = outer_value(E + r * C, H + r * dh, col, C * dh, dh, D);
    if constexpr (sizeof(T) == 2) out[r * D + col] = (uint16_t)(__float_as_uint(x) >> 16);  // x is a bf16 value already
    else out[r * D + col] = x;
}

hipError_t launch_expand_outer(const void* E, const void* H, int dtype, int64_t C, int64_t dh, int64_t rows, void* out,
                               const Dims& d, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    dim3 grid((unsigned)((d.D + 255) / 256), (unsigned)rows);
    if (dtype == SAGE_BF16)
        hipLaunchKernelGGL(expand_outer_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)E, (const uint16_t*)H, C,
                           dh, (uint16_t*)out, d.D);
    else
        hipLaunchKernelGGL(expand_outer_kernel<float>, grid, dim3(256), 0, st, (const float*)E, (const float*)H, C, dh,
                           (float*)out, d.D);
    return hipGetLastError();
}

// slab layout (NPsrc rows) -> row-major nrows x D
__global__ __launch_bounds__(256) void export_kernel(const float* __restrict__ Bblk, int NPsrc, float* __restrict__ out,
                                                     int64_t D) {
    int64_t dcol = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (dcol >= D) return;
    int r = blockIdx.y;
    out[(int64_t)r * D + dcol] = Bblk[blk_off(dcol, r, NPsrc)];
}

hipError_t launch_export_rows(const float* Bblk, int NPsrc, int nrows, float* out, const Dims& d, hipStream_t st) {
    if (nrows <= 0) return hipSuccess;
    dim3 grid((unsigned)((d.D + 255) / 256), (unsigned)nrows);
    hipLaunchKernelGGL(export_kernel, grid, dim3(256), 0, st, Bblk, NPsrc, out, d.D);
    return hipGetLastError();
}

// row-major nrows x D -> slab layout with NPdst rows; rows nrows..NPdst-1 and columns >= D are zeroed.
__global__ __launch_bounds__(256) void import_kernel(const float* __restrict__ in, int nrows, float* __restrict__ Bblk,
                                                     int NPdst, int64_t D, int64_t Dp) {
    int64_t dcol = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (dcol >= Dp) return;
    int r = blockIdx.y;
    float v = (r < nrows && dcol < D) ? in[(int64_t)r * D + dcol] : 0.f;
    Bblk[blk_off(dcol, r, NPdst)] = v;
}

hipError_t launch_import_rows(const float* in, int nrows, float* Bblk, int NPdst, const Dims& d, hipStream_t st) {
    dim3 grid((unsigned)((d.Dp + 255) / 256), (unsigned)NPdst);
    hipLaunchKernelGGL(import_kernel, grid, dim3(256), 0, st, in, nrows, Bblk, NPdst, d.D, d.Dp);
    return hipGetLastError();
}

// out[r][c] = in[map(r)][both ? map(c) : c] with map = buffer-row order -> matrix index: r < ell -> r,
// ell <= r < 2 ell -> LP + r - ell, then the padding indices in ascending order.
__device__ __forceinline__ int probe_map(int r, int LP, int ell) {
    if (r < ell) return r;
    if (r < 2 * ell) return LP + r - ell;
    int k = r - 2 * ell;                    // k-th padding index
    return k < LP - ell ? ell + k : LP + ell + (k - (LP - ell));
}
__global__ __launch_bounds__(256) void probe_permute_kernel(const double* __restrict__ in, double* __restrict__ out, int NP,
                                                            int LP, int ell, int both) {
    int r = blockIdx.x;
    int mr = probe_map(r, LP, ell);
    for (int c = threadIdx.x; c < NP; c += 256) {
        int mc = both ? probe_map(c, LP, ell) : c;
        out[(int64_t)r * NP + c] = in[(int64_t)mr * NP + mc];
    }
}

hipError_t launch_probe_permute(const double* in, double* out, int NP, int LP, int ell, bool both, hipStream_t st) {
    hipLaunchKernelGGL(probe_permute_kernel, dim3(NP), dim3(256), 0, st, in, out, NP, LP, ell, both ? 1 : 0);
    return hipGetLastError();
}

// plain copy, 16 bytes per thread (harnesses time / count it to calibrate hardware counters)
__global__ __launch_bounds__(256) void plain_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst, int64_t n16) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

hipError_t launch_plain_copy(const void* src, void* dst, int64_t bytes, hipStream_t st) {
    const int64_t n16 = bytes / 16;
    if (n16 <= 0) return hipSuccess;
    hipLaunchKernelGGL(plain_copy_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st, (const f32x4*)src,
                       (f32x4*)dst, n16);
    return hipGetLastError();
}

// Debug check of caller data: *count += the number of entries that are not finite (exponent bits all ones).
template <typename T>
__global__ __launch_bounds__(256) void count_nonfinite_kernel(const T* __restrict__ p, int64_t n, unsigned* __restrict__ count) {
    unsigned bad = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        if (sizeof(T) == 2) bad += (((unsigned)p[i]) & 0x7F80u) == 0x7F80u;
        else bad += (((unsigned)p[i]) & 0x7F800000u) == 0x7F800000u;
    }
    for (int o = 32; o >= 1; o >>= 1) bad += __shfl_xor(bad, o);
    if ((threadIdx.x & 63) == 0 && bad) atomicAdd(count, bad);
}

hipError_t launch_count_nonfinite(const void* p, int dtype, int64_t n, unsigned* count, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    if (dtype == SAGE_BF16)
        hipLaunchKernelGGL(count_nonfinite_kernel<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, st, (const uint16_t*)p, n, count);
    else
        hipLaunchKernelGGL(count_nonfinite_kernel<uint32_t>, dim3((unsigned)blocks), dim3(256), 0, st, (const uint32_t*)p, n, count);
    return hipGetLastError();
}

// zero buffer rows [r0, r1) in every slab
__global__ __launch_bounds__(256) void zero_rows_kernel(float* __restrict__ Bblk, int NP, int r0, int r1, int64_t S) {
    int per_slab = (r1 - r0) * 4;  // float4 pieces per slab
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= S * per_slab) return;
    int64_t s = i / per_slab;
    int rem = (int)(i % per_slab);
    float4* p = reinterpret_cast<float4*>(Bblk + (s * NP + r0) * DC) + rem;
    *p = make_float4(0.f, 0.f, 0.f, 0.f);
}

hipError_t launch_zero_rows(float* Bblk, int NP, int r0, int r1, const Dims& d, hipStream_t st) {
    if (r1 <= r0) return hipSuccess;
    int64_t total = d.S * (int64_t)(r1 - r0) * 4;
    hipLaunchKernelGGL(zero_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, Bblk, NP, r0, r1, d.S);
    return hipGetLastError();
}

}  // namespace sage
