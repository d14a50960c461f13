// Scoring pass, second half (Algorithm 1, Phase II: "u <- zbar/||zbar||", "alpha_i <- <zhat_i, u>",
// "Select top-k by alpha_i"): consensus direction, cosine scores, radix-select of the m-th largest score and a
// stable compaction of the selected indices in ascending order.
#include "sage_internal.h"

namespace sage {

// One wave per row (lane j holds coordinates j, j+64); every work-group first rebuilds u from the consensus sum.
// alpha_i = clamp(<zhat_i, u>, -1, 1), -0 stored as +0.
__global__ __launch_bounds__(256) void cosine_kernel(const float* __restrict__ zhat, int64_t N, int k,
                                                     const double* __restrict__ ssum, float* __restrict__ alpha) {
    __shared__ double u[128];
    __shared__ double red[128];
    const int tid = threadIdx.x;
    if (tid < 128) {
        double s = tid < k ? ssum[tid] : 0.0;
        u[tid] = s;
        red[tid] = s * s;
    }
    __syncthreads();
    for (int w = 64; w >= 1; w >>= 1) {  // fixed-shape tree
        if (tid < w) red[tid] += red[tid + w];
        __syncthreads();
    }
    const double nrm = sqrt(red[0]);
    __syncthreads();
    if (tid < 128) u[tid] = nrm > 0.0 ? u[tid] / nrm : 0.0;
    __syncthreads();
    const int wave = tid >> 6, lane = tid & 63;
    const double u0 = u[lane], u1 = u[lane + 64];
    for (int64_t r = (int64_t)blockIdx.x * 4 + wave; r < N; r += (int64_t)gridDim.x * 4) {
        const float* z = zhat + r * k;
        double a = 0.0;
        if (lane < k) a = (double)z[lane] * u0;
        if (lane + 64 < k) a += (double)z[lane + 64] * u1;
        for (int o = 32; o >= 1; o >>= 1) a += __shfl_xor(a, o);
        if (lane == 0) {
            if (a > 1.0) a = 1.0;
            if (a < -1.0) a = -1.0;
            float f = (float)a;
            if (f == 0.f) f = 0.f;  // -0 -> +0
            alpha[r] = f;
        }
    }
}

hipError_t launch_cosine(const float* zhat, int64_t N, int k, const double* ssum, float* alpha, hipStream_t st) {
    if (N <= 0) return hipSuccess;
    int64_t blocks = (N + 3) / 4;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(cosine_kernel, dim3((unsigned)blocks), dim3(256), 0, st, zhat, N, k, ssum, alpha);
    return hipGetLastError();
}

// order-preserving key: larger alpha <-> larger key; -0 and +0 share a key
__device__ __forceinline__ uint32_t score_key(float a) {
    uint32_t b = __float_as_uint(a);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// state: [0] prefix of the threshold key decided so far, [1] how many keys are still to be taken among those
// that match the prefix, [2] scratch, [3] scratch
__global__ void select_init_kernel(uint32_t* __restrict__ hist, uint32_t* __restrict__ state, uint32_t m) {
    int t = threadIdx.x;
    if (t < 256) hist[t] = 0;
    if (t == 0) { state[0] = 0; state[1] = m; state[2] = 0; state[3] = 0; }
}

// histogram of byte `shift/8` of the keys whose higher bytes equal the prefix
__global__ __launch_bounds__(256) void select_hist_kernel(const float* __restrict__ alpha, int64_t N, int shift,
                                                          const uint32_t* __restrict__ state,
                                                          uint32_t* __restrict__ hist) {
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t prefix = state[0];
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < N; i += (int64_t)gridDim.x * 256) {
        uint32_t key = score_key(alpha[i]);
        bool match = (shift == 24) ? true : ((key >> (shift + 8)) == prefix);
        if (match) atomicAdd(&h[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    uint32_t v = h[threadIdx.x];
    if (v) atomicAdd(&hist[threadIdx.x], v);
}

// walk the bins from the top until the remaining count is covered; extend the prefix; clear the histogram
__global__ void select_pick_kernel(uint32_t* __restrict__ hist, uint32_t* __restrict__ state) {
    if (threadIdx.x == 0) {
        uint32_t remaining = state[1];
        uint32_t cum = 0;
        int chosen = 0;
        for (int b = 255; b >= 0; --b) {
            uint32_t c = hist[b];
            if (cum + c >= remaining) { chosen = b; break; }
            cum += c;
        }
        state[0] = (state[0] << 8) | (uint32_t)chosen;
        state[1] = remaining - cum;
    }
    __syncthreads();
    if (threadIdx.x < 256) hist[threadIdx.x] = 0;
}

// per block of SELECT_BLOCK keys: how many are above / equal to the threshold key
__global__ __launch_bounds__(256) void select_count_kernel(const float* __restrict__ alpha, int64_t N,
                                                           const uint32_t* __restrict__ state,
                                                           uint32_t* __restrict__ blk_gt, uint32_t* __restrict__ blk_eq) {
    __shared__ uint32_t sg[256], se[256];
    const uint32_t T = state[0];
    int64_t base = (int64_t)blockIdx.x * SELECT_BLOCK + (int64_t)threadIdx.x * 8;
    uint32_t g = 0, e = 0;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        int64_t i = base + c;
        if (i < N) {
            uint32_t key = score_key(alpha[i]);
            g += key > T;
            e += key == T;
        }
    }
    sg[threadIdx.x] = g;
    se[threadIdx.x] = e;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) { sg[threadIdx.x] += sg[threadIdx.x + w]; se[threadIdx.x] += se[threadIdx.x + w]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) { blk_gt[blockIdx.x] = sg[0]; blk_eq[blockIdx.x] = se[0]; }
}

// exclusive scan of the per-block counts, in place (single work-group, sequential over chunks of 256 blocks)
__global__ __launch_bounds__(256) void select_scan_kernel(uint32_t* __restrict__ blk_gt, uint32_t* __restrict__ blk_eq,
                                                          int nblk) {
    __shared__ uint32_t sg[256], se[256];
    uint32_t carry_g = 0, carry_e = 0;
    for (int base = 0; base < nblk; base += 256) {
        int i = base + threadIdx.x;
        uint32_t g = i < nblk ? blk_gt[i] : 0, e = i < nblk ? blk_eq[i] : 0;
        sg[threadIdx.x] = g;
        se[threadIdx.x] = e;
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {  // Hillis-Steele inclusive scan
            uint32_t ag = 0, ae = 0;
            if ((int)threadIdx.x >= o) { ag = sg[threadIdx.x - o]; ae = se[threadIdx.x - o]; }
            __syncthreads();
            sg[threadIdx.x] += ag;
            se[threadIdx.x] += ae;
            __syncthreads();
        }
        if (i < nblk) {
            blk_gt[i] = carry_g + sg[threadIdx.x] - g;
            blk_eq[i] = carry_e + se[threadIdx.x] - e;
        }
        uint32_t tg = sg[255], te = se[255];
        __syncthreads();
        carry_g += tg;
        carry_e += te;
    }
}

// element i is kept when key > T, or key == T and fewer than `take` equal keys precede it; its output slot is
// (#greater before i) + min(#equal before i, take), which makes the output ascending in i.
__global__ __launch_bounds__(256) void select_emit_kernel(const float* __restrict__ alpha, int64_t N,
                                                          const uint32_t* __restrict__ state,
                                                          const uint32_t* __restrict__ blk_gt,
                                                          const uint32_t* __restrict__ blk_eq,
                                                          int64_t* __restrict__ out_idx) {
    __shared__ uint32_t sg[256], se[256];
    const uint32_t T = state[0], take = state[1];
    int64_t base = (int64_t)blockIdx.x * SELECT_BLOCK + (int64_t)threadIdx.x * 8;
    uint32_t keys[8];
    uint32_t g = 0, e = 0;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        int64_t i = base + c;
        keys[c] = 0;
        if (i < N) {
            keys[c] = score_key(alpha[i]);
            g += keys[c] > T;
            e += keys[c] == T;
        }
    }
    sg[threadIdx.x] = g;
    se[threadIdx.x] = e;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
        uint32_t ag = 0, ae = 0;
        if ((int)threadIdx.x >= o) { ag = sg[threadIdx.x - o]; ae = se[threadIdx.x - o]; }
        __syncthreads();
        sg[threadIdx.x] += ag;
        se[threadIdx.x] += ae;
        __syncthreads();
    }
    uint32_t gt_before = blk_gt[blockIdx.x] + sg[threadIdx.x] - g;
    uint32_t eq_before = blk_eq[blockIdx.x] + se[threadIdx.x] - e;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        int64_t i = base + c;
        if (i >= N) break;
        bool isg = keys[c] > T, ise = keys[c] == T;
        if (isg || (ise && eq_before < take)) {
            uint32_t slot = gt_before + (eq_before < take ? eq_before : take);
            out_idx[slot] = i;
        }
        gt_before += isg;
        eq_before += ise;
    }
}

hipError_t launch_topm(const float* alpha, int64_t N, int64_t m, int64_t* out_idx, const SelectWork& w,
                       hipStream_t st) {
    if (m <= 0 || N <= 0) return hipSuccess;
    int64_t nblk = (N + SELECT_BLOCK - 1) / SELECT_BLOCK;
    if (nblk > w.nblk_cap) return hipErrorInvalidValue;
    hipLaunchKernelGGL(select_init_kernel, dim3(1), dim3(256), 0, st, w.hist, w.state, (uint32_t)m);
    int64_t hb = (N + 255) / 256;
    if (hb > 1024) hb = 1024;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hipLaunchKernelGGL(select_hist_kernel, dim3((unsigned)hb), dim3(256), 0, st, alpha, N, shift, w.state, w.hist);
        hipLaunchKernelGGL(select_pick_kernel, dim3(1), dim3(256), 0, st, w.hist, w.state);
    }
    hipLaunchKernelGGL(select_count_kernel, dim3((unsigned)nblk), dim3(256), 0, st, alpha, N, w.state, w.blk_gt, w.blk_eq);
    hipLaunchKernelGGL(select_scan_kernel, dim3(1), dim3(256), 0, st, w.blk_gt, w.blk_eq, (int)nblk);
    hipLaunchKernelGGL(select_emit_kernel, dim3((unsigned)nblk), dim3(256), 0, st, alpha, N, w.state, w.blk_gt, w.blk_eq,
                       out_idx);
    return hipGetLastError();
}

}  // namespace sage
