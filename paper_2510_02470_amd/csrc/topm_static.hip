// Top-m selection for callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc): the radix-select work space lives in a file-scope device array instead of a per-call allocation.
// See sage_topm_static in include/sage.h.
#include <mutex>

#include "sage_internal.h"

namespace {

// Work space of one top-m run over at most SAGE_TOPM_STATIC_MAX_N keys: 256 histogram bins, 4 state words, and two
// per-block counters for every block of SELECT_BLOCK keys.
constexpr int64_t MAX_N = SAGE_TOPM_STATIC_MAX_N;
constexpr int64_t MAX_BLOCKS = (MAX_N + sage::SELECT_BLOCK - 1) / sage::SELECT_BLOCK;
constexpr size_t HIST_WORDS = 256, STATE_WORDS = 64;  // the state gets a 256-byte slot of its own
constexpr size_t SCRATCH_WORDS = HIST_WORDS + STATE_WORDS + 2 * (size_t)MAX_BLOCKS;

// One copy per GPU, at that GPU's own address; host code never uses this name as a pointer (it is a host-side stand-in
// there): it asks the runtime for the device address once per device and keeps it.
static __device__ __align__(256) uint32_t scratch[SCRATCH_WORDS];

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
uint32_t* g_ptr[MAX_DEVICES] = {nullptr};

// Device address of `scratch` on the current device (looked up on the first call per device).
int scratch_ptr(uint32_t** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return SAGE_ERR_HIP;
    }
    if (dev < 0 || dev >= MAX_DEVICES) return SAGE_ERR_ARG;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return SAGE_ERR_HIP;
        }
        g_ptr[dev] = (uint32_t*)p;
    }
    *out = g_ptr[dev];
    return SAGE_OK;
}

}  // namespace

extern "C" int sage_topm_static(const float* alpha, int64_t N, int64_t m, int64_t* out_idx, void* hip_stream) {
    if (N < 0 || m < 0 || m > N || (N > 0 && !alpha) || (m > 0 && !out_idx)) return SAGE_ERR_ARG;
    if (N > MAX_N) return SAGE_ERR_CAPACITY;
    if (m == 0) return SAGE_OK;
    uint32_t* base = nullptr;
    int rc = scratch_ptr(&base);
    if (rc != SAGE_OK) return rc;
    sage::SelectWork w{};
    w.hist = base;
    w.state = base + HIST_WORDS;
    w.blk_gt = base + HIST_WORDS + STATE_WORDS;
    w.blk_eq = w.blk_gt + MAX_BLOCKS;
    w.nblk_cap = MAX_BLOCKS;
    // the first kernel of the run clears the histogram and the state; every per-block counter that is read is
    // written earlier in the same run, so nothing of the previous call's contents is used
    if (sage::launch_topm(alpha, N, m, out_idx, w, (hipStream_t)hip_stream) != hipSuccess) {
        (void)hipGetLastError();
        return SAGE_ERR_HIP;
    }
    return SAGE_OK;
}
