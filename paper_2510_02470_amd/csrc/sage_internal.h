// Internal declarations shared by the translation units of the SAGE HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sage.h"

namespace sage {

// ---- sketch / basis layout --------------------------------------------------------------------------------
// The 2*ell x D buffer is kept as column slabs: element (row r, column d) lives at
//     ((d / DC) * NP + r) * DC + d % DC
// with DC = 16 floats (64 B) per row per slab and NP = padded row count. One slab (NP x 16 floats) is one
// contiguous block, so the Gram kernel stages a slab with linear 1 KB wave loads, and the rebuild / basis
// kernels read a 128 B line per buffer-row pair. Columns D..Dp-1 and rows beyond 2*ell are always zero.
constexpr int DC = 16;

struct Dims {
    int ell;      // sketch size
    int n;        // 2*ell buffer rows
    int LP;       // ell padded to 32 * 2^j (32, 64, 128, 256)
    int NP;       // 2*LP padded buffer rows (64 .. 512)
    int64_t D;    // columns
    int64_t S;    // slabs = ceil(D / DC)
    int64_t Dp;   // S * DC
};

__host__ __device__ inline int64_t blk_off(int64_t d, int r, int NP) {
    return ((d / DC) * NP + r) * (int64_t)DC + (d % DC);
}

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));  // indexable 16-byte piece

// fp32 matrix-core step: acc(32x32) += a(32x2) * b(2x32). Lane l supplies a[l%32][l/32] and b[l/32][l%32];
// acc element i of lane l is row 8*(i/4) + 4*(l/32) + i%4, column l%32.
__device__ __forceinline__ f32x16 mfma32(float a, float b, f32x16 acc) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

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

// An fp32 pair as three bf16 pairs hi + mid + lo (each the nearest bf16 of what the previous ones left): the three
// parts carry 24 significant bits, |x - hi - mid - lo| <= 2^-26 |x|.
__device__ __forceinline__ void split3_bf16(float x, float y, unsigned& hi, unsigned& mid, unsigned& lo) {
    hi = pack_bf16(x, y);
    const float rx = x - __uint_as_float(hi << 16), ry = y - __uint_as_float(hi & 0xffff0000u);
    mid = pack_bf16(rx, ry);
    lo = pack_bf16(rx - __uint_as_float(mid << 16), ry - __uint_as_float(mid & 0xffff0000u));
}

// The upper halves of an fp32 pair as a bf16 pair: exact when both are bf16 values (rows of a bf16 stream kept as fp32).
__device__ __forceinline__ unsigned hi_bf16(float x, float y) {
    return __builtin_amdgcn_perm(__float_as_uint(y), __float_as_uint(x), 0x07060302u);
}

// ---- kernel launchers (each enqueues on `st` and returns hipGetLastError()) ---------------------------------
// launch_util.hip: raise a kernel's dynamic LDS limit, once per (device, kernel); thread-safe
hipError_t ensure_dynamic_lds(const void* kernel, int bytes);
// fd_insert.hip
// copy `rows` batch rows into rows row0.. of a half buffer (half_rows rows per slab)
hipError_t launch_insert(const void* G, int dtype, int64_t rows, int row0, float* half, int half_rows, const Dims& d,
                         hipStream_t st);
// factored rows (E: rows x C logit errors, H: rows x dh features, both of the row type): column c*dh + t = e_c * h_t
// rounded as a stored row would be, column C*dh + c = e_c; requires D = C * (dh + 1)
hipError_t launch_insert_outer(const void* E, const void* H, int dtype, int64_t C, int64_t dh, int64_t rows, int row0,
                               float* half, int half_rows, const Dims& d, hipStream_t st);
// ... written out row-major (rows x D of the row type)
hipError_t launch_expand_outer(const void* E, const void* H, int dtype, int64_t C, int64_t dh, int64_t rows, void* out,
                               const Dims& d, hipStream_t st);
hipError_t launch_plain_copy(const void* src, void* dst, int64_t bytes, hipStream_t st);
// *count += entries of p (n values of the row type) that are not finite
hipError_t launch_count_nonfinite(const void* p, int dtype, int64_t n, unsigned* count, hipStream_t st);
hipError_t launch_probe_permute(const double* in, double* out, int NP, int LP, int ell, bool both, hipStream_t st);
hipError_t launch_export_rows(const float* Bblk, int NPsrc, int nrows, float* out, const Dims& d, hipStream_t st);
hipError_t launch_import_rows(const float* in, int nrows, float* Bblk, int NPdst, const Dims& d, hipStream_t st);
hipError_t launch_zero_rows(float* Bblk, int NP, int r0, int r1, const Dims& d, hipStream_t st);

// fd_gram.hip
// The buffer is two half buffers (top: matrix rows 0 .. LP-1, new: matrix rows LP .. NP-1, the first nfill in use).
struct GramPlan {
    int mode;         // 0: tiles t0.. of the lower triangle; 1: new rows x top rows; 2: new rows x new rows (triangle)
    int t0;           // mode 0: first tile computed (the top x top block before it is known to the caller)
    int tiles;        // 64x64 tiles computed
    int wg_per_group; // ceil(tiles / 6): a work-group computes 12 half-tiles
    int groups;       // split-K groups (multiple of 8)
    int64_t slabs_per_group;
    size_t partial_floats; // groups * tiles * 4096
    bool split = false;    // modes 1 and 2, NP = 512 only: the kernels on the bf16 matrix cores (three-way split values)
};
// The plan of the same block (mode 1 or 2) for the split-arithmetic kernels: one work-group per group, same partial
// tiles; groups > 0 overrides the group count (tiles = 0 in the result: not available for this sketch size).
GramPlan gram_plan_split(const GramPlan& base, const Dims& d, int groups);
GramPlan gram_plan(const Dims& d, int num_cu, int mode, bool skip_top, int wg_per_cu);
// new_one: every new row in use holds bf16 values (one part instead of three in the split-arithmetic kernels; the
// result has the same bits)
hipError_t launch_gram(const float* top, const float* nw, int nfill, float* partial, const GramPlan& p, const Dims& d,
                       hipStream_t st, bool new_one = false);
// C = sum of the partial tiles of launch a and (if given) launch b; known_top: the top x top block is `known`
// (LP x LP, the Gram matrix of the rows the last shrink wrote, see EigWork::known)
hipError_t launch_gram_reduce(const float* partial_a, const GramPlan& a, const float* partial_b, const GramPlan* b,
                              double* C, bool known_top, const double* known, const Dims& d, hipStream_t st);

// fd_eig.hip
struct EigWork {
    double* C;      // NP x NP, destroyed (becomes near-diagonal)
    double* Y;      // NP x NP eigenvectors in columns
    double* C2;     // ping-pong partners of C and Y for the out-of-place rotation updates
    double* Y2;
    double* Q;      // (NP/64) x 64 x 64 rotation blocks of the current step
    double* diag0;  // NP: diagonal of C before the solve
    double* stat;   // [0] trace, [1..MAXSWEEP] per-sweep max |off| / trace
    int* pos;       // NP: pos[rank] = column of Y holding the rank-th largest eigenvalue
    double* lam;    // NP: eigenvalues sorted descending
    double* known;  // LP x LP: Gram matrix of the rows the last shrink wrote, diag(w) (Y^T C Y) diag(w): diagonal
                    // lambda_j - delta (0 from row ell-1 on), off-diagonal whatever the eigensolve left (<= its tolerance)
};
constexpr int MAX_SWEEPS = 14;
// Stopping rule: a sweep records the largest |c_pq| / trace(C) it met before rotating; the solve ends after the
// first sweep whose record is <= tol. The shrink only needs the residual to be below the fp32 error of the Gram
// matrix (~1e-7 trace); the scoring basis is taken once per pass and is solved tighter.
constexpr double JACOBI_TOL_SHRINK = 1e-7;
constexpr double JACOBI_TOL_BASIS = 1e-9;
// max_sweeps <= MAX_SWEEPS sweeps are launched (sweeps after convergence return at once). acc[3] of the coefficient
// kernels then holds the sweeps that were needed, or max_sweeps + SWEEPS_NOT_CONVERGED when they did not suffice;
// acc[4] counts the solves that ended above their tolerance, acc[5] is the last solve's final off-diagonal record.
constexpr int SWEEPS_NOT_CONVERGED = 100;
hipError_t launch_eig(const EigWork& w, int NP, double tol, int max_sweeps, hipStream_t st);
// scalars on device: acc[0] sum_delta, acc[1] frob2, acc[2] last_delta, acc[3] sweeps used (as double), acc[4], acc[5]
// frob2 += diag0 over matrix indices [ra0, ra1) and [rb0, rb1) (the rows not yet counted in ||A||_F^2)
hipError_t launch_shrink_coeffs(const EigWork& w, int NP, int LP, int ell, int ra0, int ra1, int rb0, int rb1, float* Mt,
                                double* acc, double tol, hipStream_t st);
// weighted: rows sqrt(max(lambda_j - lambda_ell, 0)) v_j^T instead of v_j^T
hipError_t launch_basis_coeffs(const EigWork& w, int NP, int KP, int k, int n, int ell, bool weighted, int ra0, int ra1,
                               int rb0, int rb1, float* Mt, double* acc, double tol, hipStream_t st);

// Where the coefficient M[m][i] (output row m < MP, buffer row i < NP) is stored for the rebuild kernel: chunks of
// 16 buffer rows; inside a chunk [i & 1][m][(i & 15) >> 1], i.e. the 8 values a matrix-core lane needs are
// contiguous, and the two 16-byte halves of those 32 bytes are swapped when (m >> 3) is odd so that a quarter wave
// reading one half touches every LDS bank once.
__host__ __device__ inline int64_t coeff_offset(int i, int m, int MP) {
    const int s = (i & 15) >> 1, h = i & 1;
    const int piece = (s >> 2) ^ ((m >> 3) & 1);
    return (int64_t)(i >> 4) * 16 * MP + ((h * MP + m) * 2 + piece) * 4 + (s & 3);
}

// fd_rebuild.hip: out[0:MP] = M * B over every column, B = [top; first nfill rows of nw; zeros]; Mc holds the NP x MP
// coefficients in coeff_offset order; out has out_NP rows per slab and may be `top` itself (in place).
hipError_t launch_rebuild(const float* top, const float* nw, int nfill, const float* Mc, float* out, int out_NP, int MP,
                          const Dims& d, hipStream_t st);
// The same product on the bf16 matrix cores with both factors split into three bf16 parts (six products: 24-bit
// accuracy at 2.7 times the fp32 matrix-core rate). Mc3: work space of rebuild_split_bytes(d, MP) bytes (receives the
// split coefficients). Only for MP = 128 or 256 (rebuild_split_ok).
bool rebuild_split_ok(int MP);
size_t rebuild_split_bytes(const Dims& d, int MP);
// new_one: as for launch_gram (three products instead of six for the new half).
hipError_t launch_rebuild_split(const float* top, const float* nw, int nfill, const float* Mc, void* Mc3, float* out,
                                int out_NP, int MP, const Dims& d, hipStream_t st, bool new_one = false);

// score.hip
struct ScorePlan {
    int row_tiles;    // ceil(R / 128)
    int splits;       // split-K over D
    int64_t slabs_per_split;
    // factored rows only: the splits form a grid of class groups x feature-window groups
    int class_groups = 0, classes_per_group = 0, window_groups = 0, windows_per_group = 0;
    int bias_slots = 0, classes_per_bias_slot = 0;  // ... followed by the slots of the bias columns
};
ScorePlan score_plan(int64_t R, const Dims& d, int num_cu);
hipError_t launch_project(const void* G, int dtype, int64_t R, const float* Vblk, int KP, float* partial,
                          const ScorePlan& p, const Dims& d, hipStream_t st);
hipError_t launch_score_finalize(const float* partial, int64_t R, int KP, int k, int splits, float* zhat_out,
                                 double* cons_partial, double* ssum, int mode, float* alpha_out, hipStream_t st);

// score_split.hip: the same projection on the bf16 matrix cores with the basis split as hi + lo (bf16 each).
// The basis is kept as per-chunk LDS images built once per basis by launch_basis_split (from the fp32 slabs).
// Usable when every row starts on a 16-byte boundary (split_path_ok); ScorePlan::slabs_per_split then counts
// chunks of 128 row bytes.
bool split_path_ok(const void* G, int dtype, const Dims& d);
size_t basis_image_bytes(int KP, int dtype, const Dims& d);
hipError_t launch_basis_split(const float* Vblk, int KP, int dtype, void* img, const Dims& d, hipStream_t st);
ScorePlan score_split_plan(int64_t R, int dtype, const Dims& d, int num_cu);
hipError_t launch_project_split(const void* G, int dtype, int64_t R, const void* img, int KP, float* partial,
                                const ScorePlan& p, const Dims& d, hipStream_t st);

// The projection of factored rows (see launch_insert_outer) without storing them. Needs the images and the fp32 slabs
// of the basis; writes p.splits + p.bias_slots partial slots (the last ones hold the bias columns).
bool outer_path_ok(const void* E, const void* H, int dtype, int64_t C, int64_t dh);
ScorePlan score_outer_plan(int64_t R, int dtype, int64_t C, int64_t dh, int num_cu);
// work: outer_work_bytes(R, dtype, C) bytes (receives the transposed errors)
size_t outer_work_bytes(int64_t R, int dtype, int64_t C);
hipError_t launch_project_outer(const void* E, const void* H, int dtype, int64_t R, int64_t C, int64_t dh, void* work,
                                const void* img, const float* Vblk, int KP, float* partial, const ScorePlan& p,
                                hipStream_t st);

// select.hip
hipError_t launch_cosine(const float* zhat, int64_t N, int k, const double* ssum, float* alpha, hipStream_t st);
struct SelectWork {
    uint32_t* hist;      // 256 bins
    uint32_t* state;     // [0] prefix key, [1] remaining m, [2] count greater, [3] ties to take
    uint32_t* blk_gt;    // per block: count of keys > threshold
    uint32_t* blk_eq;    // per block: count of keys == threshold
    int64_t nblk_cap;
};
constexpr int SELECT_BLOCK = 2048;  // keys per block in the compaction passes
hipError_t launch_topm(const float* alpha, int64_t N, int64_t m, int64_t* out_idx, const SelectWork& w,
                       hipStream_t st);

// select_cb.hip: class-balanced selection (per-class centroid, cosine to it, top k_c of every class)
struct CbWork {
    long long* sums;   // C x 128 fixed-point class sums of zhat
    double* ucls;      // C x 128 unit centroids
    uint32_t* counts;  // rows per class
    uint32_t* kc;      // rows kept per class
    uint32_t* prefix;  // radix-select state: key prefix decided so far (after the index phase: index threshold)
    uint32_t* remain;  // ... keys still to take among those matching the prefix
    uint32_t* thr;     // score-key threshold per class
    uint32_t* hist;    // C x 256 bins
    uint32_t* misc;    // [0] total kept, [1] a label was out of range
    uint32_t* blk;     // per block of SELECT_BLOCK rows: rows kept (then their exclusive scan)
    uint8_t* sel;      // per row: kept
};
size_t cb_work_bytes(int C, int64_t N);
CbWork cb_work_layout(void* base, int C, int64_t N);
// rule: sage_cb_rule (how the subset size is shared out among the classes)
hipError_t launch_cb_scores(const float* zhat, const int* labels, int64_t N, int k, int C, double keep, int rule,
                            float* alpha, const CbWork& w, hipStream_t st);
hipError_t launch_cb_select(const float* alpha, const int* labels, int64_t N, int C, int64_t* out_idx, const CbWork& w,
                            hipStream_t st);

}  // namespace sage
