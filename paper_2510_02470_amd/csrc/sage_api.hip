// C ABI of the SAGE hot-path library: context, state machine and kernel sequencing. See include/sage.h.
#include <math.h>
#include <new>
#include <stdlib.h>
#include <string.h>

#include "sage_internal.h"

using namespace sage;

namespace {

constexpr int NCLASS = 9;
constexpr int64_t SCORE_CHUNK = 2048;  // rows per projection launch
enum { K_GRAM = 0, K_REDUCE, K_EIG, K_COEFF, K_REBUILD, K_INSERT, K_PROJECT, K_FINALIZE, K_SELECT };

}  // namespace

struct sage_ctx {
    Dims d{};
    int dtype = SAGE_F32;
    hipStream_t st = nullptr;
    int num_cu = 256;

    // The 2*ell-row buffer is kept as two half buffers of LP rows each (column-slab layout): `top` holds buffer rows
    // 0 .. ell-1 (after a shrink: the rows it wrote), nw[cur] holds buffer rows ell .. 2*ell-1 as they arrive. Two new
    // halves alternate so that the rows of the next cycle can be stored, and their own Gram block formed, on a side
    // stream while the eigensolve of the current cycle runs.
    float* top = nullptr;
    float* nw[2] = {nullptr, nullptr};
    int cur = 0;
    hipStream_t st2 = nullptr;                   // side stream (only when the Gram has >= 2 row panels)
    hipEvent_t ev_mark = nullptr;                // context stream: the Gram matrix of the current cycle is complete
    hipEvent_t ev_side[2] = {nullptr, nullptr};  // side stream: rows stored in nw[i] and their Gram block formed
    bool pending_shrink = false;   // the buffer is full, its shrink waits for the next update call (see sage_fd_update)
    bool pre_stored = false;       // the side stream has stored the next ell rows of the running call in nw[cur]
    bool new_block_ready = false;  // ... and their Gram block is (or will be, see ev_side) in gram_partial_new[cur]
    GramPlan gp{};        // whole lower triangle
    GramPlan gp_skip{};   // without the top x top block (known after a shrink)
    GramPlan gp_cross{};  // new rows x top rows
    // ... and their counterparts for the split-arithmetic kernels (tiles = 0: not available for this sketch size)
    GramPlan gp_cross_split{}, gp_new_split{}, gp_new2_split{};
    const GramPlan* gp_side_used[2] = {nullptr, nullptr};  // the plan the side stream's launch into gram_partial_new[i] used
    GramPlan gp_new{};    // new rows x new rows, one work-group per CU (it shares the chip with the eigensolve)
    GramPlan gp_new2{};   // the same block with the chip to itself (context stream, when there was nothing to look ahead to)
    bool top_shrunk = false;  // top holds exactly what the last shrink wrote
    float* gram_partial = nullptr;
    float* gram_partial_new[2] = {nullptr, nullptr};
    EigWork ew{};
    float* Mt = nullptr;
    void* Mt3 = nullptr;   // the rebuild's coefficients split into bf16 parts (SAGE_MM_SPLIT)
    int mm_mode = SAGE_MM_SPLIT;
    // Rows of a bf16 stream are kept as fp32 but have one bf16 part, not three: the split-arithmetic kernels then skip
    // the products with the new rows' mid and lo parts (exact zeros; same bits). nw_bf16[i]: every row in use in nw[i]
    // came from a bf16 batch (row-major or factored; not sage_fd_merge's fp32 rows). one_part: the shortcut is allowed (off under SAGE_MM_SPLIT_ALL_PARTS).
    bool nw_bf16[2] = {false, false};
    bool one_part = true;
    double* acc = nullptr;  // [0] sum_delta [1] frob2 [2] last_delta [3] sweeps [4] unconverged solves [5] last off-diagonal

    bool poisoned = false;   // a HIP call failed while work of a call was partly enqueued: the state is not trustworthy
    int fail_in = 0;         // test hook (sage_debug_fail_launch): the fail_in-th launch from now fails without running
    bool debug_checks = false;      // sage_set_debug_checks: scan caller batches for non-finite values
    unsigned* dbg_count = nullptr;  // device counter of that scan

    // Sweeps to launch for a shrink's eigensolve (a sweep that finds the matrix converged returns at once, but its 30
    // launches still cost about 50 us): what the last read-back solve needed, plus two. The count comes back through
    // pinned host memory without the host ever waiting for it.
    int sweep_cap = MAX_SWEEPS;
    int sweep_hold = 0;      // solves still to be launched with every sweep after one came back unconverged
    int sweep_recent[8] = {0, 0, 0, 0, 0, 0, 0, 0};  // sweeps the last eight reported solves needed
    int sweep_recent_at = 0;
    bool sweeps_all = false; // sage_set_sweep_policy(SAGE_SWEEPS_ALL): always launch MAX_SWEEPS
    double* h_sweeps = nullptr;                    // pinned, SWEEP_RING slots
    hipEvent_t ev_sweeps[4] = {nullptr, nullptr, nullptr, nullptr};
    bool sweeps_pending[4] = {false, false, false, false};
    int sweeps_next = 0;

    int fill_top = 0, fill_new = 0;  // rows in use in top (0..ell) and in nw[cur] (0..ell)
    int cnt_top = 0, cnt_new = 0;    // of those, rows already counted in frob2
    int64_t rows_seen = 0, n_shrinks = 0;

    bool has_basis = false;
    int k = 0, KP = 0;
    float* Vblk = nullptr;
    int Vblk_KP = 0;
    void* Vimg = nullptr;      // bf16 hi/lo chunk images of the basis (score_split.hip); built when the rows allow it
    size_t Vimg_bytes = 0;
    bool img_ok = false;       // ... and usable for row-major batches of this D
    bool img_built = false;    // the images hold the current basis
    void* stage = nullptr;     // factored rows written out, for shapes the factored projection does not take
    size_t stage_bytes = 0;
    int proj_mode = SAGE_PROJ_AUTO;
    float* zhat = nullptr;
    int64_t cap_rows = 0, n_scored = 0;
    bool store_zhat = true;   // false: zhat is not kept; alpha comes from a second pass over the rows (sage_rescore)
    int64_t n_rescored = 0;
    int* labels = nullptr;       // class label of every scored row (sage_score_labeled), same capacity as zhat
    int64_t n_labeled = 0;       // rows of the current pass that came with a label
    void* cb_work = nullptr;     // work space of the class-balanced selection
    size_t cb_work_bytes = 0;
    bool fixed_cap = false;
    float* proj_partial = nullptr;
    size_t proj_partial_floats = 0;
    double* cons_partial = nullptr;
    double* ssum = nullptr;
    float* alpha = nullptr;
    int64_t alpha_cap = 0, alpha_n = 0;
    SelectWork sw{};

    bool prof = false;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    double prof_ms[NCLASS] = {0};
    int64_t prof_n[NCLASS] = {0};
};

namespace {

// A HIP call that fails in the middle of a library call leaves work of that call partly enqueued: the context is
// marked poisoned (every later call except sage_destroy returns SAGE_ERR_STATE). `c` must be in scope.
inline int hip_failed(sage_ctx* c) {
    (void)hipGetLastError();
    c->poisoned = true;
    return SAGE_ERR_HIP;
}
#define HIPCHK(expr)                                 \
    do {                                             \
        hipError_t e_ = (expr);                      \
        if (e_ != hipSuccess) return hip_failed(c);  \
    } while (0)

// first statement of every call on a context
#define ALIVE(c)                                      \
    do {                                              \
        if (!(c)) return SAGE_ERR_ARG;                \
        if ((c)->poisoned) return SAGE_ERR_STATE;     \
    } while (0)

#define ALLOC(ptr, bytes)                                                  \
    do {                                                                   \
        if (hipMalloc((void**)&(ptr), (bytes)) != hipSuccess) {            \
            (void)hipGetLastError();                                       \
            return SAGE_ERR_ALLOC;                                         \
        }                                                                  \
    } while (0)

// run a launcher, optionally bracketed by events of kernel class `cls`
template <typename F>
int run(sage_ctx* c, int cls, F&& f) {
    if (c->fail_in > 0 && --c->fail_in == 0) return hip_failed(c);  // sage_debug_fail_launch
    if (c->prof) HIPCHK(hipEventRecord(c->ev0, c->st));
    HIPCHK(f());
    if (c->prof) {
        HIPCHK(hipEventRecord(c->ev1, c->st));
        HIPCHK(hipEventSynchronize(c->ev1));
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, c->ev0, c->ev1));
        c->prof_ms[cls] += ms;
        c->prof_n[cls] += 1;
    }
    return SAGE_OK;
}

#define RUN(cls, call)                                         \
    do {                                                       \
        int rc_ = run(c, cls, [&]() -> hipError_t { return (call); }); \
        if (rc_ != SAGE_OK) return rc_;                        \
    } while (0)

int pad_pow2_32(int v) {
    int p = 32;
    while (p < v) p *= 2;
    return p;
}

bool use_side(const sage_ctx* c) { return c->st2 != nullptr; }

// Where rows come from: a row-major batch, or the two factors of last-layer gradient rows (sage_fd_update_outer).
struct RowSrc {
    const void* G = nullptr;  // rows x D, or
    const void* E = nullptr;  // rows x C logit errors and
    const void* H = nullptr;  // rows x dh features
    int64_t C = 0, dh = 0;
    int dtype = SAGE_F32;
    bool outer() const { return G == nullptr; }
    RowSrc after(int64_t rows, int64_t D) const {
        const size_t esz = dtype == SAGE_BF16 ? 2 : 4;
        RowSrc r = *this;
        if (outer()) {
            r.E = (const char*)E + (size_t)rows * C * esz;
            r.H = (const char*)H + (size_t)rows * dh * esz;
        } else {
            r.G = (const char*)G + (size_t)rows * D * esz;
        }
        return r;
    }
};

hipError_t insert_rows(const RowSrc& s, int64_t rows, int row0, float* half, int half_rows, const Dims& d, hipStream_t st) {
    if (s.outer()) return launch_insert_outer(s.E, s.H, s.dtype, s.C, s.dh, rows, row0, half, half_rows, d, st);
    return launch_insert(s.G, s.dtype, rows, row0, half, half_rows, d, st);
}

// Rows of `s` are about to be stored in nw[i] from row row0 on.
void note_new_rows(sage_ctx* c, int i, int row0, const RowSrc& s) {
    const bool b = s.dtype == SAGE_BF16;  // factored rows of a bf16 context are rounded to bf16 when they are stored
    c->nw_bf16[i] = row0 == 0 ? b : (c->nw_bf16[i] && b);
}
bool new_one(const sage_ctx* c, int i) { return c->one_part && c->nw_bf16[i]; }

constexpr int SWEEP_RING = 4;

// Pick up the sweep counts that have arrived and set the number of sweeps to launch next.
void poll_sweeps(sage_ctx* c) {
    for (int i = 0; i < SWEEP_RING; ++i) {
        if (!c->sweeps_pending[i]) continue;
        hipError_t e = hipEventQuery(c->ev_sweeps[i]);
        if (e == hipErrorNotReady) {
            (void)hipGetLastError();
            continue;
        }
        c->sweeps_pending[i] = false;
        if (e != hipSuccess) continue;
        const int used = (int)c->h_sweeps[i];
        if (used >= SWEEPS_NOT_CONVERGED) {
            // ran out (sage_stats counts it): every sweep is launched for the solves to come
            c->sweep_cap = MAX_SWEEPS;
            c->sweep_hold = 64;
        } else {
            c->sweep_recent[c->sweep_recent_at] = used;
            c->sweep_recent_at = (c->sweep_recent_at + 1) & 7;
            if (c->sweep_hold > 0) {
                c->sweep_hold -= 1;
            } else {
                int most = used;
                for (int v : c->sweep_recent) most = v > most ? v : most;
                c->sweep_cap = most + 2 < 4 ? 4 : (most + 2 > MAX_SWEEPS ? MAX_SWEEPS : most + 2);
            }
        }
    }
}

// After a shrink's coefficient kernels: send the sweep count (acc[3]) home.
void post_sweeps(sage_ctx* c) {
    const int i = c->sweeps_next;
    if (c->sweeps_pending[i] || !c->h_sweeps) return;  // slot still in flight: skip this one
    if (hipMemcpyAsync(c->h_sweeps + i, c->acc + 3, sizeof(double), hipMemcpyDeviceToHost, c->st) != hipSuccess ||
        hipEventRecord(c->ev_sweeps[i], c->st) != hipSuccess) {
        (void)hipGetLastError();
        return;
    }
    c->sweeps_pending[i] = true;
    c->sweeps_next = (i + 1) % SWEEP_RING;
}

// Gram + eigensolve of the buffer as it stands. After a shrink the Gram matrix of the top rows is known (the shrink
// recorded it: diagonal lambda_j - delta, off-diagonal what its eigensolve left), so their block is not recomputed.
int decompose(sage_ctx* c, double tol, bool full) {
    const bool skip = !full && c->top_shrunk && c->gp_skip.t0 > 0;
    if (skip && c->fill_new == 0) {
        // Only the rows the last shrink wrote are there: the Gram matrix is the block that shrink recorded, nothing to
        // compute (its off-diagonal entries are at most the shrink's tolerance: a sweep or two at a tighter one).
        GramPlan none = c->gp_skip;
        none.tiles = 0;
        RUN(K_REDUCE, launch_gram_reduce(c->gram_partial, none, nullptr, nullptr, c->ew.C, true, c->ew.known, c->d, c->st));
        RUN(K_EIG, launch_eig(c->ew, c->d.NP, tol, MAX_SWEEPS, c->st));
        return SAGE_OK;
    }
    if (skip && c->mm_mode == SAGE_MM_SPLIT && c->gp_cross_split.tiles > 0 && c->gp_new2_split.tiles > 0 &&
        !c->new_block_ready && !c->pre_stored) {
        // the two blocks that are not known, with the split-arithmetic kernels (the side stream is idle here: its
        // partial buffer of the current half is free)
        const bool one = new_one(c, c->cur);
        RUN(K_GRAM, launch_gram(c->top, c->nw[c->cur], c->fill_new, c->gram_partial, c->gp_cross_split, c->d, c->st, one));
        RUN(K_GRAM, launch_gram(c->top, c->nw[c->cur], c->fill_new, c->gram_partial_new[c->cur], c->gp_new2_split, c->d,
                                c->st, one));
        RUN(K_REDUCE, launch_gram_reduce(c->gram_partial, c->gp_cross_split, c->gram_partial_new[c->cur], &c->gp_new2_split,
                                         c->ew.C, true, c->ew.known, c->d, c->st));
    } else {
        const GramPlan& gp = skip ? c->gp_skip : c->gp;
        RUN(K_GRAM, launch_gram(c->top, c->nw[c->cur], c->fill_new, c->gram_partial, gp, c->d, c->st));
        RUN(K_REDUCE, launch_gram_reduce(c->gram_partial, gp, nullptr, nullptr, c->ew.C, skip, c->ew.known, c->d, c->st));
    }
    RUN(K_EIG, launch_eig(c->ew, c->d.NP, tol, MAX_SWEEPS, c->st));
    return SAGE_OK;
}

// The buffer is full: shrink it (Method, FD paragraph). Leaves top = the ell new rows and the other new half current.
// next / next_rows: what is left of the running update call after this buffer. If a whole further cycle of rows is
// there, they are stored in the other new half and their own Gram block is formed on the side stream while the
// eigensolve runs on the context stream (neither needs its result, and the eigensolve leaves most of the chip idle).
// The next ell rows of the running call into the other new half and their own Gram block, on the side stream.
int side_ahead(sage_ctx* c, const RowSrc* next) {
    // The other half was last read by the rebuild before last, which precedes the mark on the context stream.
    const int LP = c->d.LP, ell = c->d.ell, o = c->cur ^ 1;
    HIPCHK(hipEventRecord(c->ev_mark, c->st));
    HIPCHK(hipStreamWaitEvent(c->st2, c->ev_mark, 0));
    note_new_rows(c, o, 0, *next);
    HIPCHK(insert_rows(*next, ell, 0, c->nw[o], LP, c->d, c->st2));
    c->gp_side_used[o] = c->mm_mode == SAGE_MM_SPLIT && c->gp_new_split.tiles > 0 ? &c->gp_new_split : &c->gp_new;
    HIPCHK(launch_gram(c->top, c->nw[o], ell, c->gram_partial_new[o], *c->gp_side_used[o], c->d, c->st2, new_one(c, o)));
    HIPCHK(hipEventRecord(c->ev_side[o], c->st2));
    return SAGE_OK;
}

int shrink(sage_ctx* c, const RowSrc* next, int64_t next_rows) {
    const int LP = c->d.LP, ell = c->d.ell;
    const bool ahead = use_side(c) && !c->prof && next && next_rows >= ell;
    if (c->new_block_ready || (c->top_shrunk && c->gp_cross.tiles > 0)) {
        // The top x top block is known. The new x new block came from the side stream, or is formed here when there
        // was nothing to look ahead to (first cycle of a call); then only new x top is left.
        const bool split = c->mm_mode == SAGE_MM_SPLIT;
        const GramPlan* gn = c->gp_side_used[c->cur];
        if (c->new_block_ready) {
            HIPCHK(hipStreamWaitEvent(c->st, c->ev_side[c->cur], 0));
        } else {
            gn = split && c->gp_new2_split.tiles > 0 ? &c->gp_new2_split : &c->gp_new2;
            RUN(K_GRAM, launch_gram(c->top, c->nw[c->cur], ell, c->gram_partial_new[c->cur], *gn, c->d, c->st,
                                    new_one(c, c->cur)));
        }
        const GramPlan& gc = split && c->gp_cross_split.tiles > 0 ? c->gp_cross_split : c->gp_cross;
        RUN(K_GRAM, launch_gram(c->top, c->nw[c->cur], ell, c->gram_partial, gc, c->d, c->st, new_one(c, c->cur)));
        RUN(K_REDUCE, launch_gram_reduce(c->gram_partial, gc, c->gram_partial_new[c->cur], gn, c->ew.C, true,
                                         c->ew.known, c->d, c->st));
    } else {
        const bool skip = c->top_shrunk && c->gp_skip.t0 > 0;
        const GramPlan& gp = skip ? c->gp_skip : c->gp;
        RUN(K_GRAM, launch_gram(c->top, c->nw[c->cur], ell, c->gram_partial, gp, c->d, c->st));
        RUN(K_REDUCE, launch_gram_reduce(c->gram_partial, gp, nullptr, nullptr, c->ew.C, skip, c->ew.known, c->d, c->st));
    }
    c->new_block_ready = false;
    if (ahead) {
        // after the Gram launches of this cycle: started beside them, the side stream's work (all of it, or the insert
        // alone) slowed the cross block more than it gained under the eigensolve (28.4 k against 29.7 k rows/s at
        // D = 2,049,000, both ways)
        int rc = side_ahead(c, next);
        if (rc != SAGE_OK) return rc;
    }
    poll_sweeps(c);
    RUN(K_EIG, launch_eig(c->ew, c->d.NP, JACOBI_TOL_SHRINK, c->sweeps_all ? MAX_SWEEPS : c->sweep_cap, c->st));
    RUN(K_COEFF, launch_shrink_coeffs(c->ew, c->d.NP, LP, ell, c->cnt_top, c->fill_top, LP + c->cnt_new, LP + c->fill_new,
                                      c->Mt, c->acc, JACOBI_TOL_SHRINK, c->st));
    if (c->mm_mode == SAGE_MM_SPLIT && c->Mt3)
        RUN(K_REBUILD, launch_rebuild_split(c->top, c->nw[c->cur], ell, c->Mt, c->Mt3, c->top, LP, LP, c->d, c->st,
                                            new_one(c, c->cur)));
    else
        RUN(K_REBUILD, launch_rebuild(c->top, c->nw[c->cur], ell, c->Mt, c->top, LP, LP, c->d, c->st));
    post_sweeps(c);
    if (use_side(c)) c->cur ^= 1;  // two new halves alternate; with a single Gram panel there is only nw[0]
    c->fill_top = ell;
    c->cnt_top = ell;
    c->fill_new = 0;
    c->cnt_new = 0;
    c->pre_stored = ahead;
    c->new_block_ready = ahead;
    c->n_shrinks += 1;
    c->top_shrunk = true;
    return SAGE_OK;
}

// A shrink that was left for the next update call: do it now (something wants to see the sketch).
int flush_pending(sage_ctx* c) {
    if (!c->pending_shrink) return SAGE_OK;
    c->pending_shrink = false;
    return shrink(c, nullptr, 0);
}

void reset_scoring(sage_ctx* c) {
    c->n_scored = 0;
    c->n_rescored = 0;
    c->n_labeled = 0;
    c->alpha_n = 0;
}

int ensure_score_buffers(sage_ctx* c) {
    if (!c->ssum) ALLOC(c->ssum, 128 * sizeof(double));
    if (!c->cons_partial) ALLOC(c->cons_partial, (size_t)(SCORE_CHUNK / 4) * 128 * sizeof(double));  // one per 4 rows
    HIPCHK(hipMemsetAsync(c->ssum, 0, 128 * sizeof(double), c->st));
    return SAGE_OK;
}

int ensure_vblk(sage_ctx* c, int KP) {
    if (c->Vblk && c->Vblk_KP == KP) return SAGE_OK;
    if (c->Vblk) {
        HIPCHK(hipStreamSynchronize(c->st));
        HIPCHK(hipFree(c->Vblk));
        c->Vblk = nullptr;
    }
    ALLOC(c->Vblk, (size_t)c->d.S * KP * DC * sizeof(float));
    c->Vblk_KP = KP;
    return SAGE_OK;
}

// The bf16 hi/lo images of the basis in Vblk (score_split.hip).
int ensure_images(sage_ctx* c) {
    if (c->img_built) return SAGE_OK;
    const size_t need = basis_image_bytes(c->KP, c->dtype, c->d);
    if (need > c->Vimg_bytes) {
        if (c->Vimg) {
            HIPCHK(hipStreamSynchronize(c->st));
            (void)hipFree(c->Vimg);
            c->Vimg = nullptr;
            c->Vimg_bytes = 0;
        }
        ALLOC(c->Vimg, need);
        c->Vimg_bytes = need;
    }
    RUN(K_REBUILD, launch_basis_split(c->Vblk, c->KP, c->dtype, c->Vimg, c->d, c->st));
    c->img_built = true;
    return SAGE_OK;
}

// After Vblk holds a new basis: build the images when the split projection can be used for row-major batches of
// this D (factored rows build them on first use otherwise).
int finish_basis(sage_ctx* c) {
    c->img_ok = false;
    c->img_built = false;
    if (c->proj_mode == SAGE_PROJ_F32) return SAGE_OK;
    if (!split_path_ok(nullptr, c->dtype, c->d)) return SAGE_OK;  // nullptr is "aligned": only D is judged here
    int rc = ensure_images(c);
    if (rc != SAGE_OK) return rc;
    c->img_ok = true;
    return SAGE_OK;
}

int64_t keep_count(double keep_rate, int64_t N) {
    double x = floor(keep_rate * (double)N + 0.5);
    int64_t m = (int64_t)x;
    if (m < 0) m = 0;
    if (m > N) m = N;
    return m;
}

int alloc_select_work(SelectWork& w, int64_t N) {
    int64_t nblk = (N + SELECT_BLOCK - 1) / SELECT_BLOCK;
    if (nblk < 1) nblk = 1;
    ALLOC(w.hist, 256 * sizeof(uint32_t));
    ALLOC(w.state, 4 * sizeof(uint32_t));
    ALLOC(w.blk_gt, (size_t)nblk * sizeof(uint32_t));
    ALLOC(w.blk_eq, (size_t)nblk * sizeof(uint32_t));
    w.nblk_cap = nblk;
    return SAGE_OK;
}

void free_select_work(SelectWork& w) {
    if (w.hist) (void)hipFree(w.hist);
    if (w.state) (void)hipFree(w.state);
    if (w.blk_gt) (void)hipFree(w.blk_gt);
    if (w.blk_eq) (void)hipFree(w.blk_eq);
    w = SelectWork{};
}

}  // namespace

extern "C" {

const char* sage_strerror(int code) {
    switch (code) {
        case SAGE_OK: return "ok";
        case SAGE_ERR_ARG: return "bad argument";
        case SAGE_ERR_STATE: return "call not allowed in this state";
        case SAGE_ERR_ALLOC: return "allocation failed";
        case SAGE_ERR_HIP: return "HIP runtime error";
        case SAGE_ERR_CAPACITY: return "capacity exceeded";
        default: return "unknown status";
    }
}

int sage_fd_create_ex(sage_ctx** out, int ell, int64_t D, sage_dtype in_dtype, int64_t max_rows, void* hip_stream) {
    if (!out) return SAGE_ERR_ARG;
    *out = nullptr;
    if (ell < 2 || ell > 256 || D < 1 || max_rows < 0) return SAGE_ERR_ARG;
    if (in_dtype != SAGE_F32 && in_dtype != SAGE_BF16) return SAGE_ERR_ARG;
    sage_ctx* c = new (std::nothrow) sage_ctx();
    if (!c) return SAGE_ERR_ALLOC;
    c->d.ell = ell;
    c->d.n = 2 * ell;
    c->d.LP = pad_pow2_32(ell);
    c->d.NP = 2 * c->d.LP;
    c->d.D = D;
    c->d.S = (D + DC - 1) / DC;
    c->d.Dp = c->d.S * DC;
    c->dtype = in_dtype;
    c->st = (hipStream_t)hip_stream;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        delete c;
        return SAGE_ERR_HIP;
    }
    c->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const int P = c->d.NP / 64;
    c->gp = gram_plan(c->d, c->num_cu, 0, false, 2);
    c->gp_skip = gram_plan(c->d, c->num_cu, 0, P >= 2, 2);
    if (P >= 2) {
        c->gp_cross = gram_plan(c->d, c->num_cu, 1, false, 2);
        c->gp_new = gram_plan(c->d, c->num_cu, 2, false, 1);
        c->gp_new2 = gram_plan(c->d, c->num_cu, 2, false, 2);
        c->gp_cross_split = gram_plan_split(c->gp_cross, c->d, 0);
        c->gp_new2_split = gram_plan_split(c->gp_new2, c->d, 0);
        // beside the eigensolve: one work-group per CU, 16 CUs left free (see gram_plan); 64, 120 and 240 work-groups
        // gave the same update rate, 480 a lower one
        c->gp_new_split = gram_plan_split(c->gp_new2, c->d, c->num_cu > 32 ? (c->num_cu - 16) / 8 * 8 : 8);
    }
    c->fixed_cap = max_rows > 0;
    c->cap_rows = max_rows > 0 ? max_rows : 65536;

    auto fail = [&](int rc) {
        sage_destroy(c);
        return rc;
    };
    const int NP = c->d.NP;
    size_t hbytes = (size_t)c->d.S * c->d.LP * DC * sizeof(float);  // one half buffer
#define CALLOC(ptr, bytes)                                                        \
    do {                                                                          \
        if (hipMalloc((void**)&(ptr), (bytes)) != hipSuccess) {                   \
            (void)hipGetLastError();                                              \
            return fail(SAGE_ERR_ALLOC);                                          \
        }                                                                         \
    } while (0)
    CALLOC(c->top, hbytes);
    CALLOC(c->nw[0], hbytes);
    {
        size_t pf = c->gp.partial_floats;
        if (c->gp_skip.partial_floats > pf) pf = c->gp_skip.partial_floats;
        if (c->gp_cross.partial_floats > pf) pf = c->gp_cross.partial_floats;
        CALLOC(c->gram_partial, pf * sizeof(float));
    }
    if (P >= 2) {
        CALLOC(c->nw[1], hbytes);
        const size_t pn = c->gp_new.partial_floats > c->gp_new2.partial_floats ? c->gp_new.partial_floats
                                                                                : c->gp_new2.partial_floats;
        CALLOC(c->gram_partial_new[0], pn * sizeof(float));
        CALLOC(c->gram_partial_new[1], pn * sizeof(float));
        if (hipStreamCreateWithFlags(&c->st2, hipStreamNonBlocking) != hipSuccess) return fail(SAGE_ERR_HIP);
        if (hipEventCreateWithFlags(&c->ev_mark, hipEventDisableTiming) != hipSuccess) return fail(SAGE_ERR_HIP);
        for (int i = 0; i < 2; ++i)
            if (hipEventCreateWithFlags(&c->ev_side[i], hipEventDisableTiming) != hipSuccess) return fail(SAGE_ERR_HIP);
    }
    CALLOC(c->ew.C, (size_t)NP * NP * sizeof(double));
    CALLOC(c->ew.Y, (size_t)NP * NP * sizeof(double));
    CALLOC(c->ew.C2, (size_t)NP * NP * sizeof(double));
    CALLOC(c->ew.Y2, (size_t)NP * NP * sizeof(double));
    CALLOC(c->ew.Q, (size_t)(NP / 64) * 4096 * sizeof(double));
    CALLOC(c->ew.diag0, (size_t)NP * sizeof(double));
    CALLOC(c->ew.stat, 32 * sizeof(double));
    CALLOC(c->ew.pos, (size_t)NP * sizeof(int));
    CALLOC(c->ew.lam, (size_t)NP * sizeof(double));
    CALLOC(c->ew.known, (size_t)c->d.LP * c->d.LP * sizeof(double));
    CALLOC(c->Mt, (size_t)NP * c->d.LP * sizeof(float));
    if (rebuild_split_ok(c->d.LP)) CALLOC(c->Mt3, rebuild_split_bytes(c->d, c->d.LP));
    CALLOC(c->acc, 8 * sizeof(double));
#undef CALLOC
    // only the top half must start as zeros: rows of a new half beyond its fill are never read
    if (hipMemsetAsync(c->top, 0, hbytes, c->st) != hipSuccess) return fail(SAGE_ERR_HIP);
    if (hipMemsetAsync(c->acc, 0, 8 * sizeof(double), c->st) != hipSuccess) return fail(SAGE_ERR_HIP);
    if (hipEventCreate(&c->ev0) != hipSuccess || hipEventCreate(&c->ev1) != hipSuccess) return fail(SAGE_ERR_HIP);
    if (hipHostMalloc((void**)&c->h_sweeps, SWEEP_RING * sizeof(double), hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        c->h_sweeps = nullptr;  // not fatal: every solve then launches all its sweeps
    }
    for (int i = 0; i < SWEEP_RING; ++i)
        if (hipEventCreateWithFlags(&c->ev_sweeps[i], hipEventDisableTiming) != hipSuccess) return fail(SAGE_ERR_HIP);
    *out = c;
    return SAGE_OK;
}

int sage_fd_create(sage_ctx** out, int ell, int64_t D) { return sage_fd_create_ex(out, ell, D, SAGE_F32, 0, nullptr); }

void sage_destroy(sage_ctx* c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->st);
    if (c->st2) (void)hipStreamSynchronize(c->st2);
    void* ptrs[] = {c->top,     c->nw[0],    c->nw[1],  c->gram_partial, c->gram_partial_new[0], c->gram_partial_new[1],
                    c->ew.C,    c->ew.Y,     c->ew.C2,  c->ew.Y2,        c->ew.Q,    c->ew.diag0, c->ew.stat,
                    c->ew.pos,  c->ew.lam,   c->ew.known, c->Mt,         c->acc,     c->Vblk,     c->Vimg,
                    c->zhat,    c->proj_partial, c->cons_partial, c->ssum, c->alpha, c->labels, c->cb_work, c->stage, c->Mt3, c->dbg_count};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    if (c->st2) (void)hipStreamDestroy(c->st2);
    if (c->h_sweeps) (void)hipHostFree(c->h_sweeps);
    hipEvent_t evs[] = {c->ev_mark, c->ev_side[0], c->ev_side[1], c->ev_sweeps[0], c->ev_sweeps[1], c->ev_sweeps[2],
                        c->ev_sweeps[3]};
    for (hipEvent_t e : evs)
        if (e) (void)hipEventDestroy(e);
    free_select_work(c->sw);
    if (c->ev0) (void)hipEventDestroy(c->ev0);
    if (c->ev1) (void)hipEventDestroy(c->ev1);
    delete c;
}

int sage_sync(sage_ctx* c) {
    ALIVE(c);
    HIPCHK(hipStreamSynchronize(c->st));
    return SAGE_OK;
}

// Rows of type `dtype` (the context's own for sage_fd_update, fp32 for sage_fd_merge) go through the insert / shrink cycle.
static int update_rows(sage_ctx* c, RowSrc g, int64_t rows) {
    ALIVE(c);
    if (rows < 0) return SAGE_ERR_ARG;
    if (rows == 0) return SAGE_OK;
    c->has_basis = false;
    const int ell = c->d.ell, LP = c->d.LP;
    if (c->pending_shrink) {
        // the buffer filled up exactly at the end of the previous call: with this call's rows at hand the shrink can
        // look ahead
        c->pending_shrink = false;
        int rc = shrink(c, &g, rows);
        if (rc != SAGE_OK) return rc;
    }
    while (rows > 0) {
        int take;
        if (c->fill_top < ell) {
            // first fill of the buffer: rows go into the top half
            take = (int)((int64_t)(ell - c->fill_top) < rows ? (ell - c->fill_top) : rows);
            RUN(K_INSERT, insert_rows(g, take, c->fill_top, c->top, LP, c->d, c->st));
            c->fill_top += take;
        } else if (c->pre_stored) {
            // the previous shrink of this call has had these ell rows stored already (side stream)
            take = ell;
            c->pre_stored = false;
            c->fill_new = ell;
        } else {
            take = (int)((int64_t)(ell - c->fill_new) < rows ? (ell - c->fill_new) : rows);
            note_new_rows(c, c->cur, c->fill_new, g);
            RUN(K_INSERT, insert_rows(g, take, c->fill_new, c->nw[c->cur], LP, c->d, c->st));
            c->fill_new += take;
        }
        c->rows_seen += take;
        g = g.after(take, c->d.D);
        rows -= take;
        if (c->fill_new == ell) {
            if (rows == 0 && use_side(c) && c->top_shrunk && !c->prof) {
                // Nothing to look ahead to: leave the shrink to the next update call, which brings rows (whoever
                // looks at the sketch first does it otherwise). The side stream may still be reading this batch for
                // the half just completed: the context stream waits for it, so that the batch is free once this
                // call's work is complete there.
                c->pending_shrink = true;
                if (c->new_block_ready) HIPCHK(hipStreamWaitEvent(c->st, c->ev_side[c->cur], 0));
            } else {
                int rc = shrink(c, &g, rows);
                if (rc != SAGE_OK) return rc;
            }
        }
    }
    return SAGE_OK;
}

// sage_set_debug_checks: a batch with a non-finite entry is refused before anything is enqueued for it (the scan
// waits for the stream; the context is left as it was).
static int check_finite(sage_ctx* c, const void* p, int dtype, int64_t n) {
    if (!c->debug_checks || n <= 0 || !p) return SAGE_OK;
    if (!c->dbg_count) ALLOC(c->dbg_count, sizeof(unsigned));
    unsigned bad = 0;
    HIPCHK(hipMemsetAsync(c->dbg_count, 0, sizeof(unsigned), c->st));
    HIPCHK(launch_count_nonfinite(p, dtype, n, c->dbg_count, c->st));
    HIPCHK(hipMemcpyAsync(&bad, c->dbg_count, sizeof(unsigned), hipMemcpyDeviceToHost, c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    return bad ? SAGE_ERR_ARG : SAGE_OK;
}

static RowSrc dense_src(const void* G, int dtype) {
    RowSrc s;
    s.G = G;
    s.dtype = dtype;
    return s;
}

// factored rows must tile the context's row exactly: D = C * (dh + 1)
static bool outer_src(const sage_ctx* c, const void* E, const void* H, int64_t C, int64_t dh, RowSrc& s) {
    if (!E || !H || C < 1 || dh < 1 || dh > ((int64_t)1 << 40) / C || C * (dh + 1) != c->d.D) return false;
    s.E = E;
    s.H = H;
    s.C = C;
    s.dh = dh;
    s.dtype = c->dtype;
    return true;
}

int sage_fd_update(sage_ctx* c, const void* G_batch, int64_t rows) {
    ALIVE(c);
    if (rows > 0 && !G_batch) return SAGE_ERR_ARG;
    if (int rc = check_finite(c, G_batch, c->dtype, rows * c->d.D); rc != SAGE_OK) return rc;
    return update_rows(c, dense_src(G_batch, c->dtype), rows);
}

int sage_fd_update_outer(sage_ctx* c, const void* E, const void* H, int64_t rows, int64_t n_classes, int64_t n_features) {
    ALIVE(c);
    if (rows < 0) return SAGE_ERR_ARG;
    if (rows == 0) return SAGE_OK;
    RowSrc s;
    if (!outer_src(c, E, H, n_classes, n_features, s)) return SAGE_ERR_ARG;
    if (int rc = check_finite(c, E, c->dtype, rows * n_classes); rc != SAGE_OK) return rc;
    if (int rc = check_finite(c, H, c->dtype, rows * n_features); rc != SAGE_OK) return rc;
    return update_rows(c, s, rows);
}

int sage_fd_merge(sage_ctx* c, const float* B_other, int64_t rows) {
    ALIVE(c);
    if (rows > 0 && !B_other) return SAGE_ERR_ARG;
    if (int rc = check_finite(c, B_other, SAGE_F32, rows * c->d.D); rc != SAGE_OK) return rc;
    return update_rows(c, dense_src(B_other, SAGE_F32), rows);
}

static int basis_impl(sage_ctx* c, int k, bool weighted);

int sage_fd_basis(sage_ctx* c, int k) { return basis_impl(c, k, false); }

int sage_fd_basis_weighted(sage_ctx* c, int k) { return basis_impl(c, k, true); }

static int basis_impl(sage_ctx* c, int k, bool weighted) {
    ALIVE(c);
    if (k < 1 || k > c->d.ell - 1 || k > 128) return SAGE_ERR_ARG;
    const int KP = pad_pow2_32(k);
    int rc = flush_pending(c);
    if (rc != SAGE_OK) return rc;
    rc = ensure_vblk(c, KP);
    if (rc != SAGE_OK) return rc;
    rc = decompose(c, JACOBI_TOL_BASIS, false);
    if (rc != SAGE_OK) return rc;
    RUN(K_COEFF, launch_basis_coeffs(c->ew, c->d.NP, KP, k, c->d.n, c->d.ell, weighted, c->cnt_top, c->fill_top,
                                     c->d.LP + c->cnt_new, c->d.LP + c->fill_new, c->Mt, c->acc, JACOBI_TOL_BASIS, c->st));
    c->cnt_top = c->fill_top;
    c->cnt_new = c->fill_new;
    if (c->mm_mode == SAGE_MM_SPLIT && c->Mt3 && rebuild_split_ok(KP) && KP <= c->d.LP)
        RUN(K_REBUILD, launch_rebuild_split(c->top, c->nw[c->cur], c->fill_new, c->Mt, c->Mt3, c->Vblk, KP, KP, c->d, c->st,
                                            c->fill_new > 0 && new_one(c, c->cur)));
    else
        RUN(K_REBUILD, launch_rebuild(c->top, c->nw[c->cur], c->fill_new, c->Mt, c->Vblk, KP, KP, c->d, c->st));
    c->k = k;
    c->KP = KP;
    rc = finish_basis(c);
    if (rc != SAGE_OK) return rc;
    c->has_basis = true;
    reset_scoring(c);
    return ensure_score_buffers(c);
}

int sage_set_projection_mode(sage_ctx* c, int mode) {
    ALIVE(c);
    if ((mode != SAGE_PROJ_AUTO && mode != SAGE_PROJ_F32)) return SAGE_ERR_ARG;
    c->proj_mode = mode;
    c->has_basis = false;
    return SAGE_OK;
}

int sage_set_update_arithmetic(sage_ctx* c, int mode) {
    ALIVE(c);
    if (mode != SAGE_MM_F32 && mode != SAGE_MM_SPLIT && mode != SAGE_MM_SPLIT_ALL_PARTS) return SAGE_ERR_ARG;
    c->mm_mode = mode == SAGE_MM_F32 ? SAGE_MM_F32 : SAGE_MM_SPLIT;
    c->one_part = mode != SAGE_MM_SPLIT_ALL_PARTS;
    return SAGE_OK;
}

int sage_set_basis(sage_ctx* c, const float* Vt, int k) {
    ALIVE(c);
    if (!Vt || k < 1 || k > 128) return SAGE_ERR_ARG;
    const int KP = pad_pow2_32(k);
    int rc = ensure_vblk(c, KP);
    if (rc != SAGE_OK) return rc;
    HIPCHK(launch_import_rows(Vt, k, c->Vblk, KP, c->d, c->st));
    c->k = k;
    c->KP = KP;
    rc = finish_basis(c);
    if (rc != SAGE_OK) return rc;
    c->has_basis = true;
    reset_scoring(c);
    return ensure_score_buffers(c);
}

// split-K partial projections of one launch
static int ensure_partial(sage_ctx* c, size_t need) {
    if (need <= c->proj_partial_floats) return SAGE_OK;
    if (c->proj_partial) {
        HIPCHK(hipStreamSynchronize(c->st));
        (void)hipFree(c->proj_partial);
        c->proj_partial = nullptr;
        c->proj_partial_floats = 0;
    }
    size_t want = (size_t)512 * 128 * 128 > need ? (size_t)512 * 128 * 128 : need;
    ALLOC(c->proj_partial, want * sizeof(float));
    c->proj_partial_floats = want;
    return SAGE_OK;
}

// staging memory of the factored scoring calls
static int ensure_stage(sage_ctx* c, size_t need) {
    if (need <= c->stage_bytes) return SAGE_OK;
    if (c->stage) {
        HIPCHK(hipStreamSynchronize(c->st));
        (void)hipFree(c->stage);
        c->stage = nullptr;
        c->stage_bytes = 0;
    }
    ALLOC(c->stage, need);
    c->stage_bytes = need;
    return SAGE_OK;
}

// The projection partials of R rows (R <= SCORE_CHUNK) in proj_partial; *slots = partial slots to sum.
static int project_rows(sage_ctx* c, const RowSrc& src, int64_t R, int* slots) {
    const void* g = src.G;
    if (src.outer()) {
        if (c->proj_mode != SAGE_PROJ_F32 && outer_path_ok(src.E, src.H, src.dtype, src.C, src.dh)) {
            int rc = ensure_images(c);
            if (rc != SAGE_OK) return rc;
            rc = ensure_stage(c, outer_work_bytes(R, src.dtype, src.C));
            if (rc != SAGE_OK) return rc;
            ScorePlan p = score_outer_plan(R, src.dtype, src.C, src.dh, c->num_cu);
            rc = ensure_partial(c, (size_t)(p.splits + p.bias_slots) * R * c->KP);
            if (rc != SAGE_OK) return rc;
            RUN(K_PROJECT, launch_project_outer(src.E, src.H, src.dtype, R, src.C, src.dh, c->stage, c->Vimg, c->Vblk,
                                                c->KP, c->proj_partial, p, c->st));
            *slots = p.splits + p.bias_slots;
            return SAGE_OK;
        }
        // any other shape: write the rows out and project them like a row-major batch
        int rc = ensure_stage(c, (size_t)R * c->d.D * (src.dtype == SAGE_BF16 ? 2 : 4));
        if (rc != SAGE_OK) return rc;
        RUN(K_INSERT, launch_expand_outer(src.E, src.H, src.dtype, src.C, src.dh, R, c->stage, c->d, c->st));
        g = c->stage;
    }
    const bool split = c->img_ok && split_path_ok(g, c->dtype, c->d);
    ScorePlan p = split ? score_split_plan(R, c->dtype, c->d, c->num_cu) : score_plan(R, c->d, c->num_cu);
    int rc = ensure_partial(c, (size_t)p.splits * R * c->KP);
    if (rc != SAGE_OK) return rc;
    if (split)
        RUN(K_PROJECT, launch_project_split(g, c->dtype, R, c->Vimg, c->KP, c->proj_partial, p, c->d, c->st));
    else
        RUN(K_PROJECT, launch_project(g, c->dtype, R, c->Vblk, c->KP, c->proj_partial, p, c->d, c->st));
    *slots = p.splits;
    return SAGE_OK;
}

static int score_impl(sage_ctx* c, RowSrc g, const int* labels, int64_t rows);

int sage_score(sage_ctx* c, const void* G_batch, int64_t rows) {
    ALIVE(c);
    if (rows > 0 && !G_batch) return SAGE_ERR_ARG;
    if (int rc = check_finite(c, G_batch, c->dtype, rows * c->d.D); rc != SAGE_OK) return rc;
    return score_impl(c, dense_src(G_batch, c->dtype), nullptr, rows);
}

int sage_score_labeled(sage_ctx* c, const void* G_batch, const int32_t* labels, int64_t rows) {
    ALIVE(c);
    if (rows > 0 && (!labels || !G_batch)) return SAGE_ERR_ARG;
    if (int rc = check_finite(c, G_batch, c->dtype, rows * c->d.D); rc != SAGE_OK) return rc;
    return score_impl(c, dense_src(G_batch, c->dtype), labels, rows);
}

int sage_score_outer(sage_ctx* c, const void* E, const void* H, const int32_t* labels, int64_t rows, int64_t n_classes,
                     int64_t n_features) {
    ALIVE(c);
    if (rows < 0) return SAGE_ERR_ARG;
    if (!c->has_basis) return SAGE_ERR_STATE;
    if (rows == 0) return SAGE_OK;
    RowSrc s;
    if (!outer_src(c, E, H, n_classes, n_features, s)) return SAGE_ERR_ARG;
    if (int rc = check_finite(c, E, c->dtype, rows * n_classes); rc != SAGE_OK) return rc;
    if (int rc = check_finite(c, H, c->dtype, rows * n_features); rc != SAGE_OK) return rc;
    return score_impl(c, s, labels, rows);
}

static int score_impl(sage_ctx* c, RowSrc g, const int* labels, int64_t rows) {
    ALIVE(c);
    if (rows < 0) return SAGE_ERR_ARG;
    if (!c->has_basis) return SAGE_ERR_STATE;
    if (rows == 0) return SAGE_OK;
    if (!c->store_zhat && (labels || c->n_rescored > 0)) return SAGE_ERR_STATE;  // no labels without zhat; pass 2 is over
    if (c->store_zhat && !c->zhat) ALLOC(c->zhat, (size_t)c->cap_rows * 128 * sizeof(float));
    if (c->store_zhat && c->n_scored + rows > c->cap_rows) {
        if (c->fixed_cap) return SAGE_ERR_CAPACITY;
        int64_t ncap = c->cap_rows;
        while (ncap < c->n_scored + rows) ncap *= 2;
        float* nz = nullptr;
        ALLOC(nz, (size_t)ncap * 128 * sizeof(float));
        if (hipMemcpyAsync(nz, c->zhat, (size_t)c->n_scored * c->k * sizeof(float), hipMemcpyDeviceToDevice, c->st) !=
                hipSuccess ||
            hipStreamSynchronize(c->st) != hipSuccess) {
            (void)hipFree(nz);
            return hip_failed(c);
        }
        (void)hipFree(c->zhat);
        c->zhat = nz;
        if (c->labels) {
            int* nl = nullptr;
            ALLOC(nl, (size_t)ncap * sizeof(int));
            if (hipMemcpyAsync(nl, c->labels, (size_t)c->n_scored * sizeof(int), hipMemcpyDeviceToDevice, c->st) !=
                    hipSuccess ||
                hipStreamSynchronize(c->st) != hipSuccess) {
                (void)hipFree(nl);
                return hip_failed(c);
            }
            (void)hipFree(c->labels);
            c->labels = nl;
        }
        c->cap_rows = ncap;
    }
    if (labels) {
        if (!c->labels) ALLOC(c->labels, (size_t)c->cap_rows * sizeof(int));
        HIPCHK(hipMemcpyAsync(c->labels + c->n_scored, labels, (size_t)rows * sizeof(int), hipMemcpyDeviceToDevice, c->st));
        if (c->n_labeled == c->n_scored) c->n_labeled += rows;  // stays behind for good once an unlabeled batch came
    }
    while (rows > 0) {
        int64_t R = rows < SCORE_CHUNK ? rows : SCORE_CHUNK;
        int slots = 0;
        int rcp = project_rows(c, g, R, &slots);
        if (rcp != SAGE_OK) return rcp;
        RUN(K_FINALIZE, launch_score_finalize(c->proj_partial, R, c->KP, c->k, slots,
                                             c->store_zhat ? c->zhat + (size_t)c->n_scored * c->k : nullptr,
                                             c->cons_partial, c->ssum, c->store_zhat ? 0 : 1, nullptr, c->st));
        c->n_scored += R;
        g = g.after(R, c->d.D);
        rows -= R;
    }
    c->alpha_n = 0;
    return SAGE_OK;
}

// alpha capacity for N rows (and the selection work space that goes with it)
static int ensure_alpha(sage_ctx* c, int64_t N) {
    if (N <= c->alpha_cap) return SAGE_OK;
    float* na = nullptr;
    int64_t ncap = N > c->cap_rows ? N : c->cap_rows;
    ALLOC(na, (size_t)ncap * sizeof(float));
    if (c->alpha) {
        // keep what a running rescoring pass has written
        if (hipMemcpyAsync(na, c->alpha, (size_t)c->alpha_cap * sizeof(float), hipMemcpyDeviceToDevice, c->st) != hipSuccess ||
            hipStreamSynchronize(c->st) != hipSuccess) {
            (void)hipFree(na);
            return hip_failed(c);
        }
        (void)hipFree(c->alpha);
    }
    c->alpha = na;
    free_select_work(c->sw);
    int rc = alloc_select_work(c->sw, ncap);
    if (rc != SAGE_OK) return rc;
    c->alpha_cap = ncap;
    return SAGE_OK;
}

int sage_set_score_store(sage_ctx* c, int store_zhat) {
    ALIVE(c);
    c->store_zhat = store_zhat != 0;
    reset_scoring(c);
    if (c->ssum) HIPCHK(hipMemsetAsync(c->ssum, 0, 128 * sizeof(double), c->st));
    return SAGE_OK;
}

static int rescore_impl(sage_ctx* c, RowSrc g, int64_t rows) {
    ALIVE(c);
    if (!c->has_basis || c->store_zhat) return SAGE_ERR_STATE;
    if (c->n_rescored + rows > c->n_scored) return SAGE_ERR_STATE;  // more rows than the first pass saw
    if (rows == 0) return SAGE_OK;
    int rc = ensure_alpha(c, c->n_scored);
    if (rc != SAGE_OK) return rc;
    while (rows > 0) {
        int64_t R = rows < SCORE_CHUNK ? rows : SCORE_CHUNK;
        int slots = 0;
        rc = project_rows(c, g, R, &slots);
        if (rc != SAGE_OK) return rc;
        RUN(K_FINALIZE, launch_score_finalize(c->proj_partial, R, c->KP, c->k, slots, nullptr, c->cons_partial, c->ssum, 2,
                                             c->alpha + c->n_rescored, c->st));
        c->n_rescored += R;
        g = g.after(R, c->d.D);
        rows -= R;
    }
    c->alpha_n = c->n_rescored == c->n_scored ? c->n_scored : 0;
    return SAGE_OK;
}

int sage_rescore(sage_ctx* c, const void* G_batch, int64_t rows) {
    ALIVE(c);
    if (rows < 0 || (rows > 0 && !G_batch)) return SAGE_ERR_ARG;
    return rescore_impl(c, dense_src(G_batch, c->dtype), rows);
}

int sage_rescore_outer(sage_ctx* c, const void* E, const void* H, int64_t rows, int64_t n_classes, int64_t n_features) {
    ALIVE(c);
    if (rows < 0) return SAGE_ERR_ARG;
    if (rows == 0) return rescore_impl(c, RowSrc{}, 0);
    RowSrc s;
    if (!outer_src(c, E, H, n_classes, n_features, s)) return SAGE_ERR_ARG;
    return rescore_impl(c, s, rows);
}

int sage_select(sage_ctx* c, double keep_rate, int64_t* out_idx, int64_t cap, int64_t* out_m) {
    ALIVE(c);
    if (!out_m || cap < 0 || !(keep_rate >= 0.0 && keep_rate <= 1.0)) return SAGE_ERR_ARG;
    if (!c->has_basis) return SAGE_ERR_STATE;
    const int64_t N = c->n_scored;
    const int64_t m = keep_count(keep_rate, N);
    *out_m = m;
    if (m > cap) return SAGE_ERR_CAPACITY;
    if (m > 0 && !out_idx) return SAGE_ERR_ARG;
    if (!c->store_zhat && c->n_rescored != N) return SAGE_ERR_STATE;  // the rescoring pass is not complete
    {
        int rc = ensure_alpha(c, N);
        if (rc != SAGE_OK) return rc;
    }
    if (c->store_zhat) RUN(K_SELECT, launch_cosine(c->zhat, N, c->k, c->ssum, c->alpha, c->st));
    c->alpha_n = N;
    RUN(K_SELECT, launch_topm(c->alpha, N, m, out_idx, c->sw, c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    return SAGE_OK;
}

int sage_select_cb(sage_ctx* c, double keep_rate, int n_classes, int64_t* out_idx, int64_t cap, int64_t* out_m) {
    return sage_select_cb_ex(c, keep_rate, n_classes, SAGE_CB_PROPORTIONAL, out_idx, cap, out_m);
}

int sage_select_cb_ex(sage_ctx* c, double keep_rate, int n_classes, int rule, int64_t* out_idx, int64_t cap,
                      int64_t* out_m) {
    ALIVE(c);
    if (!out_m || cap < 0 || !(keep_rate >= 0.0 && keep_rate <= 1.0) || n_classes < 1 || n_classes > 65536 ||
        (rule != SAGE_CB_PROPORTIONAL && rule != SAGE_CB_EQUAL))
        return SAGE_ERR_ARG;
    if (!c->has_basis) return SAGE_ERR_STATE;
    const int64_t N = c->n_scored;
    if (!c->store_zhat || c->n_labeled != N) return SAGE_ERR_STATE;  // needs zhat, and a label for every row of the pass
    *out_m = 0;
    {
        int rc = ensure_alpha(c, N);
        if (rc != SAGE_OK) return rc;
    }
    const size_t need = cb_work_bytes(n_classes, N);
    if (need > c->cb_work_bytes) {
        if (c->cb_work) {
            HIPCHK(hipStreamSynchronize(c->st));
            (void)hipFree(c->cb_work);
            c->cb_work = nullptr;
            c->cb_work_bytes = 0;
        }
        ALLOC(c->cb_work, need);
        c->cb_work_bytes = need;
    }
    const CbWork w = cb_work_layout(c->cb_work, n_classes, N);
    RUN(K_SELECT, launch_cb_scores(c->zhat, c->labels, N, c->k, n_classes, keep_rate, rule, c->alpha, w, c->st));
    c->alpha_n = N;
    uint32_t misc[2] = {0, 0};
    HIPCHK(hipMemcpyAsync(misc, w.misc, sizeof(misc), hipMemcpyDeviceToHost, c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    if (misc[1]) return SAGE_ERR_ARG;  // a label outside [0, n_classes)
    const int64_t m = (int64_t)misc[0];
    *out_m = m;
    if (m > cap) return SAGE_ERR_CAPACITY;
    if (m > 0 && !out_idx) return SAGE_ERR_ARG;
    if (m > 0) RUN(K_SELECT, launch_cb_select(c->alpha, c->labels, N, n_classes, out_idx, w, c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    return SAGE_OK;
}

int sage_topm(const float* alpha, int64_t N, int64_t m, int64_t* out_idx, void* hip_stream) {
    if (N < 0 || m < 0 || m > N || (N > 0 && !alpha) || (m > 0 && !out_idx)) return SAGE_ERR_ARG;
    if (m == 0) return SAGE_OK;
    SelectWork w{};
    int rc = alloc_select_work(w, N);
    if (rc != SAGE_OK) {
        free_select_work(w);
        return rc;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e = launch_topm(alpha, N, m, out_idx, w, st);
    hipError_t e2 = hipStreamSynchronize(st);
    free_select_work(w);
    return (e == hipSuccess && e2 == hipSuccess) ? SAGE_OK : SAGE_ERR_HIP;
}

int sage_fd_sketch_export(sage_ctx* c, float* B_out) {
    ALIVE(c);
    if (!B_out) return SAGE_ERR_ARG;
    int rcf = flush_pending(c);
    if (rcf != SAGE_OK) return rcf;
    const int ell = c->d.ell;
    HIPCHK(launch_export_rows(c->top, c->d.LP, ell, B_out, c->d, c->st));
    HIPCHK(launch_export_rows(c->nw[c->cur], c->d.LP, c->fill_new, B_out + (size_t)ell * c->d.D, c->d, c->st));
    if (c->fill_new < ell)
        HIPCHK(hipMemsetAsync(B_out + (size_t)(ell + c->fill_new) * c->d.D, 0,
                              (size_t)(ell - c->fill_new) * c->d.D * sizeof(float), c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    return SAGE_OK;
}

int sage_basis_export(sage_ctx* c, float* Vt_out) {
    ALIVE(c);
    if (!Vt_out) return SAGE_ERR_ARG;
    if (!c->has_basis) return SAGE_ERR_STATE;
    HIPCHK(launch_export_rows(c->Vblk, c->KP, c->k, Vt_out, c->d, c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    return SAGE_OK;
}

int sage_scores(sage_ctx* c, const float** alpha, int64_t* n) {
    ALIVE(c);
    if (!alpha || !n) return SAGE_ERR_ARG;
    if (!c->has_basis || c->alpha_n != c->n_scored) return SAGE_ERR_STATE;
    *alpha = c->alpha;
    *n = c->alpha_n;
    return SAGE_OK;
}

int sage_scores_export(sage_ctx* c, float* alpha_out) {
    ALIVE(c);
    if ((!alpha_out && c->n_scored > 0)) return SAGE_ERR_ARG;
    if (!c->has_basis || c->alpha_n != c->n_scored) return SAGE_ERR_STATE;
    if (c->alpha_n > 0)
        HIPCHK(hipMemcpyAsync(alpha_out, c->alpha, (size_t)c->alpha_n * sizeof(float), hipMemcpyDeviceToDevice, c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    return SAGE_OK;
}

int sage_zhat_export(sage_ctx* c, float* zhat_out) {
    ALIVE(c);
    if ((!zhat_out && c->n_scored > 0)) return SAGE_ERR_ARG;
    if (!c->has_basis || !c->store_zhat) return SAGE_ERR_STATE;
    if (c->n_scored > 0)
        HIPCHK(hipMemcpyAsync(zhat_out, c->zhat, (size_t)c->n_scored * c->k * sizeof(float), hipMemcpyDeviceToDevice,
                              c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    return SAGE_OK;
}

int sage_stats(sage_ctx* c, sage_stats_t* out) {
    ALIVE(c);
    if (!out) return SAGE_ERR_ARG;
    int rcf = flush_pending(c);
    if (rcf != SAGE_OK) return rcf;
    double acc[8];
    HIPCHK(hipMemcpyAsync(acc, c->acc, sizeof(acc), hipMemcpyDeviceToHost, c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    double pending = 0.0;
    if (c->cnt_top < c->fill_top || c->cnt_new < c->fill_new) {
        // rows inserted since the last decomposition: add their squared norms from a Gram of the buffer
        hipError_t e = launch_gram(c->top, c->nw[c->cur], c->fill_new, c->gram_partial, c->gp, c->d, c->st);
        if (e == hipSuccess)
            e = launch_gram_reduce(c->gram_partial, c->gp, nullptr, nullptr, c->ew.C, false, c->ew.known, c->d, c->st);
        if (e != hipSuccess) return hip_failed(c);
        const int NP = c->d.NP, LP = c->d.LP;
        double* diag = (double*)malloc(sizeof(double) * NP);
        if (!diag) return SAGE_ERR_ALLOC;
        e = hipMemcpy2DAsync(diag, sizeof(double), c->ew.C, (size_t)(NP + 1) * sizeof(double), sizeof(double), NP,
                             hipMemcpyDeviceToHost, c->st);
        if (e == hipSuccess) e = hipStreamSynchronize(c->st);
        if (e != hipSuccess) {
            free(diag);
            return hip_failed(c);
        }
        for (int r = c->cnt_top; r < c->fill_top; ++r) pending += diag[r];
        for (int r = c->cnt_new; r < c->fill_new; ++r) pending += diag[LP + r];
        free(diag);
    }
    out->rows_seen = c->rows_seen;
    out->n_shrinks = c->n_shrinks;
    out->n_scored = c->n_scored;
    out->sum_delta = acc[0];
    out->frob2 = acc[1] + pending;
    out->last_delta = acc[2];
    out->last_sweeps = (int)acc[3];
    out->n_unconverged = (int64_t)acc[4];
    out->last_offdiag = acc[5];
    out->fill = c->fill_top + c->fill_new;
    return SAGE_OK;
}

int sage_probe_gram_eig(sage_ctx* c, double* C_out, int eig, double* Y_out, double* lam_out, int* n_pad) {
    ALIVE(c);
    const int NP = c->d.NP, LP = c->d.LP, ell = c->d.ell;
    if (n_pad) *n_pad = NP;
    if (!C_out && !eig) return SAGE_OK;
    int rcf = flush_pending(c);
    if (rcf != SAGE_OK) return rcf;
    HIPCHK(launch_gram(c->top, c->nw[c->cur], c->fill_new, c->gram_partial, c->gp, c->d, c->st));
    HIPCHK(launch_gram_reduce(c->gram_partial, c->gp, nullptr, nullptr, c->ew.C, false, c->ew.known, c->d, c->st));
    // Inside the library matrix index LP + j stands for buffer row ell + j; the probe reports buffer-row order
    // (rows 0 .. 2*ell-1, padding last).
    if (C_out) HIPCHK(launch_probe_permute(c->ew.C, C_out, NP, LP, ell, true, c->st));
    if (eig) {
        HIPCHK(launch_eig(c->ew, NP, JACOBI_TOL_BASIS, MAX_SWEEPS, c->st));
        if (Y_out) HIPCHK(launch_probe_permute(c->ew.Y, Y_out, NP, LP, ell, false, c->st));
        if (lam_out)
            HIPCHK(hipMemcpy2DAsync(lam_out, sizeof(double), c->ew.C, (size_t)(NP + 1) * sizeof(double), sizeof(double),
                                    NP, hipMemcpyDeviceToDevice, c->st));
    }
    HIPCHK(hipStreamSynchronize(c->st));
    return SAGE_OK;
}

int sage_probe_gram_split(sage_ctx* c, double* C_out, int* n_pad) {
    ALIVE(c);
    const int NP = c->d.NP, LP = c->d.LP, ell = c->d.ell;
    if (n_pad) *n_pad = NP;
    if (c->gp_cross_split.tiles <= 0 || c->gp_new2_split.tiles <= 0) return SAGE_ERR_STATE;
    if (!C_out) return SAGE_OK;
    int rcf = flush_pending(c);
    if (rcf != SAGE_OK) return rcf;
    if (c->new_block_ready || c->pre_stored) return SAGE_ERR_STATE;  // (never after flush_pending)
    const bool one = c->fill_new > 0 && new_one(c, c->cur);
    HIPCHK(launch_gram(c->top, c->nw[c->cur], c->fill_new, c->gram_partial, c->gp_cross_split, c->d, c->st, one));
    HIPCHK(launch_gram(c->top, c->nw[c->cur], c->fill_new, c->gram_partial_new[c->cur], c->gp_new2_split, c->d, c->st, one));
    HIPCHK(launch_gram_reduce(c->gram_partial, c->gp_cross_split, c->gram_partial_new[c->cur], &c->gp_new2_split, c->ew.C,
                              false, c->ew.known, c->d, c->st));
    HIPCHK(launch_probe_permute(c->ew.C, C_out, NP, LP, ell, true, c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    return SAGE_OK;
}

int sage_probe_eig_matrix(sage_ctx* c, const double* C_in, double* Y_out, double* lam_out, double* sweep_stat_out) {
    ALIVE(c);
    if (!C_in) return SAGE_ERR_ARG;
    const int NP = c->d.NP;
    HIPCHK(hipMemcpyAsync(c->ew.C, C_in, (size_t)NP * NP * sizeof(double), hipMemcpyDeviceToDevice, c->st));
    HIPCHK(launch_eig(c->ew, NP, JACOBI_TOL_BASIS, MAX_SWEEPS, c->st));
    if (Y_out) HIPCHK(hipMemcpyAsync(Y_out, c->ew.Y, (size_t)NP * NP * sizeof(double), hipMemcpyDeviceToDevice, c->st));
    if (lam_out)
        HIPCHK(hipMemcpy2DAsync(lam_out, sizeof(double), c->ew.C, (size_t)(NP + 1) * sizeof(double), sizeof(double), NP,
                                hipMemcpyDeviceToDevice, c->st));
    if (sweep_stat_out)
        HIPCHK(hipMemcpyAsync(sweep_stat_out, c->ew.stat, 18 * sizeof(double), hipMemcpyDeviceToDevice, c->st));
    HIPCHK(hipStreamSynchronize(c->st));
    return SAGE_OK;
}

int sage_set_sweep_policy(sage_ctx* c, int policy) {
    ALIVE(c);
    if (policy != SAGE_SWEEPS_ADAPTIVE && policy != SAGE_SWEEPS_ALL) return SAGE_ERR_ARG;
    c->sweeps_all = policy == SAGE_SWEEPS_ALL;
    return SAGE_OK;
}

int sage_set_debug_checks(sage_ctx* c, int on) {
    ALIVE(c);
    c->debug_checks = on != 0;
    return SAGE_OK;
}

int sage_debug_fail_launch(sage_ctx* c, int nth) {
    ALIVE(c);
    if (nth < 0) return SAGE_ERR_ARG;
    c->fail_in = nth;
    return SAGE_OK;
}

int sage_copy_probe(void* dst, const void* src, int64_t bytes, void* hip_stream) {
    if (!dst || !src || bytes < 0 || bytes % 16 != 0 || ((uintptr_t)dst | (uintptr_t)src) % 16 != 0) return SAGE_ERR_ARG;
    if (launch_plain_copy(src, dst, bytes, (hipStream_t)hip_stream) != hipSuccess) return SAGE_ERR_HIP;
    return SAGE_OK;
}

int sage_profile_enable(sage_ctx* c, int on) {
    ALIVE(c);
    c->prof = on != 0;
    return SAGE_OK;
}

int sage_profile_read(sage_ctx* c, int which, double* ms, int64_t* launches) {
    ALIVE(c);
    if (which < 0 || which >= NCLASS || !ms || !launches) return SAGE_ERR_ARG;
    HIPCHK(hipStreamSynchronize(c->st));
    *ms = c->prof_ms[which];
    *launches = c->prof_n[which];
    c->prof_ms[which] = 0.0;
    c->prof_n[which] = 0;
    return SAGE_OK;
}

}  // extern "C"
