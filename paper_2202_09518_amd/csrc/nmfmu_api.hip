// C ABI of libnmfmu: argument checking, workspace management and the host-side
// schedules (resident loop, out-of-memory batch pipeline, CSR loop, ensemble).
// Public contract: include/nmfmu.h; the hooks of the tests: include/nmfmu_test.h.
#include "nmfmu.h"
#include "nmfmu_test.h"
#include "nmfmu_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

using namespace nmfmu;

namespace {

thread_local char t_err[256] = "";

int fail(int status, const char *fmt, const char *detail = "")
{
    snprintf(t_err, sizeof(t_err), fmt, detail);
    return status;
}

#define NMF_HIP(call)                                                         \
    do {                                                                      \
        hipError_t e_ = (call);                                               \
        if (e_ != hipSuccess) return fail(NMF_EHIP, #call ": %s", hipGetErrorString(e_)); \
    } while (0)

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// ---- process-wide device memory owned by the library ----------------------

struct State {
    std::mutex mu;
    void *ws = nullptr;         // workspace in use (owned or caller's)
    size_t ws_bytes = 0;
    bool ws_owned = true;
    void *stage = nullptr;      // staging slots of the out-of-memory path
    size_t stage_bytes = 0;
    hipStream_t copy_stream = nullptr;
    hipEvent_t ev_copied[3] = {nullptr, nullptr, nullptr};
    hipEvent_t ev_freed[3] = {nullptr, nullptr, nullptr};
    hipEvent_t ev_entry = nullptr;
    // rank-sliced out-of-memory path: up to kMaxSlots staging slots, factor rows copied back
    void *sl_stage = nullptr;
    size_t sl_stage_bytes = 0;
    hipStream_t back_stream = nullptr;
    hipEvent_t sl_copied[16] = {}, sl_done[16] = {}, sl_freed[16] = {};
};
State g;

// Workspace carving.  Slot 0 holds the arrival counters of the Gram kernels and
// must be zero whenever no kernel is running; the kernels restore that.
struct Carve {
    char *base;
    size_t off = 0;
    explicit Carve(void *b) : base(static_cast<char *>(b)) {}
    template <class T> T *take(size_t count)
    {
        T *p = reinterpret_cast<T *>(base + off);
        off = align_up(off + count * sizeof(T));
        return p;
    }
};

struct Common {
    unsigned *counters;
    float *gw, *gh, *gpart;
    float *gwp, *ghp;   // partial Gram tiles handed from one finisher to the next
    float *gws, *ghs;   // the same, added up in groups by the pass that runs in between
};

Common carve_common(Carve &c, int k)
{
    Common r;
    r.counters = c.take<unsigned>(64);
    r.gw = c.take<float>((size_t)k * k);
    r.gh = c.take<float>((size_t)k * k);
    const int kt = k_tiles(k);
    r.gpart = c.take<float>((size_t)kGramMaxBlocks * kt * kt * 1024);
    r.gwp = c.take<float>((size_t)kFinMaxBlocks * kt * kt * 1024);
    r.ghp = c.take<float>((size_t)kFinMaxBlocks * kt * kt * 1024);
    r.gws = c.take<float>((size_t)(kFinMaxBlocks / kGramGroup) * kt * kt * 1024);
    r.ghs = c.take<float>((size_t)(kFinMaxBlocks / kGramGroup) * kt * kt * 1024);
    return r;
}

size_t common_bytes(int k)
{
    Carve c(nullptr);
    carve_common(c, k);
    return c.off;
}

int ensure_workspace(size_t need, void **out)
{
    if (g.ws && g.ws_bytes >= need) {
        *out = g.ws;
        return NMF_OK;
    }
    if (!g.ws_owned) return fail(NMF_ENOMEM, "caller-provided workspace is too small%s");
    if (g.ws) {
        NMF_HIP(hipDeviceSynchronize());
        NMF_HIP(hipFree(g.ws));
        g.ws = nullptr;
        g.ws_bytes = 0;
    }
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, need);
    if (e != hipSuccess) return fail(NMF_ENOMEM, "hipMalloc(workspace): %s", hipGetErrorString(e));
    NMF_HIP(hipMemset(p, 0, kAlign));
    g.ws = p;
    g.ws_bytes = need;
    *out = p;
    return NMF_OK;
}

int check_common(const void *a, const void *w, const void *h, int64_t m, int64_t n, int32_t k,
                 int32_t iters, float eps, int32_t kmax = NMF_MU_MAX_K)
{
    if (!a || !w || !h) return fail(NMF_EINVAL, "null pointer%s");
    if (m < 1 || n < 1 || k < 1) return fail(NMF_EINVAL, "m, n, k must be >= 1%s");
    if (k > kmax) return fail(NMF_EUNSUPPORTED, "k exceeds the rank this entry point supports%s");
    if (iters < 0) return fail(NMF_EINVAL, "iters must be >= 0%s");
    if (!(eps >= 0.f) || !std::isfinite(eps)) return fail(NMF_EINVAL, "eps must be finite and >= 0%s");
    if (m > (int64_t)1 << 40 || n > (int64_t)1 << 31) return fail(NMF_EINVAL, "matrix too large%s");
    return NMF_OK;
}

// Plan of one resident dense run.  The fast plan ("mirrored") keeps A^T, W^T
// and H^T next to A, W, H, so that the A H^T product becomes the same
// row-streaming contraction as W^T A (on A^T with H^T: the two updates are
// transposes of each other) and its update the same finisher on W^T.  It costs
// one extra copy of A in the workspace; without it the direct A H^T kernel runs.
struct DensePlan {
    bool mirrored;
    Common c;
    float *ppart;              // row-split partials of either pass
    void *planes;              // bf16 piece planes of the factor a pass contracts with
    void *planes2;             // row plan: piece planes of H^T (planes then holds those of W)
    float *At, *Wt, *Ht;       // mirrored only
    int s1, s2;                // row splits of the pass over A / over A^T
    int64_t rps1, rps2;
};

size_t dense_bytes(int64_t m, int64_t n, int k, bool mirrored)
{
    const size_t p1 = (size_t)wta_splits_bound(m, n, k) * k * n, p2 = (size_t)wta_splits_bound(n, m, k) * k * m;
    size_t b = common_bytes(k) + align_up(((mirrored && p2 > p1) ? p2 : p1) * sizeof(float)) +
               align_up(planes_bytes((mirrored && n > m) ? n : m)) + align_up(planes_bytes(n));
    if (mirrored)
        b += align_up((size_t)m * n * sizeof(float)) + align_up((size_t)k * m * sizeof(float)) +
             align_up((size_t)n * k * sizeof(float));
    return b;
}

DensePlan carve_dense(void *ws, int64_t m, int64_t n, int k, bool mirrored)
{
    Carve cv(ws);
    DensePlan p;
    p.mirrored = mirrored;
    p.c = carve_common(cv, k);
    p.s1 = wta_splits(m, n, k);
    p.rps1 = wta_rows_per_split(m, p.s1);
    p.s2 = wta_splits(n, m, k);
    p.rps2 = wta_rows_per_split(n, p.s2);
    const size_t p1 = (size_t)wta_splits_bound(m, n, k) * k * n, p2 = (size_t)wta_splits_bound(n, m, k) * k * m;
    p.ppart = cv.take<float>((mirrored && p2 > p1) ? p2 : p1);
    p.planes = cv.take<char>(planes_bytes((mirrored && n > m) ? n : m));
    p.planes2 = cv.take<char>(planes_bytes(n));
    p.At = p.Wt = p.Ht = nullptr;
    if (mirrored) {
        p.At = cv.take<float>((size_t)m * n);
        p.Wt = cv.take<float>((size_t)k * m);
        p.Ht = cv.take<float>((size_t)n * k);
    }
    return p;
}

// Which plan runs.  Up to 32 factors the row plan comes first wherever its kernel applies.  From 33
// to 64 factors its A H^T pass is slower than the W^T A kernel on a transposed copy (622 against
// 525 us on 32768 x 16384, 167 against 132 us on 16384 x 8192), so there the mirrored plan comes
// first and the row plan serves when the workspace cannot hold the copy.
static bool rows_plan_first(const float *A, int64_t m, int64_t n, int k) { return k <= 32 && aht_rows_ok(A, m, n, k); }
static bool rows_plan_runs(const float *A, int64_t m, int64_t n, int k, bool mirrored)
{
    // without a transposed copy the row kernel beats the direct one on every shape it can take
    return aht_rows_can(A, n, k) && (!mirrored || rows_plan_first(A, m, n, k));
}

// Workspace for a dense run: the mirrored plan if it can be had, else the small one.
int dense_workspace(const float *A, int64_t m, int64_t n, int k, void **ws, bool *mirrored)
{
    const size_t big = dense_bytes(m, n, k, true), small = dense_bytes(m, n, k, false);
    if (rows_plan_first(A, m, n, k)) {     // the row plan streams A itself for both products
        *mirrored = false;
        return ensure_workspace(small, ws);
    }
    if (g.ws && g.ws_bytes >= big) {
        *ws = g.ws;
        *mirrored = true;
        return NMF_OK;
    }
    if (g.ws_owned && ensure_workspace(big, ws) == NMF_OK) {
        *mirrored = true;
        return NMF_OK;
    }
    (void)hipGetLastError();
    *mirrored = false;
    return ensure_workspace(small, ws);
}

constexpr int kDenseKernels = 6;

// Per-iteration objective of a dense run (device memory): out[it] after iteration it.
struct Monitor {
    double *dpart;      // kFinMaxBlocks: <numerator, new W> per finisher block
    double *normA2;     // [0] = ||A||_F^2, followed by 4096 doubles of scratch for its sum
    double *out;        // iters values
    double *res;        // direct plan: scratch of the tiled evaluation (ceil(m / 32) + 1 doubles)
    bool last_only;     // only the last iteration of the call reports (into out[0])
};

// One resident dense run on `st`.  With `ev` (kDenseKernels * iters + 1 events)
// an event is recorded before the first kernel of the loop and after every
// kernel, for per-kernel timing; slots of kernels a plan does not use collapse
// to zero duration.  `a_is_mirrored`: At already holds this A's transpose.
int dense_body(const float *A, int64_t m, int64_t n, int k, float *W, float *H, int iters,
               float eps, const DensePlan &p, hipStream_t st, bool a_is_mirrored = false,
               hipEvent_t *ev = nullptr, const BlockMap *map = nullptr, const Monitor *mon = nullptr)
{
    const Common &c = p.c;
    // The plan may have been carved for a larger rank (stacks of an ensemble): split
    // counts follow the rank actually run; the partial buffer holds the largest case.
    const int s1 = wta_splits(m, n, k), s2 = wta_splits(n, m, k);
    const int64_t rps1 = wta_rows_per_split(m, s1), rps2 = wta_rows_per_split(n, s2);
    if (rows_plan_runs(A, m, n, k, p.mirrored)) {
        // Row plan: both products stream the row-major A.  The W^T A pass reads the piece
        // planes of W and, on the side, adds the tile sets of W^T W up in groups; the H update writes
        // the planes of H^T and the tile sets of H H^T, which a small launch adds up; the A H^T pass
        // with the fused W update writes the planes of the new W and the tile sets of its W^T W.
        const int nbw = aht_rows_blocks(m, k), nbh = factor_update_blocks(n);
        const int ngw = gram_groups(nbw);
        // planes and W^T W of the W handed in, with the summation order of an updating launch
        NMF_HIP(launch_aht_rows(nullptr, m, n, k, nullptr, nullptr, W, p.planes, c.gwp, eps, st, true));
        if (ev) NMF_HIP(hipEventRecord(*ev++, st));
        for (int it = 0; it < iters; ++it) {
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            NMF_HIP(launch_wta_pass(A, m, n, k, W, p.planes, true, p.ppart, s1, rps1, false, st, c.gwp, nbw, c.gws));
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            NMF_HIP(launch_factor_update(H, nullptr, p.ppart, s1, nullptr, c.gws, ngw, c.ghp, k, n, eps, st, map, p.planes2));
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            NMF_HIP(launch_gram_sum(c.ghp, nbh, k, c.gh, st));
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            const bool report = mon && (!mon->last_only || it == iters - 1);
            NMF_HIP(launch_aht_rows(A, m, n, k, p.planes2, c.gh, W, p.planes, c.gwp, eps, st, false, map,
                                    report ? mon->dpart : nullptr));
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            if (report) {
                NMF_HIP(launch_gram_sum(c.gwp, nbw, k, c.gw, st));
                NMF_HIP(launch_objective(mon->dpart, nbw, c.gw, c.gh, k, mon->normA2,
                                         mon->out + (mon->last_only ? 0 : it), st));
            }
        }
        return NMF_OK;
    }
    if (p.mirrored) {
        if (!a_is_mirrored) NMF_HIP(launch_transpose(A, m, n, p.At, st));
        NMF_HIP(launch_transpose(W, m, k, p.Wt, st));
        NMF_HIP(launch_transpose(H, k, n, p.Ht, st));
    }
    if (p.mirrored) {
        // W^T W of the initial W as partial tiles, from the finisher in its Gram-only
        // mode (same bits as the tiles a preceding W update would have left, so that
        // a run split into two calls equals one call); afterwards every finisher
        // hands the Gram tiles of its new factor to the next one.
        NMF_HIP(launch_factor_update(p.Wt, nullptr, nullptr, 0, nullptr, nullptr, 0, c.gwp, k, m, eps, st, nullptr, p.planes));
        const int nbw = factor_update_blocks(m), nbh = factor_update_blocks(n);
        if (ev) NMF_HIP(hipEventRecord(*ev++, st));
        // The tiles of a finisher are needed, summed, by the next finisher; the pass that runs
        // in between adds them up in groups of kGramGroup on the side (its first workgroups),
        // the finisher sums the few group sets while it stages G: no launch of its own.
        const int ngw = gram_groups(nbw), ngh = gram_groups(nbh);
        for (int it = 0; it < iters; ++it) {
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            NMF_HIP(launch_wta_pass(A, m, n, k, W, p.planes, true, p.ppart, s1, rps1, false, st, c.gwp, nbw, c.gws));
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            NMF_HIP(launch_factor_update(H, p.Ht, p.ppart, s1, nullptr, c.gws, ngw, c.ghp, k, n, eps, st, map, p.planes));
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            NMF_HIP(launch_wta_pass(p.At, n, m, k, p.Ht, p.planes, true, p.ppart, s2, rps2, false, st, c.ghp, nbh, c.ghs));
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            const bool report = mon && (!mon->last_only || it == iters - 1);
            NMF_HIP(launch_factor_update(p.Wt, W, p.ppart, s2, nullptr, c.ghs, ngh, c.gwp, k, m, eps, st, map, p.planes,
                                         report ? mon->dpart : nullptr));
            if (ev) NMF_HIP(hipEventRecord(*ev++, st));
            if (report) {
                // ||A - W H||_F from what this W update leaves behind: <A H^T, W>, H H^T, W^T W
                NMF_HIP(launch_gram_sum(c.gwp, nbw, k, c.gw, st));
                NMF_HIP(launch_gram_sum(c.ghs, ngh, k, c.gh, st));
                NMF_HIP(launch_objective(mon->dpart, nbw, c.gw, c.gh, k, mon->normA2,
                                         mon->out + (mon->last_only ? 0 : it), st));
            }
        }
        return NMF_OK;
    }
    if (ev) NMF_HIP(hipEventRecord(*ev++, st));
    for (int it = 0; it < iters; ++it) {
        NMF_HIP(launch_gram_w(W, m, k, c.gw, c.gpart, c.counters, st));
        NMF_HIP(launch_split_planes(W, m, k, p.planes, st));
        if (ev) NMF_HIP(hipEventRecord(*ev++, st));
        NMF_HIP(launch_wta_pass(A, m, n, k, W, p.planes, true, p.ppart, s1, rps1, false, st));
        if (ev) NMF_HIP(hipEventRecord(*ev++, st));
        NMF_HIP(launch_factor_update(H, nullptr, p.ppart, s1, c.gw, nullptr, 0, nullptr, k, n, eps, st));
        if (ev) NMF_HIP(hipEventRecord(*ev++, st));
        NMF_HIP(launch_gram_h(H, k, n, c.gh, c.gpart, c.counters, st));
        if (ev) NMF_HIP(hipEventRecord(*ev++, st));
        NMF_HIP(launch_aht_pass(A, m, n, k, H, c.gh, W, eps, st));
        if (ev) NMF_HIP(hipEventRecord(*ev++, st));
        if (ev) NMF_HIP(hipEventRecord(*ev++, st));
        if (mon && (!mon->last_only || it == iters - 1))   // exact, tiled
            NMF_HIP(launch_residual(A, m, n, k, W, H, mon->res + 1, mon->out + (mon->last_only ? 0 : it), st));
    }
    return NMF_OK;
}

size_t csr_bytes(int64_t n, int64_t nnz, int k)
{
    return common_bytes(k) + align_up((size_t)n * k * sizeof(float)) +      // Ht
           align_up((size_t)(n + 1) * sizeof(int64_t)) +                      // column pointers
           align_up((size_t)nnz * sizeof(int32_t)) + align_up((size_t)nnz * sizeof(float)) +
           2 * align_up((size_t)(kCsrParts + 1) * sizeof(int64_t)) +          // row ranges, CSR and CSC
           2 * align_up((size_t)(nnz / kLongRow + 2) * sizeof(int32_t)) +     // long-row lists
           kAlign +                                                           // their counts
           // scratch of the one-time sort that builds the column-ordered copy
           align_up((size_t)nnz * sizeof(int32_t)) + 2 * align_up((size_t)nnz * sizeof(uint64_t)) +
           align_up(nnz ? csc_sort_temp_bytes(nnz, n) : 0);
}

// Column-ordered copy of a CSR matrix into caller-provided arrays (test hook); the sort
// scratch is transient (allocated and freed here, which synchronises with `st`).
int build_csc(const int64_t *rowptr, const int32_t *colidx, const float *vals, int64_t m,
              int64_t n, int64_t nnz, int64_t *colptr, int32_t *rowidx, float *cvals, hipStream_t st)
{
    const size_t idx_bytes = align_up((size_t)nnz * sizeof(int32_t));
    const size_t pl_bytes = align_up((size_t)nnz * sizeof(uint64_t));
    const size_t temp_bytes = nnz ? csc_sort_temp_bytes(nnz, n) : 0;
    void *scratch = nullptr;
    if (nnz) {
        hipError_t e = hipMalloc(&scratch, idx_bytes + 2 * pl_bytes + align_up(temp_bytes) + kAlign);
        if (e != hipSuccess) return fail(NMF_ENOMEM, "hipMalloc(sort scratch): %s", hipGetErrorString(e));
    }
    char *sp = static_cast<char *>(scratch);
    hipError_t e = launch_csc_build(rowptr, colidx, vals, m, n, nnz,
                                    reinterpret_cast<int32_t *>(sp + 2 * pl_bytes),
                                    reinterpret_cast<uint64_t *>(sp),
                                    reinterpret_cast<uint64_t *>(sp + pl_bytes),
                                    sp + 2 * pl_bytes + idx_bytes, temp_bytes, colptr, rowidx, cvals, st);
    hipError_t e2 = scratch ? hipStreamSynchronize(st) : hipSuccess;
    if (scratch) (void)hipFree(scratch);
    if (e != hipSuccess) return fail(NMF_EHIP, "csc build: %s", hipGetErrorString(e));
    if (e2 != hipSuccess) return fail(NMF_EHIP, "csc build: %s", hipGetErrorString(e2));
    return NMF_OK;
}

// ---- rank-sliced engine (ranks above NMF_MU_MAX_K, and the host-resident-W pipeline) ----
// Every product of the iteration is written as F^T X with F (rows x k) and X (rows x cols)
// row-major, i.e. a reduction over the rows of both, and computed 64 factor columns at a
// time by the k <= 64 pass kernel on the piece planes of that slice of F:
//   W^T A, W^T W                      F = W,  X = A or W
//   (W^T W) H                         F = W^T W (symmetric), X = H
//   A H^T, H H^T, W (H H^T)           the same three on the transposes A^T, H^T, W^T
// followed by the element-wise update.  X is read once per slice.
struct Sliced {
    void *planes;     // planes_bytes(max rows of any F)
    float *ppart;     // row-split partials of one slice: splits x 64 x max cols
    size_t planes_cap, ppart_elems;
};

int sliced_ftx(const Sliced &e, const float *F, int64_t rows, int k, const float *X, int64_t cols,
               float *out, bool accumulate, hipStream_t st)
{
    // factor columns per pass: the widest the pass kernels take from planes alone for this X
    // (the slices of F are not contiguous, so the kernel that reads the factor itself is out)
    const int kSlice = wta_planes_only_width(X, cols);
    const int splits = wta_splits(rows, cols, kSlice);
    const int64_t rps = wta_rows_per_split(rows, splits);
    const int nslices = (k + 63) / 64;
    if (kSlice == 64 && k > 64) {
        // all slices in one launch each: the slices of a tile of X run side by side and share its bytes
        if ((size_t)splits * 64 * (size_t)cols * nslices > e.ppart_elems || planes_bytes(rows) * nslices > e.planes_cap)
            return fail(NMF_EHIP, "internal: sliced scratch too small%s");
        NMF_HIP(launch_split_planes_slices(F, rows, k, e.planes, st));
        NMF_HIP(launch_wta_pass_slices(X, rows, cols, k, e.planes, e.ppart, splits, rps, st));
        NMF_HIP(launch_sum_partials_slices(e.ppart, splits, k, cols, out, st, accumulate));
        return NMF_OK;
    }
    if ((size_t)splits * kSlice * (size_t)cols > e.ppart_elems || planes_bytes(rows) > e.planes_cap)
        return fail(NMF_EHIP, "internal: sliced scratch too small%s");
    for (int c0 = 0; c0 < k; c0 += kSlice) {
        const int kc = (k - c0 < kSlice) ? k - c0 : kSlice;
        NMF_HIP(launch_split_planes_slice(F, rows, k, c0, kc, e.planes, st));
        NMF_HIP(launch_wta_pass(X, rows, cols, kc, nullptr, e.planes, true, e.ppart, splits, rps, false, st));
        NMF_HIP(launch_sum_partials(e.ppart, splits, (int64_t)kc * cols, out + (int64_t)c0 * cols, st, accumulate));
    }
    return NMF_OK;
}

// Upper bound on splits x 64 x cols over every X with at most `cols` columns: the split count is
// at most 32 and at most 512 / slabs + 1 with cols <= 256 slabs (64-factor slices; 32-factor
// slices have 128-column slabs and half the factors).
size_t sliced_ppart_elems(int64_t cols)
{
    const int64_t a = 32 * cols, b = 131072 + cols;
    return (size_t)64 * (size_t)(a < b ? a : b);
}

// Resident run of rank k > NMF_MU_MAX_K.
struct SlicedDense {
    Sliced e;
    float *At, *Wt, *Ht, *num, *den, *gw, *gh;
};

template <class T> T max3(T a, T b, T c) { return a > b ? (a > c ? a : c) : (b > c ? b : c); }

SlicedDense carve_sliced_dense(void *ws, int64_t m, int64_t n, int k, size_t *bytes)
{
    Carve cv(ws);
    SlicedDense p;
    cv.take<unsigned>(64);
    const int64_t big = m > n ? m : n;
    const size_t nslices = (size_t)(k + 63) / 64;
    p.e.planes_cap = planes_bytes(max3<int64_t>(m, n, k)) * nslices;
    p.e.ppart_elems = sliced_ppart_elems(max3<int64_t>(m, n, k)) * nslices;
    p.e.planes = cv.take<char>(p.e.planes_cap);
    // X is one of A (m x n), W (m x k), H (k x n) or a transpose of those
    p.e.ppart = cv.take<float>(p.e.ppart_elems);
    p.At = cv.take<float>((size_t)m * n);
    p.Wt = cv.take<float>((size_t)k * m);
    p.Ht = cv.take<float>((size_t)n * k);
    p.num = cv.take<float>((size_t)k * big);
    p.den = cv.take<float>((size_t)k * big);
    p.gw = cv.take<float>((size_t)k * k);
    p.gh = cv.take<float>((size_t)k * k);
    if (bytes) *bytes = cv.off;
    return p;
}

size_t sliced_dense_bytes(int64_t m, int64_t n, int k)
{
    size_t b = 0;
    carve_sliced_dense(nullptr, m, n, k, &b);
    return b;
}

int sliced_dense_body(const float *A, int64_t m, int64_t n, int k, float *W, float *H, int iters,
                      float eps, const SlicedDense &p, hipStream_t st)
{
    NMF_HIP(launch_transpose(A, m, n, p.At, st));
    NMF_HIP(launch_transpose(W, m, k, p.Wt, st));
    for (int it = 0; it < iters; ++it) {
        // H update (Algorithm 3 order): numerator W^T A, denominator (W^T W) H
        if (int rc = sliced_ftx(p.e, W, m, k, A, n, p.num, false, st)) return rc;
        if (int rc = sliced_ftx(p.e, W, m, k, W, k, p.gw, false, st)) return rc;
        if (int rc = sliced_ftx(p.e, p.gw, k, k, H, n, p.den, false, st)) return rc;
        NMF_HIP(launch_mu_apply(H, p.num, p.den, eps, (int64_t)k * n, st));
        NMF_HIP(launch_transpose(H, k, n, p.Ht, st));
        // W update with the new H, on the transposes: (A H^T)^T = H A^T, (W H H^T)^T = (H H^T) W^T
        if (int rc = sliced_ftx(p.e, p.Ht, n, k, p.At, m, p.num, false, st)) return rc;
        if (int rc = sliced_ftx(p.e, p.Ht, n, k, p.Ht, k, p.gh, false, st)) return rc;
        if (int rc = sliced_ftx(p.e, p.gh, k, k, p.Wt, m, p.den, false, st)) return rc;
        NMF_HIP(launch_mu_apply(p.Wt, p.num, p.den, eps, (int64_t)k * m, st));
        NMF_HIP(launch_transpose(p.Wt, k, m, W, st));
    }
    return NMF_OK;
}

// Out-of-memory run through the sliced engine, any supported rank; W either on the device
// (W_host == nullptr) or in host memory and streamed with the batches (Algorithm 5).
constexpr int kMaxSlots = 16;

struct SlicedOoc {
    Sliced e;
    float *Abt, *Wbt, *num_b, *den_b;   // per-batch transposes, numerator and denominator (k x rows)
    float *num, *den, *Ht, *gw, *gh;    // k x n, k x n, n x k, k x k, k x k
};

SlicedOoc carve_sliced_ooc(void *ws, int64_t rb, int64_t n, int k, size_t *bytes)
{
    Carve cv(ws);
    SlicedOoc p;
    cv.take<unsigned>(64);
    const size_t nslices = (size_t)(k + 63) / 64;
    p.e.planes_cap = planes_bytes(max3<int64_t>(rb, n, k)) * nslices;
    p.e.ppart_elems = sliced_ppart_elems(max3<int64_t>(rb, n, k)) * nslices;
    p.e.planes = cv.take<char>(p.e.planes_cap);
    p.e.ppart = cv.take<float>(p.e.ppart_elems);
    p.Abt = cv.take<float>((size_t)n * rb);
    p.Wbt = cv.take<float>((size_t)k * rb);
    p.num_b = cv.take<float>((size_t)k * rb);
    p.den_b = cv.take<float>((size_t)k * rb);
    p.num = cv.take<float>((size_t)k * n);
    p.den = cv.take<float>((size_t)k * n);
    p.Ht = cv.take<float>((size_t)n * k);
    p.gw = cv.take<float>((size_t)k * k);
    p.gh = cv.take<float>((size_t)k * k);
    if (bytes) *bytes = cv.off;
    return p;
}

size_t sliced_ooc_bytes(int64_t rb, int64_t n, int k)
{
    size_t b = 0;
    carve_sliced_ooc(nullptr, rb, n, k, &b);
    return b;
}

int sliced_ooc_run(const float *A_host, float *W_host, float *W_dev, int64_t m, int64_t n, int k,
                   float *H, int iters, float eps, int64_t batch_rows, int slots, hipStream_t st,
                   size_t *device_bytes)
{
    const bool hostw = W_host != nullptr;
    const size_t a_bytes = align_up((size_t)batch_rows * n * sizeof(float));
    const size_t w_bytes = hostw ? align_up((size_t)batch_rows * k * sizeof(float)) : 0;
    const size_t slot_bytes = a_bytes + w_bytes;
    void *ws = nullptr;
    const size_t ws_bytes = sliced_ooc_bytes(batch_rows, n, k);
    if (int rc = ensure_workspace(ws_bytes, &ws)) return rc;
    const SlicedOoc p = carve_sliced_ooc(ws, batch_rows, n, k, nullptr);
    if (g.sl_stage_bytes < slots * slot_bytes) {
        if (g.sl_stage) {
            NMF_HIP(hipDeviceSynchronize());
            NMF_HIP(hipFree(g.sl_stage));
            g.sl_stage = nullptr;
            g.sl_stage_bytes = 0;
        }
        hipError_t e = hipMalloc(&g.sl_stage, slots * slot_bytes);
        if (e != hipSuccess) return fail(NMF_ENOMEM, "hipMalloc(staging): %s", hipGetErrorString(e));
        g.sl_stage_bytes = slots * slot_bytes;
    }
    if (device_bytes) *device_bytes = ws_bytes + slots * slot_bytes;
    if (!g.copy_stream) NMF_HIP(hipStreamCreateWithFlags(&g.copy_stream, hipStreamNonBlocking));
    if (!g.ev_entry) NMF_HIP(hipEventCreateWithFlags(&g.ev_entry, hipEventDisableTiming));
    if (!g.back_stream) NMF_HIP(hipStreamCreateWithFlags(&g.back_stream, hipStreamNonBlocking));
    for (int i = 0; i < kMaxSlots; ++i) {
        if (!g.sl_copied[i]) NMF_HIP(hipEventCreateWithFlags(&g.sl_copied[i], hipEventDisableTiming));
        if (!g.sl_done[i]) NMF_HIP(hipEventCreateWithFlags(&g.sl_done[i], hipEventDisableTiming));
        if (!g.sl_freed[i]) NMF_HIP(hipEventCreateWithFlags(&g.sl_freed[i], hipEventDisableTiming));
    }
    // Staging slots may still be read by work enqueued earlier on `st`.
    NMF_HIP(hipEventRecord(g.ev_entry, st));
    NMF_HIP(hipStreamWaitEvent(g.copy_stream, g.ev_entry, 0));

    const int64_t nb = (m + batch_rows - 1) / batch_rows;
    int64_t issued = 0;
    for (int s = 0; s <= iters; ++s) {
        for (int64_t b = 0; b < nb; ++b, ++issued) {
            const int slot = (int)(issued % slots);
            const int64_t i0 = b * batch_rows;
            const int64_t rb = (i0 + batch_rows <= m) ? batch_rows : m - i0;
            char *base = static_cast<char *>(g.sl_stage) + slot * slot_bytes;
            float *Ab = reinterpret_cast<float *>(base);
            float *Wb = hostw ? reinterpret_cast<float *>(base + a_bytes) : W_dev + i0 * k;
            if (issued >= slots) NMF_HIP(hipStreamWaitEvent(g.copy_stream, g.sl_freed[slot], 0));
            NMF_HIP(hipMemcpyAsync(Ab, A_host + i0 * n, (size_t)rb * n * sizeof(float),
                                   hipMemcpyHostToDevice, g.copy_stream));
            if (hostw)
                NMF_HIP(hipMemcpyAsync(Wb, W_host + i0 * k, (size_t)rb * k * sizeof(float),
                                       hipMemcpyHostToDevice, g.copy_stream));
            NMF_HIP(hipEventRecord(g.sl_copied[slot], g.copy_stream));
            NMF_HIP(hipStreamWaitEvent(st, g.sl_copied[slot], 0));
            if (s > 0) {
                // W_b <- W_b * (A_b H^T) / (W_b H H^T + eps) on the transposes of the batch
                NMF_HIP(launch_transpose(Ab, rb, n, p.Abt, st));
                NMF_HIP(launch_transpose(Wb, rb, k, p.Wbt, st));
                if (int rc = sliced_ftx(p.e, p.Ht, n, k, p.Abt, rb, p.num_b, false, st)) return rc;
                if (int rc = sliced_ftx(p.e, p.gh, k, k, p.Wbt, rb, p.den_b, false, st)) return rc;
                NMF_HIP(launch_mu_apply(p.Wbt, p.num_b, p.den_b, eps, (int64_t)k * rb, st));
                NMF_HIP(launch_transpose(p.Wbt, k, rb, Wb, st));
            }
            if (s < iters) {
                // accumulate W_b^T A_b and W_b^T W_b with the W_b just updated
                if (int rc = sliced_ftx(p.e, Wb, rb, k, Ab, n, p.num, b > 0, st)) return rc;
                if (int rc = sliced_ftx(p.e, Wb, rb, k, Wb, k, p.gw, b > 0, st)) return rc;
            }
            if (hostw) {
                NMF_HIP(hipEventRecord(g.sl_done[slot], st));
                NMF_HIP(hipStreamWaitEvent(g.back_stream, g.sl_done[slot], 0));
                if (s > 0)
                    NMF_HIP(hipMemcpyAsync(W_host + i0 * k, Wb, (size_t)rb * k * sizeof(float),
                                           hipMemcpyDeviceToHost, g.back_stream));
                NMF_HIP(hipEventRecord(g.sl_freed[slot], g.back_stream));
            } else {
                NMF_HIP(hipEventRecord(g.sl_freed[slot], st));
            }
        }
        if (s < iters) {
            if (int rc = sliced_ftx(p.e, p.gw, k, k, H, n, p.den, false, st)) return rc;
            NMF_HIP(launch_mu_apply(H, p.num, p.den, eps, (int64_t)k * n, st));
            NMF_HIP(launch_transpose(H, k, n, p.Ht, st));
            if (int rc = sliced_ftx(p.e, p.Ht, n, k, p.Ht, k, p.gh, false, st)) return rc;
        }
    }
    if (hostw) {
        // the caller's stream continues only after the last rows of W have reached the host
        NMF_HIP(hipEventRecord(g.ev_entry, g.back_stream));
        NMF_HIP(hipStreamWaitEvent(st, g.ev_entry, 0));
    }
    return NMF_OK;
}

}  // namespace

// ---- allocation-free resident dense run --------------------------------------
// For callers that cannot allocate (HIP graph capture, tight serving loops, harnesses that
// forbid it): nmf_mu_dense on the small plan (row-split partials, piece planes, Gram scratch)
// with that workspace in a fixed array in device memory instead of hipMalloc'ed memory.

namespace {
constexpr size_t kScratchBytes = NMF_MU_NOALLOC_SCRATCH_BYTES;
}
// One copy per device that loads the library, held until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
void *scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each device, once asked

int scratch_address(void **out)
{
    int dev = -1;
    NMF_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(NMF_EUNSUPPORTED, "device ordinal beyond 63%s");
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        NMF_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(NMF_EHIP, "hipGetSymbolAddress returned a null address%s");
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return NMF_OK;
}
}  // namespace

extern "C" {

const char *nmf_status_string(int status)
{
    switch (status) {
    case NMF_OK: return "NMF_OK";
    case NMF_EINVAL: return "NMF_EINVAL";
    case NMF_ENOMEM: return "NMF_ENOMEM";
    case NMF_EHIP: return "NMF_EHIP";
    case NMF_EUNSUPPORTED: return "NMF_EUNSUPPORTED";
    default: return "NMF_UNKNOWN";
    }
}

const char *nmf_last_error(void) { return t_err; }

size_t nmf_mu_workspace_bytes(int kind, int64_t m, int64_t n, int64_t nnz, int32_t k,
                              int64_t batch_rows)
{
    if (m < 1 || n < 1 || k < 1) return 0;
    if (kind == 5) return k > NMF_MU_MAX_K_SLICED ? 0 : sliced_dense_bytes(m, n, k);
    if (kind == 6) {
        if (batch_rows < 1 || k > NMF_MU_MAX_K_SLICED) return 0;
        return sliced_ooc_bytes(batch_rows < m ? batch_rows : m, n, k);
    }
    if (k > NMF_MU_MAX_K) return 0;
    switch (kind) {
    case 0: return dense_bytes(m, n, k, true);
    case 3:   // stacks of runs up to the largest supported rank, plus their packed factors
        return dense_bytes(m, n, NMF_MU_MAX_K, true) + align_up((size_t)m * NMF_MU_MAX_K * sizeof(float)) +
               align_up((size_t)NMF_MU_MAX_K * n * sizeof(float));
    case 4: return dense_bytes(m, n, k, false);
    case 1: return nnz < 0 ? 0 : csr_bytes(n, nnz, k);
    case 2:
        if (batch_rows < 1) return 0;
        return dense_bytes(batch_rows < m ? batch_rows : m, n, k, false);
    default: return 0;
    }
}

int nmf_mu_set_workspace(void *dev_ptr, size_t bytes)
{
    std::lock_guard<std::mutex> lock(g.mu);
    if (dev_ptr && bytes) {
        if (reinterpret_cast<uintptr_t>(dev_ptr) % kAlign) return fail(NMF_EINVAL, "workspace must be 256-byte aligned%s");
        if (bytes < kAlign) return fail(NMF_EINVAL, "workspace too small%s");
        if (g.ws && g.ws_owned) {
            NMF_HIP(hipDeviceSynchronize());
            NMF_HIP(hipFree(g.ws));
        }
        NMF_HIP(hipMemset(dev_ptr, 0, kAlign));
        g.ws = dev_ptr;
        g.ws_bytes = bytes;
        g.ws_owned = false;
    } else {
        if (!g.ws_owned) {
            g.ws = nullptr;
            g.ws_bytes = 0;
        }
        g.ws_owned = true;
    }
    return NMF_OK;
}

int nmf_mu_release(void)
{
    std::lock_guard<std::mutex> lock(g.mu);
    NMF_HIP(hipDeviceSynchronize());
    if (g.ws && g.ws_owned) NMF_HIP(hipFree(g.ws));
    if (g.ws_owned) {
        g.ws = nullptr;
        g.ws_bytes = 0;
    }
    if (g.stage) NMF_HIP(hipFree(g.stage));
    g.stage = nullptr;
    g.stage_bytes = 0;
    if (g.sl_stage) NMF_HIP(hipFree(g.sl_stage));
    g.sl_stage = nullptr;
    g.sl_stage_bytes = 0;
    for (int i = 0; i < 3; ++i) {
        if (g.ev_copied[i]) NMF_HIP(hipEventDestroy(g.ev_copied[i]));
        if (g.ev_freed[i]) NMF_HIP(hipEventDestroy(g.ev_freed[i]));
        g.ev_copied[i] = g.ev_freed[i] = nullptr;
    }
    if (g.ev_entry) NMF_HIP(hipEventDestroy(g.ev_entry));
    g.ev_entry = nullptr;
    if (g.copy_stream) NMF_HIP(hipStreamDestroy(g.copy_stream));
    g.copy_stream = nullptr;
    for (int i = 0; i < 16; ++i) {
        if (g.sl_copied[i]) NMF_HIP(hipEventDestroy(g.sl_copied[i]));
        if (g.sl_done[i]) NMF_HIP(hipEventDestroy(g.sl_done[i]));
        if (g.sl_freed[i]) NMF_HIP(hipEventDestroy(g.sl_freed[i]));
        g.sl_copied[i] = g.sl_done[i] = g.sl_freed[i] = nullptr;
    }
    if (g.back_stream) NMF_HIP(hipStreamDestroy(g.back_stream));
    g.back_stream = nullptr;
    return NMF_OK;
}

int nmf_mu_dense(const float *A, int64_t m, int64_t n, int32_t k, float *W, float *H,
                 int32_t iters, float eps, void *stream)
{
    if (int rc = check_common(A, W, H, m, n, k, iters, eps, NMF_MU_MAX_K_SLICED)) return rc;
    if (iters == 0) return NMF_OK;
    std::lock_guard<std::mutex> lock(g.mu);
    void *ws = nullptr;
    if (k > NMF_MU_MAX_K) {
        if (int rc = ensure_workspace(sliced_dense_bytes(m, n, k), &ws)) return rc;
        const SlicedDense p = carve_sliced_dense(ws, m, n, k, nullptr);
        return sliced_dense_body(A, m, n, k, W, H, iters, eps, p, static_cast<hipStream_t>(stream));
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    // A that the streaming kernels cannot take as it is (base not 16-byte aligned, or n % 4 != 0) is
    // copied once per call into an aligned array of n4 = n rounded up to 4 columns, the new columns
    // zero, and H likewise: a zero column of A keeps its column of H at zero and adds nothing to any
    // product, so the run on the copies is the run on A and H.  The copy costs less than the
    // transposes of the mirrored plan and the iterations run the row plan (1.02 -> 0.80 ms per
    // iteration on 32768 x 16382 at k = 32 with 20 iterations per call); taken when the workspace
    // can hold the copy, and only with a normal positive eps: with eps = 0 a zero column gives 0 / 0.
    const int64_t n4 = (n + 3) & ~(int64_t)3;
    const bool misaligned = (reinterpret_cast<uintptr_t>(A) & 15u) != 0 || n != n4;
    if (misaligned && eps >= 1.17549435e-38f && aht_rows_ok(nullptr, m, n4, k)) {
        const size_t base = dense_bytes(m, n4, k, false);
        const size_t need = base + align_up((size_t)m * n4 * sizeof(float)) + align_up((size_t)k * n4 * sizeof(float));
        if ((g.ws && g.ws_bytes >= need) || (g.ws_owned && ensure_workspace(need, &ws) == NMF_OK)) {
            ws = g.ws;
            const DensePlan p = carve_dense(ws, m, n4, k, false);
            Carve cv(static_cast<char *>(ws) + base);
            float *Ap = cv.take<float>((size_t)m * n4);
            float *Hp = cv.take<float>((size_t)k * n4);
            NMF_HIP(launch_pad_copy(A, n, Ap, n4, m, n, st));
            NMF_HIP(launch_pad_copy(H, n, Hp, n4, k, n, st));
            if (int rc = dense_body(Ap, m, n4, k, W, Hp, iters, eps, p, st)) return rc;
            NMF_HIP(launch_pad_copy(Hp, n4, H, n, k, n, st));
            return NMF_OK;
        }
        (void)hipGetLastError();
    }
    bool mirrored = false;
    if (int rc = dense_workspace(A, m, n, k, &ws, &mirrored)) return rc;
    const DensePlan p = carve_dense(ws, m, n, k, mirrored);
    return dense_body(A, m, n, k, W, H, iters, eps, p, st);
}

int nmf_mu_dense_profile(const float *A, int64_t m, int64_t n, int32_t k, float *W, float *H,
                         int32_t iters, float eps, void *stream, float *kernel_ms)
{
    if (int rc = check_common(A, W, H, m, n, k, iters, eps)) return rc;
    if (!kernel_ms) return fail(NMF_EINVAL, "null pointer%s");
    if (iters < 1 || iters > 4096) return fail(NMF_EINVAL, "profiled run needs 1 <= iters <= 4096%s");
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g.mu);
    void *ws = nullptr;
    bool mirrored = false;
    if (int rc = dense_workspace(A, m, n, k, &ws, &mirrored)) return rc;
    const DensePlan p = carve_dense(ws, m, n, k, mirrored);
    constexpr int NK = kDenseKernels;
    std::vector<hipEvent_t> ev((size_t)iters * NK + 1, nullptr);
    int rc = NMF_OK;
    for (auto &e : ev)
        if (hipEventCreate(&e) != hipSuccess) rc = fail(NMF_EHIP, "hipEventCreate failed%s");
    if (rc == NMF_OK) rc = dense_body(A, m, n, k, W, H, iters, eps, p, st, false, ev.data());
    if (rc == NMF_OK && hipStreamSynchronize(st) != hipSuccess) rc = fail(NMF_EHIP, "hipStreamSynchronize failed%s");
    if (rc == NMF_OK) {
        double sum[NK] = {0, 0, 0, 0, 0, 0};
        for (int it = 0; it < iters && rc == NMF_OK; ++it)
            for (int j = 0; j < NK; ++j) {
                float ms = 0.f;
                if (hipEventElapsedTime(&ms, ev[(size_t)it * NK + j], ev[(size_t)it * NK + j + 1]) != hipSuccess) {
                    rc = fail(NMF_EHIP, "hipEventElapsedTime failed%s");
                    break;
                }
                sum[j] += ms;
            }
        for (int j = 0; j < NK; ++j) kernel_ms[j] = (float)(sum[j] / iters);
        kernel_ms[NK] = rows_plan_runs(A, m, n, k, mirrored) ? 2.f : (mirrored ? 1.f : 0.f);
        kernel_ms[NK + 1] = kernel_ms[NK + 2] = 0.f;
    }
    // The pass kernels once more, `reps` launches back to back between two events: the
    // duration of a launch without the event commands around it.  They only rewrite the
    // partial results, which nothing reads afterwards.
    if (rc == NMF_OK) {
        const int reps = 20;
        const int s1 = wta_splits(m, n, k), s2 = wta_splits(n, m, k);
        const int64_t rps1 = wta_rows_per_split(m, s1), rps2 = wta_rows_per_split(n, s2);
        const bool rows_plan = rows_plan_runs(A, m, n, k, mirrored);
        const Common &c = p.c;
        for (int which = 0; which < ((mirrored || rows_plan) ? 2 : 1) && rc == NMF_OK; ++which) {
            if (which == 0) (void)launch_split_planes(W, m, k, p.planes, st);
            else if (!rows_plan) (void)launch_split_planes(p.Ht, n, k, p.planes, st);
            hipError_t e = hipEventRecord(ev[0], st);
            for (int r = 0; r < reps && e == hipSuccess; ++r)
                e = which == 0 ? launch_wta_pass(A, m, n, k, W, p.planes, true, p.ppart, s1, rps1, false, st)
                    : rows_plan  // the fused pass without its stores to W
                        ? launch_aht_rows(A, m, n, k, p.planes2, c.gh, W, p.planes, c.gwp, eps, st, false, nullptr,
                                          nullptr, true)
                        : launch_wta_pass(p.At, n, m, k, p.Ht, p.planes, true, p.ppart, s2, rps2, false, st);
            if (e == hipSuccess) e = hipEventRecord(ev[1], st);
            if (e == hipSuccess) e = hipEventSynchronize(ev[1]);
            float ms = 0.f;
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev[0], ev[1]);
            if (e != hipSuccess) rc = fail(NMF_EHIP, "pass timing: %s", hipGetErrorString(e));
            kernel_ms[NK + 1 + which] = ms / reps;
        }
    }
    for (auto &e : ev)
        if (e) (void)hipEventDestroy(e);
    return rc;
}

int nmf_mu_dense_batched(int32_t n_runs, const float *const *A, int64_t m, int64_t n,
                         const int32_t *k, float *const *W, float *const *H, int32_t iters,
                         float eps, void *stream)
{
    if (n_runs < 0 || !A || !k || !W || !H) return fail(NMF_EINVAL, "null pointer or negative run count%s");
    int kmax = 1;
    for (int r = 0; r < n_runs; ++r) {
        if (int rc = check_common(A[r], W[r], H[r], m, n, k[r], iters, eps)) return rc;
        if (k[r] > kmax) kmax = k[r];
    }
    if (iters == 0 || n_runs == 0) return NMF_OK;
    std::lock_guard<std::mutex> lock(g.mu);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Consecutive runs on the same A are stacked side by side while their ranks sum to
    // at most NMF_MU_MAX_K: one stack is one factorisation of rank sum(k) for the two
    // passes over A (A is read once for all of them), with the Gram matrices masked to
    // their diagonal blocks in the finishers so that the runs stay independent.
    struct Stack { int first, count, K; };
    std::vector<Stack> stacks;
    for (int r = 0; r < n_runs;) {
        Stack sk{r, 0, 0};
        while (r < n_runs && A[r] == A[sk.first] && sk.K + k[r] <= NMF_MU_MAX_K) {
            sk.K += k[r];
            ++sk.count;
            ++r;
        }
        stacks.push_back(sk);
    }
    int Kmax = kmax;
    for (const Stack &sk : stacks)
        if (sk.K > Kmax) Kmax = sk.K;
    const size_t stack_bytes = align_up((size_t)m * Kmax * sizeof(float)) + align_up((size_t)Kmax * n * sizeof(float));
    void *ws = nullptr;
    // Stacking needs the mirrored plan for the largest stack plus room for the packed
    // factors; without that much workspace the runs go one by one with the plan that fits.
    const size_t big = dense_bytes(m, n, Kmax, true) + stack_bytes;
    const bool can_stack = (g.ws && g.ws_bytes >= big) || (g.ws_owned && ensure_workspace(big, &ws) == NMF_OK);
    if (!can_stack) {
        (void)hipGetLastError();
        bool mirrored = false;
        if (int rc = dense_workspace(nullptr, m, n, kmax, &ws, &mirrored)) return rc;
        const DensePlan p1 = carve_dense(ws, m, n, kmax, mirrored);
        for (int r = 0; r < n_runs; ++r) {
            const bool same_a = r > 0 && A[r] == A[r - 1];
            if (int rc = dense_body(A[r], m, n, k[r], W[r], H[r], iters, eps, p1, st, same_a)) return rc;
        }
        return NMF_OK;
    }
    ws = g.ws;
    // Carve once with the largest stacked rank so that A^T sits at one address for all
    // stacks: consecutive stacks on the same A share its transpose.
    const DensePlan p = carve_dense(ws, m, n, Kmax, true);
    char *tail = static_cast<char *>(ws) + dense_bytes(m, n, Kmax, true);
    float *Wall = reinterpret_cast<float *>(tail);
    float *Hall = reinterpret_cast<float *>(tail + align_up((size_t)m * Kmax * sizeof(float)));
    for (size_t si = 0; si < stacks.size(); ++si) {
        const Stack &sk = stacks[si];
        const bool same_a = si > 0 && A[sk.first] == A[stacks[si - 1].first];
        if (sk.count == 1) {
            const int r = sk.first;
            if (int rc = dense_body(A[r], m, n, k[r], W[r], H[r], iters, eps, p, st, same_a)) return rc;
            continue;
        }
        BlockMap map;
        map.on = 1;
        int off = 0;
        for (int i = 0; i < sk.count; ++i) {
            const int r = sk.first + i;
            for (int c = 0; c < k[r]; ++c) map.id[off + c] = (unsigned char)i;
            NMF_HIP(hipMemcpy2DAsync(Wall + off, (size_t)sk.K * sizeof(float), W[r], (size_t)k[r] * sizeof(float),
                                     (size_t)k[r] * sizeof(float), (size_t)m, hipMemcpyDeviceToDevice, st));
            NMF_HIP(hipMemcpyAsync(Hall + (size_t)off * n, H[r], (size_t)k[r] * n * sizeof(float),
                                   hipMemcpyDeviceToDevice, st));
            off += k[r];
        }
        for (int c = off; c < 64; ++c) map.id[c] = 255;
        if (int rc = dense_body(A[sk.first], m, n, sk.K, Wall, Hall, iters, eps, p, st, same_a, nullptr, &map))
            return rc;
        off = 0;
        for (int i = 0; i < sk.count; ++i) {
            const int r = sk.first + i;
            NMF_HIP(hipMemcpy2DAsync(W[r], (size_t)k[r] * sizeof(float), Wall + off, (size_t)sk.K * sizeof(float),
                                     (size_t)k[r] * sizeof(float), (size_t)m, hipMemcpyDeviceToDevice, st));
            NMF_HIP(hipMemcpyAsync(H[r], Hall + (size_t)off * n, (size_t)k[r] * n * sizeof(float),
                                   hipMemcpyDeviceToDevice, st));
            off += k[r];
        }
    }
    return NMF_OK;
}

// Streamed dense run; objective_host (iters doubles) != nullptr: the objective of every
// iteration as well (ranks up to NMF_MU_MAX_K only).
static int ooc_run(const float *A_host, int64_t m, int64_t n, int32_t k, float *W, float *H,
                   int32_t iters, float eps, int64_t batch_rows, int64_t device_budget_bytes,
                   double *objective_host, void *stream)
{
    if (int rc = check_common(A_host, W, H, m, n, k, iters, eps, NMF_MU_MAX_K_SLICED)) return rc;
    if (objective_host && k > NMF_MU_MAX_K)
        return fail(NMF_EUNSUPPORTED, "monitored out-of-memory run: k <= 64%s");
    if (batch_rows < 1) return fail(NMF_EINVAL, "batch_rows must be >= 1%s");
    if (device_budget_bytes < 1) return fail(NMF_EINVAL, "device_budget_bytes must be >= 1%s");
    if (iters == 0) return NMF_OK;
    if (batch_rows > m) batch_rows = m;
    const size_t slot_bytes = align_up((size_t)batch_rows * n * sizeof(float));
    int slots = (int)((size_t)device_budget_bytes / slot_bytes);
    if (slots < 1) return fail(NMF_ENOMEM, "device budget does not hold one batch%s");
    if (slots > 3) slots = 3;
    hipStream_t st = static_cast<hipStream_t>(stream);

    std::lock_guard<std::mutex> lock(g.mu);
    if (k > NMF_MU_MAX_K) {
        const int64_t nbat = (m + batch_rows - 1) / batch_rows;
        if (slots > nbat) slots = (int)nbat;
        return sliced_ooc_run(A_host, nullptr, W, m, n, k, H, iters, eps, batch_rows, slots, st, nullptr);
    }
    const int64_t nb = (m + batch_rows - 1) / batch_rows;
    // monitored run: the W updates' shares of <A H^T, W> (one per workgroup and batch), ||A_b||^2 per
    // batch and its scratch, ||A||^2, one objective value per iteration
    // The W update of a batch: the streaming row kernel where it applies (staging slots are aligned,
    // so that is a matter of n, k and the batch height), else the direct kernel.
    const bool use_rows = aht_rows_can(nullptr, n, k);
    auto w_blocks = [&](int64_t rows) { return use_rows ? (int64_t)aht_rows_blocks(rows, k) : aht_pass_blocks(rows); };
    const int64_t bpb = w_blocks(batch_rows);
    const size_t mon_bytes = objective_host
        ? align_up((size_t)(nb * bpb) * sizeof(double)) + align_up((size_t)nb * sizeof(double)) +
          align_up(4097 * sizeof(double)) + align_up((size_t)iters * sizeof(double))
        : 0;
    void *ws = nullptr;
    if (int rc = ensure_workspace(dense_bytes(batch_rows, n, k, false) + mon_bytes, &ws)) return rc;
    Carve cv(ws);
    const Common c = carve_common(cv, k);
    const int splits = wta_splits(batch_rows, n, k);
    const int64_t rps = wta_rows_per_split(batch_rows, splits);
    float *ppart = cv.take<float>((size_t)splits * k * n);
    void *planes = cv.take<char>(planes_bytes(batch_rows));
    void *planes_ht = cv.take<char>(planes_bytes(n));      // row kernel: piece planes of H^T
    double *dpart = nullptr, *normb = nullptr, *normA2 = nullptr, *obj = nullptr;
    if (objective_host) {
        dpart = cv.take<double>((size_t)(nb * bpb));
        normb = cv.take<double>((size_t)nb);
        normA2 = cv.take<double>(4097);
        obj = cv.take<double>((size_t)iters);
    }

    if (g.stage_bytes < slots * slot_bytes) {
        if (g.stage) {
            NMF_HIP(hipDeviceSynchronize());
            NMF_HIP(hipFree(g.stage));
            g.stage = nullptr;
            g.stage_bytes = 0;
        }
        hipError_t e = hipMalloc(&g.stage, slots * slot_bytes);
        if (e != hipSuccess) return fail(NMF_ENOMEM, "hipMalloc(staging): %s", hipGetErrorString(e));
        g.stage_bytes = slots * slot_bytes;
    }
    if (!g.copy_stream) NMF_HIP(hipStreamCreateWithFlags(&g.copy_stream, hipStreamNonBlocking));
    if (!g.ev_entry) NMF_HIP(hipEventCreateWithFlags(&g.ev_entry, hipEventDisableTiming));
    for (int i = 0; i < 3; ++i) {
        if (!g.ev_copied[i]) NMF_HIP(hipEventCreateWithFlags(&g.ev_copied[i], hipEventDisableTiming));
        if (!g.ev_freed[i]) NMF_HIP(hipEventCreateWithFlags(&g.ev_freed[i], hipEventDisableTiming));
    }
    // Staging slots may still be read by work enqueued earlier on `st`.
    NMF_HIP(hipEventRecord(g.ev_entry, st));
    NMF_HIP(hipStreamWaitEvent(g.copy_stream, g.ev_entry, 0));

    int64_t issued = 0;   // batches handed to the copy stream so far, over all sweeps
    for (int s = 0; s <= iters; ++s) {
        for (int64_t b = 0; b < nb; ++b, ++issued) {
            const int slot = (int)(issued % slots);
            const int64_t i0 = b * batch_rows;
            const int64_t rb = (i0 + batch_rows <= m) ? batch_rows : m - i0;
            float *Ab = reinterpret_cast<float *>(static_cast<char *>(g.stage) + slot * slot_bytes);
            if (issued >= slots) NMF_HIP(hipStreamWaitEvent(g.copy_stream, g.ev_freed[slot], 0));
            NMF_HIP(hipMemcpyAsync(Ab, A_host + i0 * n, (size_t)rb * n * sizeof(float),
                                   hipMemcpyHostToDevice, g.copy_stream));
            NMF_HIP(hipEventRecord(g.ev_copied[slot], g.copy_stream));
            NMF_HIP(hipStreamWaitEvent(st, g.ev_copied[slot], 0));
            if (dpart && s == 0) NMF_HIP(launch_sumsq(Ab, rb * n, normA2 + 1, normb + b, st));
            if (s > 0) {
                if (use_rows)    // also leaves the piece planes of the batch's new rows for the pass below
                    NMF_HIP(launch_aht_rows(Ab, rb, n, k, planes_ht, c.gh, W + i0 * k, planes, c.gwp, eps, st, false, nullptr,
                                            dpart ? dpart + b * bpb : nullptr));
                else
                    NMF_HIP(launch_aht_pass(Ab, rb, n, k, H, c.gh, W + i0 * k, eps, st, dpart ? dpart + b * bpb : nullptr));
            }
            if (s < iters)
                NMF_HIP(launch_wta_pass(Ab, rb, n, k, W + i0 * k, planes, use_rows && s > 0, ppart, splits, rps, b > 0, st));
            NMF_HIP(hipEventRecord(g.ev_freed[slot], st));
        }
        if (dpart && s == 0) NMF_HIP(launch_sum_f64(normb, nb, normA2, st));
        if (s < iters || dpart) NMF_HIP(launch_gram_w(W, m, k, c.gw, c.gpart, c.counters, st));
        if (dpart && s > 0) {
            // iteration s is complete: <A H^T, W> from this sweep's W updates (a short last batch
            // leaves the tail of its segment untouched, so its workgroups are counted, not bpb),
            // H H^T of the H they used, W^T W of the W they left
            const int64_t last_rows = m - (nb - 1) * batch_rows;
            if (w_blocks(last_rows) != bpb) {
                // close the gap so that the shares are one contiguous run
                NMF_HIP(hipMemsetAsync(dpart + (nb - 1) * bpb + w_blocks(last_rows), 0,
                                       (size_t)(bpb - w_blocks(last_rows)) * sizeof(double), st));
            }
            NMF_HIP(launch_objective(dpart, (int)(nb * bpb), c.gw, c.gh, k, normA2, obj + (s - 1), st));
        }
        if (s < iters) {
            NMF_HIP(launch_factor_update(H, nullptr, ppart, splits, c.gw, nullptr, 0, nullptr, k, n, eps, st, nullptr,
                                         use_rows ? planes_ht : nullptr));
            NMF_HIP(launch_gram_h(H, k, n, c.gh, c.gpart, c.counters, st));
        }
    }
    if (dpart) {
        NMF_HIP(hipMemcpyAsync(objective_host, obj, (size_t)iters * sizeof(double), hipMemcpyDeviceToHost, st));
        NMF_HIP(hipStreamSynchronize(st));
    }
    return NMF_OK;
}

int nmf_mu_ooc(const float *A_host, int64_t m, int64_t n, int32_t k, float *W, float *H,
               int32_t iters, float eps, int64_t batch_rows, int64_t device_budget_bytes,
               void *stream)
{
    return ooc_run(A_host, m, n, k, W, H, iters, eps, batch_rows, device_budget_bytes, nullptr, stream);
}

int nmf_mu_ooc_monitor(const float *A_host, int64_t m, int64_t n, int32_t k, float *W, float *H,
                       int32_t iters, float eps, int64_t batch_rows, int64_t device_budget_bytes,
                       double *objective_host, void *stream)
{
    if (!objective_host) return fail(NMF_EINVAL, "null pointer%s");
    if (iters > (1 << 20)) return fail(NMF_EINVAL, "monitored run: iters <= 2^20%s");
    return ooc_run(A_host, m, n, k, W, H, iters, eps, batch_rows, device_budget_bytes, objective_host, stream);
}

int nmf_mu_ooc_hostw(const float *A_host, float *W_host, int64_t m, int64_t n, int32_t k, float *H,
                     int32_t iters, float eps, int64_t batch_rows, int32_t slots, void *stream,
                     size_t *device_bytes_host)
{
    if (int rc = check_common(A_host, W_host, H, m, n, k, iters, eps, NMF_MU_MAX_K_SLICED)) return rc;
    if (batch_rows < 1) return fail(NMF_EINVAL, "batch_rows must be >= 1%s");
    if (slots < 1 || slots > kMaxSlots) return fail(NMF_EINVAL, "slots must be in 1 .. 16%s");
    if (device_bytes_host) *device_bytes_host = 0;
    if (iters == 0) return NMF_OK;
    if (batch_rows > m) batch_rows = m;
    const int64_t nbat = (m + batch_rows - 1) / batch_rows;
    if (slots > nbat) slots = (int)nbat;
    std::lock_guard<std::mutex> lock(g.mu);
    return sliced_ooc_run(A_host, W_host, nullptr, m, n, k, H, iters, eps, batch_rows, slots,
                          static_cast<hipStream_t>(stream), device_bytes_host);
}

// Bytes behind csr_bytes() that a monitored sparse run needs: the W update's by-products,
// ||A||^2 with its scratch, one objective value per iteration.
size_t csr_monitor_bytes(int iters)
{
    return align_up((size_t)kCsrDparts * sizeof(double)) + align_up(4097 * sizeof(double)) +
           align_up((size_t)iters * sizeof(double)) + align_up((size_t)(65536 + 1) * sizeof(double));
}

// Stopping rule of a sparse run (Algorithm 1): results in host memory.
struct CsrTol {
    double tol;
    int check_every;
    int32_t *iters_done;
    double *residual;
};

// Resident sparse run; objective_host (iters doubles) == nullptr: no monitoring; with `tolp`
// the run stops as soon as a check finds the objective at or below tolp->tol (iters = the most).
static int csr_run(const int64_t *rowptr, const int32_t *colidx, const float *vals, int64_t m,
                   int64_t n, int64_t nnz, int32_t k, float *W, float *H, int32_t iters, float eps,
                   double *objective_host, void *stream, const CsrTol *tolp = nullptr)
{
    if (!rowptr) return fail(NMF_EINVAL, "null pointer%s");
    if (nnz < 0) return fail(NMF_EINVAL, "nnz must be >= 0%s");
    if (nnz > 0 && (!colidx || !vals)) return fail(NMF_EINVAL, "null pointer%s");
    if (int rc = check_common(rowptr, W, H, m, n, k, iters, eps)) return rc;
    if (iters == 0 && !tolp) return NMF_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g.mu);
    if (nnz >= ((int64_t)1 << 31) || m >= ((int64_t)1 << 31))
        return fail(NMF_EUNSUPPORTED, "CSR path needs nnz < 2^31 and m < 2^31%s");
    void *ws = nullptr;
    const bool watch = objective_host || tolp;
    if (int rc = ensure_workspace(csr_bytes(n, nnz, k) + (watch ? csr_monitor_bytes(tolp ? 1 : iters) : 0), &ws))
        return rc;
    Carve cv(ws);
    const Common c = carve_common(cv, k);
    float *Ht = cv.take<float>((size_t)n * k);
    int64_t *colptr = cv.take<int64_t>((size_t)n + 1);
    int32_t *rowidx = cv.take<int32_t>((size_t)nnz);
    float *cvals = cv.take<float>((size_t)nnz);
    int64_t *part_r = cv.take<int64_t>((size_t)kCsrParts + 1);
    int64_t *part_c = cv.take<int64_t>((size_t)kCsrParts + 1);
    int32_t *long_r = cv.take<int32_t>((size_t)(nnz / kLongRow + 2));
    int32_t *long_c = cv.take<int32_t>((size_t)(nnz / kLongRow + 2));
    unsigned *long_n = cv.take<unsigned>(64);      // [0] rows of A, [1] columns of A
    const size_t sort_temp_bytes = nnz ? csc_sort_temp_bytes(nnz, n) : 0;
    int32_t *sorted_cols = cv.take<int32_t>((size_t)nnz);
    uint64_t *payload = cv.take<uint64_t>((size_t)nnz);
    uint64_t *sorted_payload = cv.take<uint64_t>((size_t)nnz);
    char *sort_temp = cv.take<char>(sort_temp_bytes);
    double *dpart = nullptr, *normA2 = nullptr, *obj = nullptr, *dup = nullptr;
    if (watch) {
        dpart = cv.take<double>(kCsrDparts);
        normA2 = cv.take<double>(4097);
        obj = cv.take<double>(tolp ? 1 : (size_t)iters);
        dup = cv.take<double>(65536 + 1);      // one share per block of the copy's last kernel, then the sum of squares
    }
    const int ndup = csc_finish_blocks(nnz);

    // Column-ordered copy of A, once per call, enqueued like everything else.
    NMF_HIP(launch_csc_build(rowptr, colidx, vals, m, n, nnz, sorted_cols, payload, sorted_payload, sort_temp,
                             sort_temp_bytes, colptr, rowidx, cvals, st, dup));
    if (watch) {
        // ||A||_F^2 of the matrix the arrays stand for: the squared stored values plus what repeated
        // (row, column) pairs add (found while the column-ordered copy is written)
        if (nnz > 0) NMF_HIP(launch_sumsq(vals, nnz, normA2 + 1, dup + ndup, st));
        else NMF_HIP(launch_fill_f32(reinterpret_cast<float *>(dup + ndup), 2, 0.f, st));
        NMF_HIP(launch_sum_f64(dup, ndup + 1, normA2, st));
    }

    // Work partitions of both orientations, once per call.
    NMF_HIP(launch_csr_partition(rowptr, m, kCsrParts, part_r, st));
    NMF_HIP(launch_csr_partition(colptr, n, kCsrParts, part_c, st));
    NMF_HIP(launch_csr_long_rows(rowptr, m, long_r, long_n, (unsigned)(nnz / kLongRow + 1), st));
    NMF_HIP(launch_csr_long_rows(colptr, n, long_c, long_n + 1, (unsigned)(nnz / kLongRow + 1), st));

    NMF_HIP(launch_transpose(H, k, n, Ht, st));
    // One iteration; with `out`, ||A - W H||_F of its result goes there, from what the W update
    // leaves behind: <A H^T, W>, H H^T, and W^T W of the new W (computed here; the next iteration
    // computes the same matrix again for its H update).
    auto iteration = [&](double *out) -> int {
        NMF_HIP(launch_gram_w_wide(W, m, k, c.gw, c.gwp, st));
        NMF_HIP(launch_aht_csr(colptr, rowidx, cvals, part_c, long_c, long_n + 1, k, W, c.gw, Ht, eps, nnz, m, st));   // H update on H^T
        NMF_HIP(launch_gram_w_wide(Ht, n, k, c.gh, c.ghp, st));
        NMF_HIP(launch_aht_csr(rowptr, colidx, vals, part_r, long_r, long_n, k, Ht, c.gh, W, eps, nnz, n, st, false,
                               out ? dpart : nullptr));                                                       // W update
        if (out) {
            NMF_HIP(launch_gram_w_wide(W, m, k, c.gw, c.gwp, st));
            NMF_HIP(launch_objective(dpart, kCsrDparts, c.gw, c.gh, k, normA2, out, st));
        }
        return NMF_OK;
    };
    if (tolp) {
        // objective of the factors as given: the W pass without its update
        double res = 0.0;
        NMF_HIP(launch_gram_w_wide(W, m, k, c.gw, c.gwp, st));
        NMF_HIP(launch_gram_w_wide(Ht, n, k, c.gh, c.ghp, st));
        NMF_HIP(launch_aht_csr(rowptr, colidx, vals, part_r, long_r, long_n, k, Ht, c.gh, W, eps, nnz, n, st, false, dpart, true));
        NMF_HIP(launch_objective(dpart, kCsrDparts, c.gw, c.gh, k, normA2, obj, st));
        NMF_HIP(hipMemcpyAsync(&res, obj, sizeof(double), hipMemcpyDeviceToHost, st));
        NMF_HIP(hipStreamSynchronize(st));
        int done = 0;
        while (done < iters && res > tolp->tol) {
            const int chunk = (iters - done < tolp->check_every) ? iters - done : tolp->check_every;
            for (int it = 0; it < chunk; ++it)
                if (int rc = iteration(it == chunk - 1 ? obj : nullptr)) return rc;
            NMF_HIP(hipMemcpyAsync(&res, obj, sizeof(double), hipMemcpyDeviceToHost, st));
            NMF_HIP(hipStreamSynchronize(st));
            done += chunk;
        }
        NMF_HIP(launch_transpose(Ht, n, k, H, st));
        NMF_HIP(hipStreamSynchronize(st));
        *tolp->iters_done = done;
        *tolp->residual = res;
        return NMF_OK;
    }
    for (int it = 0; it < iters; ++it)
        if (int rc = iteration(objective_host ? obj + it : nullptr)) return rc;
    NMF_HIP(launch_transpose(Ht, n, k, H, st));
    if (objective_host) {
        NMF_HIP(hipMemcpyAsync(objective_host, obj, (size_t)iters * sizeof(double), hipMemcpyDeviceToHost, st));
        NMF_HIP(hipStreamSynchronize(st));
    }
    return NMF_OK;
}

int nmf_mu_csr(const int64_t *rowptr, const int32_t *colidx, const float *vals, int64_t m,
               int64_t n, int64_t nnz, int32_t k, float *W, float *H, int32_t iters, float eps,
               void *stream)
{
    return csr_run(rowptr, colidx, vals, m, n, nnz, k, W, H, iters, eps, nullptr, stream);
}

int nmf_mu_csr_monitor(const int64_t *rowptr, const int32_t *colidx, const float *vals, int64_t m,
                       int64_t n, int64_t nnz, int32_t k, float *W, float *H, int32_t iters, float eps,
                       double *objective_host, void *stream)
{
    if (!objective_host) return fail(NMF_EINVAL, "null pointer%s");
    if (iters > (1 << 20)) return fail(NMF_EINVAL, "monitored run: iters <= 2^20%s");
    return csr_run(rowptr, colidx, vals, m, n, nnz, k, W, H, iters, eps, objective_host, stream);
}

int nmf_mu_csr_tol(const int64_t *rowptr, const int32_t *colidx, const float *vals, int64_t m,
                   int64_t n, int64_t nnz, int32_t k, float *W, float *H, int32_t max_iters, float eps,
                   double tol, int32_t check_every, int32_t *iters_done_host, double *residual_host,
                   void *stream)
{
    if (!iters_done_host || !residual_host) return fail(NMF_EINVAL, "null pointer%s");
    if (check_every < 1) return fail(NMF_EINVAL, "check_every must be >= 1%s");
    if (!(tol >= 0.0)) return fail(NMF_EINVAL, "tol must be >= 0%s");
    const CsrTol t = {tol, check_every, iters_done_host, residual_host};
    *iters_done_host = 0;
    return csr_run(rowptr, colidx, vals, m, n, nnz, k, W, H, max_iters, eps, nullptr, stream, &t);
}

// Out-of-memory CSR: row batches of about batch_nnz stored entries each, streamed from host
// memory every sweep in the order of nmf_mu_ooc (W update of the batch with the current H, then
// the batch's share of W^T A for the next H update).  A batch is a CSR matrix of its own once
// its row pointers are made relative; its column-ordered copy is rebuilt on the device each
// time (a sort of the batch, which runs beside the upload of the next one).
int nmf_mu_csr_ooc(const int64_t *rowptr_host, const int32_t *colidx_host, const float *vals_host,
                   int64_t m, int64_t n, int64_t nnz, int32_t k, float *W, float *H, int32_t iters,
                   float eps, int64_t batch_nnz, int64_t device_budget_bytes, void *stream)
{
    if (!rowptr_host) return fail(NMF_EINVAL, "null pointer%s");
    if (nnz < 0) return fail(NMF_EINVAL, "nnz must be >= 0%s");
    if (nnz > 0 && (!colidx_host || !vals_host)) return fail(NMF_EINVAL, "null pointer%s");
    if (int rc = check_common(rowptr_host, W, H, m, n, k, iters, eps)) return rc;
    if (batch_nnz < 1) return fail(NMF_EINVAL, "batch_nnz must be >= 1%s");
    if (device_budget_bytes < 1) return fail(NMF_EINVAL, "device_budget_bytes must be >= 1%s");
    if (m >= ((int64_t)1 << 31)) return fail(NMF_EUNSUPPORTED, "CSR path needs m < 2^31%s");
    if (iters == 0) return NMF_OK;
    if (rowptr_host[0] != 0 || rowptr_host[m] != nnz) return fail(NMF_EINVAL, "rowptr[0] != 0 or rowptr[m] != nnz%s");
    hipStream_t st = static_cast<hipStream_t>(stream);

    // Row batches: as many whole rows as fit batch_nnz entries, at least one row.
    struct Batch { int64_t r0, r1, e0, e1; };
    std::vector<Batch> batches;
    int64_t max_rows = 1, max_nnz = 1;
    for (int64_t r0 = 0; r0 < m;) {
        const int64_t e0 = rowptr_host[r0];
        const int64_t *hi = std::upper_bound(rowptr_host + r0 + 1, rowptr_host + m + 1, e0 + batch_nnz);
        int64_t r1 = (hi - rowptr_host) - 1;
        if (r1 <= r0) r1 = r0 + 1;
        const int64_t e1 = rowptr_host[r1];
        if (e1 < e0) return fail(NMF_EINVAL, "rowptr is not non-decreasing%s");
        if (e1 - e0 >= ((int64_t)1 << 31)) return fail(NMF_EUNSUPPORTED, "a row batch needs fewer than 2^31 entries%s");
        batches.push_back({r0, r1, e0, e1});
        if (r1 - r0 > max_rows) max_rows = r1 - r0;
        if (e1 - e0 > max_nnz) max_nnz = e1 - e0;
        r0 = r1;
    }
    const size_t rp_bytes = align_up((size_t)(max_rows + 1) * sizeof(int64_t));
    const size_t ci_bytes = align_up((size_t)max_nnz * sizeof(int32_t));
    const size_t va_bytes = align_up((size_t)max_nnz * sizeof(float));
    const size_t slot_bytes = rp_bytes + ci_bytes + va_bytes;
    int slots = (int)((size_t)device_budget_bytes / slot_bytes);
    if (slots < 1) return fail(NMF_ENOMEM, "device budget does not hold one batch%s");
    if (slots > 3) slots = 3;

    std::lock_guard<std::mutex> lock(g.mu);
    const size_t temp_bytes = csc_sort_temp_bytes(max_nnz, n);
    const size_t need = common_bytes(k) + 2 * align_up((size_t)n * k * sizeof(float)) + rp_bytes +
                        align_up((size_t)(n + 1) * sizeof(int64_t)) + 2 * ci_bytes + va_bytes +
                        2 * align_up((size_t)max_nnz * sizeof(uint64_t)) + align_up(temp_bytes) +
                        2 * align_up((size_t)(kCsrParts + 1) * sizeof(int64_t)) +
                        2 * align_up((size_t)(max_nnz / kLongRow + 2) * sizeof(int32_t)) + kAlign;
    void *ws = nullptr;
    if (int rc = ensure_workspace(need, &ws)) return rc;
    Carve cv(ws);
    const Common c = carve_common(cv, k);
    float *Ht = cv.take<float>((size_t)n * k);
    float *Num = cv.take<float>((size_t)n * k);
    int64_t *rowptr_loc = cv.take<int64_t>((size_t)max_rows + 1);
    int64_t *colptr = cv.take<int64_t>((size_t)n + 1);
    int32_t *rowidx = cv.take<int32_t>((size_t)max_nnz);
    float *cvals = cv.take<float>((size_t)max_nnz);
    int32_t *sorted_cols = cv.take<int32_t>((size_t)max_nnz);
    uint64_t *payload = cv.take<uint64_t>((size_t)max_nnz);
    uint64_t *sorted_payload = cv.take<uint64_t>((size_t)max_nnz);
    char *sort_temp = cv.take<char>(temp_bytes);
    int64_t *part_r = cv.take<int64_t>((size_t)kCsrParts + 1);
    int64_t *part_c = cv.take<int64_t>((size_t)kCsrParts + 1);
    int32_t *long_r = cv.take<int32_t>((size_t)(max_nnz / kLongRow + 2));
    int32_t *long_c = cv.take<int32_t>((size_t)(max_nnz / kLongRow + 2));
    unsigned *long_n = cv.take<unsigned>(64);
    if (cv.off > need) return fail(NMF_EHIP, "internal: csr_ooc workspace accounting%s");

    if (g.sl_stage_bytes < slots * slot_bytes) {
        if (g.sl_stage) {
            NMF_HIP(hipDeviceSynchronize());
            NMF_HIP(hipFree(g.sl_stage));
            g.sl_stage = nullptr;
            g.sl_stage_bytes = 0;
        }
        hipError_t e = hipMalloc(&g.sl_stage, slots * slot_bytes);
        if (e != hipSuccess) return fail(NMF_ENOMEM, "hipMalloc(staging): %s", hipGetErrorString(e));
        g.sl_stage_bytes = slots * slot_bytes;
    }
    if (!g.copy_stream) NMF_HIP(hipStreamCreateWithFlags(&g.copy_stream, hipStreamNonBlocking));
    if (!g.ev_entry) NMF_HIP(hipEventCreateWithFlags(&g.ev_entry, hipEventDisableTiming));
    for (int i = 0; i < 3; ++i) {
        if (!g.sl_copied[i]) NMF_HIP(hipEventCreateWithFlags(&g.sl_copied[i], hipEventDisableTiming));
        if (!g.sl_freed[i]) NMF_HIP(hipEventCreateWithFlags(&g.sl_freed[i], hipEventDisableTiming));
    }
    NMF_HIP(hipEventRecord(g.ev_entry, st));
    NMF_HIP(hipStreamWaitEvent(g.copy_stream, g.ev_entry, 0));

    NMF_HIP(launch_transpose(H, k, n, Ht, st));
    int64_t issued = 0;
    for (int s = 0; s <= iters; ++s) {
        if (s < iters) NMF_HIP(launch_fill_f32(Num, n * (int64_t)k, 0.f, st));
        for (size_t b = 0; b < batches.size(); ++b, ++issued) {
            const Batch &bt = batches[b];
            const int64_t rows = bt.r1 - bt.r0, cnt = bt.e1 - bt.e0;
            const int slot = (int)(issued % slots);
            char *base = static_cast<char *>(g.sl_stage) + slot * slot_bytes;
            int64_t *rp = reinterpret_cast<int64_t *>(base);
            int32_t *ci = reinterpret_cast<int32_t *>(base + rp_bytes);
            float *va = reinterpret_cast<float *>(base + rp_bytes + ci_bytes);
            if (issued >= slots) NMF_HIP(hipStreamWaitEvent(g.copy_stream, g.sl_freed[slot], 0));
            NMF_HIP(hipMemcpyAsync(rp, rowptr_host + bt.r0, (size_t)(rows + 1) * sizeof(int64_t),
                                   hipMemcpyHostToDevice, g.copy_stream));
            if (cnt > 0) {
                NMF_HIP(hipMemcpyAsync(ci, colidx_host + bt.e0, (size_t)cnt * sizeof(int32_t),
                                       hipMemcpyHostToDevice, g.copy_stream));
                NMF_HIP(hipMemcpyAsync(va, vals_host + bt.e0, (size_t)cnt * sizeof(float),
                                       hipMemcpyHostToDevice, g.copy_stream));
            }
            NMF_HIP(hipEventRecord(g.sl_copied[slot], g.copy_stream));
            NMF_HIP(hipStreamWaitEvent(st, g.sl_copied[slot], 0));
            NMF_HIP(launch_rebase_i64(rp, rows + 1, bt.e0, rowptr_loc, st));
            float *Wb = W + bt.r0 * k;
            if (s > 0) {
                NMF_HIP(launch_csr_partition(rowptr_loc, rows, kCsrParts, part_r, st));
                NMF_HIP(launch_csr_long_rows(rowptr_loc, rows, long_r, long_n, (unsigned)(max_nnz / kLongRow + 1), st));
                NMF_HIP(launch_aht_csr(rowptr_loc, ci, va, part_r, long_r, long_n, k, Ht, c.gh, Wb, eps, cnt, n, st));
            }
            if (s < iters) {
                NMF_HIP(launch_csc_build(rowptr_loc, ci, va, rows, n, cnt, sorted_cols, payload, sorted_payload,
                                         sort_temp, temp_bytes, colptr, rowidx, cvals, st));
                NMF_HIP(launch_csr_partition(colptr, n, kCsrParts, part_c, st));
                NMF_HIP(launch_csr_long_rows(colptr, n, long_c, long_n + 1, (unsigned)(max_nnz / kLongRow + 1), st));
                NMF_HIP(launch_aht_csr(colptr, rowidx, cvals, part_c, long_c, long_n + 1, k, Wb, nullptr, Num, eps,
                                       cnt, rows, st, true));
            }
            NMF_HIP(hipEventRecord(g.sl_freed[slot], st));
        }
        if (s < iters) {
            NMF_HIP(launch_gram_w_wide(W, m, k, c.gw, c.gwp, st));
            NMF_HIP(launch_row_update(Ht, Num, c.gw, k, n, eps, st));
            NMF_HIP(launch_gram_w_wide(Ht, n, k, c.gh, c.ghp, st));
        }
    }
    NMF_HIP(launch_transpose(Ht, n, k, H, st));
    return NMF_OK;
}

// ---- objective and tolerance-driven run ---------------------------------------

namespace {
// ||A - W H||_F into *out_host; synchronises `st`.  Scratch sits behind the dense plan.
int residual_to_host(const float *A, int64_t m, int64_t n, int k, const float *W, const float *H,
                     double *scratch, double *out_host, hipStream_t st)
{
    const int64_t blocks = (m + 31) / 32;
    NMF_HIP(launch_residual(A, m, n, k, W, H, scratch + 1, scratch, st));
    NMF_HIP(hipMemcpyAsync(out_host, scratch, sizeof(double), hipMemcpyDeviceToHost, st));
    NMF_HIP(hipStreamSynchronize(st));
    (void)blocks;
    return NMF_OK;
}
size_t residual_scratch_bytes(int64_t m, int64_t n) { return align_up(((size_t)residual_partials(m, n) + 1) * sizeof(double)); }
}  // namespace

int nmf_residual_dense(const float *A, int64_t m, int64_t n, int32_t k, const float *W,
                       const float *H, double *residual_host, void *stream)
{
    if (int rc = check_common(A, W, H, m, n, k, 0, 0.f)) return rc;
    if (!residual_host) return fail(NMF_EINVAL, "null pointer%s");
    std::lock_guard<std::mutex> lock(g.mu);
    void *ws = nullptr;
    if (int rc = ensure_workspace(kAlign + residual_scratch_bytes(m, n), &ws)) return rc;
    Carve cv(ws);
    cv.take<unsigned>(64);   // the arrival counters at the head of the workspace stay untouched
    double *scratch = cv.take<double>((size_t)residual_partials(m, n) + 1);
    return residual_to_host(A, m, n, k, W, H, scratch, residual_host, static_cast<hipStream_t>(stream));
}

int nmf_mu_dense_tol(const float *A, int64_t m, int64_t n, int32_t k, float *W, float *H,
                     int32_t max_iters, float eps, double tol, int32_t check_every,
                     int32_t *iters_done_host, double *residual_host, void *stream)
{
    if (int rc = check_common(A, W, H, m, n, k, max_iters, eps)) return rc;
    if (!iters_done_host || !residual_host) return fail(NMF_EINVAL, "null pointer%s");
    if (!(tol >= 0.0) || check_every < 1) return fail(NMF_EINVAL, "tol must be >= 0 and check_every >= 1%s");
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g.mu);
    void *ws = nullptr;
    bool mirrored = false;
    // the residual scratch and the monitor's few doubles ride behind whichever dense plan fits
    const size_t extra = residual_scratch_bytes(m, n) + align_up((size_t)kFinMaxBlocks * sizeof(double)) +
                         align_up(4097 * sizeof(double)) + kAlign;
    const size_t big = dense_bytes(m, n, k, true) + extra, small = dense_bytes(m, n, k, false) + extra;
    if (!rows_plan_first(A, m, n, k) &&
        ((g.ws && g.ws_bytes >= big) || (g.ws_owned && ensure_workspace(big, &ws) == NMF_OK))) {
        mirrored = true;
    } else {
        (void)hipGetLastError();
        if (int rc = ensure_workspace(small, &ws)) return rc;
    }
    ws = g.ws;
    const bool rows_plan = rows_plan_runs(A, m, n, k, mirrored);
    const bool fast = mirrored || rows_plan;   // plans whose W update leaves the objective's terms behind
    const DensePlan p = carve_dense(ws, m, n, k, mirrored);
    Carve cv(static_cast<char *>(ws) + dense_bytes(m, n, k, mirrored));
    double *scratch = cv.take<double>((size_t)residual_partials(m, n) + 1);
    Monitor mon;
    mon.dpart = cv.take<double>(kFinMaxBlocks);
    mon.normA2 = cv.take<double>(4097);
    mon.out = cv.take<double>(1);
    mon.res = scratch;
    mon.last_only = true;
    int done = 0;
    double res = 0.0;
    bool exact = true;       // `res` comes from the tiled evaluation (not from the expansion)
    if (int rc = residual_to_host(A, m, n, k, W, H, scratch, &res, st)) return rc;
    double normA2 = 0.0;
    if (fast && max_iters > 0 && res > tol) {
        NMF_HIP(launch_sumsq(A, m * n, mon.normA2 + 1, mon.normA2, st));
        NMF_HIP(hipMemcpyAsync(&normA2, mon.normA2, sizeof(double), hipMemcpyDeviceToHost, st));
        NMF_HIP(hipStreamSynchronize(st));
    }
    bool have_at = false;
    while (done < max_iters && res > tol) {
        const int chunk = (max_iters - done < check_every) ? max_iters - done : check_every;
        if (int rc = dense_body(A, m, n, k, W, H, chunk, eps, p, st, have_at, nullptr, nullptr, fast ? &mon : nullptr))
            return rc;
        have_at = mirrored;
        done += chunk;
        if (fast) {
            // The objective of the chunk's last iteration from the by-products of its W update
            // (no pass over A); its error is bounded by the fp32 sums of its three terms.  Only
            // when it comes within that bound of the tolerance is the exact value needed.
            double approx = 0.0;
            NMF_HIP(hipMemcpyAsync(&approx, mon.out, sizeof(double), hipMemcpyDeviceToHost, st));
            NMF_HIP(hipStreamSynchronize(st));
            const double slack = 1e-3 * approx + 2e-6 * normA2 / (approx > 1e-300 ? approx : 1e-300);
            if (approx > tol + slack) {
                res = approx;
                exact = false;
                continue;
            }
        }
        if (int rc = residual_to_host(A, m, n, k, W, H, scratch, &res, st)) return rc;
        exact = true;
    }
    if (!exact)
        if (int rc = residual_to_host(A, m, n, k, W, H, scratch, &res, st)) return rc;
    *iters_done_host = done;
    *residual_host = res;
    return NMF_OK;
}

int nmf_mu_dense_monitor(const float *A, int64_t m, int64_t n, int32_t k, float *W, float *H,
                         int32_t iters, float eps, double *objective_host, void *stream)
{
    if (int rc = check_common(A, W, H, m, n, k, iters, eps)) return rc;
    if (!objective_host) return fail(NMF_EINVAL, "null pointer%s");
    if (iters > (1 << 20)) return fail(NMF_EINVAL, "monitored run: iters <= 2^20%s");
    if (iters == 0) return NMF_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g.mu);
    const size_t extra = align_up((size_t)kFinMaxBlocks * sizeof(double)) + align_up(4097 * sizeof(double)) +
                         align_up((size_t)iters * sizeof(double)) + residual_scratch_bytes(m, n);
    const size_t big = dense_bytes(m, n, k, true) + extra, small = dense_bytes(m, n, k, false) + extra;
    void *ws = nullptr;
    bool mirrored = false;
    if (!rows_plan_first(A, m, n, k) &&
        ((g.ws && g.ws_bytes >= big) || (g.ws_owned && ensure_workspace(big, &ws) == NMF_OK))) {
        mirrored = true;
    } else {
        (void)hipGetLastError();
        if (int rc = ensure_workspace(small, &ws)) return rc;
    }
    ws = g.ws;
    const bool rows_plan = rows_plan_runs(A, m, n, k, mirrored);
    const DensePlan p = carve_dense(ws, m, n, k, mirrored);
    Carve cv(static_cast<char *>(ws) + dense_bytes(m, n, k, mirrored));
    Monitor mon;
    mon.dpart = cv.take<double>(kFinMaxBlocks);
    mon.normA2 = cv.take<double>(4097);
    mon.out = cv.take<double>((size_t)iters);
    mon.res = cv.take<double>((size_t)residual_partials(m, n) + 1);
    mon.last_only = false;
    if (mirrored || rows_plan) NMF_HIP(launch_sumsq(A, m * n, mon.normA2 + 1, mon.normA2, st));
    if (int rc = dense_body(A, m, n, k, W, H, iters, eps, p, st, false, nullptr, nullptr, &mon)) return rc;
    NMF_HIP(hipMemcpyAsync(objective_host, mon.out, (size_t)iters * sizeof(double), hipMemcpyDeviceToHost, st));
    NMF_HIP(hipStreamSynchronize(st));
    return NMF_OK;
}

// ---- allocation-free resident dense run --------------------------------------

int nmf_mu_dense_noalloc(const float *A, int64_t m, int64_t n, int32_t k, float *W, float *H,
                         int32_t iters, float eps, void *stream)
{
    if (int rc = check_common(A, W, H, m, n, k, iters, eps)) return rc;
    if (dense_bytes(m, n, k, false) > kScratchBytes)
        return fail(NMF_ENOMEM, "problem needs more than the fixed scratch array of nmf_mu_dense_noalloc "
                                "(see nmf_mu_workspace_bytes kind 4)%s");
    if (iters == 0) return NMF_OK;
    void *ws = nullptr;
    if (int rc = scratch_address(&ws)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The arrival counters at the head of the array must read zero when the first kernel starts;
    // the kernels restore that, but an earlier call may have been cut short.  A fill kernel, not
    // a memset: the call may be under graph capture.
    NMF_HIP(launch_fill_f32(static_cast<float *>(ws), 64, 0.f, st));
    const DensePlan p = carve_dense(ws, m, n, k, false);
    return dense_body(A, m, n, k, W, H, iters, eps, p, st);
}

// ---- single steps ----------------------------------------------------------

int nmf_csr_partition(const int64_t *rowptr, int64_t m, int32_t nparts, int64_t *part, void *stream)
{
    if (!rowptr || !part) return fail(NMF_EINVAL, "null pointer%s");
    if (m < 1 || nparts < 1) return fail(NMF_EINVAL, "bad size%s");
    NMF_HIP(launch_csr_partition(rowptr, m, nparts, part, static_cast<hipStream_t>(stream)));
    return NMF_OK;
}

int nmf_split_planes(const float *X, int64_t rows, int32_t k, uint16_t *planes, void *stream)
{
    if (!X || !planes) return fail(NMF_EINVAL, "null pointer%s");
    if (rows < 1 || k < 1) return fail(NMF_EINVAL, "bad size%s");
    if (!wta_uses_planes(k)) return fail(NMF_EUNSUPPORTED, "piece planes are used for k <= 64 only%s");
    if (reinterpret_cast<uintptr_t>(planes) % 16) return fail(NMF_EINVAL, "planes must be 16-byte aligned%s");
    NMF_HIP(launch_split_planes(X, rows, k, planes, static_cast<hipStream_t>(stream)));
    return NMF_OK;
}

int nmf_csr_to_csc(const int64_t *rowptr, const int32_t *colidx, const float *vals, int64_t m,
                   int64_t n, int64_t nnz, int64_t *colptr, int32_t *rowidx, float *cvals,
                   void *stream)
{
    if (!rowptr || !colptr) return fail(NMF_EINVAL, "null pointer%s");
    if (m < 1 || n < 1 || nnz < 0) return fail(NMF_EINVAL, "bad size%s");
    if (nnz > 0 && (!colidx || !vals || !rowidx || !cvals)) return fail(NMF_EINVAL, "null pointer%s");
    if (nnz >= ((int64_t)1 << 31) || m >= ((int64_t)1 << 31))
        return fail(NMF_EUNSUPPORTED, "CSR path needs nnz < 2^31 and m < 2^31%s");
    return build_csc(rowptr, colidx, vals, m, n, nnz, colptr, rowidx, cvals,
                     static_cast<hipStream_t>(stream));
}

int nmf_gram_w(const float *W, int64_t m, int32_t k, float *G, void *stream)
{
    if (int rc = check_common(W, W, G, m, 1, k, 0, 0.f)) return rc;
    std::lock_guard<std::mutex> lock(g.mu);
    void *ws = nullptr;
    if (int rc = ensure_workspace(common_bytes(k), &ws)) return rc;
    Carve cv(ws);
    const Common c = carve_common(cv, k);
    NMF_HIP(launch_gram_w(W, m, k, G, c.gpart, c.counters, static_cast<hipStream_t>(stream)));
    return NMF_OK;
}

int nmf_wta_dense(const float *A, int64_t m, int64_t n, int32_t k, const float *W, float *P,
                  void *stream)
{
    if (int rc = check_common(A, W, P, m, n, k, 0, 0.f)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g.mu);
    void *ws = nullptr;
    if (int rc = ensure_workspace(dense_bytes(m, n, k, false), &ws)) return rc;
    Carve cv(ws);
    carve_common(cv, k);
    const int splits = wta_splits(m, n, k);
    float *ppart = cv.take<float>((size_t)splits * k * n);
    void *planes = cv.take<char>(planes_bytes(m));
    NMF_HIP(launch_wta_pass(A, m, n, k, W, planes, false, ppart, splits, wta_rows_per_split(m, splits), false, st));
    NMF_HIP(launch_sum_partials(ppart, splits, (int64_t)k * n, P, st));
    return NMF_OK;
}

int nmf_h_update(float *H, const float *P, const float *G, int32_t k, int64_t n, float eps,
                 float *GH, void *stream)
{
    if (int rc = check_common(H, P, G, 1, n, k, 0, eps)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g.mu);
    void *ws = nullptr;
    if (int rc = ensure_workspace(common_bytes(k), &ws)) return rc;
    Carve cv(ws);
    const Common c = carve_common(cv, k);
    NMF_HIP(launch_factor_update(H, nullptr, P, 1, G, nullptr, 0, nullptr, k, n, eps, st));
    if (GH) NMF_HIP(launch_gram_h(H, k, n, GH, c.gpart, c.counters, st));
    return NMF_OK;
}

int nmf_aht_w_update_dense(const float *A, int64_t m, int64_t n, int32_t k, const float *H,
                           const float *GH, float *W, float eps, void *stream)
{
    if (int rc = check_common(A, W, H, m, n, k, 0, eps)) return rc;
    if (!GH) return fail(NMF_EINVAL, "null pointer%s");
    NMF_HIP(launch_aht_pass(A, m, n, k, H, GH, W, eps, static_cast<hipStream_t>(stream)));
    return NMF_OK;
}

}  // extern "C"
