/*
 * nmfmu.h -- C ABI of the MI355X (gfx950) multiplicative-update NMF library.
 *
 * The library runs the Frobenius-norm multiplicative-update (MU) iteration for
 * A ~= W H with W, H >= 0 (paper, section 2.1 and Algorithm 1) in the order of
 * the paper's row-partition algorithm (Algorithm 3) on a single device:
 *
 *     H <- H * (W^T A) / ((W^T W) H + eps)          H update, old H on the right
 *     W <- W * (A H^T) / (W (H H^T) + eps)          W update, uses the NEW H
 *
 * eps is added once, to the finished denominator.  Operands and results are
 * IEEE single precision.  For k <= NMF_MU_MAX_K and 16-byte aligned A the two
 * products over A are formed on the bf16 matrix cores from exact pieces: every
 * float is cut into three bf16 values that add up to it bit for bit, the
 * piece products of a term are accumulated in fp32 (each is exact there; the
 * product of the two lowest pieces, below 2^-30 of the term, is left out), and
 * no matrix accumulator runs over more than 512 terms before it is added, in
 * rounded fp32, to a running total; long sums stay within 3e-7 relative of the
 * float64 result.  Unaligned A and the Gram matrices use the fp32 matrix
 * instruction (fp32 operands, fp32 accumulation).
 *
 * Conventions shared by every entry point
 *   - All matrices are row-major and contiguous: A is m x n (leading dimension
 *     n), W is m x k (ld k), H is k x n (ld n).  Base pointers must be 4-byte
 *     aligned; the fast paths need 16-byte aligned A and H and n % 4 == 0,
 *     anything else takes a slower, equally correct path.
 *   - "device" pointers are HIP device memory of the current device; "host"
 *     pointers are host memory.  The caller owns every buffer; the library
 *     keeps no reference to them after the call's work has finished.
 *   - W and H are read and overwritten in place; after the enqueued work has
 *     completed they hold the factors after `iters` iterations.
 *   - `stream` is a hipStream_t passed as void*; NULL means the null stream.
 *     nmf_mu_dense / nmf_mu_csr / nmf_mu_dense_batched only enqueue work and
 *     return; nmf_mu_ooc also drives internal copy streams and may block the
 *     calling thread while it throttles copies, but does not synchronise the
 *     device; on return all of its work is ordered before anything enqueued
 *     on `stream` afterwards.
 *   - Scratch memory (partial sums, Gram matrices) comes from a per-process
 *     workspace that the library allocates on first use and grows on demand
 *     (growing it synchronises the device), or from a caller-provided block
 *     (nmf_mu_set_workspace).  There is one workspace per process: the calls
 *     of this header hold a lock while they enqueue, so they may be made from
 *     several threads, but work that two of them leave in flight on different
 *     streams at the same time shares the workspace and races.  Run one
 *     problem at a time per process, or order the streams with events.  Only
 *     nmf_mu_dense_noalloc has scratch of its own (shared by its own calls).
 *   - Every function returns a status code and never throws, exits or prints.
 *     Entries of A, W, H are not inspected: negative or non-finite input gives
 *     an undefined (but non-faulting) result.  iters == 0 is a successful
 *     no-op.  Supported rank: 1 <= k <= NMF_MU_MAX_K; nmf_mu_dense, nmf_mu_ooc
 *     and nmf_mu_ooc_hostw go up to NMF_MU_MAX_K_SLICED.
 */
#ifndef NMFMU_H
#define NMFMU_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    NMF_OK = 0,
    NMF_EINVAL = 1,       /* null pointer, non-positive size, bad eps/iters/batch */
    NMF_ENOMEM = 2,       /* workspace or staging buffers do not fit */
    NMF_EHIP = 3,         /* a HIP runtime call failed; see nmf_last_error() */
    NMF_EUNSUPPORTED = 4  /* rank above what the entry point supports */
};

#define NMF_MU_MAX_K 64           /* ranks served by the fused kernels */
#define NMF_MU_MAX_K_SLICED 1024  /* ranks served 64 factor columns at a time (see nmf_mu_dense) */

/* Static, human-readable name of a status code. */
const char *nmf_status_string(int status);

/* Detail of the last failure on the calling thread (thread-local storage,
 * valid until the next failing call on that thread); "" if none. */
const char *nmf_last_error(void);

/*
 * Resident dense MU (Algorithm 3 on one unit).
 *   A      device, m x n, read-only
 *   W, H   device, in/out
 *   iters  >= 0;  eps >= 0 and finite
 * Asynchronous on `stream`.  Three plans, chosen per call; they give the same
 * iteration and differ in low-order bits.  Row plan (16-byte aligned A,
 * n % 4 == 0, n < 2^24, and m >= 12288 with n >= 512, or m n <= 2^22): both products stream
 * the row-major A, the W update is fused into the A H^T pass; workspace kind 4.
 * It comes first for k <= 32.  Mirrored plan (33 <= k <= 64, and shapes the
 * row plan does not serve, if the workspace can hold a second copy of A): A is
 * transposed once per call and A^T is streamed for the A H^T product;
 * workspace kind 0.  Without room for that copy: the row plan for
 * 33 <= k <= 64 where it applies (its A H^T pass is about a fifth slower than
 * the mirrored one), else the small plan, a direct A H^T kernel on A (lanes
 * down the rows: slower); workspace kind 4.  An A whose base is not 16-byte
 * aligned or whose n is not a multiple of 4 is copied once per call, with H,
 * into aligned arrays of n rounded up to 4 columns (zero columns change no
 * result) when the workspace can hold them (about the size of kind 0) and eps
 * is a normal positive float, and the row plan runs on the copies.
 * Ranks NMF_MU_MAX_K < k <= NMF_MU_MAX_K_SLICED run the same iteration with every
 * product written as F^T X (a reduction over the rows of two row-major
 * matrices) and computed 64 factor columns of F at a time by the k <= 64 pass
 * kernel: W^T A, W^T W, (W^T W) H, and the same three on the transposes A^T,
 * H^T, W^T for the W update, followed by the element-wise update.  A is read
 * ceil(k / 64) times per product; the workspace holds A^T, W^T, H^T and two
 * k x max(m, n) arrays (nmf_mu_workspace_bytes kind 5), else NMF_ENOMEM.
 */
int nmf_mu_dense(const float *A, int64_t m, int64_t n, int32_t k,
                 float *W, float *H, int32_t iters, float eps, void *stream);

/*
 * nmf_mu_dense for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and result as nmf_mu_dense on its small plan (the direct A H^T
 * kernel; no transposed copy of A), k <= NMF_MU_MAX_K.  The scratch memory
 * (row-split partial sums, operand planes of W, Gram scratch) is a fixed array
 * of NMF_MU_NOALLOC_SCRATCH_BYTES in the library's device image instead of
 * allocated memory; every device the library runs on holds one copy until the
 * process ends.  A problem whose nmf_mu_workspace_bytes(kind 4) exceeds that
 * size is rejected with NMF_ENOMEM (32768 x 16384 with k = 32 needs 28.4 MiB).
 * The call itself makes no hipMalloc / hipFree and no allocating library call;
 * the first call on a device looks up the array's device address
 * (hipGetSymbolAddress), so make that call once outside a graph capture.
 * All calls on one device share the array: calls that overlap in time on one
 * device (two streams, two threads) race, the caller serialises them.  The
 * array is independent of the workspace of the other entry points.
 * Asynchronous on `stream`.
 */
#define NMF_MU_NOALLOC_SCRATCH_BYTES (32u << 20)
int nmf_mu_dense_noalloc(const float *A, int64_t m, int64_t n, int32_t k,
                         float *W, float *H, int32_t iters, float eps, void *stream);

/*
 * Objective of the factorisation, ||A - W H||_F (section 2.1; Algorithm 1
 * evaluates it after every iteration).  W H is formed 32 rows at a time and
 * never stored (the row tiling of section 3.2).  All of A, W, H on the device;
 * the result is written to HOST memory after `stream` has been synchronised.
 */
int nmf_residual_dense(const float *A, int64_t m, int64_t n, int32_t k,
                       const float *W, const float *H, double *residual_host, void *stream);

/*
 * Algorithm 1 with its stopping rule read as: iterate until ||A - W H||_F <= tol
 * or max_iters iterations have run.  The objective is evaluated before the first
 * iteration and then after every `check_every` iterations (each evaluation is
 * one more pass over A and a stream synchronisation; with the fast plan the
 * checks after iterations first use the expansion of nmf_mu_dense_monitor, which
 * costs no pass, and fall back to the exact evaluation only when that value is
 * within its error bound of tol, so the stopping decision is the exact one).  On return
 * *iters_done_host iterations have been applied to W, H and *residual_host is
 * the objective of the returned factors.  Blocking.
 */
int nmf_mu_dense_tol(const float *A, int64_t m, int64_t n, int32_t k, float *W, float *H,
                     int32_t max_iters, float eps, double tol, int32_t check_every,
                     int32_t *iters_done_host, double *residual_host, void *stream);

/*
 * nmf_mu_dense with the objective ||A - W H||_F reported after every iteration
 * (Algorithm 1 evaluates it every iteration), at almost no cost: the norm is
 * expanded as ||A||^2 - 2 <A H^T, W> + <H H^T, W^T W> and all three terms are
 * by-products of the W update (its numerator against the new W, and the two
 * Gram matrices); ||A||^2 is computed once per call.  The products are fp32
 * sums, so the value carries an absolute error of about 2e-7 ||A||^2 / f: exact
 * to 1e-4 relative while f >= 0.05 ||A||, a few percent at f = 0.005 ||A||;
 * nmf_residual_dense gives the exact value (one more pass over A).  When the
 * fast plan's workspace cannot be had, every value is the exact tiled one.
 * objective_host: HOST memory, iters doubles.  Blocking.  W, H as nmf_mu_dense
 * (bit-identical result).
 */
int nmf_mu_dense_monitor(const float *A, int64_t m, int64_t n, int32_t k, float *W, float *H,
                         int32_t iters, float eps, double *objective_host, void *stream);

/*
 * Resident sparse MU: the same iteration with A given in CSR (section 2.3
 * names the three CSR arrays: values, column indices, row pointers).
 *   rowptr  device, int64[m + 1], non-decreasing, rowptr[0] = 0, rowptr[m] = nnz
 *   colidx  device, int32[nnz], each in [0, n); order within a row is free and
 *           repeated (row, column) pairs add up
 *   vals    device, float[nnz]
 * The CSR arrays are read-only.  The library builds, once per call and in its
 * workspace, a column-ordered copy of the matrix (8 bytes per stored entry plus
 * 8 (n + 1) bytes) and a transposed copy of H; both products then gather rows
 * of a factor per stored entry, without atomics, so results are reproducible
 * from run to run.  Needs nnz < 2^31 and m < 2^31.  The build is a stable sort
 * by column on `stream` whose scratch (about 24 bytes per stored entry) is part
 * of the workspace; the whole call only enqueues work and returns.  The
 * structure is not validated (that would need the device's answer): entry
 * ranges and column indices are clamped to the arrays' bounds where they are
 * used, so malformed row pointers or indices give a meaningless result but no
 * out-of-range access.
 */
int nmf_mu_csr(const int64_t *rowptr, const int32_t *colidx, const float *vals,
               int64_t m, int64_t n, int64_t nnz, int32_t k,
               float *W, float *H, int32_t iters, float eps, void *stream);

/*
 * nmf_mu_csr with the objective ||A - W H||_F reported after every iteration
 * (Algorithm 1 evaluates it every iteration; for a sparse A the norm runs over
 * all m n entries, zeros included).  It is taken from the expansion
 * ||A||^2 - 2 <A H^T, W> + <H H^T, W^T W>, the only form that does not touch the
 * m n entries of W H: <A H^T, W> is summed in double inside the W update from the
 * gathered row sums against the new W, H H^T is the matrix the update used,
 * W^T W of the new W costs one more read of W per iteration, ||A||^2 once per
 * call (the squared stored values, plus the cross terms of repeated (row,
 * column) pairs, which stand for their sum).  Absolute error
 * about 2e-7 ||A||^2 / f as for nmf_mu_dense_monitor.  objective_host: HOST
 * memory, iters doubles.  Blocking.  W, H as nmf_mu_csr (bit-identical result).
 * The workspace is nmf_mu_workspace_bytes(kind 1) plus 8 (iters + 73986) bytes,
 * rounded up to 256-byte pieces.
 */
int nmf_mu_csr_monitor(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                       int64_t m, int64_t n, int64_t nnz, int32_t k,
                       float *W, float *H, int32_t iters, float eps,
                       double *objective_host, void *stream);

/*
 * Algorithm 1's loop on a CSR matrix, read as for nmf_mu_dense_tol: iterate until
 * ||A - W H||_F <= tol or max_iters iterations have run; the objective is evaluated
 * before the first iteration (one pass over the stored entries that updates
 * nothing) and after every `check_every` iterations (the expansion of
 * nmf_mu_csr_monitor: no extra pass over A, one stream synchronisation).  There is
 * no cheaper exact form for a sparse A, so the stopping decision carries that
 * expansion's error (about 2e-7 ||A||^2 / f absolute).  On return
 * *iters_done_host iterations have been applied to W, H and *residual_host is the
 * objective of the returned factors.  Blocking.
 */
int nmf_mu_csr_tol(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                   int64_t m, int64_t n, int64_t nnz, int32_t k,
                   float *W, float *H, int32_t max_iters, float eps, double tol,
                   int32_t check_every, int32_t *iters_done_host, double *residual_host,
                   void *stream);

/*
 * Out-of-memory dense MU: A stays in host memory and is streamed to the device
 * in batches of `batch_rows` rows (co-linear batching, Algorithm 5; W and H
 * stay resident on the device).  Each sweep uploads A once: a batch first gets
 * its W rows updated with the current H, then contributes W_b^T A_b and
 * W_b^T W_b of the updated rows to the next H update.  iters iterations take
 * iters + 1 sweeps and give the same sequence H1, W1, H2, W2, ... as
 * nmf_mu_dense.
 *   A_host               host, m x n; pinned memory is needed for copies to
 *                        overlap with compute (pageable memory works, slowly)
 *   batch_rows           >= 1, need not divide m
 *   device_budget_bytes  upper bound on device memory used to stage A; the
 *                        library uses min(3, what fits) staging slots of
 *                        batch_rows x n floats and fails with NMF_ENOMEM if not
 *                        even one fits
 * Ranks above NMF_MU_MAX_K take the pipeline of nmf_mu_ooc_hostw with W kept on the device.
 */
int nmf_mu_ooc(const float *A_host, int64_t m, int64_t n, int32_t k,
               float *W, float *H, int32_t iters, float eps,
               int64_t batch_rows, int64_t device_budget_bytes, void *stream);

/*
 * nmf_mu_ooc with the objective ||A - W H||_F reported after every iteration
 * (Algorithm 1 evaluates it every iteration), without another pass over A: the
 * expansion ||A||^2 - 2 <A H^T, W> + <H H^T, W^T W> of nmf_mu_dense_monitor, with
 * <A H^T, W> collected in double by the W updates of a sweep's batches, W^T W of
 * the W they leave (one more Gram after the last sweep), H H^T of the H they
 * used, and ||A||^2 summed batch by batch during the first sweep (one more read
 * of each staged batch, on the device).  Absolute error about 2e-7 ||A||^2 / f.
 * k <= NMF_MU_MAX_K.  objective_host: HOST memory, iters doubles.  Blocking.
 * W, H as nmf_mu_ooc (bit-identical result).  The workspace is
 * nmf_mu_workspace_bytes(kind 2) plus 8 bytes for each of: at most
 * ceil(batch_rows / 64) per batch, one per batch, 4097, and iters (each group
 * rounded up to 256 bytes).
 */
int nmf_mu_ooc_monitor(const float *A_host, int64_t m, int64_t n, int32_t k,
                       float *W, float *H, int32_t iters, float eps,
                       int64_t batch_rows, int64_t device_budget_bytes,
                       double *objective_host, void *stream);

/*
 * Out-of-memory dense MU with W in host memory as well (Algorithm 5 as printed:
 * per batch, W_b and A_b go to the device, W_b is updated and copied back, and
 * W_b^T A_b, W_b^T W_b are accumulated for the H update; section 4.4 is the
 * benchmark).  Same sweep order as nmf_mu_ooc.  Any rank up to
 * NMF_MU_MAX_K_SLICED; all products go through the rank-sliced engine described
 * at nmf_mu_dense, the A H^T of a batch on a transposed copy of the batch.
 *   A_host, W_host  host (pinned for overlap), m x n and m x k; W_host is
 *                   updated in place and complete once `stream` has been
 *                   synchronised
 *   H               device, k x n, in/out
 *   slots           1 .. 16 staging slots of (batch_rows x n + batch_rows x k)
 *                   floats: the stand-in for the paper's stream-queue size q_s;
 *                   uploads run `slots` - 1 batches ahead of the compute
 *                   stream, downloads of W_b on a third stream
 *   device_bytes_host  optional (host): receives the device memory the call
 *                   uses (workspace + staging), for the O(p n q_s) memory model
 */
int nmf_mu_ooc_hostw(const float *A_host, float *W_host, int64_t m, int64_t n, int32_t k,
                     float *H, int32_t iters, float eps, int64_t batch_rows, int32_t slots,
                     void *stream, size_t *device_bytes_host);

/*
 * Out-of-memory CSR MU (sections 2.3 and 3.2 together: the sparse matrix does
 * not fit the device): the CSR arrays stay in host memory (pinned for overlap)
 * and are streamed every sweep in batches of whole rows holding about
 * `batch_nnz` stored entries each (a longer single row is a batch by itself);
 * W, H and the k x k matrices stay on the device.  Sweep order and result as
 * nmf_mu_ooc / nmf_mu_csr.  Per batch: W update of its rows by the row gather;
 * a column-ordered copy of the batch (device sort) and the column gather, which
 * adds the batch's share of W^T A to an n x k numerator; after the sweep the H
 * update from that numerator.  k <= NMF_MU_MAX_K, m < 2^31, a batch < 2^31 entries.
 *   device_budget_bytes  bound on the staging memory: min(3, what fits) slots
 *                        of one batch (12 bytes per entry + 8 per row)
 * The workspace (about 40 bytes per entry of the largest batch + 8 n k bytes)
 * is sized inside the call; a caller-provided workspace must be large enough.
 * Reads rowptr_host on the calling thread to form the batches.
 */
int nmf_mu_csr_ooc(const int64_t *rowptr_host, const int32_t *colidx_host, const float *vals_host,
                   int64_t m, int64_t n, int64_t nnz, int32_t k, float *W, float *H,
                   int32_t iters, float eps, int64_t batch_nnz, int64_t device_budget_bytes,
                   void *stream);

/*
 * Ensemble of independent resident dense runs of one shape (the perturbed
 * copies times rank sweep that model selection needs, sections 1 and 4.5).
 * Run r factorises A[r] (m x n) with rank k[r] into W[r] (m x k[r]) and H[r]
 * (k[r] x n).  A[r] may be the same pointer for several runs; W[r], H[r] must
 * not overlap.  The pointer arrays and k live in HOST memory and are read
 * before the call returns; what they point to is device memory.
 * Consecutive runs that name the same A are stacked while their ranks sum to at
 * most NMF_MU_MAX_K: the two passes over A then serve the whole stack at once
 * (order the runs by A to benefit).  Results per run equal a single run's up
 * to rounding order.
 */
int nmf_mu_dense_batched(int32_t n_runs, const float *const *A, int64_t m, int64_t n,
                         const int32_t *k, float *const *W, float *const *H,
                         int32_t iters, float eps, void *stream);

/*
 * Workspace the given problem needs, in bytes.  kind: 0 dense (mirrored plan:
 * the library keeps a transposed copy of A, so this is about m*n*4 bytes plus
 * the partial sums), 4 dense (row plan and small plan: partial sums and operand
 * planes only), 1 csr (includes the scratch of the one-time sort, about 24 bytes
 * per stored entry), 2 ooc (excluding the
 * staging slots), 3 batched (enough for any mix of ranks; k is only checked),
 * 5 dense with k > NMF_MU_MAX_K (rank-sliced), 6 the rank-sliced out-of-memory
 * pipeline (nmf_mu_ooc_hostw, and nmf_mu_ooc above NMF_MU_MAX_K; excluding the
 * staging slots).  0 on invalid arguments.
 */
size_t nmf_mu_workspace_bytes(int kind, int64_t m, int64_t n, int64_t nnz,
                              int32_t k, int64_t batch_rows);

/*
 * Hand the library a device block to use as its workspace instead of its own
 * allocation (dev_ptr == NULL or bytes == 0 returns to library-owned memory).
 * The block must stay valid until replaced; 256-byte alignment required.
 */
int nmf_mu_set_workspace(void *dev_ptr, size_t bytes);

/* Free library-owned workspace and staging memory (synchronises the device). */
int nmf_mu_release(void);

#ifdef __cplusplus
}
#endif
#endif /* NMFMU_H */
