/*
 * nmfmu_test.h -- entry points of libnmfmu that exist for its tests and for
 * profiling: single steps of the iteration, the derived data structures of the
 * sparse path, the operand encoding of the passes, and a timed run.  Same
 * conventions as nmfmu.h (extern "C", status codes, device pointers, stream);
 * not part of the library's contract with applications.
 */
#ifndef NMFMU_TEST_H
#define NMFMU_TEST_H

#include "nmfmu.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * nmf_mu_dense with timing: the same launches on `stream`, with a HIP event
 * recorded between them; synchronises `stream` before returning.  On return
 * kernel_ms[0..5] (HOST memory, 9 floats) hold the average milliseconds per
 * launch of the kernels of one iteration, in launch order:
 *   [0] W^T W   [1] W^T A pass   [2] H update   [3] H H^T
 *   [4] A H^T pass (on the mirrored copy A^T, or the direct kernel with the W
 *       update fused)   [5] W update (0 for the direct kernel)
 * and kernel_ms[6] names the plan that ran: 2 the row plan (k <= 32, aligned A:
 * both passes stream the row-major A, [0], [3] and [5] are 0 because the Gram
 * matrices and the W update are by-products of the other three kernels), 1 the
 * mirrored plan (see nmf_mu_workspace_bytes), 0 the small plan.  kernel_ms[7] and
 * [8]: milliseconds per launch of the W^T A pass and (plans 1 and 2, else 0) of
 * the A H^T pass, from 20 launches back to back between two events after the
 * run, i.e. without the event commands that surround every kernel in [0..5].
 * 1 <= iters <= 4096.
 */
int nmf_mu_dense_profile(const float *A, int64_t m, int64_t n, int32_t k,
                         float *W, float *H, int32_t iters, float eps, void *stream,
                         float *kernel_ms);

/* The row-balanced work partition of the sparse kernels: part[0 .. nparts]
 * (device, int64) with part[w] = first row r such that
 * rowptr[r] + 8 r >= w * ceil((rowptr[m] + 8 m) / nparts) and part[nparts] = m;
 * wavefront w of a sparse update works on rows [part[w], part[w + 1]).  The
 * library uses nparts = 16384 and sends rows with more than 16384 stored
 * entries to a whole workgroup instead.  Asynchronous on `stream`. */
int nmf_csr_partition(const int64_t *rowptr, int64_t m, int32_t nparts, int64_t *part, void *stream);

/* The operand encoding of the W^T A pass for k <= 64.  The products of
 * Algorithms 2-5 (W^T A, and A H^T as the same product on the transposes) are
 * formed on the bf16 matrix cores from exact pieces: a float x is cut into
 * x = h + m + l, h = x with its significand truncated to 8 bits, m = x - h
 * truncated likewise, l = x - h - m (each piece is a bf16, the sum is x bit
 * for bit for |x| >= 2^-110); the piece products of a term, all but l l, are
 * accumulated in fp32.  This call writes the pieces of X (rows x k, row-major,
 * device, k <= 64) as the kernels read them, with KP = 32 factor slots per
 * row group for k <= 32 and KP = 64 above: for row group g = row / 8, piece
 * p (0: h, 1: m, 2: l) and factor c < KP, the eight bf16 of rows 8g .. 8g+7 at
 * planes[((g * 3 + p) * KP + c) * 8 ..]; rows >= `rows` and factors >= k are
 * zero.  `planes`: device, ceil(rows / 8) * 24 * KP uint16.  Asynchronous. */
int nmf_split_planes(const float *X, int64_t rows, int32_t k, uint16_t *planes, void *stream);

/* Column-ordered copy of a CSR matrix, the structure nmf_mu_csr derives for its
 * W^T A product: colptr int64[n + 1], rowidx int32[nnz], cvals float[nnz] (all
 * device, caller-allocated).  Entries of a column keep the order in which the
 * CSR arrays store them (stable).  Synchronises `stream`. */
int nmf_csr_to_csc(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                   int64_t m, int64_t n, int64_t nnz,
                   int64_t *colptr, int32_t *rowidx, float *cvals, void *stream);

/* G (k x k, ld k) = W^T W.  Algorithm 3, formation of WTW. */
int nmf_gram_w(const float *W, int64_t m, int32_t k, float *G, void *stream);

/* P (k x n, ld n) = W^T A for dense A.  Algorithm 3, formation of WTA. */
int nmf_wta_dense(const float *A, int64_t m, int64_t n, int32_t k,
                  const float *W, float *P, void *stream);

/* H <- H * P / (G H + eps) in place and GH (k x k) = H H^T of the new H.
 * Algorithm 3, the H-update line and the formation of HHT.  GH may be NULL. */
int nmf_h_update(float *H, const float *P, const float *G, int32_t k, int64_t n,
                 float eps, float *GH, void *stream);

/* W <- W * (A H^T) / (W GH + eps) in place, A dense.  Algorithm 3, formation
 * of AHT and WHHT and the W-update line, fused. */
int nmf_aht_w_update_dense(const float *A, int64_t m, int64_t n, int32_t k,
                           const float *H, const float *GH, float *W,
                           float eps, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NMFMU_TEST_H */
