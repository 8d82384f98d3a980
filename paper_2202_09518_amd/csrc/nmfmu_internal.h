// Internal declarations shared by the HIP translation units of libnmfmu.
// Not part of the public ABI (that is include/nmfmu.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace nmfmu {

// ---- launch geometry shared between the host scheduler and the kernels ----

constexpr int kWtaWaves = 4;        // waves per workgroup in the W^T A pass
constexpr int kWtaCols = 128;       // columns of A per workgroup in that pass
constexpr int kAhtWaves = 8;        // waves per workgroup in the A H^T pass
constexpr int kAhtRowTiles = 2;     // 32-row tiles per workgroup in that pass
constexpr int kGramMaxBlocks = 64;  // partial Gram matrices before the final sum
constexpr int kFinMaxBlocks = 256;  // finisher blocks when they also emit Gram partials
constexpr int kGramGroup = 16;      // sets of Gram tiles added up per group by the following pass
constexpr int kMaxKTiles = 2;       // 32-wide rank tiles: k <= 64

inline int k_tiles(int k) { return (k + 31) / 32; }

// Which independent run a factor index belongs to when several runs on the same A
// are stacked side by side (id[c] for c < k); passed to kernels by value.
struct BlockMap {
    int on;
    unsigned char id[64];
};

// Row split of the W^T A pass: number of partial k x n results, rows in each.
int wta_splits(int64_t rows, int64_t n, int k);
// Largest split count of any rank up to k on these dimensions (workspace sizing).
int wta_splits_bound(int64_t rows, int64_t n, int k);
int64_t wta_rows_per_split(int64_t rows, int splits);

// ---- kernel launchers (all asynchronous on `st`; return hipGetLastError) ----

// G (k x k, ld k) = X^T X for X rows x k (row-major, ld k).
hipError_t launch_gram_w(const float *X, int64_t rows, int k, float *G, float *gpart,
                         unsigned *counters, hipStream_t st);
// The same for a long factor (millions of rows): up to kFinMaxBlocks blocks write partial tiles
// (tiles: kFinMaxBlocks sets), summed by launch_gram_sum.
hipError_t launch_gram_w_wide(const float *X, int64_t rows, int k, float *G, float *tiles, hipStream_t st);
// G (k x k, ld k) = X X^T for X k x cols (row-major, ld cols).
hipError_t launch_gram_h(const float *X, int k, int64_t cols, float *G, float *gpart,
                         unsigned *counters, hipStream_t st);
// Ranks whose W^T A pass reads its factor as bf16 piece planes (planes_bytes(rows) bytes,
// written by launch_split_planes from the rows x k factor) instead of the floats.
inline bool wta_uses_planes(int k) { return k <= 64; }
size_t planes_bytes(int64_t rows);
// Largest rank for which launch_wta_pass on this A (n columns) reads only the planes, never
// the float factor W (which may then be null): 64 for aligned A with n % 4 == 0, else 32.
int wta_planes_only_width(const float *A, int64_t n);
hipError_t launch_split_planes(const float *X, int64_t rows, int k, void *planes, hipStream_t st);
// The same for columns c0 .. c0 + kc - 1 (kc <= 64; 32 factor slots per row group up to kc = 32, else 64)
// of X with leading dimension ld.
hipError_t launch_split_planes_slice(const float *X, int64_t rows, int64_t ld, int64_t c0, int kc,
                                     void *planes, hipStream_t st);
// ppart[s] (+)= W[r0_s:r1_s]^T A[r0_s:r1_s] for each row split s (k x n each).  `planes`:
// scratch of planes_bytes(rows) bytes (unused unless wta_uses_planes(k)); with planes_ready it
// already holds the planes of W, otherwise they are produced first.
hipError_t launch_wta_pass(const float *A, int64_t rows, int64_t n, int k, const float *W,
                           void *planes, bool planes_ready, float *ppart, int splits,
                           int64_t rows_per_split, bool accumulate, hipStream_t st,
                           const float *gtiles = nullptr, int nsets = 0, float *gsum = nullptr);
// gtiles (optional): nsets sets of partial Gram tiles for rank k that the first workgroups of
// the pass add up in groups of kGramGroup into gsum (gram_groups(nsets) sets).
inline int gram_groups(int nsets) { return (nsets + kGramGroup - 1) / kGramGroup; }
// Ranks above 64, all ceil(k / 64) slices of 64 factors in one launch each: planes of every slice of X
// (rows x k; slice z at planes + z * planes_bytes(rows)), the pass over A for every slice (aligned A,
// n % 4 == 0; partials of slice z at ppart + z * splits * 64 * n, packed for that slice's width), and
// P (k x cols) (+)= the sums over the splits.  The slices of one tile of A run side by side, so A is
// fetched from HBM about once per product.
hipError_t launch_split_planes_slices(const float *X, int64_t rows, int k, void *planes, hipStream_t st);
hipError_t launch_wta_pass_slices(const float *A, int64_t rows, int64_t n, int k, const void *planes, float *ppart,
                                  int splits, int64_t rps, hipStream_t st);
hipError_t launch_sum_partials_slices(const float *ppart, int splits, int k, int64_t cols, float *P, hipStream_t st,
                                      bool accumulate = false);
// P[e] (+)= sum_s ppart[s][e], e < count.
hipError_t launch_sum_partials(const float *ppart, int splits, int64_t count, float *P,
                               hipStream_t st, bool accumulate = false);
// X[e] <- X[e] * P[e] / (D[e] + eps), e < count.
hipError_t launch_mu_apply(float *X, const float *P, const float *D, float eps, int64_t count,
                           hipStream_t st);
// X (k x len) <- X * (sum_s part[s]) / (G X + eps), in place.  G is given complete (Gfull, ld k)
// or as nbin partial tiles (gin).  Optional: Xt (len x k) = new X^T; gout = partial Gram tiles
// of the new X, one set per block (factor_update_blocks(len) blocks); planes = the bf16 piece
// planes of the new X^T (planes_bytes(len) bytes; written only if wta_uses_planes(k)).
hipError_t launch_factor_update(float *X, float *Xt, const float *part, int splits,
                                const float *Gfull, const float *gin, int nbin, float *gout, int k,
                                int64_t len, float eps, hipStream_t st,
                                const BlockMap *map = nullptr, void *planes = nullptr,
                                double *dpart = nullptr);
// dpart (with an updating launch): per block, the sum of numerator x new value over its entries
// (factor_update_blocks(len) doubles when gout is given, else one per 64 columns).
// out[0] = sum of squares of X[0 .. count) in double; partial: 4096 doubles of scratch.
hipError_t launch_sumsq(const float *X, int64_t count, double *partial, double *out, hipStream_t st);
// out[0] = sqrt(max(0, normA2[0] - 2 sum(dpart[0 .. nb)) + <GW, GH>)).
hipError_t launch_objective(const double *dpart, int nb, const float *GW, const float *GH, int k,
                            const double *normA2, double *out, hipStream_t st);
int factor_update_blocks(int64_t len);
// G (k x k, ld k) = sum of nb sets of partial tiles.
hipError_t launch_gram_sum(const float *gpart, int nb, int k, float *G, hipStream_t st);
// Blocks (= partial tile sets) launch_gram_w uses for `rows` rows; with G == nullptr it only
// writes the partial tiles to gpart.
int gram_w_blocks(int64_t rows);
// W <- W * (A H^T) / (W GH + eps), in place, for `rows` rows of A and W.
// dpart (aht_pass_blocks(rows) doubles): per workgroup, the sum of (A H^T) x new W over its rows.
hipError_t launch_aht_pass(const float *A, int64_t rows, int64_t n, int k, const float *H,
                           const float *GH, float *W, float eps, hipStream_t st, double *dpart = nullptr);
int64_t aht_pass_blocks(int64_t rows);
// The same update for k <= 64 as one streaming pass over the row-major A (coalesced loads turned
// through LDS, exact-piece products): planesH = piece planes of H^T (what launch_factor_update
// writes for X = H), GH = H H^T (k x k).  Also written: the piece planes of the new W (planesW),
// aht_rows_blocks(rows, k) tile sets of W^T W (gout) and dpart as above (aht_rows_blocks(rows, k)
// doubles).  gram_only: no pass and no update, only planesW and gout of W as it is.  dry: the
// pass and the update without the stores to W and planesW (timing runs).  aht_rows_can: the
// operands this kernel takes; aht_rows_ok: and a shape on which it fills the chip.
bool aht_rows_can(const float *A, int64_t n, int k);
bool aht_rows_ok(const float *A, int64_t m, int64_t n, int k);
int aht_rows_blocks(int64_t rows, int k);
hipError_t launch_aht_rows(const float *A, int64_t rows, int64_t n, int k, const void *planesH,
                           const float *GH, float *W, void *planesW, float *gout, float eps, hipStream_t st,
                           bool gram_only = false, const BlockMap *map = nullptr, double *dpart = nullptr,
                           bool dry = false);
// out[0] = sum of in[0 .. count), added in a fixed order (strided per thread, then the threads in order).
hipError_t launch_sum_f64(const double *in, int64_t count, double *out, hipStream_t st);

// out[0] = ||A - W H||_F; partial: residual_partials(m, n) doubles of scratch.
int64_t residual_partials(int64_t m, int64_t n);
hipError_t launch_residual(const float *A, int64_t m, int64_t n, int k, const float *W,
                           const float *H, double *partial, double *out, hipStream_t st);

// ---- CSR (everything in terms of Ht = H^T, n x k) ----
// X[i][:] <- X[i][:] * (sum over the stored entries (i, j, a) of a * T[j][:]) / (X[i][:] G + eps)
// for i < rows.  W update: (rowptr, colidx, vals) = CSR of A, T = Ht, G = H H^T, X = W.
// H update: the CSC arrays of A, T = W, G = W^T W, X = Ht.
constexpr int kCsrParts = 16384;      // row ranges (= wavefronts) of a sparse update launch
constexpr int64_t kRowCost = 8;       // work of a row besides its entries, in entries
constexpr int64_t kLongRow = 16384;   // rows with more entries go to a whole workgroup
constexpr int kCsrLongBlocks = 256;   // workgroups of the long-row kernel
constexpr int kCsrDparts = kCsrParts / 4 + kCsrLongBlocks;
// part[0 .. nparts]: row ranges of equal work; part[w] = first row r with
// rowptr[r] + kRowCost * r >= w * ceil((rowptr[m] + kRowCost * m) / nparts), part[nparts] = m.
hipError_t launch_csr_partition(const int64_t *rowptr, int64_t m, int nparts, int64_t *part,
                                hipStream_t st);
// list[0 .. min(*count, cap)): the rows with more than kLongRow entries (cap = nnz / kLongRow + 1 slots).
hipError_t launch_csr_long_rows(const int64_t *rowptr, int64_t m, int32_t *list, unsigned *count,
                                unsigned cap, hipStream_t st);
hipError_t launch_aht_csr(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                          const int64_t *part, const int32_t *long_list, const unsigned *long_count,
                          int k, const float *Ht, const float *GH, float *W, float eps, int64_t nnz, int64_t trows,
                          hipStream_t st, bool accumulate = false, double *dpart = nullptr, bool dry = false);
// nnz, trows: lengths of the entry arrays and of the table Ht (rows); row pointers and column
// indices beyond them are pulled to the edge, so that malformed input cannot cause a stray access.
// accumulate: X[i][:] += (gathered sum) instead of the update (GH unused).
// dpart (updating launch only; kCsrDparts doubles): per workgroup of the two kernels, the sum of
// gathered sum x new value over its rows, i.e. <A H^T, W_new> in pieces (objective monitor).
// dry (needs dpart): W is left alone and dpart gets <A H^T, W> of the factors as they are.
// X[i][:] <- X[i][:] * Num[i][:] / (X[i][:] G + eps), i < rows (X, Num rows x k).
hipError_t launch_row_update(float *X, const float *Num, const float *G, int k, int64_t rows, float eps,
                             hipStream_t st);
// out[i] = in[i] - base, i < count.
hipError_t launch_rebase_i64(const int64_t *in, int64_t count, int64_t base, int64_t *out, hipStream_t st);
hipError_t launch_fill_f32(float *p, int64_t count, float v, hipStream_t st);
// Column-ordered copy (colptr int64[n+1], rowidx int32[nnz], cvals float[nnz]) of a CSR matrix
// by a stable sort on the column index.  Scratch: sorted_cols int32[nnz], payload and
// sorted_payload uint64[nnz], sort_temp of csc_sort_temp_bytes(nnz, n) bytes.
// nnz < 2^31, m < 2^31.
size_t csc_sort_temp_bytes(int64_t nnz, int64_t n);
hipError_t launch_csc_build(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                            int64_t m, int64_t n, int64_t nnz, int32_t *sorted_cols,
                            uint64_t *payload, uint64_t *sorted_payload, void *sort_temp,
                            size_t sort_temp_bytes, int64_t *colptr, int32_t *rowidx, float *cvals,
                            hipStream_t st, double *dup_part = nullptr);
// dup_part (csc_finish_blocks(nnz) doubles, at least one): their sum is what repeated (row, column)
// pairs add to the squared Frobenius norm of the matrix beyond the sum of the squared stored values.
int csc_finish_blocks(int64_t nnz);
// dst (rows x ld_dst) = the first `cols` columns of src (rows x ld_src); the columns of dst from
// `cols` on are set to zero.  Any alignment.
hipError_t launch_pad_copy(const float *src, int64_t ld_src, float *dst, int64_t ld_dst, int64_t rows, int64_t cols,
                           hipStream_t st);
// out (cols x rows) = in^T.
hipError_t launch_transpose(const float *in, int64_t rows, int64_t cols, float *out, hipStream_t st);

}  // namespace nmfmu
