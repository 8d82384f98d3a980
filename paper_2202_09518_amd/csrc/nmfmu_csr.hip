// CSR kernels of the multiplicative-update iteration for gfx950 (MI355X).
//
// With A in CSR (paper, section 2.3: values, column indices, row pointers) the
// two products over A become sums over stored entries.  Both are run as
// gathers against a row-major factor table, so that one stored entry touches
// one contiguous run of k floats and no atomics are needed:
//   A H^T : Q[i][:]  = sum over the entries (i, j, a) of row i    of a * Ht[j][:]
//   W^T A : Pt[j][:] = sum over the entries (i, j, a) of column j of a * W[i][:]
// The first walks the caller's CSR arrays (read-only, never copied); the
// second walks a column-ordered copy (CSC: column pointers, row indices,
// values) that is built once per call by a stable radix sort of the column
// indices, so entries of a column keep their row order and sums are
// reproducible.  The two updates are then one kernel used twice (the H update
// is the W update of the transposed problem), each with its update fused.
// The sparse iteration works on Ht = H^T (n x k); H is transposed on entry
// and on exit.
//
// Work mapping: a row (of A for the W update, of A^T for the H update) is
// handled by a group of LPR lanes, LPR = smallest power of two >= k (at least
// 4): lane c of the group owns factor index c.  A wave holds 64 / LPR rows, so
// short rows are packed several to a wave.  The group reads its row's entries
// LPR at a time with coalesced loads and hands them round with lane shuffles.
// Rows are dealt to wavefronts in contiguous ranges of equal work (stored
// entries plus a per-row cost), and rows too long for one group are split
// over a whole workgroup.
#include <hipcub/hipcub.hpp>

#include "nmfmu_internal.h"

namespace nmfmu {

template <int LPR>
__device__ __forceinline__ float group_bcast(float v, int src)
{
    return __shfl(v, src, LPR);
}
template <int LPR>
__device__ __forceinline__ int group_bcast(int v, int src)
{
    return __shfl(v, src, LPR);
}

// den[c] = sum_d x[d] * G[d][c] for the row whose element c this lane holds.
template <int LPR>
__device__ __forceinline__ float row_times_gram(float x, const float *Gs, int ldg, int k, int c)
{
    float d0 = 0.f, d1 = 0.f;
    const int cc = (c < k) ? c : 0;
    for (int d = 0; d + 1 < k; d += 2) {
        d0 += group_bcast<LPR>(x, d) * Gs[d * ldg + cc];
        d1 += group_bcast<LPR>(x, d + 1) * Gs[(d + 1) * ldg + cc];
    }
    if (k & 1) d0 += group_bcast<LPR>(x, k - 1) * Gs[(k - 1) * ldg + cc];
    return d0 + d1;
}

__device__ __forceinline__ void stage_gram(float *Gs, const float *__restrict__ G, int k, int ldg)
{
    for (int e = threadIdx.x; e < k * k; e += blockDim.x) Gs[(e / k) * ldg + (e % k)] = G[e];
    __syncthreads();
}

// ---------------------------------------------------------------------------
// Row-balanced work partition.  The work of row r is taken as its stored
// entries plus kRowCost (the fused update), so the running total
//     key(r) = rowptr[r] + kRowCost * r
// is increasing and part[w] = first r with key(r) >= w * share splits the rows
// into nparts contiguous ranges of (nearly) equal work, one per wavefront.
// Rows longer than kLongRow entries are taken out of the ranges (they would
// stall one wavefront) and handled by a whole workgroup each.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void csr_partition_kernel(const int64_t *__restrict__ rowptr,
                                                            int64_t m, int nparts,
                                                            int64_t *__restrict__ part)
{
    const int w = blockIdx.x * 256 + threadIdx.x;
    if (w > nparts) return;
    const int64_t total = rowptr[m] + kRowCost * m;
    const int64_t share = (total + nparts - 1) / nparts;
    const int64_t target = (int64_t)w * share;
    int64_t lo = 0, hi = m;                 // smallest r in [0, m] with key(r) >= target
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] + kRowCost * mid >= target) hi = mid;
        else lo = mid + 1;
    }
    part[w] = (w == nparts) ? m : lo;
}

// list[0 .. *count) = rows with more than kLongRow entries (any order).
// `cap` slots: row pointers that add up to nnz cannot name more such rows than nnz / kLongRow;
// malformed ones can, and what does not fit is dropped (the count keeps running).
__global__ __launch_bounds__(256) void csr_long_rows_kernel(const int64_t *__restrict__ rowptr,
                                                            int64_t m, int32_t *__restrict__ list,
                                                            unsigned *count, unsigned cap)
{
    for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < m; r += (int64_t)gridDim.x * 256)
        if (rowptr[r + 1] - rowptr[r] > kLongRow) {
            const unsigned slot = atomicAdd(count, 1u);
            if (slot < cap) list[slot] = (int32_t)r;
        }
}

__global__ void zero_u32_kernel(unsigned *p) { if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0u; }

// One gather step of a lane group: entries [e, e + LPR) of a row (fewer at its
// end), UNR at a time so that several table rows are in flight; lanes past the
// end hold (column 0, value 0): they gather row 0 of the table and add nothing.
// T has `trows` rows of k floats.
template <int LPR>
__device__ __forceinline__ float gather_chunk(const int32_t *__restrict__ colidx,
                                              const float *__restrict__ vals,
                                              const float *__restrict__ T, int trows, int k, int c,
                                              int64_t e, int64_t e1, float acc)
{
    const int64_t left = e1 - e;
    const int cnt = left < LPR ? (left > 0 ? (int)left : 0) : LPR;
    int colv = 0;
    float valv = 0.f;
    if (c < cnt) {
        colv = colidx[e + c];
        valv = vals[e + c];
    }
    constexpr int UNR = (LPR < 8) ? LPR : 8;
    const int cc = (c < k) ? c : 0;
    for (int t0 = 0; __any(t0 < cnt); t0 += UNR) {
        float a[UNR], h[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            // an index outside the table (malformed input) is pulled to its edge: no stray access
            const int col = min(max(group_bcast<LPR>(colv, t0 + u), 0), trows - 1);
            a[u] = group_bcast<LPR>(valv, t0 + u);
            h[u] = T[(int64_t)col * k + cc];
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) acc += a[u] * h[u];
    }
    return acc;
}

// The test that sends a row to the long-row kernel, on the row pointers as given (the list of
// long rows is built with the same test).
__device__ __forceinline__ bool rowptr_long(const int64_t *__restrict__ rowptr, int64_t row, bool valid)
{
    return valid && rowptr[row + 1] - rowptr[row] > kLongRow;
}

// ---------------------------------------------------------------------------
// X[i][:] <- X[i][:] * (sum over the entries (i, j, a) of row i of a T[j][:]) / (X[i][:] G + eps).
// With the CSR of A, T = Ht, G = H H^T, X = W: AHT, WHHT and the W update of
// Algorithm 3 in one kernel (the row of A H^T lives in one register per lane);
// with the column-ordered copy, T = W, G = W^T W, X = Ht: WTA and the H update.
// Wavefront gw works on rows [part[gw], part[gw + 1]), 64 / LPR rows at a time.
// accumulate != 0: no update; the gathered sums are added to W instead (the
// numerator of an update collected over several row batches of the matrix; GH unused).
// accumulate == 2: nothing is written to W (needs dpart; GH unused).
// dpart: dpart[blockIdx.x] = sum over this block's rows of gathered sum x value of W in double
// (the new value in an updating launch, the unchanged one with accumulate == 2), i.e. its
// share of <A H^T, W> for the objective ||A||^2 - 2 <A H^T, W> + <H H^T, W^T W>; lanes by
// butterfly, then the 4 waves in order.
// ---------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(256) void aht_csr_kernel(const int64_t *__restrict__ rowptr,
                                                      const int32_t *__restrict__ colidx,
                                                      const float *__restrict__ vals,
                                                      const int64_t *__restrict__ part, int k,
                                                      const float *__restrict__ Ht,
                                                      const float *__restrict__ GH, float *W,
                                                      float eps, int accumulate,
                                                      double *__restrict__ dpart, int64_t nnz, int trows)
{
    constexpr int LDG = 65, RPW = 64 / LPR;
    __shared__ float Gs[64 * LDG];
    __shared__ double dsum[4];
    if (!accumulate) stage_gram(Gs, GH, k, LDG);
    double dacc = 0.0;
    const int lane = threadIdx.x & 63;
    const int c = lane % LPR;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t r_lo = part[gw], r_hi = part[gw + 1];          // same for the whole wavefront
    for (int64_t base = r_lo; base < r_hi; base += RPW) {
        const int64_t row = base + lane / LPR;
        bool valid = row < r_hi;
        // row pointers outside [0, nnz] (malformed input) are pulled into the arrays
        int64_t e = valid ? min(max(rowptr[row], (int64_t)0), nnz) : 0;
        int64_t e1 = valid ? min(max(rowptr[row + 1], (int64_t)0), nnz) : 0;
        if (rowptr_long(rowptr, row, valid)) {       // left to the long-row kernel
            valid = false;
            e1 = e;
        }
        float acc = 0.f;
        while (__any(e < e1)) {
            acc = gather_chunk<LPR>(colidx, vals, Ht, trows, k, c, e, e1, acc);
            e += LPR;
        }
        const float w = (valid && c < k) ? W[row * k + c] : 0.f;
        if (accumulate == 2) {
            if (valid && c < k) dacc += (double)acc * (double)w;
            continue;
        }
        if (accumulate) {
            if (valid && c < k) W[row * k + c] = w + acc;
            continue;
        }
        const float den = row_times_gram<LPR>(w, Gs, LDG, k, c) + eps;
        if (valid && c < k) {
            const float wn = w * acc / den;
            W[row * k + c] = wn;
            dacc += (double)acc * (double)wn;
        }
    }
    if (dpart) {     // uniform over the grid
        for (int off = 32; off > 0; off >>= 1) dacc += __shfl_xor(dacc, off);
        if (lane == 0) dsum[threadIdx.x >> 6] = dacc;
        __syncthreads();
        if (threadIdx.x == 0) dpart[blockIdx.x] = ((dsum[0] + dsum[1]) + dsum[2]) + dsum[3];
    }
}

// The same update for the rows in `list` (more than kLongRow entries): one
// workgroup per row, its lane groups take the row's chunks round robin and
// their sums are added in group order.
template <int LPR>
__global__ __launch_bounds__(256) void aht_csr_long_kernel(const int64_t *__restrict__ rowptr,
                                                           const int32_t *__restrict__ colidx,
                                                           const float *__restrict__ vals,
                                                           const int32_t *__restrict__ list,
                                                           const unsigned *__restrict__ count, int k,
                                                           const float *__restrict__ Ht,
                                                           const float *__restrict__ GH, float *W,
                                                           float eps, int accumulate,
                                                           double *__restrict__ dpart, int64_t nnz, int trows,
                                                           unsigned list_cap)
{
    constexpr int LDG = 65, NG = 256 / LPR;
    __shared__ float Gs[64 * LDG];
    __shared__ float part_acc[NG][LPR];
    const unsigned n_long = *count < list_cap ? *count : list_cap;
    if (n_long == 0) {
        if (dpart && threadIdx.x == 0) dpart[blockIdx.x] = 0.0;
        return;
    }
    double dacc = 0.0;      // first wavefront only: it finishes the rows
    if (!accumulate) stage_gram(Gs, GH, k, LDG);
    const int c = threadIdx.x % LPR, grp = threadIdx.x / LPR;
    for (unsigned li = blockIdx.x; li < n_long; li += gridDim.x) {
        const int64_t row = list[li];
        const int64_t e0 = min(max(rowptr[row], (int64_t)0), nnz), e1 = min(max(rowptr[row + 1], (int64_t)0), nnz);
        float acc = 0.f;
        for (int64_t e = e0 + (int64_t)grp * LPR; __any(e < e1); e += (int64_t)NG * LPR)
            acc = gather_chunk<LPR>(colidx, vals, Ht, trows, k, c, e, e1, acc);
        part_acc[grp][c] = acc;
        __syncthreads();
        if (grp == 0) {        // LPR is a multiple of 64 only for LPR = 64; smaller groups share a wave
            float total = 0.f;
            for (int gI = 0; gI < NG; ++gI) total += part_acc[gI][c];
            part_acc[0][c] = total;
        }
        __syncthreads();
        if (threadIdx.x < 64) {     // first wavefront: its first group finishes the row
            const float tot = part_acc[0][c];
            const bool mine = threadIdx.x < LPR;
            const float w = (mine && c < k) ? W[row * k + c] : 0.f;
            if (accumulate == 2) {
                if (mine && c < k) dacc += (double)tot * (double)w;
            } else if (accumulate) {
                if (mine && c < k) W[row * k + c] = w + tot;
            } else {
                const float den = row_times_gram<LPR>(w, Gs, LDG, k, c) + eps;
                if (mine && c < k) {
                    const float wn = w * tot / den;
                    W[row * k + c] = wn;
                    dacc += (double)tot * (double)wn;
                }
            }
        }
        __syncthreads();
    }
    if (dpart && threadIdx.x < 64) {
        for (int off = 32; off > 0; off >>= 1) dacc += __shfl_xor(dacc, off);
        if (threadIdx.x == 0) dpart[blockIdx.x] = dacc;
    }
}

// X[i][:] <- X[i][:] * Num[i][:] / (X[i][:] G + eps) for i < rows: the update once its
// numerator has been collected (out-of-memory CSR); lane group per row as above.
template <int LPR>
__global__ __launch_bounds__(256) void row_update_kernel(float *X, const float *__restrict__ Num,
                                                         const float *__restrict__ G, int k,
                                                         int64_t rows, float eps)
{
    constexpr int LDG = 65, RPW = 64 / LPR;
    __shared__ float Gs[64 * LDG];
    stage_gram(Gs, G, k, LDG);
    const int lane = threadIdx.x & 63;
    const int c = lane % LPR;
    const int64_t waves = (int64_t)gridDim.x * 4;
    for (int64_t base = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW; base < rows; base += waves * RPW) {
        const int64_t row = base + lane / LPR;
        const bool valid = row < rows && c < k;
        const float x = valid ? X[row * k + c] : 0.f;
        const float den = row_times_gram<LPR>(x, Gs, LDG, k, c) + eps;
        if (valid) X[row * k + c] = x * Num[row * k + c] / den;
    }
}

// out[i] = in[i] - base: row pointers of a row batch made relative to the batch's first entry.
__global__ __launch_bounds__(256) void rebase_i64_kernel(const int64_t *__restrict__ in, int64_t count,
                                                         int64_t base, int64_t *__restrict__ out)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256)
        out[i] = in[i] - base;
}

__global__ __launch_bounds__(256) void fill_f32_kernel(float *p, int64_t count, float v)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256)
        p[i] = v;
}

// ---------------------------------------------------------------------------
// Column-ordered copy of the CSR matrix.
// ---------------------------------------------------------------------------
// payload[e] = (row of entry e) << 32 | bits of vals[e]; a group of 32 lanes per row.
__global__ __launch_bounds__(256) void csc_payload_kernel(const int64_t *__restrict__ rowptr,
                                                          const float *__restrict__ vals, int64_t m,
                                                          int64_t nnz, uint64_t *__restrict__ payload)
{
    const int c = threadIdx.x & 31;
    const int64_t group = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 5;
    const int64_t ngroups = (int64_t)gridDim.x * 8;
    for (int64_t row = group; row < m; row += ngroups) {
        const int64_t e1 = min(max(rowptr[row + 1], (int64_t)0), nnz);
        for (int64_t e = min(max(rowptr[row], (int64_t)0), nnz) + c; e < e1; e += 32)
            payload[e] = ((uint64_t)row << 32) | (uint64_t)__float_as_uint(vals[e]);
    }
}

// After the stable sort by column: sorted_cols[e'] is the column of the e'-th
// entry in column order and sorted_payload[e'] its (row, value).  Writes the CSC
// row indices and values and the column pointers (every column j with
// sorted_cols[e'-1] < j <= sorted_cols[e'] starts at e'; columns after the last
// stored one start at nnz).
// dup_part (optional, one double per block): repeated (row, column) pairs stand for their sum, so
// the squared norm of the matrix is the sum of the squared stored values plus, for every run of
// entries with the same row and column (adjacent here, because the sort is stable and a column's
// entries keep their row-major order), twice the products of its pairs; each entry adds
// 2 x its value x the sum of the run's entries before it.
__global__ __launch_bounds__(256) void csc_finish_kernel(const int32_t *__restrict__ sorted_cols,
                                                         const uint64_t *__restrict__ sorted_payload,
                                                         int64_t n, int64_t nnz,
                                                         int64_t *__restrict__ colptr,
                                                         int32_t *__restrict__ rowidx,
                                                         float *__restrict__ cvals,
                                                         double *__restrict__ dup_part)
{
    double corr = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * 256) {
        const uint64_t pl = sorted_payload[e];
        rowidx[e] = (int32_t)(pl >> 32);
        cvals[e] = __uint_as_float((unsigned)pl);
        if (dup_part) {
            double before = 0.0;
            for (int64_t p = e - 1; p >= 0 && sorted_cols[p] == sorted_cols[e] && (sorted_payload[p] >> 32) == (pl >> 32); --p)
                before += (double)__uint_as_float((unsigned)sorted_payload[p]);
            corr += 2.0 * (double)__uint_as_float((unsigned)pl) * before;
        }
        // column indices outside [0, n) (malformed input) are pulled to the edge
        const int64_t cur = min(max((int64_t)sorted_cols[e], (int64_t)0), n - 1);
        const int64_t prev = (e > 0) ? min(max((int64_t)sorted_cols[e - 1], (int64_t)0), n - 1) : -1;
        for (int64_t j = prev + 1; j <= cur; ++j) colptr[j] = e;
        if (e == nnz - 1)
            for (int64_t j = cur + 1; j <= n; ++j) colptr[j] = nnz;
    }
    if (dup_part) {     // uniform over the grid; lanes by butterfly, then the 4 waves in order
        __shared__ double wsum[4];
        for (int off = 32; off > 0; off >>= 1) corr += __shfl_xor(corr, off);
        if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = corr;
        __syncthreads();
        if (threadIdx.x == 0) dup_part[blockIdx.x] = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
    }
}

__global__ __launch_bounds__(256) void fill_i64_kernel(int64_t *p, int64_t count, int64_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256)
        p[i] = v;
}

// dst (rows x ld_dst) = the first `cols` columns of src (rows x ld_src), columns cols .. ld_dst - 1
// of dst set to zero (cols <= ld_dst).  One workgroup per row at a time; a wave instruction moves
// 64 consecutive floats, eight per thread in flight.  No alignment is asked of either side.
__global__ __launch_bounds__(256) void pad_copy_kernel(const float *__restrict__ src, int64_t ld_src,
                                                       float *__restrict__ dst, int64_t ld_dst, int64_t rows,
                                                       int64_t cols)
{
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const float *s = src + r * ld_src;
        float *d = dst + r * ld_dst;
        for (int64_t c0 = threadIdx.x; c0 < ld_dst; c0 += 2048) {
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int64_t c = c0 + 256 * q;
                v[q] = c < cols ? s[c] : 0.f;
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int64_t c = c0 + 256 * q;
                if (c < ld_dst) d[c] = v[q];
            }
        }
    }
}

// out (cols x rows) = in^T, in is rows x cols.
__global__ __launch_bounds__(256) void transpose_kernel(const float *__restrict__ in, int64_t rows,
                                                        int64_t cols, float *__restrict__ out)
{
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int64_t tiles_c = (cols + 31) / 32, tiles_r = (rows + 31) / 32;
    for (int64_t t = blockIdx.x; t < tiles_c * tiles_r; t += gridDim.x) {
        const int64_t r0 = (t / tiles_c) * 32, c0 = (t % tiles_c) * 32;
        for (int y = ty; y < 32; y += 8)
            if (r0 + y < rows && c0 + tx < cols) tile[y][tx] = in[(r0 + y) * cols + c0 + tx];
        __syncthreads();
        for (int y = ty; y < 32; y += 8)
            if (c0 + y < cols && r0 + tx < rows) out[(c0 + y) * rows + r0 + tx] = tile[tx][y];
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------

static int lanes_per_row(int k)
{
    int l = 4;
    while (l < k) l <<= 1;
    return l;
}

#define NMFMU_LPR_SWITCH(lpr, CALL)      \
    switch (lpr) {                        \
    case 4: { constexpr int L = 4; CALL; } break;   \
    case 8: { constexpr int L = 8; CALL; } break;   \
    case 16: { constexpr int L = 16; CALL; } break; \
    case 32: { constexpr int L = 32; CALL; } break; \
    default: { constexpr int L = 64; CALL; } break; \
    }

hipError_t launch_csr_partition(const int64_t *rowptr, int64_t m, int nparts, int64_t *part,
                                hipStream_t st)
{
    hipLaunchKernelGGL(csr_partition_kernel, dim3((nparts + 1 + 255) / 256), dim3(256), 0, st, rowptr, m, nparts, part);
    return hipGetLastError();
}

hipError_t launch_csr_long_rows(const int64_t *rowptr, int64_t m, int32_t *list, unsigned *count,
                                unsigned cap, hipStream_t st)
{
    hipLaunchKernelGGL(zero_u32_kernel, dim3(1), dim3(64), 0, st, count);
    int64_t b = (m + 255) / 256;
    if (b > 4096) b = 4096;
    hipLaunchKernelGGL(csr_long_rows_kernel, dim3((unsigned)b), dim3(256), 0, st, rowptr, m, list, count, cap);
    return hipGetLastError();
}

hipError_t launch_aht_csr(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                          const int64_t *part, const int32_t *long_list, const unsigned *long_count,
                          int k, const float *Ht, const float *GH, float *W, float eps, int64_t nnz, int64_t trows,
                          hipStream_t st, bool accumulate, double *dpart, bool dry)
{
    if (trows < 1 || trows > 0x7fffffff || nnz < 0) return hipErrorInvalidValue;
    if ((dpart && accumulate) || (dry && (!dpart || accumulate))) return hipErrorInvalidValue;
    const int lpr = lanes_per_row(k);
    const dim3 grid(kCsrParts / 4), block(256);
    const int acc = dry ? 2 : (accumulate ? 1 : 0);
    double *dlong = dpart ? dpart + kCsrParts / 4 : nullptr;
    NMFMU_LPR_SWITCH(lpr, hipLaunchKernelGGL((aht_csr_kernel<L>), grid, block, 0, st, rowptr, colidx,
                                             vals, part, k, Ht, GH, W, eps, acc, dpart, nnz, (int)trows));
    NMFMU_LPR_SWITCH(lpr, hipLaunchKernelGGL((aht_csr_long_kernel<L>), dim3(kCsrLongBlocks), block, 0, st, rowptr,
                                             colidx, vals, long_list, long_count, k, Ht, GH, W, eps, acc, dlong, nnz,
                                             (int)trows, (unsigned)(nnz / kLongRow + 1)));
    return hipGetLastError();
}

hipError_t launch_row_update(float *X, const float *Num, const float *G, int k, int64_t rows, float eps,
                             hipStream_t st)
{
    const int lpr = lanes_per_row(k);
    int64_t b = (rows * lpr / 64 + 3) / 4;
    if (b > 8192) b = 8192;
    if (b < 1) b = 1;
    const dim3 grid((unsigned)b), block(256);
    NMFMU_LPR_SWITCH(lpr, hipLaunchKernelGGL((row_update_kernel<L>), grid, block, 0, st, X, Num, G, k, rows, eps));
    return hipGetLastError();
}

hipError_t launch_rebase_i64(const int64_t *in, int64_t count, int64_t base, int64_t *out, hipStream_t st)
{
    int64_t b = (count + 255) / 256;
    if (b > 4096) b = 4096;
    hipLaunchKernelGGL(rebase_i64_kernel, dim3((unsigned)b), dim3(256), 0, st, in, count, base, out);
    return hipGetLastError();
}

hipError_t launch_fill_f32(float *p, int64_t count, float v, hipStream_t st)
{
    int64_t b = (count + 255) / 256;
    if (b > 8192) b = 8192;
    if (b < 1) b = 1;
    hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)b), dim3(256), 0, st, p, count, v);
    return hipGetLastError();
}

hipError_t launch_pad_copy(const float *src, int64_t ld_src, float *dst, int64_t ld_dst, int64_t rows, int64_t cols,
                           hipStream_t st)
{
    if (cols > ld_dst || cols > ld_src) return hipErrorInvalidValue;
    const int64_t b = rows < 8192 ? rows : 8192;
    hipLaunchKernelGGL(pad_copy_kernel, dim3((unsigned)(b < 1 ? 1 : b)), dim3(256), 0, st, src, ld_src, dst, ld_dst, rows, cols);
    return hipGetLastError();
}

hipError_t launch_transpose(const float *in, int64_t rows, int64_t cols, float *out, hipStream_t st)
{
    int64_t tiles = ((rows + 31) / 32) * ((cols + 31) / 32);
    if (tiles > 65536) tiles = 65536;
    hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)tiles), dim3(256), 0, st, in, rows, cols, out);
    return hipGetLastError();
}

static unsigned blocks_for(int64_t count)
{
    int64_t b = (count + 255) / 256;
    if (b > 65536) b = 65536;
    if (b < 1) b = 1;
    return (unsigned)b;
}

static int bits_for(int64_t n)
{
    int b = 1;
    while (((int64_t)1 << b) < n) ++b;
    return b;
}

size_t csc_sort_temp_bytes(int64_t nnz, int64_t n)
{
    size_t bytes = 0;
    const int32_t *kin = nullptr;
    int32_t *kout = nullptr;
    const uint64_t *vin = nullptr;
    uint64_t *vout = nullptr;
    (void)hipcub::DeviceRadixSort::SortPairs(nullptr, bytes, kin, kout, vin, vout, (int)nnz, 0, bits_for(n));
    return bytes;
}

hipError_t launch_csc_build(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                            int64_t m, int64_t n, int64_t nnz, int32_t *sorted_cols,
                            uint64_t *payload, uint64_t *sorted_payload, void *sort_temp,
                            size_t sort_temp_bytes, int64_t *colptr, int32_t *rowidx, float *cvals,
                            hipStream_t st, double *dup_part)
{
    if (nnz == 0) {
        hipLaunchKernelGGL(fill_i64_kernel, dim3(blocks_for(n + 1)), dim3(256), 0, st, colptr, n + 1, (int64_t)0);
        if (dup_part) hipLaunchKernelGGL(fill_i64_kernel, dim3(1), dim3(256), 0, st, reinterpret_cast<int64_t *>(dup_part), (int64_t)1, (int64_t)0);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(csc_payload_kernel, dim3(blocks_for(m * 32)), dim3(256), 0, st, rowptr, vals, m, nnz, payload);
    hipError_t e = hipcub::DeviceRadixSort::SortPairs(sort_temp, sort_temp_bytes, colidx, sorted_cols,
                                                      (const uint64_t *)payload, sorted_payload,
                                                      (int)nnz, 0, bits_for(n), st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(csc_finish_kernel, dim3(blocks_for(nnz)), dim3(256), 0, st, sorted_cols,
                       sorted_payload, n, nnz, colptr, rowidx, cvals, dup_part);
    return hipGetLastError();
}

int csc_finish_blocks(int64_t nnz) { return (int)blocks_for(nnz); }

}  // namespace nmfmu
