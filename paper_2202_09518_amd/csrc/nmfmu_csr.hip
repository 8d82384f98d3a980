// CSR kernels of the multiplicative-update iteration for gfx950 (MI355X).
//
// With A in CSR (paper, section 2.3: values, column indices, row pointers) the
// two products over A become sums over stored entries:
//   A H^T : Q[i][:]  = sum over entries (i, j, a) of a * Ht[j][:]     (gather)
//   W^T A : Pt[j][:] += a * W[i][:] for every entry (i, j, a)         (scatter)
// Both are written against a transposed factor Ht = H^T (n x k), so that one
// stored entry touches one contiguous run of k floats.  The whole sparse
// iteration therefore works on Ht; H itself is transposed once on entry and
// once on exit.
//
// Work mapping: a row (or a column of H) is handled by a group of LPR lanes,
// LPR = smallest power of two >= k (at least 4): lane c of the group owns
// factor index c.  A wave holds 64 / LPR rows, so short rows are packed
// several to a wave.  The group reads its row's entries LPR at a time with
// coalesced loads and hands them round with lane shuffles.
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
// W <- W * (A Ht) / (W GH + eps), A in CSR.  Algorithm 3: AHT, WHHT and the
// W update in one kernel; the row of A H^T lives in one register per lane.
// ---------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(256) void aht_csr_kernel(const int64_t *__restrict__ rowptr,
                                                      const int32_t *__restrict__ colidx,
                                                      const float *__restrict__ vals, int64_t m,
                                                      int k, const float *__restrict__ Ht,
                                                      const float *__restrict__ GH, float *W,
                                                      float eps)
{
    constexpr int LDG = 65;
    __shared__ float Gs[64 * LDG];
    stage_gram(Gs, GH, k, LDG);
    const int c = threadIdx.x % LPR;
    const int64_t group = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPR;
    const int64_t ngroups = (int64_t)gridDim.x * 256 / LPR;
    const int64_t trips = (m + ngroups - 1) / ngroups;     // same for every lane
    for (int64_t it = 0; it < trips; ++it) {
        const int64_t row = group + it * ngroups;
        const bool valid = row < m;
        int64_t e = valid ? rowptr[row] : 0;
        const int64_t e1 = valid ? rowptr[row + 1] : 0;
        float acc = 0.f;
        while (__any(e < e1)) {
            const int64_t left = e1 - e;
            const int cnt = left < LPR ? (left > 0 ? (int)left : 0) : LPR;
            int colv = 0;
            float valv = 0.f;
            if (c < cnt) {
                colv = colidx[e + c];
                valv = vals[e + c];
            }
            for (int t = 0; __any(t < cnt); ++t) {
                const int col = group_bcast<LPR>(colv, t);
                const float a = group_bcast<LPR>(valv, t);
                if (t < cnt && c < k) acc += a * Ht[(int64_t)col * k + c];
            }
            e += LPR;
        }
        const float w = (valid && c < k) ? W[row * k + c] : 0.f;
        const float den = row_times_gram<LPR>(w, Gs, LDG, k, c) + eps;
        if (valid && c < k) W[row * k + c] = w * acc / den;
    }
}

// ---------------------------------------------------------------------------
// Pt (n x k) += scatter of a * W[i][:] over the stored entries.  Algorithm 3,
// formation of WTA, for a CSR A; fp32 hardware atomics, order not fixed.
// ---------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(256) void wta_csr_kernel(const int64_t *__restrict__ rowptr,
                                                      const int32_t *__restrict__ colidx,
                                                      const float *__restrict__ vals, int64_t m,
                                                      int k, const float *__restrict__ W, float *Pt)
{
    const int c = threadIdx.x % LPR;
    const int64_t group = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPR;
    const int64_t ngroups = (int64_t)gridDim.x * 256 / LPR;
    const int64_t trips = (m + ngroups - 1) / ngroups;
    for (int64_t it = 0; it < trips; ++it) {
        const int64_t row = group + it * ngroups;
        const bool valid = row < m;
        int64_t e = valid ? rowptr[row] : 0;
        const int64_t e1 = valid ? rowptr[row + 1] : 0;
        const float w = (valid && c < k) ? W[row * k + c] : 0.f;
        while (__any(e < e1)) {
            const int64_t left = e1 - e;
            const int cnt = left < LPR ? (left > 0 ? (int)left : 0) : LPR;
            int colv = 0;
            float valv = 0.f;
            if (c < cnt) {
                colv = colidx[e + c];
                valv = vals[e + c];
            }
            for (int t = 0; __any(t < cnt); ++t) {
                const int col = group_bcast<LPR>(colv, t);
                const float a = group_bcast<LPR>(valv, t);
                if (t < cnt && c < k) unsafeAtomicAdd(&Pt[(int64_t)col * k + c], a * w);
            }
            e += LPR;
        }
    }
}

// ---------------------------------------------------------------------------
// X <- X * Q / (X G + eps) row by row, X and Q rows x k, G symmetric k x k.
// With X = Ht, Q = Pt, G = WTW this is the H update of Algorithm 3 written
// for the transposed factor.
// ---------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(256) void row_update_kernel(float *X, const float *__restrict__ Q,
                                                         const float *__restrict__ G, int64_t rows,
                                                         int k, float eps)
{
    constexpr int LDG = 65;
    __shared__ float Gs[64 * LDG];
    stage_gram(Gs, G, k, LDG);
    const int c = threadIdx.x % LPR;
    const int64_t group = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPR;
    const int64_t ngroups = (int64_t)gridDim.x * 256 / LPR;
    const int64_t trips = (rows + ngroups - 1) / ngroups;
    for (int64_t it = 0; it < trips; ++it) {
        const int64_t row = group + it * ngroups;
        const bool ok = row < rows && c < k;
        const float x = ok ? X[row * k + c] : 0.f;
        const float q = ok ? Q[row * k + c] : 0.f;
        const float den = row_times_gram<LPR>(x, Gs, LDG, k, c) + eps;
        if (ok) X[row * k + c] = x * q / den;
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

__global__ __launch_bounds__(256) void fill_zero_kernel(float *p, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256)
        p[i] = 0.f;
}

// ---------------------------------------------------------------------------

static int lanes_per_row(int k)
{
    int l = 4;
    while (l < k) l <<= 1;
    return l;
}

static unsigned blocks_for_groups(int64_t rows, int lpr)
{
    const int64_t groups_per_block = 256 / lpr;
    int64_t b = (rows + groups_per_block - 1) / groups_per_block;
    const int64_t cap = 256 * 16;       // 16 workgroups per compute unit, then grid-stride
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (unsigned)b;
}

#define NMFMU_LPR_SWITCH(lpr, CALL)      \
    switch (lpr) {                        \
    case 4: { constexpr int L = 4; CALL; } break;   \
    case 8: { constexpr int L = 8; CALL; } break;   \
    case 16: { constexpr int L = 16; CALL; } break; \
    case 32: { constexpr int L = 32; CALL; } break; \
    default: { constexpr int L = 64; CALL; } break; \
    }

hipError_t launch_aht_csr(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                          int64_t m, int k, const float *Ht, const float *GH, float *W, float eps,
                          hipStream_t st)
{
    const int lpr = lanes_per_row(k);
    dim3 grid(blocks_for_groups(m, lpr));
    NMFMU_LPR_SWITCH(lpr, hipLaunchKernelGGL((aht_csr_kernel<L>), grid, dim3(256), 0, st, rowptr,
                                             colidx, vals, m, k, Ht, GH, W, eps));
    return hipGetLastError();
}

hipError_t launch_wta_csr(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                          int64_t m, int k, const float *W, float *Pt, hipStream_t st)
{
    const int lpr = lanes_per_row(k);
    dim3 grid(blocks_for_groups(m, lpr));
    NMFMU_LPR_SWITCH(lpr, hipLaunchKernelGGL((wta_csr_kernel<L>), grid, dim3(256), 0, st, rowptr,
                                             colidx, vals, m, k, W, Pt));
    return hipGetLastError();
}

hipError_t launch_row_update(float *X, const float *Q, const float *G, int64_t rows, int k,
                             float eps, hipStream_t st)
{
    const int lpr = lanes_per_row(k);
    dim3 grid(blocks_for_groups(rows, lpr));
    NMFMU_LPR_SWITCH(lpr, hipLaunchKernelGGL((row_update_kernel<L>), grid, dim3(256), 0, st, X, Q,
                                             G, rows, k, eps));
    return hipGetLastError();
}

hipError_t launch_transpose(const float *in, int64_t rows, int64_t cols, float *out, hipStream_t st)
{
    int64_t tiles = ((rows + 31) / 32) * ((cols + 31) / 32);
    if (tiles > 65536) tiles = 65536;
    hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)tiles), dim3(256), 0, st, in, rows, cols, out);
    return hipGetLastError();
}

hipError_t launch_fill_zero(float *p, int64_t count, hipStream_t st)
{
    int64_t b = (count + 255) / 256;
    if (b > 8192) b = 8192;
    if (b < 1) b = 1;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)b), dim3(256), 0, st, p, count);
    return hipGetLastError();
}

}  // namespace nmfmu
