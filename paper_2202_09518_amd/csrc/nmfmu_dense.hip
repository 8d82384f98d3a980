// Dense kernels of the multiplicative-update iteration for gfx950 (MI355X).
//
// One iteration (paper, Algorithm 3 on a single unit) is
//   WTW = W^T W,  WTA = W^T A,  H <- H * WTA / (WTW H + eps),
//   HHT = H H^T (new H),  AHT = A H^T (new H),  W <- W * AHT / (W HHT + eps),
// and the two products over A are all of its memory traffic.  Here they are
// streaming passes over A on the matrix cores, with everything else folded into
// them or into one small finisher kernel:
//   wta_pass_split_buf_kernel / wta_pass_split64_wide_kernel : W^T A as row-split
//       partials; lanes run along the columns of A, the reduction over rows is the
//       reduction of the matrix instruction
//   factor_update_kernel : sums the partials, updates H (or W^T in the mirrored
//       plan), writes the operand planes and the Gram tiles of the new factor
//   aht_rows_kernel : A H^T on the row-major A (coalesced loads turned through
//       LDS) with the W update, the planes and the Gram tiles of the new W fused
//   aht_pass_kernel : the older direct A H^T kernel (lanes down the rows), for
//       shapes the others do not serve (unaligned A, short wide matrices)
//   gram_kernel, gram_sum_kernel, residual_*_kernel, objective_kernel : the small rest.
// For k <= 64 and aligned A the products are exact: fp32 operands cut into three
// bf16 pieces each, eight of the nine piece products per term (all but the lowest,
// below 2^-30 of the term) on v_mfma_f32_32x32x16_bf16 with fp32 accumulation (see
// split3 below).  wta_pass_kernel and aht_pass_kernel use
// v_mfma_f32_32x32x2_f32 on the floats themselves.
//
// Lane layout of v_mfma_f32_32x32x2_f32 (64 lanes, D = A_op B_op + C):
//   A_op (32 x 2):  lane l holds A_op[l % 32][l / 32]
//   B_op (2 x 32):  lane l holds B_op[l / 32][l % 32]
//   D    (32 x 32): lane l, register v holds D[(v % 4) + 4 (l / 32) + 8 (v / 4)][l % 32]
#include "nmfmu_internal.h"

namespace nmfmu {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x16 mfma32(float a, float b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// ---- exact fp32 products on the bf16 matrix cores ---------------------------------
// A float x is cut into three pieces h + m + l = x, each with at most 8
// significant bits (a bf16 holds 8): h = x truncated to its top 8 bits,
// m = (x - h) truncated likewise, l = the rest.  Both subtractions are exact,
// so the sum of the pieces is x bit for bit (for |x| >= 2^-110; below that the
// last piece can fall under the bf16 range and is dropped by the hardware).  A
// product of two pieces has at most 16 significant bits and is exact in the
// fp32 accumulator, so the nine piece products of x y add up to the exact x y:
// v_mfma_f32_32x32x16_bf16 on pieces computes the same sums of products as
// v_mfma_f32_32x32x2_f32 on the floats, with the roundings of the running sums
// only, at a quarter of the matrix-core time per product.
// The kernels issue eight of the nine: l_x l_y is below 2^-30 |x y| (each low piece is
// below 2^-15 of its float), a 64th of the rounding of one fp32 addition, and the passes
// are bound by the power the matrix instructions draw: leaving it out takes 4-7 % off them.
//
// Lane layout of v_mfma_f32_32x32x16_bf16: A_op (32 x 16): lane l holds
// A_op[l % 32][8 (l / 32) .. 8 (l / 32) + 7]; B_op (16 x 32): lane l holds
// B_op[8 (l / 32) .. + 7][l % 32]; D as for the fp32 instruction.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x16 mfma_bf16(u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Bit patterns of the three pieces as floats (their low 16 bits are zero, or
// dropped by pack2: the top 16 bits are the bf16).
__device__ __forceinline__ void split3(float x, unsigned &h, unsigned &m, unsigned &l)
{
    h = __float_as_uint(x) & 0xffff0000u;
    const float r = x - __uint_as_float(h);
    m = __float_as_uint(r) & 0xffff0000u;
    l = __float_as_uint(r - __uint_as_float(m));
}

// Two bf16 in one register: `even` in the low half, `odd` in the high half.
__device__ __forceinline__ unsigned pack2(unsigned even, unsigned odd)
{
    return __builtin_amdgcn_perm(odd, even, 0x07060302u);
}

// Row of the 32 x 32 accumulator held in register v of a lane in half `half`.
__device__ __forceinline__ int acc_row(int v, int half) { return (v & 3) + 4 * half + 8 * (v >> 2); }

// Running totals of the piece passes.  The bf16 matrix instruction aligns its 16 products
// and the accumulator on the largest exponent and drops what falls below its adder's
// width without rounding, so an accumulator that has grown over thousands of rows loses
// the low bits of every product it takes in, always downwards: measured on uniform data
// the sum over 2048 rows comes out 1.7e-6 low, over 4096 rows 1.1e-5, while up to 512 rows
// the loss is below 1e-7.  The pass kernels therefore keep a matrix accumulator for at most
// kFlushSteps 16-row steps and then add it, with ordinary rounded fp32 adds, into a total
// that the wave keeps in its own 16 KiB of LDS (64 accumulator registers x 64 lanes; no
// other wave touches it, so no barrier).  Slot of register r of tile q for a lane: the
// lane index is flipped by 8 q so that the epilogue, which walks columns 4 jj + q, reads
// 32 different banks.
constexpr int kFlushSteps = 32;

// Cache policy of the buffer loads that stream A: the non-temporal bit.  Every element of A is
// used once per pass, so its lines are marked for early eviction and leave the L2 and the
// Infinity Cache to the operands that are re-read (the piece planes, the partial results).
// Measured on a bare read of 32768 x 16384 floats in the pass's launch shape: 0.313 ms
// (6.85 TB/s) against 0.345 ms (6.22 TB/s) with the default policy.
constexpr int kStreamLoad = 2;
constexpr int kTotFloats = 64 * 64;
__device__ __forceinline__ int tot_slot(int q, int v, int lane) { return (q * 16 + v) * 64 + (lane ^ (8 * q)); }

__device__ __forceinline__ void tot_clear(float *tot, int lane)
{
#pragma unroll
    for (int r = 0; r < 64; ++r) tot[r * 64 + lane] = 0.f;
}

// tot += acc; acc = 0 (four column tiles of one 32-factor tile)
__device__ __forceinline__ void tot_flush4(float *tot, f32x16 (&acc)[4], int lane)
{
    // a tile at a time: 16 reads in flight, then the adds, then the writes
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float t[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) t[v] = tot[tot_slot(q, v, lane)];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            tot[tot_slot(q, v, lane)] = t[v] + acc[q][v];
            acc[q][v] = 0.f;
        }
    }
}

// Epilogue of the 128-column kernels: the four waves' totals of (factor c, column x of the
// slab), added in wave order.
__device__ __forceinline__ float tot_sum4(const float *tot, int c, int x)
{
    const int q = x & 3, jj = x >> 2, half = (c >> 2) & 1, v = (c & 3) | ((c >> 3) << 2);
    const int idx = tot_slot(q, v, 32 * half + jj);
    float val = tot[idx];
#pragma unroll
    for (int ww = 1; ww < kWtaWaves; ++ww) val += tot[ww * kTotFloats + idx];
    return val;
}

// Four consecutive elements X[row][col .. col+3] of a row-major matrix with
// `ncols` columns; elements outside the matrix (or the whole group, if !ok)
// read as zero.  VEC needs a 16-byte aligned base and ncols % 4 == 0, col % 4 == 0.
template <bool VEC>
__device__ __forceinline__ f32x4 load4(const float *__restrict__ X, int64_t ncols, int64_t row,
                                       int64_t col, bool ok)
{
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (VEC) {
        // Branch free: lanes outside the matrix read element (0, 0) and discard
        // it, so the loads of a stage stay in one basic block and the waits on
        // them can be counted exactly (needed for the software prefetch).
        const bool in = ok && col < ncols;
        const f32x4 t = *reinterpret_cast<const f32x4 *>(X + (in ? row * ncols + col : 0));
        v.x = in ? t.x : 0.f;
        v.y = in ? t.y : 0.f;
        v.z = in ? t.z : 0.f;
        v.w = in ? t.w : 0.f;
    } else {
        if (ok) {
            const float *p = X + row * ncols + col;
            if (col + 0 < ncols) v.x = p[0];
            if (col + 1 < ncols) v.y = p[1];
            if (col + 2 < ncols) v.z = p[2];
            if (col + 3 < ncols) v.w = p[3];
        }
    }
    return v;
}

// ---------------------------------------------------------------------------
// Gram matrices.  MODE 0: G = X^T X, X is rows x k (the factor W).
//                 MODE 1: G = X X^T, X is k x cols (the factor H).
// blockIdx.y selects one 32 x 32 tile (t1, t2) of G; every block sums a slice
// of the long dimension, writes its partial tile, and the block that arrives
// last adds the partials in block order (deterministic) and stores G.
// ---------------------------------------------------------------------------
template <int MODE, bool VEC>
__global__ __launch_bounds__(512) void gram_kernel(const float *__restrict__ X, int64_t len, int k,
                                                   float *__restrict__ G, float *gpart,
                                                   unsigned *counters)
{
    constexpr int NW = 8;
    __shared__ float red[1024];
    __shared__ unsigned ticket_s;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int jj = lane & 31, half = lane >> 5;
    const int kt = (k + 31) >> 5;
    const int t1 = blockIdx.y / kt, t2 = blockIdx.y % kt;
    const int c1 = 32 * t1 + jj, c2 = 32 * t2 + jj;
    const int64_t gw = (int64_t)blockIdx.x * NW + w, tw = (int64_t)gridDim.x * NW;

    // Operands of several steps are fetched before the first multiply so that
    // the loads overlap; all loads are branch free (out-of-range lanes read
    // element 0 and discard it).
    f32x16 acc = {0};
    if (MODE == 0) {
        constexpr int UN = 8;
        const int64_t npairs = (len + 1) >> 1;
        for (int64_t p = gw; p < npairs; p += tw * UN) {
            float a[UN], b[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int64_t row = 2 * (p + u * tw) + half;
                const bool in1 = row < len && c1 < k, in2 = row < len && c2 < k;
                const float va = X[in1 ? row * k + c1 : 0], vb = X[in2 ? row * k + c2 : 0];
                a[u] = in1 ? va : 0.f;
                b[u] = in2 ? vb : 0.f;
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) acc = mfma32(a[u], b[u], acc);
        }
    } else {
        constexpr int UN = 4;
        const int64_t ngroups = (len + 7) >> 3;
        for (int64_t g = gw; g < ngroups; g += tw * UN) {
            f32x4 a[UN], b[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int64_t col = 8 * (g + u * tw) + 4 * half;
                a[u] = load4<VEC>(X, len, c1, col, c1 < k);
                b[u] = load4<VEC>(X, len, c2, col, c2 < k);
            }
#pragma unroll
            for (int u = 0; u < UN; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc = mfma32(a[u][q], b[u][q], acc);
        }
    }

    // Sum the waves in wave order.
    for (int ww = 0; ww < NW; ++ww) {
        if (w == ww) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                if (ww == 0) red[v * 64 + lane] = acc[v];
                else red[v * 64 + lane] += acc[v];
            }
        }
        __syncthreads();
    }
    const int ntiles = gridDim.y;
    float *mine = gpart + ((int64_t)blockIdx.x * ntiles + blockIdx.y) * 1024;
    for (int e = tid; e < 1024; e += 64 * NW) mine[e] = red[e];
    if (G == nullptr) return;   // the consumer sums the partial tiles itself
    __threadfence();
    __syncthreads();
    if (tid == 0) ticket_s = atomicAdd(&counters[blockIdx.y], 1u);
    __syncthreads();
    if (ticket_s != gridDim.x - 1) return;
    // Last block to arrive: every partial tile is visible after this fence.
    // Loads are issued in groups of eight so that they overlap; the sum runs
    // in block order whatever the arrival order was.
    __threadfence();
    const volatile float *vp = gpart;
    for (int e = tid; e < 1024; e += 64 * NW) {
        float s = 0.f;
        const int64_t stride = (int64_t)ntiles * 1024;
        const int64_t base = (int64_t)blockIdx.y * 1024 + e;
        unsigned b = 0;
        for (; b + 8 <= gridDim.x; b += 8) {
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = vp[base + (b + u) * stride];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += t[u];
        }
        for (; b < gridDim.x; ++b) s += vp[base + b * stride];
        const int v = e >> 6, l = e & 63;
        const int r1 = 32 * t1 + acc_row(v, l >> 5), r2 = 32 * t2 + (l & 31);
        if (r1 < k && r2 < k) G[r1 * k + r2] = s;
    }
    if (tid == 0) counters[blockIdx.y] = 0u;
}

// Side job of the pass kernels: the Gram tiles a finisher left behind (nsets sets of
// kt x kt tiles of 1024 floats) are needed, summed, by the finisher AFTER this pass.  The
// first workgroups of the pass add them up in groups of kGramGroup sets (in set order) so
// that the finisher has at most kFinMaxBlocks / kGramGroup sets to sum and no separate
// launch is needed.  Job j = a quarter of the entries of group j / 4, dealt to the workgroups in order.
__device__ __forceinline__ void sum_tile_groups(const float *__restrict__ gtiles, int nsets, int k,
                                                float *__restrict__ gsum)
{
    const int ngroups = (nsets + kGramGroup - 1) / kGramGroup;
    const int kt = (k + 31) >> 5;
    const int stride = kt * kt * 1024;
    const int nwg = gridDim.x * gridDim.y;
    for (int job = blockIdx.y * gridDim.x + blockIdx.x; job < 4 * ngroups; job += nwg) {
        const int group = job >> 2, quarter = job & 3;
        const int first = group * kGramGroup;
        const int count = (nsets - first < kGramGroup) ? nsets - first : kGramGroup;
        for (int e = quarter * (stride / 4) + threadIdx.x; e < (quarter + 1) * (stride / 4); e += blockDim.x) {
            float t[kGramGroup];
#pragma unroll
            for (int b = 0; b < kGramGroup; ++b) t[b] = gtiles[(int64_t)(first + (b < count ? b : 0)) * stride + e];
            float sum = 0.f;
#pragma unroll
            for (int b = 0; b < kGramGroup; ++b) sum += (b < count) ? t[b] : 0.f;
            gsum[(int64_t)group * stride + e] = sum;
        }
    }
}

// ---------------------------------------------------------------------------
// W^T A pass.  Workgroup = 4 waves on one 128-column slab of A and one row
// split; wave w takes row pairs w, w+4, ... of the split.  Per row pair a lane
// loads four consecutive columns (one 16-byte load, 512 contiguous bytes per
// row and wave) and one element of each W row; column tile q of the wave
// therefore holds columns j0 + 4 jj + q.  MFMA roles: A_op = W rows (factor
// index across lanes), B_op = A elements (column across lanes), reduction
// over the two rows.  The waves are summed through LDS in wave order and the
// slab is written (or added) to the split's partial result.
// Registers are capped (OCC waves per SIMD) so that several workgroups share a
// compute unit: one group's reduction epilogue then hides behind the others'
// streaming, and enough loads are in flight to cover the HBM latency.
// ---------------------------------------------------------------------------
template <int KT, int U, int OCC, bool VEC>
__global__ __launch_bounds__(64 * kWtaWaves, OCC) void wta_pass_kernel(const float *__restrict__ A,
                                                       const float *__restrict__ W,
                                                       float *__restrict__ ppart, int64_t rows,
                                                       int64_t n, int k, int64_t rps,
                                                       int accumulate,
                                                       const float *__restrict__ gtiles, int nsets,
                                                       float *__restrict__ gsum)
{
    constexpr int NW = kWtaWaves;
    constexpr int LD = 132;
    __shared__ float red[KT * 32 * LD];
    if (gtiles) sum_tile_groups(gtiles, nsets, k, gsum);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int jj = lane & 31, half = lane >> 5;
    const int64_t j0 = (int64_t)blockIdx.x * kWtaCols;
    const int64_t col = j0 + 4 * jj;
    const int64_t r0 = (int64_t)blockIdx.y * rps;
    const int64_t r1 = (r0 + rps < rows) ? r0 + rps : rows;

    f32x16 acc[KT][4];
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[t][q] = f32x16{0};

    struct Stage {
        f32x4 a[U];
        float wv[U][KT];
    };
    auto load_stage = [&](Stage &s, int64_t ibase) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = ibase + 2 * NW * u + half;
            const bool ok = row < r1;
            s.a[u] = load4<VEC>(A, n, row, col, ok);
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const int c = 32 * t + jj;
                const bool in = ok && c < k;
                const float wv = W[in ? row * k + c : 0];
                s.wv[u][t] = in ? wv : 0.f;
            }
        }
    };
    const int64_t step = 2 * NW * U;
    Stage cur, nxt;
    int64_t i = r0 + 2 * w;
    load_stage(cur, i);
    for (; i < r1; i += step) {
        load_stage(nxt, i + step);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    acc[t][q] = mfma32(cur.wv[u][t], cur.a[u][q], acc[t][q]);
        cur = nxt;
    }

    for (int ww = 0; ww < NW; ++ww) {
        if (w == ww) {
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int idx = (32 * t + acc_row(v, half)) * LD + q * 32 + jj;
                        if (ww == 0) red[idx] = acc[t][q][v];
                        else red[idx] += acc[t][q][v];
                    }
        }
        __syncthreads();
    }
    float *dst = ppart + (int64_t)blockIdx.y * k * n;
    for (int e = tid; e < k * kWtaCols; e += 64 * NW) {
        const int c = e >> 7, x = e & 127;
        const int64_t cj = j0 + x;
        if (cj < n) {
            float val = red[c * LD + (x & 3) * 32 + (x >> 2)];
            float *p = dst + (int64_t)c * n + cj;
            if (accumulate) val += *p;
            *p = val;
        }
    }
}

// ---------------------------------------------------------------------------
// Piece planes of kc <= kp columns c0 .. c0 + kc - 1 of a factor X (rows x ld,
// row-major), the A_op of the passes below; kp = 32 or 64 factor slots per row group:
// planes[(g * 3 + p) * kp + c] = the eight bf16 p-th pieces (p = 0: h, 1: m, 2: l)
// of X[8 g .. 8 g + 7][c0 + c], c < kp; rows beyond `rows` and columns beyond kc are zero.
// ---------------------------------------------------------------------------
// blockIdx.y = slice: columns c0 + kp * slice onwards (at most kp of the k left), planes + slice * slice_planes.
__global__ __launch_bounds__(256) void split_planes_kernel(const float *__restrict__ X, int64_t rows,
                                                           int64_t ld, int64_t c0, int k, int kp,
                                                           u32x4 *__restrict__ planes, int64_t slice_planes)
{
    c0 += (int64_t)kp * blockIdx.y;
    k -= kp * (int)blockIdx.y;
    if (k > kp) k = kp;
    planes += (int64_t)blockIdx.y * slice_planes;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t g = t / kp;
    const int c = (int)(t % kp);
    if (g * 8 >= rows) return;
    u32x4 o[3];
#pragma unroll
    for (int pr = 0; pr < 4; ++pr) {
        unsigned h[2], m[2], l[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int64_t row = g * 8 + 2 * pr + e;
            const float x = (row < rows && c < k) ? X[row * ld + c0 + c] : 0.f;
            split3(x, h[e], m[e], l[e]);
        }
        o[0][pr] = pack2(h[0], h[1]);
        o[1][pr] = pack2(m[0], m[1]);
        o[2][pr] = pack2(l[0], l[1]);
    }
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) planes[(g * 3 + pl) * kp + c] = o[pl];
}

// ---------------------------------------------------------------------------
// W^T A pass for k <= 32 with exact products on the bf16 matrix cores (see
// split3 above).  Geometry as wta_pass_kernel: 4 waves on a 128-column slab and
// one row split, lane = 4 consecutive columns; but a wave takes 16 rows per step
// (half-wave = 8 consecutive rows, the reduction depth of one instruction), loads
// them with eight 16-byte loads per lane, cuts each element into its pieces in
// registers and reads the pieces of W ready-made (planes, 3 x 16 bytes per lane
// and step).  Per column tile the eight piece products are accumulated smallest
// first.  r0 of every split is a multiple of 16 (rps is), so a half-wave's rows
// are one 8-row group of the planes.  Two waves per SIMD (256 registers each).
// ---------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(64 * kWtaWaves, 2) void wta_pass_split_kernel(
    const float *__restrict__ A, const u32x4 *__restrict__ planes, float *__restrict__ ppart,
    int64_t rows, int64_t n, int k, int64_t rps, int accumulate,
    const float *__restrict__ gtiles, int nsets, float *__restrict__ gsum)
{
    constexpr int NW = kWtaWaves;
    __shared__ float tot[NW * kTotFloats];
    if (gtiles) sum_tile_groups(gtiles, nsets, k, gsum);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    float *mytot = tot + w * kTotFloats;
    tot_clear(mytot, lane);
    const int jj = lane & 31, half = lane >> 5;
    const int64_t j0 = (int64_t)blockIdx.x * kWtaCols;
    const int64_t col = j0 + 4 * jj;
    const int64_t r0 = (int64_t)blockIdx.y * rps;
    const int64_t r1 = (r0 + rps < rows) ? r0 + rps : rows;

    f32x16 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = f32x16{0};

    struct Stage {
        f32x4 a[8];
        u32x4 wt[3];
    };
    auto load_stage = [&](Stage &s, int64_t ibase) {
        const int64_t rb = ibase + 8 * half;
#pragma unroll
        for (int r = 0; r < 8; ++r) s.a[r] = load4<VEC>(A, n, rb + r, col, rb + r < r1);
        // rows at or beyond r1 contribute nothing because their A elements read as zero
        const int64_t g = rb >> 3;
        const bool okg = rb < r1;
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) s.wt[pl] = planes[okg ? (g * 3 + pl) * 32 + jj : 0];
    };
    const int64_t step = 16 * NW;
    Stage cur, nxt;
    int64_t i = r0 + 16 * w;
    int steps = 0;
    load_stage(cur, i);
    for (; i < r1; i += step) {
        if (++steps > kFlushSteps) {
            tot_flush4(mytot, acc, lane);
            steps = 1;
        }
        load_stage(nxt, i + step);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32x4 at[3];
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                unsigned h0, m0, l0, h1, m1, l1;
                split3(cur.a[2 * pr][q], h0, m0, l0);
                split3(cur.a[2 * pr + 1][q], h1, m1, l1);
                at[0][pr] = pack2(h0, h1);
                at[1][pr] = pack2(m0, m1);
                at[2][pr] = pack2(l0, l1);
            }
            acc[q] = mfma_bf16(cur.wt[2], at[1], acc[q]);      // eight products, smallest first (no l l)
            acc[q] = mfma_bf16(cur.wt[1], at[2], acc[q]);
            acc[q] = mfma_bf16(cur.wt[2], at[0], acc[q]);
            acc[q] = mfma_bf16(cur.wt[1], at[1], acc[q]);
            acc[q] = mfma_bf16(cur.wt[0], at[2], acc[q]);
            acc[q] = mfma_bf16(cur.wt[1], at[0], acc[q]);
            acc[q] = mfma_bf16(cur.wt[0], at[1], acc[q]);
            acc[q] = mfma_bf16(cur.wt[0], at[0], acc[q]);
        }
        cur = nxt;
    }

    tot_flush4(mytot, acc, lane);
    __syncthreads();
    float *dst = ppart + (int64_t)blockIdx.y * k * n;
    for (int e = tid; e < k * kWtaCols; e += 64 * NW) {
        const int c = e >> 7, x = e & 127;
        const int64_t cj = j0 + x;
        if (cj < n) {
            float val = tot_sum4(tot, c, x);
            float *p = dst + (int64_t)c * n + cj;
            if (accumulate) val += *p;
            *p = val;
        }
    }
}

// ---------------------------------------------------------------------------
// The same pass for 16-byte aligned A with n % 4 == 0 and 64 n < 2^31, on buffer
// loads: per 16-row step a wave builds one descriptor over those rows (base
// A + first row, extent = the rows that exist in this split) and every lane
// loads row r at byte offset (8 half + r) * 4 n + 4 col from it.  Rows past the
// end of the split are outside the extent and read as zero, without a compare
// or select per load, and the addresses cost one VALU add per load.  The planes
// are read the same way (extent = the 8-row groups that exist).  Two steps are
// written out so that the staging registers alternate without copies.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64 * kWtaWaves, 2) void wta_pass_split_buf_kernel(
    const float *__restrict__ A, const u32x4 *__restrict__ planes, float *__restrict__ ppart,
    int64_t rows, int64_t n, int k, int64_t rps, int accumulate,
    const float *__restrict__ gtiles, int nsets, float *__restrict__ gsum)
{
    constexpr int NW = kWtaWaves;
    constexpr int kRsrcFlags = 0x00020000;   // raw buffer, 32-bit data format (gfx9 family)
    __shared__ float tot[NW * kTotFloats];
    if (gtiles) sum_tile_groups(gtiles, nsets, k, gsum);
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    float *mytot = tot + w * kTotFloats;
    tot_clear(mytot, lane);
    const int jj = lane & 31, half = lane >> 5;
    const int64_t j0 = (int64_t)blockIdx.x * kWtaCols;
    int64_t col = j0 + 4 * jj;
    if (col >= n) col = 0;   // lanes past the edge read valid data that is never stored
    const int64_t r0 = (int64_t)blockIdx.y * rps;
    const int64_t r1 = (r0 + rps < rows) ? r0 + rps : rows;
    const unsigned rowb = (unsigned)(n * 4);
    const unsigned loff = (unsigned)(half * 8) * rowb + (unsigned)col * 4;
    const unsigned poff = (unsigned)(half * 3 * 32 + jj) * 16;
    const int64_t ngroups = (rows + 7) >> 3;

    f32x16 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = f32x16{0};

    struct Stage {
        u32x4 a[8];
        u32x4 wt[3];
    };
    auto load_stage = [&](Stage &s, int64_t ib) {
        int64_t av = r1 - ib;                       // rows of this step inside the split
        av = av < 0 ? 0 : (av > 16 ? 16 : av);
        const int64_t g = ib >> 3;
        int64_t ng = av ? ngroups - g : 0;          // 8-row groups of planes that exist
        ng = ng < 0 ? 0 : (ng > 2 ? 2 : ng);
        const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float *>(A + (av ? ib : 0) * n), 0, (int)(av * rowb), kRsrcFlags);
        const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<u32x4 *>(planes + (ng ? g : 0) * 3 * 32), 0, (int)(ng * 3 * 32 * 16), kRsrcFlags);
#pragma unroll
        for (int r = 0; r < 8; ++r) s.a[r] = __builtin_amdgcn_raw_buffer_load_b128(ra, loff + r * rowb, 0, kStreamLoad);
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) s.wt[pl] = __builtin_amdgcn_raw_buffer_load_b128(rp, poff + pl * 32 * 16, 0, 0);
    };
    auto compute = [&](const Stage &c) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32x4 at[3];
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                unsigned h0, m0, l0, h1, m1, l1;
                split3(__uint_as_float(c.a[2 * pr][q]), h0, m0, l0);
                split3(__uint_as_float(c.a[2 * pr + 1][q]), h1, m1, l1);
                at[0][pr] = pack2(h0, h1);
                at[1][pr] = pack2(m0, m1);
                at[2][pr] = pack2(l0, l1);
            }
            acc[q] = mfma_bf16(c.wt[2], at[1], acc[q]);      // eight products, smallest first (no l l)
            acc[q] = mfma_bf16(c.wt[1], at[2], acc[q]);
            acc[q] = mfma_bf16(c.wt[2], at[0], acc[q]);
            acc[q] = mfma_bf16(c.wt[1], at[1], acc[q]);
            acc[q] = mfma_bf16(c.wt[0], at[2], acc[q]);
            acc[q] = mfma_bf16(c.wt[1], at[0], acc[q]);
            acc[q] = mfma_bf16(c.wt[0], at[1], acc[q]);
            acc[q] = mfma_bf16(c.wt[0], at[0], acc[q]);
        }
    };
    const int64_t step = 16 * NW;
    Stage s0, s1;
    int64_t i = r0 + 16 * w;
    int pairs = 4 * w;   // the waves of a workgroup flush at different times
    load_stage(s0, i);
    while (i < r1) {
        load_stage(s1, i + step);
        compute(s0);
        i += step;
        if (i >= r1) break;
        load_stage(s0, i + step);
        compute(s1);
        i += step;
        if (++pairs == kFlushSteps / 2) {
            tot_flush4(mytot, acc, lane);
            pairs = 0;
        }
    }

    tot_flush4(mytot, acc, lane);
    __syncthreads();
    float *dst = ppart + (int64_t)blockIdx.y * k * n;
    for (int e = tid; e < k * kWtaCols; e += 64 * NW) {
        const int c = e >> 7, x = e & 127;
        const int64_t cj = j0 + x;
        if (cj < n) {
            float val = tot_sum4(tot, c, x);
            float *p = dst + (int64_t)c * n + cj;
            if (accumulate) val += *p;
            *p = val;
        }
    }
}

// ---------------------------------------------------------------------------
// The pass for 32 < k <= 64 on exact pieces (aligned A, n % 4 == 0, 64 n < 2^31; planes with
// 64 factor slots per row group).  The arithmetic of wta_pass_split_buf_kernel with two
// 32-factor accumulator tiles per column tile, and another geometry: workgroup = 256
// columns, wave w = columns 64 w .. 64 w + 63 of them (lane = 2 consecutive columns, 8-byte
// loads), and all four waves walk the same 16-row steps of the split.  The piece planes of
// a step (1.5 times the bytes of the step's A) are then fetched from L2 once per workgroup
// and hit the vector cache for the other three waves, no sum across waves is needed, and
// each wave stores its own 64 x 64 result: register v of tile (t, q) is factor
// 32 t + row(v), column 2 jj + q, so (q = 0, q = 1) pair up to 8-byte stores, 256
// contiguous bytes per row.  Loads run two steps ahead of the arithmetic (three register
// stages), held there by scheduling barriers.  Measured on 32768 x 16384, k = 64: 490 us
// against 531 us for waves interleaved down the rows of one 64-column slab; the matrix
// pipe is busy 70 % of the cycles at the 1.7 GHz the chip sustains under this load.
// ---------------------------------------------------------------------------
// Several 64-factor slices of a wider factor in one launch (SLICES; ranks above 64): a
// one-dimensional grid whose workgroup L stands for (tile, slice) with the slices of one
// tile of A (slab x row split) 8 workgroups apart, i.e. on the same XCD at about the same
// time, so that A comes from HBM once and from that XCD's L2 for the other slices (loaded
// with the default cache policy then; a single slice streams A non-temporally).  Slice z
// reads planes + z * slice_planes and writes ppart + z * slice_ppart; it holds
// min(64, ktotal - 64 z) factors.
template <bool SLICES>
__global__ __launch_bounds__(64 * kWtaWaves, 2) void wta_pass_split64_wide_kernel(
    const float *__restrict__ A, const u32x4 *__restrict__ planes, float *__restrict__ ppart,
    int64_t rows, int64_t n, int k, int64_t rps, int accumulate,
    const float *__restrict__ gtiles, int nsets, float *__restrict__ gsum,
    int gx, int gy, int nslices, int64_t slice_planes, int64_t slice_ppart)
{
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    constexpr int KP = 64;
    constexpr int kRsrcFlags = 0x00020000;   // raw buffer, 32-bit data format (gfx9 family)
    constexpr int kPolicy = SLICES ? 0 : kStreamLoad;
    __shared__ float tot[kWtaWaves * kTotFloats];
    int bx = blockIdx.x, by = blockIdx.y;
    if (SLICES) {
        const int L = blockIdx.x, within = L >> 3;
        const int z = within % nslices;
        const int t = (within / nslices) * 8 + (L & 7);
        if (t >= gx * gy) return;
        bx = t % gx;
        by = t / gx;
        planes += (int64_t)z * slice_planes;
        ppart += (int64_t)z * slice_ppart;
        k = (k - 64 * z < 64) ? k - 64 * z : 64;
    } else if (gtiles) {
        sum_tile_groups(gtiles, nsets, k, gsum);
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    float *mytot = tot + w * kTotFloats;   // register (t, q, v) of this lane at ((2 t + q) * 16 + v) * 64 + lane
    tot_clear(mytot, lane);
    const int jj = lane & 31, half = lane >> 5;
    const int64_t jw = (int64_t)bx * 256 + 64 * w;
    if (jw >= n) return;     // no barrier below: a wave wholly past the edge has nothing to do
    const int64_t colr = jw + 2 * jj;
    const int64_t col = colr < n ? colr : 0;   // lanes past the edge read valid data that is never stored
    const int64_t r0 = (int64_t)by * rps;
    const int64_t r1 = (r0 + rps < rows) ? r0 + rps : rows;
    const unsigned rowb = (unsigned)(n * 4);
    const unsigned loff = (unsigned)(half * 8) * rowb + (unsigned)col * 4;
    const unsigned poff = (unsigned)(half * 3 * KP + jj) * 16;
    const int64_t ngroups = (rows + 7) >> 3;

    f32x16 acc[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int q = 0; q < 2; ++q) acc[t][q] = f32x16{0};

    struct Stage {
        u32x2 a[8];
        u32x4 wt[2][3];
    };
    auto load_stage = [&](Stage &s, int64_t ib) {
        int64_t av = r1 - ib;                       // rows of this step inside the split
        av = av < 0 ? 0 : (av > 16 ? 16 : av);
        const int64_t g = ib >> 3;
        int64_t ng = av ? ngroups - g : 0;          // 8-row groups of planes that exist
        ng = ng < 0 ? 0 : (ng > 2 ? 2 : ng);
        const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float *>(A + (av ? ib : 0) * n), 0, (int)(av * rowb), kRsrcFlags);
        const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<u32x4 *>(planes + (ng ? g : 0) * 3 * KP), 0, (int)(ng * 3 * KP * 16), kRsrcFlags);
#pragma unroll
        for (int r = 0; r < 8; ++r) s.a[r] = __builtin_amdgcn_raw_buffer_load_b64(ra, loff + r * rowb, 0, kPolicy);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
                s.wt[t][pl] = __builtin_amdgcn_raw_buffer_load_b128(rp, poff + (pl * KP + 32 * t) * 16, 0, 0);
    };
    auto compute = [&](const Stage &c) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            u32x4 at[3];
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                unsigned h0, m0, l0, h1, m1, l1;
                split3(__uint_as_float(c.a[2 * pr][q]), h0, m0, l0);
                split3(__uint_as_float(c.a[2 * pr + 1][q]), h1, m1, l1);
                at[0][pr] = pack2(h0, h1);
                at[1][pr] = pack2(m0, m1);
                at[2][pr] = pack2(l0, l1);
            }
            constexpr int PW[8] = {2, 1, 2, 1, 0, 1, 0, 0}, PA[8] = {1, 2, 0, 1, 2, 0, 1, 0};   // smallest first, no l l
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int t = 0; t < 2; ++t) acc[t][q] = mfma_bf16(c.wt[t][PW[e]], at[PA[e]], acc[t][q]);
        }
    };
    // three steps per trip, loads two steps ahead; a step past the split loads nothing (zero
    // extent) and is skipped
    auto flush = [&]() {
        // a tile at a time: 16 reads in flight, then the adds, then the writes
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                float old[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) old[v] = mytot[((2 * t + q) * 16 + v) * 64 + lane];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    mytot[((2 * t + q) * 16 + v) * 64 + lane] = old[v] + acc[t][q][v];
                    acc[t][q][v] = 0.f;
                }
            }
    };
    Stage s0, s1, s2;
    int trips = 2 * w;   // the waves of a workgroup flush at different times
    load_stage(s0, r0);
    __builtin_amdgcn_sched_barrier(0);   // issue order = age order, also here: the waits in the loop count loads in flight
    load_stage(s1, r0 + 16);
    for (int64_t i = r0; i < r1; i += 48) {
        if (++trips > kFlushSteps / 3) {
            flush();
            trips = 1;
        }
        load_stage(s2, i + 32);
        __builtin_amdgcn_sched_barrier(0);
        compute(s0);
        __builtin_amdgcn_sched_barrier(0);
        load_stage(s0, i + 48);
        __builtin_amdgcn_sched_barrier(0);
        if (i + 16 < r1) compute(s1);
        __builtin_amdgcn_sched_barrier(0);
        load_stage(s1, i + 64);
        __builtin_amdgcn_sched_barrier(0);
        if (i + 32 < r1) compute(s2);
        __builtin_amdgcn_sched_barrier(0);
    }

    if (colr < n) {
        float *dst = ppart + (int64_t)by * k * n + colr;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int c = 32 * t + acc_row(v, half);
                if (c < k) {
                    f32x2 *p = reinterpret_cast<f32x2 *>(dst + (int64_t)c * n);
                    f32x2 val = {mytot[((2 * t) * 16 + v) * 64 + lane] + acc[t][0][v],
                                 mytot[((2 * t + 1) * 16 + v) * 64 + lane] + acc[t][1][v]};
                    if (accumulate) {
                        const f32x2 old = *p;
                        val.x += old.x;
                        val.y += old.y;
                    }
                    *p = val;
                }
            }
    }
}

// ---------------------------------------------------------------------------
// Factor update ("finisher").  For X (k x len), partials of its numerator and
// the Gram matrix G of the other factor:
//     X[c][j] <- X[c][j] * (sum_s part[s][c][j]) / (sum_d G[c][d] X[d][j] + eps).
// With X = H, part = W^T A, G = W^T W this is the H-update line of Algorithm 3;
// with X = W^T, part = (A H^T)^T, G = H H^T it is the W-update line.
// A block covers 64 columns at a time; thread (column j, group g of 8) holds
// the old column in registers and produces factor indices c = g, g+8, ...
// Every element is written by the thread that computed it, after a block
// barrier that follows all reads of the old column.
// G comes either complete (Gfull, ld k) or as `nbin` partial 32 x 32 tiles in
// accumulator layout (gin), which every block sums in block order while
// staging G into LDS.  Optional outputs: Xt (len x k), staged through LDS so a
// block stores one contiguous run of 64 k floats, and gout: this block's
// partial Gram tiles of the NEW X (X X^T), computed from the LDS copy (one tile: the
// same register as both MFMA operands; four tiles at 33 to 64 factors: each wave one
// tile over half of a chunk's columns); the next finisher consumes them, so no
// separate Gram kernel and no cross-block reduction are needed.  With
// part == nullptr (and splits == 0) nothing is updated and only gout is produced.
// ---------------------------------------------------------------------------
template <int KP>
__global__ __launch_bounds__(512) void factor_update_kernel(float *X, float *Xt,
                                                            const float *__restrict__ part,
                                                            int splits,
                                                            const float *__restrict__ Gfull,
                                                            const float *__restrict__ gin, int nbin,
                                                            float *__restrict__ gout,
                                                            u32x4 *__restrict__ planes,
                                                            double *__restrict__ dpart, int k,
                                                            int64_t len, float eps, BlockMap bm)
{
    constexpr int NW = 8, KT = KP / 32 > 0 ? KP / 32 : 1, NC = (KP + 7) / 8, LD = KP + 1;
    constexpr int LDT = 32 * KT + 1;   // the Gram tiles read 32 factor indices per tile
    // one LDS array: G and the chunk's new values during the updates, then (after a barrier)
    // the eight waves' copies of a Gram tile for the sum over waves
    constexpr int GS = KP * LD, TS = 64 * LDT;
    constexpr int SM = (GS + TS > NW * 1024) ? GS + TS : NW * 1024;
    __shared__ float Sm[SM];
    float *Gs = Sm, *Ts = Sm + GS;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int kt = (k + 31) >> 5;

    // A thread's entries of G (8 at KP = 64) are independent: the loads of up to four entries are
    // requested together, kGramGroup sets per entry at a time (each trip to L2 costs a microsecond
    // here), and each entry's sets are added in set order.
    constexpr int EPT = (KP * KP + 64 * NW - 1) / (64 * NW), EG = EPT < 4 ? EPT : 4;
    for (int i0 = 0; i0 < EPT; i0 += EG) {
        float gv[EG];
        const float *src[EG];
        bool use[EG];
        const int64_t stride = (int64_t)kt * kt * 1024;
#pragma unroll
        for (int i = 0; i < EG; ++i) {
            const int e = tid + 64 * NW * (i0 + i);
            const int c = e / KP, d = e % KP;
            // Stacked independent runs: factor indices of different runs do not interact.
            use[i] = e < KP * KP && c < k && d < k && (!bm.on || bm.id[c] == bm.id[d]);
            const int r1 = c & 31, r2 = d & 31;
            const int pos = ((r1 & 3) + 4 * (r1 >> 3)) * 64 + r2 + 32 * ((r1 >> 2) & 1);
            src[i] = Gfull ? Gfull + (use[i] ? c * k + d : 0)
                           : gin + (use[i] ? (int64_t)((c >> 5) * kt + (d >> 5)) * 1024 + pos : 0);
            gv[i] = 0.f;
        }
        if (Gfull) {
#pragma unroll
            for (int i = 0; i < EG; ++i) gv[i] = *src[i];
        } else {
            for (int b = 0; b < nbin; b += kGramGroup) {
                float t[EG][kGramGroup];
#pragma unroll
                for (int i = 0; i < EG; ++i)
#pragma unroll
                    for (int u = 0; u < kGramGroup; ++u) t[i][u] = src[i][(b + u < nbin ? b + u : 0) * stride];
#pragma unroll
                for (int i = 0; i < EG; ++i)
#pragma unroll
                    for (int u = 0; u < kGramGroup; ++u) gv[i] += b + u < nbin ? t[i][u] : 0.f;
            }
        }
#pragma unroll
        for (int i = 0; i < EG; ++i) {
            const int e = tid + 64 * NW * (i0 + i);
            if (e < KP * KP) Gs[(e / KP) * LD + e % KP] = use[i] ? gv[i] : 0.f;
        }
    }
    __syncthreads();

    // Gram tiles of the new X.  One tile (KT = 1): every wave adds up its share of the columns.
    // Four tiles (KT = 2): wave w adds up tile w % 4 over half w / 4 of a chunk's columns, which
    // leaves one accumulator per wave and one round through LDS at the end instead of four.
    constexpr bool G2 = KT == 2;
    f32x16 acc = {0};

    const int jl = lane, grp = w;
    double dacc = 0.0;   // sum over this thread's entries of numerator x new value (objective monitor)
    const int64_t nchunks = (len + 63) >> 6;
    for (int64_t ch = blockIdx.x; ch < nchunks; ch += gridDim.x) {
        const int64_t j = ch * 64 + jl;
        const bool okj = j < len;
        float h[KP];
#pragma unroll
        for (int d = 0; d < KP; ++d) {
            const bool in = okj && d < k;
            const float v = X[in ? (int64_t)d * len + j : 0];
            h[d] = in ? v : 0.f;
        }
        float p[NC];
#pragma unroll
        for (int ci = 0; ci < NC; ++ci) p[ci] = 0.f;
        // Partial sums in split order; a few splits' loads are issued together.
        constexpr int SB = (KP > 32) ? 2 : 4;
        int s = 0;
        for (; s + SB <= splits; s += SB) {
            float t[SB][NC];
#pragma unroll
            for (int u = 0; u < SB; ++u)
#pragma unroll
                for (int ci = 0; ci < NC; ++ci) {
                    const int c = grp + 8 * ci;
                    const bool in = okj && c < k;
                    const float v = part[in ? ((int64_t)(s + u) * k + c) * len + j : 0];
                    t[u][ci] = in ? v : 0.f;
                }
#pragma unroll
            for (int u = 0; u < SB; ++u)
#pragma unroll
                for (int ci = 0; ci < NC; ++ci) p[ci] += t[u][ci];
        }
        for (; s < splits; ++s) {
#pragma unroll
            for (int ci = 0; ci < NC; ++ci) {
                const int c = grp + 8 * ci;
                const bool in = okj && c < k;
                const float v = part[in ? ((int64_t)s * k + c) * len + j : 0];
                p[ci] += in ? v : 0.f;
            }
        }
        __syncthreads();   // every old value of this chunk is in registers; Ts is free
#pragma unroll
        for (int ci = 0; ci < NC; ++ci) {
            const int c = grp + 8 * ci;
            if (c < k && part == nullptr) {
                // Gram-only mode: no update, the tiles of the current X are produced
                // with exactly the summation order an updating launch would use.
                const float v = X[okj ? (int64_t)c * len + j : 0];
                Ts[jl * LDT + c] = okj ? v : 0.f;
            } else if (c < k) {
                float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
                const float *g = Gs + c * LD;
#pragma unroll
                for (int d = 0; d < KP; d += 4) {
                    d0 += g[d + 0] * h[d + 0];
                    d1 += g[d + 1] * h[d + 1];
                    d2 += g[d + 2] * h[d + 2];
                    d3 += g[d + 3] * h[d + 3];
                }
                const float den = ((d0 + d1) + (d2 + d3)) + eps;
                float nv = 0.f;
                if (okj) {
                    const int64_t at = (int64_t)c * len + j;
                    nv = X[at] * p[ci] / den;
                    X[at] = nv;
                    dacc += (double)p[ci] * (double)nv;
                }
                Ts[jl * LDT + c] = nv;   // columns past the end contribute zeros
            }
        }
        __syncthreads();
        if (Xt) {
            for (int e = tid; e < 64 * k; e += 64 * NW) {
                const int jj = e / k, c = e % k;
                if (ch * 64 + jj < len) Xt[(ch * 64 + jj) * k + c] = Ts[jj * LDT + c];
            }
        }
        constexpr int PKP = KP <= 32 ? 32 : 64;   // factor slots per row group of the planes
        if (planes && tid < 8 * PKP) {
            // bf16 piece planes of the new X^T rows of this chunk (layout of split_planes_kernel)
            const int gl = tid / PKP, c = tid % PKP;
            const int64_t grow = ch * 8 + gl;
            if (grow * 8 < len) {
                u32x4 o[3];
#pragma unroll
                for (int pr = 0; pr < 4; ++pr) {
                    unsigned hh[2], mm[2], ll[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const float x = (c < k) ? Ts[(8 * gl + 2 * pr + e) * LDT + c] : 0.f;
                        split3(x, hh[e], mm[e], ll[e]);
                    }
                    o[0][pr] = pack2(hh[0], hh[1]);
                    o[1][pr] = pack2(mm[0], mm[1]);
                    o[2][pr] = pack2(ll[0], ll[1]);
                }
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) planes[(grow * 3 + pl) * PKP + c] = o[pl];
            }
        }
        if (gout && G2) {
            const int jj = lane & 31, half = lane >> 5;
            const int ta = (w & 3) >> 1, tb = w & 1, hb = w >> 2;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int row = 32 * hb + 2 * q + half;    // column pair of this chunk
                acc = mfma32(Ts[row * LDT + 32 * ta + jj], Ts[row * LDT + 32 * tb + jj], acc);
            }
        } else if (gout) {
            const int jj = lane & 31, half = lane >> 5;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row = 2 * (w + NW * q) + half;   // column pair of this chunk
                const float va = Ts[row * LDT + jj];
                acc = mfma32(va, va, acc);
            }
        }
    }
    if (dpart) {
        // <numerator, new X> of this block, summed in a fixed order (waves, then lanes by tree)
        __shared__ double dsum[NW];
        for (int off = 32; off > 0; off >>= 1) dacc += __shfl_xor(dacc, off);
        if (lane == 0) dsum[w] = dacc;
        __syncthreads();
        if (tid == 0) {
            double t = 0.0;
            for (int i = 0; i < NW; ++i) t += dsum[i];
            dpart[blockIdx.x] = t;
        }
    }
    if (!gout) return;
    __syncthreads();   // the last chunk's readers of Ts are done: Sm changes hands
    // Rows and columns of a tile at factor indices >= k hold whatever LDS held;
    // consumers never read them.
    // every wave parks its tile, then all threads add the copies in wave order: the two halves
    // of each of four tiles, or the eight shares of the one tile
#pragma unroll
    for (int v = 0; v < 16; ++v) Sm[w * 1024 + v * 64 + lane] = acc[v];
    __syncthreads();
    if (G2) {
        for (int e = tid; e < 4096; e += 64 * NW) {
            const int a = e >> 11, b = (e >> 10) & 1;
            if (a < kt && b < kt) gout[((int64_t)blockIdx.x * kt * kt + a * kt + b) * 1024 + (e & 1023)] = Sm[e] + Sm[4096 + e];
        }
    } else {
        float *dst = gout + (int64_t)blockIdx.x * 1024;
        for (int e = tid; e < 1024; e += 64 * NW) {
            float t = Sm[e];
#pragma unroll
            for (int ww = 1; ww < NW; ++ww) t += Sm[ww * 1024 + e];
            dst[e] = t;
        }
    }
}

// ---------------------------------------------------------------------------
// A H^T pass with the W update fused.  Workgroup = 8 waves on RT*32 rows of A;
// the waves split the columns in groups of 32 (one 128-byte line per row).
// MFMA roles: A_op = A elements (row across lanes), B_op = H elements (factor
// index across lanes), reduction over two columns; a lane's 16-byte load gives
// four instructions their operands, so both A and H are read with the same
// pattern: lane l, load u -> row l % 32, columns jb + 8u + 4 (l / 32) .. +3.
// Epilogue: waves summed through LDS in wave order, then
//   W[i][c] <- W[i][c] * Q[i][c] / (sum_d W[i][d] GH[d][c] + eps).
// dpart != nullptr: dpart[blockIdx.x] = sum over the block's entries of Q x new W in double
// (its share of <A H^T, W_new> for the objective), lanes by butterfly, then the waves in order.
// ---------------------------------------------------------------------------
template <int KT, int RT, bool VEC>
__global__ __launch_bounds__(512) void aht_pass_kernel(const float *__restrict__ A,
                                                       const float *__restrict__ H,
                                                       const float *__restrict__ GH, float *W,
                                                       int64_t rows, int64_t n, int k, float eps,
                                                       double *__restrict__ dpart)
{
    constexpr int NW = kAhtWaves;
    constexpr int RB = 32 * RT;
    constexpr int KP = 32 * KT;
    constexpr int LDQ = KP + 1;
    __shared__ float Qs[RB * LDQ];
    __shared__ float Ws[RB * LDQ];
    __shared__ float Gs[KP * LDQ];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 31, half = lane >> 5;
    const int64_t i0 = (int64_t)blockIdx.x * RB;

    // Stage GH (zero padded) and the old W rows of this block.
    for (int e = tid; e < KP * KP; e += 512) {
        const int d = e / KP, c = e % KP;
        Gs[d * LDQ + c] = (d < k && c < k) ? GH[d * k + c] : 0.f;
    }
    for (int e = tid; e < RB * KP; e += 512) {
        const int i = e / KP, c = e % KP;
        Ws[i * LDQ + c] = (i0 + i < rows && c < k) ? W[(i0 + i) * k + c] : 0.f;
    }

    int64_t arow[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int64_t row = i0 + 32 * rt + r;
        arow[rt] = (row < rows) ? row : rows - 1;   // clamped rows are discarded below
    }

    f32x16 acc[RT][KT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int t = 0; t < KT; ++t) acc[rt][t] = f32x16{0};

    struct Stage {
        f32x4 a[RT][4];
        f32x4 h[KT][4];
    };
    auto load_stage = [&](Stage &s, int64_t g) {
        const int64_t jb = 32 * g + 4 * half;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) s.a[rt][u] = load4<VEC>(A, n, arow[rt], jb + 8 * u, true);
#pragma unroll
            for (int t = 0; t < KT; ++t) s.h[t][u] = load4<VEC>(H, n, 32 * t + r, jb + 8 * u, 32 * t + r < k);
        }
    };
    const int64_t ngroups = (n + 31) >> 5;
    Stage cur, nxt;
    int64_t g = w;
    load_stage(cur, g);
    for (; g < ngroups; g += NW) {
        load_stage(nxt, g + NW);   // columns >= n read as zero, no memory access
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int t = 0; t < KT; ++t)
                        acc[rt][t] = mfma32(cur.a[rt][u][q], cur.h[t][u][q], acc[rt][t]);
        cur = nxt;
    }

    for (int ww = 0; ww < NW; ++ww) {
        if (w == ww) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int t = 0; t < KT; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int idx = (32 * rt + acc_row(v, half)) * LDQ + 32 * t + r;
                        if (ww == 0) Qs[idx] = acc[rt][t][v];
                        else Qs[idx] += acc[rt][t][v];
                    }
        }
        __syncthreads();
    }

    double dacc = 0.0;
    for (int e = tid; e < RB * k; e += 512) {
        const int i = e / k, c = e % k;
        if (i0 + i < rows) {
            float d0 = 0.f, d1 = 0.f;
            for (int d = 0; d + 1 < k; d += 2) {
                d0 += Ws[i * LDQ + d] * Gs[d * LDQ + c];
                d1 += Ws[i * LDQ + d + 1] * Gs[(d + 1) * LDQ + c];
            }
            if (k & 1) d0 += Ws[i * LDQ + k - 1] * Gs[(k - 1) * LDQ + c];
            const float den = (d0 + d1) + eps;
            const float wn = Ws[i * LDQ + c] * Qs[i * LDQ + c] / den;
            W[(i0 + i) * k + c] = wn;
            dacc += (double)Qs[i * LDQ + c] * (double)wn;
        }
    }
    if (dpart) {     // uniform over the grid
        __shared__ double dsum[NW];
        for (int off = 32; off > 0; off >>= 1) dacc += __shfl_xor(dacc, off);
        if (lane == 0) dsum[w] = dacc;
        __syncthreads();
        if (tid == 0) {
            double t = 0.0;
            for (int ww = 0; ww < NW; ++ww) t += dsum[ww];
            dpart[blockIdx.x] = t;
        }
    }
}

// ---------------------------------------------------------------------------
// A H^T pass on the row-major A with the W update fused, k <= 32 KT ("row plan"; 16-byte aligned
// A, n % 4 == 0, n < 2^24; the text below describes KT = 1, the end of it what KT = 2 changes).  A workgroup of 8 waves owns 32 R rows of A and W at a time
// (row blocks blockIdx.x, + gridDim.x, ...); the waves split the 64-column chunks of the
// block between them, and a wave's sub-tile is 32 rows x 64 columns, R per chunk.  MFMA
// roles: A_op = A elements (32 rows x 16 columns, a lane holds 8 consecutive columns of one
// row, cut into bf16 pieces in registers), B_op = the piece planes of H^T (16 columns x 32
// factors: the planes the H update writes for its new H; the 48 registers of a chunk serve
// all R row tiles), so the sums are the exact-piece sums of the W^T A pass, and like there a
// matrix accumulator runs for at most 32 products deep (8 chunks) before it is added, in
// rounded fp32, to totals: here totals in LDS shared by the wave pairs (w, w + 4), because
// R accumulator tiles and R total tiles do not fit a wave's registers beside the planes.
// An operand layout with lanes down the rows would make every lane of a load touch its own
// cache line, so A is loaded coalesced (a wave instruction = 4 rows x 256 contiguous bytes,
// non-temporal) and turned through a wave-private 8 KiB tile of LDS (16-byte chunks
// swizzled by row, conflict free both ways; no barrier: only the wave itself touches its
// tile).  Every row block starts its walk over the columns at another chunk (17 x block
// index): launched in step on the same columns, the workgroups would crowd the same memory
// channels (0.338 against 0.318 ms for the bare loads on 32768 x 16384).
// LDS: 64 KiB of staging tiles + 16 R KiB of totals, dynamic (above the 64 KiB a static
// array may have; a workgroup may use all 160 KiB of a compute unit).
//
// Epilogue per row block: the four totals are added in order; W <- W * Q / (W GH + eps) for
// the block's rows with GH = H H^T (k x k, complete); then from the new rows in LDS: their
// bf16 piece planes (operand of the next W^T A pass), this workgroup's share of W^T W (fp32
// matrix instruction, one tile set per workgroup in gout, which the next W^T A pass adds up
// in groups) and, with dpart, its share of <A H^T, W_new> in double.
// KT = 2 (33 <= k <= 64): planes of 64 factor slots (96 registers per chunk), every cut of A
// feeds two accumulator chains, R = 2 (four accumulator tiles), 65-float rows in the epilogue,
// and the block's four tiles of W^T W are added to running tiles in LDS (wave w: tile w % 4
// over half w / 4 of the block's rows) instead of living in registers across row blocks.
// mode 1: no pass and no update, only the planes and the Gram share of W as it is (the
// same summation order, so that a run cut into two calls gives the same bits).  mode 2: the
// whole pass with the stores to W and its planes left out (timing).
// ---------------------------------------------------------------------------
extern __shared__ float aht_rows_lds[];
template <int R, int KT>
__global__ __launch_bounds__(512, 2) void aht_rows_kernel(
    const float *__restrict__ A, const u32x4 *__restrict__ planesH, const float *__restrict__ GH,
    float *W, u32x4 *__restrict__ planesW, float *__restrict__ gout,
    double *__restrict__ dpart, int64_t rows, int64_t n, int k, float eps, int mode, BlockMap bm)
{
    constexpr int NW = 8, RB = 32 * R, KP = 32 * KT, LDW = KP + 1, RT = R * KT * 1024;
    constexpr int kRsrcFlags = 0x00020000;   // raw buffer, 32-bit data format (gfx9 family)
    float *lds = aht_rows_lds;             // staging tiles: 8 x 2048 floats
    float *T = aht_rows_lds + NW * 2048;   // totals of the four wave pairs: 4 x (R x KT x 1024) floats
    float *Grun = T + 4 * RT;              // KT = 2: this workgroup's W^T W over its row blocks, 4 tiles
    double *dsum = reinterpret_cast<double *>(lds + 16368);      // used after the last row block only
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    float *stg = lds + w * 2048;
    const int jj = lane & 31, half = lane >> 5;
    const unsigned rowb = (unsigned)(n * 4);
    const int64_t nchunks = (n + 63) >> 6;
    const int64_t ngroups = (n + 7) >> 3;
    const int64_t nblocks = (rows + RB - 1) / RB;
    // coalesced loads: instruction u of a sub-tile covers rows 4u .. 4u+3, lane = (row, 16-byte chunk)
    const int lrow = lane >> 4, lch = lane & 15;
    const unsigned loff = (unsigned)lrow * rowb + (unsigned)lch * 16;
    // epilogue arrays (they alias the staging tiles; barriers separate the phases)
    float *Ws = lds;                      // old rows   [RB][LDW]
    float *Wn = lds + RB * LDW;           // new rows   [RB][LDW]
    float *Gs = lds + 2 * RB * LDW;       // H H^T      [KP][LDW]
    static_assert(2 * RB * LDW + KP * LDW <= 16368, "epilogue arrays must fit the staging tiles");
    f32x16 gacc = {0};                    // KT = 1: this wave's share of W^T W over all row blocks
    if (KT == 2)
        for (int e = tid; e < 4096; e += 64 * NW) Grun[e] = 0.f;   // first read after many barriers
    double dacc = 0.0;
    const int rounds = (int)((nchunks + 63) >> 6);   // a round = up to 8 chunks per wave

    for (int64_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const int64_t i0 = blk * RB;
        if (mode != 1) {
            const int64_t rot = (blk * 17) % nchunks;
            f32x16 acc[R][KT];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int ft = 0; ft < KT; ++ft) acc[r][ft] = f32x16{0};
            struct Stage { u32x4 a[8]; };
            auto phys = [&](int64_t ch) { const int64_t c = ch + rot; return c >= nchunks ? c - nchunks : c; };
            auto load_stage = [&](Stage &s, int64_t chl, int rt) {
                const int64_t rbase = i0 + 32 * rt;
                int64_t av = rows - rbase;                  // rows of this sub-tile that exist
                av = av < 0 ? 0 : (av > 32 ? 32 : av);
                if (chl >= nchunks) av = 0;                 // past the last chunk: nothing is loaded
                const int64_t ch = av ? phys(chl) : 0;
                const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<float *>(A + (av ? rbase * n + ch * 64 : 0)), 0,
                    (int)(av ? av * (int64_t)rowb - ch * 256 : 0), kRsrcFlags);
                // columns at or past n (last chunk only): the lane's offset is pushed out of range
                const unsigned lo = (ch * 64 + lch * 4 < n) ? loff : 0x7fffffffu;
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    s.a[u] = __builtin_amdgcn_raw_buffer_load_b128(ra, lo + (unsigned)(4 * u) * rowb, 0, kStreamLoad);
            };
            u32x4 bp[4][3][KT];
            auto load_b = [&](int64_t chl) {
                const int64_t g = phys(chl) * 8;
                int64_t ng = ngroups - g;                   // 8-column groups of planes that exist
                ng = ng < 0 ? 0 : (ng > 8 ? 8 : ng);
                const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<u32x4 *>(planesH + (ng ? g : 0) * 3 * KP), 0, (int)(ng * 3 * KP * 16), kRsrcFlags);
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int pl = 0; pl < 3; ++pl)
#pragma unroll
                        for (int ft = 0; ft < KT; ++ft)
                            bp[s][pl][ft] = __builtin_amdgcn_raw_buffer_load_b128(
                                rp, (unsigned)((((2 * s + half) * 3 + pl) * KP + 32 * ft + jj) * 16), 0, 0);
            };
            auto to_lds = [&](const Stage &s) {
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int row = 4 * u + lrow;
                    *reinterpret_cast<f32x4 *>(stg + row * 64 + ((lch ^ (row & 15)) << 2)) = __builtin_bit_cast(f32x4, s.a[u]);
                }
            };
            auto compute = [&](f32x16 (&a)[KT]) {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int c0 = 4 * s + 2 * half;
                    const f32x4 x0 = *reinterpret_cast<const f32x4 *>(stg + jj * 64 + ((c0 ^ (jj & 15)) << 2));
                    const f32x4 x1 = *reinterpret_cast<const f32x4 *>(stg + jj * 64 + (((c0 + 1) ^ (jj & 15)) << 2));
                    u32x4 at[3];
                    unsigned h0, m0, l0, h1, m1, l1;
                    split3(x0.x, h0, m0, l0); split3(x0.y, h1, m1, l1);
                    at[0][0] = pack2(h0, h1), at[1][0] = pack2(m0, m1), at[2][0] = pack2(l0, l1);
                    split3(x0.z, h0, m0, l0); split3(x0.w, h1, m1, l1);
                    at[0][1] = pack2(h0, h1), at[1][1] = pack2(m0, m1), at[2][1] = pack2(l0, l1);
                    split3(x1.x, h0, m0, l0); split3(x1.y, h1, m1, l1);
                    at[0][2] = pack2(h0, h1), at[1][2] = pack2(m0, m1), at[2][2] = pack2(l0, l1);
                    split3(x1.z, h0, m0, l0); split3(x1.w, h1, m1, l1);
                    at[0][3] = pack2(h0, h1), at[1][3] = pack2(m0, m1), at[2][3] = pack2(l0, l1);
                    // eight piece products (no l l), smallest first (per 32-factor tile: independent chains)
                    constexpr int PA[8] = {2, 1, 2, 1, 0, 1, 0, 0}, PB[8] = {1, 2, 0, 1, 2, 0, 1, 0};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
#pragma unroll
                        for (int ft = 0; ft < KT; ++ft) a[ft] = mfma_bf16(at[PA[e]], bp[s][PB[e]][ft], a[ft]);
                }
            };
            // Sub-tiles in the order (chunk, row tile); the loads of the next one are requested as soon
            // as the current one has gone to LDS.  After every round (8 chunks = 32 products deep) the
            // matrix accumulators are added, in rounded fp32, to totals in LDS that the waves w and w + 4
            // share: first the lower four waves, then the upper four, a barrier after each.
            Stage s0;
            load_stage(s0, w, 0);
            float *Tp = T + (w & 3) * RT;
            for (int r = 0; r < rounds; ++r) {
                for (int t = 0; t < 8; ++t) {
                    const int64_t ch = w + 8 * (int64_t)(8 * r + t);
                    if (ch >= nchunks) break;        // this wave has no more chunks (loads already requested nothing)
                    load_b(ch);
#pragma unroll
                    for (int rt = 0; rt < R; ++rt) {
                        to_lds(s0);
                        __builtin_amdgcn_sched_barrier(0);
                        if (rt + 1 < R) load_stage(s0, ch, rt + 1);
                        else load_stage(s0, ch + 8, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        compute(acc[rt]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (w < 4) {
#pragma unroll
                    for (int rt = 0; rt < R * KT; ++rt) {
                        float old[16];
#pragma unroll
                        for (int v = 0; v < 16; ++v) old[v] = r ? Tp[(rt * 16 + v) * 64 + lane] : 0.f;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            Tp[(rt * 16 + v) * 64 + lane] = old[v] + acc[rt / KT][rt % KT][v];
                            acc[rt / KT][rt % KT][v] = 0.f;
                        }
                    }
                }
                __syncthreads();
                if (w >= 4) {
#pragma unroll
                    for (int rt = 0; rt < R * KT; ++rt) {
                        float old[16];
#pragma unroll
                        for (int v = 0; v < 16; ++v) old[v] = Tp[(rt * 16 + v) * 64 + lane];
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            Tp[(rt * 16 + v) * 64 + lane] = old[v] + acc[rt / KT][rt % KT][v];
                            acc[rt / KT][rt % KT][v] = 0.f;
                        }
                    }
                }
                __syncthreads();
            }
            // the four pairs' totals, added in order, in place
            for (int e = tid; e < RT; e += 64 * NW)
                T[e] = ((T[e] + T[RT + e]) + T[2 * RT + e]) + T[3 * RT + e];
            __syncthreads();
        }
        // ---- H H^T and the block's rows of W ----
        if (mode != 1) {
            for (int e = tid; e < KP * KP; e += 64 * NW) {
                const int c = e / KP, d = e % KP;
                // stacked independent runs: factor indices of different runs do not interact
                const bool in = c < k && d < k && (!bm.on || bm.id[c] == bm.id[d]);
                const float v = GH[in ? c * k + d : 0];
                Gs[c * LDW + d] = in ? v : 0.f;
            }
        }
        for (int e = tid; e < RB * KP; e += 64 * NW) {
            const int i = e / KP, c = e % KP;
            const bool in = i0 + i < rows && c < k;
            const float v = W[in ? (i0 + i) * k + c : 0];
            (mode != 1 ? Ws : Wn)[i * LDW + c] = in ? v : 0.f;
        }
        __syncthreads();
        if (mode != 1) {
            for (int e = tid; e < RB * KP; e += 64 * NW) {
                const int i = e / KP, c = e % KP;
                float wn = 0.f;
                if (i0 + i < rows && c < k) {
                    float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
                    const float *wr = Ws + i * LDW;
#pragma unroll
                    for (int d = 0; d < KP; d += 4) {
                        d0 += wr[d + 0] * Gs[(d + 0) * LDW + c];
                        d1 += wr[d + 1] * Gs[(d + 1) * LDW + c];
                        d2 += wr[d + 2] * Gs[(d + 2) * LDW + c];
                        d3 += wr[d + 3] * Gs[(d + 3) * LDW + c];
                    }
                    const float den = ((d0 + d1) + (d2 + d3)) + eps;
                    const int r = i & 31;
                    const float q = T[(((i >> 5) * KT + (c >> 5)) * 16 + ((r & 3) | ((r >> 3) << 2))) * 64 + 32 * ((r >> 2) & 1) + (c & 31)];
                    wn = wr[c] * q / den;
                    if (mode == 0) W[(i0 + i) * k + c] = wn;
                    dacc += (double)q * (double)wn;
                }
                Wn[i * LDW + c] = wn;
            }
            __syncthreads();
        }
        // ---- by-products of the new rows: piece planes, Gram share ----
        if (tid < (RB / 8) * KP) {
            const int gl = tid / KP, c = tid % KP;
            const int64_t grow = (i0 >> 3) + gl;
            if (grow * 8 < rows && mode != 2) {
                u32x4 o[3];
#pragma unroll
                for (int pr = 0; pr < 4; ++pr) {
                    unsigned hh[2], mm[2], ll[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) split3(Wn[(8 * gl + 2 * pr + e) * LDW + c], hh[e], mm[e], ll[e]);
                    o[0][pr] = pack2(hh[0], hh[1]);
                    o[1][pr] = pack2(mm[0], mm[1]);
                    o[2][pr] = pack2(ll[0], ll[1]);
                }
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) planesW[(grow * 3 + pl) * KP + c] = o[pl];
            }
        }
        if (KT == 1) {
#pragma unroll
            for (int q = 0; q < RB / 16; ++q) {
                const float va = Wn[(2 * (w + NW * q) + half) * LDW + jj];
                gacc = mfma32(va, va, gacc);
            }
        } else {
            // the block's share of the four tiles of W^T W: wave w takes tile w % 4 over the rows of
            // half w / 4 of the block; the two halves meet in the (now free) totals and are added,
            // in order, to the running tiles
            const int ta = (w & 3) >> 1, tb = w & 1, hb = w >> 2;
            f32x16 g2 = {0};
#pragma unroll
            for (int q = 0; q < RB / 4; ++q) {
                const int row = hb * (RB / 2) + 2 * q + half;
                g2 = mfma32(Wn[row * LDW + 32 * ta + jj], Wn[row * LDW + 32 * tb + jj], g2);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) T[hb * 4096 + (w & 3) * 1024 + v * 64 + lane] = g2[v];
            __syncthreads();
            for (int e = tid; e < 4096; e += 64 * NW) Grun[e] += T[e] + T[4096 + e];
        }
        __syncthreads();                           // LDS goes back to the staging tiles
    }
    if (dpart) {
        for (int off = 32; off > 0; off >>= 1) dacc += __shfl_xor(dacc, off);
        if (lane == 0) dsum[w] = dacc;
        __syncthreads();
        if (tid == 0) { double t = 0.0; for (int i = 0; i < NW; ++i) t += dsum[i]; dpart[blockIdx.x] = t; }
    }
    if (KT == 1) {
        // this workgroup's share of W^T W: the eight waves' tiles added in wave order
#pragma unroll
        for (int v = 0; v < 16; ++v) lds[w * 1024 + v * 64 + lane] = gacc[v];
        __syncthreads();
        for (int e = tid; e < 1024; e += 64 * NW) {
            float t = lds[e];
#pragma unroll
            for (int ww = 1; ww < NW; ++ww) t += lds[ww * 1024 + e];
            gout[(int64_t)blockIdx.x * 1024 + e] = t;
        }
    } else {
        for (int e = tid; e < 4096; e += 64 * NW) gout[(int64_t)blockIdx.x * 4096 + e] = Grun[e];
    }
}

// G (k x k, ld k) = sum over nb sets of partial 32 x 32 tiles (accumulator layout).
// Eight lanes share one entry: lane q adds sets q, q+8, ... in order, then the
// eight sums are combined in a fixed tree, so the result does not depend on timing.
__global__ __launch_bounds__(256) void gram_sum_kernel(const float *__restrict__ gpart, int nb, int k,
                                                       float *__restrict__ G)
{
    const int kt = (k + 31) >> 5;
    const int64_t stride = (int64_t)kt * kt * 1024;
    const int gid = blockIdx.x * 256 + threadIdx.x;
    const int entry = gid >> 3, q = gid & 7;
    const bool ok = entry < kt * kt * 1024;
    const float *src = gpart + (ok ? entry : 0);
    float s = 0.f;
    int b = q;
    for (; b + 24 < nb; b += 32) {
        const float t0 = src[(b + 0) * stride], t1 = src[(b + 8) * stride];
        const float t2 = src[(b + 16) * stride], t3 = src[(b + 24) * stride];
        s += t0;
        s += t1;
        s += t2;
        s += t3;
    }
    for (; b < nb; b += 8) s += src[b * stride];
    s += __shfl_xor(s, 1, 8);
    s += __shfl_xor(s, 2, 8);
    s += __shfl_xor(s, 4, 8);
    if (ok && q == 0) {
        const int tile = entry >> 10, e = entry & 1023;
        const int v = e >> 6, l = e & 63;
        const int r1 = 32 * (tile / kt) + acc_row(v, l >> 5), r2 = 32 * (tile % kt) + (l & 31);
        if (r1 < k && r2 < k) G[r1 * k + r2] = s;
    }
}

// ---------------------------------------------------------------------------
// Objective ||A - W H||_F^2 in row tiles of W (the tiling of the paper's
// section 3.2 for its convergence check: W H is produced tile by tile and never
// stored).  Workgroup = 32 rows of A and W, 4 waves; a wave takes 128-column
// slabs w, w+4, ...  Per slab: X = W_tile H[:, slab] by MFMA (A_op = W tile
// from LDS, B_op = H elements, reduction over two factor indices per
// instruction; column tile q holds columns j0 + 4 jj + q), then A is loaded in
// the accumulator layout (16-byte loads, 512 contiguous bytes per row) and
// (a - x)^2 is summed.  One double per workgroup goes to `partial`.
// ---------------------------------------------------------------------------
template <int KT, bool VEC>
__global__ __launch_bounds__(256) void residual_kernel(const float *__restrict__ A,
                                                       const float *__restrict__ W,
                                                       const float *__restrict__ H, int64_t m,
                                                       int64_t n, int k, double *__restrict__ partial)
{
    constexpr int KP = 32 * KT, LDW = KP + 1;
    __shared__ float Ws[32 * LDW];
    __shared__ double wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int jj = lane & 31, half = lane >> 5;
    const int64_t i0 = (int64_t)blockIdx.x * 32;
    for (int e = tid; e < 32 * KP; e += 256) {
        const int i = e / KP, c = e % KP;
        Ws[i * LDW + c] = (i0 + i < m && c < k) ? W[(i0 + i) * k + c] : 0.f;
    }
    __syncthreads();
    const int kpairs = (k + 1) >> 1;
    float local = 0.f;
    double total = 0.0;
    const int64_t nslabs = (n + 127) >> 7;
    for (int64_t sl = w; sl < nslabs; sl += 4) {
        const int64_t col = sl * 128 + 4 * jj;
        f32x16 acc[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] = f32x16{0};
        for (int s = 0; s < kpairs; ++s) {
            const int c = 2 * s + half;
            const float a = Ws[jj * LDW + c];                 // c <= KP - 1 always; zero beyond k
            const f32x4 h = load4<VEC>(H, n, c, col, c < k);
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = mfma32(a, h[q], acc[q]);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t row = i0 + acc_row(v, half);
            const f32x4 a = load4<VEC>(A, n, row, col, row < m);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool in = row < m && col + q < n;
                const float d = in ? a[q] - acc[q][v] : 0.f;
                local += d * d;
            }
        }
        total += (double)local;     // fp32 within a slab (2048 terms per lane), double across slabs
        local = 0.f;
    }
    for (int off = 32; off > 0; off >>= 1) total += __shfl_xor(total, off);
    if (lane == 0) wsum[w] = total;
    __syncthreads();
    if (tid == 0) partial[blockIdx.x] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

// ---------------------------------------------------------------------------
// The same objective as a streaming pass for k = 16 or 32, 16-byte aligned A, W and H,
// n % 4 == 0 and m % 32 == 0 (the launcher gives the rows left over to the general kernel):
// the geometry and the exact-piece arithmetic of the W^T A pass, turned round: here the
// 32 x 32 tile of an instruction is rows of A by columns of A and the reduction runs over the
// factor index.  Workgroup = 4 waves on 256 consecutive columns and one row split; a wave
// owns 64 of the columns and walks down all the rows of the split, a lane 2 consecutive
// columns.  Once per wave its slab of H is cut into bf16 pieces (B_op: lane l holds factors
// 8 (l / 32) .. + 7 of 16 for column l % 32), kept in registers for every row tile.  Per
// 32-row tile a wave forms the two 32 x 32 tiles of W H with 2 x 8 instructions each from
// pieces of the rows of W (A_op: lane l holds 8 consecutive factors of row l % 32) that the
// workgroup makes once for its four waves (wave w cuts tile w of every group of
// four tiles into LDS, double buffered, one barrier per group), and subtracts them from the
// tile of A, loaded in the accumulator layout (lane l, register v: row (v % 4) + 4 (l / 32) +
// 8 (v / 4), its 2 columns: 8-byte loads, 1 KiB contiguous per row over the workgroup).  The
// next tile of A is requested before the current tile's arithmetic, the rows of W two groups
// ahead.  One double per workgroup.  On the 32768 x 16384, k = 32 case the kernel takes
// 0.37 ms on random operands and 0.31 ms, the time of its loads alone, on all-zero ones:
// what is left is the chip's power limit under matrix work and streaming together.
// ---------------------------------------------------------------------------
template <int KSTEPS>
__global__ __launch_bounds__(256, 2) void residual_stream_kernel(const float *__restrict__ A,
                                                                 const float *__restrict__ W,
                                                                 const float *__restrict__ H, int64_t m,
                                                                 int64_t n, int64_t rps,
                                                                 double *__restrict__ partial)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    constexpr int k = 16 * KSTEPS;
    __shared__ double wsum[4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jj = lane & 31, half = lane >> 5;
    const int64_t jw = (int64_t)blockIdx.x * 256 + 64 * w;   // this wave's 64 columns
    const int64_t col = jw + 2 * jj;
    const bool colok = col < n;                       // n is even: both columns or none
    const int64_t j0 = jw < n ? jw : 0;               // a wave wholly past column n fetches the first slab
    const int64_t r0 = (int64_t)blockIdx.y * rps;     // rps % 32 == 0
    const int64_t r1 = (r0 + rps < m) ? r0 + rps : m;

    // B_op pieces of the slab of H: hp[s][q][piece]
    u32x4 hp[KSTEPS][2][3];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
        f32x2 hv[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int c = 16 * s + 8 * half + r;
            const f32x2 t = *reinterpret_cast<const f32x2 *>(H + (colok ? (int64_t)c * n + col : 0));
            hv[r].x = colok ? t.x : 0.f;
            hv[r].y = colok ? t.y : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                unsigned h0, m0, l0, h1, m1, l1;
                split3(hv[2 * pr][q], h0, m0, l0);
                split3(hv[2 * pr + 1][q], h1, m1, l1);
                hp[s][q][0][pr] = pack2(h0, h1);
                hp[s][q][1][pr] = pack2(m0, m1);
                hp[s][q][2][pr] = pack2(l0, l1);
            }
    }

    // Requests only: nothing below reads a loaded value before the products of the previous
    // tile are issued, so the loads stay in flight.  m % 32 == 0 and rps % 32 == 0: every tile
    // is whole; a request past the split fetches tile 0 instead and is never used.
    // this lane's row of W for tile i0: 8 consecutive factors per 16-factor step
    f32x4 wv[KSTEPS][2];
    auto load_w = [&](int64_t i0) {
        const float *src = W + ((i0 < r1 ? i0 : 0) + jj) * k + 8 * half;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            wv[s][0] = *reinterpret_cast<const f32x4 *>(src + 16 * s);
            wv[s][1] = *reinterpret_cast<const f32x4 *>(src + 16 * s + 4);
        }
    };
    // A in the accumulator layout: wave-uniform row address plus one 32-bit lane offset
    // (4 n + 62 < 2^32); lanes past column n fetch the slab's first columns
    typedef f32x2 ATile[16];
    const unsigned lane_off = colok ? (unsigned)(4 * half) * (unsigned)n + 2u * jj : 0u;
    auto load_a = [&](ATile &a, int64_t i0) {
        const float *tp = A + (i0 < r1 ? i0 : 0) * n + j0;
#pragma unroll
        for (int v = 0; v < 16; ++v)
            a[v] = __builtin_nontemporal_load(reinterpret_cast<const f32x2 *>(tp + (int64_t)((v & 3) + 8 * (v >> 2)) * n + lane_off));
    };

    double total = 0.0;
    // The four waves walk the same row tiles, so the pieces of a tile of W are made once per
    // workgroup: of every group of four tiles wave w cuts tile w and stores it in LDS in
    // operand order (entry [tile][step * 3 + piece][lane], 16 bytes each), while the group
    // before it is consumed from the other buffer; one barrier per group.
    __shared__ u32x4 wlds[2][4][KSTEPS * 3][64];
    auto cut_store = [&](int buf) {
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            u32x4 wp[3];
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                unsigned h0, m0, l0, h1, m1, l1;
                split3(wv[s][pr >> 1][(2 * pr) & 3], h0, m0, l0);
                split3(wv[s][pr >> 1][(2 * pr + 1) & 3], h1, m1, l1);
                wp[0][pr] = pack2(h0, h1);
                wp[1][pr] = pack2(m0, m1);
                wp[2][pr] = pack2(l0, l1);
            }
#pragma unroll
            for (int pc = 0; pc < 3; ++pc) wlds[buf][w][s * 3 + pc][lane] = wp[pc];
        }
    };
    // one tile, its A already requested: pieces of W from LDS, products, differences.  The two
    // 32-column halves are two chains of 8 KSTEPS instructions one after the other, so the
    // differences of the first half can issue under the products of the second.
    auto tile = [&](const ATile &a, int buf, int t, bool valid) {
        u32x4 wp[KSTEPS][3];
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s)
#pragma unroll
            for (int pc = 0; pc < 3; ++pc) wp[s][pc] = wlds[buf][t][s * 3 + pc][lane];
        f32x16 acc[2];
        acc[0] = f32x16{0};
        acc[1] = f32x16{0};
        constexpr int PW[8] = {2, 1, 2, 1, 0, 1, 0, 0}, PH[8] = {1, 2, 0, 1, 2, 0, 1, 0};   // smallest first, no l l
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) acc[q] = mfma_bf16(wp[s][PW[e]], hp[s][q][PH[e]], acc[q]);
        float local = 0.f;      // 32 terms per lane in fp32, double across tiles
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float d0 = a[v].x - acc[0][v], d1 = a[v].y - acc[1][v];
            local += d0 * d0;
            local += d1 * d1;
        }
        total += valid ? (double)local : 0.0;
    };
    // four tiles per trip (every wave of the workgroup makes the same trips: r0 and r1 are the
    // workgroup's); a tile past the split is tile 0 again, and its sum is dropped
    ATile a0, a1;
    int64_t i = r0;
    load_w(i + 32 * w);
    cut_store(0);
    load_w(i + 128 + 32 * w);
    load_a(a0, i);
    __syncthreads();
    int buf = 0;
    for (; i < r1; i += 128) {
        cut_store(buf ^ 1);
        load_w(i + 256 + 32 * w);
        load_a(a1, i + 32);
        __builtin_amdgcn_sched_barrier(0);
        tile(a0, buf, 0, true);
        load_a(a0, i + 64);
        __builtin_amdgcn_sched_barrier(0);
        tile(a1, buf, 1, i + 32 < r1);
        load_a(a1, i + 96);
        __builtin_amdgcn_sched_barrier(0);
        tile(a0, buf, 2, i + 64 < r1);
        load_a(a0, i + 128);
        __builtin_amdgcn_sched_barrier(0);
        tile(a1, buf, 3, i + 96 < r1);
        __syncthreads();    // the group's buffer is free, the next group's is written
        buf ^= 1;
    }
    if (!colok) total = 0.0;   // such lanes subtracted a zero product from columns of other lanes
    for (int off = 32; off > 0; off >>= 1) total += __shfl_xor(total, off);
    if (lane == 0) wsum[w] = total;
    __syncthreads();
    if (tid == 0) partial[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

// Sum of `count` doubles by one block of 256 threads in a fixed order: thread t adds entries
// t, t + 256, ..., then thread 0 adds the 256 sums in thread order (one thread alone needs a
// dependent load per entry: 33 us for 512 entries, 0.3 ms for 4096).
__device__ __forceinline__ double block_sum_f64(const double *__restrict__ partial, int64_t count)
{
    __shared__ double part[256];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < count; i += 256) s += partial[i];
    part[threadIdx.x] = s;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0)
        for (int i = 0; i < 256; ++i) total += part[i];
    return total;     // valid in thread 0
}

// out[0] = sqrt(sum of `count` partials).  One block of 256 threads.
__global__ __launch_bounds__(256) void residual_finish_kernel(const double *__restrict__ partial, int64_t count,
                                                              double *out)
{
    const double s = block_sum_f64(partial, count);
    if (threadIdx.x == 0) out[0] = sqrt(s);
}

// partial[b] = sum of squares of a slice of X (double), for ||A||_F^2.
__global__ __launch_bounds__(256) void sumsq_kernel(const float *__restrict__ X, int64_t count,
                                                    double *__restrict__ partial)
{
    __shared__ double wsum[4];
    double acc = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256) {
        const float v = X[e];
        acc += (double)v * (double)v;
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

// out[0] = sum of `count` partials.  One block of 256 threads.
__global__ __launch_bounds__(256) void sum_f64_kernel(const double *__restrict__ partial, int64_t count, double *out)
{
    const double s = block_sum_f64(partial, count);
    if (threadIdx.x == 0) out[0] = s;
}

// Objective from quantities the W update leaves behind (the expansion of section 2.1's norm):
// ||A - W H||_F^2 = ||A||_F^2 - 2 <A H^T, W> + <H H^T, W^T W>, with <A H^T, W> = sum of dpart
// (numerator of the W update against the new W), GH = H H^T and GW = W^T W of the new factors.
// out[0] = square root of that, clamped at zero.  One block.
__global__ __launch_bounds__(256) void objective_kernel(const double *__restrict__ dpart, int nb,
                                                        const float *__restrict__ GW,
                                                        const float *__restrict__ GH, int k,
                                                        const double *__restrict__ normA2, double *out)
{
    __shared__ double part[256], dsum[256];
    double gg = 0.0, dd = 0.0;
    for (int e = threadIdx.x; e < k * k; e += 256) gg += (double)GW[e] * (double)GH[e];
    // shares b, b + 256, ... per thread, then the threads in order (the sparse and the streamed
    // runs hand over thousands of shares: one thread alone would spend 0.3 ms on them)
    for (int b = threadIdx.x; b < nb; b += 256) dd += dpart[b];
    part[threadIdx.x] = gg;
    dsum[threadIdx.x] = dd;
    __syncthreads();
    if (threadIdx.x == 0) {
        double g2 = 0.0, dot = 0.0;
        for (int i = 0; i < 256; ++i) g2 += part[i];
        for (int i = 0; i < 256; ++i) dot += dsum[i];
        const double f2 = normA2[0] - 2.0 * dot + g2;
        out[0] = f2 > 0.0 ? sqrt(f2) : 0.0;
    }
}

// P = sum over the row splits of the partial W^T A results (test entry point only).
// blockIdx.y = slice of 64 factors (ranks above 64): partials at ppart + slice * slice_ppart, `count`
// floats of P per full slice, count_last for the last one.
__global__ __launch_bounds__(256) void sum_partials_kernel(const float *__restrict__ ppart,
                                                           int splits, int64_t count,
                                                           float *__restrict__ P, int accumulate,
                                                           int64_t slice_ppart, int64_t count_last)
{
    ppart += (int64_t)blockIdx.y * slice_ppart;
    P += (int64_t)blockIdx.y * count;
    if (blockIdx.y == gridDim.y - 1) count = count_last;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256) {
        float s = 0.f;
        for (int t = 0; t < splits; ++t) s += ppart[(int64_t)t * count + e];
        P[e] = accumulate ? P[e] + s : s;
    }
}

// X <- X * P / (D + eps) element by element: the multiplicative update with its numerator P
// and the product D of the other factor's Gram matrix with X already formed (ranks above 64).
__global__ __launch_bounds__(256) void mu_apply_kernel(float *__restrict__ X, const float *__restrict__ P,
                                                       const float *__restrict__ D, float eps,
                                                       int64_t count)
{
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256)
        X[e] = X[e] * P[e] / (D[e] + eps);
}

// ---------------------------------------------------------------------------
// Host side launchers
// ---------------------------------------------------------------------------

static inline bool vec_ok(const void *p, int64_t ld)
{
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && (ld & 3) == 0;
}

int wta_splits(int64_t rows, int64_t n, int k)
{
    // Enough workgroups to fill the chip once at the kernels' occupancy (2 groups per
    // compute unit), but long row ranges per group: every split costs a k x n partial
    // result written and read again.  A workgroup covers 128 columns up to 32 factors and
    // 256 above.
    const int64_t width = k > 32 ? 256 : kWtaCols;
    const int64_t slabs = (n + width - 1) / width;
    const int64_t target = 512;
    int64_t s = (target + slabs - 1) / slabs;
    int64_t max_by_rows = (rows + 255) / 256;         // at least 256 rows per split ...
    if (slabs * max_by_rows < 128) {
        // ... unless that leaves most of the chip idle: small matrices are split down to one
        // 16-row step per wave, up to 128 workgroups (256 x 192: 19.6 instead of 26.0 us per
        // iteration; with many workgroups the fixed cost of a split outweighs it)
        const int64_t fine = (rows + 63) / 64, want = (128 + slabs - 1) / slabs;
        max_by_rows = fine < want ? fine : want;
    }
    if (s > max_by_rows) s = max_by_rows;
    // every split is a k x n partial that the finisher reads again, a few splits per trip to L2:
    // 32 at most, but up to 128 while there are fewer than 16 column slabs (1048576 x 256: the pass
    // ran on 64 workgroups)
    const int64_t cap = slabs >= 16 ? 32 : 128;
    if (s > cap) s = cap;
    if (s < 1) s = 1;
    return (int)s;
}

int wta_splits_bound(int64_t rows, int64_t n, int k)
{
    // within a column width the count shrinks as slabs grow and does not depend on k
    const int a = wta_splits(rows, n, 1), b = k > 32 ? wta_splits(rows, n, 64) : a;
    return a > b ? a : b;
}

int64_t wta_rows_per_split(int64_t rows, int splits)
{
    int64_t rps = (rows + splits - 1) / splits;
    return (rps + 15) & ~(int64_t)15;   // whole 16-row steps of a wave (and whole row pairs)
}

static int gram_blocks(int64_t len, int per_block)
{
    int64_t b = (len + per_block - 1) / per_block;
    if (b > kGramMaxBlocks) b = kGramMaxBlocks;
    if (b < 1) b = 1;
    return (int)b;
}

hipError_t launch_gram_w(const float *X, int64_t rows, int k, float *G, float *gpart,
                         unsigned *counters, hipStream_t st)
{
    const int kt = k_tiles(k);
    dim3 grid(gram_blocks(rows, 512), kt * kt);
    hipLaunchKernelGGL((gram_kernel<0, false>), grid, dim3(512), 0, st, X, rows, k, G, gpart, counters);
    return hipGetLastError();
}

hipError_t launch_gram_w_wide(const float *X, int64_t rows, int k, float *G, float *tiles, hipStream_t st)
{
    const int kt = k_tiles(k);
    int64_t nb = (rows + 511) / 512;
    if (nb > kFinMaxBlocks) nb = kFinMaxBlocks;
    if (nb < 1) nb = 1;
    hipLaunchKernelGGL((gram_kernel<0, false>), dim3((unsigned)nb, kt * kt), dim3(512), 0, st, X, rows, k,
                       static_cast<float *>(nullptr), tiles, static_cast<unsigned *>(nullptr));
    return launch_gram_sum(tiles, (int)nb, k, G, st);
}

hipError_t launch_gram_h(const float *X, int k, int64_t cols, float *G, float *gpart,
                         unsigned *counters, hipStream_t st)
{
    const int kt = k_tiles(k);
    dim3 grid(gram_blocks(cols, 512), kt * kt);
    if (vec_ok(X, cols))
        hipLaunchKernelGGL((gram_kernel<1, true>), grid, dim3(512), 0, st, X, cols, k, G, gpart, counters);
    else
        hipLaunchKernelGGL((gram_kernel<1, false>), grid, dim3(512), 0, st, X, cols, k, G, gpart, counters);
    return hipGetLastError();
}

template <int KT>
static void wta_dispatch(bool vec, dim3 grid, hipStream_t st, const float *A, const float *W,
                         float *ppart, int64_t rows, int64_t n, int k, int64_t rps, int acc,
                         const float *gtiles, int nsets, float *gsum)
{
    constexpr int U = 5, OCC = 2;
    const dim3 block(64 * kWtaWaves);
    if (vec)
        hipLaunchKernelGGL((wta_pass_kernel<KT, U, OCC, true>), grid, block, 0, st, A, W, ppart, rows, n, k, rps, acc, gtiles, nsets, gsum);
    else
        hipLaunchKernelGGL((wta_pass_kernel<KT, U, OCC, false>), grid, block, 0, st, A, W, ppart, rows, n, k, rps, acc, gtiles, nsets, gsum);
}

int wta_planes_only_width(const float *A, int64_t n)
{
    return (vec_ok(A, n) && n < ((int64_t)1 << 25)) ? 64 : 32;
}

size_t planes_bytes(int64_t rows) { return (size_t)((rows + 7) / 8) * 3 * 64 * 16; }   // 64 factor slots

hipError_t launch_split_planes_slice(const float *X, int64_t rows, int64_t ld, int64_t c0, int kc,
                                     void *planes, hipStream_t st)
{
    if (kc < 1 || kc > 64) return hipErrorInvalidValue;
    const int kp = kc <= 32 ? 32 : 64;
    const int64_t threads = ((rows + 7) / 8) * kp;
    hipLaunchKernelGGL(split_planes_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, X,
                       rows, ld, c0, kc, kp, static_cast<u32x4 *>(planes), (int64_t)0);
    return hipGetLastError();
}

hipError_t launch_split_planes_slices(const float *X, int64_t rows, int k, void *planes, hipStream_t st)
{
    const int nslices = (k + 63) / 64;
    const int64_t threads = ((rows + 7) / 8) * 64;
    hipLaunchKernelGGL(split_planes_kernel, dim3((unsigned)((threads + 255) / 256), (unsigned)nslices), dim3(256), 0, st, X,
                       rows, (int64_t)k, (int64_t)0, k, 64, static_cast<u32x4 *>(planes), (int64_t)(planes_bytes(rows) / 16));
    return hipGetLastError();
}

hipError_t launch_wta_pass_slices(const float *A, int64_t rows, int64_t n, int k, const void *planes, float *ppart,
                                  int splits, int64_t rps, hipStream_t st)
{
    if (!vec_ok(A, n) || n >= ((int64_t)1 << 25) || rps % 16 || k <= 64) return hipErrorInvalidValue;
    const int nslices = (k + 63) / 64;
    const int gx = (int)((n + 255) / 256), gy = splits;
    const int64_t tiles8 = ((int64_t)gx * gy + 7) / 8 * 8;
    hipLaunchKernelGGL((wta_pass_split64_wide_kernel<true>), dim3((unsigned)(tiles8 * nslices)), dim3(64 * kWtaWaves), 0, st, A,
                       static_cast<const u32x4 *>(planes), ppart, rows, n, k, rps, 0, static_cast<const float *>(nullptr), 0,
                       static_cast<float *>(nullptr), gx, gy, nslices, (int64_t)(planes_bytes(rows) / 16),
                       (int64_t)splits * 64 * n);
    return hipGetLastError();
}

hipError_t launch_sum_partials_slices(const float *ppart, int splits, int k, int64_t cols, float *P, hipStream_t st,
                                      bool accumulate)
{
    const int nslices = (k + 63) / 64;
    const int64_t count = 64 * cols, count_last = (int64_t)(k - 64 * (nslices - 1)) * cols;
    int64_t b = (count + 255) / 256;
    if (b > 4096) b = 4096;
    // the partials of slice z hold splits x (factors of z) x cols floats, packed for that slice's width
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)b, (unsigned)nslices), dim3(256), 0, st, ppart, splits, count, P,
                       accumulate ? 1 : 0, (int64_t)splits * 64 * cols, count_last);
    return hipGetLastError();
}

hipError_t launch_split_planes(const float *X, int64_t rows, int k, void *planes, hipStream_t st)
{
    if (!wta_uses_planes(k)) return hipSuccess;
    return launch_split_planes_slice(X, rows, k, 0, k, planes, st);
}

hipError_t launch_mu_apply(float *X, const float *P, const float *D, float eps, int64_t count,
                           hipStream_t st)
{
    int64_t b = (count + 255) / 256;
    if (b > 8192) b = 8192;
    hipLaunchKernelGGL(mu_apply_kernel, dim3((unsigned)b), dim3(256), 0, st, X, P, D, eps, count);
    return hipGetLastError();
}

hipError_t launch_wta_pass(const float *A, int64_t rows, int64_t n, int k, const float *W,
                           void *planes, bool planes_ready, float *ppart, int splits, int64_t rps,
                           bool accumulate, hipStream_t st, const float *gtiles, int nsets, float *gsum)
{
    dim3 grid((unsigned)((n + kWtaCols - 1) / kWtaCols), (unsigned)splits);
    const bool vec = vec_ok(A, n);
    const int acc = accumulate ? 1 : 0;
    if (rps % 16) return hipErrorInvalidValue;
    switch (k_tiles(k)) {
    case 1: {
        if (!planes) return hipErrorInvalidValue;
        if (!planes_ready) {
            hipError_t e = launch_split_planes(W, rows, k, planes, st);
            if (e != hipSuccess) return e;
        }
        const u32x4 *pl = static_cast<const u32x4 *>(planes);
        const dim3 block(64 * kWtaWaves);
        // buffer loads address 16 rows with 32-bit offsets: 64 n bytes must stay below 2^31
        if (vec && n < ((int64_t)1 << 25))
            hipLaunchKernelGGL(wta_pass_split_buf_kernel, grid, block, 0, st, A, pl, ppart, rows, n, k, rps, acc, gtiles, nsets, gsum);
        else
            hipLaunchKernelGGL((wta_pass_split_kernel<false>), grid, block, 0, st, A, pl, ppart, rows, n, k, rps, acc, gtiles, nsets, gsum);
        break;
    }
    case 2:
        if (vec && planes && n < ((int64_t)1 << 25)) {
            if (!planes_ready) {
                hipError_t e = launch_split_planes(W, rows, k, planes, st);
                if (e != hipSuccess) return e;
            }
            const dim3 grid256((unsigned)((n + 255) / 256), (unsigned)splits);
            hipLaunchKernelGGL((wta_pass_split64_wide_kernel<false>), grid256, dim3(64 * kWtaWaves), 0, st, A,
                               static_cast<const u32x4 *>(planes), ppart, rows, n, k, rps, acc, gtiles, nsets, gsum,
                               0, 0, 1, (int64_t)0, (int64_t)0);
        } else {
            if (!W) return hipErrorInvalidValue;   // this kernel reads the factor itself, not its planes
            wta_dispatch<2>(vec, grid, st, A, W, ppart, rows, n, k, rps, acc, gtiles, nsets, gsum);
        }
        break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

int gram_w_blocks(int64_t rows) { return gram_blocks(rows, 512); }

hipError_t launch_gram_sum(const float *gpart, int nb, int k, float *G, hipStream_t st)
{
    const int kt = k_tiles(k);
    const int threads = kt * kt * 1024 * 8;
    hipLaunchKernelGGL(gram_sum_kernel, dim3((threads + 255) / 256), dim3(256), 0, st, gpart, nb, k, G);
    return hipGetLastError();
}

int factor_update_blocks(int64_t len)
{
    int64_t b = (len + 63) / 64;
    if (b > kFinMaxBlocks) b = kFinMaxBlocks;
    return (int)b;
}

hipError_t launch_factor_update(float *X, float *Xt, const float *part, int splits,
                                const float *Gfull, const float *gin, int nbin, float *gout, int k,
                                int64_t len, float eps, hipStream_t st, const BlockMap *map,
                                void *planes, double *dpart)
{
    u32x4 *pl = wta_uses_planes(k) ? static_cast<u32x4 *>(planes) : nullptr;
    BlockMap bm;
    if (map) bm = *map;
    else bm.on = 0;
    // Without Gram output there is no reason to cap the grid: one block per chunk.
    int64_t blocks = gout ? factor_update_blocks(len) : (len + 63) / 64;
    if (blocks > 65535) blocks = 65535;
    const dim3 grid((unsigned)blocks), block(512);
    if (k <= 8)
        hipLaunchKernelGGL((factor_update_kernel<8>), grid, block, 0, st, X, Xt, part, splits, Gfull, gin, nbin, gout, pl, dpart, k, len, eps, bm);
    else if (k <= 32)
        hipLaunchKernelGGL((factor_update_kernel<32>), grid, block, 0, st, X, Xt, part, splits, Gfull, gin, nbin, gout, pl, dpart, k, len, eps, bm);
    else
        hipLaunchKernelGGL((factor_update_kernel<64>), grid, block, 0, st, X, Xt, part, splits, Gfull, gin, nbin, gout, pl, dpart, k, len, eps, bm);
    return hipGetLastError();
}

hipError_t launch_sum_partials(const float *ppart, int splits, int64_t count, float *P,
                               hipStream_t st, bool accumulate)
{
    int64_t b = (count + 255) / 256;
    if (b > 4096) b = 4096;
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)b), dim3(256), 0, st, ppart, splits, count, P, accumulate ? 1 : 0,
                       (int64_t)0, count);
    return hipGetLastError();
}

hipError_t launch_sumsq(const float *X, int64_t count, double *partial, double *out, hipStream_t st)
{
    int64_t b = (count + 256 * 64 - 1) / (256 * 64);
    if (b > 4096) b = 4096;
    if (b < 1) b = 1;
    hipLaunchKernelGGL(sumsq_kernel, dim3((unsigned)b), dim3(256), 0, st, X, count, partial);
    hipLaunchKernelGGL(sum_f64_kernel, dim3(1), dim3(256), 0, st, partial, b, out);
    return hipGetLastError();
}

hipError_t launch_objective(const double *dpart, int nb, const float *GW, const float *GH, int k,
                            const double *normA2, double *out, hipStream_t st)
{
    hipLaunchKernelGGL(objective_kernel, dim3(1), dim3(256), 0, st, dpart, nb, GW, GH, k, normA2, out);
    return hipGetLastError();
}

// Row splits of the streaming objective kernel: one resident set of workgroups, whole 32-row tiles.
static int residual_splits(int64_t m, int64_t n)
{
    const int64_t slabs = (n + 255) / 256;
    int64_t s = (512 + slabs - 1) / slabs;
    const int64_t by_rows = (m + 31) / 32;
    if (s > by_rows) s = by_rows;
    if (s < 1) s = 1;
    return (int)s;
}

int64_t residual_partials(int64_t m, int64_t n)
{
    const int64_t a = (m + 31) / 32, b = ((n + 255) / 256) * residual_splits(m & ~(int64_t)31, n) + 1;
    return a > b ? a : b;
}

hipError_t launch_residual(const float *A, int64_t m, int64_t n, int k, const float *W,
                           const float *H, double *partial, double *out, hipStream_t st)
{
    const int64_t m32 = m & ~(int64_t)31;
    // the streaming kernel adds a 32-bit lane offset of up to 4 n + 62 floats to a row address
    if (m32 > 0 && k <= 32 && k % 16 == 0 && n < ((int64_t)1 << 29) && vec_ok(A, n) && vec_ok(H, n) && vec_ok(W, k)) {
        // whole 32-row tiles by the streaming kernel, the up to 31 rows left by one workgroup
        // of the general one
        const int splits = residual_splits(m32, n);
        int64_t rps = (m32 + splits - 1) / splits;
        rps = (rps + 31) & ~(int64_t)31;
        const dim3 grid((unsigned)((n + 255) / 256), (unsigned)splits);
        int64_t count = (int64_t)grid.x * grid.y;
        if (k == 16)
            hipLaunchKernelGGL(residual_stream_kernel<1>, grid, dim3(256), 0, st, A, W, H, m32, n, rps, partial);
        else
            hipLaunchKernelGGL(residual_stream_kernel<2>, grid, dim3(256), 0, st, A, W, H, m32, n, rps, partial);
        if (m > m32) {
            hipLaunchKernelGGL((residual_kernel<1, true>), dim3(1), dim3(256), 0, st, A + m32 * n, W + m32 * k, H,
                               m - m32, n, k, partial + count);
            ++count;
        }
        hipLaunchKernelGGL(residual_finish_kernel, dim3(1), dim3(256), 0, st, (const double *)partial, count, out);
        return hipGetLastError();
    }
    const int64_t blocks = (m + 31) / 32;
    const bool vec = vec_ok(A, n) && vec_ok(H, n);
    const dim3 grid((unsigned)blocks), block(256);
    if (k_tiles(k) == 1) {
        if (vec) hipLaunchKernelGGL((residual_kernel<1, true>), grid, block, 0, st, A, W, H, m, n, k, partial);
        else hipLaunchKernelGGL((residual_kernel<1, false>), grid, block, 0, st, A, W, H, m, n, k, partial);
    } else {
        if (vec) hipLaunchKernelGGL((residual_kernel<2, true>), grid, block, 0, st, A, W, H, m, n, k, partial);
        else hipLaunchKernelGGL((residual_kernel<2, false>), grid, block, 0, st, A, W, H, m, n, k, partial);
    }
    hipLaunchKernelGGL(residual_finish_kernel, dim3(1), dim3(256), 0, st, (const double *)partial, blocks, out);
    return hipGetLastError();
}

template <int KT>
static void aht_dispatch(bool vec, dim3 grid, hipStream_t st, const float *A, const float *H,
                         const float *GH, float *W, int64_t rows, int64_t n, int k, float eps, double *dpart)
{
    constexpr int RT = kAhtRowTiles;
    if (vec)
        hipLaunchKernelGGL((aht_pass_kernel<KT, RT, true>), grid, dim3(512), 0, st, A, H, GH, W, rows, n, k, eps, dpart);
    else
        hipLaunchKernelGGL((aht_pass_kernel<KT, RT, false>), grid, dim3(512), 0, st, A, H, GH, W, rows, n, k, eps, dpart);
}

int64_t aht_pass_blocks(int64_t rows) { return (rows + 32 * kAhtRowTiles - 1) / (32 * kAhtRowTiles); }

hipError_t launch_aht_pass(const float *A, int64_t rows, int64_t n, int k, const float *H,
                           const float *GH, float *W, float eps, hipStream_t st, double *dpart)
{
    dim3 grid((unsigned)aht_pass_blocks(rows));
    const bool vec = vec_ok(A, n) && vec_ok(H, n);
    switch (k_tiles(k)) {
    case 1: aht_dispatch<1>(vec, grid, st, A, H, GH, W, rows, n, k, eps, dpart); break;
    case 2: aht_dispatch<2>(vec, grid, st, A, H, GH, W, rows, n, k, eps, dpart); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

bool aht_rows_can(const float *A, int64_t n, int k)
{
    // 32 rows of A are addressed with 32-bit byte offsets: 128 n < 2^31
    return k <= 64 && vec_ok(A, n) && n < ((int64_t)1 << 24);
}

bool aht_rows_ok(const float *A, int64_t m, int64_t n, int k)
{
    // Short and wide matrices leave most of the chip without a row block (64-row blocks: 12288 rows
    // are 192 of them), and with fewer than eight 64-column chunks some of a workgroup's waves have
    // none: such shapes do better on a transposed copy, unless the whole problem is small enough to be
    // latency bound anyway.
    return aht_rows_can(A, n, k) && ((m >= 12288 && n >= 512) || m * n <= ((int64_t)1 << 22));
}

// row tiles per workgroup: 128-row blocks when they fill the chip, else 64-row blocks; two
// 32-factor tiles leave registers for two row tiles only
static int aht_rows_tiles(int64_t rows, int k) { return k <= 32 && (rows + 127) / 128 >= 192 ? 4 : 2; }

int aht_rows_blocks(int64_t rows, int k)
{
    const int64_t rb = 32 * aht_rows_tiles(rows, k);
    int64_t b = (rows + rb - 1) / rb;
    if (b > kFinMaxBlocks) b = kFinMaxBlocks;
    return (int)b;
}

template <int R, int KT>
static hipError_t aht_rows_launch(dim3 grid, hipStream_t st, const float *A, const u32x4 *ph, const float *GH, float *W,
                                  u32x4 *pw, float *gout, double *dpart, int64_t rows, int64_t n, int k, float eps,
                                  int mode, const BlockMap &bm)
{
    constexpr int kLdsBytes = (8 * 2048 + 4 * R * KT * 1024 + (KT == 2 ? 4096 : 0)) * (int)sizeof(float);
    static bool raised = false;      // more dynamic LDS than the default limit: asked for once per process
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&aht_rows_kernel<R, KT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((aht_rows_kernel<R, KT>), grid, dim3(512), kLdsBytes, st, A, ph, GH, W, pw, gout, dpart, rows, n, k, eps, mode, bm);
    return hipGetLastError();
}

hipError_t launch_aht_rows(const float *A, int64_t rows, int64_t n, int k, const void *planesH,
                           const float *GH, float *W, void *planesW, float *gout, float eps, hipStream_t st,
                           bool gram_only, const BlockMap *map, double *dpart, bool dry)
{
    if (k > 64 || !planesW || !gout) return hipErrorInvalidValue;
    if (!gram_only && (!A || !planesH || !GH || !vec_ok(A, n) || n >= ((int64_t)1 << 24))) return hipErrorInvalidValue;
    BlockMap bm;
    if (map) bm = *map;
    else bm.on = 0;
    const dim3 grid((unsigned)aht_rows_blocks(rows, k));
    const u32x4 *ph = static_cast<const u32x4 *>(planesH);
    u32x4 *pw = static_cast<u32x4 *>(planesW);
    const int mode = gram_only ? 1 : (dry ? 2 : 0);
    if (k > 32) return aht_rows_launch<2, 2>(grid, st, A, ph, GH, W, pw, gout, dpart, rows, n, k, eps, mode, bm);
    if (aht_rows_tiles(rows, k) == 4) return aht_rows_launch<4, 1>(grid, st, A, ph, GH, W, pw, gout, dpart, rows, n, k, eps, mode, bm);
    return aht_rows_launch<2, 1>(grid, st, A, ph, GH, W, pw, gout, dpart, rows, n, k, eps, mode, bm);
}

hipError_t launch_sum_f64(const double *in, int64_t count, double *out, hipStream_t st)
{
    hipLaunchKernelGGL(sum_f64_kernel, dim3(1), dim3(256), 0, st, in, count, out);
    return hipGetLastError();
}

}  // namespace nmfmu
