// Weighted Gram matrix  M = A diag(d) A^T,  A = L(a, b)  (Sec. 3 "Computation of Gram matrix";
// App. "Fast weighted Gram matrix", Thm "Exact Gram decomposition"):
//
//   M_ij = sum_t d_t exp(-|a_i - b_t|) exp(-|a_j - b_t|)
//        = exp(-(a_hi - a_lo)) * ( U_lo + (W_hi - W_lo) + V_hi ),      lo / hi: the pair in sorted order,
//
// with, for a Gram anchor at sorted position p of the merged sequence a ++ b,
//   U = sum over middle anchors before p of  d_t exp(-2 (a - b_t))   (forward scan, doubled decay),
//   V = sum over middle anchors after  p of  d_t exp(-2 (b_t - a))   (backward scan, doubled decay),
//   W = sum over middle anchors before p of  d_t                     (plain prefix sum).
// The regions are taken by POSITION in the stable merged order, so a middle anchor equal to a Gram
// anchor lies in exactly one of them, and each region's closed form holds at a tie by continuity.
// Only non-positive numbers are ever exponentiated (the theorem's interval statistic e^{2(a_i - b_t)}
// overflows on wide intervals; the merged scan never forms it).
//
// U and V come from the scan kernels (one problem on the plan of the doubled anchors, emitted one-sided).
// This file holds W and the O(k^2) fill.  W is accumulated in fp64: the fill subtracts two prefix sums,
// and with weights of one sign an fp32 prefix of a million terms has lost the digits of a short interval.
#include "laplex_internal.h"

namespace laplex {

namespace {

constexpr int kWThreads = 256;
constexpr int kWItems = 16;
constexpr int kWTile = kWThreads * kWItems;      // merged positions per workgroup

// The weight carried by merged position j: d of a middle anchor, 0 for a Gram anchor or past the end.
__device__ __forceinline__ double weight_at(const uint32_t* __restrict__ ids, const float* __restrict__ d,
                                            uint32_t k, int64_t N, int64_t j)
{
    if (j >= N) return 0.0;
    const uint32_t id = ids[j];
    return id >= k ? (double)d[id - k] : 0.0;
}

__device__ __forceinline__ double wave_inclusive_scan_f64(double v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        const double o = __shfl_up(v, s);
        if (lane >= s) v += o;
    }
    return v;
}

// Exclusive scan of one double per thread over the workgroup (fixed order); *total = the sum.
__device__ __forceinline__ double block_exclusive_scan_f64(double v, double* total)
{
    __shared__ double wsum[kWThreads / 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const double inc = wave_inclusive_scan_f64(v);
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    double before = 0.0, all = 0.0;
#pragma unroll
    for (int w = 0; w < kWThreads / 64; ++w) {
        const double t = wsum[w];
        if (w < wave) before += t;
        all += t;
    }
    *total = all;
    __syncthreads();
    return before + inc - v;
}

// Sum of the weights of one tile of merged positions.
__global__ void __launch_bounds__(kWThreads)
k_w_tile_sums(const uint32_t* __restrict__ ids, const float* __restrict__ d, uint32_t k, int64_t N,
              double* __restrict__ tile_sum)
{
    const int64_t base = (int64_t)blockIdx.x * kWTile;
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < kWItems; ++i) s += weight_at(ids, d, k, N, base + i * kWThreads + threadIdx.x);
    double total;
    block_exclusive_scan_f64(s, &total);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

// Exclusive prefix over the tile sums, in place: one workgroup, chunks of kWThreads sums at a time.
__global__ void __launch_bounds__(kWThreads)
k_w_spine(double* __restrict__ tile_sum, int64_t tiles)
{
    double carry = 0.0;
    for (int64_t c0 = 0; c0 < tiles; c0 += kWThreads) {
        const int64_t t = c0 + threadIdx.x;
        const double v = t < tiles ? tile_sum[t] : 0.0;
        double total;
        const double ex = block_exclusive_scan_f64(v, &total);
        if (t < tiles) tile_sum[t] = carry + ex;
        carry += total;
    }
}

// W of every Gram anchor: the weights before it in merged order.  A thread owns kWItems consecutive
// positions (the tile goes through LDS so that the loads stay coalesced).
__global__ void __launch_bounds__(kWThreads)
k_w_down(const uint32_t* __restrict__ ids, const float* __restrict__ d, uint32_t k, int64_t N,
         const double* __restrict__ tile_prefix, double* __restrict__ W)
{
    __shared__ double sw[kWTile];
    __shared__ uint32_t sid[kWTile];
    const int64_t base = (int64_t)blockIdx.x * kWTile;
#pragma unroll
    for (int i = 0; i < kWItems; ++i) {
        const int slot = i * kWThreads + threadIdx.x;
        const int64_t j = base + slot;
        sw[slot] = weight_at(ids, d, k, N, j);
        sid[slot] = j < N ? ids[j] : 0xFFFFFFFFu;
    }
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < kWItems; ++i) s += sw[threadIdx.x * kWItems + i];
    double total;
    double run = tile_prefix[blockIdx.x] + block_exclusive_scan_f64(s, &total);
#pragma unroll
    for (int i = 0; i < kWItems; ++i) {
        const int slot = threadIdx.x * kWItems + i;
        const uint32_t id = sid[slot];
        if (id < k) W[id] = run;           // a Gram anchor (padding has id 0xFFFFFFFF >= k, k < 2^32 - 1)
        run += sw[slot];
    }
}

// The fill: one thread per four consecutive columns of one row.
__global__ void __launch_bounds__(256)
k_wgram_fill(const float* __restrict__ a, const float* __restrict__ U, const float* __restrict__ V,
             const double* __restrict__ W, int64_t k, float* __restrict__ M, int64_t ldm, int vec4)
{
    const int64_t i = blockIdx.x;
    const int64_t j0 = ((int64_t)blockIdx.y * blockDim.x + threadIdx.x) * 4;
    if (j0 >= k) return;
    const float ai = a[i], Ui = U[i], Vi = V[i];
    const double Wi = W[i];
    float out[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int64_t j = j0 + e < k ? j0 + e : k - 1;
        const float aj = a[j];
        // sorted order of the pair: by anchor, equal anchors by index (the stable merged order)
        const bool i_first = ai < aj || (ai == aj && i <= j);
        const float lo_u = i_first ? Ui : U[j], hi_v = i_first ? V[j] : Vi;
        const double mid = i_first ? W[j] - Wi : Wi - W[j];
        out[e] = expf(-fabsf(ai - aj)) * (lo_u + (float)mid + hi_v);
    }
    float* row = M + i * ldm;
    if (vec4 && j0 + 4 <= k) {
        typedef float v4f __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store((v4f){out[0], out[1], out[2], out[3]}, reinterpret_cast<v4f*>(row + j0));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j0 + e < k) row[j0 + e] = out[e];
    }
}

}  // namespace

int64_t wgram_tiles(int64_t N) { return (N + kWTile - 1) / kWTile; }

hipError_t launch_wgram_prefix(const uint32_t* ids, const float* d, int64_t k, int64_t N,
                               double* tile_sum, double* W, hipStream_t st)
{
    const int64_t tiles = wgram_tiles(N);
    LAPLEX_TIMED("wgram_prefix", st, hipLaunchKernelGGL(k_w_tile_sums, dim3((unsigned)tiles), dim3(kWThreads), 0, st,
                                                        ids, d, (uint32_t)k, N, tile_sum));
    LAPLEX_TIMED("wgram_prefix", st, hipLaunchKernelGGL(k_w_spine, dim3(1), dim3(kWThreads), 0, st, tile_sum, tiles));
    LAPLEX_TIMED("wgram_prefix", st, hipLaunchKernelGGL(k_w_down, dim3((unsigned)tiles), dim3(kWThreads), 0, st,
                                                        ids, d, (uint32_t)k, N, (const double*)tile_sum, W));
    return hipGetLastError();
}

hipError_t launch_wgram_fill(const float* a, const float* U, const float* V, const double* W, int64_t k,
                             float* M, int64_t ldm, hipStream_t st)
{
    const int vec4 = (reinterpret_cast<uintptr_t>(M) & 15u) == 0 && ldm % 4 == 0;
    const dim3 grid((unsigned)k, (unsigned)((k + 1023) / 1024));     // rows on x (up to 2^31 - 1), column chunks on y
    LAPLEX_TIMED("wgram_fill", st, hipLaunchKernelGGL(k_wgram_fill, grid, dim3(256), 0, st, a, U, V, W, k, M, ldm, vec4));
    return hipGetLastError();
}

}  // namespace laplex
