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
// W enters only through differences W_hi - W_lo, and two Gram anchors with no middle anchor between them must get
// the SAME number (their entry can be as small as exp(-2 gap) of the nearest middle anchor, next to which a
// rounding difference of two prefix sums associated differently is enormous).  So the prefix sum is stored once per
// middle anchor (Pb[t] = d_0 + .. + d_t in merged order), a Gram anchor records how many middle anchors precede it
// (an exact integer scan), and W is picked up afterwards as Pb[count - 1].
// The regions are taken by POSITION in the stable merged order, so a middle anchor equal to a Gram
// anchor lies in exactly one of them, and each region's closed form holds at a tie by continuity.
// Only non-positive numbers are ever exponentiated (the theorem's interval statistic e^{2(a_i - b_t)}
// overflows on wide intervals; the merged scan never forms it).
//
// U, V and W come from one three-kernel scan of their own (tile summaries, spine, downsweep) over the plan of
// the doubled anchors; a segment is summarised by (D, S) with F_out = D F_in + S in each direction.
// Everything between the fp32 anchors and the result is fp64, for the fp32 entry point too: the fill
// subtracts two prefix sums of the weights, and with weights of one sign an fp32 prefix of a million terms
// has lost the digits of a short interval; and the device's fp64 rate makes the wider type free here (the
// kernels wait for memory and for each other).  The fp64 entry point (App. "Density model", training: the
// Gram matrices run in fp64 through the same scan) differs only in the types of the weights and the result.
#include "laplex_internal.h"

namespace laplex {

namespace {

constexpr int kWThreads = 256;
constexpr int kWItems = 16;
constexpr int kWTile = kWThreads * kWItems;      // merged positions per workgroup

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

struct Pair64 { double D, S; };

__device__ __forceinline__ Pair64 pair_then(const Pair64& first, const Pair64& second)
{
    return Pair64{first.D * second.D, second.D * first.S + second.S};
}

// Exclusive scan of one pair per thread over the workgroup, in thread order; *total = all of them.
__device__ __forceinline__ Pair64 block_exclusive_scan_pair(Pair64 v, Pair64* total)
{
    __shared__ double wD[kWThreads / 64], wS[kWThreads / 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    Pair64 inc = v;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        Pair64 o{__shfl_up(inc.D, s), __shfl_up(inc.S, s)};
        if (lane >= s) inc = pair_then(o, inc);
    }
    if (lane == 63) { wD[wave] = inc.D; wS[wave] = inc.S; }
    Pair64 before{__shfl_up(inc.D, 1), __shfl_up(inc.S, 1)};
    if (lane == 0) before = Pair64{1.0, 0.0};
    __syncthreads();
    Pair64 head{1.0, 0.0}, all{1.0, 0.0};
#pragma unroll
    for (int w = 0; w < kWThreads / 64; ++w) {
        const Pair64 t{wD[w], wS[w]};
        if (w < wave) head = pair_then(head, t);
        all = pair_then(all, t);
    }
    *total = all;
    __syncthreads();
    return pair_then(head, before);
}

// Stage one tile: weights (fp64), anchors p_{j-1} .. p_{j+1} (the plan's pk, fp32: doubled anchors) and ids.
struct Tile64 {
    double* w;        // [kWTile]
    float* p;         // [kWTile + 2]: p[i] = anchor of position base + i - 1
    uint32_t* id;     // [kWTile]
};

template <typename TW>
__device__ __forceinline__ void stage_tile64(const Tile64& T, const uint32_t* __restrict__ ids, const float* __restrict__ pk,
                                             const TW* __restrict__ d, uint32_t k, int64_t N, int64_t base)
{
    for (int slot = threadIdx.x; slot < kWTile; slot += kWThreads) {
        const int64_t j = base + slot;
        uint32_t id = 0xFFFFFFFFu;
        double wv = 0.0;
        if (j < N) { id = ids[j]; if (id >= k) wv = (double)d[id - k]; }
        T.id[slot] = id;
        T.w[slot] = wv;
    }
    for (int slot = threadIdx.x; slot < kWTile + 2; slot += kWThreads) {
        const int64_t j = base + slot;                     // pk[j] = anchor of position j - 1
        T.p[slot] = pk[j <= N + 1 ? j : N + 1];
    }
    __syncthreads();
}

// decay into tile-local position i from its left neighbour / from its right neighbour; positions past
// the end are transparent
__device__ __forceinline__ double decay_left(const Tile64& T, int i, bool live)
{
    return live ? exp(-((double)T.p[i + 1] - (double)T.p[i])) : 1.0;
}
__device__ __forceinline__ double decay_right(const Tile64& T, int i, bool live)
{
    return live ? exp(-((double)T.p[i + 2] - (double)T.p[i + 1])) : 1.0;
}

#define LAPLEX_TILE64_LDS                               \
    __shared__ double t_w[kWTile];                      \
    __shared__ float t_p[kWTile + 2];                   \
    __shared__ uint32_t t_id[kWTile];                   \
    const Tile64 T{t_w, t_p, t_id}

// summ: [6][tiles] = forward (D, S), backward (D, S), sum of the weights, number of middle anchors
template <typename TW>
__global__ void __launch_bounds__(kWThreads)
k_g64_tiles(const uint32_t* __restrict__ ids, const float* __restrict__ pk, const TW* __restrict__ d,
            uint32_t k, int64_t N, int64_t tiles, double* __restrict__ summ)
{
    LAPLEX_TILE64_LDS;
    const int64_t base = (int64_t)blockIdx.x * kWTile;
    stage_tile64(T, ids, pk, d, k, N, base);
    Pair64 f{1.0, 0.0}, b{1.0, 0.0};
    double wsum = 0.0, middle = 0.0;
    const int cf = threadIdx.x * kWItems, cb = (kWThreads - 1 - threadIdx.x) * kWItems;
#pragma unroll
    for (int i = 0; i < kWItems; ++i) {
        const int u = cf + i, v = cb + kWItems - 1 - i;
        const double df = decay_left(T, u, base + u < N), db = decay_right(T, v, base + v < N);
        f = Pair64{f.D * df, df * f.S + T.w[u]};
        b = Pair64{b.D * db, db * b.S + T.w[v]};
        wsum += T.w[u];
        middle += (base + u < N && T.id[u] >= k) ? 1.0 : 0.0;       // counts stay exact in fp64
    }
    Pair64 tf, tb;
    double tw, tc;
    block_exclusive_scan_pair(f, &tf);
    block_exclusive_scan_pair(b, &tb);
    block_exclusive_scan_f64(wsum, &tw);
    block_exclusive_scan_f64(middle, &tc);
    if (threadIdx.x == 0) {
        summ[0 * tiles + blockIdx.x] = tf.D; summ[1 * tiles + blockIdx.x] = tf.S;
        summ[2 * tiles + blockIdx.x] = tb.D; summ[3 * tiles + blockIdx.x] = tb.S;
        summ[4 * tiles + blockIdx.x] = tw;
        summ[5 * tiles + blockIdx.x] = tc;
    }
}

// In place: summ[1][t] <- forward state entering tile t, summ[3][t] <- backward state entering it (from
// the right), summ[4][t] <- weights before it, summ[5][t] <- middle anchors before it.  One workgroup, kWThreads tiles at a time.
__global__ void __launch_bounds__(kWThreads)
k_g64_spine(double* __restrict__ summ, int64_t tiles)
{
    double cF = 0.0, cW = 0.0, cC = 0.0;
    for (int64_t c0 = 0; c0 < tiles; c0 += kWThreads) {
        const int64_t t = c0 + threadIdx.x;
        const bool ok = t < tiles;
        Pair64 v{ok ? summ[0 * tiles + t] : 1.0, ok ? summ[1 * tiles + t] : 0.0}, tot;
        const Pair64 ex = block_exclusive_scan_pair(v, &tot);
        double tw, tc;
        const double w = ok ? summ[4 * tiles + t] : 0.0;
        const double ew = block_exclusive_scan_f64(w, &tw);
        const double ec = block_exclusive_scan_f64(ok ? summ[5 * tiles + t] : 0.0, &tc);
        if (ok) { summ[1 * tiles + t] = ex.D * cF + ex.S; summ[4 * tiles + t] = cW + ew; summ[5 * tiles + t] = cC + ec; }
        cF = tot.D * cF + tot.S;
        cW += tw;
        cC += tc;
    }
    double cB = 0.0;
    const int64_t chunks = (tiles + kWThreads - 1) / kWThreads;
    for (int64_t c = chunks - 1; c >= 0; --c) {
        const int64_t t = c * kWThreads + (kWThreads - 1 - threadIdx.x);      // thread order = descending tiles
        const bool ok = t < tiles;
        Pair64 v{ok ? summ[2 * tiles + t] : 1.0, ok ? summ[3 * tiles + t] : 0.0}, tot;
        const Pair64 ex = block_exclusive_scan_pair(v, &tot);
        if (ok) summ[3 * tiles + t] = ex.D * cB + ex.S;
        cB = tot.D * cB + tot.S;
    }
}

template <typename TW>
__global__ void __launch_bounds__(kWThreads)
k_g64_down(const uint32_t* __restrict__ ids, const float* __restrict__ pk, const TW* __restrict__ d,
           uint32_t k, int64_t N, int64_t tiles, const double* __restrict__ summ,
           double* __restrict__ U, double* __restrict__ V, double* __restrict__ W, double* __restrict__ Pb)
{
    LAPLEX_TILE64_LDS;
    const int64_t base = (int64_t)blockIdx.x * kWTile;
    stage_tile64(T, ids, pk, d, k, N, base);
    Pair64 f{1.0, 0.0}, b{1.0, 0.0};
    double wsum = 0.0, middle = 0.0;
    const int cf = threadIdx.x * kWItems, cb = (kWThreads - 1 - threadIdx.x) * kWItems;
#pragma unroll
    for (int i = 0; i < kWItems; ++i) {
        const int u = cf + i, v = cb + kWItems - 1 - i;
        const double df = decay_left(T, u, base + u < N), db = decay_right(T, v, base + v < N);
        f = Pair64{f.D * df, df * f.S + T.w[u]};
        b = Pair64{b.D * db, db * b.S + T.w[v]};
        wsum += T.w[u];
        middle += (base + u < N && T.id[u] >= k) ? 1.0 : 0.0;
    }
    Pair64 tot;
    double tw, tc;
    const Pair64 ef = block_exclusive_scan_pair(f, &tot);
    const Pair64 eb = block_exclusive_scan_pair(b, &tot);
    double F = ef.D * summ[1 * tiles + blockIdx.x] + ef.S;
    double R = eb.D * summ[3 * tiles + blockIdx.x] + eb.S;
    double run = summ[4 * tiles + blockIdx.x] + block_exclusive_scan_f64(wsum, &tw);
    int64_t before = (int64_t)(summ[5 * tiles + blockIdx.x] + block_exclusive_scan_f64(middle, &tc));   // middle anchors before this lane's rows
#pragma unroll
    for (int i = 0; i < kWItems; ++i) {
        const int u = cf + i, v = cb + kWItems - 1 - i;
        F = decay_left(T, u, base + u < N) * F + T.w[u];
        R = decay_right(T, v, base + v < N) * R + T.w[v];
        const uint32_t iu = T.id[u], iv = T.id[v];
        // a Gram anchor carries no weight: F, R are the sums strictly beside it; its W is picked up from Pb
        // afterwards (k_g64_pick), here it records how many middle anchors precede it
        if (iu < k) { U[iu] = F; W[iu] = (double)before; }
        if (iv < k) V[iv] = R;
        run += T.w[u];
        if (base + u < N && iu >= k) { Pb[before] = run; ++before; }      // the prefix sum up to and including this middle anchor
    }
}

// W[i] <- the prefix sum at the last middle anchor before Gram anchor i (0 if there is none).
// status: the plan's status word, or null for plans that are always valid.  An invalid plan (the radix
// sort gave up a wait) turns every W[i], and with it every entry of the matrix, into a NaN.
__global__ void __launch_bounds__(256)
k_g64_pick(double* __restrict__ W, const double* __restrict__ Pb, int64_t k, const uint32_t* __restrict__ status)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= k) return;
    const int64_t c = (int64_t)W[i];
    const bool invalid = status != nullptr && *status != 0u;
    W[i] = invalid ? __longlong_as_double(0x7FF8000000000000LL) : (c > 0 ? Pb[c - 1] : 0.0);
}

// The fill: one thread per four consecutive columns of one row; lo / hi of a pair by (anchor, index), the
// stable merged order.
template <typename TM>
__global__ void __launch_bounds__(256)
k_wgram_fill(const float* __restrict__ a, const double* __restrict__ U, const double* __restrict__ V,
             const double* __restrict__ W, int64_t k, TM* __restrict__ M, int64_t ldm, int vec4)
{
    const int64_t i = blockIdx.x;
    const int64_t j0 = ((int64_t)blockIdx.y * blockDim.x + threadIdx.x) * 4;
    if (j0 >= k) return;
    const float ai = a[i];
    const double Ui = U[i], Vi = V[i], Wi = W[i];
    TM out[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int64_t j = j0 + e < k ? j0 + e : k - 1;
        const float aj = a[j];
        const bool i_first = ai < aj || (ai == aj && i <= j);
        const double inner = i_first ? Ui + (W[j] - Wi) + V[j] : U[j] + (Wi - W[j]) + Vi;
        out[e] = (TM)(exp(-fabs((double)ai - (double)aj)) * inner);
    }
    TM* row = M + i * ldm;
    if (sizeof(TM) == 4 && vec4 && j0 + 4 <= k) {
        typedef float v4f __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store((v4f){(float)out[0], (float)out[1], (float)out[2], (float)out[3]}, reinterpret_cast<v4f*>(row + j0));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j0 + e < k) row[j0 + e] = out[e];
    }
}

}  // namespace

int64_t wgram_tiles(int64_t N);

template <typename TW, typename TM>
hipError_t launch_wgram_t(const uint32_t* ids, const float* pk, const float* a, const TW* d, int64_t k, int64_t N,
                          double* summ, double* U, double* V, double* W, double* Pb, TM* M, int64_t ldm,
                          const uint32_t* status, hipStream_t st)
{
    const int64_t tiles = wgram_tiles(N);
    LAPLEX_TIMED("wgram_scan", st, hipLaunchKernelGGL((k_g64_tiles<TW>), dim3((unsigned)tiles), dim3(kWThreads), 0, st,
                                                      ids, pk, d, (uint32_t)k, N, tiles, summ));
    LAPLEX_TIMED("wgram_scan", st, hipLaunchKernelGGL(k_g64_spine, dim3(1), dim3(kWThreads), 0, st, summ, tiles));
    LAPLEX_TIMED("wgram_scan", st, hipLaunchKernelGGL((k_g64_down<TW>), dim3((unsigned)tiles), dim3(kWThreads), 0, st,
                                                      ids, pk, d, (uint32_t)k, N, tiles, (const double*)summ, U, V, W, Pb));
    LAPLEX_TIMED("wgram_scan", st, hipLaunchKernelGGL(k_g64_pick, dim3((unsigned)((k + 255) / 256)), dim3(256), 0, st,
                                                      W, (const double*)Pb, k, status));
    const int vec4 = (reinterpret_cast<uintptr_t>(M) & 15u) == 0 && ldm % 4 == 0;
    const dim3 grid((unsigned)k, (unsigned)((k + 1023) / 1024));     // rows on x (up to 2^31 - 1), column chunks on y
    LAPLEX_TIMED("wgram_fill", st, hipLaunchKernelGGL((k_wgram_fill<TM>), grid, dim3(256), 0, st,
                                                      a, (const double*)U, (const double*)V, (const double*)W, k, M, ldm, vec4));
    return hipGetLastError();
}

int64_t wgram_tiles(int64_t N) { return (N + kWTile - 1) / kWTile; }

hipError_t launch_wgram_f32(const uint32_t* ids, const float* pk, const float* a, const float* d, int64_t k, int64_t N,
                            double* summ, double* U, double* V, double* W, double* Pb, float* M, int64_t ldm,
                            const uint32_t* status, hipStream_t st)
{
    return launch_wgram_t<float, float>(ids, pk, a, d, k, N, summ, U, V, W, Pb, M, ldm, status, st);
}

hipError_t launch_wgram_f64(const uint32_t* ids, const float* pk, const float* a, const double* d, int64_t k, int64_t N,
                            double* summ, double* U, double* V, double* W, double* Pb, double* M, int64_t ldm,
                            const uint32_t* status, hipStream_t st)
{
    return launch_wgram_t<double, double>(ids, pk, a, d, k, N, summ, U, V, W, Pb, M, ldm, status, st);
}

}  // namespace laplex
