// Sorting the merged anchors (Sec. 3: "sorting raises the total cost to
// O(n log n)"; App. B "Combined complexity").  Hand-written for gfx950:
// 64-wide wavefronts, ballot-based stable ranking, LDS-staged scatter.
//
//   make_keys   a ++ b  ->  order-preserving u32 keys + ids
//   radix sort  4 LSD passes of 8 bits: per-tile digit counts, an exclusive scan
//               of the digit-major count table, and a stable scatter
//   merge       one merge-path pass when both anchor sets arrive sorted
//   decay       exp(-(p_j - p_{j-1})) between sorted neighbours, once per plan
#include "laplex_internal.h"

namespace laplex {

namespace {

__device__ __forceinline__ uint32_t float_to_key(float f)
{
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0u;                       // -0.0 sorts as +0.0
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

__device__ __forceinline__ float key_to_float(uint32_t key)
{
    return __uint_as_float(key ^ ((key >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_make_keys(const float* __restrict__ a, int64_t k, const float* __restrict__ b, int64_t n,
            uint32_t* __restrict__ keys, uint32_t* __restrict__ ids)
{
    const int64_t N = k + n;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += stride) {
        const float f = i < k ? a[i] : b[i - k];
        keys[i] = float_to_key(f);
        ids[i] = (uint32_t)i;
    }
}

// ---------------------------------------------------------------------------
// Pass step 1: digit counts of one tile -> table[digit * tiles + tile].
__global__ void __launch_bounds__(kSortThreads)
k_radix_count(const uint32_t* __restrict__ keys, int64_t N, int shift,
              uint32_t* __restrict__ table, int64_t tiles)
{
    __shared__ uint32_t hist[kSortThreads / 64][kRadix];
    const int tid = threadIdx.x, wave = tid >> 6;
    for (int i = tid; i < (kSortThreads / 64) * kRadix; i += kSortThreads) (&hist[0][0])[i] = 0u;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
    for (int i = 0; i < kSortKeysPerThread; ++i) {
        const int64_t pos = base + (int64_t)i * kSortThreads + tid;
        if (pos < N) atomicAdd(&hist[wave][(keys[pos] >> shift) & (kRadix - 1)], 1u);
    }
    __syncthreads();
    if (tid < kRadix) {
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < kSortThreads / 64; ++w) c += hist[w][tid];
        table[(int64_t)tid * tiles + blockIdx.x] = c;
    }
}

// ---------------------------------------------------------------------------
// Exclusive scan of the count table (u32), three small kernels.
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t v)
{
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(v, d);
        if (lane >= d) v += o;
    }
    return v;
}

// Exclusive scan of one value per thread over the whole workgroup; *total gets the sum.
template <int THREADS>
__device__ __forceinline__ uint32_t block_exclusive_scan_u32(uint32_t v, uint32_t* total)
{
    __shared__ uint32_t wsum[THREADS / 64];
    __shared__ uint32_t wtot;
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const uint32_t inc = wave_inclusive_scan_u32(v);
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int w = 0; w < THREADS / 64; ++w) { const uint32_t t = wsum[w]; wsum[w] = run; run += t; }
        wtot = run;
    }
    __syncthreads();
    const uint32_t r = wsum[wave] + inc - v;
    if (total) *total = wtot;
    __syncthreads();
    return r;
}

__global__ void __launch_bounds__(kTableScanThreads)
k_table_chunk_sums(const uint32_t* __restrict__ table, int64_t len, uint32_t* __restrict__ chunks)
{
    const int64_t base = (int64_t)blockIdx.x * kTableScanChunk;
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < kTableScanPerThread; ++i) {
        const int64_t p = base + (int64_t)i * kTableScanThreads + threadIdx.x;
        if (p < len) s += table[p];
    }
    uint32_t total;
    block_exclusive_scan_u32<kTableScanThreads>(s, &total);
    if (threadIdx.x == 0) chunks[blockIdx.x] = total;
}

__global__ void __launch_bounds__(1024)
k_table_chunk_scan(uint32_t* __restrict__ chunks, int64_t count)
{
    // one workgroup; each thread owns a run of consecutive chunk sums
    const int64_t per = (count + 1023) / 1024;
    const int64_t lo = (int64_t)threadIdx.x * per;
    const int64_t hi = lo + per < count ? lo + per : count;
    uint32_t s = 0;
    for (int64_t i = lo; i < hi; ++i) s += chunks[i];
    uint32_t run = block_exclusive_scan_u32<1024>(s, nullptr);
    for (int64_t i = lo; i < hi; ++i) { const uint32_t t = chunks[i]; chunks[i] = run; run += t; }
}

__global__ void __launch_bounds__(kTableScanThreads)
k_table_scan_apply(uint32_t* __restrict__ table, int64_t len, const uint32_t* __restrict__ chunks)
{
    // thread owns kTableScanPerThread consecutive entries (blocked), so the scan order is the array order
    const int64_t base = (int64_t)blockIdx.x * kTableScanChunk + (int64_t)threadIdx.x * kTableScanPerThread;
    uint32_t v[kTableScanPerThread];
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < kTableScanPerThread; ++i) {
        v[i] = base + i < len ? table[base + i] : 0u;
        s += v[i];
    }
    uint32_t run = block_exclusive_scan_u32<kTableScanThreads>(s, nullptr) + chunks[blockIdx.x];
#pragma unroll
    for (int i = 0; i < kTableScanPerThread; ++i) {
        if (base + i < len) table[base + i] = run;
        run += v[i];
    }
}

// ---------------------------------------------------------------------------
// Pass step 3: stable scatter of one tile.
//
// A wavefront owns 64 * KPT consecutive keys, item-major (item i of lane l is
// key i*64 + l of the wavefront's range), so the order (wave, item, lane) is
// the input order.  Ranking inside a wavefront: the lanes that hold the same
// digit find each other with eight ballots; the lowest of them bumps the
// wavefront's digit counter in LDS and hands the old value to its peers.
// The tile is then laid out in LDS in sorted order and written out so that
// each digit's run goes to consecutive addresses.
__global__ void __launch_bounds__(kSortThreads)
k_radix_scatter(const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ ids_in,
                uint32_t* __restrict__ keys_out, uint32_t* __restrict__ ids_out,
                int64_t N, int shift, const uint32_t* __restrict__ table, int64_t tiles)
{
    constexpr int WAVES = kSortThreads / 64;
    constexpr int KPT = kSortKeysPerThread;
    __shared__ uint32_t whist[WAVES][kRadix];     // per-wave digit counts, then offsets
    __shared__ uint32_t tile_start[kRadix];       // first local slot of each digit
    __shared__ uint32_t delta[kRadix];            // global slot of digit d = delta[d] + local slot
    __shared__ uint32_t skeys[kSortTile];
    __shared__ uint32_t sids[kSortTile];

    const int tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
    for (int i = tid; i < WAVES * kRadix; i += kSortThreads) (&whist[0][0])[i] = 0u;
    __syncthreads();

    const int64_t tile_base = (int64_t)blockIdx.x * kSortTile;
    const int64_t wave_base = tile_base + (int64_t)wave * (64 * KPT);
    const int64_t remaining = N - tile_base;
    const uint32_t valid = remaining < kSortTile ? (uint32_t)remaining : (uint32_t)kSortTile;

    uint32_t key[KPT], id[KPT], rank[KPT];
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const int64_t pos = wave_base + i * 64 + lane;
        const bool ok = pos < N;
        key[i] = ok ? keys_in[pos] : 0xFFFFFFFFu;   // padding sorts last inside the tile
        id[i] = ok ? ids_in[pos] : 0u;
    }
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const uint32_t d = (key[i] >> shift) & (kRadix - 1);
        uint64_t peers = ~0ull;
#pragma unroll
        for (int bit = 0; bit < kRadixBits; ++bit) {
            const bool one = (d >> bit) & 1u;
            const uint64_t m = __ballot(one);
            peers &= one ? m : ~m;
        }
        const int leader = __ffsll((long long)peers) - 1;
        uint32_t old = 0;
        if (lane == leader) old = atomicAdd(&whist[wave][d], (uint32_t)__popcll(peers));
        old = __shfl(old, leader);
        rank[i] = old + (uint32_t)__popcll(peers & lt_mask);
    }
    __syncthreads();

    // per digit: exclusive offsets over the wavefronts, tile-level digit starts, global deltas
    uint32_t digit_total = 0;
    if (tid < kRadix) {
#pragma unroll
        for (int w = 0; w < WAVES; ++w) { const uint32_t c = whist[w][tid]; whist[w][tid] = digit_total; digit_total += c; }
    }
    const uint32_t start = block_exclusive_scan_u32<kSortThreads>(tid < kRadix ? digit_total : 0u, nullptr);
    if (tid < kRadix) {
        tile_start[tid] = start;
        delta[tid] = table[(int64_t)tid * tiles + blockIdx.x] - start;
    }
    __syncthreads();

#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const uint32_t d = (key[i] >> shift) & (kRadix - 1);
        const uint32_t slot = tile_start[d] + whist[wave][d] + rank[i];
        skeys[slot] = key[i];
        sids[slot] = id[i];
    }
    __syncthreads();

#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const uint32_t slot = (uint32_t)(i * kSortThreads + tid);
        if (slot < valid) {
            const uint32_t kk = skeys[slot];
            const uint32_t dst = delta[(kk >> shift) & (kRadix - 1)] + slot;
            if ((int64_t)dst < N) {   // always true for a consistent count table; keeps a fault impossible
                keys_out[dst] = kk;
                ids_out[dst] = sids[slot];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Merge path: both anchor arrays ascending.  Among the first `diag` merged
// elements, how many come from a?  (a wins ties, so a[i] precedes b[j] iff
// a[i] <= b[j].)
__device__ __forceinline__ int64_t merge_split(const float* __restrict__ a, int64_t k,
                                               const float* __restrict__ b, int64_t n, int64_t diag)
{
    int64_t lo = diag > n ? diag - n : 0;
    int64_t hi = diag < k ? diag : k;
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] <= b[diag - 1 - mid]) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__global__ void __launch_bounds__(kMergeThreads)
k_merge(const float* __restrict__ a, int64_t k, const float* __restrict__ b, int64_t n,
        uint32_t* __restrict__ keys, uint32_t* __restrict__ ids)
{
    __shared__ float stage[kMergeTile];          // a-part then b-part of this tile
    __shared__ uint32_t okey[kMergeTile], oid[kMergeTile];
    __shared__ int64_t split[2];
    const int64_t N = k + n;
    const int64_t d0 = (int64_t)blockIdx.x * kMergeTile;
    const int64_t d1 = d0 + kMergeTile < N ? d0 + kMergeTile : N;
    if (threadIdx.x < 2) split[threadIdx.x] = merge_split(a, k, b, n, threadIdx.x == 0 ? d0 : d1);
    __syncthreads();
    const int64_t ia0 = split[0], ia1 = split[1];
    const int64_t ib0 = d0 - ia0, ib1 = d1 - ia1;
    const int na = (int)(ia1 - ia0), nb = (int)(ib1 - ib0);
    for (int i = threadIdx.x; i < na + nb; i += kMergeThreads)
        stage[i] = i < na ? a[ia0 + i] : b[ib0 + (i - na)];
    __syncthreads();
    const float* sa = stage;
    const float* sb = stage + na;
    for (int i = threadIdx.x; i < na + nb; i += kMergeThreads) {
        const float v = stage[i];
        int slot;
        uint32_t id;
        if (i < na) {                          // rank = own index + #b strictly below
            int lo = 0, hi = nb;
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (sb[mid] < v) lo = mid + 1; else hi = mid; }
            slot = i + lo;
            id = (uint32_t)(ia0 + i);
        } else {                               // rank = own index + #a not above
            const int j = i - na;
            int lo = 0, hi = na;
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (sa[mid] <= v) lo = mid + 1; else hi = mid; }
            slot = j + lo;
            id = (uint32_t)(k + ib0 + j);
        }
        okey[slot] = float_to_key(v);
        oid[slot] = id;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < na + nb; i += kMergeThreads) {
        keys[d0 + i] = okey[i];
        ids[d0 + i] = oid[i];
    }
}

// ---------------------------------------------------------------------------
// Decay between sorted neighbours (Sec. 3 "Symmetric case": the recurrence
// y_{i+1} = x_{i+1} + exp(a_i - a_{i+1}) y_i).  A negative entry marks "same key
// as the predecessor": the decay is exactly 1 and the position does not start
// a new run of equal anchors (needed for the strict sums of the gradients).
__global__ void __launch_bounds__(256)
k_decay(const uint32_t* __restrict__ keys, float* __restrict__ dh, int64_t N)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j <= N; j += stride) {
        float d = 0.0f;
        if (j > 0 && j < N) {
            const uint32_t k1 = keys[j], k0 = keys[j - 1];
            d = k1 == k0 ? -1.0f : expf(-(key_to_float(k1) - key_to_float(k0)));
        }
        dh[j] = d;
    }
}

__global__ void __launch_bounds__(256)
k_fill(float* __restrict__ p, int64_t rows, int64_t cols, int64_t ld, float v)
{
    const int64_t total = rows * cols;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride)
        p[(i / cols) * ld + (i % cols)] = v;
}

__global__ void __launch_bounds__(256)
k_copy_u32(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst, int64_t count)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) dst[i] = src[i];
}

inline unsigned grid_for(int64_t work, int threads, int64_t cap = 1 << 16)
{
    int64_t g = (work + threads - 1) / threads;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (unsigned)g;
}

}  // namespace

hipError_t launch_make_keys(const float* a, int64_t k, const float* b, int64_t n,
                            uint32_t* keys, uint32_t* ids, hipStream_t st)
{
    LAPLEX_TIMED("make_keys", st, hipLaunchKernelGGL(k_make_keys, dim3(grid_for(k + n, 256)), dim3(256), 0, st, a, k, b, n, keys, ids));
    return hipGetLastError();
}

hipError_t launch_radix_sort(uint32_t* keys0, uint32_t* ids0, uint32_t* keys1, uint32_t* ids1,
                             uint32_t* table, uint32_t* chunks, int64_t N, hipStream_t st)
{
    const int64_t tiles = (N + kSortTile - 1) / kSortTile;
    const int64_t len = tiles * kRadix;
    const int64_t nchunks = (len + kTableScanChunk - 1) / kTableScanChunk;
    uint32_t* kin = keys0; uint32_t* iin = ids0; uint32_t* kout = keys1; uint32_t* iout = ids1;
    for (int pass = 0; pass < kSortPasses; ++pass) {
        const int shift = pass * kRadixBits;
        LAPLEX_TIMED("radix_count", st, hipLaunchKernelGGL(k_radix_count, dim3((unsigned)tiles), dim3(kSortThreads), 0, st,
                           (const uint32_t*)kin, N, shift, table, tiles));
        LAPLEX_TIMED("table_scan", st, hipLaunchKernelGGL(k_table_chunk_sums, dim3((unsigned)nchunks), dim3(kTableScanThreads), 0, st,
                           (const uint32_t*)table, len, chunks));
        LAPLEX_TIMED("table_scan", st, hipLaunchKernelGGL(k_table_chunk_scan, dim3(1), dim3(1024), 0, st, chunks, nchunks));
        LAPLEX_TIMED("table_scan", st, hipLaunchKernelGGL(k_table_scan_apply, dim3((unsigned)nchunks), dim3(kTableScanThreads), 0, st,
                           table, len, (const uint32_t*)chunks));
        LAPLEX_TIMED("radix_scatter", st, hipLaunchKernelGGL(k_radix_scatter, dim3((unsigned)tiles), dim3(kSortThreads), 0, st,
                           (const uint32_t*)kin, (const uint32_t*)iin, kout, iout, N, shift,
                           (const uint32_t*)table, tiles));
        uint32_t* t = kin; kin = kout; kout = t;
        t = iin; iin = iout; iout = t;
    }
    return hipGetLastError();
}

hipError_t launch_merge(const float* a, int64_t k, const float* b, int64_t n,
                        uint32_t* keys, uint32_t* ids, hipStream_t st)
{
    const int64_t N = k + n;
    const int64_t tiles = (N + kMergeTile - 1) / kMergeTile;
    LAPLEX_TIMED("merge", st, hipLaunchKernelGGL(k_merge, dim3((unsigned)tiles), dim3(kMergeThreads), 0, st, a, k, b, n, keys, ids));
    return hipGetLastError();
}

hipError_t launch_decay(const uint32_t* keys, float* dh, int64_t N, hipStream_t st)
{
    LAPLEX_TIMED("decay", st, hipLaunchKernelGGL(k_decay, dim3(grid_for(N + 1, 256)), dim3(256), 0, st, keys, dh, N));
    return hipGetLastError();
}

hipError_t launch_fill(float* p, int64_t rows, int64_t cols, int64_t ld, float v, hipStream_t st)
{
    if (rows <= 0 || cols <= 0) return hipSuccess;
    LAPLEX_TIMED("fill", st, hipLaunchKernelGGL(k_fill, dim3(grid_for(rows * cols, 256)), dim3(256), 0, st, p, rows, cols, ld, v));
    return hipGetLastError();
}

hipError_t launch_copy_u32(const uint32_t* src, uint32_t* dst, int64_t count, hipStream_t st)
{
    if (count <= 0) return hipSuccess;
    LAPLEX_TIMED("copy", st, hipLaunchKernelGGL(k_copy_u32, dim3(grid_for(count, 256)), dim3(256), 0, st, src, dst, count));
    return hipGetLastError();
}

}  // namespace laplex
