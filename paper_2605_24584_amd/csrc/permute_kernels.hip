// Moving values between the caller's order and the sorted order of the plan without random accesses
// (the gather of S4 and the scatter of S7 at batch 1; Sec. 3 "Complexity": the permutation is the price
// of sorting arbitrary anchors).
//
// At batch 1 a row is one float.  Fetching x[id] for a billion sorted positions costs a 128-byte line
// per float, and storing a result at y[id] a partial line; both are bound by the number of memory
// transactions, not by bytes.  Here every value travels as a record (destination, value[, value]) through
// at most two partition passes, each of which reads its records once and writes them once in runs, and a
// last pass that places the records of one window of 16384 consecutive destinations inside LDS and writes
// the window out whole:
//
//   level 1   records -> up to 512 buckets by the top bits of the destination (only when there are more
//             than 512 windows)
//   level 2   the records of one bucket -> its (up to 512) windows
//   final     one workgroup per window: scatter inside LDS, coalesced store (destinations that no record
//             names read as zero)
//
// Destinations are positions of a permutation, so a bucket that covers C destinations receives at most C
// records: its region in the record arrays is simply the stretch [first destination, first + C).  No
// histogram pass is needed, nothing has to be stable and no tile waits for another: a tile ranks its records
// with returning LDS atomics and reserves the stretch for each of its runs with ONE returning atomic on the
// bucket's cursor (device scope).  Measured on this device: 512 such atomics per tile of 64 KB, all tiles on
// the same 512 words, cost 15 % on top of a plain copy of the tile.  The order of the records inside a bucket
// depends on the order in which the atomics land; the result does not (every destination is written once).
#include "laplex_internal.h"

#include <string>

namespace laplex {

namespace {

constexpr int kPtThreads = 1024;
constexpr int kPtPer = 16;                               // records per thread
constexpr int kPtTile = kPtThreads * kPtPer;             // 16384 records per tile: a run is 32 records on average with 512 buckets
static_assert(kPtTile == (1 << kPermuteWindowBits), "a tile of level 2 is one window's worth of records");
constexpr int kFromRecords = 3;                          // source of level 2 (beside PermuteJob::Source)

struct PartArgs {
    int mode;                      // PermuteJob::Source, or kFromRecords
    // sources
    const uint32_t* ids; uint32_t lo, hi;               // rows: destination = ids[j] - lo for lo <= ids[j] < hi
    const uint32_t* rank;                               // values: destination = rank[i]
    const float* val0; const float* val1; int64_t ld_val;
    int64_t count;                                      // source rows / values
    const uint2* in_dv; const float* in_v1;             // records of the level before: (destination, first value), second value ...
    const uint32_t* in_len;                             // ... and how many each of its buckets holds (its cursors)
    // this level
    int chain_bits;                // level 2: a bucket of the level before is read by 2^chain_bits consecutive tiles; -1: tiles over the source
    int bucket_bits, shift;        // digit = (destination >> shift) & (2^bucket_bits - 1)
    int region_shift;              // a bucket's region holds 2^region_shift records
    uint2* out_dv; float* out_v1;
    uint32_t* cursor;              // records placed so far, per bucket of this level (zero when the level starts)
    int64_t dest_count;            // destinations are below this
};

__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wsum /* kPtThreads / 64 words of LDS */)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    uint32_t before = 0;
#pragma unroll
    for (int w = 0; w < kPtThreads / 64; ++w) before += w < wave ? wsum[w] : 0u;
    __syncthreads();
    return before + inc - v;
}

// One partition level.  NV: values per record (1 or 2).
template <int MODE, int NV>
__global__ void __launch_bounds__(kPtThreads)
k_part(const PartArgs A)
{
    constexpr int kMaxBuckets = 1 << kPermuteMaxBucketBits;
    static_assert(kMaxBuckets <= kPtThreads, "one thread per bucket");
    __shared__ uint32_t hist[kMaxBuckets];          // records of the tile per bucket
    __shared__ uint32_t lstart[kMaxBuckets];        // first LDS slot of each bucket's run
    __shared__ uint32_t delta[kMaxBuckets];         // slot in the chain's output = delta[bucket] + LDS slot
    __shared__ uint32_t wsum[kPtThreads / 64];
    __shared__ uint2 sdv[kPtTile];                  // the tile's records, bucket by bucket: (destination, first value); then the second values

    const int tid = threadIdx.x;
    const int buckets = 1 << A.bucket_bits;
    if (tid < buckets) hist[tid] = 0u;
    const int64_t tile = blockIdx.x;
    const int64_t chain = A.chain_bits < 0 ? 0 : tile >> A.chain_bits;
    const int64_t chunk = A.chain_bits < 0 ? tile : tile & (((int64_t)1 << A.chain_bits) - 1);

    // the tile's source records
    int64_t src0, src1;
    if (MODE == kFromRecords) {
        uint32_t len = A.in_len[chain];                         // records of this bucket of the level before
        const uint32_t cap = 1u << (A.chain_bits + kPermuteWindowBits);
        len = len < cap ? len : cap;                            // (a valid plan never fills a region beyond its size)
        const int64_t base = chain << A.chain_bits << kPermuteWindowBits;     // 2^chain_bits tiles cover the bucket's region
        src0 = base + chunk * kPtTile;
        src1 = base + len < src0 + kPtTile ? base + len : src0 + kPtTile;
    } else {
        src0 = tile * kPtTile;
        src1 = A.count < src0 + kPtTile ? A.count : src0 + kPtTile;
    }
    if (src0 >= src1) return;

    uint32_t dest[kPtPer], slot[kPtPer];
    float v0[kPtPer], v1[NV == 2 ? kPtPer : 1];
    bool ok[kPtPer];
#pragma unroll
    for (int i = 0; i < kPtPer; ++i) {
        const int64_t j = src0 + i * kPtThreads + tid;
        const bool in = j < src1;
        const int64_t jc = in ? j : src0;
        if (MODE == kFromRecords) {
            const uint2 dv = A.in_dv[jc];
            dest[i] = dv.x; v0[i] = __uint_as_float(dv.y);
            if (NV == 2) v1[i] = A.in_v1[jc];
            ok[i] = in;
        } else if (MODE == PermuteJob::kRows) {
            const uint32_t id = A.ids[jc];
            ok[i] = in && id >= A.lo && id < A.hi;
            dest[i] = id - A.lo;
            v0[i] = A.val0[jc * A.ld_val];
            if (NV == 2) v1[i] = A.val1[jc * A.ld_val];
        } else if (MODE == PermuteJob::kRowIndex) {
            dest[i] = A.ids[jc];
            v0[i] = __uint_as_float((uint32_t)jc);
            ok[i] = in;
        } else {
            dest[i] = A.rank[jc];
            v0[i] = A.val0[jc * A.ld_val];
            if (NV == 2) v1[i] = A.val1[jc * A.ld_val];
            ok[i] = in;
        }
        ok[i] = ok[i] && (int64_t)dest[i] < A.dest_count;      // always true for a valid plan; keeps every store inside the arrays
    }
    __syncthreads();
    const uint32_t digit_mask = (uint32_t)buckets - 1u;
#pragma unroll
    for (int i = 0; i < kPtPer; ++i) {
        const uint32_t b = (dest[i] >> A.shift) & digit_mask;
        slot[i] = ok[i] ? atomicAdd(&hist[b], 1u) : 0u;         // the record's rank inside its bucket's run (any order will do)
    }
    __syncthreads();

    // thread b reserves the stretch of bucket b's region for this tile's run: one returning atomic, whose answer
    // travels while the runs are laid out in LDS
    const uint32_t cnt = tid < buckets ? hist[tid] : 0u;
    uint32_t before = 0u;
    if (cnt) before = atomicAdd(A.cursor + (chain << A.bucket_bits) + tid, cnt);
    const uint32_t ex = block_exclusive_scan(cnt, wsum);
    if (tid < buckets) lstart[tid] = ex;
    __syncthreads();
    uint32_t place[kPtPer];
#pragma unroll
    for (int i = 0; i < kPtPer; ++i) {
        place[i] = lstart[(dest[i] >> A.shift) & digit_mask] + slot[i];
        if (ok[i]) sdv[place[i]] = make_uint2(dest[i], __float_as_uint(v0[i]));
    }
    // first record of the bucket's region, relative to the chain's first region, minus the run's LDS slot
    if (tid < buckets) delta[tid] = ((uint32_t)tid << A.region_shift) + before - ex;
    __syncthreads();

    const uint32_t total = lstart[buckets - 1] + hist[buckets - 1];
    const int64_t chain_base = (chain << A.bucket_bits) << A.region_shift;
    const uint32_t region = 1u << A.region_shift;
    int64_t where[kPtPer];
#pragma unroll
    for (int i = 0; i < kPtPer; ++i) {
        const uint32_t s = (uint32_t)(i * kPtThreads + tid);
        where[i] = -1;
        if (s < total) {
            const uint2 dv = sdv[s];
            const uint32_t b = (dv.x >> A.shift) & digit_mask;
            const uint32_t off = delta[b] + s;                                  // inside the chain's output
            if (off - (b << A.region_shift) < region) {                         // a region never overflows for a permutation
                where[i] = chain_base + off;
                A.out_dv[where[i]] = dv;
            }
        }
    }
    if (NV == 2) {          // the second values through the same LDS array
        float* const sv = reinterpret_cast<float*>(sdv);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kPtPer; ++i)
            if (ok[i]) sv[place[i]] = v1[i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kPtPer; ++i)
            if (where[i] >= 0) A.out_v1[where[i]] = sv[i * kPtThreads + tid];
    }
}

struct FinalArgs {
    const uint2* in_dv; const float* in_v1;
    const uint32_t* in_len;                        // records of each window (the cursors of the level that filled them)
    float* out0; int64_t ld0; float* out1; int64_t ld1;
    int64_t dest_count;
    const uint32_t* poison;                        // the plan's status word, or null (never for the plan's own arrays)
};

// The last pass: one workgroup per window of 16384 consecutive destinations.
template <int NV>
__global__ void __launch_bounds__(kPtThreads)
k_part_final(const FinalArgs A)
{
    constexpr int W = 1 << kPermuteWindowBits;
    __shared__ float s0[W];
    __shared__ float s1[NV == 2 ? W : 1];
    const int tid = threadIdx.x;
    const int64_t w = blockIdx.x;
    uint32_t count = A.in_len[w];
    if (count > (uint32_t)W) count = (uint32_t)W;
    for (int i = tid; i < W; i += kPtThreads) { s0[i] = 0.0f; if (NV == 2) s1[i] = 0.0f; }
    __syncthreads();
    const int64_t base = w << kPermuteWindowBits;
    for (uint32_t i = tid; i < count; i += kPtThreads) {
        const uint2 dv = A.in_dv[base + i];
        const uint32_t d = dv.x & (uint32_t)(W - 1);
        s0[d] = __uint_as_float(dv.y);
        if (NV == 2) s1[d] = A.in_v1[base + i];
    }
    __syncthreads();
    const uint32_t poison = (A.poison != nullptr && *A.poison != 0u) ? 0x7FC00000u : 0u;
    for (int i = tid; i < W; i += kPtThreads) {
        const int64_t d = base + i;
        if (d < A.dest_count) {
            A.out0[d * A.ld0] = __uint_as_float(__float_as_uint(s0[i]) | poison);
            if (NV == 2) A.out1[d * A.ld1] = __uint_as_float(__float_as_uint(s1[i]) | poison);
        }
    }
}

__global__ void __launch_bounds__(256)
k_zero_words(uint32_t* __restrict__ p, int64_t count)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < count; i += stride) {
        if (i + 4 <= count) *reinterpret_cast<uint4*>(p + i) = make_uint4(0u, 0u, 0u, 0u);
        else for (int64_t j = i; j < count; ++j) p[j] = 0u;
    }
}

int ceil_log2(int64_t v) { int l = 0; while (((int64_t)1 << l) < v) ++l; return l; }

template <int NV>
void launch_level(const PartArgs& A, int64_t tiles, const char* family, hipStream_t st)
{
    const dim3 grid((unsigned)tiles), block(kPtThreads);
    switch (A.mode) {
        case PermuteJob::kRows:     LAPLEX_TIMED(family, st, hipLaunchKernelGGL((k_part<PermuteJob::kRows, NV>), grid, block, 0, st, A)); break;
        case PermuteJob::kRowIndex: LAPLEX_TIMED(family, st, hipLaunchKernelGGL((k_part<PermuteJob::kRowIndex, NV>), grid, block, 0, st, A)); break;
        case PermuteJob::kValues:   LAPLEX_TIMED(family, st, hipLaunchKernelGGL((k_part<PermuteJob::kValues, NV>), grid, block, 0, st, A)); break;
        default:                    LAPLEX_TIMED(family, st, hipLaunchKernelGGL((k_part<kFromRecords, NV>), grid, block, 0, st, A)); break;
    }
}

}  // namespace

bool permute_supported(int64_t source_count, int64_t dest_count)
{
    if (source_count <= 0 || dest_count <= 0) return false;
    const int64_t windows = (dest_count + (1 << kPermuteWindowBits) - 1) >> kPermuteWindowBits;
    return ceil_log2(windows) <= 2 * kPermuteMaxBucketBits;
}

size_t permute_cursor_words(int64_t dest_count)
{
    // level 1: at most 2^9 buckets; level 2 (or the only level): one cursor per window, padded to a power of two
    const int64_t windows = (dest_count + (1 << kPermuteWindowBits) - 1) >> kPermuteWindowBits;
    return (size_t)(((int64_t)1 << kPermuteMaxBucketBits) + ((int64_t)1 << ceil_log2(windows)));
}

hipError_t launch_permute(const PermuteJob& J, hipStream_t st)
{
    if (J.source_count <= 0 || J.dest_count <= 0) return hipSuccess;
    const int64_t windows = (J.dest_count + (1 << kPermuteWindowBits) - 1) >> kPermuteWindowBits;
    const int lw = ceil_log2(windows);
    const int p2 = lw < kPermuteMaxBucketBits ? lw : kPermuteMaxBucketBits;
    const int p1 = lw - p2;
    const int64_t tiles1 = (J.source_count + kPtTile - 1) / kPtTile;
    const int64_t tiles2 = (int64_t)1 << (p1 + p2);
    uint32_t* const cursor1 = J.cursors;                                          // level 1's buckets
    uint32_t* const cursor2 = J.cursors + ((int64_t)1 << kPermuteMaxBucketBits);  // the windows
    {
        const int64_t words = ((int64_t)1 << kPermuteMaxBucketBits) + ((int64_t)1 << lw);
        int64_t g = (words / 4 + 255) / 256; if (g < 1) g = 1;
        LAPLEX_TIMED("permute_zero", st, hipLaunchKernelGGL(k_zero_words, dim3((unsigned)g), dim3(256), 0, st, J.cursors, words));
    }

    PartArgs A{};
    A.mode = J.source;
    A.ids = J.ids; A.lo = J.lo; A.hi = J.hi; A.rank = J.rank;
    A.val0 = J.val0; A.val1 = J.val1; A.ld_val = J.ld_val; A.count = J.source_count;
    A.dest_count = J.dest_count;
    FinalArgs F{};
    F.dest_count = J.dest_count; F.out0 = J.out0; F.ld0 = J.ld0; F.out1 = J.out1; F.ld1 = J.ld1; F.poison = J.poison;
    F.in_len = cursor2;
    const std::string f1 = std::string("permute_part.") + J.tag, f2 = std::string("permute_final.") + J.tag;
    A.chain_bits = -1;
    A.out_dv = J.rec_dv[0]; A.out_v1 = J.rec_v1[0];
    if (p1 > 0) {
        // level 1: the source -> 2^p1 buckets of 2^p2 windows each, records into buffer 0
        A.bucket_bits = p1; A.shift = kPermuteWindowBits + p2; A.region_shift = kPermuteWindowBits + p2;
        A.cursor = cursor1;
        if (J.values == 2) launch_level<2>(A, tiles1, f1.c_str(), st); else launch_level<1>(A, tiles1, f1.c_str(), st);
        // level 2: each bucket -> its windows, records into buffer 1
        PartArgs B2 = A;
        B2.mode = kFromRecords;
        B2.in_dv = J.rec_dv[0]; B2.in_v1 = J.rec_v1[0]; B2.in_len = cursor1;
        B2.chain_bits = p2; B2.bucket_bits = p2; B2.shift = kPermuteWindowBits; B2.region_shift = kPermuteWindowBits;
        B2.out_dv = J.rec_dv[1]; B2.out_v1 = J.rec_v1[1];
        B2.cursor = cursor2;
        if (J.values == 2) launch_level<2>(B2, tiles2, f1.c_str(), st); else launch_level<1>(B2, tiles2, f1.c_str(), st);
        F.in_dv = J.rec_dv[1]; F.in_v1 = J.rec_v1[1];
    } else {
        // one level: the source -> windows
        A.bucket_bits = p2; A.shift = kPermuteWindowBits; A.region_shift = kPermuteWindowBits;
        A.cursor = cursor2;
        if (J.values == 2) launch_level<2>(A, tiles1, f1.c_str(), st); else launch_level<1>(A, tiles1, f1.c_str(), st);
        F.in_dv = J.rec_dv[0]; F.in_v1 = J.rec_v1[0];
    }
    if (J.values == 2) LAPLEX_TIMED(f2.c_str(), st, hipLaunchKernelGGL((k_part_final<2>), dim3((unsigned)windows), dim3(kPtThreads), 0, st, F));
    else LAPLEX_TIMED(f2.c_str(), st, hipLaunchKernelGGL((k_part_final<1>), dim3((unsigned)windows), dim3(kPtThreads), 0, st, F));
    return hipGetLastError();
}

}  // namespace laplex
