// Moving values between the caller's order and the sorted order of the plan without random accesses
// (the gather of S4 and the scatter of S7 at batch 1; Sec. 3 "Complexity": the permutation is the price
// of sorting arbitrary anchors).
//
// At batch 1 a row is one float.  Fetching x[id] for a billion sorted positions costs a 128-byte line
// per float, and storing a result at y[id] a partial line; both are bound by the number of memory
// transactions, not by bytes.  Here every value travels as a record (destination, value[, value]) through
// at most two partition passes, each of which reads its records once and writes them once in runs, and a
// last pass that places the records of one window of 8192 consecutive destinations inside LDS and writes
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
// histogram pass is needed and nothing has to be stable; a tile ranks its records with returning LDS
// atomics and learns where its runs start from a chained look-back over per-tile status words, the
// protocol of the radix sort's passes (tiles numbered by a ticket, so every predecessor of a running tile
// is running; bounded spin, so that a lost wake-up marks the plan invalid instead of hanging the device).
#include "laplex_internal.h"

#include <string>

namespace laplex {

namespace {

constexpr int kPtThreads = 512;
constexpr int kPtPer = 16;                               // records per thread
constexpr int kPtTile = kPtThreads * kPtPer;             // 8192 records per tile
static_assert(kPtTile == (1 << kPermuteWindowBits), "a tile of level 2 is one window's worth of records");
constexpr int kPtSpinLimit = 1 << 24;
constexpr uint32_t kCountMask = (1u << 30) - 1u;         // status word: state in the top two bits, a record count below

struct PartArgs {
    int mode;                      // PermuteJob::Source, or kFromRecords for the second level
    // sources
    const uint32_t* ids; uint32_t lo, hi;               // rows: destination = ids[j] - lo for lo <= ids[j] < hi
    const uint32_t* rank;                               // values: destination = rank[i]
    const float* val0; const float* val1; int64_t ld_val;
    int64_t count;                                      // source rows / values
    const uint32_t* in_d; const float* in_v0; const float* in_v1;   // records of the level before
    const uint32_t* prev_status; int64_t prev_last_tile; int prev_buckets;   // where that level left its bucket lengths
    // this level
    int chain_bits;                // a chain is 2^chain_bits consecutive tickets (one bucket of the level before); -1: one chain
    int bucket_bits, shift;        // digit = (destination >> shift) & (2^bucket_bits - 1)
    int region_shift;              // a bucket's region holds 2^region_shift records
    uint32_t* out_d; float* out_v0; float* out_v1;
    uint32_t* status; uint32_t* ticket; uint32_t* error;
    int64_t dest_count;            // destinations are below this
};

constexpr int kFromRecords = 3;

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
    __shared__ uint32_t hist[kMaxBuckets];          // records of the tile per bucket
    __shared__ uint32_t lstart[kMaxBuckets];        // first LDS slot of each bucket's run
    __shared__ uint32_t delta[kMaxBuckets];         // slot in the chain's output = delta[bucket] + LDS slot
    __shared__ uint32_t wsum[kPtThreads / 64];
    __shared__ uint32_t sd[kPtTile];
    __shared__ float sv0[kPtTile];
    __shared__ float sv1[NV == 2 ? kPtTile : 1];
    __shared__ uint32_t s_ticket;

    const int tid = threadIdx.x;
    const int buckets = 1 << A.bucket_bits;
    if (tid == 0) s_ticket = atomicAdd(A.ticket, 1u);
    for (int b = tid; b < buckets; b += kPtThreads) hist[b] = 0u;
    __syncthreads();
    const int64_t ticket = (int64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)s_ticket);
    const int64_t chain = A.chain_bits < 0 ? 0 : ticket >> A.chain_bits;
    const int64_t chunk = A.chain_bits < 0 ? ticket : ticket & (((int64_t)1 << A.chain_bits) - 1);

    // the tile's source records
    int64_t src0, src1;
    if (MODE == kFromRecords) {
        uint32_t len = A.prev_status[A.prev_last_tile * A.prev_buckets + chain] & kCountMask;   // records of this bucket
        const uint32_t cap = 1u << (A.chain_bits + kPermuteWindowBits);
        len = len < cap ? len : cap;                            // (a valid plan never fills a region beyond its size)
        const int64_t base = chain << A.chain_bits << kPermuteWindowBits;     // a chain of 2^chain_bits tiles covers its bucket's region
        src0 = base + chunk * kPtTile;
        src1 = base + len < src0 + kPtTile ? base + len : src0 + kPtTile;
    } else {
        src0 = ticket * kPtTile;
        src1 = A.count < src0 + kPtTile ? A.count : src0 + kPtTile;
    }
    if (src0 >= src1) return;        // nothing here, and nothing in any later tile of the chain: no one looks at this tile's words

    uint32_t dest[kPtPer], slot[kPtPer];
    float v0[kPtPer], v1[NV == 2 ? kPtPer : 1];
    bool ok[kPtPer];
#pragma unroll
    for (int i = 0; i < kPtPer; ++i) {
        const int64_t j = src0 + i * kPtThreads + tid;
        const bool in = j < src1;
        const int64_t jc = in ? j : src0;
        if (MODE == kFromRecords) {
            dest[i] = A.in_d[jc]; v0[i] = A.in_v0[jc];
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
    const uint32_t digit_mask = (uint32_t)buckets - 1u;
#pragma unroll
    for (int i = 0; i < kPtPer; ++i) {
        const uint32_t b = (dest[i] >> A.shift) & digit_mask;
        slot[i] = ok[i] ? atomicAdd(&hist[b], 1u) : 0u;         // the record's rank inside its bucket's run (any order will do)
    }
    __syncthreads();

    // runs in LDS: bucket order; each thread owns `per` consecutive buckets
    const int per = (buckets + kPtThreads - 1) / kPtThreads;      // 1 or 2
    uint32_t cnt[2] = {0u, 0u};
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int b = tid * per + q;
        if (q < per && b < buckets) cnt[q] = hist[b];
    }
    // publish the counts as soon as they are known: the tiles after this one wait for them
    uint32_t* const words = A.status + ticket * buckets;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int b = tid * per + q;
        if (q < per && b < buckets)
            __hip_atomic_store(words + b, ((chunk == 0 ? 2u : 1u) << 30) | cnt[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const uint32_t ex = block_exclusive_scan(cnt[0] + cnt[1], wsum);
    uint32_t before[2] = {0u, 0u};
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int b = tid * per + q;
        if (q < per && b < buckets) lstart[b] = ex + (q ? cnt[0] : 0u);
    }
    __syncthreads();

#pragma unroll
    for (int i = 0; i < kPtPer; ++i) {
        if (ok[i]) {
            const uint32_t s = lstart[(dest[i] >> A.shift) & digit_mask] + slot[i];
            sd[s] = dest[i]; sv0[s] = v0[i];
            if (NV == 2) sv1[s] = v1[i];
        }
    }

    // look-back: records of this bucket in the earlier tiles of the chain
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int b = tid * per + q;
        if (!(q < per && b < buckets)) continue;
        uint32_t sum = 0;
        bool done = chunk == 0;
        for (int64_t t = ticket - 1; !done; --t) {
            uint32_t x = __hip_atomic_load(A.status + t * buckets + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int spins = 0;
            while ((x >> 30) == 0 && spins < kPtSpinLimit) {
                __builtin_amdgcn_s_sleep(1);
                x = __hip_atomic_load(A.status + t * buckets + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ++spins;
            }
            if ((x >> 30) == 0) { *A.error = 1u; break; }       // gave up: the plan is marked invalid, nothing hangs
            sum += x & kCountMask;
            done = (x >> 30) == 2 || t == ticket - chunk;
        }
        before[q] = sum;
        if (chunk != 0)
            __hip_atomic_store(words + b, (2u << 30) | ((sum + cnt[q]) & kCountMask), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // first record of the bucket's region, relative to the chain's first region, minus the run's LDS slot
        delta[b] = ((uint32_t)b << A.region_shift) + sum - lstart[b];
    }
    __syncthreads();

    const uint32_t total = lstart[buckets - 1] + hist[buckets - 1];
    const int64_t chain_base = (chain << A.bucket_bits) << A.region_shift;
    const uint32_t region = 1u << A.region_shift;
#pragma unroll
    for (int i = 0; i < kPtPer; ++i) {
        const uint32_t s = (uint32_t)(i * kPtThreads + tid);
        if (s < total) {
            const uint32_t d = sd[s];
            const uint32_t b = (d >> A.shift) & digit_mask;
            const uint32_t off = delta[b] + s;                                  // inside the chain's output
            if (off - (b << A.region_shift) < region) {                         // a region never overflows for a permutation
                const int64_t g = chain_base + off;
                A.out_d[g] = d; A.out_v0[g] = sv0[s];
                if (NV == 2) A.out_v1[g] = sv1[s];
            }
        }
    }
}

struct FinalArgs {
    const uint32_t* in_d; const float* in_v0; const float* in_v1;
    const uint32_t* status; int buckets;           // the level that filled the windows: its status words, 2^bucket_bits per tile
    int chain_bits;                                // its chains (-1: one chain of `tiles` tiles)
    int64_t tiles;
    const uint32_t* prev_status; int64_t prev_last_tile; int prev_buckets;   // the level before it (chains only)
    float* out0; int64_t ld0; float* out1; int64_t ld1;
    int64_t dest_count;
    const uint32_t* poison;                        // the plan's status word, or null (never for the plan's own arrays)
};

// The last pass: one workgroup per window of 8192 consecutive destinations.
template <int NV>
__global__ void __launch_bounds__(kPtThreads)
k_part_final(const FinalArgs A)
{
    constexpr int W = 1 << kPermuteWindowBits;
    __shared__ float s0[W];
    __shared__ float s1[NV == 2 ? W : 1];
    const int tid = threadIdx.x;
    const int64_t w = blockIdx.x;
    // records of this window: the inclusive count that the last tile of its chain published
    int64_t last_tile;
    int bucket;
    if (A.chain_bits < 0) {
        last_tile = A.tiles - 1; bucket = (int)w;
    } else {
        const int64_t chain = w >> A.chain_bits;             // chains of level 2 have as many tiles as windows
        uint32_t len = A.prev_status[A.prev_last_tile * A.prev_buckets + chain] & kCountMask;
        const uint32_t cap = 1u << (A.chain_bits + kPermuteWindowBits);
        len = len < cap ? len : cap;
        last_tile = (chain << A.chain_bits) + ((int64_t)len + kPtTile - 1) / kPtTile - 1;
        bucket = (int)(w & (((int64_t)1 << A.chain_bits) - 1));
        if (len == 0) last_tile = -1;
    }
    uint32_t count = last_tile < 0 ? 0u : (A.status[last_tile * A.buckets + bucket] & kCountMask);
    if (count > (uint32_t)W) count = (uint32_t)W;
    for (int i = tid; i < W; i += kPtThreads) { s0[i] = 0.0f; if (NV == 2) s1[i] = 0.0f; }
    __syncthreads();
    const int64_t base = w << kPermuteWindowBits;
    for (uint32_t i = tid; i < count; i += kPtThreads) {
        const uint32_t d = A.in_d[base + i] & (uint32_t)(W - 1);
        s0[d] = A.in_v0[base + i];
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
k_zero_words(uint32_t* __restrict__ p, int64_t count, uint32_t* __restrict__ tickets)
{
    if (blockIdx.x == 0 && threadIdx.x < 2) tickets[threadIdx.x] = 0u;
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

size_t permute_status_words(int64_t source_count, int64_t dest_count)
{
    // an upper bound for every job with at most this many sources and destinations: level 1 has one tile per 8192
    // sources, level 2 one per window (padded to a power of two), and a tile has at most 2^9 words
    const int64_t tiles1 = (source_count + kPtTile - 1) / kPtTile;
    const int64_t windows = (dest_count + (1 << kPermuteWindowBits) - 1) >> kPermuteWindowBits;
    return (size_t)((tiles1 + ((int64_t)1 << ceil_log2(windows))) << kPermuteMaxBucketBits);
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
    const int64_t words1 = tiles1 * ((int64_t)1 << (p1 > 0 ? p1 : p2));
    const int64_t words2 = p1 > 0 ? tiles2 * ((int64_t)1 << p2) : 0;
    uint32_t* const status1 = J.status;
    uint32_t* const status2 = J.status + words1;

    {   // status words of both levels and the two ticket counters
        const int64_t words = words1 + words2;
        int64_t g = (words / 4 + 255) / 256; if (g < 1) g = 1; if (g > 65536) g = 65536;
        LAPLEX_TIMED("permute_zero", st, hipLaunchKernelGGL(k_zero_words, dim3((unsigned)g), dim3(256), 0, st, J.status, words, J.tickets));
    }

    PartArgs A{};
    A.mode = J.source;
    A.ids = J.ids; A.lo = J.lo; A.hi = J.hi; A.rank = J.rank;
    A.val0 = J.val0; A.val1 = J.val1; A.ld_val = J.ld_val; A.count = J.source_count;
    A.error = J.error; A.dest_count = J.dest_count;
    FinalArgs F{};
    F.dest_count = J.dest_count; F.out0 = J.out0; F.ld0 = J.ld0; F.out1 = J.out1; F.ld1 = J.ld1; F.poison = J.poison;
    const std::string f1 = std::string("permute_part.") + J.tag, f2 = std::string("permute_final.") + J.tag;
    if (p1 > 0) {
        // level 1: the source -> 2^p1 buckets of 2^p2 windows each, records into buffer A
        A.chain_bits = -1; A.bucket_bits = p1; A.shift = kPermuteWindowBits + p2; A.region_shift = kPermuteWindowBits + p2;
        A.out_d = J.rec_d[0]; A.out_v0 = J.rec_v0[0]; A.out_v1 = J.rec_v1[0];
        A.status = status1; A.ticket = J.tickets;
        if (J.values == 2) launch_level<2>(A, tiles1, f1.c_str(), st); else launch_level<1>(A, tiles1, f1.c_str(), st);
        // level 2: each bucket -> its windows, records into buffer B
        PartArgs B2 = A;
        B2.mode = kFromRecords;
        B2.in_d = J.rec_d[0]; B2.in_v0 = J.rec_v0[0]; B2.in_v1 = J.rec_v1[0];
        B2.prev_status = status1; B2.prev_last_tile = tiles1 - 1; B2.prev_buckets = 1 << p1;
        B2.chain_bits = p2; B2.bucket_bits = p2; B2.shift = kPermuteWindowBits; B2.region_shift = kPermuteWindowBits;
        B2.out_d = J.rec_d[1]; B2.out_v0 = J.rec_v0[1]; B2.out_v1 = J.rec_v1[1];
        B2.status = status2; B2.ticket = J.tickets + 1;
        if (J.values == 2) launch_level<2>(B2, tiles2, f1.c_str(), st); else launch_level<1>(B2, tiles2, f1.c_str(), st);
        F.in_d = J.rec_d[1]; F.in_v0 = J.rec_v0[1]; F.in_v1 = J.rec_v1[1];
        F.status = status2; F.buckets = 1 << p2; F.chain_bits = p2; F.tiles = tiles2;
        F.prev_status = status1; F.prev_last_tile = tiles1 - 1; F.prev_buckets = 1 << p1;
    } else {
        // one level: the source -> windows
        A.chain_bits = -1; A.bucket_bits = p2; A.shift = kPermuteWindowBits; A.region_shift = kPermuteWindowBits;
        A.out_d = J.rec_d[0]; A.out_v0 = J.rec_v0[0]; A.out_v1 = J.rec_v1[0];
        A.status = status1; A.ticket = J.tickets;
        if (J.values == 2) launch_level<2>(A, tiles1, f1.c_str(), st); else launch_level<1>(A, tiles1, f1.c_str(), st);
        F.in_d = J.rec_d[0]; F.in_v0 = J.rec_v0[0]; F.in_v1 = J.rec_v1[0];
        F.status = status1; F.buckets = 1 << p2; F.chain_bits = -1; F.tiles = tiles1;
    }
    if (J.values == 2) LAPLEX_TIMED(f2.c_str(), st, hipLaunchKernelGGL((k_part_final<2>), dim3((unsigned)windows), dim3(kPtThreads), 0, st, F));
    else LAPLEX_TIMED(f2.c_str(), st, hipLaunchKernelGGL((k_part_final<1>), dim3((unsigned)windows), dim3(kPtThreads), 0, st, F));
    return hipGetLastError();
}

}  // namespace laplex
