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
#include "permute_tile.h"

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
    int chain_bits;                // level 2: a bucket of the level before is read by 2^chain_bits consecutive tiles; -1: tiles over the source
    PartEmit emit;                 // this level
};

// One partition level.  NV: values per record (1 or 2).
template <int MODE, int NV>
__global__ void __launch_bounds__(kPtThreads)
k_part(const PartArgs A)
{
    __shared__ PartShared<kPtThreads> S;
    __shared__ uint2 sdv[kPtTile];                  // the tile's records, bucket by bucket: (destination, first value); then the second values
    const int tid = threadIdx.x;
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

    uint32_t dest[kPtPer];
    float v0[kPtPer], v1[NV == 2 ? kPtPer : 1];
    uint32_t okmask = 0u;
#pragma unroll
    for (int i = 0; i < kPtPer; ++i) {
        const int64_t j = src0 + i * kPtThreads + tid;
        const bool in = j < src1;
        const int64_t jc = in ? j : src0;
        bool ok;
        if (MODE == kFromRecords) {
            const uint2 dv = A.in_dv[jc];
            dest[i] = dv.x; v0[i] = __uint_as_float(dv.y);
            if (NV == 2) v1[i] = A.in_v1[jc];
            ok = in;
        } else if (MODE == PermuteJob::kRows) {
            const uint32_t id = A.ids[jc];
            ok = in && id >= A.lo && id < A.hi;
            dest[i] = id - A.lo;
            v0[i] = A.val0[jc * A.ld_val];
            if (NV == 2) v1[i] = A.val1[jc * A.ld_val];
        } else if (MODE == PermuteJob::kRowIndex) {
            dest[i] = A.ids[jc];
            v0[i] = __uint_as_float((uint32_t)jc);
            ok = in;
        } else {
            dest[i] = A.rank[jc];
            v0[i] = A.val0[jc * A.ld_val];
            if (NV == 2) v1[i] = A.val1[jc * A.ld_val];
            ok = in;
        }
        ok = ok && (int64_t)dest[i] < A.emit.dest_count;      // always true for a valid plan; keeps every store inside the arrays
        okmask |= ok ? 1u << i : 0u;
    }
    PartTicket<kPtPer> K;
    partition_reserve<kPtThreads, kPtPer>(A.emit, chain, dest, okmask, S, K);
    partition_place<kPtThreads, kPtPer, NV>(A.emit, chain, dest, okmask, v0, v1, S, sdv, K);
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

namespace {
struct Geom { int lw, p1, p2; int64_t windows, tiles2; };
Geom geom_of(int64_t dest_count)
{
    Geom g;
    g.windows = (dest_count + (1 << kPermuteWindowBits) - 1) >> kPermuteWindowBits;
    g.lw = ceil_log2(g.windows);
    g.p2 = g.lw < kPermuteMaxBucketBits ? g.lw : kPermuteMaxBucketBits;
    g.p1 = g.lw - g.p2;
    g.tiles2 = (int64_t)1 << (g.p1 + g.p2);
    return g;
}
}  // namespace

hipError_t permute_begin(const PermuteJob& J, PartEmit* first_level, hipStream_t st)
{
    const Geom g = geom_of(J.dest_count);
    uint32_t* const cursor1 = J.cursors;                                          // level 1's buckets
    uint32_t* const cursor2 = J.cursors + ((int64_t)1 << kPermuteMaxBucketBits);  // the windows
    const int64_t words = ((int64_t)1 << kPermuteMaxBucketBits) + ((int64_t)1 << g.lw);
    int64_t grid = (words / 4 + 255) / 256; if (grid < 1) grid = 1;
    LAPLEX_TIMED("permute_zero", st, hipLaunchKernelGGL(k_zero_words, dim3((unsigned)grid), dim3(256), 0, st, J.cursors, words));
    PartEmit E;
    E.out_dv = J.rec_dv[0]; E.out_v1 = J.rec_v1[0]; E.dest_count = J.dest_count;
    if (g.p1 > 0) {      // two levels: the first one fills 2^p1 buckets of 2^p2 windows each
        E.bucket_bits = g.p1; E.shift = kPermuteWindowBits + g.p2; E.region_shift = kPermuteWindowBits + g.p2; E.cursor = cursor1;
    } else {             // one level: straight into the windows
        E.bucket_bits = g.p2; E.shift = kPermuteWindowBits; E.region_shift = kPermuteWindowBits; E.cursor = cursor2;
    }
    *first_level = E;
    return hipGetLastError();
}

hipError_t permute_finish(const PermuteJob& J, hipStream_t st)
{
    const Geom g = geom_of(J.dest_count);
    uint32_t* const cursor1 = J.cursors;
    uint32_t* const cursor2 = J.cursors + ((int64_t)1 << kPermuteMaxBucketBits);
    const std::string f1 = std::string("permute_part.") + J.tag, f2 = std::string("permute_final.") + J.tag;
    FinalArgs F{};
    F.dest_count = J.dest_count; F.out0 = J.out0; F.ld0 = J.ld0; F.out1 = J.out1; F.ld1 = J.ld1; F.poison = J.poison;
    F.in_len = cursor2;
    F.in_dv = J.rec_dv[0]; F.in_v1 = J.rec_v1[0];
    if (g.p1 > 0) {      // level 2: each bucket of level 1 -> its windows, records into the second buffer
        PartArgs A{};
        A.mode = kFromRecords;
        A.in_dv = J.rec_dv[0]; A.in_v1 = J.rec_v1[0]; A.in_len = cursor1;
        A.chain_bits = g.p2;
        A.emit.bucket_bits = g.p2; A.emit.shift = kPermuteWindowBits; A.emit.region_shift = kPermuteWindowBits;
        A.emit.out_dv = J.rec_dv[1]; A.emit.out_v1 = J.rec_v1[1]; A.emit.cursor = cursor2; A.emit.dest_count = J.dest_count;
        if (J.values == 2) launch_level<2>(A, g.tiles2, f1.c_str(), st); else launch_level<1>(A, g.tiles2, f1.c_str(), st);
        F.in_dv = J.rec_dv[1]; F.in_v1 = J.rec_v1[1];
    }
    if (J.values == 2) LAPLEX_TIMED(f2.c_str(), st, hipLaunchKernelGGL((k_part_final<2>), dim3((unsigned)g.windows), dim3(kPtThreads), 0, st, F));
    else LAPLEX_TIMED(f2.c_str(), st, hipLaunchKernelGGL((k_part_final<1>), dim3((unsigned)g.windows), dim3(kPtThreads), 0, st, F));
    return hipGetLastError();
}

hipError_t launch_permute(const PermuteJob& J, hipStream_t st)
{
    if (J.source_count <= 0 || J.dest_count <= 0) return hipSuccess;
    PartArgs A{};
    hipError_t e = permute_begin(J, &A.emit, st);
    if (e != hipSuccess) return e;
    A.mode = J.source;
    A.ids = J.ids; A.lo = J.lo; A.hi = J.hi; A.rank = J.rank;
    A.val0 = J.val0; A.val1 = J.val1; A.ld_val = J.ld_val; A.count = J.source_count;
    A.chain_bits = -1;
    const std::string f1 = std::string("permute_part.") + J.tag;
    const int64_t tiles1 = (J.source_count + kPtTile - 1) / kPtTile;
    if (J.values == 2) launch_level<2>(A, tiles1, f1.c_str(), st); else launch_level<1>(A, tiles1, f1.c_str(), st);
    return permute_finish(J, st);
}

}  // namespace laplex
