// Internal declarations shared by the host API and the kernel files of liblaplex.
// Nothing here is part of the public boundary (that is include/laplex.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace laplex {

// ----------------------------------------------------------------------------
// Sort geometry (LSD radix sort, 8-bit digits, 4 passes over 32-bit keys).
// ----------------------------------------------------------------------------
constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kSortPasses = 4;
constexpr int kSortThreads = 512;                       // 8 wavefronts
// Keys per thread of a sort pass, hence per tile (512 x 4, 8 or 16).  A short sort is bound by the latency of one
// tile (its ranking, the hop from tile to tile), not by throughput: it gets smaller tiles, so more of them run side by side.
inline int sort_keys_per_thread(int64_t N) { return N <= (int64_t(1) << 18) ? 4 : N <= (int64_t(5) << 18) ? 8 : 16; }
inline int64_t sort_tile(int64_t N) { return (int64_t)kSortThreads * sort_keys_per_thread(N); }
// keys per workgroup of the histogram kernel (up to its grid limit): fewer for a short sort, whose histogram is bound by
// the latency of one workgroup; more for a long one, where every workgroup adds its 1024 counts to the global ones
inline int64_t sort_hist_tile(int64_t N) { return (int64_t)kSortThreads * (N <= (int64_t(1) << 18) ? 4 : 16); }
// Small state of one sort, u32 words: [0, 1024) histogram of the four digits; then the per-pass tile
// tickets, the error flag and the histogram's done counter in one cache line, and the mask of the passes that run in a line of its own.
constexpr int kSortTicketWord = 1024;
constexpr int kSortErrorWord = 1028;
constexpr int kSortDoneWord = 1029;                     // histogram workgroups that have added their counts
constexpr int kSortMaskWord = 1056;
constexpr int kSortSmallWords = 1088;
constexpr int kPlanStatusWord = 32;                     // in the plan's 64 counter words: the sort's error flag, kept with the plan
constexpr int kMergeThreads = 256;
constexpr int kMergePerThread = 8;
constexpr int kMergeTile = kMergeThreads * kMergePerThread;
// Problems with at most this many merged positions run in one launch, sorted and scanned inside one workgroup.
constexpr int kSmallMax = 8192;

// ----------------------------------------------------------------------------
// Scan geometry.  A workgroup of up to kScanWaves wavefronts owns one tile of
// consecutive merged positions ("rows").  A wavefront's 64 lanes are split into
// bv lanes across the batch (each lane holds `vec` adjacent batch columns) times
// rv = 64 / bv row-lanes; every row-lane walks `items` consecutive rows.
// ----------------------------------------------------------------------------
constexpr int kScanWaves = 8;     // wavefronts of a workgroup in the wide geometry and in the spine kernels
constexpr int kScanThreads = kScanWaves * 64;
// With 4 columns per lane and fewer than 64 lanes across the batch a block is owned by fewer wavefronts:
// the downsweep holds its rows in registers and fits one workgroup of eight per compute unit, two of
// four, and the smaller ones overlap each other's phases better (measured: 9 % on the Gram workload;
// with one column per lane it made no difference).
constexpr int kBlockWavesNarrow = 4;
constexpr int kItemsVec1 = 16;   // rows per row-lane when a lane holds 1 column
constexpr int kItemsVec4 = 8;    // rows per row-lane when a lane holds 4 columns
// A batch row narrower than this many floats is gathered once per problem and staged in sorted
// order: a random read of a few bytes costs a whole 128-byte line of HBM traffic.
constexpr int kStageMaxBatch = 8;
constexpr int kSpineItems = 8;    // tile summaries per row-lane in the chunked spine kernels, at most (ScanGeom::spine_items)
constexpr int kSpineThreads = 1024;

// ----------------------------------------------------------------------------
// Batch 1, many rows: values move between the caller's order and the sorted order as records through
// partition passes instead of by random accesses (permute_kernels.hip).  A window is the stretch of
// destinations that the last pass places inside LDS; a partition level has at most 2^9 buckets.
// ----------------------------------------------------------------------------
constexpr int kPermuteWindowBits = 14;
constexpr int kPermuteMaxBucketBits = 9;
bool permute_supported(int64_t source_count, int64_t dest_count);      // destinations fit two partition levels
size_t permute_cursor_words(int64_t dest_count);                        // the buckets' cursors of both levels
// records that a level's output array must hold for `dest_count` destinations: whole windows when one level fills
// the windows directly (at most 2^9 of them), else whole regions of 2^9 windows; and whether there are two levels
inline bool permute_two_levels(int64_t dest_count)
{
    return ((dest_count + ((int64_t)1 << kPermuteWindowBits) - 1) >> kPermuteWindowBits) > ((int64_t)1 << kPermuteMaxBucketBits);
}
inline int64_t permute_capacity(int64_t dest_count)
{
    const int64_t region = (int64_t)1 << (kPermuteWindowBits + (permute_two_levels(dest_count) ? kPermuteMaxBucketBits : 0));
    return (dest_count + region - 1) / region * region;
}

// The rows a downsweep workgroup owns are a "block" (tile_rows of them).  The spine works on
// "tiles": one block each, except in the wide geometry (64 lanes across the batch, 4 columns per
// lane, 64 rows per block), where a tile is 2^kWideSubShift consecutive blocks: a summary or a carry
// is then 4 * batch bytes per 64 * 4 * batch bytes of data, and fewer, larger ones are cheaper.
constexpr int kWideSubShift = 3;

struct ScanGeom {
    int vec;          // 1 or 4 batch columns per lane
    int items;        // rows per row-lane
    int bv;           // lanes across the batch (power of two, <= 64)
    int rv;           // row-lanes per wavefront
    int slabs;        // ceil(batch / (bv * vec)): blockIdx.y
    int waves;        // wavefronts per block workgroup
    int tile_rows;    // rows per block: waves * rv * items
    int sub_shift;    // log2(blocks per tile)
    int64_t blocks;   // ceil(N / tile_rows)
    int64_t tiles;    // ceil(blocks / 2^sub_shift)
    int spine_items;  // tile summaries per row-lane of the spine kernels: 8, or 4 when a summary is a whole wavefront wide
                      // (rv = 1): twice the workgroups, each done sooner
    int chunk_tiles;  // tiles summarised by one workgroup of the chunked spine: kScanWaves * rv * spine_items
    int64_t chunks;   // ceil(tiles / chunk_tiles)
};

inline int pow2_at_least(int64_t v) { int p = 1; while (p < v) p <<= 1; return p; }

inline ScanGeom scan_geom(int64_t N, int64_t batch, int vec)
{
    ScanGeom g;
    g.vec = vec;
    g.items = vec == 4 ? kItemsVec4 : kItemsVec1;
    const int64_t groups = (batch + vec - 1) / vec;          // column groups of `vec`
    g.bv = groups >= 64 ? 64 : pow2_at_least(groups < 1 ? 1 : groups);
    g.rv = 64 / g.bv;
    g.slabs = (int)((groups + g.bv - 1) / g.bv);
    if (g.slabs < 1) g.slabs = 1;
    g.sub_shift = (vec == 4 && g.bv == 64) ? kWideSubShift : 0;
    g.waves = (vec == 4 && !g.sub_shift) ? kBlockWavesNarrow : kScanWaves;
    g.tile_rows = g.waves * g.rv * g.items;
    g.blocks = (N + g.tile_rows - 1) / g.tile_rows;
    g.tiles = (g.blocks + (int64_t(1) << g.sub_shift) - 1) >> g.sub_shift;
    g.spine_items = g.rv == 1 ? kSpineItems / 2 : kSpineItems;
    g.chunk_tiles = kScanWaves * g.rv * g.spine_items;
    g.chunks = (g.tiles + g.chunk_tiles - 1) / g.chunk_tiles;
    return g;
}

// ----------------------------------------------------------------------------
// Workspace layout: a pure function of (merged length N, saved-scan rows,
// batch).  Plan first (ids, decays), then the saved-scan region, then scratch,
// which the sort and the scans use at different times and therefore share.
// ----------------------------------------------------------------------------
inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

struct Layout {
    int64_t N = 0, zrows = 0, batch = 0, bpad = 0;
    // plan
    size_t off_ids = 0;      // u32[N]    sorted ids
    size_t off_dh = 0;       // f32[N+1]  decay to the previous sorted key, < 0: same key
    size_t off_pk = 0;       // f32[N+2]  sorted anchors, shifted by one, between -inf and +inf sentinels
    size_t off_counters = 0; // u32[64]   words 0, 1: list lengths of the scans: zero between calls (the plan build clears them,
                             //           every scan clears them again in its last kernel); word kPlanStatusWord: 1 if the sort gave up a wait
    // saved scans
    size_t off_z = 0;        // f32[zrows][batch]
    size_t off_xs = 0;       // f32[N][batch], narrow batches only: the forward's injected rows in sorted order
    size_t off_scratch = 0;
    // scratch, sort view
    size_t off_pair0 = 0, off_pair1 = 0, off_status = 0, off_sort_small = 0;   // two buffers of (key, id) pairs
    int64_t sort_tiles = 0, status_words = 0;
    // scratch, scan view (sized for the larger of the two lane geometries)
    size_t off_agg_scalar = 0;   // float4[2][tiles]            (D, C, H, -)
    size_t off_agg_s = 0;        // f32[2][tiles][bpad]         S
    size_t off_agg_q = 0;        // f32[2][tiles][bpad]         Q
    size_t off_car_f = 0;        // f32[2][tiles][bpad]         carry F
    size_t off_car_e = 0;        // f32[2][tiles][bpad]         carry E
    size_t off_red = 0;          // f32[slabs][N]               per-slab partial row reductions
    size_t off_lists = 0;        // u32[tiles] tile list, u32[blocks] block list (sparse problems)
    size_t off_blk_flags = 0;    // u32[blocks]                 what each block holds (injected rows, result rows)
    size_t off_blk_f = 0;        // f32[2][blocks][bpad]        carry F into a block from the start of its tile (wide geometry)
    size_t off_blk_e = 0;        // f32[2][blocks][bpad]        the same, strict
    size_t off_stage = 0;        // f32[N][batch], narrow batches only: this problem's injected rows in sorted order
    // second level of the spine: the same five arrays over chunks of tiles
    size_t off_agg2_scalar = 0, off_agg2_s = 0, off_agg2_q = 0, off_car2_f = 0, off_car2_e = 0;
    int64_t max_tiles = 0, max_blocks = 0, max_chunks = 0;
    // small problems (N <= kSmallMax): f32[N][batch], the strict scans of the backward's second problem
    size_t off_small = 0;
    size_t off_pair = 0;         // f32[max(result rows)][2], batch 1 only
    // batch 1 beyond the small path: the routes through sorted order without random accesses
    bool permute = false;        // the regions below exist
    size_t off_rank = 0;         // u32[N]     plan: rank[id] = sorted position of anchor id
    size_t off_pk8 = 0;          // float2[(N+2)/8 + 1]  plan: (pk[8m], pk[8m + 1]), the anchors the sorted-order kernels need
    size_t off_rec_dv[2] = {0, 0}, off_rec_v1[2] = {0, 0};   // records of the two partition levels: (destination, value) pairs, second values
    size_t off_pt_cursors = 0;   // u32[permute_cursor_words]  records placed per bucket, both levels
    size_t total = 0;
};

inline Layout make_layout(int64_t N, int64_t zrows, int64_t batch, bool permute_regions = true)
{
    Layout L;
    L.N = N; L.zrows = zrows; L.batch = batch;
    L.bpad = (batch + 3) / 4 * 4;
    size_t o = 0;
    L.off_ids = o;  o = align_up(o + sizeof(uint32_t) * (size_t)N);
    L.off_dh = o;   o = align_up(o + sizeof(float) * (size_t)(N + 1));
    L.off_pk = o;   o = align_up(o + sizeof(float) * (size_t)(N + 2));
    L.off_counters = o; o = align_up(o + sizeof(uint32_t) * 64);
    L.off_z = o;    o = align_up(o + sizeof(float) * (size_t)zrows * (size_t)batch);
    const size_t stage_bytes = batch <= kStageMaxBatch ? sizeof(float) * (size_t)N * (size_t)batch : 0;
    L.off_xs = o;   o = align_up(o + stage_bytes);
    L.permute = permute_regions && batch == 1 && N > kSmallMax && permute_supported(N, N);
    L.off_rank = o;
    if (L.permute) o = align_up(o + sizeof(uint32_t) * (size_t)N);
    L.off_pk8 = o;
    if (L.permute) o = align_up(o + 2 * sizeof(float) * ((size_t)(N + 2) / 8 + 1));
    L.off_scratch = o;

    // sort view
    size_t s = o;
    L.sort_tiles = (N + sort_tile(N) - 1) / sort_tile(N);
    L.status_words = L.sort_tiles * kRadix;
    L.off_pair0 = s;  s = align_up(s + 2 * sizeof(uint32_t) * (size_t)N);
    L.off_pair1 = s;  s = align_up(s + 2 * sizeof(uint32_t) * (size_t)N);
    L.off_status = s;     s = align_up(s + sizeof(uint64_t) * 2 * (size_t)L.status_words);   // look-back words, two passes' worth
    L.off_sort_small = s; s = align_up(s + sizeof(uint32_t) * kSortSmallWords);            // global histogram, tickets, error, pass mask

    // scan view
    size_t c = o;
    const ScanGeom g1 = scan_geom(N, batch, 1), g4 = scan_geom(N, batch, 4);
    L.max_tiles = g1.tiles > g4.tiles ? g1.tiles : g4.tiles;
    L.max_blocks = g1.blocks > g4.blocks ? g1.blocks : g4.blocks;
    const size_t per_blk = sizeof(float) * 2 * (size_t)L.max_blocks * (size_t)L.bpad;
    const int max_slabs = g1.slabs > g4.slabs ? g1.slabs : g4.slabs;
    const size_t per = sizeof(float) * 2 * (size_t)L.max_tiles * (size_t)L.bpad;
    L.off_agg_scalar = c; c = align_up(c + sizeof(float) * 4 * 2 * (size_t)L.max_tiles);
    L.off_agg_s = c;      c = align_up(c + per);
    L.off_agg_q = c;      c = align_up(c + per);
    L.off_car_f = c;      c = align_up(c + per);
    L.off_car_e = c;      c = align_up(c + per);
    L.off_red = c;
    if (max_slabs > 1) c = align_up(c + sizeof(float) * (size_t)max_slabs * (size_t)N);
    L.off_lists = c; c = align_up(c + sizeof(uint32_t) * ((size_t)L.max_tiles + (size_t)L.max_blocks));
    L.off_blk_flags = c; c = align_up(c + sizeof(uint32_t) * (size_t)L.max_blocks);
    L.off_blk_f = c;     c = align_up(c + per_blk);
    L.off_blk_e = c;     c = align_up(c + per_blk);
    L.off_stage = c; c = align_up(c + stage_bytes);
    L.max_chunks = g1.chunks > g4.chunks ? g1.chunks : g4.chunks;
    const size_t per2 = sizeof(float) * 2 * (size_t)L.max_chunks * (size_t)L.bpad;
    L.off_agg2_scalar = c; c = align_up(c + sizeof(float) * 4 * 2 * (size_t)L.max_chunks);
    L.off_agg2_s = c;      c = align_up(c + per2);
    L.off_agg2_q = c;      c = align_up(c + per2);
    L.off_car2_f = c;      c = align_up(c + per2);
    L.off_car2_e = c;      c = align_up(c + per2);

    // batch 1: two outputs of a problem that land on the same rows (y and the saved scans; gx and gb) are written
    // as pairs and separated afterwards (two random 4-byte stores into one 8-byte slot cost what one costs, two into
    // two arrays twice that).  The pairs lie behind the scan view, on the sort view's buffers, which are dead by then.
    L.off_pair = align_up(c);
    const int64_t pair_rows = zrows > N - zrows ? zrows : N - zrows;
    if (batch == 1) c = align_up(L.off_pair + sizeof(float) * 2 * (size_t)pair_rows);
    L.total = s > c ? s : c;
    if (L.permute) {
        size_t q = align_up(L.total);
        const int64_t side = zrows > N - zrows ? zrows : N - zrows;      // result rows of a problem: at most this many
        const size_t cap1 = (size_t)permute_capacity(N), cap2 = (size_t)permute_capacity(side);
        for (int lv = 0; lv < 2; ++lv) {     // (the second level's buffers only where some move has two levels)
            L.off_rec_dv[lv] = q; if (lv == 0 || permute_two_levels(N)) q = align_up(q + 2 * sizeof(uint32_t) * cap1);
            L.off_rec_v1[lv] = q; if (lv == 0 || permute_two_levels(side)) q = align_up(q + sizeof(float) * cap2);
        }
        L.off_pt_cursors = q; q = align_up(q + sizeof(uint32_t) * permute_cursor_words(N));
        L.total = q;
    }
    L.off_small = align_up(L.total);
    if (N <= kSmallMax) L.total = align_up(L.off_small + sizeof(float) * (size_t)N * (size_t)batch);
    return L;
}

// ----------------------------------------------------------------------------
// Optional timing of one kernel family with HIP events on the launch stream
// (laplex_profile_begin / laplex_profile_end).  A no-op unless switched on.
// ----------------------------------------------------------------------------
void profile_before(const char* family, hipStream_t st);
void profile_after(const char* family, hipStream_t st);
#define LAPLEX_TIMED(family, st, launch)       \
    do {                                       \
        ::laplex::profile_before(family, st);  \
        launch;                                \
        ::laplex::profile_after(family, st);   \
    } while (0)

// ----------------------------------------------------------------------------
// Launchers (each returns the hipError_t of its launches; none synchronises).
// ----------------------------------------------------------------------------

// The anchors enter every plan scaled by the inverse temperature tau (1 = as they are).
// Stable ascending sort of the anchors a ++ b by one-sweep LSD passes.  Between passes the (key, id) pairs travel
// interleaved through the two pair buffers; the last pass that runs writes the sorted ids to `ids` and the sorted anchors
// to pk[1 .. N] (both the plan's).
// small: u32[kSortSmallWords] (global histogram, tickets, error word, pass mask); status: u64[2][tiles*256] look-back words.
hipError_t launch_onesweep_sort(const float* a, int64_t k, const float* b, int64_t n, float tau,
                                uint2* pair0, uint2* pair1, uint32_t* ids, float* pk,
                                uint32_t* small, unsigned long long* status, hipStream_t st);

// Both inputs ascending: merged keys/ids in one pass (ties: a first).
hipError_t launch_merge(const float* a, int64_t k, const float* b, int64_t n, float tau,
                        uint32_t* keys, uint32_t* ids, hipStream_t st);

// dh[j] = decay from sorted key j-1 to j (>= 0), or -1 if the two keys are equal;
// dh[0] = dh[N] = 0 (nothing beyond either end).  pk[j+1] = sorted anchor j, pk[0] = -inf, pk[N+1] = +inf.
// After the radix sort (ghist = its small words) the anchors are in pk[1 .. N] already and the kernel adds the sentinels;
// ghist == nullptr: the merge path, which leaves sorted keys in `keys`.  The last kernel of every plan build: it also
// clears the scans' list counters (64 words).
hipError_t launch_decay(const uint32_t* keys, const uint32_t* ghist, float* dh, float* pk, float2* pk8, uint32_t* counters,
                        int64_t N, hipStream_t st);

hipError_t launch_fill(float* p, int64_t rows, int64_t cols, int64_t ld, float v, hipStream_t st);
hipError_t launch_copy_u32(const uint32_t* src, uint32_t* dst, int64_t count, hipStream_t st);
// first[r * ld_first] = pairs[2r], second[r] = pairs[2r + 1]
hipError_t launch_unpair(const float* pairs, int64_t rows, float* first, int64_t ld_first, float* second, hipStream_t st);

// One scan problem over the merged sequence: inject rows of `inj` at positions
// whose id lies in [inj_lo, inj_hi), run the decayed scan in both directions and
// emit, at positions whose id lies in [res_lo, res_hi):
//   out_p[(id-res_lo)*ld_p + t] = F + R - v              (both inclusive scans)
//   out_z[(id-res_lo)*batch + t] = Z = E_right - E_left  (strict scans)
//   out_red[id-res_lo] = sum_t ( w[(id-res_lo)*ld_w + t] * Z
//                              + (zs ? v * zs[(id-res_lo)*batch + t] : 0) )
// Any of out_p / out_z / out_red may be null; strict scans run only if out_z or
// out_red is wanted.
// Where a tile places its records in one partition level (permute_tile.h).
struct PartEmit {
    int bucket_bits = 0, shift = 0;   // bucket of a record = (destination >> shift) & (2^bucket_bits - 1)
    int region_shift = 0;             // a bucket's region holds 2^region_shift records
    uint2* out_dv = nullptr;          // (destination, first value) pairs
    float* out_v1 = nullptr;          // second values
    uint32_t* cursor = nullptr;       // records placed so far, per bucket (zero when the level starts)
    int64_t dest_count = 0;           // destinations are below this
};

// One move of values between the caller's order and the sorted order (launch_permute).
//   kRows:     source row j of the sorted sequence goes to destination ids[j] - lo if lo <= ids[j] < hi (results back to
//              the caller's order); its values are val0[j * ld_val] (and val1[j * ld_val])
//   kRowIndex: destination ids[j], value j itself (as a 32-bit word): the inverse permutation
//   kValues:   source element i goes to destination rank[i] with value val0[i * ld_val] (the caller's rows into sorted order)
// The last pass writes out0[d * ld0] (and out1[d * ld1]) for EVERY destination d < dest_count: zero where no record arrived.
struct PermuteJob {
    enum Source { kRows = 0, kRowIndex = 1, kValues = 2 };
    int source = kRows;
    const uint32_t* ids = nullptr; uint32_t lo = 0, hi = 0;
    const uint32_t* rank = nullptr;
    const float* val0 = nullptr; const float* val1 = nullptr; int64_t ld_val = 1;
    int64_t source_count = 0, dest_count = 0;
    int values = 1;                                    // values per record: 1 or 2
    float* out0 = nullptr; int64_t ld0 = 1; float* out1 = nullptr; int64_t ld1 = 1;
    uint2* rec_dv[2] = {nullptr, nullptr}; float* rec_v1[2] = {nullptr, nullptr};   // records of the two levels
    uint32_t* cursors = nullptr;                       // permute_cursor_words(dest_count) words of scratch
    const uint32_t* poison = nullptr;                  // nonzero: every value written becomes a NaN (null: never)
    const char* tag = "move";                          // names the timing families permute_part.<tag>, permute_final.<tag>
};
hipError_t launch_permute(const PermuteJob& J, hipStream_t st);
// The same in two halves, for a producer that places the records of the first level itself (the batch-1 downsweep):
// permute_begin clears the cursors and says where the first level's records go; permute_finish runs what follows it.
hipError_t permute_begin(const PermuteJob& J, PartEmit* first_level, hipStream_t st);
hipError_t permute_finish(const PermuteJob& J, hipStream_t st);

// Phased backward, fused (Sec. 3 "Phased Laplace kernels"): the scan problem runs on the doubled batch
// [gy cos phi | gy sin phi] (2 * half columns) and its result rows are the inputs.  With this set, the streaming
// downsweep of the wide geometry forms, per input row j, both halves GX_c, GX_s of the plain result in registers and writes
//   gx[j]   = cos(psi_j) GX_c + sin(psi_j) GX_s,          gpsi[j] = sum_t x[j][t] (cos(psi_j) GX_s - sin(psi_j) GX_c)[t]
// and takes the weights of the row reduction (gb) from x itself, as x cos(psi_j) and x sin(psi_j); the doubled result
// matrix is only written (to out_p) for the few blocks the other downsweeps own, and a pass over those blocks merges them.
struct PhaseFuse {
    const float* psi;           // [result rows] phases of the result rows
    const float* x; int64_t ldx;    // [result rows][half] or null (no gb, no gpsi)
    float* gx; int64_t ldgx;        // [result rows][half] or null
    float* gpsi;                    // [result rows] or null
    int64_t half;                   // columns of one half; 0: off
};

// Phased kernel, input side: the injected matrix of the scan problem is [x cos psi | x sin psi] (2 * half columns) without
// being stored.  The reduce of the wide geometry reads x itself, one wavefront across both halves of a row, and forms the two
// products (rounded, as a split pass would store them) on the way in.  The downsweeps that read injected rows, or the weights
// of a row reduction, only do so in blocks that also hold rows of the other side; for those blocks the doubled rows are
// written to `x2` by a pass over the block flags after the spine:
//   split_blocks = 1: the rows of x in blocks that hold result rows (x is the injected matrix: forward, re-scan);
//   split_blocks = 2: the rows of x in blocks with more than a few injected rows (x holds the weights of the row
//                     reduction, the streaming downsweep of PhaseFuse takes them from x: backward).
struct PhaseIn {
    const float* psi;               // [rows of x] phases
    const float* x; int64_t ldx;    // [rows of x][half]
    float* x2;                      // [rows of x][2 * half] contiguous: written for the blocks named above
    uint32_t* whole;                // set to 0 by the block-wise split: x2 does not hold every row (see launch_phase_split)
    int64_t half;                   // columns of one half; 0: off
    int split_blocks;               // 0: none
    bool virtual_inj;               // the reduce reads x with the modulation instead of the injected matrix
};

struct ScanProblem {
    const uint32_t* ids; const float* dh; const float* pk; int64_t N;
    const float2* pk8 = nullptr;     // (pk[8m], pk[8m + 1]) per 8 rows, or null (batch 1 in sorted order only)
    const float* inj; int64_t ld_inj; uint32_t inj_lo, inj_hi;
    uint32_t res_lo, res_hi;
    float* out_p; int64_t ld_p;
    float* out_z;
    float* out_red; const float* w; int64_t ld_w; const float* zs;
    int64_t ld_z = 0, ld_red = 0;   // strides of out_z (0: batch) and out_red (0: 1): outputs that share rows with out_p
    int64_t batch;
    float* stage;          // narrow batches: the reduce writes the injected rows here in sorted order, the downsweep reads them back
    const float* wstage;   // narrow batches: the weights w in sorted order (an earlier problem's stage), or null
    const char* tag;   // names the timing families: scan_reduce.<tag>, scan_spine.<tag>, scan_down.<tag>
    // batch 1, routes without random accesses: `stage` already holds the injected rows in sorted order (zero elsewhere), and
    // the outputs of result row j of the sorted sequence go to out_p[j * ld_p], out_z[j * ld_z], out_red[j * ld_red]
    bool inj_sorted = false, out_sorted = false;
    // ... and with both set the results leave as records of a partition level (k_seq_down): `emit` says where they go,
    // emit_values how many outputs a record carries (2: F + R - v and the second output; 1: emit_first says which),
    // emit_strict that the second output is wanted (the strict scans Z, or w * Z when wstage is given)
    const PartEmit* emit = nullptr; int emit_values = 1; bool emit_first = true, emit_strict = false;
    const PhaseFuse* phase = nullptr;      // wide geometry, at most 256 columns per half (see PhaseFuse)
    const PhaseIn* phase_in = nullptr;     // the same geometry (see PhaseIn)
};
hipError_t launch_scan(const ScanProblem& p, const Layout& L, char* ws, hipStream_t st);

// Phase modulation of the phased kernel (phase_kernels.hip): split a (rows, batch) matrix into its
// cosine and sine halves, dst (rows, 2*batch) contiguous; merge two halves back and, if wanted, form
//   gphase[r] = sum_t other[r][t] (cos(phase_r) src2[r][batch+t] - sin(phase_r) src2[r][t]).
// `whole` (may be null): a word that says whether dst holds every row (1) or only those of some blocks (0, written by the
// block-wise split of PhaseIn); the pass sets it to 1, and with unless_whole it does nothing when the word is 1 already.
hipError_t launch_phase_split(const float* src, int64_t ld_src, const float* phase, int64_t rows, int64_t batch,
                              float* dst, hipStream_t st, uint32_t* whole = nullptr, bool unless_whole = false);
hipError_t launch_set_word(uint32_t* p, uint32_t v, hipStream_t st);      // *p = v
hipError_t launch_phase_merge(const float* src2, const float* phase, int64_t rows, int64_t batch,
                              float* dst, int64_t ld_dst, const float* other, int64_t ld_other, float* gphase,
                              hipStream_t st);

// Inverse temperature: gtau[0] = sum_i a_i ga_i + sum_j b_j gb_j (b, gb may be null with n = 0), in a fixed
// order; `partial` is scratch for kTauPartials floats.  launch_scale: p[i] *= f.
constexpr int kTauPartials = 1024;
hipError_t launch_tau_grad(const float* a, const float* ga, int64_t k, const float* b, const float* gb, int64_t n,
                           float* partial, float* gtau, hipStream_t st);
hipError_t launch_scale(float* p, int64_t count, float f, hipStream_t st);

// Small problems (small_kernels.hip): at most kSmallMax merged positions are sorted by one launch (ranks by counting)
// and scanned by one workgroup per (slab of `cols` batch columns, operator) in a second.  A SmallProblem is a ScanProblem restricted to
// out_p / out_z; pointers move by the op_* strides (in elements; op_ws in bytes) from one operator to the next.
struct SmallProblem {
    const float* inj; int64_t ld_inj; uint32_t inj_lo, inj_hi;
    uint32_t res_lo, res_hi;
    float* out_p; int64_t ld_p;     // F + R - v at the result rows, or null
    float* out_z;                   // (res rows, batch) contiguous: E_right - E_left, or null
    int64_t op_inj, op_p, op_z;
};
struct SmallArgs {
    const float* a; const float* b; int64_t k, n; float tau;
    uint32_t* ids; float* dh; float* pk;       // the plan in the workspace: written (slab 0), or read if reuse_plan
    int64_t op_a, op_b, op_ws;
    int reuse_plan;                            // the workspace holds the plan: no sort
    int write_dh;                              // set by the launcher: the decays are stored beside the plan
    int64_t batch; int cols;                   // cols: power of two <= 16
    int nprob; SmallProblem prob[2];
};
hipError_t launch_small(const SmallArgs& A, int64_t operators, hipStream_t st);
inline int small_cols(int64_t batch) { int c = 1; while (c < batch && c < 16) c <<= 1; return c; }

// LAPLEX^(r) helpers (phase_kernels.hip).  parts: r contiguous (rows, batch) matrices; w, scale: device memory.
//   combine: y = sum_q w[q] parts[q];  scale: dst (contiguous) = scale[0] * src;  accumulate: dst (+)= src (contiguous);
//   dot: out[0] = sum u .* v (v contiguous), fixed order, `partial` = kTauPartials floats of scratch.
hipError_t launch_mix_combine(const float* parts, const float* w, int64_t r, int64_t rows, int64_t batch,
                              float* y, int64_t ldy, hipStream_t st);
hipError_t launch_scale_by_device_scalar(const float* src, int64_t ld_src, const float* scale, int64_t rows, int64_t batch,
                                         float* dst, hipStream_t st);
hipError_t launch_accumulate(const float* src, int64_t rows, int64_t batch, float* dst, int64_t ld_dst, bool first,
                             hipStream_t st);
hipError_t launch_dot(const float* u, int64_t ldu, const float* v, int64_t rows, int64_t batch,
                      float* partial, float* out, hipStream_t st);
// for r operators at once: scale_ops: dst[q] (contiguous) = w[q] * src;  dot_ops: out[q] = sum u .* v[q] (v[q] contiguous,
// one after the other), partial = r * kDotGroups floats of scratch
constexpr int kDotGroups = 64;
hipError_t launch_scale_ops(const float* src, int64_t ld_src, const float* w, int64_t r, int64_t rows, int64_t batch,
                            float* dst, hipStream_t st);
hipError_t launch_dot_ops(const float* u, int64_t ldu, const float* v, int64_t r, int64_t rows, int64_t batch,
                          float* partial, float* out, hipStream_t st);

// Weighted Gram matrix (gram_kernels.hip): U, V, W (fp64, k each) by a scan of its own over the plan (ids, pk) of the
// doubled anchors, then the fill  M[i*ldm + j] = exp(-|a_i - a_j|) (U[lo] + (W[hi] - W[lo]) + V[hi]),  lo / hi the pair
// in sorted order.  summ: 6 * wgram_tiles(N) doubles of scratch; Pb: N - k doubles (the prefix sum of the weights at each
// middle anchor, in merged order).  _f32: fp32 weights and result, _f64: fp64.  status: the plan's status word (an invalid
// plan makes every entry a NaN), or null for a plan that cannot be invalid.
int64_t wgram_tiles(int64_t N);
hipError_t launch_wgram_f32(const uint32_t* ids, const float* pk, const float* a, const float* d, int64_t k, int64_t N,
                            double* summ, double* U, double* V, double* W, double* Pb, float* M, int64_t ldm,
                            const uint32_t* status, hipStream_t st);
hipError_t launch_wgram_f64(const uint32_t* ids, const float* pk, const float* a, const double* d, int64_t k, int64_t N,
                            double* summ, double* U, double* V, double* W, double* Pb, double* M, int64_t ldm,
                            const uint32_t* status, hipStream_t st);

// out[r] = sum_t u[r*ldu+t] * v[r*ldv+t]
// out[r] = sum_t (u1 v1 + u2 v2)[r, t]
// out[r] += sum_t u[r, t] * v[r, t]
hipError_t launch_add_rowdot(const float* u, int64_t ldu, const float* v, int64_t ldv, int64_t rows, int64_t batch, float* out,
                             hipStream_t st);
hipError_t launch_rowdot2(const float* u1, int64_t ldu1, const float* v1, int64_t ldv1,
                          const float* u2, int64_t ldu2, const float* v2, int64_t ldv2,
                          int64_t rows, int64_t batch, float* out, hipStream_t st);
// ... for `operators` problems at once, their matrices op_u / op_v / op_out elements apart
hipError_t launch_rowdot_ops(const float* u, int64_t ldu, int64_t op_u, const float* v, int64_t ldv, int64_t op_v,
                             int64_t rows, int64_t batch, float* out, int64_t op_out, int64_t operators, hipStream_t st);
hipError_t launch_rowdot(const float* u, int64_t ldu, const float* v, int64_t ldv,
                         int64_t rows, int64_t batch, float* out, hipStream_t st);

// Diagnostics: rows row_ids[r] of src are read (dst == nullptr) or copied to the same rows of dst.
hipError_t launch_diag_move_rows(const float* src, float* dst, const uint32_t* row_ids, int64_t rows, int64_t cols, hipStream_t st);

}  // namespace laplex
