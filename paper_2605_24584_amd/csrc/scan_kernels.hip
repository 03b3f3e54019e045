// The decayed scans over the merged, sorted anchor sequence (Sec. 3 "Symmetric
// case": y_{i+1} = x_{i+1} + exp(a_i - a_{i+1}) y_i, one prefix and one suffix
// scan; App. B.1: the associative pair operator that makes it parallel).
//
// One "scan problem" injects rows of a matrix at some positions of the merged
// sequence and reads results at others (apply forward: inject x at inputs, read
// at outputs; apply backward: inject gy at outputs, read at inputs; Gram form:
// both everywhere).  Per batch column two channels are carried:
//
//   F  inclusive decayed sum:  F_j = d_j F_{j-1} + v_j             (the paper's scan)
//   E  strict decayed sum: everything with a strictly smaller key, i.e. F at the
//      end of the previous run of equal keys, decayed once.  Needed only for
//      anchor gradients, where tied pairs must drop out (sgn(0) = 0).
//
// A run of rows is summarised by (D, S) with F_out = D F_in + S, plus, for the
// strict channel, (H, Q) with E_out = H ? D F_in + Q : E_in (the decay up to the
// last run head is D itself, since the rows after it have decay 1).  Summaries
// compose associatively, so the work splits into launches, with both directions
// done together so that the injected matrix is read once per launch:
//
//   reduce        per tile: forward and backward summary, and whether the tile
//                 holds injected rows / result rows
//   spine         exclusive scan over the tile summaries, two levels: chunks of
//                 tiles are summarised (coalesced over the batch), the chunk
//                 summaries are scanned, and the carries are pushed back down
//   downsweep     tiles with injected AND result rows: re-read the tile, seed
//                 both walks with the carries, walk forward, then backward, emit
//   downsweep_sparse  tiles with result rows but nothing injected: every row is
//                 a closed form of the two carries (the two-term evaluation of
//                 Thm "Dual reduction" inside a tile), streamed with no row state
//
// Lanes: bv lanes across the batch (vec columns each) x rv row-lanes per
// wavefront; each row-lane walks `items` consecutive rows sequentially.
#include "laplex_internal.h"
#include "permute_tile.h"

#include <string>


namespace laplex {

namespace {

struct Level {            // summaries of one level (tiles, or chunks of tiles) and the carries into them
    float4* scalar;       // [2][count]        (D, C, H, flags)
    float* s;             // [2][count][bpad]
    float* q;             // [2][count][bpad]
    float* car_f;         // [2][count][bpad]
    float* car_e;         // [2][count][bpad]
    int64_t count;
};

struct ScanArgs {
    const uint32_t* ids; const float* dh; const float* pk; int64_t N;
    const float2* pk8;                   // (pk[8m], pk[8m + 1]), or null
    const float* inj; int64_t ld_inj; uint32_t inj_lo, inj_hi;
    uint32_t res_lo, res_hi;
    float* out_p; int64_t ld_p;
    float* out_z; int64_t ld_z;          // rows of out_z are ld_z floats apart (batch, unless it shares rows with out_p)
    float* out_red; int64_t ld_red; const float* w; int64_t ld_w; const float* zs;
    float* stage; const float* wstage;   // sorted-order copies of the injected rows / of the weights (narrow batches)
    int64_t batch, bpad;
    int bv, bv_log2, rv, tile_rows, slabs, chunk_tiles, spine_items;
    // A downsweep workgroup owns a block of tile_rows rows; the spine's tiles (level 1) are
    // 2^sub_shift consecutive blocks, spine_rows rows (sub_shift > 0 in the wide geometry only).
    int sub_shift; int64_t spine_rows, blocks;
    int waves;            // wavefronts per workgroup of the block kernels (reduce, downsweeps)
    uint32_t* blk_flags;  // [blocks] kFlagInj | kFlagRes
    float* blk_f;         // [2][blocks][bpad] state entering a block when its tile starts from zero (sub_shift > 0)
    float* blk_e;         // [2][blocks][bpad] the same, strict channel
    Level l1, l2;
    float* red_partial;   // [slabs][res rows] when slabs > 1
    // sparse problems (few injected or few result rows): the metadata kernel lists the tiles that need
    // the heavy kernels, which then launch one workgroup per list entry instead of one per tile
    uint32_t* list_inj;   // tiles that hold injected rows
    uint32_t* list_both;  // blocks that hold injected and result rows
    uint32_t* counters;   // [0] = entries of list_inj, [1] = entries of list_both
    // list_inj is written by the metadata pass; list_both by the metadata pass if it runs, else by the reduce
    int reduce_from_list, down_from_list;
    int few_inj_ok, few_res_ok;   // the block flags kFlagFewInj / kFlagFewRes may be set
    int pair_out;                 // batch 1: out_p and the row's second output (out_z, else out_red) are the halves of an 8-byte slot
    int inj_sorted;               // batch 1: `stage` already holds the injected rows in sorted order: nothing is gathered
    int out_sorted;               // batch 1: outputs are indexed by the sorted row, not by the id (a later pass takes them home)
    PartEmit emit;                // batch 1, sorted order: the results leave as records of a partition level (k_seq_down)
    int emit_first;               // one value per record: the first output of a row (F + R - v), else its second
    PhaseFuse ph;                 // ph.half != 0: the phased backward's streaming downsweep merges the two halves itself
    PhaseIn pin;                  // pin.half != 0: the injected matrix (or the weights) is x modulated by its rows' phases
};

constexpr int kFlagInj = 1, kFlagRes = 2;

// An invalid plan (a tile of the radix sort gave up its bounded wait) must never pass for a result: the
// kernels that store results OR this word into every value they store.  It is 0 for a valid plan and
// turns any float into a NaN (all exponent bits and a mantissa bit) for an invalid one.
__device__ __forceinline__ uint32_t plan_poison(const uint32_t* counters) { return counters[kPlanStatusWord] ? 0x7FC00000u : 0u; }
__device__ __forceinline__ float taint(float v, uint32_t poison) { return __uint_as_float(__float_as_uint(v) | poison); }
// Block flags only (wide geometry, injected and result rows from different matrices): the block holds
// injected (result) rows, but at most kFewRows of them.  Such a block does not need the scan inside
// it: each result row is the carries' closed form plus a handful of direct terms exp(-|p_i - p_s|) v_s.
constexpr int kFlagFewInj = 4, kFlagFewRes = 8;
constexpr int kFewRows = 4;

template <int VEC, bool STRICT>
struct Seg {
    float D;        // product of the decays
    float C;        // strict channel: E_out = C * F_in + Q  (if H)
    int H;          // the rows contain the start of a run of equal keys
    float S[VEC];   // F_out = D * F_in + S
    float Q[VEC];
};

template <int VEC, bool STRICT>
__device__ __forceinline__ Seg<VEC, STRICT> seg_identity()
{
    Seg<VEC, STRICT> s;
    s.D = 1.0f; s.C = 0.0f; s.H = 0;
#pragma unroll
    for (int e = 0; e < VEC; ++e) { s.S[e] = 0.0f; s.Q[e] = 0.0f; }
    return s;
}

// s <- s followed by one row (head flag h, decay d, values v)
template <int VEC, bool STRICT>
__device__ __forceinline__ void seg_push(Seg<VEC, STRICT>& s, bool h, float d, const float* v)
{
    const float dd = h ? d : 1.0f;
    if (STRICT) {               // selects, not branches: h differs between row-lanes
        s.C = h ? dd * s.D : s.C;
        s.H |= h ? 1 : 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) s.Q[e] = h ? dd * s.S[e] : s.Q[e];
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) s.S[e] = dd * s.S[e] + v[e];
    s.D *= dd;
}

// rows of x, then rows of y
template <int VEC, bool STRICT>
__device__ __forceinline__ Seg<VEC, STRICT> seg_compose(const Seg<VEC, STRICT>& x, const Seg<VEC, STRICT>& y)
{
    Seg<VEC, STRICT> r;
    r.D = x.D * y.D;
    if (STRICT) {
        r.H = x.H | y.H;
        r.C = r.D;       // the decay up to the last run head equals the whole decay: rows after it have decay 1
#pragma unroll
        for (int e = 0; e < VEC; ++e) r.Q[e] = y.H ? y.D * x.S[e] + y.Q[e] : x.Q[e];
    } else {
        r.H = 0; r.C = 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) r.Q[e] = 0.0f;
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) r.S[e] = y.D * x.S[e] + y.S[e];
    return r;
}

template <int VEC, bool STRICT>
__device__ __forceinline__ Seg<VEC, STRICT> seg_shfl(const Seg<VEC, STRICT>& s, int src)
{
    Seg<VEC, STRICT> r;
    r.D = __shfl(s.D, src);
    if (STRICT) { r.C = __shfl(s.C, src); r.H = __shfl(s.H, src); } else { r.C = 0.0f; r.H = 0; }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        r.S[e] = __shfl(s.S[e], src);
        r.Q[e] = STRICT ? __shfl(s.Q[e], src) : 0.0f;
    }
    return r;
}

// state (F, E) after the rows summarised by s
template <int VEC, bool STRICT>
__device__ __forceinline__ void seg_apply(const Seg<VEC, STRICT>& s, float* F, float* E)
{
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        if (STRICT) E[e] = s.H ? s.D * F[e] + s.Q[e] : E[e];
        F[e] = s.D * F[e] + s.S[e];
    }
}

// Inclusive scan over the row-lanes of one wavefront, in forward (row-lane 0
// first) or backward (last row-lane first) order.  Lanes with equal (lane & (bv-1))
// hold the same batch columns.
template <bool FWD, int VEC, bool STRICT>
__device__ __forceinline__ Seg<VEC, STRICT> wave_scan(Seg<VEC, STRICT> s, int lane, int bv, int rv)
{
    const int r = lane / bv;
    for (int step = 1; step < rv; step <<= 1) {
        const int src = FWD ? lane - step * bv : lane + step * bv;
        const Seg<VEC, STRICT> o = seg_shfl<VEC, STRICT>(s, src & 63);
        const bool has = FWD ? (r >= step) : (r + step < rv);
        if (has) s = seg_compose<VEC, STRICT>(o, s);
    }
    return s;
}

typedef float v4f __attribute__((ext_vector_type(4)));

template <int VEC>
__device__ __forceinline__ void load_vec(float* dst, const float* src)
{
    if (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4*>(src);
        dst[0] = t.x; dst[1] = t.y; dst[2] = t.z; dst[3] = t.w;
    } else {
        dst[0] = src[0];
    }
}

template <int VEC>
__device__ __forceinline__ void store_vec(float* dst, const float* src)
{
    if (VEC == 4) *reinterpret_cast<float4*>(dst) = make_float4(src[0], src[1], src[2], src[3]);
    else dst[0] = src[0];
}

// The same for data that is read (written) once and not again soon: streaming accesses, which do not
// displace what the caches hold.  Used where a lane moves 16 bytes of a row; with one column per lane
// (batches of one to three columns, random 4-byte accesses) the caches are what makes the gathers
// affordable, and streaming them cost 60 % on the tie-heavy workload.
template <int VEC> constexpr bool kStreamRows = VEC == 4;
template <int VEC>
__device__ __forceinline__ void load_vec_stream(float* dst, const float* src)
{
    if (VEC == 4) {
        const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(src));
        dst[0] = t.x; dst[1] = t.y; dst[2] = t.z; dst[3] = t.w;
    } else {
        dst[0] = __builtin_nontemporal_load(src);
    }
}

template <int VEC>
__device__ __forceinline__ void store_vec_stream(float* dst, const float* src)
{
    if (VEC == 4) __builtin_nontemporal_store((v4f){src[0], src[1], src[2], src[3]}, reinterpret_cast<v4f*>(dst));
    else __builtin_nontemporal_store(src[0], dst);
}

// dst <- ok ? base[off .. off+VEC) : 0, without a branch: a row that is not wanted
// reads the first columns of row 0 (always valid, always cached) and is discarded.
template <int VEC, bool STREAM = false>
__device__ __forceinline__ void load_vec_or_zero(float* dst, const float* base, int64_t off, bool ok)
{
    float t[VEC];
    if (STREAM) load_vec_stream<VEC>(t, base + (ok ? off : 0));
    else load_vec<VEC>(t, base + (ok ? off : 0));
#pragma unroll
    for (int e = 0; e < VEC; ++e) dst[e] = ok ? t[e] : 0.0f;
}

template <int VEC>
struct TileRows {
    static constexpr int ITEMS = VEC == 4 ? kItemsVec4 : kItemsVec1;
    float dh[ITEMS + 1];      // dh[i]: decay into row i from the left; dh[i+1]: from the right
    uint32_t id[ITEMS];       // 0xFFFFFFFF past the end of the sequence
};

template <int VEC>
__device__ __forceinline__ void load_meta(const ScanArgs& A, int64_t row0, TileRows<VEC>& T)
{
    constexpr int ITEMS = TileRows<VEC>::ITEMS;
    // clamped indices and selects: no branch around any load
#pragma unroll
    for (int i = 0; i <= ITEMS; ++i) {
        const int64_t j = row0 + i;
        const float d = A.dh[j <= A.N ? j : A.N];
        T.dh[i] = j <= A.N ? d : -1.0f;
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int64_t j = row0 + i;
        const uint32_t id = A.ids[j < A.N ? j : A.N - 1];
        T.id[i] = j < A.N ? id : 0xFFFFFFFFu;
    }
}

// Row i starts a run of equal keys seen from the left / from the right.  Rows past
// the end (id 0xFFFFFFFF) are neutral: no head, decay 1, nothing injected.
template <int VEC>
__device__ __forceinline__ bool head_f(const TileRows<VEC>& T, int i) { return T.id[i] != 0xFFFFFFFFu && T.dh[i] >= 0.0f; }
template <int VEC>
__device__ __forceinline__ bool head_b(const TileRows<VEC>& T, int i) { return T.id[i] != 0xFFFFFFFFu && T.dh[i + 1] >= 0.0f; }

// Total decay over the rows [row0, row0 + count) in the forward sense (from the anchor before
// row0 to the last of the rows) and in the backward sense (from the anchor after the rows to row0),
// taken from the anchors themselves: exp(-(p_end - p_start)), one rounding whatever the count.
// pk is shifted by one between -inf / +inf sentinels, so the ends of the sequence give exactly 0;
// rows past the end do not count.
// (Branch-free: indices are clamped and an empty span is selected away afterwards, so the loads
//  are issued unconditionally next to the kernel's other loads.)
__device__ __forceinline__ float span_decay_f(const ScanArgs& A, int64_t row0, int64_t count)
{
    const int64_t lo = row0 < A.N ? row0 : A.N;
    int64_t hi = row0 + (count > 0 ? count : 0);
    hi = hi < A.N ? hi : A.N;                                        // one past the last live row
    const float d = expf(-(A.pk[hi] - A.pk[lo]));
    return hi > lo ? d : 1.0f;
}
__device__ __forceinline__ float span_decay_b(const ScanArgs& A, int64_t row0, int64_t count)
{
    const int64_t lo = row0 < A.N ? row0 : A.N;
    int64_t hi = row0 + (count > 0 ? count : 0);
    hi = hi < A.N ? hi : A.N;
    const float d = expf(-(A.pk[hi + 1] - A.pk[lo + 1]));
    return hi > lo ? d : 1.0f;
}

// Is there a run head among the rows [row0, row0 + count), seen from the left / from the right?
// Sorted anchors change somewhere in the span iff its two ends differ.
__device__ __forceinline__ bool span_head_f(const ScanArgs& A, int64_t row0, int64_t count)
{
    const int64_t lo = row0 < A.N ? row0 : A.N;
    int64_t hi = row0 + (count > 0 ? count : 0);
    hi = hi < A.N ? hi : A.N;
    return hi > lo && A.pk[hi] != A.pk[lo];
}
__device__ __forceinline__ bool span_head_b(const ScanArgs& A, int64_t row0, int64_t count)
{
    const int64_t lo = row0 < A.N ? row0 : A.N;
    int64_t hi = row0 + (count > 0 ? count : 0);
    hi = hi < A.N ? hi : A.N;
    return hi > lo && A.pk[hi + 1] != A.pk[lo + 1];
}

// State a row-lane starts from, given the carry into its tile (Fc, Ec), the summary of the rows of the
// tile that precede it applied to a ZERO state (F0 = their S, E0 = their Q), and the direct decay D /
// head flag H over those preceding rows: the carry is decayed by ONE exponential of an anchor
// difference instead of by the product of all the summaries' decays.
template <int VEC, bool STRICT>
__device__ __forceinline__ void enter_state(float* F, float* E, const float* Fc, const float* Ec, float D, bool H)
{
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const float carried = D * Fc[e];
        if (STRICT) E[e] = H ? E[e] + carried : Ec[e];
        F[e] = F[e] + carried;
    }
}

template <int VEC, bool STREAM = false>
__device__ __forceinline__ void load_injected(const ScanArgs& A, const TileRows<VEC>& T, int64_t col0, bool col_ok,
                                              float (*v)[VEC])
{
    constexpr int ITEMS = TileRows<VEC>::ITEMS;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool ok = col_ok && T.id[i] >= A.inj_lo && T.id[i] < A.inj_hi;
        load_vec_or_zero<VEC, STREAM>(v[i], A.inj, (int64_t)(T.id[i] - A.inj_lo) * A.ld_inj + col0, ok);
    }
}

// weights of the row reduction at the result rows (zero elsewhere, or when no reduction is wanted)
template <int VEC>
__device__ __forceinline__ void load_weights(const ScanArgs& A, const TileRows<VEC>& T, int64_t row0, int64_t col0,
                                             bool col_ok, bool want, float (*wv)[VEC])
{
    constexpr int ITEMS = TileRows<VEC>::ITEMS;
    if (want && A.wstage) {     // uniform: sorted-order copy, read in place of a random gather
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const bool ok = col_ok && T.id[i] >= A.res_lo && T.id[i] < A.res_hi;
            load_vec_or_zero<VEC>(wv[i], A.wstage, (row0 + i) * A.batch + col0, ok);
        }
    } else if (want) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const bool ok = col_ok && T.id[i] >= A.res_lo && T.id[i] < A.res_hi;
            load_vec_or_zero<VEC>(wv[i], A.w, (int64_t)(T.id[i] - A.res_lo) * A.ld_w + col0, ok);
        }
    } else {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
#pragma unroll
            for (int e = 0; e < VEC; ++e) wv[i][e] = 0.0f;
    }
}

// LDS exchange of per-wavefront summaries: [dir][wave] scalars and [dir][wave][column] vectors.
template <int VEC>
struct WaveSegs {
    float D[2][kScanWaves], C[2][kScanWaves];
    int H[2][kScanWaves];
    float S[2][kScanWaves][64 * VEC];
    float Q[2][kScanWaves][64 * VEC];
};

template <int VEC, bool STRICT>
__device__ __forceinline__ void put_wave_seg(WaveSegs<VEC>& W, int dir, int wave, int c, const Seg<VEC, STRICT>& s)
{
    if (c == 0) { W.D[dir][wave] = s.D; if (STRICT) { W.C[dir][wave] = s.C; W.H[dir][wave] = s.H; } }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        W.S[dir][wave][c * VEC + e] = s.S[e];
        if (STRICT) W.Q[dir][wave][c * VEC + e] = s.Q[e];
    }
}

template <int VEC, bool STRICT>
__device__ __forceinline__ Seg<VEC, STRICT> get_wave_seg(const WaveSegs<VEC>& W, int dir, int wave, int c)
{
    Seg<VEC, STRICT> s;
    s.D = W.D[dir][wave];
    s.C = STRICT ? W.C[dir][wave] : 0.0f;
    s.H = STRICT ? W.H[dir][wave] : 0;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        s.S[e] = W.S[dir][wave][c * VEC + e];
        s.Q[e] = STRICT ? W.Q[dir][wave][c * VEC + e] : 0.0f;
    }
    return s;
}

// summary `idx` of direction `dir` at one level, for the VEC columns starting at col0
template <int VEC, bool STRICT, bool FLAGGED>
__device__ __forceinline__ Seg<VEC, STRICT> load_level_seg(const Level& L, int dir, int64_t idx, int64_t bpad,
                                                           int64_t col0, bool col_ok)
{
    Seg<VEC, STRICT> s = seg_identity<VEC, STRICT>();
    const float4 sc = L.scalar[(int64_t)dir * L.count + idx];
    s.D = sc.x;
    if (STRICT) { s.C = sc.y; s.H = (int)sc.z; }
    // level 1: a tile with nothing injected has S = Q = 0 and its rows may never have been written; its
    // loads are pointed at entry 0 instead (branch-free, always cached) and the values discarded
    const bool inj = !FLAGGED || ((int)sc.w & kFlagInj) != 0;
    if (col_ok) {
        const int64_t o = inj ? ((int64_t)dir * L.count + idx) * bpad + col0 : col0;
        load_vec<VEC>(s.S, L.s + o);
        if (STRICT) load_vec<VEC>(s.Q, L.q + o);
    }
    if (FLAGGED) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { s.S[e] = inj ? s.S[e] : 0.0f; s.Q[e] = inj ? s.Q[e] : 0.0f; }
    }
    return s;
}

template <int VEC, bool STRICT>
__device__ __forceinline__ void store_level_seg(const Level& L, int dir, int64_t idx, int64_t bpad, int64_t col0,
                                                bool col_ok, bool scalar_writer, const Seg<VEC, STRICT>& s, float flags)
{
    if (scalar_writer) L.scalar[(int64_t)dir * L.count + idx] = make_float4(s.D, s.C, (float)s.H, flags);
    if (col_ok) {
        const int64_t o = ((int64_t)dir * L.count + idx) * bpad + col0;
        store_vec<VEC>(L.s + o, s.S);
        if (STRICT) store_vec<VEC>(L.q + o, s.Q);
    }
}

// Flags of a 64-row block of the wide geometry, from the masks of its injected and result rows.
__device__ __forceinline__ int block_flags(const ScanArgs& A, uint64_t inj_mask, uint64_t res_mask)
{
    int f = (inj_mask ? kFlagInj : 0) | (res_mask ? kFlagRes : 0);
    if (A.few_inj_ok && inj_mask && __popcll(inj_mask) <= kFewRows) f |= kFlagFewInj;
    if (A.few_res_ok && res_mask && __popcll(res_mask) <= kFewRows) f |= kFlagFewRes;
    return f;
}
// Does the block go on the list of the downsweeps that read the injected rows again?  (A block with
// few injected rows is handled by the streaming downsweep.)
__device__ __forceinline__ bool listed_block(int f)
{
    return (f & (kFlagInj | kFlagRes | kFlagFewInj)) == (kFlagInj | kFlagRes);
}

// ---------------------------------------------------------------------------
// metadata pass for sparse problems: one wavefront per tile, one lane per row
// (coalesced).  Writes, for every tile, its flags and the summary it has if
// nothing is injected in it (S = Q = 0, C = D: only the decays and the run heads
// matter), and lists the tiles the heavy kernels must visit.  Tiles that do hold
// injected rows get their summary overwritten by k_scan_reduce.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_scan_meta(const ScanArgs A)
{
    const int lane = threadIdx.x & 63;
    const int64_t tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= A.l1.count) return;
    int Hf = 0, Hb = 0, fl = 0;
    const int64_t base = tile * A.spine_rows;
    const float Df = span_decay_f(A, base, A.spine_rows), Db = span_decay_b(A, base, A.spine_rows);
    for (int64_t o = 0; o < A.spine_rows && base + o < A.N; o += 64) {
        const int64_t j = base + o + lane;
        const bool live = j < A.N;
        const int64_t jc = live ? j : A.N - 1;
        const uint32_t id = A.ids[jc];
        const float df = A.dh[jc], db = A.dh[jc + 1];
        Hf |= __ballot(live && df >= 0.0f) ? 1 : 0;
        Hb |= __ballot(live && db >= 0.0f) ? 1 : 0;
        const uint64_t inj_mask = __ballot(live && id >= A.inj_lo && id < A.inj_hi);
        const uint64_t res_mask = __ballot(live && id >= A.res_lo && id < A.res_hi);
        const int here = (inj_mask ? kFlagInj : 0) | (res_mask ? kFlagRes : 0);
        fl |= here;
        if (A.sub_shift && lane == 0) {     // wide geometry: these 64 rows are one block
            const int64_t blk = (base + o) >> 6;
            const int bf = block_flags(A, inj_mask, res_mask);
            A.blk_flags[blk] = (uint32_t)bf;
            if (A.down_from_list && listed_block(bf)) A.list_both[atomicAdd(&A.counters[1], 1u)] = (uint32_t)blk;
        }
    }
    if (lane == 0) {
        A.l1.scalar[tile] = make_float4(Df, Df, (float)Hf, (float)fl);
        A.l1.scalar[A.l1.count + tile] = make_float4(Db, Db, (float)Hb, (float)fl);
        // a list is built only when its kernel will be driven by it (then it is short by construction)
        if (A.reduce_from_list && (fl & kFlagInj)) A.list_inj[atomicAdd(&A.counters[0], 1u)] = (uint32_t)tile;
        if (!A.sub_shift) {                 // block = tile
            A.blk_flags[tile] = (uint32_t)fl;
            if (A.down_from_list && fl == (kFlagInj | kFlagRes)) A.list_both[atomicAdd(&A.counters[1], 1u)] = (uint32_t)tile;
        }
    }
}

// ---------------------------------------------------------------------------
// reduce: forward and backward summary of every tile, and the tile's flags
// ---------------------------------------------------------------------------
template <int VEC, bool STRICT>
__global__ void __launch_bounds__(kScanThreads)
k_scan_reduce(const ScanArgs A)
{
    constexpr int ITEMS = TileRows<VEC>::ITEMS;
    __shared__ WaveSegs<VEC> W;
    __shared__ int tile_flags;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bv = A.bv, rv = A.rv;
    const int c = lane & (bv - 1), r = lane >> A.bv_log2;
    if (A.reduce_from_list && blockIdx.x >= A.counters[0]) return;
    const int64_t tile = A.reduce_from_list ? A.list_inj[blockIdx.x] : blockIdx.x;
    const int64_t wave_row0 = tile * A.tile_rows + (int64_t)(wave * rv) * ITEMS;
    const int64_t row0 = wave_row0 + (int64_t)r * ITEMS;
    const int64_t col0 = ((int64_t)blockIdx.y * bv + c) * VEC;
    const bool col_ok = col0 < A.batch;
    if (tid == 0) tile_flags = 0;

    // decays over this row-lane's rows, this wavefront's rows and the whole tile, from the anchors
    // (not products of the rows' decays: see k_decay); asked for first so the loads go out early
    const float tile_df = span_decay_f(A, tile * A.tile_rows, A.tile_rows);
    const float tile_db = span_decay_b(A, tile * A.tile_rows, A.tile_rows);

    TileRows<VEC> T;
    load_meta<VEC>(A, row0, T);
    int mine = 0;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        mine |= (T.id[i] >= A.inj_lo && T.id[i] < A.inj_hi) ? kFlagInj : 0;
        mine |= (T.id[i] >= A.res_lo && T.id[i] < A.res_hi) ? kFlagRes : 0;
    }
    // the injected rows are asked for before the flags meet: the gathers travel while the workgroup waits at the
    // barriers (a row that is not injected is not loaded, it reads as zero)
    float v[ITEMS][VEC];
    if (A.inj_sorted) {     // uniform: the rows arrive in sorted order (zero where nothing is injected)
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
            load_vec_or_zero<VEC>(v[i], A.stage, (row0 + i) * A.batch + col0, col_ok && T.id[i] != 0xFFFFFFFFu);
    } else {
        load_injected<VEC, kStreamRows<VEC>>(A, T, col0, col_ok, v);
    }
    __syncthreads();
    if (c == 0 && mine) atomicOr(&tile_flags, mine);
    __syncthreads();
    if (tid == 0 && blockIdx.y == 0) A.blk_flags[tile] = (uint32_t)tile_flags;      // in this geometry a tile is one block
    if (!A.inj_sorted && (tile_flags & kFlagInj) && A.stage && col_ok) {     // uniform: the downsweep finds the tile's rows in sorted order
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
            if (T.id[i] != 0xFFFFFFFFu) store_vec<VEC>(A.stage + (row0 + i) * A.batch + col0, v[i]);
    }

    // The tile's summary as a weighted sum of the row-lanes' own (each from zero over its ITEMS rows): a row-lane's forward
    // state reaches the tile's last row through ONE exponential of an anchor difference, its backward state the tile's first
    // row likewise.  (Composing the row-lanes' summaries pairwise would multiply up to rv * waves decays of equal spans; on a
    // regular grid those carry equal rounding errors, and every far term of every output passes through a tile summary.)
    // Strict channel: the rows before the tile's last run head, seen from the left, are the row-lanes before the last one
    // that holds a head, whole, plus that row-lane's own strict sum (rows after the last head have decay 1).
    const int64_t tile_row0 = tile * A.tile_rows;
    const float wf = span_decay_f(A, row0 + ITEMS, tile_row0 + A.tile_rows - (row0 + ITEMS));
    const float wb = span_decay_b(A, tile_row0, row0 - tile_row0);
    Seg<VEC, STRICT> f = seg_identity<VEC, STRICT>(), b = seg_identity<VEC, STRICT>();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) seg_push<VEC, STRICT>(f, head_f<VEC>(T, i), T.dh[i], v[i]);
#pragma unroll
    for (int i = ITEMS - 1; i >= 0; --i) seg_push<VEC, STRICT>(b, head_b<VEC>(T, i), T.dh[i + 1], v[i]);
    {
        const uint64_t hf = STRICT ? __ballot(f.H != 0) : 0ull, hb = STRICT ? __ballot(b.H != 0) : 0ull;
        const int last_f = hf ? (63 - __clzll((long long)hf)) >> A.bv_log2 : -1;        // last row-lane with a head, from the left
        const int first_b = hb ? (__ffsll((long long)hb) - 1) >> A.bv_log2 : rv;        // first one, i.e. the last seen from the right
        float sf[VEC], qf[VEC], sb[VEC], qb[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            sf[e] = wf * f.S[e]; sb[e] = wb * b.S[e];
            qf[e] = r < last_f ? sf[e] : (r == last_f ? f.Q[e] : 0.0f);
            qb[e] = r > first_b ? sb[e] : (r == first_b ? b.Q[e] : 0.0f);
        }
        for (int m = bv; m < 64; m <<= 1) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                sf[e] += __shfl_xor(sf[e], m); sb[e] += __shfl_xor(sb[e], m);
                if (STRICT) { qf[e] += __shfl_xor(qf[e], m); qb[e] += __shfl_xor(qb[e], m); }
            }
        }
        if (r == 0) {
            if (c == 0 && STRICT) { W.H[0][wave] = hf != 0; W.H[1][wave] = hb != 0; }
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                W.S[0][wave][c * VEC + e] = sf[e]; W.S[1][wave][c * VEC + e] = sb[e];
                if (STRICT) { W.Q[0][wave][c * VEC + e] = qf[e]; W.Q[1][wave][c * VEC + e] = qb[e]; }
            }
        }
    }
    __syncthreads();

    if (tid < bv) {   // wavefront 0, row-lane 0: one lane per column group
        Seg<VEC, STRICT> tf = seg_identity<VEC, STRICT>(), tb = seg_identity<VEC, STRICT>();
#pragma unroll 1
        for (int w = 0; w < A.waves; ++w) {
            const bool h = STRICT && W.H[0][w] != 0;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                if (h) tf.Q[e] = tf.S[e] + W.Q[0][w][c * VEC + e];      // everything before this wavefront, and its own share
                tf.S[e] += W.S[0][w][c * VEC + e];
            }
            tf.H |= h ? 1 : 0;
        }
#pragma unroll 1
        for (int w = A.waves - 1; w >= 0; --w) {
            const bool h = STRICT && W.H[1][w] != 0;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                if (h) tb.Q[e] = tb.S[e] + W.Q[1][w][c * VEC + e];
                tb.S[e] += W.S[1][w][c * VEC + e];
            }
            tb.H |= h ? 1 : 0;
        }
        tf.D = tf.C = tile_df;
        tb.D = tb.C = tile_db;
        const bool sw = c == 0 && blockIdx.y == 0;
        // (the vectors of a tile with nothing injected are zero and never fetched: not written either)
        const bool vec_ok = col_ok && (tile_flags & kFlagInj);
        store_level_seg<VEC, STRICT>(A.l1, 0, tile, A.bpad, col0, vec_ok, sw, tf, (float)tile_flags);
        store_level_seg<VEC, STRICT>(A.l1, 1, tile, A.bpad, col0, vec_ok, sw, tb, (float)tile_flags);
    }
}

// ---------------------------------------------------------------------------
// reduce, wide batches (64 lanes across the batch, 4 columns each): a workgroup per tile of
// eight 64-row blocks, one WAVEFRONT per block.  Same outputs as k_scan_reduce, plus, for the blocks
// that hold result rows, the state the block starts from when its tile starts from zero (the
// downsweeps add the tile's carry, decayed to the block by one exponential).
//
// Lane l first looks at row l of the block: its id, its decays, and the two weights
//   wf_l = exp(-(p_last - p_l))    (row l's share in the forward summary, decayed to the block's last row)
//   wb_l = exp(-(p_l - p_first))   (its share in the backward summary, decayed to the block's first row)
// taken from the anchors with one exponential each, so the summaries are plain weighted sums
//   S_f = sum_l wf_l v_l,   S_b = sum_l wb_l v_l
// with no dependence from row to row (the recurrence of Sec. 3 unrolled; App. B.1's pair operator
// summed in closed form), and the strict sums are the part of them before the block's last run head
// (after its first one, seen from the right).  Ballots turn the per-row flags into wavefront-uniform
// masks; ids and weights reach the scalar unit with readlane.  The data rows are then streamed with
// every lane on its own 4 columns.  A summary written to memory costs far more than its share of the
// bytes (writes interleaved with a read stream), hence one per eight blocks and not one per block.
// ---------------------------------------------------------------------------

__device__ __forceinline__ float lane_f(float v, int l) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l)); }
__device__ __forceinline__ uint32_t lane_u(uint32_t v, int l) { return (uint32_t)__builtin_amdgcn_readlane((int)v, l); }

// What lane l knows about row l of a 64-row block (loads only, no arithmetic yet).
struct WideMeta {
    uint32_t id;
    float dl, dr;                                 // decay into the row from the left / from the right
    float p, p_first, p_last, p_before, p_after;  // anchors: own, the block's first and last, the neighbours outside
    bool live;                                    // false past the end of the sequence
    __device__ __forceinline__ void fetch(const ScanArgs& A, int64_t blk, int lane)
    {
        const int64_t blk_base = blk * 64, j = blk_base + lane;
        live = j < A.N;
        const int64_t jc = live ? j : A.N - 1;
        const int64_t last = blk_base + 64 <= A.N ? blk_base + 63 : A.N - 1;     // the block's last live row
        id = A.ids[jc];
        dl = A.dh[jc]; dr = A.dh[jc + 1];
        p = A.pk[jc + 1]; p_first = A.pk[blk_base + 1]; p_last = A.pk[last + 1];   // pk is shifted by one
        p_before = A.pk[blk_base]; p_after = A.pk[last + 2];
    }
};

constexpr int kWideWaves = 1 << kWideSubShift;     // one wavefront per block of the tile
constexpr int kStreamWaves = 4;                    // wavefronts (blocks) per workgroup of the kernels with one wavefront per block
static_assert(kWideWaves <= kScanWaves, "the LDS exchange has room for kScanWaves summaries");

// HALVES = 2 (phased kernel, PhaseIn): the injected matrix is [x cos psi | x sin psi]; a lane owns four columns of both
// halves, x is read once, and the two products are formed (and rounded) on the way in.  One slab then: blockIdx.y = 0.
template <bool STRICT, int HALVES>
__global__ void __launch_bounds__(kWideWaves * 64)
k_scan_reduce_wide(const ScanArgs A)
{
    constexpr int VEC = 4, ROWS = 64, CH = 8;
    static_assert(kScanWaves * kItemsVec4 == ROWS, "the wide geometry (one row-lane per wavefront) has 64 rows per block");
    __shared__ WaveSegs<VEC> W[HALVES];
    __shared__ int tile_flags, blk_flag[kWideWaves];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t half = HALVES == 2 ? A.pin.half : 0;
    const int64_t col0 = ((int64_t)(HALVES == 2 ? 0 : blockIdx.y) * 64 + lane) * VEC;
    const bool col_ok = col0 < (HALVES == 2 ? half : A.batch);
    const int64_t ld_in = HALVES == 2 ? A.pin.ldx : A.ld_inj;
    const float* const base = (HALVES == 2 ? A.pin.x : A.inj) + (col_ok ? col0 : 0);     // lanes past the last column read (and drop) columns 0..3

    if (A.reduce_from_list && blockIdx.x >= A.counters[0]) return;
    const int64_t tile = A.reduce_from_list ? (int64_t)A.list_inj[blockIdx.x] : (int64_t)blockIdx.x;
    const int64_t blk = (tile << kWideSubShift) + wave;         // this wavefront's block
    const bool blk_live = blk < A.blocks;
    if (threadIdx.x == 0) tile_flags = 0;
    __syncthreads();

    float Sf[HALVES][VEC], Qf[HALVES][VEC], Sb[HALVES][VEC], Qb[HALVES][VEC];
#pragma unroll
    for (int h = 0; h < HALVES; ++h) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { Sf[h][e] = Qf[h][e] = Sb[h][e] = Qb[h][e] = 0.0f; }
    }
    float blk_df = 1.0f, blk_db = 1.0f;
    int Hf = 0, Hb = 0, flags = 0;
    if (blk_live) {
        WideMeta M;
        M.fetch(A, blk, lane);
        const uint32_t idv = M.live ? M.id : 0xFFFFFFFFu;
        const float wf = expf(-(M.p_last - M.p)), wb = expf(-(M.p - M.p_first));
        blk_df = expf(-(M.p_last - M.p_before)); blk_db = expf(-(M.p_after - M.p_first));
        const bool inj = idv >= A.inj_lo && idv < A.inj_hi;       // never for rows past the end (id 0xFFFFFFFF)
        const bool res = idv >= A.res_lo && idv < A.res_hi;
        const uint64_t inj_mask = __ballot(inj);
        const uint64_t hf_mask = __ballot(M.live && M.dl >= 0.0f), hb_mask = __ballot(M.live && M.dr >= 0.0f);
        flags = block_flags(A, inj_mask, __ballot(res));
        Hf = hf_mask ? 1 : 0; Hb = hb_mask ? 1 : 0;
        // strict sums: rows before the last run head seen from the left / after the first one seen from the right
        const int cut_f = hf_mask ? 63 - __clzll((long long)hf_mask) : 0;      // rows i < cut_f count
        const int cut_b = hb_mask ? __ffsll((long long)hb_mask) - 1 : 63;      // rows i > cut_b count
        // the strict sums as weighted sums of their own: the same weights, zero outside their rows
        const float wqf = lane < cut_f ? wf : 0.0f, wqb = lane > cut_b ? wb : 0.0f;
        // phased: lane l holds the cosine and sine of the phase of row l
        float cph = 1.0f, sph = 0.0f;
        if (HALVES == 2 && inj) sincosf(A.pin.psi[idv - A.inj_lo], &sph, &cph);

        if (inj_mask) {
            // Straight-line code inside a group of eight rows: no branch around a load (a row that is not
            // injected reads row 0 and its bits are masked away).
            v4f buf[2][CH];
            auto issue = [&](int c0, v4f* dst) {
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    const int row = c0 + i;
                    const uint32_t id = lane_u(idv, row);
                    const int64_t r = ((inj_mask >> row) & 1ull) ? (int64_t)(id - A.inj_lo) : 0;
                    dst[i] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(base + r * ld_in));
                }
            };
            auto fold = [&](int c0, const v4f* src) {
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    const int row = c0 + i;
                    const uint32_t keep = ((inj_mask >> row) & 1ull) ? 0xFFFFFFFFu : 0u;     // scalar
                    const float f = lane_f(wf, row), b = lane_f(wb, row);
                    float x[HALVES][VEC];
#pragma unroll
                    for (int e = 0; e < VEC; ++e) x[0][e] = __uint_as_float(__float_as_uint(src[i][e]) & keep);
                    if (HALVES == 2) {
                        const float cr = lane_f(cph, row), sr = lane_f(sph, row);
#pragma unroll
                        for (int e = 0; e < VEC; ++e) { const float v = x[0][e]; x[0][e] = v * cr; x[HALVES - 1][e] = v * sr; }
                    }
#pragma unroll
                    for (int h = 0; h < HALVES; ++h) {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) { Sf[h][e] += f * x[h][e]; Sb[h][e] += b * x[h][e]; }
                    }
                    if (STRICT) {
                        const float qf = lane_f(wqf, row), qb = lane_f(wqb, row);
#pragma unroll
                        for (int h = 0; h < HALVES; ++h) {
#pragma unroll
                            for (int e = 0; e < VEC; ++e) { Qf[h][e] += qf * x[h][e]; Qb[h][e] += qb * x[h][e]; }
                        }
                    }
                }
            };
            // (groups of eight rows with nothing injected are skipped: uniform branches)
            if (inj_mask & 0xFFull) issue(0, buf[0]);
#pragma unroll
            for (int c = 0; c < ROWS / CH; ++c) {
                if (c + 1 < ROWS / CH) { if ((inj_mask >> ((c + 1) * CH)) & 0xFFull) issue((c + 1) * CH, buf[(c + 1) & 1]); }
                if ((inj_mask >> (c * CH)) & 0xFFull) fold(c * CH, buf[c & 1]);
            }
        }
        if (lane == 0 && flags) atomicOr(&tile_flags, flags & (kFlagInj | kFlagRes));
    }
    // The blocks' flags leave as one 32-byte store per tile, below, instead of a 4-byte store per block.
    if (lane == 0) blk_flag[wave] = flags;

    // The eight block summaries meet in LDS: each wavefront folds the ones before (after) its own into
    // the state its block starts from when the tile starts from zero; the last (first) one also takes
    // the tile's summary.
    Seg<VEC, STRICT> mf[HALVES], mb[HALVES];
#pragma unroll
    for (int h = 0; h < HALVES; ++h) {
        mf[h] = seg_identity<VEC, STRICT>(); mb[h] = seg_identity<VEC, STRICT>();
#pragma unroll
        for (int e = 0; e < VEC; ++e) { mf[h].S[e] = Sf[h][e]; mb[h].S[e] = Sb[h][e]; if (STRICT) { mf[h].Q[e] = Qf[h][e]; mb[h].Q[e] = Qb[h][e]; } }
        mf[h].D = mf[h].C = blk_df; mb[h].D = mb[h].C = blk_db;
        if (STRICT) { mf[h].H = Hf; mb[h].H = Hb; }
        put_wave_seg<VEC, STRICT>(W[h], 0, wave, lane, mf[h]);
        put_wave_seg<VEC, STRICT>(W[h], 1, wave, lane, mb[h]);
    }
    __syncthreads();
    const int tflags = tile_flags;
    if (wave == 0 && lane < kWideWaves && blockIdx.y == 0 && (tile << kWideSubShift) + lane < A.blocks)
        A.blk_flags[(tile << kWideSubShift) + lane] = (uint32_t)blk_flag[lane];

    const bool want_local = blk_live && (flags & kFlagRes) && (tflags & kFlagInj);     // uniform per wavefront
    const int64_t tile_base = tile * A.spine_rows;
    const bool sw = lane == 0 && blockIdx.y == 0;
#pragma unroll
    for (int h = 0; h < HALVES; ++h) {
        const int64_t colh = col0 + h * half;
        float F[VEC], E[VEC], R[VEC], G[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) { F[e] = E[e] = R[e] = G[e] = 0.0f; }
        if (want_local || wave == kWideWaves - 1) {
#pragma unroll 1
            for (int w = 0; w < wave; ++w) seg_apply<VEC, STRICT>(get_wave_seg<VEC, STRICT>(W[h], 0, w, lane), F, E);
        }
        if (want_local || wave == 0) {
#pragma unroll 1
            for (int w = kWideWaves - 1; w > wave; --w) seg_apply<VEC, STRICT>(get_wave_seg<VEC, STRICT>(W[h], 1, w, lane), R, G);
        }
        if (want_local && col_ok) {
            const int64_t o0 = blk * A.bpad + colh, o1 = (A.blocks + blk) * A.bpad + colh;
            store_vec<VEC>(A.blk_f + o0, F);
            store_vec<VEC>(A.blk_f + o1, R);
            if (STRICT) { store_vec<VEC>(A.blk_e + o0, E); store_vec<VEC>(A.blk_e + o1, G); }
        }
        if (wave == kWideWaves - 1) {           // the tile's forward summary = the state after the last block, from zero
            int Ht = 0;
            if (STRICT) { for (int w = 0; w < kWideWaves; ++w) Ht |= W[h].H[0][w]; }
            seg_apply<VEC, STRICT>(mf[h], F, E);
            Seg<VEC, STRICT> tf = seg_identity<VEC, STRICT>();
#pragma unroll
            for (int e = 0; e < VEC; ++e) { tf.S[e] = F[e]; if (STRICT) tf.Q[e] = E[e]; }
            tf.D = tf.C = span_decay_f(A, tile_base, A.spine_rows);     // from the anchors
            if (STRICT) tf.H = Ht;
            store_level_seg<VEC, STRICT>(A.l1, 0, tile, A.bpad, colh, col_ok && (tflags & kFlagInj), sw && h == 0, tf, (float)tflags);
        }
        if (wave == 0) {
            int Ht = 0;
            if (STRICT) { for (int w = 0; w < kWideWaves; ++w) Ht |= W[h].H[1][w]; }
            seg_apply<VEC, STRICT>(mb[h], R, G);
            Seg<VEC, STRICT> tb = seg_identity<VEC, STRICT>();
#pragma unroll
            for (int e = 0; e < VEC; ++e) { tb.S[e] = R[e]; if (STRICT) tb.Q[e] = G[e]; }
            tb.D = tb.C = span_decay_b(A, tile_base, A.spine_rows);
            if (STRICT) tb.H = Ht;
            store_level_seg<VEC, STRICT>(A.l1, 1, tile, A.bpad, colh, col_ok && (tflags & kFlagInj), sw && h == 0, tb, (float)tflags);
        }
    }
}

// Phased kernel, PhaseIn::split_blocks: the doubled rows [x cos psi | x sin psi] of the blocks whose rows the downsweeps
// will read (mode 1: blocks that hold result rows, x injected; mode 2: blocks with more than a few injected rows, x the
// weights of the result rows), one wavefront per eight rows of a block, row by row; the same products as k_phase_split.
__global__ void __launch_bounds__(kStreamWaves * 64)
k_phase_split_blocks(const ScanArgs A)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t part = (int64_t)blockIdx.x * kStreamWaves + wave;       // eight rows of a block per wavefront
    const int64_t blk = part >> 3;
    if (blk >= A.blocks) return;
    if (part == 0 && lane == 0 && A.pin.whole != nullptr) *A.pin.whole = 0u;       // x2 holds the rows of some blocks only
    const int flags = (int)A.blk_flags[blk];
    const int mode = A.pin.split_blocks;
    uint32_t lo, hi;          // ids of the rows of x
    if (mode == 1) {
        if (!(flags & kFlagRes) || !(flags & kFlagInj)) return;
        lo = A.inj_lo; hi = A.inj_hi;
    } else {
        if (!(flags & kFlagRes) || !(flags & kFlagInj) || (flags & kFlagFewInj)) return;
        lo = A.res_lo; hi = A.res_hi;
    }
    const int64_t j = blk * 64 + lane;
    const uint32_t idv = j < A.N ? A.ids[j] : 0xFFFFFFFFu;
    uint64_t m = __ballot(idv >= lo && idv < hi) & (0xFFull << (8 * (int)(part & 7)));
    const int64_t half = A.pin.half;
    while (m) {
        const int row = __ffsll((long long)m) - 1;
        m &= m - 1;
        const int64_t r = (int64_t)(lane_u(idv, row) - lo);
        float s, c;
        sincosf(A.pin.psi[r], &s, &c);
        const float* in = A.pin.x + r * A.pin.ldx;
        float* out = A.pin.x2 + r * 2 * half;
        for (int64_t t = lane; t < half; t += 64) {
            const float v = in[t];
            out[t] = v * c;
            out[half + t] = v * s;
        }
    }
}

// ---------------------------------------------------------------------------
// reduce, one WAVEFRONT per tile (batches that are not staged in sorted order, outside the wide
// geometry): row-lane r walks its share of the tile's rows chunk by chunk, so the summary needs no
// LDS and no barrier, and a workgroup is four independent wavefronts.  Same outputs as k_scan_reduce.
// ---------------------------------------------------------------------------
constexpr int kLoneWaves = 4;

template <int VEC, bool STRICT>
__global__ void __launch_bounds__(kLoneWaves * 64)
k_scan_reduce_wave(const ScanArgs A)
{
    constexpr int ITEMS = TileRows<VEC>::ITEMS;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int bv = A.bv, rv = A.rv;
    const int c = lane & (bv - 1), r = lane >> A.bv_log2;
    const int64_t slot = (int64_t)blockIdx.x * kLoneWaves + wave;
    if (A.reduce_from_list ? slot >= (int64_t)A.counters[0] : slot >= A.l1.count) return;
    const int64_t tile = A.reduce_from_list ? (int64_t)lane_u(A.list_inj[slot], 0) : slot;
    const int per = A.tile_rows / rv;                        // rows of a row-lane: a multiple of ITEMS
    const int64_t tile_base = tile * A.tile_rows, lane_row0 = tile_base + (int64_t)r * per;
    const int64_t col0 = ((int64_t)blockIdx.y * bv + c) * VEC;
    const bool col_ok = col0 < A.batch;
    const float lane_df = span_decay_f(A, lane_row0, per), lane_db = span_decay_b(A, lane_row0, per);
    const float tile_df = span_decay_f(A, tile_base, A.tile_rows), tile_db = span_decay_b(A, tile_base, A.tile_rows);

    Seg<VEC, STRICT> f = seg_identity<VEC, STRICT>(), b = seg_identity<VEC, STRICT>();
    int mine = 0;
    for (int k = 0; k < per; k += ITEMS) {
        const int64_t row0 = lane_row0 + k;
        TileRows<VEC> T;
        load_meta<VEC>(A, row0, T);
        int here = 0;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            here |= (T.id[i] >= A.inj_lo && T.id[i] < A.inj_hi) ? kFlagInj : 0;
            here |= (T.id[i] >= A.res_lo && T.id[i] < A.res_hi) ? kFlagRes : 0;
        }
        mine |= here;
        float v[ITEMS][VEC];
        if (__ballot(here & kFlagInj)) {                     // uniform: rows are read only where something is injected
            load_injected<VEC, kStreamRows<VEC>>(A, T, col0, col_ok, v);
        } else {
#pragma unroll
            for (int i = 0; i < ITEMS; ++i)
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[i][e] = 0.0f;
        }
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) seg_push<VEC, STRICT>(f, head_f<VEC>(T, i), T.dh[i], v[i]);
        // backward: this chunk's rows in reverse, then prepended to what the earlier chunks gave (whose
        // total decay comes from the anchors, not from the product of their rows' decays)
        Seg<VEC, STRICT> cb = seg_identity<VEC, STRICT>();
#pragma unroll
        for (int i = ITEMS - 1; i >= 0; --i) seg_push<VEC, STRICT>(cb, head_b<VEC>(T, i), T.dh[i + 1], v[i]);
        if (k > 0) b.D = span_decay_b(A, lane_row0, k);
        b = seg_compose<VEC, STRICT>(cb, b);
    }
    f.D = lane_df; b.D = lane_db;
    f = wave_scan<true, VEC, STRICT>(f, lane, bv, rv);
    b = wave_scan<false, VEC, STRICT>(b, lane, bv, rv);
    const int tile_flags = (__ballot(mine & kFlagInj) ? kFlagInj : 0) | (__ballot(mine & kFlagRes) ? kFlagRes : 0);
    if (lane == 0 && blockIdx.y == 0) A.blk_flags[tile] = (uint32_t)tile_flags;     // in this geometry a tile is one block
    const bool sw = c == 0 && blockIdx.y == 0;
    const bool vec_ok = col_ok && (tile_flags & kFlagInj);   // zero vectors are never fetched: not written either
    if (r == rv - 1) {
        f.D = f.C = tile_df;
        store_level_seg<VEC, STRICT>(A.l1, 0, tile, A.bpad, col0, vec_ok, sw, f, (float)tile_flags);
    }
    if (r == 0) {
        b.D = b.C = tile_db;
        store_level_seg<VEC, STRICT>(A.l1, 1, tile, A.bpad, col0, vec_ok, sw, b, (float)tile_flags);
    }
}

// ---------------------------------------------------------------------------
// spine, level 1 -> 2: summarise chunks of tile summaries (blockIdx.z = direction).
// Index q counts tiles in scan order; tile = q forward, count-1-q backward.
// ---------------------------------------------------------------------------
template <int VEC, bool STRICT>
__global__ void __launch_bounds__(kScanThreads)
k_spine_reduce(const ScanArgs A)
{
    __shared__ WaveSegs<VEC> W;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bv = A.bv, rv = A.rv;
    const int c = lane & (bv - 1), r = lane >> A.bv_log2;
    const int dir = blockIdx.z;
    const int64_t chunk = blockIdx.x;
    const int64_t q0 = chunk * A.chunk_tiles + (int64_t)(wave * rv + r) * A.spine_items;
    const int64_t col0 = ((int64_t)blockIdx.y * bv + c) * VEC;
    const bool col_ok = col0 < A.batch;

    Seg<VEC, STRICT> m = seg_identity<VEC, STRICT>();
#pragma unroll
    for (int i = 0; i < kSpineItems; ++i) {
        const int64_t q = q0 + i;
        if (i < A.spine_items && q < A.l1.count) {
            const int64_t t = dir == 0 ? q : A.l1.count - 1 - q;
            m = seg_compose<VEC, STRICT>(m, load_level_seg<VEC, STRICT, true>(A.l1, dir, t, A.bpad, col0, col_ok));
        }
    }
    m = wave_scan<true, VEC, STRICT>(m, lane, bv, rv);
    if (r == rv - 1) put_wave_seg<VEC, STRICT>(W, 0, wave, c, m);
    __syncthreads();
    if (tid < bv) {
        Seg<VEC, STRICT> t = seg_identity<VEC, STRICT>();
#pragma unroll 1
        for (int w = 0; w < kScanWaves; ++w) t = seg_compose<VEC, STRICT>(t, get_wave_seg<VEC, STRICT>(W, 0, w, c));
        // the chunk's total decay from the anchors, not from the product of its tiles' decays
        const int64_t tiles_here = A.l1.count - chunk * A.chunk_tiles < A.chunk_tiles ? A.l1.count - chunk * A.chunk_tiles
                                                                                      : A.chunk_tiles;
        if (dir == 0) {
            t.D = span_decay_f(A, chunk * A.chunk_tiles * A.spine_rows, tiles_here * A.spine_rows);
        } else {
            const int64_t t_hi = A.l1.count - 1 - chunk * A.chunk_tiles;          // first tile in scan order
            t.D = span_decay_b(A, (t_hi + 1 - tiles_here) * A.spine_rows, tiles_here * A.spine_rows);
        }
        store_level_seg<VEC, STRICT>(A.l2, dir, chunk, A.bpad, col0, col_ok, c == 0 && blockIdx.y == 0, t, 0.0f);
    }
}

// ---------------------------------------------------------------------------
// spine, top: exclusive scan over the chunk summaries, one workgroup per
// (column, direction).  Chunks are already numbered in scan order (chunk 0 of the
// backward direction holds the last tiles).  Each entry receives the state the
// sequence is in when it starts from zero: F_in = S, E_in = Q of all before it.
// ---------------------------------------------------------------------------
template <bool STRICT>
__global__ void __launch_bounds__(kSpineThreads)
k_spine_top(const Level L, int64_t bpad)
{
    constexpr int WAVES = kSpineThreads / 64;
    __shared__ float sD[WAVES], sC[WAVES], sS[WAVES], sQ[WAVES];
    __shared__ int sH[WAVES];
    typedef Seg<1, STRICT> S1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t col = blockIdx.x;
    const int dir = blockIdx.y;
    const int64_t count = L.count;
    const int64_t per = (count + kSpineThreads - 1) / kSpineThreads;
    const int64_t q0 = (int64_t)tid * per;
    const int64_t q1 = q0 + per < count ? q0 + per : count;

    auto entry = [&](int64_t q) { return q; };

    S1 mine = seg_identity<1, STRICT>();
    for (int64_t q = q0; q < q1; ++q)
        mine = seg_compose<1, STRICT>(mine, load_level_seg<1, STRICT, false>(L, dir, entry(q), bpad, col, true));

    const S1 inc = wave_scan<true, 1, STRICT>(mine, lane, 1, 64);
    if (lane == 63) { sD[wave] = inc.D; sC[wave] = inc.C; sH[wave] = inc.H; sS[wave] = inc.S[0]; sQ[wave] = inc.Q[0]; }
    __syncthreads();
    S1 run = seg_identity<1, STRICT>();
    for (int w = 0; w < wave; ++w) {
        S1 o; o.D = sD[w]; o.C = sC[w]; o.H = sH[w]; o.S[0] = sS[w]; o.Q[0] = sQ[w];
        run = seg_compose<1, STRICT>(run, o);
    }
    const S1 prev = seg_shfl<1, STRICT>(inc, (lane - 1) & 63);
    if (lane > 0) run = seg_compose<1, STRICT>(run, prev);

    for (int64_t q = q0; q < q1; ++q) {
        const int64_t o = ((int64_t)dir * count + entry(q)) * bpad + col;
        L.car_f[o] = run.S[0];
        if (STRICT) L.car_e[o] = run.H ? run.Q[0] : 0.0f;
        run = seg_compose<1, STRICT>(run, load_level_seg<1, STRICT, false>(L, dir, entry(q), bpad, col, true));
    }
}

// ---------------------------------------------------------------------------
// spine, level 2 -> 1: push the chunk carries down to the tiles of each chunk
// ---------------------------------------------------------------------------
template <int VEC, bool STRICT>
__global__ void __launch_bounds__(kScanThreads)
k_spine_down(const ScanArgs A)
{
    __shared__ WaveSegs<VEC> W;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bv = A.bv, rv = A.rv;
    const int c = lane & (bv - 1), r = lane >> A.bv_log2;
    const int dir = blockIdx.z;
    const int64_t chunk = blockIdx.x;

    // The list of the blocks the heavy downsweep must visit, when the reduce saw every tile itself (with a
    // metadata pass the list is already there): one workgroup per chunk compacts its blocks' flags, slots from
    // a counter in LDS, and takes its stretch of the list with ONE atomic on the shared counter (instead of one
    // per listed block from inside the reduce, each waited for by a wavefront on its way to the tile's barrier).
    if (A.down_from_list && !A.reduce_from_list && dir == 0 && blockIdx.y == 0) {
        __shared__ uint32_t l_count, l_base;
        constexpr int kMaxPer = 8;                               // a chunk has at most 4096 blocks
        if (tid == 0) l_count = 0u;
        __syncthreads();
        const int64_t b0 = (chunk * A.chunk_tiles) << A.sub_shift;
        const int64_t nb = (int64_t)A.chunk_tiles << A.sub_shift;
        uint32_t slot[kMaxPer];
#pragma unroll
        for (int q = 0; q < kMaxPer; ++q) {
            const int64_t o = (int64_t)q * kScanThreads + tid, b = b0 + o;
            const bool listed = o < nb && b < A.blocks && listed_block((int)A.blk_flags[b]);
            slot[q] = listed ? atomicAdd(&l_count, 1u) : 0xFFFFFFFFu;
        }
        __syncthreads();
        if (tid == 0) l_base = l_count ? atomicAdd(&A.counters[1], l_count) : 0u;
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kMaxPer; ++q)
            if (slot[q] != 0xFFFFFFFFu) A.list_both[l_base + slot[q]] = (uint32_t)(b0 + (int64_t)q * kScanThreads + tid);
    }
    const int64_t q0 = chunk * A.chunk_tiles + (int64_t)(wave * rv + r) * A.spine_items;
    const int64_t col0 = ((int64_t)blockIdx.y * bv + c) * VEC;
    const bool col_ok = col0 < A.batch;

    // Decay and head flag over the tiles with scan indices [qa, qb) (clipped to the tiles there are), from the anchors:
    // a composite summary never keeps the product of its parts' decays.  (Equal spans have equal decays with equal rounding
    // errors -- on a regular grid every tile's is the same -- and a chain of m of them carries m times that error.)
    const int64_t count = A.l1.count, SR = A.spine_rows;
    auto span = [&](int64_t qa, int64_t qb, float& D, bool& H) {
        qb = qb < count ? qb : count;
        D = 1.0f; H = false;
        if (qa >= qb) return;
        if (dir == 0) {
            D = span_decay_f(A, qa * SR, (qb - qa) * SR);
            H = span_head_f(A, qa * SR, (qb - qa) * SR);
        } else {                          // scan index q is tile count - 1 - q
            D = span_decay_b(A, (count - qb) * SR, (qb - qa) * SR);
            H = span_head_b(A, (count - qb) * SR, (qb - qa) * SR);
        }
    };
    Seg<VEC, STRICT> segs[kSpineItems];
    Seg<VEC, STRICT> m = seg_identity<VEC, STRICT>();
#pragma unroll
    for (int i = 0; i < kSpineItems; ++i) {
        const int64_t q = q0 + i;
        segs[i] = seg_identity<VEC, STRICT>();
        if (i < A.spine_items && q < A.l1.count) {
            const int64_t t = dir == 0 ? q : A.l1.count - 1 - q;
            segs[i] = load_level_seg<VEC, STRICT, true>(A.l1, dir, t, A.bpad, col0, col_ok);
        }
        m = seg_compose<VEC, STRICT>(m, segs[i]);
    }
    {
        float D; bool H;
        span(q0, q0 + A.spine_items, D, H);
        if (q0 < count) m.D = m.C = D;
    }
    // inclusive scan over the row-lanes of the wavefront; after every step a row-lane's summary covers the row-lanes
    // [r - 2 step + 1, r], and its decay is taken over exactly those tiles
    Seg<VEC, STRICT> inc = m;
    for (int step = 1; step < rv; step <<= 1) {
        const Seg<VEC, STRICT> o = seg_shfl<VEC, STRICT>(inc, (lane - step * bv) & 63);
        if (r >= step) {
            inc = seg_compose<VEC, STRICT>(o, inc);
            const int r_lo = r - 2 * step + 1 > 0 ? r - 2 * step + 1 : 0;
            float D; bool H;
            span(q0 - (int64_t)(r - r_lo) * A.spine_items, q0 + A.spine_items, D, H);
            inc.D = inc.C = D;
        }
    }
    if (r == rv - 1) put_wave_seg<VEC, STRICT>(W, 0, wave, c, inc);
    Seg<VEC, STRICT> exc = seg_shfl<VEC, STRICT>(inc, (lane - bv) & 63);
    if (r == 0) exc = seg_identity<VEC, STRICT>();
    __syncthreads();

    float F[VEC], E[VEC], Fc[VEC], Ec[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { F[e] = E[e] = Fc[e] = Ec[e] = 0.0f; }
    if (col_ok && A.l2.count > 1) {     // a single chunk starts from zero: the upper spine kernels have not run
        const int64_t o = ((int64_t)dir * A.l2.count + chunk) * A.bpad + col0;
        load_vec<VEC>(Fc, A.l2.car_f + o);
        if (STRICT) load_vec<VEC>(Ec, A.l2.car_e + o);
    }
#pragma unroll 1
    for (int w = 0; w < wave; ++w) seg_apply<VEC, STRICT>(get_wave_seg<VEC, STRICT>(W, 0, w, c), F, E);
    seg_apply<VEC, STRICT>(exc, F, E);
    // the chunk's carry reaches this row-lane's first tile through one exponential of an anchor difference
    if (q0 < A.l1.count) {
        float D; bool H;
        span(chunk * A.chunk_tiles, q0, D, H);
        enter_state<VEC, STRICT>(F, E, Fc, Ec, D, H);
    }
    // ... and the state at the row-lane's first tile reaches each of its tiles the same way: what the tiles in between
    // add (from zero) plus the entering state decayed over them by one exponential
    float Fl[VEC], El[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { Fl[e] = El[e] = 0.0f; }
#pragma unroll
    for (int i = 0; i < kSpineItems; ++i) {
        const int64_t q = q0 + i;
        if (i < A.spine_items && q < A.l1.count) {
            const int64_t t = dir == 0 ? q : A.l1.count - 1 - q;
            float Ft[VEC], Et[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) { Ft[e] = Fl[e]; Et[e] = El[e]; }
            float D; bool H;
            span(q0, q, D, H);
            enter_state<VEC, STRICT>(Ft, Et, F, E, D, H);
            if (col_ok) {
                const int64_t o = ((int64_t)dir * A.l1.count + t) * A.bpad + col0;
                store_vec<VEC>(A.l1.car_f + o, Ft);
                if (STRICT) store_vec<VEC>(A.l1.car_e + o, Et);
            }
            seg_apply<VEC, STRICT>(segs[i], Fl, El);
        }
    }
}

// Row reduction over the batch: sum over the bv lanes of a row-lane, then write.
__device__ __forceinline__ void emit_row_sum(const ScanArgs& A, float acc, int bv, int c, bool is_res, int64_t rr,
                                             int64_t res_rows)
{
    for (int m = 1; m < bv; m <<= 1) acc += __shfl_xor(acc, m);
    if (is_res && c == 0) {
        if (A.slabs == 1) A.out_red[rr * A.ld_red] = acc;
        else A.red_partial[(int64_t)blockIdx.y * res_rows + rr] = acc;
    }
}

// Carries into a block, forward (Fc, Ec) and backward (Rc, Gc).  A block that is a tile of its own
// reads them as the spine left them.  In the wide geometry the spine's carries belong to the tile of
// 2^sub_shift blocks: the block's carry is the tile's, decayed to the block by one exponential of an
// anchor difference, plus the state the reduce found for the block with the tile starting from zero
// (kept only for tiles that hold injected rows; zero otherwise).
template <int VEC, bool STRICT>
__device__ __forceinline__ void load_block_carries(const ScanArgs& A, int64_t blk, int64_t col0, bool col_ok,
                                                   float* Fc, float* Ec, float* Rc, float* Gc)
{
#pragma unroll
    for (int e = 0; e < VEC; ++e) { Fc[e] = Ec[e] = Rc[e] = Gc[e] = 0.0f; }
    const int64_t tile = blk >> A.sub_shift;
    float Ft[VEC], Et[VEC], Rt[VEC], Gt[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { Ft[e] = Et[e] = Rt[e] = Gt[e] = 0.0f; }
    if (col_ok) {
        const int64_t o0 = tile * A.bpad + col0, o1 = (A.l1.count + tile) * A.bpad + col0;
        load_vec<VEC>(Ft, A.l1.car_f + o0);
        load_vec<VEC>(Rt, A.l1.car_f + o1);
        if (STRICT) { load_vec<VEC>(Et, A.l1.car_e + o0); load_vec<VEC>(Gt, A.l1.car_e + o1); }
    }
    if (A.sub_shift == 0) {         // uniform
#pragma unroll
        for (int e = 0; e < VEC; ++e) { Fc[e] = Ft[e]; Ec[e] = Et[e]; Rc[e] = Rt[e]; Gc[e] = Gt[e]; }
        return;
    }
    const bool tile_inj = ((int)A.l1.scalar[tile].w & kFlagInj) != 0;
    if (tile_inj && col_ok) {
        const int64_t o0 = blk * A.bpad + col0, o1 = (A.blocks + blk) * A.bpad + col0;
        load_vec<VEC>(Fc, A.blk_f + o0);
        load_vec<VEC>(Rc, A.blk_f + o1);
        if (STRICT) { load_vec<VEC>(Ec, A.blk_e + o0); load_vec<VEC>(Gc, A.blk_e + o1); }
    }
    const int64_t tile_base = tile * A.spine_rows, blk_base = blk * A.tile_rows;
    const int64_t blk_end = blk_base + A.tile_rows, tile_end = tile_base + A.spine_rows;
    enter_state<VEC, STRICT>(Fc, Ec, Ft, Et, span_decay_f(A, tile_base, blk_base - tile_base),
                             span_head_f(A, tile_base, blk_base - tile_base));
    enter_state<VEC, STRICT>(Rc, Gc, Rt, Gt, span_decay_b(A, blk_end, tile_end - blk_end),
                             span_head_b(A, blk_end, tile_end - blk_end));
}

// ---------------------------------------------------------------------------
// downsweep: tiles that hold both injected and result rows
// ---------------------------------------------------------------------------
// WAVES: wavefronts of the workgroup (sizes the LDS buffer); RED: the row reduction is wanted (out_red);
// ZS: the reduction takes in the saved strict scans (A.zs) -- without them the kernel fits in 128 registers
// at scalar lanes, and a compute unit holds two workgroups of eight wavefronts instead of one.
template <int VEC, bool STRICT, int WAVES, bool RED, bool ZS = RED>
__global__ void __launch_bounds__(WAVES * 64)
k_scan_down(const ScanArgs A)
{
    constexpr int ITEMS = TileRows<VEC>::ITEMS;
    // One LDS buffer, used twice: first for the exchange of wavefront summaries, then (strict scans only)
    // for the per-row strict forward values, which would otherwise cost ITEMS * VEC registers per lane.
    constexpr size_t kEfBytes = STRICT ? sizeof(float) * ITEMS * WAVES * 64 * VEC : 0;
    constexpr size_t kSmem = sizeof(WaveSegs<VEC>) > kEfBytes ? sizeof(WaveSegs<VEC>) : kEfBytes;
    __shared__ __align__(16) unsigned char smem[kSmem];
    WaveSegs<VEC>& W = *reinterpret_cast<WaveSegs<VEC>*>(smem);
    float* const ef = reinterpret_cast<float*>(smem) + (size_t)threadIdx.x * VEC;   // row i at ef[i * ef_stride]
    constexpr size_t ef_stride = (size_t)WAVES * 64 * VEC;
    if (A.down_from_list && blockIdx.x >= A.counters[1]) return;
    const int64_t tile = A.down_from_list ? A.list_both[blockIdx.x] : blockIdx.x;     // the block this workgroup owns
    const int flags = (int)A.blk_flags[tile];
    if ((flags & (kFlagInj | kFlagRes | kFlagFewInj | kFlagFewRes)) != (kFlagInj | kFlagRes)) return;
    const uint32_t poison = plan_poison(A.counters);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bv = A.bv, rv = A.rv;
    const int c = lane & (bv - 1), r = lane >> A.bv_log2;
    const int64_t wave_row0 = tile * A.tile_rows + (int64_t)(wave * rv) * ITEMS;
    const int64_t row0 = wave_row0 + (int64_t)r * ITEMS;
    const int64_t col0 = ((int64_t)blockIdx.y * bv + c) * VEC;
    const bool col_ok = col0 < A.batch;

    // decays from the anchors (see k_decay), asked for first so their loads go out with the others:
    // over this row-lane's rows, over this wavefront's rows, and from the tile's ends to this row-lane
    const float lane_df = span_decay_f(A, row0, ITEMS), lane_db = span_decay_b(A, row0, ITEMS);
    const float wave_df = rv == 1 ? lane_df : span_decay_f(A, wave_row0, rv * ITEMS);
    const float wave_db = rv == 1 ? lane_db : span_decay_b(A, wave_row0, rv * ITEMS);
    const int64_t tile_base = tile * A.tile_rows, rows_after = row0 + ITEMS;
    const float enter_df = span_decay_f(A, tile_base, row0 - tile_base);
    const float enter_db = span_decay_b(A, rows_after, tile_base + A.tile_rows - rows_after);
    const bool enter_hf = span_head_f(A, tile_base, row0 - tile_base);
    const bool enter_hb = span_head_b(A, rows_after, tile_base + A.tile_rows - rows_after);

    TileRows<VEC> T;
    load_meta<VEC>(A, row0, T);
    float v[ITEMS][VEC];
    if (A.stage) {      // uniform: the reduce left this tile's injected rows in sorted order (zeros elsewhere)
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
            load_vec_or_zero<VEC>(v[i], A.stage, (row0 + i) * A.batch + col0, col_ok && T.id[i] != 0xFFFFFFFFu);
    } else {
        load_injected<VEC, kStreamRows<VEC>>(A, T, col0, col_ok, v);
    }

    constexpr bool want_red = STRICT && RED;
    // The saved strict scans enter the row reduction only through sum_t v * zs, which needs nothing from
    // the walks: their rows are asked for together with the injected rows and folded into one number per
    // row.  The weights of the reduction are fetched one row ahead of their use in the backward walk
    // (holding all rows of them would cost ITEMS * VEC registers).
    float vz[ZS ? ITEMS : 1];
#pragma unroll
    for (int i = 0; i < (ZS ? ITEMS : 1); ++i) vz[i] = 0.0f;
    if (want_red && ZS && A.zs) {                        // uniform
        float zrow[ITEMS][VEC];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const bool ok = col_ok && T.id[i] >= A.res_lo && T.id[i] < A.res_hi;
            load_vec_or_zero<VEC, kStreamRows<VEC>>(zrow[i], A.zs, ((int64_t)T.id[i] - (int64_t)A.res_lo) * A.batch + col0, ok);
        }
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
#pragma unroll
            for (int e = 0; e < VEC; ++e) vz[ZS ? i : 0] += v[i][e] * zrow[i][e];
    }
    auto fetch_row = [&](int i, float* wrow) {
        const bool ok = col_ok && T.id[i] >= A.res_lo && T.id[i] < A.res_hi;
        const int64_t rr = (int64_t)T.id[i] - (int64_t)A.res_lo;
#pragma unroll
        for (int e = 0; e < VEC; ++e) wrow[e] = 0.0f;
        if (want_red) {                                  // uniform branches
            if (A.wstage) load_vec_or_zero<VEC, kStreamRows<VEC>>(wrow, A.wstage, (row0 + i) * A.batch + col0, ok);
            else load_vec_or_zero<VEC, kStreamRows<VEC>>(wrow, A.w, rr * A.ld_w + col0, ok);
        }
    };

    // scalar lanes can afford all the weights at once (one register a row): their loads go out here, with the
    // others, instead of one row ahead of their use, where each would be waited for in turn
    constexpr bool w_ahead = want_red && VEC == 1;
    float wall[w_ahead ? ITEMS : 1][VEC];
    if (w_ahead) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) fetch_row(i, wall[i]);
    }

    // carries into the block
    float Fc[VEC], Ec[VEC], Rc[VEC], Gc[VEC];
    load_block_carries<VEC, STRICT>(A, tile, col0, col_ok, Fc, Ec, Rc, Gc);
    Seg<VEC, STRICT> fe, be;
    {
        Seg<VEC, STRICT> f = seg_identity<VEC, STRICT>();
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) seg_push<VEC, STRICT>(f, head_f<VEC>(T, i), T.dh[i], v[i]);
        f.D = lane_df;
        f = wave_scan<true, VEC, STRICT>(f, lane, bv, rv);
        if (r == rv - 1) {
            Seg<VEC, STRICT> tot = f;
            tot.D = wave_df;
            put_wave_seg<VEC, STRICT>(W, 0, wave, c, tot);
        }
        fe = seg_shfl<VEC, STRICT>(f, (lane - bv) & 63);
        if (r == 0) fe = seg_identity<VEC, STRICT>();
    }
    {
        Seg<VEC, STRICT> b = seg_identity<VEC, STRICT>();
#pragma unroll
        for (int i = ITEMS - 1; i >= 0; --i) seg_push<VEC, STRICT>(b, head_b<VEC>(T, i), T.dh[i + 1], v[i]);
        b.D = lane_db;
        b = wave_scan<false, VEC, STRICT>(b, lane, bv, rv);
        if (r == 0) {
            Seg<VEC, STRICT> tot = b;
            tot.D = wave_db;
            put_wave_seg<VEC, STRICT>(W, 1, wave, c, tot);
        }
        be = seg_shfl<VEC, STRICT>(b, (lane + bv) & 63);
        if (r == rv - 1) be = seg_identity<VEC, STRICT>();
    }
    __syncthreads();
    // entering states: what the earlier rows of the tile contribute (their summaries applied to zero) ...
    float F[VEC], E[VEC], R[VEC], G[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { F[e] = E[e] = R[e] = G[e] = 0.0f; }
#pragma unroll 1
    for (int w = 0; w < wave; ++w) seg_apply<VEC, STRICT>(get_wave_seg<VEC, STRICT>(W, 0, w, c), F, E);
#pragma unroll 1
    for (int w = WAVES - 1; w > wave; --w) seg_apply<VEC, STRICT>(get_wave_seg<VEC, STRICT>(W, 1, w, c), R, G);
    seg_apply<VEC, STRICT>(fe, F, E);
    seg_apply<VEC, STRICT>(be, R, G);
    // ... plus the tile's carries, decayed over those rows by one exponential of an anchor difference
    enter_state<VEC, STRICT>(F, E, Fc, Ec, enter_df, enter_hf);
    enter_state<VEC, STRICT>(R, G, Rc, Gc, enter_db, enter_hb);

    if (STRICT) __syncthreads();      // every wavefront is done with the summaries: the buffer now holds E per row

    // forward walk: keep F of every row in registers, E of every row in LDS
    float Ff[ITEMS][VEC];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool h = head_f<VEC>(T, i);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            E[e] = h ? T.dh[i] * F[e] : E[e];
            F[e] = (h ? E[e] : F[e]) + v[i][e];
            Ff[i][e] = F[e];
        }
        if (STRICT) store_vec<VEC>(ef + (size_t)i * ef_stride, E);
    }

    // backward walk with emission
    const int64_t res_rows = (int64_t)A.res_hi - (int64_t)A.res_lo;
    float wnext[VEC];
    if (!w_ahead) fetch_row(ITEMS - 1, wnext);
#pragma unroll
    for (int i = ITEMS - 1; i >= 0; --i) {
        float wrow[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) wrow[e] = w_ahead ? wall[w_ahead ? i : 0][e] : wnext[e];
        if (!w_ahead && i > 0) fetch_row(i - 1, wnext);
        const bool h = head_b<VEC>(T, i);
        float P[VEC], Z[VEC], Efi[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) Efi[e] = 0.0f;
        if (STRICT) load_vec<VEC>(Efi, ef + (size_t)i * ef_stride);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            G[e] = h ? T.dh[i + 1] * R[e] : G[e];
            R[e] = (h ? G[e] : R[e]) + v[i][e];
            P[e] = taint(Ff[i][e] + R[e] - v[i][e], poison);
            Z[e] = taint(G[e] - Efi[e], poison);
        }
        const bool is_res = T.id[i] >= A.res_lo && T.id[i] < A.res_hi;
        // where the row's outputs go: by its id, or (routes through sorted order) by its position in the sorted sequence
        const int64_t rr = A.out_sorted ? row0 + i : (int64_t)T.id[i] - (int64_t)A.res_lo;
        if (VEC == 1 && A.pair_out) {      // uniform; batch 1: both outputs of the row with one 8-byte store
            float second = Z[0];
            if (want_red) second = taint((ZS ? vz[ZS ? i : 0] : 0.0f) + wrow[0] * Z[0], poison);
            if (is_res && col_ok) *reinterpret_cast<float2*>(A.out_p + rr * 2) = make_float2(P[0], second);
            continue;
        }
        if (is_res && col_ok) {
            if (kStreamRows<VEC>) {
                if (A.out_p) store_vec_stream<VEC>(A.out_p + rr * A.ld_p + col0, P);
                if (STRICT && A.out_z) store_vec_stream<VEC>(A.out_z + rr * A.ld_z + col0, Z);
            } else {
                if (A.out_p) store_vec<VEC>(A.out_p + rr * A.ld_p + col0, P);
                if (STRICT && A.out_z) store_vec<VEC>(A.out_z + rr * A.ld_z + col0, Z);
            }
        }
        if (want_red) {
            float acc = ZS ? vz[ZS ? i : 0] : 0.0f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc += wrow[e] * Z[e];     // wrow is 0 off the result rows
            emit_row_sum(A, acc, bv, c, is_res, rr, res_rows);
        }
    }
}

// ---------------------------------------------------------------------------
// downsweep_sparse: tiles with result rows and nothing injected.  With no
// injection inside the tile every row is a closed form of the two carries:
//   F_j = cf_j F_in,           cf_j = product of the decays from the tile start to j
//   E_j = F_j if a run head lies at or before j inside the tile, else E_in
// and symmetrically from the right.  The decays come from the anchors directly, so
// the kernel has no scan, no LDS and no barrier; the batch columns are streamed.
// ---------------------------------------------------------------------------
template <int VEC, bool STRICT>
__global__ void __launch_bounds__(kScanThreads)
k_scan_down_sparse(const ScanArgs A)
{
    constexpr int ITEMS = TileRows<VEC>::ITEMS;
    // the last kernel of a scan: nothing reads the list lengths any more, and the next scan wants them at zero
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 2) A.counters[threadIdx.x] = 0u;
    const int64_t tile = blockIdx.x;                // the block this workgroup owns
    const int flags = (int)A.blk_flags[tile];
    // result rows and nothing injected (blocks with a few injected rows exist in the wide geometry only, which has a kernel of its own)
    if (!(flags & kFlagRes) || (flags & kFlagInj)) return;
    const uint32_t poison = plan_poison(A.counters);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bv = A.bv, rv = A.rv;
    const int c = lane & (bv - 1), r = lane >> A.bv_log2;
    const int64_t row0 = tile * A.tile_rows + (int64_t)(wave * rv + r) * ITEMS;
    const int64_t col0 = ((int64_t)blockIdx.y * bv + c) * VEC;
    const bool col_ok = col0 < A.batch;

    // everything in the tile before / after this row-lane: one exponential of an anchor difference each,
    // so no scan over the row-lanes and no LDS are needed (asked for first: the loads go out early)
    const int64_t tile_base = tile * A.tile_rows, after = row0 + ITEMS, tile_end = tile_base + A.tile_rows;
    const float Df = span_decay_f(A, tile_base, row0 - tile_base), Db = span_decay_b(A, after, tile_end - after);
    const int Hf = span_head_f(A, tile_base, row0 - tile_base) ? 1 : 0, Hb = span_head_b(A, after, tile_end - after) ? 1 : 0;

    TileRows<VEC> T;
    load_meta<VEC>(A, row0, T);
    const bool want_red = STRICT && A.out_red != nullptr;
    float wv[ITEMS][VEC];
    load_weights<VEC>(A, T, row0, col0, col_ok, want_red, wv);
    float Fin[VEC], Ein[VEC], Rin[VEC], Gin[VEC];
    load_block_carries<VEC, STRICT>(A, tile, col0, col_ok, Fin, Ein, Rin, Gin);

    // per-row cumulative decays inside this row-lane, from the left and from the right (at most ITEMS factors)
    float cf[ITEMS], cb[ITEMS];
    int hf = 0, hb = 0;               // bit i: a run head at or before (after) row i inside the row-lane
    {
        float p = 1.0f; int seen = 0;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const bool h = head_f<VEC>(T, i);
            p *= h ? T.dh[i] : 1.0f; seen |= h ? 1 : 0;
            cf[i] = p; hf |= seen << i;
        }
        p = 1.0f; seen = 0;
#pragma unroll
        for (int i = ITEMS - 1; i >= 0; --i) {
            const bool h = head_b<VEC>(T, i);
            p *= h ? T.dh[i + 1] : 1.0f; seen |= h ? 1 : 0;
            cb[i] = p; hb |= seen << i;
        }
    }
    const int64_t res_rows = (int64_t)A.res_hi - (int64_t)A.res_lo;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool is_res = T.id[i] >= A.res_lo && T.id[i] < A.res_hi;
        const int64_t rr = A.out_sorted ? row0 + i : (int64_t)T.id[i] - (int64_t)A.res_lo;
        const float kf = Df * cf[i], kb = Db * cb[i];
        const bool seen_f = Hf | ((hf >> i) & 1), seen_b = Hb | ((hb >> i) & 1);
        float P[VEC], Z[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float Fj = kf * Fin[e], Rj = kb * Rin[e];
            P[e] = taint(Fj + Rj, poison);
            Z[e] = taint((seen_b ? Rj : Gin[e]) - (seen_f ? Fj : Ein[e]), poison);
        }
        if (is_res && col_ok) {
            if (A.out_p) store_vec<VEC>(A.out_p + rr * A.ld_p + col0, P);
            if (STRICT && A.out_z) store_vec<VEC>(A.out_z + rr * A.ld_z + col0, Z);
        }
        if (want_red) {
            float acc = 0.0f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc += wv[i][e] * Z[e];      // wv is 0 off the result rows
            emit_row_sum(A, acc, bv, c, is_res, rr, res_rows);
        }
    }
}

// ---------------------------------------------------------------------------
// downsweep, wide geometry, blocks with injected rows and at most kFewRows result rows (an apply
// with few outputs): one WAVEFRONT per block.  Result row r is
//   P_r = D_f Fc + D_b Rc + sum_l exp(-|p_r - p_l|) v_l          (Sec. 1: the definition, inside the block)
//   Z_r = (strict carries) + sum_l sgn(p_l - p_r) exp(-|p_r - p_l|) v_l
// so the block's injected rows are streamed once, with one weight vector per result row (lane l
// holds the weights of row l), as in the wide reduce.  No LDS, no barrier.
// ---------------------------------------------------------------------------
constexpr int kFewWaves = 4;

template <bool STRICT>
__global__ void __launch_bounds__(kFewWaves * 64)
k_scan_down_fewres(const ScanArgs A)
{
    constexpr int VEC = 4, ROWS = 64, CH = 8, NR = kFewRows;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t slot = (int64_t)blockIdx.x * kFewWaves + wave;
    if (A.down_from_list ? slot >= (int64_t)A.counters[1] : slot >= A.blocks) return;
    const int64_t blk = A.down_from_list ? (int64_t)lane_u(A.list_both[slot], 0) : slot;
    const int flags = (int)A.blk_flags[blk];
    if ((flags & (kFlagInj | kFlagRes | kFlagFewInj | kFlagFewRes)) != (kFlagInj | kFlagRes | kFlagFewRes)) return;
    const uint32_t poison = plan_poison(A.counters);
    const int64_t col0 = ((int64_t)blockIdx.y * 64 + lane) * VEC;
    const bool col_ok = col0 < A.batch;
    const float* const base = A.inj + (col_ok ? col0 : 0);

    WideMeta M;
    M.fetch(A, blk, lane);
    float Fc[VEC], Ec[VEC], Rc[VEC], Gc[VEC];
    load_block_carries<VEC, STRICT>(A, blk, col0, col_ok, Fc, Ec, Rc, Gc);
    const uint32_t idv = M.live ? M.id : 0xFFFFFFFFu;
    const bool inj = idv >= A.inj_lo && idv < A.inj_hi;
    const uint64_t inj_mask = __ballot(inj);
    uint64_t res_mask = __ballot(idv >= A.res_lo && idv < A.res_hi);
    const uint64_t hf_mask = __ballot(M.live && M.dl >= 0.0f), hb_mask = __ballot(M.live && M.dr >= 0.0f);
    // decay of the carries to row `lane`
    const float df = expf(-(M.p - M.p_before)), db = expf(-(M.p_after - M.p));

    int rrow[NR]; bool have[NR];
    float wP[NR], wZ[NR];           // lane l: weight of injected row l for result row q
#pragma unroll
    for (int q = 0; q < NR; ++q) {
        have[q] = res_mask != 0;
        rrow[q] = have[q] ? __ffsll((long long)res_mask) - 1 : 0;
        res_mask &= res_mask - 1;
        const float pr = lane_f(M.p, rrow[q]);
        wP[q] = (have[q] && inj) ? expf(-fabsf(M.p - pr)) : 0.0f;
        wZ[q] = M.p > pr ? wP[q] : (M.p < pr ? -wP[q] : 0.0f);
    }
    float aP[NR][VEC], aZ[NR][VEC];
#pragma unroll
    for (int q = 0; q < NR; ++q)
#pragma unroll
        for (int e = 0; e < VEC; ++e) { aP[q][e] = 0.0f; aZ[q][e] = 0.0f; }

    {
        v4f buf[2][CH];
        auto issue = [&](int c0, v4f* dst) {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int row = c0 + i;
                const uint32_t id = lane_u(idv, row);
                const int64_t r = ((inj_mask >> row) & 1ull) ? (int64_t)(id - A.inj_lo) : 0;
                dst[i] = *reinterpret_cast<const v4f*>(base + r * A.ld_inj);
            }
        };
        auto fold = [&](int c0, const v4f* src) {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int row = c0 + i;
                const uint32_t keep = ((inj_mask >> row) & 1ull) ? 0xFFFFFFFFu : 0u;
                float x[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[e] = __uint_as_float(__float_as_uint(src[i][e]) & keep);
#pragma unroll
                for (int q = 0; q < NR; ++q) {
                    const float a = lane_f(wP[q], row);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) aP[q][e] += a * x[e];
                    if (STRICT) {
                        const float z = lane_f(wZ[q], row);
#pragma unroll
                        for (int e = 0; e < VEC; ++e) aZ[q][e] += z * x[e];
                    }
                }
            }
        };
        if (inj_mask & 0xFFull) issue(0, buf[0]);
#pragma unroll
        for (int c = 0; c < ROWS / CH; ++c) {
            if (c + 1 < ROWS / CH) { if ((inj_mask >> ((c + 1) * CH)) & 0xFFull) issue((c + 1) * CH, buf[(c + 1) & 1]); }
            if ((inj_mask >> (c * CH)) & 0xFFull) fold(c * CH, buf[c & 1]);
        }
    }

    const bool want_red = STRICT && A.out_red != nullptr;
    const int64_t res_rows = (int64_t)A.res_hi - (int64_t)A.res_lo;
#pragma unroll
    for (int q = 0; q < NR; ++q) {
        if (!have[q]) continue;                                     // uniform
        const int r = rrow[q];
        const float kf = lane_f(df, r), kb = lane_f(db, r);
        const bool seen_f = (hf_mask & ((2ull << r) - 1ull)) != 0;   // a run head at or before row r inside the block
        const bool seen_b = (hb_mask >> r) != 0;                     // ... at or after it, seen from the right
        const int64_t rr = (int64_t)lane_u(idv, r) - (int64_t)A.res_lo;
        float P[VEC], Z[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float Fj = kf * Fc[e], Rj = kb * Rc[e];
            P[e] = taint(aP[q][e] + Fj + Rj, poison);
            Z[e] = taint(aZ[q][e] + ((seen_b ? Rj : Gc[e]) - (seen_f ? Fj : Ec[e])), poison);
        }
        if (col_ok) {
            if (A.out_p) store_vec<VEC>(A.out_p + rr * A.ld_p + col0, P);
            if (STRICT && A.out_z) store_vec<VEC>(A.out_z + rr * A.ld_z + col0, Z);
        }
        if (want_red) {
            float wrow[VEC];
            load_vec_or_zero<VEC>(wrow, A.w, rr * A.ld_w + col0, col_ok);
            float acc = 0.0f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc += wrow[e] * Z[e];
            emit_row_sum(A, acc, 64, lane, true, rr, res_rows);
        }
    }
}

// ---------------------------------------------------------------------------
// downsweep_sparse for the wide geometry: one WAVEFRONT per 64-row block (every lane on its own 4
// columns), so the block's carries are read once and not once per wavefront of a workgroup.  Same
// closed forms as k_scan_down_sparse, with the per-row factors taken from the anchors by the lane
// that looks at the row (kf_l = exp(-(p_l - p_before)), kb_l = exp(-(p_after - p_l))) and handed to
// the scalar unit with readlane; the few rows injected inside the block add their direct terms.
// The batch reduction of eight rows at a time is a butterfly: 10 cross-lane steps for 8 row sums.
// ---------------------------------------------------------------------------

template <bool STRICT>
__global__ void __launch_bounds__(kStreamWaves * 64)
k_scan_down_sparse_wide(const ScanArgs A)
{
    constexpr int VEC = 4, ROWS = 64, CH = 8, NS = kFewRows;
    // the last kernel of a scan: nothing reads the list lengths any more, and the next scan wants them at zero
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 2) A.counters[threadIdx.x] = 0u;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t blk = (int64_t)blockIdx.x * kStreamWaves + wave;
    if (blk >= A.blocks) return;
    const int flags = (int)A.blk_flags[blk];
    // result rows, and nothing injected or at most kFewRows injected rows
    if (!(flags & kFlagRes) || ((flags & kFlagInj) && !(flags & kFlagFewInj))) return;
    const uint32_t poison = plan_poison(A.counters);
    const int64_t col0 = ((int64_t)blockIdx.y * 64 + lane) * VEC;
    const bool col_ok = col0 < A.batch;
    const int64_t colc = col_ok ? col0 : 0;      // lanes past the last column read (and drop) columns 0..3

    WideMeta M;
    M.fetch(A, blk, lane);
    float Fin[VEC], Ein[VEC], Rin[VEC], Gin[VEC];
    load_block_carries<VEC, STRICT>(A, blk, col0, col_ok, Fin, Ein, Rin, Gin);
    const uint32_t idv = M.live ? M.id : 0xFFFFFFFFu;
    const uint64_t res_mask = __ballot(idv >= A.res_lo && idv < A.res_hi);
    const uint64_t hf_mask = __ballot(M.live && M.dl >= 0.0f), hb_mask = __ballot(M.live && M.dr >= 0.0f);
    const float kf = expf(-(M.p - M.p_before)), kb = expf(-(M.p_after - M.p));

    // the few rows injected inside the block: lane l holds the weight of source q for row l
    const bool sources = (flags & kFlagFewInj) != 0;       // uniform
    float vs[NS][VEC], ws[NS], wz[NS];
#pragma unroll
    for (int q = 0; q < NS; ++q) {
        ws[q] = wz[q] = 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) vs[q][e] = 0.0f;
    }
    if (sources) {
        uint64_t m = __ballot(idv >= A.inj_lo && idv < A.inj_hi);
#pragma unroll
        for (int q = 0; q < NS; ++q) {
            const bool have = m != 0;
            const int rs = have ? __ffsll((long long)m) - 1 : 0;
            m &= m - 1;
            const float pq = lane_f(M.p, rs);
            const uint32_t idq = lane_u(idv, rs);
            if (have && col_ok) load_vec<VEC>(vs[q], A.inj + (int64_t)(idq - A.inj_lo) * A.ld_inj + col0);
            ws[q] = have ? expf(-fabsf(M.p - pq)) : 0.0f;
            wz[q] = pq > M.p ? ws[q] : (pq < M.p ? -ws[q] : 0.0f);
        }
    }

    const bool want_red = STRICT && A.out_red != nullptr;
    const int64_t res_rows = (int64_t)A.res_hi - (int64_t)A.res_lo;
#pragma unroll
    for (int c = 0; c < ROWS / CH; ++c) {
        if (!((res_mask >> (c * CH)) & 0xFFull)) continue;          // uniform: no result row among these eight
        v4f x[CH];
        if (want_red) {     // weights of the row reduction (no branch around a load: rows that are not wanted read row 0)
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int row = c * CH + i;
                const int64_t rr = ((res_mask >> row) & 1ull) ? (int64_t)(lane_u(idv, row) - A.res_lo) : 0;
                x[i] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(A.w + rr * A.ld_w + colc));
            }
        }
        float part[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int row = c * CH + i;
            const bool is_res = ((res_mask >> row) & 1ull) != 0;                  // uniform
            const float f = lane_f(kf, row), b = lane_f(kb, row);
            const bool seen_f = (hf_mask & ((2ull << row) - 1ull)) != 0;          // a run head at or before the row
            const bool seen_b = (hb_mask >> row) != 0;                            // ... at or after it, seen from the right
            float P[VEC], Z[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float Fj = f * Fin[e], Rj = b * Rin[e];
                P[e] = Fj + Rj;
                Z[e] = (seen_b ? Rj : Gin[e]) - (seen_f ? Fj : Ein[e]);
            }
            if (sources) {
#pragma unroll
                for (int q = 0; q < NS; ++q) {
                    const float a = lane_f(ws[q], row), z = lane_f(wz[q], row);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) { P[e] += a * vs[q][e]; Z[e] += z * vs[q][e]; }
                }
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e) { P[e] = taint(P[e], poison); Z[e] = taint(Z[e], poison); }
            if (is_res && col_ok) {
                const int64_t rr = (int64_t)(lane_u(idv, row) - A.res_lo);
                // the result matrix is written once and not read again by this call: streaming stores
                if (A.out_p)
                    __builtin_nontemporal_store((v4f){P[0], P[1], P[2], P[3]}, reinterpret_cast<v4f*>(A.out_p + rr * A.ld_p + col0));
                if (STRICT && A.out_z) store_vec<VEC>(A.out_z + rr * A.ld_z + col0, Z);
            }
            part[i] = 0.0f;
            if (want_red && is_res && col_ok) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) part[i] += x[i][e] * Z[e];
            }
        }
        if (want_red) {
            // eight row sums over the 64 lanes: three butterfly steps leave lane l with the sum of row
            // (l & 7) over its group of eight lanes, three more add the groups up
            float h4[4], h2[2];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool up = (lane & 4) != 0;
                const float keep = up ? part[j + 4] : part[j], send = up ? part[j] : part[j + 4];
                h4[j] = keep + __shfl_xor(send, 4);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bool up = (lane & 2) != 0;
                const float keep = up ? h4[j + 2] : h4[j], send = up ? h4[j] : h4[j + 2];
                h2[j] = keep + __shfl_xor(send, 2);
            }
            float sum;
            {
                const bool up = (lane & 1) != 0;
                const float keep = up ? h2[1] : h2[0], send = up ? h2[0] : h2[1];
                sum = keep + __shfl_xor(send, 1);
            }
            sum += __shfl_xor(sum, 8);
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            const int row = c * CH + (lane & 7);
            const uint32_t idr = __shfl(idv, row);
            if (lane < 8 && ((res_mask >> row) & 1ull)) {
                const int64_t rr = (int64_t)(idr - A.res_lo);
                if (A.slabs == 1) A.out_red[rr * A.ld_red] = sum;
                else A.red_partial[(int64_t)blockIdx.y * res_rows + rr] = sum;
            }
        }
    }
}

// Eight row sums over the 64 lanes of a wavefront (part[i]: this lane's share of row i): three butterfly steps leave lane l
// with the sum of row (l & 7) over its group of eight lanes, three more add the groups up.  Every lane returns the total of
// row (lane & 7).
__device__ __forceinline__ float row_sums8(const float* part, int lane)
{
    float h4[4], h2[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool up = (lane & 4) != 0;
        const float keep = up ? part[j + 4] : part[j], send = up ? part[j] : part[j + 4];
        h4[j] = keep + __shfl_xor(send, 4);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const bool up = (lane & 2) != 0;
        const float keep = up ? h4[j + 2] : h4[j], send = up ? h4[j] : h4[j + 2];
        h2[j] = keep + __shfl_xor(send, 2);
    }
    const bool up = (lane & 1) != 0;
    const float keep = up ? h2[1] : h2[0], send = up ? h2[0] : h2[1];
    float sum = keep + __shfl_xor(send, 1);
    sum += __shfl_xor(sum, 8);
    sum += __shfl_xor(sum, 16);
    sum += __shfl_xor(sum, 32);
    return sum;
}

// ---------------------------------------------------------------------------
// The streaming downsweep of the wide geometry for the phased backward (Sec. 3, "Phased Laplace kernels":
// cos(phi - psi) = cos phi cos psi + sin phi sin psi makes the phased product two plain ones on a doubled batch).
// The scan problem runs on [gy cos phi | gy sin phi]; a lane owns four columns of BOTH halves, so that per input row j
//   gx[j]   = cos(psi_j) GX_c[j] + sin(psi_j) GX_s[j]
//   gpsi[j] = sum_t x[j][t] (cos(psi_j) GX_s - sin(psi_j) GX_c)[j][t]
//   gb[j]   = sum_t x[j][t] cos(psi_j) Z_c[j][t] + sum_t x[j][t] sin(psi_j) Z_s[j][t]
// come out of one read of x and one write of gx: the doubled result matrix and the doubled copy of x are not touched.
// Same blocks, closed forms and direct terms as k_scan_down_sparse_wide; the products x cos(psi), x sin(psi) are rounded
// before they are used, as the split pass would have stored them.  One slab: a half has at most 256 columns.
// ---------------------------------------------------------------------------
template <bool STRICT>
__global__ void __launch_bounds__(kStreamWaves * 64)
k_scan_down_sparse_wide_phased(const ScanArgs A)
{
    constexpr int VEC = 4, ROWS = 64, CH = 8, NS = kFewRows;
    // the last kernel of a scan that looks at the list lengths: the next scan wants them at zero
    if (blockIdx.x == 0 && threadIdx.x < 2) A.counters[threadIdx.x] = 0u;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t blk = (int64_t)blockIdx.x * kStreamWaves + wave;
    if (blk >= A.blocks) return;
    const int flags = (int)A.blk_flags[blk];
    if (!(flags & kFlagRes) || ((flags & kFlagInj) && !(flags & kFlagFewInj))) return;
    const uint32_t poison = plan_poison(A.counters);
    const int64_t half = A.ph.half;
    const int64_t col0 = (int64_t)lane * VEC;
    const bool col_ok = col0 < half;
    const int64_t colc = col_ok ? col0 : 0;      // lanes past the last column read (and drop) columns 0..3

    WideMeta M;
    M.fetch(A, blk, lane);
    float Fin[2][VEC], Ein[2][VEC], Rin[2][VEC], Gin[2][VEC];
    load_block_carries<VEC, STRICT>(A, blk, col0, col_ok, Fin[0], Ein[0], Rin[0], Gin[0]);
    load_block_carries<VEC, STRICT>(A, blk, col0 + half, col_ok, Fin[1], Ein[1], Rin[1], Gin[1]);
    const uint32_t idv = M.live ? M.id : 0xFFFFFFFFu;
    const bool my_res = idv >= A.res_lo && idv < A.res_hi;
    const uint64_t res_mask = __ballot(my_res);
    const uint64_t hf_mask = __ballot(M.live && M.dl >= 0.0f), hb_mask = __ballot(M.live && M.dr >= 0.0f);
    const float kf = expf(-(M.p - M.p_before)), kb = expf(-(M.p_after - M.p));
    // lane l holds the cosine and sine of the phase of row l
    float cph = 1.0f, sph = 0.0f;
    if (my_res) sincosf(A.ph.psi[idv - A.res_lo], &sph, &cph);

    const bool sources = (flags & kFlagFewInj) != 0;       // uniform
    float vs[2][NS][VEC], ws[NS], wz[NS];
#pragma unroll
    for (int q = 0; q < NS; ++q) {
        ws[q] = wz[q] = 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) vs[0][q][e] = vs[1][q][e] = 0.0f;
    }
    if (sources) {
        uint64_t m = __ballot(idv >= A.inj_lo && idv < A.inj_hi);
#pragma unroll
        for (int q = 0; q < NS; ++q) {
            const bool have = m != 0;
            const int rs = have ? __ffsll((long long)m) - 1 : 0;
            m &= m - 1;
            const float pq = lane_f(M.p, rs);
            const uint32_t idq = lane_u(idv, rs);
            if (have && col_ok) {
                const float* row = A.inj + (int64_t)(idq - A.inj_lo) * A.ld_inj + col0;
                load_vec<VEC>(vs[0][q], row);
                load_vec<VEC>(vs[1][q], row + half);
            }
            ws[q] = have ? expf(-fabsf(M.p - pq)) : 0.0f;
            wz[q] = pq > M.p ? ws[q] : (pq < M.p ? -ws[q] : 0.0f);
        }
    }

    const bool want_x = A.ph.x != nullptr;
    const bool want_red = STRICT && A.out_red != nullptr && want_x;
    const bool want_gpsi = A.ph.gpsi != nullptr && want_x;
    const int64_t res_rows = (int64_t)A.res_hi - (int64_t)A.res_lo;
#pragma unroll
    for (int c = 0; c < ROWS / CH; ++c) {
        if (!((res_mask >> (c * CH)) & 0xFFull)) continue;          // uniform: no result row among these eight
        v4f x[CH];
        if (want_x) {       // (no branch around a load: rows that are not wanted read row 0)
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int row = c * CH + i;
                const int64_t rr = ((res_mask >> row) & 1ull) ? (int64_t)(lane_u(idv, row) - A.res_lo) : 0;
                x[i] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(A.ph.x + rr * A.ph.ldx + colc));
            }
        }
        float part_c[CH], part_s[CH], part_p[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int row = c * CH + i;
            const bool is_res = ((res_mask >> row) & 1ull) != 0;                  // uniform
            const float f = lane_f(kf, row), b = lane_f(kb, row);
            const float cr = lane_f(cph, row), sr = lane_f(sph, row);
            const bool seen_f = (hf_mask & ((2ull << row) - 1ull)) != 0;          // a run head at or before the row
            const bool seen_b = (hb_mask >> row) != 0;                            // ... at or after it, seen from the right
            float P[2][VEC], Z[2][VEC];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float Fj = f * Fin[h][e], Rj = b * Rin[h][e];
                    P[h][e] = Fj + Rj;
                    Z[h][e] = (seen_b ? Rj : Gin[h][e]) - (seen_f ? Fj : Ein[h][e]);
                }
            }
            if (sources) {
#pragma unroll
                for (int q = 0; q < NS; ++q) {
                    const float a = lane_f(ws[q], row), z = lane_f(wz[q], row);
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) { P[h][e] += a * vs[h][q][e]; Z[h][e] += z * vs[h][q][e]; }
                    }
                }
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) { P[h][e] = taint(P[h][e], poison); Z[h][e] = taint(Z[h][e], poison); }
            }
            part_c[i] = part_s[i] = part_p[i] = 0.0f;
            if (is_res && col_ok) {
                const int64_t rr = (int64_t)(lane_u(idv, row) - A.res_lo);
                if (A.ph.gx) {
                    v4f o;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) o[e] = cr * P[0][e] + sr * P[1][e];
                    __builtin_nontemporal_store(o, reinterpret_cast<v4f*>(A.ph.gx + rr * A.ph.ldgx + col0));
                }
                if (want_x) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const float xc = x[i][e] * cr, xs = x[i][e] * sr;      // the two halves of the modulated row
                        if (want_red) { part_c[i] += xc * Z[0][e]; part_s[i] += xs * Z[1][e]; }
                        part_p[i] += x[i][e] * (cr * P[1][e] - sr * P[0][e]);
                    }
                }
            }
        }
        const int row = c * CH + (lane & 7);
        const uint32_t idr = __shfl(idv, row);
        const bool writer = lane < 8 && ((res_mask >> row) & 1ull);
        const int64_t rr = (int64_t)(idr - A.res_lo);
        if (want_red) {
            const float sum_c = row_sums8(part_c, lane), sum_s = row_sums8(part_s, lane);
            if (writer) {
                if (A.slabs == 1) A.out_red[rr * A.ld_red] = sum_c + sum_s;
                else { A.red_partial[rr] = sum_c; A.red_partial[res_rows + rr] = sum_s; }     // two slabs: summed with the others'
            }
        }
        if (want_gpsi) {
            const float sum_p = row_sums8(part_p, lane);
            if (writer) A.ph.gpsi[rr] = sum_p;
        }
    }
}

// The result rows of the blocks that the kernel above does not own (blocks with more than a few injected rows: the other
// downsweeps wrote both halves of their rows to out_p): the same merge, one wavefront per eight rows of a block, row by row.
__global__ void __launch_bounds__(kStreamWaves * 64)
k_phase_merge_blocks(const ScanArgs A)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t part = (int64_t)blockIdx.x * kStreamWaves + wave;       // eight rows of a block per wavefront
    const int64_t blk = part >> 3;
    if (blk >= A.blocks) return;
    const int flags = (int)A.blk_flags[blk];
    if (!(flags & kFlagRes) || !(flags & kFlagInj) || (flags & kFlagFewInj)) return;
    const int64_t j = blk * 64 + lane;
    const uint32_t idv = j < A.N ? A.ids[j] : 0xFFFFFFFFu;
    uint64_t m = __ballot(idv >= A.res_lo && idv < A.res_hi) & (0xFFull << (8 * (int)(part & 7)));
    const int64_t half = A.ph.half;
    while (m) {
        const int row = __ffsll((long long)m) - 1;
        m &= m - 1;
        const int64_t r = (int64_t)(lane_u(idv, row) - A.res_lo);
        float s, c;
        sincosf(A.ph.psi[r], &s, &c);
        const float* in = A.out_p + r * A.ld_p;
        float acc = 0.0f;
        for (int64_t t = lane; t < half; t += 64) {
            const float u = in[t], v = in[half + t];
            if (A.ph.gx) A.ph.gx[r * A.ph.ldgx + t] = c * u + s * v;
            if (A.ph.gpsi && A.ph.x) acc += A.ph.x[r * A.ph.ldx + t] * (c * v - s * u);
        }
        if (A.ph.gpsi && A.ph.x) {
#pragma unroll
            for (int k = 32; k >= 1; k >>= 1) acc += __shfl_xor(acc, k);
            if (lane == 0) A.ph.gpsi[r] = acc;
        }
    }
}

// ---------------------------------------------------------------------------
// Batch 1, everything in sorted order (the routes through partition passes): the injected values
// arrive as a plain array over the sorted rows (zero where nothing is injected) and the weights of
// the row reduction as another (zero off the result rows); the outputs of the result rows leave as
// records (id - first result id, first output[, second output]) of the first partition level on their
// way home (permute_tile.h), so they are never written in sorted order and read again.  Every block is
// treated as holding injected and result rows, the reduce does not look at the ids at all, and the
// kernels read each array in 16-byte pieces.  Same summaries, carries and walks as k_scan_reduce / k_scan_down at one column per
// lane: 64 row-lanes per wavefront, 16 rows per row-lane, 8 wavefronts per block of 8192 rows.
// ---------------------------------------------------------------------------
// Both kernels keep the geometry of the generic ones (8 wavefronts, 16 rows per row-lane, blocks of 8192 rows).  The
// downsweep holds its rows' results in registers until they leave as records and has to stay within 128 registers for
// two workgroups to share a compute unit (one of them loads or stores while the other scans: with a single workgroup of
// 16 wavefronts and 8 rows per row-lane, which needs no care about registers, the kernel's phases simply add up — 15 ms
// instead of 9.5 at 2^31 rows): the records' destinations wait in LDS, the rows' slots are packed two to a register,
// and the variant with a row reduction asks for its rows only after the reservation.
constexpr int kSeqItems = kItemsVec1;
constexpr int kSeqDownItems = 16, kSeqDownWaves = 8, kSeqDownThreads = kSeqDownWaves * 64;
static_assert(kSeqDownItems * kSeqDownThreads == kSeqItems * kScanThreads, "both kernels own blocks of the same rows");

// exp(-x) by the hardware's base-2 exponential after one multiplication.  Only for decays that multiply a carry over a
// span of rows inside a block: the relative error is about |x| * 6e-8 (the product x * log2(e) is rounded) plus one
// unit in the last place, i.e. at most 0.37 * 6e-8 of the carry in absolute terms, whatever x; the per-row decays of
// the plan and every decay that enters a summary of the spine stay on the accurate exponential.
__device__ __forceinline__ float decay_fast(float x) { return __builtin_amdgcn_exp2f(x * -1.44269504088896340736f); }
// The sorted anchors at a position that is a multiple of 8 rows (or the end of the sequence): (pk[pos], pk[pos + 1]),
// from the packed copy of every eighth pair where the plan has one.  A lane that owns 8 or 16 consecutive rows would
// otherwise touch every 32-byte sector of pk for two values, and the kernel would fetch the whole array.
__device__ __forceinline__ float2 seq_anchor(const ScanArgs& A, int64_t pos)
{
    pos = pos < A.N ? pos : A.N;
    if (A.pk8 != nullptr && (pos & 7) == 0) return A.pk8[pos >> 3];
    return make_float2(A.pk[pos], A.pk[pos + 1]);
}
// Decays and head flags over the rows between two such positions lo <= hi (clamped to the sequence like seq_anchor's),
// forward sense (.x: from the anchor before the rows to their last) and backward sense (.y).
struct SeqSpan {
    float df, db;
    bool hf, hb;
};
__device__ __forceinline__ SeqSpan seq_span(const ScanArgs& A, int64_t lo, const float2& plo, int64_t hi, const float2& phi)
{
    lo = lo < A.N ? lo : A.N;
    hi = hi < A.N ? hi : A.N;
    SeqSpan r;
    const bool any = hi > lo;
    const float f = decay_fast(phi.x - plo.x), b = decay_fast(phi.y - plo.y);
    r.df = any ? f : 1.0f;
    r.db = any ? b : 1.0f;
    r.hf = any && phi.x != plo.x;
    r.hb = any && phi.y != plo.y;
    return r;
}

// Inclusive scan of summaries over the 64 lanes of a wavefront (one column, one row-lane per lane), forward (lane 0
// first) or backward (lane 63 first): four steps inside each row of 16 lanes with data-parallel-primitive moves (a lane
// whose source lies outside its row receives the identity, so no select is needed), then the three row totals reach
// every lane through the scalar unit.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float identity, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL, bool STRICT>
__device__ __forceinline__ Seg<1, STRICT> seg_dpp(const Seg<1, STRICT>& s)
{
    Seg<1, STRICT> r = seg_identity<1, STRICT>();
    r.D = dpp_move<CTRL>(1.0f, s.D);
    r.S[0] = dpp_move<CTRL>(0.0f, s.S[0]);
    if (STRICT) {
        r.Q[0] = dpp_move<CTRL>(0.0f, s.Q[0]);
        r.H = __builtin_amdgcn_update_dpp(0, s.H, CTRL, 0xF, 0xF, false);
    }
    return r;
}
template <bool STRICT>
__device__ __forceinline__ Seg<1, STRICT> seg_of_lane(const Seg<1, STRICT>& s, int l)     // l: uniform
{
    Seg<1, STRICT> r = seg_identity<1, STRICT>();
    r.D = lane_f(s.D, l);
    r.S[0] = lane_f(s.S[0], l);
    if (STRICT) { r.Q[0] = lane_f(s.Q[0], l); r.H = __builtin_amdgcn_readlane(s.H, l); }
    return r;
}
template <bool FWD, bool STRICT>
__device__ __forceinline__ Seg<1, STRICT> row_scan16(Seg<1, STRICT> s)
{
    // row_shr:n = 0x110 + n (lane i takes lane i - n of its row), row_shl:n = 0x100 + n
    s = seg_compose<1, STRICT>(seg_dpp<FWD ? 0x111 : 0x101, STRICT>(s), s);
    s = seg_compose<1, STRICT>(seg_dpp<FWD ? 0x112 : 0x102, STRICT>(s), s);
    s = seg_compose<1, STRICT>(seg_dpp<FWD ? 0x114 : 0x104, STRICT>(s), s);
    s = seg_compose<1, STRICT>(seg_dpp<FWD ? 0x118 : 0x108, STRICT>(s), s);
    return s;
}
template <bool FWD, bool STRICT>
__device__ __forceinline__ Seg<1, STRICT> wave_scan64(Seg<1, STRICT> s, int lane)
{
    s = row_scan16<FWD, STRICT>(s);
    // totals of the first three rows in scan order sit in the row's last lane in scan order
    const Seg<1, STRICT> t0 = seg_of_lane<STRICT>(s, FWD ? 15 : 48), t1 = seg_of_lane<STRICT>(s, FWD ? 31 : 32),
                         t2 = seg_of_lane<STRICT>(s, FWD ? 47 : 16);
    const Seg<1, STRICT> p2 = seg_compose<1, STRICT>(t0, t1), p3 = seg_compose<1, STRICT>(p2, t2);
    const int before = FWD ? lane >> 4 : 3 - (lane >> 4);       // rows ahead of this lane's in scan order
    Seg<1, STRICT> pre = seg_identity<1, STRICT>();
    pre.D = before == 1 ? t0.D : before == 2 ? p2.D : before == 3 ? p3.D : 1.0f;
    pre.S[0] = before == 1 ? t0.S[0] : before == 2 ? p2.S[0] : before == 3 ? p3.S[0] : 0.0f;
    if (STRICT) {
        pre.Q[0] = before == 1 ? t0.Q[0] : before == 2 ? p2.Q[0] : before == 3 ? p3.Q[0] : 0.0f;
        pre.H = before == 1 ? t0.H : before == 2 ? p2.H : before == 3 ? p3.H : 0;
    }
    return seg_compose<1, STRICT>(pre, s);
}

// The same scans with the decay of every composite summary re-taken from the anchors (equal spans have equal decays with
// equal rounding errors; a chain of them, as on a regular grid, multiplies the error by its length).  A lane brings the
// anchor its span starts from in scan order (pb) and the one it ends at (pe): forward the sorted anchor before its first row
// and at its last row, backward the anchor after its last row and at its first.  The decay over the lanes [lo .. lane] of a
// composite is then exp(-|pe(lane) - pb(lo)|), one fast exponential.
template <bool FWD>
__device__ __forceinline__ float anchored_decay(float pb_of_start, float pe_of_end)
{
    // (lanes past the end of the sequence bring the +inf sentinel at both ends: an empty span, decay 1)
    return pb_of_start == pe_of_end ? 1.0f : decay_fast(FWD ? pe_of_end - pb_of_start : pb_of_start - pe_of_end);
}
template <bool FWD, bool STRICT, int STEP>      // one step of the scan inside a row of 16 lanes: partners 2 * STEP - 1 .. STEP lanes back
__device__ __forceinline__ void row_step_anchored(Seg<1, STRICT>& s, float pb, float pe, float pb_row)
{
    constexpr int kBack = 2 * STEP - 1;         // after this step a lane's summary starts this many lanes back (or at the row's start)
    s = seg_compose<1, STRICT>(seg_dpp<(FWD ? 0x110 : 0x100) + STEP, STRICT>(s), s);
    const float pb_start = dpp_move<(FWD ? 0x110 : 0x100) + kBack>(pb_row, pb);
    s.D = anchored_decay<FWD>(pb_start, pe);
    if (STRICT) s.C = s.D;
}
template <bool FWD, bool STRICT>
__device__ __forceinline__ Seg<1, STRICT> wave_scan64_anchored(Seg<1, STRICT> s, float pb, float pe, int lane)
{
    const float pb_row = __shfl(pb, FWD ? lane & ~15 : lane | 15);     // where this lane's row of 16 starts in scan order
    row_step_anchored<FWD, STRICT, 1>(s, pb, pe, pb_row);
    row_step_anchored<FWD, STRICT, 2>(s, pb, pe, pb_row);
    row_step_anchored<FWD, STRICT, 4>(s, pb, pe, pb_row);
    row_step_anchored<FWD, STRICT, 8>(s, pb, pe, pb_row);
    // totals of the first three rows in scan order sit in the row's last lane in scan order
    const int l0 = FWD ? 15 : 48, l1 = FWD ? 31 : 32, l2 = FWD ? 47 : 16, first = FWD ? 0 : 63;
    const Seg<1, STRICT> t0 = seg_of_lane<STRICT>(s, l0), t1 = seg_of_lane<STRICT>(s, l1), t2 = seg_of_lane<STRICT>(s, l2);
    const float pb_first = lane_f(pb, first);
    Seg<1, STRICT> p2 = seg_compose<1, STRICT>(t0, t1);
    p2.D = anchored_decay<FWD>(pb_first, lane_f(pe, l1)); if (STRICT) p2.C = p2.D;
    Seg<1, STRICT> p3 = seg_compose<1, STRICT>(p2, t2);
    p3.D = anchored_decay<FWD>(pb_first, lane_f(pe, l2)); if (STRICT) p3.C = p3.D;
    const int before = FWD ? lane >> 4 : 3 - (lane >> 4);       // rows ahead of this lane's in scan order
    Seg<1, STRICT> pre = seg_identity<1, STRICT>();
    pre.D = before == 1 ? t0.D : before == 2 ? p2.D : before == 3 ? p3.D : 1.0f;
    pre.S[0] = before == 1 ? t0.S[0] : before == 2 ? p2.S[0] : before == 3 ? p3.S[0] : 0.0f;
    if (STRICT) {
        pre.Q[0] = before == 1 ? t0.Q[0] : before == 2 ? p2.Q[0] : before == 3 ? p3.Q[0] : 0.0f;
        pre.H = before == 1 ? t0.H : before == 2 ? p2.H : before == 3 ? p3.H : 0;
    }
    Seg<1, STRICT> r = seg_compose<1, STRICT>(pre, s);
    r.D = anchored_decay<FWD>(pb_first, pe); if (STRICT) r.C = r.D;
    return r;
}

template <int ITEMS>
struct SeqRows {
    static_assert(ITEMS % 4 == 0 && ITEMS <= 32, "a row-lane's rows are read in 16-byte pieces; one bit per row");
    float dh[ITEMS + 1];          // dh[i]: decay into row i from the left; dh[i + 1]: from the right
    uint32_t live;                // bit i: row i lies inside the sequence
    __device__ __forceinline__ bool alive(int i) const { return (live >> i) & 1u; }
};

// dst[0..ITEMS) = src[row0..row0+ITEMS), zero past the end of the sequence
template <int ITEMS>
__device__ __forceinline__ void seq_load(const float* __restrict__ src, int64_t row0, int64_t N, float* dst)
{
    if (row0 + ITEMS <= N) {
#pragma unroll
        for (int q = 0; q < ITEMS / 4; ++q) {
            const float4 t = reinterpret_cast<const float4*>(src + row0)[q];
            dst[4 * q] = t.x; dst[4 * q + 1] = t.y; dst[4 * q + 2] = t.z; dst[4 * q + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int64_t j = row0 + i;
            const float t = src[j < N ? j : N - 1];
            dst[i] = j < N ? t : 0.0f;
        }
    }
}

template <int ITEMS>
__device__ __forceinline__ void seq_meta(const ScanArgs& A, int64_t row0, SeqRows<ITEMS>& T)
{
    if (row0 + ITEMS <= A.N) {          // dh has N + 1 entries
#pragma unroll
        for (int q = 0; q < ITEMS / 4; ++q) {
            const float4 t = reinterpret_cast<const float4*>(A.dh + row0)[q];
            T.dh[4 * q] = t.x; T.dh[4 * q + 1] = t.y; T.dh[4 * q + 2] = t.z; T.dh[4 * q + 3] = t.w;
        }
        T.dh[ITEMS] = A.dh[row0 + ITEMS];
        T.live = (1u << ITEMS) - 1u;
    } else {
#pragma unroll
        for (int i = 0; i <= ITEMS; ++i) {
            const int64_t j = row0 + i;
            const float d = A.dh[j <= A.N ? j : A.N];
            T.dh[i] = j <= A.N ? d : -1.0f;
        }
        const int64_t left = A.N - row0;
        T.live = left <= 0 ? 0u : (left >= ITEMS ? (1u << ITEMS) - 1u : (1u << left) - 1u);
    }
}

// LDS exchange of the wavefronts' summaries of one block (one column): [direction][wavefront]
template <int WAVES>
struct SeqSegs {
    float D[2][WAVES], C[2][WAVES], S[2][WAVES], Q[2][WAVES];
    int H[2][WAVES];
    float preF[2][WAVES], preE[2][WAVES];     // state a wavefront starts from when its block starts from zero, per direction
    template <bool STRICT>
    __device__ __forceinline__ void put(int dir, int wave, const Seg<1, STRICT>& s)
    {
        D[dir][wave] = s.D; S[dir][wave] = s.S[0];
        if (STRICT) { C[dir][wave] = s.C; H[dir][wave] = s.H; Q[dir][wave] = s.Q[0]; }
    }
    template <bool STRICT>
    __device__ __forceinline__ Seg<1, STRICT> get(int dir, int wave) const
    {
        Seg<1, STRICT> s;
        s.D = D[dir][wave]; s.S[0] = S[dir][wave];
        s.C = STRICT ? C[dir][wave] : 0.0f; s.H = STRICT ? H[dir][wave] : 0; s.Q[0] = STRICT ? Q[dir][wave] : 0.0f;
        return s;
    }
};

template <bool STRICT>
__global__ void __launch_bounds__(kScanThreads)
k_seq_reduce(const ScanArgs A)
{
    constexpr int ITEMS = kSeqItems;
    __shared__ WaveSegs<1> W;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t tile = blockIdx.x;
    const int64_t tile_base = tile * (kScanWaves * 64 * ITEMS);
    const int64_t wave_row0 = tile_base + (int64_t)wave * 64 * ITEMS;
    const int64_t row0 = wave_row0 + (int64_t)lane * ITEMS;
    // from this row-lane's last row to the tile's last, and from its first row back to the tile's first: one exponential of
    // an anchor difference each (the tile's summary is the weighted sum of the row-lanes' own: see k_scan_reduce)
    const int64_t tile_end = tile_base + (int64_t)kScanWaves * 64 * ITEMS;
    const float2 p_lane0 = seq_anchor(A, row0), p_lane1 = seq_anchor(A, row0 + ITEMS);
    const float2 p_tile0 = seq_anchor(A, tile_base), p_tile1 = seq_anchor(A, tile_end);
    const float wf = seq_span(A, row0 + ITEMS, p_lane1, tile_end, p_tile1).df;
    const float wb = seq_span(A, tile_base, p_tile0, row0, p_lane0).db;
    SeqRows<ITEMS> T;
    seq_meta<ITEMS>(A, row0, T);
    float v[ITEMS][1];
    {
        float t[ITEMS];
        seq_load<ITEMS>(A.stage, row0, A.N, t);
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) v[i][0] = t[i];
    }
    Seg<1, STRICT> f = seg_identity<1, STRICT>(), b = seg_identity<1, STRICT>();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) seg_push<1, STRICT>(f, T.alive(i) && T.dh[i] >= 0.0f, T.dh[i], v[i]);
#pragma unroll
    for (int i = ITEMS - 1; i >= 0; --i) seg_push<1, STRICT>(b, T.alive(i) && T.dh[i + 1] >= 0.0f, T.dh[i + 1], v[i]);
    {
        const uint64_t hf = STRICT ? __ballot(f.H != 0) : 0ull, hb = STRICT ? __ballot(b.H != 0) : 0ull;
        const int last_f = hf ? 63 - __clzll((long long)hf) : -1;          // last row-lane with a run head, from the left
        const int first_b = hb ? __ffsll((long long)hb) - 1 : 64;          // first one: the last seen from the right
        float sf = wf * f.S[0], sb = wb * b.S[0];
        float qf = lane < last_f ? sf : (lane == last_f ? f.Q[0] : 0.0f);
        float qb = lane > first_b ? sb : (lane == first_b ? b.Q[0] : 0.0f);
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            sf += __shfl_xor(sf, m); sb += __shfl_xor(sb, m);
            if (STRICT) { qf += __shfl_xor(qf, m); qb += __shfl_xor(qb, m); }
        }
        if (lane == 0) {
            W.S[0][wave][0] = sf; W.S[1][wave][0] = sb;
            if (STRICT) { W.Q[0][wave][0] = qf; W.Q[1][wave][0] = qb; W.H[0][wave] = hf != 0; W.H[1][wave] = hb != 0; }
        }
    }
    __syncthreads();
    if (tid == 0) {
        Seg<1, STRICT> tf = seg_identity<1, STRICT>(), tb = seg_identity<1, STRICT>();
#pragma unroll 1
        for (int w = 0; w < kScanWaves; ++w) {
            const bool h = STRICT && W.H[0][w] != 0;
            if (h) tf.Q[0] = tf.S[0] + W.Q[0][w][0];       // everything before this wavefront, and its own share
            tf.S[0] += W.S[0][w][0];
            tf.H |= h ? 1 : 0;
        }
#pragma unroll 1
        for (int w = kScanWaves - 1; w >= 0; --w) {
            const bool h = STRICT && W.H[1][w] != 0;
            if (h) tb.Q[0] = tb.S[0] + W.Q[1][w][0];
            tb.S[0] += W.S[1][w][0];
            tb.H |= h ? 1 : 0;
        }
        tf.D = tf.C = span_decay_f(A, tile_base, A.tile_rows);
        tb.D = tb.C = span_decay_b(A, tile_base, A.tile_rows);
        const float flags = (float)(kFlagInj | kFlagRes);
        store_level_seg<1, STRICT>(A.l1, 0, tile, A.bpad, 0, true, true, tf, flags);
        store_level_seg<1, STRICT>(A.l1, 1, tile, A.bpad, 0, true, true, tb, flags);
    }
}

// RED: the second output of a row is w * Z (w = A.wstage, sorted order), else Z itself (STRICT) or nothing.
// NV: values per record that leaves (2: both outputs; 1: A.emit_first says which).
template <bool STRICT, bool RED, int NV>
__global__ void __launch_bounds__(kSeqDownThreads, 4)
k_seq_down(const ScanArgs A)
{
    constexpr int ITEMS = kSeqDownItems, WAVES = kSeqDownWaves, THREADS = kSeqDownThreads;
    // One LDS buffer, used three times: the exchange of wavefront summaries, the strict forward values per row,
    // and at the end the records of the block on their way out.
    constexpr size_t kSmem = sizeof(uint2) * ITEMS * THREADS;
    static_assert(kSmem >= sizeof(SeqSegs<WAVES>) && kSmem >= sizeof(float) * ITEMS * THREADS, "the records need the most room");
    __shared__ __align__(16) unsigned char smem[kSmem];
    __shared__ PartShared<THREADS> S;
    SeqSegs<WAVES>& W = *reinterpret_cast<SeqSegs<WAVES>*>(smem);
    float* const ef = reinterpret_cast<float*>(smem) + threadIdx.x;        // row i at ef[i * THREADS]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t tile = blockIdx.x;
    const uint32_t poison = plan_poison(A.counters);
    const int64_t tile_base = tile * (int64_t)(THREADS * ITEMS);
    const int64_t wave_row0 = tile_base + (int64_t)wave * 64 * ITEMS;
    const int64_t row0 = wave_row0 + (int64_t)lane * ITEMS;
    const int64_t rows_after = row0 + ITEMS, tile_end = tile_base + A.tile_rows;
    const float2 p_lane0 = seq_anchor(A, row0), p_lane1 = seq_anchor(A, rows_after);
    const float2 p_wave0 = seq_anchor(A, wave_row0), p_wave1 = seq_anchor(A, wave_row0 + 64 * ITEMS);
    const float2 p_tile0 = seq_anchor(A, tile_base), p_tile1 = seq_anchor(A, tile_end);
    const SeqSpan lane_span = seq_span(A, row0, p_lane0, rows_after, p_lane1);
    const SeqSpan wave_span = seq_span(A, wave_row0, p_wave0, wave_row0 + 64 * ITEMS, p_wave1);
    const SeqSpan ahead = seq_span(A, tile_base, p_tile0, row0, p_lane0);          // the rows of the block before this row-lane's
    const SeqSpan behind = seq_span(A, rows_after, p_lane1, tile_end, p_tile1);    // and after them
    const float lane_df = lane_span.df, lane_db = lane_span.db, wave_df = wave_span.df, wave_db = wave_span.db;
    const float enter_df = ahead.df, enter_db = behind.db;
    const bool enter_hf = ahead.hf, enter_hb = behind.hb;

    // The rows' decays and values are asked for at once, before the ids, unless the weights of a row reduction have to fit
    // in the registers as well: then they follow the reservation, when the ids have left (asked for early, that variant
    // spills; the others lose 10 % when they ask late).
    SeqRows<ITEMS> T;
    float v[ITEMS][1], wt[RED ? ITEMS : 1];
    float Fc[1], Ec[1], Rc[1], Gc[1];
    auto load_rows = [&]() {
        seq_meta<ITEMS>(A, row0, T);
        float t[ITEMS];
        seq_load<ITEMS>(A.stage, row0, A.N, t);
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) v[i][0] = t[i];
        load_block_carries<1, STRICT>(A, tile, 0, true, Fc, Ec, Rc, Gc);
    };
    if (!RED) load_rows();
    // The result rows will leave as records of the first partition level (destination = id - first result id).  Where
    // they go depends on the ids alone, so the stretches are reserved now, and the answers travel during the walks.
    uint32_t dest[ITEMS];
    uint32_t ok = 0u;
    if (row0 + ITEMS <= A.N) {
#pragma unroll
        for (int q = 0; q < ITEMS / 4; ++q) {
            const uint4 t = reinterpret_cast<const uint4*>(A.ids + row0)[q];
            dest[4 * q] = t.x; dest[4 * q + 1] = t.y; dest[4 * q + 2] = t.z; dest[4 * q + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) dest[i] = A.ids[row0 + i < A.N ? row0 + i : A.N - 1];
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool res = row0 + i < A.N && dest[i] >= A.res_lo && dest[i] < A.res_hi;
        dest[i] -= A.res_lo;
        ok |= (res && (int64_t)dest[i] < A.emit.dest_count) ? 1u << i : 0u;
    }
    PartSplitTicket<ITEMS> K;
    uint32_t* const sd = reinterpret_cast<uint32_t*>(smem) + ITEMS * THREADS;    // upper half: the records' destinations
    partition_reserve_split<THREADS, ITEMS>(A.emit, 0, dest, ok, S, sd, K);
    if (RED) load_rows();
    Seg<1, STRICT> fe, be;
    {
        Seg<1, STRICT> f = seg_identity<1, STRICT>();
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) seg_push<1, STRICT>(f, T.alive(i) && T.dh[i] >= 0.0f, T.dh[i], v[i]);
        f.D = lane_df;
        f = wave_scan64_anchored<true, STRICT>(f, p_lane0.x, p_lane1.x, lane);
        if (lane == 63) { Seg<1, STRICT> tot = f; tot.D = wave_df; W.template put<STRICT>(0, wave, tot); }
        fe = seg_shfl<1, STRICT>(f, (lane - 1) & 63);
        if (lane == 0) fe = seg_identity<1, STRICT>();
    }
    {
        Seg<1, STRICT> b = seg_identity<1, STRICT>();
#pragma unroll
        for (int i = ITEMS - 1; i >= 0; --i) seg_push<1, STRICT>(b, T.alive(i) && T.dh[i + 1] >= 0.0f, T.dh[i + 1], v[i]);
        b.D = lane_db;
        b = wave_scan64_anchored<false, STRICT>(b, p_lane1.y, p_lane0.y, lane);
        if (lane == 0) { Seg<1, STRICT> tot = b; tot.D = wave_db; W.template put<STRICT>(1, wave, tot); }
        be = seg_shfl<1, STRICT>(b, (lane + 1) & 63);
        if (lane == 63) be = seg_identity<1, STRICT>();
    }
    __syncthreads();
    // the state each wavefront starts from when the block starts from zero: one wavefront scans the 16 wavefront summaries
    // of each direction (lane l holds the l-th in scan order) and leaves what precedes every wavefront
    static_assert(WAVES <= 16, "the wavefront summaries fit one row of 16 lanes");
    if (wave == 0) {
        const int l = lane & 15, lw = l < WAVES ? l : WAVES - 1;
        Seg<1, STRICT> sf = W.template get<STRICT>(0, lw), sb = W.template get<STRICT>(1, WAVES - 1 - lw);
        if (l >= WAVES) sf = sb = seg_identity<1, STRICT>();
        sf = row_scan16<true, STRICT>(sf);      // lane l: wavefronts 0 .. l
        sb = row_scan16<true, STRICT>(sb);      // lane l: wavefronts WAVES - 1 .. WAVES - 1 - l
        if (lane < WAVES - 1) {
            W.preF[0][lane + 1] = sf.S[0]; W.preE[0][lane + 1] = (STRICT && sf.H) ? sf.Q[0] : 0.0f;                      // before wavefront l + 1
            W.preF[1][WAVES - 2 - lane] = sb.S[0]; W.preE[1][WAVES - 2 - lane] = (STRICT && sb.H) ? sb.Q[0] : 0.0f;      // after wavefront 14 - l
        }
        if (lane == 0) { W.preF[0][0] = W.preE[0][0] = 0.0f; W.preF[1][WAVES - 1] = W.preE[1][WAVES - 1] = 0.0f; }
    }
    __syncthreads();
    float F[1] = {W.preF[0][wave]}, E[1] = {W.preE[0][wave]}, R[1] = {W.preF[1][wave]}, G[1] = {W.preE[1][wave]};
    seg_apply<1, STRICT>(fe, F, E);
    seg_apply<1, STRICT>(be, R, G);
    enter_state<1, STRICT>(F, E, Fc, Ec, enter_df, enter_hf);
    enter_state<1, STRICT>(R, G, Rc, Gc, enter_db, enter_hb);
    if (STRICT) __syncthreads();      // every wavefront is done with the summaries: the buffer now holds E per row
    if (RED) seq_load<ITEMS>(A.wstage, row0, A.N, wt);      // (late: the weights are needed by the last loop only)

    float Ff[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool h = T.alive(i) && T.dh[i] >= 0.0f;
        E[0] = h ? T.dh[i] * F[0] : E[0];
        F[0] = (h ? E[0] : F[0]) + v[i][0];
        Ff[i] = F[0];
        if (STRICT) ef[(size_t)i * THREADS] = E[0];
    }
    float second[STRICT ? ITEMS : 1];           // (the first outputs take the place of Ff)
#pragma unroll
    for (int i = ITEMS - 1; i >= 0; --i) {
        const bool h = T.alive(i) && T.dh[i + 1] >= 0.0f;
        const float Efi = STRICT ? ef[(size_t)i * THREADS] : 0.0f;
        G[0] = h ? T.dh[i + 1] * R[0] : G[0];
        R[0] = (h ? G[0] : R[0]) + v[i][0];
        Ff[i] = taint(Ff[i] + R[0] - v[i][0], poison);
        const float Z = taint(G[0] - Efi, poison);
        if (STRICT) second[i] = RED ? taint(wt[RED ? i : 0] * Z, poison) : Z;
    }
    if (STRICT && NV == 1 && !A.emit_first) {      // uniform: the second output is the one that travels
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) Ff[i] = second[i];
    }
    partition_place_split<THREADS, ITEMS, NV>(A.emit, 0, ok, Ff, STRICT ? second : Ff, S, sd, reinterpret_cast<float*>(smem), K);
}

__global__ void __launch_bounds__(256)
k_sum_slabs(const float* __restrict__ partial, int64_t rows, int slabs, float* __restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < rows; i += stride) {
        float s = 0.0f;
        for (int k = 0; k < slabs; ++k) s += partial[(int64_t)k * rows + i];
        out[i] = s;
    }
}

// out[r] = sum_t u[r, t] * v[r, t]: one wavefront per row, fixed summation order; blockIdx.y counts operators,
// whose matrices lie op_u / op_v / op_out elements apart
__global__ void __launch_bounds__(256)
k_rowdot(const float* __restrict__ u, int64_t ldu, int64_t op_u, const float* __restrict__ v, int64_t ldv, int64_t op_v,
         int64_t rows, int64_t batch, float* __restrict__ out, int64_t op_out)
{
    u += (int64_t)blockIdx.y * op_u; v += (int64_t)blockIdx.y * op_v; out += (int64_t)blockIdx.y * op_out;
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t r = wave; r < rows; r += nwaves) {
        float s = 0.0f;
        for (int64_t t = lane; t < batch; t += 64) s += u[r * ldu + t] * v[r * ldv + t];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m);
        if (lane == 0) out[r] = s;
    }
}

// the same for a narrow batch: one thread per row
__global__ void __launch_bounds__(256)
k_rowdot_narrow(const float* __restrict__ u, int64_t ldu, int64_t op_u, const float* __restrict__ v, int64_t ldv, int64_t op_v,
                int64_t rows, int64_t batch, float* __restrict__ out, int64_t op_out)
{
    u += (int64_t)blockIdx.y * op_u; v += (int64_t)blockIdx.y * op_v; out += (int64_t)blockIdx.y * op_out;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    // rows of 4 or 8 floats that start on 16-byte boundaries are read with 128-bit loads (same summation order)
    const bool v4 = batch % 4 == 0 && ldu % 4 == 0 && ldv % 4 == 0 &&
                    ((reinterpret_cast<uintptr_t>(u) | reinterpret_cast<uintptr_t>(v)) & 15u) == 0;
    // two plain vectors (batch 1, contiguous): four rows per lane and load
    const bool vec1 = batch == 1 && ldu == 1 && ldv == 1 &&
                      ((reinterpret_cast<uintptr_t>(u) | reinterpret_cast<uintptr_t>(v) | reinterpret_cast<uintptr_t>(out)) & 15u) == 0;
    if (vec1) {
        const int64_t quads = rows >> 2;
        for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += stride) {
            const float4 x = reinterpret_cast<const float4*>(u)[q];
            const float4 y = reinterpret_cast<const float4*>(v)[q];
            reinterpret_cast<float4*>(out)[q] = make_float4(x.x * y.x, x.y * y.y, x.z * y.z, x.w * y.w);
        }
        const int64_t r = 4 * quads + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;      // the last rows
        if (r < rows) out[r] = u[r] * v[r];
        return;
    }
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += stride) {
        float s = 0.0f;
        if (v4) {
            for (int64_t t = 0; t < batch; t += 4) {
                const float4 x = *reinterpret_cast<const float4*>(u + r * ldu + t);
                const float4 y = *reinterpret_cast<const float4*>(v + r * ldv + t);
                s += x.x * y.x; s += x.y * y.y; s += x.z * y.z; s += x.w * y.w;
            }
        } else {
            for (int64_t t = 0; t < batch; ++t) s += u[r * ldu + t] * v[r * ldv + t];
        }
        out[r] = s;
    }
}

// out[r] += sum_t u[r, t] * v[r, t]: one thread per row (narrow batches)
__global__ void __launch_bounds__(256)
k_add_rowdot(const float* __restrict__ u, int64_t ldu, const float* __restrict__ v, int64_t ldv, int64_t rows, int64_t batch,
             float* __restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += stride) {
        float s = 0.0f;
        for (int64_t t = 0; t < batch; ++t) s += u[r * ldu + t] * v[r * ldv + t];
        out[r] += s;
    }
}

// out[r] = sum_t (u1[r, t] * v1[r, t] + u2[r, t] * v2[r, t]): one wavefront per row, fixed summation order
__global__ void __launch_bounds__(256)
k_rowdot2(const float* __restrict__ u1, int64_t ldu1, const float* __restrict__ v1, int64_t ldv1,
          const float* __restrict__ u2, int64_t ldu2, const float* __restrict__ v2, int64_t ldv2,
          int64_t rows, int64_t batch, float* __restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t r = wave; r < rows; r += nwaves) {
        float s = 0.0f;
        for (int64_t t = lane; t < batch; t += 64) s += u1[r * ldu1 + t] * v1[r * ldv1 + t] + u2[r * ldu2 + t] * v2[r * ldv2 + t];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m);
        if (lane == 0) out[r] = s;
    }
}

int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <int VEC, bool STRICT>
void launch_all(const ScanArgs& A, const ScanGeom& g, const std::string& tag, bool two, hipStream_t st)
{
    const dim3 block(kScanThreads);                 // spine kernels
    const dim3 bblock((unsigned)g.waves * 64);      // block kernels
    const dim3 grid((unsigned)g.blocks, (unsigned)g.slabs);
    // heavy kernels driven by the lists visit at most one tile per injected row (reduce) and one block
    // per injected and per result row (downsweep)
    const int64_t inj_rows = (int64_t)A.inj_hi - A.inj_lo, res_rows = (int64_t)A.res_hi - A.res_lo;
    const int64_t rcap = inj_rows < g.tiles ? inj_rows : g.tiles;
    const int64_t both_rows = inj_rows < res_rows ? inj_rows : res_rows;
    const int64_t dcap = both_rows < g.blocks ? both_rows : g.blocks;
    const dim3 rgrid((unsigned)(A.reduce_from_list ? rcap : g.tiles), (unsigned)g.slabs);
    const dim3 dgrid((unsigned)(A.down_from_list ? dcap : g.blocks), (unsigned)g.slabs);
    // (the list lengths are zero here: the plan build cleared them, and the last kernel of every scan does again)
    if (A.reduce_from_list) {       // else the reduce sees every tile itself and lists the blocks for the downsweep
        const std::string fm = "scan_meta." + tag;
        LAPLEX_TIMED(fm.c_str(), st, hipLaunchKernelGGL(k_scan_meta, dim3((unsigned)((g.tiles + 3) / 4)), dim3(256), 0, st, A));
    }
    const dim3 cgrid((unsigned)g.chunks, (unsigned)g.slabs, 2);
    const dim3 tgrid((unsigned)A.batch, 2);
    const std::string fr = "scan_reduce." + tag, fs = "scan_spine." + tag, fd = "scan_down." + tag,
                      fp = "scan_down_sparse." + tag;
    if (VEC == 1 && A.inj_sorted && A.out_sorted) {     // batch 1, everything in sorted order: the ids are not looked at
        LAPLEX_TIMED(fr.c_str(), st, hipLaunchKernelGGL((k_seq_reduce<STRICT>), dim3((unsigned)g.tiles), block, 0, st, A));
        if (g.chunks > 1) {
            LAPLEX_TIMED(fs.c_str(), st, hipLaunchKernelGGL((k_spine_reduce<VEC, STRICT>), cgrid, block, 0, st, A));
            LAPLEX_TIMED(fs.c_str(), st, hipLaunchKernelGGL((k_spine_top<STRICT>), tgrid, dim3(kSpineThreads), 0, st, A.l2, A.bpad));
        }
        LAPLEX_TIMED(fs.c_str(), st, hipLaunchKernelGGL((k_spine_down<VEC, STRICT>), cgrid, block, 0, st, A));
        const dim3 tiles((unsigned)g.tiles), dblock(kSeqDownThreads);
        const bool red = STRICT && A.wstage != nullptr;
        if (!STRICT) LAPLEX_TIMED(fd.c_str(), st, hipLaunchKernelGGL((k_seq_down<false, false, 1>), tiles, dblock, 0, st, A));
        else if (red && two) LAPLEX_TIMED(fd.c_str(), st, hipLaunchKernelGGL((k_seq_down<STRICT, STRICT, 2>), tiles, dblock, 0, st, A));
        else if (red) LAPLEX_TIMED(fd.c_str(), st, hipLaunchKernelGGL((k_seq_down<STRICT, STRICT, 1>), tiles, dblock, 0, st, A));
        else if (two) LAPLEX_TIMED(fd.c_str(), st, hipLaunchKernelGGL((k_seq_down<STRICT, false, 2>), tiles, dblock, 0, st, A));
        else LAPLEX_TIMED(fd.c_str(), st, hipLaunchKernelGGL((k_seq_down<STRICT, false, 1>), tiles, dblock, 0, st, A));
        return;
    }
    if (VEC == 4 && g.sub_shift) {    // wide geometry: a workgroup per tile, a wavefront per block
        if (A.pin.half && A.pin.virtual_inj)      // phased: x read once for both halves
            LAPLEX_TIMED(fr.c_str(), st, hipLaunchKernelGGL((k_scan_reduce_wide<STRICT, 2>), dim3(rgrid.x), dim3(kWideWaves * 64), 0, st, A));
        else
            LAPLEX_TIMED(fr.c_str(), st, hipLaunchKernelGGL((k_scan_reduce_wide<STRICT, 1>), rgrid, dim3(kWideWaves * 64), 0, st, A));
    } else if (!A.stage) {            // one wavefront per tile
        const dim3 lgrid((rgrid.x + kLoneWaves - 1) / kLoneWaves, rgrid.y);
        LAPLEX_TIMED(fr.c_str(), st, hipLaunchKernelGGL((k_scan_reduce_wave<VEC, STRICT>), lgrid, dim3(kLoneWaves * 64), 0, st, A));
    } else {
        LAPLEX_TIMED(fr.c_str(), st, hipLaunchKernelGGL((k_scan_reduce<VEC, STRICT>), rgrid, bblock, 0, st, A));
    }
    if (g.chunks > 1) {     // one chunk: nothing to carry between chunks, the tiles' carries come from k_spine_down alone
        LAPLEX_TIMED(fs.c_str(), st, hipLaunchKernelGGL((k_spine_reduce<VEC, STRICT>), cgrid, block, 0, st, A));
        LAPLEX_TIMED(fs.c_str(), st, hipLaunchKernelGGL((k_spine_top<STRICT>), tgrid, dim3(kSpineThreads), 0, st, A.l2, A.bpad));
    }
    LAPLEX_TIMED(fs.c_str(), st, hipLaunchKernelGGL((k_spine_down<VEC, STRICT>), cgrid, block, 0, st, A));
    if (VEC == 4 && g.sub_shift && A.pin.half && A.pin.split_blocks) {     // phased: the doubled rows the downsweeps will read
        const std::string fx = "phase_split_blocks." + tag;
        LAPLEX_TIMED(fx.c_str(), st, hipLaunchKernelGGL(k_phase_split_blocks, dim3((unsigned)((8 * g.blocks + kStreamWaves - 1) / kStreamWaves)),
                                                        dim3(kStreamWaves * 64), 0, st, A));
    }
    if (VEC == 4 && A.few_res_ok) {
        const std::string ff = "scan_down_fewres." + tag;
        const dim3 fgrid((dgrid.x + kFewWaves - 1) / kFewWaves, dgrid.y);
        LAPLEX_TIMED(ff.c_str(), st, hipLaunchKernelGGL((k_scan_down_fewres<STRICT>), fgrid, dim3(kFewWaves * 64), 0, st, A));
    }
    {
        const bool red = STRICT && A.out_red != nullptr;
        auto go = [&](auto kernel) { LAPLEX_TIMED(fd.c_str(), st, hipLaunchKernelGGL(kernel, dgrid, bblock, 0, st, A)); };
        const bool zs = red && A.zs != nullptr;
        if (g.waves == kScanWaves) {
            if (zs) go(k_scan_down<VEC, STRICT, kScanWaves, STRICT, STRICT>);
            else if (red) go(k_scan_down<VEC, STRICT, kScanWaves, STRICT, false>);
            else go(k_scan_down<VEC, STRICT, kScanWaves, false, false>);
        } else {
            if (zs) go(k_scan_down<VEC, STRICT, kBlockWavesNarrow, STRICT, STRICT>);
            else if (red) go(k_scan_down<VEC, STRICT, kBlockWavesNarrow, STRICT, false>);
            else go(k_scan_down<VEC, STRICT, kBlockWavesNarrow, false, false>);
        }
    }
    if (VEC == 4 && g.sub_shift) {
        const dim3 sgrid((unsigned)((g.blocks + kStreamWaves - 1) / kStreamWaves), (unsigned)g.slabs);
        if (A.ph.half) {     // phased backward: one wavefront merges both halves of its block's rows; the other blocks' rows after it
            const dim3 pgrid(sgrid.x);
            LAPLEX_TIMED(fp.c_str(), st, hipLaunchKernelGGL((k_scan_down_sparse_wide_phased<STRICT>), pgrid, dim3(kStreamWaves * 64), 0, st, A));
            const std::string fm = "phase_merge_blocks." + tag;
            LAPLEX_TIMED(fm.c_str(), st, hipLaunchKernelGGL(k_phase_merge_blocks, dim3((unsigned)((8 * g.blocks + kStreamWaves - 1) / kStreamWaves)),
                                                            dim3(kStreamWaves * 64), 0, st, A));
        } else {
            LAPLEX_TIMED(fp.c_str(), st, hipLaunchKernelGGL((k_scan_down_sparse_wide<STRICT>), sgrid, dim3(kStreamWaves * 64), 0, st, A));
        }
    } else {
        LAPLEX_TIMED(fp.c_str(), st, hipLaunchKernelGGL((k_scan_down_sparse<VEC, STRICT>), grid, bblock, 0, st, A));
    }
}

}  // namespace

hipError_t launch_scan(const ScanProblem& p, const Layout& L, char* ws, hipStream_t st)
{
    const bool strict = p.out_z != nullptr || p.out_red != nullptr || p.emit_strict;
    // 128-bit lanes need every row start of every matrix touched to be 16-byte aligned
    bool v4 = p.batch % 4 == 0 && p.batch >= 4;
    v4 = v4 && aligned16(p.inj) && p.ld_inj % 4 == 0;
    if (p.out_p) v4 = v4 && aligned16(p.out_p) && p.ld_p % 4 == 0;
    if (p.out_z) v4 = v4 && aligned16(p.out_z) && (p.ld_z == 0 || p.ld_z % 4 == 0);
    if (p.out_red) v4 = v4 && aligned16(p.w) && p.ld_w % 4 == 0 && (!p.zs || aligned16(p.zs));
    const ScanGeom g = scan_geom(p.N, p.batch, v4 ? 4 : 1);

    ScanArgs A;
    A.ids = p.ids; A.dh = p.dh; A.pk = p.pk; A.pk8 = p.pk8; A.N = p.N;
    A.inj = p.inj; A.ld_inj = p.ld_inj; A.inj_lo = p.inj_lo; A.inj_hi = p.inj_hi;
    A.res_lo = p.res_lo; A.res_hi = p.res_hi;
    A.out_p = p.out_p; A.ld_p = p.ld_p; A.out_z = p.out_z; A.ld_z = p.ld_z ? p.ld_z : p.batch;
    A.out_red = p.out_red; A.ld_red = p.ld_red ? p.ld_red : 1; A.w = p.w; A.ld_w = p.ld_w; A.zs = p.zs;
    A.stage = p.stage; A.wstage = p.wstage;
    A.inj_sorted = p.inj_sorted ? 1 : 0; A.out_sorted = p.out_sorted ? 1 : 0;
    if (p.emit) A.emit = *p.emit;
    A.emit_first = p.emit_first ? 1 : 0;
    A.ph = PhaseFuse{};
    if (p.phase) {
        // one wavefront must span a whole half-row: wide geometry, at most 256 columns per half, two slabs at most
        if (!v4 || !g.sub_shift || !p.out_p || p.phase->half * 2 != p.batch || p.phase->half > 256 || g.slabs > 2) return hipErrorInvalidValue;
        A.ph = *p.phase;
    }
    A.pin = PhaseIn{};
    if (p.phase_in) {
        if (!v4 || !g.sub_shift || p.phase_in->half * 2 != p.batch || p.phase_in->half > 256 || g.slabs > 2) return hipErrorInvalidValue;
        A.pin = *p.phase_in;
    }
    A.batch = p.batch; A.bpad = L.bpad;
    {
        const bool z_pair = p.out_z && !p.out_red && p.out_z == p.out_p + 1 && p.ld_z == 2;
        const bool red_pair = p.out_red && !p.out_z && p.out_red == p.out_p + 1 && p.ld_red == 2;
        A.pair_out = p.batch == 1 && p.out_p && p.ld_p == 2 && (z_pair || red_pair) && (reinterpret_cast<uintptr_t>(p.out_p) & 7u) == 0;
    }
    A.bv = g.bv; A.bv_log2 = ilog2(g.bv); A.rv = g.rv; A.tile_rows = g.tile_rows; A.slabs = g.slabs;
    A.chunk_tiles = g.chunk_tiles; A.spine_items = g.spine_items;
    A.waves = g.waves;
    A.sub_shift = g.sub_shift; A.spine_rows = (int64_t)g.tile_rows << g.sub_shift; A.blocks = g.blocks;
    A.blk_flags = reinterpret_cast<uint32_t*>(ws + L.off_blk_flags);
    A.blk_f = reinterpret_cast<float*>(ws + L.off_blk_f);
    A.blk_e = reinterpret_cast<float*>(ws + L.off_blk_e);
    A.l1 = Level{reinterpret_cast<float4*>(ws + L.off_agg_scalar), reinterpret_cast<float*>(ws + L.off_agg_s),
                 reinterpret_cast<float*>(ws + L.off_agg_q), reinterpret_cast<float*>(ws + L.off_car_f),
                 reinterpret_cast<float*>(ws + L.off_car_e), g.tiles};
    A.l2 = Level{reinterpret_cast<float4*>(ws + L.off_agg2_scalar), reinterpret_cast<float*>(ws + L.off_agg2_s),
                 reinterpret_cast<float*>(ws + L.off_agg2_q), reinterpret_cast<float*>(ws + L.off_car2_f),
                 reinterpret_cast<float*>(ws + L.off_car2_e), g.chunks};
    A.red_partial = reinterpret_cast<float*>(ws + L.off_red);
    A.list_inj = reinterpret_cast<uint32_t*>(ws + L.off_lists);
    A.list_both = A.list_inj + L.max_tiles;
    A.counters = reinterpret_cast<uint32_t*>(ws + L.off_counters);
    {   // list-driven launches pay off when the rows that force a heavy tile are few next to the tiles
        const int64_t inj_rows = (int64_t)p.inj_hi - p.inj_lo, res_rows = (int64_t)p.res_hi - p.res_lo;
        const int64_t both = inj_rows < res_rows ? inj_rows : res_rows;
        A.reduce_from_list = inj_rows * 4 <= g.tiles;
        A.down_from_list = both * 4 <= g.blocks;
        if (p.inj_sorted && p.out_sorted) A.reduce_from_list = A.down_from_list = 0;   // every block is visited
        // blocks with a handful of injected (result) rows skip the scan inside the block: wide geometry,
        // injected and result rows from different matrices, and few such rows overall
        const bool disjoint = p.inj_hi <= p.res_lo || p.res_hi <= p.inj_lo;
        A.few_inj_ok = g.sub_shift && disjoint && inj_rows * 4 <= g.blocks;
        A.few_res_ok = g.sub_shift && disjoint && res_rows * 4 <= g.blocks;
        // (the metadata pass runs before the reduce; with a dense injection the reduce then visits every
        //  tile and overwrites the provisional summaries, with a sparse one only the listed tiles)
    }

    const std::string tag = p.tag ? p.tag : "scan";
    const bool two = p.emit_values == 2;
    if (v4) { if (strict) launch_all<4, true>(A, g, tag, two, st); else launch_all<4, false>(A, g, tag, two, st); }
    else    { if (strict) launch_all<1, true>(A, g, tag, two, st); else launch_all<1, false>(A, g, tag, two, st); }
    if (p.out_red && g.slabs > 1) {
        const int64_t rows = (int64_t)p.res_hi - (int64_t)p.res_lo;
        int64_t gsz = (rows + 255) / 256; if (gsz > 65536) gsz = 65536; if (gsz < 1) gsz = 1;
        LAPLEX_TIMED("sum_slabs", st, hipLaunchKernelGGL(k_sum_slabs, dim3((unsigned)gsz), dim3(256), 0, st,
                                                         (const float*)A.red_partial, rows, g.slabs, p.out_red));
    }
    return hipGetLastError();
}

hipError_t launch_rowdot_ops(const float* u, int64_t ldu, int64_t op_u, const float* v, int64_t ldv, int64_t op_v,
                             int64_t rows, int64_t batch, float* out, int64_t op_out, int64_t operators, hipStream_t st)
{
    if (rows <= 0 || operators <= 0) return hipSuccess;
    if (batch <= 8) {
        int64_t g = (rows + 255) / 256; if (g > 65536) g = 65536;
        LAPLEX_TIMED("rowdot", st, hipLaunchKernelGGL(k_rowdot_narrow, dim3((unsigned)g, (unsigned)operators), dim3(256), 0, st,
                                                      u, ldu, op_u, v, ldv, op_v, rows, batch, out, op_out));
        return hipGetLastError();
    }
    int64_t gsz = (rows + 3) / 4; if (gsz > 65536) gsz = 65536;
    LAPLEX_TIMED("rowdot", st, hipLaunchKernelGGL(k_rowdot, dim3((unsigned)gsz, (unsigned)operators), dim3(256), 0, st,
                                                  u, ldu, op_u, v, ldv, op_v, rows, batch, out, op_out));
    return hipGetLastError();
}

hipError_t launch_add_rowdot(const float* u, int64_t ldu, const float* v, int64_t ldv, int64_t rows, int64_t batch, float* out,
                             hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    int64_t g = (rows + 255) / 256; if (g > 65536) g = 65536;
    LAPLEX_TIMED("rowdot", st, hipLaunchKernelGGL(k_add_rowdot, dim3((unsigned)g), dim3(256), 0, st, u, ldu, v, ldv, rows, batch, out));
    return hipGetLastError();
}

hipError_t launch_rowdot2(const float* u1, int64_t ldu1, const float* v1, int64_t ldv1,
                          const float* u2, int64_t ldu2, const float* v2, int64_t ldv2,
                          int64_t rows, int64_t batch, float* out, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    int64_t gsz = (rows + 3) / 4; if (gsz > 65536) gsz = 65536;
    LAPLEX_TIMED("rowdot", st, hipLaunchKernelGGL(k_rowdot2, dim3((unsigned)gsz), dim3(256), 0, st,
                                                  u1, ldu1, v1, ldv1, u2, ldu2, v2, ldv2, rows, batch, out));
    return hipGetLastError();
}

hipError_t launch_rowdot(const float* u, int64_t ldu, const float* v, int64_t ldv,
                         int64_t rows, int64_t batch, float* out, hipStream_t st)
{
    return launch_rowdot_ops(u, ldu, 0, v, ldv, 0, rows, batch, out, 0, 1, st);
}

}  // namespace laplex
