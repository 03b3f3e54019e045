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
// strict channel, (H, C, Q) with E_out = H ? C F_in + Q : E_in.  Summaries
// compose associatively, so the work splits into three launches, with both
// directions done together so that the injected matrix is read once per launch:
//
//   reduce     per tile: its forward and its backward summary
//   spine      per batch column and direction: exclusive scan over tile summaries
//   downsweep  per tile that holds result rows: re-read the tile, seed both
//              walks with the carries, walk forward then backward and emit
//
// Lanes: bv lanes across the batch (vec columns each) x rv row-lanes per
// wavefront; each row-lane walks `items` consecutive rows sequentially.
#include "laplex_internal.h"

#include <string>

namespace laplex {

namespace {

struct ScanArgs {
    const uint32_t* ids; const float* dh; int64_t N;
    const float* inj; int64_t ld_inj; uint32_t inj_lo, inj_hi;
    uint32_t res_lo, res_hi;
    float* out_p; int64_t ld_p;
    float* out_z;
    float* out_red; const float* w; int64_t ld_w; const float* zs;
    int64_t batch, bpad, tiles;
    int bv, bv_log2, rv, tile_rows, slabs;
    float4* agg_scalar; float* agg_s; float* agg_q; float* car_f; float* car_e;
    float* red_partial;   // [slabs][res rows] when slabs > 1
};

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
    if (STRICT && h) {
        s.C = dd * s.D;
        s.H = 1;
#pragma unroll
        for (int e = 0; e < VEC; ++e) s.Q[e] = dd * s.S[e];
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
        r.C = y.H ? y.C * x.D : x.C;
#pragma unroll
        for (int e = 0; e < VEC; ++e) r.Q[e] = y.H ? y.C * x.S[e] + y.Q[e] : x.Q[e];
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
        if (STRICT && s.H) E[e] = s.C * F[e] + s.Q[e];
        F[e] = s.D * F[e] + s.S[e];
    }
}

// Inclusive scan of the row-lanes of one wavefront, in forward (row-lane 0
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

template <int VEC>
struct TileRows {
    static constexpr int ITEMS = VEC == 4 ? kItemsVec4 : kItemsVec1;
    float dh[ITEMS + 1];      // dh[i]: decay into row i from the left; dh[i+1]: from the right
    uint32_t id[ITEMS];
    bool live[ITEMS];
    float v[ITEMS][VEC];
};

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

template <int VEC>
__device__ __forceinline__ void load_rows(const ScanArgs& A, int64_t row0, int64_t col0, bool col_ok,
                                          TileRows<VEC>& T)
{
    constexpr int ITEMS = TileRows<VEC>::ITEMS;
#pragma unroll
    for (int i = 0; i <= ITEMS; ++i) {
        const int64_t j = row0 + i;
        T.dh[i] = j <= A.N ? A.dh[j] : -1.0f;
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int64_t j = row0 + i;
        T.live[i] = j < A.N;
        T.id[i] = T.live[i] ? A.ids[j] : 0xFFFFFFFFu;
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool inj = col_ok && T.id[i] >= A.inj_lo && T.id[i] < A.inj_hi;
#pragma unroll
        for (int e = 0; e < VEC; ++e) T.v[i][e] = 0.0f;
        if (inj) load_vec<VEC>(T.v[i], A.inj + (int64_t)(T.id[i] - A.inj_lo) * A.ld_inj + col0);
    }
}

template <int VEC, bool STRICT>
__device__ __forceinline__ void local_segs(const TileRows<VEC>& T, Seg<VEC, STRICT>& f, Seg<VEC, STRICT>& b)
{
    constexpr int ITEMS = TileRows<VEC>::ITEMS;
    f = seg_identity<VEC, STRICT>();
    b = seg_identity<VEC, STRICT>();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) seg_push<VEC, STRICT>(f, T.live[i] && T.dh[i] >= 0.0f, T.dh[i], T.v[i]);
#pragma unroll
    for (int i = ITEMS - 1; i >= 0; --i) seg_push<VEC, STRICT>(b, T.live[i] && T.dh[i + 1] >= 0.0f, T.dh[i + 1], T.v[i]);
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

// ---------------------------------------------------------------------------
// reduce: forward and backward summary of every tile
// ---------------------------------------------------------------------------
template <int VEC, bool STRICT>
__global__ void __launch_bounds__(kScanThreads)
k_scan_reduce(const ScanArgs A)
{
    __shared__ WaveSegs<VEC> W;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bv = A.bv, rv = A.rv;
    const int c = lane & (bv - 1), r = lane >> A.bv_log2;
    const int64_t tile = blockIdx.x;
    const int64_t row0 = tile * A.tile_rows + (int64_t)(wave * rv + r) * TileRows<VEC>::ITEMS;
    const int64_t col0 = ((int64_t)blockIdx.y * bv + c) * VEC;
    const bool col_ok = col0 < A.batch;

    TileRows<VEC> T;
    load_rows<VEC>(A, row0, col0, col_ok, T);
    Seg<VEC, STRICT> f, b;
    local_segs<VEC, STRICT>(T, f, b);
    f = wave_scan<true, VEC, STRICT>(f, lane, bv, rv);
    b = wave_scan<false, VEC, STRICT>(b, lane, bv, rv);
    if (r == rv - 1) put_wave_seg<VEC, STRICT>(W, 0, wave, c, f);
    if (r == 0) put_wave_seg<VEC, STRICT>(W, 1, wave, c, b);
    __syncthreads();

    if (tid < bv) {   // wavefront 0, row-lane 0: one lane per column group
        Seg<VEC, STRICT> tf = seg_identity<VEC, STRICT>(), tb = seg_identity<VEC, STRICT>();
#pragma unroll
        for (int w = 0; w < kScanWaves; ++w) tf = seg_compose<VEC, STRICT>(tf, get_wave_seg<VEC, STRICT>(W, 0, w, c));
#pragma unroll
        for (int w = kScanWaves - 1; w >= 0; --w) tb = seg_compose<VEC, STRICT>(tb, get_wave_seg<VEC, STRICT>(W, 1, w, c));
        if (c == 0 && blockIdx.y == 0) {
            A.agg_scalar[tile] = make_float4(tf.D, tf.C, (float)tf.H, 0.0f);
            A.agg_scalar[A.tiles + tile] = make_float4(tb.D, tb.C, (float)tb.H, 0.0f);
        }
        if (col_ok) {
            const int64_t o0 = tile * A.bpad + col0, o1 = (A.tiles + tile) * A.bpad + col0;
            store_vec<VEC>(A.agg_s + o0, tf.S);
            store_vec<VEC>(A.agg_s + o1, tb.S);
            if (STRICT) { store_vec<VEC>(A.agg_q + o0, tf.Q); store_vec<VEC>(A.agg_q + o1, tb.Q); }
        }
    }
}

// ---------------------------------------------------------------------------
// spine: exclusive scan over the tile summaries, one workgroup per (column, direction).
// Carries are the state a tile starts from when the sequence starts from zero:
// F_in = S of everything before it, E_in = Q of everything before it (0 without a head).
// ---------------------------------------------------------------------------
template <bool STRICT>
__global__ void __launch_bounds__(kSpineThreads)
k_scan_spine(const ScanArgs A)
{
    constexpr int WAVES = kSpineThreads / 64;
    __shared__ float sD[WAVES], sC[WAVES], sS[WAVES], sQ[WAVES];
    __shared__ int sH[WAVES];
    typedef Seg<1, STRICT> S1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t col = blockIdx.x;
    const int dir = blockIdx.y;
    const int64_t tiles = A.tiles;
    const int64_t per = (tiles + kSpineThreads - 1) / kSpineThreads;
    const int64_t q0 = (int64_t)tid * per;
    const int64_t q1 = q0 + per < tiles ? q0 + per : tiles;
    const float4* sc = A.agg_scalar + (int64_t)dir * tiles;
    const float* as = A.agg_s + (int64_t)dir * tiles * A.bpad + col;
    const float* aq = A.agg_q + (int64_t)dir * tiles * A.bpad + col;
    float* cf = A.car_f + (int64_t)dir * tiles * A.bpad + col;
    float* ce = A.car_e + (int64_t)dir * tiles * A.bpad + col;

    auto tile_seg = [&](int64_t q) {
        const int64_t t = dir == 0 ? q : tiles - 1 - q;   // scan order -> tile index
        S1 s;
        const float4 v = sc[t];
        s.D = v.x; s.C = v.y; s.H = STRICT ? (int)v.z : 0;
        s.S[0] = as[t * A.bpad];
        s.Q[0] = STRICT ? aq[t * A.bpad] : 0.0f;
        return s;
    };

    S1 mine = seg_identity<1, STRICT>();
    for (int64_t q = q0; q < q1; ++q) mine = seg_compose<1, STRICT>(mine, tile_seg(q));

    // inclusive scan over the workgroup's threads
    S1 inc = wave_scan<true, 1, STRICT>(mine, lane, 1, 64);
    if (lane == 63) { sD[wave] = inc.D; sC[wave] = inc.C; sH[wave] = inc.H; sS[wave] = inc.S[0]; sQ[wave] = inc.Q[0]; }
    __syncthreads();
    S1 run = seg_identity<1, STRICT>();
    for (int w = 0; w < wave; ++w) {
        S1 o; o.D = sD[w]; o.C = sC[w]; o.H = sH[w]; o.S[0] = sS[w]; o.Q[0] = sQ[w];
        run = seg_compose<1, STRICT>(run, o);
    }
    S1 prev = seg_shfl<1, STRICT>(inc, (lane - 1) & 63);
    if (lane > 0) run = seg_compose<1, STRICT>(run, prev);

    for (int64_t q = q0; q < q1; ++q) {
        const int64_t t = dir == 0 ? q : tiles - 1 - q;
        cf[t * A.bpad] = run.S[0];
        if (STRICT) ce[t * A.bpad] = run.H ? run.Q[0] : 0.0f;
        run = seg_compose<1, STRICT>(run, tile_seg(q));
    }
}

// ---------------------------------------------------------------------------
// downsweep: walk every tile that holds result rows, forward then backward
// ---------------------------------------------------------------------------
template <int VEC, bool STRICT>
__global__ void __launch_bounds__(kScanThreads)
k_scan_down(const ScanArgs A)
{
    constexpr int ITEMS = TileRows<VEC>::ITEMS;
    __shared__ WaveSegs<VEC> W;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bv = A.bv, rv = A.rv;
    const int c = lane & (bv - 1), r = lane >> A.bv_log2;
    const int64_t tile = blockIdx.x;
    const int64_t row0 = tile * A.tile_rows + (int64_t)(wave * rv + r) * ITEMS;
    const int64_t col0 = ((int64_t)blockIdx.y * bv + c) * VEC;
    const bool col_ok = col0 < A.batch;

    // Does this tile hold any result row?  (ids are cheap next to the data rows.)
    {
        int any = 0;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int64_t j = row0 + i;
            if (j < A.N) { const uint32_t id = A.ids[j]; any |= (id >= A.res_lo && id < A.res_hi); }
        }
        if (!__syncthreads_or(any)) return;
    }

    TileRows<VEC> T;
    load_rows<VEC>(A, row0, col0, col_ok, T);

    // weights of the row reduction, fetched early so the loads overlap the scans
    float wv[ITEMS][VEC];
    const bool want_red = STRICT && A.out_red != nullptr;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) wv[i][e] = 0.0f;
        if (want_red && col_ok && T.id[i] >= A.res_lo && T.id[i] < A.res_hi)
            load_vec<VEC>(wv[i], A.w + (int64_t)(T.id[i] - A.res_lo) * A.ld_w + col0);
    }

    Seg<VEC, STRICT> f, b;
    local_segs<VEC, STRICT>(T, f, b);
    const Seg<VEC, STRICT> fi = wave_scan<true, VEC, STRICT>(f, lane, bv, rv);
    const Seg<VEC, STRICT> bi = wave_scan<false, VEC, STRICT>(b, lane, bv, rv);
    if (r == rv - 1) put_wave_seg<VEC, STRICT>(W, 0, wave, c, fi);
    if (r == 0) put_wave_seg<VEC, STRICT>(W, 1, wave, c, bi);
    // exclusive summaries inside the wavefront
    Seg<VEC, STRICT> fe = seg_shfl<VEC, STRICT>(fi, (lane - bv) & 63);
    Seg<VEC, STRICT> be = seg_shfl<VEC, STRICT>(bi, (lane + bv) & 63);
    if (r == 0) fe = seg_identity<VEC, STRICT>();
    if (r == rv - 1) be = seg_identity<VEC, STRICT>();
    __syncthreads();

    // entering states: tile carry, then the wavefronts before this one, then the row-lanes before this one
    float F[VEC], E[VEC], R[VEC], G[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { F[e] = E[e] = R[e] = G[e] = 0.0f; }
    if (col_ok) {
        const int64_t o0 = tile * A.bpad + col0, o1 = (A.tiles + tile) * A.bpad + col0;
        load_vec<VEC>(F, A.car_f + o0);
        load_vec<VEC>(R, A.car_f + o1);
        if (STRICT) { load_vec<VEC>(E, A.car_e + o0); load_vec<VEC>(G, A.car_e + o1); }
    }
    for (int w = 0; w < wave; ++w) seg_apply<VEC, STRICT>(get_wave_seg<VEC, STRICT>(W, 0, w, c), F, E);
    for (int w = kScanWaves - 1; w > wave; --w) seg_apply<VEC, STRICT>(get_wave_seg<VEC, STRICT>(W, 1, w, c), R, G);
    seg_apply<VEC, STRICT>(fe, F, E);
    seg_apply<VEC, STRICT>(be, R, G);

    // forward walk: keep F (and E) of every row
    float Ff[ITEMS][VEC], Ef[ITEMS][VEC];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool h = T.live[i] && T.dh[i] >= 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if (h) { E[e] = T.dh[i] * F[e]; F[e] = E[e] + T.v[i][e]; }
            else   { F[e] = F[e] + T.v[i][e]; }
            Ff[i][e] = F[e];
            Ef[i][e] = E[e];
        }
    }

    // backward walk with emission
    const int64_t res_rows = (int64_t)A.res_hi - (int64_t)A.res_lo;
#pragma unroll
    for (int i = ITEMS - 1; i >= 0; --i) {
        const bool h = T.live[i] && T.dh[i + 1] >= 0.0f;
        float P[VEC], Z[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if (h) { G[e] = T.dh[i + 1] * R[e]; R[e] = G[e] + T.v[i][e]; }
            else   { R[e] = R[e] + T.v[i][e]; }
            P[e] = Ff[i][e] + R[e] - T.v[i][e];
            Z[e] = G[e] - Ef[i][e];
        }
        const bool is_res = T.id[i] >= A.res_lo && T.id[i] < A.res_hi;
        const int64_t rr = (int64_t)T.id[i] - (int64_t)A.res_lo;
        if (is_res && col_ok) {
            if (A.out_p) store_vec<VEC>(A.out_p + rr * A.ld_p + col0, P);
            if (STRICT && A.out_z) store_vec<VEC>(A.out_z + rr * A.batch + col0, Z);
        }
        if (want_red) {
            float acc = 0.0f;
            if (is_res && col_ok) {
                float zsv[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) zsv[e] = 0.0f;
                if (A.zs) load_vec<VEC>(zsv, A.zs + rr * A.batch + col0);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc += wv[i][e] * Z[e] + T.v[i][e] * zsv[e];
            }
            for (int m = 1; m < bv; m <<= 1) acc += __shfl_xor(acc, m);
            if (is_res && c == 0) {
                if (A.slabs == 1) A.out_red[rr] = acc;
                else A.red_partial[(int64_t)blockIdx.y * res_rows + rr] = acc;
            }
        }
    }
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

// out[r] = sum_t u[r, t] * v[r, t]: one wavefront per row, fixed summation order
__global__ void __launch_bounds__(256)
k_rowdot(const float* __restrict__ u, int64_t ldu, const float* __restrict__ v, int64_t ldv,
         int64_t rows, int64_t batch, float* __restrict__ out)
{
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

int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

hipError_t launch_scan(const ScanProblem& p, const Layout& L, char* ws, hipStream_t st)
{
    const bool strict = p.out_z != nullptr || p.out_red != nullptr;
    // 128-bit lanes need every row start of every matrix touched to be 16-byte aligned
    bool v4 = p.batch % 4 == 0 && p.batch >= 4;
    v4 = v4 && aligned16(p.inj) && p.ld_inj % 4 == 0;
    if (p.out_p) v4 = v4 && aligned16(p.out_p) && p.ld_p % 4 == 0;
    if (p.out_z) v4 = v4 && aligned16(p.out_z);
    if (p.out_red) v4 = v4 && aligned16(p.w) && p.ld_w % 4 == 0 && (!p.zs || aligned16(p.zs));
    const ScanGeom g = scan_geom(p.N, p.batch, v4 ? 4 : 1);

    ScanArgs A;
    A.ids = p.ids; A.dh = p.dh; A.N = p.N;
    A.inj = p.inj; A.ld_inj = p.ld_inj; A.inj_lo = p.inj_lo; A.inj_hi = p.inj_hi;
    A.res_lo = p.res_lo; A.res_hi = p.res_hi;
    A.out_p = p.out_p; A.ld_p = p.ld_p; A.out_z = p.out_z;
    A.out_red = p.out_red; A.w = p.w; A.ld_w = p.ld_w; A.zs = p.zs;
    A.batch = p.batch; A.bpad = L.bpad; A.tiles = g.tiles;
    A.bv = g.bv; A.bv_log2 = ilog2(g.bv); A.rv = g.rv; A.tile_rows = g.tile_rows; A.slabs = g.slabs;
    A.agg_scalar = reinterpret_cast<float4*>(ws + L.off_agg_scalar);
    A.agg_s = reinterpret_cast<float*>(ws + L.off_agg_s);
    A.agg_q = reinterpret_cast<float*>(ws + L.off_agg_q);
    A.car_f = reinterpret_cast<float*>(ws + L.off_car_f);
    A.car_e = reinterpret_cast<float*>(ws + L.off_car_e);
    A.red_partial = reinterpret_cast<float*>(ws + L.off_red);

    const std::string tag = p.tag ? p.tag : "scan";
    const std::string fam_r = "scan_reduce." + tag, fam_s = "scan_spine." + tag, fam_d = "scan_down." + tag;
    const dim3 grid((unsigned)g.tiles, (unsigned)g.slabs), block(kScanThreads);
    const dim3 sgrid((unsigned)p.batch, 2), sblock(kSpineThreads);
#define LAPLEX_LAUNCH3(V, S)                                                                    \
    do {                                                                                        \
        LAPLEX_TIMED(fam_r.c_str(), st, hipLaunchKernelGGL((k_scan_reduce<V, S>), grid, block, 0, st, A)); \
        LAPLEX_TIMED(fam_s.c_str(), st, hipLaunchKernelGGL((k_scan_spine<S>), sgrid, sblock, 0, st, A));    \
        LAPLEX_TIMED(fam_d.c_str(), st, hipLaunchKernelGGL((k_scan_down<V, S>), grid, block, 0, st, A));     \
    } while (0)
    if (v4) { if (strict) LAPLEX_LAUNCH3(4, true); else LAPLEX_LAUNCH3(4, false); }
    else    { if (strict) LAPLEX_LAUNCH3(1, true); else LAPLEX_LAUNCH3(1, false); }
#undef LAPLEX_LAUNCH3
    if (p.out_red && g.slabs > 1) {
        const int64_t rows = (int64_t)p.res_hi - (int64_t)p.res_lo;
        int64_t gsz = (rows + 255) / 256; if (gsz > 65536) gsz = 65536; if (gsz < 1) gsz = 1;
        LAPLEX_TIMED("sum_slabs", st, hipLaunchKernelGGL(k_sum_slabs, dim3((unsigned)gsz), dim3(256), 0, st,
                                                         (const float*)A.red_partial, rows, g.slabs, p.out_red));
    }
    return hipGetLastError();
}

hipError_t launch_rowdot(const float* u, int64_t ldu, const float* v, int64_t ldv,
                         int64_t rows, int64_t batch, float* out, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    int64_t gsz = (rows + 3) / 4; if (gsz > 65536) gsz = 65536;
    LAPLEX_TIMED("rowdot", st, hipLaunchKernelGGL(k_rowdot, dim3((unsigned)gsz), dim3(256), 0, st, u, ldu, v, ldv, rows, batch, out));
    return hipGetLastError();
}

}  // namespace laplex
