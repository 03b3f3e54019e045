// Small problems in two launches.  When the merged sequence a ++ b has at most kSmallMax positions the
// whole path of one call (Sec. 3: sort, then the prefix recurrence and its mirror image) is one launch
// that sorts (k_small_rank: ranks by counting, over the whole device) and one that holds the plan of an
// operator in LDS and runs the decays, the decayed scans in both directions and the scatter (k_small),
// where the large path needs some thirty launches of a few microseconds each.  (App. "GPU runtime": below
// n = 2^17 the paper's curves are flat at the cost of the launches.)  Several operators (the r anchor
// pairs of a sum of operators) and several slabs of batch columns are separate workgroups of a launch.
//
// Layout of the work: a workgroup of 16 wavefronts handles C <= 16 batch columns; lane l of a wavefront
// works on column l % C and is row-lane l / C of the wavefront's 64 / C (adjacent lanes read adjacent
// columns of one row), so a column has RL = 1024 / C row-lanes, each walking 8 consecutive rows per
// sweep of RS = 8 * RL rows.  Inside a row-lane decays are multiplied up (at most 8 factors); every
// longer decay is exp of an anchor difference; row-lanes are combined by wavefront shuffles, wavefronts
// and sweeps through LDS.
// The numbers carried are those of the large path: F (inclusive decayed sum) and E (the sum over
// strictly smaller keys), summarised per segment as (D, S, H, Q):
//     F_out = D F_in + S,    E_out = H ? D F_in + Q : E_in.
#include "laplex_internal.h"

namespace laplex {

namespace {

constexpr int kSmallThreads = 1024;
constexpr int kSmallWaves = kSmallThreads / 64;
constexpr int kSmallItems = 8;

__device__ __forceinline__ uint32_t small_float_to_key(float f)
{
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0u;                       // -0.0 sorts as +0.0
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

__device__ __forceinline__ float small_key_to_float(uint32_t key)
{
    return __uint_as_float(key ^ ((key >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

struct SmallShared {
    uint32_t* id;      // [N]      sorted ids
    float* p;          // [N + 2]  sorted anchors between -inf and +inf
    float* dh;         // [N + 1]  decay into row j from row j - 1; negative: same key
};

// One direction of one scan problem.  DIR = 0: ascending keys; DIR = 1: descending (the mirror image).
// q counts rows in processing order.  The first direction parks its results at the result rows
// (out_p <- F, out_z <- -E); the second adds its own and finishes them:  out_p = F + R - v,  out_z = G - E.
template <int DIR, bool STRICT>
__device__ __forceinline__ void small_pass(const SmallProblem& P, const SmallShared& sh, int N, int64_t batch,
                                           int C, int64_t col0, float* wtot /* [4][256] */)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int RPW = 64 / C;                     // row-lanes per wavefront
    const int c = lane % C, rls = lane / C;     // adjacent lanes hold adjacent columns of a row: a load touches RPW rows
    const int RL = kSmallWaves * RPW;
    const int RS = RL * kSmallItems;
    const int64_t col = col0 + c;
    const bool col_ok = col < batch;
    const int sweeps = (N + RS - 1) / RS;
    auto pos = [&](int q) -> float { return DIR ? -sh.p[N - q] : sh.p[q + 1]; };      // q in -1 .. N
    float Fc = 0.0f, Ec = 0.0f;                 // state at the end of the previous sweep
    for (int s = 0; s < sweeps; ++s) {
        const int q0 = s * RS + (wave * RPW + rls) * kSmallItems;
        float v[kSmallItems], F0[kSmallItems], E0[kSmallItems], cf[kSmallItems];
        uint32_t idr[kSmallItems];
        int seen = 0;
        {
            float F = 0.0f, E = 0.0f, prod = 1.0f;
            int sn = 0;
#pragma unroll
            for (int i = 0; i < kSmallItems; ++i) {
                const int q = q0 + i;
                const bool live = q < N;
                const int row = live ? (DIR ? N - 1 - q : q) : 0;
                const uint32_t id = live ? sh.id[row] : 0xFFFFFFFFu;
                const float d = live ? (DIR ? sh.dh[row + 1] : sh.dh[row]) : -1.0f;     // past the end: transparent
                const bool h = d >= 0.0f;
                float val = 0.0f;
                if (live && col_ok && id >= P.inj_lo && id < P.inj_hi) val = P.inj[(int64_t)(id - P.inj_lo) * P.ld_inj + col];
                E = h ? d * F : E;
                F = (h ? E : F) + val;
                prod *= h ? d : 1.0f;
                sn |= h ? 1 : 0;
                v[i] = val; F0[i] = F; E0[i] = E; cf[i] = prod; idr[i] = id;
                seen |= sn << i;
            }
        }
        // Everything beyond a row-lane is combined with decays taken from the anchors, never with products
        // of decays (a product of m equal factors carries m times the factor's rounding error, and on a
        // regular grid the factors ARE equal).  endq(r): the last row of row-lane r of this sweep.
        auto endq = [&](int r) -> int { const int q = s * RS + (r + 1) * kSmallItems - 1; return q < N ? q : N - 1; };
        const int rl = wave * RPW + rls;
        // inclusive scan over the row-lanes of the wavefront (lanes C apart hold the same column): (S, Q, H) of
        // the row-lanes rl - 2^j + 1 .. rl; the decay across them is exp(-(anchor at their end - anchor before them))
        float S = F0[kSmallItems - 1], Q = E0[kSmallItems - 1];
        int H = (seen >> (kSmallItems - 1)) & 1;
        for (int d = 1; d < RPW; d <<= 1) {
            const float So = __shfl_up(S, d * C), Qo = __shfl_up(Q, d * C);
            const int Ho = __shfl_up(H, d * C);
            if (rls >= d) {
                const float Dl = expf(-(pos(endq(rl)) - pos(endq(rl - d))));
                Q = H ? Dl * So + Q : Qo;
                S = Dl * So + S;
                H |= Ho;
            }
        }
        if (rls == RPW - 1) {
            const int slot = wave * 16 + c;
            wtot[1 * 256 + slot] = S; wtot[2 * 256 + slot] = Q; wtot[3 * 256 + slot] = __int_as_float(H);
        }
        // the row-lanes before this one in the wavefront
        float Sb = __shfl_up(S, C), Qb = __shfl_up(Q, C);
        int Hb = __shfl_up(H, C);
        if (rls == 0) { Sb = 0.0f; Qb = 0.0f; Hb = 0; }
        // Decays from the end of wavefront u (lane u), and from the end of the previous sweep (lane 16), to the
        // row before this wavefront's first (gw) and to the end of this sweep (ge); the same for every column.
        float gw = 0.0f, ge = 0.0f;
        {
            const int q_before_wave = s * RS + wave * RPW * kSmallItems - 1;      // >= -1
            const float target_w = pos(q_before_wave < N ? q_before_wave : N - 1);
            const float target_e = pos(endq(RL - 1));
            if (lane <= kSmallWaves) {
                const float from = lane < kSmallWaves ? pos(endq((lane + 1) * RPW - 1)) : pos(s * RS - 1);
                // (the first wavefront of the first sweep has nothing before it: both anchors are the -inf sentinel)
                gw = (lane < wave || lane == kSmallWaves) && q_before_wave >= 0 ? expf(-(target_w - from)) : 0.0f;
                ge = expf(-(target_e - from));
            }
        }
        __syncthreads();
        // state entering this wavefront (Fin, Ein) and state at the end of the sweep (Fc, Ec): sums over the
        // wavefronts' summaries, each decayed to the target directly
        auto lane_value = [](float x, int l) -> float { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l)); };
        float Fin = lane_value(gw, kSmallWaves) * Fc, Ein = Ec;
        float Fe = lane_value(ge, kSmallWaves) * Fc, Ee = Ec;
#pragma unroll
        for (int u = 0; u < kSmallWaves; ++u) {
            const int slot = u * 16 + c;
            const float tS = wtot[1 * 256 + slot], tQ = wtot[2 * 256 + slot];
            const int tH = __float_as_int(wtot[3 * 256 + slot]);
            const float gwu = lane_value(gw, u), geu = lane_value(ge, u);
            if (u < wave) {
                if (tH) Ein = Fin + tQ;       // a run head inside u: everything before u, decayed, plus u's own strict sum
                Fin += gwu * tS;
            }
            if (tH) Ee = Fe + tQ;
            Fe += geu * tS;
        }
        Fc = Fe; Ec = Ee;
        __syncthreads();                                            // wtot is rewritten by the next sweep
        // ... and through the row-lanes before this one
        {
            const int qw = s * RS + wave * RPW * kSmallItems - 1;
            const float Dwl = rls == 0 ? 1.0f : expf(-(pos(q0 - 1 < N ? q0 - 1 : N - 1) - pos(qw < N ? qw : N - 1)));
            const float f = Dwl * Fin;
            Ein = Hb ? f + Qb : Ein;
            Fin = f + Sb;
        }
        // the rows
#pragma unroll
        for (int i = 0; i < kSmallItems; ++i) {
            const uint32_t id = idr[i];
            if (!(id >= P.res_lo && id < P.res_hi) || !col_ok) continue;
            const float f = cf[i] * Fin;
            const float Fi = f + F0[i];
            const float Ei = ((seen >> i) & 1) ? f + E0[i] : Ein;
            const int64_t rr = (int64_t)(id - P.res_lo);
            if (P.out_p) {
                float* o = P.out_p + rr * P.ld_p + col;
                *o = DIR == 0 ? Fi : *o + Fi - v[i];
            }
            if (STRICT && P.out_z) {
                float* o = P.out_z + rr * batch + col;
                *o = DIR == 0 ? -Ei : *o + Ei;
            }
        }
    }
}

// The sort of a small problem, spread over the whole device: the stable rank of an anchor is the number
// of pairs (key, position) below its own, and counting that by brute force costs N^2 comparisons, which
// 256 compute units do in about a microsecond for N = 8192 when the count is taken 64 comparisons at a
// time (one compare instruction, one population count of the resulting lane mask).  A workgroup takes
// a block of queries; each of its 16 wavefronts keeps 512 of the candidates in registers (8 per lane),
// counts for every query how many of them lie below it, and the 16 partial counts are added per query.
// Output: the plan's ids and sorted anchors (pk, between its two sentinels).
constexpr int kRankQueriesMax = 256;      // queries per workgroup: 32 .. 256, chosen by the launcher

__global__ void __launch_bounds__(kSmallThreads)
k_small_rank(SmallArgs A, int queries)
{
    __shared__ unsigned long long query[kRankQueriesMax];
    __shared__ uint32_t partial[kRankQueriesMax][kSmallWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t op = blockIdx.y;
    const int N = (int)(A.k + A.n);
    const float* a = A.a + op * A.op_a;
    const float* b = A.b + op * A.op_b;
    uint32_t* g_ids = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(A.ids) + op * A.op_ws);
    float* g_pk = reinterpret_cast<float*>(reinterpret_cast<char*>(A.pk) + op * A.op_ws);
    auto composite = [&](int e) -> unsigned long long {
        const float f = A.tau * (e < A.k ? a[e] : b[e - A.k]);
        return ((unsigned long long)small_float_to_key(f) << 32) | (unsigned long long)(uint32_t)e;
    };
    // candidates of this wavefront: positions wave * 512 + r * 64 + lane; a position past the end never counts
    // (one 64-bit compare per 64 candidates; splitting it into key and position compares with lane masks
    //  was four times slower)
    unsigned long long cand[kSmallItems];
#pragma unroll
    for (int r = 0; r < kSmallItems; ++r) {
        const int e = wave * 64 * kSmallItems + r * 64 + lane;
        cand[r] = e < N ? composite(e) : ~0ull;
    }
    const int q0 = blockIdx.x * queries;
    if (tid < queries) query[tid] = q0 + tid < N ? composite(q0 + tid) : 0ull;
    __syncthreads();
    const bool any = wave * 64 * kSmallItems < N;                   // uniform: does this wavefront hold candidates at all
    for (int q = 0; q < queries; ++q) {
        const unsigned long long me = query[q];                     // the same for every lane
        uint32_t below = 0u;
        if (any) {
#pragma unroll
            for (int r = 0; r < kSmallItems; ++r) below += (uint32_t)__popcll(__ballot(cand[r] < me));
        }
        if (lane == 0) partial[q][wave] = below;
    }
    __syncthreads();
    if (tid < queries && q0 + tid < N) {
        uint32_t rank = 0u;
#pragma unroll
        for (int w = 0; w < kSmallWaves; ++w) rank += partial[tid][w];
        const unsigned long long me = query[tid];
        g_ids[rank] = (uint32_t)me;
        g_pk[rank + 1] = small_key_to_float((uint32_t)(me >> 32));
    }
    if (blockIdx.x == 0 && tid == 0) { g_pk[0] = __uint_as_float(0xFF800000u); g_pk[N + 1] = __uint_as_float(0x7F800000u); }
}

__global__ void __launch_bounds__(kSmallThreads)
k_small(SmallArgs A)
{
    __shared__ unsigned long long comp[kSmallMax + 1];      // ids (first half), sorted keys / anchors (second half)
    __shared__ float sdh[kSmallMax + 1];
    __shared__ float wtot[4 * 256];                          // per sweep: (D, S, Q, H) of wavefront w, column c at [w * 16 + c]
    const int tid = threadIdx.x;
    const int64_t op = blockIdx.y;
    const int64_t N = A.k + A.n;
    const uint32_t* g_ids = reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(A.ids) + op * A.op_ws);
    float* g_dh = reinterpret_cast<float*>(reinterpret_cast<char*>(A.dh) + op * A.op_ws);
    const float* g_pk = reinterpret_cast<const float*>(reinterpret_cast<const char*>(A.pk) + op * A.op_ws);
    uint32_t* sid = reinterpret_cast<uint32_t*>(comp);
    float* sp = reinterpret_cast<float*>(comp) + kSmallMax;         // N + 2 floats, the last two in comp[kSmallMax]

    // the plan: sorted ids and anchors from the workspace (written by k_small_rank or by an earlier call);
    // the decays between neighbours are formed here (Sec. 3 "Symmetric case": exp(a_i - a_{i+1}))
    for (int64_t j = tid; j < N; j += kSmallThreads) sid[j] = g_ids[j];
    for (int64_t j = tid; j < N + 2; j += kSmallThreads) sp[j] = g_pk[j];
    __syncthreads();
    for (int64_t j = tid; j <= N; j += kSmallThreads) {
        float d = 0.0f;
        if (j > 0 && j < N) d = sp[j + 1] == sp[j] ? -1.0f : expf(-(sp[j + 1] - sp[j]));
        sdh[j] = d;
        if (blockIdx.x == 0 && A.write_dh) g_dh[j] = d;
    }
    __syncthreads();

    SmallShared sh;
    sh.id = sid; sh.p = sp; sh.dh = sdh;
    const int64_t col0 = (int64_t)blockIdx.x * A.cols;
    for (int i = 0; i < A.nprob; ++i) {
        SmallProblem P = A.prob[i];
        if (P.inj) P.inj += op * P.op_inj;
        if (P.out_p) P.out_p += op * P.op_p;
        if (P.out_z) P.out_z += op * P.op_z;
        if (P.out_z) {
            small_pass<0, true>(P, sh, (int)N, A.batch, A.cols, col0, wtot);
            __syncthreads();          // a row's two directions are walked by different threads: what the first parked must be visible
            small_pass<1, true>(P, sh, (int)N, A.batch, A.cols, col0, wtot);
        } else {
            small_pass<0, false>(P, sh, (int)N, A.batch, A.cols, col0, wtot);
            __syncthreads();
            small_pass<1, false>(P, sh, (int)N, A.batch, A.cols, col0, wtot);
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_small(const SmallArgs& A0, int64_t operators, hipStream_t st)
{
    SmallArgs A = A0;
    // Columns per workgroup: as few as still give the device a workgroup per compute unit (fewer
    // columns = more row-lanes per column = fewer sweeps, and with the device idle otherwise more workgroups beat
    // wider rows: measured on five shapes), at most 16.
    int cols = 16;
    while (cols > 1 && ((A.batch + cols - 1) / cols) * operators < 256) cols >>= 1;
    while (cols > 1 && cols / 2 >= A.batch) cols >>= 1;
    A.cols = cols;
    const int64_t slabs = (A.batch + A.cols - 1) / A.cols;
    const int64_t N = A.k + A.n;
    A.write_dh = A.reuse_plan ? 0 : 1;
    if (!A.reuse_plan) {
        int queries = 32;          // per workgroup (more per workgroup measured slower until the grid gets very large)
        while (queries < kRankQueriesMax && ((N + queries - 1) / queries) * operators > 8192) queries <<= 1;
        LAPLEX_TIMED("small_sort", st, hipLaunchKernelGGL(k_small_rank, dim3((unsigned)((N + queries - 1) / queries), (unsigned)operators),
                                                          dim3(kSmallThreads), 0, st, A, queries));
    }
    if (A.nprob > 0)
        LAPLEX_TIMED("small", st, hipLaunchKernelGGL(k_small, dim3((unsigned)slabs, (unsigned)operators), dim3(kSmallThreads), 0, st, A));
    return hipGetLastError();
}

}  // namespace laplex
