// Sorting the merged anchors (Sec. 3 "Complexity": the O(n log n) term of the method;
// App. B "Combined complexity").  Hand-written for gfx950:
// 64-wide wavefronts, ballot-based stable ranking, LDS-staged scatter.
//
//   radix sort  one-sweep LSD sort, up to 4 passes of 8 bits (a pass whose digit is the same
//               for every key is skipped): one histogram kernel (key
//               build fused: a ++ b -> order-preserving u32 keys, ids = positions),
//               then per pass one read and one write of the pairs, tile offsets
//               from a chained look-back over per-tile status words
//   merge       one merge-path pass when both anchor sets arrive sorted
//   decay       exp(-(p_j - p_{j-1})) between sorted neighbours, once per plan
#include "laplex_internal.h"

#include <type_traits>

namespace laplex {

namespace {

__device__ __forceinline__ uint32_t float_to_key(float f)
{
    const uint32_t u = __float_as_uint(f + 0.0f);       // -0.0 sorts as +0.0: the sum is +0.0, every other value is itself
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}

__device__ __forceinline__ float key_to_float(uint32_t key)
{
    return __uint_as_float(key ^ ((key >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

// ---------------------------------------------------------------------------
// Workgroup-wide exclusive scan of one u32 per thread.
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

// ---------------------------------------------------------------------------
// Ranking inside a tile (used by every pass).  A wavefront owns 64 * KPT
// consecutive keys, item-major (item i of lane l is key i*64 + l of the wavefront's
// range), so the order (wave, item, lane) is the input order.  The lanes that hold
// the same digit find each other with eight ballots; the lowest of them bumps the
// wavefront's digit counter in LDS and hands the old value to its peers.  The tile
// is then laid out in LDS in sorted order and written out so that each digit's run
// goes to consecutive addresses.
// ---------------------------------------------------------------------------
// One-sweep LSD sort.  k_sort_hist reads the anchors once and builds the global
// histogram of all four digits (the key build is fused: keys are computed from
// a and b on the fly, ids are positions).  Each of the four passes then reads its
// input once and writes it once: a tile learns how many keys with each digit lie
// in the tiles before it from a chained look-back over per-tile status words
// instead of a count pass and a table scan.
//
// Look-back protocol.  Tiles are numbered by a ticket taken when the workgroup
// starts, so every predecessor of a running tile is itself running and publishes
// its own digit counts (state 1) before it waits for anything; a tile that has
// found its prefix publishes the inclusive prefix (state 2).  A status word is a
// single 64-bit value (state in the top two bits, count below), written and read
// with agent-scope atomics, so no other memory depends on its ordering.  The
// spin is bounded: if a predecessor never shows up the tile records an error and
// goes on with what it has (the stores stay inside the buffers), so a lost wake-up
// can corrupt a result but never hang the device.
// ---------------------------------------------------------------------------
constexpr int kSpinLimit = 1 << 24;

// Status word: state in the top two bits, a key count below.  32-bit words serve up to 2^30 keys.
template <typename WORD> struct StatusBits;
template <> struct StatusBits<uint32_t> { static constexpr int shift = 30; };
template <> struct StatusBits<unsigned long long> { static constexpr int shift = 62; };

__global__ void __launch_bounds__(1024)
k_sort_reset(uint32_t* small)
{
    for (int i = threadIdx.x; i < kSortSmallWords; i += 1024) small[i] = 0u;
}

// Key of merged position `pos`; the anchors are scaled by the inverse temperature tau on the way in
// (App. A: the temperature-scaled kernel exp(-|a_i - b_j| / t); tau = 1/t; tau = 1 leaves them as they are).
__device__ __forceinline__ uint32_t anchor_key(const float* __restrict__ a, int64_t k,
                                               const float* __restrict__ b, int64_t pos, float tau)
{
    return float_to_key(tau * (pos < k ? a[pos] : b[pos - k]));
}

// Digit counters in LDS.  Two layouts:
//   plain    kHistCopies copies of the 4 x 256 counters (a lane uses copy lane % kHistCopies, and the copies start 8
//            banks apart): keys that share a digit value queue on different words.  64 lanes with unrelated digit
//            values still land 5-6 deep on the busiest of the 32 banks, and an LDS atomic is a read and a write: the
//            kernel runs at ~13 clocks per atomic instruction, which is what bounds it.
//   banked   (many keys per workgroup) every counter of the three low digits 32 times, one per bank: lane l adds to
//            word (counter << 5) + (l & 31), so an instruction touches each bank exactly twice whatever the digit
//            values are.  96 KB of LDS, one workgroup of 16 wavefronts per compute unit.
// The top digit (sign and high exponent bits) takes few values, and consecutive keys of a lane mostly share one: a lane
// counts its current run in a register and adds it to a counter (kHistCopies copies in both layouts) when the value
// changes, and once at the end.
constexpr int kHistCopies = 4;
constexpr int kHistCopyWords = kSortPasses * kRadix + 8;
constexpr int kHistBankedThreads = 1024;
constexpr int64_t kHistBankedMin = int64_t(1) << 22;     // merged positions from which the banked layout is used
constexpr int kHistBankedLowWords = (kSortPasses - 1) * kRadix * 32;
constexpr int kHistTopCopyWords = kRadix + 8;

template <bool BANKED> struct HistLds;
template <> struct HistLds<false> { uint32_t h[kHistCopies * kHistCopyWords]; };
template <> struct HistLds<true> { uint32_t low[kHistBankedLowWords]; uint32_t top[kHistCopies * kHistTopCopyWords]; };

struct TopRun {
    uint32_t cur = 0u, cnt = 0u;
};
template <bool BANKED>
__device__ __forceinline__ uint32_t* hist_top_word(HistLds<BANKED>& L, uint32_t value)
{
    const int copy = threadIdx.x & (kHistCopies - 1);
    if constexpr (BANKED) return &L.top[copy * kHistTopCopyWords + value];
    else return &L.h[copy * kHistCopyWords + (kSortPasses - 1) * kRadix + value];
}
template <bool BANKED>
__device__ __forceinline__ void hist_flush(HistLds<BANKED>& L, TopRun& run)
{
    if (run.cnt) atomicAdd(hist_top_word<BANKED>(L, run.cur), run.cnt);
    run.cnt = 0u;
}
template <bool BANKED>
__device__ __forceinline__ void hist_count(HistLds<BANKED>& L, uint32_t key, bool ok, TopRun& run)
{
    if (ok) {
#pragma unroll
        for (int p = 0; p < kSortPasses - 1; ++p) {
            const uint32_t counter = p * kRadix + ((key >> (p * kRadixBits)) & (kRadix - 1));
            if constexpr (BANKED) atomicAdd(&L.low[(counter << 5) + (threadIdx.x & 31)], 1u);
            else atomicAdd(&L.h[(threadIdx.x & (kHistCopies - 1)) * kHistCopyWords + counter], 1u);
        }
        const uint32_t top = key >> ((kSortPasses - 1) * kRadixBits);
        const uint32_t diff = top ^ run.cur;
        if (diff != 0u && run.cnt) atomicAdd(hist_top_word<BANKED>(L, run.cur), run.cnt);
        run.cnt = (run.cnt & ((diff != 0u) ? 0u : 0xFFFFFFFFu)) + 1u;       // 1 after a change, one more otherwise
        run.cur = top;
    }
}

// One anchor array: a scalar head up to the first 16-byte boundary, 16-byte loads (two in flight per lane), a scalar tail.
template <bool BANKED>
__device__ __forceinline__ void hist_stream(HistLds<BANKED>& h, const float* __restrict__ p, int64_t count, float tau, TopRun& run)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t head = (int64_t)((0u - (uint32_t)(reinterpret_cast<uintptr_t>(p) >> 2)) & 3u);
    if (head > count) head = count;
    const int64_t quads = (count - head) >> 2;
    const float4* __restrict__ p4 = reinterpret_cast<const float4*>(p + head);
    for (int64_t q0 = first; q0 < quads; q0 += 2 * stride) {
        const bool ok1 = q0 + stride < quads;
        const float4 v0 = p4[q0];
        const float4 v1 = p4[ok1 ? q0 + stride : q0];
        hist_count<BANKED>(h, float_to_key(tau * v0.x), true, run); hist_count<BANKED>(h, float_to_key(tau * v0.y), true, run);
        hist_count<BANKED>(h, float_to_key(tau * v0.z), true, run); hist_count<BANKED>(h, float_to_key(tau * v0.w), true, run);
        hist_count<BANKED>(h, float_to_key(tau * v1.x), ok1, run); hist_count<BANKED>(h, float_to_key(tau * v1.y), ok1, run);
        hist_count<BANKED>(h, float_to_key(tau * v1.z), ok1, run); hist_count<BANKED>(h, float_to_key(tau * v1.w), ok1, run);
    }
    // the head and the tail: fewer than 8 keys
    const int64_t rest = count - 4 * quads;
    if (first < rest) {
        const int64_t i = first < head ? first : 4 * quads + first;
        hist_count<BANKED>(h, float_to_key(tau * p[i]), true, run);
    }
}

template <bool BANKED>
__global__ void __launch_bounds__(BANKED ? kHistBankedThreads : kSortThreads)
k_sort_hist(const float* __restrict__ a, int64_t k, const float* __restrict__ b, int64_t n, float tau,
            uint32_t* __restrict__ ghist, unsigned long long* __restrict__ status0, int64_t status_words)
{
    constexpr int THREADS = BANKED ? kHistBankedThreads : kSortThreads;
    __shared__ HistLds<BANKED> L;
    {
        uint32_t* const words = reinterpret_cast<uint32_t*>(&L);
        for (int i = threadIdx.x; i < (int)(sizeof(L) / sizeof(uint32_t)); i += THREADS) words[i] = 0u;
    }
    __syncthreads();
    const int64_t N = k + n;
    TopRun run;
    hist_stream<BANKED>(L, a, k, tau, run);
    hist_stream<BANKED>(L, b, n, tau, run);
    hist_flush<BANKED>(L, run);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = first; i < status_words; i += stride) status0[i] = 0ull;   // look-back words of pass 0
    __syncthreads();
    uint32_t seen = 0;
    for (int i = threadIdx.x; i < kSortPasses * kRadix; i += THREADS) {
        uint32_t c = 0;
        if constexpr (BANKED) {
            if (i < (kSortPasses - 1) * kRadix) {
#pragma unroll
                for (int r = 0; r < 32; ++r) c += L.low[(i << 5) + ((r + threadIdx.x) & 31)];      // (rotated: each lane on a bank of its own)
            } else {
#pragma unroll
                for (int r = 0; r < kHistCopies; ++r) c += L.top[r * kHistTopCopyWords + i - (kSortPasses - 1) * kRadix];
            }
        } else {
#pragma unroll
            for (int r = 0; r < kHistCopies; ++r) c += L.h[r * kHistCopyWords + i];
        }
        if (c) seen |= atomicAdd(&ghist[i], c);
    }
    // (the additions return a value, and the value is waited for here: they have been performed where every
    //  workgroup sees them before this workgroup counts itself as done.  A fence would do too, but a device-wide
    //  fence writes back the whole L2 of the chiplet, once per workgroup: five times the kernel's run time.)
    asm volatile("" :: "v"(seen));
    // The workgroup that finishes last sees the whole histogram and derives the set of passes that run, once:
    // a pass whose digit takes one value over all keys would move every pair to where it already is (relative
    // to the others) and is skipped.  Bit p of ghist[kSortMaskWord] = pass p runs; if none would (all keys
    // equal) the last one runs anyway, so that the output buffers get written.
    __shared__ uint32_t s_last, constant_mask;
    __syncthreads();
    if (threadIdx.x == 0) {
        s_last = atomicAdd(&ghist[kSortDoneWord], 1u) == gridDim.x - 1 ? 1u : 0u;
        constant_mask = 0u;
    }
    __syncthreads();
    if (!s_last) return;
    for (int i = threadIdx.x; i < kSortPasses * kRadix; i += THREADS)
        if ((int64_t)__hip_atomic_load(&ghist[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == N) atomicOr(&constant_mask, 1u << (i / kRadix));
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t active = ~constant_mask & ((1u << kSortPasses) - 1u);
        if (active == 0u) active = 1u << (kSortPasses - 1);
        ghist[kSortMaskWord] = active;
    }
}

template <typename WORD, int KPT>
__global__ void __launch_bounds__(kSortThreads)
k_onesweep_pass(const float* __restrict__ a, int64_t k, const float* __restrict__ b, float tau,
                uint2* __restrict__ pair0, uint2* __restrict__ pair1,           // (key, id) pairs between passes
                uint32_t* __restrict__ ids_final, float* __restrict__ pk_final,  // the last pass's ids and anchors (the plan's)
                int64_t N, int pass, const uint32_t* __restrict__ ghist, uint32_t* __restrict__ small,
                WORD* status, WORD* status_next)
{
    constexpr int SH = StatusBits<WORD>::shift;
    constexpr WORD kMask = (WORD(1) << SH) - WORD(1);
    constexpr int WAVES = kSortThreads / 64;
    constexpr int kSortTile = kSortThreads * KPT;
    __shared__ uint32_t whist[WAVES][kRadix];     // per-wave digit counts, then offsets
    __shared__ uint32_t tile_start[kRadix];       // first local slot of each digit
    __shared__ uint32_t delta[kRadix];            // global slot of digit d = delta[d] + local slot
    __shared__ uint2 spairs[kSortTile];
    __shared__ uint32_t s_tile, s_active;

    const int tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
    const int shift = pass * kRadixBits;
    // One lane takes the ticket and fetches the pass mask for the workgroup.  (The mask has a cache line
    // of its own: a line that thousands of workgroups update with atomics is slow to read, and a load of
    // it by every wavefront cost more than the rest of the pass.)  A skipped pass takes tickets nobody
    // reads: the counters are per pass and reset with every sort.
    if (tid == 0) {
        s_tile = atomicAdd(&small[kSortTicketWord + pass], 1u);
        s_active = small[kSortMaskWord];
    }
    for (int i = tid; i < WAVES * kRadix; i += kSortThreads) (&whist[0][0])[i] = 0u;
    __syncthreads();
    const uint32_t active = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_active);   // uniform: scalar branches and addresses
    if (!((active >> pass) & 1u)) {     // skipped: only the words of the pass after this one are cleared
        if (status_next && tid < kRadix) status_next[(int64_t)blockIdx.x * kRadix + tid] = WORD(0);
        return;
    }
    // Buffers: the first pass that runs reads the anchors themselves and writes buffer 1, the next
    // reads buffer 1 and writes buffer 0, and so on.  Between passes key and id travel as one 8-byte pair: a
    // digit's run of a tile is then 256 bytes on average instead of 128 in each of two arrays (a copy with nothing
    // but this write pattern runs at 3.1 TB/s on two arrays, as fast as the pass itself used to, and at 4.1 TB/s on
    // pairs), one load and one store per key instead of two.  The last pass that runs writes the ids and the sorted
    // anchors themselves straight into the plan (k_decay adds the sentinels and the decays).
    const int before = __popc(active & ((1u << pass) - 1u));
    const bool first = before == 0;
    const bool last = (active >> pass) == 1u;            // no pass after this one runs
    const uint2* __restrict__ pairs_in = (before & 1) ? pair1 : pair0;
    uint2* __restrict__ pairs_out = (before & 1) ? pair0 : pair1;

    const int64_t tile = s_tile;
    if (status_next && tid < kRadix) status_next[tile * kRadix + tid] = WORD(0);   // words of the pass after this one

    const int64_t tile_base = tile * kSortTile;
    const int64_t wave_base = tile_base + (int64_t)wave * (64 * KPT);
    const int64_t remaining = N - tile_base;
    const uint32_t valid = remaining < kSortTile ? (uint32_t)remaining : (uint32_t)kSortTile;

    uint32_t key[KPT], id[KPT], rank[KPT];
    // two copies of the load loop, chosen once: inside one loop the choice would sit between the loads
    // and keep them from being issued back to back
    if (first) {
#pragma unroll
        for (int i = 0; i < KPT; ++i) {
            const int64_t pos = wave_base + i * 64 + lane;
            const bool ok = pos < N;
            const int64_t pc = ok ? pos : N - 1;
            const uint32_t kk = anchor_key(a, k, b, pc, tau);
            key[i] = ok ? kk : 0xFFFFFFFFu;         // padding sorts last inside the tile
            id[i] = (uint32_t)pc;
        }
    } else {
#pragma unroll
        for (int i = 0; i < KPT; ++i) {
            const int64_t pos = wave_base + i * 64 + lane;
            const bool ok = pos < N;
            const int64_t pc = ok ? pos : N - 1;
            const uint2 kv = pairs_in[pc];
            key[i] = ok ? kv.x : 0xFFFFFFFFu;
            id[i] = kv.y;
        }
    }
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const uint32_t d = (key[i] >> shift) & (kRadix - 1);
        // lanes whose digit differs from this lane's in some bit: per bit, the ballot of the bit XOR this lane's own bit
        uint32_t diff_lo = 0u, diff_hi = 0u;
#pragma unroll
        for (int bit = 0; bit < kRadixBits; ++bit) {
            const uint32_t mine = (uint32_t)(((int32_t)(d << (31 - bit))) >> 31);      // 0 or all ones
            const uint64_t m = __ballot(mine != 0u);
            diff_lo |= (uint32_t)m ^ mine;
            diff_hi |= (uint32_t)(m >> 32) ^ mine;
        }
        const uint64_t peers = ~(((uint64_t)diff_hi << 32) | diff_lo);
        const int leader = __ffsll((long long)peers) - 1;
        uint32_t old = 0;
        if (lane == leader) old = atomicAdd(&whist[wave][d], (uint32_t)__popcll(peers));
        old = __shfl(old, leader);
        rank[i] = old + (uint32_t)__popcll(peers & lt_mask);
    }
    __syncthreads();

    // per digit: exclusive offsets over the wavefronts and the tile's count (padding keys excluded)
    uint32_t digit_total = 0;
    if (tid < kRadix) {
#pragma unroll
        for (int w = 0; w < WAVES; ++w) { const uint32_t c = whist[w][tid]; whist[w][tid] = digit_total; digit_total += c; }
    }
    // Publish this tile's digit counts as soon as they are known (the tiles after this one wait for them).
    constexpr int kLook = 4;      // status words in flight per lane (more cost registers, and with them occupancy)
    uint32_t mine = digit_total;
    WORD* const word = status + tile * kRadix + (tid < kRadix ? tid : 0);
    if (tid < kRadix) {
        if (tid == kRadix - 1) mine -= (uint32_t)kSortTile - valid;        // the padding all has digit 255
        __hip_atomic_store(word, WORD((tile == 0 ? WORD(2) << SH : WORD(1) << SH) | WORD(mine)), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    const uint32_t start = block_exclusive_scan_u32<kSortThreads>(tid < kRadix ? digit_total : 0u, nullptr);
    const uint32_t gbase = block_exclusive_scan_u32<kSortThreads>(tid < kRadix ? ghist[pass * kRadix + tid] : 0u, nullptr);
    // Ask for the status words of the tiles before this one now: the answers travel while the tile is
    // laid out in LDS (a status word crosses the whole device, and with two workgroups per compute unit
    // nothing else would hide that latency).
    WORD ahead[kLook];
    if (tid < kRadix) {
        tile_start[tid] = start;
#pragma unroll
        for (int j = 0; j < kLook; ++j) {
            const int64_t t = tile - 1 - j >= 0 ? tile - 1 - j : 0;
            ahead[j] = __hip_atomic_load(status + t * kRadix + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();

#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const uint32_t d = (key[i] >> shift) & (kRadix - 1);
        const uint32_t slot = tile_start[d] + whist[wave][d] + rank[i];
        spairs[slot] = make_uint2(key[i], id[i]);
    }

    if (tid < kRadix) {
        WORD before = 0;
        bool done = false;
        // one batch of status words, newest tile first; a word not published yet is waited for
        auto take = [&](int64_t t0, const WORD* v) {
#pragma unroll
            for (int j = 0; j < kLook; ++j) {
                const int64_t t = t0 - j;
                if (done || t < 0) continue;
                WORD x = v[j];
                int spins = 0;
                while ((x >> SH) == 0 && spins < kSpinLimit) {
                    __builtin_amdgcn_s_sleep(1);
                    x = __hip_atomic_load(status + t * kRadix + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ++spins;
                }
                if ((x >> SH) == 0) { small[kSortErrorWord] = 1u; done = true; continue; }   // gave up: flag it, never hang
                before += x & kMask;
                if ((x >> SH) == 2) done = true;
            }
        };
        take(tile - 1, ahead);
        // further back, kLook status words in flight at a time (their loads are independent)
        for (int64_t t0 = tile - 1 - kLook; t0 >= 0 && !done; t0 -= kLook) {
            WORD v[kLook];
#pragma unroll
            for (int j = 0; j < kLook; ++j) {
                const int64_t t = t0 - j >= 0 ? t0 - j : 0;
                v[j] = __hip_atomic_load(status + t * kRadix + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            take(t0, v);
        }
        if (tile != 0)
            __hip_atomic_store(word, WORD((WORD(2) << SH) | (before + WORD(mine))), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        delta[tid] = gbase + (uint32_t)before - start;
    }
    __syncthreads();

    if (last) {
#pragma unroll
        for (int i = 0; i < KPT; ++i) {
            const uint32_t slot = (uint32_t)(i * kSortThreads + tid);
            if (slot < valid) {
                const uint2 kv = spairs[slot];
                const uint32_t dst = delta[(kv.x >> shift) & (kRadix - 1)] + slot;
                if ((int64_t)dst < N) {   // always true for consistent offsets; keeps a fault impossible
                    pk_final[dst + 1] = key_to_float(kv.x);      // pk[j + 1]: the anchor of sorted position j
                    ids_final[dst] = kv.y;
                }
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < KPT; ++i) {
            const uint32_t slot = (uint32_t)(i * kSortThreads + tid);
            if (slot < valid) {
                const uint2 kv = spairs[slot];
                const uint32_t dst = delta[(kv.x >> shift) & (kRadix - 1)] + slot;
                if ((int64_t)dst < N) pairs_out[dst] = kv;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Merge path: both anchor arrays ascending.  Among the first `diag` merged
// elements, how many come from a?  (a wins ties, so a[i] precedes b[j] iff
// a[i] <= b[j].)
__device__ __forceinline__ int64_t merge_split(const float* __restrict__ a, int64_t k,
                                               const float* __restrict__ b, int64_t n, int64_t diag, float tau)
{
    int64_t lo = diag > n ? diag - n : 0;
    int64_t hi = diag < k ? diag : k;
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (tau * a[mid] <= tau * b[diag - 1 - mid]) lo = mid + 1; else hi = mid;     // the scaled anchors are what is merged
    }
    return lo;
}

__global__ void __launch_bounds__(kMergeThreads)
k_merge(const float* __restrict__ a, int64_t k, const float* __restrict__ b, int64_t n, float tau,
        uint32_t* __restrict__ keys, uint32_t* __restrict__ ids)
{
    __shared__ float stage[kMergeTile];          // a-part then b-part of this tile
    __shared__ uint32_t okey[kMergeTile], oid[kMergeTile];
    __shared__ int64_t split[2];
    const int64_t N = k + n;
    const int64_t d0 = (int64_t)blockIdx.x * kMergeTile;
    const int64_t d1 = d0 + kMergeTile < N ? d0 + kMergeTile : N;
    if (threadIdx.x < 2) split[threadIdx.x] = merge_split(a, k, b, n, threadIdx.x == 0 ? d0 : d1, tau);
    __syncthreads();
    const int64_t ia0 = split[0], ia1 = split[1];
    const int64_t ib0 = d0 - ia0;
    // sorted inputs give 0 <= na, nb and na + nb = d1 - d0; inputs that are not ascending (the caller's
    // flags were wrong, or NaN anchors) can give anything, so the counts are forced into that range
    // (the result is then meaningless, but every access stays inside the arrays)
    const int span = (int)(d1 - d0);
    int na = (int)((ia1 - ia0) < 0 ? 0 : ((ia1 - ia0) > span ? span : (ia1 - ia0)));
    const int nb = span - na;
    for (int i = threadIdx.x; i < kMergeTile; i += kMergeThreads) {    // slots no rank lands on keep a valid id
        okey[i] = 0xFFFFFFFFu;
        oid[i] = (uint32_t)(d0 + i < N ? d0 + i : 0);
    }
    for (int i = threadIdx.x; i < na + nb; i += kMergeThreads)
        stage[i] = tau * (i < na ? a[ia0 + i] : b[ib0 + (i - na)]);
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
//
// The sorted anchors themselves are kept too (pk, shifted by one between a -inf and a
// +inf sentinel): a decay over more than a handful of rows is never taken as a product
// of these per-row decays but as exp(-(p_end - p_start)).  fp32 anchors make the gaps
// lattice-valued, so the rounding of the per-row decays has a systematic sign and a
// product of tens of thousands of them drifts by 1e-4 and more; key differences
// telescope exactly.  (App. B.1's pair operator adds log-decays for the same reason.)
// Each lane takes four consecutive positions: one 16-byte load of the keys, 16-byte stores of the decays and of
// the anchors (the sorted ids are in the plan already: the sort's last pass, or the merge, wrote them there).  pk[j] holds the anchor of
// position j - 1, so the four anchors a lane stores are the key before its quad and the quad's first three.
// FROM_PK: the sort's last pass has written the sorted anchors into pk[1 .. N] already; this kernel reads them there and
// adds the two sentinels.  Otherwise (the merge of two sorted anchor sets) it starts from the sorted keys.
template <bool FROM_PK>
__global__ void __launch_bounds__(256)
k_decay(const uint32_t* __restrict__ keys, const uint32_t* __restrict__ ghist, float* __restrict__ dh, float* __restrict__ pk,
        float2* __restrict__ pk8, uint32_t* __restrict__ counters, int64_t N)
{
    // list lengths of the scans that follow; and the sort's error flag moves to the plan (the sort's own words are scratch)
    if (blockIdx.x == 0 && threadIdx.x < 64)
        counters[threadIdx.x] = (threadIdx.x == kPlanStatusWord && ghist != nullptr) ? ghist[kSortErrorWord] : 0u;
    const int64_t quads = (N + 2 + 3) / 4;                       // dh has N + 1 entries, pk N + 2
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += stride) {
        const int64_t j0 = 4 * q;
        uint32_t kk[5];                                          // bits of the anchors of positions j0 - 1 .. j0 + 3 (0 where there is none)
        if (FROM_PK) {
            const uint32_t* __restrict__ bits = reinterpret_cast<const uint32_t*>(pk);      // bits[j + 1]: position j
            if (j0 > 0 && j0 + 4 <= N) {
                const uint4 v = reinterpret_cast<const uint4*>(bits)[q];
                kk[0] = v.x; kk[1] = v.y; kk[2] = v.z; kk[3] = v.w; kk[4] = bits[j0 + 4];
            } else {
#pragma unroll
                for (int u = 0; u < 5; ++u) kk[u] = (j0 + u >= 1 && j0 + u <= N) ? bits[j0 + u] : 0u;
            }
        } else {
            kk[0] = j0 > 0 && j0 - 1 < N ? keys[j0 - 1] : 0u;
            if (j0 + 3 < N) {
                const uint4 v = reinterpret_cast<const uint4*>(keys)[q];
                kk[1] = v.x; kk[2] = v.y; kk[3] = v.z; kk[4] = v.w;
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) kk[1 + u] = j0 + u < N ? keys[j0 + u] : 0u;
            }
        }
        float an[5];
#pragma unroll
        for (int u = 0; u < 5; ++u) an[u] = FROM_PK ? __uint_as_float(kk[u]) : key_to_float(kk[u]);
        float d[4], a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = j0 + u;
            d[u] = 0.0f;
            if (j > 0 && j < N) d[u] = kk[1 + u] == kk[u] ? -1.0f : expf(-(an[1 + u] - an[u]));
            a[u] = j == 0 ? __uint_as_float(0xFF800000u) : (j <= N ? an[u] : __uint_as_float(0x7F800000u));
        }
        const bool whole = j0 + 3 < N;
        if (whole) {
            reinterpret_cast<float4*>(dh)[q] = make_float4(d[0], d[1], d[2], d[3]);
            if (!FROM_PK) reinterpret_cast<float4*>(pk)[q] = make_float4(a[0], a[1], a[2], a[3]);
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (j0 + u <= N) dh[j0 + u] = d[u];
                if (!FROM_PK && j0 + u <= N + 1) pk[j0 + u] = a[u];
            }
        }
        if (FROM_PK) {      // the sentinels before the first and after the last anchor
            if (j0 == 0) pk[0] = a[0];
            if (j0 <= N + 1 && N + 1 < j0 + 4) pk[N + 1] = __uint_as_float(0x7F800000u);
        }
        // every eighth anchor with its successor once more, packed (the kernels of the sorted order of batch 1 take their
        // span decays from these instead of touching every sector of pk)
        if (pk8 != nullptr && (q & 1) == 0 && j0 <= N + 1) pk8[q >> 1] = make_float2(a[0], a[1]);
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

__global__ void __launch_bounds__(256)
k_unpair(const float2* __restrict__ pairs, int64_t rows, float* __restrict__ first, int64_t ld_first, float* __restrict__ second)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += stride) {
        const float2 p = pairs[r];
        first[r * ld_first] = p.x;
        second[r] = p.y;
    }
}

inline unsigned grid_for(int64_t work, int threads, int64_t cap = 1 << 16)
{
    int64_t g = (work + threads - 1) / threads;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (unsigned)g;
}

}  // namespace

hipError_t launch_onesweep_sort(const float* a, int64_t k, const float* b, int64_t n, float tau,
                                uint2* pair0, uint2* pair1, uint32_t* ids, float* pk,
                                uint32_t* small, unsigned long long* status, hipStream_t st)
{
    const int64_t N = k + n;
    const int64_t tiles = (N + sort_tile(N) - 1) / sort_tile(N);
    const int64_t words = tiles * kRadix;
    unsigned long long* region[2] = {status, status + words};
    LAPLEX_TIMED("sort_hist", st, hipLaunchKernelGGL(k_sort_reset, dim3(1), dim3(1024), 0, st, small));
    if (N >= kHistBankedMin) {      // one workgroup per compute unit, twice over: each clears and sums 100 KB of counters once
        int64_t hgrid = (N + (int64_t(1) << 16) - 1) >> 16;
        if (hgrid > 256) hgrid = 256;
        LAPLEX_TIMED("sort_hist", st, hipLaunchKernelGGL(k_sort_hist<true>, dim3((unsigned)hgrid), dim3(kHistBankedThreads), 0, st,
                                                         a, k, b, n, tau, small, region[0], words));
    } else {
        int64_t hgrid = (N + sort_hist_tile(N) - 1) / sort_hist_tile(N);
        if (hgrid > 2048) hgrid = 2048;
        LAPLEX_TIMED("sort_hist", st, hipLaunchKernelGGL(k_sort_hist<false>, dim3((unsigned)hgrid), dim3(kSortThreads), 0, st,
                                                         a, k, b, n, tau, small, region[0], words));
    }
    const dim3 grid((unsigned)tiles), block(kSortThreads);
    auto passes = [&](auto kernel, auto* r0, auto* r1) {
        using WORD = std::remove_pointer_t<decltype(r0)>;
        WORD* cur[4] = {r0, r1, r0, r1};
        WORD* nxt[4] = {r1, r0, r1, nullptr};
        for (int p = 0; p < kSortPasses; ++p)
            LAPLEX_TIMED("radix_scatter", st, hipLaunchKernelGGL(kernel, grid, block, 0, st,
                         a, k, b, tau, pair0, pair1, ids, pk, N, p, (const uint32_t*)small, small, cur[p], nxt[p]));
    };
    if (N <= (int64_t(1) << 30)) {
        uint32_t* r = reinterpret_cast<uint32_t*>(status);
        switch (sort_keys_per_thread(N)) {
            case 4:  passes(k_onesweep_pass<uint32_t, 4>, r, r + words); break;
            case 8:  passes(k_onesweep_pass<uint32_t, 8>, r, r + words); break;
            default: passes(k_onesweep_pass<uint32_t, 16>, r, r + words); break;
        }
    } else {
        passes(k_onesweep_pass<unsigned long long, 16>, region[0], region[1]);
    }
    return hipGetLastError();
}

hipError_t launch_merge(const float* a, int64_t k, const float* b, int64_t n, float tau,
                        uint32_t* keys, uint32_t* ids, hipStream_t st)
{
    const int64_t N = k + n;
    const int64_t tiles = (N + kMergeTile - 1) / kMergeTile;
    LAPLEX_TIMED("merge", st, hipLaunchKernelGGL(k_merge, dim3((unsigned)tiles), dim3(kMergeThreads), 0, st, a, k, b, n, tau, keys, ids));
    return hipGetLastError();
}

hipError_t launch_decay(const uint32_t* keys, const uint32_t* ghist, float* dh, float* pk, float2* pk8, uint32_t* counters,
                        int64_t N, hipStream_t st)
{
    const dim3 grid(grid_for((N + 5) / 4, 256)), block(256);
    if (ghist != nullptr) LAPLEX_TIMED("decay", st, hipLaunchKernelGGL(k_decay<true>, grid, block, 0, st, keys, ghist, dh, pk, pk8, counters, N));
    else LAPLEX_TIMED("decay", st, hipLaunchKernelGGL(k_decay<false>, grid, block, 0, st, keys, ghist, dh, pk, pk8, counters, N));
    return hipGetLastError();
}

hipError_t launch_fill(float* p, int64_t rows, int64_t cols, int64_t ld, float v, hipStream_t st)
{
    if (rows <= 0 || cols <= 0) return hipSuccess;
    LAPLEX_TIMED("fill", st, hipLaunchKernelGGL(k_fill, dim3(grid_for(rows * cols, 256)), dim3(256), 0, st, p, rows, cols, ld, v));
    return hipGetLastError();
}

hipError_t launch_unpair(const float* pairs, int64_t rows, float* first, int64_t ld_first, float* second, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    LAPLEX_TIMED("unpair", st, hipLaunchKernelGGL(k_unpair, dim3(grid_for(rows, 256)), dim3(256), 0, st,
                                                  reinterpret_cast<const float2*>(pairs), rows, first, ld_first, second));
    return hipGetLastError();
}

hipError_t launch_copy_u32(const uint32_t* src, uint32_t* dst, int64_t count, hipStream_t st)
{
    if (count <= 0) return hipSuccess;
    LAPLEX_TIMED("copy", st, hipLaunchKernelGGL(k_copy_u32, dim3(grid_for(count, 256)), dim3(256), 0, st, src, dst, count));
    return hipGetLastError();
}

}  // namespace laplex
