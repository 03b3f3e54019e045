// Device code shared by the kernels that place records into one partition level (permute_kernels.hip:
// the levels themselves; scan_kernels.hip: the batch-1 downsweep, whose results leave as records of the
// first level instead of being written in sorted order and read again).
#pragma once

#include "laplex_internal.h"

namespace laplex {

// LDS of one tile besides the staging array: per-bucket counts, run starts and output offsets.
template <int THREADS>
struct PartShared {
    uint32_t hist[1 << kPermuteMaxBucketBits];      // records of the tile per bucket
    uint32_t lstart[1 << kPermuteMaxBucketBits];    // first LDS slot of each bucket's run
    uint32_t delta[1 << kPermuteMaxBucketBits];     // slot in the chain's output = delta[bucket] + LDS slot
    uint32_t wsum[THREADS / 64];
};

template <int THREADS>
__device__ __forceinline__ uint32_t part_block_scan(uint32_t v, uint32_t* wsum)
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
    for (int w = 0; w < THREADS / 64; ++w) before += w < wave ? wsum[w] : 0u;
    __syncthreads();
    return before + inc - v;
}

// Every thread of the workgroup brings PER records (destination, one or two values; bit i of `ok`: record i exists).
// Two steps, so that a producer can put work between them while the reservations travel:
//
//   partition_reserve  needs the destinations only: the tile's records are ranked per bucket with returning LDS
//                      atomics (any order will do) and thread b reserves the stretch of bucket b's region for the
//                      tile's run with ONE returning device-scope atomic on the bucket's cursor
//   partition_place    the runs are laid out in LDS (sdv: THREADS * PER pairs) and written so that each run goes to
//                      consecutive addresses
//
// `chain` selects the group of 2^bucket_bits regions and cursors (the bucket of the level before; 0 for a first
// level).  Both must be called by all threads of the workgroup.  S must not be touched in between; sdv may alias
// LDS that the caller is done with when it calls partition_place (whose first barrier comes before anything is
// written to it).
template <int PER>
struct PartTicket {
    uint32_t slot[PER];       // rank of record i inside its bucket's run
    uint32_t before, ex;      // thread b: records of bucket b placed before this tile's run; first LDS slot of the run
};

template <int THREADS, int PER>
__device__ __forceinline__ void partition_reserve(const PartEmit& E, int64_t chain, const uint32_t* dest, uint32_t ok,
                                                  PartShared<THREADS>& S, PartTicket<PER>& K)
{
    static_assert((1 << kPermuteMaxBucketBits) <= THREADS, "one thread per bucket");
    static_assert(PER <= 32, "one bit per record");
    const int tid = threadIdx.x;
    const int buckets = 1 << E.bucket_bits;
    const uint32_t digit_mask = (uint32_t)buckets - 1u;
    if (tid < buckets) S.hist[tid] = 0u;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const uint32_t b = (dest[i] >> E.shift) & digit_mask;
        K.slot[i] = ((ok >> i) & 1u) ? atomicAdd(&S.hist[b], 1u) : 0u;
    }
    __syncthreads();
    const uint32_t cnt = tid < buckets ? S.hist[tid] : 0u;
    K.before = 0u;
    if (cnt) K.before = atomicAdd(E.cursor + (chain << E.bucket_bits) + tid, cnt);     // the answer is not waited for here
    K.ex = part_block_scan<THREADS>(cnt, S.wsum);
    if (tid < buckets) S.lstart[tid] = K.ex;
}

template <int THREADS, int PER, int NV>
__device__ __forceinline__ void partition_place(const PartEmit& E, int64_t chain, const uint32_t* dest, uint32_t ok,
                                                const float* v0, const float* v1, PartShared<THREADS>& S, uint2* sdv,
                                                const PartTicket<PER>& K)
{
    const int tid = threadIdx.x;
    const int buckets = 1 << E.bucket_bits;
    const uint32_t digit_mask = (uint32_t)buckets - 1u;
    __syncthreads();
    uint32_t place[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        place[i] = S.lstart[(dest[i] >> E.shift) & digit_mask] + K.slot[i];
        if ((ok >> i) & 1u) sdv[place[i]] = make_uint2(dest[i], __float_as_uint(v0[i]));
    }
    // first record of the bucket's region, relative to the chain's first region, minus the run's LDS slot
    if (tid < buckets) S.delta[tid] = ((uint32_t)tid << E.region_shift) + K.before - K.ex;
    __syncthreads();

    const uint32_t total = S.lstart[buckets - 1] + S.hist[buckets - 1];
    const int64_t chain_base = (chain << E.bucket_bits) << E.region_shift;
    const uint32_t region = 1u << E.region_shift;
    uint32_t where[PER];          // offset inside the chain's output (2^bucket_bits regions: below 2^32), or none
    constexpr uint32_t kNone = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const uint32_t s = (uint32_t)(i * THREADS + tid);
        where[i] = kNone;
        if (s < total) {
            const uint2 dv = sdv[s];
            const uint32_t b = (dv.x >> E.shift) & digit_mask;
            const uint32_t off = S.delta[b] + s;
            if (off - (b << E.region_shift) < region) {                         // a region never overflows for a permutation
                where[i] = off;
                E.out_dv[chain_base + off] = dv;
            }
        }
    }
    if (NV == 2) {          // the second values through the same LDS array
        float* const sv = reinterpret_cast<float*>(sdv);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if ((ok >> i) & 1u) sv[place[i]] = v1[i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (where[i] != kNone) E.out_v1[chain_base + where[i]] = sv[i * THREADS + tid];
    }
}

// The same two steps for a producer that is short of registers between them: the destinations go to their LDS slots at
// once (sd: THREADS * PER words that nobody touches until partition_place_split is through) and a thread keeps only its
// records' slots; the values follow through sv (THREADS * PER floats, which may alias LDS the caller is done with when it
// calls partition_place_split).
template <int PER>
struct PartSplitTicket {
    static_assert(PER % 2 == 0, "two slots per word");
    uint32_t slot2[PER / 2];  // LDS slots of records 2i (low half) and 2i + 1 (high half)
    uint32_t before, ex;
    __device__ __forceinline__ uint32_t slot(int i) const { return (i & 1) ? slot2[i >> 1] >> 16 : slot2[i >> 1] & 0xFFFFu; }
};

template <int THREADS, int PER>
__device__ __forceinline__ void partition_reserve_split(const PartEmit& E, int64_t chain, const uint32_t* dest, uint32_t ok,
                                                        PartShared<THREADS>& S, uint32_t* sd, PartSplitTicket<PER>& K)
{
    static_assert(THREADS * PER <= 65536, "a slot fits 16 bits");
    PartTicket<PER> T;
    partition_reserve<THREADS, PER>(E, chain, dest, ok, S, T);
    K.before = T.before; K.ex = T.ex;
    const uint32_t digit_mask = (1u << E.bucket_bits) - 1u;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const uint32_t slot = ((ok >> i) & 1u) ? T.slot[i] + S.lstart[(dest[i] >> E.shift) & digit_mask] : 0u;
        if ((ok >> i) & 1u) sd[slot] = dest[i];
        if (i & 1) K.slot2[i >> 1] |= slot << 16; else K.slot2[i >> 1] = slot;
    }
}

template <int THREADS, int PER, int NV>
__device__ __forceinline__ void partition_place_split(const PartEmit& E, int64_t chain, uint32_t ok, const float* v0, const float* v1,
                                                      PartShared<THREADS>& S, const uint32_t* sd, float* sv, const PartSplitTicket<PER>& K)
{
    const int tid = threadIdx.x;
    const int buckets = 1 << E.bucket_bits;
    const uint32_t digit_mask = (uint32_t)buckets - 1u;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PER; ++i)
        if ((ok >> i) & 1u) sv[K.slot(i)] = v0[i];
    if (tid < buckets) S.delta[tid] = ((uint32_t)tid << E.region_shift) + K.before - K.ex;
    __syncthreads();

    const uint32_t total = S.lstart[buckets - 1] + S.hist[buckets - 1];
    const int64_t chain_base = (chain << E.bucket_bits) << E.region_shift;
    const uint32_t region = 1u << E.region_shift;
    uint32_t where[PER];
    constexpr uint32_t kNone = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const uint32_t s = (uint32_t)(i * THREADS + tid);
        where[i] = kNone;
        if (s < total) {
            const uint32_t d = sd[s];
            const uint32_t b = (d >> E.shift) & digit_mask;
            const uint32_t off = S.delta[b] + s;
            if (off - (b << E.region_shift) < region) {
                where[i] = off;
                E.out_dv[chain_base + off] = make_uint2(d, __float_as_uint(sv[s]));
            }
        }
    }
    if (NV == 2) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if ((ok >> i) & 1u) sv[K.slot(i)] = v1[i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (where[i] != kNone) E.out_v1[chain_base + where[i]] = sv[i * THREADS + tid];
    }
}

}  // namespace laplex
