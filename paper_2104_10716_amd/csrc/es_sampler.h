// es_sampler.h -- the per-row edge sampler (Section 4.4 of the paper) and the wave-level LDS ordering helper.
#ifndef ES_SPMM_SAMPLER_H
#define ES_SPMM_SAMPLER_H

#include "es_common.h"

namespace {

// ---------------------------------------------------------------------------
// Sampler (Section 4.4).  One instance per lane walks the slots
// first, first + stride, first + 2*stride, ... of one row and returns the entry
// number inside the row for each.  Bucket / full / short rows: the slot number
// itself.  FastRand on a long row: (off + slot * P) mod n, kept incrementally
// (one add and one conditional subtract per slot instead of a modulo).
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint64_t splitmix64_output(uint64_t seed, uint64_t count)
{
    // `count`-th output (1-based) of SplitMix64 seeded with `seed`
    uint64_t z = seed + count * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// FastRand multiplier of a row of n entries: 577 (Equation 2), or the first of
// the next primes that does not divide n, so that the picks stay distinct.
__device__ __forceinline__ uint32_t fastrand_multiplier(uint32_t n)
{
    return (n % 577u) ? 577u : (n % 587u) ? 587u : (n % 593u) ? 593u : 599u;
}

// Per-row rotation of the FastRand picks: 0 for seed 0 (exactly Equation 2).
__device__ __forceinline__ uint32_t fastrand_offset(uint64_t seed, int64_t row, uint32_t n)
{
    if (seed == 0) return 0u;
    return (uint32_t)(splitmix64_output(seed, (uint64_t)row + 1u) >> 32) % n;
}

struct RowSampler {
    uint32_t idx;    // entry number the next call returns
    uint32_t step;   // increment per call, already reduced mod n
    uint32_t wrap;   // n for FastRand, 0xFFFFFFFF when no wrap can happen

    // requires stride <= 64
    __device__ __forceinline__ void init(int mode, uint64_t seed, int64_t row, uint32_t n,
                                         uint32_t W, uint32_t first, uint32_t stride)
    {
        if (mode != ES_FASTRAND || n <= W) {
            idx = first;
            step = stride;
            wrap = 0xFFFFFFFFu;
            return;
        }
        const uint32_t P = fastrand_multiplier(n);
        const uint32_t off = fastrand_offset(seed, row, n);
        if (first < 65536u)
            idx = (off + (first * P) % n) % n;               // both terms < n < 2^31
        else
            idx = (uint32_t)(((uint64_t)off + (uint64_t)first * P) % n);
        step = (stride * P) % n;
        wrap = n;
    }

    __device__ __forceinline__ uint32_t next()
    {
        const uint32_t cur = idx;
        uint32_t nx = idx + step;          // < 2n < 2^32
        if (nx >= wrap) nx -= wrap;
        idx = nx;
        return cur;
    }
};

// Stage 1 for one tile: lane t of a team of `team` lanes handles slots
// t, t + team, ... < count and hands (slot, entry number) to the sink.
template <class Sink>
__device__ __forceinline__ void sample_tile(RowSampler& s, int t, int team, int count, Sink&& sink)
{
    for (int i = t; i < count; i += team) sink(i, s.next());
}

// Orders a wave's LDS writes before its later LDS reads (and the reverse for
// tile reuse).  The hardware executes one wave's LDS operations in order; this
// only stops the compiler from moving them across.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace

#endif  // ES_SPMM_SAMPLER_H
