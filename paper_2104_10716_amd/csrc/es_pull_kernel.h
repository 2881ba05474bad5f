// es_pull_kernel.h -- the transposed sampled product as a gather over the transposed graph (no atomics).
#ifndef ES_SPMM_PULL_KERNEL_H
#define ES_SPMM_PULL_KERNEL_H

#include "es_tile.h"

namespace {

// ---------------------------------------------------------------------------
// dX = sample_W(A)^T dY without scattering: row c of the output sums, over the
// STORED entries (r, c) of A, the ones the sampler keeps for row r.  The
// transposed graph (built once per graph by es_spmm_transpose_graph) lists for
// every column c its entries as (row r, entry number idx inside row r, value).
// Whether the forward pass keeps entry idx of a row of n entries follows from
// inverting the sampling rule (Section 4.4):
//     full, or n <= W       kept
//     Bucket                kept iff idx < W
//     FastRand, n > W       slot i reads entry (off + i*P) mod n, so entry idx is
//                           read by slot i = ((idx - off) * P^-1) mod n
//                                          = (slot0 - shift) mod n,
//                           slot0 = idx * P^-1 mod n   (per entry, stored: it does
//                                                       not depend on W or the seed)
//                           shift = off * P^-1 mod n   (per row, recomputed per call
//                                                       from the seed: es_pull_rows_kernel)
//                           kept iff i < W.
// So one structure serves every W, mode and seed (a new seed per training
// iteration costs one pass over the rows), the per-entry test is a subtract and
// two compares, and the result is bit-reproducible.
// ---------------------------------------------------------------------------

// (a * b) mod n for a, b < n < 2^31: quotient estimated in double (off by at
// most one), remainder fixed up in integers.
__device__ __forceinline__ uint32_t mulmod31(uint32_t a, uint32_t b, uint32_t n)
{
    const uint64_t prod = (uint64_t)a * b;
    const uint64_t q = (uint64_t)((double)a * (double)b / (double)n);
    int64_t rem = (int64_t)(prod - q * n);
    if (rem < 0) rem += n;
    if (rem < 0) rem += n;
    if (rem >= (int64_t)n) rem -= n;
    if (rem >= (int64_t)n) rem -= n;
    return (uint32_t)rem;
}

// Inverse of the row's FastRand multiplier modulo its length (extended Euclid;
// the multiplier is coprime to n by construction).  One thread per row.
__global__ void __launch_bounds__(kBlockThreads)
es_pinv_kernel(const int32_t* __restrict__ rowptr, int64_t N, int32_t* __restrict__ pinv)
{
    const int64_t r = (int64_t)blockIdx.x * kBlockThreads + threadIdx.x;
    if (r >= N) return;
    const int64_t n = (int64_t)rowptr[r + 1] - rowptr[r];
    int64_t inv = 0;
    if (n > 1) {
        int64_t a = fastrand_multiplier((uint32_t)n) % n, b = n, x0 = 1, x1 = 0;   // a*x0 = a (mod n), a*x1 = b
        while (b != 0) {
            const int64_t q = a / b;
            int64_t t = a - q * b; a = b; b = t;
            t = x0 - q * x1; x0 = x1; x1 = t;
        }
        inv = x0 % n;                                   // a == gcd == 1 here
        if (inv < 0) inv += n;
    }
    pinv[r] = (int32_t)inv;
}

// After the transposed fill: turn every entry's CSR position into its entry
// number inside its row (in place) and store the slot that reads it under
// Equation 2 without rotation.
__global__ void __launch_bounds__(kBlockThreads)
es_pull_entries_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ pinv,
                       const int32_t* __restrict__ t_row, int64_t nnz, int32_t* __restrict__ t_idx,
                       int32_t* __restrict__ t_slot)
{
    for (int64_t j = (int64_t)blockIdx.x * kBlockThreads + threadIdx.x; j < nnz;
         j += (int64_t)gridDim.x * kBlockThreads) {
        const int32_t r = t_row[j];
        const int32_t base = rowptr[r];
        const uint32_t n = (uint32_t)(rowptr[r + 1] - base);
        const uint32_t idx = (uint32_t)(t_idx[j] - base);
        t_idx[j] = (int32_t)idx;
        t_slot[j] = n > 1 ? (int32_t)mulmod31(idx, (uint32_t)pinv[r], n) : 0;
    }
}

// Per call: rows[r] = (n, shift) with shift = off * P^-1 mod n for this seed.
__global__ void __launch_bounds__(kBlockThreads)
es_pull_rows_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ pinv, int64_t N,
                    int32_t mode, uint64_t seed, int32_t W, int2* __restrict__ rows)
{
    const int64_t r = (int64_t)blockIdx.x * kBlockThreads + threadIdx.x;
    if (r >= N) return;
    const uint32_t n = (uint32_t)(rowptr[r + 1] - rowptr[r]);
    uint32_t shift = 0;
    if (mode == ES_FASTRAND && n > (uint32_t)W && seed != 0)
        shift = mulmod31(fastrand_offset(seed, r, n), (uint32_t)pinv[r], n);
    rows[r] = make_int2((int)n, (int)shift);
}

// One wave per output row c, E = 64 / G edge slots.  Stage 1 reads the row's
// transposed entries 64 at a time, tests them, and packs the kept ones
// (row of dY as its key, value times the forward row factor) into the LDS tile;
// stage 2 is the forward kernel's gather.
template <int G, int CH, int VEC, bool ALIGNED, bool WIDE>
__global__ void __launch_bounds__(kBlockThreads)
es_pull_kernel(const Args a, const int32_t* __restrict__ t_ptr, const int32_t* __restrict__ t_row,
               const int32_t* __restrict__ t_idx, const int32_t* __restrict__ t_slot,
               const float* __restrict__ t_vals, const int2* __restrict__ rows)
{
    __shared__ uint2 lds[kWavesPerBlock * kWaveTileStride];
    constexpr int LOG_G = ilog2(G);
    constexpr int E = kWaveSize / G;
    constexpr int T = kTileSlots;
    using P = Pack<VEC, ALIGNED>;
    using K = RowKey<ALIGNED, WIDE>;

    // consecutive output rows go to different XCDs: under Bucket the kept entries
    // crowd into the lowest-numbered columns, and those rows are the whole work
    const uint32_t vb = blockIdx.x;
    if (vb >= a.nblocks) return;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int e = lane >> LOG_G;
    const int l = lane & (G - 1);
    uint2* tile = lds + wave * kWaveTileStride;
    const unsigned long long below_me = (1ull << lane) - 1ull;

    const int64_t c = (int64_t)vb * kWavesPerBlock + wave;
    if (c >= a.N) return;
    const int32_t begin = t_ptr[c];
    const int32_t count = t_ptr[c + 1] - begin;

    LaneCols<G, CH, VEC, ALIGNED> cols;
    cols.init(blockIdx.y * (G * CH * VEC), l, a.F);
    P acc[CH];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) acc[ch].zero();

    // kPullChunks * 64 entries per pass: all their loads are issued before the
    // first test, so that one pass costs two memory round trips, not sixteen
    constexpr int kPullChunks = 8;
    const bool need_rows = (a.mode == ES_FASTRAND && a.seed != 0) || a.norm != ES_NORM_NONE;
    int fill = 0;
    for (int j0 = 0; j0 < count; j0 += kPullChunks * kWaveSize) {
        int32_t r[kPullChunks], pick[kPullChunks];
        float v[kPullChunks];
        bool valid[kPullChunks];
#pragma unroll
        for (int q = 0; q < kPullChunks; ++q) {
            const int jj = j0 + q * kWaveSize + lane;
            valid[q] = jj < count;
            const int64_t j = (int64_t)begin + (valid[q] ? jj : 0);
            r[q] = t_row[j];
            v[q] = t_vals[j];
            pick[q] = a.mode == ES_BUCKET ? t_idx[j] : a.mode == ES_FASTRAND ? t_slot[j] : 0;
        }
        // A row's length and rotation are only needed for a rotated FastRand
        // (seed != 0) and for the row factor: without rotation the stored slot
        // (or entry number) is below n, so "n <= W or slot < W" is just "slot < W".
        int2 info[kPullChunks];
#pragma unroll
        for (int q = 0; q < kPullChunks; ++q) info[q] = need_rows ? rows[r[q]] : make_int2(INT32_MAX, 0);
#pragma unroll
        for (int q = 0; q < kPullChunks; ++q) {
            const uint32_t n = (uint32_t)info[q].x;
            int32_t slot = pick[q];                      // Bucket: entry number; FastRand: slot after rotation
            if (a.mode == ES_FASTRAND) {
                slot -= info[q].y;
                if (slot < 0) slot += (int32_t)n;
            }
            const bool keep = valid[q] && (n <= (uint32_t)a.W || (uint32_t)slot < (uint32_t)a.W);
            const unsigned long long m = __ballot(keep);
            if (keep) {
                const int k = kept_count(a.mode, (int)n, a.W);
                const float w = v[q] * row_factor(a.norm, (int)n, k);
                tile[fill + __popcll(m & below_me)] = make_uint2(K::make(r[q], a.stride_units), __float_as_uint(w));
            }
            fill += __popcll(m);
        }
        if (fill > T - kPullChunks * kWaveSize) {        // the next pass might not fit: gather what is staged
            wave_lds_fence();
            consume_tile<G, CH, VEC, ALIGNED, WIDE>(tile, fill, e, E, a.X, a.ldx, cols, acc);
            wave_lds_fence();
            fill = 0;
        }
    }
    wave_lds_fence();
    consume_tile<G, CH, VEC, ALIGNED, WIDE>(tile, fill, e, E, a.X, a.ldx, cols, acc);

#pragma unroll
    for (int m = G; m < kWaveSize; m <<= 1) {
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) acc[ch].add_xor(m);
    }
    if (e == 0) {
        float* y = a.Y + c * (int64_t)a.ldy;
#pragma unroll
        for (int ch = 0; ch < CH; ++ch)
            if (cols.ok[ch]) acc[ch].store(y + cols.off[ch], cols.first[ch]);
    }
}

}  // namespace

#endif  // ES_SPMM_PULL_KERNEL_H
