// es_fused_kernel.h -- the fused sampling + SpMM kernel (row part, long-row part) and the small kernels that zero its atomic targets.
#ifndef ES_SPMM_FUSED_KERNEL_H
#define ES_SPMM_FUSED_KERNEL_H

#include "es_tile.h"

namespace {

// ---------------------------------------------------------------------------
// Row part of the fused kernel (Algorithm 1) for workgroup `vb` of the row
// grid.  G lanes x CH chunks x VEC floats cover one block of G*CH*VEC feature
// columns (blockIdx.y selects the block).  Rows that keep more than long_k
// entries are left to the long-row part and not stored here.
// ---------------------------------------------------------------------------
template <int G, int CH, int VEC, bool ALIGNED, bool BACKWARD, bool WIDE>
__device__ __forceinline__ void row_block(const Args& a, uint32_t vb, uint2* lds)
{
    constexpr int LOG_G = ilog2(G);
    using P = Pack<VEC, ALIGNED>;

    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int logR = a.logR;
    const int team = kWaveSize >> logR;          // lanes per row
    const int rs = lane >> (6 - logR);           // row slot inside the wave
    const int t = lane & (team - 1);             // lane inside the team
    const int e = t >> LOG_G;                    // edge slot
    const int l = t & (G - 1);                   // column lane
    const int E = team >> LOG_G;                 // edge slots per row (>= 1)
    const int T = kTileSlots >> logR;            // tile slots per row
    uint2* tile = lds + wave * kWaveTileStride + rs * (T + E);   // E pad slots: the rows' reads of slots j .. j+E-1 miss each other's banks

    const int64_t r = ((((int64_t)vb * kWavesPerBlock) + wave) << logR) + rs;
    const bool rvalid = r < a.N;
    int32_t base = 0, n = 0;
    if (rvalid) {
        base = a.rowptr[r];
        n = a.rowptr[r + 1] - base;
    }
    const int k_row = kept_count(a.mode, n, a.W);
    const bool is_long = k_row > a.long_k;       // summed by the long-row part
    const int k = is_long ? 0 : k_row;

    LaneCols<G, CH, VEC, ALIGNED> cols;
    cols.init(blockIdx.y * (G * CH * VEC), l, a.F);

    RowSampler sampler;
    sampler.init(a.mode, a.seed, r, (uint32_t)n, (uint32_t)a.W, (uint32_t)t, (uint32_t)team);

    if (BACKWARD) {
        // transposed product: a.X is the upstream gradient, a.Y the (zeroed) output
        P dy[CH];
        if (k > 0) load_row_chunks<G, CH, VEC, ALIGNED>(a, r, n, k_row, cols, dy);
        for (int t0 = 0; t0 < k; t0 += T) {
            const int count = min(k - t0, T);
            stage_tile<ALIGNED, WIDE>(sampler, t, team, count, base, a.colidx, a.vals, a.stride_units, tile);
            wave_lds_fence();
            scatter_tile<G, CH, VEC, ALIGNED, WIDE>(tile, count, e, E, a.Y, a.ldy, cols, dy);
            wave_lds_fence();
        }
        return;
    }

    P acc[CH];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) acc[ch].zero();

    for (int t0 = 0; t0 < k; t0 += T) {
        const int count = min(k - t0, T);
        stage_tile<ALIGNED, WIDE>(sampler, t, team, count, base, a.colidx, a.vals, a.stride_units, tile);
        wave_lds_fence();
        consume_tile<G, CH, VEC, ALIGNED, WIDE>(tile, count, e, E, a.X, a.ldx, cols, acc);
        wave_lds_fence();
    }

    // ---- sum the E edge slots of each row, store ----------------------------
    for (int m = G; m < team; m <<= 1) {
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) acc[ch].add_xor(m);
    }
    if (rvalid && !is_long && e == 0) {
        float* y = a.Y + r * (int64_t)a.ldy;
        if (a.norm != ES_NORM_NONE) {
            const float f = row_factor(a.norm, n, k_row);
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) acc[ch].scale(f);
        }
#pragma unroll
        for (int ch = 0; ch < CH; ++ch)
            if (cols.ok[ch]) acc[ch].store_streaming(y + cols.off[ch], cols.first[ch]);
    }
}

// ---------------------------------------------------------------------------
// Long-row part.  Workgroup (bx, by) scans rows [bx*1024, bx*1024+1024) for rows
// that keep more than long_k entries, numbers their 256-slot segments with a
// prefix sum in LDS, and its 4 waves take segments gw, gw + 4*kLongSplit, ...
// (gw = by*4 + wave).  A segment is one pass of Algorithm 1 with a whole wave on
// the row; its partial sums are added to Y (zeroed beforehand by
// es_zero_long_rows_kernel) with fp32 atomics, so the summation order across
// segments is not fixed.
// ---------------------------------------------------------------------------
struct LongScratch {
    int seg_end[kLongScanRows];                  // inclusive prefix sum of segment counts
    int wave_total[kWavesPerBlock];
};

template <int G, int CH, int VEC, bool ALIGNED, bool BACKWARD, bool WIDE>
__device__ __forceinline__ void long_block(const Args& a, uint32_t bx, uint32_t by, uint2* lds,
                                           LongScratch& sc)
{
    constexpr int LOG_G = ilog2(G);
    constexpr int kRowsPerThread = kLongScanRows / kBlockThreads;
    using P = Pack<VEC, ALIGNED>;

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid >> 6;
    const int64_t row0 = (int64_t)bx * kLongScanRows;

    // thread tid owns rows row0 + tid*kRowsPerThread + i (consecutive, so the
    // prefix order is the row order)
    int nseg[kRowsPerThread];
    int mine = 0;
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {
        const int64_t r = row0 + tid * kRowsPerThread + i;
        nseg[i] = 0;
        if (r < a.N) {
            const int n = a.rowptr[r + 1] - a.rowptr[r];
            const int k = kept_count(a.mode, n, a.W);
            if (k > a.long_k) nseg[i] = (k + kLongSeg - 1) / kLongSeg;
        }
        mine += nseg[i];
    }
    if (__syncthreads_or(mine) == 0) return;     // no long row among these 1024: the common case
    int incl = mine;                             // inclusive scan inside the wave
#pragma unroll
    for (int d = 1; d < kWaveSize; d <<= 1) {
        const int up = __shfl_up(incl, d, kWaveSize);
        if (lane >= d) incl += up;
    }
    if (lane == kWaveSize - 1) sc.wave_total[wave] = incl;
    __syncthreads();
    int before = incl - mine;
    for (int w = 0; w < wave; ++w) before += sc.wave_total[w];
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {
        before += nseg[i];
        sc.seg_end[tid * kRowsPerThread + i] = before;
    }
    __syncthreads();
    const int total = sc.seg_end[kLongScanRows - 1];
    if (total == 0) return;

    const int e = lane >> LOG_G;
    const int l = lane & (G - 1);
    constexpr int E = kWaveSize / G;
    uint2* tile = lds + wave * kWaveTileStride;
    LaneCols<G, CH, VEC, ALIGNED> cols;
    cols.init(blockIdx.y * (G * CH * VEC), l, a.F);

    const int gw = by * kWavesPerBlock + wave;
    for (int task = gw; task < total; task += kLongSplit * kWavesPerBlock) {
        int lo = 0, hi = kLongScanRows - 1;      // first row whose prefix exceeds task
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (sc.seg_end[mid] > task) hi = mid; else lo = mid + 1;
        }
        const int seg = task - (lo ? sc.seg_end[lo - 1] : 0);
        const int64_t r = row0 + lo;
        const int32_t base = a.rowptr[r];
        const int n = a.rowptr[r + 1] - base;
        const int k = kept_count(a.mode, n, a.W);
        const int t0 = seg * kLongSeg;
        const int count = min(k - t0, kLongSeg);

        RowSampler sampler;
        sampler.init(a.mode, a.seed, r, (uint32_t)n, (uint32_t)a.W, (uint32_t)(t0 + lane), kWaveSize);
        stage_tile<ALIGNED, WIDE>(sampler, lane, kWaveSize, count, base, a.colidx, a.vals, a.stride_units, tile);
        wave_lds_fence();
        if (BACKWARD) {
            P dy[CH];
            load_row_chunks<G, CH, VEC, ALIGNED>(a, r, n, k, cols, dy);
            scatter_tile<G, CH, VEC, ALIGNED, WIDE>(tile, count, e, E, a.Y, a.ldy, cols, dy);
            wave_lds_fence();
            continue;
        }
        P acc[CH];
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) acc[ch].zero();
        consume_tile<G, CH, VEC, ALIGNED, WIDE>(tile, count, e, E, a.X, a.ldx, cols, acc);
        wave_lds_fence();
#pragma unroll
        for (int m = G; m < kWaveSize; m <<= 1) {
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) acc[ch].add_xor(m);
        }
        if (e == 0) {
            float* y = a.Y + r * (int64_t)a.ldy;
            if (a.norm != ES_NORM_NONE) {
                const float f = row_factor(a.norm, n, k);
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) acc[ch].scale(f);
            }
#pragma unroll
            for (int ch = 0; ch < CH; ++ch)
                if (cols.ok[ch]) acc[ch].atomic_add(y + cols.off[ch], cols.first[ch]);
        }
    }
}

// ---------------------------------------------------------------------------
// The fused kernel.  The first a.long_blocks workgroups (dispatched first, so
// the splitting of long rows overlaps the bulk of the rows) run the long-row
// part; the rest run the row part, remapped so that each XCD (hardware deals
// workgroup b to XCD b % 8; long_blocks is a multiple of 8) walks one
// contiguous range of rows.
// ---------------------------------------------------------------------------
template <int G, int CH, int VEC, bool ALIGNED, bool BACKWARD, bool WIDE>
__global__ void __launch_bounds__(kBlockThreads) es_spmm_kernel(const Args a)
{
    __shared__ uint2 lds[kWavesPerBlock * kWaveTileStride];
    __shared__ LongScratch long_scratch;

    if (blockIdx.x < a.long_blocks) {
        long_block<G, CH, VEC, ALIGNED, BACKWARD, WIDE>(a, blockIdx.x / kLongSplit, blockIdx.x % kLongSplit,
                                                  lds, long_scratch);
        return;
    }
    const uint32_t b = blockIdx.x - a.long_blocks;
    const uint32_t vb = (b % kNumXcd) * a.blocks_per_xcd + b / kNumXcd;
    if (vb >= a.nblocks) return;
    row_block<G, CH, VEC, ALIGNED, BACKWARD, WIDE>(a, vb, lds);
}

// Zero-fills an [N x F] matrix with row stride ld (the transposed product
// accumulates into its output with atomics).
__global__ void __launch_bounds__(kBlockThreads)
es_fill_zero_kernel(float* __restrict__ out, int64_t N, int32_t F, int32_t ld)
{
    const int64_t total = N * (int64_t)F;
    for (int64_t i = (int64_t)blockIdx.x * kBlockThreads + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kBlockThreads) {
        const int64_t r = i / F;
        out[r * ld + (i - r * F)] = 0.0f;
    }
}

// Zeroes Y for the rows the long-row part will accumulate into with atomics.
// Each lane tests one row; the wave then clears the flagged rows together, 64
// consecutive floats per store instruction.
__global__ void __launch_bounds__(kBlockThreads) es_zero_long_rows_kernel(const Args a)
{
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int64_t r = (int64_t)blockIdx.x * kBlockThreads + threadIdx.x;
    bool is_long = false;
    if (r < a.N) {
        const int n = a.rowptr[r + 1] - a.rowptr[r];
        is_long = kept_count(a.mode, n, a.W) > a.long_k;
    }
    unsigned long long flagged = __ballot(is_long);
    const int64_t wave_row0 = r - lane;
    while (flagged) {
        const int src = __ffsll((long long)flagged) - 1;
        flagged &= flagged - 1;
        float* y = a.Y + (wave_row0 + src) * (int64_t)a.ldy;
        for (int c = lane; c < a.F; c += kWaveSize) y[c] = 0.0f;
    }
}

}  // namespace

#endif  // ES_SPMM_FUSED_KERNEL_H
