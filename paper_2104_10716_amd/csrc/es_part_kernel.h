// es_part_kernel.h -- the column-partitioned form of the fused kernel: every XCD gathers from one eighth of X only.
#ifndef ES_SPMM_PART_KERNEL_H
#define ES_SPMM_PART_KERNEL_H

#include "es_tile.h"

namespace {

// ---------------------------------------------------------------------------
// Why: stage 2 of Algorithm 1 gathers one row of X per kept entry, and X is far
// larger than one XCD's 4 MB L2, so nearly every gather misses.  Here the
// columns of A are cut into kParts = 8 equal ranges and XCD p only ever
// multiplies entries whose column lies in range p, i.e. it only touches one
// eighth of X.  A row's sum is then built in kParts launches ("phases"): in
// phase t XCD p serves the rows of row range (p + t) mod 8 with column range p,
// so that inside one launch every row belongs to exactly one workgroup and Y
// can be updated with plain loads and stores (phase 0 stores, later phases
// add); the stream orders the phases.  The sum of a row is the same set of
// products as in the unpartitioned kernel, added in a fixed order, so results
// are bit-reproducible.
//
// A row's share of range p is the piece [cuts[r][p], cuts[r][p+1]) of its
// entries, found by binary search for the range bounds (es_cuts_kernel).  The
// cuts are forced to be non-decreasing inside [0, n], so the eight pieces tile
// the row whatever order its columns are stored in: every kept entry is
// multiplied exactly once.  Rows stored in increasing column order -- the usual
// CSR -- get the locality; other rows only lose it.
//
// A piece is short (an eighth of a row), so per-piece instructions and the chain
// "row pointers -> entries -> rows of X" weigh far more than in the plain
// kernel.  A wave therefore serves kPartGroups consecutive rows, one at a time
// with all 64 lanes: their row pointers and cuts are requested at once, and the
// first entries of row i+1 are requested before the rows of X of row i, so that
// only the gathers stay on the critical path.
//
// Degrees are skewed, so some pieces are a hundred times longer than the typical
// one, and a wave that starts such a piece near the end of a launch would keep
// the whole chip waiting for it -- eight times per call.  Every launch
// therefore sweeps its rows twice: the leading half of the grid serves only the
// pieces longer than a.long_k (most of its workgroups find none and leave at
// once), the trailing half serves the rest.  The long pieces thus start first
// and run beside the bulk of the work; each piece still has exactly one owner.
// ---------------------------------------------------------------------------
constexpr int kPartGroups = 4;       // consecutive rows one wave serves
constexpr int kPartPrefetch = 2;     // entries per lane requested one group ahead

// Eight lanes per row: lane j finds the first entry whose column is >= j * part_cols.
__global__ void __launch_bounds__(kBlockThreads)
es_cuts_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx, int64_t N,
               int32_t part_cols, int32_t* __restrict__ cuts)
{
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int j = lane & (kParts - 1);
    const int64_t r = ((int64_t)blockIdx.x * kBlockThreads + threadIdx.x) / kParts;
    int32_t base = 0, n = 0;
    if (r < N) {
        base = rowptr[r];
        n = rowptr[r + 1] - base;
    }
    const int32_t bound = j * part_cols;             // j <= 7, part_cols <= 2^28
    int32_t lo = 0, hi = (j == 0) ? 0 : n;           // lower bound of `bound` in the row
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if (colidx[(int64_t)base + mid] < bound) lo = mid + 1; else hi = mid;
    }
    // running maximum over the row's eight lanes: pieces tile [0, n] for any column order
#pragma unroll
    for (int d = 1; d < kParts; d <<= 1) {
        const int32_t up = __shfl_up(lo, d, kParts);
        if (j >= d) lo = max(lo, up);
    }
    if (r < N) cuts[r * kParts + j] = lo;
}

// Entries of one row's piece requested ahead of time.
struct AheadEntries {
    int32_t col[kPartPrefetch];
    float val[kPartPrefetch];
    bool keep[kPartPrefetch];
};

// Row part of phase a.phase: workgroup `vb` of the row grid, column range `part`.
// One row per wave at a time (the path is only taken for rows with hundreds of
// entries), all 64 lanes on the row: E = 64 / G edge slots.
template <int G, int CH, int VEC, bool ALIGNED, bool WIDE>
__device__ __forceinline__ void part_row_block(const Args& a, uint32_t vb, int part, bool long_sweep,
                                               uint2* lds)
{
    constexpr int LOG_G = ilog2(G);
    constexpr int E = kWaveSize / G;             // edge slots per row
    constexpr int B = kPartGroups;
    constexpr int PF = kPartPrefetch;
    constexpr int T = kTileSlots;
    using P = Pack<VEC, ALIGNED>;
    using K = RowKey<ALIGNED, WIDE>;

    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int e = lane >> LOG_G;                 // edge slot
    const int l = lane & (G - 1);                // column lane
    uint2* tile = lds + wave * kWaveTileStride;
    const unsigned long long below_me = (1ull << lane) - 1ull;
    const bool accumulate = a.phase != 0;        // phase 0 starts every row from zero
    const bool fastrand = a.mode == ES_FASTRAND;

    LaneCols<G, CH, VEC, ALIGNED> cols;
    cols.init(blockIdx.y * (G * CH * VEC), l, a.F);

    // ---- row pointers and cuts of all B rows, one round trip -----------------
    const int64_t row0 = ((int64_t)vb * kWavesPerBlock + wave) * B;
    int32_t base[B], n[B], lo[B], hi[B];
    int32_t slots[B];          // sampler slots to walk for the piece; 0 when the other sweep owns it
    bool mine[B];
    bool any = false;
#pragma unroll
    for (int i = 0; i < B; ++i) {
        const int64_t r = row0 + i;
        base[i] = 0; n[i] = 0; lo[i] = 0; hi[i] = 0;
        if (r < a.N) {
            base[i] = a.rowptr[r];
            n[i] = a.rowptr[r + 1] - base[i];
            const int32_t* cr = a.cuts + r * kParts;
            lo[i] = cr[part];
            hi[i] = (part + 1 < kParts) ? cr[part + 1] : n[i];
        }
        const bool strided = fastrand && n[i] > a.W;
        const int piece = hi[i] - lo[i];
        const int k_row = kept_count(a.mode, n[i], a.W);
        mine[i] = r < a.N && (min(piece, k_row) > a.long_k) == long_sweep;
        slots[i] = !mine[i] ? 0 : strided ? (piece > 0 ? k_row : 0) : piece;
        any = any || mine[i];
    }
    if (!any) return;                            // wave-uniform (the long sweep's usual case)

    // Requests the first PF entries per lane of row i's piece.  Contiguous
    // pieces (exact product, or a row kept whole): entries lo + slot.  FastRand
    // on a longer row: the slots' entry numbers, kept when they fall in [lo, hi).
    auto request = [&](int i, RowSampler& sampler, AheadEntries& ah) {
        const bool strided = fastrand && n[i] > a.W;
        if (strided) sampler.init(a.mode, a.seed, row0 + i, (uint32_t)n[i], (uint32_t)a.W, (uint32_t)lane, kWaveSize);
        else sampler.init(ES_FULL, 0, row0 + i, (uint32_t)n[i], 0u, (uint32_t)lane, kWaveSize);
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            const int slot = lane + j * kWaveSize;
            ah.keep[j] = false;
            ah.col[j] = 0;
            ah.val[j] = 0.0f;
            if (slot < min(slots[i], T)) {
                const int32_t entry = (int32_t)sampler.next();
                const bool keep = strided ? (entry >= lo[i] && entry < hi[i]) : true;
                if (keep) {
                    const int64_t p = (int64_t)base[i] + (strided ? entry : lo[i] + entry);
                    ah.col[j] = a.colidx[p];
                    ah.val[j] = a.vals ? a.vals[p] : 1.0f;
                }
                ah.keep[j] = keep;
            }
        }
    };

    // Stages slots [s0, s0 + count) of row i's piece behind the `fill` entries
    // already in the tile; returns the new fill.  Contiguous pieces keep every
    // slot, so slot numbers are tile positions; strided ones are packed.
    auto stage_more = [&](int i, RowSampler& walk, int first, int count, int fill) {
        const bool strided = fastrand && n[i] > a.W;
        for (int i0 = first; i0 < count; i0 += kWaveSize) {
            const bool valid = i0 + lane < count;
            const int32_t entry = (int32_t)walk.next();
            const bool keep = valid && (strided ? (entry >= lo[i] && entry < hi[i]) : true);
            int at = i0 + lane;
            if (strided) {
                const unsigned long long m = __ballot(keep);
                at = fill + __popcll(m & below_me);
                fill += __popcll(m);
            }
            if (keep) {
                const int64_t p = (int64_t)base[i] + (strided ? entry : lo[i] + entry);
                const float v = a.vals ? a.vals[p] : 1.0f;
                tile[at] = make_uint2(K::make(a.colidx[p], a.stride_units), __float_as_uint(v));
            }
        }
        return strided ? fill : count;
    };

    RowSampler sampler;
    AheadEntries ahead;
    request(0, sampler, ahead);

#pragma unroll
    for (int i = 0; i < B; ++i) {
        const int64_t r = row0 + i;
        const bool strided = fastrand && n[i] > a.W;
        const int k_row = kept_count(a.mode, n[i], a.W);
        float* y = a.Y + r * (int64_t)a.ldy;

        // ---- first tile: the entries requested ahead, then the rest of it ------
        const int count0 = min(slots[i], T);
        int fill = 0;                            // entries in the tile (wave-uniform)
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            if (j * kWaveSize < count0) {
                int at = lane + j * kWaveSize;
                if (strided) {
                    const unsigned long long m = __ballot(ahead.keep[j]);
                    at = fill + __popcll(m & below_me);
                    fill += __popcll(m);
                }
                if (ahead.keep[j])
                    tile[at] = make_uint2(K::make(ahead.col[j], a.stride_units), __float_as_uint(ahead.val[j]));
            }
        }
        if (!strided) fill = min(count0, PF * kWaveSize);
        RowSampler walk = sampler;               // continues after the PF slots already taken
        fill = stage_more(i, walk, PF * kWaveSize, count0, fill);
        wave_lds_fence();

        // ---- the row's earlier partial sums, and the next row's entries --------
        P prev[CH];
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) prev[ch].zero();
        if (accumulate && mine[i] && e == 0 && slots[i] > 0) {
#pragma unroll
            for (int ch = 0; ch < CH; ++ch)
                if (cols.ok[ch]) prev[ch].load(y + cols.off[ch]);
        }
        if (i + 1 < B) request(i + 1, sampler, ahead);

        P acc[CH];
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) acc[ch].zero();
        bool touched = fill > 0;                 // wave-uniform: the piece holds a kept entry
        consume_tile<G, CH, VEC, ALIGNED, WIDE>(tile, fill, e, E, a.X, a.ldx, cols, acc);
        wave_lds_fence();

        // ---- further tiles of a long piece --------------------------------------
        for (int t0 = T; t0 < slots[i]; t0 += T) {
            fill = stage_more(i, walk, 0, min(slots[i] - t0, T), 0);
            touched = touched || fill > 0;
            wave_lds_fence();
            consume_tile<G, CH, VEC, ALIGNED, WIDE>(tile, fill, e, E, a.X, a.ldx, cols, acc);
            wave_lds_fence();
        }

        // ---- sum the E edge slots, update Y ---------------------------------------
#pragma unroll
        for (int m = G; m < kWaveSize; m <<= 1) {
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) acc[ch].add_xor(m);
        }
        if (mine[i] && e == 0 && (touched || !accumulate)) {
            if (a.norm != ES_NORM_NONE) {
                const float f = row_factor(a.norm, n[i], k_row);
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) acc[ch].scale(f);
            }
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) {
                if (!cols.ok[ch]) continue;
                acc[ch].add(prev[ch]);
                acc[ch].store(y + cols.off[ch], cols.first[ch]);
            }
        }
    }
}

// One phase of the column-partitioned product.  Workgroup b runs on XCD
// p = b % 8 (hardware deals workgroups round-robin; only the speed depends on
// it, not the result) and serves column range p for the rows of row range
// (p + phase) % 8.
template <int G, int CH, int VEC, bool ALIGNED, bool WIDE>
__global__ void __launch_bounds__(kBlockThreads) es_spmm_part_kernel(const Args a)
{
    __shared__ uint2 lds[kWavesPerBlock * kWaveTileStride];
    const bool long_sweep = blockIdx.x < a.long_blocks;          // a.long_blocks is a multiple of 8
    const uint32_t b = long_sweep ? blockIdx.x : blockIdx.x - a.long_blocks;
    const uint32_t p = b % kNumXcd;
    const uint32_t q = b / kNumXcd;
    const uint32_t s = (p + (uint32_t)a.phase) % kNumXcd;
    const uint32_t vb = s * a.blocks_per_xcd + q;
    if (vb >= a.nblocks) return;
    part_row_block<G, CH, VEC, ALIGNED, WIDE>(a, vb, (int)p, long_sweep, lds);
}

}  // namespace

#endif  // ES_SPMM_PART_KERNEL_H
