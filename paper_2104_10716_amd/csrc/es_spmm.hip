// es_spmm.hip -- edge-sampled SpMM for gfx950 (MI355X), C ABI in include/es_spmm.h.
//
// Paper: Algorithm 1 ("CacheSample"): stage 1 samples at most W entries of each
// CSR row into on-chip memory (Section 4.2, sampling rules of Section 4.4 /
// Equation 2), stage 2 multiplies the staged entries with gathered rows of the
// dense matrix (Section 4.3).
//
// Mapping to CDNA4 (differs from the paper's 512-thread CUDA blocks on purpose):
//   * A wavefront (64 lanes) owns R = 2^logR consecutive rows.  The 64/R lanes of
//     a row ("team") are E x G: G lanes span the feature columns with VEC-wide
//     loads (CH column chunks per lane), E edge slots run side by side and are
//     summed with cross-lane shuffles at the end.
//   * Each wave has a private LDS tile of kTileSlots (column, value) pairs,
//     T = kTileSlots/R per row.  Stage 1: the team's lanes evaluate the sampler
//     for slots t, t+64/R, ... and copy (colidx, vals) into the tile.  Stage 2:
//     lanes read a slot as one 64-bit LDS broadcast and issue U independent
//     VEC-wide global loads of X before the first FMA.  Rows longer than a tile
//     (full mode, or W > T) refill the tile; no barrier other than wave-level
//     ordering is needed because a tile is private to its wave.
//   * Workgroup ids are remapped so each of the 8 XCDs (one L2 each) walks one
//     contiguous range of rows.
//   * Rows that keep more than `long_k` entries (full mode on skewed graphs, or a
//     very large W) would leave one wave running long after the rest of the grid
//     has drained.  The leading workgroups of the launch split each such row
//     into 256-slot segments, deal the segments to the waves of kLongSplit
//     workgroups and add the partial sums to Y with fp32 atomics (a small
//     kernel zeroes those rows of Y first); the row workgroups skip them.
//     long_k is chosen on the host so that a single wave's longest row stays a
//     few percent of the whole launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "es_spmm.h"

namespace {

constexpr int kWaveSize = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlockThreads = kWaveSize * kWavesPerBlock;
constexpr int kTileSlots = 512;                       // (col, val) slots per wave
constexpr int kWaveTileStride = kTileSlots + 64;      // + one pad slot per row slot
constexpr int kNumXcd = 8;
constexpr int kLongScanRows = 1024;                   // rows one long-row workgroup scans
constexpr int kLongSplit = 16;                        // workgroups sharing those rows
constexpr int kLongSeg = 256;                         // slots per long-row segment (<= kTileSlots)
constexpr int kLongMin = 64;                          // smallest long-row threshold the host picks
static_assert(kLongSplit % kNumXcd == 0, "long-row workgroups must not shift the XCD phase");

struct Args {
    const int32_t* rowptr;
    const int32_t* colidx;
    const float* vals;
    const float* X;
    float* Y;
    int64_t N;
    uint64_t seed;
    int32_t F, ldx, ldy, W, mode, logR;
    int32_t long_k;            // rows keeping more entries go to the long-row part  
    int32_t norm;              // es_norm_t: row factor applied before the store
    uint32_t nblocks;          // workgroups that carry rows
    uint32_t blocks_per_xcd;   // ceil(nblocks / 8)
    uint32_t long_blocks;      // leading workgroups that run the long-row part
};

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
        const uint32_t P = (n % 577u) ? 577u : (n % 587u) ? 587u : (n % 593u) ? 593u : 599u;
        uint32_t off = 0;
        if (seed != 0)
            off = (uint32_t)(splitmix64_output(seed, (uint64_t)row + 1u) >> 32) % n;
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

// ---------------------------------------------------------------------------
// VEC-wide pieces of a row of X / Y
// ---------------------------------------------------------------------------
// ALIGNED = false: rows of X / Y are only 4-byte aligned (F or a row stride is
// not a multiple of 4).  Loads stay 128-bit (the HSA ABI runs the memory
// pipeline in unaligned-access mode); a row's last, partial chunk is read as
// the row's final four floats and only its components >= `first` are kept.
typedef float float4_a4 __attribute__((ext_vector_type(4), aligned(4)));

template <int VEC, bool ALIGNED> struct Pack;
template <bool ALIGNED> struct Pack<4, ALIGNED> {
    float4 v;
    __device__ __forceinline__ void zero() { v = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ void load(const float* p)
    {
        if (ALIGNED) {
            v = *reinterpret_cast<const float4*>(p);
        } else {
            const float4_a4 t = *reinterpret_cast<const float4_a4*>(p);
            v = make_float4(t.x, t.y, t.z, t.w);
        }
    }
    __device__ __forceinline__ void store(float* p, int first) const
    {
        if (ALIGNED) {
            *reinterpret_cast<float4*>(p) = v;
        } else {
            if (first <= 0) p[0] = v.x;
            if (first <= 1) p[1] = v.y;
            if (first <= 2) p[2] = v.z;
            p[3] = v.w;
        }
    }
    __device__ __forceinline__ void atomic_add(float* p, int first) const
    {
        if (first <= 0) unsafeAtomicAdd(p, v.x);
        if (first <= 1) unsafeAtomicAdd(p + 1, v.y);
        if (first <= 2) unsafeAtomicAdd(p + 2, v.z);
        unsafeAtomicAdd(p + 3, v.w);
    }
    __device__ __forceinline__ void fma(float a, const Pack& x)
    {
        v.x = fmaf(a, x.v.x, v.x); v.y = fmaf(a, x.v.y, v.y);
        v.z = fmaf(a, x.v.z, v.z); v.w = fmaf(a, x.v.w, v.w);
    }
    __device__ __forceinline__ void scale(float f) { v.x *= f; v.y *= f; v.z *= f; v.w *= f; }
    __device__ __forceinline__ void add_xor(int mask)
    {
        v.x += __shfl_xor(v.x, mask, kWaveSize); v.y += __shfl_xor(v.y, mask, kWaveSize);
        v.z += __shfl_xor(v.z, mask, kWaveSize); v.w += __shfl_xor(v.w, mask, kWaveSize);
    }
};
template <bool ALIGNED> struct Pack<1, ALIGNED> {
    float v;
    __device__ __forceinline__ void zero() { v = 0.f; }
    __device__ __forceinline__ void load(const float* p) { v = *p; }
    __device__ __forceinline__ void store(float* p, int) const { *p = v; }
    __device__ __forceinline__ void atomic_add(float* p, int) const { unsafeAtomicAdd(p, v); }
    __device__ __forceinline__ void fma(float a, const Pack& x) { v = fmaf(a, x.v, v); }
    __device__ __forceinline__ void scale(float f) { v *= f; }
    __device__ __forceinline__ void add_xor(int mask) { v += __shfl_xor(v, mask, kWaveSize); }
};

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v >> 1); }

// Feature columns one lane covers: CH chunks of VEC floats, chunk ch at column
// colblk + (ch*G + l)*VEC.  Lanes past F re-read column 0 and never store.  In
// the unaligned variant a chunk that straddles F is moved back to end at F and
// `first` marks its first component that belongs to this lane.
template <int G, int CH, int VEC, bool ALIGNED>
struct LaneCols {
    int off[CH];
    int first[CH];
    bool ok[CH];
    __device__ __forceinline__ void init(int colblk, int l, int F)
    {
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
            const int c = colblk + (ch * G + l) * VEC;
            ok[ch] = c < F;
            off[ch] = ok[ch] ? c : 0;
            first[ch] = 0;
            if (!ALIGNED && VEC > 1 && ok[ch] && c + VEC > F) {
                off[ch] = F - VEC;
                first[ch] = c - off[ch];
            }
        }
    }
};

// Stage 1 of Algorithm 1 for one tile: copy the sampled (column, value) pairs
// of slots [0, count) into the LDS tile.
__device__ __forceinline__ void stage_tile(RowSampler& sampler, int t, int team, int count,
                                           int32_t base, const int32_t* __restrict__ colidx,
                                           const float* __restrict__ vals, uint2* tile)
{
    sample_tile(sampler, t, team, count, [&](int slot, uint32_t entry) {
        const int64_t p = (int64_t)base + entry;
        const int32_t c = colidx[p];
        const float v = vals ? vals[p] : 1.0f;
        tile[slot] = make_uint2((uint32_t)c, __float_as_uint(v));
    });
}

// Stage 2 of Algorithm 1 for one tile: this lane's edge slot e (of E) walks
// tile entries e, e+E, ... < count, U at a time: U LDS broadcasts, then U*CH
// independent loads of X, then the FMAs.
template <int G, int CH, int VEC, bool ALIGNED>
__device__ __forceinline__ void consume_tile(const uint2* tile, int count, int e, int E,
                                             const float* __restrict__ X, int64_t ldx,
                                             const LaneCols<G, CH, VEC, ALIGNED>& cols,
                                             Pack<VEC, ALIGNED> (&acc)[CH])
{
    constexpr int U = 8 / CH;
    using P = Pack<VEC, ALIGNED>;
    int j = e;
    for (; j + (U - 1) * E < count; j += U * E) {            // full batches
        uint2 ed[U];
#pragma unroll
        for (int u = 0; u < U; ++u) ed[u] = tile[j + u * E];
        P x[U][CH];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float* xr = X + (int64_t)ed[u].x * ldx;
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) x[u][ch].load(xr + cols.off[ch]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float v = __uint_as_float(ed[u].y);
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) acc[ch].fma(v, x[u][ch]);
        }
    }
    if (j < count) {                                         // last partial batch
        uint2 ed[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int jj = j + u * E;
            ok[u] = jj < count;
            ed[u] = tile[ok[u] ? jj : j];                    // absent slots re-read a present one
        }
        P x[U][CH];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float* xr = X + (int64_t)ed[u].x * ldx;
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) x[u][ch].load(xr + cols.off[ch]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float v = __uint_as_float(ed[u].y);
            if (ok[u]) {
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) acc[ch].fma(v, x[u][ch]);
            }
        }
    }
}

__device__ __forceinline__ int kept_count(int mode, int n, int W)
{
    return (mode == ES_FULL) ? n : min(n, W);
}

// Row factor of the in-kernel normalisation (Section 6.1): a function of the
// row's stored count n and kept count k; rows that keep nothing stay zero.
__device__ __forceinline__ float row_factor(int norm, int n, int k)
{
    if (norm == ES_NORM_NONE) return 1.0f;
    if (k == 0) return 0.0f;
    if (norm == ES_NORM_MEAN) return 1.0f / (float)k;
    if (norm == ES_NORM_RSQRT) return 1.0f / sqrtf((float)k);
    if (norm == ES_NORM_INV_DEGREE) return 1.0f / (float)n;
    return (float)n / (float)k;
}

// Transposed stage 2 (backward pass): every staged entry (c, v) of the tile adds
// v * dy to row c of the output with fp32 atomics; edge slot e of E walks
// entries e, e+E, ...  Atomics return nothing, so they pipeline by themselves.
template <int G, int CH, int VEC, bool ALIGNED>
__device__ __forceinline__ void scatter_tile(const uint2* tile, int count, int e, int E, float* out,
                                             int64_t ldo, const LaneCols<G, CH, VEC, ALIGNED>& cols,
                                             const Pack<VEC, ALIGNED> (&dy)[CH])
{
    for (int j = e; j < count; j += E) {
        const uint2 ed = tile[j];
        const float v = __uint_as_float(ed.y);
        float* dst = out + (int64_t)ed.x * ldo;
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
            if (cols.ok[ch]) {
                Pack<VEC, ALIGNED> t = dy[ch];
                t.scale(v);
                t.atomic_add(dst + cols.off[ch], cols.first[ch]);
            }
        }
    }
}

// This lane's chunks of row r of the upstream gradient, times the row factor.
template <int G, int CH, int VEC, bool ALIGNED>
__device__ __forceinline__ void load_row_chunks(const Args& a, int64_t r, int n, int k,
                                                const LaneCols<G, CH, VEC, ALIGNED>& cols,
                                                Pack<VEC, ALIGNED> (&dy)[CH])
{
    const float f = row_factor(a.norm, n, k);
    const float* src = a.X + r * (int64_t)a.ldx;
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        dy[ch].load(src + cols.off[ch]);
        dy[ch].scale(f);
    }
}

// ---------------------------------------------------------------------------
// Row part of the fused kernel (Algorithm 1) for workgroup `vb` of the row
// grid.  G lanes x CH chunks x VEC floats cover one block of G*CH*VEC feature
// columns (blockIdx.y selects the block).  Rows that keep more than long_k
// entries are left to the long-row part and not stored here.
// ---------------------------------------------------------------------------
template <int G, int CH, int VEC, bool ALIGNED, bool BACKWARD>
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
    uint2* tile = lds + wave * kWaveTileStride + rs * (T + 1);

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
            stage_tile(sampler, t, team, count, base, a.colidx, a.vals, tile);
            wave_lds_fence();
            scatter_tile<G, CH, VEC, ALIGNED>(tile, count, e, E, a.Y, a.ldy, cols, dy);
            wave_lds_fence();
        }
        return;
    }

    P acc[CH];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) acc[ch].zero();

    for (int t0 = 0; t0 < k; t0 += T) {
        const int count = min(k - t0, T);
        stage_tile(sampler, t, team, count, base, a.colidx, a.vals, tile);
        wave_lds_fence();
        consume_tile<G, CH, VEC, ALIGNED>(tile, count, e, E, a.X, a.ldx, cols, acc);
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
            if (cols.ok[ch]) acc[ch].store(y + cols.off[ch], cols.first[ch]);
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

template <int G, int CH, int VEC, bool ALIGNED, bool BACKWARD>
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
        stage_tile(sampler, lane, kWaveSize, count, base, a.colidx, a.vals, tile);
        wave_lds_fence();
        if (BACKWARD) {
            P dy[CH];
            load_row_chunks<G, CH, VEC, ALIGNED>(a, r, n, k, cols, dy);
            scatter_tile<G, CH, VEC, ALIGNED>(tile, count, e, E, a.Y, a.ldy, cols, dy);
            wave_lds_fence();
            continue;
        }
        P acc[CH];
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) acc[ch].zero();
        consume_tile<G, CH, VEC, ALIGNED>(tile, count, e, E, a.X, a.ldx, cols, acc);
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
template <int G, int CH, int VEC, bool ALIGNED, bool BACKWARD>
__global__ void __launch_bounds__(kBlockThreads) es_spmm_kernel(const Args a)
{
    __shared__ uint2 lds[kWavesPerBlock * kWaveTileStride];
    __shared__ LongScratch long_scratch;

    if (blockIdx.x < a.long_blocks) {
        long_block<G, CH, VEC, ALIGNED, BACKWARD>(a, blockIdx.x / kLongSplit, blockIdx.x % kLongSplit,
                                                  lds, long_scratch);
        return;
    }
    const uint32_t b = blockIdx.x - a.long_blocks;
    const uint32_t vb = (b % kNumXcd) * a.blocks_per_xcd + b / kNumXcd;
    if (vb >= a.nblocks) return;
    row_block<G, CH, VEC, ALIGNED, BACKWARD>(a, vb, lds);
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
// One thread per row; such rows are rare by construction of long_k.
__global__ void __launch_bounds__(kBlockThreads) es_zero_long_rows_kernel(const Args a)
{
    const int64_t r = (int64_t)blockIdx.x * kBlockThreads + threadIdx.x;
    if (r >= a.N) return;
    const int n = a.rowptr[r + 1] - a.rowptr[r];
    if (kept_count(a.mode, n, a.W) <= a.long_k) return;
    float* y = a.Y + r * (int64_t)a.ldy;
    for (int c = 0; c < a.F; ++c) y[c] = 0.0f;
}

// ---------------------------------------------------------------------------
// Sampler export: identical team / tile schedule, sink writes CSR positions.
// logR < 0 selects the long-row schedule instead: a whole wave per row, one
// freshly initialised sampler per kLongSeg-slot segment.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlockThreads)
es_sample_edges_kernel(const int32_t* __restrict__ rowptr, int64_t N, int32_t W, int32_t mode,
                       uint64_t seed, int32_t logR, int32_t* __restrict__ pos,
                       int32_t* __restrict__ cnt)
{
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const bool segmented = logR < 0;
    if (segmented) logR = 0;
    const int team = kWaveSize >> logR;
    const int rs = lane >> (6 - logR);
    const int t = lane & (team - 1);
    const int T = segmented ? kLongSeg : (kTileSlots >> logR);
    const int64_t r = ((((int64_t)blockIdx.x * kWavesPerBlock) + wave) << logR) + rs;
    if (r >= N) return;
    const int32_t base = rowptr[r];
    const int32_t n = rowptr[r + 1] - base;
    const int k = min(n, W);

    RowSampler sampler;
    sampler.init(mode, seed, r, (uint32_t)n, (uint32_t)W, (uint32_t)t, (uint32_t)team);
    int32_t* out = pos + r * (int64_t)W;
    for (int t0 = 0; t0 < k; t0 += T) {
        const int count = min(k - t0, T);
        if (segmented)
            sampler.init(mode, seed, r, (uint32_t)n, (uint32_t)W, (uint32_t)(t0 + t), (uint32_t)team);
        sample_tile(sampler, t, team, count,
                    [&](int slot, uint32_t entry) { out[t0 + slot] = base + (int32_t)entry; });
    }
    for (int i = k + t; i < W; i += team) out[i] = -1;
    if (t == 0) cnt[r] = k;
}

// ---------------------------------------------------------------------------
// Materialised sampled graph (the pre-sampled input of Section 5.6): row
// pointers of the kept counts by a three-step in-place scan, then the sampled
// (column, value) pairs in slot order.
// ---------------------------------------------------------------------------
constexpr int kScanRows = 1024;                       // rows per scan workgroup
constexpr int kScanPerThread = kScanRows / kBlockThreads;

// Step 1: out[r+1] = inclusive prefix, inside the row's 1024-row block, of the
// kept counts k_r (rowptr given) or of the counts already stored in out[r+1]
// (rowptr == nullptr; each thread reads its own entries before it writes them).
__global__ void __launch_bounds__(kBlockThreads)
es_kept_scan_local_kernel(const int32_t* __restrict__ rowptr, int64_t N, int32_t W, int32_t mode,
                          int32_t* out)
{
    __shared__ int wave_total[kWavesPerBlock];
    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid >> 6;
    const int64_t r0 = (int64_t)blockIdx.x * kScanRows + tid * kScanPerThread;
    int k[kScanPerThread];
    int mine = 0;
#pragma unroll
    for (int i = 0; i < kScanPerThread; ++i) {
        const int64_t r = r0 + i;
        k[i] = 0;
        if (r < N) k[i] = rowptr ? kept_count(mode, rowptr[r + 1] - rowptr[r], W) : out[r + 1];
        mine += k[i];
    }
    int incl = mine;
#pragma unroll
    for (int d = 1; d < kWaveSize; d <<= 1) {
        const int up = __shfl_up(incl, d, kWaveSize);
        if (lane >= d) incl += up;
    }
    if (lane == kWaveSize - 1) wave_total[wave] = incl;
    __syncthreads();
    int run = incl - mine;
    for (int w = 0; w < wave; ++w) run += wave_total[w];
#pragma unroll
    for (int i = 0; i < kScanPerThread; ++i) {
        run += k[i];
        if (r0 + i < N) out[r0 + i + 1] = run;
    }
    if (blockIdx.x == 0 && tid == 0) out[0] = 0;
}

// Step 2 (one workgroup): turn the block totals, stored at each block's last
// row, into global inclusive prefixes.
__global__ void __launch_bounds__(kBlockThreads)
es_kept_scan_blocks_kernel(int64_t N, int32_t* __restrict__ out)
{
    __shared__ int wave_total[kWavesPerBlock];
    __shared__ int carry_s;
    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid >> 6;
    const int64_t nblocks = (N + kScanRows - 1) / kScanRows;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (int64_t b0 = 0; b0 < nblocks; b0 += kBlockThreads) {
        const int64_t b = b0 + tid;
        const int64_t last = min((b + 1) * (int64_t)kScanRows, N);   // index of the block's total
        const int v = (b < nblocks) ? out[last] : 0;
        int incl = v;
#pragma unroll
        for (int d = 1; d < kWaveSize; d <<= 1) {
            const int up = __shfl_up(incl, d, kWaveSize);
            if (lane >= d) incl += up;
        }
        if (lane == kWaveSize - 1) wave_total[wave] = incl;
        __syncthreads();
        int run = incl + carry_s;
        for (int w = 0; w < wave; ++w) run += wave_total[w];
        if (b < nblocks) out[last] = run;
        __syncthreads();
        if (tid == kBlockThreads - 1) carry_s = run;
        __syncthreads();
    }
}

// Step 3: add the previous block's global prefix to every entry of a block
// except its last (already global).
__global__ void __launch_bounds__(kBlockThreads)
es_kept_scan_add_kernel(int64_t N, int32_t* __restrict__ out)
{
    const int64_t b = blockIdx.x + 1;                 // block 0 needs no offset
    const int offset = out[b * kScanRows];
    const int64_t last = min((b + 1) * (int64_t)kScanRows, N);
    for (int64_t i = b * kScanRows + 1 + threadIdx.x; i < last; i += kBlockThreads) out[i] += offset;
}

// One team of 64/R lanes per row, same sampler walk as stage 1 of the fused kernel.
__global__ void __launch_bounds__(kBlockThreads)
es_materialize_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                      const float* __restrict__ vals, int64_t N, int32_t W, int32_t mode,
                      uint64_t seed, int32_t logR, const int32_t* __restrict__ out_rowptr,
                      int32_t* __restrict__ out_colidx, float* __restrict__ out_vals)
{
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int team = kWaveSize >> logR;
    const int rs = lane >> (6 - logR);
    const int t = lane & (team - 1);
    const int T = kTileSlots >> logR;
    const int64_t r = ((((int64_t)blockIdx.x * kWavesPerBlock) + wave) << logR) + rs;
    if (r >= N) return;
    const int32_t base = rowptr[r];
    const int32_t n = rowptr[r + 1] - base;
    const int k = kept_count(mode, n, W);
    const int64_t obase = out_rowptr[r];

    RowSampler sampler;
    sampler.init(mode, seed, r, (uint32_t)n, (uint32_t)W, (uint32_t)t, (uint32_t)team);
    for (int t0 = 0; t0 < k; t0 += T) {
        const int count = min(k - t0, T);
        sample_tile(sampler, t, team, count, [&](int slot, uint32_t entry) {
            const int64_t p = (int64_t)base + entry;
            out_colidx[obase + t0 + slot] = colidx[p];
            out_vals[obase + t0 + slot] = vals ? vals[p] : 1.0f;
        });
    }
}

// ---------------------------------------------------------------------------
// Transposed sampled graph (the sampled graph in CSC form): count the kept
// entries per column, scan, then drop every entry into its column's segment
// through a per-column cursor.  Entries of one column arrive in no fixed order.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlockThreads) es_fill_int_kernel(int32_t* out, int64_t n, int32_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlockThreads + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * kBlockThreads)
        out[i] = v;
}

__global__ void __launch_bounds__(kBlockThreads)
es_copy_int_kernel(const int32_t* __restrict__ in, int32_t* __restrict__ out, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlockThreads + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * kBlockThreads)
        out[i] = in[i];
}

// FILL == false: out_ptr[c + 1] += 1 per kept entry with column c.
// FILL == true : the entry goes to position out_end[c]++ of out_idx / out_vals
//                (value times the row factor).
template <bool FILL>
__global__ void __launch_bounds__(kBlockThreads)
es_transpose_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                    const float* __restrict__ vals, int64_t N, int32_t W, int32_t mode, uint64_t seed,
                    int32_t norm, int32_t logR, int32_t* out_ptr, int32_t* out_end,
                    int32_t* __restrict__ out_idx, float* __restrict__ out_vals)
{
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int team = kWaveSize >> logR;
    const int rs = lane >> (6 - logR);
    const int t = lane & (team - 1);
    const int T = kTileSlots >> logR;
    const int64_t r = ((((int64_t)blockIdx.x * kWavesPerBlock) + wave) << logR) + rs;
    if (r >= N) return;
    const int32_t base = rowptr[r];
    const int32_t n = rowptr[r + 1] - base;
    const int k = kept_count(mode, n, W);
    const float f = row_factor(norm, n, k);

    RowSampler sampler;
    sampler.init(mode, seed, r, (uint32_t)n, (uint32_t)W, (uint32_t)t, (uint32_t)team);
    for (int t0 = 0; t0 < k; t0 += T) {
        const int count = min(k - t0, T);
        sample_tile(sampler, t, team, count, [&](int, uint32_t entry) {
            const int64_t p = (int64_t)base + entry;
            const int32_t c = colidx[p];
            if (!FILL) {
                atomicAdd(out_ptr + c + 1, 1);
            } else {
                const int32_t pos = atomicAdd(out_end + c, 1);
                out_idx[pos] = (int32_t)r;
                out_vals[pos] = f * (vals ? vals[p] : 1.0f);
            }
        });
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct Shape {
    int vec, G, CH;
    bool aligned;
};

int next_pow2(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

// Lanes x chunks that cover F columns: 128-bit accesses whenever F >= 4
// (aligned or not), 32-bit ones for F < 4.
Shape pick_shape(int F, bool aligned)
{
    Shape s;
    s.aligned = aligned;
    s.vec = (aligned || F >= 4) ? 4 : 1;
    const int q = (F + s.vec - 1) / s.vec;                 // accesses per row
    s.G = next_pow2(q);
    if (s.G < 4) s.G = 4;
    s.CH = 1;
    if (s.G > 64) {
        s.G = 64;
        s.CH = q > 128 ? 4 : 2;
    }
    return s;
}

// Rows per wave: enough edge slots per row to fill a batch of loads, but not
// more slots than a typical row has entries.
int pick_logR(const Shape& s, double mean_kept)
{
    const int U = 8 / s.CH;
    const int maxR = 64 / s.G;
    if (mean_kept < 1.0) mean_kept = 1.0;
    const double want = 64.0 * U / (s.G * mean_kept);      // R >= want
    int R = 1;
    while (R < maxR && R < want) R <<= 1;
    int logR = 0;
    while ((1 << logR) < R) ++logR;
    return logR;
}

template <int G, int CH, int VEC, bool ALIGNED>
hipError_t launch_forward(const Args& a, dim3 grid, hipStream_t st)
{
    if (a.long_blocks > 0) {
        const uint32_t zb = (uint32_t)((a.N + kBlockThreads - 1) / kBlockThreads);
        hipLaunchKernelGGL(es_zero_long_rows_kernel, dim3(zb), dim3(kBlockThreads), 0, st, a);
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    hipLaunchKernelGGL((es_spmm_kernel<G, CH, VEC, ALIGNED, false>), grid, dim3(kBlockThreads), 0, st, a);
    return hipGetLastError();
}

// The transposed product always runs the 32-bit interleaved column mapping
// (lane l owns columns l, l+G, ...): one atomic instruction then covers G
// consecutive floats of an output row instead of every fourth one, which is
// what the memory-side atomic units are fastest at (measured 4x over the
// 128-bit mapping); G is as wide as F allows for the same reason.
template <int G, int CH>
hipError_t launch_backward(const Args& a, dim3 grid, hipStream_t st)
{
    int64_t fb = (a.N * (int64_t)a.F + kBlockThreads * 8 - 1) / (kBlockThreads * 8);
    if (fb > 65536) fb = 65536;
    hipLaunchKernelGGL(es_fill_zero_kernel, dim3((uint32_t)fb), dim3(kBlockThreads), 0, st, a.Y, a.N, a.F,
                       a.ldy);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL((es_spmm_kernel<G, CH, 1, false, true>), grid, dim3(kBlockThreads), 0, st, a);
    return hipGetLastError();
}

// Longest row one wave may own.  A wave retires about E*U entries per memory
// round trip (~2 us under load) while the whole launch moves entries*(4F+8)
// bytes at a few TB/s; the bound keeps one wave's row near 5 % of the launch.
int32_t pick_long_k(const Shape& s, int logR, double entries, int F)
{
    const int U = 8 / s.CH;
    const int E = (64 >> logR) / s.G;
    const double k = (double)E * U * entries * (4.0 * F + 8.0) / 2.4e8;
    if (k >= (double)(INT32_MAX - kLongMin)) return INT32_MAX;
    const int32_t v = ((int32_t)k / kLongMin) * kLongMin;
    return v < kLongMin ? kLongMin : v;
}

// Process-wide overrides (relaxed atomics: a call racing with a setter sees
// either the old or the new value, never a torn one).
std::atomic<int32_t> g_force_logR{-1};   // es_spmm_set_rows_per_wave; -1 = heuristic
std::atomic<int32_t> g_force_long_k{0};  // es_spmm_set_long_row_threshold; 0 = heuristic
std::atomic<int32_t> g_force_G{0};       // es_spmm_set_lanes_per_row; 0 = heuristic

// Rows per wave for the kernels that only walk the sampler (materialise,
// transpose): about one lane per kept entry of a typical row; a whole wave per
// row when rows may be much longer than typical (full mode, W above a wave).
int walk_logR(int64_t N, int64_t nnz, int32_t Wk)
{
    if (Wk > kWaveSize) return 0;
    double mean = (double)nnz / (double)N;
    if (mean > (double)Wk) mean = (double)Wk;
    int logR = 6;
    while (logR > 0 && (double)(kWaveSize >> logR) < mean) --logR;
    return logR;
}

// Everything the host decides about one launch.
struct Plan {
    Shape s;
    int logR;                  // log2(rows per wave)
    int32_t long_k;            // long-row threshold
    int64_t nblocks;           // row workgroups that carry rows
    int64_t per_xcd;           // row workgroups per XCD
    int64_t grid_x, grid_y;    // launch grid (long-row workgroups included in grid_x)
    int64_t long_blocks;       // leading long-row workgroups
};

int check_sizes(int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W, int32_t mode,
                int32_t norm)
{
    if (norm < ES_NORM_NONE || norm > ES_NORM_INV_DEGREE) return ES_ERR_INVALID_ARG;
    if (N < 0 || nnz < 0 || nnz > INT32_MAX || F < 1 || ldx < F || ldy < F) return ES_ERR_INVALID_ARG;
    if (mode != ES_FULL && mode != ES_BUCKET && mode != ES_FASTRAND) return ES_ERR_INVALID_ARG;
    if (mode != ES_FULL && W < 1) return ES_ERR_INVALID_ARG;
    return ES_OK;
}

// Launch shape for N >= 1 rows.  `aligned`: F and both row strides are
// multiples of 4 and both matrices are 16-byte aligned.
int make_plan(int64_t N, int64_t nnz, int32_t F, int32_t W, int32_t mode, bool aligned, bool backward,
              Plan* p)
{
    Shape s = pick_shape(F, aligned);
    if (backward) {                                        // see launch_backward
        s.vec = 1; s.aligned = false;
        s.G = next_pow2(F);
        if (s.G < 4) s.G = 4;
        if (s.G > 64) s.G = 64;
        s.CH = F > 128 ? 4 : F > 64 ? 2 : 1;
    }
    const int32_t force_G = g_force_G.load(std::memory_order_relaxed);
    if (!backward && force_G > 0 && s.vec == 4 && force_G < s.G) {
        s.G = force_G;                                     // narrower column blocks, more of them
        s.CH = 1;
    }
    p->s = s;

    double mean = (double)nnz / (double)N;
    if (mode != ES_FULL && mean > (double)W) mean = (double)W;
    int logR = pick_logR(s, mean);
    const int32_t force_logR = g_force_logR.load(std::memory_order_relaxed);
    if (force_logR >= 0) {
        logR = force_logR;
        while ((64 >> logR) < s.G) --logR;                 // at least one edge slot per row
    }
    p->logR = logR;

    const int64_t rows_per_block = (int64_t)kWavesPerBlock << logR;
    p->nblocks = (N + rows_per_block - 1) / rows_per_block;
    p->per_xcd = (p->nblocks + kNumXcd - 1) / kNumXcd;
    const int cols_per_block = s.G * s.CH * s.vec;
    p->grid_y = ((int64_t)F + cols_per_block - 1) / cols_per_block;

    // rows that may keep more than long_k entries exist only in full mode or
    // for W above the bound (nnz is a hint, so it does not gate the launch)
    double entries = (double)nnz;
    if (mode != ES_FULL && entries > (double)N * W) entries = (double)N * W;
    p->long_k = pick_long_k(s, logR, entries, F);
    // the long-row part costs a second small launch and a scan of the row
    // pointers; below one tile per row that is more than the tail it removes
    if (mode != ES_FULL && p->long_k < kTileSlots) p->long_k = kTileSlots;
    const int32_t force_long_k = g_force_long_k.load(std::memory_order_relaxed);
    if (force_long_k > 0) p->long_k = force_long_k;
    const bool may_be_long = mode == ES_FULL || W > p->long_k;
    p->long_blocks = may_be_long ? ((N + kLongScanRows - 1) / kLongScanRows) * kLongSplit : 0;
    p->grid_x = p->per_xcd * kNumXcd + p->long_blocks;
    if (p->grid_x > INT32_MAX || p->grid_y > 65535) return ES_ERR_UNSUPPORTED;
    return ES_OK;
}

// Shared host path of es_spmm_norm (X -> Y) and es_spmm_backward (dY -> dX).
int es_run(const int32_t* rowptr, const int32_t* colidx, const float* vals, const float* X, float* Y,
           int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W, int32_t mode,
           uint64_t seed, int32_t norm, bool backward, void* stream)
{
    const int bad = check_sizes(N, nnz, F, ldx, ldy, W, mode, norm);
    if (bad != ES_OK) return bad;
    if (N == 0) return ES_OK;
    if (!rowptr || !X || !Y) return ES_ERR_INVALID_ARG;
    if (nnz > 0 && !colidx) return ES_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(X) % 4 || reinterpret_cast<uintptr_t>(Y) % 4)
        return ES_ERR_INVALID_ARG;
    const bool aligned = (F % 4 == 0) && (ldx % 4 == 0) && (ldy % 4 == 0) &&
                         (reinterpret_cast<uintptr_t>(X) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(Y) % 16 == 0);
    Plan p;
    const int rc = make_plan(N, nnz, F, W, mode, aligned, backward, &p);
    if (rc != ES_OK) return rc;
    const Shape& s = p.s;

    Args a;
    a.rowptr = rowptr; a.colidx = colidx; a.vals = vals; a.X = X; a.Y = Y;
    a.N = N; a.seed = seed; a.F = F; a.ldx = ldx; a.ldy = ldy;
    a.W = (mode == ES_FULL) ? INT32_MAX : W;
    a.mode = mode; a.logR = p.logR; a.norm = norm; a.long_k = p.long_k;
    a.nblocks = (uint32_t)p.nblocks; a.blocks_per_xcd = (uint32_t)p.per_xcd;
    a.long_blocks = (uint32_t)p.long_blocks;

    const dim3 grid((uint32_t)p.grid_x, (uint32_t)p.grid_y);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t err = hipErrorInvalidValue;
#define ES_CASE(G_, CH_, V_, A_)                                                   \
    if (!backward && s.G == G_ && s.CH == CH_ && s.vec == V_ && s.aligned == A_)   \
        err = launch_forward<G_, CH_, V_, A_>(a, grid, st);
    ES_CASE(4, 1, 4, true) ES_CASE(8, 1, 4, true) ES_CASE(16, 1, 4, true) ES_CASE(32, 1, 4, true)
    ES_CASE(64, 1, 4, true) ES_CASE(64, 2, 4, true) ES_CASE(64, 4, 4, true)
    ES_CASE(4, 1, 4, false) ES_CASE(8, 1, 4, false) ES_CASE(16, 1, 4, false) ES_CASE(32, 1, 4, false)
    ES_CASE(64, 1, 4, false) ES_CASE(64, 2, 4, false) ES_CASE(64, 4, 4, false)
    ES_CASE(4, 1, 1, false)
#define ES_BWD(G_, CH_) \
    if (backward && s.G == G_ && s.CH == CH_) err = launch_backward<G_, CH_>(a, grid, st);
    ES_BWD(4, 1) ES_BWD(8, 1) ES_BWD(16, 1) ES_BWD(32, 1) ES_BWD(64, 1) ES_BWD(64, 2) ES_BWD(64, 4)
#undef ES_BWD
#undef ES_CASE
    return err == hipSuccess ? ES_OK : ES_ERR_LAUNCH;
}

}  // namespace

extern "C" {

const char* es_spmm_status_string(int status)
{
    switch (status) {
        case ES_OK: return "ES_OK";
        case ES_ERR_INVALID_ARG: return "ES_ERR_INVALID_ARG: null pointer, negative size, ld < F, W < 1 or unknown mode";
        case ES_ERR_UNSUPPORTED: return "ES_ERR_UNSUPPORTED: shape outside what the kernels cover";
        case ES_ERR_LAUNCH: return "ES_ERR_LAUNCH: the HIP runtime rejected the launch";
        default: return "unknown es_spmm status";
    }
}

int32_t es_spmm_max_W(int32_t F) { return F < 1 ? 0 : INT32_MAX; }

int32_t es_spmm_tile_slots(int32_t rows_per_wave)
{
    if (rows_per_wave == 0) return kTileSlots;
    if (rows_per_wave < 1 || rows_per_wave > 64 || (rows_per_wave & (rows_per_wave - 1))) return 0;
    return kTileSlots / rows_per_wave;
}

int es_spmm_set_rows_per_wave(int32_t rows_per_wave)
{
    if (rows_per_wave == 0) { g_force_logR.store(-1, std::memory_order_relaxed); return ES_OK; }
    if (rows_per_wave < 1 || rows_per_wave > 64 || (rows_per_wave & (rows_per_wave - 1)))
        return ES_ERR_INVALID_ARG;
    int lg = 0;
    while ((1 << lg) < rows_per_wave) ++lg;
    g_force_logR.store(lg, std::memory_order_relaxed);
    return ES_OK;
}

int es_spmm_set_lanes_per_row(int32_t lanes)
{
    if (lanes != 0 && lanes != 4 && lanes != 8 && lanes != 16 && lanes != 32 && lanes != 64)
        return ES_ERR_INVALID_ARG;
    g_force_G.store(lanes, std::memory_order_relaxed);
    return ES_OK;
}

int es_spmm_set_long_row_threshold(int32_t entries)
{
    if (entries < 0) return ES_ERR_INVALID_ARG;
    g_force_long_k.store(entries, std::memory_order_relaxed);
    return ES_OK;
}

int es_spmm(const int32_t* rowptr, const int32_t* colidx, const float* vals, const float* X,
            float* Y, int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W,
            int32_t mode, uint64_t seed, void* stream)
{
    return es_spmm_norm(rowptr, colidx, vals, X, Y, N, nnz, F, ldx, ldy, W, mode, seed, ES_NORM_NONE,
                        stream);
}

int es_spmm_norm(const int32_t* rowptr, const int32_t* colidx, const float* vals, const float* X,
                 float* Y, int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W,
                 int32_t mode, uint64_t seed, int32_t norm, void* stream)
{
    return es_run(rowptr, colidx, vals, X, Y, N, nnz, F, ldx, ldy, W, mode, seed, norm, false, stream);
}

int es_spmm_backward(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                     const float* dY, float* dX, int64_t N, int64_t nnz, int32_t F, int32_t ldy,
                     int32_t ldx, int32_t W, int32_t mode, uint64_t seed, int32_t norm, void* stream)
{
    return es_run(rowptr, colidx, vals, dY, dX, N, nnz, F, ldy, ldx, W, mode, seed, norm, true, stream);
}

int es_spmm_launch_info(int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W,
                        int32_t mode, int32_t aligned16, int32_t backward, es_launch_info_t* info)
{
    if (!info) return ES_ERR_INVALID_ARG;
    const int bad = check_sizes(N, nnz, F, ldx, ldy, W, mode, ES_NORM_NONE);
    if (bad != ES_OK) return bad;
    if (N == 0) return ES_ERR_INVALID_ARG;
    const bool aligned = aligned16 && (F % 4 == 0) && (ldx % 4 == 0) && (ldy % 4 == 0);
    Plan p;
    const int rc = make_plan(N, nnz, F, W, mode, aligned, backward != 0, &p);
    if (rc != ES_OK) return rc;
    info->vector_width = p.s.vec;
    info->aligned = p.s.aligned ? 1 : 0;
    info->lanes_per_row = p.s.G;
    info->chunks_per_lane = p.s.CH;
    info->rows_per_wave = 1 << p.logR;
    info->edge_slots = (64 >> p.logR) / p.s.G;
    info->loads_in_flight = 8 / p.s.CH;
    info->tile_slots_per_row = kTileSlots >> p.logR;
    info->long_row_threshold = p.long_k;
    info->long_row_workgroups = p.long_blocks;
    info->grid_x = p.grid_x;
    info->grid_y = p.grid_y;
    return ES_OK;
}

int es_spmm_materialize(const int32_t* rowptr, const int32_t* colidx, const float* vals, int64_t N,
                        int64_t nnz, int32_t W, int32_t mode, uint64_t seed, int32_t* out_rowptr,
                        int32_t* out_colidx, float* out_vals, void* stream)
{
    if (N < 0 || nnz < 0 || nnz > INT32_MAX) return ES_ERR_INVALID_ARG;
    if (mode != ES_FULL && mode != ES_BUCKET && mode != ES_FASTRAND) return ES_ERR_INVALID_ARG;
    if (mode != ES_FULL && W < 1) return ES_ERR_INVALID_ARG;
    if (!out_rowptr) return ES_ERR_INVALID_ARG;
    if (N > 0 && (!rowptr || !out_colidx || !out_vals)) return ES_ERR_INVALID_ARG;
    if (nnz > 0 && !colidx) return ES_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t Wk = (mode == ES_FULL) ? INT32_MAX : W;
    const int64_t nscan = N == 0 ? 1 : (N + kScanRows - 1) / kScanRows;
    if (nscan > INT32_MAX) return ES_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(es_kept_scan_local_kernel, dim3((uint32_t)nscan), dim3(kBlockThreads), 0, st,
                       rowptr, N, Wk, mode, out_rowptr);
    if (hipGetLastError() != hipSuccess) return ES_ERR_LAUNCH;
    if (N == 0) return ES_OK;
    if (nscan > 1) {
        hipLaunchKernelGGL(es_kept_scan_blocks_kernel, dim3(1), dim3(kBlockThreads), 0, st, N, out_rowptr);
        if (hipGetLastError() != hipSuccess) return ES_ERR_LAUNCH;
        hipLaunchKernelGGL(es_kept_scan_add_kernel, dim3((uint32_t)(nscan - 1)), dim3(kBlockThreads), 0,
                           st, N, out_rowptr);
        if (hipGetLastError() != hipSuccess) return ES_ERR_LAUNCH;
    }
    const int logR = walk_logR(N, nnz, Wk);
    const int64_t rows_per_block = (int64_t)kWavesPerBlock << logR;
    const int64_t nblocks = (N + rows_per_block - 1) / rows_per_block;
    if (nblocks > INT32_MAX) return ES_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(es_materialize_kernel, dim3((uint32_t)nblocks), dim3(kBlockThreads), 0, st,
                       rowptr, colidx, vals, N, Wk, mode, seed, logR, out_rowptr, out_colidx, out_vals);
    return hipGetLastError() == hipSuccess ? ES_OK : ES_ERR_LAUNCH;
}

int es_spmm_materialize_transposed(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                                   int64_t N, int64_t nnz, int32_t W, int32_t mode, uint64_t seed,
                                   int32_t norm, int32_t* out_ptr, int32_t* out_end, int32_t* out_idx,
                                   float* out_vals, void* stream)
{
    if (N < 0 || nnz < 0 || nnz > INT32_MAX) return ES_ERR_INVALID_ARG;
    if (mode != ES_FULL && mode != ES_BUCKET && mode != ES_FASTRAND) return ES_ERR_INVALID_ARG;
    if (mode != ES_FULL && W < 1) return ES_ERR_INVALID_ARG;
    if (norm < ES_NORM_NONE || norm > ES_NORM_INV_DEGREE) return ES_ERR_INVALID_ARG;
    if (!out_ptr) return ES_ERR_INVALID_ARG;
    if (N > 0 && (!rowptr || !out_end || !out_idx || !out_vals)) return ES_ERR_INVALID_ARG;
    if (nnz > 0 && !colidx) return ES_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t Wk = (mode == ES_FULL) ? INT32_MAX : W;
    const int64_t nscan = N == 0 ? 1 : (N + kScanRows - 1) / kScanRows;
    if (nscan > INT32_MAX) return ES_ERR_UNSUPPORTED;
#define ES_CHECK_LAUNCH() if (hipGetLastError() != hipSuccess) return ES_ERR_LAUNCH
    int64_t fb = (N + 1 + kBlockThreads - 1) / kBlockThreads;
    if (fb > 65536) fb = 65536;
    hipLaunchKernelGGL(es_fill_int_kernel, dim3((uint32_t)fb), dim3(kBlockThreads), 0, st, out_ptr, N + 1, 0);
    ES_CHECK_LAUNCH();
    if (N == 0) return ES_OK;

    const int logR = walk_logR(N, nnz, Wk);
    const int64_t rows_per_block = (int64_t)kWavesPerBlock << logR;
    const int64_t nblocks = (N + rows_per_block - 1) / rows_per_block;
    if (nblocks > INT32_MAX) return ES_ERR_UNSUPPORTED;

    hipLaunchKernelGGL(es_transpose_kernel<false>, dim3((uint32_t)nblocks), dim3(kBlockThreads), 0, st,
                       rowptr, colidx, vals, N, Wk, mode, seed, norm, logR, out_ptr, out_end, out_idx,
                       out_vals);
    ES_CHECK_LAUNCH();
    hipLaunchKernelGGL(es_kept_scan_local_kernel, dim3((uint32_t)nscan), dim3(kBlockThreads), 0, st,
                       static_cast<const int32_t*>(nullptr), N, Wk, mode, out_ptr);
    ES_CHECK_LAUNCH();
    if (nscan > 1) {
        hipLaunchKernelGGL(es_kept_scan_blocks_kernel, dim3(1), dim3(kBlockThreads), 0, st, N, out_ptr);
        ES_CHECK_LAUNCH();
        hipLaunchKernelGGL(es_kept_scan_add_kernel, dim3((uint32_t)(nscan - 1)), dim3(kBlockThreads), 0,
                           st, N, out_ptr);
        ES_CHECK_LAUNCH();
    }
    hipLaunchKernelGGL(es_copy_int_kernel, dim3((uint32_t)fb), dim3(kBlockThreads), 0, st, out_ptr, out_end, N);
    ES_CHECK_LAUNCH();
    hipLaunchKernelGGL(es_transpose_kernel<true>, dim3((uint32_t)nblocks), dim3(kBlockThreads), 0, st,
                       rowptr, colidx, vals, N, Wk, mode, seed, norm, logR, out_ptr, out_end, out_idx,
                       out_vals);
    ES_CHECK_LAUNCH();
#undef ES_CHECK_LAUNCH
    return ES_OK;
}

int es_spmm_sample_edges(const int32_t* rowptr, int64_t N, int32_t W, int32_t mode, uint64_t seed,
                         int32_t rows_per_wave, int32_t* pos, int32_t* cnt, void* stream)
{
    if (N < 0 || W < 1) return ES_ERR_INVALID_ARG;
    if (mode != ES_BUCKET && mode != ES_FASTRAND) return ES_ERR_INVALID_ARG;
    if (rows_per_wave < -1 || rows_per_wave > 64 ||
        (rows_per_wave > 0 && (rows_per_wave & (rows_per_wave - 1))))
        return ES_ERR_INVALID_ARG;
    if (N == 0) return ES_OK;
    if (!rowptr || !pos || !cnt) return ES_ERR_INVALID_ARG;
    if (N * (int64_t)W > INT32_MAX) return ES_ERR_UNSUPPORTED;
    int logR = 0;
    while ((1 << logR) < rows_per_wave) ++logR;
    const int64_t rows_per_block = (int64_t)kWavesPerBlock << logR;
    const int64_t nblocks = (N + rows_per_block - 1) / rows_per_block;
    if (nblocks > INT32_MAX) return ES_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(es_sample_edges_kernel, dim3((uint32_t)nblocks), dim3(kBlockThreads), 0,
                       static_cast<hipStream_t>(stream), rowptr, N, W, mode, seed,
                       rows_per_wave < 0 ? -1 : logR, pos, cnt);
    return hipGetLastError() == hipSuccess ? ES_OK : ES_ERR_LAUNCH;
}

}  // extern "C"
