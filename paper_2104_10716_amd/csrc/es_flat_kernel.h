// es_flat_kernel.h -- stage 1 and stage 2 of Algorithm 1 on a flattened run of rows: edge slots are dealt entries, not rows.
#ifndef ES_SPMM_FLAT_KERNEL_H
#define ES_SPMM_FLAT_KERNEL_H

#include "es_fused_kernel.h"

namespace {

// ---------------------------------------------------------------------------
// Why: with one row (or one row per team) on a wave at a time, every row costs
// a fixed number of instructions and memory round trips, and a wave whose rows
// differ in length idles the lanes of the short ones.  Short rows -- sampled
// rows with W of 16..64, the eighth-of-a-row pieces of the column-partitioned
// product, the rows of a column slice -- then run at the instruction rate, not
// at the memory rate.  Here a wave takes NR = E or 2E consecutive rows (E =
// 64 / G edge slots), lays their kept entries end to end (each row padded to a
// multiple of E with zero-valued repeats of its first entry), stages that run
// tile by tile into LDS (stage 1 of Algorithm 1; the sample index of a slot is
// evaluated from its definition, Equation 2, since consecutive slots of a lane
// no longer belong to one row) and lets the E edge slots walk it E entries per
// step (stage 2).  Because of the padding a step never straddles two rows, so
// "a new row starts here" is a wave-uniform bit per step (scalar test): at such
// a step the slots' partial sums for the finished row are added across the wave
// with lane swaps (LDS float atomics run about a lane per cycle here: far too
// slow), written to that row's place in LDS, and the slots start over.  The
// rows' sums leave LDS once, at the end: E rows per pass, coalesced (plain
// stores, or load-add-store in the later phases of the column-partitioned
// product).
// ---------------------------------------------------------------------------
constexpr int kFlatTile = 256;                        // staged entries per tile
constexpr int kFlatLongRow = 8192;                    // kept entries above which a row goes to the long-row part (at most)
constexpr int kFlatPartRps = 2;                       // rows per edge slot in the column-partitioned product
constexpr int kFlatAccFloats = 512;                   // NR rows x 4G columns at most
constexpr int kFlatMaxRows = 32;                      // NR at most

struct FlatLds {                                      // one per wave
    uint2 tile[kFlatTile];                            // (row key, value)
    float rowacc[kFlatAccFloats];                     // [NR][4G] sums of the chunk's non-empty rows, in order
    int32_t start[kFlatMaxRows + 1];                  // padded start of each row in the run
    int32_t kept[kFlatMaxRows];                       // entries the row really keeps
    int32_t src[kFlatMaxRows];                        // CSR position of the row's (piece's) entry 0, < 2^31
    uint32_t len[kFlatMaxRows];                       // FastRand on a longer row: its length n; else 0
    uint32_t mul[kFlatMaxRows];                       //   multiplier P
    uint32_t rot[kFlatMaxRows];                       //   rotation off
};

// What the chunk's rows are: whole sampled rows (forward kernel) or the pieces
// of one column range (a phase of the column-partitioned product).
struct FlatJob {
    int part;          // column range, or -1: whole rows
    bool accumulate;   // add to Y instead of overwriting it (phases after the first)
};

// Lanes whose bit BIT (4 or 5) is clear get a + a', the others b + b', where a',
// b' are the values of the lane that differs in that bit alone: the row and
// half-wave swaps of gfx950 (odd rows of 16 lanes of the first operand trade
// places with even rows of the second; the upper half of the first with the lower
// half of the second), then one add.  No LDS traffic.
template <int BIT>
__device__ __forceinline__ float halve_add(float a, float b)
{
    static_assert(BIT == 4 || BIT == 5, "swaps of rows of 16 lanes and of half waves");
    if constexpr (BIT == 5) {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    } else {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
}

// v + the values of the lanes that differ from this one in bit BIT (2 or 3) and
// agree in the lower ones: a rotation by 2^BIT inside a row of 16 lanes.  For
// bit 2 the values must already be equal across bit 3.
template <int BIT>
__device__ __forceinline__ float all_add(float v)
{
    static_assert(BIT == 2 || BIT == 3, "rotations inside a row of 16");
    constexpr int kRowRor = 0x120 + (1 << BIT);
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), kRowRor, 0xf, 0xf, true));
}

// RPS: rows per edge slot on a wave (NR = RPS * E rows per wave).  Fewer rows per
// wave cost more set-up per row and even the waves out: 1 for the exact product
// (its rows differ most in length), 2 for sampled rows.
template <int G, bool ALIGNED, bool WIDE, bool STRIDED, int RPS>
__device__ __forceinline__ void flat_block(const Args& a, uint32_t vb, const FlatJob job, FlatLds* lds_all)
{
    constexpr int LOG_G = ilog2(G);
    constexpr int LOG_E = 6 - LOG_G;
    constexpr int E = kWaveSize / G;                  // edge slots
    constexpr int NR = RPS * E;                       // rows per wave
    constexpr int FB = 4 * G;                         // feature columns per block
    constexpr int U = E <= 8 ? 8 : kWaveSize / E;     // steps per batch = loads in flight per lane; U*E <= 64
    static_assert(NR * FB <= kFlatAccFloats && NR <= kFlatMaxRows, "row accumulators fit their LDS array");
    static_assert(U * E <= kWaveSize && kWaveSize % (U * E) == 0, "a batch lies inside 64 slots");
    using P = Pack<4, ALIGNED>;
    using K = RowKey<ALIGNED, WIDE>;

    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int e = lane >> LOG_G;
    const int l = lane & (G - 1);
    FlatLds& s = lds_all[wave];

    LaneCols<G, 1, 4, ALIGNED> cols;
    cols.init(blockIdx.y * FB, l, a.F);

    // ---- the chunk's rows: lane j describes row r0 + j -------------------------
    const int64_t r0 = ((int64_t)vb * kWavesPerBlock + wave) * NR;
    int32_t my_n = 0, my_k = 0;
    bool my_store = false;                            // this launch writes the row's Y
    uint64_t nonempty;                                // bit j: row j has entries in this run
    {
        int32_t base = 0, lo = 0, hi = 0, kj = 0;
        bool strided = false;
        const int64_t r = r0 + lane;
        if (lane < NR && r < a.N) {
            base = a.rowptr[r];
            my_n = a.rowptr[r + 1] - base;
            my_k = kept_count(a.mode, my_n, a.W);
            if (job.part < 0) {
                hi = my_k;
                my_store = my_k <= a.long_k;          // longer rows belong to the long-row part
                if (!my_store) hi = 0;
                strided = STRIDED && my_n > a.W;
            } else {
                const int32_t* cr = a.cuts + r * kParts;
                lo = __builtin_nontemporal_load(&cr[job.part]);
                hi = (job.part + 1 < kParts) ? __builtin_nontemporal_load(&cr[job.part + 1]) : my_n;
                my_store = !job.accumulate || hi > lo;
            }
            kj = hi - lo;
        }
        nonempty = __ballot(kj > 0);
        const int32_t padded = (kj + E - 1) & ~(E - 1);
        int32_t incl = padded;                        // inclusive scan over the wave
#pragma unroll
        for (int d = 1; d < kWaveSize; d <<= 1) {
            const int32_t up = __shfl_up(incl, d, kWaveSize);
            if (lane >= d) incl += up;
        }
        if (lane < NR) {
            s.start[lane + 1] = incl;
            s.kept[lane] = kj;
            s.src[lane] = base + lo;
            if constexpr (STRIDED) {
                s.len[lane] = strided ? (uint32_t)my_n : 0u;
                s.mul[lane] = strided ? fastrand_multiplier((uint32_t)my_n) : 0u;
                s.rot[lane] = strided ? fastrand_offset(a.seed, r, (uint32_t)my_n) : 0u;
            }
        }
        if (lane == 0) s.start[0] = 0;
    }
    wave_lds_fence();
    const int total = __builtin_amdgcn_readfirstlane(s.start[NR]);

    // ---- the run, tile by tile -----------------------------------------------------
    P acc;
    acc.zero();
    int cur = -1;                                     // rank of the row being summed among the non-empty ones
    int jrow = 0;                                     // row of this lane's next slot (never decreases)
    // A row ends once.  Its sum over the slots is taken so that the two steps over
    // the highest slot bits (lane bits 4 and 5: plain swaps) also halve what a lane
    // carries: after them a lane holds one of the four columns; the lower slot bits
    // are summed by rotations inside a row of 16 lanes.  The lanes of the slots
    // whose low bits are zero write the four columns side by side.
    auto flush = [&]() {
        float* dst = &s.rowacc[cur * FB + l * 4];
        if constexpr (E == 1) {
            *reinterpret_cast<float4*>(dst) = acc.v;
        } else if constexpr (E == 2) {
            const float s0 = halve_add<5>(acc.v.x, acc.v.z);
            const float s1 = halve_add<5>(acc.v.y, acc.v.w);
            *reinterpret_cast<float2*>(dst + 2 * e) = make_float2(s0, s1);
        } else {
            const float s0 = halve_add<4>(acc.v.x, acc.v.z);    // bit 4 clear: x, set: z
            const float s1 = halve_add<4>(acc.v.y, acc.v.w);    //              y       w
            float v = halve_add<5>(s0, s1);                     // bit 5 clear: s0, set: s1
            if constexpr (LOG_E > 2) v = all_add<3>(v);
            if constexpr (LOG_E > 3) v = all_add<2>(v);
            const int top = e >> (LOG_E - 2);                         // lane bits 4, 5
            if ((e & (E / 4 - 1)) == 0) dst[2 * (top & 1) + (top >> 1)] = v;
        }
    };
    // Stage 1 for one tile, up to the loads: slot -> (row, slot in row) -> sample
    // index -> CSR position, then the entry's column and value requested.  No
    // branch encloses a global load (lanes past the tile's end redo its last
    // slot; past the run's end, the run's last slot), so that all of a lane's
    // loads are in flight together, and the next tile's are in flight while this
    // tile is consumed.
    constexpr int M = kFlatTile / kWaveSize;
    struct Staged {
        int32_t col[M];
        float val[M];
        bool real[M];
        uint64_t firsts[M];                                       // bit i: slot 64m + i is the first of its row
    };
    auto request = [&](int t0, Staged& st) {
        const int count = min(total - t0, kFlatTile);             // a multiple of E; <= 0 past the run
        int64_t pos[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int at = min(m * kWaveSize + lane, count - 1);
            const int sl = t0 + at;                               // t0 - 1 at least: a slot of the run
            while (sl >= s.start[jrow + 1]) ++jrow;               // sl < total = start[NR]: stops at NR-1
            const int i = sl - s.start[jrow];
            st.real[m] = i < s.kept[jrow];
            st.firsts[m] = __ballot(i == 0 && m * kWaveSize + lane < count);
            const uint32_t slot = st.real[m] ? (uint32_t)i : 0u;  // padding repeats the row's first entry
            uint32_t entry = slot;
            if constexpr (STRIDED) {
                const uint32_t n = s.len[jrow];
                if (n) {
                    const uint32_t step = a.W < (1 << 22) ? (slot * s.mul[jrow]) % n
                                                          : (uint32_t)(((uint64_t)slot * s.mul[jrow]) % n);
                    entry = s.rot[jrow] + step;                   // both < n < 2^31
                    if (entry >= n) entry -= n;
                }
            }
            pos[m] = (int64_t)s.src[jrow] + entry;
        }
#pragma unroll
        for (int m = 0; m < M; ++m) {
            st.col[m] = __builtin_nontemporal_load(&a.colidx[pos[m]]);
            st.val[m] = a.vals ? __builtin_nontemporal_load(&a.vals[pos[m]]) : 1.0f;
        }
    };
    Staged st;
    if (total > 0) request(0, st);                                // an empty run has no slot to stand in for
    for (int t0 = 0; t0 < total; t0 += kFlatTile) {
        const int count = min(total - t0, kFlatTile);
        // the tile is filled up to whole batches with zero-valued repeats of its last
        // entry (what the lanes past its end requested), so stage 2 needs no bounds
        const int filled = (count + U * E - 1) & ~(U * E - 1);
        uint64_t firsts[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            firsts[m] = st.firsts[m];
            const int at = m * kWaveSize + lane;
            if (at < filled)
                s.tile[at] = make_uint2(K::make(st.col[m], a.stride_units),
                                        __float_as_uint(at < count && st.real[m] ? st.val[m] : 0.0f));
        }
        wave_lds_fence();
        request(t0 + kFlatTile, st);
        // stage 2: E entries per step, U steps per batch, a batch's rows of X in
        // flight together.  Rows start at multiples of E, so "step b0 + u starts a
        // row" is bit (b0 + u) * E of the tile's first-slot bits: a scalar test.
        const int steps = count >> LOG_E;
        for (int b0 = 0; b0 < steps; b0 += U) {
            const int slot0 = b0 << LOG_E;
            uint64_t word = firsts[0];
#pragma unroll
            for (int m = 1; m < M; ++m)
                if ((slot0 >> 6) == m) word = firsts[m];
            const uint64_t starts = word >> (slot0 & 63);
            uint2 ed[U];
            P x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) ed[u] = s.tile[(b0 + u) * E + e];
#pragma unroll
            for (int u = 0; u < U; ++u) {
#if defined(ES_PROBE_NO_GATHER)        // measurement builds only (wrong results): the kernel without stage 2's loads
                x[u].v = make_float4(__uint_as_float(ed[u].x), 1.f, 2.f, 3.f);
#elif defined(ES_PROBE_NEAR_GATHER)    // measurement builds only: every gather inside the first 64 KB of X
                x[u].load(K::row(a.X, ed[u].x & 0xFFFu, a.ldx) + cols.off[0]);
#else
                x[u].load(K::row(a.X, ed[u].x, a.ldx) + cols.off[0]);
#endif
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float v = __uint_as_float(ed[u].y);
                if ((starts >> (u * E)) & 1) {                     // wave-uniform; never set past the last step
                    if (cur >= 0) flush();
                    ++cur;
                    acc.mul(v, x[u]);                              // the row's first step
                } else {
                    acc.fma(v, x[u]);
                }
            }
        }
        wave_lds_fence();
    }
    if (cur >= 0) flush();
    wave_lds_fence();

    // ---- rows out: E rows per pass (earlier partial sums requested for all passes first) ----
    constexpr int PASSES = NR / E;
    P prev[PASSES];
    if (job.accumulate) {
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
            const int64_t r = min(r0 + pass * E + e, a.N - 1);     // past the end: any valid row, unused
            prev[pass].load_streaming(a.Y + r * (int64_t)a.ldy + cols.off[0]);
        }
    }
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
        const int j = pass * E + e;
        const int64_t r = r0 + j;
        const int32_t n = __shfl(my_n, j, kWaveSize);
        const int32_t k = __shfl(my_k, j, kWaveSize);
        const bool store = __shfl((int)my_store, j, kWaveSize) != 0;
        const int rank = __popcll(nonempty & ((1ull << j) - 1ull));
        P out;
        out.zero();
        if ((nonempty >> j) & 1) out.v = *reinterpret_cast<const float4*>(&s.rowacc[rank * FB + l * 4]);
        if (a.norm != ES_NORM_NONE) out.scale(row_factor(a.norm, n, k));
        if (job.accumulate) out.add(prev[pass]);
        if (store && cols.ok[0]) {
            float* y = a.Y + r * (int64_t)a.ldy + cols.off[0];
            out.store_streaming(y, cols.first[0]);                 // not read again by this launch
        }
    }
}

// The forward kernel on flattened rows: as es_spmm_kernel, the leading
// a.long_blocks workgroups split the rows that keep more than a.long_k entries
// (those rows are left out of the flattened runs), the rest serve 4 * NR rows
// each, remapped so that every XCD walks one contiguous range of rows.
template <int G, bool ALIGNED, bool WIDE, bool STRIDED, int RPS>
__global__ void __launch_bounds__(kBlockThreads) es_spmm_flat_kernel(const Args a)
{
    constexpr size_t kLongBytes = kWavesPerBlock * kWaveTileStride * sizeof(uint2) + sizeof(LongScratch);
    constexpr size_t kBytes = sizeof(FlatLds) * kWavesPerBlock > kLongBytes ? sizeof(FlatLds) * kWavesPerBlock
                                                                            : kLongBytes;
    __shared__ __align__(16) unsigned char raw[kBytes];
    if (blockIdx.x < a.long_blocks) {
        uint2* tiles = reinterpret_cast<uint2*>(raw);
        LongScratch& sc = *reinterpret_cast<LongScratch*>(raw + kWavesPerBlock * kWaveTileStride * sizeof(uint2));
        long_block<G, 1, 4, ALIGNED, false, WIDE>(a, blockIdx.x / kLongSplit, blockIdx.x % kLongSplit, tiles, sc);
        return;
    }
    const uint32_t b = blockIdx.x - a.long_blocks;
    const uint32_t vb = (b % kNumXcd) * a.blocks_per_xcd + b / kNumXcd;
    if (vb >= a.nblocks) return;
    flat_block<G, ALIGNED, WIDE, STRIDED, RPS>(a, vb, FlatJob{-1, false}, reinterpret_cast<FlatLds*>(raw));
}

// One phase of the column-partitioned exact product on flattened pieces (see
// es_part_kernel.h for the phases): XCD p = b % 8 serves column range p of the
// rows of row range (p + phase) % 8.
template <int G, bool ALIGNED, bool WIDE>
__global__ void __launch_bounds__(kBlockThreads) es_spmm_part_flat_kernel(const Args a)
{
    __shared__ FlatLds lds[kWavesPerBlock];
    const uint32_t p = blockIdx.x % kNumXcd;
    const uint32_t q = blockIdx.x / kNumXcd;
    const uint32_t sblock = (p + (uint32_t)a.phase) % kNumXcd;
    const uint32_t vb = sblock * a.blocks_per_xcd + q;
    if (vb >= a.nblocks) return;
    flat_block<G, ALIGNED, WIDE, false, kFlatPartRps>(a, vb, FlatJob{(int)p, a.phase != 0}, lds);
}

}  // namespace

#endif  // ES_SPMM_FLAT_KERNEL_H
