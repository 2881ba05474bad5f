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
// at the memory rate.  Here a wave takes NR = 4E consecutive rows (E = 64 / G
// edge slots), lays their kept entries end to end (each row padded to a
// multiple of E with zero-valued repeats of its first entry), stages that run
// tile by tile into LDS (stage 1 of Algorithm 1; the sample index of a slot is
// evaluated from its definition, Equation 2, since consecutive slots of a lane
// no longer belong to one row) and lets the E edge slots walk it E entries per
// step (stage 2).  Because of the padding a step never straddles two rows, so
// "a new row starts here" is a wave-uniform bit per step (scalar test): at such
// a step every slot adds its partial sums for the finished row into that row's
// accumulator in LDS and starts over.  The rows' sums leave LDS once, at the
// end: E rows per pass, coalesced (plain stores, or load-add-store in the later
// phases of the column-partitioned product).
// ---------------------------------------------------------------------------
constexpr int kFlatTile = 256;                        // staged entries per tile
constexpr int kFlatAccFloats = 1024;                  // NR rows x 4G columns
constexpr int kFlatMaxRows = 64;

struct FlatLds {                                      // one per wave
    uint2 tile[kFlatTile];                            // (row key, value)
    float rowacc[kFlatAccFloats];                     // [NR][4G] sums of the chunk's rows
    int32_t start[kFlatMaxRows + 1];                  // padded start of each row in the run
    int32_t kept[kFlatMaxRows];                       // entries the row really keeps
    int32_t src[kFlatMaxRows];                        // CSR position of the row's (piece's) entry 0, < 2^31
    uint32_t len[kFlatMaxRows];                       // FastRand on a longer row: its length n; else 0
    uint32_t mul[kFlatMaxRows];                       //   multiplier P
    uint32_t rot[kFlatMaxRows];                       //   rotation off
    uint32_t newrow[kFlatTile / 8];                   // bit u of word b: step 8b+u starts a row
    uint8_t steprow[kFlatTile];                       // row (0..NR-1) a step belongs to, valid where a row starts
};

// What the chunk's rows are: whole sampled rows (forward kernel) or the pieces
// of one column range (a phase of the column-partitioned product).
struct FlatJob {
    int part;          // column range, or -1: whole rows
    bool accumulate;   // add to Y instead of overwriting it (phases after the first)
};

template <int G, bool ALIGNED, bool WIDE>
__device__ __forceinline__ void flat_block(const Args& a, uint32_t vb, const FlatJob job, FlatLds* lds_all)
{
    constexpr int LOG_G = ilog2(G);
    constexpr int E = kWaveSize / G;                  // edge slots
    constexpr int NR = 4 * E;                         // rows per wave
    constexpr int FB = 4 * G;                         // feature columns per block
    constexpr int U = 8;                              // loads in flight per lane
    static_assert(NR * FB == kFlatAccFloats, "row accumulators fill their LDS array");
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
                strided = a.mode == ES_FASTRAND && my_n > a.W;
            } else {
                const int32_t* cr = a.cuts + r * kParts;
                lo = cr[job.part];
                hi = (job.part + 1 < kParts) ? cr[job.part + 1] : my_n;
                my_store = !job.accumulate || hi > lo;
            }
            kj = hi - lo;
        }
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
            s.len[lane] = strided ? (uint32_t)my_n : 0u;
            s.mul[lane] = strided ? fastrand_multiplier((uint32_t)my_n) : 0u;
            s.rot[lane] = strided ? fastrand_offset(a.seed, r, (uint32_t)my_n) : 0u;
        }
        if (lane == 0) s.start[0] = 0;
    }
#pragma unroll
    for (int i = 0; i < kFlatAccFloats / (4 * kWaveSize); ++i)
        *reinterpret_cast<float4*>(&s.rowacc[(i * kWaveSize + lane) * 4]) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_fence();
    const int total = __builtin_amdgcn_readfirstlane(s.start[NR]);

    // ---- the run, tile by tile -----------------------------------------------------
    P acc;
    acc.zero();
    int cur = -1;                                     // row being summed (wave-uniform)
    int jrow = 0;                                     // row of this lane's next slot (never decreases)
    auto flush = [&](int row) {
        if (row >= 0 && cols.ok[0]) {
            float* dst = &s.rowacc[row * FB + l * 4];
            atomicAdd(dst + 0, acc.v.x);
            atomicAdd(dst + 1, acc.v.y);
            atomicAdd(dst + 2, acc.v.z);
            atomicAdd(dst + 3, acc.v.w);
        }
    };
    for (int t0 = 0; t0 < total; t0 += kFlatTile) {
        const int count = min(total - t0, kFlatTile);             // a multiple of E
        if (lane < kFlatTile / 8) s.newrow[lane] = 0u;
        wave_lds_fence();
        // stage 1: slot -> (row, slot in row) -> sample index -> (key, value)
#pragma unroll
        for (int m = 0; m < kFlatTile / kWaveSize; ++m) {
            const int at = m * kWaveSize + lane;
            if (at < count) {
                const int sl = t0 + at;
                while (sl >= s.start[jrow + 1]) ++jrow;           // sl < total = start[NR]: stops at NR-1
                const int i = sl - s.start[jrow];
                const bool real = i < s.kept[jrow];
                const uint32_t n = s.len[jrow];
                const uint32_t slot = real ? (uint32_t)i : 0u;    // padding repeats the row's first entry
                uint32_t entry = slot;
                if (n) {
                    const uint32_t step = a.W < (1 << 22) ? (slot * s.mul[jrow]) % n
                                                          : (uint32_t)(((uint64_t)slot * s.mul[jrow]) % n);
                    entry = s.rot[jrow] + step;                   // both < n < 2^31
                    if (entry >= n) entry -= n;
                }
                const int64_t p = (int64_t)s.src[jrow] + entry;
                const float v = real ? (a.vals ? a.vals[p] : 1.0f) : 0.0f;
                s.tile[at] = make_uint2(K::make(a.colidx[p], a.stride_units), __float_as_uint(v));
                if (i == 0) {                                      // first slot of a row: its step starts the row
                    const int step = at >> (6 - LOG_G);            // at / E
                    atomicOr(&s.newrow[step >> 3], 1u << (step & 7));
                    s.steprow[step] = (uint8_t)jrow;
                }
            }
        }
        wave_lds_fence();
        // stage 2: E entries per step, U steps per batch
        const int steps = count >> (6 - LOG_G);
        for (int b0 = 0; b0 < steps; b0 += U) {
            const uint32_t starts = __builtin_amdgcn_readfirstlane(s.newrow[b0 >> 3]);
            const int nu = min(U, steps - b0);
            uint2 ed[U];
            P x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (u < nu) {
                    ed[u] = s.tile[(b0 + u) * E + e];
                    x[u].load(K::row(a.X, ed[u].x, a.ldx) + cols.off[0]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (u < nu) {
                    if (starts & (1u << u)) {                      // wave-uniform
                        flush(cur);
                        acc.zero();
                        cur = __builtin_amdgcn_readfirstlane((int)s.steprow[b0 + u]);
                    }
                    acc.fma(__uint_as_float(ed[u].y), x[u]);
                }
            }
        }
        wave_lds_fence();
    }
    flush(cur);
    wave_lds_fence();

    // ---- rows out: E rows per pass ---------------------------------------------------
#pragma unroll
    for (int pass = 0; pass < NR / E; ++pass) {
        const int j = pass * E + e;
        const int64_t r = r0 + j;
        const int32_t n = __shfl(my_n, j, kWaveSize);
        const int32_t k = __shfl(my_k, j, kWaveSize);
        const bool store = __shfl((int)my_store, j, kWaveSize) != 0;
        if (store && cols.ok[0]) {
            P out;
            out.v = *reinterpret_cast<const float4*>(&s.rowacc[j * FB + l * 4]);
            if (a.norm != ES_NORM_NONE) out.scale(row_factor(a.norm, n, k));
            float* y = a.Y + r * (int64_t)a.ldy + cols.off[0];
            if (job.accumulate) {
                P prev;
                prev.load(y);
                out.add(prev);
            }
            out.store(y, cols.first[0]);
        }
    }
}

// The forward kernel on flattened rows: as es_spmm_kernel, the leading
// a.long_blocks workgroups split the rows that keep more than a.long_k entries
// (those rows are left out of the flattened runs), the rest serve 4 * NR rows
// each, remapped so that every XCD walks one contiguous range of rows.
template <int G, bool ALIGNED, bool WIDE>
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
    flat_block<G, ALIGNED, WIDE>(a, vb, FlatJob{-1, false}, reinterpret_cast<FlatLds*>(raw));
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
    flat_block<G, ALIGNED, WIDE>(a, vb, FlatJob{(int)p, a.phase != 0}, lds);
}

}  // namespace

#endif  // ES_SPMM_FLAT_KERNEL_H
