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

#include <mutex>

#include "es_spmm.h"

#include "es_common.h"
#include "es_sampler.h"
#include "es_tile.h"
#include "es_fused_kernel.h"
#include "es_part_kernel.h"
#include "es_flat_kernel.h"
#include "es_aux_kernels.h"
#include "es_pull_kernel.h"

// Workspace of es_spmm_static_ws: the cuts array of the column-partitioned
// product for up to ES_SPMM_STATIC_WS_MAX_ROWS rows, in static device memory.
// In host code this name is only a handle for hipGetSymbolAddress; the address
// kernels receive is the per-device pointer static_scratch_address() returns.
static __device__ __align__(256) unsigned char scratch[(size_t)ES_SPMM_STATIC_WS_MAX_ROWS * kParts * sizeof(int32_t)];

namespace {

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
constexpr int kMaxDevices = 64;

// Device address of `scratch` on the current device (every GPU holds its own
// copy of the array at its own address); looked up once per device.
int static_scratch_address(void** out)
{
    static std::mutex mu;
    static void* address[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ES_ERR_LAUNCH;
    std::lock_guard<std::mutex> guard(mu);
    if (!address[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ES_ERR_LAUNCH;
        address[dev] = p;
    }
    *out = address[dev];
    return ES_OK;
}

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

template <int G, int CH, int VEC, bool ALIGNED, bool WIDE>
hipError_t launch_forward(const Args& a, dim3 grid, hipStream_t st)
{
    if (a.long_blocks > 0) {
        const uint32_t zb = (uint32_t)((a.N + kBlockThreads - 1) / kBlockThreads);
        hipLaunchKernelGGL(es_zero_long_rows_kernel, dim3(zb), dim3(kBlockThreads), 0, st, a);
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    hipLaunchKernelGGL((es_spmm_kernel<G, CH, VEC, ALIGNED, false, WIDE>), grid, dim3(kBlockThreads), 0, st, a);
    return hipGetLastError();
}

template <int G, bool ALIGNED, bool WIDE>
hipError_t launch_flat(Args a, dim3 grid, bool partition, int32_t* cuts, hipStream_t st)
{
    if (!partition) {
        if (a.long_blocks > 0) {
            const uint32_t zb = (uint32_t)((a.N + kBlockThreads - 1) / kBlockThreads);
            hipLaunchKernelGGL(es_zero_long_rows_kernel, dim3(zb), dim3(kBlockThreads), 0, st, a);
            const hipError_t err = hipGetLastError();
            if (err != hipSuccess) return err;
        }
        if (a.mode == ES_FASTRAND)                         // with Equation 2's strided slots compiled in
            hipLaunchKernelGGL((es_spmm_flat_kernel<G, ALIGNED, WIDE, true, 2>), grid, dim3(kBlockThreads), 0, st, a);
        else if (a.mode == ES_BUCKET)
            hipLaunchKernelGGL((es_spmm_flat_kernel<G, ALIGNED, WIDE, false, 2>), grid, dim3(kBlockThreads), 0, st, a);
        else
            hipLaunchKernelGGL((es_spmm_flat_kernel<G, ALIGNED, WIDE, false, 1>), grid, dim3(kBlockThreads), 0, st, a);
        return hipGetLastError();
    }
    a.cuts = cuts;
    a.part_cols = (int32_t)((a.N + kParts - 1) / kParts);
    const uint32_t cb = (uint32_t)((a.N * kParts + kBlockThreads - 1) / kBlockThreads);
    hipLaunchKernelGGL(es_cuts_kernel, dim3(cb), dim3(kBlockThreads), 0, st, a.rowptr, a.colidx, a.N,
                       a.part_cols, cuts);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    for (int phase = 0; phase < kParts; ++phase) {
        a.phase = phase;
        hipLaunchKernelGGL((es_spmm_part_flat_kernel<G, ALIGNED, WIDE>), grid, dim3(kBlockThreads), 0, st, a);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

// The transposed product always runs the 32-bit interleaved column mapping
// (lane l owns columns l, l+G, ...): one atomic instruction then covers G
// consecutive floats of an output row instead of every fourth one, which is
// what the memory-side atomic units are fastest at (measured 4x over the
// 128-bit mapping); G is as wide as F allows for the same reason.
template <int G, int CH, bool WIDE>
hipError_t launch_backward(const Args& a, dim3 grid, hipStream_t st)
{
    int64_t fb = (a.N * (int64_t)a.F + kBlockThreads * 8 - 1) / (kBlockThreads * 8);
    if (fb > 65536) fb = 65536;
    hipLaunchKernelGGL(es_fill_zero_kernel, dim3((uint32_t)fb), dim3(kBlockThreads), 0, st, a.Y, a.N, a.F,
                       a.ldy);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL((es_spmm_kernel<G, CH, 1, false, true, WIDE>), grid, dim3(kBlockThreads), 0, st, a);
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

// Per-call overrides, parsed from an es_launch_opts_t (absent = the heuristic).
struct Overrides {
    int logR = -1;             // rows_per_wave as a power of two, -1 = heuristic
    int G = 0;                 // lanes_per_row cap, 0 = heuristic, -1 = never slice
    int32_t long_k = 0;        // long-row threshold, 0 = heuristic
    int partition = 0;         // column-partitioned product: 0 = heuristic, 1 = on, -1 = off
    int kernel = 0;            // 0 = heuristic, 1 = row kernel, 2 = flattened kernel
};

int parse_opts(const es_launch_opts_t* opts, Overrides* ov)
{
    *ov = Overrides();
    if (!opts) return ES_OK;
    if (opts->column_partition < -1 || opts->column_partition > 1) return ES_ERR_INVALID_ARG;
    ov->partition = opts->column_partition;
    if (opts->kernel < 0 || opts->kernel > 2) return ES_ERR_INVALID_ARG;
    ov->kernel = opts->kernel;
    const int32_t rpw = opts->rows_per_wave;
    if (rpw != 0) {
        if (rpw < 1 || rpw > 64 || (rpw & (rpw - 1))) return ES_ERR_INVALID_ARG;
        int lg = 0;
        while ((1 << lg) < rpw) ++lg;
        ov->logR = lg;
    }
    const int32_t lanes = opts->lanes_per_row;
    if (lanes != 0 && lanes != -1 && lanes != 4 && lanes != 8 && lanes != 16 && lanes != 32 && lanes != 64)
        return ES_ERR_INVALID_ARG;
    ov->G = lanes;
    if (opts->long_row_threshold < 0) return ES_ERR_INVALID_ARG;
    ov->long_k = opts->long_row_threshold;
    return ES_OK;
}

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
    bool partition;            // column-partitioned product (kParts phases, needs a workspace)
    bool flat;                 // flattened kernel (es_flat_kernel.h) instead of the row kernel
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
// Bytes of workspace the column-partitioned product needs for N rows.
size_t part_workspace_bytes(int64_t N)
{
    return (size_t)N * kParts * sizeof(int32_t);
}

// Whether to run the column-partitioned product.  It pays when a row's piece
// inside one column range is long enough to amortise the extra pass over Y
// (kept entries per row well above kParts) and when an XCD's eighth of a
// 32-column slice of X is of the order of its L2 (measured gains on the dense
// social-like graph from 58k to 699k rows, i.e. shares of 0.9 to 11 MB).
bool pick_partition(int64_t N, double mean_kept, int32_t mode, int cols_per_block, int force)
{
    if (mode == ES_BUCKET) return false;       // first-W entries crowd into the lowest column range
    if (N < kParts * 64) return false;
    if (force > 0) return true;
    if (force < 0) return false;
    // FastRand has to walk all W slots of a row once per column range to find the
    // ones that fall inside it; measured, that costs more than the locality
    // returns (config-3 graph, W = 256: 0.8x), so it is only run on request
    if (mode == ES_FASTRAND) return false;
    if (mean_kept < 128.0) return false;
    const double share = (double)N * cols_per_block * 4.0 / kParts;
    return share >= 0.5e6 && share <= 12.0e6;
}

int make_plan(int64_t N, int64_t nnz, int32_t F, int32_t W, int32_t mode, bool aligned, bool backward,
              const Overrides& ov, bool have_workspace, Plan* p)
{
    Shape s = pick_shape(F, aligned);
    if (backward) {                                        // see launch_backward
        s.vec = 1; s.aligned = false;
        s.G = next_pow2(F);
        if (s.G < 4) s.G = 4;
        if (s.G > 64) s.G = 64;
        s.CH = F > 128 ? 4 : F > 64 ? 2 : 1;
    }
    double mean = (double)nnz / (double)N;                 // mean entries a row keeps
    const double mean_stored = mean;
    if (mode != ES_FULL && mean > (double)W) mean = (double)W;

    // Column-partitioned product?  Decided on 32-column slices, its best width on
    // all but the smallest tables.
    const int slice_cols = F < 32 ? s.G * s.CH * s.vec : 32;
    p->partition = !backward && have_workspace && pick_partition(N, mean, mode, slice_cols, ov.partition);

    // The flattened kernel applies to 128-bit accesses; FastRand in the
    // partitioned product needs the row kernel's per-row walk over all W slots.
    const bool flat_applies = !backward && s.vec == 4 && !(p->partition && mode == ES_FASTRAND);
    // chosen by rule only on 16-byte-aligned rows: 32-column slices of rows that do
    // not tile 128-byte lines fetch every line twice (F = 41: 0.7x)
    const bool flat_allowed = flat_applies && ov.kernel != 1 && s.aligned;

    // Column slicing: fewer lanes across the feature columns, the rows swept once
    // per slice, so that the part of X in use at a time is smaller.  A slice makes
    // every row short, which the row kernel pays for per row and the flattened
    // kernel does not; so the narrow (32-column) slices go with the flattened
    // kernel.  Measured (profiles/):
    //  * partitioned product: 32-column slices on the flattened kernel once an
    //    XCD's share of a 64-column slice no longer fits its L2 (1.07x..1.3x over
    //    64-column slices on the row kernel, which stay best below that);
    //  * tables of 0.3 GB and more with F >= 128: 32-column slices on the
    //    flattened kernel (1.08x..1.2x where column ids cluster, so that the X rows
    //    of a community come nearer to an L2; 0.98x..1.0x where they do not);
    //    with the row kernel forced, 64-column slices from 0.5 GB;
    //  * Bucket on rows several times longer than W: 32-column slices (its picks
    //    crowd into the lowest-numbered columns).
    // Elsewhere slicing only re-reads the CSR entries.
    int slice_G = 0;
    bool sliced_by_rule = false;
    bool want_flat = false;
    if (!backward && s.vec == 4) {
        if (ov.G > 0) slice_G = ov.G;
        else if (ov.G == 0) {
            const double table = (double)N * F * 4.0;
            if (p->partition) {
                want_flat = flat_allowed && (double)N * 32.0 > 4.0e6;
                slice_G = want_flat ? 8 : 16;
            } else if (flat_allowed && F >= 128 && table >= 300.0e6) {
                want_flat = true;
                slice_G = 8;
            } else if (mode == ES_BUCKET && F >= 64 && mean_stored >= 4.0 * W) slice_G = 8;
            else if (F >= 128 && table >= 512.0e6) slice_G = 16;
            sliced_by_rule = slice_G > 0 && slice_G < s.G;
        }
    }
    if (slice_G > 0 && slice_G < s.G) {
        s.G = slice_G;                                     // narrower column blocks, more of them
        s.CH = 1;
    }
    // The flattened kernel's row accumulators hold one column block of at most
    // 256 columns, so wider rows are sliced to that.
    p->flat = flat_applies && (ov.kernel == 2 || (ov.kernel == 0 && want_flat));
    if (p->flat) s.CH = 1;
    p->s = s;

    int logR = pick_logR(s, mean);
    // a slice gathers less per row, so sampled rows share a wave in larger numbers
    if (sliced_by_rule && mode != ES_FULL && !p->partition && (64 >> (logR + 1)) >= s.G) ++logR;
    const int32_t force_logR = ov.logR;
    if (force_logR >= 0) {
        logR = force_logR;
        while ((64 >> logR) < s.G) --logR;                 // at least one edge slot per row
    }
    p->logR = logR;

    if (p->flat) {                                         // a wave lays 1 or 2 rows per edge slot end to end
        const int rps = p->partition ? kFlatPartRps : mode == ES_FULL ? 1 : 2;
        logR = 0;
        while ((1 << logR) < rps * 64 / s.G) ++logR;
        p->logR = logR;
    }
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
    // the flattened kernel walks a long row tile by tile on one wave at no extra
    // cost per entry, so only rows that would make a tail are split: a row of k
    // entries keeps its wave busy for about k * 16 ns, the whole launch takes about
    // entries * 50 ps, and the tail should stay below a tenth of that (co-purchase
    // graph, exact product: 8192 measured 6 % faster than 2048; citation graph,
    // 2.4 M entries: 8192 would leave one 12 k row running alone for half the launch)
    if (p->flat) {
        const double tail_free = entries * 3.0e-4;
        const int32_t k = tail_free >= (double)kFlatLongRow ? kFlatLongRow : (int32_t)tail_free;
        if (p->long_k < k) p->long_k = k;
    }
    if (ov.long_k > 0) p->long_k = ov.long_k;
    const bool may_be_long = mode == ES_FULL || W > p->long_k;
    p->long_blocks = may_be_long ? ((N + kLongScanRows - 1) / kLongScanRows) * kLongSplit : 0;
    p->grid_x = p->per_xcd * kNumXcd + p->long_blocks;
    if (p->partition && p->flat) {                         // one sweep per launch, no long-piece handling
        p->long_k = INT32_MAX;
        p->long_blocks = 0;
        p->grid_x = p->per_xcd * kNumXcd;
    } else if (p->partition) {
        // a wave serves kPartGroups consecutive rows, one at a time; every launch
        // sweeps the rows twice, pieces above long_k first (es_part_kernel.h)
        p->logR = 0;
        p->long_k = ov.long_k > 0 ? ov.long_k : kPartLongPiece;
        const int64_t rows_per_part_block = (int64_t)kWavesPerBlock * kPartGroups;
        p->nblocks = (N + rows_per_part_block - 1) / rows_per_part_block;
        p->per_xcd = (p->nblocks + kNumXcd - 1) / kNumXcd;
        p->long_blocks = p->per_xcd * kNumXcd;
        p->grid_x = 2 * p->long_blocks;
    }
    if (p->grid_x > INT32_MAX || p->grid_y > 65535) return ES_ERR_UNSUPPORTED;
    return ES_OK;
}

template <int G, int CH, int VEC, bool ALIGNED, bool WIDE>
hipError_t launch_partitioned(Args a, dim3 grid, int32_t* cuts, hipStream_t st)
{
    a.cuts = cuts;
    a.part_cols = (int32_t)((a.N + kParts - 1) / kParts);
    const uint32_t cb = (uint32_t)((a.N * kParts + kBlockThreads - 1) / kBlockThreads);
    hipLaunchKernelGGL(es_cuts_kernel, dim3(cb), dim3(kBlockThreads), 0, st, a.rowptr, a.colidx, a.N,
                       a.part_cols, cuts);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    for (int phase = 0; phase < kParts; ++phase) {
        a.phase = phase;
        hipLaunchKernelGGL((es_spmm_part_kernel<G, CH, VEC, ALIGNED, WIDE>), grid, dim3(kBlockThreads), 0, st, a);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

// Shared host path of es_spmm_norm (X -> Y) and es_spmm_backward (dY -> dX).
int es_run(const int32_t* rowptr, const int32_t* colidx, const float* vals, const float* X, float* Y,
           int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W, int32_t mode,
           uint64_t seed, int32_t norm, bool backward, const es_launch_opts_t* opts, void* workspace,
           size_t workspace_bytes, void* stream)
{
    const int bad = check_sizes(N, nnz, F, ldx, ldy, W, mode, norm);
    if (bad != ES_OK) return bad;
    Overrides ov;
    const int bad_opts = parse_opts(opts, &ov);
    if (bad_opts != ES_OK) return bad_opts;
    if (N == 0) return ES_OK;
    if (!rowptr || !X || !Y) return ES_ERR_INVALID_ARG;
    if (nnz > 0 && !colidx) return ES_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(X) % 4 || reinterpret_cast<uintptr_t>(Y) % 4)
        return ES_ERR_INVALID_ARG;
    const bool aligned = (F % 4 == 0) && (ldx % 4 == 0) && (ldy % 4 == 0) &&
                         (reinterpret_cast<uintptr_t>(X) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(Y) % 16 == 0);
    if (workspace && reinterpret_cast<uintptr_t>(workspace) % 16) return ES_ERR_INVALID_ARG;
    const bool have_ws = workspace && workspace_bytes >= part_workspace_bytes(N);
    Plan p;
    const int rc = make_plan(N, nnz, F, W, mode, aligned, backward, ov, have_ws, &p);
    if (rc != ES_OK) return rc;
    const Shape& s = p.s;

    Args a;
    a.rowptr = rowptr; a.colidx = colidx; a.vals = vals; a.X = X; a.Y = Y;
    a.N = N; a.seed = seed; a.F = F; a.ldx = ldx; a.ldy = ldy;
    a.W = (mode == ES_FULL) ? INT32_MAX : W;
    a.mode = mode; a.logR = p.logR; a.norm = norm; a.long_k = p.long_k;
    a.nblocks = (uint32_t)p.nblocks; a.blocks_per_xcd = (uint32_t)p.per_xcd;
    a.long_blocks = (uint32_t)p.long_blocks;
    a.cuts = nullptr; a.part_cols = 0; a.phase = 0;

    const dim3 grid((uint32_t)p.grid_x, (uint32_t)p.grid_y);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t err = hipErrorInvalidValue;
    // RowKey form: the gathered matrix is X (forward) or dX (backward, the
    // matrix passed as Y here); its largest row offset in RowKey units must fit 32 bits
    const int64_t gather_ld = backward ? ldy : ldx;
    const bool key_aligned = !backward && s.aligned;
    const int64_t stride_units = key_aligned ? gather_ld / 4 : gather_ld;
    const bool wide = (uint64_t)N * (uint64_t)stride_units > 0xFFFFFFFFull;
    a.stride_units = wide ? 0u : (uint32_t)stride_units;
#define ES_LAUNCH(G_, CH_, V_, A_, W_)                                                              \
    (p.partition ? launch_partitioned<G_, CH_, V_, A_, W_>(a, grid, static_cast<int32_t*>(workspace), st) \
                 : launch_forward<G_, CH_, V_, A_, W_>(a, grid, st))
#define ES_CASE(G_, CH_, V_, A_)                                                          \
    if (!backward && !p.flat && s.G == G_ && s.CH == CH_ && s.vec == V_ && s.aligned == A_) \
        err = wide ? ES_LAUNCH(G_, CH_, V_, A_, true) : ES_LAUNCH(G_, CH_, V_, A_, false);
    ES_CASE(4, 1, 4, true) ES_CASE(8, 1, 4, true) ES_CASE(16, 1, 4, true) ES_CASE(32, 1, 4, true)
    ES_CASE(64, 1, 4, true) ES_CASE(64, 2, 4, true) ES_CASE(64, 4, 4, true)
    ES_CASE(4, 1, 4, false) ES_CASE(8, 1, 4, false) ES_CASE(16, 1, 4, false) ES_CASE(32, 1, 4, false)
    ES_CASE(64, 1, 4, false) ES_CASE(64, 2, 4, false) ES_CASE(64, 4, 4, false)
    ES_CASE(4, 1, 1, false)
#define ES_BWD(G_, CH_)                         \
    if (backward && s.G == G_ && s.CH == CH_)   \
        err = wide ? launch_backward<G_, CH_, true>(a, grid, st) : launch_backward<G_, CH_, false>(a, grid, st);
    ES_BWD(4, 1) ES_BWD(8, 1) ES_BWD(16, 1) ES_BWD(32, 1) ES_BWD(64, 1) ES_BWD(64, 2) ES_BWD(64, 4)
#define ES_FLAT(G_, A_)                                                                         \
    if (p.flat && s.G == G_ && s.aligned == A_)                                                 \
        err = wide ? launch_flat<G_, A_, true>(a, grid, p.partition, static_cast<int32_t*>(workspace), st)  \
                   : launch_flat<G_, A_, false>(a, grid, p.partition, static_cast<int32_t*>(workspace), st);
    ES_FLAT(4, true) ES_FLAT(8, true) ES_FLAT(16, true) ES_FLAT(32, true) ES_FLAT(64, true)
    ES_FLAT(4, false) ES_FLAT(8, false) ES_FLAT(16, false) ES_FLAT(32, false) ES_FLAT(64, false)
#undef ES_FLAT
#undef ES_BWD
#undef ES_CASE
#undef ES_LAUNCH
    return err == hipSuccess ? ES_OK : ES_ERR_LAUNCH;
}

int build_transposed(const int32_t* rowptr, const int32_t* colidx, const float* vals, int64_t N,
                     int64_t nnz, int32_t W, int32_t mode, uint64_t seed, int32_t norm, int32_t* out_ptr,
                     int32_t* out_end, int32_t* out_idx, float* out_vals, int32_t* out_pos, void* stream);

}  // namespace

extern "C" {

const char* es_spmm_status_string(int status)
{
    switch (status) {
        case ES_OK: return "ES_OK";
        case ES_ERR_INVALID_ARG: return "ES_ERR_INVALID_ARG: null pointer, negative size, ld < F, W < 1 or unknown mode";
        case ES_ERR_UNSUPPORTED:
            return "ES_ERR_UNSUPPORTED: shape outside what the kernels cover (or more rows than "
                   "es_spmm_static_ws holds a workspace for: use es_spmm_ws)";
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
    return es_run(rowptr, colidx, vals, X, Y, N, nnz, F, ldx, ldy, W, mode, seed, norm, false, nullptr,
                  nullptr, 0, stream);
}

int es_spmm_ex(const int32_t* rowptr, const int32_t* colidx, const float* vals, const float* X,
               float* Y, int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W,
               int32_t mode, uint64_t seed, int32_t norm, const es_launch_opts_t* opts, void* stream)
{
    return es_run(rowptr, colidx, vals, X, Y, N, nnz, F, ldx, ldy, W, mode, seed, norm, false, opts,
                  nullptr, 0, stream);
}

size_t es_spmm_workspace_bytes(int64_t N) { return N < 0 ? 0 : part_workspace_bytes(N); }

int es_spmm_ws(const int32_t* rowptr, const int32_t* colidx, const float* vals, const float* X,
               float* Y, int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W,
               int32_t mode, uint64_t seed, int32_t norm, const es_launch_opts_t* opts, void* workspace,
               size_t workspace_bytes, void* stream)
{
    return es_run(rowptr, colidx, vals, X, Y, N, nnz, F, ldx, ldy, W, mode, seed, norm, false, opts,
                  workspace, workspace_bytes, stream);
}

int es_spmm_static_ws(const int32_t* rowptr, const int32_t* colidx, const float* vals, const float* X,
                      float* Y, int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W,
                      int32_t mode, uint64_t seed, int32_t norm, const es_launch_opts_t* opts, void* stream)
{
    // argument errors first (as every entry point), then the capacity of the
    // static array, then -- the first thing that touches the GPU -- its address
    const int bad = check_sizes(N, nnz, F, ldx, ldy, W, mode, norm);
    if (bad != ES_OK) return bad;
    Overrides ov;
    const int bad_opts = parse_opts(opts, &ov);
    if (bad_opts != ES_OK) return bad_opts;
    if (N > ES_SPMM_STATIC_WS_MAX_ROWS) return ES_ERR_UNSUPPORTED;
    if (N == 0) return ES_OK;
    if (!rowptr || !X || !Y || (nnz > 0 && !colidx)) return ES_ERR_INVALID_ARG;
    void* ws = nullptr;
    const int rc = static_scratch_address(&ws);
    if (rc != ES_OK) return rc;
    return es_run(rowptr, colidx, vals, X, Y, N, nnz, F, ldx, ldy, W, mode, seed, norm, false, opts, ws,
                  sizeof(scratch), stream);
}

int es_spmm_backward(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                     const float* dY, float* dX, int64_t N, int64_t nnz, int32_t F, int32_t ldy,
                     int32_t ldx, int32_t W, int32_t mode, uint64_t seed, int32_t norm, void* stream)
{
    return es_run(rowptr, colidx, vals, dY, dX, N, nnz, F, ldy, ldx, W, mode, seed, norm, true, nullptr,
                  nullptr, 0, stream);
}

int es_spmm_backward_ex(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                        const float* dY, float* dX, int64_t N, int64_t nnz, int32_t F, int32_t ldy,
                        int32_t ldx, int32_t W, int32_t mode, uint64_t seed, int32_t norm,
                        const es_launch_opts_t* opts, void* stream)
{
    return es_run(rowptr, colidx, vals, dY, dX, N, nnz, F, ldy, ldx, W, mode, seed, norm, true, opts,
                  nullptr, 0, stream);
}

int es_spmm_launch_info(int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W,
                        int32_t mode, int32_t aligned16, int32_t backward,
                        const es_launch_opts_t* opts, es_launch_info_t* info)
{
    if (!info) return ES_ERR_INVALID_ARG;
    Overrides ov;
    const int bad_opts = parse_opts(opts, &ov);
    if (bad_opts != ES_OK) return bad_opts;
    const int bad = check_sizes(N, nnz, F, ldx, ldy, W, mode, ES_NORM_NONE);
    if (bad != ES_OK) return bad;
    if (N == 0) return ES_ERR_INVALID_ARG;
    const bool aligned = aligned16 && (F % 4 == 0) && (ldx % 4 == 0) && (ldy % 4 == 0);
    Plan p;
    const int rc = make_plan(N, nnz, F, W, mode, aligned, backward != 0, ov, true, &p);
    if (rc != ES_OK) return rc;
    info->vector_width = p.s.vec;
    info->aligned = p.s.aligned ? 1 : 0;
    info->lanes_per_row = p.s.G;
    info->chunks_per_lane = p.s.CH;
    info->rows_per_wave = 1 << p.logR;
    info->edge_slots = p.flat ? 64 / p.s.G : (64 >> p.logR) / p.s.G;
    info->loads_in_flight = 8 / p.s.CH;
    info->tile_slots_per_row = kTileSlots >> p.logR;
    info->long_row_threshold = p.long_k;
    info->long_row_workgroups = p.long_blocks;
    info->grid_x = p.grid_x;
    info->grid_y = p.grid_y;
    info->flattened = p.flat ? 1 : 0;
    info->column_ranges = p.partition ? kParts : 1;
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
    return build_transposed(rowptr, colidx, vals, N, nnz, W, mode, seed, norm, out_ptr, out_end, out_idx,
                            out_vals, nullptr, stream);
}

int es_spmm_transpose_graph(const int32_t* rowptr, const int32_t* colidx, const float* vals, int64_t N,
                            int64_t nnz, int32_t* t_ptr, int32_t* t_end, int32_t* t_row, int32_t* t_idx,
                            int32_t* t_slot, float* t_vals, int32_t* t_pinv, void* stream)
{
    if (N > 0 && (!t_idx || !t_slot || !t_pinv)) return ES_ERR_INVALID_ARG;
    // t_idx first receives every entry's CSR position, then becomes its entry number
    const int rc = build_transposed(rowptr, colidx, vals, N, nnz, 0, ES_FULL, 0, ES_NORM_NONE, t_ptr, t_end,
                                    t_row, t_vals, t_idx, stream);
    if (rc != ES_OK || N == 0) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t pb = (N + kBlockThreads - 1) / kBlockThreads;
    if (pb > INT32_MAX) return ES_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(es_pinv_kernel, dim3((uint32_t)pb), dim3(kBlockThreads), 0, st, rowptr, N, t_pinv);
    if (hipGetLastError() != hipSuccess) return ES_ERR_LAUNCH;
    int64_t eb = (nnz + kBlockThreads - 1) / kBlockThreads;
    if (eb > 65536) eb = 65536;
    if (eb > 0) {
        hipLaunchKernelGGL(es_pull_entries_kernel, dim3((uint32_t)eb), dim3(kBlockThreads), 0, st, rowptr,
                           t_pinv, t_row, nnz, t_idx, t_slot);
        if (hipGetLastError() != hipSuccess) return ES_ERR_LAUNCH;
    }
    return ES_OK;
}

int es_spmm_backward_pull(const int32_t* rowptr, const int32_t* t_ptr, const int32_t* t_row,
                          const int32_t* t_idx, const int32_t* t_slot, const float* t_vals,
                          const int32_t* t_pinv, int32_t* t_rows, const float* dY, float* dX, int64_t N,
                          int64_t nnz, int32_t F, int32_t ldy, int32_t ldx, int32_t W, int32_t mode,
                          uint64_t seed, int32_t norm, void* stream)
{
    const int bad = check_sizes(N, nnz, F, ldy, ldx, W, mode, norm);
    if (bad != ES_OK) return bad;
    if (N == 0) return ES_OK;
    if (!rowptr || !t_ptr || !dY || !dX) return ES_ERR_INVALID_ARG;
    if (!t_pinv || !t_rows || reinterpret_cast<uintptr_t>(t_rows) % 8) return ES_ERR_INVALID_ARG;
    if (nnz > 0 && (!t_row || !t_idx || !t_slot || !t_vals)) return ES_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(dY) % 4 || reinterpret_cast<uintptr_t>(dX) % 4) return ES_ERR_INVALID_ARG;
    const bool aligned = (F % 4 == 0) && (ldx % 4 == 0) && (ldy % 4 == 0) &&
                         (reinterpret_cast<uintptr_t>(dY) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(dX) % 16 == 0);
    const Shape s = pick_shape(F, aligned);
    Args a;
    a.rowptr = rowptr; a.colidx = nullptr; a.vals = nullptr; a.X = dY; a.Y = dX;
    a.N = N; a.seed = seed; a.F = F; a.ldx = ldy; a.ldy = ldx;
    a.W = (mode == ES_FULL) ? INT32_MAX : W;
    a.mode = mode; a.logR = 0; a.norm = norm; a.long_k = INT32_MAX;
    const int64_t nblocks = (N + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t per_xcd = (nblocks + kNumXcd - 1) / kNumXcd;
    a.nblocks = (uint32_t)nblocks; a.blocks_per_xcd = (uint32_t)per_xcd; a.long_blocks = 0;
    a.cuts = nullptr; a.part_cols = 0; a.phase = 0;
    const int cols_per_block = s.G * s.CH * s.vec;
    const int64_t grid_y = ((int64_t)F + cols_per_block - 1) / cols_per_block;
    if (per_xcd * kNumXcd > INT32_MAX || grid_y > 65535) return ES_ERR_UNSUPPORTED;
    const int64_t stride_units = s.aligned ? ldy / 4 : ldy;          // rows of dY are what gets gathered
    const bool wide = (uint64_t)N * (uint64_t)stride_units > 0xFFFFFFFFull;
    a.stride_units = wide ? 0u : (uint32_t)stride_units;
    const dim3 grid((uint32_t)(per_xcd * kNumXcd), (uint32_t)grid_y);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // per-row (length, rotation) of this call
    int2* rows = reinterpret_cast<int2*>(t_rows);
    const int64_t rb = (N + kBlockThreads - 1) / kBlockThreads;
    if (rb > INT32_MAX) return ES_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(es_pull_rows_kernel, dim3((uint32_t)rb), dim3(kBlockThreads), 0, st, rowptr, t_pinv, N,
                       mode, seed, a.W, rows);
    if (hipGetLastError() != hipSuccess) return ES_ERR_LAUNCH;
    bool launched = false;
#define ES_PULL(G_, CH_, V_, A_)                                                                     \
    if (s.G == G_ && s.CH == CH_ && s.vec == V_ && s.aligned == A_) {                                \
        if (wide)                                                                                    \
            hipLaunchKernelGGL((es_pull_kernel<G_, CH_, V_, A_, true>), grid, dim3(kBlockThreads), 0, st, a,  \
                               t_ptr, t_row, t_idx, t_slot, t_vals, rows);                                 \
        else                                                                                         \
            hipLaunchKernelGGL((es_pull_kernel<G_, CH_, V_, A_, false>), grid, dim3(kBlockThreads), 0, st, a, \
                               t_ptr, t_row, t_idx, t_slot, t_vals, rows);                                 \
        launched = true;                                                                             \
    }
    ES_PULL(4, 1, 4, true) ES_PULL(8, 1, 4, true) ES_PULL(16, 1, 4, true) ES_PULL(32, 1, 4, true)
    ES_PULL(64, 1, 4, true) ES_PULL(64, 2, 4, true) ES_PULL(64, 4, 4, true)
    ES_PULL(4, 1, 4, false) ES_PULL(8, 1, 4, false) ES_PULL(16, 1, 4, false) ES_PULL(32, 1, 4, false)
    ES_PULL(64, 1, 4, false) ES_PULL(64, 2, 4, false) ES_PULL(64, 4, 4, false)
    ES_PULL(4, 1, 1, false)
#undef ES_PULL
    if (!launched) return ES_ERR_UNSUPPORTED;
    return hipGetLastError() == hipSuccess ? ES_OK : ES_ERR_LAUNCH;
}

}  // extern "C"

namespace {

// Transposed (sampled) graph: count the kept entries per column, scan, then
// drop every entry into its column's segment through a per-column cursor.
int build_transposed(const int32_t* rowptr, const int32_t* colidx, const float* vals, int64_t N,
                     int64_t nnz, int32_t W, int32_t mode, uint64_t seed, int32_t norm, int32_t* out_ptr,
                     int32_t* out_end, int32_t* out_idx, float* out_vals, int32_t* out_pos, void* stream)
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
                       out_vals, out_pos);
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
                       out_vals, out_pos);
    ES_CHECK_LAUNCH();
#undef ES_CHECK_LAUNCH
    return ES_OK;
}

}  // namespace

extern "C" {

int es_spmm_validate_csr(const int32_t* rowptr, const int32_t* colidx, int64_t N, int64_t nnz,
                         int32_t* report, void* stream)
{
    if (N < 0 || nnz < 0 || nnz > INT32_MAX || !rowptr || !report) return ES_ERR_INVALID_ARG;
    if (nnz > 0 && !colidx) return ES_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(es_fill_int_kernel, dim3(1), dim3(kBlockThreads), 0, st, report, (int64_t)4, 0);
    if (hipGetLastError() != hipSuccess) return ES_ERR_LAUNCH;
    int64_t blocks = (N + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks < 1) blocks = 1;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(es_validate_csr_kernel, dim3((uint32_t)blocks), dim3(kBlockThreads), 0, st, rowptr,
                       colidx, N, nnz, report);
    return hipGetLastError() == hipSuccess ? ES_OK : ES_ERR_LAUNCH;
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
