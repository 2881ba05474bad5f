// es_aux_kernels.h -- kernels that only walk the sampler: edge-list export, materialised sampled graph (scan + write), its transpose.
#ifndef ES_SPMM_AUX_KERNELS_H
#define ES_SPMM_AUX_KERNELS_H

#include "es_tile.h"

namespace {

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
//                (value times the row factor) and, if asked for, out_pos (its
//                position in the original CSR arrays).
template <bool FILL>
__global__ void __launch_bounds__(kBlockThreads)
es_transpose_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                    const float* __restrict__ vals, int64_t N, int32_t W, int32_t mode, uint64_t seed,
                    int32_t norm, int32_t logR, int32_t* out_ptr, int32_t* out_end,
                    int32_t* __restrict__ out_idx, float* __restrict__ out_vals,
                    int32_t* __restrict__ out_pos)
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
                if (out_pos) out_pos[pos] = (int32_t)p;      // where the entry sits in the original CSR
            }
        });
    }
}

// ---------------------------------------------------------------------------
// CSR check: what es_spmm takes on trust (row pointers that start at 0, never
// decrease and end at nnz; column ids inside [0, N)).  One wave per row; a
// row's entries are only read when its own pointer pair lies inside [0, nnz].
// report[0] = bad row-pointer pairs (plus 1 each if rowptr[0] != 0 or
// rowptr[N] != nnz), report[1] = column ids outside [0, N), report[2] = rows
// whose column ids are not strictly increasing, report[3] = longest row.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlockThreads)
es_validate_csr_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                       int64_t N, int64_t nnz, int32_t* report)
{
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t waves = (int64_t)gridDim.x * kWavesPerBlock;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (rowptr[0] != 0) atomicAdd(report + 0, 1);
        if ((int64_t)rowptr[N] != nnz) atomicAdd(report + 0, 1);
    }
    for (int64_t r = (int64_t)blockIdx.x * kWavesPerBlock + wave; r < N; r += waves) {
        const int64_t b = rowptr[r], e = rowptr[r + 1];
        if (b < 0 || e < b || e > nnz) {
            if (lane == 0) atomicAdd(report + 0, 1);
            continue;
        }
        int bad_col = 0, unsorted = 0;
        for (int64_t p = b + lane; p < e; p += kWaveSize) {
            const int32_t c = colidx[p];
            if (c < 0 || (int64_t)c >= N) ++bad_col;
            if (p > b && colidx[p - 1] >= c) unsorted = 1;
        }
#pragma unroll
        for (int m = 1; m < kWaveSize; m <<= 1) {
            bad_col += __shfl_xor(bad_col, m, kWaveSize);
            unsorted |= __shfl_xor(unsorted, m, kWaveSize);
        }
        if (lane == 0) {
            if (bad_col) atomicAdd(report + 1, bad_col);
            if (unsorted) atomicAdd(report + 2, 1);
            atomicMax(report + 3, (int32_t)(e - b));
        }
    }
}

}  // namespace

#endif  // ES_SPMM_AUX_KERNELS_H
