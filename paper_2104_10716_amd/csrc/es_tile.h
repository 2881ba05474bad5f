// es_tile.h -- per-lane column packs and the two stages of Algorithm 1 on one LDS tile (stage, consume / scatter).
#ifndef ES_SPMM_TILE_H
#define ES_SPMM_TILE_H

#include "es_sampler.h"

namespace {

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
    // as load(), marked as data this kernel reads once
    __device__ __forceinline__ void load_streaming(const float* p)
    {
        if (ALIGNED) {
            typedef float float4_v __attribute__((ext_vector_type(4)));
            const float4_v t = __builtin_nontemporal_load(reinterpret_cast<const float4_v*>(p));
            v = make_float4(t.x, t.y, t.z, t.w);
        } else {
            load(p);
        }
    }
    // as store(), marked as data this kernel will not read again (kept out of the way of X in the L2)
    __device__ __forceinline__ void store_streaming(float* p, int first) const
    {
        if (ALIGNED) {
            typedef float float4_v __attribute__((ext_vector_type(4)));
            float4_v t = {v.x, v.y, v.z, v.w};
            __builtin_nontemporal_store(t, reinterpret_cast<float4_v*>(p));
        } else {
            store(p, first);
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
    __device__ __forceinline__ void mul(float a, const Pack& x) { v.x = a * x.v.x; v.y = a * x.v.y; v.z = a * x.v.z; v.w = a * x.v.w; }
    __device__ __forceinline__ void scale(float f) { v.x *= f; v.y *= f; v.z *= f; v.w *= f; }
    __device__ __forceinline__ void add(const Pack& o) { v.x += o.v.x; v.y += o.v.y; v.z += o.v.z; v.w += o.v.w; }
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
    __device__ __forceinline__ void store_streaming(float* p, int) const { __builtin_nontemporal_store(v, p); }
    __device__ __forceinline__ void atomic_add(float* p, int) const { unsafeAtomicAdd(p, v); }
    __device__ __forceinline__ void fma(float a, const Pack& x) { v = fmaf(a, x.v, v); }
    __device__ __forceinline__ void scale(float f) { v *= f; }
    __device__ __forceinline__ void add(const Pack& o) { v += o.v; }
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

// How a staged column id turns into the address of that row of the dense
// matrix.  WIDE == false: stage 1 stores the row's offset, column * stride,
// as a 32-bit count of UNIT floats (UNIT = 4 for 16-byte aligned rows, else 1),
// so that stage 2 forms an address with one shift-add instead of a 64-bit
// multiply per gathered row; the host picks this form whenever the largest
// offset fits 32 bits (matrices up to 64 GB, or 16 GB for unaligned rows).
// WIDE == true: the column id is stored and multiplied in stage 2.
template <bool ALIGNED, bool WIDE>
struct RowKey {
    static constexpr int UNIT = ALIGNED ? 4 : 1;
    __device__ __forceinline__ static uint32_t make(int32_t col, uint32_t stride_units)
    {
        return WIDE ? (uint32_t)col : (uint32_t)col * stride_units;
    }
    __device__ __forceinline__ static const float* row(const float* base, uint32_t key, int64_t stride)
    {
        return WIDE ? base + (int64_t)key * stride : base + (size_t)key * UNIT;
    }
    __device__ __forceinline__ static float* row(float* base, uint32_t key, int64_t stride)
    {
        return WIDE ? base + (int64_t)key * stride : base + (size_t)key * UNIT;
    }
};

// Stage 1 of Algorithm 1 for one tile: copy the sampled (column, value) pairs
// of slots [0, count) into the LDS tile (the column as its RowKey).
template <bool ALIGNED, bool WIDE>
__device__ __forceinline__ void stage_tile(RowSampler& sampler, int t, int team, int count,
                                           int32_t base, const int32_t* __restrict__ colidx,
                                           const float* __restrict__ vals, uint32_t stride_units, uint2* tile)
{
    sample_tile(sampler, t, team, count, [&](int slot, uint32_t entry) {
        const int64_t p = (int64_t)base + entry;
        const int32_t c = colidx[p];
        const float v = vals ? vals[p] : 1.0f;
        tile[slot] = make_uint2(RowKey<ALIGNED, WIDE>::make(c, stride_units), __float_as_uint(v));
    });
}

// Stage 2 of Algorithm 1 for one tile: this lane's edge slot e (of E) walks
// tile entries e, e+E, ... < count, U at a time: U LDS broadcasts, then U*CH
// independent loads of X, then the FMAs.
template <int G, int CH, int VEC, bool ALIGNED, bool WIDE>
__device__ __forceinline__ void consume_tile(const uint2* tile, int count, int e, int E,
                                             const float* __restrict__ X, int64_t ldx,
                                             const LaneCols<G, CH, VEC, ALIGNED>& cols,
                                             Pack<VEC, ALIGNED> (&acc)[CH])
{
    constexpr int U = 8 / CH;
    using P = Pack<VEC, ALIGNED>;
    using K = RowKey<ALIGNED, WIDE>;
    int j = e;
    for (; j + (U - 1) * E < count; j += U * E) {            // full batches
        uint2 ed[U];
#pragma unroll
        for (int u = 0; u < U; ++u) ed[u] = tile[j + u * E];
        P x[U][CH];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float* xr = K::row(X, ed[u].x, ldx);
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
            const float* xr = K::row(X, ed[u].x, ldx);
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
template <int G, int CH, int VEC, bool ALIGNED, bool WIDE>
__device__ __forceinline__ void scatter_tile(const uint2* tile, int count, int e, int E, float* out,
                                             int64_t ldo, const LaneCols<G, CH, VEC, ALIGNED>& cols,
                                             const Pack<VEC, ALIGNED> (&dy)[CH])
{
    for (int j = e; j < count; j += E) {
        const uint2 ed = tile[j];
        const float v = __uint_as_float(ed.y);
        float* dst = RowKey<ALIGNED, WIDE>::row(out, ed.x, ldo);
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

}  // namespace

#endif  // ES_SPMM_TILE_H
