// es_common.h -- constants and the kernel argument block shared by every kernel of the library.
#ifndef ES_SPMM_COMMON_H
#define ES_SPMM_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>
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
constexpr int kParts = kNumXcd;                       // column ranges of the partitioned product
constexpr int kPartLongPiece = 256;                   // pieces above this many entries start first
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
    uint32_t stride_units;     // row stride of the gathered (scattered) matrix in RowKey units
    int32_t long_k;            // rows keeping more entries go to the long-row part  
    int32_t norm;              // es_norm_t: row factor applied before the store
    uint32_t nblocks;          // workgroups that carry rows
    uint32_t blocks_per_xcd;   // ceil(nblocks / 8)
    uint32_t long_blocks;      // leading workgroups that run the long-row part
    // column-partitioned product only
    const int32_t* cuts;       // [N x kParts]: row r's piece of column range j starts at entry cuts[r][j]
    int32_t part_cols;         // columns per range, ceil(N / kParts)
    int32_t phase;             // 0 .. kParts-1: which row range each XCD serves in this launch
};

}  // namespace

#endif  // ES_SPMM_COMMON_H
