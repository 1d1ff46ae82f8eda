// Shared by the fused attention kernels: the LDS layout of a [64 rows x head-dim] bf16 tile that is
// read both row-wise (MFMA operands with the head dimension as K) and with transposing reads
// (operands with the tile's rows as K).
#pragma once
#include "gemm_bf16_dtl.hip.h"

namespace mecefo {

// XOR swizzle of the 16-byte chunk index inside a tile row.  Two access patterns must stay free of
// bank conflicts: 16 lanes reading one chunk column of 16 consecutive rows (A operands), and 32 lanes
// reading 64 bytes of each of four consecutive rows (transposing B-operand reads).  The first needs
// 16 distinct chunk positions over 16 rows, the second needs rows that differ in their low bits to land
// in different 64-byte groups, hence the low row bits go to the high chunk bits.
template <int DH> __device__ inline int tile_swz(int row) {
  if constexpr (DH == 128) return ((row & 3) << 2) | ((row >> 2) & 3);     // 16 chunks per 256-byte row
  else return ((row >> 1) & 1) << 2 | ((row >> 2) & 1) << 1 | ((row >> 3) & 1);   // 8 chunks per 128-byte row
}

}  // namespace mecefo
