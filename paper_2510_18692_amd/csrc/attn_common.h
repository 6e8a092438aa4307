// Pieces shared by the forward and backward group-attention kernels.
#pragma once

#include "lds_pipe.h"

namespace moga {

constexpr int kHeadDim = 128;  // head_dim of the bf16 MFMA kernels

// Tile schedule.  Every group g with n_g rows contributes ceil(n_g / rows_per_tile) tiles;
// tiles never straddle a group boundary.  `tile` is a flat index over all groups in order.
// Every thread of the block must call this (it contains block-wide barriers).  Returns false
// when `tile` lies beyond the last real tile (the grid is sized from an upper bound because
// the group sizes live on the device).
struct TileInfo {
  int group;      // group id
  int row_begin;  // first row of the group (sorted slot)
  int row_end;    // one past the last row of the group
  int tile_row;   // first row of this tile
};

__device__ __forceinline__ bool find_tile(const int32_t* __restrict__ cu_seqlens, int M,
                                          int rows_per_tile, int tile, int* s_start /*[M+1]*/,
                                          int* s_found, TileInfo& out) {
  const int lane = threadIdx.x & 63;
  if (threadIdx.x < 64) {
    int running = 0;
    for (int g0 = 0; g0 < M; g0 += 64) {
      const int g = g0 + lane;
      const int n = g < M ? cu_seqlens[g + 1] - cu_seqlens[g] : 0;
      const int t = (n + rows_per_tile - 1) / rows_per_tile;
      int incl = t;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += up;
      }
      if (g < M) s_start[g] = running + incl - t;
      running += __shfl(incl, 63, kWave);
    }
    if (lane == 0) { s_start[M] = running; *s_found = -1; }
  }
  __syncthreads();
  for (int g = threadIdx.x; g < M; g += blockDim.x)
    if (s_start[g] <= tile && tile < s_start[g + 1]) *s_found = g;
  __syncthreads();
  const int g = *s_found;
  if (g < 0) return false;
  out.group = g;
  out.row_begin = cu_seqlens[g];
  out.row_end = cu_seqlens[g + 1];
  out.tile_row = out.row_begin + (tile - s_start[g]) * rows_per_tile;
  return true;
}

// The same lookup for calls with many groups: `tile_start[g]` (M + 1 entries, written by
// tile_start_kernel) is the flat index of group g's first tile; every thread binary-searches it.
__device__ __forceinline__ bool find_tile_presummed(const int32_t* __restrict__ tile_start,
                                                    const int32_t* __restrict__ cu_seqlens, int M,
                                                    int rows_per_tile, int tile, TileInfo& out) {
  if (tile >= tile_start[M]) return false;
  int lo = 0, hi = M;   // invariant: tile_start[lo] <= tile < tile_start[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tile_start[mid] <= tile) lo = mid; else hi = mid;
  }
  out.group = lo;
  out.row_begin = cu_seqlens[lo];
  out.row_end = cu_seqlens[lo + 1];
  out.tile_row = out.row_begin + (tile - tile_start[lo]) * rows_per_tile;
  return true;
}

// One block: exclusive scan of ceil(n_g / rows_per_tile) over the groups, M + 1 results.
static __global__ __launch_bounds__(1024) void tile_start_kernel(const int32_t* __restrict__ cu_seqlens, int M,
                                                                 int rows_per_tile, int32_t* __restrict__ tile_start) {
  __shared__ int s_wave[16];
  __shared__ int s_carry;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) s_carry = 0;
  __syncthreads();
  for (int g0 = 0; g0 < M; g0 += 1024) {
    const int g = g0 + threadIdx.x;
    const int n = g < M ? cu_seqlens[g + 1] - cu_seqlens[g] : 0;
    const int t = n > 0 ? (n + rows_per_tile - 1) / rows_per_tile : 0;
    int incl = t;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o, kWave);
      if (lane >= o) incl += up;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    int before = s_carry;
    for (int w = 0; w < wave; ++w) before += s_wave[w];
    if (g < M) tile_start[g] = before + incl - t;
    __syncthreads();
    if (threadIdx.x == 1023) s_carry = before + incl;
    __syncthreads();
  }
  if (threadIdx.x == 0) tile_start[M] = s_carry;
}

// Upper bound on the number of tiles for N rows in M groups (host side).
inline int64_t max_tiles(int64_t N, int M, int rows_per_tile) {
  return (N + rows_per_tile - 1) / rows_per_tile + M;
}

// Work item of a block: blocks are dealt round-robin to the 8 XCDs by the hardware, so block
// b runs on XCD b % 8.  Give each XCD one contiguous eighth of the (head-major) work list, so
// that the K/V tiles of a head are streamed through a single L2.
__device__ __forceinline__ int64_t xcd_work_index(int64_t block, int64_t total) {
  const int64_t per = (total + 7) / 8;
  return (block & 7) * per + (block >> 3);
}

// Row permutation that makes the 32x32 MFMA accumulator registers of a lane hold eight
// consecutive contraction indices: swap bits 2 and 3 of the row index.
__device__ __forceinline__ int swap_bits_2_3(int x) {
  return (x & ~12) | ((x & 4) << 1) | ((x & 8) >> 1);
}

// XOR swizzle of the 16-byte chunk index inside an unpadded 256-byte LDS row (128 bf16):
// chunk' = chunk ^ lds_swizzle(row).  The two low row bits land in chunk bits 3:2 and row bits
// 3:2 in chunk bits 1:0, which spreads both the row-per-lane 16-byte reads and the 4-row
// transposed reads over all banks.
__device__ __forceinline__ int lds_swizzle(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

}  // namespace moga
