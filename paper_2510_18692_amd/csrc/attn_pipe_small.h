// bf16 forward kernel of the group attention for SMALL groups (head_dim 128): the static groups of
// Section 3.2 have a few hundred to a few thousand rows, where the 256-row, 8-wave kernel of
// attn_pipe.h wastes most of its last query tile and its three-tile prologue is not amortised.
//
// Same step (pipe_step) and operand layouts, but a block is 4 waves x 32 query rows (128-row
// tiles) and streams K/V in tiles of 32 keys through a ring of four 8 KB + 8 KB slots: 64 KB of
// LDS, so TWO blocks share a CU.  They run independently: one block's prologue, epilogue and
// barrier waits are covered by the other block's waves on the same SIMDs.
#pragma once

#include "attn_pipe.h"

namespace moga {

constexpr int kSmallTileBytes = 32 * kHeadDim * 2;   // 8 KB per K (or V) tile of 32 keys

// Issue the loads of the 32-key tile starting at group-relative row kv0 into ring slot `buf`:
// two rounds, each of the 4 waves moving 4 rows of K and 4 rows of V per round.
__device__ __forceinline__ void small_issue_tile(const PipeDma& d, int kv0, int buf) {
  const unsigned boff = (unsigned)buf * kSmallTileBytes;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = min(kv0 + d.row0 + 16 * i, d.last_row);
    const unsigned off = (unsigned)row * (kHeadDim * 2) + d.chunk_off;
    lds_dma16_soff(d.kbase, off, d.lds_k + boff + i * 4096);
    lds_dma16_soff(d.vbase, off, d.lds_v + boff + i * 4096);
  }
}

// Arguments as attn_fwd_bf16_pipe_kernel (no gather mode); tiles of 128 query rows.
__global__ __launch_bounds__(256, 2) void attn_fwd_bf16_small_kernel(
    const unsigned short* __restrict__ qh, const unsigned short* __restrict__ kh,
    const unsigned short* __restrict__ vh, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_k, const int32_t* __restrict__ tile_start, int M,
    int64_t Nq, int64_t Nk, int H, float scale, int tiles_per_head, unsigned short* __restrict__ oh,
    float* __restrict__ lse) {
  constexpr int NW = 4, QW = 1, BM = 128;
  constexpr int kDmaPerTile = 4;   // direct-to-LDS instructions per thread per tile
  constexpr int kAhead = 2;        // tiles in flight beyond the one being waited for
  __shared__ __attribute__((aligned(1024))) unsigned short Ks[4][32 * kHeadDim];
  __shared__ __attribute__((aligned(1024))) unsigned short Vs[4][32 * kHeadDim];
  __shared__ int s_start[MOGA_MAX_GROUPS + 1];
  __shared__ int s_found;

  const int64_t total = (int64_t)H * tiles_per_head;
  const int64_t work = xcd_work_index(blockIdx.x, total);
  if (work >= total) return;
  const int head = (int)(work / tiles_per_head);
  const int tile = (int)(work - (int64_t)head * tiles_per_head);
  TileInfo ti;
  if (tile_start) {
    if (!find_tile_presummed(tile_start, cu_q, M, BM, tile, ti)) return;
  } else if (!find_tile(cu_q, M, BM, tile, s_start, &s_found, ti)) {
    return;
  }
  const int ge = ti.row_end, q0 = ti.tile_row;   // query rows of the group end at ge
  const int gs = cu_k[ti.group];                 // first key row of the group
  const int n = cu_k[ti.group + 1] - gs;         // number of keys

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int r = lane & 31, h = lane >> 5;
  const int64_t head_off = (int64_t)head * Nq;
  const int64_t head_off_k = (int64_t)head * Nk;
  const float c = scale * 1.4426950408889634f;
  const float tau = 8.f / c;
  const int qrow = q0 + wave * 32 + r;

  if (n <= 0) {   // queries without keys: zero output, lse = -inf (block-uniform branch)
    if (qrow < ge) {
      uintx4_t* op = (uintx4_t*)(oh + (head_off + qrow) * kHeadDim + 64 * h);
      const uintx4_t z = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int i = 0; i < 8; ++i) op[i] = z;
      if (h == 0) lse[head_off + qrow] = -INFINITY;
    }
    return;
  }

  // Q fragments (B operand): lane (r, h) holds Q[q = r][d = 16*ks + 8*h + 0..7]
  bf16x8_t qf[QW][8];
  {
    const int qr = qrow > ge - 1 ? ge - 1 : qrow;
    const unsigned short* qp = qh + (head_off + qr) * kHeadDim + 8 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[0][ks] = *(const bf16x8_t*)(qp + 16 * ks);
  }

  PipeDma dma;
  dma.kbase = uniform_ptr(kh + (head_off_k + gs) * kHeadDim);
  dma.vbase = uniform_ptr(vh + (head_off_k + gs) * kHeadDim);
  dma.lds_k = lds_addr_uniform(&Ks[0][0]) + wave * 1024;
  dma.lds_v = lds_addr_uniform(&Vs[0][0]) + wave * 1024;
  dma.row0 = 4 * wave + (lane >> 4);
  dma.chunk_off = (unsigned)(((lane & 15) ^ lds_swizzle(dma.row0)) * 16);
  dma.last_row = n - 1;
#pragma unroll
  for (int t = 0; t <= kAhead; ++t) small_issue_tile(dma, 32 * t, t);   // rows are clamped: always issued

  PipeLane ln;
  {
    const int krow_a = swap_bits_2_3(r);
    const int k_sw = lds_swizzle(krow_a);
    const unsigned kb = (unsigned)(uintptr_t)&Ks[0][0] + krow_a * 256;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) ln.k_addr[ks] = kb + (((2 * ks + h) ^ k_sw) << 4);
    const int tr_r = 8 * h + ((lane & 15) >> 2);
    const int tr_c = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
    const int tr_e = 4 * (lane & 1);
    const unsigned vb = (unsigned)(uintptr_t)&Vs[0][0] + tr_e * 2;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      ln.v_addr[dt][0] = vb + tr_r * 256 + (((4 * dt + tr_c) ^ lds_swizzle(tr_r)) << 4);
      ln.v_addr[dt][1] = vb + (tr_r + 4) * 256 + (((4 * dt + tr_c) ^ lds_swizzle(tr_r + 4)) << 4);
    }
  }

  PipeState<QW> st;
  st.m[0] = -INFINITY;
  st.l[0] = 0.f;
  st.negmc[0] = 0.f;
  st.thresh[0] = -INFINITY;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) st.o[0][dt][v] = 0.f;

  const int nsteps = (n + 31) >> 5;
  const int nfull = n >> 5;   // steps whose 32 keys are all inside the group

  // prologue: scores of step 0 (tile 0)
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * kAhead));
  __syncthreads();
  if (q0 + wave * 32 >= ge) {
    // every query row of this wave lies past the end of the group: it only moves its share of the K/V
    // tiles and keeps the barriers of the loops below, one per step
    for (int s = 0; s < nsteps; ++s) {
      __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * (kAhead - 1)));
      __syncthreads();
      small_issue_tile(dma, 32 * (s + 1 + kAhead), (s + 1 + kAhead) & 3);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    return;
  }
  floatx16_t s_a[QW], s_b[QW];   // scores of even / odd steps
  float mx[QW];
  {
    bf16x8_t kf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kf[ks] = lds_read_b128(ln.k_addr[ks]);
#pragma unroll
    for (int v = 0; v < 16; ++v) s_a[0][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      s_a[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[0][ks], s_a[0], 0, 0, 0);
    if (nfull == 0) mask_step(s_a[0], 0, h, n);
    mx[0] = step_max(s_a[0]);
  }

  // main loop.  Step s (= tile s) lives in ring slot s % 4: it reads its values from that slot and
  // the keys of step s+1 from the next one.  At the top of a step the block waits for tile s+1 and
  // refills the slot of tile s-1 with tile s+3.  Four steps per iteration: every LDS offset is an
  // immediate.
  int s = 0;
#define MOGA_SMALL_STEP(B, SA, SB)                                                        \
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * (kAhead - 1)));                     \
  __syncthreads();                                                                        \
  small_issue_tile(dma, 32 * (s + (B) + 1 + kAhead), ((B) + 1 + kAhead) & 3);             \
  maybe_rescale<QW>(st, mx, c, tau);                                                      \
  pipe_step<QW, true, (((B) + 1) & 3) * kSmallTileBytes, (B) * kSmallTileBytes>(ln, 0, 0, qf, st, SA, SB, mx, c);
  for (; s + 4 <= nfull - 1; s += 4) {   // steps s .. s+3 and their successors are full
    MOGA_SMALL_STEP(0, s_a, s_b)
    MOGA_SMALL_STEP(1, s_b, s_a)
    MOGA_SMALL_STEP(2, s_a, s_b)
    MOGA_SMALL_STEP(3, s_b, s_a)
  }
#undef MOGA_SMALL_STEP

  // tail: at most four steps and a partial one (s is a multiple of 4 here), ring offsets at run time
  for (; s < nsteps; ++s) {
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * (kAhead - 1)));
    __syncthreads();
    small_issue_tile(dma, 32 * (s + 1 + kAhead), (s + 1 + kAhead) & 3);
    const bool has_next = s + 1 < nsteps;
    maybe_rescale<QW>(st, mx, c, tau);
    const unsigned voff = (unsigned)(s & 3) * kSmallTileBytes;
    const unsigned koff = (unsigned)((s + 1) & 3) * kSmallTileBytes;
    if (has_next) {
      pipe_step<QW, true>(ln, koff, voff, qf, st, s_a, s_b, mx, c);
      if (s + 1 >= nfull) mask_step(s_b[0], 32 * (s + 1), h, n);
      s_a[0] = s_b[0];
      if (s + 1 >= nfull) mx[0] = step_max(s_a[0]);
    } else {
      pipe_step<QW, false>(ln, koff, voff, qf, st, s_a, s_b, mx, c);
    }
  }

  // epilogue: register v of d tile dt is d = 32*dt + 8*(v/4) + 4*h + v%4 of query column r
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // drain the look-ahead loads before the LDS is released
  {
    const auto rr = __builtin_amdgcn_permlane32_swap(__float_as_uint(st.l[0]), __float_as_uint(st.l[0]), false, false);
    const float lt = __uint_as_float(rr[0]) + __uint_as_float(rr[1]);
    const float inv = 1.f / lt;
    if (qrow < ge) {
      unsigned short* op = oh + (head_off + qrow) * kHeadDim + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          uintx2_t pk = {pack_bf16x2(st.o[0][dt][4 * b] * inv, st.o[0][dt][4 * b + 1] * inv),
                         pack_bf16x2(st.o[0][dt][4 * b + 2] * inv, st.o[0][dt][4 * b + 3] * inv)};
          *(uintx2_t*)(op + 32 * dt + 8 * b) = pk;
        }
      if (h == 0) lse[head_off + qrow] = st.m[0] * scale + logf(lt);
    }
  }
}

}  // namespace moga
