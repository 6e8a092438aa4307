// bf16 backward kernels of the group attention (head_dim 128) on the LDS ring of attn_pipe.h.
//
//   attn_bwd_dq_pipe_kernel   : a wave owns 32*QW query rows (Q, dO fragments, lse, delta and
//                               the dQ^T accumulators in registers) and sweeps 64-key tiles of
//                               K and V; three MFMA products per tile (S^T, dP^T, dQ^T).
//   attn_bwd_dkdv_ab_kernel   : a pair of waves on one SIMD owns 32 key rows and sweeps 64-query
//                               tiles of Q, dO, lse and delta; one wave computes S, P and dV^T,
//                               the other dP, dS and dK^T (P handed over through LDS).
// Tiles are streamed global -> LDS by direct-to-LDS loads into a ring of four slots, two tiles
// ahead; one block-wide barrier per tile.  Both kernels also come as 4-wave blocks with a two-slot
// ring (64 KB of LDS), two blocks per CU, for groups of a few thousand rows or less.
#pragma once

#include "attn_pipe.h"

namespace moga {

__device__ __forceinline__ void lds_dma4_soff(const void* base, unsigned byte_off, unsigned lds_wave_base) {
  lds_wave_base = __builtin_amdgcn_readfirstlane(lds_wave_base);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :
               : "s"(lds_wave_base), "v"(byte_off), "s"(base)
               : "memory");
}

__device__ __forceinline__ floatx4_t lds_read_f32x4(unsigned addr) {
  return *(const floatx4_t __attribute__((address_space(3)))*)(uintptr_t)addr;
}

// dQ kernel: P = exp2(s*c - lse2) and dS = P * (dP - delta) for the 16 scores of a lane (one query
// column per lane, so lse2 and delta are per-lane scalars), dS packed to bf16.
// `limit`: keys >= limit (relative to the step's first) get P = 0 (MASK only).
template <bool MASK>
__device__ __forceinline__ void softmax_bwd_cols(const floatx16_t& s, const floatx16_t& dp, float lse2,
                                                 float dlt, float c, int h, int limit, bf16x8_t (&dsf)[2]) {
#pragma unroll
  for (int kstep = 0; kstep < 2; ++kstep) {
    unsigned int dd[4];
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
      const int v = 8 * kstep + j;
      float pa = fast_exp2(fmaf(s[v], c, -lse2));
      float pb = fast_exp2(fmaf(s[v + 1], c, -lse2));
      if (MASK) {
        const int idx = 16 * kstep + 8 * h + j;
        if (idx >= limit) pa = 0.f;
        if (idx + 1 >= limit) pb = 0.f;
      }
      dd[j >> 1] = pack_bf16x2(pa * (dp[v] - dlt), pb * (dp[v + 1] - dlt));
    }
    const uintx4_t du = {dd[0], dd[1], dd[2], dd[3]};
    dsf[kstep] = __builtin_bit_cast(bf16x8_t, du);
  }
}

// ---------------------------------------------------------------------------------------
// dQ: query-stationary
// ---------------------------------------------------------------------------------------
struct DqLane {
  unsigned k_nat[8];     // K fragment (row = permuted lane row) for d chunk pair ks, slot 0, half 0
  unsigned v_nat[8];     // same for V
  unsigned k_tr[4][2];   // transposed K read for d tile dt, rows +0 / +4
};

// S^T = K Q^T and dP^T = V dO^T for one 32-key half of a tile
template <int QW, int SOFF>
__device__ __forceinline__ void dq_scores(const DqLane& ln, unsigned off, const bf16x8_t (&qf)[QW][8],
                                          const bf16x8_t (&dof)[QW][8], floatx16_t (&s)[QW],
                                          floatx16_t (&dp)[QW]) {
#pragma unroll
  for (int qw = 0; qw < QW; ++qw)
#pragma unroll
    for (int v = 0; v < 16; ++v) { s[qw][v] = 0.f; dp[qw][v] = 0.f; }
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const bf16x8_t kf = lds_read_b128(ln.k_nat[ks] + off + SOFF);
    const bf16x8_t vf = lds_read_b128(ln.v_nat[ks] + off + SOFF);
#pragma unroll
    for (int qw = 0; qw < QW; ++qw) {
      s[qw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qw][ks], s[qw], 0, 0, 0);
      dp[qw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[qw][ks], dp[qw], 0, 0, 0);
    }
  }
}

// dQ^T += K^T dS^T for one 32-key half
template <int QW, int SOFF>
__device__ __forceinline__ void dq_accumulate(const DqLane& ln, unsigned off, const bf16x8_t (&dsf)[QW][2],
                                              floatx16_t (&dq)[QW][4]) {
#pragma unroll
  for (int kstep = 0; kstep < 2; ++kstep)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      const bf16x8_t a = concat_tr(lds_read_tr16_addr(ln.k_tr[dt][0] + off + SOFF + kstep * 16 * 256),
                                   lds_read_tr16_addr(ln.k_tr[dt][1] + off + SOFF + kstep * 16 * 256));
#pragma unroll
      for (int qw = 0; qw < QW; ++qw)
        dq[qw][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dsf[qw][kstep], dq[qw][dt], 0, 0, 0);
    }
}

// One 64-key tile in four phases, so that the vector work of one half overlaps the matrix
// work of the other: scores(A) | scores(B) + softmax(A) | dQ(A) + softmax(B) | dQ(B).
template <int QW, bool MASK, int SOFF>
__device__ __forceinline__ void dq_tile(const DqLane& ln, unsigned off, const bf16x8_t (&qf)[QW][8],
                                        const bf16x8_t (&dof)[QW][8], const float (&lse2)[QW],
                                        const float (&dlt)[QW], floatx16_t (&dq)[QW][4], float c, int h,
                                        int left) {
  floatx16_t s_a[QW], dp_a[QW], s_b[QW], dp_b[QW];
  bf16x8_t dsf_a[QW][2], dsf_b[QW][2];
  dq_scores<QW, SOFF>(ln, off, qf, dof, s_a, dp_a);
  __builtin_amdgcn_sched_barrier(0);
  dq_scores<QW, SOFF + 8192>(ln, off, qf, dof, s_b, dp_b);
#pragma unroll
  for (int qw = 0; qw < QW; ++qw)
    softmax_bwd_cols<MASK>(s_a[qw], dp_a[qw], lse2[qw], dlt[qw], c, h, left, dsf_a[qw]);
  __builtin_amdgcn_sched_barrier(0);
  dq_accumulate<QW, SOFF>(ln, off, dsf_a, dq);
#pragma unroll
  for (int qw = 0; qw < QW; ++qw)
    softmax_bwd_cols<MASK>(s_b[qw], dp_b[qw], lse2[qw], dlt[qw], c, h, left - 32, dsf_b[qw]);
  __builtin_amdgcn_sched_barrier(0);
  dq_accumulate<QW, SOFF + 8192>(ln, off, dsf_b, dq);
}

// GATHER (both backward kernels): d_oh, qh, kh, vh and the gradient outputs are token-major
// [N, H, 128] and row j of a group is token perm[j]; neg_lse_over_scale / neg_delta stay in
// sorted order [H, N] and carry the gate (see attn_bwd_fused_prepass_kernel), so d_oh is the
// raw upstream gradient of the gated output.
// NB: ring slots of 64 keys (4: two tiles ahead, one block per CU; 2: one tile ahead, 64 KB of LDS, so
// that two 4-wave blocks share a CU -- the variant for small groups).
template <int NW, int QW, bool GATHER = false, int NB = 4>
__global__ __launch_bounds__(NW * 64, NB == 2 ? 2 : 1) void attn_bwd_dq_pipe_kernel(
    const unsigned short* __restrict__ d_oh, const unsigned short* __restrict__ qh,
    const unsigned short* __restrict__ kh, const unsigned short* __restrict__ vh,
    const float* __restrict__ neg_lse_over_scale, const float* __restrict__ neg_delta,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_k,
    const int32_t* __restrict__ tile_start, int M, int64_t Nq, int64_t Nk, int H, float scale,
    int tiles_per_head, unsigned short* __restrict__ d_qh, const int32_t* __restrict__ perm = nullptr) {
  constexpr int BM = NW * 32 * QW;
  constexpr int kDmaPerTile = 2 * (16 / NW);
  constexpr int kAhead = NB - 2;   // tiles in flight beyond the one being waited for
  __shared__ __attribute__((aligned(1024))) unsigned short Ks[NB][64 * kHeadDim];
  __shared__ __attribute__((aligned(1024))) unsigned short Vs[NB][64 * kHeadDim];
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

  if (n <= 0) {   // queries without keys: zero gradient (block-uniform branch)
#pragma unroll
    for (int qw = 0; qw < QW; ++qw) {
      const int qrow = q0 + (wave * QW + qw) * 32 + r;
      if (qrow < ge) {
        const int64_t orow = GATHER ? (int64_t)perm[qrow] * H + head : head_off + qrow;
        uintx4_t* op = (uintx4_t*)(d_qh + orow * kHeadDim + 64 * h);
        const uintx4_t z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 8; ++i) op[i] = z;
      }
    }
    return;
  }

  bf16x8_t qf[QW][8], dof[QW][8];
  float lq[QW], dl[QW];
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    int qrow = q0 + (wave * QW + qw) * 32 + r;
    if (qrow > ge - 1) qrow = ge - 1;
    const int64_t irow = GATHER ? (int64_t)perm[qrow] * H + head : head_off + qrow;
    const unsigned short* qp = qh + irow * kHeadDim + 8 * h;
    const unsigned short* dp = d_oh + irow * kHeadDim + 8 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      qf[qw][ks] = *(const bf16x8_t*)(qp + 16 * ks);
      dof[qw][ks] = *(const bf16x8_t*)(dp + 16 * ks);
    }
    lq[qw] = -neg_lse_over_scale[head_off + qrow] * c;   // lse * log2(e)
    dl[qw] = -neg_delta[head_off + qrow];
  }

  PipeDma dma;
  dma.kbase = uniform_ptr(GATHER ? kh + (int64_t)head * kHeadDim : kh + (head_off_k + gs) * kHeadDim);
  dma.vbase = uniform_ptr(GATHER ? vh + (int64_t)head * kHeadDim : vh + (head_off_k + gs) * kHeadDim);
  dma.lds_k = lds_addr_uniform(&Ks[0][0]) + wave * 1024;
  dma.lds_v = lds_addr_uniform(&Vs[0][0]) + wave * 1024;
  dma.row0 = 4 * wave + (lane >> 4);
  dma.chunk_off = (unsigned)(((lane & 15) ^ lds_swizzle(dma.row0)) * 16);
  dma.last_row = n - 1;
  if (GATHER) {
    dma.rows = (const int32_t*)uniform_ptr(perm + gs);
    dma.tok_stride = (int64_t)H * kHeadDim * 2;
    dma.wave_row = 4 * wave;
    dma.last_index = (int)(Nk - 1) - gs;
    pipe_load_tokens<NW>(dma, 0);
  }
#pragma unroll
  for (int t = 0; t <= kAhead; ++t) pipe_issue<NW, GATHER>(dma, 64 * t, t);

  DqLane ln;
  {
    const int krow_a = swap_bits_2_3(r);
    const int k_sw = lds_swizzle(krow_a);
    const unsigned kb = (unsigned)(uintptr_t)&Ks[0][0];
    const unsigned vb = (unsigned)(uintptr_t)&Vs[0][0];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      ln.k_nat[ks] = kb + krow_a * 256 + (((2 * ks + h) ^ k_sw) << 4);
      ln.v_nat[ks] = vb + krow_a * 256 + (((2 * ks + h) ^ k_sw) << 4);
    }
    const int tr_r = 8 * h + ((lane & 15) >> 2);
    const int tr_c = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
    const int tr_e = 4 * (lane & 1);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      ln.k_tr[dt][0] = kb + tr_e * 2 + tr_r * 256 + (((4 * dt + tr_c) ^ lds_swizzle(tr_r)) << 4);
      ln.k_tr[dt][1] = kb + tr_e * 2 + (tr_r + 4) * 256 + (((4 * dt + tr_c) ^ lds_swizzle(tr_r + 4)) << 4);
    }
  }

  floatx16_t dq[QW][4];
#pragma unroll
  for (int qw = 0; qw < QW; ++qw)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) dq[qw][dt][v] = 0.f;

  // tile T lives in ring slot T % 4; at the top of tile T the block waits for it, and refills the
  // slot of tile T-1 (which every wave has left) with tile T+3
  const int nfull = n >> 6;   // tiles whose 64 keys are all inside the group
  // a wave whose query rows all lie past the end of the group only moves its share of the tiles
  const bool active = q0 + wave * 32 * QW < ge;
  int T = 0;
#define MOGA_DQ_TILE(B)                                                                  \
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * kAhead));                      \
  __syncthreads();                                                                       \
  pipe_issue<NW, GATHER>(dma, 64 * (T + (B) + 1 + kAhead), ((B) + 1 + kAhead) & (NB - 1)); \
  if (active) dq_tile<QW, false, ((B) & (NB - 1)) * kPipeTileBytes>(ln, 0, qf, dof, lq, dl, dq, c, h, 64);
  for (; T + 4 <= nfull; T += 4) {   // four tiles per iteration: every LDS offset is an immediate
    MOGA_DQ_TILE(0)
    MOGA_DQ_TILE(1)
    MOGA_DQ_TILE(2)
    MOGA_DQ_TILE(3)
  }
#undef MOGA_DQ_TILE
  for (; T < nfull; ++T) {
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * kAhead));
    __syncthreads();
    pipe_issue<NW, GATHER>(dma, 64 * (T + 1 + kAhead), (T + 1 + kAhead) & (NB - 1));
    if (active) dq_tile<QW, false, 0>(ln, ((unsigned)T & (unsigned)(NB - 1)) * kPipeTileBytes, qf, dof, lq, dl, dq, c, h, 64);
  }
  if (n & 63) {   // last, partial tile: masked keys contribute zero
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * kAhead));
    __syncthreads();
    if (active) dq_tile<QW, true, 0>(ln, ((unsigned)T & (unsigned)(NB - 1)) * kPipeTileBytes, qf, dof, lq, dl, dq, c, h, n - 64 * T);
  }

  __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // drain the look-ahead loads before the LDS is released
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    const int qrow = q0 + (wave * QW + qw) * 32 + r;
    if (qrow < ge) {
      const int64_t orow = GATHER ? (int64_t)perm[qrow] * H + head : head_off + qrow;
      unsigned short* op = d_qh + orow * kHeadDim + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          uintx2_t pk = {pack_bf16x2(dq[qw][dt][4 * b] * scale, dq[qw][dt][4 * b + 1] * scale),
                         pack_bf16x2(dq[qw][dt][4 * b + 2] * scale, dq[qw][dt][4 * b + 3] * scale)};
          *(uintx2_t*)(op + 32 * dt + 8 * b) = pk;
        }
    }
  }
}

// ---------------------------------------------------------------------------------------
// dK, dV with two waves per SIMD: the four products are split between two waves that own the
// same 32 key rows.  Wave A (waves 0-3) holds K and the dV^T accumulators: it computes S = Q K^T,
// P = exp2(c*S - lse*log2e), hands P to its partner through LDS and accumulates dV^T += dO^T P.
// Wave B (waves 4-7, same SIMD as its partner) holds V and the dK^T accumulators: it computes
// dP = dO V^T - delta, waits for P, forms dS = P * dP and accumulates dK^T += Q^T dS.  Each wave
// needs 64 accumulator registers instead of 128, so two waves fit on a SIMD and fill each other's
// waits.  One block-wide barrier per 64-query tile (tile landed, ring slot free); P is handed over
// inside the pair with a flag in LDS (release store by A, acquire spin by B), so the pairs and the
// two roles drift apart instead of meeting twice per tile.  A never waits for B outside the block
// barrier, so every spin ends.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void lds_write_b128(unsigned addr, bf16x8_t v) {
  *(bf16x8_t __attribute__((address_space(3)))*)(uintptr_t)addr = v;
}

struct AbLane {
  unsigned nat[8];      // rows of Q (A) or dO (B): A operand of the score product, slot 0, half 0
  unsigned tr[4][2];    // transposed reads of dO (A) or Q (B) for d tile dt, rows +0 / +4
  unsigned init_addr;   // -lse/scale (A) or -delta (B) of the lane's first row
  unsigned p_addr;      // this lane's 16 bytes in the pair's P buffer (unit 0, kstep 0)
};

// scores of one 32-query unit: acc starts from the per-row constants, then 8 chained MFMAs
template <int SOFF, int SROW>
__device__ __forceinline__ void ab_scores(const AbLane& ln, unsigned off, unsigned off_row,
                                          const bf16x8_t (&kvf)[8], floatx16_t& acc) {
  bf16x8_t nat[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) nat[ks] = lds_read_b128(ln.nat[ks] + off + SOFF);
#pragma unroll
  for (int kstep = 0; kstep < 2; ++kstep)
#pragma unroll
    for (int half4 = 0; half4 < 2; ++half4) {
      const floatx4_t iv = lds_read_f32x4(ln.init_addr + off_row + SROW + (16 * kstep + 4 * half4) * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[8 * kstep + 4 * half4 + e] = iv[e];
    }
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(nat[ks], kvf[ks], acc, 0, 0, 0);
}

template <int SOFF>
__device__ __forceinline__ void ab_load_tr(const AbLane& ln, unsigned off, bf16x8_t (&tr)[2][4]) {
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int kstep = 0; kstep < 2; ++kstep)
      tr[kstep][dt] = concat_tr(lds_read_tr16_addr(ln.tr[dt][0] + off + SOFF + kstep * 16 * 256),
                                lds_read_tr16_addr(ln.tr[dt][1] + off + SOFF + kstep * 16 * 256));
}

__device__ __forceinline__ void ab_accumulate(const bf16x8_t (&tr)[2][4], const bf16x8_t (&bop)[2],
                                              floatx16_t (&acc)[4]) {
#pragma unroll
  for (int kstep = 0; kstep < 2; ++kstep)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
      acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr[kstep][dt], bop[kstep], acc[dt], 0, 0, 0);
}

// A: P of one 32-query unit from its scores, also written to LDS for the partner.
template <bool MASK>
__device__ __forceinline__ void ab_make_p(const AbLane& ln, const floatx16_t& sc, float c, int h, int left, int u,
                                          bf16x8_t (&pf)[2]) {
#pragma unroll
  for (int kstep = 0; kstep < 2; ++kstep) {
    unsigned int pp[4];
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
      const int v = 8 * kstep + j;
      float pa = fast_exp2(sc[v] * c), pb = fast_exp2(sc[v + 1] * c);
      if (MASK) {
        const int idx = 32 * u + 16 * kstep + 8 * h + j;
        if (idx >= left) pa = 0.f;
        if (idx + 1 >= left) pb = 0.f;
      }
      pp[j >> 1] = pack_bf16x2(pa, pb);
    }
    const uintx4_t pu = {pp[0], pp[1], pp[2], pp[3]};
    pf[kstep] = __builtin_bit_cast(bf16x8_t, pu);
    lds_write_b128(ln.p_addr + u * 2048 + kstep * 1024, pf[kstep]);
  }
}

// B: dS = P * dP of one unit, P read from LDS.
__device__ __forceinline__ void ab_take_p(const AbLane& ln, const floatx16_t& dp, int u, bf16x8_t (&dsf)[2]) {
#pragma unroll
  for (int kstep = 0; kstep < 2; ++kstep) {
    const uintx4_t pu = __builtin_bit_cast(uintx4_t, lds_read_b128(ln.p_addr + u * 2048 + kstep * 1024));
    unsigned int dd[4];
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
      const int v = 8 * kstep + j;
      dd[j >> 1] = pack_bf16x2(bf16_lo_to_f32(pu[j >> 1]) * dp[v], bf16_hi_to_f32(pu[j >> 1]) * dp[v + 1]);
    }
    const uintx4_t du = {dd[0], dd[1], dd[2], dd[3]};
    dsf[kstep] = __builtin_bit_cast(bf16x8_t, du);
  }
}

// One 64-query tile for either role (role is wave-uniform; the common parts are written once so that
// the two roles share one instruction stream, with one short role-specific piece in the middle):
//   A: S(u0), S(u1) | P -> LDS, stamp          | dV(u0), dV(u1)
//   B: dP(u0), dP(u1) | wait for the stamp, dS = P * dP | dK(u0), dK(u1)
// `left`: valid query rows of the tile (MASK only).  The stamp of tile t is t + 1.
// The wait of B is bounded: after `spin_limit` polls it records a give-up in *status and goes on
// with whatever P holds (wrong numbers, but the kernel drains normally and the host can tell).
// Progress does not depend on the bound: A publishes the stamp of tile t before it reaches the
// block barrier of tile t + 1 and never waits for B anywhere else, and the single P buffer of a
// pair is only rewritten after that barrier, which B reaches only after it has consumed P.
template <bool MASK, int SOFF, int SROW>
__device__ __forceinline__ void ab_tile(const AbLane& ln, int role, unsigned off, unsigned off_row,
                                        const bf16x8_t (&kvf)[8], floatx16_t (&acc)[4], float c, int h, int left,
                                        int* flag, int tile_no, int spin_limit, int* status) {
  floatx16_t sc[2];   // S (A) or dP (B) of the two 32-query units
  bf16x8_t bop[2][2]; // B operand of the second product: P (A) or dS (B), per unit and 16-query step
  bf16x8_t tr0[2][4], tr1[2][4];
  ab_scores<SOFF, SROW>(ln, off, off_row, kvf, sc[0]);
  ab_scores<SOFF + 8192, SROW + 128>(ln, off, off_row, kvf, sc[1]);
  ab_load_tr<SOFF>(ln, off, tr0);   // in flight while P is computed (A) or awaited (B)
  __builtin_amdgcn_sched_barrier(0);
  if (role == 0) {
    ab_make_p<MASK>(ln, sc[0], c, h, left, 0, bop[0]);
    ab_make_p<MASK>(ln, sc[1], c, h, left, 1, bop[1]);
    __hip_atomic_store(flag, tile_no, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);   // P of this tile is in LDS
  } else {
    int polls = 0;
    while (__hip_atomic_load(flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < tile_no) {
      if (++polls > spin_limit) {   // wave-uniform
        if ((threadIdx.x & 63) == 0) atomicOr(status, 1);
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    ab_take_p(ln, sc[0], 0, bop[0]);
    ab_take_p(ln, sc[1], 1, bop[1]);
  }
  ab_load_tr<SOFF + 8192>(ln, off, tr1);   // in flight while the first unit is accumulated
  ab_accumulate(tr0, bop[0], acc);
  ab_accumulate(tr1, bop[1], acc);
}

// NPAIR: wave pairs per block (4: 128 keys, partners on one SIMD; 2: 64 keys, for small groups).
// NB: ring slots of 64 queries (4 or 2, as in the dQ kernel).
template <bool GATHER = false, int NPAIR = 4, int NB = 4>
__global__ __launch_bounds__(NPAIR * 128, NB == 2 ? 2 : 1) void attn_bwd_dkdv_ab_kernel(
    const unsigned short* __restrict__ d_oh, const unsigned short* __restrict__ qh,
    const unsigned short* __restrict__ kh, const unsigned short* __restrict__ vh,
    const float* __restrict__ neg_lse_over_scale, const float* __restrict__ neg_delta,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_k,
    const int32_t* __restrict__ tile_start, int M, int64_t Nq, int64_t Nk, int H, float scale,
    int tiles_per_head, unsigned short* __restrict__ d_kh, unsigned short* __restrict__ d_vh,
    int spin_limit, int* __restrict__ status, const int32_t* __restrict__ perm = nullptr) {
  constexpr int NW = 2 * NPAIR;
  constexpr int BK = 32 * NPAIR;                   // pairs of waves x 32 keys
  constexpr int kAhead = NB - 2;
  constexpr int kDmaPerTile = 2 * (16 / NW) + 2;
  __shared__ __attribute__((aligned(1024))) unsigned short Qs[NB][64 * kHeadDim];
  __shared__ __attribute__((aligned(1024))) unsigned short dOs[NB][64 * kHeadDim];
  __shared__ __attribute__((aligned(1024))) unsigned char Ps[NPAIR][4096];   // P of one tile, per pair
  __shared__ __attribute__((aligned(256))) float Ls[NB][64];      // -lse / scale
  __shared__ __attribute__((aligned(256))) float Ds[NB][64];      // -delta
  __shared__ int s_flag[NPAIR];   // per pair: number of tiles whose P has been written
  __shared__ int s_start[MOGA_MAX_GROUPS + 1];
  __shared__ int s_found;

  const int64_t total = (int64_t)H * tiles_per_head;
  const int64_t work = xcd_work_index(blockIdx.x, total);
  if (work >= total) return;
  const int head = (int)(work / tiles_per_head);
  const int tile = (int)(work - (int64_t)head * tiles_per_head);
  if (threadIdx.x < NPAIR) s_flag[threadIdx.x] = 0;   // ordered before its first use by the barriers below
  TileInfo ti;   // tiles run over the key rows of the groups
  if (tile_start) {
    if (!find_tile_presummed(tile_start, cu_k, M, BK, tile, ti)) return;
  } else if (!find_tile(cu_k, M, BK, tile, s_start, &s_found, ti)) {
    return;
  }
  const int ge = ti.row_end, k0 = ti.tile_row;
  const int gs = cu_q[ti.group];
  const int n = cu_q[ti.group + 1] - gs;

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int role = wave / NPAIR, pair = wave % NPAIR;
  int* flag = &s_flag[pair];
  const int r = lane & 31, h = lane >> 5;
  const int64_t head_off = (int64_t)head * Nk;
  const int64_t head_off_q = (int64_t)head * Nq;
  const float c = scale * 1.4426950408889634f;
  const int krow = k0 + pair * 32 + r;
  unsigned short* outp = role == 0 ? d_vh : d_kh;

  if (n <= 0) {   // keys without queries: zero gradient (block-uniform branch)
    if (krow < ge) {
      const int64_t orow = GATHER ? (int64_t)perm[krow] * H + head : head_off + krow;
      uintx4_t* o4 = (uintx4_t*)(outp + orow * kHeadDim + 64 * h);
      const uintx4_t z = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int i = 0; i < 8; ++i) o4[i] = z;
    }
    return;
  }

  // K (A) or V (B) fragments of the pair's 32 key rows: B operand, lane (r, h) holds row r, d = 16*ks + 8*h + 0..7
  const int krow_c = krow < ge ? krow : ge - 1;
  bf16x8_t kvf[8];
  {
    const int64_t irow = GATHER ? (int64_t)perm[krow_c] * H + head : head_off + krow_c;
    const unsigned short* kp = (role == 0 ? kh : vh) + irow * kHeadDim + 8 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kvf[ks] = *(const bf16x8_t*)(kp + 16 * ks);
  }

  PipeDma dma;   // "k" = Q rows, "v" = dO rows of this head's group
  dma.kbase = uniform_ptr(GATHER ? qh + (int64_t)head * kHeadDim : qh + (head_off_q + gs) * kHeadDim);
  dma.vbase = uniform_ptr(GATHER ? d_oh + (int64_t)head * kHeadDim : d_oh + (head_off_q + gs) * kHeadDim);
  dma.lds_k = lds_addr_uniform(&Qs[0][0]) + wave * 1024;
  dma.lds_v = lds_addr_uniform(&dOs[0][0]) + wave * 1024;
  dma.row0 = 4 * wave + (lane >> 4);
  dma.chunk_off = (unsigned)(((lane & 15) ^ lds_swizzle(dma.row0)) * 16);
  dma.last_row = n - 1;
  if (GATHER) {
    dma.rows = (const int32_t*)uniform_ptr(perm + gs);
    dma.tok_stride = (int64_t)H * kHeadDim * 2;
    dma.wave_row = 4 * wave;
    dma.last_index = (int)(Nq - 1) - gs;
    pipe_load_tokens<NW>(dma, 0);
  }
  const void* lbase = uniform_ptr(neg_lse_over_scale + head_off_q + gs);
  const void* dbase = uniform_ptr(neg_delta + head_off_q + gs);
  const unsigned lds_l = lds_addr_uniform(&Ls[0][0]), lds_d = lds_addr_uniform(&Ds[0][0]);
  auto issue_tile = [&](int T) {   // every wave issues the (identical) row-constant loads so that all count alike
    const int slot = T & (NB - 1);
    pipe_issue<NW, GATHER>(dma, 64 * T, slot);
    const unsigned roff = (unsigned)min(64 * T + lane, n - 1) * 4u;
    lds_dma4_soff(lbase, roff, lds_l + slot * 256);
    lds_dma4_soff(dbase, roff, lds_d + slot * 256);
  };
#pragma unroll
  for (int t = 0; t <= kAhead; ++t) issue_tile(t);

  AbLane ln;
  {
    const int row_a = swap_bits_2_3(r);
    const int sw = lds_swizzle(row_a);
    const unsigned nb = role == 0 ? (unsigned)(uintptr_t)&Qs[0][0] : (unsigned)(uintptr_t)&dOs[0][0];
    const unsigned tb = role == 0 ? (unsigned)(uintptr_t)&dOs[0][0] : (unsigned)(uintptr_t)&Qs[0][0];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) ln.nat[ks] = nb + row_a * 256 + (((2 * ks + h) ^ sw) << 4);
    const int tr_r = 8 * h + ((lane & 15) >> 2);
    const int tr_c = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
    const int tr_e = 4 * (lane & 1);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      ln.tr[dt][0] = tb + tr_e * 2 + tr_r * 256 + (((4 * dt + tr_c) ^ lds_swizzle(tr_r)) << 4);
      ln.tr[dt][1] = tb + tr_e * 2 + (tr_r + 4) * 256 + (((4 * dt + tr_c) ^ lds_swizzle(tr_r + 4)) << 4);
    }
    ln.init_addr = (role == 0 ? (unsigned)(uintptr_t)&Ls[0][0] : (unsigned)(uintptr_t)&Ds[0][0]) + 8 * h * 4;
    ln.p_addr = (unsigned)(uintptr_t)&Ps[0][0] + pair * 4096 + lane * 16;
  }

  floatx16_t acc[4];   // dV^T (A) or dK^T (B): 128 x 32
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[dt][v] = 0.f;

  const int nfull = n >> 6;   // tiles whose 64 queries are all inside the group
  // a pair whose 32 key rows lie past the end of the group (both of its waves) only moves its share of the tiles
  const bool active = k0 + pair * 32 < ge;
  int T = 0;
#define MOGA_AB_TILE(B)                                                          \
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * kAhead));              \
  __syncthreads();                                                               \
  issue_tile(T + (B) + 1 + kAhead);                                          \
  if (active)                                                                    \
    ab_tile<false, ((B) & (NB - 1)) * kPipeTileBytes, ((B) & (NB - 1)) * 256>(ln, role, 0, 0, kvf, acc, c, h, 64, flag, \
                                                                              T + (B) + 1, spin_limit, status);
  for (; T + 4 <= nfull; T += 4) {   // four tiles per iteration: every LDS offset is an immediate
    MOGA_AB_TILE(0)
    MOGA_AB_TILE(1)
    MOGA_AB_TILE(2)
    MOGA_AB_TILE(3)
  }
#undef MOGA_AB_TILE
  for (; T < nfull; ++T) {
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * kAhead));
    __syncthreads();
    issue_tile(T + 1 + kAhead);
    if (active)
      ab_tile<false, 0, 0>(ln, role, ((unsigned)T & (unsigned)(NB - 1)) * kPipeTileBytes,
                           ((unsigned)T & (unsigned)(NB - 1)) * 256, kvf, acc, c, h, 64, flag, T + 1, spin_limit, status);
  }
  if (n & 63) {   // last, partial tile: masked queries get P = 0 and contribute nothing
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * kAhead));
    __syncthreads();
    if (active)
      ab_tile<true, 0, 0>(ln, role, ((unsigned)T & (unsigned)(NB - 1)) * kPipeTileBytes,
                          ((unsigned)T & (unsigned)(NB - 1)) * 256, kvf, acc, c, h, n - 64 * T, flag, T + 1, spin_limit, status);
  }

  __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // drain the look-ahead loads before the LDS is released
  if (krow < ge) {
    const float f = role == 0 ? 1.f : scale;
    const int64_t orow = GATHER ? (int64_t)perm[krow] * H + head : head_off + krow;
    unsigned short* op = outp + orow * kHeadDim + 4 * h;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        uintx2_t pk = {pack_bf16x2(acc[dt][4 * b] * f, acc[dt][4 * b + 1] * f),
                       pack_bf16x2(acc[dt][4 * b + 2] * f, acc[dt][4 * b + 3] * f)};
        *(uintx2_t*)(op + 32 * dt + 8 * b) = pk;
      }
  }
}

}  // namespace moga
