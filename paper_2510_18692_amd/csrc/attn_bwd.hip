// Backward of the variable-length group attention (derivative of Eq. 1 inside each group).
//
// With P = exp(scale*S - lse) and delta = rowsum(dO * O):
//   dV = P^T dO,  dP = dO V^T,  dS = P * (dP - delta),  dQ = scale dS K,  dK = scale dS^T Q.
//
// Three kernels, no atomics, results independent of scheduling:
//   attn_bwd_delta   : delta[h][j] = sum_c dO[h][j][c] * O[h][j][c]
//   attn_bwd_dkdv    : a wave owns 32 key rows (K, V fragments and the dK^T, dV^T accumulators
//                      live in registers) and sweeps the query tiles of its group;
//   attn_bwd_dq      : a wave owns 32*QW query rows and sweeps the key tiles (mirror of forward).
// Both MFMA kernels keep the contraction index of the second product in the accumulator
// registers of the first (row permutation of the LDS operand), and read the transposed
// operands (dO^T, Q^T, K^T) from row-major LDS tiles with the transposing LDS read.
#include <stdlib.h>

#include "attn_common.h"
#include "attn_bwd_pipe.h"

namespace moga {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kBwdTile = 64;              // rows of the streamed tile (queries in dkdv, keys in dq)
constexpr int kBwdStride = kHeadDim + 8;  // bf16 per LDS row

// ---------------------------------------------------------------------------------------
template <int LPR, bool BF16>
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(const uintx4_t* __restrict__ d_oh,
                                                             const uintx4_t* __restrict__ oh,
                                                             const float* __restrict__ lse, int64_t rows,
                                                             float* __restrict__ delta,
                                                             float* __restrict__ lse2) {
  const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPR;
  const int part = threadIdx.x % LPR;
  float s = 0.f;
  if (row < rows) {
    const uintx4_t a = d_oh[row * LPR + part], b = oh[row * LPR + part];
    if (BF16) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        s = fmaf(bf16_lo_to_f32(a[i]), bf16_lo_to_f32(b[i]), s);
        s = fmaf(bf16_hi_to_f32(a[i]), bf16_hi_to_f32(b[i]), s);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) s = fmaf(__uint_as_float(a[i]), __uint_as_float(b[i]), s);
    }
  }
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, kWave);
  if (row < rows && part == 0) {
    delta[row] = s;
    if (lse2) lse2[row] = lse[row] * kLog2e;   // the bf16 kernels exponentiate in base 2
  }
}

// ---------------------------------------------------------------------------------------
// dK, dV: key-stationary
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_bwd_dkdv_bf16_kernel(
    const unsigned short* __restrict__ d_oh, const unsigned short* __restrict__ qh,
    const unsigned short* __restrict__ kh, const unsigned short* __restrict__ vh,
    const float* __restrict__ lse, const float* __restrict__ delta,
    const int32_t* __restrict__ cu_seqlens, int M, int64_t N, int H, float scale,
    int tiles_per_head, unsigned short* __restrict__ d_kh, unsigned short* __restrict__ d_vh) {
  constexpr int BK = 128;  // key rows per block: 4 waves x 32
  __shared__ __attribute__((aligned(16))) unsigned short Qs[kBwdTile][kBwdStride];
  __shared__ __attribute__((aligned(16))) unsigned short dOs[kBwdTile][kBwdStride];
  __shared__ __attribute__((aligned(16))) float s_lse[kBwdTile];    // lse * log2(e); +inf on padding rows
  __shared__ __attribute__((aligned(16))) float s_delta[kBwdTile];
  __shared__ int s_start[MOGA_MAX_GROUPS + 1];
  __shared__ int s_found;

  const int64_t total = (int64_t)H * tiles_per_head;
  const int64_t work = xcd_work_index(blockIdx.x, total);
  if (work >= total) return;
  const int head = (int)(work / tiles_per_head);
  const int tile = (int)(work - (int64_t)head * tiles_per_head);
  TileInfo ti;
  if (!find_tile(cu_seqlens, M, BK, tile, s_start, &s_found, ti)) return;
  const int gs = ti.row_begin, ge = ti.row_end, k0 = ti.tile_row;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 31, h = lane >> 5;
  const int64_t head_off = (int64_t)head * N;
  const float c = scale * kLog2e;

  // K, V fragments of this wave's 32 key rows: B operand, lane (r, h) holds row r, d = 16*ks + 8*h + 0..7
  const int krow = k0 + wave * 32 + r;
  const int krow_c = krow < ge ? krow : ge - 1;
  bf16x8_t kf[8], vf[8];
  {
    const unsigned short* kp = kh + (head_off + krow_c) * kHeadDim + 8 * h;
    const unsigned short* vp = vh + (head_off + krow_c) * kHeadDim + 8 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      kf[ks] = *(const bf16x8_t*)(kp + 16 * ks);
      vf[ks] = *(const bf16x8_t*)(vp + 16 * ks);
    }
  }
  floatx16_t dk_acc[4], dv_acc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk_acc[dt][v] = 0.f; dv_acc[dt][v] = 0.f; }

  const int qrow_a = swap_bits_2_3(r);
  const int tr_row = (lane & 15) >> 2;
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

  for (int q0 = gs; q0 < ge; q0 += kBwdTile) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = threadIdx.x + 256 * i;
      const int row = idx >> 4, ch = idx & 15;
      const int grow = q0 + row;
      uintx4_t qq = {0u, 0u, 0u, 0u}, dd = {0u, 0u, 0u, 0u};
      if (grow < ge) {
        qq = *(const uintx4_t*)(qh + (head_off + grow) * kHeadDim + ch * 8);
        dd = *(const uintx4_t*)(d_oh + (head_off + grow) * kHeadDim + ch * 8);
      }
      *(uintx4_t*)&Qs[row][ch * 8] = qq;
      *(uintx4_t*)&dOs[row][ch * 8] = dd;
    }
    if (threadIdx.x < kBwdTile) {
      const int grow = q0 + threadIdx.x;
      s_lse[threadIdx.x] = grow < ge ? lse[head_off + grow] * kLog2e : INFINITY;
      s_delta[threadIdx.x] = grow < ge ? delta[head_off + grow] : 0.f;
    }
    __syncthreads();

#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      // S = Q K^T and dP = dO V^T: rows are queries (permuted), column r is this lane's key
      floatx16_t s_acc, dp_acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) { s_acc[v] = 0.f; dp_acc[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8_t aq = *(const bf16x8_t*)&Qs[sub * 32 + qrow_a][ks * 16 + h * 8];
        const bf16x8_t ad = *(const bf16x8_t*)&dOs[sub * 32 + qrow_a][ks * 16 + h * 8];
        s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq, kf[ks], s_acc, 0, 0, 0);
        dp_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ad, vf[ks], dp_acc, 0, 0, 0);
      }
      // register v is query 32*sub + 16*(v/8) + 8*h + v%8 of the tile
      bf16x8_t pf[2], dsf[2];
#pragma unroll
      for (int kstep = 0; kstep < 2; ++kstep) {
        const int qb = 32 * sub + 16 * kstep + 8 * h;
        const floatx4_t l0 = *(const floatx4_t*)&s_lse[qb], l1 = *(const floatx4_t*)&s_lse[qb + 4];
        const floatx4_t d0 = *(const floatx4_t*)&s_delta[qb], d1 = *(const floatx4_t*)&s_delta[qb + 4];
        unsigned int pp[4], dd[4];
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
          const float la = j < 4 ? l0[j] : l1[j - 4], lb = j + 1 < 4 ? l0[j + 1] : l1[j - 3];
          const float da = j < 4 ? d0[j] : d1[j - 4], db = j + 1 < 4 ? d0[j + 1] : d1[j - 3];
          const float pa = fast_exp2(fmaf(s_acc[8 * kstep + j], c, -la));
          const float pb = fast_exp2(fmaf(s_acc[8 * kstep + j + 1], c, -lb));
          const float dsa = pa * (dp_acc[8 * kstep + j] - da);
          const float dsb = pb * (dp_acc[8 * kstep + j + 1] - db);
          pp[j >> 1] = pack_bf16x2(pa, pb);
          dd[j >> 1] = pack_bf16x2(dsa, dsb);
        }
        uintx4_t pu = {pp[0], pp[1], pp[2], pp[3]}, du = {dd[0], dd[1], dd[2], dd[3]};
        pf[kstep] = __builtin_bit_cast(bf16x8_t, pu);
        dsf[kstep] = __builtin_bit_cast(bf16x8_t, du);
      }
      // dV^T += dO^T P,  dK^T += Q^T dS   (d x key; A operand read transposed from LDS)
#pragma unroll
      for (int kstep = 0; kstep < 2; ++kstep) {
        const int qb = sub * 32 + kstep * 16 + 8 * h + tr_row;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const bf16x8_t a_do = concat_tr(lds_read_tr16(&dOs[qb][dt * 32 + tr_col]),
                                          lds_read_tr16(&dOs[qb + 4][dt * 32 + tr_col]));
          const bf16x8_t a_q = concat_tr(lds_read_tr16(&Qs[qb][dt * 32 + tr_col]),
                                         lds_read_tr16(&Qs[qb + 4][dt * 32 + tr_col]));
          dv_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_do, pf[kstep], dv_acc[dt], 0, 0, 0);
          dk_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_q, dsf[kstep], dk_acc[dt], 0, 0, 0);
        }
      }
    }
  }

  if (krow < ge) {
    unsigned short* dkp = d_kh + (head_off + krow) * kHeadDim + 4 * h;
    unsigned short* dvp = d_vh + (head_off + krow) * kHeadDim + 4 * h;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        uintx2_t pk = {pack_bf16x2(dk_acc[dt][4 * b] * scale, dk_acc[dt][4 * b + 1] * scale),
                       pack_bf16x2(dk_acc[dt][4 * b + 2] * scale, dk_acc[dt][4 * b + 3] * scale)};
        uintx2_t pv = {pack_bf16x2(dv_acc[dt][4 * b], dv_acc[dt][4 * b + 1]),
                       pack_bf16x2(dv_acc[dt][4 * b + 2], dv_acc[dt][4 * b + 3])};
        *(uintx2_t*)(dkp + 32 * dt + 8 * b) = pk;
        *(uintx2_t*)(dvp + 32 * dt + 8 * b) = pv;
      }
  }
}

// ---------------------------------------------------------------------------------------
// dQ: query-stationary
// ---------------------------------------------------------------------------------------
template <int QW>
__global__ __launch_bounds__(256) void attn_bwd_dq_bf16_kernel(
    const unsigned short* __restrict__ d_oh, const unsigned short* __restrict__ qh,
    const unsigned short* __restrict__ kh, const unsigned short* __restrict__ vh,
    const float* __restrict__ lse, const float* __restrict__ delta,
    const int32_t* __restrict__ cu_seqlens, int M, int64_t N, int H, float scale,
    int tiles_per_head, unsigned short* __restrict__ d_qh) {
  constexpr int BM = 128 * QW;
  __shared__ __attribute__((aligned(16))) unsigned short Ks[kBwdTile][kBwdStride];
  __shared__ __attribute__((aligned(16))) unsigned short Vs[kBwdTile][kBwdStride];
  __shared__ int s_start[MOGA_MAX_GROUPS + 1];
  __shared__ int s_found;

  const int64_t total = (int64_t)H * tiles_per_head;
  const int64_t work = xcd_work_index(blockIdx.x, total);
  if (work >= total) return;
  const int head = (int)(work / tiles_per_head);
  const int tile = (int)(work - (int64_t)head * tiles_per_head);
  TileInfo ti;
  if (!find_tile(cu_seqlens, M, BM, tile, s_start, &s_found, ti)) return;
  const int gs = ti.row_begin, ge = ti.row_end, q0 = ti.tile_row;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 31, h = lane >> 5;
  const int64_t head_off = (int64_t)head * N;
  const float c = scale * kLog2e;

  bf16x8_t qf[QW][8], dof[QW][8];
  float lse2[QW], dlt[QW];
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    int qrow = q0 + (wave * QW + qw) * 32 + r;
    if (qrow > ge - 1) qrow = ge - 1;
    const unsigned short* qp = qh + (head_off + qrow) * kHeadDim + 8 * h;
    const unsigned short* dp = d_oh + (head_off + qrow) * kHeadDim + 8 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      qf[qw][ks] = *(const bf16x8_t*)(qp + 16 * ks);
      dof[qw][ks] = *(const bf16x8_t*)(dp + 16 * ks);
    }
    lse2[qw] = lse[head_off + qrow] * kLog2e;
    dlt[qw] = delta[head_off + qrow];
  }
  floatx16_t dq_acc[QW][4];
#pragma unroll
  for (int qw = 0; qw < QW; ++qw)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) dq_acc[qw][dt][v] = 0.f;

  const int krow_a = swap_bits_2_3(r);
  const int tr_row = (lane & 15) >> 2;
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

  for (int kv0 = gs; kv0 < ge; kv0 += kBwdTile) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = threadIdx.x + 256 * i;
      const int row = idx >> 4, ch = idx & 15;
      const int grow = kv0 + row;
      uintx4_t kk = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
      if (grow < ge) {
        kk = *(const uintx4_t*)(kh + (head_off + grow) * kHeadDim + ch * 8);
        vv = *(const uintx4_t*)(vh + (head_off + grow) * kHeadDim + ch * 8);
      }
      *(uintx4_t*)&Ks[row][ch * 8] = kk;
      *(uintx4_t*)&Vs[row][ch * 8] = vv;
    }
    __syncthreads();

#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      floatx16_t s_acc[QW], dp_acc[QW];
#pragma unroll
      for (int qw = 0; qw < QW; ++qw)
#pragma unroll
        for (int v = 0; v < 16; ++v) { s_acc[qw][v] = 0.f; dp_acc[qw][v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8_t ak = *(const bf16x8_t*)&Ks[sub * 32 + krow_a][ks * 16 + h * 8];
        const bf16x8_t av = *(const bf16x8_t*)&Vs[sub * 32 + krow_a][ks * 16 + h * 8];
#pragma unroll
        for (int qw = 0; qw < QW; ++qw) {
          s_acc[qw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, qf[qw][ks], s_acc[qw], 0, 0, 0);
          dp_acc[qw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, dof[qw][ks], dp_acc[qw], 0, 0, 0);
        }
      }
      // register v is key kv0 + 32*sub + 16*(v/8) + 8*h + v%8; keys past the group end get P = 0
      bf16x8_t dsf[QW][2];
#pragma unroll
      for (int qw = 0; qw < QW; ++qw) {
#pragma unroll
        for (int kstep = 0; kstep < 2; ++kstep) {
          unsigned int dd[4];
#pragma unroll
          for (int j = 0; j < 8; j += 2) {
            const int kv = kv0 + 32 * sub + 16 * kstep + 8 * h + j;
            float pa = fast_exp2(fmaf(s_acc[qw][8 * kstep + j], c, -lse2[qw]));
            float pb = fast_exp2(fmaf(s_acc[qw][8 * kstep + j + 1], c, -lse2[qw]));
            if (kv >= ge) pa = 0.f;
            if (kv + 1 >= ge) pb = 0.f;
            dd[j >> 1] = pack_bf16x2(pa * (dp_acc[qw][8 * kstep + j] - dlt[qw]),
                                     pb * (dp_acc[qw][8 * kstep + j + 1] - dlt[qw]));
          }
          uintx4_t du = {dd[0], dd[1], dd[2], dd[3]};
          dsf[qw][kstep] = __builtin_bit_cast(bf16x8_t, du);
        }
      }
      // dQ^T += K^T dS^T
#pragma unroll
      for (int kstep = 0; kstep < 2; ++kstep) {
        const int kvb = sub * 32 + kstep * 16 + 8 * h + tr_row;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const bf16x8_t a = concat_tr(lds_read_tr16(&Ks[kvb][dt * 32 + tr_col]),
                                       lds_read_tr16(&Ks[kvb + 4][dt * 32 + tr_col]));
#pragma unroll
          for (int qw = 0; qw < QW; ++qw)
            dq_acc[qw][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dsf[qw][kstep], dq_acc[qw][dt], 0, 0, 0);
        }
      }
    }
  }

#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    const int qrow = q0 + (wave * QW + qw) * 32 + r;
    if (qrow < ge) {
      unsigned short* op = d_qh + (head_off + qrow) * kHeadDim + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          uintx2_t pk = {pack_bf16x2(dq_acc[qw][dt][4 * b] * scale, dq_acc[qw][dt][4 * b + 1] * scale),
                         pack_bf16x2(dq_acc[qw][dt][4 * b + 2] * scale, dq_acc[qw][dt][4 * b + 3] * scale)};
          *(uintx2_t*)(op + 32 * dt + 8 * b) = pk;
        }
    }
  }
}

// ---------------------------------------------------------------------------------------
// fp32 (head_dim 64): one thread per row
// ---------------------------------------------------------------------------------------
constexpr int kF32BM = 64, kF32BN = 32;

template <int D>
__global__ __launch_bounds__(64) void attn_bwd_dq_f32_kernel(
    const float* __restrict__ d_oh, const float* __restrict__ qh, const float* __restrict__ kh,
    const float* __restrict__ vh, const float* __restrict__ lse, const float* __restrict__ delta,
    const int32_t* __restrict__ cu_seqlens, int M, int64_t N, int H, float scale, int tiles_per_head,
    float* __restrict__ d_qh) {
  __shared__ __attribute__((aligned(16))) float Ks[kF32BN][D];
  __shared__ __attribute__((aligned(16))) float Vs[kF32BN][D];
  __shared__ int s_start[MOGA_MAX_GROUPS + 1];
  __shared__ int s_found;
  const int head = blockIdx.x / tiles_per_head;
  const int tile = blockIdx.x - head * tiles_per_head;
  TileInfo ti;
  if (!find_tile(cu_seqlens, M, kF32BM, tile, s_start, &s_found, ti)) return;
  const int ge = ti.row_end;
  const int64_t head_off = (int64_t)head * N;
  const int row = ti.tile_row + threadIdx.x;
  const bool valid = row < ge;
  const int64_t rr = head_off + (valid ? row : ge - 1);
  float q[D], dO[D], dq[D];
#pragma unroll
  for (int cI = 0; cI < D; ++cI) { q[cI] = qh[rr * D + cI]; dO[cI] = d_oh[rr * D + cI]; dq[cI] = 0.f; }
  const float l = lse[rr], dl = delta[rr];

  for (int kv0 = ti.row_begin; kv0 < ge; kv0 += kF32BN) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < kF32BN * (D / 4); idx += 64) {
      const int r2 = idx / (D / 4), c4 = (idx - r2 * (D / 4)) * 4;
      floatx4_t kk = {0.f, 0.f, 0.f, 0.f}, vv = {0.f, 0.f, 0.f, 0.f};
      if (kv0 + r2 < ge) {
        kk = *(const floatx4_t*)(kh + (head_off + kv0 + r2) * D + c4);
        vv = *(const floatx4_t*)(vh + (head_off + kv0 + r2) * D + c4);
      }
      *(floatx4_t*)&Ks[r2][c4] = kk;
      *(floatx4_t*)&Vs[r2][c4] = vv;
    }
    __syncthreads();
    const int nk = min(kF32BN, ge - kv0);
    for (int j = 0; j < nk; ++j) {
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int cI = 0; cI < D; ++cI) { s = fmaf(q[cI], Ks[j][cI], s); dp = fmaf(dO[cI], Vs[j][cI], dp); }
      const float p = expf(s * scale - l);
      const float ds = p * (dp - dl);
#pragma unroll
      for (int cI = 0; cI < D; ++cI) dq[cI] = fmaf(ds, Ks[j][cI], dq[cI]);
    }
  }
  if (valid) {
#pragma unroll
    for (int cI = 0; cI < D; ++cI) d_qh[rr * D + cI] = dq[cI] * scale;
  }
}

template <int D>
__global__ __launch_bounds__(64) void attn_bwd_dkdv_f32_kernel(
    const float* __restrict__ d_oh, const float* __restrict__ qh, const float* __restrict__ kh,
    const float* __restrict__ vh, const float* __restrict__ lse, const float* __restrict__ delta,
    const int32_t* __restrict__ cu_seqlens, int M, int64_t N, int H, float scale, int tiles_per_head,
    float* __restrict__ d_kh, float* __restrict__ d_vh) {
  __shared__ __attribute__((aligned(16))) float Qs[kF32BN][D];
  __shared__ __attribute__((aligned(16))) float dOs[kF32BN][D];
  __shared__ float s_lse[kF32BN], s_delta[kF32BN];
  __shared__ int s_start[MOGA_MAX_GROUPS + 1];
  __shared__ int s_found;
  const int head = blockIdx.x / tiles_per_head;
  const int tile = blockIdx.x - head * tiles_per_head;
  TileInfo ti;
  if (!find_tile(cu_seqlens, M, kF32BM, tile, s_start, &s_found, ti)) return;
  const int ge = ti.row_end;
  const int64_t head_off = (int64_t)head * N;
  const int row = ti.tile_row + threadIdx.x;
  const bool valid = row < ge;
  const int64_t rr = head_off + (valid ? row : ge - 1);
  float k[D], v[D], dk[D], dv[D];
#pragma unroll
  for (int cI = 0; cI < D; ++cI) { k[cI] = kh[rr * D + cI]; v[cI] = vh[rr * D + cI]; dk[cI] = 0.f; dv[cI] = 0.f; }

  for (int q0 = ti.row_begin; q0 < ge; q0 += kF32BN) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < kF32BN * (D / 4); idx += 64) {
      const int r2 = idx / (D / 4), c4 = (idx - r2 * (D / 4)) * 4;
      floatx4_t qq = {0.f, 0.f, 0.f, 0.f}, dd = {0.f, 0.f, 0.f, 0.f};
      if (q0 + r2 < ge) {
        qq = *(const floatx4_t*)(qh + (head_off + q0 + r2) * D + c4);
        dd = *(const floatx4_t*)(d_oh + (head_off + q0 + r2) * D + c4);
      }
      *(floatx4_t*)&Qs[r2][c4] = qq;
      *(floatx4_t*)&dOs[r2][c4] = dd;
    }
    if (threadIdx.x < kF32BN) {
      const int g = q0 + threadIdx.x;
      s_lse[threadIdx.x] = g < ge ? lse[head_off + g] : INFINITY;
      s_delta[threadIdx.x] = g < ge ? delta[head_off + g] : 0.f;
    }
    __syncthreads();
    const int nq = min(kF32BN, ge - q0);
    for (int i = 0; i < nq; ++i) {
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int cI = 0; cI < D; ++cI) { s = fmaf(k[cI], Qs[i][cI], s); dp = fmaf(v[cI], dOs[i][cI], dp); }
      const float p = expf(s * scale - s_lse[i]);
      const float ds = p * (dp - s_delta[i]);
#pragma unroll
      for (int cI = 0; cI < D; ++cI) { dv[cI] = fmaf(p, dOs[i][cI], dv[cI]); dk[cI] = fmaf(ds, Qs[i][cI], dk[cI]); }
    }
  }
  if (valid) {
#pragma unroll
    for (int cI = 0; cI < D; ++cI) { d_kh[rr * D + cI] = dk[cI] * scale; d_vh[rr * D + cI] = dv[cI]; }
  }
}

}  // namespace moga

using namespace moga;

extern "C" size_t moga_attn_bwd_ws_bytes(int64_t N, int H, int D, int dtype) {
  (void)D; (void)dtype;
  if (N <= 0 || H < 1) return 0;
  return 2 * (size_t)N * (size_t)H * sizeof(float);   // delta, lse * log2(e)
}

extern "C" int moga_group_attn_bwd(const void* d_oh, const void* qh, const void* kh, const void* vh,
                                   const void* oh, const float* lse, int dtype, int64_t N, int H,
                                   int D, const int32_t* cu_seqlens, int M, float softmax_scale,
                                   void* d_qh, void* d_kh, void* d_vh, void* ws, size_t ws_bytes,
                                   void* stream) {
  if (N < 0 || H < 1 || D < 1 || M < 1) return MOGA_ERR_INVALID_ARG;
  if (!(softmax_scale > 0.f) || !(softmax_scale < INFINITY)) return MOGA_ERR_INVALID_ARG;
  if (dtype != MOGA_F32 && dtype != MOGA_BF16) return MOGA_ERR_UNSUPPORTED;
  if (M > MOGA_MAX_GROUPS || N >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  if (dtype == MOGA_BF16 && D != 128) return MOGA_ERR_UNSUPPORTED;
  if (dtype == MOGA_F32 && D != 64) return MOGA_ERR_UNSUPPORTED;
  if (N == 0) return MOGA_OK;
  if (!d_oh || !qh || !kh || !vh || !oh || !lse || !cu_seqlens || !d_qh || !d_kh || !d_vh)
    return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(d_oh) && aligned16(qh) && aligned16(kh) && aligned16(vh) && aligned16(oh) &&
        aligned16(d_qh) && aligned16(d_kh) && aligned16(d_vh)))
    return MOGA_ERR_INVALID_ARG;
  const size_t need = moga_attn_bwd_ws_bytes(N, H, D, dtype);
  if (!ws || ws_bytes < need) return MOGA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  float* delta = (float*)ws;
  const int64_t rows = N * (int64_t)H;
  if (dtype == MOGA_BF16) {
    float* lse2 = delta + rows;
    attn_bwd_delta_kernel<16, true><<<(unsigned)((rows * 16 + 255) / 256), 256, 0, st>>>(
        (const uintx4_t*)d_oh, (const uintx4_t*)oh, lse, rows, delta, lse2);
    const char* ev = getenv("MOGA_BWD_VARIANT");
    const int variant = ev ? atoi(ev) : 0;
    {
      const int64_t tiles = max_tiles(N, M, 128);
      const int64_t blocks = (tiles * H + 7) / 8 * 8;
      if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
      if (variant == 1)
        attn_bwd_dkdv_bf16_kernel<<<(unsigned)blocks, 256, 0, st>>>(
            (const unsigned short*)d_oh, (const unsigned short*)qh, (const unsigned short*)kh,
            (const unsigned short*)vh, lse, delta, cu_seqlens, M, N, H, softmax_scale, (int)tiles,
            (unsigned short*)d_kh, (unsigned short*)d_vh);
      else
        attn_bwd_dkdv_pipe_kernel<4><<<(unsigned)blocks, 256, 0, st>>>(
            (const unsigned short*)d_oh, (const unsigned short*)qh, (const unsigned short*)kh,
            (const unsigned short*)vh, lse2, delta, cu_seqlens, M, N, H, softmax_scale, (int)tiles,
            (unsigned short*)d_kh, (unsigned short*)d_vh);
    }
    {
      const int64_t tiles = max_tiles(N, M, 256);
      const int64_t blocks = (tiles * H + 7) / 8 * 8;
      if (variant == 1)
        attn_bwd_dq_bf16_kernel<2><<<(unsigned)blocks, 256, 0, st>>>(
            (const unsigned short*)d_oh, (const unsigned short*)qh, (const unsigned short*)kh,
            (const unsigned short*)vh, lse, delta, cu_seqlens, M, N, H, softmax_scale, (int)tiles,
            (unsigned short*)d_qh);
      else
        attn_bwd_dq_pipe_kernel<8, 1><<<(unsigned)blocks, 512, 0, st>>>(
            (const unsigned short*)d_oh, (const unsigned short*)qh, (const unsigned short*)kh,
            (const unsigned short*)vh, lse2, delta, cu_seqlens, M, N, H, softmax_scale, (int)tiles,
            (unsigned short*)d_qh);
    }
  } else {
    attn_bwd_delta_kernel<16, false><<<(unsigned)((rows * 16 + 255) / 256), 256, 0, st>>>(
        (const uintx4_t*)d_oh, (const uintx4_t*)oh, lse, rows, delta, nullptr);
    const int64_t tiles = max_tiles(N, M, kF32BM);
    const int64_t blocks = tiles * H;
    if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
    attn_bwd_dkdv_f32_kernel<64><<<(unsigned)blocks, 64, 0, st>>>(
        (const float*)d_oh, (const float*)qh, (const float*)kh, (const float*)vh, lse, delta,
        cu_seqlens, M, N, H, softmax_scale, (int)tiles, (float*)d_kh, (float*)d_vh);
    attn_bwd_dq_f32_kernel<64><<<(unsigned)blocks, 64, 0, st>>>(
        (const float*)d_oh, (const float*)qh, (const float*)kh, (const float*)vh, lse, delta,
        cu_seqlens, M, N, H, softmax_scale, (int)tiles, (float*)d_qh);
  }
  return launch_status();
}
