// Variable-length attention inside groups (Alg. 1 step 3 of the paper; Eq. 1 per group/head).
//
// bf16 kernel, head_dim 128, 32x32x16 bf16 MFMA:
//   * scores are computed transposed, S^T = K Q^T, so that each lane owns one query column:
//     its softmax statistics are per-lane scalars and a row reduction is 16 registers plus
//     one exchange with the other half of the wave;
//   * the K rows fed to the MFMA are permuted (bits 2,3 of the row swapped) so a lane's
//     accumulator registers hold 8 consecutive keys -- exactly the B operand of the second
//     product O^T = V^T P^T, which therefore needs no data movement for P;
//   * V^T is read from the row-major V tile in LDS with the transposing LDS read.
// fp32 kernel: one thread per query row, plain FMA, for the full-precision configuration.
#include "attn_common.h"

namespace moga {

constexpr int kFwdBN = 64;                   // keys per tile
constexpr int kKStride = kHeadDim + 8;       // bf16 per K row in LDS (+16 B pad: b128 reads)
constexpr int kVStride = kHeadDim + 32;      // bf16 per V row in LDS (+64 B pad: transposed reads)

template <int QW>  // 32-query sub-tiles per wave; the block owns 128*QW query rows
__global__ __launch_bounds__(256) void attn_fwd_bf16_kernel(
    const unsigned short* __restrict__ qh, const unsigned short* __restrict__ kh,
    const unsigned short* __restrict__ vh, const int32_t* __restrict__ cu_seqlens, int M,
    int64_t N, int H, float scale, int tiles_per_head, unsigned short* __restrict__ oh,
    float* __restrict__ lse) {
  constexpr int BM = 128 * QW;
  __shared__ __attribute__((aligned(16))) unsigned short Ks[kFwdBN][kKStride];
  __shared__ __attribute__((aligned(16))) unsigned short Vs[kFwdBN][kVStride];
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
  const float c = scale * 1.4426950408889634f;  // scores are exponentiated in base 2

  // Q fragments stay in registers: B operand, lane (r, h) holds Q[q = r][d = 16*ks + 8*h + 0..7]
  bf16x8_t qf[QW][8];
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    int qrow = q0 + (wave * QW + qw) * 32 + r;
    if (qrow > ge - 1) qrow = ge - 1;
    const unsigned short* qp = qh + (head_off + qrow) * kHeadDim + 8 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[qw][ks] = *(const bf16x8_t*)(qp + 16 * ks);
  }

  float m_run[QW], l_run[QW];
  floatx16_t o_acc[QW][4];
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    m_run[qw] = -INFINITY;
    l_run[qw] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) o_acc[qw][dt][v] = 0.f;
  }

  const int krow_a = swap_bits_2_3(r);
  const int tr_row = (lane & 15) >> 2;                       // row inside a 4-row transposed read
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);  // column inside a 32-wide d tile

  for (int kv0 = gs; kv0 < ge; kv0 += kFwdBN) {
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

    // S^T = K Q^T for two 32-key sub-tiles
    floatx16_t s_acc[QW][2];
#pragma unroll
    for (int qw = 0; qw < QW; ++qw)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int v = 0; v < 16; ++v) s_acc[qw][sub][v] = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8_t a = *(const bf16x8_t*)&Ks[sub * 32 + krow_a][ks * 16 + h * 8];
#pragma unroll
        for (int qw = 0; qw < QW; ++qw)
          s_acc[qw][sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qw][ks], s_acc[qw][sub], 0, 0, 0);
      }
    }
    // register v of sub-tile `sub` is key kv0 + 32*sub + 16*(v/8) + 8*h + v%8
    if (kv0 + kFwdBN > ge) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int kv = kv0 + 32 * sub + 16 * (v >> 3) + 8 * h + (v & 7);
          if (kv >= ge) {
#pragma unroll
            for (int qw = 0; qw < QW; ++qw) s_acc[qw][sub][v] = -INFINITY;
          }
        }
    }

    // online softmax, one query column per lane
    bf16x8_t pf[QW][2][2];
#pragma unroll
    for (int qw = 0; qw < QW; ++qw) {
      float mx = -INFINITY;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s_acc[qw][sub][v]);
      mx = fmaxf(mx, other_half(mx));
      const float m_new = fmaxf(m_run[qw], mx);
      const float alpha = fast_exp2((m_run[qw] - m_new) * c);
      m_run[qw] = m_new;
      const float mc = m_new * c;
      float rs = 0.f;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        unsigned int pk[8];
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
          const float p0 = fast_exp2(fmaf(s_acc[qw][sub][v], c, -mc));
          const float p1 = fast_exp2(fmaf(s_acc[qw][sub][v + 1], c, -mc));
          rs += p0 + p1;
          pk[v >> 1] = pack_bf16x2(p0, p1);
        }
        uintx4_t lo = {pk[0], pk[1], pk[2], pk[3]}, hi = {pk[4], pk[5], pk[6], pk[7]};
        pf[qw][sub][0] = __builtin_bit_cast(bf16x8_t, lo);
        pf[qw][sub][1] = __builtin_bit_cast(bf16x8_t, hi);
      }
      l_run[qw] = l_run[qw] * alpha + rs;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[qw][dt][v] *= alpha;
    }

    // O^T += V^T P^T
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int kstep = 0; kstep < 2; ++kstep) {
        const int kvb = sub * 32 + kstep * 16 + 8 * h + tr_row;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const short4_t a_lo = lds_read_tr16(&Vs[kvb][dt * 32 + tr_col]);
          const short4_t a_hi = lds_read_tr16(&Vs[kvb + 4][dt * 32 + tr_col]);
          const bf16x8_t a = concat_tr(a_lo, a_hi);
#pragma unroll
          for (int qw = 0; qw < QW; ++qw)
            o_acc[qw][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[qw][sub][kstep], o_acc[qw][dt], 0, 0, 0);
        }
      }
    }
  }

  // epilogue: register v of d tile dt is d = 32*dt + 8*(v/4) + 4*h + v%4 of query column r
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    const float lt = l_run[qw] + other_half(l_run[qw]);
    const float inv = 1.f / lt;
    const int qrow = q0 + (wave * QW + qw) * 32 + r;
    if (qrow < ge) {
      unsigned short* op = oh + (head_off + qrow) * kHeadDim + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          uintx2_t pk = {pack_bf16x2(o_acc[qw][dt][4 * b] * inv, o_acc[qw][dt][4 * b + 1] * inv),
                         pack_bf16x2(o_acc[qw][dt][4 * b + 2] * inv, o_acc[qw][dt][4 * b + 3] * inv)};
          *(uintx2_t*)(op + 32 * dt + 8 * b) = pk;
        }
      if (h == 0) lse[head_off + qrow] = m_run[qw] * scale + logf(lt);
    }
  }
}

// ---------------------------------------------------------------------------------------
// fp32: one thread per query row
// ---------------------------------------------------------------------------------------
constexpr int kF32BM = 64, kF32BN = 32;

template <int D>
__global__ __launch_bounds__(64) void attn_fwd_f32_kernel(
    const float* __restrict__ qh, const float* __restrict__ kh, const float* __restrict__ vh,
    const int32_t* __restrict__ cu_seqlens, int M, int64_t N, int H, float scale,
    int tiles_per_head, float* __restrict__ oh, float* __restrict__ lse) {
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
  const float* qp = qh + (head_off + (valid ? row : ge - 1)) * D;
  float q[D], o[D];
#pragma unroll
  for (int cI = 0; cI < D; cI += 4) {
    const floatx4_t t = *(const floatx4_t*)(qp + cI);
    q[cI] = t[0]; q[cI + 1] = t[1]; q[cI + 2] = t[2]; q[cI + 3] = t[3];
  }
#pragma unroll
  for (int cI = 0; cI < D; ++cI) o[cI] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  for (int kv0 = ti.row_begin; kv0 < ge; kv0 += kF32BN) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < kF32BN * (D / 4); idx += 64) {
      const int rr = idx / (D / 4), c4 = (idx - rr * (D / 4)) * 4;
      floatx4_t kk = {0.f, 0.f, 0.f, 0.f}, vv = {0.f, 0.f, 0.f, 0.f};
      if (kv0 + rr < ge) {
        kk = *(const floatx4_t*)(kh + (head_off + kv0 + rr) * D + c4);
        vv = *(const floatx4_t*)(vh + (head_off + kv0 + rr) * D + c4);
      }
      *(floatx4_t*)&Ks[rr][c4] = kk;
      *(floatx4_t*)&Vs[rr][c4] = vv;
    }
    __syncthreads();
    const int nk = min(kF32BN, ge - kv0);
    float s[kF32BN];
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < kF32BN; ++j) {
      float dot = 0.f;
#pragma unroll
      for (int cI = 0; cI < D; cI += 4) {
        const floatx4_t kk = *(const floatx4_t*)&Ks[j][cI];
        dot = fmaf(q[cI], kk[0], dot);
        dot = fmaf(q[cI + 1], kk[1], dot);
        dot = fmaf(q[cI + 2], kk[2], dot);
        dot = fmaf(q[cI + 3], kk[3], dot);
      }
      s[j] = j < nk ? dot * scale : -INFINITY;
      mx = fmaxf(mx, s[j]);
    }
    const float m_new = fmaxf(m_run, mx);
    const float alpha = expf(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int cI = 0; cI < D; ++cI) o[cI] *= alpha;
#pragma unroll
    for (int j = 0; j < kF32BN; ++j) {
      const float p = expf(s[j] - m_new);
      l_run += p;
#pragma unroll
      for (int cI = 0; cI < D; cI += 4) {
        const floatx4_t vv = *(const floatx4_t*)&Vs[j][cI];
        o[cI] = fmaf(p, vv[0], o[cI]);
        o[cI + 1] = fmaf(p, vv[1], o[cI + 1]);
        o[cI + 2] = fmaf(p, vv[2], o[cI + 2]);
        o[cI + 3] = fmaf(p, vv[3], o[cI + 3]);
      }
    }
  }
  if (valid) {
    const float inv = 1.f / l_run;
    float* op = oh + (head_off + row) * D;
#pragma unroll
    for (int cI = 0; cI < D; cI += 4) {
      floatx4_t t = {o[cI] * inv, o[cI + 1] * inv, o[cI + 2] * inv, o[cI + 3] * inv};
      *(floatx4_t*)(op + cI) = t;
    }
    lse[head_off + row] = m_run + logf(l_run);
  }
}

}  // namespace moga

using namespace moga;

extern "C" int moga_group_attn_fwd(const void* qh, const void* kh, const void* vh, int dtype,
                                   int64_t N, int H, int D, const int32_t* cu_seqlens, int M,
                                   float softmax_scale, void* oh, float* lse, void* ws,
                                   size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  if (N < 0 || H < 1 || D < 1 || M < 1) return MOGA_ERR_INVALID_ARG;
  if (!(softmax_scale > 0.f) || !(softmax_scale < INFINITY)) return MOGA_ERR_INVALID_ARG;
  if (dtype != MOGA_F32 && dtype != MOGA_BF16) return MOGA_ERR_UNSUPPORTED;
  if (M > MOGA_MAX_GROUPS || N >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  if (dtype == MOGA_BF16 && D != 128) return MOGA_ERR_UNSUPPORTED;
  if (dtype == MOGA_F32 && D != 64 && D != 128) return MOGA_ERR_UNSUPPORTED;
  if (N == 0) return MOGA_OK;
  if (!qh || !kh || !vh || !cu_seqlens || !oh || !lse) return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(qh) && aligned16(kh) && aligned16(vh) && aligned16(oh))) return MOGA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == MOGA_BF16) {
    // 256-row query tiles once there is enough work to fill the chip with them
    const bool big = N * (int64_t)H >= (int64_t)256 * 256 * 4;
    const int bm = big ? 256 : 128;
    const int64_t tiles = max_tiles(N, M, bm);
    const int64_t total = tiles * H;
    const int64_t blocks = (total + 7) / 8 * 8;
    if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
    if (big)
      attn_fwd_bf16_kernel<2><<<(unsigned)blocks, 256, 0, st>>>(
          (const unsigned short*)qh, (const unsigned short*)kh, (const unsigned short*)vh,
          cu_seqlens, M, N, H, softmax_scale, (int)tiles, (unsigned short*)oh, lse);
    else
      attn_fwd_bf16_kernel<1><<<(unsigned)blocks, 256, 0, st>>>(
          (const unsigned short*)qh, (const unsigned short*)kh, (const unsigned short*)vh,
          cu_seqlens, M, N, H, softmax_scale, (int)tiles, (unsigned short*)oh, lse);
  } else {
    const int64_t tiles = max_tiles(N, M, kF32BM);
    const int64_t blocks = tiles * H;
    if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
    if (D == 64)
      attn_fwd_f32_kernel<64><<<(unsigned)blocks, 64, 0, st>>>(
          (const float*)qh, (const float*)kh, (const float*)vh, cu_seqlens, M, N, H,
          softmax_scale, (int)tiles, (float*)oh, lse);
    else
      attn_fwd_f32_kernel<128><<<(unsigned)blocks, 64, 0, st>>>(
          (const float*)qh, (const float*)kh, (const float*)vh, cu_seqlens, M, N, H,
          softmax_scale, (int)tiles, (float*)oh, lse);
  }
  return launch_status();
}
