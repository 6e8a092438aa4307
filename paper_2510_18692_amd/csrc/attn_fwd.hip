// Variable-length attention inside groups (Alg. 1 step 3 of the paper; Eq. 1 per group/head).
//
// bf16 kernel, head_dim 128, 32x32x16 bf16 MFMA:
//   * scores are computed transposed, S^T = K Q^T, so that each lane owns one query column:
//     its softmax statistics are per-lane scalars and a row reduction is 16 registers plus
//     one exchange with the other half of the wave;
//   * the K rows fed to the MFMA are permuted (bits 2,3 of the row swapped) so a lane's
//     accumulator registers hold 8 consecutive keys -- exactly the B operand of the second
//     product O^T = V^T P^T, which therefore needs no data movement for P;
//   * V^T is read from the row-major V tile in LDS with the transposing LDS read;
//   * the kernel itself (software pipeline, LDS ring, direct-to-LDS loads) is in attn_pipe.h.
// fp32 kernel: one thread per query row, plain FMA, for the full-precision configuration.
#include "attn_common.h"
#include "attn_pipe.h"

namespace moga {

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
    const int64_t tiles = max_tiles(N, M, 256);
    const int64_t blocks = (tiles * H + 7) / 8 * 8;
    if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
    attn_fwd_bf16_pipe_kernel<8, 1><<<(unsigned)blocks, 512, 0, st>>>(
        (const unsigned short*)qh, (const unsigned short*)kh, (const unsigned short*)vh, cu_seqlens, M,
        N, H, softmax_scale, (int)tiles, (unsigned short*)oh, lse);
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
