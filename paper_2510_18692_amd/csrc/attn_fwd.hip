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
#include "attn_pipe_small.h"

namespace moga {

// ---------------------------------------------------------------------------------------
// fp32: one thread per query row
// ---------------------------------------------------------------------------------------
constexpr int kF32BM = 64, kF32BN = 32;
constexpr int64_t kSmallGroupRows = 2560;   // mean rows per group below which the small-group bf16 kernel runs
                                            // (927 against 886 TFLOP/s at 1,560 rows, 1052 against 1063 at 3,224)

template <int D>
__global__ __launch_bounds__(64) void attn_fwd_f32_kernel(
    const float* __restrict__ qh, const float* __restrict__ kh, const float* __restrict__ vh,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_k,
    const int32_t* __restrict__ tile_start, int M, int64_t Nq, int64_t Nk, int H, float scale,
    int tiles_per_head, float* __restrict__ oh, float* __restrict__ lse) {
  __shared__ __attribute__((aligned(16))) float Ks[kF32BN][D];
  __shared__ __attribute__((aligned(16))) float Vs[kF32BN][D];
  __shared__ int s_start[MOGA_MAX_GROUPS + 1];
  __shared__ int s_found;
  const int head = blockIdx.x / tiles_per_head;
  const int tile = blockIdx.x - head * tiles_per_head;
  TileInfo ti;
  if (tile_start) {
    if (!find_tile_presummed(tile_start, cu_q, M, kF32BM, tile, ti)) return;
  } else if (!find_tile(cu_q, M, kF32BM, tile, s_start, &s_found, ti)) {
    return;
  }
  const int ge = ti.row_end;
  const int kbeg = cu_k[ti.group], kend = cu_k[ti.group + 1];   // key rows of the group
  const int64_t head_off = (int64_t)head * Nq;
  const int64_t head_off_k = (int64_t)head * Nk;
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

  for (int kv0 = kbeg; kv0 < kend; kv0 += kF32BN) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < kF32BN * (D / 4); idx += 64) {
      const int rr = idx / (D / 4), c4 = (idx - rr * (D / 4)) * 4;
      floatx4_t kk = {0.f, 0.f, 0.f, 0.f}, vv = {0.f, 0.f, 0.f, 0.f};
      if (kv0 + rr < kend) {
        kk = *(const floatx4_t*)(kh + (head_off_k + kv0 + rr) * D + c4);
        vv = *(const floatx4_t*)(vh + (head_off_k + kv0 + rr) * D + c4);
      }
      *(floatx4_t*)&Ks[rr][c4] = kk;
      *(floatx4_t*)&Vs[rr][c4] = vv;
    }
    __syncthreads();
    const int nk = min(kF32BN, kend - kv0);
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
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;   // no keys: zero output, lse = -inf
    float* op = oh + (head_off + row) * D;
#pragma unroll
    for (int cI = 0; cI < D; cI += 4) {
      floatx4_t t = {o[cI] * inv, o[cI + 1] * inv, o[cI + 2] * inv, o[cI + 3] * inv};
      *(floatx4_t*)(op + cI) = t;
    }
    lse[head_off + row] = l_run > 0.f ? m_run + logf(l_run) : -INFINITY;
  }
}

}  // namespace moga

using namespace moga;

// Shared launcher.  tile_start == NULL: tile lookup inside the kernels (M <= MOGA_MAX_GROUPS).
static int launch_attn_fwd(const void* qh, const void* kh, const void* vh, int dtype, int64_t Nq,
                           int64_t Nk, int H, int D, const int32_t* cu_q, const int32_t* cu_k,
                           int32_t* tile_start, int M, float softmax_scale, void* oh, float* lse,
                           hipStream_t st) {
  // bf16: groups of a few thousand rows or less (the static groups of Section 3.2) take the kernel
  // with 128-row tiles and two 4-wave blocks per CU; the host only knows the mean group size
  const bool small = dtype == MOGA_BF16 && use_small_group_kernels(Nq, M, kSmallGroupRows);
  const int bm = dtype == MOGA_BF16 ? (small ? 128 : 256) : kF32BM;
  const int64_t tiles = max_tiles(Nq, M, bm);
  const int64_t blocks = dtype == MOGA_BF16 ? (tiles * H + 7) / 8 * 8 : tiles * H;
  if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  if (tile_start) tile_start_kernel<<<1, 1024, 0, st>>>(cu_q, M, bm, tile_start);
  if (small) {
    attn_fwd_bf16_small_kernel<<<(unsigned)blocks, 256, 0, st>>>(
        (const unsigned short*)qh, (const unsigned short*)kh, (const unsigned short*)vh, cu_q, cu_k,
        tile_start, M, Nq, Nk, H, softmax_scale, (int)tiles, (unsigned short*)oh, lse);
  } else if (dtype == MOGA_BF16) {
    attn_fwd_bf16_pipe_kernel<8, 1><<<(unsigned)blocks, 512, 0, st>>>(
        (const unsigned short*)qh, (const unsigned short*)kh, (const unsigned short*)vh, cu_q, cu_k,
        tile_start, M, Nq, Nk, H, softmax_scale, (int)tiles, (unsigned short*)oh, lse);
  } else if (D == 64) {
    attn_fwd_f32_kernel<64><<<(unsigned)blocks, 64, 0, st>>>(
        (const float*)qh, (const float*)kh, (const float*)vh, cu_q, cu_k, tile_start, M, Nq, Nk, H,
        softmax_scale, (int)tiles, (float*)oh, lse);
  } else {
    attn_fwd_f32_kernel<128><<<(unsigned)blocks, 64, 0, st>>>(
        (const float*)qh, (const float*)kh, (const float*)vh, cu_q, cu_k, tile_start, M, Nq, Nk, H,
        softmax_scale, (int)tiles, (float*)oh, lse);
  }
  return launch_status();
}

static int check_attn_args(int64_t Nq, int64_t Nk, int H, int D, int M, float softmax_scale, int dtype) {
  if (Nq < 0 || Nk < 0 || H < 1 || D < 1 || M < 1) return MOGA_ERR_INVALID_ARG;
  if (!(softmax_scale > 0.f) || !(softmax_scale < INFINITY)) return MOGA_ERR_INVALID_ARG;
  if (dtype != MOGA_F32 && dtype != MOGA_BF16) return MOGA_ERR_UNSUPPORTED;
  if (Nq >= ((int64_t)1 << 31) || Nk >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  if (dtype == MOGA_BF16 && D != 128) return MOGA_ERR_UNSUPPORTED;
  if (dtype == MOGA_F32 && D != 64 && D != 128) return MOGA_ERR_UNSUPPORTED;
  // the bf16 kernels form per-lane byte offsets `row * 256` in 32 bits, relative to the first row
  // of a group: a group (hence a tensor) must have fewer than 2^24 rows
  if (dtype == MOGA_BF16 && (Nq >= ((int64_t)1 << 24) || Nk >= ((int64_t)1 << 24))) return MOGA_ERR_UNSUPPORTED;
  return MOGA_OK;
}

extern "C" int moga_group_attn_fwd(const void* qh, const void* kh, const void* vh, int dtype,
                                   int64_t N, int H, int D, const int32_t* cu_seqlens, int M,
                                   float softmax_scale, void* oh, float* lse, void* ws,
                                   size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  const int bad = check_attn_args(N, N, H, D, M, softmax_scale, dtype);
  if (bad) return bad;
  if (M > MOGA_MAX_GROUPS) return MOGA_ERR_UNSUPPORTED;
  if (N == 0) return MOGA_OK;
  if (!qh || !kh || !vh || !cu_seqlens || !oh || !lse) return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(qh) && aligned16(kh) && aligned16(vh) && aligned16(oh))) return MOGA_ERR_INVALID_ARG;
  return launch_attn_fwd(qh, kh, vh, dtype, N, N, H, D, cu_seqlens, cu_seqlens, nullptr, M,
                         softmax_scale, oh, lse, (hipStream_t)stream);
}

extern "C" int moga_fused_attn_fwd(const void* q, const void* k, const void* v, int dtype, int64_t N,
                                   int H, int D, const int32_t* perm, const float* gate,
                                   const int32_t* cu_seqlens, int M, float softmax_scale, void* o,
                                   float* lse, void* stream) {
  const int bad = check_attn_args(N, N, H, D, M, softmax_scale, dtype);
  if (bad) return bad;
  if (M > MOGA_MAX_GROUPS || dtype != MOGA_BF16) return MOGA_ERR_UNSUPPORTED;
  if (N == 0) return MOGA_OK;
  if (!q || !k || !v || !perm || !gate || !cu_seqlens || !o || !lse) return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(o))) return MOGA_ERR_INVALID_ARG;
  const int64_t tiles = max_tiles(N, M, 256);
  const int64_t blocks = (tiles * H + 7) / 8 * 8;
  if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  attn_fwd_bf16_pipe_kernel<8, 1, true><<<(unsigned)blocks, 512, 0, (hipStream_t)stream>>>(
      (const unsigned short*)q, (const unsigned short*)k, (const unsigned short*)v, cu_seqlens, cu_seqlens,
      nullptr, M, N, N, H, softmax_scale, (int)tiles, (unsigned short*)o, lse, perm, gate);
  return launch_status();
}

extern "C" size_t moga_varlen_attn_fwd_ws_bytes(int G) { return ((size_t)G + 1) * sizeof(int32_t); }

extern "C" int moga_varlen_attn_fwd(const void* qh, const void* kh, const void* vh, int dtype,
                                    int64_t Nq, int64_t Nk, int H, int D,
                                    const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int G,
                                    float softmax_scale, void* oh, float* lse, void* ws,
                                    size_t ws_bytes, void* stream) {
  const int bad = check_attn_args(Nq, Nk, H, D, G, softmax_scale, dtype);
  if (bad) return bad;
  if (G > MOGA_MAX_SEGMENTS) return MOGA_ERR_UNSUPPORTED;
  if (Nq == 0) return MOGA_OK;
  if (!qh || !cu_seqlens_q || !cu_seqlens_k || !oh || !lse) return MOGA_ERR_INVALID_ARG;
  if (Nk > 0 && (!kh || !vh)) return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(qh) && aligned16(kh) && aligned16(vh) && aligned16(oh))) return MOGA_ERR_INVALID_ARG;
  if (!ws || ws_bytes < moga_varlen_attn_fwd_ws_bytes(G)) return MOGA_ERR_WORKSPACE;
  return launch_attn_fwd(qh, kh, vh, dtype, Nq, Nk, H, D, cu_seqlens_q, cu_seqlens_k, (int32_t*)ws, G,
                         softmax_scale, oh, lse, (hipStream_t)stream);
}
