// Backward of the variable-length group attention (derivative of Eq. 1 inside each group).
//
// With P = exp(scale*S - lse) and delta = rowsum(dO * O):
//   dV = P^T dO,  dP = dO V^T,  dS = P * (dP - delta),  dQ = scale dS K,  dK = scale dS^T Q.
//
// Three kernels, no atomics, results independent of scheduling:
//   attn_bwd_delta   : delta[h][j] = sum_c dO[h][j][c] * O[h][j][c]
//   attn_bwd_dkdv    : a wave owns 32 key rows (K, V fragments and the dK^T, dV^T accumulators
//                      live in registers) and sweeps the query tiles of its group;
//   attn_bwd_dq      : a wave owns 32 query rows and sweeps the key tiles (mirror of forward).
// The bf16 MFMA kernels are in attn_bwd_pipe.h: they keep the contraction index of the second
// product in the accumulator registers of the first (row permutation of the LDS operand), and
// read the transposed operands (dO^T, Q^T, K^T) from row-major LDS tiles with the transposing
// LDS read.  The fp32 kernels below use one thread per row.
#include <atomic>

#include "attn_common.h"
#include "attn_bwd_pipe.h"

namespace moga {


// ---------------------------------------------------------------------------------------
template <int LPR, bool BF16>
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(const uintx4_t* __restrict__ d_oh,
                                                             const uintx4_t* __restrict__ oh,
                                                             const float* __restrict__ lse, int64_t rows,
                                                             float inv_scale, float* __restrict__ delta,
                                                             float* __restrict__ neg_lse_over_scale,
                                                             int* __restrict__ status) {
  if (status && blockIdx.x == 0 && threadIdx.x == 0) *status = 0;   // read by the kernels that follow
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
    if (neg_lse_over_scale) {   // bf16 kernels: both arrays negated, ready to start an accumulator from
      delta[row] = -s;
      neg_lse_over_scale[row] = -lse[row] * inv_scale;
    } else {
      delta[row] = s;
    }
  }
}

// Pre-pass of the gather-fused backward (bf16, head_dim 128; token-major inputs).  With O = gate * A
// (Eq. 5) and dO the upstream gradient of O:  delta = rowsum(dA * A) = rowsum(dO * O) =: dot, and the
// kernels can consume the raw dO rows if the gate is folded into the per-row constants:
//   P' = gate * P = exp(S - (lse - ln gate)),   dS = P' * (dO V^T - dot / gate),   dV = P'^T dO.
// Writes, in sorted order [H, N]:  -(lse - ln gate) / scale  and  -dot / gate;  and per token
// d_gate = sum over heads of dot / gate.  16 tokens per block, 16 lanes per (token, head) row.
__global__ __launch_bounds__(256) void attn_bwd_fused_prepass_kernel(
    const uintx4_t* __restrict__ d_o, const uintx4_t* __restrict__ o, const float* __restrict__ lse,
    const int32_t* __restrict__ inv_perm, const float* __restrict__ gate, int64_t N, int H,
    float inv_scale, float* __restrict__ neg_lse_over_scale, float* __restrict__ neg_delta,
    float* __restrict__ d_gate, int* __restrict__ status) {
  __shared__ float s_part[4][16];
  if (blockIdx.x == 0 && threadIdx.x == 0) *status = 0;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int part = lane & 15, rsub = lane >> 4;
  const int64_t t0 = (int64_t)blockIdx.x * 16;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  int64_t slot[4];
  float g[4], lg[4];
  bool ok[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int64_t t = t0 + it * 4 + rsub;
    ok[it] = t < N;
    slot[it] = ok[it] ? inv_perm[t] : 0;
    g[it] = ok[it] ? gate[t] : 1.f;
    lg[it] = logf(g[it]);
  }
  for (int h = wave; h < H; h += 4) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      if (!ok[it]) continue;
      const int64_t t = t0 + it * 4 + rsub;
      const uintx4_t a = d_o[(t * H + h) * 16 + part], b = o[(t * H + h) * 16 + part];
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        s = fmaf(bf16_lo_to_f32(a[i]), bf16_lo_to_f32(b[i]), s);
        s = fmaf(bf16_hi_to_f32(a[i]), bf16_hi_to_f32(b[i]), s);
      }
#pragma unroll
      for (int o2 = 8; o2 > 0; o2 >>= 1) s += __shfl_xor(s, o2, kWave);
      const float dg = s / g[it];
      acc[it] += dg;
      if (part == 0) {
        const int64_t idx = (int64_t)h * N + slot[it];
        neg_lse_over_scale[idx] = -(lse[idx] - lg[it]) * inv_scale;
        neg_delta[idx] = -dg;
      }
    }
  }
#pragma unroll
  for (int it = 0; it < 4; ++it)
    if (part == 0) s_part[wave][it * 4 + rsub] = acc[it];
  __syncthreads();
  if (threadIdx.x < 16) {
    const int64_t t = t0 + threadIdx.x;
    if (t < N)
      d_gate[t] = (s_part[0][threadIdx.x] + s_part[1][threadIdx.x]) + (s_part[2][threadIdx.x] + s_part[3][threadIdx.x]);
  }
}

// ---------------------------------------------------------------------------------------
// fp32 (head_dim 64): one thread per row
// ---------------------------------------------------------------------------------------
constexpr int kF32BM = 64, kF32BN = 32;
constexpr int64_t kSmallGroupRows = 1280;   // mean rows per group below which the small-group bf16 kernels run
                                            // (398 against 334 TFLOP/s at 312 rows, equal at 1,560, slower above)

template <int D>
__global__ __launch_bounds__(64) void attn_bwd_dq_f32_kernel(
    const float* __restrict__ d_oh, const float* __restrict__ qh, const float* __restrict__ kh,
    const float* __restrict__ vh, const float* __restrict__ lse, const float* __restrict__ delta,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_k,
    const int32_t* __restrict__ tile_start, int M, int64_t Nq, int64_t Nk, int H, float scale,
    int tiles_per_head, float* __restrict__ d_qh) {
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
  const int64_t rr = head_off + (valid ? row : ge - 1);
  float q[D], dO[D], dq[D];
#pragma unroll
  for (int cI = 0; cI < D; ++cI) { q[cI] = qh[rr * D + cI]; dO[cI] = d_oh[rr * D + cI]; dq[cI] = 0.f; }
  const float l = lse[rr], dl = delta[rr];

  for (int kv0 = kbeg; kv0 < kend; kv0 += kF32BN) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < kF32BN * (D / 4); idx += 64) {
      const int r2 = idx / (D / 4), c4 = (idx - r2 * (D / 4)) * 4;
      floatx4_t kk = {0.f, 0.f, 0.f, 0.f}, vv = {0.f, 0.f, 0.f, 0.f};
      if (kv0 + r2 < kend) {
        kk = *(const floatx4_t*)(kh + (head_off_k + kv0 + r2) * D + c4);
        vv = *(const floatx4_t*)(vh + (head_off_k + kv0 + r2) * D + c4);
      }
      *(floatx4_t*)&Ks[r2][c4] = kk;
      *(floatx4_t*)&Vs[r2][c4] = vv;
    }
    __syncthreads();
    const int nk = min(kF32BN, kend - kv0);
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
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_k,
    const int32_t* __restrict__ tile_start, int M, int64_t Nq, int64_t Nk, int H, float scale,
    int tiles_per_head, float* __restrict__ d_kh, float* __restrict__ d_vh) {
  __shared__ __attribute__((aligned(16))) float Qs[kF32BN][D];
  __shared__ __attribute__((aligned(16))) float dOs[kF32BN][D];
  __shared__ float s_lse[kF32BN], s_delta[kF32BN];
  __shared__ int s_start[MOGA_MAX_GROUPS + 1];
  __shared__ int s_found;
  const int head = blockIdx.x / tiles_per_head;
  const int tile = blockIdx.x - head * tiles_per_head;
  TileInfo ti;   // tiles run over the key rows of the groups
  if (tile_start) {
    if (!find_tile_presummed(tile_start, cu_k, M, kF32BM, tile, ti)) return;
  } else if (!find_tile(cu_k, M, kF32BM, tile, s_start, &s_found, ti)) {
    return;
  }
  const int ge = ti.row_end;
  const int qbeg = cu_q[ti.group], qend = cu_q[ti.group + 1];   // query rows of the group
  const int64_t head_off = (int64_t)head * Nk;     // key-side tensors
  const int64_t head_off_q = (int64_t)head * Nq;   // query-side tensors
  const int row = ti.tile_row + threadIdx.x;
  const bool valid = row < ge;
  const int64_t rr = head_off + (valid ? row : ge - 1);
  float k[D], v[D], dk[D], dv[D];
#pragma unroll
  for (int cI = 0; cI < D; ++cI) { k[cI] = kh[rr * D + cI]; v[cI] = vh[rr * D + cI]; dk[cI] = 0.f; dv[cI] = 0.f; }

  for (int q0 = qbeg; q0 < qend; q0 += kF32BN) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < kF32BN * (D / 4); idx += 64) {
      const int r2 = idx / (D / 4), c4 = (idx - r2 * (D / 4)) * 4;
      floatx4_t qq = {0.f, 0.f, 0.f, 0.f}, dd = {0.f, 0.f, 0.f, 0.f};
      if (q0 + r2 < qend) {
        qq = *(const floatx4_t*)(qh + (head_off_q + q0 + r2) * D + c4);
        dd = *(const floatx4_t*)(d_oh + (head_off_q + q0 + r2) * D + c4);
      }
      *(floatx4_t*)&Qs[r2][c4] = qq;
      *(floatx4_t*)&dOs[r2][c4] = dd;
    }
    if (threadIdx.x < kF32BN) {
      const int g = q0 + threadIdx.x;
      s_lse[threadIdx.x] = g < qend ? lse[head_off_q + g] : INFINITY;
      s_delta[threadIdx.x] = g < qend ? delta[head_off_q + g] : 0.f;
    }
    __syncthreads();
    const int nq = min(kF32BN, qend - q0);
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

// Workspace layout of the backward calls: [-delta: rows floats][-lse/scale: rows floats][status:
// 16 bytes, first int32 used], rows = Nq * H; the varlen call appends its two tile-start lists.
static size_t bwd_rows_bytes(int64_t Nq, int H) { return round_up(2 * (size_t)Nq * (size_t)H * sizeof(float), 16); }

extern "C" size_t moga_attn_bwd_status_offset(int64_t Nq, int H) {
  if (Nq <= 0 || H < 1) return 0;
  return bwd_rows_bytes(Nq, H);
}

extern "C" size_t moga_attn_bwd_ws_bytes(int64_t N, int H, int D, int dtype) {
  (void)D; (void)dtype;
  if (N <= 0 || H < 1) return 0;
  return bwd_rows_bytes(N, H) + 16;
}

// Polls after which a wave of the dK/dV kernel that waits for its partner's P gives up (and sets the
// status word).  In normal operation a wait lasts a few hundred polls at most.
static std::atomic<int> g_spin_limit{1 << 24};
extern "C" void moga_debug_set_spin_limit(int polls) { g_spin_limit.store(polls < 0 ? 0 : polls); }

// The bf16 kernels form per-lane byte offsets `row * 256` in 32 bits, relative to the first row of
// a group: a group (hence a tensor) must have fewer than 2^24 rows.
static bool bf16_rows_ok(int64_t Nq, int64_t Nk) { return Nq < ((int64_t)1 << 24) && Nk < ((int64_t)1 << 24); }

// Shared launcher.  ts_q / ts_k: NULL (tile lookup inside the kernels, M <= MOGA_MAX_GROUPS) or
// space for the pre-summed first-tile indices over query rows / key rows (M + 1 ints each).
static int launch_attn_bwd(const void* d_oh, const void* qh, const void* kh, const void* vh,
                           const void* oh, const float* lse, int dtype, int64_t Nq, int64_t Nk, int H, int D,
                           const int32_t* cu_q, const int32_t* cu_k, int32_t* ts_q, int32_t* ts_k,
                           int M, float softmax_scale, void* d_qh, void* d_kh, void* d_vh,
                           float* delta, hipStream_t st) {
  const int64_t rows = Nq * (int64_t)H;
  if ((rows * 32 + 255) / 256 >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;   // grid of the delta kernel
  if (dtype == MOGA_BF16) {
    if (!bf16_rows_ok(Nq, Nk)) return MOGA_ERR_UNSUPPORTED;
    float* lse2 = delta + rows;   // holds -lse/scale; `delta` holds -delta
    int* status = (int*)((char*)delta + bwd_rows_bytes(Nq, H));
    attn_bwd_delta_kernel<16, true><<<(unsigned)((rows * 16 + 255) / 256), 256, 0, st>>>(
        (const uintx4_t*)d_oh, (const uintx4_t*)oh, lse, rows, 1.f / softmax_scale, delta, lse2, status);
    // groups of a few thousand rows or less (the static groups of Section 3.2): 4-wave blocks with a
    // two-slot ring, two blocks per CU, and tiles half as large; the host only knows the mean group size
    const bool small = use_small_group_kernels(Nq, M, kSmallGroupRows);
    if (Nk > 0) {
      const int bk = small ? 64 : 128;
      const int64_t tiles = max_tiles(Nk, M, bk);
      const int64_t blocks = (tiles * H + 7) / 8 * 8;
      if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
      if (ts_k) tile_start_kernel<<<1, 1024, 0, st>>>(cu_k, M, bk, ts_k);
      if (small)
        attn_bwd_dkdv_ab_kernel<false, 2, 2><<<(unsigned)blocks, 256, 0, st>>>(
            (const unsigned short*)d_oh, (const unsigned short*)qh, (const unsigned short*)kh,
            (const unsigned short*)vh, lse2, delta, cu_q, cu_k, ts_k, M, Nq, Nk, H, softmax_scale,
            (int)tiles, (unsigned short*)d_kh, (unsigned short*)d_vh, g_spin_limit.load(), status);
      else
        attn_bwd_dkdv_ab_kernel<false><<<(unsigned)blocks, 512, 0, st>>>(
            (const unsigned short*)d_oh, (const unsigned short*)qh, (const unsigned short*)kh,
            (const unsigned short*)vh, lse2, delta, cu_q, cu_k, ts_k, M, Nq, Nk, H, softmax_scale,
            (int)tiles, (unsigned short*)d_kh, (unsigned short*)d_vh, g_spin_limit.load(), status);
    }
    {
      const int bm = small ? 128 : 256;
      const int64_t tiles = max_tiles(Nq, M, bm);
      const int64_t blocks = (tiles * H + 7) / 8 * 8;
      if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
      if (ts_q) tile_start_kernel<<<1, 1024, 0, st>>>(cu_q, M, bm, ts_q);
      if (small)
        attn_bwd_dq_pipe_kernel<4, 1, false, 2><<<(unsigned)blocks, 256, 0, st>>>(
            (const unsigned short*)d_oh, (const unsigned short*)qh, (const unsigned short*)kh,
            (const unsigned short*)vh, lse2, delta, cu_q, cu_k, ts_q, M, Nq, Nk, H, softmax_scale,
            (int)tiles, (unsigned short*)d_qh);
      else
        attn_bwd_dq_pipe_kernel<8, 1><<<(unsigned)blocks, 512, 0, st>>>(
            (const unsigned short*)d_oh, (const unsigned short*)qh, (const unsigned short*)kh,
            (const unsigned short*)vh, lse2, delta, cu_q, cu_k, ts_q, M, Nq, Nk, H, softmax_scale,
            (int)tiles, (unsigned short*)d_qh);
    }
  } else {
    if (D == 64)
      attn_bwd_delta_kernel<16, false><<<(unsigned)((rows * 16 + 255) / 256), 256, 0, st>>>(
          (const uintx4_t*)d_oh, (const uintx4_t*)oh, lse, rows, 1.f, delta, nullptr, nullptr);
    else
      attn_bwd_delta_kernel<32, false><<<(unsigned)((rows * 32 + 255) / 256), 256, 0, st>>>(
          (const uintx4_t*)d_oh, (const uintx4_t*)oh, lse, rows, 1.f, delta, nullptr, nullptr);
    if (Nk > 0) {
      const int64_t tiles = max_tiles(Nk, M, kF32BM);
      const int64_t blocks = tiles * H;
      if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
      if (ts_k) tile_start_kernel<<<1, 1024, 0, st>>>(cu_k, M, kF32BM, ts_k);
      if (D == 64)
        attn_bwd_dkdv_f32_kernel<64><<<(unsigned)blocks, 64, 0, st>>>(
            (const float*)d_oh, (const float*)qh, (const float*)kh, (const float*)vh, lse, delta,
            cu_q, cu_k, ts_k, M, Nq, Nk, H, softmax_scale, (int)tiles, (float*)d_kh, (float*)d_vh);
      else
        attn_bwd_dkdv_f32_kernel<128><<<(unsigned)blocks, 64, 0, st>>>(
            (const float*)d_oh, (const float*)qh, (const float*)kh, (const float*)vh, lse, delta,
            cu_q, cu_k, ts_k, M, Nq, Nk, H, softmax_scale, (int)tiles, (float*)d_kh, (float*)d_vh);
    }
    const int64_t tiles = max_tiles(Nq, M, kF32BM);
    const int64_t blocks = tiles * H;
    if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
    if (ts_q) tile_start_kernel<<<1, 1024, 0, st>>>(cu_q, M, kF32BM, ts_q);
    if (D == 64)
      attn_bwd_dq_f32_kernel<64><<<(unsigned)blocks, 64, 0, st>>>(
          (const float*)d_oh, (const float*)qh, (const float*)kh, (const float*)vh, lse, delta,
          cu_q, cu_k, ts_q, M, Nq, Nk, H, softmax_scale, (int)tiles, (float*)d_qh);
    else
      attn_bwd_dq_f32_kernel<128><<<(unsigned)blocks, 64, 0, st>>>(
          (const float*)d_oh, (const float*)qh, (const float*)kh, (const float*)vh, lse, delta,
          cu_q, cu_k, ts_q, M, Nq, Nk, H, softmax_scale, (int)tiles, (float*)d_qh);
  }
  return launch_status();
}

static int check_attn_bwd_args(int64_t Nq, int64_t Nk, int H, int D, int M, float softmax_scale, int dtype) {
  if (Nq < 0 || Nk < 0 || H < 1 || D < 1 || M < 1) return MOGA_ERR_INVALID_ARG;
  if (!(softmax_scale > 0.f) || !(softmax_scale < INFINITY)) return MOGA_ERR_INVALID_ARG;
  if (dtype != MOGA_F32 && dtype != MOGA_BF16) return MOGA_ERR_UNSUPPORTED;
  if (Nq >= ((int64_t)1 << 31) || Nk >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  if (dtype == MOGA_BF16 && D != 128) return MOGA_ERR_UNSUPPORTED;
  if (dtype == MOGA_F32 && D != 64 && D != 128) return MOGA_ERR_UNSUPPORTED;
  return MOGA_OK;
}

extern "C" int moga_group_attn_bwd(const void* d_oh, const void* qh, const void* kh, const void* vh,
                                   const void* oh, const float* lse, int dtype, int64_t N, int H,
                                   int D, const int32_t* cu_seqlens, int M, float softmax_scale,
                                   void* d_qh, void* d_kh, void* d_vh, void* ws, size_t ws_bytes,
                                   void* stream) {
  const int bad = check_attn_bwd_args(N, N, H, D, M, softmax_scale, dtype);
  if (bad) return bad;
  if (M > MOGA_MAX_GROUPS) return MOGA_ERR_UNSUPPORTED;
  if (N == 0) return MOGA_OK;
  if (!d_oh || !qh || !kh || !vh || !oh || !lse || !cu_seqlens || !d_qh || !d_kh || !d_vh)
    return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(d_oh) && aligned16(qh) && aligned16(kh) && aligned16(vh) && aligned16(oh) &&
        aligned16(d_qh) && aligned16(d_kh) && aligned16(d_vh)))
    return MOGA_ERR_INVALID_ARG;
  const size_t need = moga_attn_bwd_ws_bytes(N, H, D, dtype);
  if (!ws || ws_bytes < need) return MOGA_ERR_WORKSPACE;
  return launch_attn_bwd(d_oh, qh, kh, vh, oh, lse, dtype, N, N, H, D, cu_seqlens, cu_seqlens, nullptr,
                         nullptr, M, softmax_scale, d_qh, d_kh, d_vh, (float*)ws, (hipStream_t)stream);
}

extern "C" size_t moga_varlen_attn_bwd_ws_bytes(int64_t Nq, int H, int G) {
  if (Nq <= 0 || H < 1) return 0;
  return bwd_rows_bytes(Nq, H) + 16 + 2 * ((size_t)G + 1) * sizeof(int32_t);
}

extern "C" int moga_varlen_attn_bwd(const void* d_oh, const void* qh, const void* kh, const void* vh,
                                    const void* oh, const float* lse, int dtype, int64_t Nq,
                                    int64_t Nk, int H, int D, const int32_t* cu_seqlens_q,
                                    const int32_t* cu_seqlens_k, int G, float softmax_scale,
                                    void* d_qh, void* d_kh, void* d_vh, void* ws, size_t ws_bytes,
                                    void* stream) {
  const int bad = check_attn_bwd_args(Nq, Nk, H, D, G, softmax_scale, dtype);
  if (bad) return bad;
  if (G > MOGA_MAX_SEGMENTS) return MOGA_ERR_UNSUPPORTED;
  if (Nq == 0 && Nk == 0) return MOGA_OK;
  if (!cu_seqlens_q || !cu_seqlens_k) return MOGA_ERR_INVALID_ARG;
  if (Nq > 0 && (!d_oh || !qh || !oh || !lse || !d_qh)) return MOGA_ERR_INVALID_ARG;
  if (Nk > 0 && (!kh || !vh || !d_kh || !d_vh)) return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(d_oh) && aligned16(qh) && aligned16(kh) && aligned16(vh) && aligned16(oh) &&
        aligned16(d_qh) && aligned16(d_kh) && aligned16(d_vh)))
    return MOGA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (Nq == 0) {   // keys without any query: zero gradients
    const int64_t nf = Nk * (int64_t)H * D / (dtype == MOGA_BF16 ? 2 : 1);
    if ((nf + 255) / 256 >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;   // grid of the fill kernel
    fill_zero_kernel<<<(unsigned)((nf + 255) / 256), 256, 0, st>>>((float*)d_kh, nf);
    fill_zero_kernel<<<(unsigned)((nf + 255) / 256), 256, 0, st>>>((float*)d_vh, nf);
    return launch_status();
  }
  const size_t need = moga_varlen_attn_bwd_ws_bytes(Nq, H, G);
  if (!ws || ws_bytes < need || !aligned16(ws)) return MOGA_ERR_WORKSPACE;
  int32_t* ts_q = (int32_t*)((char*)ws + bwd_rows_bytes(Nq, H) + 16);
  int32_t* ts_k = ts_q + (G + 1);
  return launch_attn_bwd(d_oh, qh, kh, vh, oh, lse, dtype, Nq, Nk, H, D, cu_seqlens_q, cu_seqlens_k, ts_q,
                         ts_k, G, softmax_scale, d_qh, d_kh, d_vh, (float*)ws, st);
}

extern "C" int moga_fused_attn_bwd(const void* d_o, const void* q, const void* k, const void* v,
                                   const void* o, const float* lse, int dtype, int64_t N, int H, int D,
                                   const int32_t* perm, const int32_t* inv_perm, const float* gate,
                                   const int32_t* cu_seqlens, int M, float softmax_scale, void* d_q,
                                   void* d_k, void* d_v, float* d_gate, void* ws, size_t ws_bytes,
                                   void* stream) {
  const int bad = check_attn_bwd_args(N, N, H, D, M, softmax_scale, dtype);
  if (bad) return bad;
  if (M > MOGA_MAX_GROUPS || dtype != MOGA_BF16 || !bf16_rows_ok(N, N)) return MOGA_ERR_UNSUPPORTED;
  if (N == 0) return MOGA_OK;
  if (!d_o || !q || !k || !v || !o || !lse || !perm || !inv_perm || !gate || !cu_seqlens || !d_q || !d_k ||
      !d_v || !d_gate)
    return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(d_o) && aligned16(q) && aligned16(k) && aligned16(v) && aligned16(o) && aligned16(d_q) &&
        aligned16(d_k) && aligned16(d_v)))
    return MOGA_ERR_INVALID_ARG;
  const size_t need = moga_attn_bwd_ws_bytes(N, H, D, dtype);
  if (!ws || ws_bytes < need) return MOGA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  float* delta = (float*)ws;
  float* lse2 = delta + N * (int64_t)H;
  int* status = (int*)((char*)ws + bwd_rows_bytes(N, H));
  attn_bwd_fused_prepass_kernel<<<(unsigned)((N + 15) / 16), 256, 0, st>>>(
      (const uintx4_t*)d_o, (const uintx4_t*)o, lse, inv_perm, gate, N, H, 1.f / softmax_scale, lse2, delta, d_gate,
      status);
  {
    const int64_t tiles = max_tiles(N, M, 128);
    const int64_t blocks = (tiles * H + 7) / 8 * 8;
    if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
    attn_bwd_dkdv_ab_kernel<true><<<(unsigned)blocks, 512, 0, st>>>(
        (const unsigned short*)d_o, (const unsigned short*)q, (const unsigned short*)k, (const unsigned short*)v,
        lse2, delta, cu_seqlens, cu_seqlens, nullptr, M, N, N, H, softmax_scale, (int)tiles, (unsigned short*)d_k,
        (unsigned short*)d_v, g_spin_limit.load(), status, perm);
  }
  {
    const int64_t tiles = max_tiles(N, M, 256);
    const int64_t blocks = (tiles * H + 7) / 8 * 8;
    if (blocks >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
    attn_bwd_dq_pipe_kernel<8, 1, true><<<(unsigned)blocks, 512, 0, st>>>(
        (const unsigned short*)d_o, (const unsigned short*)q, (const unsigned short*)k, (const unsigned short*)v,
        lse2, delta, cu_seqlens, cu_seqlens, nullptr, M, N, N, H, softmax_scale, (int)tiles, (unsigned short*)d_q,
        perm);
  }
  return launch_status();
}
