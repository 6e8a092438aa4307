// Token router of MoGA (Eqs. 2-4 of the paper) and its backward through the gate of Eq. 5.
//
//   logits = X W^T, probs = softmax(logits), group = argmax, gate = probs[group].
//
// Two forward kernels:
//   * route_mfma_kernel: bf16 X.  logits^T = W X^T on bf16 MFMA with fp32-GEMM semantics:
//     each fp32 weight is split exactly into three bf16 limbs (hi + mid + lo == w), every
//     limb product with a bf16 activation is exact in fp32, and only the accumulation
//     rounds.  Groups are the MFMA rows and tokens the columns, so a lane ends up holding
//     half of one token's logits: argmax / softmax need one exchange between wave halves.
//   * route_generic_kernel: any dtype / shape; one wave per token, fp32 FMA.
#include "moga_common.h"

namespace moga {

// ---------------------------------------------------------------------------------------
// generic: one wave per token
// ---------------------------------------------------------------------------------------
template <typename XT> __device__ __forceinline__ float load_x(const XT* p);
template <> __device__ __forceinline__ float load_x<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_x<unsigned short>(const unsigned short* p) {
  return bf16_bits_to_f32(*p);
}

template <typename XT>
__global__ __launch_bounds__(256) void route_generic_kernel(
    const XT* __restrict__ x, const float* __restrict__ w, const float* __restrict__ bias,
    int64_t N, int d, int M, int32_t* __restrict__ group, float* __restrict__ gate,
    float* __restrict__ probs, float* __restrict__ logits) {
  __shared__ float s_logit[4][MOGA_MAX_GROUPS];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int64_t tok = (int64_t)blockIdx.x * 4 + wave;
  const bool valid = tok < N;
  if (!valid) tok = N - 1;
  const XT* xr = x + tok * (int64_t)d;

  for (int j0 = 0; j0 < M; j0 += 8) {
    float acc[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) acc[jj] = 0.f;
    for (int c = lane; c < d; c += 64) {
      const float xv = load_x<XT>(xr + c);
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        const int j = min(j0 + jj, M - 1);
        acc[jj] = fmaf(xv, w[(int64_t)j * d + c], acc[jj]);
      }
    }
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      const float r = wave_sum(acc[jj]);
      if (lane == jj && j0 + jj < M) s_logit[wave][j0 + jj] = r + (bias ? bias[j0 + jj] : 0.f);
    }
  }
  __syncthreads();

  // argmax (lowest index on ties) and softmax over the M logits of this wave's token
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int j = lane; j < M; j += 64) {
    const float r = s_logit[wave][j];
    if (r > best) { best = r; bi = j; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, kWave);
    const int oi = __shfl_xor(bi, o, kWave);
    if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
  }
  float sum = 0.f;
  for (int j = lane; j < M; j += 64) sum += expf(s_logit[wave][j] - best);
  sum = wave_sum(sum);
  const float g = 1.f / sum;
  if (valid) {
    if (lane == 0) { group[tok] = bi; gate[tok] = g; }
    for (int j = lane; j < M; j += 64) {
      const float r = s_logit[wave][j];
      if (probs) probs[tok * M + j] = expf(r - best) * g;
      if (logits) logits[tok * M + j] = r;
    }
  }
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA path (M <= 32, d_model % 64 == 0)
// ---------------------------------------------------------------------------------------
constexpr int kRouteKC = 256;              // k-chunk of W staged in LDS
constexpr int kRouteStride = kRouteKC + 8; // bf16 elements per LDS row (+16 B against bank conflicts)

// Split an fp32 value into three bf16 limbs whose sum is exactly the value.
__device__ __forceinline__ void split3(float w, unsigned short& hi, unsigned short& mid,
                                       unsigned short& lo) {
  hi = f32_to_bf16_bits(w);
  const float r1 = w - bf16_bits_to_f32(hi);
  mid = f32_to_bf16_bits(r1);
  const float r2 = r1 - bf16_bits_to_f32(mid);
  lo = f32_to_bf16_bits(r2);
}

template <int TT>  // 32-token tiles per wave
__global__ __launch_bounds__(256, 2) void route_mfma_kernel(
    const unsigned short* __restrict__ x, const float* __restrict__ w,
    const float* __restrict__ bias, int64_t N, int d, int M, int32_t* __restrict__ group,
    float* __restrict__ gate, float* __restrict__ probs, float* __restrict__ logits) {
  __shared__ __attribute__((aligned(16))) unsigned short s_w[3][32][kRouteStride];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 31, h = lane >> 5;
  const int64_t tok0 = ((int64_t)blockIdx.x * 4 + wave) * (32 * TT);

  const unsigned short* xrow[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    int64_t tok = tok0 + 32 * t + r;
    if (tok > N - 1) tok = N - 1;
    xrow[t] = x + tok * (int64_t)d + 32 * h;
  }

  floatx16_t total[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) total[t][v] = 0.f;

  // Within a 64-wide k block, lane half h reads elements [32h, 32h+32) of its row as four
  // 16-byte pieces; piece s feeds MFMA k-step s.  The weight operand uses the same map.
  uintx4_t xb[TT][4];
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int s = 0; s < 4; ++s) xb[t][s] = *(const uintx4_t*)(xrow[t] + 8 * s);

  for (int k0 = 0; k0 < d; k0 += kRouteKC) {
    const int kc = min(kRouteKC, d - k0);
    __syncthreads();
    const int q4 = kc >> 2;
    for (int idx = threadIdx.x; idx < 32 * q4; idx += 256) {
      const int row = idx / q4, c = (idx - row * q4) * 4;
      floatx4_t wv = {0.f, 0.f, 0.f, 0.f};
      if (row < M) wv = *(const floatx4_t*)(w + (int64_t)row * d + k0 + c);
      unsigned short hi[4], mid[4], lo[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) split3(wv[e], hi[e], mid[e], lo[e]);
      uintx2_t ph = {hi[0] | ((unsigned)hi[1] << 16), hi[2] | ((unsigned)hi[3] << 16)};
      uintx2_t pm = {mid[0] | ((unsigned)mid[1] << 16), mid[2] | ((unsigned)mid[3] << 16)};
      uintx2_t pl = {lo[0] | ((unsigned)lo[1] << 16), lo[2] | ((unsigned)lo[3] << 16)};
      *(uintx2_t*)&s_w[0][row][c] = ph;
      *(uintx2_t*)&s_w[1][row][c] = pm;
      *(uintx2_t*)&s_w[2][row][c] = pl;
    }
    __syncthreads();

    floatx16_t acc[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

    for (int kb = 0; kb < kc; kb += 64) {
      // prefetch the next 64-wide block of X (clamped to the row's last block at the very end)
      uintx4_t xn[TT][4];
      const int knext = min(k0 + kb + 64, d - 64);
#pragma unroll
      for (int t = 0; t < TT; ++t)
#pragma unroll
        for (int s = 0; s < 4; ++s) xn[t][s] = *(const uintx4_t*)(xrow[t] + knext + 8 * s);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int limb = 0; limb < 3; ++limb) {
          const bf16x8_t a = *(const bf16x8_t*)&s_w[limb][r][kb + 32 * h + 8 * s];
#pragma unroll
          for (int t = 0; t < TT; ++t)
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                a, __builtin_bit_cast(bf16x8_t, xb[t][s]), acc[t], 0, 0, 0);
        }
      }
#pragma unroll
      for (int t = 0; t < TT; ++t)
#pragma unroll
        for (int s = 0; s < 4; ++s) xb[t][s] = xn[t][s];
    }
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) total[t][v] += acc[t][v];
  }

  // Epilogue: accumulator register v of lane (r, h) is group row 8*(v/4) + 4*h + v%4 of token r.
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int64_t tok = tok0 + 32 * t + r;
    float vals[16];
    float best = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = 8 * (v >> 2) + 4 * h + (v & 3);
      float val = total[t][v];
      if (row < M) {
        if (bias) val += bias[row];
      } else {
        val = -INFINITY;
      }
      vals[v] = val;
      if (val > best) { best = val; bi = row; }
    }
    const float ob = other_half(best);
    const int oi = other_half_i(bi);
    if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
    float sum = 0.f;
    float e[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) { e[v] = expf(vals[v] - best); sum += e[v]; }
    sum += other_half(sum);
    const float g = 1.f / sum;
    if (tok < N) {
      if (h == 0) { group[tok] = bi; gate[tok] = g; }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = 8 * (v >> 2) + 4 * h + (v & 3);
        if (row < M) {
          if (probs) probs[tok * M + row] = e[v] * g;
          if (logits) logits[tok * M + row] = vals[v];
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// backward: dr = d_gate * gate * (onehot(group) - probs);  dW = dr^T X;  dX = dr W
// ---------------------------------------------------------------------------------------
constexpr int kRbTok = 64;  // tokens per staged tile
constexpr int kRbMB = 32;   // groups per pass

template <typename XT>
__global__ __launch_bounds__(256) void route_bwd_dw_partial_kernel(
    const XT* __restrict__ x, const float* __restrict__ probs, const int32_t* __restrict__ group,
    const float* __restrict__ gate, const float* __restrict__ d_gate, int64_t N, int d, int M,
    int64_t tokens_per_split, float* __restrict__ partial /* [splits][M][d] */) {
  __shared__ float s_dr[kRbTok][kRbMB];
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int split = blockIdx.y;
  const int j0 = blockIdx.z * kRbMB;
  const int mb = min(kRbMB, M - j0);
  const int64_t t0 = (int64_t)split * tokens_per_split;
  const int64_t t1 = min(N, t0 + tokens_per_split);
  float acc[kRbMB];
#pragma unroll
  for (int j = 0; j < kRbMB; ++j) acc[j] = 0.f;

  for (int64_t tb = t0; tb < t1; tb += kRbTok) {
    const int nt = (int)min((int64_t)kRbTok, t1 - tb);
    __syncthreads();
    for (int idx = threadIdx.x; idx < kRbTok * kRbMB; idx += 256) {
      const int ti = idx / kRbMB, j = idx - ti * kRbMB;
      float v = 0.f;
      if (ti < nt && j < mb) {
        const int64_t tok = tb + ti;
        const float coef = d_gate[tok] * gate[tok];
        const float onehot = (group[tok] == j0 + j) ? 1.f : 0.f;
        v = coef * (onehot - probs[tok * M + j0 + j]);
      }
      s_dr[ti][j] = v;
    }
    __syncthreads();
    if (c < d) {
      for (int ti = 0; ti < nt; ++ti) {
        const float xv = load_x<XT>(x + (tb + ti) * (int64_t)d + c);
#pragma unroll
        for (int j = 0; j < kRbMB; ++j) acc[j] = fmaf(s_dr[ti][j], xv, acc[j]);
      }
    }
  }
  if (c < d) {
    for (int j = 0; j < mb; ++j)
      partial[((int64_t)split * M + j0 + j) * d + c] = acc[j];
  }
}

__global__ __launch_bounds__(256) void route_bwd_dw_reduce_kernel(
    const float* __restrict__ partial, int splits, int64_t md, float* __restrict__ d_w) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= md) return;
  float s = 0.f;
  for (int k = 0; k < splits; ++k) s += partial[(int64_t)k * md + i];
  d_w[i] = s;
}

__global__ __launch_bounds__(256) void route_bwd_dx_kernel(
    const float* __restrict__ w, const float* __restrict__ probs,
    const int32_t* __restrict__ group, const float* __restrict__ gate,
    const float* __restrict__ d_gate, int64_t N, int d, int M, float* __restrict__ d_x) {
  __shared__ float s_dr[kRbTok][kRbMB];
  const int c = blockIdx.y * 256 + threadIdx.x;
  const int64_t tb = (int64_t)blockIdx.x * kRbTok;
  const int nt = (int)min((int64_t)kRbTok, N - tb);
  float out[kRbTok];
#pragma unroll
  for (int ti = 0; ti < kRbTok; ++ti) out[ti] = 0.f;
  for (int j0 = 0; j0 < M; j0 += kRbMB) {
    const int mb = min(kRbMB, M - j0);
    __syncthreads();
    for (int idx = threadIdx.x; idx < kRbTok * kRbMB; idx += 256) {
      const int ti = idx / kRbMB, j = idx - ti * kRbMB;
      float v = 0.f;
      if (ti < nt && j < mb) {
        const int64_t tok = tb + ti;
        const float coef = d_gate[tok] * gate[tok];
        const float onehot = (group[tok] == j0 + j) ? 1.f : 0.f;
        v = coef * (onehot - probs[tok * M + j0 + j]);
      }
      s_dr[ti][j] = v;
    }
    __syncthreads();
    if (c < d) {
      for (int j = 0; j < mb; ++j) {
        const float wv = w[(int64_t)(j0 + j) * d + c];
#pragma unroll
        for (int ti = 0; ti < kRbTok; ++ti) out[ti] = fmaf(s_dr[ti][j], wv, out[ti]);
      }
    }
  }
  if (c < d) {
#pragma unroll
    for (int ti = 0; ti < kRbTok; ++ti)
      if (ti < nt) d_x[(tb + ti) * (int64_t)d + c] = out[ti];
  }
}

static int route_bwd_splits(int64_t N) {
  int64_t s = (N + 2047) / 2048;
  if (s < 1) s = 1;
  if (s > 64) s = 64;
  return (int)s;
}

}  // namespace moga

using namespace moga;

extern "C" size_t moga_route_bwd_ws_bytes(int64_t N, int M, int d_model) {
  return (size_t)route_bwd_splits(N) * (size_t)M * (size_t)d_model * sizeof(float);
}

extern "C" int moga_route(const void* x, int x_dtype, const float* w, const float* bias,
                          int64_t N, int d_model, int M, int32_t* group, float* gate,
                          float* probs, float* logits, void* ws, size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  if (N < 0 || d_model < 1 || M < 1) return MOGA_ERR_INVALID_ARG;
  if (x_dtype != MOGA_F32 && x_dtype != MOGA_BF16) return MOGA_ERR_UNSUPPORTED;
  if (M > MOGA_MAX_GROUPS || N >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  if (N == 0) return MOGA_OK;
  if (!x || !w || !group || !gate) return MOGA_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(w)) return MOGA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (x_dtype == MOGA_BF16 && M <= 32 && d_model % 64 == 0) {
    if (N >= 65536) {
      const unsigned blocks = (unsigned)((N + 255) / 256);
      route_mfma_kernel<2><<<blocks, 256, 0, st>>>((const unsigned short*)x, w, bias, N, d_model, M,
                                                  group, gate, probs, logits);
    } else {
      const unsigned blocks = (unsigned)((N + 127) / 128);
      route_mfma_kernel<1><<<blocks, 256, 0, st>>>((const unsigned short*)x, w, bias, N, d_model, M,
                                                  group, gate, probs, logits);
    }
  } else {
    const unsigned blocks = (unsigned)((N + 3) / 4);
    if (x_dtype == MOGA_F32)
      route_generic_kernel<float><<<blocks, 256, 0, st>>>((const float*)x, w, bias, N, d_model, M,
                                                         group, gate, probs, logits);
    else
      route_generic_kernel<unsigned short><<<blocks, 256, 0, st>>>(
          (const unsigned short*)x, w, bias, N, d_model, M, group, gate, probs, logits);
  }
  return launch_status();
}

extern "C" int moga_route_bwd(const void* x, int x_dtype, const float* w, const float* probs,
                              const int32_t* group, const float* gate, const float* d_gate,
                              int64_t N, int d_model, int M, float* d_w, float* d_x,
                              void* ws, size_t ws_bytes, void* stream) {
  if (N < 0 || d_model < 1 || M < 1) return MOGA_ERR_INVALID_ARG;
  if (x_dtype != MOGA_F32 && x_dtype != MOGA_BF16) return MOGA_ERR_UNSUPPORTED;
  if (M > MOGA_MAX_GROUPS || N >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  if (!d_w) return MOGA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  const int64_t md = (int64_t)M * d_model;
  if (N == 0) {
    fill_zero_kernel<<<(unsigned)((md + 255) / 256), 256, 0, st>>>(d_w, md);
    return launch_status();
  }
  if (!x || !w || !probs || !group || !gate || !d_gate) return MOGA_ERR_INVALID_ARG;
  const size_t need = moga_route_bwd_ws_bytes(N, M, d_model);
  if (!ws || ws_bytes < need) return MOGA_ERR_WORKSPACE;
  const int splits = route_bwd_splits(N);
  int64_t tps = (N + splits - 1) / splits;
  tps = (tps + kRbTok - 1) / kRbTok * kRbTok;
  dim3 grid((d_model + 255) / 256, splits, (M + kRbMB - 1) / kRbMB);
  float* partial = (float*)ws;
  if (x_dtype == MOGA_F32)
    route_bwd_dw_partial_kernel<float><<<grid, 256, 0, st>>>((const float*)x, probs, group, gate,
                                                            d_gate, N, d_model, M, tps, partial);
  else
    route_bwd_dw_partial_kernel<unsigned short><<<grid, 256, 0, st>>>(
        (const unsigned short*)x, probs, group, gate, d_gate, N, d_model, M, tps, partial);
  route_bwd_dw_reduce_kernel<<<(unsigned)((md + 255) / 256), 256, 0, st>>>(partial, splits, md, d_w);
  if (d_x) {
    dim3 gx((unsigned)((N + kRbTok - 1) / kRbTok), (d_model + 255) / 256);
    route_bwd_dx_kernel<<<gx, 256, 0, st>>>(w, probs, group, gate, d_gate, N, d_model, M, d_x);
  }
  return launch_status();
}
