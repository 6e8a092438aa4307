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
// Backward: dr = d_gate * gate * (onehot(group) - probs), dW = dr^T X on bf16 MFMA (dr split in two
// bf16 limbs) for bf16 X, else with fp32 FMAs; optional dX = dr W.
#include <algorithm>

#include "lds_pipe.h"

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
constexpr int kRouteKC = 128;              // k-chunk of W staged in LDS (two 64-wide k blocks)
constexpr int kRouteStride = kRouteKC + 8; // bf16 elements per LDS row (+16 B against bank conflicts)
// float4 loads of W per thread and chunk in a block of NWV waves
template <int NWV> constexpr int kRouteWLoads = 32 * (kRouteKC / 4) / (64 * NWV);

// Split an fp32 value into three bf16 limbs whose sum is exactly the value.
__device__ __forceinline__ void split3(float w, unsigned short& hi, unsigned short& mid,
                                       unsigned short& lo) {
  hi = f32_to_bf16_bits(w);
  const float r1 = w - bf16_bits_to_f32(hi);
  mid = f32_to_bf16_bits(r1);
  const float r2 = r1 - bf16_bits_to_f32(mid);
  lo = f32_to_bf16_bits(r2);
}

// One thread's share of a weight chunk: rows of W beyond M and columns beyond d read as zero.
template <int NWV>
__device__ __forceinline__ void route_load_w(const float* __restrict__ w, int d, int M, int k0,
                                             floatx4_t (&wv)[kRouteWLoads<NWV>]) {
#pragma unroll
  for (int i = 0; i < kRouteWLoads<NWV>; ++i) {
    const int idx = threadIdx.x + 64 * NWV * i;
    const int row = idx / (kRouteKC / 4), c = (idx % (kRouteKC / 4)) * 4;
    const floatx4_t z = {0.f, 0.f, 0.f, 0.f};
    wv[i] = (row < M && k0 + c < d) ? *(const floatx4_t*)(w + (int64_t)row * d + k0 + c) : z;
  }
}

template <int NWV>
__device__ __forceinline__ void route_store_w(unsigned short (&sw)[3][32][kRouteStride],
                                              const floatx4_t (&wv)[kRouteWLoads<NWV>]) {
#pragma unroll
  for (int i = 0; i < kRouteWLoads<NWV>; ++i) {
    const int idx = threadIdx.x + 64 * NWV * i;
    const int row = idx / (kRouteKC / 4), c = (idx % (kRouteKC / 4)) * 4;
    unsigned short hi[4], mid[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) split3(wv[i][e], hi[e], mid[e], lo[e]);
    const uintx2_t ph = {hi[0] | ((unsigned)hi[1] << 16), hi[2] | ((unsigned)hi[3] << 16)};
    const uintx2_t pm = {mid[0] | ((unsigned)mid[1] << 16), mid[2] | ((unsigned)mid[3] << 16)};
    const uintx2_t pl = {lo[0] | ((unsigned)lo[1] << 16), lo[2] | ((unsigned)lo[3] << 16)};
    *(uintx2_t*)&sw[0][row][c] = ph;
    *(uintx2_t*)&sw[1][row][c] = pm;
    *(uintx2_t*)&sw[2][row][c] = pl;
  }
}

// A 64-wide k block of X as a wave's MFMA B operands: lane half h holds elements [32h, 32h+32) of
// its token's row as four 16-byte pieces; piece s feeds MFMA k-step s (the weight operand uses
// the same map).
template <int TT>
struct RouteXBlock {
  uintx4_t v[TT][4];
};

template <int TT>
__device__ __forceinline__ void route_load_x(RouteXBlock<TT>& b, const unsigned short* const (&xrow)[TT],
                                             int koff) {
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int s = 0; s < 4; ++s) b.v[t][s] = *(const uintx4_t*)(xrow[t] + koff + 8 * s);
}

template <int TT>
__device__ __forceinline__ void route_mfma_block(floatx16_t (&acc)[TT],
                                                 const unsigned short (&sw)[3][32][kRouteStride],
                                                 int col0, int r, int h, const RouteXBlock<TT>& b) {
#pragma unroll
  for (int s = 0; s < 4; ++s) {
#pragma unroll
    for (int limb = 0; limb < 3; ++limb) {
      const bf16x8_t a = *(const bf16x8_t*)&sw[limb][r][col0 + 32 * h + 8 * s];
#pragma unroll
      for (int t = 0; t < TT; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            a, __builtin_bit_cast(bf16x8_t, b.v[t][s]), acc[t], 0, 0, 0);
    }
  }
}

// The weight chunk is double-buffered: while the matrix cores work on chunk c, the fp32 weights of
// chunk c+1 are in flight from L2; they are split and stored after the chunk's MFMAs, one block
// barrier per chunk.  X lives in a ring of four k-block register sets with fixed roles (the loop
// is unrolled over two chunks, so no set is ever copied): a set is refilled, four k blocks ahead,
// right after its MFMAs, which keeps 16-32 KB of loads per wave in flight across the barriers.
template <int TT, int NWV>  // 32-token tiles per wave, waves per block
__global__ __launch_bounds__(64 * NWV, 2) void route_mfma_kernel(
    const unsigned short* __restrict__ x, const float* __restrict__ w,
    const float* __restrict__ bias, int64_t N, int d, int M, int32_t* __restrict__ group,
    float* __restrict__ gate, float* __restrict__ probs, float* __restrict__ logits) {
  __shared__ __attribute__((aligned(16))) unsigned short s_w[2][3][32][kRouteStride];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 31, h = lane >> 5;
  const int64_t tok0 = ((int64_t)blockIdx.x * NWV + wave) * (32 * TT);

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

  // k blocks past the end of the row are clamped to the last one (loaded, never used)
  const int last_kb = d - 64;
  RouteXBlock<TT> b0, b1, b2, b3;
  route_load_x<TT>(b0, xrow, 0);
  route_load_x<TT>(b1, xrow, min(64, last_kb));
  route_load_x<TT>(b2, xrow, min(128, last_kb));
  route_load_x<TT>(b3, xrow, min(192, last_kb));
  floatx4_t wv[kRouteWLoads<NWV>];
  route_load_w<NWV>(w, d, M, 0, wv);
  route_store_w<NWV>(s_w[0], wv);
  __syncthreads();

  const int nchunks = (d + kRouteKC - 1) / kRouteKC;
  // One chunk: k blocks (BA, BB) against weight buffer BUF.
#define MOGA_ROUTE_CHUNK(BA, BB, BUF, C)                                          \
  {                                                                                \
    const int k0 = (C) * kRouteKC;                                                 \
    const bool more = (C) + 1 < nchunks;                                           \
    if (more) route_load_w<NWV>(w, d, M, k0 + kRouteKC, wv);                         \
    floatx16_t acc[TT];                                                            \
    _Pragma("unroll") for (int t = 0; t < TT; ++t)                                 \
      _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;              \
    route_mfma_block<TT>(acc, s_w[BUF], 0, r, h, BA);                              \
    route_load_x<TT>(BA, xrow, min(k0 + 256, last_kb));                            \
    if (k0 + 64 < d) route_mfma_block<TT>(acc, s_w[BUF], 64, r, h, BB);            \
    route_load_x<TT>(BB, xrow, min(k0 + 320, last_kb));                            \
    _Pragma("unroll") for (int t = 0; t < TT; ++t)                                 \
      _Pragma("unroll") for (int v = 0; v < 16; ++v) total[t][v] += acc[t][v];     \
    if (more) route_store_w<NWV>(s_w[(BUF) ^ 1], wv);                                \
    __syncthreads();                                                               \
  }
  for (int c = 0; c < nchunks; c += 2) {
    MOGA_ROUTE_CHUNK(b0, b1, 0, c)
    if (c + 1 < nchunks) MOGA_ROUTE_CHUNK(b2, b3, 1, c + 1)
  }
#undef MOGA_ROUTE_CHUNK

  // Epilogue: accumulator register v of lane (r, h) is group row 8*(v/4) + 4*h + v%4 of token r.
  const bool vec4 = (M & 3) == 0 && (((uintptr_t)probs | (uintptr_t)logits) & 15) == 0;
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
      if (vec4) {   // a lane's registers 4q .. 4q+3 are four consecutive groups: one 16-byte store
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row = 8 * q + 4 * h;
          if (row < M) {
            if (probs) {
              const floatx4_t pv = {e[4 * q] * g, e[4 * q + 1] * g, e[4 * q + 2] * g, e[4 * q + 3] * g};
              *(floatx4_t*)(probs + tok * M + row) = pv;
            }
            if (logits) {
              const floatx4_t lv = {vals[4 * q], vals[4 * q + 1], vals[4 * q + 2], vals[4 * q + 3]};
              *(floatx4_t*)(logits + tok * M + row) = lv;
            }
          }
        }
      } else {
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

// dX for M <= 32 and d a multiple of 4: a thread owns four adjacent columns and keeps their 32
// weights in registers; a block sweeps kDxTokens tokens in tiles of kRbTok, whose dr rows are staged
// in LDS and read back as broadcast 16-byte pieces (8 LDS reads for 128 FMAs per token).  Every
// output row leaves as 16-byte stores, 1 KB contiguous per wave.  Sums run over the groups in
// ascending order: exact fp32 FMA chains, the same for every launch.
constexpr int kDxTokens = 512;   // tokens per block

__global__ __launch_bounds__(256) void route_bwd_dx_cols_kernel(
    const float* __restrict__ w, const float* __restrict__ probs,
    const int32_t* __restrict__ group, const float* __restrict__ gate,
    const float* __restrict__ d_gate, int64_t N, int d, int M, float* __restrict__ d_x) {
  __shared__ __attribute__((aligned(16))) float s_dr[kRbTok][32];
  const int c0 = (blockIdx.y * 256 + threadIdx.x) * 4;
  const bool valid = c0 < d;
  floatx4_t wreg[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const floatx4_t z = {0.f, 0.f, 0.f, 0.f};
    wreg[j] = (valid && j < M) ? *(const floatx4_t*)(w + (int64_t)j * d + c0) : z;
  }
  const int64_t t_begin = (int64_t)blockIdx.x * kDxTokens;
  const int64_t t_end = min(N, t_begin + kDxTokens);
  for (int64_t tb = t_begin; tb < t_end; tb += kRbTok) {
    const int nt = (int)min((int64_t)kRbTok, t_end - tb);
    __syncthreads();
    for (int idx = threadIdx.x; idx < kRbTok * 32; idx += 256) {
      const int ti = idx >> 5, j = idx & 31;
      float v = 0.f;
      if (ti < nt && j < M) {
        const int64_t tok = tb + ti;
        const float coef = d_gate[tok] * gate[tok];
        const float onehot = (group[tok] == j) ? 1.f : 0.f;
        v = coef * (onehot - probs[tok * M + j]);
      }
      s_dr[ti][j] = v;
    }
    __syncthreads();
    if (valid) {
      for (int ti = 0; ti < nt; ++ti) {
        floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j4 = 0; j4 < 8; ++j4) {
          const floatx4_t r = *(const floatx4_t*)&s_dr[ti][4 * j4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const floatx4_t wv = wreg[4 * j4 + e];
            acc[0] = fmaf(r[e], wv[0], acc[0]);
            acc[1] = fmaf(r[e], wv[1], acc[1]);
            acc[2] = fmaf(r[e], wv[2], acc[2]);
            acc[3] = fmaf(r[e], wv[3], acc[3]);
          }
        }
        *(floatx4_t*)(d_x + (tb + ti) * (int64_t)d + c0) = acc;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// dW on the matrix cores (bf16 X, M <= 32, d a multiple of 256).
//
// dW^T[c, j] = sum_t X[t, c] dr[t, j] is a contraction over tokens.  A pre-pass writes dr as two
// bf16 limbs (hi + lo carries 16 mantissa bits) in the B-operand order of the 32x32x16 MFMA:
// [token block of 8][group 0..31][8 tokens], zero beyond M and beyond N.  The main kernel runs
// one wave per block: the wave owns 256 columns of X and a range of 16-token steps, streams
// [16 tokens x 256 columns] tiles of X plus the two dr limb tiles into its own LDS ring with
// direct-to-LDS loads (three stages in flight, no barriers: a wave only reads what it loaded),
// reads X^T fragments with transposed LDS reads and accumulates eight 32x32 blocks of dW^T.
// Partial sums go to partial[split][c][32] and a second kernel reduces over the splits.
// ---------------------------------------------------------------------------------------
constexpr int kDwCols = 256;                          // columns of X per wave
constexpr int kDwTok = 16;                            // tokens per stage = one MFMA contraction step
constexpr int kDwStages = 4;                          // ring slots
constexpr int kDwXBytes = kDwTok * kDwCols * 2;       // 8 KB
constexpr int kDwStageBytes = kDwXBytes + 2048;       // + dr hi, dr lo (1 KB each)
constexpr int kDwDmaPerStage = kDwXBytes / 1024 + 2;  // direct-to-LDS instructions per stage

__global__ __launch_bounds__(256) void route_bwd_dr_pack_kernel(
    const float* __restrict__ probs, const int32_t* __restrict__ group,
    const float* __restrict__ gate, const float* __restrict__ d_gate, int64_t N, int M,
    int64_t blocks8, uintx4_t* __restrict__ dr_hi, uintx4_t* __restrict__ dr_lo) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t tb = idx >> 5;
  const int j = (int)(idx & 31);
  if (tb >= blocks8) return;
  unsigned short hi[8], lo[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t tok = tb * 8 + i;
    float v = 0.f;
    if (tok < N && j < M) {
      const float coef = d_gate[tok] * gate[tok];
      const float onehot = (group[tok] == j) ? 1.f : 0.f;
      v = coef * (onehot - probs[tok * M + j]);
    }
    hi[i] = f32_to_bf16_bits(v);
    lo[i] = f32_to_bf16_bits(v - bf16_bits_to_f32(hi[i]));
  }
  const uintx4_t ph = {hi[0] | ((unsigned)hi[1] << 16), hi[2] | ((unsigned)hi[3] << 16),
                       hi[4] | ((unsigned)hi[5] << 16), hi[6] | ((unsigned)hi[7] << 16)};
  const uintx4_t pl = {lo[0] | ((unsigned)lo[1] << 16), lo[2] | ((unsigned)lo[3] << 16),
                       lo[4] | ((unsigned)lo[5] << 16), lo[6] | ((unsigned)lo[7] << 16)};
  dr_hi[idx] = ph;
  dr_lo[idx] = pl;
}

// Chunk swizzle of the X tile in LDS (rows of 512 B = 32 chunks of 16 B): chunk' = chunk ^ this.
// The four rows a transposed read touches land in four different 64-byte bank groups.
__device__ __forceinline__ int dw_swizzle(int row) { return (row & 3) << 2; }

__global__ __launch_bounds__(64) void route_bwd_dw_mfma_kernel(
    const unsigned short* __restrict__ x, const uintx4_t* __restrict__ dr_hi,
    const uintx4_t* __restrict__ dr_lo, int64_t N, int d, int nslabs, int splits,
    int64_t steps_per_split, int64_t total_steps, float* __restrict__ partial) {
  __shared__ __attribute__((aligned(1024))) unsigned char ring[kDwStages * kDwStageBytes];
  const int lane = threadIdx.x;
  const int r = lane & 31, h = lane >> 5;
  // Blocks are dealt round-robin to the 8 XCDs; consecutive blocks of one XCD take the column
  // slabs of one token split, so its dr tiles are shared through that XCD's L2.
  const int64_t k = blockIdx.x >> 3;
  const int split = (int)(k / nslabs) * 8 + (int)(blockIdx.x & 7);
  const int slab = (int)(k % nslabs);
  if (split >= splits) return;
  const int64_t s0 = (int64_t)split * steps_per_split;
  const int64_t s1 = min(total_steps, s0 + steps_per_split);
  const int nst = (int)(s1 - s0);

  floatx16_t acc[8];
#pragma unroll
  for (int cb = 0; cb < 8; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[cb][v] = 0.f;

  const unsigned lds0 = lds_addr_uniform(&ring[0]);
  // direct-to-LDS: instruction q of a stage covers token rows 2q, 2q+1 (32 chunks each)
  const int dma_row = lane >> 5, dma_pos = lane & 31;
  const unsigned short* xslab = x + (int64_t)slab * kDwCols;
  auto issue = [&](int64_t step, int slot) {
    if (step > total_steps - 1) step = total_steps - 1;   // beyond the range: valid memory, never read back
    const int64_t tok0 = step * kDwTok;
    const int last = (int)min((int64_t)(kDwTok - 1), N - 1 - tok0);
    const void* xb = uniform_ptr(xslab + tok0 * (int64_t)d);
    const unsigned base = lds0 + slot * kDwStageBytes;
#pragma unroll
    for (int q = 0; q < kDwTok / 2; ++q) {
      const int row = 2 * q + dma_row;
      const unsigned off = (unsigned)min(row, last) * (unsigned)(d * 2) + ((dma_pos ^ dw_swizzle(row)) << 4);
      lds_dma16_soff(xb, off, base + q * 1024);
    }
    const int64_t tb = step * 2 * 32;   // two 8-token blocks of 32 groups, 16 bytes each
    lds_dma16_soff(uniform_ptr(dr_hi + tb), (unsigned)lane * 16u, base + kDwXBytes);
    lds_dma16_soff(uniform_ptr(dr_lo + tb), (unsigned)lane * 16u, base + kDwXBytes + 1024);
  };

  // transposed reads: lane gets X^T[column 32*cb + lane%32][tokens 8h .. 8h+7] from rows tr_r + {0..3}
  // (and + 4), 16-byte chunk 4*cb + tr_c, element offset tr_e
  const int tr_r = 8 * h + ((lane & 15) >> 2);
  const int tr_c = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
  const int tr_e = 4 * (lane & 1);
  unsigned a_addr[8];
#pragma unroll
  for (int cb = 0; cb < 8; ++cb)
    a_addr[cb] = (unsigned)(uintptr_t)&ring[0] + tr_r * 512 + (((4 * cb + tr_c) ^ dw_swizzle(tr_r)) << 4) + tr_e * 2;
  const unsigned b_addr = (unsigned)(uintptr_t)&ring[0] + kDwXBytes + lane * 16;

#pragma unroll
  for (int t = 0; t < kDwStages - 1; ++t) issue(s0 + t, t);
  for (int s = 0; s < nst; ++s) {
    issue(s0 + s + kDwStages - 1, (s + kDwStages - 1) & (kDwStages - 1));
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kDwDmaPerStage * (kDwStages - 1)) : "memory");
    const unsigned so = (unsigned)(s & (kDwStages - 1)) * kDwStageBytes;
    const bf16x8_t bh = lds_read_b128(b_addr + so);
    const bf16x8_t bl = lds_read_b128(b_addr + so + 1024);
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
      const bf16x8_t a = concat_tr(lds_read_tr16_addr(a_addr[cb] + so), lds_read_tr16_addr(a_addr[cb] + so + 4 * 512));
      acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bh, acc[cb], 0, 0, 0);
      acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bl, acc[cb], 0, 0, 0);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may land in LDS after the block ends

  // accumulator register v of lane (r, h): column 8*(v/4) + 4*h + v%4 of the block, group r
  float* out = partial + ((int64_t)split * d + (int64_t)slab * kDwCols) * 32 + r;
#pragma unroll
  for (int cb = 0; cb < 8; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v)
      out[(int64_t)(32 * cb + 8 * (v >> 2) + 4 * h + (v & 3)) * 32] = acc[cb][v];
}

__global__ __launch_bounds__(256) void route_bwd_dw_reduce_t_kernel(
    const float* __restrict__ partial /* [splits][d][32] */, int splits, int d, int M,
    float* __restrict__ d_w) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t n = (int64_t)d * 32;
  if (i >= n) return;
  float s = 0.f;
  for (int k = 0; k < splits; ++k) s += partial[(int64_t)k * n + i];
  const int c = (int)(i >> 5), j = (int)(i & 31);
  if (j < M) d_w[(int64_t)j * d + c] = s;
}

static int route_bwd_splits(int64_t N) {
  int64_t s = (N + 2047) / 2048;
  if (s < 1) s = 1;
  if (s > 64) s = 64;
  return (int)s;
}

// Launch plan of the matrix-core dW path.
struct DwPlan {
  int nslabs, splits;
  int64_t total_steps, steps_per_split;
  size_t dr_bytes, partial_bytes;   // one dr limb array; the partial sums
};

static bool route_bwd_mfma_ok(int x_dtype, int M, int d) {
  return x_dtype == MOGA_BF16 && M <= 32 && d % kDwCols == 0;
}

static DwPlan route_bwd_plan(int64_t N, int d) {
  DwPlan p;
  p.nslabs = d / kDwCols;
  p.total_steps = (N + kDwTok - 1) / kDwTok;
  // 40 KB of LDS per one-wave block: 4 blocks per CU, 1024 on the chip; three rounds of them measured
  // best at 580k tokens (1.21 ms against 1.29 ms for two or four rounds)
  int64_t splits = 3072 / p.nslabs;
  splits = std::min<int64_t>(splits, (p.total_steps + 7) / 8);   // at least 128 tokens per split
  splits = std::max<int64_t>(1, std::min<int64_t>(splits, 256));
  p.steps_per_split = (p.total_steps + splits - 1) / splits;
  p.splits = (int)((p.total_steps + p.steps_per_split - 1) / p.steps_per_split);   // no empty split
  p.dr_bytes = (size_t)p.total_steps * 2 * 32 * 16;
  p.partial_bytes = (size_t)p.splits * (size_t)d * 32 * sizeof(float);
  return p;
}

}  // namespace moga

using namespace moga;

extern "C" size_t moga_route_bwd_ws_bytes(int64_t N, int M, int d_model) {
  // the larger of the two paths, so the size does not depend on the dtype of X
  size_t need = (size_t)route_bwd_splits(N) * (size_t)M * (size_t)d_model * sizeof(float);
  if (N > 0 && route_bwd_mfma_ok(MOGA_BF16, M, d_model)) {
    const DwPlan p = route_bwd_plan(N, d_model);
    need = std::max(need, 2 * p.dr_bytes + p.partial_bytes);
  }
  return need;
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
      // 8 waves share one staged weight chunk, one 32-token tile per wave: 16 waves per CU keep more
      // loads in flight than 4-wave blocks with two tiles per wave (5.1 against 4.7 TB/s at 580k tokens)
      const unsigned blocks = (unsigned)((N + 255) / 256);
      route_mfma_kernel<1, 8><<<blocks, 512, 0, st>>>((const unsigned short*)x, w, bias, N, d_model, M,
                                                     group, gate, probs, logits);
    } else {
      const unsigned blocks = (unsigned)((N + 127) / 128);
      route_mfma_kernel<1, 4><<<blocks, 256, 0, st>>>((const unsigned short*)x, w, bias, N, d_model, M,
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
  if (d_model > (1 << 24)) return MOGA_ERR_UNSUPPORTED;   // keeps every grid size below 2^31 blocks
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
  if (route_bwd_mfma_ok(x_dtype, M, d_model)) {
    if (!aligned16(x) || !aligned16(ws)) return MOGA_ERR_INVALID_ARG;
    const DwPlan p = route_bwd_plan(N, d_model);
    uintx4_t* dr_hi = (uintx4_t*)ws;
    uintx4_t* dr_lo = (uintx4_t*)((char*)ws + p.dr_bytes);
    float* partial = (float*)((char*)ws + 2 * p.dr_bytes);
    const int64_t blocks8 = p.total_steps * 2;
    route_bwd_dr_pack_kernel<<<(unsigned)((blocks8 * 32 + 255) / 256), 256, 0, st>>>(
        probs, group, gate, d_gate, N, M, blocks8, dr_hi, dr_lo);
    const unsigned blocks = (unsigned)((p.splits + 7) / 8 * 8 * p.nslabs);
    route_bwd_dw_mfma_kernel<<<blocks, 64, 0, st>>>((const unsigned short*)x, dr_hi, dr_lo, N, d_model,
                                                    p.nslabs, p.splits, p.steps_per_split,
                                                    p.total_steps, partial);
    route_bwd_dw_reduce_t_kernel<<<(unsigned)(((int64_t)d_model * 32 + 255) / 256), 256, 0, st>>>(
        partial, p.splits, d_model, M, d_w);
  } else {
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
  }
  if (d_x) {
    if (M <= 32 && d_model % 4 == 0 && aligned16(d_x) && aligned16(w)) {
      dim3 gx((unsigned)((N + kDxTokens - 1) / kDxTokens), (d_model + 1023) / 1024);
      route_bwd_dx_cols_kernel<<<gx, 256, 0, st>>>(w, probs, group, gate, d_gate, N, d_model, M, d_x);
    } else {
      dim3 gx((unsigned)((N + kRbTok - 1) / kRbTok), (d_model + 255) / 256);
      route_bwd_dx_kernel<<<gx, 256, 0, st>>>(w, probs, group, gate, d_gate, N, d_model, M, d_x);
    }
  }
  return launch_status();
}
