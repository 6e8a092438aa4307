// Group balancing loss of MoGA (Eqs. 6-8 of the paper) and its gradient with respect to the gate.
//
//   F_i = (1/N) #{x : g(x) = i}                      fraction of tokens assigned to group i (Eq. 7)
//   P_i = (1/N) sum_{x : g(x) = i} p(g(x) | x)       router probability mass of those tokens (Eq. 8)
//   L   = alpha * M * sum_i F_i * P_i                (Eq. 6)
//
// The per-group sums are accumulated as integers (counts, and gates in 2^-32 fixed point), so
// the result does not depend on the order in which tokens are added: LDS atomics per block,
// then one global atomic per block and group.  A last block turns the sums into F, P and L in
// double precision.  F is piecewise constant in the router weights, so the gradient flows through
// P only: dL/d gate[x] = alpha * M * F_{g(x)} / N.
#include <algorithm>

#include "moga_common.h"

namespace moga {

constexpr double kGateFixedScale = 4294967296.0;   // 2^32

struct BalanceAcc {
  unsigned long long gate_sum;   // sum of round(gate * 2^32), two's complement
  unsigned long long count;
};

__global__ __launch_bounds__(256) void balance_accumulate_kernel(
    const int32_t* __restrict__ group, const float* __restrict__ gate, int64_t N, int M,
    BalanceAcc* __restrict__ acc) {
  __shared__ unsigned long long s_sum[MOGA_MAX_GROUPS];
  __shared__ unsigned int s_cnt[MOGA_MAX_GROUPS];
  for (int j = threadIdx.x; j < M; j += 256) { s_sum[j] = 0ull; s_cnt[j] = 0u; }
  __syncthreads();
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < N; t += stride) {
    const int g = group[t];
    if (g >= 0 && g < M) {
      const long long fx = __double2ll_rn((double)gate[t] * kGateFixedScale);
      atomicAdd(&s_sum[g], (unsigned long long)fx);
      atomicAdd(&s_cnt[g], 1u);
    }
  }
  __syncthreads();
  for (int j = threadIdx.x; j < M; j += 256) {
    if (s_cnt[j]) {
      atomicAdd(&acc[j].gate_sum, s_sum[j]);
      atomicAdd(&acc[j].count, (unsigned long long)s_cnt[j]);
    }
  }
}

__global__ __launch_bounds__(256) void balance_finalize_kernel(
    const BalanceAcc* __restrict__ acc, int64_t N, int M, float alpha, float* __restrict__ loss,
    float* __restrict__ frac, float* __restrict__ prob) {
  __shared__ double s_fp[MOGA_MAX_GROUPS];
  const double inv_n = 1.0 / (double)N;
  for (int j = threadIdx.x; j < M; j += 256) {
    const double f = (double)acc[j].count * inv_n;
    const double p = (double)(long long)acc[j].gate_sum / kGateFixedScale * inv_n;
    frac[j] = (float)f;
    prob[j] = (float)p;
    s_fp[j] = f * p;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int j = 0; j < M; ++j) s += s_fp[j];
    loss[0] = (float)((double)alpha * (double)M * s);
  }
}

__global__ __launch_bounds__(256) void balance_bwd_kernel(
    const int32_t* __restrict__ group, const float* __restrict__ frac, int64_t N, int M, float coef,
    const float* __restrict__ d_loss_dev, int accumulate, float* __restrict__ d_gate) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= N) return;
  if (d_loss_dev) coef *= d_loss_dev[0];   // upstream gradient kept on the device: no host synchronisation
  const int g = group[t];
  const float v = (g >= 0 && g < M) ? coef * frac[g] : 0.f;
  d_gate[t] = accumulate ? d_gate[t] + v : v;
}

}  // namespace moga

using namespace moga;

extern "C" size_t moga_balance_ws_bytes(int M) { return (size_t)M * sizeof(BalanceAcc); }

extern "C" int moga_balance_loss(const int32_t* group, const float* gate, int64_t N, int M,
                                 float alpha, float* loss, float* frac, float* prob, void* ws,
                                 size_t ws_bytes, void* stream) {
  if (N < 0 || M < 1) return MOGA_ERR_INVALID_ARG;
  if (M > MOGA_MAX_GROUPS || N >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  if (!loss || !frac || !prob) return MOGA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (N == 0) {   // no tokens: F = P = 0, L = 0
    fill_zero_kernel<<<1, 256, 0, st>>>(frac, M);
    fill_zero_kernel<<<1, 256, 0, st>>>(prob, M);
    fill_zero_kernel<<<1, 256, 0, st>>>(loss, 1);
    return launch_status();
  }
  if (!group || !gate) return MOGA_ERR_INVALID_ARG;
  if (!ws || ws_bytes < moga_balance_ws_bytes(M)) return MOGA_ERR_WORKSPACE;
  if (!aligned16(ws)) return MOGA_ERR_INVALID_ARG;
  BalanceAcc* acc = (BalanceAcc*)ws;
  const int64_t ws_floats = (int64_t)(moga_balance_ws_bytes(M) / sizeof(float));
  fill_zero_kernel<<<(unsigned)((ws_floats + 255) / 256), 256, 0, st>>>((float*)ws, ws_floats);
  const unsigned blocks = (unsigned)std::min<int64_t>(1024, (N + 1023) / 1024);
  balance_accumulate_kernel<<<blocks, 256, 0, st>>>(group, gate, N, M, acc);
  balance_finalize_kernel<<<1, 256, 0, st>>>(acc, N, M, alpha, loss, frac, prob);
  return launch_status();
}

extern "C" int moga_balance_loss_bwd(const int32_t* group, const float* frac, int64_t N, int M,
                                     float alpha, float d_loss, const float* d_loss_device_or_null,
                                     int accumulate, float* d_gate, void* stream) {
  if (N < 0 || M < 1) return MOGA_ERR_INVALID_ARG;
  if (M > MOGA_MAX_GROUPS || N >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  if (N == 0) return MOGA_OK;
  if (!group || !frac || !d_gate) return MOGA_ERR_INVALID_ARG;
  const float coef = (float)((double)d_loss * (double)alpha * (double)M / (double)N);
  balance_bwd_kernel<<<(unsigned)((N + 255) / 256), 256, 0, (hipStream_t)stream>>>(
      group, frac, N, M, coef, d_loss_device_or_null, accumulate, d_gate);
  return launch_status();
}
