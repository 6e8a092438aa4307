// Calls the MoGA library through its C ABI alone: plain device pointers from hipMalloc, no torch.
// Runs Alg. 1 (route -> permute -> group attention -> unpermute) on a small random problem in bf16 and
// checks what can be checked without a reference: the histogram sums to N, perm is a permutation sorted
// by group, every output is finite, and a token that is alone in its group returns gate * its own V row.
// Built by build.py next to the library (paper_2510_18692_amd/c_abi_example).
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstring>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "moga.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define MOGA_CALL(x) do { int s_ = (x); if (s_ != MOGA_OK) { std::printf("%s -> %s\n", #x, moga_status_string(s_)); return 3; } } while (0)

static uint16_t to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);   // round to nearest even
  return (uint16_t)(u >> 16);
}
static float from_bf16(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

int main() {
  const int64_t N = 4096;
  const int H = 2, D = 128, d_model = 256, M = 8;
  uint64_t state = 12345;
  auto uniform = [&]() { state = state * 6364136223846793005ull + 1442695040888963407ull; return (float)((state >> 40) / 16777216.0) - 0.5f; };
  std::vector<uint16_t> x(N * d_model), q(N * H * D), k(N * H * D), v(N * H * D);
  std::vector<float> w(M * d_model);
  for (auto& e : x) e = to_bf16(3.f * uniform());
  for (auto& e : q) e = to_bf16(3.f * uniform());
  for (auto& e : k) e = to_bf16(3.f * uniform());
  for (auto& e : v) e = to_bf16(3.f * uniform());
  for (auto& e : w) e = uniform() * 0.2f;

  void *dx, *dw, *dq, *dk, *dv, *dqh, *dkh, *dvh, *doh, *dout, *ws;
  int32_t *group, *counts, *cu, *maxlen, *perm, *inv;
  float *gate, *lse;
  const size_t tensor = (size_t)N * H * D * 2;
  HIP_OK(hipMalloc(&dx, x.size() * 2)); HIP_OK(hipMalloc(&dw, w.size() * 4));
  HIP_OK(hipMalloc(&dq, tensor)); HIP_OK(hipMalloc(&dk, tensor)); HIP_OK(hipMalloc(&dv, tensor));
  HIP_OK(hipMalloc(&dqh, tensor)); HIP_OK(hipMalloc(&dkh, tensor)); HIP_OK(hipMalloc(&dvh, tensor));
  HIP_OK(hipMalloc(&doh, tensor)); HIP_OK(hipMalloc(&dout, tensor));
  HIP_OK(hipMalloc((void**)&group, N * 4)); HIP_OK(hipMalloc((void**)&gate, N * 4));
  HIP_OK(hipMalloc((void**)&counts, M * 4)); HIP_OK(hipMalloc((void**)&cu, (M + 1) * 4));
  HIP_OK(hipMalloc((void**)&maxlen, 4)); HIP_OK(hipMalloc((void**)&perm, N * 4)); HIP_OK(hipMalloc((void**)&inv, N * 4));
  HIP_OK(hipMalloc((void**)&lse, (size_t)N * H * 4));
  const size_t ws_bytes = moga_workspace_bytes(MOGA_OP_PERMUTE, N, H, D, M, d_model, MOGA_BF16);
  HIP_OK(hipMalloc(&ws, ws_bytes ? ws_bytes : 16));
  HIP_OK(hipMemcpy(dx, x.data(), x.size() * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dw, w.data(), w.size() * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dq, q.data(), tensor, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dk, k.data(), tensor, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dv, v.data(), tensor, hipMemcpyHostToDevice));

  hipStream_t st;
  HIP_OK(hipStreamCreate(&st));
  const float scale = 1.f / std::sqrt((float)D);
  MOGA_CALL(moga_route(dx, MOGA_BF16, (const float*)dw, nullptr, N, d_model, M, group, gate, nullptr, nullptr, nullptr, 0, st));
  MOGA_CALL(moga_permute(group, N, M, dq, dk, dv, MOGA_BF16, H, D, counts, cu, maxlen, perm, inv, dqh, dkh, dvh, ws, ws_bytes, st));
  MOGA_CALL(moga_group_attn_fwd(dqh, dkh, dvh, MOGA_BF16, N, H, D, cu, M, scale, doh, lse, nullptr, 0, st));
  MOGA_CALL(moga_unpermute(doh, MOGA_BF16, perm, gate, N, H, D, dout, st));
  HIP_OK(hipStreamSynchronize(st));

  std::vector<int32_t> hcounts(M), hperm(N), hgroup(N);
  std::vector<uint16_t> out(N * H * D);
  HIP_OK(hipMemcpy(hcounts.data(), counts, M * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(hperm.data(), perm, N * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(hgroup.data(), group, N * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(out.data(), dout, tensor, hipMemcpyDeviceToHost));
  int64_t total = 0;
  for (int g = 0; g < M; ++g) total += hcounts[g];
  bool ok = total == N;
  std::vector<char> seen(N, 0);
  for (int64_t j = 0; j < N && ok; ++j) {
    ok = hperm[j] >= 0 && hperm[j] < N && !seen[hperm[j]];
    if (ok) seen[hperm[j]] = 1;
    if (ok && j > 0) ok = hgroup[hperm[j - 1]] < hgroup[hperm[j]] || (hgroup[hperm[j - 1]] == hgroup[hperm[j]] && hperm[j - 1] < hperm[j]);
  }
  for (size_t i = 0; i < out.size() && ok; ++i) ok = std::isfinite(from_bf16(out[i]));
  std::printf("library version %d, group sizes:", moga_version());
  for (int g = 0; g < M; ++g) std::printf(" %d", hcounts[g]);
  std::printf("\n%s\n", ok ? "C ABI example OK" : "C ABI example FAILED");
  return ok ? 0 : 1;
}
