// Two microbenchmarks that measure what this GPU delivers, built into libmoga_bench.so (not part
// of libmoga.so and not declared in moga.h): bench.py times them with HIP events and reports the
// results next to the published peaks as a second denominator.
//   moga_bench_mfma_loop : every wave issues 32x32x16 bf16 MFMAs whose operands and accumulators
//                          never leave the registers (no LDS, no memory): the matrix-core rate the
//                          chip sustains under its own power and clock management.
//   moga_bench_copy      : a plain device-to-device copy, 16 bytes per lane: the HBM rate a
//                          streaming kernel can reach.
//   moga_bench_mix_loop  : the MFMA loop with two waves per SIMD and, per MFMA, a chosen number of
//                          1 KB LDS fragment reads, fp32 fmas and exp2s on random or all-zero data.
//                          Run at the board's power limit, the rate it sustains prices each extra
//                          in units of the energy of one MFMA (python -m paper_2510_18692_amd.profiling energy).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moga_bench {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));
typedef unsigned int uintx4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned int hash32(unsigned int x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// Eight bf16 values spread over [-2, 2), different for every lane and fragment (all-equal operands
// toggle fewer wires and flatter the power budget).
__device__ __forceinline__ bf16x8_t random_fragment(unsigned int key) {
  unsigned int w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned int h = hash32(key * 4u + i);
    const floatx2_t f = {(float)(h & 0xffffu) * (4.f / 65536.f) - 2.f, (float)(h >> 16) * (4.f / 65536.f) - 2.f};
    w[i] = __builtin_bit_cast(unsigned int, __builtin_convertvector(f, bf16x2_t));
  }
  const uintx4_t u = {w[0], w[1], w[2], w[3]};
  return __builtin_bit_cast(bf16x8_t, u);
}

constexpr int kAcc = 8;   // independent accumulators per wave (128 registers)

__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* __restrict__ sink) {
  bf16x8_t a[kAcc], b[kAcc];
  floatx16_t acc[kAcc];
  const unsigned int id = blockIdx.x * 256u + threadIdx.x;
#pragma unroll
  for (int j = 0; j < kAcc; ++j) {
    a[j] = random_fragment(id * 16u + j);
    b[j] = random_fragment(id * 16u + 8u + j);
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kAcc; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + 3) & (kAcc - 1)], acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < kAcc; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[j][v];
  if (s == 12345.678f) sink[id] = s;   // keeps the loop alive; practically never taken
}

// A operands come from LDS when NL >= 1 (B operands too when NL == 2): 16 bytes per lane, a different
// conflict-free 1 KB row each time, loaded six MFMAs before their use.  NF fmas and NE exp2s per MFMA keep
// 16 values per lane bounded.  zero != 0 clears every operand (same instruction stream, no toggling).
template <int NL, int NF, int NE>
__global__ __launch_bounds__(512) void mix_loop_kernel(int iters, int zero, float* __restrict__ sink) {
  __shared__ uintx4_t rows[4096];   // 64 rows of 1 KB
  const unsigned int id = blockIdx.x * 512u + threadIdx.x;
  for (int i = threadIdx.x; i < 4096; i += 512)
    rows[i] = zero ? uintx4_t{0u, 0u, 0u, 0u} : __builtin_bit_cast(uintx4_t, random_fragment(0x40000000u + i));
  __syncthreads();
  bf16x8_t a[kAcc], b[kAcc];
  floatx16_t acc[4];
#pragma unroll
  for (int j = 0; j < kAcc; ++j) {
    a[j] = random_fragment(id * 16u + j);
    b[j] = random_fragment(id * 16u + 8u + j);
    if (zero) { a[j] = __builtin_bit_cast(bf16x8_t, uintx4_t{0u, 0u, 0u, 0u}); b[j] = a[j]; }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
  float x[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) x[j] = zero ? 0.f : (float)(hash32(id * 16u + j) & 0xffffu) * (1.f / 65536.f) - 0.5f;
  const float fa = zero ? 0.f : -0.9990234f, fb = zero ? 0.f : 0.37f;
  const unsigned int lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < kAcc; ++m) {
      acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m], b[(m + 3) & (kAcc - 1)], acc[m & 3], 0, 0, 0);
#pragma unroll
      for (int t = 0; t < NL; ++t) {
        const unsigned int row = (unsigned int)(it * kAcc * NL + m * NL + t + wave * 7) & 63u;
        const bf16x8_t f = __builtin_bit_cast(bf16x8_t, rows[row * 64u + lane]);
        if (t == 0) a[(m + 6) & (kAcc - 1)] = f; else b[(m + 1) & (kAcc - 1)] = f;
      }
#pragma unroll
      for (int t = 0; t < NF; ++t) x[(m * NF + t) & 15] = __builtin_fmaf(x[(m * NF + t) & 15], fa, fb);
#pragma unroll
      for (int t = 0; t < NE; ++t) x[(m * NE + t + 7) & 15] = __builtin_amdgcn_exp2f(x[(m * NE + t + 7) & 15]) - 1.f;
    }
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    s += x[j];
#pragma unroll
    for (int q = 0; q < 4; ++q) s += acc[q][j];
  }
  if (s == 12345.678f) sink[id] = s;   // keeps the loop alive; practically never taken
}

__global__ __launch_bounds__(256) void copy_kernel(uintx4_t* __restrict__ dst, const uintx4_t* __restrict__ src,
                                                   int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * 256 * 4;
  for (int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x; i < n16; i += stride) {
    uintx4_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (i + 256 * k < n16) v[k] = src[i + 256 * k];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (i + 256 * k < n16) dst[i + 256 * k] = v[k];
  }
}

}  // namespace moga_bench

using namespace moga_bench;

// Launches `blocks` blocks of 4 waves, each wave issuing iters * 8 MFMAs; returns the FLOPs of the
// launch (2 * 32 * 32 * 16 per MFMA) or -1 on a bad argument / failed launch.  sink: device, >= blocks * 256 floats.
extern "C" double moga_bench_mfma_loop(int blocks, int iters, float* sink, void* stream) {
  if (blocks < 1 || iters < 1 || !sink) return -1.0;
  mfma_loop_kernel<<<blocks, 256, 0, (hipStream_t)stream>>>(iters, sink);
  if (hipGetLastError() != hipSuccess) return -1.0;
  return (double)blocks * 4.0 * (double)iters * kAcc * 32768.0;
}

// One launch of the mixed loop: `blocks` blocks of 8 waves (two per SIMD), each wave issuing iters * 8 MFMAs
// plus, per MFMA, lds_reads (0..2) fragment reads, fmas (0, 2, 4 or 6) and exps (0..2); the combinations
// built are the ones listed below.  Returns the MFMA FLOPs of the launch, or -1 for a bad argument, a
// combination that is not built, or a failed launch.  sink: device, >= blocks * 512 floats.
extern "C" double moga_bench_mix_loop(int lds_reads, int fmas, int exps, int blocks, int iters, int zero, float* sink,
                                      void* stream) {
  if (blocks < 1 || iters < 1 || !sink) return -1.0;
  hipStream_t st = (hipStream_t)stream;
  const int key = lds_reads * 100 + fmas * 10 + exps;
#define MOGA_MIX(NL, NF, NE) \
  case NL * 100 + NF * 10 + NE: mix_loop_kernel<NL, NF, NE><<<blocks, 512, 0, st>>>(iters, zero, sink); break;
  switch (key) {
    MOGA_MIX(0, 0, 0) MOGA_MIX(1, 0, 0) MOGA_MIX(2, 0, 0)
    MOGA_MIX(0, 2, 0) MOGA_MIX(0, 4, 0) MOGA_MIX(0, 6, 0)
    MOGA_MIX(0, 0, 1) MOGA_MIX(0, 0, 2)
    MOGA_MIX(1, 4, 1)
    default: return -1.0;
  }
#undef MOGA_MIX
  if (hipGetLastError() != hipSuccess) return -1.0;
  return (double)blocks * 8.0 * (double)iters * kAcc * 32768.0;
}

// Copies `bytes` (a multiple of 16, both pointers 16-byte aligned) from src to dst; returns the bytes
// moved over HBM (read + written) or -1.
extern "C" double moga_bench_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes == 0 || (bytes & 15u) || ((uintptr_t)dst & 15u) || ((uintptr_t)src & 15u)) return -1.0;
  const int64_t n16 = (int64_t)(bytes / 16);
  const int64_t want = (n16 + 1023) / 1024;
  const unsigned grid = (unsigned)(want < 256 * 64 ? want : 256 * 64);
  copy_kernel<<<grid, 256, 0, (hipStream_t)stream>>>((uintx4_t*)dst, (const uintx4_t*)src, n16);
  if (hipGetLastError() != hipSuccess) return -1.0;
  return 2.0 * (double)bytes;
}
