// Two microbenchmarks that measure what this GPU delivers, built into libmoga_bench.so (not part
// of libmoga.so and not declared in moga.h): bench.py times them with HIP events and reports the
// results next to the published peaks as a second denominator.
//   moga_bench_mfma_loop : every wave issues 32x32x16 bf16 MFMAs whose operands and accumulators
//                          never leave the registers (no LDS, no memory): the matrix-core rate the
//                          chip sustains under its own power and clock management.
//   moga_bench_copy      : a plain device-to-device copy, 16 bytes per lane: the HBM rate a
//                          streaming kernel can reach.
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
