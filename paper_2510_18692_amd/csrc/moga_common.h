// Shared device helpers and host-side launch checks for the gfx950 MoGA kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moga.h"

namespace moga {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));
typedef unsigned int uintx2_t __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4_t __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// fp32 <-> bf16 (round to nearest even), packed two at a time (one v_cvt_pk_bf16_f32).
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi) {
  floatx2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(unsigned int, b);
}
__device__ __forceinline__ float bf16_lo_to_f32(unsigned int packed) {
  return __uint_as_float(packed << 16);
}
__device__ __forceinline__ float bf16_hi_to_f32(unsigned int packed) {
  return __uint_as_float(packed & 0xffff0000u);
}
__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) {
  return __uint_as_float(((unsigned int)b) << 16);
}
__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f) {
  return (unsigned short)(pack_bf16x2(f, 0.f) & 0xffffu);
}

// Butterfly reductions over the 64 lanes of a wave.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Value held by the lane 32 away (the other half of the wave).
__device__ __forceinline__ float other_half(float v) { return __shfl_xor(v, 32, kWave); }
__device__ __forceinline__ int other_half_i(int v) { return __shfl_xor(v, 32, kWave); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Zero fill as a kernel (a memset node inside a captured graph is avoided on purpose).
[[maybe_unused]] static __global__ void fill_zero_kernel(float* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

// ---- host side ------------------------------------------------------------
// true when groups of mean size rows / groups should run on the small-group bf16 attention kernels
bool use_small_group_kernels(int64_t rows, int groups, int64_t default_threshold);
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int launch_status() { return hipGetLastError() == hipSuccess ? MOGA_OK : MOGA_ERR_HIP; }
inline size_t round_up(size_t a, size_t b) { return (a + b - 1) / b * b; }
inline size_t elem_size(int dtype) { return dtype == MOGA_F32 ? 4 : 2; }

// Number of wave-sized token chunks the permutation uses for N tokens, and their length.
inline int perm_chunk_len(int64_t N) {
  int64_t len = 512;
  while ((N + len - 1) / len > 8192) len *= 2;
  return (int)len;
}
inline int perm_num_chunks(int64_t N) {
  int len = perm_chunk_len(N);
  return (int)((N + len - 1) / len);
}

}  // namespace moga
