// Generic pieces for kernels that stream tiles global -> LDS with direct-to-LDS loads and read
// them back as MFMA operands (plain 16-byte and transposed reads).
#pragma once

#include "moga_common.h"

namespace moga {

// Transposed LDS read: the 16 lanes of a block each point at 4 consecutive bf16; lane i gets,
// for e = 0..3, element i%4 of the 4 bf16 that lane 4e + i/4 pointed at.
__device__ __forceinline__ short4_t lds_read_tr16(const unsigned short* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (short4_t __attribute__((address_space(3)))*)(p));
}

// Direct global -> LDS load of 16 bytes per lane: the wave writes 1 KB starting at the
// wave-uniform LDS byte address `lds_wave_base`, lane i at byte 16*i.  Issued through inline
// assembly so that the compiler does not make later LDS reads of *other* buffers wait for it;
// the caller waits (s_waitcnt vmcnt(0)) and synchronises before anyone reads the target.
__device__ __forceinline__ void lds_dma16(const void* gptr, unsigned lds_wave_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_wave_base), "v"(gptr)
               : "memory");
}

// LDS byte address of a __shared__ object, made wave-uniform.
__device__ __forceinline__ unsigned lds_addr_uniform(const void* p) {
  return __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)p);
}

__device__ __forceinline__ bf16x8_t concat_tr(short4_t lo, short4_t hi) {
  typedef short short8_t __attribute__((ext_vector_type(8)));
  short8_t s = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8_t, s);
}

// s_waitcnt immediates (gfx9 encoding): vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8.
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// A pointer every lane agrees on, moved to scalar registers.
__device__ __forceinline__ const void* uniform_ptr(const void* p) {
  const uint64_t v = (uint64_t)(uintptr_t)p;
  // readfirstlane returns a signed int: go through unsigned so the low half is not sign-extended
  const uint64_t lo = (unsigned)__builtin_amdgcn_readfirstlane((unsigned)v);
  const uint64_t hi = (unsigned)__builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return (const void*)(uintptr_t)(lo | (hi << 32));
}

// Direct-to-LDS load with a wave-uniform 64-bit base (scalar registers) and a 32-bit per-lane
// byte offset.
__device__ __forceinline__ void lds_dma16_soff(const void* base, unsigned byte_off, unsigned lds_wave_base) {
  lds_wave_base = __builtin_amdgcn_readfirstlane(lds_wave_base);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_wave_base), "v"(byte_off), "s"(base)
               : "memory");
}

__device__ __forceinline__ bf16x8_t lds_read_b128(unsigned addr) {
  return *(const bf16x8_t __attribute__((address_space(3)))*)(uintptr_t)addr;
}
__device__ __forceinline__ short4_t lds_read_tr16_addr(unsigned addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4_t __attribute__((address_space(3)))*)(uintptr_t)addr);
}

}  // namespace moga
