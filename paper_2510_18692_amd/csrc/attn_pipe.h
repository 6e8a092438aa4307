// Software-pipelined bf16 forward kernel of the group attention (head_dim 128).
//
// 8 waves per block, 32 query rows per wave (256-row query tiles), two waves per SIMD.
// Keys are consumed in steps of 32.  While the matrix cores compute the scores of step s+1
// (S^T = K Q^T), the vector units exponentiate the scores of step s; while the matrix cores
// accumulate O^T += V^T P^T of step s, the vector units reduce the maximum of step s+1.
// K/V tiles of 64 keys (two steps) are streamed global -> LDS with direct-to-LDS loads into
// a ring of four buffers, two tiles ahead of their use; one block-wide barrier per tile.
#pragma once

#include "attn_common.h"

namespace moga {

constexpr int kPipeNBuf = 4;                      // LDS ring: tiles of 64 keys
constexpr int kPipeAhead = 2;                     // tiles in flight beyond the one being waited for
constexpr int kPipeTileBytes = 64 * kHeadDim * 2; // 16 KB per K (or V) tile

struct PipeLane {
  // per-lane LDS byte addresses inside buffer 0 (swizzle applied); other buffers, the second
  // 32-key half and the second 16-key MFMA step are compile-time offsets
  unsigned k_addr[8];      // K fragment for d chunk pair ks (row = permuted lane row)
  unsigned v_addr[4][2];   // transposed V read for d tile dt, rows +0 / +4
};

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// Maximum of a lane's 16 scores combined with the other wave half (all 32 keys of the step).
__device__ __forceinline__ float step_max(const floatx16_t& s) {
  float t = max3(s[0], s[1], s[2]);
  t = max3(t, s[3], s[4]);
  t = max3(t, s[5], s[6]);
  t = max3(t, s[7], s[8]);
  t = max3(t, s[9], s[10]);
  t = max3(t, s[11], s[12]);
  t = max3(t, s[13], s[14]);
  t = fmaxf(t, s[15]);
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// keys of this lane in a 32-key step: register v is key 16*(v/8) + 8*h + v%8
__device__ __forceinline__ void mask_step(floatx16_t& s, int first_key, int h, int end) {
#pragma unroll
  for (int v = 0; v < 16; ++v)
    if (first_key + 16 * (v >> 3) + 8 * h + (v & 7) >= end) s[v] = -INFINITY;
}

template <int QW>
struct PipeState {
  floatx16_t o[QW][4];
  float m[QW], l[QW], negmc[QW];   // running max (raw score units), row sum, -m*c
  float thresh[QW];                // m + tau: the max is raised only when a score exceeds this
};

template <int QW>
__device__ __forceinline__ void maybe_rescale(PipeState<QW>& st, const float (&mx)[QW], float c, float tau) {
  bool need = false;
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) need |= mx[qw] > st.thresh[qw];
  if (__any(need)) {   // wave-uniform; after the first step this is rare
#pragma unroll
    for (int qw = 0; qw < QW; ++qw) {
      const float m_new = fmaxf(st.m[qw], mx[qw]);
      const float alpha = fast_exp2((st.m[qw] - m_new) * c);
      st.m[qw] = m_new;
      st.negmc[qw] = -m_new * c;
      st.thresh[qw] = m_new + tau;
      st.l[qw] *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) st.o[qw][dt][v] *= alpha;
    }
  }
}

// One pipeline step.  koff: byte offset (ring slot + half) of the NEXT step's keys; voff: byte
// offset of the CURRENT step's values.  s_cur holds the current step's raw scores; s_next
// receives the next step's raw scores (if HAS_NEXT) and mx their maximum.
template <int QW, bool HAS_NEXT, int KOFF = 0, int VOFF = 0>
__device__ __forceinline__ void pipe_step(const PipeLane& ln, unsigned koff, unsigned voff,
                                          const bf16x8_t (&qf)[QW][8], PipeState<QW>& st,
                                          const floatx16_t (&s_cur)[QW], floatx16_t (&s_next)[QW],
                                          float (&mx)[QW], float c) {
  bf16x8_t kf[8];
  if (HAS_NEXT) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kf[ks] = lds_read_b128(ln.k_addr[ks] + koff + KOFF);
  }
  bf16x8_t vf[2][4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    const unsigned a0 = ln.v_addr[dt][0] + voff + VOFF, a1 = ln.v_addr[dt][1] + voff + VOFF;
#pragma unroll
    for (int kstep = 0; kstep < 2; ++kstep)
      vf[kstep][dt] = concat_tr(lds_read_tr16_addr(a0 + kstep * 16 * 256), lds_read_tr16_addr(a1 + kstep * 16 * 256));
  }

  // P = exp2(S*c - m*c), packed to bf16; row sum from the rounded values
  typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
  const bf16x2v ones = {(__bf16)1.0f, (__bf16)1.0f};
  unsigned int pk[QW][8];
  if (HAS_NEXT) {
#pragma unroll
    for (int qw = 0; qw < QW; ++qw)
#pragma unroll
      for (int v = 0; v < 16; ++v) s_next[qw][v] = 0.f;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
#pragma unroll
    for (int qw = 0; qw < QW; ++qw) {
      if (HAS_NEXT) s_next[qw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[qw][i], s_next[qw], 0, 0, 0);
      const float p0 = fast_exp2(fmaf(s_cur[qw][2 * i], c, st.negmc[qw]));
      const float p1 = fast_exp2(fmaf(s_cur[qw][2 * i + 1], c, st.negmc[qw]));
      pk[qw][i] = pack_bf16x2(p0, p1);
      st.l[qw] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2v, pk[qw][i]), ones, st.l[qw], false);
    }
  }
  bf16x8_t pf[QW][2];
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    const uintx4_t plo = {pk[qw][0], pk[qw][1], pk[qw][2], pk[qw][3]};
    const uintx4_t phi = {pk[qw][4], pk[qw][5], pk[qw][6], pk[qw][7]};
    pf[qw][0] = __builtin_bit_cast(bf16x8_t, plo);
    pf[qw][1] = __builtin_bit_cast(bf16x8_t, phi);
  }
#pragma unroll
  for (int kstep = 0; kstep < 2; ++kstep)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int qw = 0; qw < QW; ++qw)
        st.o[qw][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kstep][dt], pf[qw][kstep], st.o[qw][dt], 0, 0, 0);
  if (HAS_NEXT) {
#pragma unroll
    for (int qw = 0; qw < QW; ++qw) mx[qw] = step_max(s_next[qw]);
  }
}

struct PipeDma {
  const void* kbase;   // first K row of this head's group (wave-uniform)
  const void* vbase;
  unsigned lds_k, lds_v;   // LDS byte address of this wave's first row in buffer 0 (wave-uniform)
  int row0;                // this lane's row inside a tile for round 0 (round i is + 4*NW*i)
  unsigned chunk_off;      // swizzled 16-byte chunk inside the row, in bytes
  int last_row;            // last valid row, relative to the group's first row
  // gather mode: rows are fetched through an index list from token-major tensors; kbase / vbase
  // then point at token 0 of this head
  const int32_t* rows;     // index list at the group's first row (wave-uniform)
  int64_t tok_stride;      // bytes between two tokens
  int wave_row;            // 4 * wave (wave-uniform)
  int last_index;          // last readable entry of `rows` (the list ends there; entries past the
                           // group's own rows belong to other groups and are harmless: those rows are masked)
  // tokens of the rows this wave moves in the next tile to be issued, rounds 0 and 1 (wave-uniform;
  // separate scalars so that they stay in scalar registers)
  int ta0, ta1, ta2, ta3, tb0, tb1, tb2, tb3;
};

// Issue the loads of the 64-key tile starting at group-relative row kv0 into ring slot `buf`:
// 16/NW rounds, each wave moving 4 rows of K and 4 rows of V per round.
template <int NW>
__device__ __forceinline__ void pipe_issue_tile(const PipeDma& d, int kv0, int buf) {
  const unsigned boff = (unsigned)buf * kPipeTileBytes;
#pragma unroll
  for (int i = 0; i < 16 / NW; ++i) {
    const int row = min(kv0 + d.row0 + 4 * NW * i, d.last_row);
    const unsigned off = (unsigned)row * (kHeadDim * 2) + d.chunk_off;
    lds_dma16_soff(d.kbase, off, d.lds_k + boff + i * 4 * NW * 256);
    lds_dma16_soff(d.vbase, off, d.lds_v + boff + i * 4 * NW * 256);
  }
}

// Gather mode: the tokens of the tile's rows were read (as scalars) while the previous tile was
// issued; select this lane's token, form the two 64-bit addresses, issue, then read the tokens of
// the following tile.
// Scalar (constant-address-space) read of one index: address and result are wave-uniform.
__device__ __forceinline__ int scalar_load_index(const int32_t* p, int i) {
  typedef const int32_t __attribute__((address_space(4))) * cptr;
  return __builtin_amdgcn_readfirstlane(((cptr)(uintptr_t)p)[i]);
}

typedef int intx4_t __attribute__((ext_vector_type(4)));

// Four consecutive indices with one 16-byte scalar load.
__device__ __forceinline__ intx4_t scalar_load_index4(const int32_t* p, int i) {
  typedef const intx4_t __attribute__((address_space(4), aligned(4))) * cptr4;
  return *(cptr4)(uintptr_t)(p + i);
}

template <int NW>
__device__ __forceinline__ void pipe_load_tokens(PipeDma& d, int kv0) {
  const int r0 = kv0 + d.wave_row;
  if (NW == 8 && r0 + 35 <= d.last_index) {   // the common case: two 16-byte scalar loads, no clamping
    const intx4_t a = scalar_load_index4(d.rows, r0), b = scalar_load_index4(d.rows, r0 + 32);
    d.ta0 = __builtin_amdgcn_readfirstlane(a[0]);
    d.ta1 = __builtin_amdgcn_readfirstlane(a[1]);
    d.ta2 = __builtin_amdgcn_readfirstlane(a[2]);
    d.ta3 = __builtin_amdgcn_readfirstlane(a[3]);
    d.tb0 = __builtin_amdgcn_readfirstlane(b[0]);
    d.tb1 = __builtin_amdgcn_readfirstlane(b[1]);
    d.tb2 = __builtin_amdgcn_readfirstlane(b[2]);
    d.tb3 = __builtin_amdgcn_readfirstlane(b[3]);
    return;
  }
  d.ta0 = scalar_load_index(d.rows, min(r0 + 0, d.last_row));
  d.ta1 = scalar_load_index(d.rows, min(r0 + 1, d.last_row));
  d.ta2 = scalar_load_index(d.rows, min(r0 + 2, d.last_row));
  d.ta3 = scalar_load_index(d.rows, min(r0 + 3, d.last_row));
  if (NW == 8) {
    d.tb0 = scalar_load_index(d.rows, min(r0 + 32, d.last_row));
    d.tb1 = scalar_load_index(d.rows, min(r0 + 33, d.last_row));
    d.tb2 = scalar_load_index(d.rows, min(r0 + 34, d.last_row));
    d.tb3 = scalar_load_index(d.rows, min(r0 + 35, d.last_row));
  }
}

__device__ __forceinline__ int select4(int sub, int a, int b, int c, int e) {
  int t = a;
  t = sub == 1 ? b : t;
  t = sub == 2 ? c : t;
  t = sub == 3 ? e : t;
  return t;
}

template <int NW>
__device__ __forceinline__ void pipe_issue_tile_gather(PipeDma& d, int kv0, int buf) {
  static_assert(NW == 8, "gather mode moves two rounds of four rows per wave");
  const unsigned boff = (unsigned)buf * kPipeTileBytes;
  const int sub = d.row0 & 3;
  const int64_t off_a = (int64_t)select4(sub, d.ta0, d.ta1, d.ta2, d.ta3) * d.tok_stride + d.chunk_off;
  const int64_t off_b = (int64_t)select4(sub, d.tb0, d.tb1, d.tb2, d.tb3) * d.tok_stride + d.chunk_off;
  lds_dma16((const char*)d.kbase + off_a, d.lds_k + boff);
  lds_dma16((const char*)d.vbase + off_a, d.lds_v + boff);
  lds_dma16((const char*)d.kbase + off_b, d.lds_k + boff + 4 * NW * 256);
  lds_dma16((const char*)d.vbase + off_b, d.lds_v + boff + 4 * NW * 256);
  pipe_load_tokens<NW>(d, kv0 + 64);
}

template <int NW, bool GATHER>
__device__ __forceinline__ void pipe_issue(PipeDma& d, int kv0, int buf) {
  if constexpr (GATHER) pipe_issue_tile_gather<NW>(d, kv0, buf);
  else pipe_issue_tile<NW>(d, kv0, buf);
}

// Queries are the rows cu_q[g] .. cu_q[g+1] of qh [H, Nq, 128]; their keys and values the rows
// cu_k[g] .. cu_k[g+1] of kh, vh [H, Nk, 128] (cu_k == cu_q and Nk == Nq for MoGA's groups).
// tile_start: NULL (tile lookup from cu_q inside the block, M <= MOGA_MAX_GROUPS) or the
// pre-summed first-tile index of every group.
//
// GATHER: qh, kh, vh and oh are token-major [N, H, 128]; row j of a group is token perm[j] (the
// permutation of Alg. 1 is applied while loading, nothing is materialised) and the output row is
// multiplied by gate[token] (Eq. 5) and written to its token.  lse stays in sorted order [H, N].
template <int NW, int QW, bool GATHER = false>
__global__ __launch_bounds__(NW * 64) void attn_fwd_bf16_pipe_kernel(
    const unsigned short* __restrict__ qh, const unsigned short* __restrict__ kh,
    const unsigned short* __restrict__ vh, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_k, const int32_t* __restrict__ tile_start, int M,
    int64_t Nq, int64_t Nk, int H, float scale, int tiles_per_head, unsigned short* __restrict__ oh,
    float* __restrict__ lse, const int32_t* __restrict__ perm = nullptr,
    const float* __restrict__ gate = nullptr) {
  constexpr int BM = NW * 32 * QW;
  constexpr int kDmaPerTile = 2 * (16 / NW);   // direct-to-LDS instructions per thread per tile
  static_assert(NW == 4 || NW == 8, "4 or 8 waves");
  __shared__ __attribute__((aligned(1024))) unsigned short Ks[kPipeNBuf][64 * kHeadDim];
  __shared__ __attribute__((aligned(1024))) unsigned short Vs[kPipeNBuf][64 * kHeadDim];
  __shared__ int s_start[MOGA_MAX_GROUPS + 1];
  __shared__ int s_found;

  const int64_t total = (int64_t)H * tiles_per_head;
  const int64_t work = xcd_work_index(blockIdx.x, total);
  if (work >= total) return;
  const int head = (int)(work / tiles_per_head);
  const int tile = (int)(work - (int64_t)head * tiles_per_head);
  TileInfo ti;
  if (tile_start) {
    if (!find_tile_presummed(tile_start, cu_q, M, BM, tile, ti)) return;
  } else if (!find_tile(cu_q, M, BM, tile, s_start, &s_found, ti)) {
    return;
  }
  const int ge = ti.row_end, q0 = ti.tile_row;   // query rows of the group end at ge
  const int gs = cu_k[ti.group];                 // first key row of the group
  const int n = cu_k[ti.group + 1] - gs;         // number of keys

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int r = lane & 31, h = lane >> 5;
  const int64_t head_off = (int64_t)head * Nq;
  const int64_t head_off_k = (int64_t)head * Nk;
  const float c = scale * 1.4426950408889634f;
  const float tau = 8.f / c;

  if (n <= 0) {   // queries without keys: zero output, lse = -inf (block-uniform branch)
#pragma unroll
    for (int qw = 0; qw < QW; ++qw) {
      const int qrow = q0 + (wave * QW + qw) * 32 + r;
      if (qrow < ge) {
        const int64_t orow = GATHER ? (int64_t)perm[qrow] * H + head : head_off + qrow;
        uintx4_t* op = (uintx4_t*)(oh + orow * kHeadDim + 64 * h);
        const uintx4_t z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 8; ++i) op[i] = z;
        if (h == 0) lse[head_off + qrow] = -INFINITY;
      }
    }
    return;
  }

  // ---- Q fragments (B operand): lane (r, h) holds Q[q = r][d = 16*ks + 8*h + 0..7]
  bf16x8_t qf[QW][8];
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    int qrow = q0 + (wave * QW + qw) * 32 + r;
    if (qrow > ge - 1) qrow = ge - 1;
    const int64_t irow = GATHER ? (int64_t)perm[qrow] * H + head : head_off + qrow;
    const unsigned short* qp = qh + irow * kHeadDim + 8 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[qw][ks] = *(const bf16x8_t*)(qp + 16 * ks);
  }

  // ---- direct-to-LDS loads: first kPipeAhead + 1 tiles (always issued; rows are clamped)
  PipeDma dma;
  dma.kbase = uniform_ptr(GATHER ? kh + (int64_t)head * kHeadDim : kh + (head_off_k + gs) * kHeadDim);
  dma.vbase = uniform_ptr(GATHER ? vh + (int64_t)head * kHeadDim : vh + (head_off_k + gs) * kHeadDim);
  dma.lds_k = lds_addr_uniform(&Ks[0][0]) + wave * 1024;
  dma.lds_v = lds_addr_uniform(&Vs[0][0]) + wave * 1024;
  dma.row0 = 4 * wave + (lane >> 4);
  dma.chunk_off = (unsigned)(((lane & 15) ^ lds_swizzle(dma.row0)) * 16);
  dma.last_row = n - 1;
  if constexpr (GATHER) {
    dma.rows = (const int32_t*)uniform_ptr(perm + gs);
    dma.tok_stride = (int64_t)H * kHeadDim * 2;
    dma.wave_row = 4 * wave;
    dma.last_index = (int)(Nk - 1) - gs;
    pipe_load_tokens<NW>(dma, 0);
  }
#pragma unroll
  for (int t = 0; t <= kPipeAhead; ++t) pipe_issue<NW, GATHER>(dma, 64 * t, t);

  // ---- per-lane LDS read addresses
  PipeLane ln;
  {
    const int krow_a = swap_bits_2_3(r);
    const int k_sw = lds_swizzle(krow_a);
    const unsigned kb = (unsigned)(uintptr_t)&Ks[0][0] + krow_a * 256;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) ln.k_addr[ks] = kb + (((2 * ks + h) ^ k_sw) << 4);
    const int tr_r = 8 * h + ((lane & 15) >> 2);
    const int tr_c = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
    const int tr_e = 4 * (lane & 1);
    const unsigned vb = (unsigned)(uintptr_t)&Vs[0][0] + tr_e * 2;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      ln.v_addr[dt][0] = vb + tr_r * 256 + (((4 * dt + tr_c) ^ lds_swizzle(tr_r)) << 4);
      ln.v_addr[dt][1] = vb + (tr_r + 4) * 256 + (((4 * dt + tr_c) ^ lds_swizzle(tr_r + 4)) << 4);
    }
  }

  PipeState<QW> st;
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    st.m[qw] = -INFINITY;
    st.l[qw] = 0.f;
    st.negmc[qw] = 0.f;
    st.thresh[qw] = -INFINITY;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) st.o[qw][dt][v] = 0.f;
  }

  const int nsteps = (n + 31) >> 5;
  const int nfull = n >> 5;   // steps whose 32 keys are all inside the group

  // ---- prologue: scores of step 0
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * kPipeAhead));
  __syncthreads();
  if (q0 + wave * 32 * QW >= ge) {
    // Every query row of this wave lies past the end of the group (last tile of a group): it only moves
    // its share of the K/V tiles and keeps the barriers of the loops below, one for one, so that no
    // matrix or vector work is spent on padding.
    int s = 0;
    for (; s + 8 <= nfull - 1; s += 8) {
#pragma unroll
      for (int B = 0; B < 4; ++B) {
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * (kPipeAhead - 1)));
        __syncthreads();
        pipe_issue<NW, GATHER>(dma, 32 * s + 64 * (B + 1 + kPipeAhead), (B + 1 + kPipeAhead) & 3);
      }
    }
    while (s + 2 <= nfull - 1) {
      __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * (kPipeAhead - 1)));
      __syncthreads();
      pipe_issue<NW, GATHER>(dma, 32 * (s + 2) + 64 * kPipeAhead, ((s >> 1) + 1 + kPipeAhead) & 3);
      s += 2;
    }
    for (; s < nsteps; ++s) {
      if ((s & 1) == 1 && s + 1 < nsteps) {
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * (kPipeAhead - 1)));
        __syncthreads();
        pipe_issue<NW, GATHER>(dma, 32 * (s + 1) + 64 * kPipeAhead, (((s >> 1) & 3) + 1 + kPipeAhead) & 3);
      }
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    return;
  }
  floatx16_t s_a[QW], s_b[QW];   // scores of even / odd steps
  float mx[QW];
  {
    bf16x8_t kf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kf[ks] = lds_read_b128(ln.k_addr[ks]);
#pragma unroll
    for (int qw = 0; qw < QW; ++qw) {
#pragma unroll
      for (int v = 0; v < 16; ++v) s_a[qw][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        s_a[qw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[qw][ks], s_a[qw], 0, 0, 0);
      if (nfull == 0) mask_step(s_a[qw], 0, h, n);
      mx[qw] = step_max(s_a[qw]);
    }
  }

  // ---- main loop.  Tile T (64 keys, two steps) lives in ring slot T % 4.  Step 2T reads its
  // values and the next step's keys from that slot; then the block waits for tile T+1, refills
  // the slot of tile T-1 with tile T+3, and step 2T+1 reads the keys of step 2T+2 from the slot
  // of tile T+1.  Four tiles per iteration so that every LDS offset is an immediate.
  int s = 0;
#define MOGA_FWD_TILE(B)                                                                        \
  maybe_rescale<QW>(st, mx, c, tau);                                                            \
  pipe_step<QW, true, (B) * kPipeTileBytes + 8192, (B) * kPipeTileBytes>(ln, 0, 0, qf, st, s_a, s_b, mx, c); \
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * (kPipeAhead - 1)));                       \
  __syncthreads();                                                                              \
  pipe_issue<NW, GATHER>(dma, 32 * s + 64 * ((B) + 1 + kPipeAhead), ((B) + 1 + kPipeAhead) & 3); \
  maybe_rescale<QW>(st, mx, c, tau);                                                            \
  pipe_step<QW, true, (((B) + 1) & 3) * kPipeTileBytes, (B) * kPipeTileBytes + 8192>(ln, 0, 0, qf, st, s_b, s_a, mx, c);
  for (; s + 8 <= nfull - 1; s += 8) {   // steps s .. s+7 and their successors are full
    MOGA_FWD_TILE(0)
    MOGA_FWD_TILE(1)
    MOGA_FWD_TILE(2)
    MOGA_FWD_TILE(3)
  }
#undef MOGA_FWD_TILE
  // remaining whole tiles, ring offsets at run time (s / 2 is a multiple of 4 on entry)
  while (s + 2 <= nfull - 1) {
    const unsigned slot = ((unsigned)(s >> 1) & 3u) * kPipeTileBytes;
    const unsigned slot_next = ((unsigned)((s >> 1) + 1) & 3u) * kPipeTileBytes;
    maybe_rescale<QW>(st, mx, c, tau);
    pipe_step<QW, true>(ln, slot + 8192, slot, qf, st, s_a, s_b, mx, c);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * (kPipeAhead - 1)));
    __syncthreads();
    pipe_issue<NW, GATHER>(dma, 32 * (s + 2) + 64 * kPipeAhead, ((s >> 1) + 1 + kPipeAhead) & 3);
    maybe_rescale<QW>(st, mx, c, tau);
    pipe_step<QW, true>(ln, slot_next, slot + 8192, qf, st, s_b, s_a, mx, c);
    s += 2;
  }

  // ---- tail: at most three steps (s is even here), the last one possibly partial
  for (; s < nsteps; ++s) {
    const int buf = (s >> 1) & 3, half = s & 1;
    const bool has_next = s + 1 < nsteps;
    if (half == 1 && has_next) {   // the next step starts a new tile
      __builtin_amdgcn_s_waitcnt(waitcnt_vm(kDmaPerTile * (kPipeAhead - 1)));
      __syncthreads();
      pipe_issue<NW, GATHER>(dma, 32 * (s + 1) + 64 * kPipeAhead, (buf + 1 + kPipeAhead) & 3);
    }
    maybe_rescale<QW>(st, mx, c, tau);
    const unsigned voff = buf * kPipeTileBytes + half * 8192;
    const unsigned koff = (half ? ((buf + 1) & 3) : buf) * kPipeTileBytes + (half ? 0 : 8192);
    if (has_next) {
      pipe_step<QW, true>(ln, koff, voff, qf, st, s_a, s_b, mx, c);
#pragma unroll
      for (int qw = 0; qw < QW; ++qw) {
        if (s + 1 >= nfull) mask_step(s_b[qw], 32 * (s + 1), h, n);
        s_a[qw] = s_b[qw];
        if (s + 1 >= nfull) mx[qw] = step_max(s_a[qw]);
      }
    } else {
      pipe_step<QW, false>(ln, koff, voff, qf, st, s_a, s_b, mx, c);
    }
  }

  // ---- epilogue: register v of d tile dt is d = 32*dt + 8*(v/4) + 4*h + v%4 of query column r
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // drain the look-ahead loads before the LDS is released
#pragma unroll
  for (int qw = 0; qw < QW; ++qw) {
    const auto rr = __builtin_amdgcn_permlane32_swap(__float_as_uint(st.l[qw]), __float_as_uint(st.l[qw]), false, false);
    const float lt = __uint_as_float(rr[0]) + __uint_as_float(rr[1]);
    float inv = 1.f / lt;
    const int qrow = q0 + (wave * QW + qw) * 32 + r;
    if (qrow < ge) {
      int64_t orow = head_off + qrow;
      if (GATHER) {
        const int tok = perm[qrow];
        orow = (int64_t)tok * H + head;
        inv *= gate[tok];
      }
      unsigned short* op = oh + orow * kHeadDim + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          uintx2_t pk = {pack_bf16x2(st.o[qw][dt][4 * b] * inv, st.o[qw][dt][4 * b + 1] * inv),
                         pack_bf16x2(st.o[qw][dt][4 * b + 2] * inv, st.o[qw][dt][4 * b + 3] * inv)};
          *(uintx2_t*)(op + 32 * dt + 8 * b) = pk;
        }
      if (h == 0) lse[head_off + qrow] = st.m[qw] * scale + logf(lt);
    }
  }
}

}  // namespace moga
