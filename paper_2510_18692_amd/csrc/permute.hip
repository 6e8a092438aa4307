// permute / repermute of MoGA (Alg. 1 steps 2 and 4) and their backward.
//
// Integer part: a stable counting sort of tokens by group id, without atomics deciding any
// order.  Tokens are cut into chunks, one wave per chunk:
//   1. chunk_hist  : per-chunk histogram by wave ballots, accumulated in LDS owned by the wave;
//   2. chunk_scan  : one block; per group a wave scan over the chunks gives every chunk its
//                    first slot for that group; also counts, cu_seqlens, max_seqlen;
//   3. chunk_rank  : each wave walks its chunk in token order; a token's slot is its chunk's
//                    running base for the group plus its rank among equal ids in the batch.
// Data part: 16-byte-per-lane row copies between token order [N, H, D] and head-major
// group-contiguous order [H, N, D]; the scatter back multiplies by the gate (Eq. 5).
#include <mutex>

#include "moga_common.h"

namespace moga {

// Lanes of this wave (among `valid` ones) that hold the same group id as the caller.
__device__ __forceinline__ unsigned long long match_group(int g, bool valid, int nbits) {
  unsigned long long mask = __ballot(valid);
  for (int b = 0; b < nbits; ++b) {
    const bool bit = (g >> b) & 1;
    const unsigned long long bal = __ballot(bit);
    mask &= bit ? bal : ~bal;
  }
  return mask;
}

__device__ __forceinline__ int clamp_group(int g, int M) { return g < 0 ? 0 : (g >= M ? M - 1 : g); }

__global__ __launch_bounds__(256) void chunk_hist_kernel(const int32_t* __restrict__ group,
                                                         int64_t N, int M, int nbits,
                                                         int chunk_len, int num_chunks,
                                                         int32_t* __restrict__ hist) {
  __shared__ int s_hist[4][MOGA_MAX_GROUPS];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int chunk = blockIdx.x * 4 + wave;
  volatile int* my = s_hist[wave];
  for (int j = lane; j < M; j += 64) my[j] = 0;
  if (chunk < num_chunks) {
    const int64_t t0 = (int64_t)chunk * chunk_len;
    const int64_t t1 = min(N, t0 + chunk_len);
    for (int64_t tb = t0; tb < t1; tb += 64) {
      const int64_t tok = tb + lane;
      const bool valid = tok < t1;
      const int g = valid ? clamp_group(group[tok], M) : 0;
      const unsigned long long mask = match_group(g, valid, nbits);
      const unsigned long long below = mask & ((1ull << lane) - 1ull);
      if (valid && below == 0) my[g] += __popcll(mask);  // one leader per distinct id
    }
    for (int j = lane; j < M; j += 64) hist[(int64_t)chunk * M + j] = my[j];
  }
}

// One block of 1024 threads.  hist [num_chunks][M] is overwritten with each chunk's first slot.
__global__ __launch_bounds__(1024) void chunk_scan_kernel(int32_t* __restrict__ hist,
                                                          int num_chunks, int M, int64_t N,
                                                          int32_t* __restrict__ counts,
                                                          int32_t* __restrict__ cu_seqlens,
                                                          int32_t* __restrict__ max_seqlen) {
  __shared__ int s_count[MOGA_MAX_GROUPS];
  __shared__ int s_cu[MOGA_MAX_GROUPS + 1];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int g = wave; g < M; g += 16) {
    int tot = 0;
    for (int c = lane; c < num_chunks; c += 64) tot += hist[(int64_t)c * M + g];
    tot = wave_sum_i(tot);
    if (lane == 0) s_count[g] = tot;
  }
  __syncthreads();
  if (wave == 0) {
    int running = 0, mx = 0;
    for (int g0 = 0; g0 < M; g0 += 64) {
      const int g = g0 + lane;
      const int v = g < M ? s_count[g] : 0;
      int incl = v;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += up;
      }
      if (g < M) {
        s_cu[g] = running + incl - v;
        cu_seqlens[g] = running + incl - v;
        counts[g] = v;
      }
      running += __shfl(incl, 63, kWave);
      int m = v;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) m = max(m, __shfl_xor(m, o, kWave));
      mx = max(mx, m);
    }
    if (lane == 0) {
      s_cu[M] = running;
      cu_seqlens[M] = running;
      max_seqlen[0] = mx;
    }
  }
  __syncthreads();
  for (int g = wave; g < M; g += 16) {
    int running = s_cu[g];
    for (int c0 = 0; c0 < num_chunks; c0 += 64) {
      const int c = c0 + lane;
      const int v = c < num_chunks ? hist[(int64_t)c * M + g] : 0;
      int incl = v;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += up;
      }
      if (c < num_chunks) hist[(int64_t)c * M + g] = running + incl - v;
      running += __shfl(incl, 63, kWave);
    }
  }
}

__global__ __launch_bounds__(256) void chunk_rank_kernel(const int32_t* __restrict__ group,
                                                         int64_t N, int M, int nbits,
                                                         int chunk_len, int num_chunks,
                                                         const int32_t* __restrict__ base,
                                                         int32_t* __restrict__ perm,
                                                         int32_t* __restrict__ inv_perm) {
  __shared__ int s_next[4][MOGA_MAX_GROUPS];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int chunk = blockIdx.x * 4 + wave;
  if (chunk >= num_chunks) return;  // no block-wide barrier below
  volatile int* next = s_next[wave];
  for (int j = lane; j < M; j += 64) next[j] = base[(int64_t)chunk * M + j];
  const int64_t t0 = (int64_t)chunk * chunk_len;
  const int64_t t1 = min(N, t0 + chunk_len);
  for (int64_t tb = t0; tb < t1; tb += 64) {
    const int64_t tok = tb + lane;
    const bool valid = tok < t1;
    const int g = valid ? clamp_group(group[tok], M) : 0;
    const unsigned long long mask = match_group(g, valid, nbits);
    const int rank = __popcll(mask & ((1ull << lane) - 1ull));
    int slot = 0;
    if (valid) slot = next[g] + rank;
    __builtin_amdgcn_wave_barrier();
    if (valid) {
      perm[slot] = (int32_t)tok;
      inv_perm[tok] = slot;
      if (rank == 0) next[g] += __popcll(mask);
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// ---------------------------------------------------------------------------------------
// row movers.  A (token, head) row is D*elem bytes = LPR lanes of 16 bytes.
// ---------------------------------------------------------------------------------------
constexpr int kSlotsPerBlock = 16;

struct Rows3 {
  const void* src[3];
  void* dst[3];
};

// token order -> head-major sorted order:  dst[h][j] = src[perm[j]][h]
template <int LPR>
__global__ __launch_bounds__(256) void gather_rows_kernel(Rows3 p, const int32_t* __restrict__ perm,
                                                          int64_t N, int H) {
  constexpr int RPW = 64 / LPR;  // rows per wave instruction
  constexpr int IT = kSlotsPerBlock / RPW;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int part = lane % LPR, rsub = lane / LPR;
  const int64_t j0 = (int64_t)blockIdx.x * kSlotsPerBlock;
  const uintx4_t* __restrict__ src = (const uintx4_t*)p.src[blockIdx.y];
  uintx4_t* __restrict__ dst = (uintx4_t*)p.dst[blockIdx.y];
  int64_t tok[IT];
  bool ok[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int64_t j = j0 + it * RPW + rsub;
    ok[it] = j < N;
    tok[it] = ok[it] ? perm[j] : 0;
  }
  for (int h = wave; h < H; h += 4) {
    uintx4_t v[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it)
      if (ok[it]) v[it] = src[(tok[it] * H + h) * LPR + part];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int64_t j = j0 + it * RPW + rsub;
      if (ok[it]) dst[((int64_t)h * N + j) * LPR + part] = v[it];
    }
  }
}

template <bool BF16>
__device__ __forceinline__ uintx4_t scale16(uintx4_t v, float g) {
  uintx4_t r;
  if (BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      r[i] = pack_bf16x2(bf16_lo_to_f32(v[i]) * g, bf16_hi_to_f32(v[i]) * g);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = __float_as_uint(__uint_as_float(v[i]) * g);
  }
  return r;
}

template <bool BF16>
__device__ __forceinline__ float dot16(uintx4_t a, uintx4_t b) {
  float s = 0.f;
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
  return s;
}

// head-major sorted order -> token order: dst[perm[j]][h] = gate[perm[j]] * src[h][j]
template <int LPR, bool BF16>
__global__ __launch_bounds__(256) void scatter_rows_kernel(Rows3 p, const int32_t* __restrict__ perm,
                                                           const float* __restrict__ gate,
                                                           int64_t N, int H) {
  constexpr int RPW = 64 / LPR;
  constexpr int IT = kSlotsPerBlock / RPW;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int part = lane % LPR, rsub = lane / LPR;
  const int64_t j0 = (int64_t)blockIdx.x * kSlotsPerBlock;
  const uintx4_t* __restrict__ src = (const uintx4_t*)p.src[blockIdx.y];
  uintx4_t* __restrict__ dst = (uintx4_t*)p.dst[blockIdx.y];
  int64_t tok[IT];
  float g[IT];
  bool ok[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int64_t j = j0 + it * RPW + rsub;
    ok[it] = j < N;
    tok[it] = ok[it] ? perm[j] : 0;
    g[it] = (gate && ok[it]) ? gate[tok[it]] : 1.f;
  }
  for (int h = wave; h < H; h += 4) {
    uintx4_t v[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int64_t j = j0 + it * RPW + rsub;
      if (ok[it]) v[it] = src[((int64_t)h * N + j) * LPR + part];
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      if (ok[it]) {
        uintx4_t o = gate ? scale16<BF16>(v[it], g[it]) : v[it];
        dst[(tok[it] * H + h) * LPR + part] = o;
      }
    }
  }
}

// d_oh[h][j] = gate[t] * d_o[t][h],  d_gate[t] = sum_{h,c} d_o[t][h][c] * oh[h][j][c],  t = perm[j]
template <int LPR, bool BF16>
__global__ __launch_bounds__(256) void unpermute_bwd_kernel(
    const uintx4_t* __restrict__ d_o, const uintx4_t* __restrict__ oh,
    const int32_t* __restrict__ perm, const float* __restrict__ gate, int64_t N, int H,
    uintx4_t* __restrict__ d_oh, float* __restrict__ d_gate) {
  constexpr int RPW = 64 / LPR;
  constexpr int IT = kSlotsPerBlock / RPW;
  __shared__ float s_part[4][kSlotsPerBlock];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int part = lane % LPR, rsub = lane / LPR;
  const int64_t j0 = (int64_t)blockIdx.x * kSlotsPerBlock;
  int64_t tok[IT];
  float g[IT], acc[IT];
  bool ok[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int64_t j = j0 + it * RPW + rsub;
    ok[it] = j < N;
    tok[it] = ok[it] ? perm[j] : 0;
    g[it] = ok[it] ? gate[tok[it]] : 0.f;
    acc[it] = 0.f;
  }
  for (int h = wave; h < H; h += 4) {
    uintx4_t a[IT], b[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int64_t j = j0 + it * RPW + rsub;
      if (ok[it]) {
        a[it] = d_o[(tok[it] * H + h) * LPR + part];
        b[it] = oh[((int64_t)h * N + j) * LPR + part];
      }
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int64_t j = j0 + it * RPW + rsub;
      if (ok[it]) {
        acc[it] += dot16<BF16>(a[it], b[it]);
        d_oh[((int64_t)h * N + j) * LPR + part] = scale16<BF16>(a[it], g[it]);
      }
    }
  }
  // reduce over the LPR lanes of a row, then over the four waves
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    float s = acc[it];
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, kWave);
    if (part == 0) s_part[wave][it * RPW + rsub] = s;
  }
  __syncthreads();
  if (threadIdx.x < kSlotsPerBlock) {
    const int64_t j = j0 + threadIdx.x;
    if (j < N) {
      const float s = (s_part[0][threadIdx.x] + s_part[1][threadIdx.x]) +
                      (s_part[2][threadIdx.x] + s_part[3][threadIdx.x]);
      d_gate[perm[j]] = s;
    }
  }
}

// ---------------------------------------------------------------------------------------
// Static branches (Section 3.2): gradient of a gather whose index lists a token several times,
// and the mean of the dynamic branch and two static branches fused into one scatter.
// ---------------------------------------------------------------------------------------
template <bool BF16>
__device__ __forceinline__ void add16(float (&acc)[8], uintx4_t v) {
  if (BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { acc[2 * i] += bf16_lo_to_f32(v[i]); acc[2 * i + 1] += bf16_hi_to_f32(v[i]); }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] += __uint_as_float(v[i]);
  }
}

template <bool BF16>
__device__ __forceinline__ uintx4_t pack16(const float (&acc)[8]) {
  uintx4_t r;
  if (BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = pack_bf16x2(acc[2 * i], acc[2 * i + 1]);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = __float_as_uint(acc[i]);
  }
  return r;
}

// d_src[t][h] (+)= sum over the slots j that list token t (inv_slots[inv_cu[t] .. inv_cu[t+1]),
// ascending) of d_dst[h][j]; fp32 sums in a fixed order.
template <int LPR, bool BF16>
__global__ __launch_bounds__(256) void gather_rows_bwd_kernel(
    const uintx4_t* __restrict__ d_dst, const int32_t* __restrict__ inv_cu,
    const int32_t* __restrict__ inv_slots, int64_t N, int64_t Nk, int H, int accumulate,
    uintx4_t* __restrict__ d_src) {
  constexpr int RPW = 64 / LPR;
  constexpr int IT = kSlotsPerBlock / RPW;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int part = lane % LPR, rsub = lane / LPR;
  const int64_t t0 = (int64_t)blockIdx.x * kSlotsPerBlock;
  for (int it = 0; it < IT; ++it) {
    const int64_t t = t0 + it * RPW + rsub;
    if (t >= N) continue;
    const int beg = inv_cu[t], end = inv_cu[t + 1];
    for (int h = wave; h < H; h += 4) {
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      uintx4_t* dp = d_src + (t * H + h) * LPR + part;
      if (accumulate) add16<BF16>(acc, *dp);
      for (int j = beg; j < end; ++j)
        add16<BF16>(acc, d_dst[((int64_t)h * Nk + inv_slots[j]) * LPR + part]);
      *dp = pack16<BF16>(acc);
    }
  }
}

// Gradient of a token-order tensor that fed all three branches (Q, K or V of Section 3.2's block):
//   d_src[t][h] = g_m[h][inv_m[t]] + sum over the slots j of t of g_s[h][j] + g_f[h][inv_f[t]]
// (inv_f NULL = identity).  One fp32 sum per element in this fixed order, rounded once: a single
// pass instead of a scatter followed by two accumulating gather-backwards.
template <int LPR, bool BF16>
__global__ __launch_bounds__(256) void gather3_bwd_kernel(
    const uintx4_t* __restrict__ g_m, const int32_t* __restrict__ inv_m,
    const uintx4_t* __restrict__ g_s, const int32_t* __restrict__ inv_cu,
    const int32_t* __restrict__ inv_slots, int64_t Nk, const uintx4_t* __restrict__ g_f,
    const int32_t* __restrict__ inv_f, int64_t N, int H, uintx4_t* __restrict__ d_src) {
  constexpr int RPW = 64 / LPR;
  constexpr int IT = kSlotsPerBlock / RPW;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int part = lane % LPR, rsub = lane / LPR;
  const int64_t t0 = (int64_t)blockIdx.x * kSlotsPerBlock;
  int64_t jm[IT], jf[IT];
  int beg[IT], end[IT];
  bool ok[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int64_t t = t0 + it * RPW + rsub;
    ok[it] = t < N;
    jm[it] = ok[it] ? inv_m[t] : 0;
    jf[it] = ok[it] ? (inv_f ? inv_f[t] : t) : 0;
    beg[it] = ok[it] ? inv_cu[t] : 0;
    end[it] = ok[it] ? inv_cu[t + 1] : 0;
  }
  for (int h = wave; h < H; h += 4) {
    uintx4_t vm[IT], vf[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it)
      if (ok[it]) {
        vm[it] = g_m[((int64_t)h * N + jm[it]) * LPR + part];
        vf[it] = g_f[((int64_t)h * N + jf[it]) * LPR + part];
      }
#pragma unroll
    for (int it = 0; it < IT; ++it)
      if (ok[it]) {
        const int64_t t = t0 + it * RPW + rsub;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        add16<BF16>(acc, vm[it]);
        for (int j = beg[it]; j < end[it]; ++j)
          add16<BF16>(acc, g_s[((int64_t)h * Nk + inv_slots[j]) * LPR + part]);
        add16<BF16>(acc, vf[it]);
        d_src[(t * H + h) * LPR + part] = pack16<BF16>(acc);
      }
  }
}

// o[t][h] = alpha * (gate[t] * a_m[h][inv_m[t]] + a_s[h][inv_s[t]] + a_f[h][inv_f[t]]); a NULL
// inverse list means the identity (the branch keeps token order).
template <int LPR, bool BF16>
__global__ __launch_bounds__(256) void merge3_fwd_kernel(
    const uintx4_t* __restrict__ a_m, const uintx4_t* __restrict__ a_s, const uintx4_t* __restrict__ a_f,
    const int32_t* __restrict__ inv_m, const int32_t* __restrict__ inv_s, const int32_t* __restrict__ inv_f,
    const float* __restrict__ gate, float alpha, int64_t N, int H, uintx4_t* __restrict__ o) {
  constexpr int RPW = 64 / LPR;
  constexpr int IT = kSlotsPerBlock / RPW;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int part = lane % LPR, rsub = lane / LPR;
  const int64_t t0 = (int64_t)blockIdx.x * kSlotsPerBlock;
  int64_t jm[IT], js[IT], jf[IT];
  float g[IT];
  bool ok[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int64_t t = t0 + it * RPW + rsub;
    ok[it] = t < N;
    jm[it] = ok[it] ? (inv_m ? inv_m[t] : t) : 0;
    js[it] = ok[it] ? (inv_s ? inv_s[t] : t) : 0;
    jf[it] = ok[it] ? (inv_f ? inv_f[t] : t) : 0;
    g[it] = ok[it] ? gate[t] : 0.f;
  }
  for (int h = wave; h < H; h += 4) {
    uintx4_t vm[IT], vs[IT], vf[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it)
      if (ok[it]) {
        vm[it] = a_m[((int64_t)h * N + jm[it]) * LPR + part];
        vs[it] = a_s[((int64_t)h * N + js[it]) * LPR + part];
        vf[it] = a_f[((int64_t)h * N + jf[it]) * LPR + part];
      }
#pragma unroll
    for (int it = 0; it < IT; ++it)
      if (ok[it]) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        add16<BF16>(acc, vm[it]);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= g[it];
        add16<BF16>(acc, vs[it]);
        add16<BF16>(acc, vf[it]);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= alpha;
        const int64_t t = t0 + it * RPW + rsub;
        o[(t * H + h) * LPR + part] = pack16<BF16>(acc);
      }
  }
}

// Backward of merge3_fwd: d_m[h][inv_m[t]] = alpha * gate[t] * d_o[t][h], d_s / d_f = alpha * d_o[t][h],
// d_gate[t] = alpha * sum_{h,c} d_o[t][h][c] * a_m[h][inv_m[t]][c].
template <int LPR, bool BF16>
__global__ __launch_bounds__(256) void merge3_bwd_kernel(
    const uintx4_t* __restrict__ d_o, const uintx4_t* __restrict__ a_m,
    const int32_t* __restrict__ inv_m, const int32_t* __restrict__ inv_s, const int32_t* __restrict__ inv_f,
    const float* __restrict__ gate, float alpha, int64_t N, int H, uintx4_t* __restrict__ d_m,
    uintx4_t* __restrict__ d_s, uintx4_t* __restrict__ d_f, float* __restrict__ d_gate) {
  constexpr int RPW = 64 / LPR;
  constexpr int IT = kSlotsPerBlock / RPW;
  __shared__ float s_part[4][kSlotsPerBlock];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int part = lane % LPR, rsub = lane / LPR;
  const int64_t t0 = (int64_t)blockIdx.x * kSlotsPerBlock;
  int64_t jm[IT], js[IT], jf[IT];
  float g[IT], acc[IT];
  bool ok[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int64_t t = t0 + it * RPW + rsub;
    ok[it] = t < N;
    jm[it] = ok[it] ? (inv_m ? inv_m[t] : t) : 0;
    js[it] = ok[it] ? (inv_s ? inv_s[t] : t) : 0;
    jf[it] = ok[it] ? (inv_f ? inv_f[t] : t) : 0;
    g[it] = ok[it] ? gate[t] * alpha : 0.f;
    acc[it] = 0.f;
  }
  for (int h = wave; h < H; h += 4) {
    uintx4_t a[IT], b[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it)
      if (ok[it]) {
        const int64_t t = t0 + it * RPW + rsub;
        a[it] = d_o[(t * H + h) * LPR + part];
        b[it] = a_m[((int64_t)h * N + jm[it]) * LPR + part];
      }
#pragma unroll
    for (int it = 0; it < IT; ++it)
      if (ok[it]) {
        acc[it] += dot16<BF16>(a[it], b[it]);
        d_m[((int64_t)h * N + jm[it]) * LPR + part] = scale16<BF16>(a[it], g[it]);
        const uintx4_t sc = scale16<BF16>(a[it], alpha);
        d_s[((int64_t)h * N + js[it]) * LPR + part] = sc;
        d_f[((int64_t)h * N + jf[it]) * LPR + part] = sc;
      }
  }
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    float s = acc[it];
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, kWave);
    if (part == 0) s_part[wave][it * RPW + rsub] = s;
  }
  __syncthreads();
  if (threadIdx.x < kSlotsPerBlock) {
    const int64_t t = t0 + threadIdx.x;
    if (t < N)
      d_gate[t] = alpha * ((s_part[0][threadIdx.x] + s_part[1][threadIdx.x]) +
                           (s_part[2][threadIdx.x] + s_part[3][threadIdx.x]));
  }
}

static int bits_for(int M) {
  int b = 0;
  while ((1 << b) < M) ++b;
  return b;
}

template <int LPR>
static void launch_gather(const Rows3& p, int ntensors, const int32_t* perm, int64_t N, int H,
                          hipStream_t st) {
  dim3 grid((unsigned)((N + kSlotsPerBlock - 1) / kSlotsPerBlock), ntensors);
  gather_rows_kernel<LPR><<<grid, 256, 0, st>>>(p, perm, N, H);
}

template <int LPR, bool BF16>
static void launch_scatter(const Rows3& p, int ntensors, const int32_t* perm, const float* gate,
                           int64_t N, int H, hipStream_t st) {
  dim3 grid((unsigned)((N + kSlotsPerBlock - 1) / kSlotsPerBlock), ntensors);
  scatter_rows_kernel<LPR, BF16><<<grid, 256, 0, st>>>(p, perm, gate, N, H);
}

// Returns lanes per (token, head) row, or 0 when the combination is not covered.
static int lanes_per_row(int dtype, int D) {
  if (dtype == MOGA_F32 && (D == 64 || D == 128)) return D / 4;
  if (dtype == MOGA_BF16 && D == 128) return 16;
  return 0;
}

static int check_rows_args(int dtype, int64_t N, int H, int D) {
  if (N < 0 || H < 1 || D < 1) return MOGA_ERR_INVALID_ARG;
  if (dtype != MOGA_F32 && dtype != MOGA_BF16) return MOGA_ERR_UNSUPPORTED;
  if (N >= ((int64_t)1 << 31) || lanes_per_row(dtype, D) == 0) return MOGA_ERR_UNSUPPORTED;
  return MOGA_OK;
}

}  // namespace moga

using namespace moga;

extern "C" size_t moga_permute_ws_bytes(int64_t N, int M) {
  return (size_t)perm_num_chunks(N) * (size_t)M * sizeof(int32_t);
}

// Shared body of moga_permute and moga_permute_static: `hist` holds num_chunks * M int32.
static int permute_impl(const int32_t* group, int64_t N, int M, const void* q, const void* k,
                        const void* v, int dtype, int H, int D, int32_t* counts,
                        int32_t* cu_seqlens, int32_t* max_seqlen, int32_t* perm,
                        int32_t* inv_perm, void* qh, void* kh, void* vh, int32_t* hist,
                        hipStream_t st) {
  const bool with_data = q || k || v;
  const int chunk_len = perm_chunk_len(N);
  const int num_chunks = perm_num_chunks(N);
  const int nbits = bits_for(M);
  if (num_chunks > 0)
    chunk_hist_kernel<<<(num_chunks + 3) / 4, 256, 0, st>>>(group, N, M, nbits, chunk_len,
                                                           num_chunks, hist);
  chunk_scan_kernel<<<1, 1024, 0, st>>>(hist, num_chunks, M, N, counts, cu_seqlens, max_seqlen);
  if (num_chunks > 0)
    chunk_rank_kernel<<<(num_chunks + 3) / 4, 256, 0, st>>>(group, N, M, nbits, chunk_len,
                                                           num_chunks, hist, perm, inv_perm);
  if (with_data && N > 0) {
    Rows3 p;
    p.src[0] = q; p.src[1] = k; p.src[2] = v;
    p.dst[0] = qh; p.dst[1] = kh; p.dst[2] = vh;
    switch (lanes_per_row(dtype, D)) {
      case 16: launch_gather<16>(p, 3, perm, N, H, st); break;
      case 32: launch_gather<32>(p, 3, perm, N, H, st); break;
      default: return MOGA_ERR_UNSUPPORTED;
    }
  }
  return launch_status();
}

// Host-side argument checks shared by the two permute entry points.
static int permute_check(const int32_t* group, int64_t N, int M, const void* q, const void* k,
                         const void* v, int dtype, int H, int D, const int32_t* counts,
                         const int32_t* cu_seqlens, const int32_t* max_seqlen,
                         const int32_t* perm, const int32_t* inv_perm, const void* qh,
                         const void* kh, const void* vh) {
  if (N < 0 || M < 1) return MOGA_ERR_INVALID_ARG;
  if (M > MOGA_MAX_GROUPS || N >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  const bool with_data = q || k || v;
  if (with_data) {
    const int rc = check_rows_args(dtype, N, H, D);
    if (rc != MOGA_OK) return rc;
  }
  if (!counts || !cu_seqlens || !max_seqlen) return MOGA_ERR_INVALID_ARG;
  if (N > 0) {
    if (!group || !perm || !inv_perm) return MOGA_ERR_INVALID_ARG;
    if (with_data && (!q || !k || !v || !qh || !kh || !vh)) return MOGA_ERR_INVALID_ARG;
    if (with_data && !(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(qh) &&
                       aligned16(kh) && aligned16(vh)))
      return MOGA_ERR_INVALID_ARG;
  }
  return MOGA_OK;
}

extern "C" int moga_permute(const int32_t* group, int64_t N, int M, const void* q, const void* k,
                            const void* v, int dtype, int H, int D, int32_t* counts,
                            int32_t* cu_seqlens, int32_t* max_seqlen, int32_t* perm,
                            int32_t* inv_perm, void* qh, void* kh, void* vh, void* ws,
                            size_t ws_bytes, void* stream) {
  const int rc = permute_check(group, N, M, q, k, v, dtype, H, D, counts, cu_seqlens, max_seqlen,
                               perm, inv_perm, qh, kh, vh);
  if (rc != MOGA_OK) return rc;
  const size_t need = moga_permute_ws_bytes(N, M);
  if (need > 0 && (!ws || ws_bytes < need)) return MOGA_ERR_WORKSPACE;
  return permute_impl(group, N, M, q, k, v, dtype, H, D, counts, cu_seqlens, max_seqlen, perm,
                      inv_perm, qh, kh, vh, (int32_t*)ws, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------
// moga_permute_static: the same call for callers that cannot allocate.  The per-chunk
// histograms live in a file-scope device array; every GPU holds its own copy, whose address is
// looked up once per device (the array's name is only a host-side handle, never a device
// address).  chunk_hist overwrites every entry it later reads, so nothing has to be cleared
// between calls; two calls that overlap on one GPU would share the array and race.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) int32_t scratch[MOGA_PERMUTE_STATIC_MAX_BYTES / sizeof(int32_t)];

static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static int32_t* g_scratch_ptr[kMaxDevices];  // per device, filled on the first call there

// Device address of `scratch` on the current device, or nullptr when HIP reports an error.
static int32_t* static_scratch_for_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = (int32_t*)ptr;
  }
  return g_scratch_ptr[dev];
}

extern "C" int moga_permute_static(const int32_t* group, int64_t N, int M, const void* q,
                                   const void* k, const void* v, int dtype, int H, int D,
                                   int32_t* counts, int32_t* cu_seqlens, int32_t* max_seqlen,
                                   int32_t* perm, int32_t* inv_perm, void* qh, void* kh,
                                   void* vh, void* stream) {
  const int rc = permute_check(group, N, M, q, k, v, dtype, H, D, counts, cu_seqlens, max_seqlen,
                               perm, inv_perm, qh, kh, vh);
  if (rc != MOGA_OK) return rc;
  if (moga_permute_ws_bytes(N, M) > (size_t)MOGA_PERMUTE_STATIC_MAX_BYTES)
    return MOGA_ERR_UNSUPPORTED;  // more chunk histograms than the static array holds
  int32_t* hist = static_scratch_for_current_device();
  if (!hist) return MOGA_ERR_HIP;
  return permute_impl(group, N, M, q, k, v, dtype, H, D, counts, cu_seqlens, max_seqlen, perm,
                      inv_perm, qh, kh, vh, hist, (hipStream_t)stream);
}

static int scatter_dispatch(const Rows3& p, int ntensors, int dtype, int D, const int32_t* perm,
                            const float* gate, int64_t N, int H, hipStream_t st) {
  const int lpr = lanes_per_row(dtype, D);
  if (dtype == MOGA_BF16) {
    launch_scatter<16, true>(p, ntensors, perm, gate, N, H, st);
  } else if (lpr == 16) {
    launch_scatter<16, false>(p, ntensors, perm, gate, N, H, st);
  } else {
    launch_scatter<32, false>(p, ntensors, perm, gate, N, H, st);
  }
  return launch_status();
}

extern "C" int moga_unpermute(const void* oh, int dtype, const int32_t* perm, const float* gate,
                              int64_t N, int H, int D, void* o, void* stream) {
  const int rc = check_rows_args(dtype, N, H, D);
  if (rc != MOGA_OK) return rc;
  if (N == 0) return MOGA_OK;
  if (!oh || !perm || !o) return MOGA_ERR_INVALID_ARG;
  if (!aligned16(oh) || !aligned16(o)) return MOGA_ERR_INVALID_ARG;
  Rows3 p;
  p.src[0] = oh; p.dst[0] = o;
  p.src[1] = p.src[2] = nullptr; p.dst[1] = p.dst[2] = nullptr;
  return scatter_dispatch(p, 1, dtype, D, perm, gate, N, H, (hipStream_t)stream);
}

extern "C" int moga_permute_bwd(const void* d_qh, const void* d_kh, const void* d_vh, int dtype,
                                const int32_t* perm, int64_t N, int H, int D, void* d_q,
                                void* d_k, void* d_v, void* stream) {
  const int rc = check_rows_args(dtype, N, H, D);
  if (rc != MOGA_OK) return rc;
  if (N == 0) return MOGA_OK;
  if (!d_qh || !d_kh || !d_vh || !perm || !d_q || !d_k || !d_v) return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(d_qh) && aligned16(d_kh) && aligned16(d_vh) && aligned16(d_q) &&
        aligned16(d_k) && aligned16(d_v)))
    return MOGA_ERR_INVALID_ARG;
  Rows3 p;
  p.src[0] = d_qh; p.src[1] = d_kh; p.src[2] = d_vh;
  p.dst[0] = d_q; p.dst[1] = d_k; p.dst[2] = d_v;
  return scatter_dispatch(p, 3, dtype, D, perm, nullptr, N, H, (hipStream_t)stream);
}

extern "C" int moga_unpermute_bwd(const void* d_o, const void* oh, int dtype, const int32_t* perm,
                                  const float* gate, int64_t N, int H, int D, void* d_oh,
                                  float* d_gate, void* stream) {
  const int rc = check_rows_args(dtype, N, H, D);
  if (rc != MOGA_OK) return rc;
  if (N == 0) return MOGA_OK;
  if (!d_o || !oh || !perm || !gate || !d_oh || !d_gate) return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(d_o) && aligned16(oh) && aligned16(d_oh))) return MOGA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  const unsigned blocks = (unsigned)((N + kSlotsPerBlock - 1) / kSlotsPerBlock);
  const int lpr = lanes_per_row(dtype, D);
  if (dtype == MOGA_BF16)
    unpermute_bwd_kernel<16, true><<<blocks, 256, 0, st>>>(
        (const uintx4_t*)d_o, (const uintx4_t*)oh, perm, gate, N, H, (uintx4_t*)d_oh, d_gate);
  else if (lpr == 16)
    unpermute_bwd_kernel<16, false><<<blocks, 256, 0, st>>>(
        (const uintx4_t*)d_o, (const uintx4_t*)oh, perm, gate, N, H, (uintx4_t*)d_oh, d_gate);
  else
    unpermute_bwd_kernel<32, false><<<blocks, 256, 0, st>>>(
        (const uintx4_t*)d_o, (const uintx4_t*)oh, perm, gate, N, H, (uintx4_t*)d_oh, d_gate);
  return launch_status();
}

// ---------------------------------------------------------------------------------------
// static branches
// ---------------------------------------------------------------------------------------
extern "C" int moga_gather_rows(const void* src, int dtype, const int32_t* index, int64_t Nk, int H,
                                int D, void* dst, void* stream) {
  const int bad = check_rows_args(dtype, Nk, H, D);
  if (bad) return bad;
  if (Nk == 0) return MOGA_OK;
  if (!src || !index || !dst || !aligned16(src) || !aligned16(dst)) return MOGA_ERR_INVALID_ARG;
  Rows3 p{};
  p.src[0] = src;
  p.dst[0] = dst;
  const int lpr = lanes_per_row(dtype, D);
  if (lpr == 16) launch_gather<16>(p, 1, index, Nk, H, (hipStream_t)stream);
  else launch_gather<32>(p, 1, index, Nk, H, (hipStream_t)stream);
  return launch_status();
}

extern "C" int moga_gather_rows_bwd(const void* d_dst, int dtype, const int32_t* inv_cu,
                                    const int32_t* inv_slots, int64_t N, int64_t Nk, int H, int D,
                                    int accumulate, void* d_src, void* stream) {
  const int bad = check_rows_args(dtype, N, H, D);
  if (bad) return bad;
  if (Nk < 0 || Nk >= ((int64_t)1 << 31)) return MOGA_ERR_INVALID_ARG;
  if (N == 0) return MOGA_OK;
  if (!inv_cu || !d_src || (Nk > 0 && (!d_dst || !inv_slots))) return MOGA_ERR_INVALID_ARG;
  if (!aligned16(d_dst) || !aligned16(d_src)) return MOGA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  const unsigned blocks = (unsigned)((N + kSlotsPerBlock - 1) / kSlotsPerBlock);
  const int lpr = lanes_per_row(dtype, D);
  if (dtype == MOGA_BF16)
    gather_rows_bwd_kernel<16, true><<<blocks, 256, 0, st>>>((const uintx4_t*)d_dst, inv_cu, inv_slots, N, Nk, H,
                                                             accumulate, (uintx4_t*)d_src);
  else if (lpr == 16)
    gather_rows_bwd_kernel<16, false><<<blocks, 256, 0, st>>>((const uintx4_t*)d_dst, inv_cu, inv_slots, N, Nk, H,
                                                              accumulate, (uintx4_t*)d_src);
  else
    gather_rows_bwd_kernel<32, false><<<blocks, 256, 0, st>>>((const uintx4_t*)d_dst, inv_cu, inv_slots, N, Nk, H,
                                                              accumulate, (uintx4_t*)d_src);
  return launch_status();
}

extern "C" int moga_gather3_bwd(const void* g_moga, const int32_t* inv_moga, const void* g_stga,
                                const int32_t* inv_cu, const int32_t* inv_slots, int64_t Nk,
                                const void* g_frame, const int32_t* inv_frame, int dtype, int64_t N,
                                int H, int D, void* d_src, void* stream) {
  const int bad = check_rows_args(dtype, N, H, D);
  if (bad) return bad;
  if (Nk < 0 || Nk >= ((int64_t)1 << 31)) return MOGA_ERR_INVALID_ARG;
  if (N == 0) return MOGA_OK;
  if (!g_moga || !inv_moga || !inv_cu || !g_frame || !d_src || (Nk > 0 && (!g_stga || !inv_slots)))
    return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(g_moga) && aligned16(g_stga) && aligned16(g_frame) && aligned16(d_src)))
    return MOGA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  const unsigned blocks = (unsigned)((N + kSlotsPerBlock - 1) / kSlotsPerBlock);
  const int lpr = lanes_per_row(dtype, D);
#define MOGA_GATHER3(LPR, BF)                                                                         \
  gather3_bwd_kernel<LPR, BF><<<blocks, 256, 0, st>>>((const uintx4_t*)g_moga, inv_moga,              \
                                                      (const uintx4_t*)g_stga, inv_cu, inv_slots, Nk, \
                                                      (const uintx4_t*)g_frame, inv_frame, N, H,      \
                                                      (uintx4_t*)d_src)
  if (dtype == MOGA_BF16) MOGA_GATHER3(16, true);
  else if (lpr == 16) MOGA_GATHER3(16, false);
  else MOGA_GATHER3(32, false);
#undef MOGA_GATHER3
  return launch_status();
}

extern "C" int moga_merge3_fwd(const void* a_moga, const void* a_stga, const void* a_frame, int dtype,
                               const int32_t* inv_moga, const int32_t* inv_stga, const int32_t* inv_frame,
                               const float* gate, int64_t N, int H, int D, void* o, void* stream) {
  const int bad = check_rows_args(dtype, N, H, D);
  if (bad) return bad;
  if (N == 0) return MOGA_OK;
  if (!a_moga || !a_stga || !a_frame || !gate || !o) return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(a_moga) && aligned16(a_stga) && aligned16(a_frame) && aligned16(o))) return MOGA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  const unsigned blocks = (unsigned)((N + kSlotsPerBlock - 1) / kSlotsPerBlock);
  const float alpha = 1.f / 3.f;
  const int lpr = lanes_per_row(dtype, D);
#define MOGA_MERGE_FWD(LPR, BF)                                                                          \
  merge3_fwd_kernel<LPR, BF><<<blocks, 256, 0, st>>>((const uintx4_t*)a_moga, (const uintx4_t*)a_stga,   \
                                                     (const uintx4_t*)a_frame, inv_moga, inv_stga,       \
                                                     inv_frame, gate, alpha, N, H, (uintx4_t*)o)
  if (dtype == MOGA_BF16) MOGA_MERGE_FWD(16, true);
  else if (lpr == 16) MOGA_MERGE_FWD(16, false);
  else MOGA_MERGE_FWD(32, false);
#undef MOGA_MERGE_FWD
  return launch_status();
}

extern "C" int moga_merge3_bwd(const void* d_o, const void* a_moga, int dtype, const int32_t* inv_moga,
                               const int32_t* inv_stga, const int32_t* inv_frame, const float* gate,
                               int64_t N, int H, int D, void* d_a_moga, void* d_a_stga, void* d_a_frame,
                               float* d_gate, void* stream) {
  const int bad = check_rows_args(dtype, N, H, D);
  if (bad) return bad;
  if (N == 0) return MOGA_OK;
  if (!d_o || !a_moga || !gate || !d_a_moga || !d_a_stga || !d_a_frame || !d_gate) return MOGA_ERR_INVALID_ARG;
  if (!(aligned16(d_o) && aligned16(a_moga) && aligned16(d_a_moga) && aligned16(d_a_stga) && aligned16(d_a_frame)))
    return MOGA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  const unsigned blocks = (unsigned)((N + kSlotsPerBlock - 1) / kSlotsPerBlock);
  const float alpha = 1.f / 3.f;
  const int lpr = lanes_per_row(dtype, D);
#define MOGA_MERGE_BWD(LPR, BF)                                                                          \
  merge3_bwd_kernel<LPR, BF><<<blocks, 256, 0, st>>>((const uintx4_t*)d_o, (const uintx4_t*)a_moga,      \
                                                     inv_moga, inv_stga, inv_frame, gate, alpha, N, H,   \
                                                     (uintx4_t*)d_a_moga, (uintx4_t*)d_a_stga,           \
                                                     (uintx4_t*)d_a_frame, d_gate)
  if (dtype == MOGA_BF16) MOGA_MERGE_BWD(16, true);
  else if (lpr == 16) MOGA_MERGE_BWD(16, false);
  else MOGA_MERGE_BWD(32, false);
#undef MOGA_MERGE_BWD
  return launch_status();
}
