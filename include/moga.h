/*
 * moga.h -- C ABI of the MI355X (gfx950) Mixture-of-Groups Attention library.
 *
 * The calls follow the MoGA paper (arXiv 2510.18692): Alg. 1 is
 *     g = router(X);  Q^,K^,V^,cu_seqlen,max_seqlen,permute_index = permute(Q,K,V,g);
 *     O^ = varlen_attention(Q^,K^,V^,cu_seqlen);  O = repermute(O^, permute_index)
 * with the router of Eqs. 2-4 (one linear layer, softmax, top-1) and the output of
 * Eq. 5 (the attention result of a token is multiplied by its router probability).
 * The *_bwd calls are the derivative of Eq. 5 with the assignment g held constant.
 *
 * Conventions shared by every call
 *   - Every pointer argument except `stream` is a DEVICE pointer owned by the caller;
 *     tensors must be 16-byte aligned and must not alias each other.  The library
 *     allocates nothing, keeps no state between calls, and uses only the caller's
 *     workspace `ws` (size from moga_workspace_bytes; NULL allowed when that size is 0).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work: they never synchronise the host, and outputs are valid in stream order.
 *   - Return value is a moga_status.  No exceptions, no abort, no printing.  Arguments are
 *     validated on the host before anything is launched; N == 0 is a successful no-op.
 *   - Notation: N tokens (batch 1), d_model router input width, M groups, H heads,
 *     D head_dim.  Token-order tensors are [N, H, D] row-major; group-contiguous
 *     ("hat") tensors are head-major [H, N, D], row j of a head being sorted slot j.
 *   - Supported: M in [1, 256]; N < 2^31 (N < 2^24 for the BF16 attention calls, whose kernels
 *     address the rows of a group with 32-bit byte offsets); dtype F32 with D in {64, 128} and
 *     dtype BF16 with D = 128.  Anything else returns MOGA_ERR_UNSUPPORTED.
 */
#ifndef MOGA_H_
#define MOGA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOGA_MAX_GROUPS 256          /* router groups M */
#define MOGA_MAX_SEGMENTS (1 << 24)  /* static groups G of the moga_varlen_* calls */

typedef enum {
  MOGA_OK = 0,
  MOGA_ERR_INVALID_ARG = -1, /* NULL required pointer, negative size, misaligned pointer, bad scale */
  MOGA_ERR_UNSUPPORTED = -2, /* shape / dtype combination the kernels do not cover */
  MOGA_ERR_WORKSPACE = -3,   /* ws is NULL or smaller than moga_workspace_bytes says */
  MOGA_ERR_HIP = -4          /* a kernel launch failed (hipGetLastError) */
} moga_status;

typedef enum { MOGA_F32 = 0, MOGA_BF16 = 1 } moga_dtype;

typedef enum {
  MOGA_OP_ROUTE = 0,
  MOGA_OP_PERMUTE = 1,
  MOGA_OP_ATTN_FWD = 2,
  MOGA_OP_ATTN_BWD = 3,
  MOGA_OP_ROUTE_BWD = 4,
  MOGA_OP_BALANCE_LOSS = 5,
  MOGA_OP_VARLEN_ATTN_FWD = 6, /* N = Nq, M = G */
  MOGA_OP_VARLEN_ATTN_BWD = 7  /* N = Nq, M = G */
} moga_op;

/* Human-readable name of a status code (static storage, never NULL). */
const char* moga_status_string(int status);
/* Library version, major*10000 + minor*100 + patch. */
int moga_version(void);

/* Bytes of device workspace the given call needs for these sizes (0 if none). Host-only. */
size_t moga_workspace_bytes(int op, int64_t N, int H, int D, int M, int d_model, int dtype);

/*
 * Router, Eqs. 2-4, plus the gate that Eq. 5 multiplies by.
 *   logits[i][j] = sum_c x[i][c] * w[j][c] (+ bias[j])      fp32-GEMM semantics
 *   group[i]     = argmax_j logits[i][j], lowest j on ties   (Eq. 4; softmax is monotone)
 *   probs[i][j]  = softmax_j(logits[i])                      (Eq. 3)
 *   gate[i]      = probs[i][group[i]]
 * x [N, d_model] of x_dtype; w [M, d_model] fp32; bias [M] fp32 or NULL.
 * Outputs: group [N] int32, gate [N] fp32; probs [N, M] fp32 (NULL to skip; the backward
 * needs it); logits [N, M] fp32 (NULL to skip).  One group and one gate per token,
 * shared by all heads (Section 3.2).
 */
int moga_route(const void* x, int x_dtype, const float* w, const float* bias_or_null,
               int64_t N, int d_model, int M,
               int32_t* group, float* gate, float* probs_or_null, float* logits_or_null,
               void* ws, size_t ws_bytes, void* stream);

/*
 * permute of Alg. 1: histogram, exclusive prefix sum, stable counting-sort permutation,
 * and the gather of Q, K, V into group-contiguous head-major layout.
 *   counts[g]      = #{i : group[i] == g}                       [M]
 *   cu_seqlens     = exclusive prefix sum of counts, cu[M] = N   [M + 1]
 *   max_seqlen     = max_g counts[g]                             [1]
 *   perm[j]        = token in sorted slot j; keys (group, token index) ascending   [N]
 *   inv_perm[i]    = slot of token i                             [N]
 *   qh[h][j][:]    = q[perm[j]][h][:]   (same for k, v)
 * group ids outside [0, M) are clamped into range.  q, k, v may all be NULL to compute
 * only the integer outputs (then qh, kh, vh are ignored).  All int32 outputs stay on the device.
 */
int moga_permute(const int32_t* group, int64_t N, int M,
                 const void* q, const void* k, const void* v, int dtype, int H, int D,
                 int32_t* counts, int32_t* cu_seqlens, int32_t* max_seqlen,
                 int32_t* perm, int32_t* inv_perm,
                 void* qh, void* kh, void* vh,
                 void* ws, size_t ws_bytes, void* stream);

/*
 * moga_permute for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * (minus ws), same kernels and bit-identical outputs; the per-chunk histograms live in a static
 * device array of MOGA_PERMUTE_STATIC_MAX_BYTES that each GPU the library runs on holds until
 * the process ends.  The call allocates nothing.  Sizes whose chunk histograms
 * (moga_workspace_bytes(MOGA_OP_PERMUTE, N, .., M, ..)) exceed that limit return
 * MOGA_ERR_UNSUPPORTED: with at most 8192 chunks, every N < 2^31 fits for M <= 64.  All calls
 * on one GPU share the array: calls that overlap on one GPU (two streams, two threads) race;
 * calls in stream order on one stream do not.
 */
#define MOGA_PERMUTE_STATIC_MAX_BYTES (2u << 20)
int moga_permute_static(const int32_t* group, int64_t N, int M,
                        const void* q, const void* k, const void* v, int dtype, int H, int D,
                        int32_t* counts, int32_t* cu_seqlens, int32_t* max_seqlen,
                        int32_t* perm, int32_t* inv_perm,
                        void* qh, void* kh, void* vh, void* stream);

/*
 * Variable-length attention of Alg. 1 step 3: Eq. 1 applied independently inside each
 * group and head, bidirectional:
 *   oh[h][j] = softmax_k(softmax_scale * qh[h][j] . kh[h][k]) vh[h][k],  k over j's group
 *   lse[h][j] = log sum_k exp(softmax_scale * qh[h][j] . kh[h][k])      [H, N] fp32
 * Groups are the row ranges cu_seqlens[g]..cu_seqlens[g+1] (device, [M + 1]); empty groups
 * do nothing.  softmax_scale must be finite and > 0.  BF16: bf16 MFMA inputs, fp32
 * accumulation and softmax statistics; F32: fp32 throughout.
 */
int moga_group_attn_fwd(const void* qh, const void* kh, const void* vh, int dtype,
                        int64_t N, int H, int D, const int32_t* cu_seqlens, int M,
                        float softmax_scale, void* oh, float* lse,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * repermute of Alg. 1 with the gate of Eq. 5:
 *   o[perm[j]][h][:] = gate[perm[j]] * oh[h][j][:]      (gate NULL: plain scatter)
 */
int moga_unpermute(const void* oh, int dtype, const int32_t* perm, const float* gate_or_null,
                   int64_t N, int H, int D, void* o, void* stream);

/*
 * Backward of moga_unpermute (derivative of Eq. 5 w.r.t. the attention output and the gate):
 *   d_oh[h][j][:] = gate[perm[j]] * d_o[perm[j]][h][:]
 *   d_gate[perm[j]] = sum_{h,c} d_o[perm[j]][h][c] * oh[h][j][c]      [N] fp32
 */
int moga_unpermute_bwd(const void* d_o, const void* oh, int dtype, const int32_t* perm,
                       const float* gate, int64_t N, int H, int D,
                       void* d_oh, float* d_gate, void* stream);

/*
 * Backward of moga_group_attn_fwd, per group and head, with P = exp(scale*S - lse):
 *   delta = rowsum(d_oh * oh);  dV = P^T d_oh;  dP = d_oh V^T;  dS = P * (dP - delta)
 *   dQ = scale * dS K;  dK = scale * dS^T Q
 * All tensors [H, N, D] in group-contiguous order; lse from the forward call.
 */
int moga_group_attn_bwd(const void* d_oh, const void* qh, const void* kh, const void* vh,
                        const void* oh, const float* lse, int dtype,
                        int64_t N, int H, int D, const int32_t* cu_seqlens, int M,
                        float softmax_scale, void* d_qh, void* d_kh, void* d_vh,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * Diagnostics of the BF16 backward calls (moga_group_attn_bwd, moga_varlen_attn_bwd,
 * moga_fused_attn_bwd).  Inside the dK/dV kernel one wave of a pair waits for values its partner
 * publishes through LDS; the wait is bounded, and a wave that gives up sets an int32 status word in
 * the workspace to a nonzero value and carries on, so the kernel always drains (the gradients of
 * that call are then invalid).  The word lies at byte offset moga_attn_bwd_status_offset(Nq, H) of
 * ws, is cleared by every call and is valid in stream order after it; it reads 0 after every
 * correct run.  moga_debug_set_spin_limit sets the number of polls before a give-up (default 2^24;
 * 0 makes every not-yet-satisfied wait give up at once: for tests of this path only).  Host-only.
 */
size_t moga_attn_bwd_status_offset(int64_t Nq, int H);
void moga_debug_set_spin_limit(int polls);

/*
 * The BF16 attention calls have two sets of kernels: 8-wave blocks with 256-row (forward, dQ) or
 * 128-row (dK/dV) tiles, and 4-wave blocks with tiles half as large, two blocks per CU, for the small
 * static groups of Section 3.2.  The group sizes live on the device, so a call chooses by the mean
 * group size N / M (forward: below 2560 rows; backward: below 1280).  Both sets give the same results up
 * to rounding order.  moga_debug_set_small_group_rows overrides both thresholds (0: never the small
 * kernels; a huge value: always; negative: the defaults) so that tests can run either set on any shape.
 */
void moga_debug_set_small_group_rows(int64_t rows);

/* Backward of the gather in moga_permute: d_q[perm[j]][h][:] = d_qh[h][j][:] (same for k, v). */
int moga_permute_bwd(const void* d_qh, const void* d_kh, const void* d_vh, int dtype,
                     const int32_t* perm, int64_t N, int H, int D,
                     void* d_q, void* d_k, void* d_v, void* stream);

/*
 * Backward of the router through the gate (the assignment is a constant):
 *   dr[i][j] = d_gate[i] * gate[i] * ([j == group[i]] - probs[i][j])
 *   d_w[j][c] = sum_i dr[i][j] * x[i][c]            [M, d_model] fp32
 *   d_x[i][c] = sum_j dr[i][j] * w[j][c]            [N, d_model] fp32, NULL to skip
 */
int moga_route_bwd(const void* x, int x_dtype, const float* w, const float* probs,
                   const int32_t* group, const float* gate, const float* d_gate,
                   int64_t N, int d_model, int M, float* d_w, float* d_x_or_null,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * Alg. 1 steps 3-4 without materialising the permuted tensors: the kernel loads the rows of group g
 * through perm (row j of the sorted order is token perm[j]) from the token-order tensors
 * q, k, v [N, H, D], and writes o[perm[j]][h][:] = gate[perm[j]] * attention row j (Eq. 5) in
 * token order.  perm, cu_seqlens as written by moga_permute (which may be called with NULL
 * q, k, v so that it only builds the index); gate from moga_route.  lse [H, N] fp32 stays in
 * sorted order.  BF16, D = 128 only.  Same result as moga_permute + moga_group_attn_fwd +
 * moga_unpermute up to one bf16 rounding (the ungated output is never rounded).
 */
int moga_fused_attn_fwd(const void* q, const void* k, const void* v, int dtype, int64_t N, int H, int D,
                        const int32_t* perm, const float* gate, const int32_t* cu_seqlens, int M,
                        float softmax_scale, void* o, float* lse, void* stream);

/*
 * Backward of moga_fused_attn_fwd, again without permuted tensors.  d_o [N, H, D] is the gradient of
 * the gated output o; q, k, v, o token order; lse [H, N] from the fused forward; perm / inv_perm /
 * cu_seqlens from moga_permute; gate (> 0) from moga_route.  Outputs in token order: d_q, d_k, d_v
 * [N, H, D] and d_gate [N] fp32 (= sum over heads and channels of d_o * o / gate, the input of
 * moga_route_bwd).  The gate is folded into the per-row constants of the kernels
 * (lse - ln gate, rowsum(d_o * o) / gate), so neither the ungated output nor a scaled copy of d_o is
 * ever written.  BF16, D = 128 only.  Workspace: MOGA_OP_ATTN_BWD.
 */
int moga_fused_attn_bwd(const void* d_o, const void* q, const void* k, const void* v, const void* o,
                        const float* lse, int dtype, int64_t N, int H, int D,
                        const int32_t* perm, const int32_t* inv_perm, const float* gate,
                        const int32_t* cu_seqlens, int M, float softmax_scale,
                        void* d_q, void* d_k, void* d_v, float* d_gate,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * Attention inside static groups whose queries and keys are listed separately (Section 3.2,
 * "Spatial-Temporal Group Attention": a group's keys and values may hold more rows than its
 * queries, e.g. latent frames added from adjacent shots).  Group g attends the query rows
 * cu_seqlens_q[g] .. cu_seqlens_q[g+1] of qh [H, Nq, D] to the key/value rows
 * cu_seqlens_k[g] .. cu_seqlens_k[g+1] of kh, vh [H, Nk, D]; Eq. 1 per group and head, as in
 * moga_group_attn_fwd (which is the case cu_seqlens_k == cu_seqlens_q, Nk == Nq).
 * cu_seqlens_q, cu_seqlens_k: [G + 1] int32 on the device, non-decreasing, first entry 0, last
 * entry Nq / Nk.  G in [1, MOGA_MAX_SEGMENTS].  Queries of a group without keys get oh = 0 and
 * lse = -inf.  Outputs oh [H, Nq, D], lse [H, Nq] fp32.  Workspace: MOGA_OP_VARLEN_ATTN_FWD.
 */
int moga_varlen_attn_fwd(const void* qh, const void* kh, const void* vh, int dtype,
                         int64_t Nq, int64_t Nk, int H, int D,
                         const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int G,
                         float softmax_scale, void* oh, float* lse,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * Backward of moga_varlen_attn_fwd (same formulas as moga_group_attn_bwd, per group and head).
 * d_oh, oh, d_qh [H, Nq, D]; d_kh, d_vh [H, Nk, D]: one gradient row per listed key row (a token
 * listed as a key by several groups has several rows; moga_gather_rows_bwd adds them up).
 * Keys of a group without queries, and queries of a group without keys, get zero gradients.
 * Workspace: MOGA_OP_VARLEN_ATTN_BWD.
 */
int moga_varlen_attn_bwd(const void* d_oh, const void* qh, const void* kh, const void* vh,
                         const void* oh, const float* lse, int dtype,
                         int64_t Nq, int64_t Nk, int H, int D,
                         const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int G,
                         float softmax_scale, void* d_qh, void* d_kh, void* d_vh,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * Static groups of Section 3.2 ("Spatial-Temporal Group Attention"), built on the HOST: the lists
 * depend only on the latent grid (T frames of Hh x Ww tokens, token = (t*Hh + y)*Ww + x), the window
 * (wh x ww, non-overlapping, ragged at the border), the run length tg (consecutive frames of one
 * shot; the last run of a shot may be shorter) and the shot of every frame.  A group is
 * (run, window); its queries are its own tokens; its keys are its own tokens followed by the tokens
 * of the same window in the last a_prev frames of the previous shot and the first a_next frames of
 * the next shot (the paper adds two latent frames from the adjacent shots: a_prev = a_next = 1).
 * EVERY pointer of these two calls is a HOST pointer; shot_of_frame [T] must be non-decreasing.
 *   moga_stga_index_sizes: *n_groups = G, *n_keys = Nk (total listed keys).
 *   moga_stga_build_index: q_index [N] (queries of group g: q_index[cu_q[g] .. cu_q[g+1]), ascending),
 *     q_slot [N] (inverse of q_index), cu_q [G+1], kv_index [Nk], cu_k [G+1], and for the backward
 *     of the key gather inv_cu [N+1], inv_slots [Nk]: token t is listed at the key slots
 *     inv_slots[inv_cu[t] .. inv_cu[t+1]), ascending.
 * The per-frame groups of the same section need no lists: group f = frame f, cu[f] = f*Hh*Ww.
 */
int moga_stga_index_sizes(int T, int Hh, int Ww, int wh, int ww, int tg, const int32_t* shot_of_frame,
                          int a_prev, int a_next, int64_t* n_groups, int64_t* n_keys);
int moga_stga_build_index(int T, int Hh, int Ww, int wh, int ww, int tg, const int32_t* shot_of_frame,
                          int a_prev, int a_next, int32_t* q_index, int32_t* q_slot, int32_t* cu_q,
                          int32_t* kv_index, int32_t* cu_k, int32_t* inv_cu, int32_t* inv_slots);

/*
 * Gather through an index list (device pointers again): dst[h][j][:] = src[index[j]][h][:],
 * src [N, H, D] token order, dst [H, Nk, D]; index [Nk] int32 with values in [0, N), repeats allowed.
 */
int moga_gather_rows(const void* src, int dtype, const int32_t* index, int64_t Nk, int H, int D,
                     void* dst, void* stream);

/*
 * Backward of moga_gather_rows: d_src[t][h][:] (+)= sum of d_dst[h][j][:] over the slots j that
 * list token t (inv_cu [N+1], inv_slots [Nk] as built by moga_stga_build_index); fp32 sums in
 * ascending slot order, so the result is reproducible.  accumulate != 0 adds to d_src [N, H, D],
 * otherwise d_src is overwritten (tokens listed nowhere get zero).
 */
int moga_gather_rows_bwd(const void* d_dst, int dtype, const int32_t* inv_cu, const int32_t* inv_slots,
                         int64_t N, int64_t Nk, int H, int D, int accumulate, void* d_src, void* stream);

/*
 * Gradient of a token-order tensor (Q, K or V) that fed all three branches of Section 3.2, in one
 * pass:  d_src[t][h][:] = g_moga[h][inv_moga[t]][:]
 *                         + sum of g_stga[h][j][:] over the slots j that list token t
 *                         + g_frame[h][inv_frame[t]][:]
 * g_moga, g_frame [H, N, D]; g_stga [H, Nk, D]; inv_moga [N] (the inv_perm of moga_permute);
 * inv_cu [N+1], inv_slots [Nk] as for moga_gather_rows_bwd (for the queries, which are listed
 * once: inv_cu = 0..N and inv_slots = q_slot); inv_frame [N] or NULL for the identity.  One fp32
 * sum per element in the order written above (slots ascending), rounded once; d_src [N, H, D] is
 * overwritten.  Equivalent to moga_permute_bwd followed by two accumulating
 * moga_gather_rows_bwd calls, with half the memory traffic and one rounding instead of three.
 */
int moga_gather3_bwd(const void* g_moga, const int32_t* inv_moga, const void* g_stga,
                     const int32_t* inv_cu, const int32_t* inv_slots, int64_t Nk,
                     const void* g_frame, const int32_t* inv_frame, int dtype, int64_t N, int H,
                     int D, void* d_src, void* stream);

/*
 * Mean of the three branches of Section 3.2 fused into one scatter:
 *   o[t][h][:] = ( gate[t] * a_moga[h][inv_moga[t]][:] + a_stga[h][inv_stga[t]][:]
 *                  + a_frame[h][inv_frame[t]][:] ) / 3
 * a_* are [H, N, D] in each branch's own row order; inv_* [N] maps a token to its row there
 * (inv_perm of moga_permute, q_slot of moga_stga_build_index; NULL = identity).  Only the dynamic
 * branch is gated (Eq. 5).  o [N, H, D].
 */
int moga_merge3_fwd(const void* a_moga, const void* a_stga, const void* a_frame, int dtype,
                    const int32_t* inv_moga, const int32_t* inv_stga, const int32_t* inv_frame,
                    const float* gate, int64_t N, int H, int D, void* o, void* stream);

/*
 * Backward of moga_merge3_fwd: d_a_moga[h][inv_moga[t]] = gate[t] * d_o[t][h] / 3,
 * d_a_stga / d_a_frame likewise without the gate, d_gate[t] = sum_{h,c} d_o[t][h][c] * a_moga[h][inv_moga[t]][c] / 3.
 */
int moga_merge3_bwd(const void* d_o, const void* a_moga, int dtype, const int32_t* inv_moga,
                    const int32_t* inv_stga, const int32_t* inv_frame, const float* gate,
                    int64_t N, int H, int D, void* d_a_moga, void* d_a_stga, void* d_a_frame,
                    float* d_gate, void* stream);

/*
 * Group balancing loss, Eqs. 6-8 (Section 3.2; alpha = 0.1 in the paper's training setup):
 *   frac[i] = (1/N) #{x : group[x] = i}                   (Eq. 7)
 *   prob[i] = (1/N) sum_{x : group[x] = i} gate[x]        (Eq. 8: the sum runs over the tokens
 *                                                          assigned to i, gate = p(g(x)|x))
 *   loss    = alpha * M * sum_i frac[i] * prob[i]         (Eq. 6)
 * group [N] int32 and gate [N] fp32 as written by moga_route.  Outputs (device, fp32): loss [1],
 * frac [M], prob [M], all required.  Sums are order-independent (integer accumulation), so the
 * result is bit-reproducible.  Tokens whose group lies outside [0, M) are ignored.
 */
int moga_balance_loss(const int32_t* group, const float* gate, int64_t N, int M, float alpha,
                      float* loss, float* frac, float* prob, void* ws, size_t ws_bytes, void* stream);

/*
 * Gradient of the balancing loss with respect to the gate (frac is piecewise constant in the
 * router weights, so only prob carries a gradient):
 *   d_gate[x] (+)= d_loss * alpha * M * frac[group[x]] / N
 * frac [M] from moga_balance_loss.  The upstream scalar gradient is d_loss (a host value) times
 * d_loss_device_or_null[0] when that device pointer is given (an autograd caller keeps its
 * gradient on the device and passes d_loss = 1: no host synchronisation), else d_loss alone.
 * With accumulate != 0 the term is added to d_gate (e.g. the output of moga_unpermute_bwd, before
 * moga_route_bwd); otherwise d_gate is overwritten.
 */
int moga_balance_loss_bwd(const int32_t* group, const float* frac, int64_t N, int M, float alpha,
                          float d_loss, const float* d_loss_device_or_null, int accumulate,
                          float* d_gate, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOGA_H_ */
