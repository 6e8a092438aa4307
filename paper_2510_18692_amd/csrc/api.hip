// Host-only entry points of the C ABI: status strings, version, workspace sizes.
#include <atomic>

#include "moga_common.h"

extern "C" size_t moga_permute_ws_bytes(int64_t N, int M);
extern "C" size_t moga_route_bwd_ws_bytes(int64_t N, int M, int d_model);
extern "C" size_t moga_attn_bwd_ws_bytes(int64_t N, int H, int D, int dtype);
extern "C" size_t moga_balance_ws_bytes(int M);
extern "C" size_t moga_varlen_attn_fwd_ws_bytes(int G);
extern "C" size_t moga_varlen_attn_bwd_ws_bytes(int64_t Nq, int H, int G);

extern "C" const char* moga_status_string(int status) {
  switch (status) {
    case MOGA_OK: return "MOGA_OK";
    case MOGA_ERR_INVALID_ARG: return "MOGA_ERR_INVALID_ARG";
    case MOGA_ERR_UNSUPPORTED: return "MOGA_ERR_UNSUPPORTED";
    case MOGA_ERR_WORKSPACE: return "MOGA_ERR_WORKSPACE";
    case MOGA_ERR_HIP: return "MOGA_ERR_HIP";
    default: return "MOGA_ERR_UNKNOWN";
  }
}

extern "C" int moga_version(void) { return 104; }

// Test hook: overrides the mean group size below which the bf16 attention calls pick their
// small-group kernels (negative: each call's own default).
static std::atomic<long long> g_small_group_rows{-1};
extern "C" void moga_debug_set_small_group_rows(int64_t rows) { g_small_group_rows.store(rows); }
namespace moga {
bool use_small_group_kernels(int64_t rows, int groups, int64_t default_threshold) {
  const long long o = g_small_group_rows.load();
  return rows / (groups > 0 ? groups : 1) < (o >= 0 ? o : default_threshold);
}
}  // namespace moga

extern "C" size_t moga_workspace_bytes(int op, int64_t N, int H, int D, int M, int d_model,
                                       int dtype) {
  if (N <= 0 || M < 1) return 0;
  switch (op) {
    case MOGA_OP_PERMUTE: return moga_permute_ws_bytes(N, M);
    case MOGA_OP_ATTN_BWD: return moga_attn_bwd_ws_bytes(N, H, D, dtype);
    case MOGA_OP_ROUTE_BWD: return moga_route_bwd_ws_bytes(N, M, d_model);
    case MOGA_OP_BALANCE_LOSS: return moga_balance_ws_bytes(M);
    case MOGA_OP_VARLEN_ATTN_FWD: return moga_varlen_attn_fwd_ws_bytes(M);
    case MOGA_OP_VARLEN_ATTN_BWD: return moga_varlen_attn_bwd_ws_bytes(N, H, M);
    default: return 0;
  }
}
