#include "attn_common.h"
extern "C" size_t moga_attn_bwd_ws_bytes(int64_t N, int H, int D, int dtype) { return (size_t)N * H * 4; }
extern "C" int moga_group_attn_bwd(const void* d_oh, const void* qh, const void* kh, const void* vh,
                        const void* oh, const float* lse, int dtype,
                        int64_t N, int H, int D, const int32_t* cu_seqlens, int M,
                        float softmax_scale, void* d_qh, void* d_kh, void* d_vh,
                        void* ws, size_t ws_bytes, void* stream) { return MOGA_ERR_UNSUPPORTED; }
