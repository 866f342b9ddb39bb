// Prefill-time attention (query tiles on MFMA): placeholder until the tiled kernels land.
#include "common.h"

namespace rtp {
int32_t prefill_range_attn(const char* who, bool dense, const rtp_layer_desc* L, const void* q, const void* K,
                           const void* V, int64_t row_stride, int64_t head_stride, const int64_t* seq_start,
                           const int32_t* ctx_len, const int32_t* q_start, int32_t B, int32_t n_q, int64_t max_ctx,
                           void* out, float* lse, hipStream_t s) {
  return fail(RTP_ERR_UNSUPPORTED, "%s: prefill mode is not built yet", who);
}
}  // namespace rtp

using namespace rtp;

extern "C" size_t rtp_sparse_attn_prefill_workspace_bytes(const rtp_layer_desc* layer, int32_t T, int64_t chunk_start) {
  return 256;
}
extern "C" int32_t rtp_sparse_attn_prefill(const rtp_layer_desc* layer, const void* q_pre, const void* q, const float* WQ,
                                           const void* kI, int64_t kI_head_stride,
                                           const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                                           int64_t chunk_start, int32_t T, float p, void* out, float* lse,
                                           float* tau, int32_t* count, float* mass,
                                           void* ws, size_t ws_bytes, void* stream) {
  return fail(RTP_ERR_UNSUPPORTED, "rtp_sparse_attn_prefill: not built yet");
}
