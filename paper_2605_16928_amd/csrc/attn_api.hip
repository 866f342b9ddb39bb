// Entry points rtp_local_attn / rtp_dense_attn: dispatch between the decode kernels (one query per
// sequence, HBM-bound row streaming) and the prefill kernels (query tiles on MFMA).
#include "attn_decode_shared.h"

namespace rtp {

int32_t prefill_range_attn(const char* who, bool dense, const rtp_layer_desc* L, const void* q, const void* K,
                           const void* V, int64_t row_stride, int64_t head_stride, const int64_t* seq_start,
                           const int32_t* ctx_len, const int32_t* q_start, int32_t B, int32_t n_q, int64_t max_ctx,
                           void* out, float* lse, hipStream_t s);
}  // namespace rtp

using namespace rtp;

static int32_t range_attn(const char* who, bool dense, const rtp_layer_desc* layer, const void* q,
                          const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                          const int64_t* seq_start, const int32_t* ctx_len, const int32_t* q_start,
                          int32_t B, int32_t n_q, int64_t max_ctx, void* out, float* lse,
                          void* ws, size_t ws_bytes, void* stream) {
  if (n_q <= 0) return fail(RTP_ERR_INVALID_ARG, "%s: n_q must be positive", who);
  if (!q_start) {
    if (n_q != 1) return fail(RTP_ERR_INVALID_ARG, "%s: decode (q_start == NULL) needs n_q == 1", who);
    return decode_range_attn(who, dense, layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len, B,
                             max_ctx, out, lse, ws, ws_bytes, (hipStream_t)stream);
  }
  return prefill_range_attn(who, dense, layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len, q_start,
                            B, n_q, max_ctx, out, lse, (hipStream_t)stream);
}

extern "C" size_t rtp_local_attn_workspace_bytes(const rtp_layer_desc* layer, int32_t B, int32_t n_q, int64_t max_ctx) {
  (void)n_q;
  size_t w = decode_range_ws(false, layer, B, max_ctx);
  return w ? w : 256;
}
extern "C" size_t rtp_dense_attn_workspace_bytes(const rtp_layer_desc* layer, int32_t B, int32_t n_q, int64_t max_ctx) {
  (void)n_q;
  size_t w = decode_range_ws(true, layer, B, max_ctx);
  return w ? w : 256;
}

extern "C" int32_t rtp_local_attn(const rtp_layer_desc* layer, const void* q,
                                  const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                                  const int64_t* seq_start, const int32_t* ctx_len, const int32_t* q_start,
                                  int32_t B, int32_t n_q, int64_t max_ctx, void* out, float* lse,
                                  void* ws, size_t ws_bytes, void* stream) {
  return range_attn("rtp_local_attn", false, layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len,
                    q_start, B, n_q, max_ctx, out, lse, ws, ws_bytes, stream);
}

extern "C" int32_t rtp_dense_attn(const rtp_layer_desc* layer, const void* q,
                                  const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                                  const int64_t* seq_start, const int32_t* ctx_len, const int32_t* q_start,
                                  int32_t B, int32_t n_q, int64_t max_ctx, void* out, float* lse,
                                  void* ws, size_t ws_bytes, void* stream) {
  return range_attn("rtp_dense_attn", true, layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len,
                    q_start, B, n_q, max_ctx, out, lse, ws, ws_bytes, stream);
}
