// Bounded KV cache of the KV heads whose query heads are all local (decode).
//
// The paper keeps the full KV cache for retrieval heads only (Sec. 2.1); the other heads see the sink tokens
// and a sliding window (Sec. 3.2, Sec. 4.2).  The cache is per KV head (Sec. 3.2, last paragraph), so under
// GQA a KV head can drop remote tokens when every query head mapped to it is local.  Such a head keeps
// cap = sink + window rows per sequence: row i < sink holds token i, token t >= sink lives in row
// sink + (t - sink) mod window (the layout is this library's; the paper gives none).
//
//   rtp_kv_ring_heads   which KV heads those are (host-side helper)
//   rtp_kv_ring_append  one new token per sequence: 2 x 256 bytes per bounded head
//   rtp_kv_ring_fill    hand-over after prefill: the rows of the full cache that are still inside
// A softmax over a set does not depend on the order of its members, so attention reads the first
// min(ctx, cap) rows as they lie (rtp_local_attn_ring, attn_decode.hip).
#include "common.h"

namespace rtp {

constexpr int kRingThreads = 256;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct RingArgs {
  const uint16_t* K;          // append: bf16 [B, n_kv_heads, 128]; fill: the full cache
  const uint16_t* V;
  int64_t row_stride, head_stride;   // fill only
  const int64_t* seq_start;          // fill only
  const int32_t* n_or_pos;    // append: position of the new token per sequence; fill: ctx_len
  uint16_t* ringK;
  uint16_t* ringV;
  int64_t ring_row_stride, ring_head_stride;
  const int64_t* ring_seq_start;
  int32_t n_kv_heads, n_ring, sink, window;
  int32_t ring_heads[128];    // KV head of bounded head i
};

// Host: the all-local KV heads, ascending.  Returns their number.
int ring_heads_of(const rtp_layer_desc* L, int32_t* heads /*[n_kv_heads] or NULL*/, int8_t* ring_of_kv /*[128] or NULL*/) {
  const int g = L->n_q_heads / L->n_kv_heads;
  bool is_ret[128] = {};
  for (int j = 0; j < L->n_ret; ++j) is_ret[L->ret_heads[j]] = true;
  int n = 0;
  for (int kv = 0; kv < L->n_kv_heads; ++kv) {
    bool any = false;
    for (int h = kv * g; h < (kv + 1) * g; ++h) any = any || is_ret[h];
    if (ring_of_kv) ring_of_kv[kv] = any ? (int8_t)-1 : (int8_t)n;
    if (!any) {
      if (heads) heads[n] = kv;
      ++n;
    }
  }
  return n;
}

__device__ __forceinline__ int ring_slot(int t, int sink, int window) { return t < sink ? t : sink + (t - sink) % window; }

// One workgroup per sequence; a 16-lane group moves one 256-byte row (K or V of one bounded head).
__global__ __launch_bounds__(kRingThreads) void kv_ring_append_kernel(const RingArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int t = a.n_or_pos[b];
  if (t < 0) return;
  const int slot = ring_slot(t, a.sink, a.window);
  const int piece = tid & 15;
  for (int job = tid >> 4; job < 2 * a.n_ring; job += kRingThreads / 16) {
    const int i = job >> 1, which = job & 1;
    const uint16_t* src = (which ? a.V : a.K) + ((int64_t)b * a.n_kv_heads + a.ring_heads[i]) * kHeadDim + piece * 8;
    uint16_t* dst = (which ? a.ringV : a.ringK) + (int64_t)i * a.ring_head_stride +
                    (a.ring_seq_start[b] + slot) * a.ring_row_stride + piece * 8;
    *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(src);
  }
}

// grid (row blocks of 16, B, n_ring): row s of the bounded cache <- the token that occupies it after ctx_len appends.
__global__ __launch_bounds__(kRingThreads) void kv_ring_fill_kernel(const RingArgs a) {
  const int b = blockIdx.y, i = blockIdx.z, tid = threadIdx.x;
  const int n = a.n_or_pos[b];
  const int cap = a.sink + a.window;
  const int s = blockIdx.x * (kRingThreads / 16) + (tid >> 4), piece = tid & 15;
  if (s >= min(n, cap)) return;
  int t = s;
  if (s >= a.sink) {
    const int base = max(a.sink, n - a.window);        // oldest token of the window
    int off = (s - a.sink - (base - a.sink)) % a.window;
    if (off < 0) off += a.window;
    t = base + off;
  }
  const int64_t src = (int64_t)a.ring_heads[i] * a.head_stride + (a.seq_start[b] + t) * a.row_stride + piece * 8;
  const int64_t dst = (int64_t)i * a.ring_head_stride + (a.ring_seq_start[b] + s) * a.ring_row_stride + piece * 8;
  *reinterpret_cast<u32x4*>(a.ringK + dst) = *reinterpret_cast<const u32x4*>(a.K + src);
  *reinterpret_cast<u32x4*>(a.ringV + dst) = *reinterpret_cast<const u32x4*>(a.V + src);
}

static int32_t check_ring(const char* who, const rtp_layer_desc* L, const void* ring_K, const void* ring_V,
                          int64_t ring_row_stride, int64_t ring_head_stride, const void* ring_seq_start) {
  if (!ring_K || !ring_V || !ring_seq_start) return fail(RTP_ERR_INVALID_ARG, "%s: NULL ring pointer", who);
  if (((uintptr_t)ring_K & 15) || ((uintptr_t)ring_V & 15))
    return fail(RTP_ERR_INVALID_ARG, "%s: ring_K and ring_V must be 16-byte aligned", who);
  if (ring_row_stride < kHeadDim || (ring_row_stride & 7) || (ring_head_stride & 7) || ring_head_stride < 0)
    return fail(RTP_ERR_INVALID_ARG, "%s: ring_row_stride must be >= 128, ring strides multiples of 8", who);
  if (L->window <= 0) return fail(RTP_ERR_INVALID_ARG, "%s: a bounded cache needs window > 0", who);
  return RTP_OK;
}

static void fill_ring_args(RingArgs& a, const rtp_layer_desc* L, void* ring_K, void* ring_V, int64_t ring_row_stride,
                           int64_t ring_head_stride, const int64_t* ring_seq_start) {
  a.ringK = (uint16_t*)ring_K;
  a.ringV = (uint16_t*)ring_V;
  a.ring_row_stride = ring_row_stride;
  a.ring_head_stride = ring_head_stride;
  a.ring_seq_start = ring_seq_start;
  a.n_kv_heads = L->n_kv_heads;
  a.sink = L->sink;
  a.window = L->window;
  for (int i = 0; i < 128; ++i) a.ring_heads[i] = 0;
  a.n_ring = ring_heads_of(L, a.ring_heads, nullptr);
}

}  // namespace rtp

using namespace rtp;

extern "C" int32_t rtp_kv_ring_heads(const rtp_layer_desc* layer, int32_t* kv_heads) {
  const char* who = "rtp_kv_ring_heads";
  const int32_t rc = check_layer(layer, who);
  if (rc != RTP_OK) return -1;
  clear_error();
  return ring_heads_of(layer, kv_heads, nullptr);
}

extern "C" int32_t rtp_kv_ring_append(const rtp_layer_desc* layer, const void* k_new, const void* v_new,
                                      const int32_t* pos, int32_t B, void* ring_K, void* ring_V,
                                      int64_t ring_row_stride, int64_t ring_head_stride,
                                      const int64_t* ring_seq_start, void* stream) {
  const char* who = "rtp_kv_ring_append";
  int32_t rc = check_layer(layer, who);
  if (rc != RTP_OK) return rc;
  if (!k_new || !v_new || !pos) return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (((uintptr_t)k_new & 15) || ((uintptr_t)v_new & 15)) return fail(RTP_ERR_INVALID_ARG, "%s: k_new and v_new must be 16-byte aligned", who);
  if (B <= 0) return fail(RTP_ERR_INVALID_ARG, "%s: B must be positive", who);
  rc = check_ring(who, layer, ring_K, ring_V, ring_row_stride, ring_head_stride, ring_seq_start);
  if (rc != RTP_OK) return rc;
  clear_error();
  RingArgs a;
  fill_ring_args(a, layer, ring_K, ring_V, ring_row_stride, ring_head_stride, ring_seq_start);
  if (a.n_ring == 0) return RTP_OK;
  a.K = (const uint16_t*)k_new;
  a.V = (const uint16_t*)v_new;
  a.row_stride = a.head_stride = 0;
  a.seq_start = nullptr;
  a.n_or_pos = pos;
  RTP_LAUNCH(kv_ring_append_kernel, dim3((unsigned)B), dim3(kRingThreads), 0, (hipStream_t)stream, a);
  return check_launch(who);
}

extern "C" int32_t rtp_kv_ring_fill(const rtp_layer_desc* layer, const void* K, const void* V, int64_t kv_row_stride,
                                    int64_t kv_head_stride, const int64_t* seq_start, const int32_t* ctx_len, int32_t B,
                                    void* ring_K, void* ring_V, int64_t ring_row_stride, int64_t ring_head_stride,
                                    const int64_t* ring_seq_start, void* stream) {
  const char* who = "rtp_kv_ring_fill";
  int32_t rc = check_layer(layer, who);
  if (rc != RTP_OK) return rc;
  if (!K || !V || !seq_start || !ctx_len) return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (((uintptr_t)K & 15) || ((uintptr_t)V & 15)) return fail(RTP_ERR_INVALID_ARG, "%s: K and V must be 16-byte aligned", who);
  if (kv_row_stride < kHeadDim || (kv_row_stride & 7) || (kv_head_stride & 7) || kv_head_stride < 0)
    return fail(RTP_ERR_INVALID_ARG, "%s: kv_row_stride must be >= 128, strides multiples of 8", who);
  if (B <= 0 || B > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: B must be in [1, 65535]", who);
  rc = check_ring(who, layer, ring_K, ring_V, ring_row_stride, ring_head_stride, ring_seq_start);
  if (rc != RTP_OK) return rc;
  clear_error();
  RingArgs a;
  fill_ring_args(a, layer, ring_K, ring_V, ring_row_stride, ring_head_stride, ring_seq_start);
  if (a.n_ring == 0) return RTP_OK;
  a.K = (const uint16_t*)K;
  a.V = (const uint16_t*)V;
  a.row_stride = kv_row_stride;
  a.head_stride = kv_head_stride;
  a.seq_start = seq_start;
  a.n_or_pos = ctx_len;
  const int64_t cap = (int64_t)layer->sink + layer->window;
  const unsigned row_blocks = (unsigned)((cap + kRingThreads / 16 - 1) / (kRingThreads / 16));
  RTP_LAUNCH(kv_ring_fill_kernel, dim3(row_blocks, (unsigned)B, (unsigned)a.n_ring), dim3(kRingThreads), 0,
                     (hipStream_t)stream, a);
  return check_launch(who);
}
