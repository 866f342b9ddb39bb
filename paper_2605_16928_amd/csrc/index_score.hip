// rtp_index_score: the indexer score pass (paper Sec. 3.2, indexer equation).
//
// HBM-bound streaming kernel.  Index keys are 32-byte rows (16 x bf16); a lane loads 16-byte pieces
// at consecutive addresses so that every wave-wide load instruction covers one contiguous 1 KiB
// (eight full 128-byte lines).  A lane multiplies its half row with the matching half of the index
// query, lanes 2i and 2i+1 exchange their partial sums through DPP, and even/odd lanes write the
// scores of two consecutive load rounds, which keeps the fp32 stores full-line as well.
// Algorithmic traffic: 32 B read + 4 B written per (token, retrieval head).
//
// Optionally the pass also accumulates the first level of the top-p mass histogram of every row
// (topp_common.h) while the scores are still in registers: the exponentials run in the shadow of the
// HBM stream and the selector then starts at its second level.
#include "topp_common.h"

namespace rtp {

// tokens per workgroup: 2048 (64 KiB of index keys) for the plain pass; the pass that also builds the
// histogram takes 4096 so that half as many workgroups zero, scan and flush a 2048-bin LDS histogram
// (measured on batch 8 x 131072: 27.5 us against 28.4 us with 2048; the plain pass prefers 2048)
constexpr int kIsThreads = 256;
constexpr int kIsChunkPlain = 8 * kIsThreads, kIsChunkHist = 16 * kIsThreads;
constexpr int kIsBatch = 16;             // 16-byte loads in flight per lane

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct IndexScoreArgs {
  const uint16_t* q_in;
  const float* WQ;
  const uint16_t* kI;
  int64_t kI_head_stride;
  const int64_t* seq_start;
  const int32_t* ctx_len;
  const int32_t* q_start;
  int32_t n_q, n_ret, n_q_heads;
  float index_scale;
  float* scores;
  int64_t score_stride;
  uint16_t* qI_out;
  uint64_t* hist;          // level-1 histograms of the selector's workspace or NULL
  int64_t hist_stride;     // words per row; n_sub copies of level 1 per row (topp_common.h)
  int32_t n_sub;
  int32_t ret_heads[64];
};

__device__ __forceinline__ float dot8(const u32x4 v, const float (&q)[8]) {
  float acc = bf16_lo(v.x) * q[0];
  acc = fmaf(bf16_hi(v.x), q[1], acc);
  acc = fmaf(bf16_lo(v.y), q[2], acc);
  acc = fmaf(bf16_hi(v.y), q[3], acc);
  acc = fmaf(bf16_lo(v.z), q[4], acc);
  acc = fmaf(bf16_hi(v.z), q[5], acc);
  acc = fmaf(bf16_lo(v.w), q[6], acc);
  acc = fmaf(bf16_hi(v.w), q[7], acc);
  return acc;
}

// PROBE: the same grid, loads and stores with the arithmetic taken out (the stored word is a piece of the key
// row): what the chip sustains for this traffic mix, 32 bytes read for every 4 written.
template <bool HIST, bool PROBE = false>
__global__ __launch_bounds__(kIsThreads) void index_score_kernel(const IndexScoreArgs a) {
  constexpr int kIsChunk = HIST ? kIsChunkHist : kIsChunkPlain;
  static_assert((kIsChunk * 2) % (kIsThreads * kIsBatch) == 0, "a chunk is a whole number of load batches");
  const int bj = blockIdx.z;
  const int b = bj / a.n_ret, j = bj - b * a.n_ret, t = blockIdx.y;
  const int n_ctx = a.ctx_len[b];
  const int64_t n0 = (int64_t)blockIdx.x * kIsChunk;
  if (n0 >= n_ctx) return;
  const int tid = threadIdx.x;

  // ---- issue the first batch of key loads before anything else: they depend on nothing the prologue
  // computes, so the projection and the histogram set-up run under their latency ----
  const int limit = a.q_start ? min(n_ctx, a.q_start[b] + t + 1) : n_ctx;   // candidates: n < limit
  const int n_here = (int)min((int64_t)kIsChunk, (int64_t)n_ctx - n0);     // chunk tokens inside the context
  const int lim_here = (int)min((int64_t)n_here, (int64_t)limit - n0);     // chunk tokens that are candidates
  const u32x4* src = reinterpret_cast<const u32x4*>(a.kI + (int64_t)j * a.kI_head_stride +
                                                    (a.seq_start[b] + n0) * kIndexDim);
  const bool full = (n_here == kIsChunk);
  u32x4 v[kIsBatch];
  auto load_batch = [&](int batch) {
#pragma unroll
    for (int u = 0; u < kIsBatch; ++u) {
      const int piece = (batch * kIsBatch + u) * kIsThreads + tid;
      if (full || (piece >> 1) < n_here) {
        v[u] = __builtin_nontemporal_load(src + piece);
      } else {
        v[u] = (u32x4){0u, 0u, 0u, 0u};
      }
    }
  };
  load_batch(0);

  __shared__ uint64_t lh[HIST ? kBins1 : 1];
  __shared__ double tab[HIST ? 256 : 1];
  if (HIST) {
    for (int i = tid; i < kBins1; i += kIsThreads) lh[i] = 0;
    fill_exp_table(tab);
  }
  const int shift = fixed_shift(n_ctx);

  // ---- the index query of this row: 16 floats in LDS (bf16 values) ----
  __shared__ float sq[kIndexDim];
  const int64_t qi_off = (((int64_t)b * a.n_ret + j) * a.n_q + t) * kIndexDim;
  if (a.WQ) {
    if (tid < 256) {
      const int i = tid >> 4, part = tid & 15;   // 16 output dims x 16 lanes, 8 terms each
      const float* w = a.WQ + ((int64_t)j * kIndexDim + i) * kHeadDim + part * 8;
      const uint16_t* x = a.q_in + (((int64_t)b * a.n_q + t) * a.n_q_heads + a.ret_heads[j]) * kHeadDim + part * 8;
      double acc = 0.0;
#pragma unroll
      for (int c = 0; c < 8; ++c) acc = fma((double)w[c], (double)bf16_to_f32(x[c]), acc);
      acc += __shfl_xor(acc, 1);
      acc += __shfl_xor(acc, 2);
      acc += __shfl_xor(acc, 4);
      acc += __shfl_xor(acc, 8);
      if (part == 0) {
        const uint16_t qb = f64_to_bf16_rne(acc);
        sq[i] = bf16_to_f32(qb);
        if (blockIdx.x == 0 && a.qI_out) a.qI_out[qi_off + i] = qb;
      }
    }
  } else if (tid < kIndexDim) {
    const uint16_t qb = a.q_in[qi_off + tid];
    sq[tid] = bf16_to_f32(qb);
    if (blockIdx.x == 0 && a.qI_out) a.qI_out[qi_off + tid] = qb;
  }
  __syncthreads();

  const int half = tid & 1;
  float qv[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) qv[c] = sq[half * 8 + c];

  float* dst = a.scores + ((int64_t)bj * a.n_q + t) * a.score_stride + n0;
  const float ninf = -__builtin_huge_valf();

#pragma unroll
  for (int batch = 0; batch < (kIsChunk * 2) / (kIsThreads * kIsBatch); ++batch) {
    if (batch > 0) load_batch(batch);
#pragma unroll
    for (int u = 0; u < kIsBatch; u += 2) {
      const float d0 = PROBE ? __uint_as_float(v[u].x & 0x3fffffffu) : pair_sum(dot8(v[u], qv));
      const float d1 = PROBE ? __uint_as_float(v[u + 1].x & 0x3fffffffu) : pair_sum(dot8(v[u + 1], qv));
      const int tok = (((batch * kIsBatch + u + half) * kIsThreads) + tid) >> 1;
      float val = (half ? d1 : d0) * a.index_scale;
      if (tok >= lim_here) val = ninf;
      if (tok < n_here) {
        dst[tok] = val;
        if (HIST) level1_add(lh, val, shift, tab);
      }
    }
  }
  if (HIST) {
    __syncthreads();
    flush_hist(lh, a.hist + ((int64_t)bj * a.n_q + t) * a.hist_stride + level1_copy_offset((int)(blockIdx.x % a.n_sub)), kBins1,
               kIsThreads);
  }
}

}  // namespace rtp

using namespace rtp;

static int32_t run_index_score(const char* who, bool probe, const rtp_layer_desc* layer, const void* q_in, const float* WQ,
                               const void* kI, int64_t kI_head_stride,
                               const int64_t* seq_start, const int32_t* ctx_len, const int32_t* q_start,
                               int32_t B, int32_t n_q, int64_t max_ctx,
                               float* scores, int64_t score_stride, void* qI_out,
                               void* topp_ws, size_t topp_ws_bytes, void* stream) {
  int32_t rc = check_layer(layer, who);
  if (rc != RTP_OK) return rc;
  if (!q_in || !kI || !seq_start || !ctx_len || !scores)
    return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (B <= 0 || n_q <= 0 || max_ctx <= 0) return fail(RTP_ERR_INVALID_ARG, "%s: B, n_q and max_ctx must be positive", who);
  if (!q_start && n_q != 1) return fail(RTP_ERR_INVALID_ARG, "%s: decode (q_start == NULL) needs n_q == 1", who);
  if (n_q > 65535 || (int64_t)B * layer->n_ret > 65535)
    return fail(RTP_ERR_INVALID_ARG, "%s: n_q and B * n_ret are limited to 65535", who);
  if (max_ctx > RTP_MAX_ROW_LEN) return fail(RTP_ERR_INVALID_ARG, "%s: max_ctx exceeds %d", who, RTP_MAX_ROW_LEN);
  if (score_stride < max_ctx || (score_stride & 3))
    return fail(RTP_ERR_INVALID_ARG, "%s: score_stride must be >= max_ctx and a multiple of 4", who);
  if (((uintptr_t)scores & 15) || ((uintptr_t)kI & 15) || (kI_head_stride & 7) || kI_head_stride < 0)
    return fail(RTP_ERR_INVALID_ARG, "%s: scores/kI must be 16-byte aligned, kI_head_stride a multiple of 8", who);
  uint64_t* hist = nullptr;
  int64_t hist_stride = 0;
  int32_t n_sub = 1;
  if (topp_ws) {
    const int64_t rows = (int64_t)B * layer->n_ret * n_q;
    if (rows > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: more than 65535 score rows", who);
    const TopPLayout l = topp_layout((int32_t)rows, max_ctx);
    if (((uintptr_t)topp_ws & 255) || topp_ws_bytes < l.total)
      return fail(RTP_ERR_WORKSPACE, "%s: top-p workspace of %zu bytes (256-byte aligned) required, got %zu", who,
                  l.total, topp_ws_bytes);
    hist = (uint64_t*)((char*)topp_ws + l.hist_off);
    hist_stride = l.hist_stride;
    n_sub = l.n_sub;
  }
  clear_error();
  if (layer->n_ret == 0) return RTP_OK;

  IndexScoreArgs a;
  a.hist = hist;
  a.hist_stride = hist_stride;
  a.n_sub = n_sub;
  a.q_in = (const uint16_t*)q_in;
  a.WQ = WQ;
  a.kI = (const uint16_t*)kI;
  a.kI_head_stride = kI_head_stride;
  a.seq_start = seq_start;
  a.ctx_len = ctx_len;
  a.q_start = q_start;
  a.n_q = n_q;
  a.n_ret = layer->n_ret;
  a.n_q_heads = layer->n_q_heads;
  a.index_scale = index_scale_of(layer);
  a.scores = scores;
  a.score_stride = score_stride;
  a.qI_out = (uint16_t*)qI_out;
  for (int j = 0; j < 64; ++j) a.ret_heads[j] = j < layer->n_ret ? layer->ret_heads[j] : 0;

  const int64_t chunk = hist ? kIsChunkHist : kIsChunkPlain;
  dim3 grid((unsigned)((max_ctx + chunk - 1) / chunk), (unsigned)n_q, (unsigned)(B * layer->n_ret));
  if (probe) RTP_LAUNCH((index_score_kernel<false, true>), grid, dim3(kIsThreads), 0, (hipStream_t)stream, a);
  else if (hist) RTP_LAUNCH(index_score_kernel<true>, grid, dim3(kIsThreads), 0, (hipStream_t)stream, a);
  else RTP_LAUNCH(index_score_kernel<false>, grid, dim3(kIsThreads), 0, (hipStream_t)stream, a);
  return check_launch(who);
}

extern "C" int32_t rtp_index_score(const rtp_layer_desc* layer, const void* q_in, const float* WQ,
                                   const void* kI, int64_t kI_head_stride,
                                   const int64_t* seq_start, const int32_t* ctx_len, const int32_t* q_start,
                                   int32_t B, int32_t n_q, int64_t max_ctx,
                                   float* scores, int64_t score_stride, void* qI_out,
                                   void* topp_ws, size_t topp_ws_bytes, void* stream) {
  return run_index_score("rtp_index_score", false, layer, q_in, WQ, kI, kI_head_stride, seq_start, ctx_len, q_start, B, n_q,
                         max_ctx, scores, score_stride, qI_out, topp_ws, topp_ws_bytes, stream);
}

extern "C" int32_t rtp_index_score_traffic_probe(const rtp_layer_desc* layer, const void* q_in, const float* WQ,
                                                 const void* kI, int64_t kI_head_stride,
                                                 const int64_t* seq_start, const int32_t* ctx_len, const int32_t* q_start,
                                                 int32_t B, int32_t n_q, int64_t max_ctx,
                                                 float* scores, int64_t score_stride, void* stream) {
  return run_index_score("rtp_index_score_traffic_probe", true, layer, q_in, WQ, kI, kI_head_stride, seq_start, ctx_len,
                         q_start, B, n_q, max_ctx, scores, score_stride, nullptr, nullptr, 0, stream);
}
