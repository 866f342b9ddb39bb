// rtp_sparsity_stats: the decode-time sparsity figures of the paper's Sec. 3.2 (last paragraph) and
// Sec. 4.2 ("Sparsity Analysis" and its table), per sequence of one decode step:
//   compute sparsity  1 - (mean over QUERY heads of the number of attended tokens) / context
//   memory sparsity   1 - (mean over KV heads of the size of the UNION of the token sets of the query
//                     heads mapped to that KV head) / context
//   active tokens     mean selected-set size over the retrieval heads
//   attention mass    mean over the retrieval heads of the probability the FULL softmax attention puts on
//                     the selected set, exp(lse_selected - lse_full), from the log-sum-exps the attention
//                     entry points return
// A local head attends the sink + window set; a retrieval head its selected list.  The union of a KV
// group is counted without a bitmap: the local set is two ranges, the selected lists are ascending
// (as rtp_topp_select, rtp_topk_select and rtp_block_topp_select write them), so "already counted"
// is a range test plus a binary search in the lists of the group's earlier retrieval heads.
// One workgroup per sequence; integer counts, fixed order: deterministic.
#include "common.h"

namespace rtp {

constexpr int kStThreads = 256;

struct StatsArgs {
  const int32_t* ctx_len;
  const int32_t* sel_idx;
  int64_t sel_stride;
  const int32_t* sel_count;
  const float* lse_sel;     // optional [B, n_q_heads]
  const float* lse_full;    // optional [B, n_q_heads]
  float* stats;             // [B, 4]
  int32_t* union_size;      // optional [B, n_kv_heads]
  int32_t n_q_heads, n_kv_heads, n_ret, sink, window;
  int32_t ret_heads[64];
};

__device__ __forceinline__ bool list_has(const int32_t* lst, int n, int v) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (lst[mid] < v) lo = mid + 1; else hi = mid;
  }
  return lo < n && lst[lo] == v;
}

__device__ __forceinline__ long long block_sum(long long v, long long* sh) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  long long t = 0;
#pragma unroll
  for (int i = 0; i < kStThreads / 64; ++i) t += sh[i];
  return t;
}

__global__ __launch_bounds__(kStThreads) void sparsity_stats_kernel(const StatsArgs a) {
  __shared__ long long sh[kStThreads / 64];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int n = max(a.ctx_len[b], 0);
  const int G = a.n_q_heads / a.n_kv_heads;
  // local set: [0, s0) U [w0, n)
  const int s0 = min(a.sink, n);
  const int w0 = max(a.sink, n - a.window);
  const long long n_local = s0 + max(0, n - w0);
  long long attended = 0, unions = 0, active = 0;
  int jr = 0;                                      // retrieval heads are ascending: walk them with the KV heads
  for (int g = 0; g < a.n_kv_heads; ++g) {
    const int j0 = jr;
    while (jr < a.n_ret && a.ret_heads[jr] < (g + 1) * G) ++jr;
    const int n_ret_here = jr - j0;
    const bool has_local = n_ret_here < G;
    long long u = has_local ? n_local : 0;
    attended += (long long)(G - n_ret_here) * n_local;
    for (int j = j0; j < jr; ++j) {
      const int row = b * a.n_ret + j;
      const int cnt = max(a.sel_count[row], 0);
      const int32_t* lst = a.sel_idx + (int64_t)row * a.sel_stride;
      attended += cnt;
      active += cnt;
      long long fresh = 0;
      for (int e = tid; e < cnt; e += kStThreads) {
        const int v = lst[e];
        bool seen = has_local && (v < s0 || v >= w0);
        for (int jp = j0; jp < j && !seen; ++jp) {
          const int rp = b * a.n_ret + jp;
          seen = list_has(a.sel_idx + (int64_t)rp * a.sel_stride, max(a.sel_count[rp], 0), v);
        }
        fresh += seen ? 0 : 1;
      }
      u += block_sum(fresh, sh);
    }
    unions += u;
    if (a.union_size && tid == 0) a.union_size[b * a.n_kv_heads + g] = (int32_t)u;
  }
  if (tid != 0) return;
  float* o = a.stats + (int64_t)b * 4;
  const double nn = n > 0 ? (double)n : 1.0;
  o[0] = (float)(1.0 - (double)attended / ((double)a.n_q_heads * nn));
  o[1] = (float)(1.0 - (double)unions / ((double)a.n_kv_heads * nn));
  o[2] = a.n_ret > 0 ? (float)((double)active / a.n_ret) : 0.f;
  float mass = __builtin_nanf("");
  if (a.lse_sel && a.lse_full && a.n_ret > 0) {
    double m = 0.0;
    for (int j = 0; j < a.n_ret; ++j) {
      const int64_t i = (int64_t)b * a.n_q_heads + a.ret_heads[j];
      m += exp((double)a.lse_sel[i] - (double)a.lse_full[i]);
    }
    mass = (float)(m / a.n_ret);
  }
  o[3] = mass;
}

}  // namespace rtp

using namespace rtp;

extern "C" int32_t rtp_sparsity_stats(const rtp_layer_desc* layer, const int32_t* ctx_len,
                                      const int32_t* sel_idx, int64_t sel_stride, const int32_t* sel_count,
                                      const float* lse_selected, const float* lse_full, int32_t B,
                                      float* stats, int32_t* union_size, void* stream) {
  const char* who = "rtp_sparsity_stats";
  HeadTable ht;
  int32_t rc = fill_head_table(layer, &ht, who);
  if (rc != RTP_OK) return rc;
  if (!ctx_len || !stats) return fail(RTP_ERR_INVALID_ARG, "%s: NULL ctx_len/stats", who);
  if (layer->n_ret > 0 && (!sel_idx || !sel_count)) return fail(RTP_ERR_INVALID_ARG, "%s: NULL sel_idx/sel_count", who);
  if ((lse_selected == nullptr) != (lse_full == nullptr))
    return fail(RTP_ERR_INVALID_ARG, "%s: pass both log-sum-exp arrays or neither", who);
  if (B <= 0 || B > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: B must be in [1, 65535]", who);
  if (sel_stride < 0) return fail(RTP_ERR_INVALID_ARG, "%s: sel_stride must be >= 0", who);
  clear_error();
  StatsArgs a;
  a.ctx_len = ctx_len;
  a.sel_idx = sel_idx;
  a.sel_stride = sel_stride;
  a.sel_count = sel_count;
  a.lse_sel = lse_selected;
  a.lse_full = lse_full;
  a.stats = stats;
  a.union_size = union_size;
  a.n_q_heads = layer->n_q_heads;
  a.n_kv_heads = layer->n_kv_heads;
  a.n_ret = layer->n_ret;
  a.sink = layer->sink;
  a.window = layer->window;
  for (int j = 0; j < 64; ++j) a.ret_heads[j] = ht.ret_heads[j];
  RTP_LAUNCH(sparsity_stats_kernel, dim3((unsigned)B), dim3(kStThreads), 0, (hipStream_t)stream, a);
  return check_launch(who);
}
