// rtp_index_project: the low-rank indexer projections of the paper's Sec. 3.2 (indexer equation),
//   kI[j, n, :] = bf16( W^K_{h_j} k^pre_{n, kv(h_j)} )     (key side: appended tokens, once per token)
//   qI[j, t, :] = bf16( W^Q_{h_j} q^pre_{t, h_j} )          (query side)
// for the j-th retrieval query head h_j.  The 128-term sums run in fp64 (every bf16 x fp32 product is
// exact there) and are rounded to bf16 ONCE, so the bits do not depend on the summation order and equal
// a correctly rounded reference.
//
// A workgroup takes 64 tokens of one retrieval head.  W_j sits in LDS as fp64, transposed to
// [c][16] so that the four outputs a thread owns are two 16-byte reads that the whole wave shares
// per quarter; a thread owns (token, 4 outputs), streams its token's 256-byte row in 16-byte pieces and
// does 512 fp64 FMAs.  fp64 vector rate and the HBM read of the rows (256 B per token and KV head)
// are of the same order, so neither a matrix-core formulation nor a finer split would buy much.
#include "common.h"

namespace rtp {

constexpr int kIbThreads = 256;
constexpr int kIbTokens = 64;     // tokens per workgroup

struct IndexBuildArgs {
  const float* W;           // [n_ret, 16, 128]
  const uint16_t* x;        // bf16 [T, n_x_heads, 128]
  uint16_t* out;            // bf16: (j, t, i) at out[j * out_head_stride + (out_t0 + t) * 16 + i]
  int64_t out_head_stride, out_t0;
  int32_t T, n_x_heads;
  int32_t x_head[64];       // head of x that retrieval head j projects
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kIbThreads) void index_build_kernel(const IndexBuildArgs a) {
  __shared__ double Wt[kHeadDim][kIndexDim];           // 16 KB
  const int j = blockIdx.y, tid = threadIdx.x;
  const float* Wj = a.W + (int64_t)j * kIndexDim * kHeadDim;
  for (int e = tid; e < kIndexDim * kHeadDim; e += kIbThreads) {
    const int i = e >> 7, c = e & 127;                 // coalesced read of W[j][i][c]
    Wt[c][i] = (double)Wj[e];
  }
  __syncthreads();
  const int t = blockIdx.x * kIbTokens + (tid >> 2), qd = tid & 3;   // token, quarter of the 16 outputs
  if (t >= a.T) return;
  const uint16_t* row = a.x + ((int64_t)t * a.n_x_heads + a.x_head[j]) * kHeadDim;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
  for (int c8 = 0; c8 < kHeadDim; c8 += 8) {
    const u32x4 raw = *reinterpret_cast<const u32x4*>(row + c8);
    const float xf[8] = {bf16_lo(raw.x), bf16_hi(raw.x), bf16_lo(raw.y), bf16_hi(raw.y),
                         bf16_lo(raw.z), bf16_hi(raw.z), bf16_lo(raw.w), bf16_hi(raw.w)};
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const double xv = (double)xf[k];
      const double* w = &Wt[c8 + k][qd * 4];
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = fma(w[i], xv, acc[i]);
    }
  }
  uint16_t* o = a.out + (int64_t)j * a.out_head_stride + (a.out_t0 + t) * kIndexDim + qd * 4;
  const uint32_t lo = (uint32_t)f64_to_bf16_rne(acc[0]) | ((uint32_t)f64_to_bf16_rne(acc[1]) << 16);
  const uint32_t hi = (uint32_t)f64_to_bf16_rne(acc[2]) | ((uint32_t)f64_to_bf16_rne(acc[3]) << 16);
  *reinterpret_cast<uint2*>(o) = make_uint2(lo, hi);
}

}  // namespace rtp

using namespace rtp;

extern "C" int32_t rtp_index_project(const rtp_layer_desc* layer, const float* W, const void* x_pre, int32_t side,
                                     int32_t T, void* xI_out, int64_t out_head_stride, int64_t out_t0, void* stream) {
  const char* who = "rtp_index_project";
  HeadTable ht;
  int32_t rc = fill_head_table(layer, &ht, who);
  if (rc != RTP_OK) return rc;
  if (!W || !x_pre || !xI_out) return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (side != RTP_SIDE_QUERY && side != RTP_SIDE_KEY) return fail(RTP_ERR_INVALID_ARG, "%s: side must be RTP_SIDE_QUERY or RTP_SIDE_KEY", who);
  if (T <= 0 || out_t0 < 0) return fail(RTP_ERR_INVALID_ARG, "%s: T must be positive and out_t0 >= 0", who);
  if (out_head_stride < 0 || (out_head_stride & 3)) return fail(RTP_ERR_INVALID_ARG, "%s: out_head_stride must be a non-negative multiple of 4", who);
  if (((uintptr_t)x_pre & 15) || ((uintptr_t)xI_out & 7) || ((uintptr_t)W & 3))
    return fail(RTP_ERR_INVALID_ARG, "%s: x_pre must be 16-byte and xI_out 8-byte aligned", who);
  const int64_t blocks = ((int64_t)T + kIbTokens - 1) / kIbTokens;
  if (blocks > 0x7fffffffLL) return fail(RTP_ERR_INVALID_ARG, "%s: T too large", who);
  clear_error();
  if (layer->n_ret == 0) return RTP_OK;
  IndexBuildArgs a;
  a.W = W;
  a.x = (const uint16_t*)x_pre;
  a.out = (uint16_t*)xI_out;
  a.out_head_stride = out_head_stride;
  a.out_t0 = out_t0;
  a.T = T;
  const int G = layer->n_q_heads / layer->n_kv_heads;
  a.n_x_heads = side == RTP_SIDE_QUERY ? layer->n_q_heads : layer->n_kv_heads;
  for (int j = 0; j < 64; ++j) {
    const int h = j < layer->n_ret ? layer->ret_heads[j] : 0;
    a.x_head[j] = side == RTP_SIDE_QUERY ? h : h / G;
  }
  RTP_LAUNCH(index_build_kernel, dim3((unsigned)blocks, (unsigned)layer->n_ret), dim3(kIbThreads), 0,
                     (hipStream_t)stream, a);
  return check_launch(who);
}
