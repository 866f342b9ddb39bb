// Decode-time attention over a token set: rtp_sparse_attn_decode (paper Sec. 3.2, sparse-attention
// equation), rtp_local_attn in decode mode (sink + window rule, Sec. 3.2 / Sec. 4.2) and the dense
// comparison rtp_dense_attn in decode mode.
//
// All three stream K/V rows with a different token source: an index list (sparse), or the ranges
// [0, sink) U [ctx - window, ctx) (local) / [0, ctx) (dense).  Two kernels share the work-item plan, the
// partial format and the merge launch: the vector-ALU kernel described next (one query head per row:
// the selected-token source, and range sources without GQA), and attn_decode_gqa_kernel further down
// (a GQA group per row: the scores go to the matrix cores).  One K or V row is 256 bytes
// = 16 lanes x 16 bytes, so a 64-lane wave loads four rows per instruction; the 16 lanes of a DPP row
// own one token, multiply their 8 dims with the query and reduce with four DPP adds.  Each 16-lane
// group keeps its own online-softmax state (max, sum, 8 output dims per lane) in registers for all
// G query heads that share the KV head, so every K/V row is read once per KV head.  U tokens per
// group are in flight at a time (all K and V loads are issued before the arithmetic).
//
// Load balance without host knowledge of the set sizes: a persistent grid; every workgroup derives
// the same plan from the device-side counts -- split length ST = total tokens / grid size (rounded
// up to 128), unit u contributes ceil(n_u / ST) work items -- and walks the items blockIdx.x,
// blockIdx.x + gridDim.x, ...  Each item leaves a partial (m, l, acc[128]) per head; a second small
// kernel merges the partials of a unit (the split-KV reduction of Sec. 3.4, as a separate launch).
// Algorithmic traffic: 512 B per attended token and KV head (+ 4 B per token for the index list).
#include "attn_decode_shared.h"

#include <stdlib.h>

namespace rtp {

// Exclusive prefix sum over the block (256 threads); *total gets the block sum.
__device__ __forceinline__ int block_excl_scan(int v, int* sh_w /*[4]*/, int* total) {
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(incl, o);
    if ((threadIdx.x & 63) >= o) incl += t;
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 63) sh_w[threadIdx.x >> 6] = incl;
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kAdThreads / 64; ++i) {
    if (i < (int)(threadIdx.x >> 6)) off += sh_w[i];
    tot += sh_w[i];
  }
  *total = tot;
  return off + incl - v;
}

// Every workgroup computes the same plan: split length and the exclusive item prefix per unit.
template <int SRC>
__device__ __forceinline__ void build_plan(const AttnDecodeArgs& a, int* sh_prefix /*[kAdMaxUnits+1]*/, int* sh_w,
                                           int* split_tokens, int* n_items) {
  const int tid = threadIdx.x;
  int cnt[kAdMaxUnits / kAdThreads];
  int mine = 0;
#pragma unroll
  for (int i = 0; i < kAdMaxUnits / kAdThreads; ++i) {
    const int u = tid * (kAdMaxUnits / kAdThreads) + i;
    cnt[i] = u < a.units ? unit_tokens<SRC>(a, u) : 0;
    mine += (cnt[i] + 127) >> 7;          // in blocks of 128 tokens, so the total cannot overflow int
  }
  int total128;
  block_excl_scan(mine, sh_w, &total128);
  // at least kMinSplitBlocks * 128 tokens per item: shorter items spend their time in the prologue and the merge
  int st = (total128 + a.target_items - 1) / max(a.target_items, 1);
  st = max(st, a.min_split_blocks) * 128;
  int items = 0;
#pragma unroll
  for (int i = 0; i < kAdMaxUnits / kAdThreads; ++i) {
    cnt[i] = (cnt[i] + st - 1) / st;
    items += cnt[i];
  }
  int tot;
  int off = block_excl_scan(items, sh_w, &tot);
#pragma unroll
  for (int i = 0; i < kAdMaxUnits / kAdThreads; ++i) {
    const int u = tid * (kAdMaxUnits / kAdThreads) + i;
    sh_prefix[u] = off;
    off += cnt[i];
  }
  if (tid == kAdThreads - 1) sh_prefix[kAdMaxUnits] = off;
  __syncthreads();
  *split_tokens = st;
  *n_items = tot;
}

__device__ __forceinline__ int find_unit(const int* sh_prefix, int units, int item) {
  int lo = 0, hi = units - 1;             // largest u with prefix[u] <= item
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (sh_prefix[mid] <= item) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Merge online-softmax state (mo, lo, acco) into (m, l, acc); log2-domain maxima.
__device__ __forceinline__ void merge_state(float& m, float& l, float (&acc)[8], float mo, float lo,
                                            const float (&acco)[8]) {
  const float M = fmaxf(m, mo);
  if (M == -__builtin_huge_valf()) return;
  const float ca = fast_exp2(m - M), cb = fast_exp2(mo - M);
  l = l * ca + lo * cb;
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = acc[c] * ca + acco[c] * cb;
  m = M;
}

// PAGED (selected-token source only): token position p of sequence b lives in row
// page_table[b][p >> page_shift] * page_size + p % page_size of a pool shared by all sequences.  The lookup is
// one more dependent load in front of the K/V rows, so the index list runs TWO rounds ahead and the page
// lookups one round ahead: both stay in the shadow of the row loads.
template <int G, int SRC, int U, bool PAGED = false, bool F16 = false>
__global__ __launch_bounds__(kAdThreads) void attn_decode_kernel(const AttnDecodeArgs a) {
  static_assert(!PAGED || SRC != kSrcDense, "paging is implemented for the selected-token and the local source");
  __shared__ int sh_prefix[kAdMaxUnits + 1];
  __shared__ int sh_w[kAdThreads / 64];
  __shared__ float sh_m[kAdThreads / 64][G], sh_l[kAdThreads / 64][G];
  __shared__ float sh_acc[kAdThreads / 64][G][kHeadDim];

  int ST, n_items;
  if (SRC == kSrcSparse) {
    build_plan<SRC>(a, sh_prefix, sh_w, &ST, &n_items);
  } else {
    ST = a.split_tokens;
    n_items = a.units * a.n_splits;
  }

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = wave * 4 + (lane >> 4);   // 16 groups of 16 lanes
  const int piece = lane & 15;              // which 8 of the 128 dims
  const float ninf = -__builtin_huge_valf();
  const int group_size = a.n_q_heads / a.n_kv_heads;

  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    int unit, split;
    if (SRC == kSrcSparse) {
      unit = find_unit(sh_prefix, a.units, item);
      split = item - sh_prefix[unit];
    } else {
      unit = item / a.n_splits;
      split = item - unit * a.n_splits;
    }
    int b, kvh, h0;
    if (SRC == kSrcSparse) {
      b = unit / a.n_ret;
      h0 = a.ret_heads[unit - b * a.n_ret];
      kvh = h0 / group_size;
    } else {
      b = unit / a.n_kv_heads;
      kvh = unit - b * a.n_kv_heads;
      h0 = kvh * G;
    }
    const int n_tok = unit_tokens<SRC>(a, unit);
    const int t_begin = split * ST, t_end = min(n_tok, t_begin + ST);
    if (t_begin >= n_tok) continue;        // (fixed plan only) this split lies beyond the unit's tokens
    // local source: logical token i maps to position i (sinks) or w0 + (i - s0) (window)
    int s0 = 0, w0 = 0;
    if (SRC == kSrcLocal) {
      const int n = a.ctx_len[b];
      s0 = max(min(a.sink, n), 0);
      w0 = max(a.sink, n - a.window);
    }
    const int32_t* idx = (SRC == kSrcSparse) ? a.sel_idx + (int64_t)unit * a.sel_stride : nullptr;
    const int64_t seq0 = PAGED ? 0 : a.seq_start[b];      // PAGED: rows are pool rows, no per-sequence offset
    const uint16_t* Kb = a.K + (int64_t)kvh * a.head_stride + seq0 * a.row_stride + piece * 8;
    const uint16_t* Vb = a.V + (int64_t)kvh * a.head_stride + seq0 * a.row_stride + piece * 8;
    int64_t row_stride = a.row_stride;
    const int32_t* pt = PAGED ? a.page_table + (int64_t)b * a.pt_stride : nullptr;
    const int page_mask = (1 << a.page_shift) - 1;
    auto pool_row = [&](int p) { return (pt[p >> a.page_shift] << a.page_shift) | (p & page_mask); };
    bool paged_rows = PAGED;
    if (SRC == kSrcLocal && a.ringK && a.ring_of_kv[kvh] >= 0) {
      // bounded cache: its first n_tok rows are exactly this unit's tokens, in some order
      paged_rows = false;
      const int64_t off = (int64_t)a.ring_of_kv[kvh] * a.ring_head_stride + a.ring_seq_start[b] * a.ring_row_stride + piece * 8;
      Kb = a.ringK + off;
      Vb = a.ringV + off;
      row_stride = a.ring_row_stride;
      s0 = n_tok;                         // logical token i is row i
    }

    float qv[G][8];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
      const u32x4 qraw = *reinterpret_cast<const u32x4*>(a.q + ((int64_t)b * a.n_q_heads + h0 + hh) * kHeadDim + piece * 8);
      unpack8<F16>(qraw, qv[hh]);
#pragma unroll
      for (int c = 0; c < 8; ++c) qv[hh][c] *= a.scale_log2;
    }
    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
      m[hh] = ninf;
      l[hh] = 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[hh][c] = 0.f;
    }

    int nxt[U];                 // rows of the coming round (positions, or pool rows when PAGED)
    int ahead[PAGED ? U : 1];   // PAGED: positions of the round after it
    if (SRC == kSrcSparse) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = t_begin + u * 16 + grp;
        nxt[u] = i < t_end ? idx[i] : 0;
        if (PAGED) {
          ahead[u] = i + 16 * U < t_end ? idx[i + 16 * U] : 0;
          nxt[u] = i < t_end ? pool_row(nxt[u]) : 0;
        }
      }
    }
    for (int base = t_begin; base < t_end; base += 16 * U) {
      u32x4 kr[U], vr[U];
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = base + u * 16 + grp;
        ok[u] = i < t_end;
        int pos;
        if (SRC == kSrcSparse) pos = nxt[u];
        else if (SRC == kSrcLocal) pos = i < s0 ? i : w0 + (i - s0);
        else pos = i;
        if (PAGED && SRC == kSrcLocal && paged_rows && ok[u]) pos = pool_row(pos);
        if (ok[u]) {
          kr[u] = *reinterpret_cast<const u32x4*>(Kb + (int64_t)pos * row_stride);
          vr[u] = *reinterpret_cast<const u32x4*>(Vb + (int64_t)pos * row_stride);
        } else {
          kr[u] = (u32x4){0u, 0u, 0u, 0u};
          vr[u] = (u32x4){0u, 0u, 0u, 0u};
        }
      }
      if (SRC == kSrcSparse) {   // index list of the next round, under the shadow of the K/V loads
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int i = base + 16 * U + u * 16 + grp;
          if (PAGED) {
            nxt[u] = i < t_end ? pool_row(ahead[u]) : 0;               // its positions arrived a round ago
            ahead[u] = i + 16 * U < t_end ? idx[i + 16 * U] : 0;
          } else {
            nxt[u] = i < t_end ? idx[i] : 0;
          }
        }
      }
      float s[G][U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float kf[8];
        unpack8<F16>(kr[u], kf);
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
          float d = kf[0] * qv[hh][0];
#pragma unroll
          for (int c = 1; c < 8; ++c) d = fmaf(kf[c], qv[hh][c], d);
          d = row16_sum(d);
          s[hh][u] = ok[u] ? d : ninf;
        }
      }
#pragma unroll
      for (int hh = 0; hh < G; ++hh) {
        float mx = s[hh][0];
#pragma unroll
        for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[hh][u]);
        const float mn = fmaxf(m[hh], mx);
        if (mn != ninf) {
          const float corr = fast_exp2(m[hh] - mn);
          l[hh] *= corr;
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[hh][c] *= corr;
          m[hh] = mn;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float vf[8];
        unpack8<F16>(vr[u], vf);
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
          const float pw = (s[hh][u] == ninf) ? 0.f : fast_exp2(s[hh][u] - m[hh]);
          l[hh] += pw;
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[hh][c] = fmaf(pw, vf[c], acc[hh][c]);
        }
      }
    }

    // ---- merge the four 16-lane groups of each wave in registers, then the four waves through LDS ----
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const float mo = __shfl_xor(m[hh], o), lo = __shfl_xor(l[hh], o);
        float ao[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) ao[c] = __shfl_xor(acc[hh][c], o);
        merge_state(m[hh], l[hh], acc[hh], mo, lo, ao);
      }
    }
    __syncthreads();   // previous item's readers are done with the LDS buffers
    if (lane < 16) {
#pragma unroll
      for (int hh = 0; hh < G; ++hh) {
        if (piece == 0) { sh_m[wave][hh] = m[hh]; sh_l[wave][hh] = l[hh]; }
#pragma unroll
        for (int c = 0; c < 8; ++c) sh_acc[wave][hh][piece * 8 + c] = acc[hh][c];
      }
    }
    __syncthreads();
    float* pout = a.part + (int64_t)item * G * kPartStride;
    for (int e = tid; e < G * kHeadDim; e += kAdThreads) {
      const int hh = e >> 7, d = e & 127;
      float M = sh_m[0][hh];
#pragma unroll
      for (int w = 1; w < kAdThreads / 64; ++w) M = fmaxf(M, sh_m[w][hh]);
      float L = 0.f, A = 0.f;
      if (M != ninf) {
#pragma unroll
        for (int w = 0; w < kAdThreads / 64; ++w) {
          const float cw = fast_exp2(sh_m[w][hh] - M);
          L += sh_l[w][hh] * cw;
          A += sh_acc[w][hh][d] * cw;
        }
      }
      pout[hh * kPartStride + 4 + d] = A;
      if (d == 0) { pout[hh * kPartStride] = M; pout[hh * kPartStride + 1] = L; }
    }
  }
}

// ---- GQA groups on the matrix cores ---------------------------------------------------------------
// With G >= 2 query heads per KV row the kernel above spends its time on the vector ALU (every head
// repeats the 128-term dot product and its DPP reduction per row).  Here the scores of 16 tokens x G
// heads are four v_mfma_f32_16x16x32_bf16 (A = the K rows in the MFMA operand layout: lane = token +
// 16 * quarter, loaded straight from global memory, 64 contiguous bytes per row and instruction; B = the
// G queries in 16 columns, zero beyond G).  The softmax runs in the MFMA result layout (lane = head +
// 16 * row group, four tokens per lane), where a head's running maximum is uniform over its four lanes
// after two cross-row exchanges.  The PV product stays on the vector ALU in the row-streaming layout
// of the kernel above (16 lanes per token, 8 dims per lane): token 4 * grp + j of a tile is loaded by
// lane group grp in round j, so the probability it needs sits in ITS OWN 16-lane row at lane = head,
// register j, and one DPP row_share brings it to all 16 lanes.  Work items, partials and the merge
// launch are those of the kernel above.
template <int G, int SRC, bool F16 = false, bool PAGED = false>
__global__ __launch_bounds__(kAdThreads) void attn_decode_gqa_kernel(const AttnDecodeArgs a) {
  gqa_decode_items<G, SRC, kAdThreads, 2, F16, PAGED>(a, blockIdx.x, gridDim.x);
}

// Merges the partials of one (unit, head) per workgroup: 8 slices of 32 lanes, each lane owns 4 of the
// 128 output dims and walks the unit's work items slice, slice + 8, ...; LDS merges the 8 slices.
template <int G, int SRC>
__global__ __launch_bounds__(kAdThreads) void attn_decode_combine_kernel(const AttnDecodeArgs a) {
  __shared__ int sh_prefix[SRC == kSrcSparse ? kAdMaxUnits + 1 : 1];
  __shared__ int sh_w[kAdThreads / 64];
  const int unit = blockIdx.x / G, hh = blockIdx.x - unit * G;
  int b, h, i0, i1;
  if (SRC == kSrcSparse) {
    int ST, n_items;
    build_plan<SRC>(a, sh_prefix, sh_w, &ST, &n_items);
    b = unit / a.n_ret;
    h = a.ret_heads[unit - b * a.n_ret];
    i0 = sh_prefix[unit];
    i1 = (unit + 1 < a.units) ? sh_prefix[unit + 1] : n_items;
  } else {
    b = unit / a.n_kv_heads;
    h = (unit - b * a.n_kv_heads) * G + hh;
    if (SRC == kSrcLocal && a.is_ret[h]) return;
    i0 = unit * a.n_splits;
    i1 = i0 + (unit_tokens<SRC>(a, unit) + a.split_tokens - 1) / a.split_tokens;
  }
  merge_partials_to_out(a, G, hh, b, h, i0, i1);
}

struct DecodePlanHost {
  int32_t units, target_items, grid, split_tokens, n_splits;
  size_t ws_bytes;
};

// Sparse: the set sizes are only known on the device, so the host gives a target item count and a
// persistent grid; the device derives the split length from the actual counts.
static DecodePlanHost plan_host_sparse(int32_t units, int64_t max_tok) {
  DecodePlanHost p = {};
  p.units = units;
  const int64_t cap = 1024;
  int64_t blocks128 = (int64_t)units * ((max_tok + 127) / 128);
  int64_t tgt = blocks128 < 1 ? 1 : (blocks128 > cap ? cap : blocks128);
  p.target_items = (int32_t)tgt;
  p.grid = (int32_t)tgt;
  // items <= total128 / ceil(total128 / target) + units <= target + units
  p.ws_bytes = align_up((size_t)(tgt + units) * kPartStride * sizeof(float), 256);
  return p;
}

// Local / dense: every unit has at most max_tok tokens, so the split is fixed on the host.
static DecodePlanHost plan_host_range(int32_t units, int64_t max_tok, int32_t G) {
  DecodePlanHost p = {};
  p.units = units;
  // about 512 tokens per item, between 256 and 1024 items: a short local window cut finer than that only
  // buys launch and merge overhead (measured on batch 8: 2052 tokens per unit, 256 items 24.2 us, 1024 items 26.5 us)
  int64_t dflt = (int64_t)units * max_tok / 512;
  dflt = dflt < 256 ? 256 : (dflt > 1024 ? 1024 : dflt);
  const int64_t cap = dflt;
  const int64_t blocks = (max_tok + 127) / 128;
  int64_t ns = cap / units;
  if (ns < 1) ns = 1;
  if (ns > blocks) ns = blocks;
  int64_t st = ((max_tok + ns - 1) / ns + 127) / 128 * 128;
  ns = (max_tok + st - 1) / st;
  p.split_tokens = (int32_t)st;
  p.n_splits = (int32_t)ns;
  p.grid = (int32_t)(units * ns);
  p.ws_bytes = align_up((size_t)units * ns * G * kPartStride * sizeof(float), 256);
  return p;
}

template <int SRC, bool F16>
static int32_t launch_decode_t(const AttnDecodeArgs& a, int G, int grid, hipStream_t s, const char* who) {
  const int cgrid = a.units * G;
  // one head per K/V row (always so for the selected-token source): the vector-ALU kernel;
  // a GQA group per row: scores on the matrix cores
  constexpr bool kCanPage = SRC != kSrcDense;
#define RTP_LAUNCH_GQA(GG)                                                                                   \
  if (kCanPage && a.page_table)                                                                              \
    RTP_LAUNCH((attn_decode_gqa_kernel<GG, SRC == kSrcSparse ? kSrcDense : SRC, F16, kCanPage>), dim3(grid), dim3(kAdThreads), 0, s, a); \
  else                                                                                                       \
    RTP_LAUNCH((attn_decode_gqa_kernel<GG, SRC == kSrcSparse ? kSrcDense : SRC, F16>), dim3(grid), dim3(kAdThreads), 0, s, a); \
  RTP_LAUNCH((attn_decode_combine_kernel<GG, SRC>), dim3(cgrid), dim3(kAdThreads), 0, s, a);
  if (SRC == kSrcSparse || G == 1) {
    if (kCanPage && a.page_table) RTP_LAUNCH((attn_decode_kernel<1, SRC, 8, kCanPage, F16>), dim3(grid), dim3(kAdThreads), 0, s, a);
    else RTP_LAUNCH((attn_decode_kernel<1, SRC, 8, false, F16>), dim3(grid), dim3(kAdThreads), 0, s, a);
    RTP_LAUNCH((attn_decode_combine_kernel<1, SRC>), dim3(cgrid), dim3(kAdThreads), 0, s, a);
  } else {
    switch (G) {
      case 2: RTP_LAUNCH_GQA(2) break;
      case 4: RTP_LAUNCH_GQA(4) break;
      case 8: RTP_LAUNCH_GQA(8) break;
      default: return fail(RTP_ERR_UNSUPPORTED, "%s: group size %d", who, G);
    }
  }
#undef RTP_LAUNCH_GQA
  return check_launch(who);
}
template <int SRC>
static int32_t launch_decode(const AttnDecodeArgs& a, int G, int grid, hipStream_t s, const char* who) {
  return a.f16 ? launch_decode_t<SRC, true>(a, G, grid, s, who) : launch_decode_t<SRC, false>(a, G, grid, s, who);
}

static int32_t check_kv(const char* who, const void* q, const void* K, const void* V, int64_t row_stride,
                        int64_t head_stride, const void* out) {
  if (!q || !K || !V || !out) return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (row_stride < kHeadDim || (row_stride & 7) || (head_stride & 7) || head_stride < 0)
    return fail(RTP_ERR_INVALID_ARG, "%s: kv_row_stride must be >= 128, strides multiples of 8", who);
  if (((uintptr_t)q & 15) || ((uintptr_t)K & 15) || ((uintptr_t)V & 15) || ((uintptr_t)out & 15))
    return fail(RTP_ERR_INVALID_ARG, "%s: q, K, V and out must be 16-byte aligned", who);
  return RTP_OK;
}

static void fill_common(AttnDecodeArgs& a, const rtp_layer_desc* L, const HeadTable& ht, const void* q, const void* K,
                        const void* V, int64_t row_stride, int64_t head_stride, const int64_t* seq_start,
                        const int32_t* ctx_len, void* out, float* lse, void* ws) {
  a.q = (const uint16_t*)q;
  a.K = (const uint16_t*)K;
  a.V = (const uint16_t*)V;
  a.row_stride = row_stride;
  a.head_stride = head_stride;
  a.seq_start = seq_start;
  a.ctx_len = ctx_len;
  a.sel_idx = nullptr;
  a.sel_stride = 0;
  a.sel_count = nullptr;
  a.n_q_heads = L->n_q_heads;
  a.n_kv_heads = L->n_kv_heads;
  a.n_ret = L->n_ret;
  a.sink = L->sink;
  a.window = L->window;
  a.scale_log2 = softmax_scale_of(L) * 1.4426950408889634f;
  a.part = (float*)ws;
  a.out = (uint16_t*)out;
  a.lse = lse;
  a.f16 = L->kv_dtype == RTP_DTYPE_FP16;
  for (int j = 0; j < 64; ++j) a.ret_heads[j] = ht.ret_heads[j];
  for (int h = 0; h < 128; ++h) a.is_ret[h] = ht.is_ret[h];
  a.ringK = a.ringV = nullptr;
  a.ring_row_stride = a.ring_head_stride = 0;
  a.ring_seq_start = nullptr;
  for (int h = 0; h < 128; ++h) a.ring_of_kv[h] = -1;
  a.page_table = nullptr;
  a.pt_stride = 0;
  a.page_shift = 0;
}

// Decode-mode local / dense attention (called from attn_api.hip).
int ring_heads_of(const rtp_layer_desc* L, int32_t* heads, int8_t* ring_of_kv);

// Checks the arguments of a range-source decode call and fills the kernels' argument block and grid.
// *launch = false: nothing to compute (no local head).  Also used by the selector's launch that carries the
// local heads' work items (topp.hip).
int32_t decode_range_prepare(const char* who, bool dense, const rtp_layer_desc* L, const void* q, const void* K,
                             const void* V, int64_t row_stride, int64_t head_stride, const int64_t* seq_start,
                             const int32_t* ctx_len, int32_t B, int64_t max_ctx, void* out, float* lse, void* ws,
                             size_t ws_bytes, const RingSource* ring, AttnDecodeArgs* args, int* grid, bool* launch,
                             const PageSource* pages) {
  *launch = false;
  HeadTable ht;
  int32_t rc = fill_head_table(L, &ht, who);
  if (rc != RTP_OK) return rc;
  rc = check_kv(who, q, K, V, row_stride, head_stride, out);
  if (rc != RTP_OK) return rc;
  if ((!seq_start && !pages) || !ctx_len) return fail(RTP_ERR_INVALID_ARG, "%s: NULL seq_start/ctx_len", who);
  if (B <= 0 || max_ctx <= 0) return fail(RTP_ERR_INVALID_ARG, "%s: B and max_ctx must be positive", who);
  int page_shift = 0;
  if (pages) {
    if (dense) return fail(RTP_ERR_UNSUPPORTED, "%s: the dense comparison does not read a paged cache", who);
    rc = check_pages(who, pages, max_ctx, &page_shift);
    if (rc != RTP_OK) return rc;
  }
  const int G = L->n_q_heads / L->n_kv_heads;
  const int64_t units = (int64_t)B * L->n_kv_heads;
  if (units > kAdMaxUnits) return fail(RTP_ERR_UNSUPPORTED, "%s: B * n_kv_heads = %lld exceeds %d", who, (long long)units, kAdMaxUnits);
  const int64_t max_tok = dense ? max_ctx : (max_ctx < (int64_t)L->sink + L->window ? max_ctx : (int64_t)L->sink + L->window);
  const DecodePlanHost p = plan_host_range((int32_t)units, max_tok, G);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < p.ws_bytes)
    return fail(RTP_ERR_WORKSPACE, "%s: workspace of %zu bytes (256-byte aligned) required, got %zu", who, p.ws_bytes, ws_bytes);
  clear_error();
  if (!dense && L->n_ret == L->n_q_heads) return RTP_OK;   // no local head
  AttnDecodeArgs& a = *args;
  fill_common(a, L, ht, q, K, V, row_stride, head_stride, seq_start, ctx_len, out, lse, ws);
  a.units = p.units;
  a.target_items = 0;
  a.min_split_blocks = 1;
  a.split_tokens = p.split_tokens;
  a.n_splits = p.n_splits;
  if (pages) {
    a.page_table = pages->table;
    a.pt_stride = pages->stride;
    a.page_shift = page_shift;
  }
  if (ring) {
    a.ringK = (const uint16_t*)ring->K;
    a.ringV = (const uint16_t*)ring->V;
    a.ring_row_stride = ring->row_stride;
    a.ring_head_stride = ring->head_stride;
    a.ring_seq_start = ring->seq_start;
    ring_heads_of(L, nullptr, a.ring_of_kv);
  }
  *grid = p.grid;
  *launch = true;
  return RTP_OK;
}

static int32_t decode_range_attn_from(const char* who, bool dense, const rtp_layer_desc* L, const void* q, const void* K,
                                      const void* V, int64_t row_stride, int64_t head_stride, const int64_t* seq_start,
                                      const int32_t* ctx_len, int32_t B, int64_t max_ctx, void* out, float* lse, void* ws,
                                      size_t ws_bytes, hipStream_t s, const RingSource* ring,
                                      const PageSource* pages = nullptr) {
  AttnDecodeArgs a;
  int grid = 0;
  bool launch = false;
  const int32_t rc = decode_range_prepare(who, dense, L, q, K, V, row_stride, head_stride, seq_start, ctx_len, B, max_ctx,
                                          out, lse, ws, ws_bytes, ring, &a, &grid, &launch, pages);
  if (rc != RTP_OK || !launch) return rc;
  const int G = L->n_q_heads / L->n_kv_heads;
  return dense ? launch_decode<kSrcDense>(a, G, grid, s, who) : launch_decode<kSrcLocal>(a, G, grid, s, who);
}

int32_t decode_range_attn(const char* who, bool dense, const rtp_layer_desc* L, const void* q, const void* K,
                          const void* V, int64_t row_stride, int64_t head_stride, const int64_t* seq_start,
                          const int32_t* ctx_len, int32_t B, int64_t max_ctx, void* out, float* lse, void* ws,
                          size_t ws_bytes, hipStream_t s, const PageSource* pages) {
  return decode_range_attn_from(who, dense, L, q, K, V, row_stride, head_stride, seq_start, ctx_len, B, max_ctx, out, lse,
                                ws, ws_bytes, s, nullptr, pages);
}

int32_t check_pages(const char* who, const PageSource* pages, int64_t max_ctx, int* page_shift) {
  if (!pages->table) return fail(RTP_ERR_INVALID_ARG, "%s: NULL page_table", who);
  const int32_t ps = pages->page_size;
  if (ps < 16 || (ps & (ps - 1)) || ps > (1 << 20))
    return fail(RTP_ERR_INVALID_ARG, "%s: page_size must be a power of two in [16, 2^20]", who);
  int sh = 0;
  while ((1 << sh) < ps) ++sh;
  if (pages->stride < (max_ctx + ps - 1) / ps) return fail(RTP_ERR_INVALID_ARG, "%s: pt_stride must cover max_ctx tokens", who);
  *page_shift = sh;
  return RTP_OK;
}

size_t decode_range_ws(bool dense, const rtp_layer_desc* L, int32_t B, int64_t max_ctx) {
  if (!L || B <= 0 || max_ctx <= 0 || L->n_kv_heads <= 0 || L->n_q_heads <= 0) return 0;
  const int G = L->n_q_heads / L->n_kv_heads;
  const int64_t max_tok = dense ? max_ctx : (max_ctx < (int64_t)L->sink + L->window ? max_ctx : (int64_t)L->sink + L->window);
  return plan_host_range(B * L->n_kv_heads, max_tok, G).ws_bytes;
}

}  // namespace rtp

using namespace rtp;

extern "C" size_t rtp_sparse_attn_decode_workspace_bytes(const rtp_layer_desc* layer, int32_t B, int64_t max_sel) {
  if (!layer || B <= 0 || max_sel <= 0 || layer->n_ret <= 0) return 256;
  return plan_host_sparse(B * layer->n_ret, max_sel).ws_bytes;
}

static int32_t sparse_attn_decode_impl(const char* who, const rtp_layer_desc* layer, const void* q,
                                       const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                                       const int64_t* seq_start, const int32_t* page_table, int64_t pt_stride,
                                       int32_t page_size,
                                       const int32_t* sel_idx, int64_t sel_stride, const int32_t* sel_count,
                                       int64_t max_sel, int32_t B, void* out, float* lse,
                                       void* ws, size_t ws_bytes, void* stream) {
  HeadTable ht;
  int32_t rc = fill_head_table(layer, &ht, who);
  if (rc != RTP_OK) return rc;
  rc = check_kv(who, q, K, V, kv_row_stride, kv_head_stride, out);
  if (rc != RTP_OK) return rc;
  if ((!seq_start && !page_table) || !sel_idx || !sel_count)
    return fail(RTP_ERR_INVALID_ARG, "%s: NULL seq_start/page_table/sel_idx/sel_count", who);
  int page_shift = 0;
  if (page_table) {
    if (page_size < 16 || (page_size & (page_size - 1)) || page_size > (1 << 20))
      return fail(RTP_ERR_INVALID_ARG, "%s: page_size must be a power of two in [16, 2^20]", who);
    while ((1 << page_shift) < page_size) ++page_shift;
    if (pt_stride < (max_sel + page_size - 1) / page_size)
      return fail(RTP_ERR_INVALID_ARG, "%s: pt_stride must cover max_sel tokens", who);
  }
  if (B <= 0 || max_sel <= 0) return fail(RTP_ERR_INVALID_ARG, "%s: B and max_sel must be positive", who);
  if (sel_stride < max_sel) return fail(RTP_ERR_INVALID_ARG, "%s: sel_stride must be >= max_sel", who);
  const int64_t units = (int64_t)B * layer->n_ret;
  if (units > kAdMaxUnits) return fail(RTP_ERR_UNSUPPORTED, "%s: B * n_ret = %lld exceeds %d", who, (long long)units, kAdMaxUnits);
  if (layer->n_ret == 0) { clear_error(); return RTP_OK; }
  const DecodePlanHost p = plan_host_sparse((int32_t)units, max_sel);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < p.ws_bytes)
    return fail(RTP_ERR_WORKSPACE, "%s: workspace of %zu bytes (256-byte aligned) required, got %zu", who, p.ws_bytes, ws_bytes);
  clear_error();
  AttnDecodeArgs a;
  fill_common(a, layer, ht, q, K, V, kv_row_stride, kv_head_stride, seq_start, nullptr, out, lse, ws);
  a.sel_idx = sel_idx;
  a.sel_stride = sel_stride;
  a.sel_count = sel_count;
  a.units = p.units;
  a.target_items = p.target_items;
  a.min_split_blocks = 5;
  a.split_tokens = 0;
  a.n_splits = 0;
  a.page_table = page_table;
  a.pt_stride = pt_stride;
  a.page_shift = page_shift;
  return launch_decode<kSrcSparse>(a, 1, p.grid, (hipStream_t)stream, who);
}

extern "C" int32_t rtp_sparse_attn_decode(const rtp_layer_desc* layer, const void* q,
                                          const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                                          const int64_t* seq_start,
                                          const int32_t* sel_idx, int64_t sel_stride, const int32_t* sel_count,
                                          int64_t max_sel, int32_t B, void* out, float* lse,
                                          void* ws, size_t ws_bytes, void* stream) {
  if (!seq_start) return fail(RTP_ERR_INVALID_ARG, "rtp_sparse_attn_decode: NULL seq_start/sel_idx/sel_count");
  return sparse_attn_decode_impl("rtp_sparse_attn_decode", layer, q, K, V, kv_row_stride, kv_head_stride, seq_start,
                                 nullptr, 0, 0, sel_idx, sel_stride, sel_count, max_sel, B, out, lse, ws, ws_bytes, stream);
}

extern "C" int32_t rtp_sparse_attn_decode_paged(const rtp_layer_desc* layer, const void* q,
                                                const void* K, const void* V, int64_t kv_row_stride,
                                                int64_t kv_head_stride, const int32_t* page_table, int64_t pt_stride,
                                                int32_t page_size,
                                                const int32_t* sel_idx, int64_t sel_stride, const int32_t* sel_count,
                                                int64_t max_sel, int32_t B, void* out, float* lse,
                                                void* ws, size_t ws_bytes, void* stream) {
  if (!page_table) return fail(RTP_ERR_INVALID_ARG, "rtp_sparse_attn_decode_paged: NULL page_table");
  return sparse_attn_decode_impl("rtp_sparse_attn_decode_paged", layer, q, K, V, kv_row_stride, kv_head_stride, nullptr,
                                 page_table, pt_stride, page_size, sel_idx, sel_stride, sel_count, max_sel, B, out, lse, ws,
                                 ws_bytes, stream);
}

extern "C" size_t rtp_local_attn_ring_workspace_bytes(const rtp_layer_desc* layer, int32_t B, int64_t max_ctx) {
  const size_t w = decode_range_ws(false, layer, B, max_ctx);
  return w ? w : 256;
}

extern "C" int32_t rtp_local_attn_ring(const rtp_layer_desc* layer, const void* q,
                                       const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                                       const int64_t* seq_start,
                                       const void* ring_K, const void* ring_V, int64_t ring_row_stride,
                                       int64_t ring_head_stride, const int64_t* ring_seq_start,
                                       const int32_t* ctx_len, int32_t B, int64_t max_ctx, void* out, float* lse,
                                       void* ws, size_t ws_bytes, void* stream) {
  const char* who = "rtp_local_attn_ring";
  int32_t rc = check_layer(layer, who);
  if (rc != RTP_OK) return rc;
  if (!ring_K || !ring_V || !ring_seq_start) return fail(RTP_ERR_INVALID_ARG, "%s: NULL ring pointer", who);
  if (((uintptr_t)ring_K & 15) || ((uintptr_t)ring_V & 15))
    return fail(RTP_ERR_INVALID_ARG, "%s: ring_K and ring_V must be 16-byte aligned", who);
  if (ring_row_stride < kHeadDim || (ring_row_stride & 7) || (ring_head_stride & 7) || ring_head_stride < 0)
    return fail(RTP_ERR_INVALID_ARG, "%s: ring_row_stride must be >= 128, ring strides multiples of 8", who);
  if (layer->window <= 0) return fail(RTP_ERR_INVALID_ARG, "%s: a bounded cache needs window > 0", who);
  const RingSource ring = {ring_K, ring_V, ring_row_stride, ring_head_stride, ring_seq_start};
  return decode_range_attn_from(who, false, layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len, B, max_ctx,
                                out, lse, ws, ws_bytes, (hipStream_t)stream, &ring);
}
