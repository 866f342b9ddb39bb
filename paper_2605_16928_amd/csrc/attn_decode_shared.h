// Pieces of the decode attention kernels that other launches reuse (attn_decode.hip holds the kernels and
// describes the design): the argument block, the GQA work-item loop as a device function -- the selector can
// carry the local heads' work items in one of its own launches -- and the merge of partials.
#pragma once

#include "common.h"

namespace rtp {

constexpr int kAdThreads = 256;
constexpr int kAdMaxUnits = 1024;
constexpr int kPartStride = kHeadDim + 4;   // m, l, 2 pad, acc[128]  (floats)

enum { kSrcSparse = 0, kSrcLocal = 1, kSrcDense = 2 };

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct AttnDecodeArgs {
  const uint16_t* q;
  const uint16_t* K;
  const uint16_t* V;
  int64_t row_stride, head_stride;
  const int64_t* seq_start;
  const int32_t* ctx_len;
  const int32_t* sel_idx;
  int64_t sel_stride;
  const int32_t* sel_count;
  int32_t n_q_heads, n_kv_heads, n_ret, sink, window;
  int32_t units;           // B * n_ret (sparse) or B * n_kv_heads
  int32_t target_items;    // sparse: host hint, aim for this many work items
  int32_t min_split_blocks;  // sparse: shortest split, in blocks of 128 tokens
  int32_t split_tokens;    // local / dense: tokens per work item, fixed by the host
  int32_t n_splits;        // local / dense: work items per unit
  float scale_log2;        // softmax scale * log2(e)
  float* part;             // [items, G, kPartStride]
  uint16_t* out;
  float* lse;
  int32_t ret_heads[64];
  uint8_t is_ret[128];
  // local source only: bounded (sink + window rows) cache of the KV heads whose query heads are all local;
  // NULL = every head reads the full cache.  ring_of_kv[kv] = its index among the bounded heads, or -1.
  const uint16_t* ringK;
  const uint16_t* ringV;
  int64_t ring_row_stride, ring_head_stride;
  const int64_t* ring_seq_start;
  int8_t ring_of_kv[128];
  // selected-token source only: paged cache (NULL = contiguous sequences at seq_start)
  const int32_t* page_table;   // [B, pt_stride] pool pages
  int64_t pt_stride;
  int32_t page_shift;          // log2(page size in tokens)
  int32_t f16;                 // q, K, V and out are fp16 (else bf16)
};

template <int SRC>
__device__ __forceinline__ int unit_tokens(const AttnDecodeArgs& a, int unit) {
  if (SRC == kSrcSparse) return max(a.sel_count[unit], 0);
  const int n = a.ctx_len[unit / a.n_kv_heads];
  if (SRC == kSrcDense) return max(n, 0);
  const int s0 = min(a.sink, n);
  const int w0 = max(a.sink, n - a.window);
  return max(s0, 0) + max(0, n - w0);
}

template <bool F16 = false>
__device__ __forceinline__ void unpack8(const u32x4 v, float (&f)[8]) {
  f[0] = lo16<F16>(v.x); f[1] = hi16<F16>(v.x); f[2] = lo16<F16>(v.y); f[3] = hi16<F16>(v.y);
  f[4] = lo16<F16>(v.z); f[5] = hi16<F16>(v.z); f[6] = lo16<F16>(v.w); f[7] = hi16<F16>(v.w);
}


typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
// 16 x 16 x 32 MFMA on 16-bit operands of either format, fp32 accumulation
template <bool F16>
__device__ __forceinline__ f32x4_t mfma16(const u32x4 a, const u32x4 b, const f32x4_t c) {
  if constexpr (F16) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  else return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

template <int H>
__device__ __forceinline__ float row_share(float x) {      // every lane reads lane H of its own 16-lane row
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + H, 0xf, 0xf, false));
}

// The work items first_item, first_item + item_step, ... of a workgroup of THREADS threads, TILES tiles per wave
// in flight (alone in its launch the kernel runs 256 threads and 2 tiles: 1, 3 and 4 measured slower).
// PAGED: token position p of sequence b lives in pool row page_table[b][p >> page_shift] * page_size + p % page_size
// (rows of a bounded cache are never paged).
template <int G, int SRC, int THREADS, int TILES, bool F16 = false, bool PAGED = false>
__device__ __forceinline__ void gqa_decode_items(const AttnDecodeArgs& a, const int first_item, const int item_step,
                                                 const int item_end = -1) {
  static_assert(SRC != kSrcSparse && G >= 2 && G <= 16, "range sources, GQA groups");
  constexpr int kTile = 16;                 // tokens per MFMA tile
  constexpr int kTilesInFlight = TILES;     // 8 x 16-byte loads per lane and tile in flight
  constexpr int kAdThreads = THREADS;       // (shadows the stand-alone kernels' workgroup size)
  __shared__ float sh_m[kAdThreads / 64][G], sh_l[kAdThreads / 64][G];
  __shared__ float sh_acc[kAdThreads / 64][G][kHeadDim];

  const int ST = a.split_tokens;
  const int n_items = item_end >= 0 ? item_end : a.units * a.n_splits;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = lane >> 4, piece = lane & 15;
  const float ninf = -__builtin_huge_valf();

  for (int item = first_item; item < n_items; item += item_step) {
    const int unit = item / a.n_splits, split = item - unit * a.n_splits;
    const int b = unit / a.n_kv_heads, kvh = unit - b * a.n_kv_heads, h0 = kvh * G;
    const int n_tok = unit_tokens<SRC>(a, unit);
    const int t_begin = split * ST, t_end = min(n_tok, t_begin + ST);
    if (t_begin >= n_tok) continue;
    int s0 = 0, w0 = 0;
    if (SRC == kSrcLocal) {
      const int n = a.ctx_len[b];
      s0 = max(min(a.sink, n), 0);
      w0 = max(a.sink, n - a.window);
    }
    const int64_t seq0 = PAGED ? 0 : a.seq_start[b];
    const uint16_t* Kb = a.K + (int64_t)kvh * a.head_stride + seq0 * a.row_stride;
    const uint16_t* Vb = a.V + (int64_t)kvh * a.head_stride + seq0 * a.row_stride;
    int64_t row_stride = a.row_stride;
    const int32_t* pt = PAGED ? a.page_table + (int64_t)b * a.pt_stride : nullptr;
    const int page_mask = (1 << a.page_shift) - 1;
    if (SRC == kSrcLocal && a.ringK && a.ring_of_kv[kvh] >= 0) {
      pt = nullptr;
      // bounded cache: its first n_tok rows are exactly this unit's tokens, in some order
      const int64_t off = (int64_t)a.ring_of_kv[kvh] * a.ring_head_stride + a.ring_seq_start[b] * a.ring_row_stride;
      Kb = a.ringK + off;
      Vb = a.ringV + off;
      row_stride = a.ring_row_stride;
      s0 = n_tok;                         // logical token i is row i
    }
    auto pos_of = [&](int i) {
      const int p = SRC == kSrcLocal ? (i < s0 ? i : w0 + (i - s0)) : i;
      if (PAGED && pt) return (pt[p >> a.page_shift] << a.page_shift) | (p & page_mask);
      return p;
    };

    // B operand: column piece = head (zero beyond G), k slice grp * 8 .. + 7 of each 32-dim step
    u32x4 qB[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      qB[kk] = (u32x4){0u, 0u, 0u, 0u};
      if (piece < G) qB[kk] = *reinterpret_cast<const u32x4*>(a.q + ((int64_t)b * a.n_q_heads + h0 + piece) * kHeadDim + kk * 32 + grp * 8);
    }
    float m_run = ninf, l_run = 0.f;         // head `piece`: maximum uniform over its four lanes, sum per lane
    float acc[G][8];
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[hh][c] = 0.f;

    // the wave's tiles: base, base + 4 * 16, ...; kTilesInFlight of them per round
    const int wave_first = t_begin + wave * kTile;
    for (int base = wave_first; base < t_end; base += (kAdThreads / 64) * kTile * kTilesInFlight) {
      u32x4 kr[kTilesInFlight][4], vr[kTilesInFlight][4];
#pragma unroll
      for (int tl = 0; tl < kTilesInFlight; ++tl) {
        const int tb = base + tl * (kAdThreads / 64) * kTile;
        // K: lane (token piece, quarter grp) of the tile; rows past the end repeat the last valid one (masked below)
        const int ik = min(tb + piece, t_end - 1);
        const uint16_t* krow = Kb + (int64_t)pos_of(ik) * row_stride + grp * 8;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) kr[tl][kk] = *reinterpret_cast<const u32x4*>(krow + kk * 32);
        // V: round j, lane group grp -> token 4 * grp + j, 8 dims per lane
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int iv = min(tb + 4 * grp + j, t_end - 1);
          vr[tl][j] = *reinterpret_cast<const u32x4*>(Vb + (int64_t)pos_of(iv) * row_stride + piece * 8);
        }
      }
#pragma unroll
      for (int tl = 0; tl < kTilesInFlight; ++tl) {
        const int tb = base + tl * (kAdThreads / 64) * kTile;
        if (tb >= t_end) continue;                                   // wave-uniform
        f32x4_t S = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          S = mfma16<F16>(kr[tl][kk], qB[kk], S);
        // lane (head piece, row group grp) holds tokens tb + 4 * grp + i, i < 4
        float sc[4];
        float mx = ninf;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          sc[i] = (tb + 4 * grp + i < t_end) ? S[i] * a.scale_log2 : ninf;
          mx = fmaxf(mx, sc[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);                       // finite: the tile has a valid token
        const float corr = fast_exp2(m_run - m_new);                // 0 on the first tile (m_run = -inf)
        float pw[4];
        float ls = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          pw[i] = fast_exp2(sc[i] - m_new);                         // exp2(-inf) = 0 for masked tokens
          ls += pw[i];
        }
        l_run = l_run * corr + ls;
        m_run = m_new;
        // rescale the accumulators: head hh's factor sits in lane hh of every row
        if (__ballot(corr != 1.f) != 0ull) {
#pragma unroll
          for (int hh = 0; hh < G; ++hh) {
            const float ch = __shfl(corr, hh);
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[hh][c] *= ch;
          }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float vf[8];
          unpack8<F16>(vr[tl][j], vf);
          // probability of token 4 * grp + j for head hh: register j of lane hh of this lane's own row
          float ph[G];
          ph[0] = row_share<0>(pw[j]);
          if (G > 1) ph[1] = row_share<1>(pw[j]);
          if (G > 2) { ph[2] = row_share<2>(pw[j]); ph[3] = row_share<3>(pw[j]); }
          if (G > 4) { ph[4] = row_share<4>(pw[j]); ph[5] = row_share<5>(pw[j]); ph[6] = row_share<6>(pw[j]); ph[7] = row_share<7>(pw[j]); }
#pragma unroll
          for (int hh = 0; hh < G; ++hh)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[hh][c] = fmaf(ph[hh], vf[c], acc[hh][c]);
        }
      }
    }

    // ---- the wave's result: sums over its four lane groups (they share the head maxima), then LDS ----
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        acc[hh][c] += __shfl_xor(acc[hh][c], 16);
        acc[hh][c] += __shfl_xor(acc[hh][c], 32);
      }
    __syncthreads();   // previous item's readers are done with the LDS buffers
    if (lane < G) { sh_m[wave][lane] = m_run; sh_l[wave][lane] = l_run; }
    if (lane < 16) {
#pragma unroll
      for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int c = 0; c < 8; ++c) sh_acc[wave][hh][piece * 8 + c] = acc[hh][c];
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

// Merges the partials i0 .. i1-1 of head slot hh (of G per partial) and writes query head h of sequence b:
// 256 threads = 8 slices of 32 lanes, each lane owns 4 of the 128 output dims and walks the partials slice,
// slice + 8, ...; LDS merges the 8 slices.
__device__ __forceinline__ void merge_partials_to_out(const AttnDecodeArgs& a, int G, int hh, int b, int h, int i0, int i1) {
  __shared__ float sh_m[8], sh_l[8];
  __shared__ float sh_acc[8][kHeadDim];
  const int tid = threadIdx.x;
  const float ninf = -__builtin_huge_valf();
  const int d4 = tid & 31, slice = tid >> 5;
  float M = ninf, L = 0.f;
  float4 A = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int i = i0 + slice; i < i1; i += 8) {
    const float* p = a.part + ((int64_t)i * G + hh) * kPartStride;
    const float m = p[0], l = p[1];
    const float4 v = *reinterpret_cast<const float4*>(p + 4 + d4 * 4);
    const float Mn = fmaxf(M, m);
    if (Mn != ninf) {
      const float c0 = fast_exp2(M - Mn), c1 = fast_exp2(m - Mn);
      L = L * c0 + l * c1;
      A.x = A.x * c0 + v.x * c1; A.y = A.y * c0 + v.y * c1;
      A.z = A.z * c0 + v.z * c1; A.w = A.w * c0 + v.w * c1;
      M = Mn;
    }
  }
  if (d4 == 0) { sh_m[slice] = M; sh_l[slice] = L; }
  *reinterpret_cast<float4*>(&sh_acc[slice][d4 * 4]) = A;
  __syncthreads();
  if (tid < kHeadDim) {
    float Mt = sh_m[0];
#pragma unroll
    for (int s = 1; s < 8; ++s) Mt = fmaxf(Mt, sh_m[s]);
    float Lt = 0.f, At = 0.f;
    if (Mt != ninf) {
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const float cw = fast_exp2(sh_m[s] - Mt);
        Lt += sh_l[s] * cw;
        At += sh_acc[s][tid] * cw;
      }
    }
    const int64_t o = ((int64_t)b * a.n_q_heads + h);
    a.out[o * kHeadDim + tid] = f32_to_16(Lt > 0.f ? At / Lt : 0.f, a.f16 != 0);
    if (a.lse && tid == 0) a.lse[o] = Lt > 0.f ? (Mt + log2f(Lt)) * 0.6931471805599453f : ninf;
  }
}

struct RingSource {       // bounded cache of the all-local KV heads (see kv_ring.hip)
  const void* K;
  const void* V;
  int64_t row_stride, head_stride;
  const int64_t* seq_start;
};
struct PageSource {       // K and V are pools of pages: sequence b's page i is pool page table[b * stride + i]
  const int32_t* table;
  int64_t stride;
  int32_t page_size;
};
// checks a page table's shape for contexts of up to max_ctx tokens and gives log2(page_size)
int32_t check_pages(const char* who, const PageSource* pages, int64_t max_ctx, int* page_shift);

// attn_decode.hip: argument checks + plan of a range-source (local / dense) decode call, without the launch
int32_t decode_range_prepare(const char* who, bool dense, const rtp_layer_desc* L, const void* q, const void* K,
                             const void* V, int64_t row_stride, int64_t head_stride, const int64_t* seq_start,
                             const int32_t* ctx_len, int32_t B, int64_t max_ctx, void* out, float* lse, void* ws,
                             size_t ws_bytes, const RingSource* ring, AttnDecodeArgs* args, int* grid, bool* launch,
                             const PageSource* pages = nullptr);
int32_t decode_range_attn(const char* who, bool dense, const rtp_layer_desc* L, const void* q, const void* K,
                          const void* V, int64_t row_stride, int64_t head_stride, const int64_t* seq_start,
                          const int32_t* ctx_len, int32_t B, int64_t max_ctx, void* out, float* lse, void* ws,
                          size_t ws_bytes, hipStream_t s, const PageSource* pages = nullptr);
size_t decode_range_ws(bool dense, const rtp_layer_desc* L, int32_t B, int64_t max_ctx);

}  // namespace rtp
