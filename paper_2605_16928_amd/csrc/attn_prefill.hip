// Prefill-time attention on bf16 MFMA: rtp_local_attn / rtp_dense_attn with q_start != NULL, and the
// p >= 1 case of rtp_sparse_attn_prefill (the paper's prefill rule: retrieval heads dense, local heads
// sink + window; Sec. 3.2 and Sec. 4.2).
//
// Flash-style tiling written for the CDNA MFMA register layout.  A wave owns 32 queries and computes
// the TRANSPOSED score tile  S^T = K Q^T  with v_mfma_f32_32x32x16_bf16: the K tile is the A operand
// (read from LDS, row-major, 16-byte reads), Q^T the B operand (held in registers for the whole
// kernel).  In the accumulator layout a lane then holds 16 keys of ONE query (column = lane % 32), so
// the online-softmax state (running max, running sum, rescale factor) is a per-lane scalar and the
// only cross-lane traffic is one exchange with lane ^ 32 per tile.  The probabilities stay in place:
// the accumulator registers, rounded to bf16, ARE the B operand of  O^T = V^T P^T  (the key order
// inside the contraction is permuted identically for both operands), so P never touches LDS.  Only V
// has to be transposed, once per tile, on its way into LDS.
//
// Workgroup = 4 waves = 128 queries of one (sequence, head); key tiles of 64; heads of one KV group
// are adjacent in the grid so that they meet in L2; late (long) query tiles are scheduled first.
#include "common.h"

#include <algorithm>
#include <type_traits>
#include <vector>

namespace rtp {

constexpr int kPfThreads = 256;
constexpr int kPfQ = 128;          // queries per workgroup
constexpr int kPfK = 64;           // keys per tile
constexpr int kKsStride = 136;     // bf16 per K row in LDS   (128 + 8: rows start 4 banks apart)
constexpr int kVtStride = 72;      // bf16 per V^T row in LDS (64 + 8)
constexpr int kPfPart = kHeadDim + 4;   // floats per partial row: max, sum, 2 pad, unnormalised output[128]

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct PrefillArgs {
  const uint16_t* q;
  const uint16_t* K;
  const uint16_t* V;
  int64_t row_stride, head_stride;
  const int64_t* seq_start;     // NULL: one sequence starting at token 0
  const int32_t* q_start;       // NULL: q_start_host
  int64_t q_start_host;
  int32_t n_q, n_q_heads, n_kv_heads, sink, window;
  float scale, scale_log2;
  uint16_t* out;
  float* lse;
  int32_t n_heads;
  uint8_t heads[128];           // query heads this launch computes
  int32_t n_splits;             // dense mode: key range of every query tile cut into this many parts
  float* part;                  // n_splits > 1: partial results [split, head slot, query, kPfPart]
  // sparse mode only (per-query top-p over the indexer scores):
  const uint16_t* qI;           // bf16 [n_ret, n_q, 16]
  const uint16_t* kI;           // bf16 [n_ret, >= pos0 + n_q, 16]
  int64_t kI_head_stride;
  float p, index_scale;
  float* tau;                   // optional [n_ret, n_q]
  int32_t* count;
  float* mass;
  float* sel_thr;               // [n_ret, n_q]: a candidate is kept iff its raw index product is >= this
  int32_t f16;                  // q, K, V and out are fp16 (else bf16)
  // selecting mode: which key tiles can hold a kept pair at all
  float* tile_max;              // [n_ret * ceil(n_q / 32), n_t64]: largest raw index product of a 32-query group in a 64-key tile
  int32_t n_t64;                // row length of tile_max
  int32_t* act_list;            // [n_ret, ceil(n_q / 256), n_t64]: the 64-key tiles a 256-query tile has to visit, ascending
  int32_t* act_count;           // [n_ret, ceil(n_q / 256)]
  int32_t* act_range;           // {longest list, shortest list} of the launch (the search resets, the list kernel updates)
  int32_t n_splits_even;        // key ranges per query tile when the lists are about equally long
};

// Key ranges a selecting launch behind a threshold search really uses: the grid is sized for lists that differ
// wildly in length (many short ranges); when the shortest list is at least half the longest there is nothing to
// even out and the few long ranges of the dense rule are cheaper (fewer partials to write and merge).
__device__ __forceinline__ int listed_splits(const PrefillArgs& a) {
  const int longest = a.act_range[0], shortest = a.act_range[1];
  return (2 * shortest >= longest) ? min(a.n_splits_even, a.n_splits) : a.n_splits;
}

enum { kModeDense = 0, kModeLocal = 1, kModeSparse = 2 };
// Per-query threshold search of the sparse mode: a score s is mapped to the integer
// q = floor((M - s) * 2^17) (M = row maximum; q clamps at 2^21 - 1, i.e. 16 below the maximum) and
// the threshold is the smallest q whose cumulative mass from q = 0 reaches p * Z, found digit by
// digit in base 128 (bin widths 1/8, 1/1024, 1/131072 in score units).  Masses are summed in fp64.
constexpr int kSelBins = 128;
constexpr float kSelScale = 131072.0f;
constexpr int kSelQMax = (1 << 21) - 1;
constexpr int kTileHalfs = kPfK * kKsStride + kHeadDim * kVtStride;   // bf16 elements of one staged K + V^T tile
constexpr int kSmemDense = kTileHalfs * 2 * 2;                        // two buffers
constexpr int kSelListCap = 16;      // entries per lane: what one tile can add (lists are emptied after every tile)
constexpr int kSelMfma = 2;          // index-score MFMAs of a wave in flight (the SIMD's other wave covers their latency)
constexpr int kSelRing = 4;          // index-key tiles in flight per wave during the threshold search

__device__ __forceinline__ int sel_q_of_t(float tt) {       // tt = M - s >= 0
  return (int)fminf(tt * kSelScale, (float)kSelQMax);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const f32x2 f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}
// The attention tensors' element type is a template flag of the kernels (F16 = IEEE binary16, else bf16): two
// floats rounded (nearest even) and packed, and the 32 x 32 x 16 MFMA on 16-bit operands with fp32 accumulation.
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
template <bool F16> __device__ __forceinline__ uint32_t pack16(float a, float b) {
  if constexpr (F16) {
    const f32x2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2));
  } else {
    return pack_bf16(a, b);
  }
}
template <bool F16> __device__ __forceinline__ f32x16 mfma32(const u32x4 a, const u32x4 b, const f32x16 c) {
  if constexpr (F16) return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int MODE, bool F16 = false>
__global__ __launch_bounds__(kPfThreads, 2) void flash_prefill_kernel(const PrefillArgs a) {
  constexpr bool LOCAL = MODE == kModeLocal;
  static_assert(MODE == kModeDense || MODE == kModeLocal, "the selecting mode lives in the wide kernel");
  __shared__ __attribute__((aligned(16))) unsigned char smem[kSmemDense];
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;
  const int h = a.heads[blockIdx.x];
  const int n_splits = LOCAL ? 1 : a.n_splits;
  const int b = blockIdx.z / n_splits;
  const int split = blockIdx.z - b * n_splits;
  const int t0 = ((int)gridDim.y - 1 - (int)blockIdx.y) * kPfQ;
  const int kvh = h / (a.n_q_heads / a.n_kv_heads);
  const int pos0 = a.q_start ? a.q_start[b] : (int)a.q_start_host;
  const int64_t tok0 = a.seq_start ? a.seq_start[b] : 0;
  const float ninf = -__builtin_huge_valf();

  // ---- this lane's query (column r of the wave's 32) ----
  const int t = t0 + wave * 32 + r;
  const bool qok = t < a.n_q;
  const int m = pos0 + t;
  const int64_t qrow = (((int64_t)b * a.n_q + t) * a.n_q_heads + h) * kHeadDim;
  u32x4 qreg[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    qreg[kk] = qok ? *reinterpret_cast<const u32x4*>(a.q + qrow + kk * 16 + g * 8) : (u32x4){0u, 0u, 0u, 0u};
  }

  // ---- key tiles this workgroup needs ----
  const int m_lo = pos0 + t0;
  const int m_hi = pos0 + min(t0 + kPfQ, a.n_q) - 1;
  const int kt_end = m_hi / kPfK;                       // inclusive
  int kt_w0 = 0, ks_end = 0;
  if (LOCAL) {
    const int lo = max(a.sink, m_lo - a.window + 1);
    kt_w0 = lo / kPfK;
    ks_end = min((a.sink + kPfK - 1) / kPfK, kt_w0);    // sink tiles not already inside the band
  }
  const int n_tiles = ks_end + (kt_end - kt_w0 + 1);

  const uint16_t* Kg = a.K + (int64_t)kvh * a.head_stride + tok0 * a.row_stride;
  const uint16_t* Vg = a.V + (int64_t)kvh * a.head_stride + tok0 * a.row_stride;

  f32x16 O[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) O[db][i] = 0.f;
  float mrow = ninf, lrow = 0.f;
  const float c = a.scale_log2;
  const int m_wave_lo = pos0 + t0 + wave * 32;
  const int m_wave_hi = pos0 + min(t0 + wave * 32 + 32, a.n_q) - 1;

  // ---- tile movers -------------------------------------------------------------------------------
  // K: thread handles chunks idx = i * 256 + tid -> (key idx / 16, 16-byte chunk idx % 16).
  // V: thread handles keys wave * 16 + (lane / 16) * 4 + {0..3} at chunk lane % 16, so that it can
  //    transpose a 4 x 8 block in registers and write 8-byte runs of V^T.
  u32x4 kr[4], vr[4];
  const int v_ck = lane & 15;
  const int v_key0 = wave * 16 + (lane >> 4) * 4;
  auto load_tile = [&](int n0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = i * kPfThreads + tid;
      const int n = n0 + (idx >> 4);
      kr[i] = (u32x4){0u, 0u, 0u, 0u};
      if (n <= m_hi) kr[i] = *reinterpret_cast<const u32x4*>(Kg + (int64_t)n * a.row_stride + (idx & 15) * 8);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = n0 + v_key0 + i;
      vr[i] = (u32x4){0u, 0u, 0u, 0u};
      if (n <= m_hi) vr[i] = *reinterpret_cast<const u32x4*>(Vg + (int64_t)n * a.row_stride + v_ck * 8);
    }
  };
  // V^T row d holds the tile's 64 keys in the order the PV MFMAs consume them: inside every 32-key
  // block, position = tt*16 + g*8 + hi*4 + j for key = tt*16 + hi*8 + g*4 + j, so the 8 keys a lane
  // needs for one MFMA are one 16-byte read.  16-byte units are XOR-swizzled with bits of d so that
  // the transposing 8-byte writes spread over the banks.
  auto store_tile = [&](int buf) {
    uint16_t* ks = Ks + buf * (kTileHalfs);
    uint16_t* vt = ks + kPfK * kKsStride;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = i * kPfThreads + tid;
      *reinterpret_cast<u32x4*>(&ks[(idx >> 4) * kKsStride + (idx & 15) * 8]) = kr[i];
    }
    const int pos0v = (v_key0 & 32) + ((v_key0 >> 4) & 1) * 16 + ((v_key0 >> 2) & 1) * 8 + ((v_key0 >> 3) & 1) * 4;
    const uint32_t w0[4] = {vr[0].x, vr[0].y, vr[0].z, vr[0].w};
    const uint32_t w1[4] = {vr[1].x, vr[1].y, vr[1].z, vr[1].w};
    const uint32_t w2[4] = {vr[2].x, vr[2].y, vr[2].z, vr[2].w};
    const uint32_t w3[4] = {vr[3].x, vr[3].y, vr[3].z, vr[3].w};
#pragma unroll
    for (int aa = 0; aa < 4; ++aa) {
#pragma unroll
      for (int hl = 0; hl < 2; ++hl) {
        const int d = v_ck * 8 + aa * 2 + hl;
        const uint32_t sel = hl ? 0x07060302u : 0x05040100u;      // high / low halves of (second, first)
        const u32x2 val = (u32x2){__builtin_amdgcn_perm(w1[aa], w0[aa], sel), __builtin_amdgcn_perm(w3[aa], w2[aa], sel)};
        const int off = d * kVtStride + ((((pos0v >> 3) ^ ((d >> 4) & 7))) << 3) + (pos0v & 7);
        *reinterpret_cast<u32x2*>(&vt[off]) = val;
      }
    }
  };

  // ---- one key tile: S^T = K Q^T, online softmax, O^T += V^T P^T -----------------------------------
  auto compute_tile = [&](int buf, int n0) {
    const uint16_t* ks = Ks + buf * (kTileHalfs);
    const uint16_t* vt = ks + kPfK * kKsStride;
    f32x16 S[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) S[kb][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const u32x4 ka = *reinterpret_cast<const u32x4*>(&ks[(kb * 32 + r) * kKsStride + kk * 16 + g * 8]);
        S[kb] = mfma32<F16>(ka, qreg[kk], S[kb]);
      }
    }
    // interior tiles (every key visible to every query of the wave) skip the mask arithmetic
    const bool edge = (n0 + kPfK - 1 > m_wave_lo) || (LOCAL && n0 <= m_wave_hi - a.window);
    float mx = ninf;
    if (edge) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int n = n0 + kb * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
          bool ok = qok && n <= m;
          if (LOCAL) ok = ok && (n < a.sink || n > m - a.window);
          S[kb][i] = ok ? S[kb][i] : ninf;
          mx = max_nn(mx, S[kb][i]);
        }
      }
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = max_nn(mx, S[kb][i]);
    }
    mx = max_nn(mx, __shfl_xor(mx, 32));
    const float mnew = fmaxf(mrow, mx);
    uint32_t P[2][8];
    if (mnew == ninf) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 8; ++i) P[kb][i] = 0u;
    } else {
      const float mc = mnew * c;
      float lsum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const float p0 = fast_exp2(fmaf(S[kb][i], c, -mc));
          const float p1 = fast_exp2(fmaf(S[kb][i + 1], c, -mc));
          lsum += p0 + p1;
          P[kb][i >> 1] = pack16<F16>(p0, p1);
        }
      }
      const float corr = fast_exp2((mrow - mnew) * c);     // 1 where the maximum did not move
      lrow = lrow * corr + lsum;
      if (__ballot(mnew > mrow) != 0ull) {                   // rescale only when some query's maximum grew
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) O[db][i] *= corr;
      }
      mrow = mnew;
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const u32x4 pb = (u32x4){P[kb][4 * tt], P[kb][4 * tt + 1], P[kb][4 * tt + 2], P[kb][4 * tt + 3]};
        const int pos8 = kb * 4 + tt * 2 + g;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const int d = db * 32 + r;
          const u32x4 va = *reinterpret_cast<const u32x4*>(&vt[d * kVtStride + ((pos8 ^ ((d >> 4) & 7)) << 3)]);
          O[db] = mfma32<F16>(va, pb, O[db]);
        }
      }
    }
  };

  {
    // Software pipeline: the global loads of tile it+1 are in flight while tile it is computed from
    // the other LDS buffer; one barrier per tile.
    auto tile_n0 = [&](int it) { return (it < ks_end ? it : kt_w0 + (it - ks_end)) * kPfK; };
    const int it_lo = (int)((int64_t)n_tiles * split / n_splits);
    const int it_hi = (int)((int64_t)n_tiles * (split + 1) / n_splits);
    if (it_lo < it_hi) {
      load_tile(tile_n0(it_lo));
      store_tile(it_lo & 1);
      __syncthreads();
    }
    for (int it = it_lo; it < it_hi; ++it) {
      const bool has_next = it + 1 < it_hi;
      if (has_next) load_tile(tile_n0(it + 1));
      compute_tile(it & 1, tile_n0(it));
      if (has_next) store_tile((it + 1) & 1);
      __syncthreads();
    }
  }

  // ---- normalise and store ----
  const float ltot = lrow + __shfl_xor(lrow, 32);
  if (!qok) return;
  if (n_splits > 1) {
    // partial result of this key range: merged by prefill_combine_kernel
    float* prow = a.part + (((int64_t)split * a.n_heads + blockIdx.x) * a.n_q + t) * kPfPart;
    if (g == 0) { prow[0] = mrow; prow[1] = ltot; }
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4)
        *reinterpret_cast<float4*>(prow + 4 + db * 32 + i4 * 8 + g * 4) =
            make_float4(O[db][i4 * 4], O[db][i4 * 4 + 1], O[db][i4 * 4 + 2], O[db][i4 * 4 + 3]);
    return;
  }
  const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
  uint16_t* orow = a.out + qrow;
#pragma unroll
  for (int db = 0; db < 4; ++db) {
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const u32x2 w = (u32x2){pack16<F16>(O[db][i4 * 4] * inv, O[db][i4 * 4 + 1] * inv),
                              pack16<F16>(O[db][i4 * 4 + 2] * inv, O[db][i4 * 4 + 3] * inv)};
      *reinterpret_cast<u32x2*>(orow + db * 32 + i4 * 8 + g * 4) = w;
    }
  }
  if (a.lse && g == 0) {
    a.lse[((int64_t)b * a.n_q + t) * a.n_q_heads + h] = ltot > 0.f ? mrow * a.scale + logf(ltot) : ninf;
  }
}

// ---- per-query top-p threshold search (selecting mode of rtp_sparse_attn_prefill) ---------------------
// Sec. 3.2, S = Top-P(s(m, .), p), applied to every prefill query over its causal candidates n <= m.
//
// 32 queries of one retrieval head form a group, whose waves sweep the index keys 0..m up to four times:
// sweep 0 finds the row maximum M; sweeps 1-3 histogram the softmax mass over the integer
// q = floor(min((M - s) * 2^17, 2^21 - 1)) one base-128 digit at a time (all candidates in sweep 1, only
// the members of the digit prefix found so far in sweeps 2 and 3) and scan the histogram from the top of
// the score range for the bin where the cumulative mass reaches p * Z.  The index-score tile of 32 keys
// x 32 queries is ONE MFMA (K = 16) in the transposed layout, so a lane holds 16 keys of its own query.
//
// What makes the sweeps cheap:
//  - index keys are fetched kSelRing tiles ahead into registers (two waves share a SIMD: not enough to
//    hide a load's latency by themselves);
//  - interior tiles (every key a candidate of every query of the wave) carry no mask arithmetic;
//  - the histogram of a group is laid out [bin][query]: the 32 queries of a wave sit in 32 different
//    LDS bank pairs whatever their bins, so an fp64 LDS atomic of the wave sees only the two-way
//    conflict between the two lanes of one query;
//  - q is a monotone function of the raw MFMA product x (s = x * index_scale), so "q lies in the digit
//    prefix" is an interval of x.  Its two end points are found once per query and sweep by bisection
//    over the float bit patterns, evaluating the very expression that defines q -- the comparisons of
//    sweeps 2, 3 and of the attention kernel are then exact restatements of that definition, two
//    (one) compare per pair, and only members do any further arithmetic;
//  - sweep 0 records the largest product of the group in every pair of key tiles, and sweeps 2 and 3 -- whose
//    members all lie at or above a known bound -- pass over the pairs that cannot hold one.
// t = M - x * index_scale as ONE fused operation (one rounding): the definition every sweep, the end points
// of the digit intervals and the final threshold share
__device__ __forceinline__ float sel_t(float M, float x, float index_scale) { return __builtin_fmaf(-x, index_scale, M); }

// Smallest float x (as a raw product) with sel_t(M, x) < bound; -inf if every finite x qualifies.
// sel_t is non-increasing in x, so the predicate flips once from false to true.
__device__ __forceinline__ float sel_first_below(float M, float index_scale, float bound) {
  if (bound == __builtin_huge_valf()) return -__builtin_huge_valf();
  uint32_t lo = float_key(-__builtin_huge_valf()), hi = float_key(__builtin_huge_valf());
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if (sel_t(M, key_float(mid), index_scale) < bound) hi = mid; else lo = mid + 1;
  }
  return key_float(lo);
}

//
// KS waves share one group of 32 queries and split its key range between them; a workgroup is eight waves -- two
// per SIMD, so that one wave's vector instructions issue under the other's latencies -- i.e. 8 / KS groups.  The
// waves of a group add into ONE histogram (LDS atomics; 32 KB per group); the per-lane member lists of sweeps 2
// and 3 hold one tile's worth of entries (16) and are emptied after every tile that added one.  All waves of the
// workgroup meet at barriers around every scan, so the phases are uniform over the workgroup.
// The library launches KS = 8, one group per workgroup: on score laws that keep thousands of tokens per query it
// runs as fast as two or four groups per workgroup (25.6 ms against 25.7 and 25.6 on the last 8192-query chunk of
// a 1,048,576-token context), and when a few queries of a chunk have their threshold deep in the background
// while the others' sweeps 2 and 3 visit a handful of tiles, short workgroups in four times the number let the
// dispatcher even the load out (19.0 ms against 24.1).
//
// A threshold inside the open-ended last coarse bin (candidates 15.875 or more below the row maximum) is not
// taken as "keep everything": the workgroup repeats sweep 1 with the reference lowered by 15.875 for the queries
// concerned -- the mass above that bin is already known, the bin's members are spread over 128 new coarse bins --
// until the threshold bin is an ordinary one (or 24 rounds, about 380 score units, are used up).
constexpr int kSelThreads = 512;
constexpr float kSelLumpT = 15.875f;               // (kSelBins - 1) / 8: where the open-ended bin starts
constexpr double kSelLumpScale = 7843180.797657975;   // exp(15.875)
constexpr int kSelMaxRounds = 24;

template <int KS>
__global__ __launch_bounds__(kSelThreads, 2) void prefill_select_kernel(const PrefillArgs a) {
  constexpr int NW = kSelThreads / 64;                             // waves per workgroup
  constexpr int NG = NW / KS;                                      // query groups per workgroup
  constexpr int kSelQ = 32 * NG;                                   // queries per workgroup
  static_assert(NG >= 1 && NG <= 4, "at most four histograms fit");
  __shared__ double hist_all[NG][kSelBins][32];                    // 32 KB per group
  __shared__ float list_all[NW][kSelListCap][64];                  // per-lane member lists of sweeps 2 and 3 (32 KB)
  float (*max_all)[32] = reinterpret_cast<float (*)[32]>(&list_all[0][0][0]);   // sweep 0: the waves' row maxima
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;
  // Workgroups go round-robin over the chip's 8 dies, each with its own L2.  The 1-D grid is decoded so
  // that a die works on ONE head (8 / n_heads dies per head): all its waves then stream the same index
  // keys and meet in that L2.
  int j, qtile;
  const int n_qtiles = (a.n_q + kSelQ - 1) / kSelQ;
  if (a.n_heads <= 8 && 8 % a.n_heads == 0) {
    const int per_head = 8 / a.n_heads;                            // dies per head
    const int die = blockIdx.x & 7, k = blockIdx.x >> 3;
    j = die / per_head;
    qtile = k * per_head + die % per_head;
  } else {
    j = blockIdx.x % a.n_heads;
    qtile = blockIdx.x / a.n_heads;
  }
  if (blockIdx.x == 0 && tid == 0) {                               // for prefill_active_tiles_kernel, which runs next
    a.act_range[0] = 0;
    a.act_range[1] = 0x7fffffff;
  }
  if (qtile >= n_qtiles) return;                                   // (the whole workgroup)
  const int t0 = (n_qtiles - 1 - qtile) * kSelQ;                   // long rows first
  const int qgroup = wave / KS, part = wave - qgroup * KS;         // this wave's queries and its share of their keys
  const int tw = t0 + qgroup * 32;                                 // first query of the group
  const bool idle = tw >= a.n_q;                                   // no query in this group (the wave still goes to the barriers)
  const int pos0 = (int)a.q_start_host;
  const int t = tw + r;
  const bool qok = t < a.n_q;
  const int m = pos0 + t;
  const float ninf = -__builtin_huge_valf(), pinf = __builtin_huge_valf();
  const float cs = a.index_scale;
  const uint16_t* kIg = a.kI + (int64_t)j * a.kI_head_stride;
  u32x4 qIreg = (u32x4){0u, 0u, 0u, 0u};
  if (qok) qIreg = *reinterpret_cast<const u32x4*>(a.qI + ((int64_t)j * a.n_q + t) * kIndexDim + g * 8);
  const int n_rows = pos0 + a.n_q;                                 // index-key rows that exist
  const int m_wave_lo = pos0 + tw;
  const int m_wave_hi = pos0 + min(tw + 32, a.n_q) - 1;
  const bool wave_partial = tw + 32 > a.n_q;
  const int n_tiles = idle ? 0 : m_wave_hi / 32 + 1;
  const int n_interior = (wave_partial || idle) ? 0 : (m_wave_lo + 1) / 32;  // tiles with nb + 31 <= m_wave_lo
  double (*hist)[32] = hist_all[qgroup];
  float (*lst)[64] = list_all[wave];
  // this group's row of the tile-maximum table: written in sweep 0 (one entry per pair of key tiles, i.e. per 64
  // keys), read in sweeps 2 and 3, whose members all lie at or above x_lo -- a tile pair whose maximum is below
  // every query's x_lo holds none.  Sweep 3 replaces the entries of the pairs it visits by +inf (some query of
  // the group has a product at or above its own x_lo there, so it may keep a key) or -inf (none can); the pairs
  // it skips keep a maximum below every x_lo.  The attention launch's tile lists are built from the result.
  float* tmx = a.tile_max + ((int64_t)j * ((a.n_q + 31) / 32) + (idle ? 0 : tw / 32)) * a.n_t64;
  float xlo_wave = ninf;            // smallest x_lo over the wave's queries
  float xlo_wave_top = ninf;        // and the largest
  bool reach_known = false;         // sweep 3: the tile in hand is certain to hold a product at or above its query's x_lo
  int n_looked = 0, n_needed = 0;   // sweep 3: tile pairs whose reach was worked out, and those found within reach
  int lcnt = 0;                     // entries in this lane's member list
  const uint32_t lst_base = (uint32_t)(size_t)(__attribute__((address_space(3))) float*)&lst[0][lane];

  auto load_k = [&](int tile) {
    const int nrow = min(tile * 32 + r, n_rows - 1);               // rows past the chunk are causally masked anyway
    return *reinterpret_cast<const u32x4*>(kIg + (int64_t)nrow * kIndexDim + g * 8);
  };
  // the group's waves clear their histogram together (followed by a barrier at the call sites)
  auto zero_hist = [&]() {
    double* h = &hist[0][0];
    for (int i = part * 64 + lane; i < kSelBins * 32; i += KS * 64) h[i] = 0.0;
  };
  // One candidate's mass into bin `bin` of this lane's query.
  auto add_mass = [&](int bin, float tt) {
    const float wgt = fast_exp2(tt * -1.4426950408889634f);        // exp(s - M)
    atomicAdd(&hist[bin][r], (double)wgt);
  };

  float selM = ninf;                // the query's reference: its row maximum, lowered by 15.875 per repeat of sweep 1
  float selM8 = ninf;               // 8 * selM and 8 * index_scale for sweep 1
  const float cs8 = cs * 8.0f;
  float x_lo = ninf, x_top = pinf;  // sweeps 2, 3: members of the prefix have x_lo <= x <= x_top
  int shift = 0;
  float mxs[kSelMfma];
#pragma unroll
  for (int u = 0; u < kSelMfma; ++u) mxs[u] = ninf;

  // Weighs the listed members of every lane: lane-private lists, so the only cross-lane step is the
  // loop bound.
  auto drain_list = [&]() {
    for (int k = 0; __ballot(k < lcnt) != 0ull; ++k) {
      if (k < lcnt) {
        const float tt = sel_t(selM, lst[k][lane], cs);
        add_mass((sel_q_of_t(tt) >> shift) & (kSelBins - 1), tt);
      }
    }
    lcnt = 0;
  };

  // What one tile contributes in phase PH (0: maximum, 1: all candidates, 4: the candidates at or below the
  // lowered reference of a repeated sweep 1, 2 / 3: members of the digit prefix): SI = its 32 x 32 index
  // products, nb = its first key.
  auto tile_work = [&](auto PH, auto EDGE, const f32x16& SI, int nb, float& mxacc) -> float {
    constexpr int phase = decltype(PH)::value;
    constexpr bool edge = decltype(EDGE)::value;
    if (phase == 0) {
      // scaling by a positive constant is monotone, so the maximum is taken on the raw products
      float v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int n = nb + (i >> 2) * 8 + g * 4 + (i & 3);
        v[i] = (!edge || (qok && n <= m)) ? SI[i] : ninf;
      }
#pragma unroll
      for (int st = 8; st > 0; st >>= 1)
#pragma unroll
        for (int i = 0; i < st; ++i) v[i] = max_nn(v[i], v[i + st]);
      mxacc = fmaxf(mxacc, v[0]);
      return v[0];
    } else if (phase == 1 || phase == 4) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int n = nb + (i >> 2) * 8 + g * 4 + (i & 3);
        // 8 * (M - x * scale) straight from 8 M and 8 * scale: scaling by a power of two commutes with both
        // roundings, so this IS 8 * sel_t(M, x, scale), one multiplication less per pair
        const float tt8 = sel_t(selM8, SI[i], cs8);
        // a repeated sweep takes the candidates at or below the lowered reference only (the others were
        // counted above the open-ended bin); a query that does not repeat has reference -inf and takes none
        const bool cand = (!edge || (qok && n <= m)) && (phase == 1 || tt8 >= 0.f);
        if (cand) {
          // first digit of q: floor(min(tt * 2^17, 2^21 - 1)) >> 14 == floor(min(tt * 8, (2^21 - 1) / 2^14))
          const int bin = (int)fminf(tt8, 127.99993896484375f);
          // exp(s - M) = exp2(tt * -log2(e)); the constant carries the 1/8, again exactly
          atomicAdd(&hist[bin][r], (double)fast_exp2(tt8 * -0.18033688011112042f));
        }
      }
    } else {
      // Members of the digit prefix (about one pair in a hundred in sweep 2, one in ten thousand in
      // sweep 3) are only noted here -- their raw product goes to the lane's list -- and weighed
      // with all lanes busy (drain_list); weighing them where they turn up would run the exponential
      // and the atomic for one or two active lanes at a time.
      // Membership x_lo <= x <= x_top is one median and one comparison on the vector ALU (going through
      // scalar condition registers costs a vector-to-scalar hand-off per pair).  Appending is branch-free:
      // every pair writes its product at the list's end, members advance the end.  Sweep 3 first counts the
      // tile's members and skips the appends when the whole wave has none (nearly always).
      auto member = [&](int i) {
        const int n = nb + (i >> 2) * 8 + g * 4 + (i & 3);
        const bool in = __builtin_amdgcn_fmed3f(SI[i], x_lo, x_top) == SI[i];
        return edge ? (in && qok && n <= m) : in;
      };
      bool go = true;
      float reach = 0.f;
      if (phase == 3) {
        // does any lane have a member in this tile?  The comparisons' lane masks are OR-ed on the scalar side
        // (no vector instruction beyond the median and the comparison per pair)
        uint64_t any = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) any |= __ballot(member(i));
        go = any != 0ull;
        // can some query of the wave keep a key of this tile?  Its final threshold is at or above x_lo, so a
        // tile whose largest visible product is below x_lo for every query holds no kept pair
        reach = 1.f;
        if (!reach_known) {
        float v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int n = nb + (i >> 2) * 8 + g * 4 + (i & 3);
          v[i] = (!edge || (qok && n <= m)) ? SI[i] : ninf;
        }
#pragma unroll
        for (int st = 8; st > 0; st >>= 1)
#pragma unroll
          for (int i = 0; i < st; ++i) v[i] = max_nn(v[i], v[i + st]);
        const float top = v[0];
        reach = __ballot(top >= x_lo) != 0ull ? 1.f : 0.f;
        }
      }
      if (go) {
        // The list holds 16 entries per lane; a half tile adds at most 8, so it is emptied when some lane holds
        // more than 8 before a half tile starts.  The list's end travels as an LDS address.
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          if (__ballot(lcnt > kSelListCap - 8) != 0ull) drain_list();
          uint32_t end = lst_base + (uint32_t)lcnt * 256u;
#pragma unroll
          for (int i = hf * 8; i < hf * 8 + 8; ++i) {
            *reinterpret_cast<float __attribute__((address_space(3)))*>(end) = SI[i];
            end += member(i) ? 256u : 0u;
          }
          lcnt = (int)((end - lst_base) >> 8);
        }
      }
      return reach;
    }
    return 0.f;
  };

  // One sweep over the tiles [tile_begin, tile_end) in rounds of 2 * kSelRing: two groups of index-key
  // registers alternate, each refilled (for two groups ahead) as soon as its MFMAs have read it, so a
  // load has a whole group's arithmetic to land in; the kSelRing MFMAs of a group are issued together and
  // their latency hides behind one another.  No tail test: the interior range is a whole number of
  // rounds, and in the edge range a tile past the last one holds only keys n > m, which the causal mask drops.
  // LOOK (sweeps 2 and 3): consult the maximum table pair by pair -- skip what cannot hold a member, and in sweep 3
  // note which pairs a query can keep a key in.  Without it the sweep is the plain streaming one, which is what a
  // stretch where nearly every pair can hold a member gets (looking would cost more than it saves there; the
  // pairs keep their maxima in the table, which is the conservative answer).
  auto sweep = [&](auto PH, auto EDGE, auto LOOK, int tile_begin, int tile_end) {
    if (tile_begin >= tile_end) return;
    constexpr int phase_ = decltype(PH)::value;
    constexpr bool kSkip = (phase_ == 2 || phase_ == 3) && decltype(LOOK)::value;
    if (!kSkip) reach_known = true;
    static_assert(kSelMfma == 2, "a batch of MFMAs is one 64-key tile of the maximum table");
    u32x4 ringA[kSelRing], ringB[kSelRing];
    float tmA[kSelRing / 2], tmB[kSelRing / 2];                    // the table entries of the tile pairs in the rings
#pragma unroll
    for (int u = 0; u < kSelRing; ++u) {
      ringA[u] = load_k(tile_begin + u);
      ringB[u] = load_k(tile_begin + kSelRing + u);
    }
    if (kSkip) {
#pragma unroll
      for (int u = 0; u < kSelRing / 2; ++u) {
        tmA[u] = tmx[(tile_begin >> 1) + u];
        tmB[u] = tmx[((tile_begin + kSelRing) >> 1) + u];
      }
    }
    auto group = [&](u32x4 (&ring)[kSelRing], float (&tm)[kSelRing / 2], int first) {
#pragma unroll
      for (int hb = 0; hb < kSelRing; hb += kSelMfma) {            // kSelMfma MFMAs in flight at a time
        // no member possible in this pair of tiles: only the prefetches for two groups ahead are issued
        bool skip = false;
        if (kSkip) {
          const float pair_max = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(tm[hb / 2])));
          skip = pair_max < xlo_wave;
          // a maximum at or above EVERY query's x_lo is at or above its own query's: no need to look
          reach_known = pair_max >= xlo_wave_top;
          tm[hb / 2] = tmx[((first + 2 * kSelRing + hb) >> 1)];
        }
        if (skip) {
#pragma unroll
          for (int u = 0; u < kSelMfma; ++u) ring[hb + u] = load_k(first + 2 * kSelRing + hb + u);
          continue;
        }
        f32x16 SI[kSelMfma];
#pragma unroll
        for (int u = 0; u < kSelMfma; ++u) {
#pragma unroll
          for (int i = 0; i < 16; ++i) SI[u][i] = 0.f;
          SI[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ring[hb + u]),
                                                          __builtin_bit_cast(bf16x8, qIreg), SI[u], 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kSelMfma; ++u) ring[hb + u] = load_k(first + 2 * kSelRing + hb + u);
        float tmax = ninf;
#pragma unroll
        for (int u = 0; u < kSelMfma; ++u) {
          __builtin_amdgcn_sched_barrier(0);       // one tile at a time: hoisting four tiles' operands runs out of registers
          tmax = fmaxf(tmax, tile_work(PH, EDGE, SI[u], (first + hb + u) * 32, mxs[u]));
        }
        if (phase_ == 0) {                         // the pair's maximum over the wave's 32 queries x 64 keys
          const float wm = wave_max_f32(tmax);
          if (lane == 0) tmx[(first + hb) >> 1] = wm;
        }
        // the last sweep knows better than the maximum: can one of the wave's queries keep a key of the pair?
        // (a pair known to reach keeps its maximum, which says the same)
        if (phase_ == 3 && !reach_known) {
          n_looked += 1;
          n_needed += tmax > 0.f ? 1 : 0;
          if (lane == 0) tmx[(first + hb) >> 1] = tmax > 0.f ? pinf : ninf;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
#pragma unroll 1
    for (int base = tile_begin; base < tile_end; base += 2 * kSelRing) {
      group(ringA, tmA, base);
      group(ringB, tmB, base + kSelRing);
    }
  };
  const int n_plain = n_interior / (2 * kSelRing) * (2 * kSelRing);   // whole rounds of interior tiles run without masks
  // this wave's share: an equal run of the mask-free rounds; the last wave of the group also takes the edge
  const int rounds = n_plain / (2 * kSelRing);
  const int plain_lo = (rounds * part / KS) * (2 * kSelRing), plain_hi = (rounds * (part + 1) / KS) * (2 * kSelRing);
  // Sweeps 2 and 3 over the mask-free range, 512 tiles (256 entries of the maximum table) at a time: where at most
  // a quarter of the tile pairs can hold a member, only those are fetched and looked at -- with a peaked score
  // law that is a handful of pairs in a million keys --; otherwise the streaming sweep above runs over the stretch,
  // consulting the table per pair unless that can skip next to nothing and, in sweep 3, nine in ten of the pairs
  // the wave has looked at turned out to hold a product some query can keep (a group with one moderately hard query
  // among easy ones is not such a case: looking tells which pairs that query really keeps a key in).
  auto sweep_picked = [&](auto PH, int tile_begin, int tile_end) {
    constexpr int phase_ = decltype(PH)::value;
#pragma unroll 1
    for (int tb = tile_begin; tb < tile_end; tb += 512) {
      const int te = min(tb + 512, tile_end);
      float tmv[4];
      uint64_t on[4];
      int n_on = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int pair = (tb >> 1) + k * 64 + lane;
        tmv[k] = pair < (te >> 1) ? tmx[pair] : ninf;
        on[k] = __ballot(tmv[k] >= xlo_wave);
        n_on += __popcll(on[k]);
      }
      // next to nothing to skip, and (sweep 3) the pairs looked at so far nearly all turned out to be needed:
      // stream, do not look
      if (n_on > 240 && (phase_ == 2 || (n_looked >= 64 && 10 * n_needed >= 9 * n_looked))) {
        sweep(PH, std::false_type{}, std::false_type{}, tb, te);
        continue;
      }
      if (n_on > 64) {
        sweep(PH, std::false_type{}, std::true_type{}, tb, te);
        continue;
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        uint64_t todo = on[k];
        while (todo != 0ull) {
          const int pl = __builtin_ctzll(todo);
          todo &= todo - 1ull;
          const int tile = tb + 2 * (k * 64 + pl);
          reach_known = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(tmv[k]), pl)) >= xlo_wave_top;
          f32x16 SI[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int i = 0; i < 16; ++i) SI[u][i] = 0.f;
            SI[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, load_k(tile + u)),
                                                            __builtin_bit_cast(bf16x8, qIreg), SI[u], 0, 0, 0);
          }
          float tmax = ninf;
#pragma unroll
          for (int u = 0; u < 2; ++u) tmax = fmaxf(tmax, tile_work(PH, std::false_type{}, SI[u], (tile + u) * 32, mxs[u]));
          if (phase_ == 3 && !reach_known && lane == 0) tmx[tile >> 1] = tmax > 0.f ? pinf : ninf;
        }
      }
    }
  };
  auto sweep_all = [&](auto PH) {
    constexpr int phase_ = decltype(PH)::value;
    if constexpr (phase_ == 2 || phase_ == 3) sweep_picked(PH, plain_lo, plain_hi);
    else sweep(PH, std::false_type{}, std::false_type{}, plain_lo, plain_hi);
    if (part == KS - 1) sweep(PH, std::true_type{}, std::true_type{}, n_plain, n_tiles);
    if (phase_ == 2 || phase_ == 3) drain_list();
  };

  double Z = 0.0, above = 0.0;
  int prefix = 0;                 // digits of the threshold found so far
  float sel_mass = 1.f;
  float cut = pinf;               // keep a candidate iff reference - s < cut
  double cum = 0.0, hsel = 0.0;
  int bsel = kSelBins - 1;
  // this query's bins from the top of the score range (bin 0) down; both lanes of the pair and every wave of
  // the group run the same scan on the same numbers
  auto scan = [&](double target) {
    cum = above;
    hsel = 0.0;
    bsel = kSelBins - 1;
    bool found = false;
    for (int i = 0; i < kSelBins; ++i) {
      const double hv = hist[i][r];
      if (!found) {
        if (cum + hv >= target) { bsel = i; hsel = hv; found = true; }
        else cum += hv;
      }
    }
  };

  // ---- sweep 0: the row maxima ----
  sweep_all(std::integral_constant<int, 0>{});
  {
    float mx = mxs[0];
#pragma unroll
    for (int u = 1; u < kSelMfma; ++u) mx = fmaxf(mx, mxs[u]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (g == 0) max_all[wave][r] = mx;
    zero_hist();
    __syncthreads();
#pragma unroll
    for (int k = 0; k < KS; ++k) mx = fmaxf(mx, max_all[qgroup * KS + k][r]);
    selM = mx * cs;
  }
  __syncthreads();                                                  // the maxima are read: the lists' memory is free again

  // ---- sweep 1: the first digit; repeated with a lowered reference while some query's threshold lies in the
  // open-ended bin ----
  bool repeat_me = false, rebased = false;
  for (int round = 0; round < kSelMaxRounds; ++round) {
    selM8 = (round == 0 || repeat_me) ? selM * 8.0f : ninf;         // (exact unless it overflows)
    if (round == 0) sweep_all(std::integral_constant<int, 1>{});
    else sweep_all(std::integral_constant<int, 4>{});
    __syncthreads();                                                // every wave of the group has added its masses
    if (round == 0) {
      Z = 0.0;
      for (int i = 0; i < kSelBins; ++i) Z += hist[i][r];
    }
    if (round == 0 || repeat_me) scan((double)a.p * Z);
    // the threshold in the open-ended bin: everything above it is counted (cum), its members go round again
    repeat_me = (round == 0 || repeat_me) && !idle && qok && bsel == kSelBins - 1 && hsel > 0.0 && round + 1 < kSelMaxRounds;
    // does any query of the workgroup repeat?  (flags in the lists' memory, idle in this phase; the barrier also
    // says that every wave has read the histograms)
    int* flags = reinterpret_cast<int*>(&list_all[0][0][0]);
    const bool mine = __ballot(repeat_me) != 0ull;
    if (lane == 0) flags[wave] = mine ? 1 : 0;
    __syncthreads();
    int any = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) any |= flags[w];
    if (!any) break;
    if (repeat_me) {
      rebased = true;
      selM -= kSelLumpT;
      Z *= kSelLumpScale;
      above = cum * kSelLumpScale;
    }
    zero_hist();
    __syncthreads();
  }
  prefix = bsel;
  above = cum;

  // ---- sweeps 2 and 3: the second and third digit among the members of the prefix ----
#pragma unroll 1
  for (int phase = 2; phase < 4; ++phase) {
    // members of the prefix: prefix << shift <= q < (prefix + 1) << shift; for the non-negative
    // tt = M - s of a candidate that is qlo / 2^17 <= tt < qhi / 2^17 (the last bin is open-ended),
    // and in terms of the raw product x: first x with tt < hi bound <= x < first x with tt < lo bound
    shift = 7 * (4 - phase);                                        // of the prefix found so far: 14, then 7
    const int qlo = prefix << shift, qhi = (prefix + 1) << shift;
    const float lo_t = (float)qlo * (1.0f / kSelScale);
    const float hi_t = qhi > kSelQMax ? pinf : (float)qhi * (1.0f / kSelScale);
    x_lo = sel_first_below(selM, cs, hi_t);
    // the largest x that is still a member: the float just below the first x with tt < lo bound
    x_top = key_float(float_key(sel_first_below(selM, cs, lo_t)) - 1u);
    // the very first range of a reference that is the row maximum is open upwards: t of the maximum itself is the
    // rounding error of M = max * scale and may be a hair below zero (a lowered reference keeps its bound:
    // what lies above it has been counted)
    if (qlo == 0 && !rebased) x_top = pinf;
    xlo_wave = -wave_max_f32((qok && !idle) ? -x_lo : ninf);
    xlo_wave_top = wave_max_f32((qok && !idle) ? x_lo : ninf);
    shift -= 7;                                                     // of this sweep's digit: 7, then 0
    zero_hist();
    __syncthreads();
    if (phase == 2) sweep_all(std::integral_constant<int, 2>{});
    else sweep_all(std::integral_constant<int, 3>{});
    __syncthreads();
    scan((double)a.p * Z);
    prefix = (prefix << 7) | bsel;
    above = cum;
    __syncthreads();                                                // every wave has read the histograms
  }
  // a threshold inside the open-ended last coarse bin (only after the last repeat) keeps every candidate
  const bool lump = (prefix >> 14) == kSelBins - 1;
  cut = lump ? pinf : (float)(prefix + 1) * (1.0f / kSelScale);
  sel_mass = (lump || !(Z > 0.0)) ? 1.f : (float)((cum + hsel) / Z);
  if (!qok || g != 0 || part != 0) return;
  const int64_t o = (int64_t)j * a.n_q + t;
  a.sel_thr[o] = sel_first_below(selM, cs, cut);
  if (a.mass) a.mass[o] = sel_mass;
  // kept: candidates with floor((M - s) * 2^17) <= the threshold's digit string, i.e. s > M - cut
  if (a.tau) a.tau[o] = cut != pinf ? selM - cut : ninf;
}

// ---- the wide kernel: dense and selecting modes ------------------------------------------------------
// Same data flow as above for a workgroup of 256 queries whose waves share every staged K/V tile, in
// one of two shapes (QB = 32-query column blocks per wave):
//   QB = 1 (default): eight waves of 32 queries, two per SIMD, at most 256 registers each;
//   QB = 2: four waves of 64 queries, one per SIMD.  Every A operand read from LDS (a K row block, a
//           V^T row block) feeds two MFMAs, which halves the LDS operand traffic per flop; the price is
//           registers (2 x 64 output accumulators, 64 for the two Q operand sets).
// Measured on the chip: a lone wave on a SIMD issues an independent 32x32x16 MFMA every 38 cycles and
// a vector instruction every ~6, two waves reach the pipes' 32 and 4; in this kernel's own address
// patterns eight waves read K rows from LDS at ~250 bytes per clock and V^T (the transposing read) at
// ~96, four waves at ~160 and ~63 -- enough for either shape, so the second instruction stream wins:
// QB = 1 is 3 to 16 % faster than QB = 2 at every depth of the 131072- and 1048576-token configurations.
//
// Nothing hides latency by itself at one or two waves per SIMD, so the loop is software-pipelined over
// 32-key blocks: while the softmax of block i runs on the vector ALU, the matrix pipe executes the PV
// MFMAs of block i-1; the two are independent instruction streams inside one basic block and are
// interleaved with scheduling-group hints.  For that the accumulators must never be touched by the
// vector ALU inside the loop (the register allocator would otherwise shuttle them between the two
// register files), so there is no running maximum: every query takes a FIXED reference
// maximum from the scores of the first key tile and the probabilities are exp2(s - ref), which fp32 and
// bf16 represent over +-126 binades.  After the pass the row sums tell whether a reference was off by
// more than that leaves room for (sum outside [2^-60, 2^100], or not finite); the workgroup then
// repeats its keys with the classical running-maximum recurrence (exact_pass).  Real score rows
// have their maximum at the first tokens; the repeat exists for correctness, not for speed.
// K/V tiles rotate through three LDS buffers (the PV of a tile's last block reads its V^T while the
// next tile is current), one workgroup barrier per 64-key tile.
constexpr int kPwQ = 256;
constexpr int kPwStages = 3;
// One staged tile: 64 K rows then 64 V rows, 256 bytes each, no padding -- the tiles are written by
// direct global->LDS loads (16 bytes per lane, a wave's 64 lanes fill 1 KiB contiguously), so bank
// spreading comes from the order of the 16-byte chunks inside a row instead: K row n keeps chunk c at
// position c ^ (n % 16) (the MFMA operand read takes one chunk of 16 consecutive rows), V row n keeps
// 32-byte unit u at position u ^ 2 (n % 4): a transposing operand read has each half-wave take, from four rows,
// the two units 2 db and 2 db + 1 (its two 16-lane groups), and with this order those eight (row, unit) pieces
// land on the eight different bank groups of a row (u ^ (n % 8), the first layout, put the two groups' pieces on
// the same four: a third of the kernel's LDS cycles were bank conflicts by the counters, none now; the kernel is
// bound by instruction issue and runs as long).
constexpr int kPwTileBytes = 2 * kPfK * kHeadDim * 2;
constexpr int kSmemWide = kPwTileBytes * kPwStages;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));


template <int MODE, int QB, bool F16 = false>
__global__ __launch_bounds__(64 * (8 / QB), QB == 1 ? 2 : 1) void flash_prefill_wide_kernel(const PrefillArgs a) {
  constexpr int NW = 8 / QB;                 // waves per workgroup; each owns QB blocks of 32 queries
  constexpr int RG = 4 * NW;                 // tile rows one load instruction of the whole workgroup covers
  constexpr int GH = 64 / RG;                // such loads per wave for the K rows of a tile (and as many for V)
  constexpr bool LOCAL = MODE == kModeLocal;
  constexpr bool SPARSE = MODE == kModeSparse;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kSmemWide];
  unsigned char* const Ls = smem;       // stage s: K rows at Ls + s * kPwTileBytes, V rows 16 KiB further

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;
  // A selecting launch behind a threshold search (one sequence) is laid out (key range, query tile, head slot): the
  // query tiles' lists differ wildly in length, and with the key range as the fastest index the ranges of a long
  // list go round all eight dies (workgroups are dealt to the dies in turn) instead of piling up on one.
  // The grid of such a launch is sized for the finer cut; the ranges really used (listed_splits) take the
  // first workgroups of the grid in the same (key range, query tile, head slot) order, the others leave.
  const bool listed = SPARSE && a.p < 1.f;
  const int n_splits = LOCAL ? 1 : (listed ? listed_splits(a) : a.n_splits);
  int hslot = blockIdx.x, split, qt_rev = blockIdx.y, b = 0;
  if (listed) {
    const int lin = (int)blockIdx.x + (int)gridDim.x * ((int)blockIdx.y + (int)gridDim.y * (int)blockIdx.z);
    split = lin % n_splits;
    qt_rev = (lin / n_splits) % (int)gridDim.y;
    hslot = lin / (n_splits * (int)gridDim.y);
    if (hslot >= (int)gridDim.z) return;
  } else {
    b = blockIdx.z / n_splits;
    split = (int)blockIdx.z - b * n_splits;
  }
  const int h = a.heads[hslot];
  const int t0 = ((int)gridDim.y - 1 - qt_rev) * kPwQ;
  const int kvh = h / (a.n_q_heads / a.n_kv_heads);
  const int pos0 = a.q_start ? a.q_start[b] : (int)a.q_start_host;
  const int64_t tok0 = a.seq_start ? a.seq_start[b] : 0;
  const float ninf = -__builtin_huge_valf();

  // ---- this lane's queries (column r of each of the wave's QB blocks) ----
  int tq[QB], mq[QB];
  bool qok[QB];
  int64_t qrow[QB];
  u32x4 qreg[QB][8];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    tq[qb] = t0 + wave * (32 * QB) + qb * 32 + r;
    qok[qb] = tq[qb] < a.n_q;
    mq[qb] = pos0 + tq[qb];
    qrow[qb] = (((int64_t)b * a.n_q + tq[qb]) * a.n_q_heads + h) * kHeadDim;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      qreg[qb][kk] = qok[qb] ? *reinterpret_cast<const u32x4*>(a.q + qrow[qb] + kk * 16 + g * 8) : (u32x4){0u, 0u, 0u, 0u};
  }

  // ---- key tiles this workgroup needs ----
  const int m_lo = pos0 + t0;
  const int m_hi = pos0 + min(t0 + kPwQ, a.n_q) - 1;
  const int kt_end = m_hi / kPfK;                       // inclusive
  int kt_w0 = 0, ks_end = 0;
  if (LOCAL) {
    const int lo = max(a.sink, m_lo - a.window + 1);
    kt_w0 = lo / kPfK;
    ks_end = min((a.sink + kPfK - 1) / kPfK, kt_w0);    // sink tiles not already inside the band
  }
  // selecting mode with a threshold search in front: only the tiles on this query tile's list (ascending
  // 64-key tile numbers, written by prefill_active_tiles_kernel) can hold a kept pair
  const int qt_list = (int)gridDim.y - 1 - qt_rev;
  const int32_t* const alist = listed ? a.act_list + ((int64_t)hslot * gridDim.y + qt_list) * a.n_t64 : nullptr;
  const int n_tiles = listed ? a.act_count[(int64_t)hslot * gridDim.y + qt_list] : ks_end + (kt_end - kt_w0 + 1);
  const uint16_t* Kg = a.K + (int64_t)kvh * a.head_stride + tok0 * a.row_stride;
  const uint16_t* Vg = a.V + (int64_t)kvh * a.head_stride + tok0 * a.row_stride;

  f32x16 O[QB][4];
  float mrow[QB], lrow[QB];
  const float c = a.scale_log2;
  const int q_last = pos0 + a.n_q - 1;
  const int m_w_lo = pos0 + t0 + wave * (32 * QB);             // the wave's first query position
  const int m_w_hi = min(m_w_lo + 32 * QB - 1, q_last);          // and its last (< m_w_lo: the wave has no queries)

  // ---- selecting mode: a key is kept by a query iff the raw index product reaches the query's
  // threshold (found by prefill_select_kernel; -inf keeps every candidate).  The index-score block of
  // 32 keys x 32 queries is one MFMA (K = 16) in the layout of the attention scores. ----
  u32x4 qIreg[QB];
  float selThr[QB];
  int sel_cnt[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    qIreg[qb] = (u32x4){0u, 0u, 0u, 0u};
    selThr[qb] = ninf;
    sel_cnt[qb] = 0;
  }
  const uint16_t* kIg = nullptr;
  const int n_rows = pos0 + a.n_q;                      // index-key rows that exist
  if (SPARSE) {
    const int j = hslot;
    kIg = a.kI + (int64_t)j * a.kI_head_stride;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if (qok[qb]) {
        qIreg[qb] = *reinterpret_cast<const u32x4*>(a.qI + ((int64_t)j * a.n_q + tq[qb]) * kIndexDim + g * 8);
        if (a.p < 1.f) selThr[qb] = a.sel_thr[(int64_t)j * a.n_q + tq[qb]];
      }
    }
  }
  // index keys of the 32-key block at nb0 (rows past the chunk repeat the last one: causally masked anyway)
  auto load_ki = [&](int nb0) __attribute__((always_inline)) {
    const int nrow = min(nb0 + r, n_rows - 1);
    return *reinterpret_cast<const u32x4*>(kIg + (int64_t)nrow * kIndexDim + g * 8);
  };
  // drops the keys a query does not keep from its scores and counts the kept ones; run AFTER mask_block
  // (causality shows as -inf there)
  auto select_block = [&](f32x16 (&S)[QB], const u32x4 ki) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      f32x16 SI;
#pragma unroll
      for (int i = 0; i < 16; ++i) SI[i] = 0.f;
      SI = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ki), __builtin_bit_cast(bf16x8, qIreg[qb]), SI, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const bool keep = SI[i] >= selThr[qb] && S[qb][i] != ninf;
        sel_cnt[qb] += keep ? 1 : 0;
        S[qb][i] = keep ? S[qb][i] : ninf;
      }
    }
  };

  // ---- tile movers: direct global->LDS loads, no staging registers (rows past the last needed key
  // repeat that key: they are masked for every query, and real data keeps 0 * V finite) ----
  // Load j (0..GH-1: K, GH..2GH-1: V) of a wave covers rows RG * (j % GH) + 4 * wave + lane / 16 of the
  // tile, lane % 16 is the 16-byte position inside the row; the lane fetches the chunk that belongs there.
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)Ls;
  const int ld_row = 4 * wave + (lane >> 4);
  const int ld_pos = lane & 15;
  const int ld_ck = ld_pos ^ (ld_row & 15);                                          // K chunk of this lane
  const int ld_cv = ((((ld_pos >> 1) ^ (2 * (ld_row & 3))) << 1) | (ld_pos & 1));    // V chunk of this lane
  auto load_piece = [&](int n0, int slot, int j) __attribute__((always_inline)) {
    const int jj = j % GH;
    const int n = min(n0 + RG * jj + ld_row, m_hi);
    const uint16_t* src = (j < GH ? Kg + ld_ck * 8 : Vg + ld_cv * 8) + (int64_t)n * a.row_stride;
    const uint32_t dst = lds_base + slot * kPwTileBytes + (j < GH ? 0 : kPwTileBytes / 2) + (jj * NW + uwave) * 1024;
    // Written as assembly on purpose: through the compiler's own intrinsic every later LDS read waits
    // for ALL outstanding direct loads (it cannot tell the buffers apart), which serialises the
    // pipeline; completion is awaited explicitly (loads_landed) before the barrier that publishes a tile.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(src) : "memory", "m0");
  };
  // The same for a tile that lies wholly inside the key range (every tile but the last): the tile's first
  // K and V rows as scalar base addresses, the lane's place inside the tile as a 32-bit offset computed
  // once -- no vector arithmetic per load (the general form costs seven vector instructions per piece,
  // two of them quarter-rate multiplies, a tenth of the kernel's issue slots).
  uint32_t off_k[GH], off_v[GH];
#pragma unroll
  for (int jj = 0; jj < GH; ++jj) {
    off_k[jj] = (uint32_t)(((int64_t)(RG * jj + ld_row) * a.row_stride + ld_ck * 8) * 2);
    off_v[jj] = (uint32_t)(((int64_t)(RG * jj + ld_row) * a.row_stride + ld_cv * 8) * 2);
  }
  auto load_piece_full = [&](int n0, int slot, int j) __attribute__((always_inline)) {
    const int jj = j % GH;
    const unsigned char* base = reinterpret_cast<const unsigned char*>((j < GH ? Kg : Vg) + (int64_t)n0 * a.row_stride);
    const uint32_t dst = lds_base + slot * kPwTileBytes + (j < GH ? 0 : kPwTileBytes / 2) + (jj * NW + uwave) * 1024;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(j < GH ? off_k[jj] : off_v[jj]), "s"(base)
                 : "memory", "m0");
  };
  auto load_tile = [&](int n0, int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 2 * GH; ++j) load_piece(n0, slot, j);
  };
  auto loads_landed = [&]() __attribute__((always_inline)) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
  // operand read addresses (bytes inside a staged tile)
  const int rd_k = r * 256, rd_kx = (g ^ (r & 15)) << 4;                              // K: + kb * 8192, chunk (2 kk) ^ ...
  const int rd_j = lane & 15, rd_G = (lane >> 4) & 1;
  const int rd_v = kPwTileBytes / 2 + (4 * g + (rd_j >> 2)) * 256 + 8 * (rd_j & 3);   // V: + (kb * 32 + 16 tt + 8 h) * 256
  const int rd_vx = (rd_G ^ (2 * (rd_j >> 2))) << 5;                                  //    unit (2 db) ^ ...
  auto read_k = [&](const unsigned char* tile, int kb, int kk) __attribute__((always_inline)) {
    return *reinterpret_cast<const u32x4*>(tile + kb * 8192 + rd_k + ((kk << 5) ^ rd_kx));
  };
  // the 8 keys x 1 dim a lane needs of V^T for MFMA (tt, db): two transposing reads of 4 keys each
  auto read_v = [&](const unsigned char* tile, int kb, int tt, int db) __attribute__((always_inline)) {
    const unsigned char* p0 = tile + rd_v + (kb * 32 + 16 * tt) * 256 + ((db << 6) ^ rd_vx);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * 256));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };

  // ---- MFMA streams ----
  // scores of key block kb of the staged tile, for the wave's query blocks
  auto mfma_S = [&](const unsigned char* tile, int kb, f32x16 (&S)[QB]) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) S[qb][i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const u32x4 ka = read_k(tile, kb, kk);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) S[qb] = mfma32<F16>(ka, qreg[qb][kk], S[qb]);
    }
  };
  // The same MFMAs with their K operands read three steps ahead and a slice of other work (issuing
  // the loads of a later tile) between every pair; scheduling fences keep the order.
  auto scores_beside = [&](const unsigned char* tile, int kb, f32x16 (&S)[QB], auto&& work) __attribute__((always_inline)) {
    u32x4 ka[8];
    ka[0] = read_k(tile, kb, 0);
    ka[1] = read_k(tile, kb, 1);
    ka[2] = read_k(tile, kb, 2);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) S[qb][i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      if (kk + 3 < 8) ka[kk + 3] = read_k(tile, kb, kk + 3);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        S[qb] = mfma32<F16>(ka[kk], qreg[qb][kk], S[qb]);
        if (qb == 0) work(kk);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  // O^T += V^T P^T for key block kb of the staged tile
  auto mfma_PV = [&](const unsigned char* tile, int kb, const uint32_t (&P)[QB][8]) __attribute__((always_inline)) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const u32x4 va = __builtin_bit_cast(u32x4, read_v(tile, kb, tt, db));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          const u32x4 pb = (u32x4){P[qb][4 * tt], P[qb][4 * tt + 1], P[qb][4 * tt + 2], P[qb][4 * tt + 3]};
          O[qb][db] = mfma32<F16>(va, pb, O[qb][db]);
        }
      }
    }
  };
  // per-element visibility without control flow: key nb0 + off, off = (i / 4) * 8 + g * 4 + i % 4, is
  // visible iff off <= hi and (LOCAL) off > lo or off < sk, three per-lane bounds
  auto mask_block = [&](f32x16 (&S)[QB], int nb0) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int base = nb0 + g * 4;
      const int hi = qok[qb] ? mq[qb] - base : -1;
      const int lo = mq[qb] - a.window - base;
      const int sk = a.sink - base;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int off = (i >> 2) * 8 + (i & 3);
        bool ok = off <= hi;
        if (LOCAL) ok = ok & ((off > lo) | (off < sk));
        S[qb][i] = ok ? S[qb][i] : ninf;
      }
    }
  };
  // probabilities against the fixed reference; masked scores are -inf and give exactly 0
  auto softmax_fixed = [&](const f32x16 (&S)[QB], uint32_t (&P)[QB][8]) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float mc = mrow[qb] * c;
      float lsum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = fast_exp2(fmaf(S[qb][i], c, -mc));
        const float p1 = fast_exp2(fmaf(S[qb][i + 1], c, -mc));
        lsum += p0 + p1;
        P[qb][i >> 1] = pack16<F16>(p0, p1);
      }
      lrow[qb] += lsum;
    }
  };
  // l += both halves of a packed pair of probabilities, i.e. the values as rounded to bf16 (what the PV
  // product multiplies): one instruction, and of a kind the compiler leaves where it is written (plain
  // additions get collected behind the last MFMA of the sequence, where nothing hides them)
  // (the compiler's own dot product intrinsic gets collected the same way).  The result of a dot
  // instruction must not be read by another kind of vector instruction for three wait states, and
  // the compiler does not look into assembly text: row_sum_settled() goes between the last
  // row_sum_add and the first use.
  auto row_sum_settled = [&](float& l) __attribute__((always_inline)) { asm volatile("s_nop 3" : "+v"(l)); };
  auto row_sum_add = [&](float& l, uint32_t pk) __attribute__((always_inline)) {
    if constexpr (F16) asm volatile("v_dot2c_f32_f16 %0, %1, %2" : "+v"(l) : "v"(pk), "v"(0x3c003c00u));
    else asm volatile("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(l) : "v"(pk), "v"(0x3f803f80u));
  };
  // The steady-state step: the PV MFMAs of the previous block and the softmax of the current block as
  // ONE hand-interleaved instruction sequence -- per MFMA (32 cycles of the matrix pipe) one pair of
  // probabilities (2 fma, 2 exp, 1 convert, 1 packed dot product on the vector ALU); scheduling fences
  // keep the compiler from regrouping it, V^T operands are read two steps ahead.  SEL (the selecting
  // mode): the block's index-score MFMAs in front and every probability gated by its query's keep test
  // (one compare, one select, one add for the count per probability).
  auto pv_beside_softmax = [&](auto sel_tag, const unsigned char* tile, int kb, const uint32_t (&Pin)[QB][8], const f32x16 (&S)[QB],
                               uint32_t (&Pout)[QB][8], const u32x4 ki) __attribute__((always_inline)) {
    constexpr bool SEL = decltype(sel_tag)::value;
    f32x16 SI[QB];
    float mc[QB], l[QB];
    int cnt[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      mc[qb] = mrow[qb] * c;
      l[qb] = 0.f;
      cnt[qb] = 0;
      if (SEL) {
#pragma unroll
        for (int i = 0; i < 16; ++i) SI[qb][i] = 0.f;
        SI[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ki), __builtin_bit_cast(bf16x8, qIreg[qb]), SI[qb], 0, 0, 0);
      }
    }
    s16x8 va[8];
    auto read_va = [&](int k) __attribute__((always_inline)) { va[k] = read_v(tile, kb, k >> 2, k & 3); };   // k = tt * 4 + db
    read_va(0);
    read_va(1);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int tt = k >> 2, db = k & 3;
      if (k + 2 < 8) read_va(k + 2);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const u32x4 pb = (u32x4){Pin[qb][4 * tt], Pin[qb][4 * tt + 1], Pin[qb][4 * tt + 2], Pin[qb][4 * tt + 3]};
        O[qb][db] = mfma32<F16>(__builtin_bit_cast(u32x4, va[k]), pb, O[qb][db]);
        {
          float p0 = fast_exp2(fmaf(S[qb][2 * k], c, -mc[qb]));
          float p1 = fast_exp2(fmaf(S[qb][2 * k + 1], c, -mc[qb]));
          if (SEL) {
            const bool k0 = SI[qb][2 * k] >= selThr[qb], k1 = SI[qb][2 * k + 1] >= selThr[qb];
            p0 = k0 ? p0 : 0.f;
            p1 = k1 ? p1 : 0.f;
            cnt[qb] += (k0 ? 1 : 0) + (k1 ? 1 : 0);
          }
          Pout[qb][k] = pack16<F16>(p0, p1);
          row_sum_add(l[qb], Pout[qb][k]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      row_sum_settled(l[qb]);
      lrow[qb] += l[qb];
      if (SEL) sel_cnt[qb] += cnt[qb];
    }
  };
  // does the 32-key block starting at nb0 need per-element masks for some query of this wave?
  auto needs_mask = [&](int nb0) __attribute__((always_inline)) {
    bool e = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int m_b_lo = m_w_lo + qb * 32;
      const int m_b_hi = min(m_b_lo + 31, q_last);
      e = e || (m_b_hi < m_b_lo) || (nb0 + 31 > m_b_lo) || (LOCAL && !(nb0 > m_b_hi - a.window || nb0 + 31 < a.sink));
    }
    return e;
  };
  // can some query of this wave see a key of the block at all?
  auto is_active = [&](int nb0) __attribute__((always_inline)) {
    if (m_w_hi < m_w_lo || nb0 > m_w_hi) return false;
    if (LOCAL && nb0 >= a.sink && nb0 + 31 <= m_w_lo - a.window) return false;
    return true;
  };

  auto tile_n0 = [&](int it) __attribute__((always_inline)) {
    if (SPARSE && listed) return alist[it] * kPfK;
    return (it < ks_end ? it : kt_w0 + (it - ks_end)) * kPfK;
  };
  const int it_lo = (int)((int64_t)n_tiles * split / n_splits);
  const int it_hi = (int)((int64_t)n_tiles * (split + 1) / n_splits);
  auto slot_of = [&](int it) __attribute__((always_inline)) { return (it - it_lo) % kPwStages; };
  auto tile_at = [&](int it) __attribute__((always_inline)) { return Ls + slot_of(it) * kPwTileBytes; };

  bool redo = false;
  if (it_lo < it_hi) {
    f32x16 S[QB];
    uint32_t P0[QB][8], P1[QB][8];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      lrow[qb] = 0.f;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[qb][db][i] = 0.f;
    }
    // first keys of tiles it, it + 1, it + 2 (clamped to the range's last tile) and, one iteration ahead of its
    // first use, it + 3: a listed tile's number comes from memory
    int n_t0 = tile_n0(it_lo), n_t1 = tile_n0(min(it_lo + 1, it_hi - 1)), n_t2 = tile_n0(min(it_lo + 2, it_hi - 1));
    int n_t3 = tile_n0(min(it_lo + 3, it_hi - 1));
    load_tile(n_t0, 0);
    load_tile(n_t1, 1);
    loads_landed();
    __syncthreads();
    // reference maxima: the largest score of the first tile, masks ignored (always finite)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) mrow[qb] = ninf;
#pragma unroll
    for (int kb = 1; kb >= 0; --kb) {
      mfma_S(Ls, kb, S);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float mx = S[qb][0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, S[qb][i]);
        mrow[qb] = fmaxf(mrow[qb], fmaxf(mx, __shfl_xor(mx, 32)));
      }
    }                                                    // S now holds block (it_lo, 0)

    // Invariant at the start of half hf of tile it: S holds the scores of that block if it is active
    // for this wave; if `pend`, the probabilities of the last active block wait in P1 (hf = 0, V in
    // the previous tile's buffer) or P0 (hf = 1); tiles it and it + 1 are in LDS.  The loads of tile
    // it + 2 go out during half 1 (their buffer held tile it - 1, last read in half 0) and every wave
    // waits for its own before the barrier that ends half 0 of tile it + 1.
    bool pend = false;
    u32x4 ki0 = (u32x4){0u, 0u, 0u, 0u}, ki1 = ki0;       // index keys of the current tile's two key blocks
    if (SPARSE) {
      ki0 = load_ki(n_t0);
      ki1 = load_ki(n_t0 + 32);
    }
    auto half = [&](int it, auto hf_tag) __attribute__((always_inline)) {
      constexpr int hf = decltype(hf_tag)::value;
      const int nb0 = n_t0 + hf * 32;
      const unsigned char* t_pend = hf == 0 ? tile_at(it - 1) : tile_at(it);
      const uint32_t (&Pin)[QB][8] = hf == 0 ? P1 : P0;
      uint32_t (&Pout)[QB][8] = hf == 0 ? P0 : P1;
      if (!is_active(nb0)) {
        if (pend) mfma_PV(t_pend, 1 - hf, Pin);
        pend = false;
      } else if (pend && !needs_mask(nb0)) {
        // steady state: PV of the previous block beside the softmax of this one
        pv_beside_softmax(std::integral_constant<bool, SPARSE>{}, t_pend, 1 - hf, Pin, S, Pout, hf == 0 ? ki0 : ki1);
      } else {
        if (pend) mfma_PV(t_pend, 1 - hf, Pin);
        mask_block(S, nb0);
        if (SPARSE) select_block(S, hf == 0 ? ki0 : ki1);
        softmax_fixed(S, Pout);
        pend = true;
      }
      if (SPARSE && hf == 1) {                             // the next tile's index keys: a tile's time to arrive
        ki0 = load_ki(n_t1);
        ki1 = load_ki(n_t1 + 32);
      }
      if (hf == 0) {
        if (is_active(nb0 + 32)) scores_beside(tile_at(it), 1, S, [&](int) __attribute__((always_inline)) {});
        loads_landed();
        __syncthreads();
      } else {
        // past the last tile the same loads re-fetch it into a buffer nobody reads: no branches
        const int n2 = n_t2;
        const int s2 = slot_of(it + 2);
        const bool next_active = it + 1 < it_hi && is_active(n_t1);
        if (n2 + kPfK - 1 <= m_hi) {                       // a whole tile (all but the last of the range)
          if (next_active) {
            scores_beside(tile_at(it + 1), 0, S, [&](int kk) __attribute__((always_inline)) { if (kk < 2 * GH) load_piece_full(n2, s2, kk); });
          } else {
#pragma unroll
            for (int j = 0; j < 2 * GH; ++j) load_piece_full(n2, s2, j);
          }
        } else if (next_active) {
          scores_beside(tile_at(it + 1), 0, S, [&](int kk) __attribute__((always_inline)) { if (kk < 2 * GH) load_piece(n2, s2, kk); });
        } else {
          load_tile(n2, s2);
        }
      }
    };
    for (int it = it_lo; it < it_hi; ++it) {
      half(it, std::integral_constant<int, 0>{});
      half(it, std::integral_constant<int, 1>{});
      n_t0 = n_t1;
      n_t1 = n_t2;
      n_t2 = n_t3;
      n_t3 = tile_n0(min(it + 4, it_hi - 1));
    }
    if (pend) mfma_PV(tile_at(it_hi - 1), 1, P1);        // drain: PV of the last block
    loads_landed();

    // was every reference within reach?  A query that can see a key of this key range (always, with
    // the whole band of a local launch; from the range's first key on, in a dense one) must have a sum
    // in the comfortable middle of the fp32 range; everything else (0, tiny, huge, inf, NaN) repeats.
    bool bad = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float ltot = lrow[qb] + __shfl_xor(lrow[qb], 32);
      // selecting mode: a query that kept no key of this range legitimately sums to zero
      const bool sees_key = SPARSE ? (sel_cnt[qb] + __shfl_xor(sel_cnt[qb], 32) > 0)
                                   : (qok[qb] && (LOCAL || tile_n0(it_lo) <= mq[qb]));
      // (fp16 probabilities: nothing above 65504 -- a larger one is infinite and shows in the sum -- and a
      // row whose largest probability is below 2^-6 has most of its mass in subnormals or flushed to zero)
      bad = bad || (sees_key && !(ltot > (F16 ? 0x1p-6f : 0x1p-60f) && ltot < 0x1p100f));
    }
    redo = __syncthreads_or(bad ? 1 : 0) != 0;
  }

  if (redo) {
    // ---- exact pass: running maximum, accumulators rescaled in place; no pipelining (rare) ----
    f32x16 S[QB];
    uint32_t P[QB][8];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      mrow[qb] = ninf;
      lrow[qb] = 0.f;
      sel_cnt[qb] = 0;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[qb][db][i] = 0.f;
    }
    for (int it = it_lo; it < it_hi; ++it) {
      __syncthreads();
      load_tile(tile_n0(it), 0);
      loads_landed();
      __syncthreads();
      for (int kb = 0; kb < 2; ++kb) {
        const int nb0 = tile_n0(it) + kb * 32;
        if (!is_active(nb0)) continue;
        if (kb == 0) mfma_S(Ls, 0, S); else mfma_S(Ls, 1, S);
        mask_block(S, nb0);
        if (SPARSE) select_block(S, load_ki(nb0));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          float mx = S[qb][0];
#pragma unroll
          for (int i = 1; i < 16; ++i) mx = fmaxf(mx, S[qb][i]);
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          const float mnew = fmaxf(mrow[qb], mx);
          const float msafe = mnew == ninf ? 0.f : mnew;
          const float mc = msafe * c;
          float lsum = 0.f;
#pragma unroll
          for (int i = 0; i < 16; i += 2) {
            const float p0 = fast_exp2(fmaf(S[qb][i], c, -mc));
            const float p1 = fast_exp2(fmaf(S[qb][i + 1], c, -mc));
            lsum += p0 + p1;
            P[qb][i >> 1] = pack16<F16>(p0, p1);
          }
          const float corr = fast_exp2((mrow[qb] - msafe) * c);
          lrow[qb] = lrow[qb] * corr + lsum;
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[qb][db][i] *= corr;
          mrow[qb] = mnew;
        }
        if (kb == 0) mfma_PV(Ls, 0, P); else mfma_PV(Ls, 1, P);
      }
    }
  }

  // ---- normalise and store ----
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float ltot = (it_lo < it_hi) ? lrow[qb] + __shfl_xor(lrow[qb], 32) : 0.f;
    if (!qok[qb]) continue;
    const float mfin = (it_lo < it_hi && ltot > 0.f) ? mrow[qb] : ninf;
    const int kept = sel_cnt[qb] + __shfl_xor(sel_cnt[qb], 32);
    if (SPARSE && g == 0 && split == 0 && !(a.p < 1.f)) {   // keep-all: the threshold search did not run
      const int64_t o = (int64_t)hslot * a.n_q + tq[qb];
      if (a.mass) a.mass[o] = 1.f;
      if (a.tau) a.tau[o] = ninf;
    }
    if (n_splits > 1) {
      float* prow = a.part + (((int64_t)split * a.n_heads + hslot) * a.n_q + tq[qb]) * kPfPart;
      if (g == 0) { prow[0] = mfin; prow[1] = ltot; prow[2] = __int_as_float(kept); }
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
          *reinterpret_cast<float4*>(prow + 4 + db * 32 + i4 * 8 + g * 4) =
              ltot > 0.f ? make_float4(O[qb][db][i4 * 4], O[qb][db][i4 * 4 + 1], O[qb][db][i4 * 4 + 2], O[qb][db][i4 * 4 + 3])
                         : make_float4(0.f, 0.f, 0.f, 0.f);
      continue;
    }
    const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
    uint16_t* orow = a.out + qrow[qb];
#pragma unroll
    for (int db = 0; db < 4; ++db) {
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const u32x2 w = ltot > 0.f ? (u32x2){pack16<F16>(O[qb][db][i4 * 4] * inv, O[qb][db][i4 * 4 + 1] * inv),
                                             pack16<F16>(O[qb][db][i4 * 4 + 2] * inv, O[qb][db][i4 * 4 + 3] * inv)}
                                   : (u32x2){0u, 0u};
        *reinterpret_cast<u32x2*>(orow + db * 32 + i4 * 8 + g * 4) = w;
      }
    }
    if (a.lse && g == 0) {
      a.lse[((int64_t)b * a.n_q + tq[qb]) * a.n_q_heads + h] = ltot > 0.f ? mfin * a.scale + logf(ltot) : ninf;
    }
    if (SPARSE && a.count && g == 0) a.count[(int64_t)hslot * a.n_q + tq[qb]] = kept;
  }
}

// The 64-key tiles a 256-query tile of the selecting attention launch has to visit: tile n is on the list iff, for
// one of the tile's eight 32-query groups, the group's largest index product in the tile (tile_max, written by the
// first sweep of prefill_select_kernel) reaches the group's smallest threshold.  Every other tile holds no kept
// pair -- the keep test is product >= threshold -- so leaving it out changes no output, count or sum.
// Grid (query tiles, retrieval heads), 256 threads; the list is ascending.
__global__ __launch_bounds__(256) void prefill_active_tiles_kernel(const PrefillArgs a) {
  const int j = blockIdx.y, qt = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = qt * kPwQ;
  __shared__ float thr[kPwQ / 32];
  __shared__ int wave_n[4];
  {
    const int t = t0 + tid;
    float v = t < a.n_q ? a.sel_thr[(int64_t)j * a.n_q + t] : __builtin_huge_valf();
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o));
    if ((tid & 31) == 0) thr[tid >> 5] = v;
  }
  __syncthreads();
  const int pos0 = (int)a.q_start_host;
  const int n_pairs = (pos0 + min(t0 + kPwQ, a.n_q) - 1) / kPfK + 1;
  const float* tm = a.tile_max + ((int64_t)j * ((a.n_q + 31) / 32) + t0 / 32) * a.n_t64;
  int32_t* list = a.act_list + ((int64_t)j * gridDim.x + qt) * a.n_t64;
  int base = 0;
  for (int p0 = 0; p0 < n_pairs; p0 += 256) {
    const int p = p0 + tid;
    bool on = false;
    if (p < n_pairs) {
#pragma unroll
      for (int i = 0; i < kPwQ / 32; ++i) {
        const int tw = t0 + 32 * i;
        // the group's row of the table reaches as far as its last query sees
        if (tw < a.n_q && p * kPfK <= pos0 + min(tw + 32, a.n_q) - 1) on = on || tm[(int64_t)i * a.n_t64 + p] >= thr[i];
      }
    }
    const uint64_t bal = __ballot(on);
    if (lane == 0) wave_n[wave] = __popcll(bal);
    __syncthreads();
    int before = base;
    for (int w = 0; w < wave; ++w) before += wave_n[w];
    if (on) list[before + __popcll(bal & ((1ull << lane) - 1ull))] = p;
    base += wave_n[0] + wave_n[1] + wave_n[2] + wave_n[3];
    __syncthreads();
  }
  if (tid == 0) {
    a.act_count[(int64_t)j * gridDim.x + qt] = base;
    atomicMax(&a.act_range[0], base);
    atomicMin(&a.act_range[1], base);
  }
}

// qI[j, t, :] = bf16( W[j] . x[t, ret_heads[j], :] ), the 128-term sums in fp64, one rounding
// (Sec. 3.2, indexer equation, query side).  16 queries per workgroup: thread = (query, output dim).
struct ProjectArgs {
  const float* W;
  const uint16_t* x;
  uint16_t* out;
  int32_t n_q, n_q_heads, n_ret;
  int32_t ret_heads[64];
};

__global__ __launch_bounds__(256) void index_project_kernel(const ProjectArgs a) {
  const int j = blockIdx.y;
  const int t = blockIdx.x * 16 + (threadIdx.x >> 4), i = threadIdx.x & 15;
  if (t >= a.n_q) return;
  const float* w = a.W + ((int64_t)j * kIndexDim + i) * kHeadDim;
  const uint16_t* x = a.x + ((int64_t)t * a.n_q_heads + a.ret_heads[j]) * kHeadDim;
  double acc = 0.0;
  for (int c = 0; c < kHeadDim; ++c) acc = fma((double)w[c], (double)bf16_to_f32(x[c]), acc);
  a.out[((int64_t)j * a.n_q + t) * kIndexDim + i] = f64_to_bf16_rne(acc);
}

// Merges the key-range partials of one (query, head): thread = output dim, two queries per block.
__global__ __launch_bounds__(256) void prefill_combine_kernel(const PrefillArgs a) {
  const int t = blockIdx.x * 2 + (threadIdx.x >> 7), d = threadIdx.x & 127, hs = blockIdx.y;
  if (t >= a.n_q) return;
  const float ninf = -__builtin_huge_valf();
  const int n_splits = a.act_range ? listed_splits(a) : a.n_splits;     // (a listed launch decides on the device)
  float M = ninf;
  for (int s = 0; s < n_splits; ++s) M = fmaxf(M, a.part[(((int64_t)s * a.n_heads + hs) * a.n_q + t) * kPfPart]);
  if (a.count && d == 0) {                                 // selecting mode: kept keys over all key ranges
    int kept = 0;
    for (int s = 0; s < n_splits; ++s) kept += __float_as_int(a.part[(((int64_t)s * a.n_heads + hs) * a.n_q + t) * kPfPart + 2]);
    a.count[(int64_t)hs * a.n_q + t] = kept;
  }
  float L = 0.f, A = 0.f;
  if (M != ninf) {
    for (int s = 0; s < n_splits; ++s) {
      const float* p = a.part + (((int64_t)s * a.n_heads + hs) * a.n_q + t) * kPfPart;
      if (p[0] == ninf) continue;
      const float cw = fast_exp2((p[0] - M) * a.scale_log2);
      L += p[1] * cw;
      A += p[4 + d] * cw;
    }
  }
  const int h = a.heads[hs];
  const int64_t o = (int64_t)t * a.n_q_heads + h;        // single sequence
  a.out[o * kHeadDim + d] = f32_to_16(L > 0.f ? A / L : 0.f, a.f16 != 0);
  if (a.lse && d == 0) a.lse[o] = L > 0.f ? M * a.scale + logf(L) : ninf;
}

// Compute units of the current device (256 on the target; also the answer where no device is visible,
// as when only a workspace size is asked for).
static int compute_units() {
  static const int v = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
      (void)hipGetLastError();
      n = 256;
    }
    return n;
  }();
  return v;
}

// Number of key-range splits for a dense launch with few workgroups (long context, few heads).  A
// compute unit holds ONE workgroup of the wide kernel (its LDS), so a launch runs in rounds of as many
// workgroups as there are compute units: the split count is the one that fills its last round best (at
// most 8, at least 32 key tiles per part), a smaller count winning near-ties because every part costs a
// partial result to write and merge.  Measured on the 131072- and 1048576-token configurations (64 and 128
// query-tile workgroups): 4 and 2 parts beat the former 8 by 4 and 2 %, 3 or 6 parts lose 15 to 20 %.
static int choose_splits(int n_heads, int32_t T, int64_t chunk_start) {
  const int64_t wgs = (int64_t)n_heads * ((T + kPwQ - 1) / kPwQ);
  const int64_t avg_tiles = (chunk_start + T / 2) / kPfK + 1;
  int64_t smax = avg_tiles / 32;
  if (smax > 8) smax = 8;
  if (wgs <= 0 || smax <= 1) return 1;
  const int64_t cus = compute_units();
  int best = 1;
  double best_cost = 0.0;
  for (int s = 1; s <= (int)smax; ++s) {
    const int64_t total = wgs * s, rounds = (total + cus - 1) / cus;
    const double cost = (double)(rounds * cus) / (double)total * (1.0 + 0.02 * (s - 1));
    if (s == 1 || cost < best_cost) {
      best = s;
      best_cost = cost;
    }
  }
  return best;
}

// Key ranges of a selecting launch that follows a threshold search: the query tiles' lists differ in length by
// orders of magnitude (a tile with one hard query visits everything, its neighbour a few dozen tiles), and the
// host does not see the lengths.  Ranges of at most ~512 listed tiles, many more workgroups than compute units:
// the hardware's workgroup dispatch does the balancing, a workgroup with an empty range leaves at once.
static int choose_splits_listed(int n_heads, int32_t T, int64_t chunk_start) {
  const int64_t max_tiles = (chunk_start + T - 1) / kPfK + 1;
  int64_t s = (max_tiles + 511) / 512;
  if (s > 32) s = 32;
  const int base = choose_splits(n_heads, T, chunk_start);
  return s > base ? (int)s : base;
}

static int32_t launch_prefill(const char* who, bool local, PrefillArgs& a, int32_t B, hipStream_t s) {
  if (a.n_heads == 0) return RTP_OK;
  if (a.n_splits < 1) a.n_splits = 1;
  // dense launches take the wide kernel; the local band (a few dozen key tiles per query tile, many of
  // them masked) stays on the 128-query kernel, whose masked tiles cost less (the wide kernel takes
  // twice as long for the band: its masked blocks leave the pipelined path)
  const int qt = local ? kPfQ : kPwQ;
  dim3 grid((unsigned)a.n_heads, (unsigned)((a.n_q + qt - 1) / qt), (unsigned)(B * (local ? 1 : a.n_splits)));
  if (grid.y > 65535 || grid.z > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: n_q / B too large for one launch", who);
  if (local) {
    if (a.f16) RTP_LAUNCH((flash_prefill_kernel<kModeLocal, true>), grid, dim3(kPfThreads), 0, s, a);
    else RTP_LAUNCH(flash_prefill_kernel<kModeLocal>, grid, dim3(kPfThreads), 0, s, a);
  } else if (a.f16) RTP_LAUNCH((flash_prefill_wide_kernel<kModeDense, 1, true>), grid, dim3(512), 0, s, a);
  else RTP_LAUNCH((flash_prefill_wide_kernel<kModeDense, 1>), grid, dim3(512), 0, s, a);
  if (!local && a.n_splits > 1)
    RTP_LAUNCH(prefill_combine_kernel, dim3((unsigned)((a.n_q + 1) / 2), (unsigned)a.n_heads), dim3(256), 0, s, a);
  return check_launch(who);
}

static int32_t check_prefill_common(const char* who, const void* q, const void* K, const void* V, int64_t row_stride,
                                    int64_t head_stride, const void* out) {
  if (!q || !K || !V || !out) return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (row_stride < kHeadDim || (row_stride & 7) || (head_stride & 7) || head_stride < 0)
    return fail(RTP_ERR_INVALID_ARG, "%s: kv_row_stride must be >= 128, strides multiples of 8", who);
  if (row_stride > (1 << 24))   // a 64-row tile must span less than 4 GiB (32-bit lane offsets inside a tile)
    return fail(RTP_ERR_INVALID_ARG, "%s: kv_row_stride must be at most 2^24 elements", who);
  if (((uintptr_t)q & 15) || ((uintptr_t)K & 15) || ((uintptr_t)V & 15) || ((uintptr_t)out & 15))
    return fail(RTP_ERR_INVALID_ARG, "%s: q, K, V and out must be 16-byte aligned", who);
  return RTP_OK;
}

// rtp_local_attn / rtp_dense_attn with q_start != NULL.
int32_t prefill_range_attn(const char* who, bool dense, const rtp_layer_desc* L, const void* q, const void* K,
                           const void* V, int64_t row_stride, int64_t head_stride, const int64_t* seq_start,
                           const int32_t* ctx_len, const int32_t* q_start, int32_t B, int32_t n_q, int64_t max_ctx,
                           void* out, float* lse, hipStream_t s) {
  HeadTable ht;
  int32_t rc = fill_head_table(L, &ht, who);
  if (rc != RTP_OK) return rc;
  rc = check_prefill_common(who, q, K, V, row_stride, head_stride, out);
  if (rc != RTP_OK) return rc;
  if (!seq_start || !ctx_len || !q_start) return fail(RTP_ERR_INVALID_ARG, "%s: NULL seq_start/ctx_len/q_start", who);
  if (B <= 0 || n_q <= 0 || max_ctx <= 0) return fail(RTP_ERR_INVALID_ARG, "%s: B, n_q and max_ctx must be positive", who);
  if (max_ctx > 0x7fffffffLL - kPwQ) return fail(RTP_ERR_INVALID_ARG, "%s: max_ctx too large", who);
  clear_error();
  PrefillArgs a = {};
  a.q = (const uint16_t*)q;
  a.K = (const uint16_t*)K;
  a.V = (const uint16_t*)V;
  a.row_stride = row_stride;
  a.head_stride = head_stride;
  a.seq_start = seq_start;
  a.q_start = q_start;
  a.n_q = n_q;
  a.n_q_heads = L->n_q_heads;
  a.n_kv_heads = L->n_kv_heads;
  a.sink = L->sink;
  a.window = L->window;
  a.scale = softmax_scale_of(L);
  a.f16 = L->kv_dtype == RTP_DTYPE_FP16;
  a.scale_log2 = a.scale * 1.4426950408889634f;
  a.out = (uint16_t*)out;
  a.lse = lse;
  a.n_heads = 0;
  for (int h = 0; h < L->n_q_heads; ++h)
    if (dense || !ht.is_ret[h]) a.heads[a.n_heads++] = (uint8_t)h;
  return launch_prefill(who, !dense, a, B, s);
}

// Sizes of the tile bookkeeping of a selecting launch.  A table row has one entry per 64 keys of the context, plus
// the entries the threshold search touches past a group's last tile (its sweeps run in whole rounds of 8 tiles of
// 32 keys and read the table one round ahead).
struct PrefillTileWs {
  int32_t n_t64;
  size_t table_bytes, list_bytes, count_bytes;
};
static PrefillTileWs prefill_tile_ws(int32_t n_ret, int32_t T, int64_t chunk_start) {
  PrefillTileWs w;
  w.n_t64 = (int32_t)(((chunk_start + T + 31) / 32 + 32) / 2 + 1);
  w.table_bytes = align_up((size_t)n_ret * ((T + 31) / 32) * w.n_t64 * sizeof(float), 256);
  w.list_bytes = align_up((size_t)n_ret * ((T + kPwQ - 1) / kPwQ) * w.n_t64 * sizeof(int32_t), 256);
  w.count_bytes = align_up(((size_t)n_ret * ((T + kPwQ - 1) / kPwQ) + 2) * sizeof(int32_t), 256);   // + {longest, shortest}
  return w;
}

}  // namespace rtp

using namespace rtp;

extern "C" size_t rtp_sparse_attn_prefill_workspace_bytes(const rtp_layer_desc* layer, int32_t T, int64_t chunk_start) {
  if (!layer || T <= 0 || layer->n_ret <= 0) return 256;
  // selecting mode: projected index queries, then one threshold per (retrieval head, query)
  const size_t proj = align_up((size_t)layer->n_ret * T * kIndexDim * sizeof(uint16_t), 256);
  const size_t state = align_up((size_t)layer->n_ret * T * sizeof(float), 256);
  // both rules: key-range partials
  const int ns = choose_splits_listed(layer->n_ret, T, chunk_start < 0 ? 0 : chunk_start);   // (the larger of the two rules)
  const size_t part = ns > 1 ? align_up((size_t)ns * layer->n_ret * T * kPfPart * sizeof(float), 256) : 0;
  // selecting mode: the tile-maximum table and the query tiles' lists of tiles to visit
  const PrefillTileWs tw = prefill_tile_ws(layer->n_ret, T, chunk_start < 0 ? 0 : chunk_start);
  return proj + state + part + tw.table_bytes + tw.list_bytes + tw.count_bytes;
}

extern "C" int32_t rtp_sparse_attn_prefill(const rtp_layer_desc* layer, const void* q_pre, const void* q, const float* WQ,
                                           const void* kI, int64_t kI_head_stride,
                                           const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                                           int64_t chunk_start, int32_t T, float p, void* out, float* lse,
                                           float* tau, int32_t* count, float* mass,
                                           void* ws, size_t ws_bytes, void* stream) {
  const char* who = "rtp_sparse_attn_prefill";
  HeadTable ht;
  int32_t rc = fill_head_table(layer, &ht, who);
  if (rc != RTP_OK) return rc;
  rc = check_prefill_common(who, q, K, V, kv_row_stride, kv_head_stride, out);
  if (rc != RTP_OK) return rc;
  if (T <= 0 || chunk_start < 0) return fail(RTP_ERR_INVALID_ARG, "%s: T must be positive and chunk_start >= 0", who);
  if (chunk_start + T > 0x7fffffffLL - kPwQ) return fail(RTP_ERR_INVALID_ARG, "%s: context too long", who);
  if (!(p > 0.f)) return fail(RTP_ERR_INVALID_ARG, "%s: p must be > 0", who);
  if ((T + kPfQ - 1) / kPfQ > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: T too large for one launch", who);
  const bool sparse = p < 1.f || tau || count || mass;
  if (sparse) {
    if (!q_pre || !kI) return fail(RTP_ERR_INVALID_ARG, "%s: NULL index tensors", who);
    if (((uintptr_t)q_pre & 15) || ((uintptr_t)kI & 15) || (kI_head_stride & 7) || kI_head_stride < 0)
      return fail(RTP_ERR_INVALID_ARG, "%s: index tensors must be 16-byte aligned, kI_head_stride a multiple of 8", who);
    if (layer->n_ret > 0) {
      const size_t need = rtp_sparse_attn_prefill_workspace_bytes(layer, T, chunk_start);
      if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)
        return fail(RTP_ERR_WORKSPACE, "%s: workspace of %zu bytes (256-byte aligned) required, got %zu", who, need, ws_bytes);
    }
  }
  clear_error();
  if (layer->n_ret == 0) return RTP_OK;
  PrefillArgs a = {};
  a.q = (const uint16_t*)q;
  a.K = (const uint16_t*)K;
  a.V = (const uint16_t*)V;
  a.row_stride = kv_row_stride;
  a.head_stride = kv_head_stride;
  a.seq_start = nullptr;
  a.q_start = nullptr;
  a.q_start_host = chunk_start;
  a.n_q = T;
  a.n_q_heads = layer->n_q_heads;
  a.n_kv_heads = layer->n_kv_heads;
  a.sink = layer->sink;
  a.window = layer->window;
  a.scale = softmax_scale_of(layer);
  a.f16 = layer->kv_dtype == RTP_DTYPE_FP16;
  a.scale_log2 = a.scale * 1.4426950408889634f;
  a.out = (uint16_t*)out;
  a.lse = lse;
  a.n_heads = layer->n_ret;
  for (int j = 0; j < layer->n_ret; ++j) a.heads[j] = (uint8_t)layer->ret_heads[j];
  if (!sparse) {                                     // the paper's dense prefill rule
    a.n_splits = choose_splits(layer->n_ret, T, chunk_start);
    if (a.n_splits > 1) {
      const size_t need = rtp_sparse_attn_prefill_workspace_bytes(layer, T, chunk_start);
      if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need) a.n_splits = 1;   // no scratch: run unsplit
      a.part = (float*)ws;
    }
    return launch_prefill(who, false, a, 1, (hipStream_t)stream);
  }

  // index queries: given, or projected in fp64 into the workspace first
  const uint16_t* qI = (const uint16_t*)q_pre;
  if (WQ) {
    ProjectArgs pa;
    pa.W = WQ;
    pa.x = (const uint16_t*)q_pre;
    pa.out = (uint16_t*)ws;
    pa.n_q = T;
    pa.n_q_heads = layer->n_q_heads;
    pa.n_ret = layer->n_ret;
    for (int j = 0; j < 64; ++j) pa.ret_heads[j] = j < layer->n_ret ? layer->ret_heads[j] : 0;
    RTP_LAUNCH(index_project_kernel, dim3((unsigned)((T + 15) / 16), (unsigned)layer->n_ret), dim3(256), 0,
                       (hipStream_t)stream, pa);
    qI = (const uint16_t*)ws;
  }
  a.qI = qI;
  a.kI = (const uint16_t*)kI;
  a.kI_head_stride = kI_head_stride;
  a.p = p;
  a.index_scale = index_scale_of(layer);
  a.tau = tau;
  a.count = count;
  a.mass = mass;
  const size_t proj_bytes = align_up((size_t)layer->n_ret * T * kIndexDim * sizeof(uint16_t), 256);
  const size_t state_bytes = align_up((size_t)layer->n_ret * T * sizeof(float), 256);
  a.sel_thr = (float*)((char*)ws + proj_bytes);
  a.part = (float*)((char*)ws + proj_bytes + state_bytes);
  a.n_splits = p < 1.f ? choose_splits_listed(layer->n_ret, T, chunk_start) : choose_splits(layer->n_ret, T, chunk_start);
  {
    // (the layout does not depend on p: the partials' region has the size of the larger rule)
    const int ns_ws = choose_splits_listed(layer->n_ret, T, chunk_start);
    const size_t part_bytes = ns_ws > 1 ? align_up((size_t)ns_ws * layer->n_ret * T * kPfPart * sizeof(float), 256) : 0;
    const PrefillTileWs tw = prefill_tile_ws(layer->n_ret, T, chunk_start);
    char* at = (char*)ws + proj_bytes + state_bytes + part_bytes;
    a.n_t64 = tw.n_t64;
    a.tile_max = (float*)at;
    a.act_list = (int32_t*)(at + tw.table_bytes);
    a.act_count = (int32_t*)(at + tw.table_bytes + tw.list_bytes);
    if (p < 1.f) {
      // (the last two ints of the counts' region)
      a.act_range = a.act_count + (tw.count_bytes / sizeof(int32_t) - 2);
      a.n_splits_even = std::max(2, choose_splits(layer->n_ret, T, chunk_start));
    }
  }
  if (p < 1.f) {
    constexpr int ks = 8;                                  // waves per 32-query group (see the kernel's header)
    static_assert(ks == 8, "the launch below names the instantiation");
    const unsigned n_qtiles = (unsigned)((T + 256 / ks - 1) / (256 / ks));
    // 1-D grid, padded so that every die gets whole (head, query tile) columns (see the kernel's decoding)
    unsigned wgs = (unsigned)a.n_heads * n_qtiles;
    if (a.n_heads <= 8 && 8 % a.n_heads == 0) {
      const unsigned per_head = 8u / (unsigned)a.n_heads;
      wgs = 8u * ((n_qtiles + per_head - 1) / per_head);
    }
    RTP_LAUNCH(prefill_select_kernel<8>, dim3(wgs), dim3(kSelThreads), 0, (hipStream_t)stream, a);
    RTP_LAUNCH(prefill_active_tiles_kernel, dim3((unsigned)((T + kPwQ - 1) / kPwQ), (unsigned)a.n_heads), dim3(256), 0,
               (hipStream_t)stream, a);
  }
  dim3 grid((unsigned)a.n_heads, (unsigned)((T + kPwQ - 1) / kPwQ), (unsigned)a.n_splits);
  if (p < 1.f) grid = dim3((unsigned)a.n_splits, (unsigned)((T + kPwQ - 1) / kPwQ), (unsigned)a.n_heads);
  if (a.f16) RTP_LAUNCH((flash_prefill_wide_kernel<kModeSparse, 1, true>), grid, dim3(512), 0, (hipStream_t)stream, a);
  else RTP_LAUNCH((flash_prefill_wide_kernel<kModeSparse, 1>), grid, dim3(512), 0, (hipStream_t)stream, a);
  if (a.n_splits > 1)
    RTP_LAUNCH(prefill_combine_kernel, dim3((unsigned)((T + 1) / 2), (unsigned)a.n_heads), dim3(256), 0,
                       (hipStream_t)stream, a);
  return check_launch(who);
}

extern "C" int32_t rtp_sparse_attn_prefill_tile_stats(const rtp_layer_desc* layer, int32_t T, int64_t chunk_start,
                                                      const void* ws, size_t ws_bytes, void* stream,
                                                      int64_t* tiles_visited, int64_t* tiles_causal) {
  const char* who = "rtp_sparse_attn_prefill_tile_stats";
  HeadTable ht;
  int32_t rc = fill_head_table(layer, &ht, who);
  if (rc != RTP_OK) return rc;
  if (T <= 0 || chunk_start < 0 || !tiles_visited || !tiles_causal)
    return fail(RTP_ERR_INVALID_ARG, "%s: T must be positive, chunk_start >= 0, outputs non-NULL", who);
  if (layer->n_ret <= 0) {
    *tiles_visited = *tiles_causal = 0;
    return RTP_OK;
  }
  const size_t need = rtp_sparse_attn_prefill_workspace_bytes(layer, T, chunk_start);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)
    return fail(RTP_ERR_WORKSPACE, "%s: the workspace of the rtp_sparse_attn_prefill call (%zu bytes) is required", who, need);
  clear_error();
  const PrefillTileWs tw = prefill_tile_ws(layer->n_ret, T, chunk_start);
  const int n_qt = (T + kPwQ - 1) / kPwQ;
  std::vector<int32_t> counts((size_t)layer->n_ret * n_qt);
  // the counts are the last region of the workspace
  const char* at = (const char*)ws + need - tw.count_bytes;
  hipError_t e = hipStreamSynchronize((hipStream_t)stream);
  if (e == hipSuccess) e = hipMemcpy(counts.data(), at, counts.size() * sizeof(int32_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail(RTP_ERR_HIP, "%s: %s", who, hipGetErrorString(e));
  int64_t vis = 0, causal = 0;
  for (size_t i = 0; i < counts.size(); ++i) vis += counts[i];
  for (int qt = 0; qt < n_qt; ++qt) {
    const int64_t m_hi = chunk_start + (int64_t)std::min(qt * kPwQ + kPwQ, T) - 1;
    causal += (m_hi / kPfK + 1) * layer->n_ret;
  }
  *tiles_visited = vis;
  *tiles_causal = causal;
  return RTP_OK;
}
