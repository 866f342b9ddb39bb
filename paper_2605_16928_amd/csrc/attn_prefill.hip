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
};

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
constexpr int kSmemSparse = (kPfThreads / 64) * 32 * kSelBins * 8;

__device__ __forceinline__ int sel_q(float M, float s) {
  return (int)fminf((M - s) * kSelScale, (float)kSelQMax);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const f32x2 f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

template <int MODE>
__global__ __launch_bounds__(kPfThreads, 2) void flash_prefill_kernel(const PrefillArgs a) {
  constexpr bool LOCAL = MODE == kModeLocal;
  constexpr bool SPARSE = MODE == kModeSparse;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SPARSE ? (kSmemSparse > kSmemDense ? kSmemSparse : kSmemDense)
                                                                    : kSmemDense];
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;
  const int h = a.heads[blockIdx.x];
  const int n_splits = SPARSE || LOCAL ? 1 : a.n_splits;
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

  // ---- sparse mode: per-query top-p threshold over the indexer scores (three sweeps over kI) ----
  // Every wave works alone on its 32 queries.  The index-score tile is ONE MFMA (K = 16) in the same
  // transposed layout as the attention scores, so a lane sees 16 keys of its own query.
  u32x4 qIreg = (u32x4){0u, 0u, 0u, 0u};
  const uint16_t* kIg = nullptr;
  float selM = ninf;          // row maximum of the index scores
  int selQ = 0x7fffffff;      // keep a candidate iff sel_q(selM, s) <= selQ; the default keeps everything
  float sel_mass = 1.f;
  int sel_cnt = 0;
  if (SPARSE) {
    const int j = blockIdx.x;
    kIg = a.kI + (int64_t)j * a.kI_head_stride;
    if (qok) qIreg = *reinterpret_cast<const u32x4*>(a.qI + ((int64_t)j * a.n_q + t) * kIndexDim + g * 8);
    const int n_rows = pos0 + a.n_q;                          // index-key rows that exist
    const int m_wave_hi = pos0 + min(t0 + wave * 32 + 32, a.n_q) - 1;
    double* hist = reinterpret_cast<double*>(smem) + (wave * 32 + r) * kSelBins;   // this query's bins
    const bool keep_all = !(a.p < 1.f);
    double Z = 0.0, above = 0.0;
    int prefix = 0;            // digits of the threshold found so far
    // Control flow around the barriers is uniform: every thread runs all four sweeps (or none when
    // p >= 1); per-lane state only decides what a lane accumulates.
    for (int phase = 0; phase < 4 && !keep_all; ++phase) {
      if (phase > 0) {
        for (int i = g; i < kSelBins; i += 2) hist[i] = 0.0;
        __syncthreads();
      }
      const int shift = 7 * (3 - phase);                      // phase 1: 14, phase 2: 7, phase 3: 0
      float mx = ninf;
      for (int nb = 0; nb <= m_wave_hi; nb += 32) {
        const int nrow = nb + r;
        u32x4 ka = (u32x4){0u, 0u, 0u, 0u};
        if (nrow < n_rows) ka = *reinterpret_cast<const u32x4*>(kIg + (int64_t)nrow * kIndexDim + g * 8);
        f32x16 SI;
#pragma unroll
        for (int i = 0; i < 16; ++i) SI[i] = 0.f;
        SI = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka), __builtin_bit_cast(bf16x8, qIreg),
                                                     SI, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int n = nb + (i >> 2) * 8 + g * 4 + (i & 3);
          const bool ok = qok && n <= m;
          const float sv = SI[i] * a.index_scale;
          if (phase == 0) {
            mx = fmaxf(mx, ok ? sv : ninf);
          } else if (ok) {
            const int qv = sel_q(selM, sv);
            if (phase == 1 || (qv >> (shift + 7)) == prefix) {
              const float wgt = fast_exp2((sv - selM) * 1.4426950408889634f);
              atomicAdd(&hist[(qv >> shift) & (kSelBins - 1)], (double)wgt);
            }
          }
        }
      }
      if (phase == 0) {
        selM = fmaxf(mx, __shfl_xor(mx, 32));
      } else {
        __syncthreads();
        // scan this query's bins from the top of the score range (bin 0) down; both lanes of the
        // pair run the same scan on the same numbers
        if (phase == 1) {
          Z = 0.0;
          for (int i = 0; i < kSelBins; ++i) Z += hist[i];
        }
        const double target = (double)a.p * Z;
        double cum = above, hsel = 0.0;
        int bsel = kSelBins - 1;
        bool found = false;
        for (int i = 0; i < kSelBins; ++i) {
          const double hv = hist[i];
          if (!found) {
            if (cum + hv >= target) { bsel = i; hsel = hv; found = true; }
            else cum += hv;
          }
        }
        prefix = (prefix << 7) | bsel;
        above = cum;
        if (phase == 3) {
          // a threshold inside the open-ended last coarse bin keeps every candidate
          const bool lump = (prefix >> 14) == kSelBins - 1;
          selQ = lump ? 0x7fffffff : prefix;
          sel_mass = (lump || !(Z > 0.0)) ? 1.f : (float)((cum + hsel) / Z);
        }
        __syncthreads();
      }
    }
    __syncthreads();             // the histogram memory becomes the K/V tile buffers
  }

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
  auto compute_tile = [&](int buf, int n0, const uint32_t (&selmask)[2]) {
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
        S[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka),
                                                        __builtin_bit_cast(bf16x8, qreg[kk]), S[kb], 0, 0, 0);
      }
    }
    // interior tiles (every key visible to every query of the wave) skip the mask arithmetic
    const bool masked = SPARSE || (n0 + kPfK - 1 > m_wave_lo) || (LOCAL && n0 <= m_wave_hi - a.window);
    float mx = ninf;
    if (masked) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int n = n0 + kb * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
          bool ok = qok && n <= m;
          if (LOCAL) ok = ok && (n < a.sink || n > m - a.window);
          if (SPARSE) ok = (selmask[kb] >> i) & 1u;
          S[kb][i] = ok ? S[kb][i] : ninf;
          mx = fmaxf(mx, S[kb][i]);
        }
      }
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[kb][i]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
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
          P[kb][i >> 1] = pack_bf16(p0, p1);
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
          O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va),
                                                          __builtin_bit_cast(bf16x8, pb), O[db], 0, 0, 0);
        }
      }
    }
  };

  if (SPARSE) {
    // Selecting mode: a tile is staged only if some query of the workgroup keeps one of its keys.
    const int n_rows = pos0 + a.n_q;
    for (int kt = 0; kt <= kt_end; ++kt) {
      const int n0 = kt * kPfK;
      uint32_t selmask[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const int nrow = n0 + kb * 32 + r;
        u32x4 ka = (u32x4){0u, 0u, 0u, 0u};
        if (nrow < n_rows) ka = *reinterpret_cast<const u32x4*>(kIg + (int64_t)nrow * kIndexDim + g * 8);
        f32x16 SI;
#pragma unroll
        for (int i = 0; i < 16; ++i) SI[i] = 0.f;
        SI = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka), __builtin_bit_cast(bf16x8, qIreg),
                                                     SI, 0, 0, 0);
        uint32_t mk = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int n = n0 + kb * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
          bool keep = qok && n <= m;
          if (selQ != 0x7fffffff) keep = keep && sel_q(selM, SI[i] * a.index_scale) <= selQ;
          mk |= (keep ? 1u : 0u) << i;
        }
        selmask[kb] = mk;
        sel_cnt += __popc(mk);
      }
      const int wave_any = (__ballot((selmask[0] | selmask[1]) != 0u) != 0ull) ? 1 : 0;
      if (!__syncthreads_or(wave_any)) continue;     // nobody in the workgroup needs this key tile
      load_tile(n0);
      store_tile(0);
      __syncthreads();
      if (wave_any) compute_tile(0, n0, selmask);
    }
  } else {
    // Software pipeline: the global loads of tile it+1 are in flight while tile it is computed from
    // the other LDS buffer; one barrier per tile.
    const uint32_t nomask[2] = {0xffffu, 0xffffu};
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
      compute_tile(it & 1, tile_n0(it), nomask);
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
      const u32x2 w = (u32x2){pack_bf16(O[db][i4 * 4] * inv, O[db][i4 * 4 + 1] * inv),
                              pack_bf16(O[db][i4 * 4 + 2] * inv, O[db][i4 * 4 + 3] * inv)};
      *reinterpret_cast<u32x2*>(orow + db * 32 + i4 * 8 + g * 4) = w;
    }
  }
  if (a.lse && g == 0) {
    a.lse[((int64_t)b * a.n_q + t) * a.n_q_heads + h] = ltot > 0.f ? mrow * a.scale + logf(ltot) : ninf;
  }
  if (SPARSE) {
    const int cnt = sel_cnt + __shfl_xor(sel_cnt, 32);
    if (g == 0) {
      const int64_t o = (int64_t)blockIdx.x * a.n_q + t;
      if (a.count) a.count[o] = cnt;
      if (a.mass) a.mass[o] = sel_mass;
      // kept: scores s with floor((M - s) * 2^17) <= selQ, i.e. s > M - (selQ + 1) / 2^17
      if (a.tau) a.tau[o] = selQ != 0x7fffffff ? selM - (float)(selQ + 1) * (1.0f / kSelScale) : ninf;
    }
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
  float M = ninf;
  for (int s = 0; s < a.n_splits; ++s) M = fmaxf(M, a.part[(((int64_t)s * a.n_heads + hs) * a.n_q + t) * kPfPart]);
  float L = 0.f, A = 0.f;
  if (M != ninf) {
    for (int s = 0; s < a.n_splits; ++s) {
      const float* p = a.part + (((int64_t)s * a.n_heads + hs) * a.n_q + t) * kPfPart;
      if (p[0] == ninf) continue;
      const float cw = fast_exp2((p[0] - M) * a.scale_log2);
      L += p[1] * cw;
      A += p[4 + d] * cw;
    }
  }
  const int h = a.heads[hs];
  const int64_t o = (int64_t)t * a.n_q_heads + h;        // single sequence
  a.out[o * kHeadDim + d] = f32_to_bf16_rne(L > 0.f ? A / L : 0.f);
  if (a.lse && d == 0) a.lse[o] = L > 0.f ? M * a.scale + logf(L) : ninf;
}

// Number of key-range splits for a dense launch with few workgroups (long context, few heads).
static int choose_splits(int n_heads, int32_t T, int64_t chunk_start) {
  const int64_t wgs = (int64_t)n_heads * ((T + kPfQ - 1) / kPfQ);
  const int64_t avg_tiles = (chunk_start + T / 2) / kPfK + 1;
  int64_t s = 1024 / (wgs > 0 ? wgs : 1);
  if (s > avg_tiles / 32) s = avg_tiles / 32;
  if (s > 8) s = 8;
  return s < 1 ? 1 : (int)s;
}

static int32_t launch_prefill(const char* who, bool local, PrefillArgs& a, int32_t B, hipStream_t s) {
  if (a.n_heads == 0) return RTP_OK;
  if (a.n_splits < 1) a.n_splits = 1;
  dim3 grid((unsigned)a.n_heads, (unsigned)((a.n_q + kPfQ - 1) / kPfQ), (unsigned)(B * (local ? 1 : a.n_splits)));
  if (grid.y > 65535 || grid.z > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: n_q / B too large for one launch", who);
  if (local) hipLaunchKernelGGL(flash_prefill_kernel<kModeLocal>, grid, dim3(kPfThreads), 0, s, a);
  else hipLaunchKernelGGL(flash_prefill_kernel<kModeDense>, grid, dim3(kPfThreads), 0, s, a);
  if (!local && a.n_splits > 1)
    hipLaunchKernelGGL(prefill_combine_kernel, dim3((unsigned)((a.n_q + 1) / 2), (unsigned)a.n_heads), dim3(256), 0, s, a);
  return check_launch(who);
}

static int32_t check_prefill_common(const char* who, const void* q, const void* K, const void* V, int64_t row_stride,
                                    int64_t head_stride, const void* out) {
  if (!q || !K || !V || !out) return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (row_stride < kHeadDim || (row_stride & 7) || (head_stride & 7) || head_stride < 0)
    return fail(RTP_ERR_INVALID_ARG, "%s: kv_row_stride must be >= 128, strides multiples of 8", who);
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
  if (max_ctx > 0x7fffffffLL - kPfQ) return fail(RTP_ERR_INVALID_ARG, "%s: max_ctx too large", who);
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
  a.scale_log2 = a.scale * 1.4426950408889634f;
  a.out = (uint16_t*)out;
  a.lse = lse;
  a.n_heads = 0;
  for (int h = 0; h < L->n_q_heads; ++h)
    if (dense || !ht.is_ret[h]) a.heads[a.n_heads++] = (uint8_t)h;
  return launch_prefill(who, !dense, a, B, s);
}

}  // namespace rtp

using namespace rtp;

extern "C" size_t rtp_sparse_attn_prefill_workspace_bytes(const rtp_layer_desc* layer, int32_t T, int64_t chunk_start) {
  if (!layer || T <= 0 || layer->n_ret <= 0) return 256;
  const size_t proj = align_up((size_t)layer->n_ret * T * kIndexDim * sizeof(uint16_t), 256);   // projected index queries
  const int ns = choose_splits(layer->n_ret, T, chunk_start < 0 ? 0 : chunk_start);
  const size_t part = ns > 1 ? align_up((size_t)ns * layer->n_ret * T * kPfPart * sizeof(float), 256) : 0;
  return proj > part ? proj : part;
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
  if (chunk_start + T > 0x7fffffffLL - kPfQ) return fail(RTP_ERR_INVALID_ARG, "%s: context too long", who);
  if (!(p > 0.f)) return fail(RTP_ERR_INVALID_ARG, "%s: p must be > 0", who);
  const bool sparse = p < 1.f || tau || count || mass;
  if (sparse) {
    if (!q_pre || !kI) return fail(RTP_ERR_INVALID_ARG, "%s: NULL index tensors", who);
    if (((uintptr_t)q_pre & 15) || ((uintptr_t)kI & 15) || (kI_head_stride & 7) || kI_head_stride < 0)
      return fail(RTP_ERR_INVALID_ARG, "%s: index tensors must be 16-byte aligned, kI_head_stride a multiple of 8", who);
    if (layer->n_ret > 0 && WQ) {
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
    hipLaunchKernelGGL(index_project_kernel, dim3((unsigned)((T + 15) / 16), (unsigned)layer->n_ret), dim3(256), 0,
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
  dim3 grid((unsigned)a.n_heads, (unsigned)((T + kPfQ - 1) / kPfQ), 1);
  if (grid.y > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: T too large for one launch", who);
  hipLaunchKernelGGL(flash_prefill_kernel<kModeSparse>, grid, dim3(kPfThreads), 0, (hipStream_t)stream, a);
  return check_launch(who);
}
