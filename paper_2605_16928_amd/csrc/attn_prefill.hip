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
constexpr int kSmemDense = (kPfK * kKsStride + kHeadDim * kVtStride) * 2;
constexpr int kSmemSparse = (kPfThreads / 64) * 32 * kSelBins * 8;

__device__ __forceinline__ int sel_q(float M, float s) {
  return (int)fminf((M - s) * kSelScale, (float)kSelQMax);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const f32x2 f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

template <int MODE>
__global__ __launch_bounds__(kPfThreads) void flash_prefill_kernel(const PrefillArgs a) {
  constexpr bool LOCAL = MODE == kModeLocal;
  constexpr bool SPARSE = MODE == kModeSparse;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SPARSE ? (kSmemSparse > kSmemDense ? kSmemSparse : kSmemDense)
                                                                    : kSmemDense];
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);
  uint16_t* Vt = Ks + kPfK * kKsStride;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;
  const int h = a.heads[blockIdx.x];
  const int b = blockIdx.z;
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

  for (int it = 0; it < n_tiles; ++it) {
    const int kt = it < ks_end ? it : kt_w0 + (it - ks_end);
    const int n0 = kt * kPfK;

    // ---- sparse mode: which (key, query) pairs of this tile are in the active sets ----
    uint32_t selmask[2] = {0xffffu, 0xffffu};       // bit i: accumulator element i of block kb is kept
    if (SPARSE) {
      const int n_rows = pos0 + a.n_q;
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
    }

    // ---- stage K (row-major) and V (transposed) in LDS ----
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = i * kPfThreads + tid;
      const int key = idx >> 4, ck = idx & 15;
      const int n = n0 + key;
      u32x4 v = (u32x4){0u, 0u, 0u, 0u};
      if (n <= m_hi) v = *reinterpret_cast<const u32x4*>(Kg + (int64_t)n * a.row_stride + ck * 8);
      *reinterpret_cast<u32x4*>(&Ks[key * kKsStride + ck * 8]) = v;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int key = i * 16 + (tid & 15), ck = tid >> 4;
      const int n = n0 + key;
      u32x4 v = (u32x4){0u, 0u, 0u, 0u};
      if (n <= m_hi) v = *reinterpret_cast<const u32x4*>(Vg + (int64_t)n * a.row_stride + ck * 8);
      uint16_t* dst = &Vt[(ck * 8) * kVtStride + key];
      dst[0 * kVtStride] = (uint16_t)(v.x & 0xffffu);
      dst[1 * kVtStride] = (uint16_t)(v.x >> 16);
      dst[2 * kVtStride] = (uint16_t)(v.y & 0xffffu);
      dst[3 * kVtStride] = (uint16_t)(v.y >> 16);
      dst[4 * kVtStride] = (uint16_t)(v.z & 0xffffu);
      dst[5 * kVtStride] = (uint16_t)(v.z >> 16);
      dst[6 * kVtStride] = (uint16_t)(v.w & 0xffffu);
      dst[7 * kVtStride] = (uint16_t)(v.w >> 16);
    }
    __syncthreads();

    // ---- S^T = K Q^T : two 32-key blocks ----
    f32x16 S[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) S[kb][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const u32x4 ka = *reinterpret_cast<const u32x4*>(&Ks[(kb * 32 + r) * kKsStride + kk * 16 + g * 8]);
        S[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka),
                                                        __builtin_bit_cast(bf16x8, qreg[kk]), S[kb], 0, 0, 0);
      }
    }

    // ---- mask, online softmax (per-lane state: this lane's query) ----
    float mx = ninf;
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
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mnew = fmaxf(mrow, mx);
    uint32_t P[2][8];
    if (mnew == ninf) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 8; ++i) P[kb][i] = 0u;
    } else {
      const float corr = fast_exp2((mrow - mnew) * c);
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
      lrow = lrow * corr + lsum;
      mrow = mnew;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[db][i] *= corr;
    }

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const u32x4 pb = (u32x4){P[kb][4 * tt], P[kb][4 * tt + 1], P[kb][4 * tt + 2], P[kb][4 * tt + 3]};
        const int kbase = kb * 32 + tt * 16 + g * 4;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const uint16_t* vrow = &Vt[(db * 32 + r) * kVtStride + kbase];
          const u32x2 lo = *reinterpret_cast<const u32x2*>(vrow);
          const u32x2 hi = *reinterpret_cast<const u32x2*>(vrow + 8);
          const u32x4 va = (u32x4){lo.x, lo.y, hi.x, hi.y};
          O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va),
                                                          __builtin_bit_cast(bf16x8, pb), O[db], 0, 0, 0);
        }
      }
    }
    __syncthreads();
  }

  // ---- normalise and store ----
  const float ltot = lrow + __shfl_xor(lrow, 32);
  if (!qok) return;
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

static int32_t launch_prefill(const char* who, bool local, PrefillArgs& a, int32_t B, hipStream_t s) {
  if (a.n_heads == 0) return RTP_OK;
  dim3 grid((unsigned)a.n_heads, (unsigned)((a.n_q + kPfQ - 1) / kPfQ), (unsigned)B);
  if (grid.y > 65535 || grid.z > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: n_q / B too large for one launch", who);
  if (local) hipLaunchKernelGGL(flash_prefill_kernel<kModeLocal>, grid, dim3(kPfThreads), 0, s, a);
  else hipLaunchKernelGGL(flash_prefill_kernel<kModeDense>, grid, dim3(kPfThreads), 0, s, a);
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
  (void)chunk_start;
  if (!layer || T <= 0 || layer->n_ret <= 0) return 256;
  return align_up((size_t)layer->n_ret * T * kIndexDim * sizeof(uint16_t), 256);   // projected index queries
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
  if (!sparse) return launch_prefill(who, false, a, 1, (hipStream_t)stream);   // the paper's dense prefill rule

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
