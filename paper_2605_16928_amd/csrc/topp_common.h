// Pieces of the top-p threshold search shared by the selector (topp.hip) and the score pass
// (index_score.hip), which can accumulate the first histogram level while it produces the scores.
//
// The search works on the order-preserving 32-bit key of an fp32 score, in three radix levels of
// 11 + 11 + 10 bits.  A level histograms softmax MASS per bin.  Masses are 64-bit integers:
//   w = floor-rounded( exp(s - ref) * 2^shift ),  ref = the upper edge of the element's LEVEL-1 bin,
// so that no row maximum is needed before the first pass (every bin has its own reference, exp <= 1)
// and sums do not depend on the order in which atomics land.  The scan of level 1 rescales the bins to
// a common reference in fp64; levels 2 and 3 live inside one level-1 bin and stay pure integer.
#pragma once

#include "common.h"
#include "exp2_table.h"

namespace rtp {

constexpr int kBins1 = 2048, kBins2 = 2048, kBins3 = 1024;
constexpr int kBinsTotal = kBins1 + kBins2 + kBins3;

// weights are <= 2^shift and a row has n of them: n * 2^shift must stay below 2^63; shift <= 51 keeps
// every weight below 2^52, which the integer conversion in fixed_weight relies on
__device__ __forceinline__ int fixed_shift(int n) {
  const int lg = 32 - __clz(max(n, 2) - 1);      // ceil(log2 n)
  return min(51, 62 - lg);
}

// Upper edge (as a finite float) of level-1 bin `bin` = the reference of every score in that bin.
__device__ __forceinline__ float bin_ref(int bin) {
  const float f = key_float(((uint32_t)bin << 21) | 0x1fffffu);
  const uint32_t u = __float_as_uint(f);
  if ((u & 0x7f800000u) == 0x7f800000u) return __uint_as_float((u & 0x80000000u) | 0x7f7fffffu);   // inf/nan bins
  return f;
}

// The same edge straight from a finite score: the low 21 bits set for s >= 0, cleared for s < 0.
__device__ __forceinline__ float score_ref(float s) {
  const uint32_t u = __float_as_uint(s);
  const uint32_t neg = (uint32_t)((int32_t)u >> 31) & 0x1fffffu;
  return __uint_as_float((u | 0x1fffffu) ^ neg);
}

// 2^(j/256), j < 256: the table behind fixed_weight, copied into LDS (256 threads, then a barrier).  The
// values are constants (exp2_table.h): computing them costs every workgroup a double-precision exp2 per thread
// at the very start, when all workgroups of a launch do the same thing at once.
__device__ __forceinline__ void fill_exp_table(double* tab) {
  if (threadIdx.x < 256) tab[threadIdx.x] = kExp2Frac256[threadIdx.x];
}

// exp(x) for x <= 0 as m * 2^e with m in [1, 2): x * 256 / ln 2 = k + f, k integer, f in [0, 1);
// exp(x) = 2^(k >> 8) * T[k & 255] * P(t), P a degree-4 polynomial in t = f * ln 2 / 256 < 2.8e-3
// (~1e-15 relative).  Arguments below about -80 return e = -119 or so: far under any resolution used.
__device__ __forceinline__ double exp_parts(double x, const double* __restrict__ tab, int* e, double y_min = -30000.0) {
  const double y = fmax(fmin(x, 0.0) * 369.3299304675746, y_min);      // 256 / ln 2
  const double k = floor(y);
  const double t = (y - k) * 0.0027076061740622863;                    // ln 2 / 256
  const int ki = (int)k;
  double pl = fma(t, 1.0 / 24.0, 1.0 / 6.0);
  pl = fma(t, pl, 0.5);
  pl = fma(t, pl, 1.0);
  pl = fma(t, pl, 1.0);
  *e = ki >> 8;
  return tab[ki & 255] * pl;
}

// round-to-nearest-even( exp(s - ref) * 2^shift ) as an integer, s <= ref, shift <= 51.  The value is
// below 2^52, so adding 2^52 leaves the rounded integer in the low 52 bits of the sum.
__device__ __forceinline__ uint64_t fixed_weight(float s, float ref, int shift, const double* __restrict__ tab) {
  int e;
  // s lies in the bin whose upper edge ref is: same binade, so the fp32 difference is exact
  const double m = exp_parts((double)(s - ref), tab, &e);
  const double r = ldexp(m, shift + e) + 4503599627370496.0;
  return (uint64_t)__double_as_longlong(r) & 0xFFFFFFFFFFFFFull;
}

// Level-1 bins are quarter binades of the score.  While |s| < 128 a bin is at most 16 wide, so a weight is
// at least e^-16 * 2^shift (>= 2^8 for the longest row) and keeps a relative resolution of 2^-8 or far better.
// From |s| = 128 on the bins are 32 and more wide and a weight relative to the bin's edge can round to
// nothing; a row whose LARGEST score lies out there cannot be resolved and is reported as unsupported
// (sel_count = -2) instead: such scores still mark their bin (weight 1), so the scan sees where the row's top is.
constexpr int kBin1FirstWidePos = 1024 + 134 * 4;     // first bin of s >= 128
constexpr int kBin1LastWideNeg = 1023 - 134 * 4;      // last bin (from below) of s <= -128
__device__ __forceinline__ bool level1_bin_is_wide(int bin) { return bin >= kBin1FirstWidePos || bin <= kBin1LastWideNeg; }

// Adds one score to a level-1 LDS histogram (2048 x u64).  -inf scores carry no mass; +inf and NaN
// scores are not supported (they land in the top bins with weight 2^shift).
__device__ __forceinline__ void level1_add(uint64_t* lh, float s, int shift, const double* tab) {
  if (s == -__builtin_huge_valf()) return;
  const int bin = (int)(float_key(s) >> 21);
  uint64_t w = fixed_weight(s, fminf(score_ref(s), 3.4028234663852886e38f), shift, tab);
  if (!w && level1_bin_is_wide(bin)) w = 1;
  if (w) atomicAdd((unsigned long long*)&lh[bin], (unsigned long long)w);
}

// Adds the non-empty bins of an LDS histogram to a global one.
__device__ __forceinline__ void flush_hist(const uint64_t* lh, uint64_t* gh, int nbins, int nthreads) {
  for (int i = threadIdx.x; i < nbins; i += nthreads) {
    const uint64_t v = lh[i];
    if (v) atomicAdd((unsigned long long*)&gh[i], (unsigned long long)v);
  }
}

// Workspace of one rtp_topp_select call (R rows of at most max_len scores).  rtp_index_score uses
// the same layout when it is asked to accumulate level 1.
struct TopPLayout {
  size_t ccnt_off, hist_off, state_off, bn_off, bucket_off, total;
  // A row's histograms: level 1 (copy 0), level 2, level 3, then n_sub - 1 more copies of level 1.  With few
  // rows every workgroup of a long row would add its level-1 bins to the same hundred addresses (256
  // workgroups per row at 1M tokens), and those atomics queue up at the end of the score pass; the workgroups
  // of a row therefore spread over n_sub copies, which the level-2 prologue adds up.
  int32_t n_sub;
  int64_t hist_stride;     // 64-bit words per row
};
// where copy `sub` of a row's level-1 histogram starts, in words from the row's start
__host__ __device__ inline int64_t level1_copy_offset(int sub) { return sub == 0 ? 0 : kBinsTotal + (int64_t)(sub - 1) * kBins1; }
TopPLayout topp_layout(int32_t R, int64_t max_len);

}  // namespace rtp
