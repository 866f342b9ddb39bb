// rtp_topp_select: sort-free dynamic top-p (paper Sec. 3.2, S = Top-P(s, p); Sec. 3.4, the threshold
// "at which the cumulative attention mass reaches p").
//
// Design (ours, for gfx950; the paper's kernel uses one 256-bin histogram of block maxima):
// a three-level radix search over the order-preserving 32-bit key of each fp32 score
// (11 + 11 + 10 bits).  Level L histograms the softmax mass w = exp(s - max) of the elements whose
// higher key bits equal the prefix found so far; scanning the histogram from the top finds the bin in
// which the descending cumulative mass crosses p * Z.  After three levels the threshold key is exact.
// Masses are fp64 exponentials converted to 64-bit fixed point, so every sum is an integer sum and
// the result is independent of the order in which atomics land.
//
// Launches: init (row maxima per chunk, zero histograms) -> level 1 -> level 2 -> level 3 -> count -> write.
// The selected positions come out in ascending order (deterministic, and friendly to the K/V gather).
// There is no "last block" hand-off: each level's histogram is scanned redundantly in the prologue
// of every workgroup of the NEXT launch, so kernel boundaries provide all ordering.
// A row is cut into chunks of kChunk scores, one workgroup each; histograms live in LDS and only
// non-empty bins are flushed with 64-bit global atomics.
#include "common.h"

#include <stdlib.h>

namespace rtp {

constexpr int kTpThreads = 256;
#ifndef RTP_TP_CHUNK
#define RTP_TP_CHUNK 4096
#endif
constexpr int kTpChunk = RTP_TP_CHUNK;     // scores per workgroup (2048, 4096 or 8192)
constexpr int kTpVec = kTpChunk / (kTpThreads * 4);   // float4 loads per thread = 8
constexpr int kBins1 = 2048, kBins2 = 2048, kBins3 = 1024;
constexpr int kBinsTotal = kBins1 + kBins2 + kBins3;

struct RowState {          // one per row and level (3 per row)
  uint64_t above;          // fixed-point mass of keys strictly above the current prefix range
  uint64_t target;         // fixed-point p * Z
  uint64_t total;          // fixed-point Z
  uint32_t prefix;         // key bits resolved so far (right-aligned)
  int32_t flags;           // 0 ok, 1 = keep everything (p >= 1), -1 = invalid p
  float smax;
  int32_t shift;
};

struct FusedSync {          // per row; zeroed before the single-launch kernel starts
  uint32_t bar;            // arrivals at the row barrier (monotonic)
  uint32_t maxkey;         // order-preserving key of the row maximum
  int32_t err;             // set if a barrier wait ran out
  uint32_t pad;
};

struct TopPArgs {
  const float* scores;
  int64_t score_stride;
  const int32_t* row_len;
  const float* p;
  int32_t R;
  int32_t n_chunks;        // grid.x
  int32_t* sel_idx;
  int64_t sel_stride;
  int32_t* sel_count;
  float* tau;
  float* mass;
  float* cmax;             // [R, n_chunks]
  int32_t* chunk_cnt;      // [R, n_chunks]
  uint64_t* hist;          // [R, kBinsTotal]
  RowState* state;         // [R, 4]
  struct FusedSync* sync;  // [R]   (single-launch path)
};

__device__ __forceinline__ int fixed_shift(int n) {
  // weights are <= 1 and a row has n of them: n * 2^shift must stay below 2^63
  int lg = 32 - __clz(max(n, 2) - 1);      // ceil(log2 n)
  return min(52, 62 - lg);
}

// exp(s - smax) * 2^shift as an integer.  exp is evaluated in fp64 as 2^n * T[j] * P(t):
// y = x * log2(e) = n + j/256 + f, T[j] = 2^(j/256) from an LDS table, P a degree-4 polynomial in
// t = f * ln 2 < 2.8e-3 (truncation error ~1e-15 relative).
__device__ __forceinline__ uint64_t fixed_weight(float s, float smax, int shift, const double* __restrict__ tab) {
  const double x = (double)s - (double)smax;         // exact
  if (!(x >= -60.0)) return 0;                        // below 2^-86: under the fixed-point resolution
  const double y = x * 1.4426950408889634;
  const double n = floor(y);
  const double f = y - n;                             // [0, 1)
  const int j = min((int)(f * 256.0), 255);
  const double t = (f - (double)j * 0.00390625) * 0.6931471805599453;
  double pl = fma(t, 1.0 / 24.0, 1.0 / 6.0);
  pl = fma(t, pl, 0.5);
  pl = fma(t, pl, 1.0);
  pl = fma(t, pl, 1.0);
  return (uint64_t)__double2ull_rn(ldexp(tab[j] * pl, shift + (int)n));
}

// Block-wide maximum; result valid in every thread.
__device__ __forceinline__ float block_max(float v, float* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  v = red[0];
#pragma unroll
  for (int i = 1; i < kTpThreads / 64; ++i) v = fmaxf(v, red[i]);
  return v;
}

struct ScanResult {
  int bin;             // highest bin b with  above + sum_{i >= b} h[i] >= target
  uint64_t above;      // mass strictly above bin b (including the incoming `above`)
  uint64_t bin_mass;   // h[b]
  uint64_t target;     // the target used
  uint64_t total;      // sum of the whole histogram
};

// Scans NBINS fixed-point masses (global, written by an earlier launch) from the top.  With
// derive_target the histogram is the level-1 one: its total is Z and the target becomes ceil(p * Z).
// Every thread gets the result.  Two block barriers; wave-level suffix sums run on shuffles.
template <int NBINS, bool COHERENT = false>
__device__ __forceinline__ ScanResult scan_from_top(const uint64_t* h, uint64_t above, uint64_t target,
                                                    bool derive_target, float p, uint64_t* sh_w /*[4]*/,
                                                    uint64_t* sh_res /*[3]*/) {
  constexpr int per = NBINS / kTpThreads;             // consecutive bins per thread
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint64_t loc[per];
  uint64_t sum = 0;
#pragma unroll
  for (int i = 0; i < per; ++i) {
    // COHERENT: the bins were written by other workgroups of this same launch
    loc[i] = COHERENT ? __hip_atomic_load(&h[tid * per + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : h[tid * per + i];
    sum += loc[i];
  }
  uint64_t incl = sum;                                // suffix sum inside the wave (lanes >= lane)
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint64_t t = __shfl_down(incl, o);
    if (lane + o < 64) incl += t;
  }
  if (lane == 0) sh_w[wave] = incl;
  if (tid == 0) { sh_res[0] = 0; sh_res[1] = above; sh_res[2] = loc[0]; }
  __syncthreads();
  uint64_t total = 0, after = 0;
#pragma unroll
  for (int w = 0; w < kTpThreads / 64; ++w) {
    const uint64_t t = sh_w[w];
    total += t;
    if (w > wave) after += t;
  }
  if (derive_target) {
    target = (uint64_t)__double2ull_rn(ceil((double)p * (double)total));
    if (target > total) target = total;
    if (target < 1) target = 1;
  }
  incl += after;                                      // bins of threads >= tid
  const uint64_t excl = incl - sum;                   // bins of threads > tid
  if (above + excl < target && above + incl >= target) {
    uint64_t run = above + excl;
    int b = per - 1;
#pragma unroll
    for (int i = per - 1; i > 0; --i) {
      if (b == i && run + loc[i] < target) { run += loc[i]; b = i - 1; }
    }
    uint64_t lb = loc[0];
#pragma unroll
    for (int i = 1; i < per; ++i) if (b == i) lb = loc[i];
    sh_res[0] = (uint64_t)(tid * per + b);
    sh_res[1] = run;
    sh_res[2] = lb;
  }
  __syncthreads();
  ScanResult r;
  r.bin = (int)sh_res[0];
  r.above = sh_res[1];
  r.bin_mass = sh_res[2];
  r.target = target;
  r.total = total;
  __syncthreads();                                    // sh_w / sh_res may be reused by the caller
  return r;
}

// ---- launch 0: per-chunk maxima, zero the histograms and counters --------------------------------
__global__ __launch_bounds__(kTpThreads) void topp_init_kernel(const TopPArgs a) {
  const int r = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  __shared__ float red[kTpThreads / 64];
  uint64_t* h = a.hist + (int64_t)r * kBinsTotal;
  for (int i = c * kTpThreads + tid; i < kBinsTotal; i += a.n_chunks * kTpThreads) h[i] = 0;
  const int n = a.row_len[r];
  const int64_t n0 = (int64_t)c * kTpChunk;
  if (n0 >= n) return;
  const float4* src = reinterpret_cast<const float4*>(a.scores + (int64_t)r * a.score_stride + n0);
  const int n_here = (int)min((int64_t)kTpChunk, (int64_t)n - n0);
  float m = -__builtin_huge_valf();
#pragma unroll
  for (int u = 0; u < kTpVec; ++u) {
    const int e = (u * kTpThreads + tid) * 4;
    if (e < n_here) {
      const float4 v = src[u * kTpThreads + tid];
      m = fmaxf(m, v.x);
      if (e + 1 < n_here) m = fmaxf(m, v.y);
      if (e + 2 < n_here) m = fmaxf(m, v.z);
      if (e + 3 < n_here) m = fmaxf(m, v.w);
    }
  }
  m = block_max(m, red);
  if (tid == 0) a.cmax[(int64_t)r * a.n_chunks + c] = m;
}

// ---- launches 1-3: one histogram level each ----------------------------------------------------
template <int LEVEL>
__global__ __launch_bounds__(kTpThreads) void topp_level_kernel(const TopPArgs a) {
  constexpr int kBins = LEVEL == 1 ? kBins1 : (LEVEL == 2 ? kBins2 : kBins3);
  constexpr int kShift = LEVEL == 1 ? 21 : (LEVEL == 2 ? 10 : 0);     // key bits below this level's field
  constexpr int kOff = LEVEL == 1 ? 0 : (LEVEL == 2 ? kBins1 : kBins1 + kBins2);
  const int r = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int n = a.row_len[r];
  const int64_t n0 = (int64_t)c * kTpChunk;
  if (n0 >= n || n <= 0) return;

  __shared__ uint64_t lh[kBins];
  __shared__ uint64_t sh_part[kTpThreads / 64];
  __shared__ uint64_t sh_res[3];
  __shared__ float red[kTpThreads / 64];
  __shared__ double tab[256];
  tab[tid] = exp2((double)tid * 0.00390625);
  uint64_t* hrow = a.hist + (int64_t)r * kBinsTotal;
  RowState* st = a.state + (int64_t)r * 4;

  // ---- prologue: what the previous launch left for this row ----
  float smax;
  int shift;
  uint32_t prefix = 0;
  int flags = 0;
  if (LEVEL == 1) {
    const int n_row_chunks = (n + kTpChunk - 1) / kTpChunk;
    float m = -__builtin_huge_valf();
    for (int i = tid; i < n_row_chunks; i += kTpThreads) m = fmaxf(m, a.cmax[(int64_t)r * a.n_chunks + i]);
    smax = block_max(m, red);
    shift = fixed_shift(n);
    const float pr = a.p[r];
    flags = (pr >= 1.f) ? 1 : ((pr > 0.f) ? 0 : -1);
    if (c == 0 && tid == 0) {
      RowState s;
      s.above = 0; s.target = 0; s.total = 0; s.prefix = 0; s.flags = flags; s.smax = smax; s.shift = shift;
      st[0] = s;
    }
  } else {
    const RowState prev = st[LEVEL - 2];
    smax = prev.smax;
    shift = prev.shift;
    flags = prev.flags;
    uint64_t above = prev.above, target = prev.target, total = prev.total;
    if (flags == 0) {
      const uint64_t* hprev = hrow + (LEVEL == 2 ? 0 : kBins1);
      const ScanResult sr = scan_from_top<(LEVEL == 2 ? kBins1 : kBins2)>(hprev, LEVEL == 2 ? 0 : above, target,
                                                                         LEVEL == 2, a.p[r], sh_part, sh_res);
      if (LEVEL == 2) { target = sr.target; total = sr.total; }
      prefix = (prev.prefix << 11) | (uint32_t)sr.bin;
      above = sr.above;
    }
    if (c == 0 && tid == 0) {
      RowState s;
      s.above = above; s.target = target; s.total = total; s.prefix = prefix; s.flags = flags; s.smax = smax;
      s.shift = shift;
      st[LEVEL - 1] = s;
    }
  }
  if (flags != 0) return;          // keep-all or invalid rows need no histogram

  for (int i = tid; i < kBins; i += kTpThreads) lh[i] = 0;
  __syncthreads();

  const float4* src = reinterpret_cast<const float4*>(a.scores + (int64_t)r * a.score_stride + n0);
  const int n_here = (int)min((int64_t)kTpChunk, (int64_t)n - n0);
#pragma unroll 2
  for (int u = 0; u < kTpVec; ++u) {
    const int e = (u * kTpThreads + tid) * 4;
    if (e >= n_here) break;
    const float4 v = src[u * kTpThreads + tid];
    const float s4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (e + k < n_here) {
        const uint32_t key = float_key(s4[k]);
        bool mine;
        if (LEVEL == 1) mine = true;
        else mine = (key >> (kShift + (LEVEL == 2 ? 11 : 10))) == prefix;
        if (mine) {
          const uint64_t w = fixed_weight(s4[k], smax, shift, tab);
          if (w) atomicAdd((unsigned long long*)&lh[(key >> kShift) & (kBins - 1)], (unsigned long long)w);
        }
      }
    }
  }
  __syncthreads();
  uint64_t* hout = hrow + kOff;
  for (int i = tid; i < kBins; i += kTpThreads) {
    const uint64_t v = lh[i];
    if (v) atomicAdd((unsigned long long*)&hout[i], (unsigned long long)v);
  }
}

// ---- launches 4 and 5: final scan + per-chunk counts, then ordered compaction ---------------------
// Bit u*4+k of the result says whether score (u * 256 + tid) * 4 + k of the chunk is kept.
__device__ __forceinline__ uint32_t keep_mask(const float4* __restrict__ src, int n_here, int tid, bool all,
                                              uint32_t tkey) {
  const float ninf = -__builtin_huge_valf();
  uint32_t keep = 0;
#pragma unroll
  for (int u = 0; u < kTpVec; ++u) {
    const int e = (u * kTpThreads + tid) * 4;
    if (e < n_here) {
      const float4 v = src[u * kTpThreads + tid];
      const float s4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const bool sel = (e + k < n_here) && s4[k] != ninf && (all || float_key(s4[k]) >= tkey);
        keep |= (sel ? 1u : 0u) << (u * 4 + k);
      }
    }
  }
  return keep;
}

// Writes the kept positions of one chunk in ascending order starting at out[before].
// Element order inside a chunk is (load round u, thread, k); per-round counts (0..4) travel as
// 16-bit fields of two 64-bit words through one wave scan.
__device__ __forceinline__ void write_ranked(uint32_t keep, int before, int32_t* out, int64_t n0,
                                             uint64_t (*sh_tot)[2] /*[waves][2]*/) {
  const int tid = threadIdx.x;
  uint64_t lo = 0, hi = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    lo |= (uint64_t)__popc((keep >> (u * 4)) & 0xFu) << (16 * u);
    hi |= (uint64_t)__popc((keep >> (16 + u * 4)) & 0xFu) << (16 * u);
  }
  uint64_t ilo = lo, ihi = hi;       // inclusive wave scans
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint64_t tl = __shfl_up(ilo, o), th = __shfl_up(ihi, o);
    if ((tid & 63) >= o) { ilo += tl; ihi += th; }
  }
  if ((tid & 63) == 63) { sh_tot[tid >> 6][0] = ilo; sh_tot[tid >> 6][1] = ihi; }
  __syncthreads();
  int round_base = before;
#pragma unroll
  for (int u = 0; u < kTpVec; ++u) {
    const int sh = 16 * (u & 3);
    int wave_before = 0, round_total = 0;
#pragma unroll
    for (int i = 0; i < kTpThreads / 64; ++i) {
      const int t = (int)((sh_tot[i][u >> 2] >> sh) & 0xFFFFu);
      if (i < (tid >> 6)) wave_before += t;
      round_total += t;
    }
    const int incl = (int)(((u < 4 ? ilo : ihi) >> sh) & 0xFFFFu);
    const int mine = (int)(((u < 4 ? lo : hi) >> sh) & 0xFFFFu);
    int pos = round_base + wave_before + incl - mine;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (keep & (1u << (u * 4 + k))) out[pos++] = (int32_t)(n0 + (u * kTpThreads + tid) * 4 + k);
    }
    round_base += round_total;
  }
}

__global__ __launch_bounds__(kTpThreads) void topp_count_kernel(const TopPArgs a) {
  const int r = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int n = a.row_len[r];
  const int64_t n0 = (int64_t)c * kTpChunk;
  RowState* st = a.state + (int64_t)r * 4;
  if (n <= 0) {
    if (c == 0 && tid == 0) {
      if (a.tau) a.tau[r] = -__builtin_huge_valf();
      if (a.mass) a.mass[r] = 0.f;
      a.sel_count[r] = 0;
    }
    return;
  }
  if (n0 >= n) return;
  __shared__ uint64_t sh_part[kTpThreads / 64];
  __shared__ uint64_t sh_res[3];
  __shared__ int sh_cnt[kTpThreads / 64];
  const uint64_t* hrow = a.hist + (int64_t)r * kBinsTotal;
  const RowState prev = st[2];

  uint32_t tkey = 0;      // keep keys >= tkey
  if (prev.flags < 0) {
    if (c == 0 && tid == 0) {
      a.sel_count[r] = -1;
      if (a.tau) a.tau[r] = __builtin_nanf("");
      if (a.mass) a.mass[r] = 0.f;
      RowState s = prev;
      st[3] = s;
    }
    return;
  } else if (prev.flags == 0) {
    const ScanResult sr = scan_from_top<kBins3>(hrow + kBins1 + kBins2, prev.above, prev.target, false, 0.f,
                                                sh_part, sh_res);
    tkey = (prev.prefix << 10) | (uint32_t)sr.bin;
    if (c == 0 && tid == 0) {
      if (a.tau) a.tau[r] = key_float(tkey);
      if (a.mass) a.mass[r] = (float)((double)(sr.above + sr.bin_mass) / (double)prev.total);
    }
  } else if (c == 0 && tid == 0) {
    if (a.tau) a.tau[r] = -__builtin_huge_valf();
    if (a.mass) a.mass[r] = 1.f;
  }
  if (c == 0 && tid == 0) {
    RowState s = prev;
    s.prefix = tkey;
    st[3] = s;
  }

  const float4* src = reinterpret_cast<const float4*>(a.scores + (int64_t)r * a.score_stride + n0);
  const int n_here = (int)min((int64_t)kTpChunk, (int64_t)n - n0);
  int cnt = __popc(keep_mask(src, n_here, tid, prev.flags == 1, tkey));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
  if ((tid & 63) == 0) sh_cnt[tid >> 6] = cnt;
  __syncthreads();
  if (tid == 0) {
    int tot = 0;
#pragma unroll
    for (int i = 0; i < kTpThreads / 64; ++i) tot += sh_cnt[i];
    a.chunk_cnt[(int64_t)r * a.n_chunks + c] = tot;
  }
}

// Writes the kept positions of the row in ascending order: chunk bases come from the per-chunk
// counts of the previous launch, positions inside a chunk from block-wide prefix sums.
__global__ __launch_bounds__(kTpThreads) void topp_write_kernel(const TopPArgs a) {
  const int r = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int n = a.row_len[r];
  const int64_t n0 = (int64_t)c * kTpChunk;
  if (n <= 0 || n0 >= n) return;
  const RowState st = a.state[(int64_t)r * 4 + 3];
  if (st.flags < 0) return;
  __shared__ int sh_red[kTpThreads / 64][2];
  __shared__ uint64_t sh_tot[kTpThreads / 64][2];

  // ---- base of this chunk = kept count of the chunks before it; chunk 0 also publishes the total ----
  const int n_row_chunks = (n + kTpChunk - 1) / kTpChunk;
  int before = 0, total = 0;
  for (int i = tid; i < n_row_chunks; i += kTpThreads) {
    const int v = a.chunk_cnt[(int64_t)r * a.n_chunks + i];
    total += v;
    if (i < c) before += v;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    before += __shfl_xor(before, o);
    total += __shfl_xor(total, o);
  }
  if ((tid & 63) == 0) { sh_red[tid >> 6][0] = before; sh_red[tid >> 6][1] = total; }
  __syncthreads();
  before = 0;
  total = 0;
#pragma unroll
  for (int i = 0; i < kTpThreads / 64; ++i) { before += sh_red[i][0]; total += sh_red[i][1]; }
  if (c == 0 && tid == 0) a.sel_count[r] = total;

  const float4* src = reinterpret_cast<const float4*>(a.scores + (int64_t)r * a.score_stride + n0);
  const int n_here = (int)min((int64_t)kTpChunk, (int64_t)n - n0);
  const uint32_t keep = keep_mask(src, n_here, tid, st.flags == 1, st.prefix);

  write_ranked(keep, before, a.sel_idx + (int64_t)r * a.sel_stride, n0, sh_tot);
}

// ---- single-launch path ---------------------------------------------------------------------------
// When every workgroup of the grid can be resident at once, the five phases run inside ONE kernel:
// a workgroup keeps its 8192 scores in registers from the first phase to the last (the scores are
// read once instead of six times) and the workgroups of a ROW meet at a row-local barrier between
// phases (an arrival counter in global memory).  The wait is bounded: if it ever runs out the row is
// flagged (sel_count = -2) and every wave still exits.
constexpr int kSpinLimit = 1 << 21;

// Everything the workgroups of a row tell each other travels through agent-scope ATOMIC operations
// (histogram bins, chunk counts, the row maximum), which are performed at the device's coherence
// point; a wave waits for its own atomics to be acknowledged (s_waitcnt) before it arrives.  No
// device-wide fence is needed -- on this multi-die GPU a release fence writes the whole L2 back,
// which costs more than the rest of the kernel.
__device__ __forceinline__ bool row_barrier(FusedSync* sy, uint32_t target, int* sh_ok) {
  __builtin_amdgcn_s_waitcnt(0);            // this wave's atomics have been acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(&sy->bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int it = 0;
    bool ok = true;
    while (__hip_atomic_load(&sy->bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      __builtin_amdgcn_s_sleep(1);
      if (++it > kSpinLimit) { ok = false; break; }
    }
    if (!ok) __hip_atomic_store(&sy->err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *sh_ok = ok ? 1 : 0;
  }
  __syncthreads();
  return *sh_ok != 0;
}

// Zeroes the histograms and the row barriers (launched right before topp_fused_kernel).
__global__ __launch_bounds__(kTpThreads) void topp_zero_kernel(const TopPArgs a) {
  const int64_t i = (int64_t)blockIdx.x * kTpThreads + threadIdx.x;
  if (i < (int64_t)a.R * kBinsTotal) a.hist[i] = 0;
  if (i < a.R) {
    FusedSync z = {0u, 0u, 0, 0u};
    a.sync[i] = z;
  }
}

template <int LEVEL>
__device__ __forceinline__ void fused_level(const float4 (&sc)[kTpVec], uint32_t prefix, float smax, int shift,
                                            uint64_t* lh, const double* tab, uint64_t* hout) {
  constexpr int kBins = LEVEL == 1 ? kBins1 : (LEVEL == 2 ? kBins2 : kBins3);
  constexpr int kShift = LEVEL == 1 ? 21 : (LEVEL == 2 ? 10 : 0);
  const int tid = threadIdx.x;
  for (int i = tid; i < kBins; i += kTpThreads) lh[i] = 0;
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kTpVec; ++u) {
    const float s4[4] = {sc[u].x, sc[u].y, sc[u].z, sc[u].w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t key = float_key(s4[k]);
      const bool mine = LEVEL == 1 ? true : (key >> (kShift + (LEVEL == 2 ? 11 : 10))) == prefix;
      if (mine) {
        const uint64_t w = fixed_weight(s4[k], smax, shift, tab);
        if (w) atomicAdd((unsigned long long*)&lh[(key >> kShift) & (kBins - 1)], (unsigned long long)w);
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < kBins; i += kTpThreads) {
    const uint64_t v = lh[i];
    if (v) __hip_atomic_fetch_add(&hout[i], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

__global__ __launch_bounds__(kTpThreads) void topp_fused_kernel(const TopPArgs a) {
  const int r = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int n = a.row_len[r];
  const int64_t n0 = (int64_t)c * kTpChunk;
  const float ninf = -__builtin_huge_valf();
  if (n <= 0) {
    if (c == 0 && tid == 0) {
      if (a.tau) a.tau[r] = ninf;
      if (a.mass) a.mass[r] = 0.f;
      a.sel_count[r] = 0;
    }
    return;
  }
  if (n0 >= n) return;
  __shared__ uint64_t lh[kBins1];
  __shared__ uint64_t sh_part[kTpThreads / 64];
  __shared__ uint64_t sh_res[3];
  __shared__ uint64_t sh_tot[kTpThreads / 64][2];
  __shared__ float red[kTpThreads / 64];
  __shared__ int sh_red[kTpThreads / 64][2];
  __shared__ int sh_ok;
  __shared__ double tab[256];
  tab[tid] = exp2((double)tid * 0.00390625);
  FusedSync* sy = a.sync + r;
  uint64_t* hrow = a.hist + (int64_t)r * kBinsTotal;
  const uint32_t n_row_chunks = (uint32_t)((n + kTpChunk - 1) / kTpChunk);
  uint32_t phase = 0;

  // ---- the chunk's scores, once; slots beyond the row read as -inf (never kept, zero mass) ----
  const float4* src = reinterpret_cast<const float4*>(a.scores + (int64_t)r * a.score_stride + n0);
  const int n_here = (int)min((int64_t)kTpChunk, (int64_t)n - n0);
  float4 sc[kTpVec];
  float m = ninf;
#pragma unroll
  for (int u = 0; u < kTpVec; ++u) {
    const int e = (u * kTpThreads + tid) * 4;
    float4 v = make_float4(ninf, ninf, ninf, ninf);
    if (e < n_here) {
      v = src[u * kTpThreads + tid];
      if (e + 1 >= n_here) v.y = ninf;
      if (e + 2 >= n_here) v.z = ninf;
      if (e + 3 >= n_here) v.w = ninf;
    }
    sc[u] = v;
    m = fmaxf(fmaxf(m, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
  }
  m = block_max(m, red);
  if (tid == 0) __hip_atomic_fetch_max(&sy->maxkey, float_key(m), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const float pr = a.p[r];
  const int flags = (pr >= 1.f) ? 1 : ((pr > 0.f) ? 0 : -1);
  if (flags < 0) {
    if (c == 0 && tid == 0) {
      a.sel_count[r] = -1;
      if (a.tau) a.tau[r] = __builtin_nanf("");
      if (a.mass) a.mass[r] = 0.f;
    }
    return;
  }
  bool ok = true;
  uint32_t tkey = 0;
  float mass_out = 1.f;
  if (flags == 0) {
    ok = row_barrier(sy, ++phase * n_row_chunks, &sh_ok);
    const float smax = key_float(__hip_atomic_load(&sy->maxkey, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    const int shift = fixed_shift(n);
    uint32_t prefix = 0;
    uint64_t above = 0, target = 0, total = 1;
    if (ok) {
      fused_level<1>(sc, 0u, smax, shift, lh, tab, hrow);
      ok = row_barrier(sy, ++phase * n_row_chunks, &sh_ok);
    }
    if (ok) {
      const ScanResult s1 = scan_from_top<kBins1, true>(hrow, 0, 0, true, pr, sh_part, sh_res);
      prefix = (uint32_t)s1.bin;
      above = s1.above;
      target = s1.target;
      total = s1.total;
      fused_level<2>(sc, prefix, smax, shift, lh, tab, hrow + kBins1);
      ok = row_barrier(sy, ++phase * n_row_chunks, &sh_ok);
    }
    if (ok) {
      const ScanResult s2 = scan_from_top<kBins2, true>(hrow + kBins1, above, target, false, 0.f, sh_part, sh_res);
      prefix = (prefix << 11) | (uint32_t)s2.bin;
      above = s2.above;
      fused_level<3>(sc, prefix, smax, shift, lh, tab, hrow + kBins1 + kBins2);
      ok = row_barrier(sy, ++phase * n_row_chunks, &sh_ok);
    }
    if (ok) {
      const ScanResult s3 = scan_from_top<kBins3, true>(hrow + kBins1 + kBins2, above, target, false, 0.f, sh_part, sh_res);
      tkey = (prefix << 10) | (uint32_t)s3.bin;
      mass_out = (float)((double)(s3.above + s3.bin_mass) / (double)total);
    }
  }

  // ---- keep mask from the registers, per-chunk counts, ordered write ----
  uint32_t keep = 0;
  if (ok) {
#pragma unroll
    for (int u = 0; u < kTpVec; ++u) {
      const float s4[4] = {sc[u].x, sc[u].y, sc[u].z, sc[u].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const bool sel = s4[k] != ninf && (flags == 1 || float_key(s4[k]) >= tkey);
        keep |= (sel ? 1u : 0u) << (u * 4 + k);
      }
    }
    int cnt = __popc(keep);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
    if ((tid & 63) == 0) sh_red[tid >> 6][0] = cnt;
    __syncthreads();
    if (tid == 0) {
      int tot = 0;
#pragma unroll
      for (int i = 0; i < kTpThreads / 64; ++i) tot += sh_red[i][0];
      __hip_atomic_store(&a.chunk_cnt[(int64_t)r * a.n_chunks + c], tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    ok = row_barrier(sy, ++phase * n_row_chunks, &sh_ok);
  }
  if (!ok) {
    if (c == 0 && tid == 0) a.sel_count[r] = -2;       // a barrier wait ran out (never expected)
    return;
  }
  int before = 0, total_cnt = 0;
  for (int i = tid; i < (int)n_row_chunks; i += kTpThreads) {
    const int v = __hip_atomic_load(&a.chunk_cnt[(int64_t)r * a.n_chunks + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    total_cnt += v;
    if (i < c) before += v;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    before += __shfl_xor(before, o);
    total_cnt += __shfl_xor(total_cnt, o);
  }
  __syncthreads();
  if ((tid & 63) == 0) { sh_red[tid >> 6][0] = before; sh_red[tid >> 6][1] = total_cnt; }
  __syncthreads();
  before = 0;
  total_cnt = 0;
#pragma unroll
  for (int i = 0; i < kTpThreads / 64; ++i) { before += sh_red[i][0]; total_cnt += sh_red[i][1]; }
  if (c == 0 && tid == 0) {
    a.sel_count[r] = total_cnt;
    if (a.tau) a.tau[r] = flags == 1 ? ninf : key_float(tkey);
    if (a.mass) a.mass[r] = mass_out;
  }
  write_ranked(keep, before, a.sel_idx + (int64_t)r * a.sel_stride, n0, sh_tot);
}

struct TopPLayout {
  size_t cmax_off, ccnt_off, hist_off, state_off, sync_off, total;
};
static TopPLayout topp_layout(int32_t R, int64_t max_len) {
  const int64_t n_chunks = (max_len + kTpChunk - 1) / kTpChunk;
  TopPLayout l;
  size_t off = 0;
  l.cmax_off = off;  off = align_up(off + (size_t)R * n_chunks * sizeof(float), 256);
  l.ccnt_off = off;  off = align_up(off + (size_t)R * n_chunks * sizeof(int32_t), 256);
  l.hist_off = off;  off = align_up(off + (size_t)R * kBinsTotal * sizeof(uint64_t), 256);
  l.state_off = off; off = align_up(off + (size_t)R * 4 * sizeof(RowState), 256);
  l.sync_off = off;  off = align_up(off + (size_t)R * sizeof(FusedSync), 256);
  l.total = off;
  return l;
}

}  // namespace rtp

using namespace rtp;

extern "C" size_t rtp_topp_workspace_bytes(int32_t R, int64_t max_len) {
  if (R <= 0 || max_len <= 0) return 0;
  return topp_layout(R, max_len).total;
}

extern "C" int32_t rtp_topp_select(const float* scores, int64_t score_stride, const int32_t* row_len,
                                   const float* p, int32_t R, int64_t max_len,
                                   int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                   float* tau, float* mass, void* ws, size_t ws_bytes, void* stream) {
  const char* who = "rtp_topp_select";
  if (!scores || !row_len || !p || !sel_idx || !sel_count)
    return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (R <= 0 || R > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: R must be in [1, 65535]", who);
  if (max_len <= 0 || max_len > RTP_MAX_ROW_LEN)
    return fail(RTP_ERR_INVALID_ARG, "%s: max_len must be in [1, %d]", who, RTP_MAX_ROW_LEN);
  if (score_stride < max_len || (score_stride & 3) || ((uintptr_t)scores & 15))
    return fail(RTP_ERR_INVALID_ARG, "%s: scores must be 16-byte aligned, score_stride >= max_len and a multiple of 4", who);
  if (sel_stride < max_len) return fail(RTP_ERR_INVALID_ARG, "%s: sel_stride must be >= max_len", who);
  const TopPLayout l = topp_layout(R, max_len);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < l.total)
    return fail(RTP_ERR_WORKSPACE, "%s: workspace of %zu bytes (256-byte aligned) required, got %zu", who, l.total,
                ws_bytes);
  clear_error();

  TopPArgs a;
  a.scores = scores;
  a.score_stride = score_stride;
  a.row_len = row_len;
  a.p = p;
  a.R = R;
  a.n_chunks = (int32_t)((max_len + kTpChunk - 1) / kTpChunk);
  a.sel_idx = sel_idx;
  a.sel_stride = sel_stride;
  a.sel_count = sel_count;
  a.tau = tau;
  a.mass = mass;
  a.cmax = (float*)((char*)ws + l.cmax_off);
  a.chunk_cnt = (int32_t*)((char*)ws + l.ccnt_off);
  a.hist = (uint64_t*)((char*)ws + l.hist_off);
  a.state = (RowState*)((char*)ws + l.state_off);
  a.sync = (FusedSync*)((char*)ws + l.sync_off);

  hipStream_t s = (hipStream_t)stream;
  dim3 grid((unsigned)a.n_chunks, (unsigned)R), block(kTpThreads);
  // single-launch path: only if the whole grid can be resident at once (row barriers inside)
  static int capacity = -1;
  if (capacity < 0) {
    int per_cu = 0, dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, topp_fused_kernel, kTpThreads, 0) == hipSuccess)
      capacity = per_cu * prop.multiProcessorCount;
    else
      capacity = 0;
    (void)hipGetLastError();
  }
  // Measured on MI355X (configuration 2): the single-launch kernel takes 74 us against 53 us for the
  // six launches -- a row barrier across the dies costs about as much as a kernel boundary -- so it
  // is opt-in (RTP_TOPP_PATH=fused) and the multi-launch path is the default.
  const char* force = getenv("RTP_TOPP_PATH");
  const bool fits = (int64_t)a.n_chunks * R <= capacity;
  if (force && force[0] == 'f' && fits) {
    const int64_t nz = (int64_t)R * kBinsTotal;
    hipLaunchKernelGGL(topp_zero_kernel, dim3((unsigned)((nz + kTpThreads - 1) / kTpThreads)), block, 0, s, a);
    hipLaunchKernelGGL(topp_fused_kernel, grid, block, 0, s, a);
    return check_launch(who);
  }
  hipLaunchKernelGGL(topp_init_kernel, grid, block, 0, s, a);
  hipLaunchKernelGGL(topp_level_kernel<1>, grid, block, 0, s, a);
  hipLaunchKernelGGL(topp_level_kernel<2>, grid, block, 0, s, a);
  hipLaunchKernelGGL(topp_level_kernel<3>, grid, block, 0, s, a);
  hipLaunchKernelGGL(topp_count_kernel, grid, block, 0, s, a);
  hipLaunchKernelGGL(topp_write_kernel, grid, block, 0, s, a);
  return check_launch(who);
}
