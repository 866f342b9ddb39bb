// rtp_topp_select: sort-free dynamic top-p (paper Sec. 3.2, S = Top-P(s, p); Sec. 3.4, the score
// threshold where the descending cumulative softmax mass first reaches p).
//
// Design (ours, for gfx950; the paper's kernel uses one 256-bin histogram of block maxima):
// a three-level radix search over the order-preserving 32-bit key of each fp32 score
// (11 + 11 + 10 bits).  Level L histograms the softmax mass of the elements whose higher key bits
// equal the prefix found so far; scanning the histogram from the top finds the bin in which the
// descending cumulative mass crosses p * Z.  After three levels the threshold key is exact.
// Masses are integers (see topp_common.h), so the result does not depend on atomic ordering.
//
// Launches: [zero] -> level 1 -> level 2 -> level 3 -> write.  The first two disappear when
// the score pass has already accumulated level 1 (level1_ready).  Level 3 also leaves, per chunk, the
// number of scores strictly above the 22-bit prefix (certainly kept) and appends the few scores that
// share the prefix to a short per-row list; the write launch finds the exact threshold from the
// level-3 histogram and takes the kept list members' positions into its chunk offsets, so no separate
// counting pass over the scores is needed.  (A row whose list overflows -- thousands of scores equal
// in their top 22 key bits -- is still written correctly: its workgroups count their predecessors'
// kept scores themselves.)  There is no "last block" hand-off:
// each level's histogram is scanned redundantly in the prologue of every workgroup of the NEXT
// launch, so kernel boundaries provide all the ordering.  A row is cut into chunks of kTpChunk
// scores, one workgroup each; histograms live in LDS and only non-empty bins are flushed with 64-bit
// global atomics.  The selected positions come out in ascending order (deterministic, and friendly to
// the K/V gather).
//
// (A single-launch variant with row-local barriers between the phases was measured on MI355X at 74 us
// against 53 us for the separate launches on batch 8 x 131072: a barrier across the chip's dies costs
// about as much as a kernel boundary.  It is not kept.)
#include "topp_common.h"
#include "attn_decode_shared.h"

#include <stdlib.h>

#include <mutex>

namespace rtp {

// Workgroup shape, measured on batch 8 x 131072 and batch 1 x 1048576 (whole decode step, us):
//   256 threads x 4096 scores 108.8 / 118.9 | 512 x 8192 107.3 / 110.3 | 1024 x 16384 113.6 / 109.5 |
//   256 x 8192 111.8 / 113.9 | 512 x 4096 111.6 / 120.7 | 512 x 16384 111.4 / 109.5.
// Every workgroup repeats the scan of the previous level, and the workgroups resident on a compute unit
// run their phases in step and share its vector ALUs: fewer, larger workgroups repeat less (and start
// sooner: a launch of 1024 workgroups takes 2.5 us to get them all going), smaller ones balance better.
constexpr int kTpThreads = 512;
constexpr int kTpChunk = 8192;             // scores per workgroup
constexpr int kTpVec = kTpChunk / (kTpThreads * 4);   // float4 loads per thread

struct RowState {          // one per row and launch (levels 2 and 3 leave one each)
  double above_base;       // mass strictly above the level-1 threshold bin, in that bin's integer units
  double total_d;          // Z in the same units
  uint64_t above;          // integer mass above the current prefix range INSIDE the level-1 bin
  uint64_t target;         // integer mass to reach inside the level-1 bin
  uint32_t prefix;         // key bits resolved so far (right-aligned)
  int32_t flags;           // 0 ok, 1 = keep everything (p >= 1), -1 = invalid p, 2 = no finite score,
                           // -2 = the row's largest score lies outside (-128, 128)
  float ref;               // reference score of the level-1 threshold bin
  int32_t shift;
};

constexpr int kBucketCap = 1024;

struct TopPArgs {
  const float* scores;
  int64_t score_stride;
  const int32_t* row_len;
  const float* p;
  int32_t R;
  int32_t n_chunks;        // grid.x
  int32_t rezero;          // write launch leaves the histograms zeroed (level1_ready protocol)
  int32_t balance;         // gathering write launch: rows with one overfull chunk share their ranks out equally
  const int32_t* kcount;   // NULL: top-p by softmax mass; else static top-k, every score weighs 1 and
                           // the target is kcount[r] (rtp_topk_select)
  int32_t* sel_idx;
  int64_t sel_stride;
  int32_t* sel_count;
  float* tau;
  float* mass;
  int32_t* chunk_cnt;      // [R, n_chunks]: scores of the chunk strictly above the level-2 prefix (or all finite ones)
  uint64_t* hist;          // [R, hist_stride]
  int64_t hist_stride;
  int32_t n_sub;           // copies of level 1 per row (topp_common.h)
  RowState* state;         // [R, 3]
  int32_t* bucket_n;       // [R]: scores that share the level-2 prefix (may exceed kBucketCap)
  uint2* bucket;           // [R, kBucketCap]: (key, position) of the first kBucketCap of them
};

TopPLayout topp_layout(int32_t R, int64_t max_len) {
  const int64_t n_chunks = (max_len + kTpChunk - 1) / kTpChunk;
  TopPLayout l;
  size_t off = 0;
  l.n_sub = R >= 16 ? 1 : (R >= 8 ? 2 : (R >= 4 ? 4 : 8));
  l.hist_stride = kBinsTotal + (int64_t)(l.n_sub - 1) * kBins1;
  l.hist_off = off;  off = align_up(off + (size_t)R * l.hist_stride * sizeof(uint64_t), 256);
  l.ccnt_off = off;  off = align_up(off + (size_t)R * n_chunks * sizeof(int32_t), 256);
  l.state_off = off; off = align_up(off + (size_t)R * 3 * sizeof(RowState), 256);
  l.bn_off = off;    off = align_up(off + (size_t)R * sizeof(int32_t), 256);
  l.bucket_off = off; off = align_up(off + (size_t)R * kBucketCap * sizeof(uint2), 256);
  l.total = off;
  return l;
}

// ---- histogram scans -------------------------------------------------------------------------------
struct Scan1Result {       // level 1: bins carry different references, the scan runs in fp64
  int bin;                 // threshold bin (-1: the row has no mass at all)
  int top;                 // highest bin that holds a score
  double above_base, total_d;
  uint64_t target;         // integer mass still to reach inside the threshold bin (1 .. bin mass)
  float ref;
};

// Every thread gets the result; all workgroups of a row compute the same numbers in the same order.
// Threads own `per` consecutive bins in order FROM THE TOP of the score range (thread 0 the highest bins),
// so "the mass above" is an ordinary inclusive prefix sum over lanes and waves.
// The bins arrive in registers (load_bins): a kernel issues those loads first thing, so that they are in
// flight while it finds out what else it needs.
template <int NBINS>
__device__ __forceinline__ void load_bins(const uint64_t* __restrict__ h, uint64_t (&loc)[NBINS / kTpThreads]) {
  const int first = (kTpThreads - 1 - (int)threadIdx.x) * (NBINS / kTpThreads);
#pragma unroll
  for (int i = 0; i < NBINS / kTpThreads; ++i) loc[i] = h[first + i];
}

__device__ __forceinline__ Scan1Result scan_level1(const uint64_t (&loc)[kBins1 / kTpThreads], float p, double* sh_d /*[4]*/,
                                                   int* sh_i /*[4]*/, double* sh_res /*[3]*/,
                                                   const double* __restrict__ tab /* filled by the caller */) {
  constexpr int per = kBins1 / kTpThreads;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int first = (kTpThreads - 1 - tid) * per;     // this thread's lowest bin
  int top = -1;
#pragma unroll
  for (int i = 0; i < per; ++i) {
    if (loc[i]) top = first + i;
  }
  top = wave_max_ge_m1(top);
  if (lane == 0) sh_i[wave] = top;
  __syncthreads();
  top = sh_i[0];
#pragma unroll
  for (int w = 1; w < kTpThreads / 64; ++w) top = max(top, sh_i[w]);
  Scan1Result res;
  res.bin = -1; res.top = top; res.above_base = 0.0; res.total_d = 0.0; res.target = 1; res.ref = 0.f;
  if (top < 0) { __syncthreads(); return res; }       // uniform: every thread sees the same `top`
  const double R = (double)bin_ref(top);
  double md[per];
  double sum = 0.0;
#pragma unroll
  for (int i = 0; i < per; ++i) {
    md[i] = 0.0;
    if (loc[i]) {
      int e;
      const double m = exp_parts((double)bin_ref(first + i) - R, tab, &e);
      md[i] = (double)loc[i] * ldexp(m, e);
    }
    sum += md[i];
  }
  double incl = wave_incl_scan(sum);                  // this thread's bins and every higher bin of the wave
  if (lane == 63) sh_d[wave] = incl;
  // defaults (nobody crosses): the top bin, nothing above it -- left by the thread that owns that bin
  if (top >= first && top < first + per) {
    uint64_t lt = loc[0];
#pragma unroll
    for (int i = 1; i < per; ++i) if (top - first == i) lt = loc[i];
    sh_res[0] = (double)top; sh_res[1] = 0.0; sh_res[2] = __longlong_as_double((long long)lt);
  }
  __syncthreads();
  double total = 0.0, before = 0.0;
#pragma unroll
  for (int w = 0; w < kTpThreads / 64; ++w) {         // fixed order: identical in every workgroup
    if (w < wave) before += sh_d[w];
    total += sh_d[w];
  }
  const double target = (double)p * total;
  incl += before;
  const double excl = incl - sum;
  // the crossing thread: the mass above its bins is below the target, the mass including them reaches it.
  // (if rounding left the target unreachable nobody matches and the defaults -- top bin -- stand, which
  // cannot happen for p < 1 because the whole-row sum is the largest partial sum)
  if (excl < target && incl >= target) {
    double run = excl;
    int b = per - 1;
#pragma unroll
    for (int i = per - 1; i > 0; --i) {
      if (b == i && !(loc[i] && run + md[i] >= target)) { run += md[i]; b = i - 1; }
    }
    uint64_t lb = loc[0];
#pragma unroll
    for (int i = 1; i < per; ++i) if (b == i) lb = loc[i];
    sh_res[0] = (double)(first + b);
    sh_res[1] = run;
    sh_res[2] = __longlong_as_double((long long)lb);
  }
  __syncthreads();
  const int b1 = (int)sh_res[0];
  const double above_true = sh_res[1];
  const uint64_t hb = (uint64_t)__double_as_longlong(sh_res[2]);
  const float ref1 = bin_ref(b1);
  // exp(R - ref1) >= 1 as the reciprocal of the table-based exponential of the negative argument (which
  // may underflow to 0 here: the reciprocal is then capped)
  int es;
  const double ms = exp_parts((double)ref1 - R, tab, &es, -300000.0);
  const double scale = fmin(1.0 / ldexp(ms, es), 1e250);
  double t2 = ceil((target - above_true) * scale);
  if (!(t2 >= 1.0)) t2 = 1.0;
  uint64_t tgt = (uint64_t)__double2ull_rn(fmin(t2, 1.8e19));
  if (tgt > hb) tgt = hb;
  if (tgt < 1) tgt = 1;
  res.bin = b1;
  res.above_base = above_true * scale;
  res.total_d = total * scale;
  res.target = tgt;
  res.ref = ref1;
  __syncthreads();
  return res;
}

struct ScanResult {
  int bin;             // highest bin b with  above + sum_{i >= b} h[i] >= target
  uint64_t above;      // mass strictly above bin b (including the incoming `above`)
  uint64_t bin_mass;   // h[b]
  uint64_t total;      // above + sum of all bins
};

// Levels 2 and 3: integer masses with one reference.  Same thread order as above (thread 0 owns the
// highest bins); two block barriers.
template <int NBINS>
__device__ __forceinline__ ScanResult scan_from_top(const uint64_t (&loc)[NBINS / kTpThreads], uint64_t above, uint64_t target,
                                                    uint64_t* sh_w /*[4]*/, uint64_t* sh_res /*[3]*/) {
  constexpr int per = NBINS / kTpThreads;             // consecutive bins per thread
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int first = (kTpThreads - 1 - tid) * per;     // this thread's lowest bin
  uint64_t sum = 0;
#pragma unroll
  for (int i = 0; i < per; ++i) sum += loc[i];
  uint64_t incl = wave_incl_scan(sum);                // this thread's bins and every higher bin of the wave
  if (lane == 63) sh_w[wave] = incl;
  if (first == 0) { sh_res[0] = 0; sh_res[1] = above; sh_res[2] = loc[0]; }   // defaults: bin 0
  __syncthreads();
  uint64_t before = 0, total = above;
#pragma unroll
  for (int w = 0; w < kTpThreads / 64; ++w) {
    if (w < wave) before += sh_w[w];
    total += sh_w[w];
  }
  incl += before;                                     // bins of threads <= tid
  const uint64_t excl = incl - sum;                   // bins of threads < tid: everything above this thread's
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
    sh_res[0] = (uint64_t)(first + b);
    sh_res[1] = run;
    sh_res[2] = lb;
  }
  __syncthreads();
  ScanResult r;
  r.bin = (int)sh_res[0];
  r.above = sh_res[1];
  r.bin_mass = sh_res[2];
  r.total = total;
  __syncthreads();                                    // sh_w / sh_res may be reused by the caller
  return r;
}

// The chunk's scores, issued as the first loads of a launch so that the prologue (state, histogram
// scan) runs under their latency.  Vectors wholly past the row end are not read.
__device__ __forceinline__ void load_chunk(const float4* __restrict__ src, int n_here, int tid, float4 (&v)[kTpVec]) {
#pragma unroll
  for (int u = 0; u < kTpVec; ++u) {
    const int e = (u * kTpThreads + tid) * 4;
    if (e < n_here) v[u] = src[u * kTpThreads + tid];
    else v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
}

// ---- launch 0 (only when level 1 is not supplied): zero the histograms -------------------------------
__global__ __launch_bounds__(kTpThreads) void topp_zero_kernel(uint64_t* hist, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kTpThreads + threadIdx.x;
  if (i < n) hist[i] = 0;
}

// Sum of `cnt` over the workgroup, stored by thread 0 (two barriers).
__device__ __forceinline__ void block_count_to(int cnt, int32_t* dst, int* sh_i /*[waves]*/) {
  cnt = wave_sum(cnt);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh_i[threadIdx.x >> 6] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    int tot = 0;
#pragma unroll
    for (int i = 0; i < kTpThreads / 64; ++i) tot += sh_i[i];
    *dst = tot;
  }
}

// ---- launches 1-3: one histogram level each ----------------------------------------------------
template <int LEVEL>
__device__ __forceinline__ void level_body(const TopPArgs& a, const int c, const int r) {
  constexpr int kBins = LEVEL == 1 ? kBins1 : (LEVEL == 2 ? kBins2 : kBins3);
  constexpr int kShift = LEVEL == 1 ? 21 : (LEVEL == 2 ? 10 : 0);     // key bits below this level's field
  constexpr int kOff = LEVEL == 1 ? 0 : (LEVEL == 2 ? kBins1 : kBins1 + kBins2);
  const int tid = threadIdx.x;
  // what the previous launch left for this row: in flight before anything else (levels 2 and 3 scan the
  // histogram of the level before in their prologue)
  static_assert(kBins1 == kBins2, "one register array serves the scans of levels 2 and 3");
  uint64_t prev_bins[kBins1 / kTpThreads];
  if (LEVEL >= 2) load_bins<kBins1>(a.hist + (int64_t)r * a.hist_stride + (LEVEL == 3 ? kBins1 : 0), prev_bins);
  if (LEVEL == 2) {      // level 1 may be spread over several copies
    for (int sub = 1; sub < a.n_sub; ++sub) {
      uint64_t more[kBins1 / kTpThreads];
      load_bins<kBins1>(a.hist + (int64_t)r * a.hist_stride + level1_copy_offset(sub), more);
#pragma unroll
      for (int i = 0; i < kBins1 / kTpThreads; ++i) prev_bins[i] += more[i];
    }
  }
  const int n = a.row_len[r];
  const int64_t n0 = (int64_t)c * kTpChunk;
  if (n0 >= n || n <= 0) return;
  const int n_here = (int)min((int64_t)kTpChunk, (int64_t)n - n0);
  float4 v[kTpVec];
  load_chunk(reinterpret_cast<const float4*>(a.scores + (int64_t)r * a.score_stride + n0), n_here, tid, v);

  __shared__ uint64_t lh[kBins];
  __shared__ uint64_t sh_part[kTpThreads / 64];
  __shared__ uint64_t sh_res[3];
  __shared__ double sh_d[kTpThreads / 64];
  __shared__ double sh_dres[3];
  __shared__ int sh_i[kTpThreads / 64];
  __shared__ double tab[256];
  fill_exp_table(tab);
  uint64_t* hrow = a.hist + (int64_t)r * a.hist_stride;
  RowState* st = a.state + (int64_t)r * 3;
  // Level 3's histogram and the row's short list are written by the NEXT launch and were last read by the
  // write launch of the previous call: the level-2 launch clears them -- as the last thing it does, because a
  // workgroup barrier waits for the stores issued before it, and the prologue below is a chain of barriers.
  auto clear_level3 = [&]() {
    if (LEVEL != 2) return;
    const int active = (n + kTpChunk - 1) / kTpChunk;
    for (int i = c * kTpThreads + tid; i < kBins3; i += active * kTpThreads) hrow[kBins1 + kBins2 + i] = 0;
    if (c == 0 && tid == 0) a.bucket_n[r] = 0;
  };

  // ---- prologue: what the previous launch left for this row ----
  const int shift = fixed_shift(n);
  uint32_t prefix = 0;
  float ref = 0.f;
  int flags = 0;
  const bool by_count = a.kcount != nullptr;
  if (LEVEL == 1) {
    if (by_count) {
      flags = a.kcount[r] > 0 ? 0 : -1;
    } else {
      const float pr = a.p[r];
      flags = (pr >= 1.f) ? 1 : ((pr > 0.f) ? 0 : -1);
    }
  } else if (LEVEL == 2) {
    const float pr = by_count ? 0.5f : a.p[r];
    flags = by_count ? (a.kcount[r] > 0 ? 0 : -1) : ((pr >= 1.f) ? 1 : ((pr > 0.f) ? 0 : -1));
    RowState s;
    s.above_base = 0.0; s.total_d = 0.0; s.above = 0; s.target = 1; s.prefix = 0; s.flags = flags; s.ref = 0.f;
    s.shift = shift;
    if (flags == 0 && by_count) {
      // static top-k: level 1 holds plain counts; the k-th best score lies in the bin where the count
      // from the top reaches k.  A budget that covers every finite score keeps them all.
      const uint64_t k = (uint64_t)a.kcount[r];
      const ScanResult s1 = scan_from_top<kBins1>(prev_bins, 0, k, sh_part, sh_res);
      if (s1.total == 0) {
        flags = 2;
      } else if (k >= s1.total) {
        flags = 1;
      } else {
        prefix = (uint32_t)s1.bin;
        s.target = k - s1.above;              // still to find inside the bin
        s.prefix = prefix;
      }
      s.flags = flags;
    } else if (flags == 0) {
      const Scan1Result s1 = scan_level1(prev_bins, pr, sh_d, sh_i, sh_dres, tab);
      if (s1.bin < 0) {
        flags = 2;
      } else if (level1_bin_is_wide(s1.top)) {
        flags = -2;
      } else {
        prefix = (uint32_t)s1.bin;
        ref = s1.ref;
        s.above_base = s1.above_base; s.total_d = s1.total_d; s.target = s1.target; s.prefix = prefix; s.ref = ref;
      }
      s.flags = flags;
    }
    if (c == 0 && tid == 0) st[0] = s;
  } else {
    // Field-wise access on purpose: a RowState copied as a whole through a local makes the compiler
    // park the untouched fields in LDS indexed by a flat thread id, which it derives from the dispatch
    // packet -- a read from host memory in every wave that tripled this launch's duration.
    flags = st[0].flags;
    ref = st[0].ref;
    uint64_t above3 = 0;
    if (flags == 0) {
      const ScanResult sr = scan_from_top<kBins2>(prev_bins, 0, st[0].target, sh_part, sh_res);
      prefix = (st[0].prefix << 11) | (uint32_t)sr.bin;
      above3 = sr.above;
    }
    if (c == 0 && tid == 0) {
      st[1].above_base = st[0].above_base;
      st[1].total_d = st[0].total_d;
      st[1].above = above3;
      st[1].target = st[0].target;
      st[1].prefix = prefix;
      st[1].flags = flags;
      st[1].ref = ref;
      st[1].shift = st[0].shift;
    }
  }
  if (LEVEL == 3 && flags == 1) {
    // keep-everything rows: the write launch needs the number of finite scores per chunk
    int cnt = 0;
#pragma unroll
    for (int u = 0; u < kTpVec; ++u) {
      const int e = (u * kTpThreads + tid) * 4;
      const float s4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) cnt += (e + k < n_here && s4[k] != -__builtin_huge_valf()) ? 1 : 0;
    }
    block_count_to(cnt, a.chunk_cnt + (int64_t)r * a.n_chunks + c, sh_i);
  }
  if (flags != 0) {                // keep-all, invalid or empty rows need no histogram
    clear_level3();
    return;
  }

  // Levels 2 and 3 weigh only the members of the prefix bin (a few percent of the chunk at level 2,
  // a handful at level 3).  At level 2, weighing them where they sit would run the fp64 arithmetic in
  // nearly every wave instruction slot for one or two active lanes, so the members are first packed
  // into an LDS list (order is irrelevant: integer masses) and then weighed densely.  At level 3 almost
  // every slot is empty and skipped as it is; packing costs more than it saves there.
  __shared__ float sh_list[LEVEL == 2 ? kTpChunk : 1];
  __shared__ int sh_n;
  static_assert(kTpVec * 4 <= 32, "member mask is one 32-bit word");
  for (int i = tid; i < kBins; i += kTpThreads) lh[i] = 0;
  if (tid == 0) sh_n = 0;
  __syncthreads();

  if (LEVEL == 1) {
#pragma unroll
    for (int u = 0; u < kTpVec; ++u) {
      const int e = (u * kTpThreads + tid) * 4;
      const float s4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (e + k >= n_here) continue;
        if (!by_count) level1_add(lh, s4[k], shift, tab);
        else if (s4[k] != -__builtin_huge_valf()) atomicAdd((unsigned long long*)&lh[float_key(s4[k]) >> 21], 1ull);
      }
    }
  } else if (LEVEL == 3) {
    // scores strictly above the prefix are certainly kept: count them; the few that share the prefix go
    // into the level-3 histogram and onto the row's short list (key, position)
    int cnt_above = 0;
#pragma unroll
    for (int u = 0; u < kTpVec; ++u) {
      const int e = (u * kTpThreads + tid) * 4;
      const float s4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t key = float_key(s4[k]);
        const bool ok = e + k < n_here && s4[k] != -__builtin_huge_valf();
        cnt_above += (ok && (key >> 10) > prefix) ? 1 : 0;
        if (ok && (key >> 10) == prefix) {
          const uint64_t w = by_count ? 1ull : fixed_weight(s4[k], ref, shift, tab);
          if (w) atomicAdd((unsigned long long*)&lh[key & (kBins - 1)], (unsigned long long)w);
          const int slot = atomicAdd(&a.bucket_n[r], 1);
          if (slot < kBucketCap) a.bucket[(int64_t)r * kBucketCap + slot] = make_uint2(key, (uint32_t)(n0 + e + k));
        }
      }
    }
    block_count_to(cnt_above, a.chunk_cnt + (int64_t)r * a.n_chunks + c, sh_i);
  } else {
    constexpr int kAbove = kShift + 11;                          // key bits of the prefix start here
    uint32_t member = 0;
#pragma unroll
    for (int u = 0; u < kTpVec; ++u) {
      const int e = (u * kTpThreads + tid) * 4;
      const float s4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const bool in = (e + k < n_here) && (float_key(s4[k]) >> kAbove) == prefix && s4[k] != -__builtin_huge_valf();
        member |= (in ? 1u : 0u) << (u * 4 + k);
      }
    }
    const int lane = tid & 63;
    const int cnt = __popc(member);
    const int incl = wave_incl_scan(cnt);
    int base = 0;
    if (lane == 63 && incl > 0) base = atomicAdd(&sh_n, incl);
    base = wave_last(base);
    int pos = base + incl - cnt;
#pragma unroll
    for (int u = 0; u < kTpVec; ++u) {
      const float s4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (member & (1u << (u * 4 + k))) sh_list[pos++] = s4[k];
    }
    __syncthreads();
    const int total = sh_n;
    for (int i = tid; i < total; i += kTpThreads) {
      const float sv = sh_list[i];
      const uint64_t w = by_count ? 1ull : fixed_weight(sv, ref, shift, tab);
      if (w) atomicAdd((unsigned long long*)&lh[(float_key(sv) >> kShift) & (kBins - 1)], (unsigned long long)w);
    }
  }
  __syncthreads();
  flush_hist(lh, hrow + (LEVEL == 1 ? level1_copy_offset(c % a.n_sub) : kOff), kBins, kTpThreads);
  clear_level3();
}

template <int LEVEL>
__global__ __launch_bounds__(kTpThreads) void topp_level_kernel(const TopPArgs a) {
  level_body<LEVEL>(a, blockIdx.x, blockIdx.y);
}

// A level-2 or level-3 launch with local heads of the same decode step on board (rtp_decode_attention): the
// first n_ride workgroups run the work items item_lo .. item_hi-1 of the local-attention plan
// (attn_decode_shared.h), the others are the level's own workgroups.  The selector's middle launches are
// latency-bound and leave HBM idle, which is where the local heads' K/V rows get streamed; as riders they need
// no second stream (a fork and a join per step cost more than the overlap they buy).  Two workgroups per
// compute unit, i.e. at most 128 vector registers: one tile per wave in flight (groups of 8 need 163 and
// get one workgroup per compute unit).
template <int LEVEL, int G, bool F16 = false, bool PAGED = false>
__global__ __launch_bounds__(kTpThreads, G == 8 ? 2 : 4) void topp_level_ride_kernel(const TopPArgs a, const AttnDecodeArgs la,
                                                                        const int n_ride, const int item_lo,
                                                                        const int item_hi) {
  const int bid = blockIdx.x;
  if (bid < n_ride) {
    gqa_decode_items<G, kSrcLocal, kTpThreads, 1, F16, PAGED>(la, item_lo + bid, n_ride, item_hi);
    return;
  }
  const int r = (bid - n_ride) / a.n_chunks;
  level_body<LEVEL>(a, (bid - n_ride) - r * a.n_chunks, r);
}

// ---- launches 4 and 5: final scan + per-chunk counts, then ordered compaction ---------------------
// Bit u*4+k of the result says whether score (u * 256 + tid) * 4 + k of the chunk is kept.
__device__ __forceinline__ uint32_t keep_mask(const float4 (&v)[kTpVec], int n_here, int tid, bool all, uint32_t tkey) {
  const float ninf = -__builtin_huge_valf();
  uint32_t keep = 0;
#pragma unroll
  for (int u = 0; u < kTpVec; ++u) {
    const int e = (u * kTpThreads + tid) * 4;
    const float s4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const bool sel = (e + k < n_here) && s4[k] != ninf && (all || float_key(s4[k]) >= tkey);
      keep |= (sel ? 1u : 0u) << (u * 4 + k);
    }
  }
  return keep;
}

// Writes the kept positions of one chunk in ascending order starting at out[before].
// Element order inside a chunk is (load round u, thread, k); per-round counts (0..4) travel as
// 16-bit fields of two 64-bit words through one wave scan.
// `local` (optional, LDS) receives the positions of ranks win_lo <= rank < win_hi at local[rank - win_lo]
// (by default all of the chunk's, starting at local[0]).  Returns the chunk's kept count.
__device__ __forceinline__ int write_ranked(uint32_t keep, int before, int32_t* out, int64_t n0,
                                            uint64_t (*sh_tot)[2] /*[waves][2]*/, int32_t* local = nullptr,
                                            int win_lo = -1, int win_hi = 0x7fffffff) {
  if (win_lo < 0) win_lo = before;
  const int tid = threadIdx.x;
  uint64_t lo = 0, hi = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    lo |= (uint64_t)__popc((keep >> (u * 4)) & 0xFu) << (16 * u);
    hi |= (uint64_t)__popc((keep >> (16 + u * 4)) & 0xFu) << (16 * u);
  }
  const uint64_t ilo = wave_incl_scan(lo), ihi = wave_incl_scan(hi);
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
      if (keep & (1u << (u * 4 + k))) {
        const int32_t where = (int32_t)(n0 + (u * kTpThreads + tid) * 4 + k);
        if (out) out[pos] = where;
        if (local && pos >= win_lo && pos < win_hi) local[pos - win_lo] = where;
        ++pos;
      }
    }
    round_base += round_total;
  }
  return round_base - before;
}

// ---- launch 4: exact threshold, chunk offsets, ordered compaction -----------------------------------
// Every workgroup of a row repeats the final scan (level-3 histogram -> threshold key) and derives its
// chunk's offset: the certainly-kept counts of the chunks before it (level-3 launch) plus the kept
// members of the row's short list that lie before it.  Positions inside a chunk come from block-wide
// prefix sums, so the row's kept positions are ascending.
//
// ATTEND: the same launch goes on to the sparse-attention step of Sec. 3.2 for its chunk -- the kept
// positions stay in LDS, their K/V rows are gathered and a partial softmax state (m, l, acc[128]) is left
// per (row, chunk) for select_attend_combine_kernel.  One launch and one pass over the index list less than
// selecting and attending separately; rows are the retrieval heads of a decode batch, r = b * n_ret + j.
struct GatherArgs {
  const uint16_t* q;
  const uint16_t* K;
  const uint16_t* V;
  int64_t row_stride, head_stride;
  const int64_t* seq_start;
  int32_t n_q_heads, n_kv_heads, n_ret;
  float scale_log2;        // softmax scale * log2(e)
  float* part;             // [R, n_chunks, kSaPart]
  uint16_t* out;
  float* lse;
  int32_t f16;             // q, K, V and out are fp16 (else bf16)
  const int32_t* page_table;   // paged cache: [B, pt_stride] pool pages (NULL: contiguous sequences at seq_start)
  int64_t pt_stride;
  int32_t page_shift;
  int32_t ret_heads[64];
};
constexpr int kSaPart = kHeadDim + 4;      // m, l, 2 pad, acc[128]  (floats)
constexpr int kScanCost = 128;             // repeating a chunk's compaction costs about what gathering this many rows does
constexpr int kSaInFlight = 8;             // K/V rows in flight per 16-lane group (two register sets taking turns,
                                           // or more rows, measured no faster: the gather is bandwidth-bound)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// PAGED (ATTEND only): the K/V rows of a sequence live in pool pages; the kept positions are translated to pool
// rows once, into a second LDS list, before the gather starts.
template <bool ATTEND, bool F16 = false, bool PAGED = false>
__global__ __launch_bounds__(kTpThreads) void topp_write_kernel(const TopPArgs a, const GatherArgs ga) {
  const int r = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  __shared__ int32_t sh_list[ATTEND ? kTpChunk : 1];
  __shared__ int32_t sh_rows[(ATTEND && PAGED) ? kTpChunk : 1];
  // Levels 1 and 2 were last read by the level-2 / level-3 launches; every workgroup of the grid clears its
  // share on its way out (not on its way in: the barriers below would wait for the stores).
  // The same goes for the row's scalar results (chunk 0 stores them at the end).
  float res_tau = 0.f, res_mass = 0.f;
  int res_count = 0;
  bool have_res = false;
  auto rezero = [&]() {
    if (have_res && c == 0 && tid == 0) {
      a.sel_count[r] = res_count;
      if (a.tau) a.tau[r] = res_tau;
      if (a.mass) a.mass[r] = res_mass;
    }
    if (!a.rezero) return;
    uint64_t* h = a.hist + (int64_t)r * a.hist_stride;
    for (int i = c * kTpThreads + tid; i < kBins1 + kBins2; i += a.n_chunks * kTpThreads) h[i] = 0;
    for (int i = kBinsTotal + c * kTpThreads + tid; i < a.hist_stride; i += a.n_chunks * kTpThreads) h[i] = 0;
  };
  // what the level-3 launch left for this row, in flight before anything else: its histogram, the per-chunk
  // counts (one per thread: that covers rows of kTpThreads chunks) and the row's short list
  uint64_t l3_bins[kBins3 / kTpThreads];
  load_bins<kBins3>(a.hist + (int64_t)r * a.hist_stride + kBins1 + kBins2, l3_bins);
  const int cc_mine = tid < a.n_chunks ? a.chunk_cnt[(int64_t)r * a.n_chunks + tid] : 0;
  const int listed_raw = a.bucket_n[r];
  uint2 be[kBucketCap / kTpThreads];
#pragma unroll
  for (int k = 0; k < kBucketCap / kTpThreads; ++k) be[k] = a.bucket[(int64_t)r * kBucketCap + k * kTpThreads + tid];
  const int n = a.row_len[r];
  const int64_t n0 = (int64_t)c * kTpChunk;
  const float ninf = -__builtin_huge_valf();
  if (n <= 0) {
    have_res = true; res_tau = ninf; res_mass = 0.f; res_count = 0;
    rezero();
    return;
  }
  if (n0 >= n) {
    rezero();
    return;
  }
  const int n_here = (int)min((int64_t)kTpChunk, (int64_t)n - n0);
  float4 v[kTpVec];
  load_chunk(reinterpret_cast<const float4*>(a.scores + (int64_t)r * a.score_stride + n0), n_here, tid, v);
  __shared__ uint64_t sh_part[kTpThreads / 64];
  __shared__ uint64_t sh_res[3];
  __shared__ int sh_red[kTpThreads / 64][3];
  __shared__ uint64_t sh_tot[kTpThreads / 64][2];
  __shared__ int sh_cnt[ATTEND ? kTpThreads : 1], sh_pre[ATTEND ? kTpThreads : 1];   // balanced gather: kept per chunk, and before it
  const uint64_t* hrow = a.hist + (int64_t)r * a.hist_stride;
  // level 2 always leaves st[0]; level 3 leaves st[1] (a copy of st[0] for rows that carry no search)
  const RowState prev = a.state[(int64_t)r * 3 + 1];

  int kept_here = 0, kept_base = 0;
  bool balanced = false;          // ATTEND: gather an equal share of the row's ranks instead of this chunk's own tokens
  const bool empty_row = prev.flags < 0 || prev.flags == 2;      // the same in every workgroup of the row
  if (empty_row) {
    have_res = true;
    res_count = prev.flags < 0 ? prev.flags : 0;
    res_tau = prev.flags < 0 ? __builtin_nanf("") : ninf;
    res_mass = 0.f;
    if (!ATTEND) {
      rezero();
      return;
    }
  } else {
  uint32_t tkey = 0;      // keep keys >= tkey
  if (prev.flags == 0) {
    const ScanResult sr = scan_from_top<kBins3>(l3_bins, prev.above, prev.target, sh_part, sh_res);
    tkey = (prev.prefix << 10) | (uint32_t)sr.bin;
    res_tau = key_float(tkey);
    res_mass = a.kcount ? __builtin_nanf("") : (float)((prev.above_base + (double)(sr.above + sr.bin_mass)) / prev.total_d);
  } else {
    res_tau = ninf;
    res_mass = 1.f;
  }
  have_res = true;

  // ---- offset of this chunk = kept scores of the chunks before it; chunk 0 also publishes the total ----
  const int n_row_chunks = (n + kTpChunk - 1) / kTpChunk;
  const int listed = prev.flags == 0 ? listed_raw : 0;
  int before = 0, total = 0;
  if (listed <= kBucketCap) {
    if (tid < n_row_chunks) {
      total += cc_mine;
      if (tid < c) before += cc_mine;
    }
    for (int i = tid + kTpThreads; i < n_row_chunks; i += kTpThreads) {      // longer rows
      const int cv = a.chunk_cnt[(int64_t)r * a.n_chunks + i];
      total += cv;
      if (i < c) before += cv;
    }
#pragma unroll
    for (int k = 0; k < kBucketCap / kTpThreads; ++k) {
      if (k * kTpThreads + tid < listed && be[k].x >= tkey) {
        total += 1;
        if ((int64_t)be[k].y < n0) before += 1;
      }
    }
  } else {
    // more scores share the 22-bit prefix than the list holds: count the kept scores before this chunk
    // (and, for chunk 0, of the whole row) straight from the scores
    const float* row = a.scores + (int64_t)r * a.score_stride;
    const int64_t upto = c == 0 ? n : n0;
    for (int64_t i = tid; i < upto; i += kTpThreads) {
      const float sv = row[i];
      const int k1 = (sv != ninf && float_key(sv) >= tkey) ? 1 : 0;
      total += k1;
      if (i < n0) before += k1;
    }
  }
  before = wave_sum(before);
  total = wave_sum(total);
  // ATTEND: the fullest chunk of the row (certainly-kept counts; the short list adds at most kBucketCap)
  const int fullest_w = ATTEND ? wave_max_ge_m1(tid < n_row_chunks ? cc_mine : 0) : 0;   // (counts past the row's own chunks are stale)
  if ((tid & 63) == 0) { sh_red[tid >> 6][0] = before; sh_red[tid >> 6][1] = total; sh_red[tid >> 6][2] = fullest_w; }
  __syncthreads();
  before = 0;
  total = 0;
  int fullest = 0;
#pragma unroll
  for (int i = 0; i < kTpThreads / 64; ++i) { before += sh_red[i][0]; total += sh_red[i][1]; fullest = max(fullest, sh_red[i][2]); }
  res_count = total;

  const uint32_t keep = keep_mask(v, n_here, tid, prev.flags == 1, tkey);
  // The gather below is split by chunk, which is even only as far as the kept tokens are spread over the
  // row.  Where one chunk holds far more than its share (the same verdict in every workgroup of the row),
  // each workgroup gathers an equal share of the row's RANKS instead: it finds the chunks that hold its
  // ranks from the exact per-chunk counts and repeats their compaction (a 32 KB read each).  That costs
  // about 6 us per call, what the fullest chunk's workgroup needs for some 400 rows more than its share:
  // hence the threshold (configuration 2 itself: 575 kept tokens per chunk, 766 in the fullest).
  balanced = ATTEND && a.balance && prev.flags == 0 && listed <= kBucketCap && n_row_chunks > 1 && n_row_chunks <= kTpThreads &&
             fullest > 5 * (total / n_row_chunks) / 4 + 256;
  if (!balanced) {
    // ATTEND: the positions go to LDS only for now and to memory after the gather (same reason as above: the
    // gather starts behind a barrier, and every wait for a K/V row would also wait for stores in flight)
    kept_here = write_ranked(keep, before, ATTEND ? nullptr : a.sel_idx + (int64_t)r * a.sel_stride, n0, sh_tot,
                             ATTEND ? sh_list : nullptr);
    kept_base = before;
  } else {
    write_ranked(keep, before, a.sel_idx + (int64_t)r * a.sel_stride, n0, sh_tot, nullptr);   // this chunk's part of the list
    // exact kept count of every chunk: the level-3 launch's count + the kept members of the short list
    sh_cnt[tid] = tid < n_row_chunks ? cc_mine : 0;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kBucketCap / kTpThreads; ++k)
      if (k * kTpThreads + tid < listed && be[k].x >= tkey) atomicAdd(&sh_cnt[be[k].y / kTpChunk], 1);
    __syncthreads();
    // Shares are equal in COST: a chunk that holds kept tokens costs its kept count plus kScanCost (what
    // repeating its compaction takes, in gathered tokens), laid out along one axis in chunk order with the
    // scan cost first; workgroup c takes the c-th of n_row_chunks equal pieces of that axis and with it the
    // ranks of the tokens that lie inside -- a contiguous run of ranks, from one chunk or a few.
    const int mine = sh_cnt[tid];
    const int my_scan = mine > 0 ? kScanCost : 0;
    const uint64_t packed = ((uint64_t)(uint32_t)(mine + my_scan) << 32) | (uint32_t)mine;
    const uint64_t incl = wave_incl_scan(packed);
    if ((tid & 63) == 63) sh_tot[tid >> 6][0] = incl;
    __syncthreads();
    uint64_t waves_before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < kTpThreads / 64; ++i) {
      waves_before += i < (tid >> 6) ? sh_tot[i][0] : 0;
      all += sh_tot[i][0];
    }
    const uint64_t excl = waves_before + incl - packed;
    const int q0 = (int)(excl >> 32);                    // cost before this thread's chunk
    sh_pre[tid] = (int)(uint32_t)excl;                   // kept tokens before it
    const int64_t cost_all = (int64_t)(all >> 32);
    const int w_lo = (int)(cost_all * c / n_row_chunks), w_hi = (int)(cost_all * (c + 1) / n_row_chunks);
    // ranks below a point x of the cost axis: this chunk's share, summed over the chunks
    auto below = [&](int x) { return min(max(x - q0 - my_scan, 0), mine); };
    const int lo_w = wave_sum(below(w_lo)), hi_w = wave_sum(below(w_hi));
    if ((tid & 63) == 0) { sh_red[tid >> 6][0] = lo_w; sh_red[tid >> 6][1] = hi_w; }
    __syncthreads();
    int g_lo = 0, g_hi = 0;
#pragma unroll
    for (int i = 0; i < kTpThreads / 64; ++i) { g_lo += sh_red[i][0]; g_hi += sh_red[i][1]; }
    for (int i = 0; i < n_row_chunks; ++i) {
      __syncthreads();                                   // sh_pre written / sh_tot of the last compaction read
      const int p0 = sh_pre[i], p1 = p0 + sh_cnt[i];
      if (p1 == p0 || p1 <= g_lo || p0 >= g_hi) continue;   // (the same for every thread)
      uint32_t kp = keep;                                // this workgroup's own chunk: already in registers
      if (i != c) {
        const int nh = (int)min((int64_t)kTpChunk, (int64_t)n - (int64_t)i * kTpChunk);
        float4 vv[kTpVec];
        load_chunk(reinterpret_cast<const float4*>(a.scores + (int64_t)r * a.score_stride + (int64_t)i * kTpChunk), nh, tid, vv);
        kp = keep_mask(vv, nh, tid, false, tkey);
      }
      write_ranked(kp, p0, nullptr, (int64_t)i * kTpChunk, sh_tot, sh_list, g_lo, g_hi);
    }
    kept_here = g_hi - g_lo;
  }
  }
  if (!ATTEND) {
    rezero();
    return;
  }

  // ---- attention over this chunk's kept positions: groups of 16 lanes, one K/V row (256 bytes) per
  // group and load, kSaInFlight rows per group in flight; a lane owns 8 of the 128 dims ----
  __shared__ float sh_m[kTpThreads / 64], sh_l[kTpThreads / 64];
  __shared__ float sh_acc[kTpThreads / 64][kHeadDim];
  __syncthreads();                           // the list is complete
  const int lane = tid & 63, wave = tid >> 6;
  const int grp = wave * 4 + (lane >> 4), piece = lane & 15;
  const int b = r / ga.n_ret;
  const int h = ga.ret_heads[r - b * ga.n_ret];
  const int kvh = h / (ga.n_q_heads / ga.n_kv_heads);
  const int64_t seq0 = PAGED ? 0 : ga.seq_start[b];
  const uint16_t* Kb = ga.K + (int64_t)kvh * ga.head_stride + seq0 * ga.row_stride + piece * 8;
  const uint16_t* Vb = ga.V + (int64_t)kvh * ga.head_stride + seq0 * ga.row_stride + piece * 8;
  if (PAGED) {
    const int32_t* pt = ga.page_table + (int64_t)b * ga.pt_stride;
    const int mask = (1 << ga.page_shift) - 1;
    for (int i = tid; i < kept_here; i += kTpThreads) {
      const int p = sh_list[i];
      sh_rows[i] = (pt[p >> ga.page_shift] << ga.page_shift) | (p & mask);
    }
    __syncthreads();
  }
  const int32_t* rows = PAGED ? sh_rows : sh_list;
  float qv[8];
  unpack8<F16>(*reinterpret_cast<const u32x4*>(ga.q + ((int64_t)b * ga.n_q_heads + h) * kHeadDim + piece * 8), qv);
#pragma unroll
  for (int d = 0; d < 8; ++d) qv[d] *= ga.scale_log2;
  float m = ninf, l = 0.f, acc[8];
#pragma unroll
  for (int d = 0; d < 8; ++d) acc[d] = 0.f;
  constexpr int kGroups = kTpThreads / 16;   // 16-lane groups of the workgroup, one K/V row each per load
  for (int base = 0; base < kept_here; base += kGroups * kSaInFlight) {
    u32x4 kr[kSaInFlight], vr[kSaInFlight];
    bool ok[kSaInFlight];
#pragma unroll
    for (int u = 0; u < kSaInFlight; ++u) {
      const int i = base + u * kGroups + grp;
      ok[u] = i < kept_here;
      if (ok[u]) {
        const int64_t pos = rows[i];
        kr[u] = *reinterpret_cast<const u32x4*>(Kb + pos * ga.row_stride);
        vr[u] = *reinterpret_cast<const u32x4*>(Vb + pos * ga.row_stride);
      } else {
        kr[u] = (u32x4){0u, 0u, 0u, 0u};
        vr[u] = (u32x4){0u, 0u, 0u, 0u};
      }
    }
    float sc[kSaInFlight];
    float mx = ninf;
#pragma unroll
    for (int u = 0; u < kSaInFlight; ++u) {
      float kf[8];
      unpack8<F16>(kr[u], kf);
      float d = kf[0] * qv[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) d = fmaf(kf[e], qv[e], d);
      d = row16_sum(d);
      sc[u] = ok[u] ? d : ninf;
      mx = fmaxf(mx, sc[u]);
    }
    const float mn = fmaxf(m, mx);
    if (mn != ninf) {
      const float corr = fast_exp2(m - mn);
      l *= corr;
#pragma unroll
      for (int d = 0; d < 8; ++d) acc[d] *= corr;
      m = mn;
    }
#pragma unroll
    for (int u = 0; u < kSaInFlight; ++u) {
      float vf[8];
      unpack8<F16>(vr[u], vf);
      const float pw = (sc[u] == ninf) ? 0.f : fast_exp2(sc[u] - m);
      l += pw;
#pragma unroll
      for (int d = 0; d < 8; ++d) acc[d] = fmaf(pw, vf[d], acc[d]);
    }
  }
  // the four groups of a wave in registers, the four waves through LDS
#pragma unroll
  for (int o = 16; o <= 32; o <<= 1) {
    const float mo = __shfl_xor(m, o), lo = __shfl_xor(l, o);
    float ao[8];
#pragma unroll
    for (int d = 0; d < 8; ++d) ao[d] = __shfl_xor(acc[d], o);
    const float M = fmaxf(m, mo);
    if (M != ninf) {
      const float ca = fast_exp2(m - M), cb = fast_exp2(mo - M);
      l = l * ca + lo * cb;
#pragma unroll
      for (int d = 0; d < 8; ++d) acc[d] = acc[d] * ca + ao[d] * cb;
      m = M;
    }
  }
  if (lane < 16) {
    if (piece == 0) { sh_m[wave] = m; sh_l[wave] = l; }
#pragma unroll
    for (int d = 0; d < 8; ++d) sh_acc[wave][piece * 8 + d] = acc[d];
  }
  __syncthreads();
  if (tid < kHeadDim) {
    float M = sh_m[0];
#pragma unroll
    for (int w = 1; w < kTpThreads / 64; ++w) M = fmaxf(M, sh_m[w]);
    float L = 0.f, A = 0.f;
    if (M != ninf) {
#pragma unroll
      for (int w = 0; w < kTpThreads / 64; ++w) {
        const float cw = fast_exp2(sh_m[w] - M);
        L += sh_l[w] * cw;
        A += sh_acc[w][tid] * cw;
      }
    }
    float* pout = ga.part + ((int64_t)r * a.n_chunks + c) * kSaPart;
    pout[4 + tid] = A;
    if (tid == 0) { pout[0] = M; pout[1] = L; }
  }
  if (!balanced) {   // the chunk's positions, in one coalesced piece (after the last barrier)
    int32_t* dst = a.sel_idx + (int64_t)r * a.sel_stride + kept_base;
    for (int i = tid; i < kept_here; i += kTpThreads) dst[i] = sh_list[i];
  }
  rezero();
}

// Merges the (row, chunk) partials of one row: 8 slices of 32 lanes walk the chunks slice, slice + 8, ...
// (each lane owns 4 of the 128 output dims); LDS merges the slices.  Rows without a kept token give zeros.
// Workgroups past the R rows (rtp_decode_attention only) merge the local heads' partials, one (unit, head) each.
template <int RIDE_G>
__global__ __launch_bounds__(256) void select_attend_combine_kernel(const TopPArgs a, const GatherArgs ga,
                                                                    const AttnDecodeArgs la) {
  if (RIDE_G > 0 && (int)blockIdx.x >= a.R) {
    const int blk = (int)blockIdx.x - a.R;
    const int unit = blk / RIDE_G, hh = blk - unit * RIDE_G;
    const int b = unit / la.n_kv_heads, h = (unit - b * la.n_kv_heads) * RIDE_G + hh;
    if (la.is_ret[h]) return;
    const int i0 = unit * la.n_splits;
    const int i1 = i0 + (unit_tokens<kSrcLocal>(la, unit) + la.split_tokens - 1) / la.split_tokens;
    merge_partials_to_out(la, RIDE_G, hh, b, h, i0, i1);
    return;
  }
  __shared__ float sh_m[8], sh_l[8];
  __shared__ float sh_acc[8][kHeadDim];
  const int r = blockIdx.x, tid = threadIdx.x;
  const float ninf = -__builtin_huge_valf();
  const int n = a.row_len[r];
  const int n_row_chunks = n > 0 ? (n + kTpChunk - 1) / kTpChunk : 0;
  const int d4 = tid & 31, slice = tid >> 5;
  float M = ninf, L = 0.f;
  float4 A = make_float4(0.f, 0.f, 0.f, 0.f);
  // four partials in flight per slice: a long row has hundreds of chunks and each load is a round trip
  for (int i0 = slice; i0 < n_row_chunks; i0 += 8 * 4) {
    float pm[4], pl[4];
    float4 pv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * 8;
      pm[u] = ninf; pl[u] = 0.f; pv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < n_row_chunks) {
        const float* p = ga.part + ((int64_t)r * a.n_chunks + i) * kSaPart;
        pm[u] = p[0]; pl[u] = p[1];
        pv[u] = *reinterpret_cast<const float4*>(p + 4 + d4 * 4);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float Mn = fmaxf(M, pm[u]);
      if (Mn != ninf) {
        const float c0 = fast_exp2(M - Mn), c1 = fast_exp2(pm[u] - Mn);
        L = L * c0 + pl[u] * c1;
        A.x = A.x * c0 + pv[u].x * c1; A.y = A.y * c0 + pv[u].y * c1;
        A.z = A.z * c0 + pv[u].z * c1; A.w = A.w * c0 + pv[u].w * c1;
        M = Mn;
      }
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
    const int b = r / ga.n_ret;
    const int64_t o = (int64_t)b * ga.n_q_heads + ga.ret_heads[r - b * ga.n_ret];
    ga.out[o * kHeadDim + tid] = f32_to_16(Lt > 0.f ? At / Lt : 0.f, ga.f16 != 0);
    if (ga.lse && tid == 0) ga.lse[o] = Lt > 0.f ? (Mt + log2f(Lt)) * 0.6931471805599453f : ninf;
  }
}

}  // namespace rtp

using namespace rtp;

extern "C" size_t rtp_topp_workspace_bytes(int32_t R, int64_t max_len) {
  if (R <= 0 || max_len <= 0) return 0;
  return topp_layout(R, max_len).total;
}

extern "C" int32_t rtp_topp_workspace_init(void* ws, size_t ws_bytes, void* stream) {
  const char* who = "rtp_topp_workspace_init";
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes == 0 || (ws_bytes & 7))
    return fail(RTP_ERR_WORKSPACE, "%s: workspace must be 256-byte aligned and a multiple of 8 bytes", who);
  clear_error();
  const int64_t n = (int64_t)(ws_bytes / 8);
  RTP_LAUNCH(topp_zero_kernel, dim3((unsigned)((n + kTpThreads - 1) / kTpThreads)), dim3(kTpThreads), 0,
                     (hipStream_t)stream, (uint64_t*)ws, n);
  return check_launch(who);
}

// Shared body of rtp_topp_select (p != NULL) and rtp_topk_select (kcount != NULL).
static int32_t run_select(const char* who, const float* scores, int64_t score_stride, const int32_t* row_len,
                          const float* p, const int32_t* kcount, int32_t R, int64_t max_len,
                          int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                          float* tau, float* mass, int32_t level1_ready,
                          void* ws, size_t ws_bytes, void* stream, const GatherArgs* attend = nullptr,
                          const AttnDecodeArgs* ride = nullptr, int ride_G = 0) {
  if (!scores || !row_len || (!p && !kcount) || !sel_idx || !sel_count)
    return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (R <= 0 || R > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: R must be in [1, 65535]", who);
  if (max_len <= 0 || max_len > RTP_MAX_ROW_LEN)
    return fail(RTP_ERR_INVALID_ARG, "%s: max_len must be in [1, %d]", who, RTP_MAX_ROW_LEN);
  if (score_stride < max_len || (score_stride & 3) || ((uintptr_t)scores & 15))
    return fail(RTP_ERR_INVALID_ARG, "%s: scores must be 16-byte aligned, score_stride >= max_len and a multiple of 4", who);
  if (sel_stride < max_len) return fail(RTP_ERR_INVALID_ARG, "%s: sel_stride must be >= max_len", who);
  if (level1_ready != 0 && level1_ready != 1) return fail(RTP_ERR_INVALID_ARG, "%s: level1_ready must be 0 or 1", who);
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
  a.kcount = kcount;
  a.R = R;
  a.n_chunks = (int32_t)((max_len + kTpChunk - 1) / kTpChunk);
  a.rezero = level1_ready;
  a.balance = 1;
  a.sel_idx = sel_idx;
  a.sel_stride = sel_stride;
  a.sel_count = sel_count;
  a.tau = tau;
  a.mass = mass;
  a.chunk_cnt = (int32_t*)((char*)ws + l.ccnt_off);
  a.hist = (uint64_t*)((char*)ws + l.hist_off);
  a.hist_stride = l.hist_stride;
  a.n_sub = l.n_sub;
  a.state = (RowState*)((char*)ws + l.state_off);
  a.bucket_n = (int32_t*)((char*)ws + l.bn_off);
  a.bucket = (uint2*)((char*)ws + l.bucket_off);

  hipStream_t s = (hipStream_t)stream;
  dim3 grid((unsigned)a.n_chunks, (unsigned)R), block(kTpThreads);
  if (!level1_ready) {
    const int64_t nz = (int64_t)R * l.hist_stride;
    RTP_LAUNCH(topp_zero_kernel, dim3((unsigned)((nz + kTpThreads - 1) / kTpThreads)), block, 0, s, a.hist, nz);
    RTP_LAUNCH(topp_level_kernel<1>, grid, block, 0, s, a);
  }
  if (ride) {
    // the local heads' work items travel in the level-2 launch (the longer of the two middle launches; giving
    // level 3 a share was measured slower: a carried item costs its chain of load rounds whichever launch it is
    // in); at most one carried workgroup per compute unit
    const int n_items = ride->units * ride->n_splits;
    const int n_ride = n_items < 256 ? n_items : 256;
    const dim3 grid2((unsigned)(n_ride + a.n_chunks * R));
    const bool paged = ride->page_table != nullptr;
#define RTP_RIDE(GG)                                                                                                   \
  do {                                                                                                                  \
    if (ride->f16 && paged) RTP_LAUNCH((topp_level_ride_kernel<2, GG, true, true>), grid2, block, 0, s, a, *ride, n_ride, 0, n_items);        \
    else if (ride->f16) RTP_LAUNCH((topp_level_ride_kernel<2, GG, true, false>), grid2, block, 0, s, a, *ride, n_ride, 0, n_items);           \
    else if (paged) RTP_LAUNCH((topp_level_ride_kernel<2, GG, false, true>), grid2, block, 0, s, a, *ride, n_ride, 0, n_items);               \
    else RTP_LAUNCH((topp_level_ride_kernel<2, GG>), grid2, block, 0, s, a, *ride, n_ride, 0, n_items);                                       \
  } while (0)
    if (ride_G == 2) RTP_RIDE(2);
    else if (ride_G == 4) RTP_RIDE(4);
    else RTP_RIDE(8);
#undef RTP_RIDE
    RTP_LAUNCH(topp_level_kernel<3>, grid, block, 0, s, a);
  } else {
    RTP_LAUNCH(topp_level_kernel<2>, grid, block, 0, s, a);
    RTP_LAUNCH(topp_level_kernel<3>, grid, block, 0, s, a);
  }
  if (attend) {
    const bool paged = attend->page_table != nullptr;
    if (attend->f16 && paged) RTP_LAUNCH((topp_write_kernel<true, true, true>), grid, block, 0, s, a, *attend);
    else if (attend->f16) RTP_LAUNCH((topp_write_kernel<true, true>), grid, block, 0, s, a, *attend);
    else if (paged) RTP_LAUNCH((topp_write_kernel<true, false, true>), grid, block, 0, s, a, *attend);
    else RTP_LAUNCH(topp_write_kernel<true>, grid, block, 0, s, a, *attend);
    if (ride) {
      const dim3 cgrid((unsigned)(R + ride->units * ride_G));
      if (ride_G == 2) RTP_LAUNCH(select_attend_combine_kernel<2>, cgrid, dim3(256), 0, s, a, *attend, *ride);
      else if (ride_G == 4) RTP_LAUNCH(select_attend_combine_kernel<4>, cgrid, dim3(256), 0, s, a, *attend, *ride);
      else RTP_LAUNCH(select_attend_combine_kernel<8>, cgrid, dim3(256), 0, s, a, *attend, *ride);
    } else {
      RTP_LAUNCH(select_attend_combine_kernel<0>, dim3((unsigned)R), dim3(256), 0, s, a, *attend, AttnDecodeArgs{});
    }
  } else {
    RTP_LAUNCH(topp_write_kernel<false>, grid, block, 0, s, a, GatherArgs{});
  }
  return check_launch(who);
}

extern "C" int32_t rtp_topp_select(const float* scores, int64_t score_stride, const int32_t* row_len,
                                   const float* p, int32_t R, int64_t max_len,
                                   int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                   float* tau, float* mass, int32_t level1_ready,
                                   void* ws, size_t ws_bytes, void* stream) {
  if (!p) return fail(RTP_ERR_INVALID_ARG, "rtp_topp_select: NULL tensor pointer");
  return run_select("rtp_topp_select", scores, score_stride, row_len, p, nullptr, R, max_len, sel_idx, sel_stride,
                    sel_count, tau, mass, level1_ready, ws, ws_bytes, stream);
}

// ---- rtp_topp_select for callers that cannot allocate --------------------------------------------------
// The workspace of the call is a file-scope device array instead of a caller buffer.  In host code the
// array's name is only a stand-in: its device address is asked for once per device (with that device
// current) and kept; every launch takes that address.
constexpr size_t kNoAllocBytes = RTP_TOPP_NOALLOC_WS_BYTES;
static __device__ __align__(256) unsigned char g_noalloc_scratch[kNoAllocBytes];
constexpr int kNoAllocMaxDevices = 64;
static void* g_noalloc_ptr[kNoAllocMaxDevices];          // per device; written once under the mutex below
static std::mutex g_noalloc_mutex;

static int32_t noalloc_scratch(const char* who, void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kNoAllocMaxDevices)
    return fail(RTP_ERR_HIP, "%s: no current device (or device index >= %d)", who, kNoAllocMaxDevices);
  std::lock_guard<std::mutex> lock(g_noalloc_mutex);
  if (!g_noalloc_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_noalloc_scratch));
    if (e != hipSuccess || !ptr)
      return fail(RTP_ERR_HIP, "%s: hipGetSymbolAddress failed: %s", who, hipGetErrorString(e));
    g_noalloc_ptr[dev] = ptr;
  }
  *out = g_noalloc_ptr[dev];
  return RTP_OK;
}

extern "C" int32_t rtp_topp_select_noalloc(const float* scores, int64_t score_stride, const int32_t* row_len,
                                           const float* p, int32_t R, int64_t max_len,
                                           int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                           float* tau, float* mass, void* stream) {
  const char* who = "rtp_topp_select_noalloc";
  if (!p) return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (R <= 0 || R > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: R must be in [1, 65535]", who);
  if (max_len <= 0 || max_len > RTP_MAX_ROW_LEN)
    return fail(RTP_ERR_INVALID_ARG, "%s: max_len must be in [1, %d]", who, RTP_MAX_ROW_LEN);
  const size_t need = topp_layout(R, max_len).total;
  if (need > kNoAllocBytes)
    return fail(RTP_ERR_WORKSPACE, "%s: R = %d rows of up to %lld scores need %zu bytes of scratch, the built-in "
                "buffer holds %zu (use rtp_topp_select with a workspace of your own)", who, R, (long long)max_len, need,
                kNoAllocBytes);
  void* ws = nullptr;
  const int32_t rc = noalloc_scratch(who, &ws);
  if (rc != RTP_OK) return rc;
  return run_select(who, scores, score_stride, row_len, p, nullptr, R, max_len, sel_idx, sel_stride, sel_count, tau, mass,
                    0, ws, kNoAllocBytes, stream);
}

extern "C" int32_t rtp_topk_select(const float* scores, int64_t score_stride, const int32_t* row_len,
                                   const int32_t* k, int32_t R, int64_t max_len,
                                   int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count, float* tau,
                                   void* ws, size_t ws_bytes, void* stream) {
  if (!k) return fail(RTP_ERR_INVALID_ARG, "rtp_topk_select: NULL tensor pointer");
  return run_select("rtp_topk_select", scores, score_stride, row_len, nullptr, k, R, max_len, sel_idx, sel_stride,
                    sel_count, tau, nullptr, 0, ws, ws_bytes, stream);
}

extern "C" size_t rtp_select_attend_decode_workspace_bytes(const rtp_layer_desc* layer, int32_t B, int64_t max_ctx) {
  if (!layer || B <= 0 || max_ctx <= 0 || layer->n_ret <= 0) return 256;
  const int64_t n_chunks = (max_ctx + kTpChunk - 1) / kTpChunk;
  return align_up((size_t)B * layer->n_ret * n_chunks * kSaPart * sizeof(float), 256);
}

// Argument checks of the selection + attention call and its gather arguments (shared by the two entry points).
static int32_t prepare_select_attend(const char* who, const rtp_layer_desc* layer, const float* p, int32_t B, int64_t max_ctx,
                                     const void* q, const void* K, const void* V, int64_t kv_row_stride,
                                     int64_t kv_head_stride, const int64_t* seq_start, void* out, float* lse,
                                     void* attn_ws, size_t attn_ws_bytes, GatherArgs* ga, int64_t* R,
                                     const PageSource* pages = nullptr) {
  HeadTable ht;
  int32_t rc = fill_head_table(layer, &ht, who);
  if (rc != RTP_OK) return rc;
  if (!p || !q || !K || !V || !out || (!seq_start && !pages)) return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  int page_shift = 0;
  if (pages) {
    rc = check_pages(who, pages, max_ctx, &page_shift);
    if (rc != RTP_OK) return rc;
  }
  if (kv_row_stride < kHeadDim || (kv_row_stride & 7) || (kv_head_stride & 7) || kv_head_stride < 0)
    return fail(RTP_ERR_INVALID_ARG, "%s: kv_row_stride must be >= 128, strides multiples of 8", who);
  if (((uintptr_t)q & 15) || ((uintptr_t)K & 15) || ((uintptr_t)V & 15) || ((uintptr_t)out & 15))
    return fail(RTP_ERR_INVALID_ARG, "%s: q, K, V and out must be 16-byte aligned", who);
  if (B <= 0) return fail(RTP_ERR_INVALID_ARG, "%s: B must be positive", who);
  *R = (int64_t)B * layer->n_ret;
  if (*R > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: B * n_ret is limited to 65535", who);
  if (layer->n_ret == 0) return RTP_OK;
  const size_t need = rtp_select_attend_decode_workspace_bytes(layer, B, max_ctx);
  if (!attn_ws || ((uintptr_t)attn_ws & 255) || attn_ws_bytes < need)
    return fail(RTP_ERR_WORKSPACE, "%s: attention workspace of %zu bytes (256-byte aligned) required, got %zu", who, need,
                attn_ws_bytes);
  ga->q = (const uint16_t*)q;
  ga->K = (const uint16_t*)K;
  ga->V = (const uint16_t*)V;
  ga->row_stride = kv_row_stride;
  ga->head_stride = kv_head_stride;
  ga->seq_start = seq_start;
  ga->n_q_heads = layer->n_q_heads;
  ga->n_kv_heads = layer->n_kv_heads;
  ga->n_ret = layer->n_ret;
  ga->scale_log2 = softmax_scale_of(layer) * 1.4426950408889634f;
  ga->part = (float*)attn_ws;
  ga->out = (uint16_t*)out;
  ga->lse = lse;
  ga->f16 = layer->kv_dtype == RTP_DTYPE_FP16;
  ga->page_table = pages ? pages->table : nullptr;
  ga->pt_stride = pages ? pages->stride : 0;
  ga->page_shift = page_shift;
  for (int j = 0; j < 64; ++j) ga->ret_heads[j] = ht.ret_heads[j];
  return RTP_OK;
}

extern "C" int32_t rtp_select_attend_decode(const rtp_layer_desc* layer, const float* scores, int64_t score_stride,
                                            const int32_t* row_len, const float* p, int32_t B, int64_t max_ctx,
                                            const void* q, const void* K, const void* V, int64_t kv_row_stride,
                                            int64_t kv_head_stride, const int64_t* seq_start,
                                            int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                            float* tau, float* mass, int32_t level1_ready, void* out, float* lse,
                                            void* topp_ws, size_t topp_ws_bytes, void* attn_ws, size_t attn_ws_bytes,
                                            void* stream) {
  const char* who = "rtp_select_attend_decode";
  GatherArgs ga;
  int64_t R = 0;
  const int32_t rc = prepare_select_attend(who, layer, p, B, max_ctx, q, K, V, kv_row_stride, kv_head_stride, seq_start, out,
                                           lse, attn_ws, attn_ws_bytes, &ga, &R);
  if (rc != RTP_OK) return rc;
  if (layer->n_ret == 0) { clear_error(); return RTP_OK; }
  return run_select(who, scores, score_stride, row_len, p, nullptr, (int32_t)R, max_ctx, sel_idx, sel_stride, sel_count,
                    tau, mass, level1_ready, topp_ws, topp_ws_bytes, stream, &ga);
}

static int32_t decode_attention_impl(const char* who, const PageSource* pages,
                                     const rtp_layer_desc* layer, const float* scores, int64_t score_stride,
                                     const int32_t* row_len, const float* p, const int32_t* ctx_len, int32_t B,
                                     int64_t max_ctx, const void* q, const void* K, const void* V,
                                     int64_t kv_row_stride, int64_t kv_head_stride, const int64_t* seq_start,
                                     int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                     float* tau, float* mass, int32_t level1_ready, void* out, float* lse,
                                     void* topp_ws, size_t topp_ws_bytes, void* attn_ws, size_t attn_ws_bytes,
                                     void* local_ws, size_t local_ws_bytes, void* stream) {
  GatherArgs ga;
  int64_t R = 0;
  int32_t rc = prepare_select_attend(who, layer, p, B, max_ctx, q, K, V, kv_row_stride, kv_head_stride, seq_start, out, lse,
                                     attn_ws, attn_ws_bytes, &ga, &R, pages);
  if (rc != RTP_OK) return rc;
  AttnDecodeArgs la;
  int lgrid = 0;
  bool have_local = false;
  rc = decode_range_prepare(who, false, layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len, B, max_ctx, out,
                            lse, local_ws, local_ws_bytes, nullptr, &la, &lgrid, &have_local, pages);
  if (rc != RTP_OK) return rc;
  const int G = layer->n_q_heads / layer->n_kv_heads;
  hipStream_t s = (hipStream_t)stream;
  if (layer->n_ret == 0) {               // nothing to select: the local heads are the whole layer
    return have_local ? decode_range_attn(who, false, layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len, B,
                                          max_ctx, out, lse, local_ws, local_ws_bytes, s, pages)
                      : RTP_OK;
  }
  // groups of 8 need 163 vector registers for a carried item, which costs the level-2 launch a resident
  // workgroup per compute unit: worth it while every carrier has one item (batch 8 x 131072 with 32 query /
  // 4 KV heads: 97 against 101 us per step), not for the long item chains of a large batch (a ragged batch of
  // 32 with 64 / 8 heads: 1.21 against 1.15 ms)
  const bool ride = have_local && (G == 2 || G == 4 || (G == 8 && (int64_t)la.units * la.n_splits <= 256));
  if (!ride) {
    // group sizes (or workloads) the carried form does not cover: the two parts one after the other
    rc = run_select(who, scores, score_stride, row_len, p, nullptr, (int32_t)R, max_ctx, sel_idx, sel_stride, sel_count, tau,
                    mass, level1_ready, topp_ws, topp_ws_bytes, stream, &ga);
    if (rc != RTP_OK || !have_local) return rc;
    return decode_range_attn(who, false, layer, q, K, V, kv_row_stride, kv_head_stride, seq_start, ctx_len, B, max_ctx, out,
                             lse, local_ws, local_ws_bytes, s, pages);
  }
  return run_select(who, scores, score_stride, row_len, p, nullptr, (int32_t)R, max_ctx, sel_idx, sel_stride, sel_count, tau,
                    mass, level1_ready, topp_ws, topp_ws_bytes, stream, &ga, &la, G);
}

extern "C" int32_t rtp_decode_attention(const rtp_layer_desc* layer, const float* scores, int64_t score_stride,
                                        const int32_t* row_len, const float* p, const int32_t* ctx_len, int32_t B,
                                        int64_t max_ctx, const void* q, const void* K, const void* V,
                                        int64_t kv_row_stride, int64_t kv_head_stride, const int64_t* seq_start,
                                        int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                        float* tau, float* mass, int32_t level1_ready, void* out, float* lse,
                                        void* topp_ws, size_t topp_ws_bytes, void* attn_ws, size_t attn_ws_bytes,
                                        void* local_ws, size_t local_ws_bytes, void* stream) {
  if (!seq_start) return fail(RTP_ERR_INVALID_ARG, "rtp_decode_attention: NULL tensor pointer");
  return decode_attention_impl("rtp_decode_attention", nullptr, layer, scores, score_stride, row_len, p, ctx_len, B, max_ctx, q,
                               K, V, kv_row_stride, kv_head_stride, seq_start, sel_idx, sel_stride, sel_count, tau, mass,
                               level1_ready, out, lse, topp_ws, topp_ws_bytes, attn_ws, attn_ws_bytes, local_ws,
                               local_ws_bytes, stream);
}

extern "C" int32_t rtp_decode_attention_paged(const rtp_layer_desc* layer, const float* scores, int64_t score_stride,
                                              const int32_t* row_len, const float* p, const int32_t* ctx_len, int32_t B,
                                              int64_t max_ctx, const void* q, const void* K, const void* V,
                                              int64_t kv_row_stride, int64_t kv_head_stride,
                                              const int32_t* page_table, int64_t pt_stride, int32_t page_size,
                                              int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                              float* tau, float* mass, int32_t level1_ready, void* out, float* lse,
                                              void* topp_ws, size_t topp_ws_bytes, void* attn_ws, size_t attn_ws_bytes,
                                              void* local_ws, size_t local_ws_bytes, void* stream) {
  const PageSource pages = {page_table, pt_stride, page_size};
  return decode_attention_impl("rtp_decode_attention_paged", &pages, layer, scores, score_stride, row_len, p, ctx_len, B,
                               max_ctx, q, K, V, kv_row_stride, kv_head_stride, nullptr, sel_idx, sel_stride, sel_count, tau,
                               mass, level1_ready, out, lse, topp_ws, topp_ws_bytes, attn_ws, attn_ws_bytes, local_ws,
                               local_ws_bytes, stream);
}
