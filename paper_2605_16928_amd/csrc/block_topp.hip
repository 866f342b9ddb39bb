// rtp_block_topp_select: the block-wise, sort-free top-p selector the paper describes for its decode
// kernel (Sec. 3.4, "Sort-free top-p via histogram"; block size 64 in its configuration table):
//   1. the candidates are cut into blocks of 64 consecutive tokens; a block is reduced to its
//      log-sum-exp pair (m_b = max score, l_b = sum exp(s - m_b));
//   2. the block deposits its mass l_b * exp(m_b) into the bin of a 256-bin histogram that m_b falls into;
//   3. the histogram is scanned from the highest bin down to the bin where the cumulative mass reaches p;
//   4. the mask keeps every block at or above that bin.
// Readings where the section is silent: bins are uniform in score (bin = floor((m_b - bin_lo) /
// bin_width), clamped to [0, 255]); deposits are integers -- every token's exp(s - upper edge of its
// block's bin) in fixed point, so a bin's content does not depend on the order of the atomics -- and the
// scan brings the bins to one scale in fp64.  Scores above the binned range count with the mass of the
// range's upper edge (the caller picks a range that covers its scores).
//
// What differs from the section's kernel (written for another GPU): it runs as its own launches behind
// the score pass instead of inside it, and the scan is repeated in the prologue of every workgroup of
// the next launch instead of being handed to the last workgroup to finish -- on this chip a hand-off
// between workgroups costs as much as a kernel boundary.  The kept tokens are written as an ascending
// index list, the format rtp_sparse_attn_decode consumes.
#include "topp_common.h"

namespace rtp {

constexpr int kBtThreads = 256;
constexpr int kBtChunk = 4096;                 // scores per workgroup = 64 blocks
constexpr int kBtBlock = 64;
constexpr int kBtBins = 256;
constexpr int kBtVec = kBtChunk / (kBtThreads * 4);
constexpr int kBtBlocksPerChunk = kBtChunk / kBtBlock;

struct BlockRowState {
  int32_t thr_bin;      // keep blocks whose bin is >= thr_bin
  int32_t flags;        // 0 ok, 1 keep everything (p >= 1), -1 invalid p, 2 no mass at all
};

struct BlockTopPArgs {
  const float* scores;
  int64_t score_stride;
  const int32_t* row_len;
  const float* p;
  int32_t R, n_chunks;
  float bin_lo, bin_width;
  int32_t* sel_idx;
  int64_t sel_stride;
  int32_t* sel_count;
  int32_t* thr_out;      // optional [R]
  float* mass;           // optional [R]
  uint8_t* mask_out;     // optional [R, mask_stride]
  int64_t mask_stride;
  uint64_t* hist;        // [R, 256]
  uint8_t* block_bin;    // [R, n_chunks * 64]
  int32_t* chunk_cnt;    // [R, n_chunks]
  BlockRowState* state;  // [R]
};

struct BlockLayout {
  size_t hist_off, bin_off, ccnt_off, state_off, total;
};
static BlockLayout block_layout(int32_t R, int64_t max_len) {
  const int64_t n_chunks = (max_len + kBtChunk - 1) / kBtChunk;
  BlockLayout l;
  size_t off = 0;
  l.hist_off = off;  off = align_up(off + (size_t)R * kBtBins * sizeof(uint64_t), 256);
  l.bin_off = off;   off = align_up(off + (size_t)R * n_chunks * kBtBlocksPerChunk, 256);
  l.ccnt_off = off;  off = align_up(off + (size_t)R * n_chunks * sizeof(int32_t), 256);
  l.state_off = off; off = align_up(off + (size_t)R * sizeof(BlockRowState), 256);
  l.total = off;
  return l;
}

__device__ __forceinline__ float row16_max(float x) {
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, true)));
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, true)));
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, true)));
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xf, 0xf, true)));
  return x;
}

// Bin of a block maximum, in fp64 like the definition; -inf (a block without a finite score) goes to bin 0.
__device__ __forceinline__ int bin_of(float m, double lo, double width) {
  const double q = floor(((double)m - lo) / width);
  return q >= (double)(kBtBins - 1) ? kBtBins - 1 : (q > 0.0 ? (int)q : 0);
}

__global__ __launch_bounds__(kBtThreads) void block_zero_kernel(uint64_t* hist, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBtThreads + threadIdx.x;
  if (i < n) hist[i] = 0;
}

__device__ __forceinline__ void load_chunk_bt(const float4* __restrict__ src, int n_here, int tid, float4 (&v)[kBtVec]) {
  const float ninf = -__builtin_huge_valf();
#pragma unroll
  for (int u = 0; u < kBtVec; ++u) {
    const int e = (u * kBtThreads + tid) * 4;
    if (e < n_here) v[u] = src[u * kBtThreads + tid];
    else v[u] = make_float4(ninf, ninf, ninf, ninf);
    if (e + 1 >= n_here) v[u].y = ninf;     // a vector that straddles the row end
    if (e + 2 >= n_here) v[u].z = ninf;
    if (e + 3 >= n_here) v[u].w = ninf;
  }
}

// ---- launch 1: block pairs -> histogram ---------------------------------------------------------------
// A block of 64 scores is 16 consecutive lanes (one DPP row) of one load round: its maximum is a row
// reduction, its mass the row sum of the lanes' fixed-point weights.
__global__ __launch_bounds__(kBtThreads) void block_stats_kernel(const BlockTopPArgs a) {
  const int r = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int n = a.row_len[r];
  const int64_t n0 = (int64_t)c * kBtChunk;
  if (n <= 0 || n0 >= n) return;
  const float pr = a.p[r];
  if (!(pr > 0.f) || pr >= 1.f) return;        // invalid or keep-all rows need no histogram
  const int n_here = (int)min((int64_t)kBtChunk, (int64_t)n - n0);
  float4 v[kBtVec];
  load_chunk_bt(reinterpret_cast<const float4*>(a.scores + (int64_t)r * a.score_stride + n0), n_here, tid, v);
  __shared__ uint64_t lh[kBtBins];
  __shared__ double tab[256];
  fill_exp_table(tab);
  lh[tid] = 0;
  __syncthreads();
  const int shift = fixed_shift(n);
  const double lo = (double)a.bin_lo, width = (double)a.bin_width;
  uint8_t* bins = a.block_bin + (int64_t)r * a.n_chunks * kBtBlocksPerChunk + (int64_t)c * kBtBlocksPerChunk;
#pragma unroll
  for (int u = 0; u < kBtVec; ++u) {
    const int blk = u * (kBtThreads / 16) + (tid >> 4);            // block of the chunk this lane's row covers
    if (blk * kBtBlock >= n_here) continue;                        // uniform over the 16-lane row
    const float s4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
    const float m_b = row16_max(fmaxf(fmaxf(s4[0], s4[1]), fmaxf(s4[2], s4[3])));
    const int bin = bin_of(m_b, lo, width);
    const double edge = lo + (double)(bin + 1) * width;
    uint64_t w = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (s4[k] == -__builtin_huge_valf()) continue;
      int e;
      const double mant = exp_parts((double)s4[k] - edge, tab, &e);   // arguments above 0 count as 0
      const double rr = ldexp(mant, shift + e) + 4503599627370496.0;
      w += (uint64_t)__double_as_longlong(rr) & 0xFFFFFFFFFFFFFull;
    }
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) w += __shfl_xor((unsigned long long)w, o);
    if ((tid & 15) == 0) {
      if (w) atomicAdd((unsigned long long*)&lh[bin], (unsigned long long)w);
      bins[blk] = (uint8_t)bin;
    }
  }
  __syncthreads();
  flush_hist(lh, a.hist + (int64_t)r * kBtBins, kBtBins, kBtThreads);
}

// Threshold bin of a row: every thread of the workgroup gets the same answer (fixed summation order).
// thread t holds bin t.  Returns -1 if the row has no mass.  *kept_frac: kept mass / total.
__device__ __forceinline__ int scan_block_hist(const uint64_t* __restrict__ h, float p, double lo, double width,
                                               double* sh /*[256]*/, int* sh_top, float* kept_frac) {
  const int tid = threadIdx.x;
  const uint64_t mine = h[tid];
  if (tid == 0) *sh_top = -1;
  __syncthreads();
  if (mine) atomicMax(sh_top, tid);
  __syncthreads();
  const int top = *sh_top;
  if (top < 0) { *kept_frac = 0.f; return -1; }
  // bring bin t to the scale of the top bin's edge
  sh[tid] = mine ? (double)mine * exp((double)(tid - top) * width) : 0.0;
  __syncthreads();
  double total = 0.0;
  for (int k = kBtBins - 1; k >= 0; --k) total += sh[k];
  const double target = (double)p * total;
  double cum = 0.0;
  int thr = 0;
  for (int k = kBtBins - 1; k >= 0; --k) {
    cum += sh[k];
    if (cum >= target) { thr = k; break; }
  }
  *kept_frac = (float)(cum / total);
  __syncthreads();
  return thr;
}

// Tokens of the chunk that belong to kept blocks; also fills keep bits (bit b = block b of the chunk).
__device__ __forceinline__ int chunk_kept(const uint8_t* bins, int n_here, int thr, bool all, uint64_t* keep_bits) {
  const int lane = threadIdx.x & 63;            // every wave computes the same 64-block picture
  const int n_blocks = (n_here + kBtBlock - 1) / kBtBlock;
  const bool keep = lane < n_blocks && (all || (int)bins[lane] >= thr);
  const uint64_t bits = __ballot(keep);
  *keep_bits = bits;
  int tokens = __popcll(bits) * kBtBlock;
  if ((n_here & (kBtBlock - 1)) && ((bits >> (n_blocks - 1)) & 1ull)) tokens -= kBtBlock - (n_here & (kBtBlock - 1));
  return tokens;
}

// ---- launch 2: scan + per-chunk kept-token counts --------------------------------------------------------
__global__ __launch_bounds__(kBtThreads) void block_count_kernel(const BlockTopPArgs a) {
  const int r = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int n = a.row_len[r];
  const int64_t n0 = (int64_t)c * kBtChunk;
  __shared__ double sh[kBtBins];
  __shared__ int sh_top;
  const float pr = a.p[r];
  int flags = (pr >= 1.f) ? 1 : ((pr > 0.f) ? 0 : -1);
  if (n <= 0) flags = flags < 0 ? -1 : 2;
  int thr = 0;
  float frac = 1.f;
  if (flags == 0) {
    thr = scan_block_hist(a.hist + (int64_t)r * kBtBins, pr, (double)a.bin_lo, (double)a.bin_width, sh, &sh_top, &frac);
    if (thr < 0) { flags = 2; thr = 0; }
  }
  if (c == 0 && tid == 0) {
    BlockRowState s;
    s.thr_bin = thr;
    s.flags = flags;
    a.state[r] = s;
    if (a.thr_out) a.thr_out[r] = flags == 0 ? thr : (flags == 1 ? 0 : -1);
    if (a.mass) a.mass[r] = flags == 0 ? frac : (flags == 1 ? 1.f : 0.f);
    if (flags < 0 || flags == 2) a.sel_count[r] = flags < 0 ? -1 : 0;
  }
  if (flags < 0 || flags == 2 || n0 >= n) return;
  const int n_here = (int)min((int64_t)kBtChunk, (int64_t)n - n0);
  const uint8_t* bins = a.block_bin + (int64_t)r * a.n_chunks * kBtBlocksPerChunk + (int64_t)c * kBtBlocksPerChunk;
  uint64_t bits;
  const int tokens = chunk_kept(bins, n_here, thr, flags == 1, &bits);
  if (tid == 0) a.chunk_cnt[(int64_t)r * a.n_chunks + c] = tokens;
}

// ---- launch 3: ascending token list of the kept blocks ---------------------------------------------------
__global__ __launch_bounds__(kBtThreads) void block_write_kernel(const BlockTopPArgs a) {
  const int r = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int n = a.row_len[r];
  const int64_t n0 = (int64_t)c * kBtChunk;
  if (n <= 0 || n0 >= n) return;
  const BlockRowState st = a.state[r];
  if (st.flags < 0 || st.flags == 2) return;
  __shared__ int sh_red[kBtThreads / 64][2];
  const int n_row_chunks = (n + kBtChunk - 1) / kBtChunk;
  int before = 0, total = 0;
  for (int i = tid; i < n_row_chunks; i += kBtThreads) {
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
  for (int i = 0; i < kBtThreads / 64; ++i) { before += sh_red[i][0]; total += sh_red[i][1]; }
  if (c == 0 && tid == 0) a.sel_count[r] = total;

  const int n_here = (int)min((int64_t)kBtChunk, (int64_t)n - n0);
  const uint8_t* bins = a.block_bin + (int64_t)r * a.n_chunks * kBtBlocksPerChunk + (int64_t)c * kBtBlocksPerChunk;
  uint64_t bits;
  chunk_kept(bins, n_here, st.thr_bin, st.flags == 1, &bits);
  if (a.mask_out && tid < kBtBlocksPerChunk && tid * kBtBlock < n_here)
    a.mask_out[(int64_t)r * a.mask_stride + (int64_t)c * kBtBlocksPerChunk + tid] = (uint8_t)((bits >> tid) & 1ull);
  int32_t* out = a.sel_idx + (int64_t)r * a.sel_stride + before;
  // every block before the row's last is full, so a kept token's slot is 64 * (kept blocks before its own) + its offset
  for (int e = tid; e < n_here; e += kBtThreads) {
    const int blk = e >> 6;
    if ((bits >> blk) & 1ull) {
      const int kb = __popcll(bits & ((1ull << blk) - 1ull));
      out[kb * kBtBlock + (e & 63)] = (int32_t)(n0 + e);
    }
  }
}

}  // namespace rtp

using namespace rtp;

extern "C" size_t rtp_block_topp_workspace_bytes(int32_t R, int64_t max_len) {
  if (R <= 0 || max_len <= 0) return 0;
  return block_layout(R, max_len).total;
}

extern "C" int32_t rtp_block_topp_select(const float* scores, int64_t score_stride, const int32_t* row_len,
                                         const float* p, int32_t R, int64_t max_len,
                                         int32_t block, float bin_lo, float bin_width,
                                         int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                         int32_t* threshold_bin, float* mass, uint8_t* block_mask, int64_t mask_stride,
                                         void* ws, size_t ws_bytes, void* stream) {
  const char* who = "rtp_block_topp_select";
  if (!scores || !row_len || !p || !sel_idx || !sel_count) return fail(RTP_ERR_INVALID_ARG, "%s: NULL tensor pointer", who);
  if (block != kBtBlock) return fail(RTP_ERR_UNSUPPORTED, "%s: block size %d unsupported (must be 64)", who, block);
  if (R <= 0 || R > 65535) return fail(RTP_ERR_INVALID_ARG, "%s: R must be in [1, 65535]", who);
  if (max_len <= 0 || max_len > RTP_MAX_ROW_LEN)
    return fail(RTP_ERR_INVALID_ARG, "%s: max_len must be in [1, %d]", who, RTP_MAX_ROW_LEN);
  if (score_stride < max_len || (score_stride & 3) || ((uintptr_t)scores & 15))
    return fail(RTP_ERR_INVALID_ARG, "%s: scores must be 16-byte aligned, score_stride >= max_len and a multiple of 4", who);
  if (sel_stride < max_len) return fail(RTP_ERR_INVALID_ARG, "%s: sel_stride must be >= max_len", who);
  if (!(bin_width > 0.f) || !(bin_lo == bin_lo) || !(bin_width < 3.0e38f))
    return fail(RTP_ERR_INVALID_ARG, "%s: bin_width must be positive and finite, bin_lo a number", who);
  if (block_mask && mask_stride < (max_len + kBtBlock - 1) / kBtBlock)
    return fail(RTP_ERR_INVALID_ARG, "%s: mask_stride must cover ceil(max_len / 64) blocks", who);
  const BlockLayout l = block_layout(R, max_len);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < l.total)
    return fail(RTP_ERR_WORKSPACE, "%s: workspace of %zu bytes (256-byte aligned) required, got %zu", who, l.total, ws_bytes);
  clear_error();
  BlockTopPArgs a;
  a.scores = scores;
  a.score_stride = score_stride;
  a.row_len = row_len;
  a.p = p;
  a.R = R;
  a.n_chunks = (int32_t)((max_len + kBtChunk - 1) / kBtChunk);
  a.bin_lo = bin_lo;
  a.bin_width = bin_width;
  a.sel_idx = sel_idx;
  a.sel_stride = sel_stride;
  a.sel_count = sel_count;
  a.thr_out = threshold_bin;
  a.mass = mass;
  a.mask_out = block_mask;
  a.mask_stride = mask_stride;
  a.hist = (uint64_t*)((char*)ws + l.hist_off);
  a.block_bin = (uint8_t*)((char*)ws + l.bin_off);
  a.chunk_cnt = (int32_t*)((char*)ws + l.ccnt_off);
  a.state = (BlockRowState*)((char*)ws + l.state_off);
  hipStream_t s = (hipStream_t)stream;
  dim3 grid((unsigned)a.n_chunks, (unsigned)R), blk(kBtThreads);
  const int64_t nz = (int64_t)R * kBtBins;
  RTP_LAUNCH(block_zero_kernel, dim3((unsigned)((nz + kBtThreads - 1) / kBtThreads)), blk, 0, s, a.hist, nz);
  RTP_LAUNCH(block_stats_kernel, grid, blk, 0, s, a);
  RTP_LAUNCH(block_count_kernel, grid, blk, 0, s, a);
  RTP_LAUNCH(block_write_kernel, grid, blk, 0, s, a);
  return check_launch(who);
}
