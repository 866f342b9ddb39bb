/*
 * rtp.h -- C ABI of the RTPurbo sparse-attention hot path for AMD MI355X (gfx950).
 *
 * The library implements, for ONE attention layer on ONE GPU, the inference-time
 * attention rule of the paper's Section 3.2 ("Adaptive Sparse Attention Mechanism"):
 *
 *   retrieval heads   index score  s_h(m,n) = <W^Q_h q^pre_{m,h}, W^K_h k^pre_{n,h}>   (indexer equation)
 *                     active set   S_h(m)   = Top-P(s_h(m,.), p)                        (sparse-attention equation)
 *                     output       O_h(m)   = sum_{n in S} softmax_S(q.k_n/sqrt(d_h)) v_n
 *   local heads       attention over `sink` first tokens + the `window` most recent ones (Sec. 3.2, Sec. 4.2)
 *   dense comparison  causal softmax attention over every token (the paper's comparison system is
 *                     a dense flash-attention kernel, Sec. 4.2 "Runtime Analysis"; this one is in-house)
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every tensor pointer is a DEVICE pointer owned by the caller.  The library never allocates,
 *    frees, copies to the host or synchronises: all work is enqueued on `stream` (a hipStream_t
 *    passed as void*; NULL = the default stream) and the call returns at once.
 *  - `rtp_layer_desc` and its `ret_heads` array are HOST memory, read during the call only.
 *  - Scratch memory comes from the caller: `ws` (device, 256-byte aligned) of at least the size
 *    the matching *_workspace_bytes() function returns.  Contents are undefined before and after.
 *  - 16-bit tensors are raw bit patterns.  The attention tensors q, K, V and out are bf16, or fp16 (IEEE binary16)
 *    when the layer says kv_dtype = RTP_DTYPE_FP16; both are read exactly, accumulated in fp32 and the output is
 *    rounded once to the same type.  Everything on the indexer side (q_pre, k_pre, kI, qI) is bf16 either way.
 *    head_dim must be 128 and index_dim 16.
 *  - K and V caches: bf16, element (kvh, token, c) at  base[kvh * kv_head_stride + token * kv_row_stride + c],
 *    strides in ELEMENTS, kv_row_stride >= 128 and a multiple of 8 (256 with V = K + 128 gives
 *    interleaved K|V rows; the prefill calls also require kv_row_stride <= 2^24).  Sequences are packed along the token axis: sequence b owns tokens
 *    seq_start[b] .. seq_start[b] + ctx_len[b] - 1  (seq_start int64, ctx_len int32, both device).
 *  - Index-key cache kI = bf16(W^K_h k^pre): element (j, token, i) at kI[j * kI_head_stride + token * 16 + i],
 *    one stream per RETRIEVAL QUERY head j (j-th entry of ret_heads).
 *  - GQA: query head h reads KV head h / (n_q_heads / n_kv_heads).
 *  - Query positions: `q_start` (device int32 [B]) NULL means decode -- n_q must be 1 and the query of
 *    sequence b sits at position ctx_len[b] - 1 (the caller appends the new token's K/V/kI row first,
 *    so it is a candidate).  Otherwise query t of sequence b sits at position q_start[b] + t, sees
 *    tokens n <= q_start[b] + t (causal), and q_start[b] + n_q <= ctx_len[b] must hold.
 *  - Queries and outputs: bf16 [B, n_q, n_q_heads, 128].  Retrieval-head entry points write only the
 *    rows of retrieval heads, rtp_local_attn only the rows of the other heads, so the two may run
 *    concurrently on two streams.  `lse` (optional, fp32 [B, n_q, n_q_heads]) receives the natural-log
 *    sum of exponentials of the scaled logits over the attended set.
 *  - Return value: RTP_OK or a negative error code.  Every argument check happens on the host before
 *    the first launch; on error nothing has been enqueued.  rtp_last_error() gives a thread-local
 *    message for the last failing call of the calling thread.
 *  - Calls on different streams may overlap if their outputs and workspaces are disjoint.
 *  - Size limits of the decode calls (n_q = 1): rtp_local_attn, rtp_dense_attn, rtp_local_attn_ring and
 *    rtp_decode_attention serve at most 1024 (sequence, KV head) pairs per call (B * n_kv_heads <= 1024),
 *    rtp_sparse_attn_decode and its paged form at most 1024 (sequence, retrieval head) rows (B * n_ret <= 1024):
 *    RTP_ERR_UNSUPPORTED beyond that, before anything is enqueued -- split the batch.
 */
#ifndef RTP_H_
#define RTP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RTP_OK                 0
#define RTP_ERR_INVALID_ARG   (-1)   /* null pointer, non-positive size, bad head list, bad stride */
#define RTP_ERR_UNSUPPORTED   (-2)   /* head_dim != 128, index_dim != 16, group size not in {1,2,4,8} */
#define RTP_ERR_WORKSPACE     (-3)   /* workspace missing, misaligned or too small */
#define RTP_ERR_HIP           (-4)   /* a launch failed; the HIP error text is in rtp_last_error() */

#define RTP_DTYPE_BF16  0
#define RTP_DTYPE_FP16  1            /* IEEE binary16, the format the paper's decode kernel loads (Sec. 3.4) */

#define RTP_HEAD_DIM   128
#define RTP_INDEX_DIM  16
#define RTP_MAX_ROW_LEN (1 << 24)    /* longest score row rtp_topp_select accepts */

/* One attention layer (host struct).  Values used by the paper's configuration table:
 * index_dim 16, sink 4, window 8192, 15 % of the heads retrieval. */
typedef struct rtp_layer_desc {
  int32_t n_q_heads;         /* query heads                                   */
  int32_t n_kv_heads;        /* KV heads; n_q_heads / n_kv_heads in {1,2,4,8} */
  int32_t head_dim;          /* 128                                           */
  int32_t index_dim;         /* 16                                            */
  int32_t n_ret;             /* number of retrieval query heads (may be 0)    */
  const int32_t* ret_heads;  /* HOST, strictly ascending query-head ids       */
  int32_t sink;              /* local heads: first `sink` tokens ...          */
  int32_t window;            /* ... plus the `window` most recent, own position included */
  float softmax_scale;       /* 0 => 1/sqrt(head_dim)   (sparse-attention equation) */
  float index_scale;         /* 0 => 1                  (the indexer equation has no scale) */
  int32_t kv_dtype;          /* element type of q, K, V and out: RTP_DTYPE_BF16 (0, default) or RTP_DTYPE_FP16 */
} rtp_layer_desc;

/* Message for the last error on this thread ("" if none).  Never NULL. */
const char* rtp_last_error(void);
/* Library version, e.g. "rtp-gfx950 0.1". */
const char* rtp_version(void);

/* ---------------------------------------------------------------------------------------------
 * (1) Indexer score pass -- Sec. 3.2, indexer equation.
 *
 * For every row (b, j, t) -- sequence b, j-th retrieval head, query t -- and every cached token n of
 * sequence b:   scores[row * score_stride + n] = index_scale * sum_{i<16} qI[i] * kI[j, seq_start[b]+n, i]
 * accumulated in fp32 (the bf16*bf16 products are exact), row = (b * n_ret + j) * n_q + t.
 * Non-candidates (n > query position) inside [0, ctx_len[b]) are written as -inf; entries at
 * n >= ctx_len[b] are not written.
 *
 * The index query: if WQ != NULL, q_in is the PRE-RoPE query tensor bf16 [B, n_q, n_q_heads, 128] and
 * qI = bf16_rne( WQ[j] . q_in[b, t, ret_heads[j], :] ) with WQ fp32 [n_ret, 16, 128]; the 128-term sum
 * runs in fp64 and is rounded to bf16 once.  If WQ == NULL, q_in already holds qI, bf16 [B, n_ret, n_q, 16].
 * qI_out (optional, bf16 [B, n_ret, n_q, 16]) receives the index queries used.
 *
 * max_ctx: host upper bound of ctx_len[] (sizes the grid).  score_stride >= max_ctx, multiple of 4;
 * `scores` 16-byte aligned.
 *
 * topp_ws (optional): the workspace of the rtp_topp_select call that will consume these scores, sized
 * by rtp_topp_workspace_bytes(B * n_ret * n_q, max_ctx) and INITIALISED (rtp_topp_workspace_init once
 * after allocation; rtp_topp_select with level1_ready = 1 leaves it initialised again).  When given,
 * the score pass also accumulates the first level of the selector's mass histogram while the scores
 * are in registers, and the following rtp_topp_select(..., level1_ready = 1, same workspace, row_len =
 * ctx_len of each row, max_len = max_ctx) skips its first two launches.
 */
int32_t rtp_index_score(const rtp_layer_desc* layer, const void* q_in, const float* WQ,
                        const void* kI, int64_t kI_head_stride,
                        const int64_t* seq_start, const int32_t* ctx_len, const int32_t* q_start,
                        int32_t B, int32_t n_q, int64_t max_ctx,
                        float* scores, int64_t score_stride, void* qI_out,
                        void* topp_ws, size_t topp_ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * (2) Dynamic top-p selection -- Sec. 3.2 (S = Top-P(s, p)) and Sec. 3.4 (the threshold is found
 * without sorting, as the score where the descending cumulative softmax mass first reaches p).
 *
 * For each of R independent rows: w_n = exp(s_n - max_n s_n), Z = sum w_n; the selected set is
 * { n : s_n >= tau } where tau is the largest score whose descending cumulative mass reaches p * Z.
 * This is the smallest such set up to ties AT tau, all of which are kept.  The search is a three-level
 * radix histogram over the order-preserving 32-bit key of the fp32 score (exact: no sort, no sampling);
 * masses are accumulated as 64-bit fixed point of fp64 exponentials, so the result does not depend on
 * summation order.  The fixed-point reference of a score is the upper edge of its quarter binade, at most 16
 * away while |s| < 128 (a weight then keeps a relative resolution of 2^-8 or far better for the longest row);
 * a row whose LARGEST finite score lies outside (-128, 128) cannot be resolved that way and is reported as
 * unsupported: sel_count = -2, nothing selected (lower scores of any magnitude are fine).
 *
 *   scores    fp32 [R, score_stride] (16-byte aligned, score_stride multiple of 4); row r uses
 *             entries [0, row_len[r]); -inf entries are never selected.
 *   row_len   device int32 [R], each <= max_len (host bound, <= RTP_MAX_ROW_LEN).
 *   p         device fp32 [R], one value per row; p >= 1 keeps every entry of the row (tau = -inf);
 *             p <= 0 or NaN marks the row invalid: sel_count = -1, nothing selected.
 *             (sel_count = -2: the row's largest score lies outside (-128, 128), see above.)
 *   sel_idx   out, int32 [R, sel_stride], sel_stride >= max_len; the selected positions in
 *             ascending order (the result is deterministic: same inputs, same bits).
 *   sel_count out, int32 [R].   tau, mass: optional outputs fp32 [R] (threshold score; selected mass / Z).
 *   level1_ready  0: the call is self-contained and the workspace contents do not matter.
 *             1: rtp_index_score has accumulated the first histogram level into this (initialised)
 *             workspace; the call starts at level 2 and leaves the workspace initialised for the next step.
 */
size_t rtp_topp_workspace_bytes(int32_t R, int64_t max_len);
/* Zero-fills a top-p workspace (needed once before it is first handed to rtp_index_score). */
int32_t rtp_topp_workspace_init(void* ws, size_t ws_bytes, void* stream);
int32_t rtp_topp_select(const float* scores, int64_t score_stride, const int32_t* row_len,
                        const float* p, int32_t R, int64_t max_len,
                        int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                        float* tau, float* mass, int32_t level1_ready,
                        void* ws, size_t ws_bytes, void* stream);

/* rtp_topp_select for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation): the same kernels, results and argument
 * rules as rtp_topp_select(..., level1_ready = 0, ...), with the scratch in a buffer built into the library
 * (RTP_TOPP_NOALLOC_WS_BYTES of device memory per GPU, held until the process ends).  The call allocates
 * nothing and records kernel launches only.  Shapes whose scratch, rtp_topp_workspace_bytes(R, max_len), exceeds
 * the buffer are refused with RTP_ERR_WORKSPACE before anything is enqueued (32 rows of 131072 scores need
 * 1.5 MiB, 64 rows 3.0 MiB, 8 rows of 1048576 scores 0.5 MiB).  Every call on a GPU uses that GPU's one buffer:
 * calls that overlap in time on the same GPU (different streams or threads) race; calls on one stream are fine.
 */
#define RTP_TOPP_NOALLOC_WS_BYTES (4u << 20)
int32_t rtp_topp_select_noalloc(const float* scores, int64_t score_stride, const int32_t* row_len,
                                const float* p, int32_t R, int64_t max_len,
                                int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                float* tau, float* mass, void* stream);

/* ---------------------------------------------------------------------------------------------
 * (3) Exact softmax attention over the selected tokens, decode, retrieval heads only --
 * Sec. 3.2, sparse-attention equation.
 *
 * Row (b, j) attends query q[b, 0, ret_heads[j], :] to tokens sel_idx[(b*n_ret+j)*sel_stride + i],
 * i < sel_count[b*n_ret+j] (positions relative to seq_start[b]), of KV head kv(ret_heads[j]), and
 * writes out[b, 0, ret_heads[j], :].  Rows with sel_count <= 0 write zeros (lse = -inf).
 * max_sel: host upper bound of sel_count[] (sizes the grid and the workspace).
 */
size_t rtp_sparse_attn_decode_workspace_bytes(const rtp_layer_desc* layer, int32_t B, int64_t max_sel);
int32_t rtp_sparse_attn_decode(const rtp_layer_desc* layer, const void* q,
                               const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                               const int64_t* seq_start,
                               const int32_t* sel_idx, int64_t sel_stride, const int32_t* sel_count,
                               int64_t max_sel, int32_t B, void* out, float* lse,
                               void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * (4) Causal prefill chunk for the retrieval heads of ONE sequence: index score + per-query top-p +
 * attention over each query's own active set, fused (no T x N score matrix is materialised).
 * The paper runs retrieval heads dense in prefill (Sec. 3.2, Sec. 4.2) -- that is p >= 1 here; p < 1
 * applies its decode rule (Top-P over the causal candidates n <= m) to every prefill query.
 *
 * Pointers K, V, kI address token 0 of the sequence.  Queries t = 0..T-1 sit at positions
 * chunk_start + t; rows [0, chunk_start + T) of K/V/kI must exist.  q: bf16 [T, n_q_heads, 128]
 * (post-RoPE).  Index queries as in (1): WQ != NULL => q_pre bf16 [T, n_q_heads, 128], else q_pre holds
 * qI bf16 [n_ret, T, 16].  out: bf16 [T, n_q_heads, 128], retrieval rows only.
 * Optional per-(j, t) statistics, fp32/int32 [n_ret, T]: tau (threshold used), count (tokens kept),
 * mass (indexer mass kept).  For p < 1 the threshold search works on floor((ref - s) * 2^17), ref = the row
 * maximum, so the kept set is the exact top-p set plus any token whose score lies within 2^-17 (7.6e-6) below
 * its threshold.  One pass resolves the 15.875 score units below its reference; a threshold deeper than that
 * (p within ~1e-5 of 1 on a peaked row) makes the search lower the reference and repeat, so the resolution is the
 * same at any depth.  Masses are fp32 exponentials (relative error up to 2^-22) summed in fp64: where single
 * tokens weigh less than 3e-7 of a row's mass, the kept count can differ from the fp64 count by the tokens
 * inside that margin.
 * For p < 1 the attention visits only the 64-key tiles in which some query of a 256-query tile can keep a key (the
 * search leaves, per 32-query group and tile, whether a product reaches the group's thresholds); outputs, counts and
 * sums are those of visiting every tile.  The workspace holds that table (4 B per group and 64 keys of context),
 * the tile lists and the key-range partials: about 630 MB for T = 8192 at chunk_start = 1,040,384 with 4
 * retrieval heads, 40 MB for T = 4096 at 126,976.
 */
size_t rtp_sparse_attn_prefill_workspace_bytes(const rtp_layer_desc* layer, int32_t T, int64_t chunk_start);
int32_t rtp_sparse_attn_prefill(const rtp_layer_desc* layer, const void* q_pre, const void* q, const float* WQ,
                                const void* kI, int64_t kI_head_stride,
                                const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                                int64_t chunk_start, int32_t T, float p, void* out, float* lse,
                                float* tau, int32_t* count, float* mass,
                                void* ws, size_t ws_bytes, void* stream);

/*
 * How much of the causal key range the last rtp_sparse_attn_prefill call with p < 1 on this workspace visited
 * (a measurement aid for the block-sparse prefill discussion of Sec. 3.4: the threshold search records the largest
 * index score of every 32-query group in every 64-key tile, and the attention launch visits a tile only if some
 * query of its 256-query tile can keep a key there).  layer, T and chunk_start as in that call; waits for `stream`,
 * then writes two host values: tiles_visited (64-key tiles visited, summed over retrieval heads and 256-query
 * tiles) and tiles_causal (what plain causal attention visits).  Allocates nothing on the device.
 */
int32_t rtp_sparse_attn_prefill_tile_stats(const rtp_layer_desc* layer, int32_t T, int64_t chunk_start,
                                           const void* ws, size_t ws_bytes, void* stream,
                                           int64_t* tiles_visited, int64_t* tiles_causal);

/* ---------------------------------------------------------------------------------------------
 * (5) Sink + sliding-window attention for every NON-retrieval head -- Sec. 3.2 (first sentence),
 * Sec. 4.2 (the evaluated setting: sink = 4, window = 8192).
 *
 * A query at position m attends tokens { n < sink } U { max(sink, m - window + 1) <= n <= m }.
 * Decode (q_start == NULL, n_q == 1) reads each needed K/V row once per KV head and serves the whole
 * GQA group from it; prefill (q_start != NULL) runs banded causal MFMA tiles.
 * max_ctx: host upper bound of ctx_len[].
 */
size_t rtp_local_attn_workspace_bytes(const rtp_layer_desc* layer, int32_t B, int32_t n_q, int64_t max_ctx);
int32_t rtp_local_attn(const rtp_layer_desc* layer, const void* q,
                       const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                       const int64_t* seq_start, const int32_t* ctx_len, const int32_t* q_start,
                       int32_t B, int32_t n_q, int64_t max_ctx, void* out, float* lse,
                       void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * In-house dense comparison: causal softmax attention over ALL tokens for ALL heads (same tensors,
 * same conventions as (5)).  Stands in for the dense flash-attention baseline of Sec. 4.2.
 */
size_t rtp_dense_attn_workspace_bytes(const rtp_layer_desc* layer, int32_t B, int32_t n_q, int64_t max_ctx);
int32_t rtp_dense_attn(const rtp_layer_desc* layer, const void* q,
                       const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                       const int64_t* seq_start, const int32_t* ctx_len, const int32_t* q_start,
                       int32_t B, int32_t n_q, int64_t max_ctx, void* out, float* lse,
                       void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Per-kernel timing for measurements (the paper reports run time per attention layer, Sec. 4.2 "Runtime
 * Analysis"; a per-kernel split needs clocks between the launches of one call).  Between rtp_profile_start and
 * rtp_profile_stop every kernel launch of the library, from any thread of the process, carries a start and a stop
 * event stamped with the dispatch's own begin and end times (at most max_launches launches are recorded, further
 * ones pass untimed).
 * rtp_profile_stop waits for the recorded launches, writes up to out_cap (kernel name, microseconds) pairs in
 * launch order and *n_out, and releases the events.  The names are static strings of the library.  Recording
 * serialises nothing; do not record inside a stream capture.
 */
typedef struct {
  const char* kernel;
  float us;
} rtp_launch_time;
/* Measurement only: rtp_index_score's launch (same grid, same loads of the index keys, same stores) with the
 * arithmetic taken out -- `scores` receives meaningless words.  Its duration is what the chip sustains for the
 * score pass's traffic mix (32 bytes read for every 4 written), the ceiling the real pass is priced against. */
int32_t rtp_index_score_traffic_probe(const rtp_layer_desc* layer, const void* q_in, const float* WQ,
                                      const void* kI, int64_t kI_head_stride,
                                      const int64_t* seq_start, const int32_t* ctx_len, const int32_t* q_start,
                                      int32_t B, int32_t n_q, int64_t max_ctx,
                                      float* scores, int64_t score_stride, void* stream);
int32_t rtp_profile_start(int32_t max_launches);
int32_t rtp_profile_stop(rtp_launch_time* out, int32_t out_cap, int32_t* n_out);

/* =============================================================================================
 * Entry points beside the five above: the index-key build, the two other selectors the paper
 * discusses, and its sparsity figures.
 * ============================================================================================= */

/* ---------------------------------------------------------------------------------------------
 * Indexer projections -- Sec. 3.2, indexer equation: kI = bf16(W^K_h k^pre), qI = bf16(W^Q_h q^pre).
 *
 * For the j-th retrieval query head h_j and token t < T:
 *   xI_out[j * out_head_stride + (out_t0 + t) * 16 + i] = bf16_rne( sum_c W[j, i, c] * x_pre[t, xh(j), c] ),  i < 16,
 * the 128-term sum in fp64, rounded once.  W: fp32 [n_ret, 16, 128].  side = RTP_SIDE_KEY: x_pre is the
 * PRE-rotary key tensor bf16 [T, n_kv_heads, 128] and xh(j) = kv(h_j) -- the call that appends T tokens to
 * the index-key cache at token offset out_t0 (out_head_stride = the cache's kI_head_stride).
 * side = RTP_SIDE_QUERY: x_pre is the pre-rotary query tensor bf16 [T, n_q_heads, 128] and xh(j) = h_j.
 * x_pre 16-byte aligned, xI_out 8-byte aligned, out_head_stride a multiple of 4.  No workspace.
 */
#define RTP_SIDE_QUERY 0
#define RTP_SIDE_KEY   1
int32_t rtp_index_project(const rtp_layer_desc* layer, const float* W, const void* x_pre, int32_t side,
                          int32_t T, void* xI_out, int64_t out_head_stride, int64_t out_t0, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Static top-k selection -- the fixed-budget rule the paper compares its dynamic top-p against
 * (Sec. 2.3, top-k / top-p table; Sec. 4.1 "Baselines", k = 4096).
 *
 * Row r keeps its k[r] highest scores (k: device int32 [R]); all scores tied with the k-th are kept, so
 * sel_count can exceed k[r] by the ties; a budget that covers every finite score keeps them all;
 * k[r] <= 0 marks the row invalid (sel_count = -1).  Same radix search, tensors, ordering (ascending
 * positions, deterministic) and workspace (rtp_topp_workspace_bytes) as rtp_topp_select, with counts in
 * place of masses.  tau (optional): the k-th best score.
 */
int32_t rtp_topk_select(const float* scores, int64_t score_stride, const int32_t* row_len,
                        const int32_t* k, int32_t R, int64_t max_len,
                        int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count, float* tau,
                        void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Block-wise top-p selection -- Sec. 3.4, "Sort-free top-p via histogram" (block size 64 in the
 * paper's configuration table).
 *
 * Row r is cut into blocks of `block` (= 64) consecutive scores.  Block b has the log-sum-exp pair
 * m_b = max s, l_b = sum exp(s - m_b) and deposits the mass l_b * exp(m_b) into bin
 * clamp(floor((m_b - bin_lo) / bin_width), 0, 255) of a 256-bin histogram.  The histogram is scanned from
 * the highest bin down; the threshold bin is the first at which the cumulative mass reaches p[r] times the
 * total; every block whose bin is at or above it is kept WHOLE -- the kept mass overshoots p by up to the
 * mass of the threshold bin (the price of the one-pass, sort-free search; rtp_topp_select is the
 * token-exact selector).  The paper gives neither the bin mapping nor the scale of the deposits; uniform
 * bins over a caller-chosen range and exact integer deposits are this library's reading.  Scores above
 * bin_lo + 256 * bin_width count with the mass of that upper edge: choose a range that covers the scores.
 * p >= 1 keeps every block; p <= 0 or NaN: sel_count = -1.
 *
 *   sel_idx / sel_count  the tokens of the kept blocks, ascending (what rtp_sparse_attn_decode reads).
 *   threshold_bin (optional int32 [R]), mass (optional fp32 [R]: kept mass / total),
 *   block_mask (optional uint8 [R, mask_stride], 1 = kept, mask_stride >= ceil(max_len / 64)).
 */
size_t rtp_block_topp_workspace_bytes(int32_t R, int64_t max_len);
int32_t rtp_block_topp_select(const float* scores, int64_t score_stride, const int32_t* row_len,
                              const float* p, int32_t R, int64_t max_len,
                              int32_t block, float bin_lo, float bin_width,
                              int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                              int32_t* threshold_bin, float* mass, uint8_t* block_mask, int64_t mask_stride,
                              void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Sparsity figures of one decode step -- Sec. 3.2 (last paragraph: compute vs memory sparsity under
 * GQA), Sec. 4.2 ("Sparsity Analysis" and its table).
 *
 * stats[b] = { compute sparsity, memory sparsity, active tokens, attention mass } (fp32 [B, 4]):
 *   compute sparsity = 1 - (mean over query heads of attended tokens) / ctx_len[b], a local head attending
 *                      its sink + window set, a retrieval head its selected list;
 *   memory sparsity  = 1 - (mean over KV heads of the size of the union of its query heads' sets) / ctx_len[b];
 *   active tokens    = mean sel_count over the retrieval heads;
 *   attention mass   = mean over the retrieval heads of exp(lse_selected - lse_full): the probability the
 *                      full softmax attention puts on the selected set.  lse_selected / lse_full are the
 *                      lse outputs (fp32 [B, n_q_heads], n_q = 1) of rtp_sparse_attn_decode and
 *                      rtp_dense_attn; pass both or neither (NaN then).
 * sel_idx rows must be ascending (every selector of this library writes them so).
 * union_size (optional int32 [B, n_kv_heads]): the union sizes themselves.
 */
int32_t rtp_sparsity_stats(const rtp_layer_desc* layer, const int32_t* ctx_len,
                           const int32_t* sel_idx, int64_t sel_stride, const int32_t* sel_count,
                           const float* lse_selected, const float* lse_full, int32_t B,
                           float* stats, int32_t* union_size, void* stream);

/* ---------------------------------------------------------------------------------------------
 * (3) with the retrieval heads' cache held in pages (a storage layout; the arithmetic is the
 * sparse-attention equation of Sec. 3.2 unchanged).
 *
 * K and V are pools of rows shared by all sequences: token position t of sequence b lives in pool row
 * page_table[b * pt_stride + t / page_size] * page_size + t % page_size, element (kvh, row, c) at
 * base[kvh * kv_head_stride + row * kv_row_stride + c].  page_table: device int32; page_size: a power
 * of two >= 16; pt_stride >= ceil(max_sel / page_size).  Everything else as in rtp_sparse_attn_decode
 * (same workspace size, same plan, bit-identical results for the same rows).  The bounded cache of the
 * all-local KV heads (rtp_kv_ring_*) needs no paging; local heads that share their KV head with a
 * retrieval head are not covered by this entry point.
 */
int32_t rtp_sparse_attn_decode_paged(const rtp_layer_desc* layer, const void* q,
                                     const void* K, const void* V, int64_t kv_row_stride,
                                     int64_t kv_head_stride, const int32_t* page_table, int64_t pt_stride,
                                     int32_t page_size,
                                     const int32_t* sel_idx, int64_t sel_stride, const int32_t* sel_count,
                                     int64_t max_sel, int32_t B, void* out, float* lse,
                                     void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * (2) + (3) in one call for a decode step -- Sec. 3.2 (S = Top-P(s, p), then exact softmax attention
 * over S).  Sec. 3.4 saves a launch per step by fusing neighbouring stages (there: scoring and selection);
 * the pair fused here is the last selection launch and the attention.
 *
 * The results are those of rtp_topp_select followed by rtp_sparse_attn_decode on the same tensors
 * (sel_idx, sel_count, tau, mass bit-identical; out and lse equal up to the order of the fp32 partial
 * sums), with one launch and one pass over the index list less: the launch that writes the ordered
 * positions of a chunk of the row (8192 scores) keeps them in LDS, gathers their K/V rows and leaves a partial softmax
 * state per (row, chunk); a merge launch finishes each row.
 * The gather is thereby split by score chunk, which is even as far as the kept tokens are spread over the
 * context.  A row with one overfull chunk (more than 1.25 x the mean + 256 kept tokens) is shared out
 * differently: every workgroup of the row takes an equal share of the row's ranks -- weighed with the cost
 * of repeating a chunk's compaction -- and finds the positions in whichever chunks hold them.
 *
 * Rows are the retrieval heads of the batch: row r = b * n_ret + j scores the cached tokens of sequence b
 * for head ret_heads[j] (the layout rtp_index_score writes with n_q = 1), R = B * n_ret rows.
 *   scores, score_stride, row_len, p, sel_idx, sel_stride, sel_count, tau, mass, level1_ready, topp_ws:
 *             as in rtp_topp_select with R = B * n_ret and max_len = max_ctx.
 *   q, K, V, kv_row_stride, kv_head_stride, seq_start, out, lse: as in rtp_sparse_attn_decode.
 *   attn_ws   rtp_select_attend_decode_workspace_bytes(layer, B, max_ctx) bytes, 256-byte aligned.
 * Rows that select nothing (invalid p, no finite score, row_len <= 0) write zeros and lse = -inf.
 */
size_t rtp_select_attend_decode_workspace_bytes(const rtp_layer_desc* layer, int32_t B, int64_t max_ctx);
int32_t rtp_select_attend_decode(const rtp_layer_desc* layer, const float* scores, int64_t score_stride,
                                 const int32_t* row_len, const float* p, int32_t B, int64_t max_ctx,
                                 const void* q, const void* K, const void* V, int64_t kv_row_stride,
                                 int64_t kv_head_stride, const int64_t* seq_start,
                                 int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                 float* tau, float* mass, int32_t level1_ready, void* out, float* lse,
                                 void* topp_ws, size_t topp_ws_bytes, void* attn_ws, size_t attn_ws_bytes,
                                 void* stream);

/* ---------------------------------------------------------------------------------------------
 * (2) + (3) + (4) in one call for a decode step: everything after the score pass -- Sec. 3.2 (Top-P
 * selection, attention of the retrieval heads over the selected tokens, sink + window attention of the
 * other heads).
 *
 * The results are those of rtp_select_attend_decode followed by rtp_local_attn (n_q = 1) on the same
 * tensors.  With 2 or 4 query heads per KV head (and with 8 while the batch is small enough for one work
 * item per carrying workgroup) the local heads' work items are carried by the selector's second launch,
 * which is latency-bound and leaves HBM idle: one stream, no fork and join, four launches after the score
 * pass.  Otherwise the two parts run one after the other.
 *
 *   ctx_len   device int32 [B]: cached tokens per sequence (row_len[b * n_ret + j] must equal ctx_len[b]).
 *   local_ws  rtp_local_attn_workspace_bytes(layer, B, 1, max_ctx) bytes, 256-byte aligned.
 *   every other argument as in rtp_select_attend_decode.
 */
int32_t rtp_decode_attention(const rtp_layer_desc* layer, const float* scores, int64_t score_stride,
                             const int32_t* row_len, const float* p, const int32_t* ctx_len, int32_t B,
                             int64_t max_ctx, const void* q, const void* K, const void* V,
                             int64_t kv_row_stride, int64_t kv_head_stride, const int64_t* seq_start,
                             int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                             float* tau, float* mass, int32_t level1_ready, void* out, float* lse,
                             void* topp_ws, size_t topp_ws_bytes, void* attn_ws, size_t attn_ws_bytes,
                             void* local_ws, size_t local_ws_bytes, void* stream);

/* rtp_decode_attention with the whole K/V cache held in pages (a storage layout; the arithmetic is that of
 * Sec. 3.2 unchanged -- Sec. 2.1: the retrieval heads keep the full cache, which is the one a server pages).
 * K and V address pools [n_kv_heads, pool rows, 128]; token t of sequence b lives in pool row
 * page_table[b * pt_stride + t / page_size] * page_size + t % page_size for every KV head (page_table device int32,
 * page_size a power of two in [16, 2^20], pt_stride >= ceil(max_ctx / page_size)).  Both the gathered rows of the
 * retrieval heads and the sink + window rows of the local heads are read through the table; selections and
 * outputs are bit-identical to rtp_decode_attention on the same tokens laid out contiguously.
 */
int32_t rtp_decode_attention_paged(const rtp_layer_desc* layer, const float* scores, int64_t score_stride,
                                   const int32_t* row_len, const float* p, const int32_t* ctx_len, int32_t B,
                                   int64_t max_ctx, const void* q, const void* K, const void* V,
                                   int64_t kv_row_stride, int64_t kv_head_stride,
                                   const int32_t* page_table, int64_t pt_stride, int32_t page_size,
                                   int32_t* sel_idx, int64_t sel_stride, int32_t* sel_count,
                                   float* tau, float* mass, int32_t level1_ready, void* out, float* lse,
                                   void* topp_ws, size_t topp_ws_bytes, void* attn_ws, size_t attn_ws_bytes,
                                   void* local_ws, size_t local_ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Bounded KV cache of the all-local KV heads, decode -- Sec. 2.1 (the full KV cache is kept for
 * retrieval heads only, the other heads drop remote tokens) and Sec. 3.2, last paragraph (memory is
 * counted per KV head: under GQA a KV head can drop them when EVERY query head mapped to it is local).
 *
 * Such a KV head keeps cap = sink + window rows per sequence.  Layout (this library's; the paper gives
 * none): row i < sink holds token i; token t >= sink lives in row sink + (t - sink) mod window.  Row s of
 * bounded head i (the i-th all-local KV head in ascending order) of sequence b is at
 * ring_K + i * ring_head_stride + (ring_seq_start[b] + s) * ring_row_stride (bf16, 16-byte aligned,
 * ring_row_stride >= 128 and a multiple of 8; ring_seq_start: device int64 [B]); ring_V likewise.
 *
 *   rtp_kv_ring_heads   host helper: the all-local KV heads (kv_heads: host int32 [n_kv_heads] or NULL);
 *                       returns their number, -1 on a bad descriptor.
 *   rtp_kv_ring_append  stores the new token of every sequence: k_new, v_new bf16 [B, n_kv_heads, 128]
 *                       (post-rotary), pos device int32 [B] = its position (pos < 0: sequence skipped).
 *   rtp_kv_ring_fill    hand-over after prefill: copies from the full cache (layout of rtp_local_attn)
 *                       the rows that are inside the bounded cache after ctx_len[b] tokens.
 *   rtp_local_attn_ring rtp_local_attn for n_q = 1 with the bounded cache as the source of the all-local
 *                       KV heads: they attend the first min(ctx_len, cap) rows as they lie (a softmax over a
 *                       set does not depend on the order of its members).  Local heads that share their KV
 *                       head with a retrieval head still read K, V (the full cache, whose rows for the
 *                       bounded heads are never touched and need not be backed by memory).
 *                       Workspace: rtp_local_attn_ring_workspace_bytes(layer, B, max_ctx).
 */
int32_t rtp_kv_ring_heads(const rtp_layer_desc* layer, int32_t* kv_heads);
int32_t rtp_kv_ring_append(const rtp_layer_desc* layer, const void* k_new, const void* v_new,
                           const int32_t* pos, int32_t B, void* ring_K, void* ring_V,
                           int64_t ring_row_stride, int64_t ring_head_stride,
                           const int64_t* ring_seq_start, void* stream);
int32_t rtp_kv_ring_fill(const rtp_layer_desc* layer, const void* K, const void* V, int64_t kv_row_stride,
                         int64_t kv_head_stride, const int64_t* seq_start, const int32_t* ctx_len, int32_t B,
                         void* ring_K, void* ring_V, int64_t ring_row_stride, int64_t ring_head_stride,
                         const int64_t* ring_seq_start, void* stream);
size_t rtp_local_attn_ring_workspace_bytes(const rtp_layer_desc* layer, int32_t B, int64_t max_ctx);
int32_t rtp_local_attn_ring(const rtp_layer_desc* layer, const void* q,
                            const void* K, const void* V, int64_t kv_row_stride, int64_t kv_head_stride,
                            const int64_t* seq_start,
                            const void* ring_K, const void* ring_V, int64_t ring_row_stride,
                            int64_t ring_head_stride, const int64_t* ring_seq_start,
                            const int32_t* ctx_len, int32_t B, int64_t max_ctx, void* out, float* lse,
                            void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RTP_H_ */
