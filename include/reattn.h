/*
 * libreattn -- ReAttention's per-layer attention hot path on AMD MI355X (gfx950).
 *
 * C ABI.  Every call takes a host pointer to a plain `reattn_params` and raw
 * DEVICE pointers for tensors; nothing is allocated, freed or retained by the
 * library, and no call synchronises: work is enqueued on `stream` (a
 * hipStream_t passed as void*; NULL is the default stream) and the call returns.
 * Return value: REATTN_OK or a negative reattn_status.  All argument errors are
 * detected on the host before anything is launched; REATTN_ERR_HIP reports a
 * failed launch.  q, k_cache and v_cache are never written: the cache stays
 * free of positional encoding (paper, Method, "Training-Free Integration").
 *
 * Notation (paper Eq. 1-3): Hq query heads, Hkv KV heads, G = Hq/Hkv, D head
 * dimension, N cached tokens INCLUDING the M current ones as the last M rows
 * (the appendix pseudocode appends before it selects), s = n_sink = l_global,
 * l = n_local = l_local.  Clamped partition (Eq. 1):
 *     s_eff = min(s, N), l_eff = min(l, N - s_eff), N_mid = N - s_eff - l_eff,
 *     k_eff = min(top_k, N_mid), S = s_eff + k_eff + l_eff   ("scope").
 * sink = [0, s_eff), middle = [s_eff, N - l_eff), local = [N - l_eff, N).
 *
 * Layouts (row-major, contiguous innermost D):
 *     q        [M][Hq][D]        storage dtype (fp32, bf16 or fp16), WITHOUT rotary encoding
 *     k_cache  [Hkv][N][D]       storage dtype, WITHOUT rotary encoding; strides in params
 *     v_cache  [Hkv][N][D]       storage dtype; strides in params
 *     scores   [M][Hkv][N_mid]   fp32
 *     idx      [M][Hkv][k_eff]   int32, ABSOLUTE cache positions, strictly ascending
 *     k_sel    [M][Hkv][S][D]    fp32, rotary-encoded at re-assigned position r = 0..S-1
 *     v_sel    [M][Hkv][S][D]    storage dtype (copied rows)
 *     out      [M][Hq][D]        fp32
 * Query i is cache token N - M + i; for M > 1 it sees the local part only up to
 * its own token (causal), and M <= l is required (a chunk lies inside the local
 * window: paper, hyper-parameter discussion of the chunk size) unless the middle is
 * empty: then the kept entries are all N tokens in order and any M <= N is plain
 * causal attention (the first prefill chunk of l_global + l_local tokens).
 */
#ifndef REATTN_H_
#define REATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  REATTN_OK = 0,
  REATTN_ERR_NULL = -1,      /* a required pointer is NULL */
  REATTN_ERR_SHAPE = -2,     /* heads / head_dim / strides not supported */
  REATTN_ERR_DTYPE = -3,     /* unknown storage dtype or aggregation */
  REATTN_ERR_RANGE = -4,     /* n_ctx, n_query, n_sink, n_local or top_k out of range */
  REATTN_ERR_WINDOW = -5,    /* scope S exceeds max_position */
  REATTN_ERR_WORKSPACE = -6, /* ws is NULL or smaller than reattn_workspace_bytes() */
  REATTN_ERR_ALIGN = -7,     /* a pointer or stride breaks the 16-byte row alignment */
  REATTN_ERR_HIP = -8,       /* the HIP runtime refused a launch */
  REATTN_ERR_STATIC_LIMIT = -9 /* reattn_decode_step_static: the step needs more than REATTN_STATIC_SCRATCH_BYTES */
} reattn_status;

/* Storage of q, k_cache, v_cache, v_sel.  All arithmetic is fp32 on exactly widened inputs (the
 * matrix-core paths split what they must round into hi + lo halves).  REATTN_F16 (IEEE half, the
 * precision of the paper's own runs) takes the same kernels as bf16: the streaming kernels of a decode
 * step, the matrix cores (f16 MFMA instructions) for chunks and for the vote selection. */
typedef enum { REATTN_F32 = 0, REATTN_BF16 = 1, REATTN_F16 = 2 } reattn_dtype;

/* How the G heads of one GQA group are combined into one score per KV head (paper Eq. 2 scores one head;
 * the paper's own way of combining heads, votes over per-head lists, is the reattn_vote_* family below, which
 * ignores this field).  REATTN_AGG_SUM: sum_g q_g . k, every path.  REATTN_AGG_MAX: max_g q_g . k; the scores
 * are then formed by the streaming scan for every M (the matrix-core contraction and the filter route score
 * group sums and are not taken), everything behind the scores is the same. */
typedef enum { REATTN_AGG_SUM = 0, REATTN_AGG_MAX = 1 } reattn_agg;

typedef struct reattn_params {
  int32_t n_q_heads;    /* Hq, multiple of n_kv_heads, G <= 16 */
  int32_t n_kv_heads;   /* Hkv */
  int32_t head_dim;     /* D: 64 or 128 */
  int32_t dtype;        /* reattn_dtype of q, k_cache, v_cache, v_sel */
  int64_t n_ctx;        /* N >= 1 (and N - 1 must fit int32 indices) */
  int32_t n_query;      /* M >= 1; M == 1 is a decode step; M <= n_local, M <= N */
  int32_t n_sink;       /* s >= 0 */
  int32_t n_local;      /* l >= 1 */
  int32_t top_k;        /* k >= 0; clamped to N_mid */
  float   rope_theta;   /* rotary base (> 1), e.g. 10000 or 500000 */
  int32_t max_position; /* S must not exceed it; 0 disables the check */
  int32_t agg;          /* reattn_agg */
  float   softmax_scale;/* 0 selects 1/sqrt(D) */
  int64_t k_stride_head, k_stride_tok; /* in elements; 0,0 means contiguous [Hkv][N][D] */
  int64_t v_stride_head, v_stride_tok;
  /* Paged cache (NULL / 0: none).  k_cache and v_cache are then pools [Hkv][P * page_size][D] of P pages
   * per head, and token t of the sequence sits in row page_table[t / page_size] * page_size + t % page_size
   * of every head's slice.  page_table is a DEVICE array of ceil(N / page_size) int32 page numbers in
   * [0, P); the library cannot read it on the host, so entries outside the pool are the caller's fault.
   * page_size is a power of two >= 64; the four strides must be given (stride_head >= P * page_size * D).
   * Every call that reads or writes a cache takes paged params (decode steps and chunks of both selections,
   * the chunk loop, the decode token, reattn_cache_append).  Indices (idx, sel, head_topk) stay token
   * positions of the sequence. */
  const int32_t* page_table;
  int32_t page_size;
  /* Which way a decode step (M == 1) over a middle of more than 65,536 tokens finds its top-k (Eq. 2); the
   * results are the same either way.  REATTN_ROUTE_SCORES: the scan writes one fp32 score per key, a radix
   * select runs over them.  REATTN_ROUTE_FILTER: no score is written; a strided sample of the scores gives a
   * lower bound of the k-th score, the scan keeps only the (score, position) pairs at or above it and one
   * workgroup per KV head picks the k best of them exactly (rows whose bound missed are redone exactly).
   * REATTN_ROUTE_AUTO (0) takes the filter from 2^22 scored keys per step (n_mid * Hkv) upwards.  A tuning
   * and testing aid: shapes the filter does not take (short middles, top_k so large that the kept pairs
   * would outgrow the pick, REATTN_AGG_MAX) use the scores whatever is asked for. */
  int32_t route;
  /* A decode step (reattn_decode_step, _static, _timed; reattn_vote_layer and its _timed form with n_query == 1)
   * normally starts with a launch that zeroes its histograms and builds its rotary table (the vote layer's: the
   * table only).  Nonzero ws_warm is the caller's promise that this launch is not needed: the last call that
   * wrote `ws` was the same kind of decode step with the same head counts, head_dim, dtype, n_sink, n_local,
   * top_k (vote selection: the same reattn_vote), rope_theta and paging, over a context of at least
   * n_sink + top_k + n_local tokens (vote: n_sink + n_centres * span + n_local), so that the scope S, and with
   * it the table, is the same (n_ctx itself may have grown); that call was enqueued on the same stream or has
   * completed; and nothing else has written `ws` since.  Every step leaves the histograms zeroed behind it,
   * and both sit at the front of the workspace at offsets that do not depend on n_ctx.  A promise that does not
   * hold gives wrong results, not an error: the library cannot see it.  Other calls ignore the field. */
  int32_t ws_warm;
} reattn_params;
typedef enum { REATTN_ROUTE_AUTO = 0, REATTN_ROUTE_FILTER = 1, REATTN_ROUTE_SCORES = 2 } reattn_route;

/* Library version (major*10000 + minor*100 + patch) and a static message for a status. */
int reattn_version(void);
const char* reattn_status_string(int status);
/* sizeof(reattn_params) / sizeof(reattn_vote) as this library was compiled: a binding that declares the
 * structs by hand (ctypes, an FFI) compares them with its own before the first call. */
size_t reattn_params_bytes(void);
size_t reattn_vote_bytes(void);

/* Host-only checks of `p` (no GPU needed).  REATTN_OK or the first error found. */
int reattn_validate(const reattn_params* p);

/* Eq. 1 with the clamping rules above.  Any output pointer may be NULL.  Host only. */
int reattn_scope(const reattn_params* p, int64_t* n_sink_eff, int64_t* n_local_eff,
                 int64_t* n_mid, int64_t* k_eff, int64_t* scope);

/* Bytes of device scratch every call below accepts for these params (0 if `p` is
 * invalid).  The buffer must be 256-byte aligned; its contents are garbage in and
 * garbage out, and two calls that share it must be ordered on one stream. */
size_t reattn_workspace_bytes(const reattn_params* p);

/* Eq. 2, first line: scores[i][h][j] = sum over the G heads of group h of
 * q[i][hG+g] . k_cache[h][s_eff + j], j in [0, N_mid); no rotary encoding, no
 * scaling; fp32 accumulation.  M == 1 streams the cache once (HBM-bound) and
 * needs no workspace (ws may be NULL); M > 1 with bf16 / fp16 storage and D == 128 runs
 * the MFMA contraction and uses ws; other M > 1 shapes stream once per query.
 * N_mid == 0 is a no-op. */
int reattn_score(const reattn_params* p, const void* q, const void* k_cache,
                 float* scores, void* ws, size_t ws_bytes, void* stream);

/* Eq. 2: per (query, KV head) row of `scores`, the k_eff largest entries as
 * absolute ascending cache indices.  Ties: higher score first, then lower index.
 * Deterministic.  k_eff == 0 is a no-op.  `scores` is read only. */
int reattn_topk(const reattn_params* p, const float* scores, int32_t* idx,
                void* ws, size_t ws_bytes, void* stream);

/* Eq. 3, first line + PE on the keys: gathers [sink, idx, local] rows of K and V
 * per (query, KV head); K rows are rotary-encoded in fp32 at slot r (pair
 * (c, c + D/2), angle r * theta^(-2c/D)); V rows are copied.  Rows of a query
 * beyond its causal cut are zero-filled.  Needs M*Hkv*S*D*(4 + elem) bytes. */
int reattn_gather_rope(const reattn_params* p, const void* k_cache, const void* v_cache,
                       const int32_t* idx, float* k_sel, void* v_sel, void* stream);

/* Eq. 3, second line: out[i][hq] = softmax(q~ . k_sel[i][hq/G]^T * scale) v_sel[i][hq/G]
 * over the first S - (M - 1 - i) slots, with q~ the query rotary-encoded at the
 * slot of its own key (the last one it sees).  fp32 throughout. */
int reattn_attend(const reattn_params* p, const void* q, const float* k_sel, const void* v_sel,
                  float* out, void* ws, size_t ws_bytes, void* stream);

/* One decode step of one layer (appendix, decoding phase, the lines from the
 * score to rope_attention): score -> top-k -> concat -> PE -> attention, with the
 * gather and the rotary encoding done on the fly (nothing of size S*D is
 * materialised).  Requires M == 1.  idx_out may be NULL. */
int reattn_decode_step(const reattn_params* p, const void* q, const void* k_cache,
                       const void* v_cache, int32_t* idx_out, float* out,
                       void* ws, size_t ws_bytes, void* stream);

/* reattn_decode_step for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus the workspace,
 * same kernels, same results; the step's scratch (scores, histograms, candidate lists, selection bitmap,
 * rotary table, split-S partials) is a fixed array of REATTN_STATIC_SCRATCH_BYTES inside the library's
 * device image, which every GPU the library runs on holds until the process ends.  The call allocates
 * nothing and frees nothing.  Steps whose reattn_workspace_bytes() exceeds the array (a bf16 cache of
 * 8 KV heads past ~500K tokens) return REATTN_ERR_STATIC_LIMIT before anything is launched.  All calls
 * on one GPU share that GPU's array: calls that overlap on one GPU (two streams, two threads) race; order
 * them on one stream.  Nothing the next call relies on is kept between calls, unless the caller sets
 * reattn_params.ws_warm: the array is then the workspace the promise is about (the previous step through this
 * entry point on this GPU). */
#define REATTN_STATIC_SCRATCH_BYTES (32u << 20)
size_t reattn_static_scratch_bytes(void);
int reattn_decode_step_static(const reattn_params* p, const void* q, const void* k_cache,
                              const void* v_cache, int32_t* idx_out, float* out, void* stream);

/* One prefill chunk of one layer (appendix, prefilling phase, same lines) for
 * M >= 1 queries: per-query scores, per-query top-k, causal attention over
 * [sink, selected_i, local up to token i].  idx_out may be NULL. */
int reattn_prefill_chunk(const reattn_params* p, const void* q, const void* k_cache,
                         const void* v_cache, int32_t* idx_out, float* out,
                         void* ws, size_t ws_bytes, void* stream);

/* ---- Vote selection -------------------------------------------------------------------
 * The paper's way of combining heads and query rows (Method, "Full-Context Cache
 * Selection", last paragraph; Setup: k = 4, k' = 127, span 32): every (query row, query
 * head) votes for its own `vote_k` best middle tokens by raw score
 * q[i][hq] . k_cache[hq/G][j]; votes of all heads and all M query rows are pooled; the
 * `n_centres` most voted tokens (ties: lower index; tokens without a vote never) are kept
 * together with their `span` neighbouring entries [c - span/2, c - span/2 + span), clipped
 * to the middle, overlaps deduplicated.  The result is ONE ascending index list per layer,
 * shared by all heads and query rows, of data-dependent length n_sel <= cap =
 * min(n_centres * span, N_mid).  In these calls p->top_k is ignored, the scope is
 * S = s_eff + n_sel + l_eff (query i sits at slot s_eff + n_sel + l_eff - M + i) and
 * p->max_position is checked against s_eff + cap + l_eff.
 * Supported: every shape reattn_validate accepts (G <= 16), vote_k <= 8, n_centres <= 1024.  16-bit storage with
 * D = 128 scores on the matrix cores; fp32 storage and D = 64 on the vector ALU (the keys are then streamed
 * once per query row, and once more per 8 (D = 64, or fp32 D = 64) or 16 (fp32 D = 128) heads of a group).
 *
 * Batches: with n_seq > 1 the head axis holds n_seq equal-length sequences of a decode step (M = 1),
 * sequence b owning query heads [b * Hq/n_seq, ...) and KV heads [b * Hkv/n_seq, ...) of q / the caches;
 * votes are pooled per sequence, sel is [n_seq][cap] and n_sel [n_seq] (cap = min(n_centres * span,
 * N_mid)), and every sequence attends over its own selection.  Hq/n_seq * vote_k <= 1024. */
typedef struct reattn_vote {
  int32_t vote_k;     /* k: entries per (query row, head) list, 1..8; clamped to N_mid */
  int32_t n_centres;  /* k': 1..1024 */
  int32_t span;       /* m >= 1 */
  int32_t n_seq;      /* sequences folded into the head axis; 0 or 1 = one */
} reattn_vote;

/* Bytes of device scratch the vote calls accept for (p, v); 0 if either is invalid. */
size_t reattn_vote_workspace_bytes(const reattn_params* p, const reattn_vote* v);

/* Fused score + top-k of the selection: head_topk[i][hq][kk], kk = min(vote_k, N_mid),
 * ascending absolute indices of the kk largest raw scores of query row i, head hq (ties:
 * lower index).  The key cache is streamed once per query row; no score is written. */
int reattn_vote_topk(const reattn_params* p, const reattn_vote* v, const void* q,
                     const void* k_cache, int32_t* head_topk, void* ws, size_t ws_bytes,
                     void* stream);

/* Votes -> centres -> spans: sel[0 .. *n_sel) ascending absolute indices (sel holds cap
 * entries), *n_sel a DEVICE int32.  Pure integer work on the given lists; a list entry that
 * lies outside the middle [s_eff, N - l_eff) is ignored (it casts no vote). */
int reattn_vote_merge(const reattn_params* p, const reattn_vote* v, const int32_t* head_topk,
                      int32_t* sel, int32_t* n_sel, void* ws, size_t ws_bytes, void* stream);

/* One layer step with the vote selection for M >= 1 query rows: reattn_vote_topk ->
 * reattn_vote_merge -> attention of every query row over [sink, sel, local up to its own
 * token] with sequential positions (Eq. 3).  sel_out (cap entries) and n_sel_out (device
 * int32) may be NULL.  out: [M][Hq][D] fp32. */
int reattn_vote_layer(const reattn_params* p, const reattn_vote* v, const void* q,
                      const void* k_cache, const void* v_cache, int32_t* sel_out,
                      int32_t* n_sel_out, float* out, void* ws, size_t ws_bytes, void* stream);

/* ---- Streaming prefill of one layer ------------------------------------------------------
 * The chunk loop of the appendix's prefilling phase for ONE layer: chunk 0 holds the first
 * min(L, l_global + l_local) tokens, every later chunk `chunk` tokens (the last one what is
 * left); each chunk's keys and values are appended to the cache, then its query rows select
 * from the middle as it stands and attend (Eq. 1-3).  In these calls p->n_ctx = L is the
 * whole sequence, p->n_query is ignored, and the strides describe the cache
 * ([Hkv][>= L][D]; 0,0 = contiguous [Hkv][L][D]).  1 <= chunk <= n_local (a chunk lies inside
 * the local window: paper, hyper-parameter discussion of the chunk size). */

/* cache[h][first_tok + t][:] = new[t][h][:] for t < n_tok: k_new, v_new are token-major
 * [n_tok][Hkv][D] device buffers (as the projections deliver them); first_tok + n_tok <= n_ctx. */
int reattn_cache_append(const reattn_params* p, int64_t first_tok, int32_t n_tok, const void* k_new,
                        const void* v_new, void* k_cache, void* v_cache, void* stream);

/* Chunk c of the loop: its tokens are [*first, *end) (the chunk's query rows; the cache holds *end tokens when
 * it selects).  REATTN_ERR_RANGE past the last chunk.  Either output may be NULL.  Host only.  A caller sizes
 * idx_out of reattn_prefill_sequence by asking reattn_scope for every chunk's (n_ctx = *end, n_query = *end - *first). */
int reattn_prefill_sequence_chunk_bounds(const reattn_params* p, int32_t chunk, int64_t c, int64_t* first, int64_t* end);

/* Number of chunks of the loop (0 if p or chunk is invalid) and the scratch bytes the whole loop
 * accepts (the largest any chunk needs; v == NULL: per-query top-k, else the vote selection). */
int64_t reattn_prefill_sequence_chunks(const reattn_params* p, int32_t chunk);
size_t reattn_prefill_sequence_workspace_bytes(const reattn_params* p, const reattn_vote* v, int32_t chunk);

/* The loop.  q [L][Hq][D], k_new, v_new [L][Hkv][D], out [L][Hq][D] fp32; k_cache, v_cache are WRITTEN
 * (rows [0, L)).  v == NULL selects per query row and KV head as reattn_prefill_chunk does; then idx_out
 * (nullable) receives the chunks' index sets back to back, chunk c as [M_c][Hkv][k_eff_c].  v != NULL
 * uses the vote selection; then sel_out (nullable, [n_chunks][cap_L], cap_L = min(n_centres * span,
 * middle of the whole sequence)) and n_sel_out (nullable, [n_chunks] device int32) receive every
 * chunk's shared selection.  Everything is enqueued on `stream`; nothing synchronises. */
int reattn_prefill_sequence(const reattn_params* p, const reattn_vote* v, int32_t chunk, const void* q,
                            const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                            float* out, int32_t* idx_out, int32_t* sel_out, int32_t* n_sel_out,
                            void* ws, size_t ws_bytes, void* stream);

/* One decode token through n_layers layers (appendix, decoding phase: the loop over the layers, without
 * the projections and the feed-forward blocks that separate them in a model): for layer l the token's rows
 * k_new[l], v_new[l] ([Hkv][D]) are appended at position N - 1 of that layer's cache (p->n_ctx = N counts
 * the new token; the strides describe every layer's cache), then the layer's decode step runs with q[l]
 * ([Hq][D]) into out[l] ([Hq][D] fp32).  q, k_new, v_new, k_cache, v_cache, out are HOST arrays of
 * n_layers DEVICE pointers.  v == NULL: per-KV-head top-k (reattn_decode_step); else the vote selection.
 * One workspace (reattn_workspace_bytes / reattn_vote_workspace_bytes for M = 1) serves all layers. */
int reattn_decode_token(const reattn_params* p, const reattn_vote* v, int32_t n_layers,
                        const void* const* q, const void* const* k_new, const void* const* v_new,
                        void* const* k_cache, void* const* v_cache, float* const* out,
                        void* ws, size_t ws_bytes, void* stream);

/* Measurement aid: reattn_decode_step with HIP events recorded on `stream` at the
 * stage boundaries; it WAITS for the step to finish and fills the HOST array
 * stage_ms[REATTN_N_STAGES] with the elapsed milliseconds of
 *   [0] prep (histogram clear + rotary table), [1] the key scan of Eq. 2,
 *   [2] top-k (pivot, select, refine, emit),   [3] attention of Eq. 3 (+ combine).
 * Creates and destroys its events, so it is not for the serving loop. */
#define REATTN_N_STAGES 4
int reattn_decode_step_timed(const reattn_params* p, const void* q, const void* k_cache,
                             const void* v_cache, int32_t* idx_out, float* out,
                             void* ws, size_t ws_bytes, void* stream, float* stage_ms);

/* Measurement aid: reattn_prefill_chunk on the MFMA path (bf16 / fp16, D == 128, M > 1, k_eff > 0;
 * other shapes return REATTN_ERR_SHAPE) with HIP events at the stage boundaries; WAITS and
 * fills the HOST array stage_ms[REATTN_N_STAGES] with
 *   [0] prep + query split + sampled scores + per-row thresholds,
 *   [1] the fused MFMA score contraction with threshold filter (Eq. 2 for all M queries),
 *   [2] exact per-row top-k over the candidates (+ redo rows), [3] attention of Eq. 3. */
int reattn_prefill_chunk_timed(const reattn_params* p, const void* q, const void* k_cache,
                               const void* v_cache, int32_t* idx_out, float* out,
                               void* ws, size_t ws_bytes, void* stream, float* stage_ms);

/* Measurement aid: reattn_vote_layer with HIP events at the stage boundaries; WAITS and fills
 * the HOST array stage_ms[REATTN_N_VOTE_STAGES] with
 *   [0] the fused score + per-head top-k scan of the key cache (+ the merge of the workgroups'
 *       lists),  [1] votes -> centres -> spans,  [2] rotary table + attention of Eq. 3. */
#define REATTN_N_VOTE_STAGES 3
int reattn_vote_layer_timed(const reattn_params* p, const reattn_vote* v, const void* q,
                            const void* k_cache, const void* v_cache, int32_t* sel_out,
                            int32_t* n_sel_out, float* out, void* ws, size_t ws_bytes, void* stream,
                            float* stage_ms);

/* Diagnostic: where, inside the workspace of reattn_decode_step / reattn_prefill_chunk for these params,
 * the last call left its redo list: a uint32 count of score rows whose sampled lower bound of the k-th
 * score (Eq. 2) did not yield an exact selection by the fast route (bound above the k-th score, or more
 * candidates than the fast route holds) and that were therefore selected exactly over all their scores.
 * For a chunk (M > 1) the count is followed by that many uint32 row ids h * M + i.  *offset is in bytes.
 * REATTN_ERR_SHAPE when the params take a route without such a list (short middles, other storage). */
int reattn_redo_list_offset(const reattn_params* p, size_t* offset);

/* Measurement aid: streams `bytes` of the device buffer `buf` (16-byte aligned)
 * `iters` times with the key scan's load shape and nothing else (no arithmetic, no
 * stores) and reports the rate in GB/s into the HOST float *gb_per_s: the practical
 * read ceiling reports are normalised against next to the data-sheet peak.  Waits. */
int reattn_probe_read_bandwidth(const void* buf, size_t bytes, int iters, void* stream,
                                float* gb_per_s);

#ifdef __cplusplus
}
#endif
#endif /* REATTN_H_ */
