/*
 * samkv.h - C ABI of the SamKV hot path on one MI355X (gfx950).
 *
 * SamKV (Sparse Attention across Multiple-context KV Cache) sparsifies N independently prefilled
 * per-document KV caches against the user query, then recomputes the kept tokens locally so that
 * they see the other documents.  This library holds the data-parallel part of one layer:
 *
 *   samkv_score           personalized query vector per document (Sec. 3.1, Eq. 1) and the inner
 *                         product of every cached key with it (Sec. 3.2, Table 2 "<.,.>")
 *   samkv_topk_select     per document and KV head, keep the top share of the scores (Sec. 3.2);
 *                         initial and local positions may be forced in (Sec. 3.2, Setup)
 *   samkv_gather          concatenate the kept K/V of all documents into one compacted cache, in
 *                         document order and original position order (Sec. 3.2, last paragraph)
 *   samkv_recompute_attn  attention of the kept tokens over the compacted cache, causal across
 *                         document boundaries: the attention inside the recomputation (Sec. 3.3)
 *   samkv_query_attn      attention of the user query's tokens over the compacted cache: the final
 *                         incremental prefill of the query (Sec. 3.3, last paragraph)
 *   samkv_kv_update       overwrite or fuse (Eq. 4) recomputed K/V rows into the compacted cache
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer unless the comment says "host".  Host arrays (len,
 *     pointer tables, cu_k_host) are read or written before the call returns.
 *   - The caller owns every buffer, including the workspace; the library allocates nothing and keeps
 *     no state between calls.  A workspace of samkv_workspace_bytes(...) bytes, 256-byte aligned,
 *     serves any of the calls; its contents are scratch.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the default stream).
 *     No call synchronises with the device.
 *   - Tensors are dense, row-major, innermost dimension = head_dim.  `dtype` is the storage type of
 *     K, V and all Q tensors.  Scores, attention outputs and log-sum-exp are always float32.
 *   - Grouped-query attention: query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - Return value: SAMKV_OK or a negative error.  Argument errors are found before anything is
 *     launched and leave the outputs untouched.  Results are deterministic (no float atomics).
 *   - HIP graphs: every call only enqueues kernels (no memsets, no copies, no allocation), so a sequence of calls
 *     can be captured.  The first attention call on a device raises the dynamic-LDS limit of every attention kernel
 *     variant with hipFuncSetAttribute; make one attention call (any shape) before capturing.
 *   - Alignment: every K, V and Q tensor, the compacted caches and the attention outputs must be 16-byte aligned
 *     (rows are moved with 16-byte accesses); scores, positions and log-sum-exp 4-byte aligned.  Anything else is
 *     SAMKV_EINVAL, found before any launch.
 *   - Limits: head_dim in {64, 128}; n_ctx <= SAMKV_MAX_CTX; each document at most SAMKV_MAX_LEN
 *     tokens; n_q_heads a multiple of n_kv_heads.
 */
#ifndef SAMKV_H_
#define SAMKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SAMKV_MAX_CTX 128
#define SAMKV_MAX_LEN 65536

typedef enum { SAMKV_F32 = 0, SAMKV_BF16 = 1 } samkv_dtype;

enum {
  SAMKV_OK = 0,
  SAMKV_EINVAL = -1,       /* NULL pointer, non-positive size, inconsistent shapes, ratio outside (0, 1] */
  SAMKV_EUNSUPPORTED = -2, /* head_dim, dtype, n_ctx or document length outside the limits above */
  SAMKV_EWORKSPACE = -3,   /* workspace missing or smaller than samkv_workspace_bytes(...) */
  SAMKV_EDEVICE = -4       /* the HIP runtime refused a launch */
};

/* The N per-document caches of one layer.  In the paper's problem statement (Abstract, Sec. 1) every
 * retrieved document's KV cache was prefilled and stored on its own, without seeing the others.
 * Host struct. */
typedef struct {
  int32_t n_ctx;            /* D in the paper: number of documents                              */
  int32_t n_q_heads;        /* Hq                                                                */
  int32_t n_kv_heads;       /* Hkv                                                               */
  int32_t head_dim;         /* d                                                                 */
  int32_t dtype;            /* samkv_dtype of k, v and of every Q tensor passed with this struct */
  const int32_t* len;       /* host [n_ctx]: tokens per document, each >= 1                      */
  const void* const* k;     /* host [n_ctx] of device pointers, document i: [Hkv][len[i]][d]     */
  const void* const* v;     /* same for V; may be NULL for samkv_score and samkv_topk_select     */
} samkv_caches;

/* Human-readable name of an error code (static string). */
const char* samkv_strerror(int code);

/* Number of tokens kept per (document, KV head) for a document of `len` tokens at budget `ratio`:
 * ceil(ratio * len), at least 1, at most len; the product is shrunk by 2^-22 before the ceiling so
 * that the float32 rounding of the ratio cannot push an integral budget up (0.1 * 20 gives 2).
 * Returns 0 for invalid arguments. */
int32_t samkv_kept_count(int32_t len, float ratio);

/* Bytes of workspace that serve every call below for these sizes.  m_total = sum of kept counts
 * (length of the compacted cache); n_q_tok = user-query tokens; w_loc = rows of a local Q cache. */
size_t samkv_workspace_bytes(int32_t n_ctx, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                             int32_t n_q_tok, int32_t m_total);

/* Sec. 3.1 + Sec. 3.2 scoring.
 *   Q_que[h]     = mean over the n_q_tok rows of q_tok[h]                      (generic query vector)
 *   Q_loc_j[h]   = mean over the w_loc rows of q_loc[j][h]                     (document j's local Q cache)
 *   Q^_i[h]      = Q_que[h] + 1/(N-1) * sum_{j != i} |cos(Q_que[h], Q_loc_j[h])| * Q_loc_j[h]      (Eq. 1)
 *   scores[g][cu_len[i] + t] = mean over the query heads h of KV head g of <Q^_i[h], K_i[g][t][:]>
 * with cu_len the exclusive prefix sum of caches->len.  q_loc == NULL or n_ctx == 1 drops the bias
 * term; a cosine whose argument has norm below 1e-20 counts as 0.
 *   q_tok   [Hq][n_q_tok][d]            dtype of caches
 *   q_loc   [n_ctx][Hq][w_loc][d]       dtype of caches, or NULL
 *   scores  [Hkv][sum len]  float32     written
 * Arithmetic: float32 accumulation of exact products. */
int samkv_score(const samkv_caches* caches, const void* q_tok, int32_t n_q_tok, const void* q_loc,
                int32_t w_loc, float* scores, void* ws, size_t ws_bytes, void* stream);

/* samkv_score for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, arithmetic and results as
 * samkv_score; the few vectors of Eq. 1 that samkv_score keeps in the caller's workspace live in a fixed
 * SAMKV_NOALLOC_SCRATCH_BYTES area inside the library's device image instead (every GPU the library runs on holds one
 * copy until the process ends).  The call allocates nothing and frees nothing.
 *   - Sizes whose vectors do not fit the area (about 4 * head_dim * n_q_heads * (n_ctx + 2) + 4 * head_dim *
 *     n_kv_heads * n_ctx bytes) are SAMKV_EUNSUPPORTED; every other error as in samkv_score.
 *   - All calls on one GPU share that GPU's area: two calls that overlap in time on one GPU (different streams, or
 *     different threads) race and give undefined scores.  Calls on one stream are ordered and safe.  Nothing in the
 *     area has to survive or be cleared between calls.
 *   - The first call on a device looks the area's address up (hipGetSymbolAddress); make that call outside a capture. */
#define SAMKV_NOALLOC_SCRATCH_BYTES (8u << 20)
int samkv_score_noalloc(const samkv_caches* caches, const void* q_tok, int32_t n_q_tok, const void* q_loc,
                        int32_t w_loc, float* scores, void* stream);

/* Sec. 3.2 selection with a fixed budget.  For document i and KV head g, keep k_i =
 * samkv_kept_count(len[i], ratio) positions: first the n_sink initial and n_local last positions
 * (they count towards k_i; n_sink + n_local > k_i for any document is SAMKV_EINVAL), then the
 * largest scores; equal scores go to the lower position.
 *   scores     [Hkv][sum len] float32, as written by samkv_score
 *   idx        [Hkv][M] int32 written: document-local positions, documents in order, ascending
 *              inside each document; M = sum k_i
 *   cu_k_dev   [n_ctx + 1] int32 device, written (exclusive prefix sum of k_i); may be NULL
 *   cu_k_host  [n_ctx + 1] int32 host, written before the call returns; may be NULL
 * caches->k and caches->v are not read. */
int samkv_topk_select(const float* scores, const samkv_caches* caches, float ratio, int32_t n_sink,
                      int32_t n_local, int32_t* idx, int32_t* cu_k_dev, int32_t* cu_k_host, void* ws,
                      size_t ws_bytes, void* stream);

/* samkv_score and samkv_topk_select as one call that passes over K once: a workgroup owns one (document, KV head)
 * row, keeps its scores on chip and selects from there.  Arguments as in the two calls; the kept positions are
 * bit-identical to theirs.  `scores` may be NULL when the caller does not need them; documents longer than 8192
 * tokens fall back to the two kernels and then need `scores` as their buffer (NULL is SAMKV_EINVAL there). */
int samkv_score_select(const samkv_caches* caches, const void* q_tok, int32_t n_q_tok, const void* q_loc,
                       int32_t w_loc, float ratio, int32_t n_sink, int32_t n_local, float* scores, int32_t* idx,
                       int32_t* cu_k_dev, int32_t* cu_k_host, void* ws, size_t ws_bytes, void* stream);

/* samkv_score_select and samkv_gather (Sec. 3.2: score, select, concatenate the kept rows) as one call: the workgroup
 * that has selected a (document, KV head) row also copies its kept K and V rows into the compacted cache, so short
 * inputs pay one launch instead of two.  Arguments and results as in the two calls (idx is written as well; k_c and
 * v_c [Hkv][M][d], dtype of caches, must not be NULL; caches->v is read).  Documents longer than 8192 tokens fall back
 * to the separate kernels and need `scores` as their buffer. */
int samkv_score_select_gather(const samkv_caches* caches, const void* q_tok, int32_t n_q_tok, const void* q_loc,
                              int32_t w_loc, float ratio, int32_t n_sink, int32_t n_local, float* scores, int32_t* idx,
                              int32_t* cu_k_dev, int32_t* cu_k_host, void* k_c, void* v_c, void* ws, size_t ws_bytes,
                              void* stream);

/* Sec. 3.2, dynamic Top-P (Eq. 2 and Eq. 3).  HOST arithmetic on a handful of scalars, no device work:
 *   P^(n)_i = (s_max - s_anc) / (s_max - s_min)  if s_min < s_anc <= s_max, else 0                  (Eq. 2)
 *   P_i     = mean over the n_layers stable layers of P^(n)_i                                        (Eq. 3)
 * s_anc, s_max, s_min: host [n_layers][n_ctx], the scores <Q^_i, K> of document i's anchor block, of its
 * most-attended and of its least-attended middle block in each stable layer (which blocks those are comes
 * from the paper's offline attention analysis and is the caller's knowledge; the scores themselves can be
 * read off samkv_score's output).  p: host [n_ctx], written. */
int samkv_top_p(const float* s_anc, const float* s_max, const float* s_min, int32_t n_layers, int32_t n_ctx,
                float* p);

/* Kept tokens of a document of `len` tokens whose n_sink initial and n_local last positions are kept in full
 * while the middle is sparsified to the share p in [0, 1] (Sec. 3.2: initial and local positions are not
 * sparsified): n_sink + n_local + ceil(p * (len - n_sink - n_local)), at most len.  0 for invalid arguments. */
int32_t samkv_kept_count_mid(int32_t len, float p, int32_t n_sink, int32_t n_local);

/* samkv_topk_select with one share per document (the P_i of Eq. 3) applied to the middle segment:
 * k_i = samkv_kept_count_mid(len[i], p[i], n_sink, n_local).  p: host [n_ctx], each in [0, 1]; a document
 * may keep nothing, the total must be at least one token.  Everything else as in samkv_topk_select. */
int samkv_topk_select_v(const float* scores, const samkv_caches* caches, const float* p, int32_t n_sink,
                        int32_t n_local, int32_t* idx, int32_t* cu_k_dev, int32_t* cu_k_host, void* ws,
                        size_t ws_bytes, void* stream);

/* Sec. 3.2, block-level retrieval: the cache is managed in blocks of `block` consecutive tokens and a block is
 * represented by the mean of its keys (Setup: 64-token blocks).  The inner product is linear, so the score of a
 * block is the mean of its tokens' scores:
 *   bscores[g][cu_b[i] + b] = mean over t in [b*block, min(len[i], (b+1)*block)) of scores[g][cu_len[i] + t]
 * with cu_b the exclusive prefix sum of ceil(len[i] / block); a document's last block may be short.
 *   scores   [Hkv][sum len] float32 (samkv_score's output);   bscores [Hkv][sum ceil(len/block)] float32 written
 *   1 <= block <= 4096.   caches->k and caches->v are not read. */
int samkv_block_scores(const float* scores, const samkv_caches* caches, int32_t block, float* bscores,
                       void* stream);

/* Workspace of samkv_block_select, bytes (0 for invalid arguments). */
size_t samkv_block_workspace_bytes(const samkv_caches* caches, int32_t block);

/* Sec. 3.2 selection at block granularity.  Per document i and KV head g: the first n_init_blocks and the last
 * n_local_blocks blocks are always kept (Setup: 1 and 2), and of the B_i - n_init_blocks - n_local_blocks middle
 * blocks the ceil(p[i] * middle) with the largest block scores (ties to the lower block).  The kept blocks are
 * written out as the positions of their tokens, so the result feeds samkv_gather_v / samkv_gather_q unchanged:
 *   idx        [Hkv][M] int32 written: document-local token positions, ascending inside each document
 *   cu_k_dev / cu_k_host   [n_ctx + 1] exclusive prefix sum of the kept TOKENS per document (either may be NULL)
 *   p          host [n_ctx], each in [0, 1] (the P_i of Eq. 3)
 * Every head must keep the same number of tokens, so a short last block has to be kept by all heads or by none:
 * with n_local_blocks == 0 a document whose length is not a multiple of `block` is SAMKV_EINVAL unless it keeps
 * all of its blocks or none.  ws: samkv_block_workspace_bytes(caches, block) bytes, 256-byte aligned.
 * The second, cross-document filter that the paper applies to the retrieved blocks is not part of this call:
 * the paper does not define the normalisation it compares blocks of different documents under. */
int samkv_block_select(const float* bscores, const samkv_caches* caches, int32_t block, const float* p,
                       int32_t n_init_blocks, int32_t n_local_blocks, int32_t* idx, int32_t* cu_k_dev,
                       int32_t* cu_k_host, void* ws, size_t ws_bytes, void* stream);

/* Tokens per KV head that samkv_block_select keeps, M (host arithmetic); 0 for invalid arguments. */
int32_t samkv_block_select_count(const samkv_caches* caches, int32_t block, const float* p,
                                 int32_t n_init_blocks, int32_t n_local_blocks);

/* Sec. 3.2, second filter across documents, on top of samkv_block_select.  Per KV head: the candidates are the
 * middle blocks that the per-document selection retrieved; each document's candidate scores are normalised, the
 * candidates of all documents are compared, and keep = ceil(candidates / n_ctx) of them survive (the paper: the
 * total block count divided by the number of documents).  Forced initial / local blocks always survive.
 * READING, not fixed by the paper (it names a normalisation but does not define it): min-max per document and KV
 * head over its candidates, (s - min) / (max - min) in float32, 1 when max == min; equal normalised scores go to
 * the earlier document, then the lower block.
 * The documents' shares now differ from head to head, so the result is one row of GLOBAL token positions per
 * head (position in the concatenation of all documents, cu_len[i] + t), ascending:
 *   gidx   [Hkv][M] int32 written, M = samkv_block_filter_count(...) (same for every head)
 *   ws     samkv_block_workspace_bytes(caches, block) bytes, 256-byte aligned
 * Every candidate must be a full block: a document with a short last block needs n_local_blocks >= 1
 * (SAMKV_EINVAL otherwise); more than SAMKV_MAX_LEN retrieved blocks in total is SAMKV_EUNSUPPORTED. */
int samkv_block_select_filter(const float* bscores, const samkv_caches* caches, int32_t block, const float* p,
                              int32_t n_init_blocks, int32_t n_local_blocks, int32_t* gidx, void* ws,
                              size_t ws_bytes, void* stream);

/* Tokens per KV head that samkv_block_select_filter keeps (host arithmetic); 0 for invalid arguments. */
int32_t samkv_block_filter_count(const samkv_caches* caches, int32_t block, const float* p,
                                 int32_t n_init_blocks, int32_t n_local_blocks);

/* Compaction by global token positions: K_c[g][m][:] = K_i[g][gidx[g][m] - cu_len[i]][:] with i the document that
 * holds the position, same for V; bit-exact copies.  gidx [Hkv][m_total] device (out-of-range values are clamped);
 * k_c, v_c [Hkv][m_total][d] written. */
int samkv_gather_g(const samkv_caches* caches, const int32_t* gidx, int32_t m_total, void* k_c, void* v_c,
                   void* stream);

/* The same for the stored Q caches (as samkv_gather_q): q_rec[h][m][:] = Q_i[h][gidx[h / G][m] - cu_len[i]][:]. */
int samkv_gather_q_g(const samkv_caches* caches, const void* const* q_cache, const int32_t* gidx, int32_t m_total,
                     void* q_rec, void* stream);

/* samkv_gather with the kept counts given explicitly: cu_k_host is host [n_ctx + 1], the exclusive prefix
 * sum that the selection returned. */
int samkv_gather_v(const samkv_caches* caches, const int32_t* idx, const int32_t* cu_k_host, void* k_c,
                   void* v_c, void* stream);

/* Sec. 3.2 compaction: K_c[g][cu_k[i] + m][:] = K_i[g][idx[g][cu_k[i] + m]][:], same for V; bit-exact
 * copies.  The kept counts are recomputed from caches->len and `ratio` exactly as in
 * samkv_topk_select, so idx must come from a selection at the same ratio.
 *   idx   [Hkv][M] int32 device (values outside [0, len[i]) are clamped, never dereferenced raw)
 *   k_c, v_c  [Hkv][M][d]  dtype of caches, written */
int samkv_gather(const samkv_caches* caches, const int32_t* idx, float ratio, void* k_c, void* v_c,
                 void* stream);

/* Same compaction for the per-document Q caches the method also stores (Table 2: the notation covers Q
 * caches as well): q_rec[h][cu_k[i] + m][:] = Q_i[h][idx[h / G][cu_k[i] + m]][:], bit-exact copies.  This
 * yields the query states of the kept tokens that samkv_recompute_attn takes.
 *   q_cache  host [n_ctx] of device pointers, document i: [Hq][len[i]][d], dtype of caches
 *   q_rec    [Hq][M][d] written.   caches->k and caches->v are not read. */
int samkv_gather_q(const samkv_caches* caches, const void* const* q_cache, const int32_t* idx, float ratio,
                   void* q_rec, void* stream);

/* samkv_gather_q with the kept counts given explicitly (cu_k_host as in samkv_gather_v). */
int samkv_gather_q_v(const samkv_caches* caches, const void* const* q_cache, const int32_t* idx,
                     const int32_t* cu_k_host, void* q_rec, void* stream);

/* Sec. 3.3 recomputation, attention part.  Row p of query head h is the query state of the token
 * that KV head g(h) keeps at compacted position p; it attends to compacted positions 0..p (itself
 * included), across document boundaries:
 *   out[h][p][:] = sum_{j <= p} softmax_j(scale * <q_rec[h][p], k_c[g][j]>) * v_c[g][j]
 *   lse[h][p]    = log sum_{j <= p} exp(scale * <q_rec[h][p], k_c[g][j]>)
 *   q_rec [Hq][M][d], k_c, v_c [Hkv][M][d] in `dtype`; out [Hq][M][d], lse [Hq][M] float32.
 * bf16: scores on the bf16 matrix cores, softmax statistics and accumulators float32.  The second product runs on
 * the half-precision matrix cores: the softmax weights are rounded to IEEE half precision (11-bit significand), and
 * V is first rewritten into the workspace as half precision, each KV head scaled by a power of two so that nothing
 * overflows and bf16 values down to 2^-32 of the head's largest magnitude stay exact (smaller ones lose at most
 * 2^-40 of that magnitude).  f32: float32 throughout.
 * ws: samkv_workspace_bytes(...) bytes, 256-byte aligned, for bf16 (SAMKV_EWORKSPACE otherwise); f32 needs none. */
int samkv_recompute_attn(const void* q_rec, const void* k_c, const void* v_c, int32_t m_total,
                         int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t dtype,
                         float scale, float* out, float* lse, void* ws, size_t ws_bytes, void* stream);

/* Sec. 3.3, last paragraph: the user query's tokens attend over the whole compacted cache (every
 * cached token precedes the query, so there is no mask):
 *   out[h][t][:] = sum_{j < M} softmax_j(scale * <q_tok[h][t], k_c[g][j]>) * v_c[g][j],  lse likewise.
 *   q_tok [Hq][n_q_tok][d]; out [Hq][n_q_tok][d], lse [Hq][n_q_tok] float32.
 * Arithmetic as in samkv_recompute_attn, with one difference for bf16 with fewer than 512 query rows per KV head
 * (G * n_q_tok < 512: the call is bound by latency or by HBM, and rewriting V would cost more than the products):
 * V is read as stored and every softmax weight enters the second product as the sum of two bf16 terms
 * (16 significant bits), on the bf16 matrix cores; no copy of V is made.  Long caches are cut into key chunks whose
 * partial results are merged by their log-sum-exp, in chunk order (deterministic).
 * ws: samkv_workspace_bytes(...) bytes, 256-byte aligned: the half-precision copy of V (bf16, when made) and the
 * chunk partials; f32 with a single chunk needs none.  Too small or missing: SAMKV_EWORKSPACE. */
int samkv_query_attn(const void* q_tok, int32_t n_q_tok, const void* k_c, const void* v_c,
                     int32_t m_total, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                     int32_t dtype, float scale, float* out, float* lse, void* ws, size_t ws_bytes,
                     void* stream);

/* samkv_recompute_attn followed by samkv_query_attn over the same compacted cache, as one call (Sec. 3.3: the kept
 * tokens are recomputed, then the query is prefilled over the result; here both read k_c, v_c as they stand).  The
 * half-precision copy of V that the bf16 kernels read is made once and serves both.  bf16: both attentions run in ONE
 * kernel launch; the query attention's workgroups are handed out first and each walks all keys of its rows in one
 * chunk (no partial results, no merge), which takes as long as the causal problem's longest row tile, so the query
 * attention hides inside the causal one.  The recompute outputs are bit-identical to samkv_recompute_attn's; the query
 * outputs follow the same definition as samkv_query_attn's but sum the keys in one chunk instead of several, so they
 * agree with it to rounding (both within the stated precision), not bit for bit.  float32: the two kernels one after
 * the other, bit-identical to the two calls.  Arguments as in the two calls; ws as for samkv_query_attn.  A caller
 * that updates the cache between the two attentions (samkv_kv_update) uses the separate calls. */
int samkv_recompute_query_attn(const void* q_rec, const void* q_tok, int32_t n_q_tok, const void* k_c, const void* v_c,
                               int32_t m_total, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t dtype,
                               float scale, float* rec_out, float* rec_lse, float* q_out, float* q_lse, void* ws,
                               size_t ws_bytes, void* stream);

/* The same prefill with the query's own keys and values: query token t attends to the whole compacted
 * cache and to query tokens 0..t (itself included), which is what an incremental prefill of the query
 * after the cached documents computes (Sec. 3.3, last paragraph).
 *   k_self, v_self  [Hkv][n_q_tok][d]  the query tokens' own K/V, dtype as the other tensors
 * Computed as two partial attentions (cache: no mask; self: causal) merged by their log-sum-exp.
 * Needs a workspace (samkv_workspace_bytes covers it). */
int samkv_query_attn_self(const void* q_tok, int32_t n_q_tok, const void* k_c, const void* v_c,
                          int32_t m_total, const void* k_self, const void* v_self, int32_t n_q_heads,
                          int32_t n_kv_heads, int32_t head_dim, int32_t dtype, float scale, float* out,
                          float* lse, void* ws, size_t ws_bytes, void* stream);

/* Sec. 3.3, cache update after recomputation.  k_c, v_c [Hkv][M][d] hold the old compacted cache and are
 * updated in place from the recomputed rows k_new, v_new (same shape and dtype):
 *   mode SAMKV_OVERWRITE: row <- new row
 *   mode SAMKV_FUSION (Eq. 4): theta = cos(new row, old row); row <- theta * new + (1 - theta) * old,
 *     per compacted position and KV head, separately for K and for V; float32 arithmetic, one rounding
 *     to `dtype` at the end; theta = 1 when either row has norm below 1e-20.
 * The new rows come from the model's K/V projections of the recomputed tokens, which are outside this
 * library; samkv_query_attn then attends over the updated cache. */
enum { SAMKV_OVERWRITE = 0, SAMKV_FUSION = 1 };
int samkv_kv_update(void* k_c, void* v_c, const void* k_new, const void* v_new, int32_t m_total,
                    int32_t n_kv_heads, int32_t head_dim, int32_t dtype, int32_t mode, void* stream);

/* Diagnostics, not part of the method: two micro-kernels with which a benchmark measures what this device
 * sustains, to quote kernel rates against the measured ceiling as well as the published one.  The caller times the
 * launch (HIP events on `stream`).
 *   samkv_peak_mfma_bf16  n_blocks workgroups of 4 waves, each wave issues iters * 16 independent
 *                         v_mfma_f32_32x32x16_bf16: n_blocks * 4 * iters * 16 * 32768 flop.  sink: 4 bytes, untouched.
 *   samkv_peak_copy       dst[0..bytes) = src[0..bytes), 16-byte aligned, bytes a multiple of 16.
 *   samkv_peak_read       reads src[0..bytes) once (16-byte aligned, a multiple of 16); sink: 4 bytes, untouched. */
int samkv_peak_mfma_bf16(float* sink, int32_t n_blocks, int32_t iters, void* stream);
/* The same loop with a chosen operand pattern: 0 small integers (what samkv_peak_mfma_bf16 uses), 1 zeros, 2
 * pseudo-random values with full mantissas.  The sustained rate depends on it: the device holds its power limit by
 * lowering the clock, and the matrix unit draws more the more operand bits toggle.  Pattern 2 is the ceiling for a
 * kernel that multiplies real data.  Other patterns: SAMKV_EINVAL. */
int samkv_peak_mfma_bf16_data(float* sink, int32_t n_blocks, int32_t iters, int32_t pattern, void* stream);
int samkv_peak_copy(const void* src, void* dst, size_t bytes, void* stream);
int samkv_peak_read(const void* src, size_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SAMKV_H_ */
