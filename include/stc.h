/*
 * stc.h - C ABI of libstc: decode-step attention over a two-level compressed KV
 * cache on AMD MI355X (gfx950).
 *
 * Level 1 is Quest-style page selection over the cached keys (the paper's
 * Stage I, Sec. 3.2, with the chunk size 16 of its LLM training-config table in
 * App. C.1).  Level 2 is sub-token value-group routing (Stage II, Sec. 3.3): the
 * value vector of every cached token is split into G groups (the paper's S), a
 * per-token bitmask records which groups the router kept, and only kept groups
 * are stored ("group-packed store").  Attention follows the equation of
 * Sec. 3.3: softmax(q K^T / sqrt(d_h)) applied to the routed value matrix;
 * queries and keys are never compressed, dropped groups contribute nothing and
 * the softmax is not renormalised over kept groups.
 *
 * Calls
 *   cache construction   stc_build_page_bounds, stc_route_and_pack_values (per-token top-K,
 *                        given masks, or the global token-group budget of the LLM setting),
 *                        stc_router_logits (the router's projection), stc_compact_tokens
 *                        (token-level compaction helper)
 *   decode step          stc_select_pages (+ stc_score_pages: its scoring half alone),
 *                        stc_decode_attention; stc_decode_step does both in one call
 *                        (stc_decode_step_tail: with the uncompressed tail;
 *                        stc_decode_step_static: without a caller-provided workspace)
 *   recent tokens        stc_append_tail, stc_decode_attention_tail (uncompressed tail),
 *                        stc_flush_tail (tail tokens into the compressed cache, in place)
 *   per-query-head form  stc_select_pages_per_head, stc_decode_attention_per_head,
 *                        stc_union_pages + stc_decode_attention_union (shared K/V reads)
 *   helpers              stc_workspace_bytes, stc_bounds_bytes, stc_status_string, stc_version
 *
 * Conventions shared by every call
 *   - "stream" = one (batch b, KV head h) pair; streams are independent.
 *     Query head j belongs to KV head j / (Hq/Hkv).
 *   - Every data pointer is a DEVICE pointer owned by the caller, 16-byte
 *     aligned, to a contiguous row-major tensor of the stated shape.  It is
 *     borrowed until the work enqueued by the call has completed.
 *     stc_shape_t is HOST memory, read during the call only.
 *   - bf16 tensors are passed as void* (2 bytes per element).
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No call synchronises, allocates, frees or keeps
 *     state between calls (the library only remembers, per device, that it has
 *     raised the LDS limit of its own kernels).
 *   - Return value: STC_OK (0) or a negative STC_ERR_* code.  On error nothing
 *     has been enqueued.  Inputs are expected to be finite (no NaN/Inf).
 *   - Ties in every top-k are broken towards the lowest index.
 */
#ifndef STC_H
#define STC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct stc_shape {
  int32_t B;            /* batch size, >= 1 */
  int32_t Hq;           /* query heads; Hq % Hkv == 0, Hq/Hkv <= 16 */
  int32_t Hkv;          /* KV heads */
  int32_t D;            /* head dimension: 64 or 128 */
  int32_t N;            /* cached tokens per stream, >= 1 */
  int32_t P;            /* page size in tokens: 16 */
  int32_t G;            /* value groups per token (paper's S): 1..16, D % G == 0,
                           group width gd = D/G >= 8 (16-byte multiples) */
  int32_t N_cap;        /* token capacity of K, mask, tok_off and bounds per stream: their
                           per-stream strides.  0 means N (no room to grow); else >= N. */
  int64_t v_cap_groups; /* capacity of each stream's packed value store, in groups */
} stc_shape_t;

enum {
  STC_OK = 0,
  STC_ERR_NULL = -1,      /* a required pointer is NULL */
  STC_ERR_SHAPE = -2,     /* a shape constraint above is violated, or k/mode out of range */
  STC_ERR_ALIGN = -3,     /* a pointer is not 16-byte aligned */
  STC_ERR_WORKSPACE = -4, /* workspace missing or smaller than stc_workspace_bytes() */
  STC_ERR_LAUNCH = -5     /* the HIP runtime refused a launch */
};

/* which_call values for stc_workspace_bytes */
enum {
  STC_WS_ROUTE = 1,
  STC_WS_SELECT = 2,
  STC_WS_ATTENTION = 3,
  STC_WS_ATTENTION_TAIL = 4,
  STC_WS_SELECT_PER_HEAD = 5,
  STC_WS_ATTENTION_PER_HEAD = 6,
  STC_WS_STEP = 7,
  STC_WS_STEP_TAIL = 8
};

/* routing modes of stc_route_and_pack_values */
enum {
  STC_ROUTE_MASK = 0, /* mask_in gives the kept groups (bits >= G are ignored) */
  STC_ROUTE_TOPK = 1, /* top-k of `logits` per token; count from kcount[] or fixed_k */
  STC_ROUTE_GLOBAL = 2, /* the N*fixed_k largest of a stream's N*G logits */
  /* flag, OR-ed into a mode: logits, kcount and mask_in hold ONE set per batch element
   * ([B, 1, N, ...]) that all KV heads of the element read -- the router gives one mask per
   * token and layer (App. B.1); stc_router_logits with Hkv = 1 writes logits of that shape */
  STC_ROUTE_SHARED = 0x100
};

int stc_version(void);
const char *stc_status_string(int status);

/* Bytes of device workspace the given call needs for this shape (0 = none).
 * k_pages is not used by STC_WS_ROUTE.  For STC_WS_ATTENTION_TAIL and STC_WS_STEP_TAIL it is
 * the number of selected pages plus ceil(n_tail / P), at their largest.  Returns 0 for an
 * invalid shape (the call itself then reports the error). */
size_t stc_workspace_bytes(const stc_shape_t *shape, int which_call, int k_pages);

/*
 * Quest page summary (Stage I, Sec. 3.2; chunk 16, App. C.1): for every page p < NP =
 * ceil(N/P) and channel c, the minimum and the maximum of K[t, c] over the page's valid
 * tokens (t < N).  Exact (comparisons only); -0 orders below +0.
 *   K      [B, Hkv, Ncap, D]  bf16, in (Ncap = N_cap, or N when N_cap is 0; rows >= N unused)
 *   bounds stc_bounds_bytes(shape) bytes, out.  A layout made for the scoring kernel:
 *          dwords [B*Hkv][NT][D/32][2][8][4][4] with NT = ceil(ceil(Ncap/16)/8) tiles of 8
 *          pages;
 *          element [s][t][j][g][e][col][w] is page 8*t + 4*g + col, channel
 *          e*(D/8) + 4*j + w of stream s: bf16 minimum in the low half of the dword,
 *          bf16 maximum in the high half.  Pages >= NP of the last tile hold zeros.
 */
int stc_build_page_bounds(const stc_shape_t *shape, const void *K, void *bounds,
                          void *stream);

/* Size in bytes of the bounds buffer of stc_build_page_bounds (0 for an invalid shape). */
size_t stc_bounds_bytes(const stc_shape_t *shape);

/*
 * Routing mask and group-packed value store (Stage II, Sec. 3.3 "Value-group
 * decomposition" and "Routing mask"; fixed per-token K of App. B.1).
 *   mode STC_ROUTE_TOPK: bit g of mask[t] is set iff group g is among the c_t
 *        largest of logits[t, 0..G) (equal logits: lower g first), where
 *        c_t = kcount[t] (clamped to G) if kcount != NULL, else fixed_k (0..G).
 *   mode STC_ROUTE_MASK: mask[t] = mask_in[t] & ((1<<G)-1).
 *   mode STC_ROUTE_GLOBAL (global token-group budget, Sec. 3.4 and App. B.1): per stream the
 *        M = N*fixed_k token-group pairs of largest logit over the whole [N, G] grid are
 *        kept (fixed_k in 0..G; equal logits, -0 == +0: lower t*G+g first), so a token keeps
 *        anything from 0 to G groups.  kcount is ignored.
 *   mode | STC_ROUTE_SHARED: the three routing inputs below are [B, 1, ...] and shared by the
 *        KV heads of a batch element (every head of the element then gets the same mask).
 *   V       [B, Hkv, N, D] bf16, in
 *   logits  [B, Hkv, N, G] float, in (TOPK and GLOBAL)
 *   kcount  [B, Hkv, N] uint8, in (TOPK, may be NULL)
 *   mask_in [B, Hkv, N] uint16, in (MASK only; must not alias mask when shared)
 *   mask    [B, Hkv, Ncap] uint16, out (may alias mask_in when Ncap == N)
 *   tok_off [B, Hkv, Ncap+1] uint32, out: exclusive prefix sum of popcount(mask)
 *           per stream, in group units; tok_off[N] = kept groups of the stream
 *   vpacked [B, Hkv, v_cap_groups, D/G] bf16, out: group g of token t (if kept)
 *           is stored at group slot tok_off[t] + popcount(mask[t] & ((1<<g)-1));
 *           slots >= tok_off[N] are left untouched
 *   dev_status int32 on the device, out (may be NULL): set to 1 if any stream's
 *           tok_off[N] exceeds v_cap_groups; writes beyond the capacity are
 *           dropped, mask and tok_off are still exact.  The caller zeroes it.
 *   ws      device workspace of stc_workspace_bytes(shape, STC_WS_ROUTE, 0) bytes
 */
int stc_route_and_pack_values(const stc_shape_t *shape, int mode, const void *V,
                              const float *logits, const uint8_t *kcount, int fixed_k,
                              const uint16_t *mask_in, uint16_t *mask, uint32_t *tok_off,
                              void *vpacked, int32_t *dev_status, void *ws, size_t ws_bytes,
                              void *stream);

/*
 * Query-aware page selection (Quest upper-bound score, top-k pages).
 *   per query head h and page p, in float:
 *     U_h[p] = sum_c max(q_h[c]*min[p,c], q_h[c]*max[p,c])
 *   the D terms are summed by a balanced tree over adjacent channels
 *   ((c0+c1)+(c2+c3))+..., every addition rounded to float;
 *   score[p] = max over the query heads of the stream's KV head; -0 becomes +0.
 *   The k_eff = min(k_pages, NP) pages of largest score (ties: lowest p) are
 *   written in ascending order of p.
 *   A query or bound that is subnormal as bf16 (|x| < 2^-126) counts as zero; products must
 *   stay finite in float.
 *   q          [B, Hq, D] bf16, in
 *   bounds     as written by stc_build_page_bounds, in (not read when k_pages >= NP)
 *   page_idx   [B, Hkv, k_eff] int32, out
 *   page_score [B, Hkv, NP] float, out, may be NULL (then the scores live in ws);
 *              not written when k_pages >= NP
 *   ws         stc_workspace_bytes(shape, STC_WS_SELECT, k_pages) bytes
 */
int stc_select_pages(const stc_shape_t *shape, const void *q, const void *bounds, int k_pages,
                     int32_t *page_idx, float *page_score, void *ws, size_t ws_bytes,
                     void *stream);

/*
 * The scoring half of stc_select_pages alone (same arithmetic, same bits): writes
 * the Quest upper-bound score of every page of every stream and selects nothing.
 *   q [B, Hq, D] bf16, in;  bounds as written by stc_build_page_bounds, in
 *   page_score [B, Hkv, NP] float, out
 */
int stc_score_pages(const stc_shape_t *shape, const void *q, const void *bounds,
                    float *page_score, void *stream);

/*
 * Routed decode attention over the selected pages (attention equation of
 * Sec. 3.3 with the routed value matrix).  With T = all tokens t < N of the
 * listed pages and s_t = (q_h . K[t]) / sqrt(D):
 *   out_h[g*gd + j] = sum_{t in T, bit g of mask[t]} softmax_T(s)_t *
 *                     vpacked[tok_off[t] + popcount(mask[t] & ((1<<g)-1))][j]
 * bf16 inputs, float accumulation, float output.
 *   q, K as above; vpacked, mask, tok_off as written by stc_route_and_pack_values
 *   page_idx [B, Hkv, k_pages] int32, in; 1 <= k_pages <= NP; entries outside
 *            [0, NP) are skipped; a page must not be listed twice.  NULL stands for
 *            pages 0 .. k_pages-1 of every stream (with k_pages == NP: the whole cache,
 *            no selection call needed)
 *   out      [B, Hq, D] float, out
 *   ws       stc_workspace_bytes(shape, STC_WS_ATTENTION, k_pages) bytes
 * Value slots at or beyond v_cap_groups are treated as dropped; v_cap_groups >= 1.
 * One stream's keys (N*D*2 bytes) and packed store (v_cap_groups*(D/G)*2 bytes) must
 * each stay below 4 GiB.
 */
int stc_decode_attention(const stc_shape_t *shape, const void *q, const void *K,
                         const void *vpacked, const uint16_t *mask, const uint32_t *tok_off,
                         const int32_t *page_idx, int k_pages, float *out, void *ws,
                         size_t ws_bytes, void *stream);

/*
 * One decode step of the compressed cache: the page selection of stc_select_pages (Quest
 * bound scores, top-k_pages per stream; Sec. 3.4) followed by the attention of
 * stc_decode_attention over the selected pages (Sec. 3.3), with the same results bit for
 * bit as the two calls in a row.  The attention workgroups select their stream's pages from
 * the page scores themselves, which saves the launch that orders the scores.
 *   q, bounds, K, vpacked, mask, tok_off, k_pages, out: as in the two calls
 *   page_idx [B, Hkv, k_pages] int32, out: the selected pages, ascending (required)
 *   ws       stc_workspace_bytes(shape, STC_WS_STEP, k_pages) bytes
 */
int stc_decode_step(const stc_shape_t *shape, const void *q, const void *bounds, const void *K,
                    const void *vpacked, const uint16_t *mask, const uint32_t *tok_off,
                    int k_pages, int32_t *page_idx, float *out, void *ws, size_t ws_bytes,
                    void *stream);

/*
 * stc_decode_step for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same
 * kernels and the same results bit for bit; the page scores and split partials live in a
 * scratch array that is part of the library's device image (STC_STATIC_SCRATCH_BYTES per GPU
 * the library runs on, held until the process ends).  The call allocates and frees nothing;
 * its first call on a device looks the array's address up (make that call outside a graph
 * capture).
 *   arguments as stc_decode_step, without ws / ws_bytes
 *   STC_ERR_WORKSPACE if stc_workspace_bytes(shape, STC_WS_STEP, k_pages) exceeds
 *   STC_STATIC_SCRATCH_BYTES (nothing is enqueued); STC_ERR_LAUNCH if the address look-up fails.
 * All calls on one GPU share that GPU's array: two calls whose work overlaps in time (different
 * streams, or threads) race on it; calls on one stream are ordered and safe.  Nothing in the
 * array needs to start at zero: every byte a step reads it has written before.
 */
#define STC_STATIC_SCRATCH_BYTES (8 * 1024 * 1024)
int stc_decode_step_static(const stc_shape_t *shape, const void *q, const void *bounds,
                           const void *K, const void *vpacked, const uint16_t *mask,
                           const uint32_t *tok_off, int k_pages, int32_t *page_idx, float *out,
                           void *stream);

/*
 * Routed decode attention with an uncompressed tail of recent tokens: the tokens generated
 * since the cache was built (the paper leaves query-region tokens uncompressed, Sec. 3.4)
 * are kept with full-width values in a small dense store and are always attended, next to
 * the selected pages of the compressed cache, under one softmax.  Everything else as
 * stc_decode_attention.
 *   K_tail, V_tail [B, Hkv, tail_cap, D] bf16, in: rows 0 .. n_tail-1 of every stream are
 *            attended (0 <= n_tail <= tail_cap; may be NULL when n_tail == 0);
 *            tail_cap*D*2 bytes must stay below 4 GiB
 *   ws       stc_workspace_bytes(shape, STC_WS_ATTENTION_TAIL, k_pages + ceil(n_tail/P))
 */
int stc_decode_attention_tail(const stc_shape_t *shape, const void *q, const void *K,
                              const void *vpacked, const uint16_t *mask, const uint32_t *tok_off,
                              const int32_t *page_idx, int k_pages, const void *K_tail,
                              const void *V_tail, int n_tail, int tail_cap, float *out, void *ws,
                              size_t ws_bytes, void *stream);

/*
 * stc_decode_step with the uncompressed tail of stc_decode_attention_tail: the same results bit
 * for bit as stc_select_pages followed by stc_decode_attention_tail.
 *   ws       stc_workspace_bytes(shape, STC_WS_STEP_TAIL, k_pages + ceil(n_tail/P)) bytes, the
 *            second argument at its largest (as for STC_WS_ATTENTION_TAIL)
 */
int stc_decode_step_tail(const stc_shape_t *shape, const void *q, const void *bounds,
                         const void *K, const void *vpacked, const uint16_t *mask,
                         const uint32_t *tok_off, int k_pages, const void *K_tail,
                         const void *V_tail, int n_tail, int tail_cap, int32_t *page_idx,
                         float *out, void *ws, size_t ws_bytes, void *stream);

/*
 * Per-step append: writes the new token's key and value of every stream (k_new, v_new
 * [B, Hkv, D] bf16) to row n_tail of K_tail / V_tail (n_tail < tail_cap); the caller then
 * attends n_tail + 1 tail tokens.  Moving old tail tokens into the compressed cache (routing
 * and packing them) is a cache-construction step and not done here.
 */
int stc_append_tail(const stc_shape_t *shape, const void *k_new, const void *v_new, void *K_tail,
                    void *V_tail, int n_tail, int tail_cap, void *stream);

/*
 * Per-query-head page selection and attention: the other reading of Quest under grouped-query
 * attention.  Every query head scores the pages with its own upper bound U_h[p] (no maximum
 * over the heads of its KV head), keeps its own k pages, and attends them; heads of one KV
 * head then read that head's cache independently (pages chosen by several heads are read
 * once per head).  For Hq == Hkv both calls equal stc_select_pages / stc_decode_attention.
 *   page_idx   [B, Hq, k_eff] int32;  page_score [B, Hq, NP] float (may be NULL)
 *   ws         stc_workspace_bytes(shape, STC_WS_SELECT_PER_HEAD / STC_WS_ATTENTION_PER_HEAD,
 *              k_pages); B*Hq must not exceed 65535 for the attention call.
 * Everything else as in the calls they mirror.
 */
int stc_select_pages_per_head(const stc_shape_t *shape, const void *q, const void *bounds,
                              int k_pages, int32_t *page_idx, float *page_score, void *ws,
                              size_t ws_bytes, void *stream);
int stc_decode_attention_per_head(const stc_shape_t *shape, const void *q, const void *K,
                                  const void *vpacked, const uint16_t *mask,
                                  const uint32_t *tok_off, const int32_t *page_idx, int k_pages,
                                  float *out, void *ws, size_t ws_bytes, void *stream);

/*
 * Moves the oldest n_flush tokens of the uncompressed tail into the compressed cache, in
 * place: they become tokens N .. N+n_flush-1 of every stream (N = shape->N, the count before
 * the call; N + n_flush <= N_cap).  Keys are copied, values are routed and packed behind the
 * stream's packed store, tok_off[N+1 .. N+n_flush] continue from tok_off[N], and the bounds of
 * every page holding a new token are recomputed.  The arrays then equal, bit for bit, what
 * cache construction over all N + n_flush tokens writes.  The rows that stay in the tail
 * (n_flush .. n_tail-1) are moved to its front; the caller continues with shape->N + n_flush
 * cached and n_tail - n_flush tail tokens.
 *   K_tail, V_tail [B, Hkv, tail_cap, D] bf16, in/out: rows 0 .. n_flush-1 are moved into the
 *            cache, rows n_flush .. n_tail-1 to rows 0 .. (1 <= n_flush <= n_tail <= tail_cap)
 *   mode     STC_ROUTE_MASK (mask_in [B, Hkv, n_flush]) or STC_ROUTE_TOPK (logits
 *            [B, Hkv, n_flush, G], kcount [B, Hkv, n_flush] or fixed_k), as in
 *            stc_route_and_pack_values; a global budget cannot be continued
 *   K, bounds, mask, tok_off, vpacked, dev_status: the cache arrays, updated in place
 */
int stc_flush_tail(const stc_shape_t *shape, void *K_tail, void *V_tail, int n_flush, int n_tail,
                   int tail_cap, int mode, const float *logits, const uint8_t *kcount,
                   int fixed_k, const uint16_t *mask_in, void *K, void *bounds, uint16_t *mask,
                   uint32_t *tok_off, void *vpacked, int32_t *dev_status, void *stream);

/*
 * Per-query-head selection without reading a page once per head: stc_union_pages merges the
 * page lists of the query heads of every KV head into one ascending list plus, per page, the
 * set of heads that selected it; stc_decode_attention_union attends that list with all heads
 * of the group sharing every K page and V run, a head giving no weight to the tokens of pages
 * it did not select.  The output equals stc_decode_attention_per_head up to rounding.
 *   page_idx_per_head [B, Hq, k_pages] int32, in: ascending lists (as written by
 *               stc_select_pages_per_head)
 *   union_idx   [B, Hkv, union_cap] int32, out: selected pages ascending, then -1
 *   union_heads [B, Hkv, union_cap] uint16, out: bit r = head r of the group selected the page
 *   union_cap   >= min(NP, (Hq/Hkv) * k_pages) and <= NP; (Hq/Hkv) * k_pages <= 16384
 *   ws          stc_workspace_bytes(shape, STC_WS_ATTENTION, union_cap) bytes
 */
int stc_union_pages(const stc_shape_t *shape, const int32_t *page_idx_per_head, int k_pages,
                    int32_t *union_idx, uint16_t *union_heads, int union_cap, void *stream);
int stc_decode_attention_union(const stc_shape_t *shape, const void *q, const void *K,
                               const void *vpacked, const uint16_t *mask,
                               const uint32_t *tok_off, const int32_t *union_idx,
                               const uint16_t *union_heads, int union_cap, float *out, void *ws,
                               size_t ws_bytes, void *stream);

/*
 * Value-group router (App. B.1: the S group logits of a token are one learned linear map of
 * its hidden state at the layer input), for feeding stc_route_and_pack_values:
 *   logits[b, kvh, t, g] = sum_c h[b, t, c] * W[g, c] (+ bias[g]), the same for every kvh
 *   (the router gives one mask per token and layer).  With Hkv = 1 a single copy is written,
 *   for stc_route_and_pack_values with STC_ROUTE_SHARED.
 * Float arithmetic in a fixed order, because masks are decided on these numbers: chunks of
 * 128 adjacent channels are summed as a balanced tree over adjacent channels, chunk sums are
 * accumulated left to right, the bias is added last.
 *   h      [B, N, d_model] bf16, in; d_model a multiple of 128
 *   W      [G, d_model] bf16, in; G in {1, 2, 4, 8, 16}
 *   bias   [G] float (bias_per_batch == 0) or [B, G] float (bias_per_batch == 1), in, may be
 *          NULL.  The per-element form carries the query term of the LLM setting's router
 *          (Sec. 3.4: the group scores are a function of the token state and a summary s_Q of
 *          the query region; for one linear map of the two, W [h; s_Q] + b = W_h h + (W_q s_Q +
 *          b), the bracket is one vector per batch element: this routine on the summaries,
 *          N = 1, gives it)
 *   logits [B, Hkv, N, G] float, out
 * An element of h or W that is subnormal as bf16 (|x| < 2^-126) counts as zero; products must
 * stay finite in float.
 */
int stc_router_logits(int32_t B, int32_t Hkv, int32_t N, int32_t d_model, int32_t G,
                      const void *h, const void *W, const float *bias, int32_t bias_per_batch,
                      float *logits, void *stream);

/*
 * Token-level compaction helper for caches reduced by a visual-token method
 * (Stage I for VLMs, Sec. 3.2: only the retained tokens stay in the cache).
 * Gathers rows of a [B, Hkv, N_src, D] bf16 tensor:
 *   dst[b, h, i, :] = src[b, h, token_idx[b, i], :],  i < n_keep.
 *   token_idx [B, n_keep] int32, in; an index outside [0, N_src) writes a zero
 *             row and sets *dev_status (device int32, may be NULL) to 1.
 */
int stc_compact_tokens(const void *src, const int32_t *token_idx, void *dst, int32_t B,
                       int32_t Hkv, int32_t N_src, int32_t n_keep, int32_t D,
                       int32_t *dev_status, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* STC_H */
