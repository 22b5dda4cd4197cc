/*
 * citrus.h - C ABI of the CItruS chunk-eviction hot path for AMD MI355X (gfx950).
 *
 * CItruS = Chunked Instruction-aware State Eviction (arXiv 2406.12018).  A long
 * document is read chunk by chunk against a bounded key/value cache; after each
 * chunk the cache is cut back to its budget k by keeping the states with the
 * highest attention-based importance.  This library implements the per-chunk,
 * per-layer step of that procedure for all (document, layer, head) units at
 * once:
 *
 *   citrus_chunk_attn       the chunk's queries attend causally over
 *                           [retained cache ; chunk]            (Section 4.1, step 1)
 *   citrus_instr_score      the instruction's queries attend over the same
 *                           keys; softmax weights are summed per key
 *                                                               (Eq. (1) with s = I, Section 4.2)
 *   citrus_topk_select      keep the k highest scores           (Eq. (2)-(3), (4)-(5))
 *   citrus_kv_compact       gather the kept K/V rows into the new cache
 *                                                               (Eq. (3), (5))
 *   citrus_process_document the chunk loop around those four    (Section 4.1 "Overall
 *                                                               process", Section 4.3)
 *
 * General rules, valid for every entry point
 * ------------------------------------------
 * Memory.  Every pointer is a DEVICE pointer unless its comment says "host".
 *   The caller owns all buffers, including the workspace; the library allocates
 *   and frees no device memory.  The only state it keeps between calls is, per
 *   device, the dynamic-LDS limits it has raised for its kernels, the device's
 *   number of compute units and the address of its static scratch array (see
 *   citrus_evict_cache_static); all are atomics, so host threads may call any
 *   entry point concurrently.
 * Tensors.  A citrus_tensor is a base pointer plus ELEMENT strides for the
 *   document (b), layer (l), head (h) and sequence (s) axes; the head_dim axis is
 *   contiguous (stride 1).  Rows (one head_dim vector) must start on a 16-byte
 *   boundary, i.e. ptr is 16-byte aligned and every stride is a multiple of
 *   8 (bf16) or 4 (f32) elements.  Element type is citrus_config.dtype.
 *   The rows of one (b, l, h) unit that a call touches must span less than
 *   2 GiB ((rows - 1) * stride_s + head_dim elements): the kernels address a
 *   unit's rows with 32-bit byte offsets.  Larger spans: CITRUS_ERR_SHAPE.
 *   bf16 is the 16-bit brain-float, stored as its raw bits.
 * Heads.  Query head h reads KV head h / G with G = q_heads / kv_heads
 *   (contiguous groups).
 * Candidates.  The keys a step works on are the concatenation
 *   [cache rows 0..cache_len-1 ; chunk rows 0..chunk_len-1]; n = cache_len +
 *   chunk_len.  Candidate index j < cache_len is cache row j, otherwise chunk
 *   row j - cache_len.
 * Streams.  hip_stream is a hipStream_t (NULL = the default stream).  Calls
 *   only enqueue work and return; results are valid once the stream has been
 *   synchronised by the caller.  No call synchronises the device.
 * Capture.  A call enqueues kernel launches only (plus, with a side stream, one
 *   event record / wait pair per step), so it may be made while hip_stream is
 *   being captured into a HIP graph, citrus_process_document with the resident
 *   provider included.  The first call that reaches a kernel on a device raises
 *   that kernel's dynamic-LDS limit (and citrus_evict_cache_static looks up its
 *   array): make one eager call of the same shape on the device before capturing.
 * Errors.  Every entry point returns a citrus_status.  Arguments are validated
 *   on the host before anything is launched; on a validation error nothing is
 *   launched and outputs are untouched.  A failed launch maps to
 *   CITRUS_ERR_DEVICE.  Nothing throws or aborts across this boundary.
 * Determinism.  No floating-point atomics are used anywhere: the same inputs
 *   give bit-identical outputs from run to run.
 * Concurrency.  Calls that share a workspace or an output buffer must be
 *   ordered on one stream (or by the caller); otherwise calls are independent.
 */
#ifndef CITRUS_H
#define CITRUS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CITRUS_ABI_VERSION 10
#define CITRUS_EVENTS_PER_STEP 8

typedef enum {
  CITRUS_OK = 0,
  CITRUS_ERR_NULL = 1,        /* a required pointer is NULL                          */
  CITRUS_ERR_SHAPE = 2,       /* sizes/strides inconsistent or out of range          */
  CITRUS_ERR_UNSUPPORTED = 3, /* dtype / head_dim / mode not implemented             */
  CITRUS_ERR_WORKSPACE = 4,   /* workspace NULL or smaller than citrus_workspace_bytes */
  CITRUS_ERR_DEVICE = 5,      /* the HIP runtime reported an error at launch         */
  CITRUS_ERR_PROVIDER = 6     /* the chunk provider returned a negative value        */
} citrus_status;

typedef enum { CITRUS_F32 = 0, CITRUS_BF16 = 1 } citrus_dtype;

/* Cache designs of Section 4.2.  INSTR and SHARED run the same kernel sequence
 * on one cache that the chunk attends over and the instruction scores (with
 * layer-independent synthetic inputs there is no separate language-modelling
 * cache to differ from); DUAL keeps a language-modelling cache, scored by the
 * chunk's own attention (Eq. (1) with s = chunk), next to the instruction cache.
 * STANDARD is the Standard CSE process of Section 4.1 on its own: one cache
 * (budget `budget`), evicted by the document's chunks; the instruction takes no
 * part in the loop, and the extra eviction by the instruction after the last
 * chunk is citrus_evict_cache. */
typedef enum {
  CITRUS_CACHE_INSTR = 0,
  CITRUS_CACHE_SHARED = 1,
  CITRUS_CACHE_DUAL = 2,
  CITRUS_CACHE_STANDARD = 3
} citrus_cache_mode;

/* How the cache that the document's own chunks evict (the language-modelling cache of DUAL, the only cache
 * of STANDARD; budget_lm reads budget for the latter) is evicted.
 * SCORE_AFTER_APPEND: the chunk's own causal attention scores [cache ; chunk] in the step that encodes it.
 * EVICT_THEN_APPEND:  the three steps of Section 4.1 in the order printed: the chunk is encoded given the
 *   cache (which still holds the whole previous chunk: up to budget_lm + chunk_len states), the states of
 *   the cache are scored by Eq. (1) with s = the chunk and the softmax normalised over the cache states
 *   only, the budget_lm best stay, and then all states of the chunk are put into the cache.
 * The instruction cache is the same computation in both orderings (hoisted by one step). */
typedef enum { CITRUS_LM_SCORE_AFTER_APPEND = 0, CITRUS_LM_EVICT_THEN_APPEND = 1 } citrus_lm_ordering;

/* What the selection of the instruction-scored cache ranks.
 * PER_STEP:    this step's Eq. (1) score (the paper's method).
 * ACCUMULATED: the sum of the Eq. (1) scores a state has received from the instruction in every step since
 *              it entered the cache: the accumulative-attention rule of H2O that Section 5.2 ("Baselines")
 *              combines with the instruction-aware cache ("H2O + Shared Cache").  INSTR / SHARED only. */
typedef enum { CITRUS_SCORE_PER_STEP = 0, CITRUS_SCORE_ACCUMULATED = 1 } citrus_score_mode;

/* PER_KV_HEAD: one index set per (document, layer, KV head).
 * PER_LAYER:   scores of all KV heads are added first and one index set is used
 *              by the whole layer (the layer-wise eviction of Section 4.1).     */
typedef enum { CITRUS_SELECT_PER_KV_HEAD = 0, CITRUS_SELECT_PER_LAYER = 1 } citrus_select_mode;

/* Plain data, passed by pointer, read during the call only. */
typedef struct {
  int32_t batch;          /* B  documents                                    >= 1 */
  int32_t layers;         /* L                                               >= 1;  B*L <= 65535 */
  int32_t q_heads;        /* Hq, a multiple of kv_heads, <= 65535; and B*L*Hq*ceil(max(chunk_len, instr_len)/32)
                             < 2^28 (the largest launch: 8 workgroups per 32 rows of a head); else CITRUS_ERR_SHAPE */
  int32_t kv_heads;       /* Hkv                                             >= 1 */
  int32_t head_dim;       /* d: 64 or 128.  The matrix-core (MFMA) kernels exist for bf16 with d = 128 only;
                             bf16 with d = 64 and every f32 configuration run on plain vector kernels (one
                             wavefront per query row), which are meant for tests and small shapes        */
  int32_t chunk_len;      /* l_s: maximum chunk length c                     >= 1 */
  int32_t budget;         /* k: states kept in the (instruction) cache       >= 1 */
  int32_t budget_lm;      /* DUAL: budget of the language-modelling cache; else ignored */
  int32_t instr_len;      /* n_i: instruction tokens                         >= 1 */
  int32_t cache_capacity; /* rows per head of every cache buffer, >= max(budget, budget_lm) */
  int32_t dtype;          /* citrus_dtype                                        */
  int32_t cache_mode;     /* citrus_cache_mode                                   */
  int32_t select_mode;    /* citrus_select_mode                                  */
  int32_t start_size;     /* leading document states that are never evicted (appendix "Analysis on
                             initial tokens"); 0 = plain Eq. (2)-(3); < budget (and < budget_lm)  */
  int32_t lm_ordering;    /* citrus_lm_ordering (DUAL, STANDARD); EVICT_THEN_APPEND needs cache_capacity >=
                             budget_lm + chunk_len (DUAL) or budget + chunk_len (STANDARD)             */
  int32_t score_mode;     /* citrus_score_mode                                   */
  int32_t position_shift; /* 0 / 1: the position shift of Section 5.3 in the chunk loop (INSTR / SHARED / DUAL):
                             the provider hands over q, k and q_instr WITHOUT rotary embedding and every step
                             rotates them to the positions of the cache (see citrus_rope); with DUAL each of
                             the two caches has its own slots                                          */
  float rope_base;        /* base of the rotary frequencies; 0 -> 10000                                */
  float softmax_scale;    /* 0 -> 1/sqrt(head_dim), the scaling of Eq. (1)       */
} citrus_config;

typedef struct {
  void* ptr;
  int64_t stride_b, stride_l, stride_h, stride_s; /* in elements */
} citrus_tensor;

/* Bytes of workspace that is enough for any entry point under this
 * configuration (0 if cfg is NULL or invalid). */
size_t citrus_workspace_bytes(const citrus_config* cfg);

/* Static, NUL-terminated description of a status code (host pointer). */
const char* citrus_status_string(int32_t status);

int32_t citrus_abi_version(void);

/*
 * Chunk attention (Section 4.1, step 1: "encode the current text chunk given
 * the cache"; softmax and 1/sqrt(d_k) scaling as written inside Eq. (1)).
 *
 *   out[b,l,h,t,:] = sum_j softmax_j( scale * q[b,l,h,t,:] . Kcat[b,l,h/G,j,:] ) * Vcat[b,l,h/G,j,:]
 *   over candidates j <= cache_len + t (the whole cache and the causal prefix
 *   of the chunk).
 *
 * q, out      [B, L, Hq, chunk_len, d]
 * k_cache, v_cache [B, L, Hkv, >= cache_len, d]   (ptr may be NULL iff cache_len == 0)
 * k_chunk, v_chunk [B, L, Hkv, chunk_len, d]
 * cache_len   0 .. cfg->cache_capacity;  chunk_len 1 .. cfg->chunk_len
 * lse         optional, dense [B, L, Hq, chunk_len] f32: log-sum-exp of each
 *             row's scaled logits over the candidates it sees
 * lse_cache   optional (cache_len >= 1), dense [B, L, Hq, chunk_len] f32: the same
 *             over the cache states alone, i.e. the normaliser of Eq. (1) as
 *             printed; citrus_cache_score takes it.  A by-product of the bf16
 *             d=128 kernel when cache_len is a multiple of 32, else one more pass.
 * lm_score    optional, dense [B, L, Hkv, n] f32: chunk-scored importance,
 *             lm_score[b,l,g,j] = sum over heads h of group g and chunk rows t
 *             of the attention probability p[h,t,j] (0 where masked); Eq. (1)
 *             with s = the chunk, as a sum (divide by chunk_len*G for the mean).
 *             Needs lse: if lse is NULL the workspace is used for it.
 * Compute: bf16 inputs, f32 accumulation, probabilities rounded to bf16 before
 * the P.V product, bf16 output; f32 mode computes in f32 throughout.
 */
int32_t citrus_chunk_attn(const citrus_config* cfg, citrus_tensor q, citrus_tensor k_cache, citrus_tensor v_cache,
                          int32_t cache_len, citrus_tensor k_chunk, citrus_tensor v_chunk, int32_t chunk_len,
                          citrus_tensor out, float* lse, float* lse_cache, float* lm_score, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/*
 * Instruction-aware importance (Eq. (1) with the instruction I in the role of
 * the chunk: Imp(I, c^I) / Imp(I, c) of Section 4.2), as a sum:
 *
 *   score[b,l,g,j] = sum_{h in group g} sum_{u < instr_len}
 *                    softmax_j( scale * q_instr[b,l,h,u,:] . Kcat[b,l,g,j,:] )
 *
 * with the softmax over all n candidates, no mask.  Each row of score sums to
 * instr_len * G; Imp = score / (instr_len * G).
 *
 * q_instr [B, L, Hq, instr_len, d];  K segments as in citrus_chunk_attn.
 * score   dense [B, L, Hkv, n] f32.
 * workspace: >= citrus_workspace_bytes(cfg).
 */
int32_t citrus_instr_score(const citrus_config* cfg, citrus_tensor q_instr, citrus_tensor k_cache, int32_t cache_len,
                           citrus_tensor k_chunk, int32_t chunk_len, float* score, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

/*
 * Importance of the cache states exactly as Eq. (1) prints it: attention of the rows of q to the states of
 * the cache, softmax normalised over the cache states alone, summed over the rows and over the query heads of
 * each KV group (divide by rows*G for the mean):
 *   score[b,l,g,j] = sum_{h in g} sum_{t < rows} softmax_{j' < cache_len}(scale * q[b,l,h,t,:] . K[b,l,g,j',:])_j
 * Used with q = the chunk's queries by the EVICT_THEN_APPEND ordering (Section 4.1, step 2) and with q = the
 * instruction's queries by the extra eviction after the last chunk; every row sees the whole cache, so there
 * is no mask.
 *
 * q       [B, L, Hq, rows, d]; rows >= 1 and at most cfg->instr_len, or at most cfg->chunk_len when the
 *         configuration runs a cache in the EVICT_THEN_APPEND order (the workspace is sized by these);
 *         more rows: CITRUS_ERR_SHAPE
 * k_cache [B, L, Hkv, >= cache_len, d], 1 <= cache_len <= cfg->cache_capacity
 * lse_cache optional, dense [B, L, Hq, rows] f32: the rows' log-sum-exp over the cache states, as
 *         citrus_chunk_attn returns it for the same q and cache; then only the column sums are computed
 *         (one pass over the keys instead of two), no workspace is needed and rows may go up to
 *         max(chunk_len, instr_len) in any configuration
 * score   dense [B, L, Hkv, cache_len] f32
 * workspace: >= citrus_workspace_bytes(cfg) (may be NULL when lse_cache is given).
 */
int32_t citrus_cache_score(const citrus_config* cfg, citrus_tensor q, int32_t rows, citrus_tensor k_cache,
                           int32_t cache_len, const float* lse_cache, float* score, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

/*
 * One eviction of a cache by a text (Section 4.1 step 2; with the instruction as the text: the additional
 * eviction after the last chunk, which removes the bias towards that chunk and leaves the k states the
 * instruction and the response are encoded with): citrus_cache_score of q over the cache, selection of the
 * min(k, cache_len) best as in citrus_topk_select (cfg->select_mode, cfg->start_size), and the kept K/V rows
 * written to k_new / v_new rows 0 .. min(k, cache_len)-1 in their order, as in citrus_kv_compact.  A cache
 * of at most k states is copied whole.
 *
 * q, rows, k_cache, cache_len   as in citrus_cache_score; v_cache like k_cache
 * k       1 .. cfg->budget
 * k_new, v_new [B, L, Hkv, >= min(k, cache_len), d]; must not overlap the sources
 * idx     optional dense int32 [B, L, Hsel, k]: the kept positions (NULL: kept in the workspace only)
 */
int32_t citrus_evict_cache(const citrus_config* cfg, citrus_tensor q, int32_t rows, citrus_tensor k_cache,
                           citrus_tensor v_cache, int32_t cache_len, int32_t k, citrus_tensor k_new,
                           citrus_tensor v_new, int32_t* idx, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * citrus_evict_cache for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical results; the partial softmax sums, the scores and (with idx == NULL) the kept positions live
 * in a fixed array of citrus_static_scratch_bytes() bytes (16 MiB) inside the library's device image instead
 * of a workspace.  Every GPU the library runs on holds its own copy of that array until the process ends.
 * The call allocates and frees nothing and synchronises nothing.  Its need,
 *   max(B*L*Hq*rows*64, S) + B*L*Hkv*cache_len*4 + B*L*Hsel*k*4 bytes (each term rounded up to 256), with
 *   S = B*L*Hkv*ceil(G*r/32)*min(cache_len, 2560)*8, the partial sums of the row strips of a small launch:
 *   r = the largest row count <= rows with G*r <= 512 and B*L*Hkv*ceil(G*r/64) <= 608 (S = 0 if there is none),
 * must fit the array, else CITRUS_ERR_WORKSPACE (nothing is launched; use citrus_evict_cache).
 * The array keeps the previous call's contents and every part a call reads is written by that call first.
 * All calls on one GPU share the array: two calls that overlap in time on one GPU (different streams or
 * host threads) race; order them on one stream or with events.
 */
size_t citrus_static_scratch_bytes(void);
int32_t citrus_evict_cache_static(const citrus_config* cfg, citrus_tensor q, int32_t rows, citrus_tensor k_cache,
                                  citrus_tensor v_cache, int32_t cache_len, int32_t k, citrus_tensor k_new,
                                  citrus_tensor v_new, int32_t* idx, void* hip_stream);

/*
 * Rotary position embedding at explicit positions (the position shift mechanism of Section 5.3,
 * "Hyperparameters": the cache always uses the same positional embeddings, so a state's position is its
 * slot in the cache and not its place in the document).  Convention of the Llama / Mistral models:
 * pairs (i, i + d/2), angle a = (pos0 + s) * rope_base^(-2 i / d):
 *   y[b,l,h,s,i]       = x[b,l,h,s,i] cos a - x[b,l,h,s,i+d/2] sin a
 *   y[b,l,h,s,i+d/2]   = x[b,l,h,s,i+d/2] cos a + x[b,l,h,s,i] sin a        for h < heads, s < rows
 * x, y  [B, L, heads, >= rows, d]; y may be x itself (in place) but must not overlap it otherwise
 * heads 1 .. 65535;  rows >= 0;  pos0 >= 0
 * bf16: f32 arithmetic, result rounded to bf16; f32: angles and products in f64.
 * With cfg->position_shift the chunk loop applies it, every step, to the candidates [cache ; chunk]
 * (position = index j), to the chunk's queries (cache_len + t) and to the instruction's queries
 * (cache_len + chunk_len + u), for each cache with that cache's own length; the caches keep the unrotated keys.
 */
int32_t citrus_rope(const citrus_config* cfg, citrus_tensor x, int32_t heads, int32_t rows, int32_t pos0,
                    citrus_tensor y, void* hip_stream);

/*
 * One decoding step of the response over the retained states (Section 4.3: the k states left by the last
 * eviction encode the instruction and the response; nothing is evicted while the response is generated).
 * The new token's key and value become row cache_len of the cache and its query attends over rows
 * 0 .. cache_len (softmax with the scaling of Eq. (1)):
 *   out[b,l,h,0,:] = softmax_j(scale * q[b,l,h,0,:] . K[b,l,h/G,j,:]) . V[b,l,h/G,j,:],  j <= cache_len
 *
 * q              [B, L, Hq, 1, d]
 * k_new, v_new   [B, L, Hkv, 1, d]: the token's own state
 * k_cache, v_cache [B, L, Hkv, >= cache_len + 1, d], in/out: rows 0 .. cache_len-1 are read, row cache_len
 *                is written with k_new / v_new (bit copies); 0 <= cache_len < cfg->cache_capacity.
 *                The caller's cache length becomes cache_len + 1.
 * out            [B, L, Hq, 1, d]
 * workspace      >= citrus_workspace_bytes(cfg)
 */
int32_t citrus_decode_step(const citrus_config* cfg, citrus_tensor q, citrus_tensor k_new, citrus_tensor v_new,
                           citrus_tensor k_cache, citrus_tensor v_cache, int32_t cache_len, citrus_tensor out,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The two steps of the ACCUMULATED score mode around the selection (Section 5.2, H2O's accumulative
 * attention score on the instruction-aware cache):
 *   citrus_score_accumulate  score[b,l,g,j] += acc[b,l,g,j] for j < cache_len: a cache state's sum so far is
 *                            added to this step's score; candidates from the chunk start at their own score.
 *   citrus_score_gather      acc_new[b,l,g,r] = score[b,l,g, idx[b,l,g',r]] for r < m: the kept states carry
 *                            their sums on (g' = g, or 0 for PER_LAYER, as in citrus_kv_compact).
 * score    dense [B, L, Hkv, n] f32 (in/out for accumulate), 1 <= n <= cache_capacity + chunk_len
 * acc, acc_new  dense [B, L, Hkv, cfg->cache_capacity] f32, distinct buffers; 0 <= cache_len <= min(n, capacity)
 * idx      dense int32 with row pitch idx_pitch >= m, values in [0, n); 1 <= m <= cfg->cache_capacity
 */
int32_t citrus_score_accumulate(const citrus_config* cfg, float* score, int32_t n, const float* acc,
                                int32_t cache_len, void* hip_stream);
int32_t citrus_score_gather(const citrus_config* cfg, const float* score, int32_t n, const int32_t* idx,
                            int32_t idx_pitch, int32_t m, float* acc_new, void* hip_stream);

/*
 * Selection (Eq. (2)-(3)): the positions of the min(k, n) highest scores.
 * Equal scores: the lower position wins.  Output positions are ascending, so
 * kept states stay in their original order.  n <= k keeps everything
 * (0..n-1), as the first chunk does in the paper.  With cfg->start_size = s > 0
 * (appendix "Analysis on initial tokens") and n > k, candidates 0..min(s,k)-1 are
 * always kept and the other places go to the best of the remaining candidates.
 *
 * score dense [B, L, Hkv, n] f32 (finite values).
 * idx   dense int32, row pitch k:  [B, L, Hkv, k] (PER_KV_HEAD) or [B, L, 1, k]
 *       (PER_LAYER, scores added over Hkv in head order first).  Entries
 *       min(k,n).. of a row are left untouched.
 * n >= 1, k >= 1.  No workspace needed (arguments kept for symmetry; may be NULL/0).
 */
int32_t citrus_topk_select(const citrus_config* cfg, const float* score, int32_t n, int32_t k, int32_t* idx,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Compaction (Eq. (3), (5): the evicted cache holds exactly the selected
 * states):  k_new[b,l,g,r,:] = Kcat[b,l,g, idx[b,l,g',r], :], same for V, for
 * r < m, where g' = g (PER_KV_HEAD) or 0 (PER_LAYER).  Bit copies.
 *
 * idx   dense int32 with row pitch idx_pitch (>= m), values in [0, n).
 * m     rows to write per head, 1 .. cfg->cache_capacity.
 * k_new, v_new [B, L, Hkv, >= m, d]; must not overlap any source.
 */
int32_t citrus_kv_compact(const citrus_config* cfg, citrus_tensor k_cache, citrus_tensor v_cache, int32_t cache_len,
                          citrus_tensor k_chunk, citrus_tensor v_chunk, int32_t chunk_len, const int32_t* idx,
                          int32_t idx_pitch, int32_t m, citrus_tensor k_new, citrus_tensor v_new, void* hip_stream);

/* One chunk's tensors, filled in by the provider. */
typedef struct {
  citrus_tensor q;       /* [B, L, Hq,  chunk_len, d]                         */
  citrus_tensor k, v;    /* [B, L, Hkv, chunk_len, d]                         */
  citrus_tensor q_instr; /* [B, L, Hq,  instr_len, d] instruction queries for this step */
  citrus_tensor out;     /* [B, L, Hq,  chunk_len, d] where to write the attention output */
  int32_t chunk_len;     /* 1 .. cfg->chunk_len (the last chunk may be short)  */
} citrus_chunk_io;

/* Host callback.  Must fill *io for chunk `chunk_index` (buffers valid on
 * hip_stream until the stream has passed this step) and return 0; return 1
 * for "no more chunks", a negative value to abort. */
typedef int32_t (*citrus_chunk_provider)(void* user, int32_t chunk_index, void* hip_stream, citrus_chunk_io* io);

/* A ready-made provider for documents that are resident in device memory:
 * pass citrus_resident_provider as `next` and a (host) pointer to this struct
 * as `user`.  Chunk i covers document positions i*chunk_len .. min(doc_len,
 * (i+1)*chunk_len)-1. */
typedef struct {
  citrus_tensor q;       /* [B, L, Hq,  doc_len, d]                            */
  citrus_tensor k, v;    /* [B, L, Hkv, doc_len, d]                            */
  citrus_tensor out;     /* [B, L, Hq,  doc_len, d]                            */
  citrus_tensor q_instr; /* [B, L, Hq,  instr_len, d] for chunk 0 ...          */
  int64_t q_instr_stride_chunk; /* ... plus this many elements per chunk (0 = same queries every chunk) */
  int32_t doc_len;
  int32_t chunk_len;     /* must equal cfg->chunk_len                          */
  int32_t dtype;         /* citrus_dtype of the tensors (must equal cfg->dtype) */
} citrus_resident_doc;
int32_t citrus_resident_provider(void* user, int32_t chunk_index, void* hip_stream, citrus_chunk_io* io);

/*
 * The chunk loop (Section 4.1 "Overall process", Section 4.3).  For chunk
 * index i = first_chunk, first_chunk+1, ... until `max_chunks` steps are done
 * or the provider returns 1:
 *   INSTR / SHARED:  chunk_attn over [cache ; chunk] -> io.out;
 *                    instr_score over the same keys; topk_select(budget);
 *                    kv_compact into the other buffer of the ping-pong pair.
 *   DUAL:            chunk_attn (+ chunk-scored importance) over
 *                    [LM cache ; chunk], topk_select(budget_lm), kv_compact of
 *                    the LM pair; then instr_score / topk_select(budget) /
 *                    kv_compact on the instruction pair.
 *   DUAL with lm_ordering = EVICT_THEN_APPEND: chunk_attn over [LM cache ; chunk]
 *                    where the LM cache holds up to budget_lm + chunk_len states;
 *                    (with its cache-only log-sum-exp as a by-product);
 *                    cache_score of the chunk's queries over the LM cache alone,
 *                    topk_select(budget_lm) among its states, then the kept states
 *                    followed by all states of the chunk are written to the other LM
 *                    buffer (cache_len_lm grows to kept + chunk_len; no eviction
 *                    happens after the last chunk).  idx_history_lm then holds the
 *                    kept positions of the LM cache (not the appended chunk rows).
 *   INSTR / SHARED with score_mode = ACCUMULATED: score_accumulate between
 *                    instr_score and topk_select, score_gather next to kv_compact.
 *   INSTR / SHARED with position_shift: before these, rope of the cache keys
 *                    (position 0 ..), the chunk keys and queries (cache_len ..)
 *                    and the instruction queries (cache_len + chunk_len ..) into
 *                    the workspace; attention and scores read the rotated
 *                    copies, kv_compact gathers the unrotated keys.
 *   DUAL with position_shift: the same per cache.  The chunk's queries and the
 *                    candidates [LM cache ; chunk] are rotated to the LM cache's
 *                    positions (its state j -> j, chunk token t -> cache_len_lm + t)
 *                    for the attention and the chunk's scores; the candidates
 *                    [instruction cache ; chunk] and the instruction queries to the
 *                    instruction cache's (j, cache_len + chunk_len + u).
 *   STANDARD:        the language-modelling steps of DUAL (in either ordering) on
 *                    the only cache pair with budget `budget`; io.q_instr is not
 *                    read and may be NULL; idx_history holds its selections.
 * An empty cache (length 0) is the start of a document: the first chunk enters
 * whole if it fits the budget.
 *
 * k_cache[2], v_cache[2]        ping-pong buffers [B, L, Hkv, cache_capacity, d]
 *                               of the instruction (or only) cache
 * k_cache_lm[2], v_cache_lm[2]  DUAL only (else may be NULL pointers)
 * cache_len, cache_len_lm       host, in/out: valid rows on entry / on return
 *                               (cache_len_lm may be NULL unless DUAL)
 * buffer_index, buffer_index_lm host, in/out: which buffer of the pair is
 *                               current (0/1) on entry / on return.  Passing
 *                               the values a previous call returned, with the
 *                               same buffers, resumes a document bit-exactly.
 * acc_score[2]    score_mode = ACCUMULATED only (else may be NULL): two dense f32
 *                 buffers [B, L, Hkv, cache_capacity] holding the accumulated
 *                 scores of the cache rows; they follow buffer_index like
 *                 k_cache / v_cache and belong to the state a resume needs
 * idx_history     optional dense int32 [steps, B, L, Hsel, budget]: the
 *                 selection of every step done by this call (step 0 = chunk
 *                 first_chunk); Hsel = Hkv or 1 (PER_LAYER)
 * idx_history_lm  same for the LM cache with pitch budget_lm (DUAL)
 * chunks_done     host, optional: number of steps performed
 * phase_events    host, optional: array of hipEvent_t handles created by the
 *                 caller (with timing enabled), CITRUS_EVENTS_PER_STEP per step.
 *                 Step s records event [s*CITRUS_EVENTS_PER_STEP + p] on
 *                 hip_stream at these points: p=0 step start, 1 after chunk
 *                 attention, 2 after the chunk-scored importance, 3 after the
 *                 LM selection, 4 after the LM compaction (2..4 coincide with 1
 *                 unless DUAL), 5 after the instruction score, 6 after the
 *                 selection, 7 after the compaction.  A NULL entry is skipped (every
 *                 recorded event costs a few microseconds of stream time).  For
 *                 per-phase timing only.
 * side            optional (NULL: every launch goes to hip_stream in the order a1 .. a4).  A second stream
 *                 of the same device and two events, all created by the caller.  In the single-cache
 *                 modes (INSTR, SHARED) a step then runs its instruction score first, and its selection
 *                 and gather on side->stream NEXT TO its chunk attention on hip_stream: neither reads
 *                 what the other writes (the attention reads the current buffer of the pair and the
 *                 chunk, the gather writes the other buffer), and the gather's waves fit beside the
 *                 attention's on a compute unit.  fork_event orders the side stream behind the
 *                 instruction score, join_event orders hip_stream behind the gather before the next
 *                 step; on return everything the call enqueued is ordered before later work on
 *                 hip_stream.  Results are bit-identical with and without it.  Phase events 6 and 7 are
 *                 then recorded on the side stream and event 5 (after the instruction score) comes
 *                 before the attention: the attention launch is bracketed by events 5 and 1.  Other
 *                 cache modes ignore it.
 * No host/device synchronisation happens inside the loop.
 */
typedef struct citrus_side_stream {
  void* stream;     /* hipStream_t */
  void* fork_event; /* hipEvent_t */
  void* join_event; /* hipEvent_t */
} citrus_side_stream;

int32_t citrus_process_document(const citrus_config* cfg, citrus_chunk_provider next, void* user,
                                int32_t first_chunk, int32_t max_chunks,
                                const citrus_tensor* k_cache, const citrus_tensor* v_cache,
                                const citrus_tensor* k_cache_lm, const citrus_tensor* v_cache_lm,
                                int32_t* cache_len, int32_t* cache_len_lm,
                                int32_t* buffer_index, int32_t* buffer_index_lm,
                                float* const* acc_score,
                                int32_t* idx_history, int32_t* idx_history_lm, int32_t* chunks_done,
                                void* const* phase_events,
                                void* workspace, size_t workspace_bytes, void* hip_stream,
                                const citrus_side_stream* side);

/*
 * Measurement aid, not a step of the method: launches a kernel in which every wave (two workgroups of eight
 * waves per compute unit) issues 16 * iters independent v_mfma_f32_32x32x16_bf16 back to back and touches no
 * memory until the end; the caller times the launch (events on hip_stream) and divides.  bench.py reports the
 * rate it reaches next to the published bf16 peak.
 * iters       1 .. 2^20
 * sink        device, >= 1024 floats per compute unit (one value per lane is written so that the work is kept)
 * mfma_count  host, out: MFMA instructions the launch issues; each is 2 * 32 * 32 * 16 = 32768 flop
 */
int32_t citrus_probe_mfma(int32_t iters, float* sink, size_t sink_floats, int64_t* mfma_count, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CITRUS_H */
