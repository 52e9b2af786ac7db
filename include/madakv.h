/*
 * madakv.h - C ABI of the MadaKV eviction + ragged-decode hot path for one AMD
 * MI355X (gfx950).
 *
 * The calls follow the method of "MadaKV: Adaptive Modality-Perception KV Cache
 * Eviction" (arxiv 2506.15724), Section 3:
 *
 *   madakv_score          Sec. 3.3 Eq. 7 (proxy-token scores), Eq. 6 (modality
 *                         mass), Eq. 9 (theta-mass sparsity counts), plus score
 *                         pooling used for ranking only
 *   madakv_allocate       Sec. 3.3 Eq. 8 (per-head, per-modality budgets) and
 *                         Eq. 10-11 (layer compensation, budget recurrence)
 *   madakv_select_gather  Sec. 3.3, end of the MPA paragraph: per-head,
 *                         per-modality eviction; builds the reduced KV cache
 *   madakv_decode_attn    Sec. 3.1 Eq. 3-5: append K_t, V_t and attend over the
 *                         reduced cache
 *   madakv_evict          Sec. 3.3 Eq. 6-11 and the eviction itself: the first three calls in one
 *   madakv_score_lse      Sec. 3.3 Eq. 7 with the softmax normalisers of the proxy rows given
 *                         (the prefill attention of Sec. 3.1 Eq. 5 has them)
 *   madakv_window_attn_score  that prefill attention for the proxy rows (Sec. 3.1 Eq. 5) with Eq. 7, 6, 9 as
 *                         by-products of the same pass
 *
 * General rules
 *   - Plain C, no exceptions.  Every call returns a madakv_status (0 = OK).
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, contiguous,
 *     row-major in the stated shape.  Q/K/V-like tensors (q_win, k, v, k_c, v_c, q,
 *     k_new, v_new, out) and the workspaces must be aligned to 16 bytes; the other
 *     arrays to their element size (kv_off 8, float / int32 arrays and stats 4).
 *     The library never allocates, frees or keeps tensor memory.  A null or
 *     misaligned pointer gives MADAKV_ERR_INVALID_ARG; nothing is enqueued then.
 *   - All work is ordered on the caller's stream (a hipStream_t passed as void*, NULL = the
 *     null stream): it starts after what the stream held before the call and is complete, as far
 *     as the stream is concerned, before anything enqueued after it.  madakv_allocate
 *     and madakv_decode_attn enqueue on that stream only.  madakv_score, madakv_score_lse,
 *     madakv_select_gather and madakv_evict over four or more layers also use the handle's own
 *     stream for the per-head statistics / selection kernels of one layer group while another
 *     group is scored or gathered; that stream forks from and joins the caller's stream through
 *     events inside the call.  No call synchronises the device.
 *   - Arguments are validated on the host before anything is enqueued.  Errors
 *     found there leave all outputs untouched.
 *   - The handle belongs to the HIP device that was current in madakv_create; that device must
 *     be current in every later call on it.  It owns a few KB of device memory (carry state of
 *     the layer recurrence and cache cursors; with a paged cache its page table; for contexts of
 *     four or more 16384-token chunks on at most 128 heads per layer a few MB of histograms that
 *     the per-head statistics and selection kernels share between launches), a little pinned
 *     host memory, one extra stream of default priority and a few events.  Calls on one handle
 *     must not overlap.
 *   - Layers are addressed as a range [layer0, layer0 + n).  Tensor arguments hold
 *     only the n layers of the call, layer-major.  madakv_allocate and
 *     madakv_select_gather carry state from layer to layer and must be called in
 *     increasing layer order, starting at layer 0 (which resets the state).
 *   - Modality ids: 0 = text, 1 = image (2, 3: further modalities when n_modalities says so).
 *     Query head j reads KV head j / G,
 *     G = n_q_heads / n_kv_heads.
 */
#ifndef MADAKV_H
#define MADAKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MADAKV_OK = 0,
  MADAKV_ERR_INVALID_ARG = -1,        /* null / misaligned pointer, bad layer range, out of decode slack */
  MADAKV_ERR_BAD_SHAPE = -2,          /* n_q_heads % n_kv_heads, window > ctx_len, unsupported head_dim ... */
  MADAKV_ERR_BAD_BUDGET = -3,         /* budget <= window while budget < ctx_len */
  MADAKV_ERR_WORKSPACE_TOO_SMALL = -4,
  MADAKV_ERR_UNSUPPORTED_DTYPE = -5,
  MADAKV_ERR_HIP = -6,                /* see madakv_last_hip_error */
  MADAKV_ERR_UNIMPLEMENTED = -7
} madakv_status;

enum { MADAKV_FP32 = 0, MADAKV_BF16 = 1 };

/* Hyper-parameters and shapes.  The paper names the proxy-token count, theta and
 * the layer budget (Sec. 3.3) without giving values; they are set here. */
typedef struct {
  int32_t n_layers;        /* 1 .. 1024 */
  int32_t batch;           /* >= 1 */
  int32_t n_q_heads;       /* multiple of n_kv_heads */
  int32_t n_kv_heads;      /* 1 .. 64 */
  int32_t head_dim;        /* 64 or 128 */
  int32_t ctx_len;         /* L, prompt length, <= 2^20 */
  int32_t window;          /* W = number of proxy tokens (the last W prompt positions); G*W <= 256 */
  int32_t budget;          /* tokens kept per KV head per layer, window included; >= ctx_len keeps all */
  int32_t dtype;           /* MADAKV_FP32 / MADAKV_BF16: type of Q, K, V and of the reduced cache */
  int32_t pool_k;          /* odd, 1 .. 63: max-pool width on the scores used for ranking; 1 = none */
  int32_t mpa_mode;        /* 1 = Eq. 8 modality split; 0 = modality-agnostic top-k; 2 / 3 = fixed priority
                              baselines: text / image takes all it can, the other modality the rest */
  int32_t hcc_mode;        /* 1 = Eq. 9-11 compensation, head totals follow demand; 0 = every head gets
                              budget - window; 2 = Eq. 9-11 layer totals shared equally by the heads */
  int32_t hcc_rho;         /* >= 1: demand clamp ratio around the running nominal budget */
  float   theta;           /* Eq. 9 threshold, in (0, 1] */
  float   softmax_scale;   /* 0 = 1/sqrt(head_dim) */
  int32_t max_new_tokens;  /* decode slack per head in the reduced cache */
  int32_t out_fp32;        /* decode output: 1 = float, 0 = same as dtype */
  int32_t pool_mode;       /* 0 = max-pool, 1 = average-pool (same clipped neighbourhood) */
  int32_t share_mode;      /* Eq. 6 masses over 0 = the candidates, 1 = all L columns (window included) */
  int32_t select_mode;     /* 0 = top scores per modality; 1 = score-free baseline: the first sink_tokens
                              candidates and the most recent ones, b_t + b_v in total */
  int32_t sink_tokens;     /* >= 0, used by select_mode 1 */
  int32_t cache_fp8;       /* 1 = the reduced cache k_c, v_c holds 8-bit floats (OCP E4M3: round to nearest even,
                              magnitudes above 448 saturate), one byte per element, instead of dtype; needs
                              dtype = MADAKV_BF16.  Q, K, V, k_new, v_new and out stay in dtype. */
  int32_t n_modalities;    /* M, 2 .. 4: modality ids in the mask are 0 .. M-1 (the paper has text = 0 and
                              image = 1; more modalities are the extension its Sec. 6 names) */
  int32_t page_rows;       /* 0 = every head's segment of the reduced cache is its kept rows followed by
                              max_new_tokens free rows; 16, 32, 64, 128 or 256 = paged reduced cache: a segment
                              is the kept rows rounded up to whole pages of that many rows, and the rows decode
                              appends (Sec. 3.1 Eq. 4) continue in pages taken on demand from a pool all heads
                              of a batch item share, so no head reserves room for generation up front */
} madakv_config;

/* Per-head statistics that madakv_score hands to madakv_allocate: a record of M floats
 * (Eq. 6 attention mass per modality) followed by M int32 (Eq. 9 theta-mass counts).  With
 * two modalities the record is this struct. */
typedef struct {
  float   w_t, w_v;        /* Eq. 6 attention mass on text / image candidates */
  int32_t k_t, k_v;        /* Eq. 9 theta-mass counts */
} madakv_head_stats;

typedef struct madakv_handle madakv_handle;

/* Creates a handle on the current HIP device.  *out is set only on success.
 * Errors: INVALID_ARG (null), BAD_SHAPE, BAD_BUDGET, UNSUPPORTED_DTYPE, HIP. */
int32_t madakv_create(const madakv_config* cfg, madakv_handle** out);
int32_t madakv_destroy(madakv_handle* h);

/* hipError_t of the last failing HIP call made through this handle (0 if none). */
int32_t madakv_last_hip_error(const madakv_handle* h);

/* Bytes of caller-provided scratch each call needs when it covers n layers (the
 * worst case over layer ranges of that size).  Any out pointer may be NULL. */
int32_t madakv_workspace_bytes(const madakv_handle* h, int32_t n_layers_per_call,
                               size_t* score_ws, size_t* select_ws, size_t* decode_ws);

/* Rows (tokens) the reduced cache k_c / v_c and kept_idx must hold for the whole
 * model: n_layers * batch * n_kv_heads * (min(budget, ctx_len) + max_new_tokens); with a paged
 * cache n_layers * batch * n_kv_heads * (ceil(min(budget, ctx_len) / page_rows) + 1 +
 * ceil(max_new_tokens / page_rows)) pages of page_rows rows.
 * Known without a device sync because the sum of budgets is conserved exactly. */
int32_t madakv_compact_capacity_tokens(const madakv_handle* h, int64_t* tokens);

/* Environment variables (diagnostics, read at every call they concern; not needed in normal use):
 *   MADAKV_SCORE_TWO_SWEEPS=1   score with the two-sweep kernels (K read twice) everywhere
 *   MADAKV_SCORE_SPIN_LIMIT=n   polls a workgroup of the one-sweep scoring kernel spends on a missing word
 *                               before it computes the head's row statistics alone (default 65536)
 *   MADAKV_LAYER_GROUPS=n       layer groups a call over several layers is pipelined in (1..4; default: as many as
 *                               leave a group 256 heads)
 *   MADAKV_SCORE_NO_PARKED_CHUNKS=1   long heads: all chunks of a head in one launch of the one-sweep kernel, also
 *                               where a few of them are in the way of one more head fitting the chip */

/* Eq. 7, Eq. 6, Eq. 9 and pooling for layers [layer0, layer0 + n).
 *   q_win    [n, B, Hq, W, d]  queries of the last W prompt positions
 *   k        [n, B, H, L, d]   prompt keys
 *   mask     [B, L] uint8      modality id per position
 *   psi      [n, B, H, L]      out: psi(i) = sum over the G*W proxy rows of the causal
 *                              softmax(scale * q k^T) they pay to key i
 *   psi_pool [n, B, H, L-W]    out: max of psi over |j - i| <= (pool_k-1)/2 within the
 *                              candidates [0, L-W)
 *   stats    [n, B, H]         out: records {float w[M]; int32 k[M]} over the candidates
 *   n_mod    [B, M] int32      out: candidate count per modality
 * ws / ws_bytes: scratch of at least score_ws bytes.  Its first int32 is a diagnostic counter the
 * library only ever adds to: workgroups of the one-sweep scoring kernel that gave up waiting for the
 * row statistics of their head's other workgroups and computed them alone (0 in normal operation if
 * the caller cleared it). */
int32_t madakv_score(madakv_handle* h, int32_t layer0, int32_t n,
                     const void* q_win, const void* k, const uint8_t* mask,
                     float* psi, float* psi_pool, void* stats, int32_t* n_mod,
                     void* ws, size_t ws_bytes, void* stream);

/* Sec. 3.3 Eq. 7 (then Eq. 6, Eq. 9, pooling as in madakv_score) for a caller whose prefill attention
 * (Sec. 3.1 Eq. 5 on the last W prompt positions) kept the softmax normalisers of the proxy
 * rows (any flash-attention kernel has them): with
 *   row_lse  [n, B, Hq, W] float  natural log of sum_i exp(scale * q_r . k_i) over the keys row r sees
 * the first of the two passes over K is not needed and psi costs one pass.  Everything else as
 * in madakv_score; the results are the same up to the rounding of row_lse. */
int32_t madakv_score_lse(madakv_handle* h, int32_t layer0, int32_t n,
                         const void* q_win, const void* k, const uint8_t* mask, const float* row_lse,
                         float* psi, float* psi_pool, void* stats, int32_t* n_mod,
                         void* ws, size_t ws_bytes, void* stream);

/* The step before the eviction path, fused with its first step: the prefill attention of the last W prompt
 * positions (Sec. 3.1 Eq. 5 for the proxy rows of Sec. 3.3), whose softmax rows are the alpha of Eq. 7.  One pass
 * over K and V gives
 *   out      [n, B, Hq, W, d]  softmax(scale * q_win k^T) v over the keys each proxy row sees (float if out_fp32
 *                              else dtype)
 *   row_lse  [n, B, Hq, W]     optional (may be NULL): natural log-sum-exp of each row
 * and psi, psi_pool, stats, n_mod exactly as madakv_score defines them (up to the rounding order of psi).  A model
 * whose prefill calls this for its last W positions needs no scoring sweep of its own: madakv_allocate and
 * madakv_select_gather follow directly.  v [n, B, H, L, d]; ws: madakv_window_attn_workspace_bytes(h, n) bytes;
 * everything else as in madakv_score.  With more than 32 proxy rows (grouped queries, wide windows) the rows are
 * taken in blocks of 32, each with a pass over K and V of its own.  MADAKV_ERR_UNIMPLEMENTED unless dtype is bf16
 * and ctx_len <= 131072 (head_dim 128) / 196608 (head_dim 64). */
int32_t madakv_window_attn_workspace_bytes(const madakv_handle* h, int32_t n_layers_per_call, size_t* bytes);
int32_t madakv_window_attn_score(madakv_handle* h, int32_t layer0, int32_t n,
                                 const void* q_win, const void* k, const void* v, const uint8_t* mask,
                                 void* out, float* row_lse,
                                 float* psi, float* psi_pool, void* stats, int32_t* n_mod,
                                 void* ws, size_t ws_bytes, void* stream);

/* Eq. 8, Eq. 10-11 for layers [layer0, layer0 + n) in order.
 *   stats    [n, B, H]        from madakv_score
 *   n_mod    [B, M]
 *   budgets  [n, B, H, M] int32  out: candidate tokens to keep per modality ((b_t, b_v) for M = 2);
 *                              their sum over modalities, heads and the whole model is
 *                              exactly n_layers * H * (budget - W) per batch item.
 *                              With mpa_mode = 0 the head total is in slot 0, the others are 0.
 * The remaining pool of each batch item is carried in the handle; layer0 = 0 resets it. */
int32_t madakv_allocate(madakv_handle* h, int32_t layer0, int32_t n,
                        const void* stats, const int32_t* n_mod,
                        int32_t* budgets, void* stream);

/* Per head and modality: keep the b_m candidates with the largest psi_pool (equal scores:
 * lower position first), in ascending position, then the W window positions; copy their
 * K and V rows into the reduced cache.
 *   psi_pool [n, B, H, L-W], mask [B, L], budgets [n, B, H, M] (0 <= b_m <= n_mod[m])
 *   k, v     [n, B, H, L, d]
 *   kept_idx int32, ragged  out: head (l,b,h) owns kept_idx[kv_off .. kv_off + kv_len)
 *   kv_off   [n, B, H] int64 out: first row of the head's segment in k_c / v_c / kept_idx
 *   kv_len   [n, B, H] int32 out: sum of the head's budgets + W
 *   k_c, v_c [capacity_tokens, d]  out: the reduced cache (dtype, or bytes with cache_fp8); a head's segment has kv_len
 *                              rows followed by max_new_tokens free rows
 * Batch item b owns rows [b, b+1) * capacity_tokens / B; inside, layers then heads follow
 * each other.  Budgets from madakv_allocate fill that space exactly.  If hand-made budgets
 * add up to more, the first head that does not fit and every head after it in the batch
 * item get an empty segment (kv_len = 0): nothing is written for them, decode neither
 * appends to them nor produces a finite output for them.  The write cursor per batch item is carried in the handle; layer0 = 0
 * resets it.  The decode-step counters of the layers in the call are reset. */
int32_t madakv_select_gather(madakv_handle* h, int32_t layer0, int32_t n,
                             const float* psi_pool, const uint8_t* mask, const int32_t* budgets,
                             const void* k, const void* v,
                             int32_t* kept_idx, int64_t* kv_off, int32_t* kv_len,
                             void* k_c, void* v_c,
                             void* ws, size_t ws_bytes, void* stream);

/* Sec. 3.3 as a whole (Eq. 7, 6, 9, then Eq. 8, 10, 11, then the per-head, per-modality eviction):
 * madakv_score + madakv_allocate + madakv_select_gather for layers [layer0, layer0 + n) in one call,
 * with the same arguments and the same results bit for bit.  A call over four or more layers is
 * cut into four layer groups: the statistics, allocation and selection of a group run on a side
 * stream while the caller's stream holds the score passes of the next group and the gather of the
 * group before.  Keep-all configurations (budget >= ctx_len) have nothing to score: use
 * madakv_select_gather for them.  score_ws / select_ws: at least what madakv_workspace_bytes
 * reports for n layers. */
int32_t madakv_evict(madakv_handle* h, int32_t layer0, int32_t n,
                     const void* q_win, const void* k, const void* v, const uint8_t* mask,
                     float* psi, float* psi_pool, void* stats, int32_t* n_mod, int32_t* budgets,
                     int32_t* kept_idx, int64_t* kv_off, int32_t* kv_len, void* k_c, void* v_c,
                     void* score_ws, size_t score_ws_size, void* select_ws, size_t select_ws_size, void* stream);

/* One decode step for layers [layer0, layer0 + n): append k_new, v_new to every head's
 * segment (Eq. 4), then out = softmax(scale * q k_c^T) v_c over the head's rows (Eq. 5).
 *   q        [n, B, Hq, d]
 *   k_new, v_new [n, B, H, d]  both NULL = attend only
 *   k_c, v_c, kv_off          as produced by madakv_select_gather
 *   kv_len   [n, B, H]        in/out: the array madakv_select_gather filled (the library sizes
 *                              its launch from the lengths it produced); incremented by the append
 *   out      [n, B, Hq, d]    float if out_fp32 else dtype
 * INVALID_ARG if a layer in the range has already appended max_new_tokens rows. */
int32_t madakv_decode_attn(madakv_handle* h, int32_t layer0, int32_t n,
                           const void* q, const void* k_new, const void* v_new,
                           void* k_c, void* v_c, const int64_t* kv_off, int32_t* kv_len,
                           void* out, void* ws, size_t ws_bytes, void* stream);

/* Re-eviction during generation (the paper evicts once, after the prefill, Sec. 3.3; its Sec. 6 leaves long
 * generation open).  After some decode steps every head's segment holds its kept rows, the W window rows and
 * the appended rows.  The call brings each head of layers [layer0, layer0 + n) back to the length the prompt
 * eviction gave it, in place:
 *   - the last W rows of the segment are the new proxy set; q_recent holds their queries;
 *   - every earlier row is a candidate, scored as in Eq. 7 over the rows of the segment (proxy row r sees
 *     the rows up to its own), pooled over neighbouring rows as configured;
 *   - the head's total stays budgets_total = (length after the last (re-)eviction) - W: the layer
 *     compensation of Eq. 9-11 is a prefill decision and is not re-run;
 *   - the total is split over the modalities by the current masses (Eq. 6, Eq. 8, same integer rules as
 *     madakv_allocate; a prompt token has the modality of its position in `mask`, a generated token is text);
 *   - per modality the best-scored candidates survive (equal scores: lower row), in row order, followed by
 *     the W proxy rows; K, V and kept_idx rows move down inside the segment.
 *   q_recent [n, B, Hq, W, d]   queries of the tokens in the last W rows of every segment, oldest first
 *   mask     [B, L]
 *   k_c, v_c, kept_idx, kv_off  as left by madakv_select_gather / madakv_evict and madakv_decode_attn;
 *                               kept_idx entries of generated tokens read ctx_len + (index of the token
 *                               in the generation) afterwards
 *   kv_len   [n, B, H]          in/out: back to its value after the prompt eviction
 *   budgets  [n, B, H, M]       out: the new split
 *   ws                          madakv_reevict_workspace_bytes(h, n) bytes
 * The decode-step counters of the layers are reset: max_new_tokens rows can be appended again.
 * An 8-bit cache is scored and moved as it is stored (E4M3 rows).  A paged cache is re-evicted as a whole
 * (layer0 = 0, n = n_layers, else MADAKV_ERR_INVALID_ARG): the survivors end up in the heads' initial pages
 * and every page taken since the eviction goes back to the pools, which all layers share; the work is done
 * on a linear copy of the rows in the workspace (as many rows as the cache holds).
 * MADAKV_ERR_UNIMPLEMENTED with dtype fp32 or segments longer than 64 chunks of the
 * scoring kernel (65536 rows at G * W <= 32, 49152 beyond); MADAKV_ERR_BAD_BUDGET when budget >= ctx_len
 * (nothing was evicted). */
int32_t madakv_reevict_workspace_bytes(const madakv_handle* h, int32_t n_layers_per_call, size_t* bytes);
int32_t madakv_reevict(madakv_handle* h, int32_t layer0, int32_t n,
                       const void* q_recent, const uint8_t* mask,
                       void* k_c, void* v_c, int32_t* kept_idx, const int64_t* kv_off, int32_t* kv_len,
                       int32_t* budgets, void* ws, size_t ws_bytes, void* stream);

/* Paged reduced cache (page_rows > 0): where the rows of a head are.  Rows [0, table[0] * page_rows) of head
 * (l, b, h) sit at kv_off[l, b, h] + r (its initial pages follow each other); row r beyond that sits in page
 * table[1 + (r - table[0] * page_rows) / page_rows] at slot r % page_rows, a page p covering rows
 * [p * page_rows, (p + 1) * page_rows) of k_c / v_c.  *table is a device pointer into the handle (valid
 * until madakv_destroy, NULL without paging) to int32 [n_layers * batch * n_kv_heads][*entries_per_head],
 * head-major in (layer, batch, head) order; madakv_select_gather / madakv_evict write entry 0,
 * madakv_decode_attn the others as pages get taken (from the top of the batch item's region downwards;
 * a new pass starting at layer 0 returns them all). */
int32_t madakv_page_table(const madakv_handle* h, const int32_t** table, int32_t* entries_per_head);

/* madakv_decode_attn for callers that cannot allocate device memory and so have no workspace to
 * pass: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, kernels and results as madakv_decode_attn, without ws: the partial
 * results of heads that are cut into several chunks go to an array of
 * MADAKV_STATIC_SCRATCH_BYTES bytes that is part of the library's device code (one copy per GPU,
 * held until the process ends).  The call allocates and frees nothing.
 *   - MADAKV_ERR_WORKSPACE_TOO_SMALL if this launch needs more than the array holds: the need is
 *     (heads in the call) * (chunks of the longest head) * G * (head_dim + 2) * 4 bytes, with
 *     chunks of 256 .. 1024 rows (512 once the call covers >= 1024 heads); the longest head is
 *     taken from what the eviction produced once that has reached the host, from ctx_len +
 *     max_new_tokens before.  One layer of 128 heads of up to 16K rows fits.  Nothing is
 *     enqueued in that case.
 *   - Every call on one GPU, from any handle, uses the same array: calls that may run
 *     concurrently on one GPU (different streams) race on it and must not be issued.  Nothing in
 *     the array has to survive between calls.
 *   - On a stream under graph capture (this call or madakv_decode_attn) the launch is sized for every
 *     row the segments have room for, so that the captured step can be replayed while the heads
 *     grow; each replay appends a row like a call would, but the library's count of appended rows
 *     only sees the capture itself: the caller must not replay beyond max_new_tokens rows per
 *     head, and takes up eager calls again only after a new eviction or re-eviction. */
#define MADAKV_STATIC_SCRATCH_BYTES ((size_t)8 << 20)
int32_t madakv_decode_attn_static(madakv_handle* h, int32_t layer0, int32_t n,
                                  const void* q, const void* k_new, const void* v_new,
                                  void* k_c, void* v_c, const int64_t* kv_off, int32_t* kv_len,
                                  void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MADAKV_H */
