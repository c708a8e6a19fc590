/*
 * sepattn.h -- C ABI of libsepattn: SepAttention (SepLLM, arXiv 2412.12094) on AMD MI355X (gfx950).
 *
 * SepAttention is causal softmax attention in which query i sees only
 *   - the first `a` tokens of its sequence                     (Initial Tokens,     Sec. 3.1),
 *   - every separator token at or before i                     (Separator Tokens,   Sec. 3.1),
 *   - its n closest tokens  i-n < j <= i                       (Neighboring Tokens, Sec. 3.1),
 * i.e. the binary mask M of Eq. 2, applied as in Eq. 1:  A = Softmax(QK^T/sqrt(d_k) | M), O = A V.
 * The library provides the training / prefill forward and backward of Eq. 1 (also over rows packed
 * from several documents), single-query decode over the four-block KV cache (optionally with the
 * rotary encoding applied by position within the cache), and the cache steps of Sec. 3.3 ("Tailored
 * Streaming Design"): hand-over from a prefill, append, compression.
 *
 * Conventions common to every call
 *   - Pointers marked DEVICE address memory of the current HIP device; HOST pointers address
 *     ordinary host memory.  The caller owns every buffer, including workspaces; the library
 *     allocates no device memory and keeps no state between calls (the fixed scratch array of
 *     sepattn_decode_noalloc aside).
 *   - Alignment: token_ids, Q, K, V, O, dO, dQ, dK, dV, q, Kc, Vc, out, k_new, v_new and rope tables
 *     must be 16-byte aligned, is_sep 4-byte aligned, workspaces 256-byte aligned; a misaligned
 *     buffer is refused with SEPATTN_ERR_PARAM (workspaces: SEPATTN_ERR_WORKSPACE).
 *   - Tensors are dense and contiguous with the head dimension d innermost.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls validate their
 *     arguments synchronously, enqueue their kernels on `stream` and return without waiting.
 *     Nothing is enqueued when a validation error (any status but SEPATTN_ERR_HIP) is returned.
 *     SEPATTN_ERR_HIP means the runtime refused a launch of this call; a call that consists of
 *     several kernels may then have enqueued the earlier ones, and its outputs are unspecified.
 *     An error left pending in the HIP runtime by the caller's own earlier calls is discarded at
 *     entry, not reported.
 *   - Return value: SEPATTN_OK (0) or a positive sepattn_status.  No call throws or exits.
 *   - Outputs must not alias inputs, except where a call is documented as in-place.
 *   - All results are bit-reproducible run to run (no floating-point atomics).
 */
#ifndef SEPATTN_H
#define SEPATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SEPATTN_OK = 0,
    SEPATTN_ERR_NULL = 1,      /* a required pointer is NULL                                   */
    SEPATTN_ERR_SHAPE = 2,     /* a size is non-positive, too large, or inconsistent            */
    SEPATTN_ERR_PARAM = 3,     /* a hyper-parameter is out of range (n < 1, a < 0, a+s+w >= c),
                                  or a buffer is not aligned as the conventions above require  */
    SEPATTN_ERR_DTYPE = 4,     /* dtype is not a sepattn_dtype / unsupported head dimension     */
    SEPATTN_ERR_WORKSPACE = 5, /* workspace missing or smaller than *_workspace_bytes reports   */
    SEPATTN_ERR_CAPACITY = 6,  /* an index list capacity is too small to be usable              */
    SEPATTN_ERR_HIP = 7        /* the HIP runtime reported an error at launch                   */
} sepattn_status;

typedef enum {
    SEPATTN_BF16 = 0, /* bfloat16 storage, fp32 softmax and accumulation, MFMA contractions    */
    SEPATTN_FP32 = 1  /* fp32 storage and arithmetic: slow debug path                          */
} sepattn_dtype;

#define SEPATTN_MAX_SEP_IDS 64

/* Static, NUL-terminated description of a status code (HOST pointer, never freed). */
const char *sepattn_status_string(int status);

/* ------------------------------------------------------------------------------------------
 * Separator marking (Sec. 4.1 "Parameter Setting": the separator set; a token is a separator
 * iff its id is in the caller's set).
 *   token_ids  DEVICE int32 [B, L]
 *   sep_ids    HOST   int32 [n_sep], 1 <= n_sep <= SEPATTN_MAX_SEP_IDS (copied before returning)
 *   is_sep     DEVICE uint8 [B, L]  out: 1 for separators, 0 otherwise
 * ------------------------------------------------------------------------------------------ */
int sepattn_mark_separators(const int32_t *token_ids, int B, int L, const int32_t *sep_ids,
                            int n_sep, uint8_t *is_sep, void *stream);

/* Fixed-interval variant (the appendix "Fixed-Interval Variant", FixLLM): instead of the separators,
 * one token in every `delta` is attended to between the initial and the neighbouring tokens.  Writes
 * is_sep[b, j] = (j % delta == phase); everything downstream (compaction, forward, backward, the
 * cache calls) takes this bitmap in place of the separator flags.
 *   delta >= 1, 0 <= phase < delta (SEPATTN_ERR_PARAM otherwise)
 *   is_sep     DEVICE uint8 [B, L]  out, 4-byte aligned
 */
int sepattn_mark_interval(int B, int L, int delta, int phase, uint8_t *is_sep, void *stream);

/* ------------------------------------------------------------------------------------------
 * Separator compaction: the index form of the separator part of mask M (Eq. 2), shared by all
 * layers and heads of a batch.
 *   is_sep      DEVICE uint8 [B, L]
 *   sep_idx     DEVICE int32 [B, cap]  out: ascending separator positions of each sequence;
 *                                       entries at and beyond min(count, cap) are left untouched
 *   sep_count   DEVICE int32 [B]       out: true number of separators, even when it exceeds cap
 *   sep_prefix  DEVICE int32 [B, L+1]  out: sep_prefix[b,j] = number of separators at positions
 *                                       < j  (exclusive prefix count; sep_prefix[b,L] = count).
 *                                       May be NULL when only the list and the count are wanted
 *                                       (forward / backward / the hand-over need it).
 *   workspace   DEVICE, at least sepattn_compact_workspace_bytes(B, L) bytes, 4-byte aligned
 * cap >= 1.  A caller that wants forward / backward to see every separator passes cap >= count
 * (cap = L always suffices).
 * ------------------------------------------------------------------------------------------ */
size_t sepattn_compact_workspace_bytes(int B, int L);
int sepattn_compact_indices(const uint8_t *is_sep, int B, int L, int32_t *sep_idx, int cap,
                            int32_t *sep_count, int32_t *sep_prefix, void *workspace,
                            size_t workspace_bytes, void *stream);

/* Marking and compaction in one call (Sec. 4.1 "Parameter Setting" and Eq. 2): exactly the outputs
 * of sepattn_mark_separators followed by sepattn_compact_indices, arguments as there (is_sep is an
 * output here; sep_prefix may be NULL; the workspace is the one of the compaction).  Sequences of up
 * to 8192 tokens take one kernel launch instead of two, which matters because at these sizes the
 * kernels last no longer than their launch; longer ones run the separate kernels.
 */
int sepattn_mark_compact(const int32_t *token_ids, int B, int L, const int32_t *sep_ids, int n_sep,
                         uint8_t *is_sep, int32_t *sep_idx, int cap, int32_t *sep_count,
                         int32_t *sep_prefix, void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Training / prefill attention (Eq. 1 with the mask of Eq. 2).
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    int B;       /* sequences                                                                  */
    int Hq;      /* query heads                                                                */
    int Hkv;     /* key/value heads; Hq % Hkv == 0; query head h reads KV head h / (Hq/Hkv)     */
    int L;       /* sequence length (the paper's m); L * d * 4 < 2^32, else SEPATTN_ERR_SHAPE   */
    int d;       /* head dimension d_k = d_v: 64 or 128                                        */
    int a;       /* number of initial tokens kept, a >= 0                                      */
    int n;       /* number of neighbouring tokens kept, the token itself included, n >= 1      */
    float scale; /* multiplies QK^T; 1/sqrt(d) in Eq. 1                                        */
    int dtype;   /* sepattn_dtype of Q, K, V, O, dO, dQ, dK, dV                                */
    int cap;     /* row pitch of sep_idx                                                       */
} sepattn_params;

/*   Q          DEVICE dtype [B, Hq,  L, d]
 *   K, V       DEVICE dtype [B, Hkv, L, d]
 *   sep_idx, sep_count, sep_prefix   DEVICE, as written by sepattn_compact_indices for the same
 *                                    (B, L) with pitch p->cap; sep_count[b] <= cap is required
 *   O          DEVICE dtype [B, Hq, L, d]  out
 *   LSE        DEVICE fp32  [B, Hq, L]     out: natural log of sum_j exp(scale*<Q_i,K_j>) over the
 *                                           visible keys j of row i
 *   ws         DEVICE, >= sepattn_forward_workspace_bytes(p) bytes (may be NULL when that is 0),
 *              256-byte aligned
 */
size_t sepattn_forward_workspace_bytes(const sepattn_params *p);
int sepattn_forward(const sepattn_params *p, const void *Q, const void *K, const void *V,
                    const int32_t *sep_idx, const int32_t *sep_count, const int32_t *sep_prefix,
                    void *O, float *LSE, void *ws, size_t ws_bytes, void *stream);

/* Gradient of Eq. 1 (the paper trains through Sep-Attention, Sec. 4.3; it prints no formula, this
 * is the analytic gradient): given dO, with D_i = <dO_i, O_i>, A_ij = exp(scale*<Q_i,K_j> - LSE_i):
 *   dV_j = sum_i A_ij dO_i,  dS_ij = A_ij (<dO_i,V_j> - D_i),
 *   dQ_i = scale sum_j dS_ij K_j,  dK_j = scale sum_i dS_ij Q_i,
 * dK and dV of a KV head summed over the Hq/Hkv query heads that read it.  LSE carries no gradient.
 *   O, LSE     DEVICE, as written by sepattn_forward for the same inputs
 *   dO         DEVICE dtype [B, Hq, L, d]
 *   dQ         DEVICE dtype [B, Hq,  L, d]  out
 *   dK, dV     DEVICE dtype [B, Hkv, L, d]  out
 *   ws         DEVICE, >= sepattn_backward_workspace_bytes(p) bytes, 256-byte aligned
 */
size_t sepattn_backward_workspace_bytes(const sepattn_params *p);
int sepattn_backward(const sepattn_params *p, const void *Q, const void *K, const void *V,
                     const void *O, const float *LSE, const void *dO, const int32_t *sep_idx,
                     const int32_t *sep_count, const int32_t *sep_prefix, void *dQ, void *dK,
                     void *dV, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Packed documents (training batches packed from several documents; the paper is silent on them:
 * every document is taken as a sequence of its own, i.e. Eq. 1 / Eq. 2 per document: its first a
 * tokens are its initial tokens and a query sees no key outside its document).
 *
 * Preparation, per row of the batch: sepattn_doc_bounds turns the cumulative lengths into the two
 * per-position bounds and marks the first a tokens of every document in the row's marker bitmap;
 * the bitmap then goes through sepattn_compact_indices as usual, and the packed calls run with
 * p->a == 0 (SEPATTN_ERR_PARAM otherwise): the documents' initial tokens are list entries.
 *   cu_seqlens  DEVICE int32 [n_docs+1]: cu[0] = 0 < cu[1] < ... < cu[n_docs] = L
 *   doc_start   DEVICE int32 [L]  out: first position of each position's document
 *   doc_end     DEVICE int32 [L]  out: one past its last position
 *   is_sep      DEVICE uint8 [L]  in/out, may be NULL: one row of the marker bitmap
 * sepattn_forward_packed / sepattn_backward_packed: as sepattn_forward / sepattn_backward, plus
 *   doc_start, doc_end  DEVICE int32 [B, L] (bounds that contradict each other cannot fault: they
 *   are clamped around the position; the result is then unspecified).
 * ------------------------------------------------------------------------------------------ */
int sepattn_doc_bounds(const int32_t *cu_seqlens, int n_docs, int L, int a, int32_t *doc_start,
                       int32_t *doc_end, uint8_t *is_sep, void *stream);
int sepattn_forward_packed(const sepattn_params *p, const int32_t *doc_start, const int32_t *doc_end,
                           const void *Q, const void *K, const void *V, const int32_t *sep_idx,
                           const int32_t *sep_count, const int32_t *sep_prefix, void *O, float *LSE,
                           void *ws, size_t ws_bytes, void *stream);
int sepattn_backward_packed(const sepattn_params *p, const int32_t *doc_start,
                            const int32_t *doc_end, const void *Q, const void *K, const void *V,
                            const void *O, const float *LSE, const void *dO, const int32_t *sep_idx,
                            const int32_t *sep_count, const int32_t *sep_prefix, void *dQ, void *dK,
                            void *dV, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Head-wise neighbour windows (Sec. 4.6 "Comparison with More Baselines and Variants": some heads
 * keep a short window, the others see everything; also the per-layer hybrids of Sec. 4.3 when the
 * caller batches them): forward and backward of Eq. 1 with a mask of Eq. 2 whose n is a per-head
 * value, n_per_head[h] for query head h (n_per_head[h] >= L is full causal attention for that
 * head).  Initial tokens and separators are visible to every head as before.
 *   n_per_head   HOST int32 [Hq], every entry >= 1 (copied before returning); p->n is ignored.
 *                Hq <= SEPATTN_MAX_HEADWISE_HEADS (SEPATTN_ERR_SHAPE otherwise).
 * Everything else as sepattn_forward / sepattn_backward; the backward workspace is the one of a
 * call with n = max_h n_per_head[h] (sepattn_backward_headwise_workspace_bytes).  The heads of a
 * KV head share its K/V tiles, so a call costs about what the largest window of each group costs.
 * ------------------------------------------------------------------------------------------ */
#define SEPATTN_MAX_HEADWISE_HEADS 128
int sepattn_forward_headwise(const sepattn_params *p, const int32_t *n_per_head, const void *Q,
                             const void *K, const void *V, const int32_t *sep_idx,
                             const int32_t *sep_count, const int32_t *sep_prefix, void *O, float *LSE,
                             void *ws, size_t ws_bytes, void *stream);
size_t sepattn_backward_headwise_workspace_bytes(const sepattn_params *p, const int32_t *n_per_head);
int sepattn_backward_headwise(const sepattn_params *p, const int32_t *n_per_head, const void *Q,
                              const void *K, const void *V, const void *O, const float *LSE,
                              const void *dO, const int32_t *sep_idx, const int32_t *sep_count,
                              const int32_t *sep_prefix, void *dQ, void *dK, void *dV, void *ws,
                              size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Streaming generation on the four-block KV cache (Sec. 3.3).
 * Cache layout, per (sequence, KV head): c slots of d values,
 *     [0, a)       Initial Cache
 *     [a, a+s)     Separator Cache, a ring: separator k (oldest first) sits in slot
 *                  a + (head_sep + k) mod s
 *     [a+s, c)     window, a ring of c-a-s slots: entry u (oldest first: the Past Window Cache,
 *                  then the Local Window Cache) sits at window index (head_win + u) mod (c-a-s),
 *                  i.e. in slot a+s + that index; win_is_sep is indexed by window index
 * sizes[S, SEPKV_SIZES_COLS = 6] = (Size_init, Size_sep, Size_past_w, Size_local_w, head_sep, head_win):
 * valid entries of each block and the two ring heads (0 for a cache that has never dropped
 * anything).  The rings are what lets the compression step move only the rows the method says
 * must move: dropping the oldest separators or the Past Window advances a head.  Requires
 * 0 <= Size_init <= a, 0 <= Size_sep <= s, Size_past_w + Size_local_w <= c-a-s,
 * 0 <= head_sep < max(s, 1), 0 <= head_win < c-a-s; sizes are read on the device and clamped to
 * these ranges there (a value outside them gives wrong results, never an access out of bounds).
 * "Position within the cache" (sepattn_decode_rope) is the rank of an entry in age order over
 * Initial, Separator, Past Window, Local Window, whatever slots the entries occupy.
 * ------------------------------------------------------------------------------------------ */
#define SEPKV_SIZES_COLS 6
typedef struct {
    int S;       /* sequences                                                                  */
    int Hq;      /* query heads                                                                */
    int Hkv;     /* key/value heads, Hq % Hkv == 0                                             */
    int d;       /* head dimension: 64 or 128                                                  */
    int a;       /* capacity of the Initial Cache                                              */
    int s;       /* capacity of the Separator Cache                                            */
    int w;       /* capacity of the Local Window Cache                                         */
    int c;       /* capacity of the whole cache; a + s + w < c                                 */
    float scale; /* multiplies q K^T                                                           */
    int dtype;   /* sepattn_dtype of q, Kc, Vc, out                                            */
} sepkv_params;

/* One query token per sequence attends to every valid cache entry (Sec. 3.2 "Generation": only
 * the KV of initial, separator and neighbouring tokens is kept, and all of it is visible).  The
 * caller appends the current token's K/V before calling.
 *   q        DEVICE dtype [S, Hq, d]
 *   Kc, Vc   DEVICE dtype [S, Hkv, c, d]
 *   sizes    DEVICE int32 [S, 6]; a sequence with no valid entry yields out = 0, lse = -inf
 *   out      DEVICE dtype [S, Hq, d]  out
 *   lse      DEVICE fp32  [S, Hq]     out, may be NULL
 *   ws       DEVICE, >= sepattn_decode_workspace_bytes(p) bytes, 256-byte aligned
 */
size_t sepattn_decode_workspace_bytes(const sepkv_params *p);
int sepattn_decode(const sepkv_params *p, const void *q, const void *Kc, const void *Vc,
                   const int32_t *sizes, void *out, float *lse, void *ws, size_t ws_bytes,
                   void *stream);

/* Decode with positions within the cache (Sec. 3.3 "Positional Encoding"; Sec. 4.6, the ablation
 * of the positional shifting): q and the cached keys are stored WITHOUT position encoding; the
 * valid entries of a sequence, oldest first (Initial, Separator, Past Window, Local Window Cache),
 * are at positions 0 .. nv-1 and the query, the newest entry's token, at nv-1.  Keys and query are
 * turned by the rotary encoding of the backbones the paper evaluates (dimension i < d/2 pairs with
 * i + d/2; the pair at position t is rotated by t * base^(-2i/d)) inside the kernel, so entries
 * that move or drop out of the cache never have to be re-encoded in memory.
 *   sepkv_rope_table: fills  table  DEVICE fp32 [n_pos, 2, d/2]  (16-byte aligned; cos, then sin, of
 *       position * base^(-2i/d); computed in double, rounded to fp32); d is 64 or 128, base > 1.
 *       Build it once per (d, base); the caller owns it.
 *   sepattn_decode_rope: as sepattn_decode, plus  rope_table  from sepkv_rope_table with
 *       n_pos >= c (SEPATTN_ERR_SHAPE otherwise).  The table must be complete before the call
 *       runs (same stream, or synchronised).
 */
int sepkv_rope_table(int n_pos, int d, double base, float *table, void *stream);
int sepattn_decode_rope(const sepkv_params *p, const void *q, const void *Kc, const void *Vc,
                        const int32_t *sizes, const float *rope_table, int n_pos, void *out,
                        float *lse, void *ws, size_t ws_bytes, void *stream);

/* sepattn_decode for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as sepattn_decode, without ws / ws_bytes: the partial results of
 * the cache slices live in a fixed array of SEPATTN_DECODE_NOALLOC_SCRATCH_BYTES inside the library
 * (one copy per GPU the library runs on, held until the process ends).  The call allocates and
 * frees nothing and clears nothing.
 *   - SEPATTN_ERR_WORKSPACE if the shape needs more than the fixed array, i.e. if
 *     sepattn_decode_noalloc_scratch_bytes(p) (= sepattn_decode_workspace_bytes(p)) exceeds
 *     SEPATTN_DECODE_NOALLOC_SCRATCH_BYTES; nothing is enqueued then.
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (on
 *     different streams, or from different threads) race on it.  Calls on one stream are ordered
 *     and safe.
 */
#define SEPATTN_DECODE_NOALLOC_SCRATCH_BYTES (4u << 20)
size_t sepattn_decode_noalloc_scratch_bytes(const sepkv_params *p);
int sepattn_decode_noalloc(const sepkv_params *p, const void *q, const void *Kc, const void *Vc,
                           const int32_t *sizes, void *out, float *lse, void *stream);

/* A new token enters the cache of every sequence (Sec. 3.3 "Framework"): the first a tokens of a
 * sequence go to the Initial Cache; a later token is written behind the newest window entry and
 * joins the Local Window Cache, and once that holds more than w its oldest entry passes to the
 * Past Window Cache.  A sequence whose window region is full (Size_past_w + Size_local_w = c-a-s)
 * is left unchanged: run sepkv_evict_window first (its sizes tell: they did not change).
 *   k_new, v_new  DEVICE dtype [S, Hkv, d]      the token's key and value (copied bit-exactly)
 *   is_sep_new    DEVICE uint8 [S]              whether the token is a separator
 *   Kc, Vc        DEVICE dtype [S, Hkv, c, d]   in/out
 *   win_is_sep    DEVICE uint8 [S, c-a-s]       in/out
 *   sizes         DEVICE int32 [S, 6]           in/out
 */
int sepkv_append(const sepkv_params *p, const void *k_new, const void *v_new,
                 const uint8_t *is_sep_new, void *Kc, void *Vc, uint8_t *win_is_sep,
                 int32_t *sizes, void *stream);

/* Compression step (Sec. 3.3; caption of the streaming-design figure): the separators of the Past
 * Window Cache are appended to the Separator Cache, its other entries are dropped, and the Local
 * Window becomes the whole window.  If the Separator Cache would exceed s, its oldest entries are
 * dropped (first in, first out).  IN PLACE; rows are copied bit-exactly, and only the kept
 * Past-Window rows are copied at all: the rest is a change of the ring heads.
 *   Kc, Vc      DEVICE dtype [S, Hkv, c, d]  in/out
 *   win_is_sep  DEVICE uint8 [S, c-a-s]      separator flag by window index; not written (the
 *                                            flags of the surviving Local Window stay in place)
 *   sizes       DEVICE int32 [S, 6]          in/out: becomes (Size_init, min(s, Size_sep + k), 0,
 *                                            Size_local_w, head_sep + dropped separators mod s,
 *                                            head_win + Size_past_w mod (c-a-s)), k = number of
 *                                            flagged Past-Window entries
 *   ws          not used: the step needs no scratch memory, sepkv_evict_workspace_bytes returns 0
 *               and ws may be NULL (the two arguments are kept for callers written against a
 *               workspace)
 * Slots outside the valid entries hold unspecified data afterwards.  The caller decides when to call
 * (the paper triggers it when Size_run reaches c).
 */
size_t sepkv_evict_workspace_bytes(const sepkv_params *p);
int sepkv_evict_window(const sepkv_params *p, void *Kc, void *Vc, const uint8_t *win_is_sep,
                       int32_t *sizes, void *ws, size_t ws_bytes, void *stream);

/* Hand-over from prefill to the cache (Sec. 3.2 "Generation": only the KV of initial, separator and
 * neighbouring tokens is kept; Sec. 3.3 for the block layout): after L prompt tokens the cache of
 * each sequence receives
 *     Initial Cache    positions 0 .. min(a, L) - 1
 *     Separator Cache  the newest (at most s) separators among the positions [min(a, L), L - nw),
 *                      oldest first; older ones are dropped, as the compression step would drop them
 *     window           the last nw positions, oldest first; the newest min(w, nw) are the Local Window
 * i.e. the state the append / compression policy reaches after L tokens when its window then holds
 * nw entries (the caller knows nw: the policy's n after L tokens).  Rows are copied bit-exactly.
 *   L            prompt length;  nw  window entries, 0 <= nw <= min(c - a - s, L - min(a, L))
 *   K, V         DEVICE dtype [S, Hkv, L, d]     the prefill's keys and values
 *   is_sep       DEVICE uint8 [S, L]             as from sepattn_mark_separators
 *   sep_idx      DEVICE int32 [S, cap], sep_prefix DEVICE int32 [S, L+1]: as from
 *                sepattn_compact_indices (cap >= the number of separators, else the newest listed ones)
 *   Kc, Vc       DEVICE dtype [S, Hkv, c, d]     out; slots beyond the new sizes are left untouched
 *   win_is_sep   DEVICE uint8 [S, c-a-s]         out: separator flag of each window entry
 *   sizes        DEVICE int32 [S, 6]             out: (min(a, L), kept separators, nw - Size_local_w, Size_local_w, 0, 0)
 * Errors: SEPATTN_ERR_PARAM if nw is out of range.
 */
int sepkv_fill_from_prefill(const sepkv_params *p, int L, int nw, const void *K, const void *V,
                            const uint8_t *is_sep, const int32_t *sep_idx, int cap,
                            const int32_t *sep_prefix, void *Kc, void *Vc, uint8_t *win_is_sep,
                            int32_t *sizes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Measurement hooks (not part of the method).  A benchmark that times whole steps can also report one
 * kernel's own duration: it creates a handle for that kernel, attaches it to the thread that makes
 * the library calls, and from then on every launch of the kernel by that thread is bracketed by a
 * pair of HIP events recorded on the stream the kernel is launched on, until the handle is detached.
 * The handle and everything it records belong to the caller; the library keeps no process-wide state,
 * only, per thread, which handle is attached.  Different threads may use different handles at the
 * same time; one handle must not be attached to two threads.
 *   sepattn_profile_create   kernel: a sepattn_kernel_id; max_records: events are created up front
 *                            for this many launches, further launches are not recorded;
 *                            *out receives the handle (HOST)
 *   sepattn_profile_attach   SEPATTN_ERR_PARAM if this thread already has a handle attached
 *   sepattn_profile_detach   SEPATTN_ERR_PARAM if h is not the handle attached to this thread
 *   sepattn_profile_read     waits for the recorded events (call it after the timed region);
 *                            ms HOST float [max_records] out: elapsed milliseconds per recorded
 *                            launch; *n_records out: how many were written
 *   sepattn_profile_destroy  frees the events and the handle (detaches it from this thread first)
 * ------------------------------------------------------------------------------------------ */
typedef enum {
    SEPATTN_K_MARK = 0,
    SEPATTN_K_COMPACT_COUNT = 1,
    SEPATTN_K_COMPACT_WRITE = 2,
    SEPATTN_K_FORWARD = 3,
    SEPATTN_K_BWD_DQ = 4,
    SEPATTN_K_BWD_DKV = 5,
    SEPATTN_K_BWD_COMBINE = 6,
    SEPATTN_K_DECODE_SPLIT = 7,
    SEPATTN_K_DECODE_MERGE = 8,
    SEPATTN_K_EVICT_SIZES = 9,
    SEPATTN_K_EVICT_MOVE = 10,
    SEPATTN_K_CACHE_FILL = 11,
    SEPATTN_K_ROPE_TABLE = 12,
    SEPATTN_K_CACHE_APPEND = 13,
    SEPATTN_K_MARK_INTERVAL = 14,
    SEPATTN_K_DOC_BOUNDS = 15,
    SEPATTN_K_MARK_COMPACT = 16,
    SEPATTN_K_COUNT = 17
} sepattn_kernel_id;
const char *sepattn_kernel_name(int kernel);
typedef struct sepattn_profile sepattn_profile;
int sepattn_profile_create(int kernel, int max_records, sepattn_profile **out);
int sepattn_profile_attach(sepattn_profile *h);
int sepattn_profile_detach(sepattn_profile *h);
int sepattn_profile_read(sepattn_profile *h, float *ms, int max_records, int *n_records);
void sepattn_profile_destroy(sepattn_profile *h);

#ifdef __cplusplus
}
#endif
#endif /* SEPATTN_H */
