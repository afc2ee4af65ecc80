/*
 * ltea.h — C ABI of the SWA + learnable-token-eviction (LTE) token mixer for
 * AMD MI355X (gfx950).
 *
 * The method (paper Sections 3.1.1 and 3.1.3): per KV head a small 1-D CNN over
 * neighbouring past and future tokens scores every KV pair; when a token leaves
 * the sliding window it is kept only if its score passes the threshold (or it
 * is an attention sink), and at most `budget` such pairs per head survive (the
 * highest-scoring ones); each query attends to its window plus its head's
 * retained set.
 *
 * General rules of this boundary
 *   - plain C: no C++ types, no exceptions, no global state; reentrant
 *     (one documented exception: ltea_decode_step_static).
 *   - every pointer that is not a pointer to one of the config structs below is
 *     a DEVICE pointer, allocated, owned and freed by the caller.  The config
 *     structs themselves (ltea_cfg, ltea_cnn, ltea_cache) live in HOST memory
 *     and are read during the call only.
 *   - the library never allocates device memory, never synchronises and never
 *     touches the default stream: kernels are enqueued on `stream` (a
 *     hipStream_t passed as void*, NULL = the null stream) and the call
 *     returns at once.
 *   - all arguments are validated on the host before anything is enqueued: a
 *     negative return value means nothing was launched and no state changed.
 *   - results are deterministic: same inputs, same bits.
 *   - positions are 0-based inside each sequence.  `window` counts the current
 *     token (query i sees i-window+1 .. i).  Token j is an eviction candidate
 *     iff j < sink or logit_j > tau_logit (tau_logit = 0 is the paper's
 *     "retention score > 0.5"); NaN logits never pass.  Candidates are ranked by
 *     (key descending, position ascending) with key = +inf for sinks, else the
 *     fp32 logit; the first `budget` are kept.
 *   - activations (Q, K, V, O, caches, conv weights) are all of cfg->dtype;
 *     logits, scores and biases are fp32; accumulation is fp32.
 */
#ifndef LTEA_H
#define LTEA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LTEA_MAX_CNN_LAYERS 4

typedef enum { LTEA_F32 = 0, LTEA_BF16 = 1 } ltea_dtype;

typedef enum {
  LTEA_OK = 0,
  LTEA_EINVAL = -1,        /* null pointer, bad size, bad stride, inconsistent config      */
  LTEA_EUNSUPPORTED = -2,  /* valid request outside what the kernels implement             */
  LTEA_EWORKSPACE = -3,    /* workspace missing or smaller than ltea_*workspace_bytes says */
  LTEA_EHIP = -4           /* a kernel launch was rejected by the HIP runtime              */
} ltea_status;

/* Scoring CNN of the LTE module (Section 3.1.1; Appendix A): per KV head, a
 * stack of 1-D convolutions over concat(key, value) features (keys in channels
 * 0..D-1, values in D..2D-1), each followed by Swish (beta = 1), then a
 * per-head linear map to one logit.  Each conv is a cross-correlation with
 * "same" zero padding: tap t of layer l reads position
 * j + (t - (kernel[l]-1)/2) * dilation[l]; positions outside the sequence
 * contribute zero at every layer. */
typedef struct ltea_cnn {
  int32_t n_layers;                       /* 1 .. LTEA_MAX_CNN_LAYERS                        */
  int32_t kernel[LTEA_MAX_CNN_LAYERS];    /* odd, >= 1                                       */
  int32_t dilation[LTEA_MAX_CNN_LAYERS];  /* >= 1                                            */
  int32_t c_out[LTEA_MAX_CNN_LAYERS];     /* output channels; input of layer 0 is 2*D        */
  const void *w[LTEA_MAX_CNN_LAYERS];     /* [Hkv][c_out][c_in][kernel], cfg->dtype, device  */
  const float *bias[LTEA_MAX_CNN_LAYERS]; /* [Hkv][c_out] fp32, device                       */
  const void *w_out;                      /* [Hkv][c_out of last layer], cfg->dtype, device  */
  const float *b_out;                     /* [Hkv] fp32, device                              */
  const void *panels;                     /* optional, device: what ltea_cnn_prepare wrote for exactly these weights
                                             and this cfg; NULL: the weights are re-laid on every call (workspace)  */
} ltea_cnn;

typedef struct ltea_cfg {
  int32_t Hq, Hkv, D;      /* query heads, KV heads (Hq % Hkv == 0), head dim in {64, 128}  */
  int32_t window;          /* >= 2*rho+1 where rho = sum_l dilation[l]*(kernel[l]-1)/2       */
  int32_t budget;          /* >= 0, retained KV pairs per (sequence, KV head)                */
  int32_t sink;            /* >= 0, first `sink` positions are always candidates             */
  float tau_logit;         /* candidate iff logit > tau_logit; -INFINITY = pure top-budget   */
  float softmax_scale;     /* <= 0 selects 1/sqrt(D)                                         */
  int32_t dtype;           /* ltea_dtype                                                     */
} ltea_cfg;

/* Cache state of B sequences (Section 3.1.3, cache-layout figure): a circular
 * sliding-window segment plus a compact out-of-window segment per
 * (sequence, KV head).  All arrays are device memory owned by the caller and
 * are updated in place.  The physical order inside the compact segment is not
 * part of the contract (prefill leaves it ascending by position; decode
 * appends or overwrites single slots). */
typedef struct ltea_cache {
  void *k_win, *v_win;   /* [B][Hkv][window][D]  ring; position p lives in slot p % window   */
  float *win_score;      /* [B][Hkv][window]     logits of ring tokens; final for p < n_scored */
  void *k_ret, *v_ret;   /* [B][Hkv][budget][D]  retained KV pairs                            */
  float *ret_score;      /* [B][Hkv][budget]     their selection keys (+inf for sinks)        */
  int32_t *ret_pos;      /* [B][Hkv][budget]     their positions                              */
  int32_t *ret_count;    /* [B][Hkv]             valid entries, <= budget                     */
  int32_t *n_seen;       /* [B]                  tokens consumed so far                       */
  int32_t *n_scored;     /* [B]                  = max(0, n_seen - rho) after every call      */
} ltea_cache;

/* The matrix-core scoring kernels read the conv weights re-laid as tap-major panels.  By default every call that
 * scores re-lays them: inside the scoring launch itself where the weights fit the register file (bf16, D = 64: one
 * layer of kernel size 3 or 5, and the three-layer stack of Appendix A) and the weight tensors are 16-byte aligned,
 * else with a launch of its own into the workspace (a few microseconds); weights that do not change between calls
 * can be prepared once instead: ltea_cnn_prepare fills `panels` (device, ltea_cnn_panels_bytes bytes, 0 if this
 * configuration runs on kernels that need none), and a ltea_cnn whose `panels` member points there makes every
 * entry point skip the re-layout.  The caller keeps `panels` alive and redoes the preparation when the weights
 * change; cnn->panels is ignored by ltea_cnn_prepare itself. */
size_t ltea_cnn_panels_bytes(const ltea_cfg *cfg, const ltea_cnn *cnn);
int ltea_cnn_prepare(const ltea_cfg *cfg, const ltea_cnn *cnn, void *panels, size_t panels_bytes, void *stream);

/* Human-readable text for a status code (static storage). */
const char *ltea_strerror(int status);

/* Bytes of device workspace ltea_score / ltea_retain / ltea_sparse_attention /
 * ltea_prefill need for these sizes (0 is a valid answer).  Returns 0 on
 * invalid arguments as well; the entry points report those themselves.
 * Every workspace pointer of this library, here and below, must be 256-byte
 * aligned (device allocations are); a misaligned one is LTEA_EINVAL. */
size_t ltea_workspace_bytes(const ltea_cfg *cfg, const ltea_cnn *cnn, int32_t n_seqs, int64_t total_tokens,
                            int32_t max_seqlen);

/* Bytes of device workspace ltea_decode_step needs for n_seqs sequences (contents need no initialisation
 * and need not be preserved between steps).  With `cnn` given the size also covers the faster scoring path of
 * multi-layer bf16 CNNs (receptive-field windows of the whole batch packed and scored by the fused prefill kernel);
 * with cnn == NULL, or a smaller workspace passed to ltea_decode_step, that CNN is scored per (sequence, head). */
size_t ltea_decode_workspace_bytes(const ltea_cfg *cfg, const ltea_cnn *cnn, int32_t n_seqs);

/* (a) Scoring (Section 3.1.1): logits[h][t] for every packed token t and KV
 * head h.  k, v: [total_tokens][Hkv][D] views with element strides stride_tok
 * and stride_head (innermost dimension contiguous).  cu_seqlens: device int32
 * [n_seqs+1], non-decreasing, cu_seqlens[0] = 0, cu_seqlens[n_seqs] =
 * total_tokens; max_seqlen >= every length.  The convolution never crosses a
 * sequence boundary.  logits: [Hkv][total_tokens] fp32 (the last rho logits of
 * each sequence are provisional: their right context is zero padding). */
int ltea_score(const ltea_cfg *cfg, const ltea_cnn *cnn, const void *k, const void *v, int64_t stride_tok,
               int64_t stride_head, const int32_t *cu_seqlens, int32_t n_seqs, int64_t total_tokens,
               int32_t max_seqlen, float *logits, void *workspace, size_t workspace_bytes, void *stream);

/* (b) Retention and cache fill (eq. 5; Section 3.1.3 "Capped capacity" and
 * "Cached prefilling"): from given logits [Hkv][total_tokens], select per
 * (sequence, KV head) the kept out-of-window positions, gather their K, V, key
 * and position ascending by position into the compact segment, copy the last
 * min(n, window) tokens and their logits into the ring, and set ret_count,
 * n_seen = n and n_scored = max(0, n - rho).  Unused compact slots are left
 * untouched.  cache arrays are sized for B = n_seqs. */
int ltea_retain(const ltea_cfg *cfg, const float *logits, const void *k, const void *v, int64_t stride_tok,
                int64_t stride_head, const int32_t *cu_seqlens, int32_t n_seqs, int64_t total_tokens,
                int32_t max_seqlen, int32_t rho, const ltea_cache *cache, void *workspace, size_t workspace_bytes,
                void *stream);

/* (c) Prefill attention over window + retained set (Section 3.1.3): for query
 * i of a sequence and query head hq (KV head hq / (Hq/Hkv)),
 *   out_i = softmax_j(scale * q_i . k_j) v_j  over
 *   { max(0, i-window+1) <= j <= i }  union  { retained j : j <= i - window }.
 * Reads only ret_pos / ret_count / k_ret / v_ret of `cache`.  q: view
 * [total_tokens][Hq][D] with element strides q_stride_tok / q_stride_head;
 * out: contiguous [total_tokens][Hq][D]. */
int ltea_sparse_attention(const ltea_cfg *cfg, const void *q, int64_t q_stride_tok, int64_t q_stride_head,
                          const void *k, const void *v, int64_t kv_stride_tok, int64_t kv_stride_head,
                          const int32_t *cu_seqlens, int32_t n_seqs, int64_t total_tokens, int32_t max_seqlen,
                          const ltea_cache *cache, void *out, void *workspace, size_t workspace_bytes,
                          void *stream);

/* (a)+(b)+(c): scores every token, fills the cache state of all n_seqs
 * sequences, and writes the attention output of every token.  Mid-sequence
 * queries see the FINAL capped retained set of their sequence, restricted to
 * positions that have left their window.  logits_or_null, if given, receives
 * the [Hkv][total_tokens] logits. */
int ltea_prefill(const ltea_cfg *cfg, const ltea_cnn *cnn, const void *q, int64_t q_stride_tok,
                 int64_t q_stride_head, const void *k, const void *v, int64_t kv_stride_tok, int64_t kv_stride_head,
                 const int32_t *cu_seqlens, int32_t n_seqs, int64_t total_tokens, int32_t max_seqlen, void *out,
                 const ltea_cache *cache, float *logits_or_null, void *workspace, size_t workspace_bytes,
                 void *stream);

/* ltea_prefill for models whose cached keys differ from the keys the scoring CNN is trained on (rotary position
 * encoding: Section 3.1.1 scores keys as they are before the rotation, the cache holds them after it): k_feat, a view
 * with the strides of k, is what the CNN scores; k is what is cached and attended.  ltea_prefill is this call with
 * k_feat = k.  (Such a cache is continued with ltea_prefill_append_feat and decoded with ltea_decode_step_feat or
 * ltea_decode_step_lazy + ltea_rescore, all of which take the model's rotary tables.) */
int ltea_prefill_feat(const ltea_cfg *cfg, const ltea_cnn *cnn, const void *q, int64_t q_stride_tok,
                      int64_t q_stride_head, const void *k, const void *v, const void *k_feat, int64_t kv_stride_tok,
                      int64_t kv_stride_head, const int32_t *cu_seqlens, int32_t n_seqs, int64_t total_tokens,
                      int32_t max_seqlen, void *out, const ltea_cache *cache, float *logits_or_null, void *workspace,
                      size_t workspace_bytes, void *stream);

/* (d) One decode step for n_seqs sequences (Section 3.1.3, cache replacement
 * and lazy scoring paragraphs): for sequence b with t = n_seen[b],
 *   1. the logit of position t - rho becomes final (its receptive field
 *      t-2rho .. t is the 2*rho newest ring rows plus the incoming token);
 *   2. position e = t - window leaves the window: if it is a candidate it is
 *      appended to the compact segment, or, when that is full, overwrites the
 *      entry with the lowest key (among equal keys the latest position) iff
 *      its own key is strictly higher;
 *   3. k_t, v_t go to ring slot t % window; n_seen, n_scored advance;
 *   4. out = attention of q_t over the ring's valid rows plus the compact rows.
 * q: contiguous [n_seqs][Hq][D]; k, v: contiguous [n_seqs][Hkv][D]; out:
 * contiguous [n_seqs][Hq][D].  Requires the invariant n_scored = max(0,
 * n_seen - rho) on entry (true after ltea_retain / ltea_prefill / a previous
 * step, and for an all-zero fresh cache).  Concurrent calls on the same cache or
 * the same workspace race.  A CNN whose per-step activation rows, 2 * (2*rho+1) *
 * max(2*D, widest layer) floats, exceed 48 KB of LDS is scored through the prefill
 * kernels instead (as ltea_decode_step_feat does): that needs the workspace
 * ltea_decode_workspace_bytes(cfg, cnn, n_seqs) reports, LTEA_EWORKSPACE otherwise. */
int ltea_decode_step(const ltea_cfg *cfg, const ltea_cnn *cnn, const void *q, const void *k, const void *v,
                     void *out, const ltea_cache *cache, int32_t n_seqs, void *workspace, size_t workspace_bytes,
                     void *stream);

/* ltea_decode_step for callers that cannot allocate device memory or pass a workspace: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * ltea_decode_step, minus the workspace: the step's scratch (split partials, finalised logits, step indices) is a
 * fixed device array of LTEA_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process
 * ends.  This is the one entry point with state of its own, so unlike the rest of the boundary it is not
 * reentrant: every call on a GPU shares that GPU's array, and calls that overlap in time on one GPU (different
 * streams or threads) race.  Nothing is carried from one call to the next.  Calls no hipMalloc, hipFree or other
 * allocating routine; the first call on a device looks the array's device address up once.
 * Returns LTEA_EWORKSPACE, before anything is launched, when ltea_decode_workspace_bytes(cfg, cnn, n_seqs) exceeds
 * LTEA_STATIC_SCRATCH_BYTES (decode_bf16's 64 sequences x 16 heads x D = 128 need about 2.2 MB). */
#define LTEA_STATIC_SCRATCH_BYTES (8u << 20)
int ltea_decode_step_static(const ltea_cfg *cfg, const ltea_cnn *cnn, const void *q, const void *k, const void *v,
                            void *out, const ltea_cache *cache, int32_t n_seqs, void *stream);

/* Continues a prefill on an existing cache state (the chunked / multi-token form of (a)+(b)+(c)): sequence s of
 * `cache` holds n_seen[s] tokens (from ltea_prefill, ltea_decode_step or an earlier call of this function) and
 * receives cu_new[s+1] - cu_new[s] >= 0 new tokens (q, k, v: packed views as in ltea_prefill; out: contiguous
 * [total_new][Hq][D]).  Outputs and the final state equal those rows and that state of one ltea_prefill over the
 * whole history: new queries see their window plus the final capped retained set restricted to positions that have
 * left their window; the retained set is re-selected among the old retained entries and the tokens that leave the
 * window now (tokens dropped earlier stay dropped, which is what a one-shot prefill would also have decided).
 * Workspace: ltea_append_workspace_bytes. */
size_t ltea_append_workspace_bytes(const ltea_cfg *cfg, const ltea_cnn *cnn, int32_t n_seqs, int64_t total_new,
                                   int32_t max_new);
int ltea_prefill_append(const ltea_cfg *cfg, const ltea_cnn *cnn, const void *q, int64_t q_stride_tok,
                        int64_t q_stride_head, const void *k, const void *v, int64_t kv_stride_tok,
                        int64_t kv_stride_head, const int32_t *cu_new, int32_t n_seqs, int64_t total_new,
                        int32_t max_new, void *out, const ltea_cache *cache, void *workspace, size_t workspace_bytes,
                        void *stream);

/* ---- lazy scoring during decode (Section 3.1.3, lazy scoring paragraph) ------------------------------------
 * Instead of finalising one logit per step, the caller may run ltea_decode_step_lazy (no scoring at all) and call
 * ltea_rescore every so often, which finalises the logits of all positions n_scored .. n_seen - rho - 1 of every
 * sequence in one batched pass over the ring and restores n_scored = max(0, n_seen - rho).  A token's logit is
 * needed when it leaves the window, and its receptive field must still be in the ring when it is scored, so at
 * most ltea_lazy_period() = window - 2*rho lazy steps may follow ltea_prefill / ltea_retain / ltea_prefill_append /
 * ltea_rescore / an eager step before the next ltea_rescore.  The resulting cache state and outputs equal those
 * of eager steps.  ltea_decode_step and ltea_prefill_append expect the invariant n_scored = max(0, n_seen - rho):
 * call ltea_rescore before going back to them.
 *
 * Violations of the period cannot be seen from the host; they are reported through `status`, an optional device
 * int32 the kernels OR bits into (the caller zeroes it and reads it when convenient): */
#define LTEA_LATE_SCORING 1 /* set by ltea_rescore when the left context of an unscored token has already left the
                               window (the period was exceeded: the logits it writes for that sequence are
                               unspecified), and by ltea_decode_step_lazy when the token that leaves the window has
                               no final logit (that step's output rows of the sequence are NaN and its kept set is
                               unspecified from then on)                                                           */
#define LTEA_ROPE_RANGE 2   /* a cached position lies beyond the rotary tables: that key was left as it is          */

/* Rotary position encoding as the model holds it ("cached sinusoids"): row p of the tables rotates pair i of a
 * key at position p, (a, b) -> (a cos - b sin, a sin + b cos), with pair i = (x[i], x[i + rot_dim/2]), or
 * (x[2i], x[2i+1]) when `interleaved`; features from rot_dim on are not rotated.  Given to ltea_rescore,
 * ltea_decode_step_feat or ltea_prefill_append_feat, the cache is taken to hold rotated keys and the scoring CNN sees
 * them rotated back (same tables, negated sines, each row at its own position), rounded to cfg->dtype. */
typedef struct ltea_rope {
  const float *cos, *sin; /* [n_pos][rot_dim/2] fp32, device                                    */
  int32_t n_pos;          /* table rows; every cached position must be below it                  */
  int32_t rot_dim;        /* multiple of 16, <= D                                                */
  int32_t interleaved;    /* 0 or 1                                                              */
} ltea_rope;

/* window - 2*rho (>= 1), or 0 on invalid arguments. */
int32_t ltea_lazy_period(const ltea_cfg *cfg, const ltea_cnn *cnn);

/* Workspace of ltea_rescore: the packed ring rows of all sequences, their logits and the scoring kernels' own
 * workspace (about 2 * n_seqs * window * Hkv * D elements). */
size_t ltea_rescore_workspace_bytes(const ltea_cfg *cfg, const ltea_cnn *cnn, int32_t n_seqs);

/* Batched scoring of the unscored in-window positions (see above).  rope_or_null: NULL scores the cached keys as
 * they are.  Only win_score and n_scored of `cache` are written. */
int ltea_rescore(const ltea_cfg *cfg, const ltea_cnn *cnn, const ltea_rope *rope_or_null, const ltea_cache *cache,
                 int32_t n_seqs, int32_t *status_or_null, void *workspace, size_t workspace_bytes, void *stream);

/* ltea_decode_step for models that cache rotated keys: the keys in the receptive field of the token being finalised
 * (ring rows of positions t - 2*rho .. t - 1) are rotated back with `rope` before the CNN sees them; the incoming
 * token's scoring key is k_feat_or_null (contiguous [n_seqs][Hkv][D], the key before the rotation) or, when NULL, k
 * rotated back at position t.  k, the rotated key, is what is cached and attended.  Same state and outputs as
 * ltea_decode_step_lazy followed by ltea_rescore after every step.  rope == NULL scores the keys as they are (then
 * k_feat must be NULL too).  status_or_null receives LTEA_ROPE_RANGE.  Works for every CNN shape ltea_score
 * accepts (the windows are packed and scored by the prefill kernels: three more launches than ltea_decode_step).
 * Workspace: ltea_decode_feat_workspace_bytes. */
size_t ltea_decode_feat_workspace_bytes(const ltea_cfg *cfg, const ltea_cnn *cnn, int32_t n_seqs);
int ltea_decode_step_feat(const ltea_cfg *cfg, const ltea_cnn *cnn, const ltea_rope *rope_or_null, const void *q,
                          const void *k, const void *v, const void *k_feat_or_null, void *out, const ltea_cache *cache,
                          int32_t n_seqs, int32_t *status_or_null, void *workspace, size_t workspace_bytes,
                          void *stream);

/* ltea_prefill_append for models that cache rotated keys.  rope_or_null: the ring's keys are rotated back at their
 * positions for the scoring CNN, exactly as ltea_rescore does it.  k_feat_or_null: the new tokens' keys as they
 * were before the rotation (same strides as k); NULL rotates the new keys back too (positions n_seen[s] + i), so the
 * caller need not keep them.  k, the rotated keys, are what is cached and attended.  Results equal ltea_prefill_feat
 * over the whole history up to the rounding of the keys that are rotated back.  status_or_null receives
 * LTEA_ROPE_RANGE when a position lies beyond the tables (that key is scored as cached).  rope == NULL with
 * k_feat == NULL is ltea_prefill_append; k_feat without rope is LTEA_EINVAL.  Requires n_scored = max(0, n_seen - rho)
 * on entry like ltea_prefill_append.  Workspace: ltea_append_workspace_bytes. */
int ltea_prefill_append_feat(const ltea_cfg *cfg, const ltea_cnn *cnn, const ltea_rope *rope_or_null, const void *q,
                             int64_t q_stride_tok, int64_t q_stride_head, const void *k, const void *v,
                             const void *k_feat_or_null, int64_t kv_stride_tok, int64_t kv_stride_head,
                             const int32_t *cu_new, int32_t n_seqs, int64_t total_new, int32_t max_new, void *out,
                             const ltea_cache *cache, int32_t *status_or_null, void *workspace, size_t workspace_bytes,
                             void *stream);

/* ltea_decode_step without step 1: position t - window is evicted on the logit win_score already holds for it,
 * n_scored is left alone.  Arguments as ltea_decode_step; workspace: ltea_decode_workspace_bytes(cfg, NULL, n_seqs). */
int ltea_decode_step_lazy(const ltea_cfg *cfg, const void *q, const void *k, const void *v, void *out,
                          const ltea_cache *cache, int32_t n_seqs, int32_t *status_or_null, void *workspace,
                          size_t workspace_bytes, void *stream);

/* ---- training side (Section 3.1.2 "Adaptive training"; Algorithm 1) -----------------------------------------
 * During training no cap applies: query i sees its window plus every candidate (sink, or logit > tau_logit) that
 * has left it; cfg->budget is ignored by these entry points.  The forward is ltea_prefill's pipeline with the cap
 * lifted and also returns the softmax normalisers; the state it leaves in `workspace` (the compacted candidates)
 * must reach ltea_train_backward unchanged.  The CNN's own backward (d logits -> d weights, d features) is
 * ltea_cnn_backward below; its dropout is not part of this library. */
/* cnn may be NULL (logits supplied by the caller). */
size_t ltea_train_workspace_bytes(const ltea_cfg *cfg, const ltea_cnn *cnn, int32_t n_seqs, int64_t total_tokens,
                                  int32_t max_seqlen);

/* out: contiguous [total_tokens][Hq][D]; lse: [Hq][total_tokens] fp32, natural log of sum_j exp(scale q_i.k_j) over
 * the keys query i sees; logits: [Hkv][total_tokens] fp32.  With `cnn` given the logits are computed and written
 * (rho is ignored).  With cnn == NULL the logits are an INPUT: a framework that runs the scoring CNN under its own
 * autograd passes its logits here (and rho, the CNN's look-ahead, which must satisfy window >= 2*rho + 1) and feeds
 * the d logits of ltea_train_backward back into its graph; a rotary model passes the logits ltea_score gives for its
 * unrotated keys, k here being the rotated ones (and hands the same unrotated keys to ltea_cnn_backward).  Other
 * arguments as ltea_prefill. */
int ltea_train_forward(const ltea_cfg *cfg, const ltea_cnn *cnn, const void *q, int64_t q_stride_tok,
                       int64_t q_stride_head, const void *k, const void *v, int64_t kv_stride_tok,
                       int64_t kv_stride_head, const int32_t *cu_seqlens, int32_t n_seqs, int64_t total_tokens,
                       int32_t max_seqlen, int32_t rho, void *out, float *lse, float *logits, void *workspace,
                       size_t workspace_bytes, void *stream);

/* Gradients for d(loss)/d(out) = dout (contiguous [total_tokens][Hq][D], cfg->dtype):
 *   dq [total_tokens][Hq][D], dk, dv [total_tokens][Hkv][D] (contiguous, cfg->dtype, fp32 accumulation; dk and dv
 *   are the attention's gradients only: what flows into k, v through the scoring CNN is the caller's);
 *   dz [Hkv][total_tokens] fp32 = (<v_j, dv_j> + lambda[h] * 1[logit_j > tau_logit]) * r_j (1 - r_j), r = sigmoid(logit):
 *   the straight-through surrogate d(loss)/d r_j := <v_j, d(loss)/d v_j> plus the gradient of the sparsity penalty
 *   sum_h lambda_h sum_j ReLU(r_j - sigmoid(tau_logit));
 *   counts [n_seqs][Hkv] int32 = #{j : logit_j > tau_logit} (the c of the penalty-weight feedback).
 * q, k, v, cu_seqlens, out, lse, logits: what ltea_train_forward was given / returned; lambda: [Hkv] fp32, device. */
int ltea_train_backward(const ltea_cfg *cfg, const void *q, int64_t q_stride_tok, int64_t q_stride_head,
                        const void *k, const void *v, int64_t kv_stride_tok, int64_t kv_stride_head,
                        const int32_t *cu_seqlens, int32_t n_seqs, int64_t total_tokens, int32_t max_seqlen,
                        const void *out, const void *dout, const float *lse, const float *logits, const float *lambda,
                        void *dq, void *dk, void *dv, float *dz, int32_t *counts, void *workspace,
                        size_t workspace_bytes, void *stream);

/* Backward of the scoring CNN (the module of Section 3.1.1, trained through the d logits above): gradients of
 * L = sum_{h,t} dz[h][t] * logit[h][t] with respect to every parameter and to the input features.  `grad` holds device
 * fp32 arrays of the shapes of the weights (w[l]: [Hkv][c_out][c_in][kernel], bias[l]: [Hkv][c_out], w_out:
 * [Hkv][c_out of the last layer], b_out: [Hkv]); they are overwritten, not accumulated into (sums over all tokens of
 * all sequences, fp32, fixed order).  dk_feat_or_null / dv_or_null: contiguous [total_tokens][Hkv][D] of cfg->dtype,
 * the gradient that reaches the scored keys and the values through the CNN (to be added to the attention's dk / dv
 * by a caller that trains them through this path too).  k_feat, v, cu_seqlens: as given to ltea_score /
 * ltea_train_forward (k_feat = the keys the CNN scores).  cnn->panels is not used.  fp32-accurate arithmetic for every
 * CNN shape and storage type: products on the fp32 matrix instruction, or, on bf16 storage where one operand is a
 * bf16 value, on the bf16 one with the fp32 operand split into three bf16 terms. */
typedef struct ltea_cnn_grad {
  float *w[LTEA_MAX_CNN_LAYERS];
  float *bias[LTEA_MAX_CNN_LAYERS];
  float *w_out;
  float *b_out;
} ltea_cnn_grad;
size_t ltea_cnn_backward_workspace_bytes(const ltea_cfg *cfg, const ltea_cnn *cnn, int64_t total_tokens);
int ltea_cnn_backward(const ltea_cfg *cfg, const ltea_cnn *cnn, const void *k_feat, const void *v, int64_t stride_tok,
                      int64_t stride_head, const int32_t *cu_seqlens, int32_t n_seqs, int64_t total_tokens,
                      int32_t max_seqlen, const float *dz, const ltea_cnn_grad *grad, void *dk_feat_or_null,
                      void *dv_or_null, void *workspace, size_t workspace_bytes, void *stream);

/* One feedback step on n penalty weights (Algorithm 1), on HOST arrays: lambda_i is multiplied by alpha where the
 * averaged count c_bar_i exceeds cap, divided by alpha where it is below 0.95 cap, clamped to <= 1, flushed to 0
 * below 1e-9, and restarted from 1e-9 where it is 0 while c_bar_i > cap. */
int ltea_lambda_update(float *lambda, const float *c_bar, int32_t n, float cap, float alpha);

/* ---- measurement aids (not part of the method; the hot-path entry points above never call them) ----------
 * What the chip sustains on the two resources the roofline figures are quoted against, so that a report can
 * give a fraction of the measured ceiling next to the fraction of the datasheet peak.  Both launch
 * LTEA_DIAG_BLOCKS workgroups of 256 threads on `stream` and return at once; `sink` is device memory of at
 * least ltea_diag_sink_bytes() bytes that receives per-thread checksums (so the work cannot be elided). */
#define LTEA_DIAG_BLOCKS 4096
size_t ltea_diag_sink_bytes(void);

/* Register-resident loop of bf16 32x32x16 MFMAs, 8 per iteration per wave, no memory traffic.  *flops_out
 * (host, optional) receives the floating-point operations one launch performs. */
int ltea_diag_mfma_loop(int32_t iters, void *sink, double *flops_out, void *stream);

/* Reads every byte of [src, src+bytes) once with 16-byte loads, one contiguous share per workgroup
 * (bytes % 16 == 0, src 16-byte aligned). */
int ltea_diag_stream_read(const void *src, size_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LTEA_H */
