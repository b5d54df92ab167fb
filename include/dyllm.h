/*
 * dyllm.h - C ABI of the MI355X (gfx950) library for DyLLM's per-denoising-step
 * sparse layer update.
 *
 * One call = one transformer layer, one denoising step.  The salient tokens of
 * the step get their K/V rows refreshed, their exact attention rows recomputed
 * against all keys, a cosine test against the cached previous context, and --
 * for those that pass the test -- output projection and FFN; every other token
 * reuses its cached K, V, context and layer output.
 * [App. C.3, Alg. 3 (SparseStep), layer body; Sec. 3.1-3.3]
 *
 * Conventions (all entry points)
 *  - Every tensor pointer is DEVICE memory owned by the caller (allocated and
 *    freed by the caller); the library owns only the scratch workspace of its
 *    context.  Pointers named host_* are host memory.
 *  - Tensors are dense row-major (the weight matrices of bf16 contexts excepted:
 *    see dyllm_layer_weights).  A "token id" is b*L + i for position i of
 *    sequence b; T = B*L.  Element type is the context's dtype (fp32 or bf16)
 *    unless a parameter says otherwise.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work on it: no device synchronisation, no device-to-host
 *    copy.  Row counts stay on the device (offsets[B]).
 *  - Return value: 0 on success, a negative DYLLM_ERR_* code otherwise.
 *    Argument and shape errors are found on the host before anything is
 *    launched.  Nothing throws, aborts or prints.  dyllm_last_error gives a
 *    message for the last failing call on a context.
 *  - A context is not thread-safe; calls that share a context must be ordered
 *    on one stream.
 */
#ifndef DYLLM_H
#define DYLLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DYLLM_OK 0
#define DYLLM_ERR_INVALID_ARG (-1) /* NULL pointer, negative size, bad enum */
#define DYLLM_ERR_BAD_SHAPE (-2)   /* sizes inconsistent with the context's configuration */
#define DYLLM_ERR_UNSUPPORTED (-3) /* shape the kernels are not written for */
#define DYLLM_ERR_NO_MEM (-4)      /* workspace allocation failed */
#define DYLLM_ERR_HIP (-5)         /* a HIP runtime call failed */
#define DYLLM_ERR_CAPACITY (-6)    /* an index list did not fit its capacity (see dyllm_poll_status) */

typedef struct dyllm_ctx dyllm_ctx; /* opaque; owns only scratch workspace */

typedef enum { DYLLM_F32 = 0, DYLLM_BF16 = 1 } dyllm_dtype;

/* Layer configuration.  hidden must equal n_heads*head_dim is NOT required;
 * n_heads must be a multiple of n_kv_heads (query head h reads KV head
 * h / (n_heads/n_kv_heads)).  Kernel limits: head_dim 64 or 128; hidden,
 * n_heads*head_dim and ffn_dim multiples of 64 (bf16: of 128). */
typedef struct {
  int32_t hidden;     /* d */
  int32_t n_heads;    /* H */
  int32_t n_kv_heads; /* Hkv */
  int32_t head_dim;   /* dh */
  int32_t ffn_dim;    /* F */
  int32_t max_batch;  /* largest B of any call */
  int32_t max_seq;    /* largest L of any call */
  int32_t max_rows;   /* largest number of rows one call recomputes (capacity of its index
                         lists); 0 means max_batch*max_seq, which dyllm_full_step needs */
  int32_t dtype;      /* dyllm_dtype: storage type of weights, activations and caches */
  float rms_eps;      /* added to the mean square inside RMSNorm's square root */
  float rope_theta;   /* rotary base */
} dyllm_layer_cfg;

/* Weights of one layer, y = W x (+ b); the shapes below are [out, in].
 * DYLLM_F32 contexts read every matrix row-major.  DYLLM_BF16 contexts read every matrix in the
 * panel layout written by dyllm_pack_weight (the GEMM kernels stream each tile's share of a matrix
 * as contiguous 4 KB runs instead of one 128-byte piece per row); biases and gains are plain
 * vectors in both. */
typedef struct {
  const void *wq;     /* [H*dh, d] */
  const void *wk;     /* [Hkv*dh, d] */
  const void *wv;     /* [Hkv*dh, d] */
  const void *wo;     /* [d, H*dh] */
  const void *w_gate; /* [F, d] */
  const void *w_up;   /* [F, d] */
  const void *w_down; /* [d, F] */
  const void *bq;     /* [H*dh] or NULL */
  const void *bk;     /* [Hkv*dh] or NULL */
  const void *bv;     /* [Hkv*dh] or NULL */
  const void *g_attn; /* [d] RMSNorm gain before attention */
  const void *g_ffn;  /* [d] RMSNorm gain before the FFN */
} dyllm_layer_weights;

/* The four per-layer caches [Alg. 1 initialisation; Alg. 2 / Alg. 3 cache lines], updated in place,
 * and an optional fifth one for the reused-normaliser form of the approximate update. */
typedef struct {
  void *k;   /* [B, L, Hkv, dh]  keys, stored AFTER the rotary embedding */
  void *v;   /* [B, L, Hkv, dh] */
  void *c;   /* [B, L, H*dh]     attention context, before the output projection */
  void *out; /* [B, L, d]        layer output hidden state ("FFN output cache") */
  float *lse; /* NULL, or [B, L, H] fp32: log(sum_j exp(q.k_j/sqrt(dh))) of every token's last EXACT
                 attention row; written by the dense step and for the exact rows of every sparse step */
} dyllm_layer_cache;

/* A set of tokens: ascending, unique token ids, grouped by sequence. */
typedef struct {
  int32_t *idx;     /* [cap] token ids b*L+i; entries beyond the count are undefined; may be NULL
                       if cap is 0 */
  int32_t *offsets; /* [B+1] offsets[b]..offsets[b+1] = entries of sequence b; offsets[B] = count */
  int32_t cap;      /* capacity of idx (host value); the count on the device must not exceed it */
} dyllm_index_list;

/* Re-lays a row-major bf16 matrix src [n_out, n_in] (device) into dst (device, same number of
 * bytes, must not overlap src) in the layout the bf16 GEMMs of Alg. 3's projection and FFN lines
 * read: panels of 32 output rows, each panel stored K-slice-major,
 *   dst[((n/32) * (n_in/64) + k/64) * 2048 + (n%32) * 64 + k%64] = src[n * n_in + k].
 * Call once per matrix when the weights are loaded; the row-major copy is not needed afterwards.
 * Only enqueues on `stream`.  Errors: INVALID_ARG (NULL, src == dst, sizes <= 0), UNSUPPORTED
 * (n_out not a multiple of 32 or n_in not a multiple of 64), HIP. */
int dyllm_pack_weight(const void *src, int32_t n_out, int32_t n_in, void *dst, void *stream);

/* Bytes of device scratch a context with this configuration allocates. */
int dyllm_workspace_bytes(const dyllm_layer_cfg *cfg, size_t *host_bytes);

/* Creates a context on the current HIP device (allocates its workspace once).
 * Errors: INVALID_ARG, UNSUPPORTED (kernel limits above), NO_MEM. */
int dyllm_create(const dyllm_layer_cfg *cfg, dyllm_ctx **host_ctx_out);
/* Frees the workspace.  The caller must have synchronised the streams it used. */
int dyllm_destroy(dyllm_ctx *ctx);

const char *dyllm_strerror(int code);
const char *dyllm_last_error(const dyllm_ctx *ctx);

/* Copies the context's device status word (0, or DYLLM_ERR_CAPACITY if some kernel since the
 * last poll found more rows than a list's capacity and dropped the excess) to *host_status.
 * This is the one call that synchronises `stream`. */
int dyllm_poll_status(dyllm_ctx *ctx, int32_t *host_status, void *stream);

/* Temporal cosine similarity and the salient test.  [Sec. 3.1; Sec. 3.2: A = {i : s_i < tau}]
 *   rows != NULL: c_new is [count, D] (row j belongs to token rows->idx[j]) and is compared with
 *                 c_cache[rows->idx[j]]; cos_out / flag_out are [rows->cap] (count entries written).
 *   rows == NULL: c_new and c_cache are both [B*L, D]; cos_out / flag_out are [B*L].
 * D = n_heads*head_dim.  s = <a,b> / (max(|a|,1e-8) * max(|b|,1e-8)), accumulated in fp32 over the
 * stored values; flag = (s < tau), strict.  With commit != 0 the old cache row is read first and
 * then overwritten with the new row [Alg. 3 cache commit]; commit requires rows != NULL or
 * c_new != c_cache.  cos_out may be NULL. */
int dyllm_saliency(dyllm_ctx *ctx, const void *c_new, void *c_cache, const dyllm_index_list *rows,
                   int32_t B, int32_t L, float tau, float *cos_out, uint8_t *flag_out, int commit,
                   void *stream);

/* Stable compaction of the flagged tokens into an ascending index list.  [Alg. 3: where(...)]
 * flag[j] != 0 selects token rows->idx[j] (rows != NULL, j < count) or token j (rows == NULL,
 * j < B*L).  Writes out->idx, out->offsets[0..B].  If more than out->cap tokens are flagged the
 * excess is dropped and the status word is set (dyllm_poll_status). */
int dyllm_compact(dyllm_ctx *ctx, const uint8_t *flag, const dyllm_index_list *rows, int32_t B,
                  int32_t L, dyllm_index_list *out, void *stream);

/* dyllm_compact for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  It takes no context (dyllm_create allocates one)
 * and calls no allocating routine; the few counter and partial-count words its kernel needs live in a
 * fixed array inside the library's code object (4352 bytes per GPU, held until the process ends).
 * Same inputs, outputs and results as dyllm_compact.  B*L (rows == NULL) or rows->cap may be at most
 * DYLLM_COMPACT_STATIC_MAX_ROWS; a larger request returns DYLLM_ERR_CAPACITY and launches nothing.
 * status: NULL, or a device word that receives DYLLM_ERR_CAPACITY when more than out->cap tokens are
 * flagged (the excess is dropped); it is not written otherwise.
 * Every call on one GPU shares that GPU's array: calls that may overlap on one GPU (different
 * streams without an ordering between them) race; calls on one stream are safe.  The first call on
 * a device looks the array's address up once (no allocation), so make it outside stream capture. */
#define DYLLM_COMPACT_STATIC_MAX_ROWS (1 << 20)
int dyllm_compact_static(const uint8_t *flag, const dyllm_index_list *rows, int32_t B, int32_t L,
                         dyllm_index_list *out, int32_t *status, void *stream);

/* K/V refresh of the salient rows.  [Alg. 3: norm, q_proj, k_proj / v_proj merge lines]
 * For every token r in rows: n = RMSNorm(x[r]; g_attn); q, k, v = W n (+ b); q and k rotated by the
 * rotary embedding at position r mod L; cache->k[r] = k, cache->v[r] = v (other rows untouched);
 * q_sal_out[j] = q for the j-th entry of rows, layout [rows->cap, H, dh]. */
int dyllm_qkv_refresh(dyllm_ctx *ctx, const dyllm_layer_weights *w, const void *x,
                      const dyllm_index_list *rows, int32_t B, int32_t L, dyllm_layer_cache *cache,
                      void *q_sal_out, void *stream);

/* Exact attention rows for the salient queries against ALL keys and values of their own sequence,
 * bidirectional (no mask), softmax scale 1/sqrt(dh).  [Sec. 3.3 salient path; Alg. 3: C_sal]
 * q_sal: [rows->cap, H, dh] (count rows used); k_cache, v_cache: [B, L, Hkv, dh];
 * c_sal_out: [rows->cap, H*dh]. */
int dyllm_partial_attention(dyllm_ctx *ctx, const void *q_sal, const void *k_cache,
                            const void *v_cache, const dyllm_index_list *rows, int32_t B, int32_t L,
                            void *c_sal_out, void *stream);

/* Output projection + residual, RMSNorm, SwiGLU FFN + residual for the tokens in rows_out, written
 * into out_cache at those rows only.  [Alg. 3: out_proj / FFN / cache lines; Sec. 3.2]
 *   h = x[r] + Wo c[r];  y = h + Wdown( silu(Wgate f) * (Wup f) ), f = RMSNorm(h; g_ffn);
 *   out_cache[r] = y.
 * x: [B*L, d] layer input; c: [B*L, H*dh] merged attention context (the context cache after its
 * commit); out_cache: [B*L, d]. */
int dyllm_salient_ffn(dyllm_ctx *ctx, const dyllm_layer_weights *w, const void *x, const void *c,
                      const dyllm_index_list *rows_out, int32_t B, int32_t L, void *out_cache,
                      void *stream);

/* One layer of SparseStep on the salient path.  [Alg. 3 layer body; Sec. 3.2-3.3]
 * = dyllm_qkv_refresh(idx_in) -> dyllm_partial_attention -> dyllm_saliency(commit) ->
 *   dyllm_compact -> dyllm_salient_ffn(idx_out), all enqueued on `stream`.
 * x: [B, L, d] layer input (must not alias cache->out).  idx_in: tokens to recompute (the salient
 * set handed over by the previous layer or step).  idx_out: receives the tokens whose cosine fell
 * below tau (a subset of idx_in); it is the next layer's idx_in.  cos_out: [idx_in->cap] or NULL.
 * The layer's output is cache->out (all rows).  An empty idx_in changes no cache byte and yields
 * an empty idx_out. */
int dyllm_layer_step(dyllm_ctx *ctx, const dyllm_layer_weights *w, dyllm_layer_cache *cache,
                     const void *x, const dyllm_index_list *idx_in, int32_t B, int32_t L, float tau,
                     dyllm_index_list *idx_out, float *cos_out, void *stream);

/* One layer of SparseStep with both attention paths: exact rows for the tokens of idx_in, and for
 * every other token of the step the approximate update of its cached context.  [Sec. 3.3; Alg. 3
 * layer body; Alg. 4; Eq. 3]
 *   The step's tokens are the positions [row_lo, L) of every sequence: row_lo = 0 is a whole-sequence
 *   step, row_lo = L_P a response-only step (Sec. 3.5), in which the tokens below row_lo keep every
 *   cache row and take no part in the test, while keys and values still cover the whole sequence
 *   (App. C.4).  idx_in must hold tokens of the step only.
 *   q of ALL tokens of the step is recomputed from x; K, V of the tokens in idx_in are recomputed and
 *   merged into the caches, dV = V_new - V_cache of those tokens taken before the merge;
 *   C[idx_in]  = softmax(q K^T / sqrt(dh)) V            (against the merged caches),
 *   C[others] = C_cache + softmax(q K^T / sqrt(dh))[:, idx_in] dV   (normalised over ALL keys);
 *   the cosine test then runs over ALL tokens of the step (new context against the cached one), the
 *   context cache takes the new rows, and idx_out receives every token whose cosine fell below tau --
 *   it may hold tokens outside idx_in, so idx_out->cap should be B*(L-row_lo) (overflow sets
 *   DYLLM_ERR_CAPACITY in the status word as for dyllm_compact).  Out-projection and FFN run for
 *   idx_out only.
 * cached_norm != 0 selects a variant that is NOT the printed Alg. 4: the weight of candidate key j for
 *   query i is exp(q_i.k_j/sqrt(dh) - cache->lse[i]), i.e. the softmax normaliser is the one cached at
 *   token i's last exact evaluation instead of a sum over all keys now, so that only the candidates'
 *   keys are scored -- the O(N |A| d) cost that Sec. 3.3 states.  It equals Alg. 4 whenever the
 *   cached normalisers are current; needs cache->lse.
 * cos_out: [B*L] indexed by token (entries of tokens outside the step are not written) or NULL.
 * Needs a context with max_rows covering B*L.  An empty idx_in leaves every cached value unchanged
 * and yields an empty idx_out. */
int dyllm_layer_step_approx(dyllm_ctx *ctx, const dyllm_layer_weights *w, dyllm_layer_cache *cache,
                            const void *x, const dyllm_index_list *idx_in, int32_t B, int32_t L,
                            int32_t row_lo, float tau, int32_t cached_norm, dyllm_index_list *idx_out,
                            float *cos_out, void *stream);

/* dyllm_layer_step_approx through a stack of n_layers layers, chained like dyllm_stack_step.  [Alg. 3,
 * loop over l]  The selections may grow from layer to layer: every idx_out[l] should have capacity
 * B*(L-row_lo).  cos_out: NULL or [n_layers, B*L]. */
int dyllm_stack_step_approx(dyllm_ctx *ctx, int32_t n_layers, const dyllm_layer_weights *w,
                            dyllm_layer_cache *caches, const void *x, const dyllm_index_list *idx_in,
                            int32_t B, int32_t L, int32_t row_lo, float tau, int32_t cached_norm,
                            dyllm_index_list *idx_out, float *cos_out, void *stream);

/* out = the ascending, duplicate-free union of the token lists a and b (either may be NULL), kept to
 * the tokens at positions >= pos_lo of their sequence, with per-sequence offsets.  Serves the carry
 * of the salient set from one denoising step to the next and the restriction of a response-only step
 * to the response.  [App. C.1, Alg. 1: idx_sal across iterations; Sec. 3.5]
 * out must not share buffers with a or b; more tokens than out->cap: the excess is dropped and the
 * status word is set.  Needs a context with max_rows covering B*L. */
int dyllm_merge_lists(dyllm_ctx *ctx, const dyllm_index_list *a, const dyllm_index_list *b, int32_t B,
                      int32_t L, int32_t pos_lo, dyllm_index_list *out, void *stream);

/* The step schedule of the generation loop.  [App. C.1, Alg. 1; Sec. 3.2; Sec. 3.5] */
typedef struct {
  int32_t t_full;      /* the first t_full steps are dense (FullStep) */
  int32_t full_period; /* a later step t takes the whole sequence when t % full_period == 0 (the paper
                          uses 4), the response only otherwise; <= 1: always the whole sequence */
  int32_t prompt_len;  /* L_P: positions [0, L_P) of every sequence are the prompt */
  int32_t approx;      /* 0: exact rows only; 1: approximate update of the non-salient tokens (Sec. 3.3,
                          Alg. 4); 2: the same with reused normalisers (see dyllm_layer_step_approx) */
  float tau;
} dyllm_schedule;
#define DYLLM_STEP_DENSE 0
#define DYLLM_STEP_FULL 1
#define DYLLM_STEP_RESPONSE 2
/* DYLLM_STEP_* of step t, or DYLLM_ERR_INVALID_ARG.  Host only. */
int dyllm_step_kind(const dyllm_schedule *sched, int32_t t);

/* One iteration of the generation loop without its token side (embedding, logits and unmasking stay
 * with the caller).  [App. C.1, Alg. 1]
 *   dense step:  dyllm_stack_full_step; decoded, carry, cand and idx_out are not used.
 *   sparse step: cand = merge(carry, decoded) kept to the step's tokens (all, or the response), then
 *     dyllm_stack_step (approx == 0; a response-only step then differs from a whole-sequence step only
 *     by that restriction) or dyllm_stack_step_approx with cand as the first layer's idx_in.
 * x: [B, L, d] hidden states of the whole sequence (a response-only step reads its response rows).
 * decoded: tokens unmasked by the previous step, or NULL.  carry: idx_out[n_layers-1] of the previous
 * sparse step, or NULL after a dense step (Alg. 1 then starts from the decoded positions alone).
 * Reading taken where Alg. 1 is silent: later steps join the newly decoded positions to the carried
 * set, since a token whose input embedding changed has to be recomputed.
 * cand: scratch list that receives the candidates; idx_out: host array of n_layers lists as in
 * dyllm_stack_step; idx_out[n_layers-1] is the next step's carry (it may be the same buffers as this
 * step's carry: the carry is consumed before any layer writes).  cand must
 * not share buffers with carry, decoded or idx_out[0]. */
int dyllm_denoise_step(dyllm_ctx *ctx, const dyllm_schedule *sched, int32_t t, int32_t n_layers,
                       const dyllm_layer_weights *w, dyllm_layer_cache *caches, const void *x,
                       const dyllm_index_list *decoded, const dyllm_index_list *carry, int32_t B,
                       int32_t L, dyllm_index_list *cand, dyllm_index_list *idx_out, void *stream);

/* Dense pass of one layer over all B*L rows; fills all four caches.  [App. C.2, Alg. 2]
 * Needs a context with max_rows covering B*L. */
int dyllm_full_step(dyllm_ctx *ctx, const dyllm_layer_weights *w, dyllm_layer_cache *cache,
                    const void *x, int32_t B, int32_t L, void *stream);

/* SparseStep through a stack of n_layers layers, enqueued as one sequence.  [Alg. 3, loop over l]
 * w, caches and idx_out are HOST arrays of n_layers entries (their members are device pointers).
 * Layer 0 reads x and idx_in; layer l > 0 reads caches[l-1].out (all rows: recomputed and reused
 * alike) as its input and idx_out[l-1] as its candidates, and writes idx_out[l]; idx_out[n_layers-1]
 * is the set carried to the next denoising step.  idx_out[l] must not share buffers with
 * idx_out[l-1] (or idx_in for l = 0); lists two layers apart may share them.  Every selection is a
 * subset of idx_in, so a capacity of idx_in->cap suffices for each list.  cos_out: NULL, or
 * [n_layers, idx_in->cap] (row l: cosines of layer l's candidates).  All arguments of all layers
 * are checked before the first launch. */
int dyllm_stack_step(dyllm_ctx *ctx, int32_t n_layers, const dyllm_layer_weights *w,
                     dyllm_layer_cache *caches, const void *x, const dyllm_index_list *idx_in,
                     int32_t B, int32_t L, float tau, dyllm_index_list *idx_out, float *cos_out,
                     void *stream);

/* FullStep through a stack of n_layers layers: layer l > 0 reads caches[l-1].out.  [Alg. 2, loop
 * over l]  w and caches are host arrays of n_layers entries. */
int dyllm_stack_full_step(dyllm_ctx *ctx, int32_t n_layers, const dyllm_layer_weights *w,
                          dyllm_layer_cache *caches, const void *x, int32_t B, int32_t L,
                          void *stream);

/* Per-stage timing of dyllm_layer_step / dyllm_full_step for measurement.  After
 * dyllm_profile_begin the next max_calls (<= 4096) step calls on this context record a HIP event on
 * their stream after every stage (gather+norm, q/k/v GEMM, rotation+merge, attention, saliency,
 * compaction, out-projection GEMM, FFN norm, gate/up GEMM, down GEMM).  dyllm_profile_end waits for
 * those events, writes the mean milliseconds per stage into host_stage_ms[dyllm_stage_count()] and
 * the number of recorded calls into *host_calls, and switches profiling off.  A stage's time runs
 * from the end of the previous stage to its own end on the stream. */
int dyllm_profile_begin(dyllm_ctx *ctx, int32_t max_calls);
int dyllm_profile_end(dyllm_ctx *ctx, float *host_stage_ms, int32_t *host_calls);
int dyllm_stage_count(void);
const char *dyllm_stage_name(int stage);

#ifdef __cplusplus
}
#endif
#endif /* DYLLM_H */
