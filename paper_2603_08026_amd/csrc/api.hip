// C ABI of the library: context, argument checks on the host, and the composition of the
// kernels into the boundary calls.  Everything is enqueued on the caller's stream; row counts stay
// on the device.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "../../include/dyllm.h"
#include "kernels.h"

using namespace dy;

struct dyllm_ctx {
  dyllm_layer_cfg cfg;
  int rows_cap;  // max rows of one call
  int dq, dkv;
  size_t esz;
  char *ws;  // one device allocation, carved below
  size_t ws_bytes;
  // carved buffers
  void *ns;        // [R, d]        normalised salient rows
  void *qs;        // [R, dq]       rotated queries
  float *part_o;   // fp32 scratch shared by consecutive stages: raw GEMM results / attention partials
  float *part_ml;
  size_t part_elems;
  void *dv_full;   // [R, dkv] value residuals of the approximate path; all zero between calls
  void *dc;        // [R, dq] approximate context residual of every token
  void *csal;      // [R, dq] exact context rows of the salient tokens (approximate path)
  int32_t *pos;    // [R] position+1 of a token in the salient list; all zero between calls
  int32_t *win_idx, *win_off;  // [R], [max_batch+1]: the tokens of a response-only step as a list
  void *ksal;      // [R, dkv] compact copy of the candidates' new key rows (reused-normaliser variant)
  float *cosb;     // [R]
  uint8_t *flag;   // [R]
  float *hs;       // [R, d]        x + Wo c (fp32)
  void *fs;        // [R, d]        RMSNorm(h)
  void *act;       // [R, F]        silu(gate)*up
  int32_t *status; // device status word
  int32_t *scan;   // words of the chained compaction kernel; all zero between calls
  float *rope;     // [max_seq, dh/2, 2]
  // optional per-stage timing (dyllm_profile_begin / _end)
  std::vector<hipEvent_t> *prof_events;
  int prof_max_calls, prof_calls;
  hipEvent_t *prof_cur;
  char err[256];
};

namespace {

struct Layout {
  size_t ns, qs, part_o, part_ml, cosb, flag, hs, fs, act, status, rope, dv_full, dc, csal, pos, win_idx, win_off, ksal, scan, total;
  size_t part_elems;
};

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

Layout make_layout(const dyllm_layer_cfg &c) {
  Layout l;
  const size_t R = c.max_rows > 0 ? (size_t)c.max_rows : (size_t)c.max_batch * c.max_seq;
  const size_t e = c.dtype == DYLLM_F32 ? 4 : 2;
  const size_t d = c.hidden, dq = (size_t)c.n_heads * c.head_dim, dkv = (size_t)c.n_kv_heads * c.head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  l.ns = take(R * d * e);
  l.qs = take(R * dq * e);
  // fp32 scratch: 16 attention splits of up to 2048 rows, or one raw GEMM result of R rows
  const size_t prow = R < 2048 ? R : 2048;
  const size_t widest = dq + 2 * dkv > d ? dq + 2 * dkv : d;
  l.part_elems = 16 * prow * dq > R * widest ? 16 * prow * dq : R * widest;
  l.part_o = take(l.part_elems * 4);
  l.part_ml = take(l.part_elems / c.head_dim * 2 * 4);
  l.cosb = take(R * 4);
  l.flag = take(R);
  l.hs = take(R * d * 4);
  l.fs = take(R * d * e);
  l.act = take(R * (size_t)c.ffn_dim * e);
  l.status = take(256);
  l.rope = take((size_t)c.max_seq * (c.head_dim / 2) * 2 * 4);
  l.dv_full = take(R * dkv * e);
  l.dc = take(R * dq * e);
  l.csal = take(R * dq * e);
  l.pos = take(R * 4);
  l.win_idx = take(R * 4);
  l.win_off = take(((size_t)c.max_batch + 1) * 4);
  l.ksal = take(R * dkv * e);
  l.scan = take((size_t)compact_scan_words() * 4);
  l.total = off;
  return l;
}

// Device words of dyllm_compact_static, the entry point that allocates nothing.  In host code the
// array's name is only a handle for the symbol lookup: kernels get the address that
// hipGetSymbolAddress returns for the current device (every GPU holds its own copy).
constexpr int kScratchWords = 1088;  // COMPACT_SCAN_WORDS + the spare status word, padded to 4352 bytes
static_assert(kScratchWords > COMPACT_SCAN_WORDS, "room for the spare status word");
static __device__ __align__(256) int32_t scratch[kScratchWords];
constexpr int kMaxDevices = 64;
int32_t *g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mu;

// address of `scratch` on the current device, looked up once per device
int static_scratch(int32_t **words) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DYLLM_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return DYLLM_ERR_HIP;
    }
    g_scratch_ptr[dev] = (int32_t *)p;
  }
  *words = g_scratch_ptr[dev];
  return DYLLM_OK;
}

int check_cfg(const dyllm_layer_cfg *c) {
  if (!c) return DYLLM_ERR_INVALID_ARG;
  if (c->dtype != DYLLM_F32 && c->dtype != DYLLM_BF16) return DYLLM_ERR_INVALID_ARG;
  if (c->hidden <= 0 || c->n_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->ffn_dim <= 0 ||
      c->max_batch <= 0 || c->max_seq <= 0 || c->max_rows < 0)
    return DYLLM_ERR_INVALID_ARG;
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return DYLLM_ERR_INVALID_ARG;
  if (c->n_heads % c->n_kv_heads) return DYLLM_ERR_BAD_SHAPE;
  if ((long)c->max_batch * c->max_seq > (1l << 30)) return DYLLM_ERR_UNSUPPORTED;
  if (c->max_rows > 0 && (long)c->max_rows > (long)c->max_batch * c->max_seq) return DYLLM_ERR_BAD_SHAPE;
  if (c->head_dim != 64 && c->head_dim != 128) return DYLLM_ERR_UNSUPPORTED;
  if (c->hidden > 16384) return DYLLM_ERR_UNSUPPORTED;  // a row kernel keeps one row per workgroup in registers
  const int q = c->dtype == DYLLM_BF16 ? 128 : 64;
  if (c->hidden % q || c->ffn_dim % q || (c->n_heads * c->head_dim) % q) return DYLLM_ERR_UNSUPPORTED;
  return DYLLM_OK;
}

int fail(dyllm_ctx *ctx, int code, const char *what) {
  if (ctx) snprintf(ctx->err, sizeof(ctx->err), "%s: %s", dyllm_strerror(code), what);
  return code;
}

int hip_fail(dyllm_ctx *ctx, hipError_t e, const char *where) {
  if (ctx) ctx->prof_cur = nullptr;
  if (ctx) snprintf(ctx->err, sizeof(ctx->err), "HIP error at %s: %s", where, hipGetErrorString(e));
  return DYLLM_ERR_HIP;
}

int check_launch(dyllm_ctx *ctx, const char *where) {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DYLLM_OK : hip_fail(ctx, e, where);
}

int check_bl(dyllm_ctx *ctx, int B, int L) {
  if (B <= 0 || L <= 0) return fail(ctx, DYLLM_ERR_INVALID_ARG, "B and L must be positive");
  if (B > ctx->cfg.max_batch || L > ctx->cfg.max_seq)
    return fail(ctx, DYLLM_ERR_BAD_SHAPE, "B or L exceeds the context's max_batch / max_seq");
  return DYLLM_OK;
}

int check_list(dyllm_ctx *ctx, const dyllm_index_list *l, const char *name) {
  if (!l || !l->offsets) return fail(ctx, DYLLM_ERR_INVALID_ARG, name);
  if (l->cap < 0) return fail(ctx, DYLLM_ERR_INVALID_ARG, "negative list capacity");
  if (!l->idx && l->cap > 0) return fail(ctx, DYLLM_ERR_INVALID_ARG, name);  // idx may be NULL only for cap 0
  if (l->cap > ctx->rows_cap) return fail(ctx, DYLLM_ERR_CAPACITY, "list capacity exceeds the context's max_rows");
  return DYLLM_OK;
}

Rows rows_of(const dyllm_index_list *l, int B) { return Rows{l->idx, l->offsets + B, l->cap}; }

DType dt(const dyllm_ctx *c) { return c->cfg.dtype == DYLLM_F32 ? F32 : BF16; }

// Stages of a step in execution order; with profiling on, an event is recorded after each.
enum Stage {
  ST_GATHER_NORM = 0, ST_GEMM_QKV, ST_ROPE_SCATTER, ST_ATTENTION, ST_SALIENCY, ST_COMPACT, ST_GEMM_OPROJ,
  ST_NORM_FFN, ST_GEMM_SWIGLU, ST_GEMM_DOWN, N_STAGES
};
const char *const kStageNames[N_STAGES] = {
    "gather_rmsnorm", "gemm_qkv", "rope_scatter", "partial_attention", "saliency_compact", "marker_overhead",
    "gemm_oproj", "rmsnorm_ffn", "gemm_swiglu", "gemm_down"};

void prof_begin_call(dyllm_ctx *ctx, hipStream_t s) {
  ctx->prof_cur = nullptr;
  if (!ctx->prof_events || ctx->prof_calls >= ctx->prof_max_calls) return;
  ctx->prof_cur = ctx->prof_events->data() + (size_t)ctx->prof_calls * (N_STAGES + 1);
  ++ctx->prof_calls;
  (void)hipEventRecord(ctx->prof_cur[0], s);
}
void prof_mark(dyllm_ctx *ctx, int stage, hipStream_t s) {
  if (ctx->prof_cur) (void)hipEventRecord(ctx->prof_cur[stage + 1], s);
}

// gather + norm, q/k/v projection, rotation, K/V merge  [Alg. 3: norm / q_proj / k_proj / v_proj lines]
int enqueue_qkv(dyllm_ctx *ctx, const dyllm_layer_weights *w, const void *x, Rows rows, int L,
                dyllm_layer_cache *cache, void *q_out, hipStream_t s) {
  const dyllm_layer_cfg &c = ctx->cfg;
  launch_gather_rmsnorm(dt(ctx), x, w->g_attn, rows, c.hidden, c.rms_eps, ctx->ns, s);
  prof_mark(ctx, ST_GATHER_NORM, s);
  WSeg seg;
  seg.w[0] = w->wq; seg.w[1] = w->wk; seg.w[2] = w->wv;
  seg.n_end[0] = ctx->dq; seg.n_end[1] = ctx->dq + ctx->dkv; seg.n_end[2] = ctx->dq + 2 * ctx->dkv;
  const Splits splits = launch_gemm_raw(dt(ctx), GemmA{ctx->ns, nullptr, c.hidden}, rows, c.hidden, seg,
                                     ctx->part_o, ctx->part_elems, s);
  prof_mark(ctx, ST_GEMM_QKV, s);
  launch_qkv_finalize(dt(ctx), ctx->part_o, splits, (size_t)rows.cap * seg.n_end[2], ctx->rope, rows, L,
                      c.n_heads, c.n_kv_heads, c.head_dim, w->bq, w->bk, w->bv, q_out, cache->k,
                      cache->v, nullptr, 0, nullptr, 0, nullptr, 0, s);
  prof_mark(ctx, ST_ROPE_SCATTER, s);
  return check_launch(ctx, "qkv refresh");
}

AttnArgs attn_args(dyllm_ctx *ctx, const void *q, const void *k, const void *v, Rows rows,
                   const int32_t *offsets, int B, int L, void *out, int partial) {
  const dyllm_layer_cfg &c = ctx->cfg;
  AttnArgs a;
  a.q = q; a.q_by_token = 0; a.k = k; a.v = v; a.rows = rows; a.offsets = offsets;
  a.key_offsets = nullptr; a.lse_out = nullptr; a.c_commit = nullptr; a.cos_part = nullptr;
  a.B = B; a.L = L; a.H = c.n_heads; a.Hkv = c.n_kv_heads; a.dh = c.head_dim;
  const int rows_per_seq = offsets ? (rows.cap + B - 1) / B : L;
  attention_plan(dt(ctx), B, L, c.n_heads, c.head_dim, rows.cap, rows_per_seq, ctx->part_elems, &a,
                 c.n_heads / c.n_kv_heads);
  a.partial = partial;
  a.part_o = ctx->part_o; a.part_ml = ctx->part_ml; a.out = out;
  return a;
}

// exact attention rows, merged into `out`  [Alg. 3: C_sal]
int enqueue_attention(dyllm_ctx *ctx, const void *q, const void *k, const void *v, Rows rows,
                      const int32_t *offsets, int B, int L, void *out, hipStream_t s) {
  const AttnArgs a = attn_args(ctx, q, k, v, rows, offsets, B, L, out, 0);
  launch_attention(dt(ctx), a, s);
  prof_mark(ctx, ST_ATTENTION, s);
  return check_launch(ctx, "partial attention");
}

// out-projection + residual, norm, SwiGLU FFN + residual, scatter into the output cache
// [Alg. 3: out_proj / FFN / cache lines]
int enqueue_ffn(dyllm_ctx *ctx, const dyllm_layer_weights *w, const void *x, const void *c_all,
                Rows rows, void *out_cache, size_t n_tokens, hipStream_t s) {
  const dyllm_layer_cfg &c = ctx->cfg;
  const Splits splits = launch_gemm_raw(dt(ctx), GemmA{c_all, rows.idx, ctx->dq, n_tokens}, rows, ctx->dq,
                                     wseg_one(w->wo, c.hidden), ctx->part_o, ctx->part_elems, s);
  prof_mark(ctx, ST_GEMM_OPROJ, s);
  launch_oproj_finalize(dt(ctx), ctx->part_o, splits, (size_t)rows.cap * c.hidden, x, w->g_ffn, rows,
                        c.hidden, c.rms_eps, ctx->hs, ctx->fs, s);
  prof_mark(ctx, ST_NORM_FFN, s);
  launch_gemm_swiglu(dt(ctx), GemmA{ctx->fs, nullptr, c.hidden}, rows, c.hidden, c.ffn_dim, w->w_gate,
                     w->w_up, ctx->act, ctx->part_o, ctx->part_elems, s);
  prof_mark(ctx, ST_GEMM_SWIGLU, s);
  launch_gemm_down(dt(ctx), GemmA{ctx->act, nullptr, c.ffn_dim}, rows, c.ffn_dim, c.hidden, w->w_down,
                   ctx->hs, out_cache, ctx->part_o, ctx->part_elems, s);
  prof_mark(ctx, ST_GEMM_DOWN, s);
  return check_launch(ctx, "salient ffn");
}

int check_weights(dyllm_ctx *ctx, const dyllm_layer_weights *w, bool attn, bool ffn) {
  if (!w) return fail(ctx, DYLLM_ERR_INVALID_ARG, "weights is NULL");
  if (attn && (!w->wq || !w->wk || !w->wv || !w->g_attn))
    return fail(ctx, DYLLM_ERR_INVALID_ARG, "wq / wk / wv / g_attn is NULL");
  if (ffn && (!w->wo || !w->w_gate || !w->w_up || !w->w_down || !w->g_ffn))
    return fail(ctx, DYLLM_ERR_INVALID_ARG, "wo / w_gate / w_up / w_down / g_ffn is NULL");
  return DYLLM_OK;
}

int check_cache(dyllm_ctx *ctx, const dyllm_layer_cache *c) {
  if (!c || !c->k || !c->v || !c->c || !c->out) return fail(ctx, DYLLM_ERR_INVALID_ARG, "cache pointer is NULL");
  return DYLLM_OK;
}

int check_dense_layer(dyllm_ctx *ctx, const dyllm_layer_weights *w, const dyllm_layer_cache *cache,
                      const void *x) {
  int rc;
  if ((rc = check_weights(ctx, w, true, true))) return rc;
  if ((rc = check_cache(ctx, cache))) return rc;
  if (!x) return fail(ctx, DYLLM_ERR_INVALID_ARG, "x is NULL");
  if (x == cache->out) return fail(ctx, DYLLM_ERR_INVALID_ARG, "x aliases cache->out");
  return DYLLM_OK;
}

int check_sparse_layer(dyllm_ctx *ctx, const dyllm_layer_weights *w, const dyllm_layer_cache *cache,
                       const void *x, const dyllm_index_list *idx_in, const dyllm_index_list *idx_out) {
  int rc;
  if ((rc = check_dense_layer(ctx, w, cache, x))) return rc;
  if ((rc = check_list(ctx, idx_in, "idx_in"))) return rc;
  if ((rc = check_list(ctx, idx_out, "idx_out"))) return rc;
  if ((idx_out->idx && idx_out->idx == idx_in->idx) || idx_out->offsets == idx_in->offsets)
    return fail(ctx, DYLLM_ERR_INVALID_ARG, "idx_out aliases idx_in");
  return DYLLM_OK;
}

// one layer of the sparse step, arguments already checked  [Alg. 3 layer body]
int enqueue_sparse_layer(dyllm_ctx *ctx, const dyllm_layer_weights *w, dyllm_layer_cache *cache,
                         const void *x, const dyllm_index_list *idx_in, int B, int L, float tau,
                         dyllm_index_list *idx_out, float *cos_out, hipStream_t s) {
  int rc;
  const Rows rin = rows_of(idx_in, B);
  prof_begin_call(ctx, s);
  if ((rc = enqueue_qkv(ctx, w, x, rin, L, cache, ctx->qs, s))) return rc;
  {
    AttnArgs a = attn_args(ctx, ctx->qs, cache->k, cache->v, rin, idx_in->offsets, B, L, nullptr, 1);
    a.lse_out = (float *)cache->lse;  // optional fifth cache: log-normalisers of the exact rows
    if (dt(ctx) == BF16 && ctx->cfg.head_dim == 128 && a.splits == 1) {
      // one key split: the attention kernel commits its rows itself and leaves per-head sums for the
      // cosine (no fp32 partial result, no second pass over the rows); the cosine test of a row then
      // rides on the compaction kernel
      a.c_commit = cache->c;
      a.cos_part = ctx->part_o;
      launch_attention(dt(ctx), a, s);
      prof_mark(ctx, ST_ATTENTION, s);
      launch_cos_compact(ctx->part_o, ctx->cfg.n_heads, tau, cos_out ? cos_out : ctx->cosb, ctx->flag, rin, B, L,
                         idx_out->idx, idx_out->offsets, idx_out->cap, ctx->status, ctx->scan, s);
    } else {
      // attention leaves per-split partials; their merge is fused with the cosine test and the commit
      launch_attention(dt(ctx), a, s);
      prof_mark(ctx, ST_ATTENTION, s);
      // ... and the last workgroup of that kernel compacts the flags into idx_out
      launch_attn_finalize(dt(ctx), a, cache->c, tau, cos_out ? cos_out : ctx->cosb, ctx->flag,
                           idx_out->idx, idx_out->offsets, idx_out->cap, ctx->status, ctx->status + 1, s);
    }
    prof_mark(ctx, ST_SALIENCY, s);
    prof_mark(ctx, ST_COMPACT, s);
  }
  if ((rc = check_launch(ctx, "saliency / compact"))) return rc;
  // idx_out is a subset of idx_in: its count never exceeds idx_in's capacity, which sizes the grids
  Rows rout = rows_of(idx_out, B);
  if (rout.cap > idx_in->cap) rout.cap = idx_in->cap;
  rc = enqueue_ffn(ctx, w, x, cache->c, rout, cache->out, (size_t)B * L, s);
  ctx->prof_cur = nullptr;
  return rc;
}

// The tokens of a step: all B*L (row_lo = 0) or the positions [row_lo, L) of every sequence, as a list
// in the context's workspace  [Sec. 3.5: response-only steps]
struct Window { Rows rows; const int32_t *offsets; int lo; };
Window make_window(dyllm_ctx *ctx, int B, int L, int row_lo, hipStream_t s) {
  if (row_lo <= 0) return Window{Rows{nullptr, nullptr, B * L}, nullptr, 0};
  launch_make_window(B, L, row_lo, ctx->win_idx, ctx->win_off, s);
  return Window{Rows{ctx->win_idx, nullptr, B * (L - row_lo)}, ctx->win_off, row_lo};
}

// one layer of the sparse step with both attention paths, arguments already checked
// [Alg. 3 layer body; Sec. 3.3: exact rows for the salient tokens, approximate update for the others]
int enqueue_approx_layer(dyllm_ctx *ctx, const dyllm_layer_weights *w, dyllm_layer_cache *cache,
                         const void *x, const dyllm_index_list *idx_in, int B, int L, Window win, float tau,
                         int cached_norm, dyllm_index_list *idx_out, float *cos_out, hipStream_t s) {
  const dyllm_layer_cfg &c = ctx->cfg;
  const Rows all = win.rows;
  const Rows rin = rows_of(idx_in, B);
  const int by_token = all.idx != nullptr;  // a window keeps q at its token's row, so that both
                                            // attention passes find it from a token id
  int rc;
  ctx->prof_cur = nullptr;  // no per-stage timing on this path
  // norm and q projection (+ rotation) of EVERY token of the step  [Alg. 3: Q <- q_proj(x)]
  launch_gather_rmsnorm(dt(ctx), x, w->g_attn, all, c.hidden, c.rms_eps, ctx->ns, s);
  {
    const Splits splits = launch_gemm_raw(dt(ctx), GemmA{ctx->ns, nullptr, c.hidden}, all, c.hidden,
                                       wseg_one(w->wq, ctx->dq), ctx->part_o, ctx->part_elems, s);
    launch_qkv_finalize(dt(ctx), ctx->part_o, splits, (size_t)all.cap * ctx->dq, ctx->rope, all, L, c.n_heads,
                        0, c.head_dim, w->bq, nullptr, nullptr, ctx->qs, nullptr, nullptr, nullptr, by_token,
                        nullptr, 0, nullptr, 0, s);
  }
  // k, v of the salient tokens: norm, projection, rotation, value residual, merge into the caches
  launch_gather_rmsnorm(dt(ctx), x, w->g_attn, rin, c.hidden, c.rms_eps, ctx->fs, s);
  {
    WSeg seg;
    seg.w[0] = w->wk; seg.w[1] = w->wv; seg.w[2] = w->wv;
    seg.n_end[0] = ctx->dkv; seg.n_end[1] = 2 * ctx->dkv; seg.n_end[2] = 2 * ctx->dkv;
    const Splits splits = launch_gemm_raw(dt(ctx), GemmA{ctx->fs, nullptr, c.hidden}, rin, c.hidden, seg,
                                       ctx->part_o, ctx->part_elems, s);
    // value residual: by token into the zero-padded [T, dkv] buffer (Alg. 4 as printed), or by list
    // entry next to a compact copy of the new keys (reused normalisers: only candidates are scored)
    launch_qkv_finalize(dt(ctx), ctx->part_o, splits, (size_t)rin.cap * 2 * ctx->dkv, ctx->rope, rin, L, 0,
                        c.n_kv_heads, c.head_dim, nullptr, w->bk, w->bv, nullptr, cache->k, cache->v,
                        cached_norm ? ctx->dc : ctx->dv_full, 0, cached_norm ? ctx->ksal : nullptr,
                        cached_norm, ctx->pos, win.lo, s);  // also marks the step's candidates in the token -> entry map
  }
  if ((rc = check_launch(ctx, "approx: projections"))) return rc;
  // exact rows of the salient tokens  [Alg. 3: C_sal]; q is stored by token here.  With a cache of
  // log-normalisers the rows go through the merge kernel, which stores theirs.
  {
    const int keep_lse = cache->lse != nullptr;
    AttnArgs a = attn_args(ctx, ctx->qs, cache->k, cache->v, rin, idx_in->offsets, B, L, ctx->csal, keep_lse);
    a.q_by_token = 1;
    a.lse_out = (float *)cache->lse;
    launch_attention(dt(ctx), a, s);
    if (keep_lse) launch_attn_combine(dt(ctx), a, s);
  }
  if (!cached_norm) {
    // approximate residual of every token of the step: the full softmax against the merged keys times
    // the value residual, which is zero outside the salient rows  [Alg. 4]
    AttnArgs a = attn_args(ctx, ctx->qs, cache->k, ctx->dv_full, all, win.offsets, B, L, ctx->dc, 0);
    a.q_by_token = by_token;
    launch_attention(dt(ctx), a, s);
    if ((rc = check_launch(ctx, "approx: attention"))) return rc;
    // new contexts of the step's tokens, cosine test, commit; then the scratch maps go back to zero
    launch_saliency_approx(dt(ctx), all, ctx->dq, ctx->csal, ctx->dc, ctx->pos, cache->c, tau, cos_out, ctx->flag,
                           nullptr, nullptr, L, s);
    launch_clear_rows(dt(ctx), rin, ctx->dv_full, ctx->dkv, s);  // the residual buffer goes back to zero
  } else {
    // Reused normalisers (Sec. 3.3's O(N |A| d) form): every token of the step is scored against the
    // candidates' keys only -- compact rows, sequence b's at [offsets[b], offsets[b+1]) -- and the
    // un-normalised partial sums are scaled by the log-normaliser cached at the token's last exact
    // evaluation instead of a softmax over all keys.
    int lk_max = rin.cap < L ? rin.cap : L;
    if (lk_max < 1) lk_max = 1;
    AttnArgs a = attn_args(ctx, ctx->qs, ctx->ksal, ctx->dc, all, win.offsets, B, L, nullptr, 1);
    // key splits over the longest possible candidate run; the query side still walks sequences of L
    attention_plan(dt(ctx), B, lk_max, c.n_heads, c.head_dim, all.cap, win.offsets ? (all.cap + B - 1) / B : L,
                   ctx->part_elems, &a, c.n_heads / c.n_kv_heads);
    a.q_by_token = by_token;
    a.key_offsets = idx_in->offsets;
    launch_attention(dt(ctx), a, s);
    if ((rc = check_launch(ctx, "approx: attention"))) return rc;
    launch_saliency_approx(dt(ctx), all, ctx->dq, ctx->csal, nullptr, ctx->pos, cache->c, tau, cos_out, ctx->flag,
                           &a, (const float *)cache->lse, L, s);
  }
  launch_compact(ctx->flag, all, B, L, idx_out->idx, idx_out->offsets, idx_out->cap, ctx->status, ctx->scan, s);
  if ((rc = check_launch(ctx, "approx: saliency / compact"))) return rc;
  return enqueue_ffn(ctx, w, x, cache->c, rows_of(idx_out, B), cache->out, (size_t)B * L, s);
}

// out = ascending unique union of a and b (either may be null), kept to positions >= pos_lo
int enqueue_merge(dyllm_ctx *ctx, const dyllm_index_list *a, const dyllm_index_list *b, int B, int L,
                  int pos_lo, dyllm_index_list *out, hipStream_t s) {
  const int T = B * L;
  launch_fill_i32((int32_t *)ctx->flag, 0, (T + 3) / 4, s);
  if (a) launch_mark_flags(rows_of(a, B), T, L, pos_lo, ctx->flag, s);
  if (b) launch_mark_flags(rows_of(b, B), T, L, pos_lo, ctx->flag, s);
  launch_compact(ctx->flag, Rows{nullptr, nullptr, T}, B, L, out->idx, out->offsets, out->cap, ctx->status, ctx->scan, s);
  return check_launch(ctx, "list merge");
}

// dense pass of one layer, arguments already checked  [Alg. 2 layer body]
int enqueue_dense_layer(dyllm_ctx *ctx, const dyllm_layer_weights *w, dyllm_layer_cache *cache,
                        const void *x, int B, int L, hipStream_t s) {
  int rc;
  const Rows all{nullptr, nullptr, B * L};
  prof_begin_call(ctx, s);
  if ((rc = enqueue_qkv(ctx, w, x, all, L, cache, ctx->qs, s))) return rc;
  // every row is a query: the context cache is written directly
  if (cache->lse) {  // ... through the merge kernel when the log-normalisers are kept as well
    AttnArgs a = attn_args(ctx, ctx->qs, cache->k, cache->v, all, nullptr, B, L, cache->c, 1);
    a.lse_out = (float *)cache->lse;
    launch_attention(dt(ctx), a, s);
    launch_attn_combine(dt(ctx), a, s);
    prof_mark(ctx, ST_ATTENTION, s);
    if ((rc = check_launch(ctx, "attention"))) return rc;
  } else if ((rc = enqueue_attention(ctx, ctx->qs, cache->k, cache->v, all, nullptr, B, L, cache->c, s))) {
    return rc;
  }
  prof_mark(ctx, ST_SALIENCY, s);
  prof_mark(ctx, ST_COMPACT, s);
  rc = enqueue_ffn(ctx, w, x, cache->c, all, cache->out, (size_t)B * L, s);
  ctx->prof_cur = nullptr;
  return rc;
}

}  // namespace

extern "C" {

const char *dyllm_strerror(int code) {
  switch (code) {
    case DYLLM_OK: return "ok";
    case DYLLM_ERR_INVALID_ARG: return "invalid argument";
    case DYLLM_ERR_BAD_SHAPE: return "bad shape";
    case DYLLM_ERR_UNSUPPORTED: return "unsupported configuration";
    case DYLLM_ERR_NO_MEM: return "out of device memory";
    case DYLLM_ERR_HIP: return "HIP runtime error";
    case DYLLM_ERR_CAPACITY: return "index list capacity exceeded";
    default: return "unknown error";
  }
}

const char *dyllm_last_error(const dyllm_ctx *ctx) { return ctx ? ctx->err : "no context"; }

int dyllm_workspace_bytes(const dyllm_layer_cfg *cfg, size_t *host_bytes) {
  if (!host_bytes) return DYLLM_ERR_INVALID_ARG;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  *host_bytes = make_layout(*cfg).total;
  return DYLLM_OK;
}

int dyllm_create(const dyllm_layer_cfg *cfg, dyllm_ctx **out) {
  if (!out) return DYLLM_ERR_INVALID_ARG;
  *out = nullptr;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  dyllm_ctx *ctx = new (std::nothrow) dyllm_ctx;
  if (!ctx) return DYLLM_ERR_NO_MEM;
  memset(ctx, 0, sizeof(*ctx));
  ctx->cfg = *cfg;
  ctx->rows_cap = cfg->max_rows > 0 ? cfg->max_rows : cfg->max_batch * cfg->max_seq;
  ctx->dq = cfg->n_heads * cfg->head_dim;
  ctx->dkv = cfg->n_kv_heads * cfg->head_dim;
  ctx->esz = cfg->dtype == DYLLM_F32 ? 4 : 2;
  const Layout l = make_layout(*cfg);
  ctx->ws_bytes = l.total;
  if (hipMalloc((void **)&ctx->ws, l.total) != hipSuccess) {
    (void)hipGetLastError();
    delete ctx;
    return DYLLM_ERR_NO_MEM;
  }
  char *b = ctx->ws;
  ctx->ns = b + l.ns; ctx->qs = b + l.qs;
  ctx->part_o = (float *)(b + l.part_o); ctx->part_ml = (float *)(b + l.part_ml);
  ctx->part_elems = l.part_elems;
  ctx->cosb = (float *)(b + l.cosb); ctx->flag = (uint8_t *)(b + l.flag);
  ctx->hs = (float *)(b + l.hs); ctx->fs = b + l.fs; ctx->act = b + l.act;
  ctx->status = (int32_t *)(b + l.status); ctx->rope = (float *)(b + l.rope);
  ctx->dv_full = b + l.dv_full; ctx->dc = b + l.dc; ctx->csal = b + l.csal; ctx->pos = (int32_t *)(b + l.pos);
  ctx->win_idx = (int32_t *)(b + l.win_idx); ctx->win_off = (int32_t *)(b + l.win_off);
  ctx->ksal = b + l.ksal; ctx->scan = (int32_t *)(b + l.scan);

  // rotary table in double precision on the host, cleared status word
  const int half = cfg->head_dim / 2;
  std::vector<float> tab((size_t)cfg->max_seq * half * 2);
  for (int p = 0; p < cfg->max_seq; ++p)
    for (int j = 0; j < half; ++j) {
      const double ang = (double)p * pow((double)cfg->rope_theta, -2.0 * j / cfg->head_dim);
      tab[((size_t)p * half + j) * 2] = (float)cos(ang);
      tab[((size_t)p * half + j) * 2 + 1] = (float)sin(ang);
    }
  hipError_t e = hipMemcpy(ctx->rope, tab.data(), tab.size() * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemset(ctx->status, 0, 256);
  if (e == hipSuccess) e = hipMemset(ctx->dv_full, 0, l.dc - l.dv_full);
  if (e == hipSuccess) e = hipMemset(ctx->pos, 0, l.win_idx - l.pos);
  if (e == hipSuccess) e = hipMemset(ctx->scan, 0, (size_t)compact_scan_words() * 4);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    (void)hipFree(ctx->ws);
    delete ctx;
    return DYLLM_ERR_HIP;
  }
  *out = ctx;
  return DYLLM_OK;
}

int dyllm_profile_begin(dyllm_ctx *ctx, int32_t max_calls) {
  if (!ctx || max_calls <= 0 || max_calls > 4096) return DYLLM_ERR_INVALID_ARG;
  if (ctx->prof_events) return fail(ctx, DYLLM_ERR_INVALID_ARG, "profiling already on");
  auto *ev = new (std::nothrow) std::vector<hipEvent_t>((size_t)max_calls * (N_STAGES + 1));
  if (!ev) return DYLLM_ERR_NO_MEM;
  for (size_t i = 0; i < ev->size(); ++i)
    if (hipEventCreate(&(*ev)[i]) != hipSuccess) {
      for (size_t k = 0; k < i; ++k) (void)hipEventDestroy((*ev)[k]);
      delete ev;
      return hip_fail(ctx, hipGetLastError(), "hipEventCreate");
    }
  ctx->prof_events = ev;
  ctx->prof_max_calls = max_calls;
  ctx->prof_calls = 0;
  ctx->prof_cur = nullptr;
  return DYLLM_OK;
}

int dyllm_profile_end(dyllm_ctx *ctx, float *host_stage_ms, int32_t *host_calls) {
  if (!ctx || !host_stage_ms || !host_calls) return DYLLM_ERR_INVALID_ARG;
  if (!ctx->prof_events) return fail(ctx, DYLLM_ERR_INVALID_ARG, "profiling is not on");
  std::vector<hipEvent_t> &ev = *ctx->prof_events;
  int rc = DYLLM_OK;
  for (int i = 0; i < N_STAGES; ++i) host_stage_ms[i] = 0.f;
  for (int c = 0; c < ctx->prof_calls && rc == DYLLM_OK; ++c) {
    hipEvent_t *e = ev.data() + (size_t)c * (N_STAGES + 1);
    if (hipEventSynchronize(e[N_STAGES]) != hipSuccess) rc = hip_fail(ctx, hipGetLastError(), "event sync");
    for (int i = 0; i < N_STAGES && rc == DYLLM_OK; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, e[i], e[i + 1]) != hipSuccess) rc = hip_fail(ctx, hipGetLastError(), "event elapsed");
      host_stage_ms[i] += ms;
    }
  }
  *host_calls = ctx->prof_calls;
  if (rc == DYLLM_OK && ctx->prof_calls > 0)
    for (int i = 0; i < N_STAGES; ++i) host_stage_ms[i] /= (float)ctx->prof_calls;
  for (hipEvent_t e : ev) (void)hipEventDestroy(e);
  delete ctx->prof_events;
  ctx->prof_events = nullptr;
  ctx->prof_cur = nullptr;
  return rc;
}

int dyllm_stage_count(void) { return N_STAGES; }
const char *dyllm_stage_name(int stage) { return (stage >= 0 && stage < N_STAGES) ? kStageNames[stage] : ""; }

int dyllm_destroy(dyllm_ctx *ctx) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  if (ctx->prof_events) {
    for (hipEvent_t e : *ctx->prof_events) (void)hipEventDestroy(e);
    delete ctx->prof_events;
  }
  hipError_t e = hipFree(ctx->ws);
  delete ctx;
  return e == hipSuccess ? DYLLM_OK : DYLLM_ERR_HIP;
}

int dyllm_poll_status(dyllm_ctx *ctx, int32_t *host_status, void *stream) {
  if (!ctx || !host_status) return DYLLM_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e = hipMemcpyAsync(host_status, ctx->status, 4, hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return hip_fail(ctx, e, "poll_status copy");
  launch_fill_i32(ctx->status, 0, 1, s);
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) return hip_fail(ctx, e, "poll_status sync");
  return DYLLM_OK;
}

int dyllm_saliency(dyllm_ctx *ctx, const void *c_new, void *c_cache, const dyllm_index_list *rows,
                   int32_t B, int32_t L, float tau, float *cos_out, uint8_t *flag_out, int commit,
                   void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  if (!c_new || !c_cache || !flag_out) return fail(ctx, DYLLM_ERR_INVALID_ARG, "NULL tensor");
  int rc = check_bl(ctx, B, L);
  if (rc) return rc;
  Rows r;
  if (rows) {
    if ((rc = check_list(ctx, rows, "rows"))) return rc;
    r = rows_of(rows, B);
  } else {
    if (commit && c_new == c_cache) return fail(ctx, DYLLM_ERR_INVALID_ARG, "commit onto itself");
    r = Rows{nullptr, nullptr, B * L};
  }
  launch_saliency(dt(ctx), c_new, c_cache, r, ctx->dq, tau, cos_out, flag_out, commit, (hipStream_t)stream);
  return check_launch(ctx, "saliency");
}

int dyllm_compact(dyllm_ctx *ctx, const uint8_t *flag, const dyllm_index_list *rows, int32_t B,
                  int32_t L, dyllm_index_list *out, void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  if (!flag || !out || !out->offsets || out->cap < 0 || (!out->idx && out->cap > 0))
    return fail(ctx, DYLLM_ERR_INVALID_ARG, "NULL flag or output list");
  int rc = check_bl(ctx, B, L);
  if (rc) return rc;
  Rows r;
  if (rows) {
    if ((rc = check_list(ctx, rows, "rows"))) return rc;
    r = rows_of(rows, B);
  } else {
    r = Rows{nullptr, nullptr, B * L};
  }
  launch_compact(flag, r, B, L, out->idx, out->offsets, out->cap, ctx->status, ctx->scan, (hipStream_t)stream);
  return check_launch(ctx, "compact");
}

int dyllm_compact_static(const uint8_t *flag, const dyllm_index_list *rows, int32_t B, int32_t L,
                         dyllm_index_list *out, int32_t *status, void *stream) {
  if (!flag || !out || !out->offsets || out->cap < 0 || (!out->idx && out->cap > 0)) return DYLLM_ERR_INVALID_ARG;
  if (B <= 0 || L <= 0) return DYLLM_ERR_INVALID_ARG;
  if ((long)B * L > (1l << 30)) return DYLLM_ERR_UNSUPPORTED;
  Rows r;
  if (rows) {
    if (!rows->offsets || rows->cap < 0 || (!rows->idx && rows->cap > 0)) return DYLLM_ERR_INVALID_ARG;
    r = rows_of(rows, B);
  } else {
    r = Rows{nullptr, nullptr, B * L};
  }
  if (r.cap > DYLLM_COMPACT_STATIC_MAX_ROWS) return DYLLM_ERR_CAPACITY;
  int32_t *words = nullptr;
  const int rc = static_scratch(&words);
  if (rc) return rc;
  // words [0, COMPACT_SCAN_WORDS): the kernel's scan words, zero between calls (the kernel clears
  // them itself); the word behind them takes the overflow code when the caller gives no status word
  launch_compact(flag, r, B, L, out->idx, out->offsets, out->cap, status ? status : words + COMPACT_SCAN_WORDS,
                 words, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? DYLLM_OK : DYLLM_ERR_HIP;
}

int dyllm_qkv_refresh(dyllm_ctx *ctx, const dyllm_layer_weights *w, const void *x,
                      const dyllm_index_list *rows, int32_t B, int32_t L, dyllm_layer_cache *cache,
                      void *q_sal_out, void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  int rc;
  if ((rc = check_weights(ctx, w, true, false))) return rc;
  if (!x || !q_sal_out || !cache || !cache->k || !cache->v) return fail(ctx, DYLLM_ERR_INVALID_ARG, "NULL tensor");
  if ((rc = check_bl(ctx, B, L))) return rc;
  if ((rc = check_list(ctx, rows, "rows"))) return rc;
  return enqueue_qkv(ctx, w, x, rows_of(rows, B), L, cache, q_sal_out, (hipStream_t)stream);
}

int dyllm_partial_attention(dyllm_ctx *ctx, const void *q_sal, const void *k_cache,
                            const void *v_cache, const dyllm_index_list *rows, int32_t B, int32_t L,
                            void *c_sal_out, void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  if (!q_sal || !k_cache || !v_cache || !c_sal_out) return fail(ctx, DYLLM_ERR_INVALID_ARG, "NULL tensor");
  int rc;
  if ((rc = check_bl(ctx, B, L))) return rc;
  if ((rc = check_list(ctx, rows, "rows"))) return rc;
  return enqueue_attention(ctx, q_sal, k_cache, v_cache, rows_of(rows, B), rows->offsets, B, L,
                           c_sal_out, (hipStream_t)stream);
}

int dyllm_salient_ffn(dyllm_ctx *ctx, const dyllm_layer_weights *w, const void *x, const void *c,
                      const dyllm_index_list *rows_out, int32_t B, int32_t L, void *out_cache,
                      void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  int rc;
  if ((rc = check_weights(ctx, w, false, true))) return rc;
  if (!x || !c || !out_cache) return fail(ctx, DYLLM_ERR_INVALID_ARG, "NULL tensor");
  if (x == out_cache) return fail(ctx, DYLLM_ERR_INVALID_ARG, "x aliases out_cache");
  if ((rc = check_bl(ctx, B, L))) return rc;
  if ((rc = check_list(ctx, rows_out, "rows_out"))) return rc;
  return enqueue_ffn(ctx, w, x, c, rows_of(rows_out, B), out_cache, (size_t)B * L, (hipStream_t)stream);
}

int dyllm_layer_step(dyllm_ctx *ctx, const dyllm_layer_weights *w, dyllm_layer_cache *cache,
                     const void *x, const dyllm_index_list *idx_in, int32_t B, int32_t L, float tau,
                     dyllm_index_list *idx_out, float *cos_out, void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  int rc;
  if ((rc = check_bl(ctx, B, L))) return rc;
  if ((rc = check_sparse_layer(ctx, w, cache, x, idx_in, idx_out))) return rc;
  return enqueue_sparse_layer(ctx, w, cache, x, idx_in, B, L, tau, idx_out, cos_out, (hipStream_t)stream);
}

int check_window(dyllm_ctx *ctx, int B, int L, int row_lo) {
  if (row_lo < 0 || row_lo >= L) return fail(ctx, DYLLM_ERR_INVALID_ARG, "row_lo must lie in [0, L)");
  if ((long)B * L > ctx->rows_cap) return fail(ctx, DYLLM_ERR_CAPACITY, "B*L exceeds the context's max_rows");
  return DYLLM_OK;
}

int check_cached_norm(dyllm_ctx *ctx, int cached_norm, const dyllm_layer_cache *cache) {
  if (cached_norm && !cache->lse)
    return fail(ctx, DYLLM_ERR_INVALID_ARG, "reused normalisers need cache->lse");
  return DYLLM_OK;
}

int dyllm_layer_step_approx(dyllm_ctx *ctx, const dyllm_layer_weights *w, dyllm_layer_cache *cache,
                            const void *x, const dyllm_index_list *idx_in, int32_t B, int32_t L,
                            int32_t row_lo, float tau, int32_t cached_norm, dyllm_index_list *idx_out,
                            float *cos_out, void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  int rc;
  if ((rc = check_bl(ctx, B, L))) return rc;
  if ((rc = check_window(ctx, B, L, row_lo))) return rc;
  if ((rc = check_sparse_layer(ctx, w, cache, x, idx_in, idx_out))) return rc;
  if ((rc = check_cached_norm(ctx, cached_norm, cache))) return rc;
  const Window win = make_window(ctx, B, L, row_lo, (hipStream_t)stream);
  return enqueue_approx_layer(ctx, w, cache, x, idx_in, B, L, win, tau, cached_norm != 0, idx_out, cos_out,
                              (hipStream_t)stream);
}

int dyllm_stack_step_approx(dyllm_ctx *ctx, int32_t n_layers, const dyllm_layer_weights *w,
                            dyllm_layer_cache *caches, const void *x, const dyllm_index_list *idx_in,
                            int32_t B, int32_t L, int32_t row_lo, float tau, int32_t cached_norm,
                            dyllm_index_list *idx_out, float *cos_out, void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  if (n_layers <= 0 || !w || !caches || !idx_out) return fail(ctx, DYLLM_ERR_INVALID_ARG, "empty stack or NULL array");
  int rc;
  if ((rc = check_bl(ctx, B, L))) return rc;
  if ((rc = check_window(ctx, B, L, row_lo))) return rc;
  for (int l = 0; l < n_layers; ++l) {
    const void *xl = l ? caches[l - 1].out : x;
    const dyllm_index_list *in = l ? &idx_out[l - 1] : idx_in;
    if ((rc = check_sparse_layer(ctx, &w[l], &caches[l], xl, in, &idx_out[l]))) return rc;
    if ((rc = check_cached_norm(ctx, cached_norm, &caches[l]))) return rc;
  }
  const Window win = make_window(ctx, B, L, row_lo, (hipStream_t)stream);
  const dyllm_index_list *in = idx_in;
  for (int l = 0; l < n_layers; ++l) {
    float *cos_l = cos_out ? cos_out + (size_t)l * B * L : nullptr;
    if ((rc = enqueue_approx_layer(ctx, &w[l], &caches[l], l ? caches[l - 1].out : x, in, B, L, win, tau,
                                   cached_norm != 0, &idx_out[l], cos_l, (hipStream_t)stream)))
      return rc;
    in = &idx_out[l];
  }
  return DYLLM_OK;
}

int dyllm_merge_lists(dyllm_ctx *ctx, const dyllm_index_list *a, const dyllm_index_list *b, int32_t B,
                      int32_t L, int32_t pos_lo, dyllm_index_list *out, void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  int rc;
  if ((rc = check_bl(ctx, B, L))) return rc;
  if ((rc = check_window(ctx, B, L, pos_lo))) return rc;
  if (a && (rc = check_list(ctx, a, "a"))) return rc;
  if (b && (rc = check_list(ctx, b, "b"))) return rc;
  if ((rc = check_list(ctx, out, "out"))) return rc;
  if ((a && (out->offsets == a->offsets || (out->idx && out->idx == a->idx))) ||
      (b && (out->offsets == b->offsets || (out->idx && out->idx == b->idx))))
    return fail(ctx, DYLLM_ERR_INVALID_ARG, "out aliases an input list");
  return enqueue_merge(ctx, a, b, B, L, pos_lo, out, (hipStream_t)stream);
}

int dyllm_pack_weight(const void *src, int32_t n_out, int32_t n_in, void *dst, void *stream) {
  if (!src || !dst || src == dst) return DYLLM_ERR_INVALID_ARG;
  if (n_out <= 0 || n_in <= 0) return DYLLM_ERR_INVALID_ARG;
  if (n_out % 32 || n_in % 64) return DYLLM_ERR_UNSUPPORTED;
  launch_pack_weight(src, n_out, n_in, dst, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? DYLLM_OK : DYLLM_ERR_HIP;
}

int dyllm_step_kind(const dyllm_schedule *sched, int32_t t) {
  if (!sched || t < 0) return DYLLM_ERR_INVALID_ARG;
  if (t < sched->t_full) return DYLLM_STEP_DENSE;
  return (sched->full_period <= 1 || t % sched->full_period == 0) ? DYLLM_STEP_FULL : DYLLM_STEP_RESPONSE;
}

int dyllm_denoise_step(dyllm_ctx *ctx, const dyllm_schedule *sched, int32_t t, int32_t n_layers,
                       const dyllm_layer_weights *w, dyllm_layer_cache *caches, const void *x,
                       const dyllm_index_list *decoded, const dyllm_index_list *carry, int32_t B,
                       int32_t L, dyllm_index_list *cand, dyllm_index_list *idx_out, void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  if (!sched) return fail(ctx, DYLLM_ERR_INVALID_ARG, "schedule is NULL");
  const int kind = dyllm_step_kind(sched, t);
  if (kind < 0) return fail(ctx, DYLLM_ERR_INVALID_ARG, "negative step number");
  if (sched->t_full < 0 || sched->prompt_len < 0) return fail(ctx, DYLLM_ERR_INVALID_ARG, "negative schedule field");
  if (kind == DYLLM_STEP_DENSE) return dyllm_stack_full_step(ctx, n_layers, w, caches, x, B, L, stream);
  if (!cand || !idx_out) return fail(ctx, DYLLM_ERR_INVALID_ARG, "cand / idx_out is NULL");
  const int row_lo = kind == DYLLM_STEP_FULL ? 0 : sched->prompt_len;
  int rc;
  if ((rc = dyllm_merge_lists(ctx, carry, decoded, B, L, row_lo, cand, stream))) return rc;
  if (sched->approx)
    return dyllm_stack_step_approx(ctx, n_layers, w, caches, x, cand, B, L, row_lo, sched->tau,
                                   sched->approx == 2, idx_out, nullptr, stream);
  return dyllm_stack_step(ctx, n_layers, w, caches, x, cand, B, L, sched->tau, idx_out, nullptr, stream);
}

int dyllm_full_step(dyllm_ctx *ctx, const dyllm_layer_weights *w, dyllm_layer_cache *cache,
                    const void *x, int32_t B, int32_t L, void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  int rc;
  if ((rc = check_bl(ctx, B, L))) return rc;
  if ((long)B * L > ctx->rows_cap) return fail(ctx, DYLLM_ERR_CAPACITY, "B*L exceeds the context's max_rows");
  if ((rc = check_dense_layer(ctx, w, cache, x))) return rc;
  return enqueue_dense_layer(ctx, w, cache, x, B, L, (hipStream_t)stream);
}

int dyllm_stack_step(dyllm_ctx *ctx, int32_t n_layers, const dyllm_layer_weights *w,
                     dyllm_layer_cache *caches, const void *x, const dyllm_index_list *idx_in,
                     int32_t B, int32_t L, float tau, dyllm_index_list *idx_out, float *cos_out,
                     void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  if (n_layers <= 0 || !w || !caches || !idx_out) return fail(ctx, DYLLM_ERR_INVALID_ARG, "empty stack or NULL array");
  int rc;
  if ((rc = check_bl(ctx, B, L))) return rc;
  // every argument of every layer is checked before the first launch
  for (int l = 0; l < n_layers; ++l) {
    const void *xl = l ? caches[l - 1].out : x;
    const dyllm_index_list *in = l ? &idx_out[l - 1] : idx_in;
    if ((rc = check_sparse_layer(ctx, &w[l], &caches[l], xl, in, &idx_out[l]))) return rc;
  }
  // a layer's selection is a subset of the first layer's candidates: that capacity sizes every grid
  const int cap0 = idx_in->cap;
  dyllm_index_list in = *idx_in;
  for (int l = 0; l < n_layers; ++l) {
    dyllm_index_list out = idx_out[l];
    if (out.cap > cap0) out.cap = cap0;
    float *cos_l = cos_out ? cos_out + (size_t)l * cap0 : nullptr;
    if ((rc = enqueue_sparse_layer(ctx, &w[l], &caches[l], l ? caches[l - 1].out : x, &in, B, L, tau,
                                   &out, cos_l, (hipStream_t)stream)))
      return rc;
    in = out;
  }
  return DYLLM_OK;
}

int dyllm_stack_full_step(dyllm_ctx *ctx, int32_t n_layers, const dyllm_layer_weights *w,
                          dyllm_layer_cache *caches, const void *x, int32_t B, int32_t L,
                          void *stream) {
  if (!ctx) return DYLLM_ERR_INVALID_ARG;
  if (n_layers <= 0 || !w || !caches) return fail(ctx, DYLLM_ERR_INVALID_ARG, "empty stack or NULL array");
  int rc;
  if ((rc = check_bl(ctx, B, L))) return rc;
  if ((long)B * L > ctx->rows_cap) return fail(ctx, DYLLM_ERR_CAPACITY, "B*L exceeds the context's max_rows");
  for (int l = 0; l < n_layers; ++l)
    if ((rc = check_dense_layer(ctx, &w[l], &caches[l], l ? caches[l - 1].out : x))) return rc;
  for (int l = 0; l < n_layers; ++l)
    if ((rc = enqueue_dense_layer(ctx, &w[l], &caches[l], l ? caches[l - 1].out : x, B, L,
                                  (hipStream_t)stream)))
      return rc;
  return DYLLM_OK;
}

}  // extern "C"
