// Host-side launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dy {

enum DType { F32 = 0, BF16 = 1 };

// A list of token rows living on the device.  idx == nullptr means the identity (row j = token j);
// count == nullptr means exactly `cap` rows.  The device count is clamped to cap by every kernel.
struct Rows {
  const int32_t *idx;
  const int32_t *count;
  int32_t cap;
};

// K splits of a raw GEMM result: the rows below tail_from hold n partial sums each, the rows from
// tail_from on (a short last row tile that a launch of its own computed) n_tail.
struct Splits {
  int n = 1, tail_from = 0x7fffffff, n_tail = 1;
  int done_to = 0;  // down projection: rows below it need no sum kernel (the GEMM's own epilogue wrote them)
  __host__ __device__ int of(int j) const { return j < tail_from ? n : n_tail; }
};

// ---- row kernels (HBM-bound) ------------------------------------------------------------------
// out[j,:] = RMSNorm(x[row_j,:]) * gain            x: [T,d] T-typed, out: [cap,d] T-typed
void launch_gather_rmsnorm(DType t, const void *x, const void *gain, Rows rows, int d, float eps,
                           void *out, hipStream_t s);
// The GEMMs leave fp32 "raw" results part[z][j][n] (z = K split, j = position in the row list); the
// finalize kernels below sum the splits and apply the fused tail of the step, one workgroup per row.
//
// q/k/v: sum of splits + bias, rotary embedding of q and k by the table entry of position
// (row mod L), q_out[j] (T-typed [cap,dq]; q_out[row_j] when q_by_token), k and v rows scattered into
// the caches at row_j; dv_out (may be nullptr) takes v - v_cache of those rows before the merge, at
// row_j or (dv_by_entry) at j; ksal_out (may be nullptr) takes a copy of the rotated k rows at j.
// rope_tab: [max_seq, dh/2, 2] fp32 (cos, sin).  dh is 64 or 128.
// dv_out (optional, [T, Hkv*dh] T-typed): value residual new - cached of the rows, taken before the merge
// entry_of (optional, [T] int32): entry_of[row_j] = j + 1, the map from a token to its list entry, written
// for the rows at positions >= entry_lo of their sequence only
void launch_qkv_finalize(DType t, const float *part, Splits splits, size_t split_stride,
                         const float *rope_tab, Rows rows, int L, int H, int Hkv, int dh,
                         const void *bq, const void *bk, const void *bv, void *q_out, void *k_cache,
                         void *v_cache, void *dv_out, int q_by_token, void *ksal_out, int dv_by_entry,
                         int32_t *entry_of, int entry_lo, hipStream_t s);
// out-projection: h[j] = x[row_j] + sum of splits (fp32 [cap,d]); f[j] = RMSNorm(h[j]) * gain (T-typed)
void launch_oproj_finalize(DType t, const float *part, Splits splits, size_t split_stride, const void *x,
                           const void *gain, Rows rows, int d, float eps, float *h, void *f,
                           hipStream_t s);
// down projection after a K split: out_cache[row_j] = h[j] + sum of splits, for the rows from
// splits.done_to on (the rows below it were written by the GEMM's own epilogue)
void launch_down_finalize(DType t, const float *part, Splits splits, size_t split_stride, const float *h,
                          Rows rows, int d, void *out_cache, hipStream_t s);
// cosine of c_new[j] vs c_cache[row_j], flag = cos < tau, optional commit of the new row.
void launch_saliency(DType t, const void *c_new, void *c_cache, Rows rows, int D, float tau,
                     float *cos_out, uint8_t *flag_out, int commit, hipStream_t s);
// stable compaction over up to 1024 chained workgroups; out_offsets[b] = #selected tokens with id < b*L.
// scan: compact_scan_words() device ints, all zero before the launch; the kernel leaves them zero.
// Launches that share `scan` must not overlap.
void launch_compact(const uint8_t *flag, Rows rows, int B, int L, int32_t *out_idx,
                    int32_t *out_offsets, int out_cap, int32_t *status, int32_t *scan, hipStream_t s);
constexpr int COMPACT_SCAN_WORDS = 2 + 1024;
inline int compact_scan_words() { return COMPACT_SCAN_WORDS; }

// The cosine test from per-head sums, then the same compaction: entry j of `rows` has
// cos = sum_h p[j][h][0] / (max(sqrt(sum_h p[j][h][1]), 1e-8) * max(sqrt(sum_h p[j][h][2]), 1e-8)),
// flag = cos < tau; cos_out[j] and flag_out[j] are written, the flagged tokens compacted as by
// launch_compact.  cos_part: [cap, H, 4] fp32.
void launch_cos_compact(const float *cos_part, int H, float tau, float *cos_out, uint8_t *flag_out, Rows rows,
                        int B, int L, int32_t *out_idx, int32_t *out_offsets, int out_cap, int32_t *status,
                        int32_t *scan, hipStream_t s);

// ---- attention ---------------------------------------------------------------------------------
struct AttnArgs {
  const void *q;        // [cap, H, dh] T-typed; with q_by_token: [T, H, dh], row of query j = rows.idx[j]
  int q_by_token;
  const void *k, *v;    // [B, L, Hkv, dh] T-typed; with key_offsets: compact rows [*, Hkv, dh]
  const int32_t *key_offsets;  // nullptr, or [B+1]: the keys of sequence b are rows [key_offsets[b],
                               // key_offsets[b+1]) of k / v (a split past a sequence's last key writes nothing)
  float *lse_out;       // nullptr, or [T, H]: the merge kernels store log(sum exp) of every merged row here
  Rows rows;            // token ids of the query rows (idx may be nullptr = identity)
  const int32_t *offsets;  // [B+1] per-sequence offsets into rows, or nullptr = every sequence has L rows
  int B, L, H, Hkv, dh;
  int splits;           // key range split into this many parts (>= 1), none of them empty
  int chunk;            // keys per split (multiple of the key tile); split s covers [s*chunk, min(L,(s+1)*chunk))
  int bq;               // query rows per workgroup the plan chose (bf16: 128 or 64; fp32: 16)
  int partial;          // 1: leave partials even for a single split (a finalize kernel follows)
  float *part_o;        // [splits, cap, H*dh] fp32 un-normalised partial outputs
  float *part_ml;       // [splits, cap, H, 2] fp32 (running max in natural-log units, running sum)
  void *out;            // [cap, H*dh] T-typed (unused when partials are left)
  // Fused commit (bf16, head_dim 128, one key split; null otherwise): the attention kernel itself
  // normalises its rows, rounds them to the storage type, reads the cached context row of the query's
  // token (rows.idx, or the identity), overwrites it with the new one, and leaves the three sums the
  // cosine needs -- <new, old>, |new|^2, |old|^2 over the head's dh columns -- in cos_part[j][h][0..2]
  // (fp32, [cap, H, 4]); no partial output is written.
  void *c_commit;       // [T, H*dh] T-typed context cache
  float *cos_part;
};
// attention rows; merges the splits into a.out unless a.partial is set
void launch_attention(DType t, const AttnArgs &a, hipStream_t s);
// merge of the attention partials of a call that left them (a.partial) into a.out (and a.lse_out)
void launch_attn_combine(DType t, const AttnArgs &a, hipStream_t s);
// merge of the attention partials fused with the saliency test and the context commit:
// new = merged row (rounded to T), cos against c_cache[row_j], flag = cos < tau, c_cache[row_j] = new.
// The workgroup that finishes last also compacts the flags into (out_idx, out_offsets) like
// launch_compact; `counter` is a zero-initialised device word the kernel leaves at zero.
void launch_attn_finalize(DType t, const AttnArgs &a, void *c_cache, float tau, float *cos_out,
                          uint8_t *flag_out, int32_t *out_idx, int32_t *out_offsets, int out_cap,
                          int32_t *status, int32_t *counter, hipStream_t s);
// Chooses the query tile, the number of key splits and the keys per split for a call (host);
// rows_per_seq = expected query rows per sequence (capacity / B for a row list, L for a dense step);
// grouped_heads = query heads per KV head.
void attention_plan(DType t, int B, int L, int H, int dh, int cap, int rows_per_seq, size_t part_elems,
                    AttnArgs *a, int grouped_heads);

// ---- GEMMs  C[m,n] = sum_k A[m,k] * W[n,k]  (W [N,K]: row-major for fp32, 32-row panels for bf16) --
struct GemmA {
  const void *a;        // T-typed, row stride lda
  const int32_t *gather;  // nullptr, or row j of the GEMM reads a[gather[j], :]
  int lda;
  // rows of the buffer `a` points to when `gather` is set (without it the row list's capacity bounds
  // the rows read); 0 = unknown.  Kernels that address the operand with 32-bit offsets need it.
  size_t a_rows = 0;
};
// Up to three weight matrices stacked along N (q | k | v); the bf16 kernels look the matrix up per
// tile row, so a column tile may span two of them.
struct WSeg {
  const void *w[3];
  int n_end[3];  // exclusive end column of each segment; N = n_end[2]
};
inline WSeg wseg_one(const void *w, int N) {
  WSeg s;
  s.w[0] = s.w[1] = s.w[2] = w;
  s.n_end[0] = s.n_end[1] = s.n_end[2] = N;
  return s;
}
// raw GEMM: part[z][j][n] = sum over K split z of A[j,:] * W[n,:] (fp32, split stride cap*N);
// returns the numbers of splits used (>= 1), chosen from the capacity, N and K.
Splits launch_gemm_raw(DType t, GemmA A, Rows rows, int K, WSeg seg, float *part, size_t part_elems,
                    hipStream_t s);
// up: act[j,:] = silu(A w_gate^T) * (A w_up^T), T-typed out [cap, N]
// `scratch` holds the raw gate|up result in the weight-streaming regime (then a row kernel applies
// the SwiGLU); otherwise the epilogue is fused.
void launch_gemm_swiglu(DType t, GemmA A, Rows rows, int K, int N, const void *w_gate,
                        const void *w_up, void *act, float *scratch, size_t scratch_elems,
                        hipStream_t s);
// down: out_cache[row_j,:] = h[j,:] + A[j,:] * w_down^T, T-typed scatter into [T, N]; `scratch`
// holds K-split partials when the launcher decides to split.
void launch_gemm_down(DType t, GemmA A, Rows rows, int K, int N, const void *w_down, const float *h,
                      void *out_cache, float *scratch, size_t scratch_elems, hipStream_t s);

// row-major [n_out, n_in] (2-byte elements; n_out % 32 == 0, n_in % 64 == 0) -> weight panels of the bf16 GEMMs
void launch_pack_weight(const void *src, int n_out, int n_in, void *dst, hipStream_t s);
void launch_fill_i32(int32_t *p, int32_t v, int n, hipStream_t s);

// ---- approximate (column-sparse) context update of the non-salient rows  [Sec. 3.3; Alg. 3, Alg. 4]
// pos[row_j] = j + 1 for the candidates among the step's tokens (written by the k|v finalize kernel of
// the step through its entry_of argument, consumed and zeroed by launch_saliency_approx; pos is zero
// elsewhere, before and after a step)
// For every entry j of the window `win` (token r = win.idx[j], or j): new context = c_sal[pos[r]-1]
// where pos[r] != 0, else c_cache[r] + residual (rounded to T); cosine against the cached row, commit;
// cos_out[r] (may be nullptr), flag_out[j] = cos < tau.  The residual is dc[j], or (cached != nullptr)
// sum over the key splits s of part_o[s][j] * exp(m_s - lse[r, h]) from the partials of an attention
// pass over the compact candidate keys (cached->key_offsets) -- the normalisers are NOT recomputed.
// Every pos entry that is read non-zero is set back to zero.
void launch_saliency_approx(DType t, Rows win, int D, const void *c_sal, const void *dc, int32_t *pos,
                            void *c_cache, float tau, float *cos_out, uint8_t *flag_out,
                            const AttnArgs *cached, const float *lse, int L, hipStream_t s);
// idx/off := the tokens at positions [lo, L) of each of the B sequences, as an index list
void launch_make_window(int B, int L, int lo, int32_t *idx, int32_t *off, hipStream_t s);
// flag[r] = 1 for every token r < T of the list whose position in its sequence is >= lo
void launch_mark_flags(Rows rows, int T, int L, int lo, uint8_t *flag, hipStream_t s);
// dv[row_j, :] = 0 for the rows of the list
void launch_clear_rows(DType t, Rows rows, void *dv, int dkv, hipStream_t s);

}  // namespace dy
