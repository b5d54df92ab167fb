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

// ---- row kernels (HBM-bound) ------------------------------------------------------------------
// out[j,:] = RMSNorm(x[row_j,:]) * gain            x: [T,d] T-typed, out: [cap,d] T-typed
void launch_gather_rmsnorm(DType t, const void *x, const void *gain, Rows rows, int d, float eps,
                           void *out, hipStream_t s);
// out[j,:] = RMSNorm(h[j,:]) * gain                h: [cap,d] fp32, out: [cap,d] T-typed
void launch_rmsnorm_f32in(DType t, const float *h, const void *gain, Rows rows, int d, float eps,
                          void *out, hipStream_t s);
// qkv: [cap, dq+2dkv] fp32 (unrotated, bias not yet added).  Adds bias, rotates q and k by the
// table entry of position (row mod L), writes q_out[j] (T-typed [cap,dq]) and scatters k, v rows
// into the caches at row_j.  rope_tab: [max_seq, dh/2, 2] fp32 (cos, sin).
void launch_rope_scatter(DType t, const float *qkv, const float *rope_tab, Rows rows, int L, int H,
                         int Hkv, int dh, const void *bq, const void *bk, const void *bv,
                         void *q_out, void *k_cache, void *v_cache, hipStream_t s);
// cosine of c_new[j] vs c_cache[row_j], flag = cos < tau, optional commit of the new row.
void launch_saliency(DType t, const void *c_new, void *c_cache, Rows rows, int D, float tau,
                     float *cos_out, uint8_t *flag_out, int commit, hipStream_t s);
// stable compaction (single workgroup); out_offsets[b] = #selected tokens with id < b*L.
void launch_compact(const uint8_t *flag, Rows rows, int B, int L, int32_t *out_idx,
                    int32_t *out_offsets, int out_cap, int32_t *status, hipStream_t s);

// ---- attention ---------------------------------------------------------------------------------
struct AttnArgs {
  const void *q;        // [cap, H, dh] T-typed
  const void *k, *v;    // [B, L, Hkv, dh] T-typed
  Rows rows;            // token ids of the query rows (idx may be nullptr = identity)
  const int32_t *offsets;  // [B+1] per-sequence offsets into rows, or nullptr = every sequence has L rows
  int B, L, H, Hkv, dh;
  int splits;           // key range split into this many parts (>= 1), none of them empty
  int chunk;            // keys per split (multiple of the key tile); split s covers [s*chunk, min(L,(s+1)*chunk))
  float *part_o;        // [splits, cap, H*dh] fp32 un-normalised partial outputs (splits > 1)
  float *part_ml;       // [splits, cap, H, 2] fp32 (running max, running sum)     (splits > 1)
  void *out;            // [cap, H*dh] T-typed
};
void launch_attention(DType t, const AttnArgs &a, hipStream_t s);
// Chooses splits and chunk for a call (host).
void attention_plan(DType t, int B, int L, int H, int dh, int cap, size_t part_elems, int *splits,
                    int *chunk);

// ---- GEMMs  C[m,n] = sum_k A[m,k] * W[n,k]  (W is [N,K] row-major) -----------------------------
struct GemmA {
  const void *a;        // T-typed, row stride lda
  const int32_t *gather;  // nullptr, or row j of the GEMM reads a[gather[j], :]
  int lda;
};
// qkv: out[j, 0:dq | dq:dq+dkv | dq+dkv:] = A[j,:] * (wq | wk | wv)^T, fp32 out [cap, dq+2dkv]
// `scratch` (fp32, scratch_elems) holds K-split partial sums when a launcher decides to split K.
void launch_gemm_qkv(DType t, GemmA A, Rows rows, int K, const void *wq, const void *wk,
                     const void *wv, int dq, int dkv, float *out, float *scratch,
                     size_t scratch_elems, hipStream_t s);
// o-proj: h[j,:] = x[row_j,:] + A[j,:] * wo^T, fp32 out [cap, N]; x T-typed [T, N]
void launch_gemm_oproj(DType t, GemmA A, Rows rows, int K, int N, const void *wo, const void *x,
                       float *h, float *scratch, size_t scratch_elems, hipStream_t s);
// up: act[j,:] = silu(A w_gate^T) * (A w_up^T), T-typed out [cap, N]
void launch_gemm_swiglu(DType t, GemmA A, Rows rows, int K, int N, const void *w_gate,
                        const void *w_up, void *act, float *scratch, size_t scratch_elems,
                        hipStream_t s);
// down: out_cache[row_j,:] = h[j,:] + A[j,:] * w_down^T, T-typed scatter into [T, N]
void launch_gemm_down(DType t, GemmA A, Rows rows, int K, int N, const void *w_down, const float *h,
                      void *out_cache, float *scratch, size_t scratch_elems, hipStream_t s);

void launch_fill_i32(int32_t *p, int32_t v, int n, hipStream_t s);

}  // namespace dy
