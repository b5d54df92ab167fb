// Dispatch of the salient-row GEMMs by storage type: fp32 -> FMA kernels, bf16 -> MFMA kernels.
#include "kernels.h"

namespace dy {

void gemm_f32_qkv(DType, GemmA, Rows, int, const void *, const void *, const void *, int, int, float *, hipStream_t);
void gemm_f32_oproj(DType, GemmA, Rows, int, int, const void *, const void *, float *, hipStream_t);
void gemm_f32_swiglu(DType, GemmA, Rows, int, int, const void *, const void *, void *, hipStream_t);
void gemm_f32_down(DType, GemmA, Rows, int, int, const void *, const float *, void *, hipStream_t);

void gemm_bf16_qkv(GemmA, Rows, int, const void *, const void *, const void *, int, int, float *, float *, size_t, hipStream_t);
void gemm_bf16_oproj(GemmA, Rows, int, int, const void *, const void *, float *, float *, size_t, hipStream_t);
void gemm_bf16_swiglu(GemmA, Rows, int, int, const void *, const void *, void *, float *, size_t, hipStream_t);
void gemm_bf16_down(GemmA, Rows, int, int, const void *, const float *, void *, float *, size_t, hipStream_t);

void launch_gemm_qkv(DType t, GemmA A, Rows rows, int K, const void *wq, const void *wk,
                     const void *wv, int dq, int dkv, float *out, float *scratch,
                     size_t scratch_elems, hipStream_t s) {
  if (t == F32) gemm_f32_qkv(t, A, rows, K, wq, wk, wv, dq, dkv, out, s);
  else gemm_bf16_qkv(A, rows, K, wq, wk, wv, dq, dkv, out, scratch, scratch_elems, s);
}

void launch_gemm_oproj(DType t, GemmA A, Rows rows, int K, int N, const void *wo, const void *x,
                       float *h, float *scratch, size_t scratch_elems, hipStream_t s) {
  if (t == F32) gemm_f32_oproj(t, A, rows, K, N, wo, x, h, s);
  else gemm_bf16_oproj(A, rows, K, N, wo, x, h, scratch, scratch_elems, s);
}

void launch_gemm_swiglu(DType t, GemmA A, Rows rows, int K, int N, const void *w_gate,
                        const void *w_up, void *act, float *scratch, size_t scratch_elems,
                        hipStream_t s) {
  if (t == F32) gemm_f32_swiglu(t, A, rows, K, N, w_gate, w_up, act, s);
  else gemm_bf16_swiglu(A, rows, K, N, w_gate, w_up, act, scratch, scratch_elems, s);
}

void launch_gemm_down(DType t, GemmA A, Rows rows, int K, int N, const void *w_down, const float *h,
                      void *out_cache, float *scratch, size_t scratch_elems, hipStream_t s) {
  if (t == F32) gemm_f32_down(t, A, rows, K, N, w_down, h, out_cache, s);
  else gemm_bf16_down(A, rows, K, N, w_down, h, out_cache, scratch, scratch_elems, s);
}

}  // namespace dy
