// bf16 salient-row GEMMs (placeholder: routes through the FMA kernels until the MFMA kernels land).
#include "kernels.h"

namespace dy {

void gemm_f32_qkv(DType, GemmA, Rows, int, const void *, const void *, const void *, int, int, float *, hipStream_t);
void gemm_f32_oproj(DType, GemmA, Rows, int, int, const void *, const void *, float *, hipStream_t);
void gemm_f32_swiglu(DType, GemmA, Rows, int, int, const void *, const void *, void *, hipStream_t);
void gemm_f32_down(DType, GemmA, Rows, int, int, const void *, const float *, void *, hipStream_t);

void gemm_bf16_qkv(GemmA A, Rows rows, int K, const void *wq, const void *wk, const void *wv, int dq,
                   int dkv, float *out, hipStream_t s) {
  gemm_f32_qkv(BF16, A, rows, K, wq, wk, wv, dq, dkv, out, s);
}
void gemm_bf16_oproj(GemmA A, Rows rows, int K, int N, const void *wo, const void *x, float *h,
                     hipStream_t s) {
  gemm_f32_oproj(BF16, A, rows, K, N, wo, x, h, s);
}
void gemm_bf16_swiglu(GemmA A, Rows rows, int K, int N, const void *wg, const void *wu, void *act,
                      hipStream_t s) {
  gemm_f32_swiglu(BF16, A, rows, K, N, wg, wu, act, s);
}
void gemm_bf16_down(GemmA A, Rows rows, int K, int N, const void *wd, const float *h, void *out,
                    hipStream_t s) {
  gemm_f32_down(BF16, A, rows, K, N, wd, h, out, s);
}

}  // namespace dy
