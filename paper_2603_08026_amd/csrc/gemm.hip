// Dispatch of the salient-row GEMMs by storage type: fp32 -> FMA kernels, bf16 -> MFMA kernels.
#include "kernels.h"

namespace dy {

void gemm_f32_raw(DType, GemmA, Rows, int, WSeg, float *, hipStream_t);
void gemm_f32_swiglu(DType, GemmA, Rows, int, int, const void *, const void *, void *, hipStream_t);
void gemm_f32_down(DType, GemmA, Rows, int, int, const void *, const float *, void *, hipStream_t);

Splits gemm_bf16_raw(GemmA, Rows, int, WSeg, float *, size_t, hipStream_t);
void gemm_bf16_swiglu(GemmA, Rows, int, int, const void *, const void *, void *, float *, size_t, hipStream_t);
void gemm_bf16_down(GemmA, Rows, int, int, const void *, const float *, void *, float *, size_t, hipStream_t);

Splits launch_gemm_raw(DType t, GemmA A, Rows rows, int K, WSeg seg, float *part, size_t part_elems,
                       hipStream_t s) {
  if (t == F32) {
    gemm_f32_raw(t, A, rows, K, seg, part, s);
    return Splits{};
  }
  return gemm_bf16_raw(A, rows, K, seg, part, part_elems, s);
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
