// Epilogues of the salient-row GEMMs.  Each takes the fp32 accumulator(s) of output element
// (j, n) -- j = position in the row list, n = output column -- and finishes the fused step:
//   EpiStoreF32 ... plain fp32 store (raw result; a finalize row kernel follows)
//   EpiSwiGLU ..... act = silu(acc_gate) * acc_up           [Alg. 3: FFN, first half]
//   EpiDown ....... out_cache[row_j] = h + acc              [Alg. 3: FFN second half + cache commit]
#pragma once
#include "common.h"
#include "kernels.h"

namespace dy {

struct EpiStoreF32 {
  static constexpr bool DUAL = false;
  float *out;
  int ldo;
  __device__ __forceinline__ void operator()(int j, int row, int n, float acc, float) const {
    (void)row;
    out[(size_t)j * ldo + n] = acc;
  }
};

template <typename T> struct EpiSwiGLU {
  static constexpr bool DUAL = true;
  T *act;  // [cap, N]
  int N;
  __device__ __forceinline__ void operator()(int j, int row, int n, float gate, float up) const {
    (void)row;
    const float s = gate / (1.0f + __expf(-gate));
    act[(size_t)j * N + n] = from_f<T>(s * up);
  }
};

template <typename T> struct EpiDown {
  static constexpr bool DUAL = false;
  const float *h;  // [cap, N]
  T *out;          // [T, N]
  int N;
  __device__ __forceinline__ void operator()(int j, int row, int n, float acc, float) const {
    out[(size_t)row * N + n] = from_f<T>(h[(size_t)j * N + n] + acc);
  }
};

}  // namespace dy
