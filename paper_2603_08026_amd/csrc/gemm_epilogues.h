// Epilogues of the salient-row GEMMs.  Each takes the fp32 accumulator(s) of output element
// (j, n) -- j = position in the row list, n = output column -- and finishes the fused step:
//   EpiStoreF32 ... plain fp32 store (raw result; a finalize row kernel follows)
//   EpiSwiGLU ..... act = silu(acc_gate) * acc_up           [Alg. 3: FFN, first half]
//   EpiDown ....... out_cache[row_j] = h + acc              [Alg. 3: FFN second half + cache commit]
//   EpiSwiGLUHalves  the same SwiGLU for the weight-streaming regime: a column tile holds HALF gate
//                   columns followed by the HALF up columns of the same outputs (the kernel looks the
//                   weight rows up that way), so one matrix serves per tile and the product never
//                   leaves the registers
// INTERLEAVE = that HALF (0: the tile's columns are consecutive rows of the stacked matrices).
#pragma once
#include "common.h"
#include "kernels.h"

namespace dy {

struct EpiStoreF32 {
  static constexpr bool DUAL = false;
  static constexpr int INTERLEAVE = 0;
  static constexpr bool PRELOAD = false;
  float *out;
  int ldo;
  __device__ __forceinline__ void operator()(int j, int row, int n, float acc, float) const {
    (void)row;
    out[(size_t)j * ldo + n] = acc;
  }
};

template <typename T> struct EpiSwiGLU {
  static constexpr bool DUAL = true;
  static constexpr int INTERLEAVE = 0;
  static constexpr bool PRELOAD = false;
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
  static constexpr int INTERLEAVE = 0;
  // The residual is read before the result is written.  h and out may alias as far as the compiler
  // knows, so element by element every load would wait for the store before it; the kernel instead
  // loads a block's residuals (load) and then stores the block (store).
  static constexpr bool PRELOAD = true;
  const float *h;  // [cap, N]
  T *out;          // [T, N]
  int N;
  __device__ __forceinline__ float load(int j, int n) const { return h[(size_t)j * N + n]; }
  __device__ __forceinline__ void store(int row, int n, float acc, float hv) const {
    out[(size_t)row * N + n] = from_f<T>(hv + acc);
  }
  __device__ __forceinline__ void operator()(int j, int row, int n, float acc, float) const {
    store(row, n, acc, load(j, n));
  }
};

template <typename T, int HALF> struct EpiSwiGLUHalves {
  static constexpr bool DUAL = false;
  static constexpr int INTERLEAVE = HALF;  // 48 (96-column tiles) or 64 (128-column tiles)
  static constexpr bool PRELOAD = false;
  T *act;  // [cap, F]
  int F;
  // f = output column of the FFN's hidden layer
  __device__ __forceinline__ void store(int j, int f, float gate, float up) const {
    const float s = gate / (1.0f + __expf(-gate));
    act[(size_t)j * F + f] = from_f<T>(s * up);
  }
  __device__ __forceinline__ void operator()(int, int, int, float, float) const {}
};

}  // namespace dy
