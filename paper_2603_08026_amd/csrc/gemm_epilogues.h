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
//
// Full tiles address their results as a wave-uniform element offset u = row * ld + col (held in
// scalar registers) plus one byte offset per lane that is fixed for the whole tile (lane_bytes: the
// lane's 4 * (lane / 32) rows and lane % 32 columns), so a store costs no vector address arithmetic:
// put(u, lane_bytes, ...).
#pragma once
#include "common.h"
#include "kernels.h"

namespace dy {

// x * sigmoid(x) in fp32.  For 2-byte outputs the hardware reciprocal (1 ulp) replaces the division:
// its error is far below the rounding of the result, and the division is a ten-instruction sequence
// per element of the epilogue.
template <typename T> __device__ __forceinline__ float silu_for(float x) {
  if constexpr (sizeof(T) == 2) return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x));
  else return x / (1.0f + __expf(-x));
}

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
  __device__ __forceinline__ int ld() const { return ldo; }
  __device__ __forceinline__ uint32_t lane_bytes(int lhi, int l32) const { return ((uint32_t)(4 * lhi) * ldo + l32) * 4u; }
  __device__ __forceinline__ void put(size_t u, uint32_t lb, float acc, float) const {
    *reinterpret_cast<float *>(reinterpret_cast<char *>(out + u) + lb) = acc;
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
    const float s = silu_for<T>(gate);
    act[(size_t)j * N + n] = from_f<T>(s * up);
  }
  __device__ __forceinline__ int ld() const { return N; }
  __device__ __forceinline__ uint32_t lane_bytes(int lhi, int l32) const {
    return ((uint32_t)(4 * lhi) * N + l32) * (uint32_t)sizeof(T);
  }
  __device__ __forceinline__ void put(size_t u, uint32_t lb, float gate, float up) const {
    const float s = silu_for<T>(gate);
    *reinterpret_cast<T *>(reinterpret_cast<char *>(act + u) + lb) = from_f<T>(s * up);
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
  __device__ __forceinline__ int ld() const { return N; }
  __device__ __forceinline__ uint32_t lane_bytes(int lhi, int l32) const {
    return ((uint32_t)(4 * lhi) * N + l32) * (uint32_t)sizeof(T);
  }
  __device__ __forceinline__ uint32_t lane_bytes_h(int lhi, int l32) const { return ((uint32_t)(4 * lhi) * N + l32) * 4u; }
  __device__ __forceinline__ float get(size_t u, uint32_t lbh) const {
    return *reinterpret_cast<const float *>(reinterpret_cast<const char *>(h + u) + lbh);
  }
  // row j of the list is written where it is (no scatter)
  __device__ __forceinline__ void put(size_t u, uint32_t lb, float acc, float hv) const {
    *reinterpret_cast<T *>(reinterpret_cast<char *>(out + u) + lb) = from_f<T>(hv + acc);
  }
  // scatter: start of the lane's run in row `row` (column n), then blocks of 32 columns
  __device__ __forceinline__ T *row_ptr(int row, int n) const { return out + (size_t)row * N + n; }
};

template <typename T, int HALF> struct EpiSwiGLUHalves {
  static constexpr bool DUAL = false;
  static constexpr int INTERLEAVE = HALF;  // 48 (96-column tiles) or 64 (128-column tiles)
  static constexpr bool PRELOAD = false;
  T *act;  // [cap, F]
  int F;
  // f = output column of the FFN's hidden layer
  __device__ __forceinline__ void store(int j, int f, float gate, float up) const {
    const float s = silu_for<T>(gate);
    act[(size_t)j * F + f] = from_f<T>(s * up);
  }
  __device__ __forceinline__ void operator()(int, int, int, float, float) const {}
};

}  // namespace dy
