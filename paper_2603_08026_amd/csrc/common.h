// Shared device helpers of the gfx950 kernels: storage types, wave64 reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dy {

constexpr int WAVE = 64;

typedef uint16_t bf16_t;  // raw bf16 bits

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two floats -> packed bf16 pair (lo in bits 0..15), round to nearest even: one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)(pack_bf16(f, 0.f) & 0xffffu); }

template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v) { return bf2f(v); }

template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return f2bf(v); }

// 16-byte vector of storage elements
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float4 raw;
  __device__ __forceinline__ float get(int i) const { return (&raw.x)[i]; }
  __device__ __forceinline__ void set(int i, float v) { (&raw.x)[i] = v; }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  uint4 raw;
  __device__ __forceinline__ float get(int i) const {
    uint32_t w = (&raw.x)[i >> 1];
    return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
  }
  __device__ __forceinline__ void set(int i, float v) {
    uint32_t b = f2bf(v);
    uint32_t &w = (&raw.x)[i >> 1];
    w = (i & 1) ? ((w & 0x0000ffffu) | (b << 16)) : ((w & 0xffff0000u) | b);
  }
};

template <typename T> __device__ __forceinline__ Vec16<T> ld16(const T *p) {
  Vec16<T> v;
  v.raw = *reinterpret_cast<const decltype(v.raw) *>(p);
  return v;
}
template <typename T> __device__ __forceinline__ void st16(T *p, const Vec16<T> &v) {
  *reinterpret_cast<decltype(v.raw) *>(p) = v.raw;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

// Sum over a workgroup of NT threads (NT multiple of 64, <= 1024); result valid in every thread.
// `red` is LDS scratch of at least NT/64 floats; the call contains barriers.
template <int NT> __device__ __forceinline__ float block_sum(float v, float *red) {
  v = wave_sum(v);
  const int w = threadIdx.x / WAVE, l = threadIdx.x % WAVE;
  __syncthreads();
  if (l == 0) red[w] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NT / WAVE; ++i) s += red[i];
  return s;
}

// Sums of three values over a workgroup in one pass (two barriers); red: 3*NT/64 floats of LDS.
template <int NT>
__device__ __forceinline__ void block_sum3(float &a, float &b, float &c, float *red) {
  a = wave_sum(a); b = wave_sum(b); c = wave_sum(c);
  const int w = threadIdx.x / WAVE, l = threadIdx.x % WAVE;
  __syncthreads();
  if (l == 0) { red[3 * w] = a; red[3 * w + 1] = b; red[3 * w + 2] = c; }
  __syncthreads();
  a = b = c = 0.f;
#pragma unroll
  for (int i = 0; i < NT / WAVE; ++i) { a += red[3 * i]; b += red[3 * i + 1]; c += red[3 * i + 2]; }
}

// Asynchronous global -> LDS copy: lane i moves the 16 bytes at its own global address g to
// LDS[lds_base + 16*i]; lds_base is wave-uniform.  Completion is tracked by vmcnt.
__device__ __forceinline__ void dma16(const void *g, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_base), "v"(g)
               : "memory", "m0");
}

// The same copy with a wave-uniform base address (held in scalar registers) and a 32-bit byte
// offset per lane: no 64-bit vector address arithmetic per copy.
__device__ __forceinline__ void dma16_s(const void *sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_base), "v"(voff), "s"(sbase)
               : "memory", "m0");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// all LDS reads of this wave have returned their data
__device__ __forceinline__ void wait_lgkmcnt0() { asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory"); }

__device__ __forceinline__ uint32_t lds_offset_of(const void *p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

}  // namespace dy
