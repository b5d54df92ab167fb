// bf16 salient-row GEMM kernel for the gfx950 matrix cores:  C[j,n] = sum_k A[row_j,k] * W[n,k].
//
// Both operands are K-contiguous ([M,K] activations, [N,K] weights), which is exactly what
// v_mfma_f32_32x32x16_bf16 wants: lane l feeds 8 consecutive k of row (l % 32) for A and of
// column (l % 32) for B, k offset 8*(l/32).  A workgroup of 4 waves owns a BM x BN output tile
// (x2 matrices for the fused gate/up GEMM), streams K in slices of 64 through a double-buffered,
// padded LDS tile (row stride 72 elements: the 16-byte operand reads of 8 neighbouring lanes fall
// into 32 distinct banks), prefetching the next slice into registers while the MFMAs of the
// current one run.  The fp32 accumulator block of a wave is laid out as
//   row = 8*(r/4) + 4*(l/32) + (r%4),  col = l%32   for register r = 0..15 of lane l.
//
// The row count M lives on the device.  The grid is sized from the list capacity; workgroups
// walk the existing tiles in a grouped order (GROUP_M row tiles x all column tiles) after a
// remap that keeps neighbouring tiles on one XCD (workgroup i runs on XCD i % 8), so that the A
// tiles and weight tiles a group shares stay in that XCD's L2.
//
// Two tile shapes: a large one for the MFMA-bound regime (hundreds of rows or more) and a skinny
// one (all rows in one 128-row tile, narrow column tiles, optional split of K) for the
// weight-streaming-bound regime of a few dozen rows.
#pragma once
#include "gemm_epilogues.h"
#include "kernels.h"

namespace dy {
namespace mm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int NT = 256;    // threads per workgroup
constexpr int BK = 64;     // K slice
constexpr int LDK = BK + 8;  // padded LDS row stride (elements)
constexpr int N_XCD = 8;

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, bool DUAL_> struct Shape {
  static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr bool DUAL = DUAL_;
  static constexpr int NMAT = DUAL ? 2 : 1;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int MB = WM / 32, NB = WN / 32;
  static constexpr int A_CH = BM * BK / 8 / NT;  // 16-byte chunks per thread and slice
  static constexpr int B_CH = BN * BK / 8 / NT;
  static constexpr int STAGE = (BM + NMAT * BN) * LDK;  // elements per LDS stage
  static constexpr size_t LDS_BYTES = (size_t)2 * STAGE * sizeof(bf16_t);
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 blocks");
  static_assert(A_CH >= 1 && B_CH >= 1, "tile too small for the load mapping");
};

struct SplitStore {  // epilogue of a K-split: fp32 partial tile part[z][j][n]
  float *part;
  size_t split_stride;
  int N;
};

// One K slice, global -> registers: A_CH + NMAT*B_CH 16-byte chunks per thread.
template <typename SH>
__device__ __forceinline__ void load_slice(uint4 (&ra)[SH::A_CH], uint4 (&rb)[SH::NMAT][SH::B_CH],
                                           const bf16_t *const (&ap)[SH::A_CH], const bf16_t *wbase,
                                           const bf16_t *w2base, int ldw, int ko, int tid) {
#pragma unroll
  for (int i = 0; i < SH::A_CH; ++i) ra[i] = *reinterpret_cast<const uint4 *>(ap[i] + ko);
#pragma unroll
  for (int i = 0; i < SH::B_CH; ++i) {
    const int c = tid + NT * i;
    const size_t off = (size_t)(c / 8) * ldw + (c % 8) * 8 + ko;
    rb[0][i] = *reinterpret_cast<const uint4 *>(wbase + off);
    if (SH::DUAL) rb[SH::NMAT - 1][i] = *reinterpret_cast<const uint4 *>(w2base + off);
  }
}

// registers -> one LDS stage ([BM + NMAT*BN] rows of LDK elements)
template <typename SH>
__device__ __forceinline__ void store_slice(const uint4 (&ra)[SH::A_CH],
                                            const uint4 (&rb)[SH::NMAT][SH::B_CH], bf16_t *stage, int tid) {
  bf16_t *sb = stage + SH::BM * LDK;
#pragma unroll
  for (int i = 0; i < SH::A_CH; ++i) {
    const int c = tid + NT * i;
    *reinterpret_cast<uint4 *>(stage + (c / 8) * LDK + (c % 8) * 8) = ra[i];
  }
#pragma unroll
  for (int t = 0; t < SH::NMAT; ++t)
#pragma unroll
    for (int i = 0; i < SH::B_CH; ++i) {
      const int c = tid + NT * i;
      *reinterpret_cast<uint4 *>(sb + t * SH::BN * LDK + (c / 8) * LDK + (c % 8) * 8) = rb[t][i];
    }
}

// MFMAs of one LDS stage for this wave's tile
template <typename SH>
__device__ __forceinline__ void mma_slice(floatx16 (&acc)[SH::NMAT][SH::MB][SH::NB], const bf16_t *stage,
                                          int wm0, int wn0, int l32, int lhi) {
  const bf16_t *sa = stage + (wm0 + l32) * LDK + lhi * 8;
  const bf16_t *sb = stage + SH::BM * LDK + (wn0 + l32) * LDK + lhi * 8;
#pragma unroll
  for (int kk = 0; kk < BK / 16; ++kk) {
    bf16x8 af[SH::MB], bfr[SH::NMAT][SH::NB];
#pragma unroll
    for (int i = 0; i < SH::MB; ++i) af[i] = *reinterpret_cast<const bf16x8 *>(sa + i * 32 * LDK + kk * 16);
#pragma unroll
    for (int t = 0; t < SH::NMAT; ++t)
#pragma unroll
      for (int j = 0; j < SH::NB; ++j)
        bfr[t][j] = *reinterpret_cast<const bf16x8 *>(sb + t * SH::BN * LDK + j * 32 * LDK + kk * 16);
#pragma unroll
    for (int t = 0; t < SH::NMAT; ++t)
#pragma unroll
      for (int i = 0; i < SH::MB; ++i)
#pragma unroll
        for (int j = 0; j < SH::NB; ++j)
          acc[t][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[t][j], acc[t][i][j], 0, 0, 0);
  }
}

template <typename SH, typename Epi>
__global__ __launch_bounds__(NT) void k_gemm_bf16(const bf16_t *__restrict__ A,
                                                   const int32_t *__restrict__ gather, int lda,
                                                   Rows rows, int N, WSeg seg,
                                                   const bf16_t *__restrict__ W2, int ldw, int kchunk,
                                                   int group_m, Epi epi, SplitStore split) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *smem = reinterpret_cast<bf16_t *>(smem_raw);
  constexpr int BM = SH::BM, BN = SH::BN, MB = SH::MB, NB = SH::NB, NMAT = SH::NMAT;

  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
  const int total = tiles_m * tiles_n;
  const int tid = threadIdx.x, lane = tid % WAVE, wave = tid / WAVE;
  const int wm0 = (wave / SH::WAVES_N) * SH::WM, wn0 = (wave % SH::WAVES_N) * SH::WN;
  const int l32 = lane % 32, lhi = lane / 32;
  const int z = blockIdx.y;  // K split
  const int kbeg = z * kchunk;
  const int KT = kchunk / BK;

  // XCD-aware walk: position p of the padded tile sequence is worked by workgroup p % grid; map it
  // to a logical tile so that one XCD (p % 8) gets a contiguous range of logical tiles.
  const int per_xcd = (total + N_XCD - 1) / N_XCD;
  const int total_pad = per_xcd * N_XCD;

  for (int p = blockIdx.x; p < total_pad; p += gridDim.x) {
    const int logical = (p % N_XCD) * per_xcd + p / N_XCD;
    if (logical >= total) continue;  // uniform for the workgroup
    // grouped order: group_m row tiles share a sweep over all column tiles
    const int gsz = group_m * tiles_n;
    const int g = logical / gsz, r = logical % gsz;
    const int gm = min(group_m, tiles_m - g * group_m);
    const int tm = g * group_m + r % gm, tn = r / gm;
    const int m0 = tm * BM, n0 = tn * BN;

    // per-thread source pointers of the 16-byte chunks it moves every slice
    const bf16_t *ap[SH::A_CH];
#pragma unroll
    for (int i = 0; i < SH::A_CH; ++i) {
      const int c = tid + NT * i;
      int j = m0 + c / 8;
      j = j < M ? j : M - 1;  // rows past the end are clamped; their results are never stored
      const int src = gather ? gather[j] : j;
      ap[i] = A + (size_t)src * lda + kbeg + (c % 8) * 8;
    }
    int sg = 0;
    while (sg < 2 && n0 >= seg.n_end[sg]) ++sg;
    const int seg_start = sg ? seg.n_end[sg - 1] : 0;
    const bf16_t *wbase = (const bf16_t *)seg.w[sg] + (size_t)(n0 - seg_start) * ldw + kbeg;
    const bf16_t *w2base = SH::DUAL ? W2 + (size_t)n0 * ldw + kbeg : nullptr;

    floatx16 acc[NMAT][MB][NB];
#pragma unroll
    for (int t = 0; t < NMAT; ++t)
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[t][i][j][e] = 0.f;

    uint4 ra[SH::A_CH], rb[NMAT][SH::B_CH];
    __syncthreads();  // LDS free (previous tile of this workgroup fully consumed)
    load_slice<SH>(ra, rb, ap, wbase, w2base, ldw, 0, tid);
    store_slice<SH>(ra, rb, smem, tid);
    __syncthreads();
    for (int kt = 0; kt + 1 < KT; ++kt) {
      const int cur = kt & 1;
      load_slice<SH>(ra, rb, ap, wbase, w2base, ldw, (kt + 1) * BK, tid);
      mma_slice<SH>(acc, smem + cur * SH::STAGE, wm0, wn0, l32, lhi);
      store_slice<SH>(ra, rb, smem + (cur ^ 1) * SH::STAGE, tid);
      __syncthreads();
    }
    mma_slice<SH>(acc, smem + ((KT - 1) & 1) * SH::STAGE, wm0, wn0, l32, lhi);

    // epilogue
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int j = m0 + wm0 + i * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
        if (j < M) {
          if (split.part) {
#pragma unroll
            for (int jn = 0; jn < NB; ++jn)
              split.part[(size_t)z * split.split_stride + (size_t)j * split.N + n0 + wn0 + jn * 32 + l32] =
                  acc[0][i][jn][e];
          } else {
            const int row = rows.idx ? rows.idx[j] : j;
#pragma unroll
            for (int jn = 0; jn < NB; ++jn)
              epi(j, row, n0 + wn0 + jn * 32 + l32, acc[0][i][jn][e], acc[NMAT - 1][i][jn][e]);
          }
        }
      }
  }
}

// Sum of K-split partials, then the real epilogue, one thread per output element.
template <typename Epi>
__global__ __launch_bounds__(NT) void k_split_reduce(SplitStore split, int splits, Rows rows, Epi epi) {
  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  const size_t total = (size_t)M * split.N;
  for (size_t e = (size_t)blockIdx.x * NT + threadIdx.x; e < total; e += (size_t)gridDim.x * NT) {
    const int j = (int)(e / split.N), n = (int)(e % split.N);
    float s = 0.f;
    for (int z = 0; z < splits; ++z) s += split.part[(size_t)z * split.split_stride + e];
    epi(j, rows.idx ? rows.idx[j] : j, n, s, 0.f);
  }
}

inline WSeg one(const void *w, int N) {
  WSeg s;
  s.w[0] = s.w[1] = s.w[2] = w;
  s.n_end[0] = s.n_end[1] = s.n_end[2] = N;
  return s;
}

template <typename SH, typename Epi> void set_lds_once() {
  static bool done = false;
  if (!done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_bf16<SH, Epi>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::LDS_BYTES);
    done = true;
  }
}


}  // namespace mm
}  // namespace dy
