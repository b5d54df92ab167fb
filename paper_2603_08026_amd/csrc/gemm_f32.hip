// Salient-row GEMMs for the fp32 storage type: C[j,n] = sum_k A[row_j,k] * W[n,k] with fused
// epilogues.  64x64 output tile per workgroup, K staged through LDS in slices of 16, 4x4 outputs
// per thread, plain fp32 FMAs (the fp32 path is the accuracy reference of the library; the bf16
// path has MFMA kernels of its own).  The row count lives on the device: the grid is sized for the
// list's capacity and each workgroup loops over the tiles that exist.
#include "gemm_epilogues.h"
#include "kernels.h"

namespace dy {

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <typename T, typename Epi>
__global__ __launch_bounds__(256) void k_gemm_f32(const T *__restrict__ A, const int32_t *gather,
                                                   int lda, Rows rows, int K, int N, WSeg seg,
                                                   const T *__restrict__ W2, Epi epi) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[TK][TN + 4];
  __shared__ float B2s[Epi::DUAL ? TK : 1][TN + 4];

  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  const int tiles_n = N / TN, tiles_m = (M + TM - 1) / TM;
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  const int lr = tid / 4, lk = (tid % 4) * 4;  // load mapping: row lr of the tile, k offset lk..lk+3

  for (int tile = blockIdx.x; tile < tiles_m * tiles_n; tile += gridDim.x) {
    const int tm = tile / tiles_n, tn = tile % tiles_n;
    const int m0 = tm * TM, n0 = tn * TN;
    // A row of this thread's load slot
    const int jm = m0 + lr;
    const T *arow = nullptr;
    if (jm < M) arow = A + (size_t)(gather ? gather[jm] : jm) * lda;
    // weight row of this thread's load slot, looked up in the stacked weight matrices
    const int nw = n0 + lr;
    const bool in1 = nw >= seg.n_end[0], in2 = nw >= seg.n_end[1];
    const int seg_start = in2 ? seg.n_end[1] : in1 ? seg.n_end[0] : 0;
    const T *wrow = (const T *)(in2 ? seg.w[2] : in1 ? seg.w[1] : seg.w[0]) + (size_t)(nw - seg_start) * K;
    const T *w2row = Epi::DUAL ? W2 + (size_t)(n0 + lr) * K : nullptr;

    float acc[4][4], acc2[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = acc2[i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += TK) {
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        As[lk + i][lr] = arow ? to_f<T>(arow[k0 + lk + i]) : 0.f;
        Bs[lk + i][lr] = to_f<T>(wrow[k0 + lk + i]);
        if (Epi::DUAL) B2s[lk + i][lr] = to_f<T>(w2row[k0 + lk + i]);
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < TK; ++kk) {
        float a[4], b[4], b2[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
        if (Epi::DUAL) {
#pragma unroll
          for (int j = 0; j < 4; ++j) b2[j] = B2s[kk][tx * 4 + j];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            acc[i][j] += a[i] * b[j];
            if (Epi::DUAL) acc2[i][j] += a[i] * b2[j];
          }
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = m0 + ty * 4 + i;
      if (j < M) {
        const int row = rows.idx ? rows.idx[j] : j;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) epi(j, row, n0 + tx * 4 + jj, acc[i][jj], acc2[i][jj]);
      }
    }
  }
}

inline int gemm_grid(int cap, int N) {
  long t = (long)((cap + TM - 1) / TM) * (N / TN);
  if (t < 1) t = 1;
  return (int)(t > 4096 ? 4096 : t);
}

template <typename T, typename Epi>
void run(GemmA A, Rows rows, int K, int N, WSeg seg, const void *w2, Epi epi, hipStream_t s) {
  if (rows.cap <= 0) return;
  k_gemm_f32<T, Epi><<<gemm_grid(rows.cap, N), 256, 0, s>>>((const T *)A.a, A.gather, A.lda, rows, K,
                                                            N, seg, (const T *)w2, epi);
}

}  // namespace

void gemm_f32_raw(DType t, GemmA A, Rows rows, int K, WSeg seg, float *part, hipStream_t s) {
  const int N = seg.n_end[2];
  EpiStoreF32 e{part, N};
  if (t == F32) run<float>(A, rows, K, N, seg, nullptr, e, s);
  else run<bf16_t>(A, rows, K, N, seg, nullptr, e, s);
}

void gemm_f32_swiglu(DType t, GemmA A, Rows rows, int K, int N, const void *w_gate, const void *w_up,
                     void *act, hipStream_t s) {
  if (t == F32) run<float>(A, rows, K, N, wseg_one(w_gate, N), w_up, EpiSwiGLU<float>{(float *)act, N}, s);
  else run<bf16_t>(A, rows, K, N, wseg_one(w_gate, N), w_up, EpiSwiGLU<bf16_t>{(bf16_t *)act, N}, s);
}

void gemm_f32_down(DType t, GemmA A, Rows rows, int K, int N, const void *w_down, const float *h,
                   void *out_cache, hipStream_t s) {
  if (t == F32) run<float>(A, rows, K, N, wseg_one(w_down, N), nullptr, EpiDown<float>{h, (float *)out_cache, N}, s);
  else run<bf16_t>(A, rows, K, N, wseg_one(w_down, N), nullptr, EpiDown<bf16_t>{h, (bf16_t *)out_cache, N}, s);
}

}  // namespace dy
