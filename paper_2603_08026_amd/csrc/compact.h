// Stream compaction of salient flags into an ascending token list  [Alg. 3: idx_sal <- where(cos < tau)]
// as a workgroup-level routine, so that it can run as a kernel of its own or as the tail of the
// kernel that produces the flags.
#pragma once
#include "common.h"
#include "kernels.h"

namespace dy {

constexpr int CB = 1024;  // threads of the stand-alone compaction kernel

// One workgroup of NT threads sweeps n flags in chunks of NT: wave64 ballot + popcount give each
// flagged lane its rank inside the wave, the 16 per-wave totals are combined through LDS.  The output
// keeps the input order, so it is ascending.  Per-sequence offsets: the first candidate of every
// sequence writes its own exclusive rank for all sequences that start at or before it.
// `coherent` makes the flag reads bypass the per-CU cache (flags written by other workgroups of the
// same launch).  wave_cnt: LDS scratch of NT/64 ints.
template <int NT>
__device__ __forceinline__ void compact_block(const uint8_t *flag, const Rows &rows, int n, int B, int L,
                                              int32_t *out_idx, int32_t *out_off, int out_cap,
                                              int32_t *status, int overflow_code, bool coherent,
                                              int *wave_cnt) {
  const int tid = threadIdx.x, lane = tid % WAVE, w = tid / WAVE;
  int base = 0;
  for (int start = 0; start < n; start += NT) {
    const int j = start + tid;
    bool f = false;
    int row = 0, sprev = -1;
    if (j < n) {
      const uint8_t fv = coherent ? __hip_atomic_load(flag + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                  : flag[j];
      f = fv != 0;
      row = rows.idx ? rows.idx[j] : j;
      if (j > 0) sprev = (rows.idx ? rows.idx[j - 1] : j - 1) / L;
    }
    const unsigned long long bal = __ballot(f);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wave_cnt[w] = __popcll(bal);
    __syncthreads();
    int woff = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NT / WAVE; ++i) {
      const int c = wave_cnt[i];
      woff += (i < w) ? c : 0;
      tot += c;
    }
    if (j < n) {
      const int p = base + woff + before;  // flagged candidates in front of j
      if (f && p < out_cap) out_idx[p] = row;
      const int sj = row / L;
      for (int b = sprev + 1; b <= sj; ++b) out_off[b] = min(p, out_cap);
    }
    base += tot;
    __syncthreads();
  }
  if (base > out_cap && tid == 0) *status = overflow_code;
  const int s_last = n > 0 ? (rows.idx ? rows.idx[n - 1] : n - 1) / L : -1;
  for (int b = s_last + 1 + tid; b <= B; b += NT) out_off[b] = min(base, out_cap);
}

}  // namespace dy
