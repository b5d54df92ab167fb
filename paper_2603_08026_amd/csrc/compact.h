// Stream compaction of salient flags into an ascending token list  [Alg. 3: idx_sal <- where(cos < tau)]
// as workgroup-level routines, so that it can run as a kernel of its own (one workgroup, or many
// workgroups chained through a few words of device memory) or as the tail of the kernel that
// produces the flags.
#pragma once
#include "common.h"
#include "kernels.h"

namespace dy {

constexpr int CB = 256;       // threads of a workgroup of the stand-alone compaction kernel
constexpr int CMAXG = 1024;   // most workgroups of one stand-alone launch
static_assert(COMPACT_SCAN_WORDS == 2 + CMAXG, "scan words: ticket, finished count, one word per workgroup");

// sequence of a token id, never past the last sequence (an id outside [0, B*L) must not index past
// offsets[B])
__device__ __forceinline__ int seq_of(int row, int B, int L) {
  const unsigned s = (unsigned)row / (unsigned)L;
  return s < (unsigned)B ? (int)s : B - 1;
}

// One workgroup of NT threads sweeps the flags [lo, hi) in chunks of NT: wave64 ballot + popcount give
// each flagged lane its rank inside the wave, the per-wave totals are combined through LDS.  `base`
// flagged entries precede lo.  The output keeps the input order, so it is ascending.  Per-sequence
// offsets: the first entry of every sequence writes its own exclusive rank for all sequences that
// start at or before it.  `coherent` makes the flag reads bypass the per-CU cache (flags written by
// other workgroups of the same launch).  wave_cnt: LDS scratch of NT/64 ints.  Returns base + the
// number of flagged entries in [lo, hi).
template <int NT>
__device__ __forceinline__ int compact_range(const uint8_t *flag, const Rows &rows, int lo, int hi, int base,
                                             int B, int L, int32_t *out_idx, int32_t *out_off, int out_cap,
                                             bool coherent, int *wave_cnt) {
  const int tid = threadIdx.x, lane = tid % WAVE, w = tid / WAVE;
  for (int start = lo; start < hi; start += NT) {
    const int j = start + tid;
    bool f = false;
    int row = 0, sprev = -1;
    if (j < hi) {
      const uint8_t fv = coherent ? __hip_atomic_load(flag + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                  : flag[j];
      f = fv != 0;
      row = rows.idx ? rows.idx[j] : j;
      if (j > 0) sprev = seq_of(rows.idx ? rows.idx[j - 1] : j - 1, B, L);
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
    if (j < hi) {
      const int p = base + woff + before;  // flagged entries in front of j
      if (f && p < out_cap) out_idx[p] = row;
      const int sj = seq_of(row, B, L);
      for (int b = sprev + 1; b <= sj; ++b) out_off[b] = min(p, out_cap);
    }
    base += tot;
    __syncthreads();
  }
  return base;
}

// After the last entry: the offsets of the sequences behind it (and offsets[B]) take the total; a
// total beyond the capacity is reported.
template <int NT>
__device__ __forceinline__ void compact_tail(const Rows &rows, int n, int total, int B, int L, int32_t *out_off,
                                             int out_cap, int32_t *status, int overflow_code) {
  const int tid = threadIdx.x;
  if (total > out_cap && tid == 0) *status = overflow_code;
  const int s_last = n > 0 ? seq_of(rows.idx ? rows.idx[n - 1] : n - 1, B, L) : -1;
  for (int b = s_last + 1 + tid; b <= B; b += NT) out_off[b] = min(total, out_cap);
}

// The whole list in one workgroup.
template <int NT>
__device__ __forceinline__ void compact_block(const uint8_t *flag, const Rows &rows, int n, int B, int L,
                                              int32_t *out_idx, int32_t *out_off, int out_cap,
                                              int32_t *status, int overflow_code, bool coherent,
                                              int *wave_cnt) {
  const int total = compact_range<NT>(flag, rows, 0, n, 0, B, L, out_idx, out_off, out_cap, coherent, wave_cnt);
  compact_tail<NT>(rows, n, total, B, L, out_off, out_cap, status, overflow_code);
}

}  // namespace dy
