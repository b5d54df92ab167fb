// Partial (row-sparse) attention, fp32 arithmetic: exact attention rows for the salient queries
// against all keys/values of their sequence, no mask.  [Sec. 3.3 salient path; Alg. 3: C_sal]
//
// Flash-style: a workgroup owns BQ query rows of one (sequence, head) and streams the keys in
// tiles of BK through LDS with an online softmax.  The key range can be split over several
// workgroups (few query rows, small batch); partial (max, sum, un-normalised output) triples are
// merged by k_attn_combine.  This file serves the fp32 storage type; the bf16 type has an MFMA
// kernel of its own and shares only the combine kernel and the tile-to-sequence mapping.
#include "attention_common.h"

namespace dy {

namespace {

template <int DH> struct F32Tile {
  static constexpr int BQ = 16, BK = 32, NT = 256;
  static constexpr int OPT = DH / 16;  // output columns per thread
};

template <typename T, int DH>
__global__ __launch_bounds__(256) void k_attn_f32(AttnArgs a) {
  using TL = F32Tile<DH>;
  constexpr int BQ = TL::BQ, BK = TL::BK, OPT = TL::OPT;
  __shared__ float Qs[BQ][DH];
  __shared__ float Ks[BK][DH + 1];
  __shared__ float Vs[BK][DH];
  __shared__ float Ps[BQ][BK + 1];
  __shared__ int tile_info[3];

  const int tid = threadIdx.x;
  if (tid == 0) find_tile(a, BQ, blockIdx.x, tile_info);
  __syncthreads();
  const int b = tile_info[0];
  if (b < 0) return;  // uniform: no such tile
  const int j0 = tile_info[1], nq = tile_info[2];
  const int h = blockIdx.y, kvh = h / (a.H / a.Hkv), split = blockIdx.z;
  const int kbase = a.key_offsets ? a.key_offsets[b] : b * a.L;
  const int Lk = a.key_offsets ? a.key_offsets[b + 1] - kbase : a.L;
  const int k_lo = split * a.chunk, k_hi = min(Lk, k_lo + a.chunk);
  if (k_lo >= k_hi) return;  // uniform

  const T *q = (const T *)a.q;
  const T *kc = (const T *)a.k + ((size_t)kbase * a.Hkv + kvh) * DH;
  const T *vc = (const T *)a.v + ((size_t)kbase * a.Hkv + kvh) * DH;
  const size_t kv_stride = (size_t)a.Hkv * DH;
  const float scale = 1.0f / sqrtf((float)DH);

  for (int e = tid; e < BQ * DH; e += 256) {
    const int r = e / DH, c = e % DH;
    const size_t qrow = (r < nq) ? (a.q_by_token ? (size_t)a.rows.idx[j0 + r] : (size_t)(j0 + r)) : 0;
    Qs[r][c] = (r < nq) ? to_f<T>(q[(qrow * a.H + h) * DH + c]) * scale : 0.f;
  }

  const int row = tid / 16, sub = tid % 16;
  float o[OPT];
#pragma unroll
  for (int i = 0; i < OPT; ++i) o[i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  for (int k0 = k_lo; k0 < k_hi; k0 += BK) {
    __syncthreads();  // previous tile fully consumed (also orders the Qs fill)
    for (int e = tid; e < BK * DH; e += 256) {
      const int r = e / DH, c = e % DH;
      const bool ok = (k0 + r) < k_hi;
      Ks[r][c] = ok ? to_f<T>(kc[(size_t)(k0 + r) * kv_stride + c]) : 0.f;
      Vs[r][c] = ok ? to_f<T>(vc[(size_t)(k0 + r) * kv_stride + c]) : 0.f;
    }
    __syncthreads();
    float s0 = 0.f, s1 = 0.f;
#pragma unroll 8
    for (int e = 0; e < DH; ++e) {
      const float qv = Qs[row][e];
      s0 += qv * Ks[sub][e];
      s1 += qv * Ks[sub + 16][e];
    }
    if (k0 + sub >= k_hi) s0 = -INFINITY;
    if (k0 + sub + 16 >= k_hi) s1 = -INFINITY;
    float mt = fmaxf(s0, s1);
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) mt = fmaxf(mt, __shfl_xor(mt, off, 16));
    const float m_new = fmaxf(m_run, mt);  // finite: every tile holds at least one valid key
    const float corr = __expf(m_run - m_new);
    const float p0 = __expf(s0 - m_new), p1 = __expf(s1 - m_new);
    float ps = p0 + p1;
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) ps += __shfl_xor(ps, off, 16);
    l_run = l_run * corr + ps;
    m_run = m_new;
    Ps[row][sub] = p0;
    Ps[row][sub + 16] = p1;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < OPT; ++i) o[i] *= corr;
    for (int kk = 0; kk < BK; ++kk) {
      const float p = Ps[row][kk];
#pragma unroll
      for (int i = 0; i < OPT; ++i) o[i] += p * Vs[kk][sub + 16 * i];
    }
  }

  if (row < nq) {
    const int j = j0 + row;
    if (a.splits == 1 && !a.partial) {
      T *out = (T *)a.out + ((size_t)j * a.H + h) * DH;
      const float inv = 1.0f / l_run;
#pragma unroll
      for (int i = 0; i < OPT; ++i) out[sub + 16 * i] = from_f<T>(o[i] * inv);
    } else {
      float *po = a.part_o + (((size_t)split * a.rows.cap + j) * a.H + h) * DH;
#pragma unroll
      for (int i = 0; i < OPT; ++i) po[sub + 16 * i] = o[i];
      if (sub == 0) {
        float *ml = a.part_ml + (((size_t)split * a.rows.cap + j) * a.H + h) * 2;
        ml[0] = m_run;
        ml[1] = l_run;
      }
    }
  }
}

}  // namespace

void launch_attention_f32(DType t, const AttnArgs &a, hipStream_t s) {
  constexpr int BQ = 16;
  dim3 grid(max_q_tiles(a, BQ), a.H, a.splits);
  if (t == F32) {
    if (a.dh == 64) k_attn_f32<float, 64><<<grid, 256, 0, s>>>(a);
    else k_attn_f32<float, 128><<<grid, 256, 0, s>>>(a);
  } else {
    if (a.dh == 64) k_attn_f32<bf16_t, 64><<<grid, 256, 0, s>>>(a);
    else k_attn_f32<bf16_t, 128><<<grid, 256, 0, s>>>(a);
  }
}

}  // namespace dy
