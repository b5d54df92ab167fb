// Partial attention: dispatch, key-split choice and the merge of split partial results.
#include "attention_common.h"
#include "compact.h"

namespace dy {

namespace {

// One workgroup per query row, a thread per 4 neighbouring columns (all of one head).  For every
// head: M = max_s m_s, l = sum_s l_s e^{m_s - M}, out = sum_s o_s e^{m_s - M} / l  (the usual merge
// of online-softmax partials).
__device__ __forceinline__ float4 merge_splits(const AttnArgs &a, int j, int c, int D) {
  const int h = c / a.dh;
  float M = -INFINITY;
  for (int s = 0; s < a.splits; ++s) M = fmaxf(M, a.part_ml[(((size_t)s * a.rows.cap + j) * a.H + h) * 2]);
  float l = 0.f;
  float4 acc{0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < a.splits; ++s) {
    const float2 ml = *reinterpret_cast<const float2 *>(a.part_ml + (((size_t)s * a.rows.cap + j) * a.H + h) * 2);
    const float w = __expf(ml.x - M);
    const float4 o = *reinterpret_cast<const float4 *>(a.part_o + ((size_t)s * a.rows.cap + j) * D + c);
    l += ml.y * w;
    acc.x += o.x * w; acc.y += o.y * w; acc.z += o.z * w; acc.w += o.w * w;
  }
  const float inv = 1.0f / l;
  return float4{acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv};
}

template <typename T>
__global__ __launch_bounds__(1024) void k_attn_combine(AttnArgs a) {
  const int n = a.rows.count ? min(*a.rows.count, a.rows.cap) : a.rows.cap;
  const int D = a.H * a.dh;
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    T *orow = (T *)a.out + (size_t)j * D;
    for (int c = threadIdx.x * 4; c < D; c += 4096) {
      const float4 o = merge_splits(a, j, c, D);
      orow[c] = from_f<T>(o.x); orow[c + 1] = from_f<T>(o.y);
      orow[c + 2] = from_f<T>(o.z); orow[c + 3] = from_f<T>(o.w);
    }
  }
}

// Merge of the partials fused with the temporal cosine similarity, the salient test and the context
// commit  [Sec. 3.1, Sec. 3.2; Alg. 3: cosine line and cache commit].  The new context is rounded to
// the storage type first; the cosine is taken over the stored values (so an unchanged context gives
// exactly the cached row and s = 1), the old cache row is read before it is overwritten.
// Tail: the workgroup that finishes last (device counter) compacts the flags of the whole launch
// into the next index list, which saves a launch on a latency-bound step.
struct CompactOut {
  int32_t *idx, *off, *status, *counter;
  int cap, B, L, overflow_code;
};

template <typename T>
__global__ __launch_bounds__(1024) void k_attn_finalize(AttnArgs a, T *c_cache, float tau,
                                                        float *__restrict__ cos_out, uint8_t *flag_out,
                                                        CompactOut co) {
  __shared__ float red[3 * 1024 / WAVE];
  __shared__ int wave_cnt[CB / WAVE];
  __shared__ int is_last;
  const int n = a.rows.count ? min(*a.rows.count, a.rows.cap) : a.rows.cap;
  const int D = a.H * a.dh;
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    const int r = a.rows.idx ? a.rows.idx[j] : j;
    T *crow = c_cache + (size_t)r * D;
    float dot = 0.f, na = 0.f, nb = 0.f;
    for (int c = threadIdx.x * 4; c < D; c += 4096) {
      const float4 o = merge_splits(a, j, c, D);
      const T n0 = from_f<T>(o.x), n1 = from_f<T>(o.y), n2 = from_f<T>(o.z), n3 = from_f<T>(o.w);
      const float f0 = to_f<T>(n0), f1 = to_f<T>(n1), f2 = to_f<T>(n2), f3 = to_f<T>(n3);
      const float b0 = to_f<T>(crow[c]), b1 = to_f<T>(crow[c + 1]), b2 = to_f<T>(crow[c + 2]), b3 = to_f<T>(crow[c + 3]);
      dot += f0 * b0 + f1 * b1 + f2 * b2 + f3 * b3;
      na += f0 * f0 + f1 * f1 + f2 * f2 + f3 * f3;
      nb += b0 * b0 + b1 * b1 + b2 * b2 + b3 * b3;
      crow[c] = n0; crow[c + 1] = n1; crow[c + 2] = n2; crow[c + 3] = n3;
    }
    block_sum3<1024>(dot, na, nb, red);
    if (threadIdx.x == 0) {
      const float s = dot / (fmaxf(sqrtf(na), 1e-8f) * fmaxf(sqrtf(nb), 1e-8f));
      if (cos_out) cos_out[j] = s;
      flag_out[j] = (s < tau) ? 1 : 0;
    }
  }
  // flags of this workgroup are out (thread 0 wrote them); count finished workgroups
  if (threadIdx.x == 0) {
    __threadfence();
    const int done = atomicAdd(co.counter, 1);
    is_last = (done == (int)gridDim.x - 1);
    if (is_last) *co.counter = 0;  // ready for the next launch on the stream
  }
  __syncthreads();
  if (is_last) {
    __threadfence();
    compact_block(flag_out, a.rows, n, co.B, co.L, co.idx, co.off, co.cap, co.status, co.overflow_code,
                  true, wave_cnt);
  }
}

}  // namespace

void launch_attn_combine(DType t, const AttnArgs &a, hipStream_t s) {
  int grid = a.rows.cap > 8192 ? 8192 : a.rows.cap;
  if (grid < 1) return;
  if (t == F32) k_attn_combine<float><<<grid, 1024, 0, s>>>(a);
  else k_attn_combine<bf16_t><<<grid, 1024, 0, s>>>(a);
}

void launch_attn_finalize(DType t, const AttnArgs &a, void *c_cache, float tau, float *cos_out,
                          uint8_t *flag_out, int32_t *out_idx, int32_t *out_offsets, int out_cap,
                          int32_t *status, int32_t *counter, hipStream_t s) {
  // an empty list still needs its offsets written: one workgroup runs the (empty) compaction
  int grid = a.rows.cap > 8192 ? 8192 : a.rows.cap;
  if (grid < 1) grid = 1;
  CompactOut co{out_idx, out_offsets, status, counter, out_cap, a.B, a.L, -6};
  if (t == F32)
    k_attn_finalize<float><<<grid, 1024, 0, s>>>(a, (float *)c_cache, tau, cos_out, flag_out, co);
  else
    k_attn_finalize<bf16_t><<<grid, 1024, 0, s>>>(a, (bf16_t *)c_cache, tau, cos_out, flag_out, co);
}

// Query tile and key splits: enough workgroups to cover the chip once when there are few
// (sequence, head, query tile) triples; the splits' partials cost HBM traffic and a merge, so no more
// than that.  Bounded by the partial buffer and by one key tile per split.
void attention_plan(DType t, int B, int L, int H, int dh, int cap, int rows_per_seq, size_t part_elems,
                    AttnArgs *a) {
  const int BK = (t == F32) ? 64 : 128;
  const int n_opt = (t == F32) ? 1 : 2;
  const int bq_opt[2] = {(t == F32) ? 16 : 128, 64};
  const long target = 256;  // workgroups that cover the 256 CUs once
  // 128-row query tiles when sequences bring that many rows, else 64-row tiles
  const int best_bq = (n_opt == 1) ? bq_opt[0] : (rows_per_seq > 80 ? 128 : 64);
  long tiles = (long)((rows_per_seq + best_bq - 1) / best_bq) * B * H;
  if (tiles < 1) tiles = 1;  // empty list
  const int best_s = (int)((target + tiles - 1) / tiles);
  int s = best_s;
  const int max_by_keys = (L + BK - 1) / BK;
  if (s > max_by_keys) s = max_by_keys;
  if (s > 16) s = 16;
  const size_t per_split = (size_t)cap * H * dh;
  if (per_split > 0 && (size_t)s * per_split > part_elems) s = (int)(part_elems / per_split);
  if (s < 1) s = 1;
  const int c = split_chunk(L, s, BK);
  a->bq = best_bq;
  a->chunk = c;
  a->splits = (L + c - 1) / c;  // drops splits that would be empty
}

void launch_attention(DType t, const AttnArgs &a, hipStream_t s) {
  if (a.rows.cap <= 0) return;
  if (t == F32) launch_attention_f32(t, a, s);
  else launch_attention_bf16(a, s);
  if (a.splits > 1 && !a.partial) launch_attn_combine(t, a, s);
}

}  // namespace dy
