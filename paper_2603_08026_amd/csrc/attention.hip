// Partial attention: dispatch, key-split choice and the merge of split partial results.
#include "attention_common.h"
#include "compact.h"

namespace dy {

namespace {

// One workgroup per query row, a thread per 16 bytes of the row in the storage type (V = 4 or 8
// neighbouring columns, all of one head).  For every head: M = max_s m_s, l = sum_s l_s e^{m_s - M},
// out = sum_s o_s e^{m_s - M} / l  (the usual merge of online-softmax partials).
// lse (optional) receives log(sum_keys exp(score)) of the row's head: M + log l.
template <int V>
__device__ __forceinline__ void merge_splits(const AttnArgs &a, int j, int c, int D, float (&out)[V],
                                             float *lse = nullptr) {
  const int h = c / a.dh;
  if (a.splits == 1) {  // one partial: nothing to weigh, and one dependent load less
    const float2 ml = *reinterpret_cast<const float2 *>(a.part_ml + ((size_t)j * a.H + h) * 2);
    const float4 *po = reinterpret_cast<const float4 *>(a.part_o + (size_t)j * D + c);
    const float inv = 1.0f / ml.y;
#pragma unroll
    for (int q = 0; q < V / 4; ++q) {
      const float4 o = po[q];
      out[4 * q] = o.x * inv; out[4 * q + 1] = o.y * inv; out[4 * q + 2] = o.z * inv; out[4 * q + 3] = o.w * inv;
    }
    if (lse) *lse = ml.x + __logf(ml.y);
    return;
  }
  float M = -INFINITY;
  for (int s = 0; s < a.splits; ++s) M = fmaxf(M, a.part_ml[(((size_t)s * a.rows.cap + j) * a.H + h) * 2]);
  float l = 0.f;
#pragma unroll
  for (int e = 0; e < V; ++e) out[e] = 0.f;
  for (int s = 0; s < a.splits; ++s) {
    const float2 ml = *reinterpret_cast<const float2 *>(a.part_ml + (((size_t)s * a.rows.cap + j) * a.H + h) * 2);
    const float w = __expf(ml.x - M);
    const float4 *po = reinterpret_cast<const float4 *>(a.part_o + ((size_t)s * a.rows.cap + j) * D + c);
    l += ml.y * w;
#pragma unroll
    for (int q = 0; q < V / 4; ++q) {
      const float4 o = po[q];
      out[4 * q] += o.x * w; out[4 * q + 1] += o.y * w; out[4 * q + 2] += o.z * w; out[4 * q + 3] += o.w * w;
    }
  }
  const float inv = 1.0f / l;
#pragma unroll
  for (int e = 0; e < V; ++e) out[e] *= inv;
  if (lse) *lse = M + __logf(l);
}

constexpr int FIN_NT = 512;  // threads of the merge kernels

template <typename T>
__global__ __launch_bounds__(FIN_NT) void k_attn_combine(AttnArgs a) {
  constexpr int V = Vec16<T>::N;
  const int n = a.rows.count ? min(*a.rows.count, a.rows.cap) : a.rows.cap;
  const int D = a.H * a.dh;
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    T *orow = (T *)a.out + (size_t)j * D;
    const int r = a.rows.idx ? a.rows.idx[j] : j;
    for (int c = threadIdx.x * V; c < D; c += FIN_NT * V) {
      float o[V], lse;
      merge_splits<V>(a, j, c, D, o, &lse);
      if (a.lse_out && c % a.dh == 0) a.lse_out[(size_t)r * a.H + c / a.dh] = lse;
      Vec16<T> v;
#pragma unroll
      for (int e = 0; e < V; ++e) v.set(e, o[e]);
      st16(orow + c, v);
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
__global__ __launch_bounds__(FIN_NT) void k_attn_finalize(AttnArgs a, T *c_cache, float tau,
                                                          float *__restrict__ cos_out, uint8_t *flag_out,
                                                          CompactOut co) {
  constexpr int V = Vec16<T>::N;
  __shared__ float red[3 * FIN_NT / WAVE];
  __shared__ int wave_cnt[FIN_NT / WAVE];
  __shared__ int is_last;
  const int n = a.rows.count ? min(*a.rows.count, a.rows.cap) : a.rows.cap;
  const int D = a.H * a.dh;
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    const int r = a.rows.idx ? a.rows.idx[j] : j;
    T *crow = c_cache + (size_t)r * D;
    float dot = 0.f, na = 0.f, nb = 0.f;
    for (int c = threadIdx.x * V; c < D; c += FIN_NT * V) {
      float o[V], lse;
      merge_splits<V>(a, j, c, D, o, &lse);
      if (a.lse_out && c % a.dh == 0) a.lse_out[(size_t)r * a.H + c / a.dh] = lse;
      const Vec16<T> old = ld16(crow + c);
      Vec16<T> nw;
#pragma unroll
      for (int e = 0; e < V; ++e) nw.set(e, o[e]);
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const float f = nw.get(e), b = old.get(e);  // the stored (rounded) values
        dot += f * b;
        na += f * f;
        nb += b * b;
      }
      st16(crow + c, nw);
    }
    block_sum3<FIN_NT>(dot, na, nb, red);
    if (threadIdx.x == 0) {
      const float s = dot / (fmaxf(sqrtf(na), 1e-8f) * fmaxf(sqrtf(nb), 1e-8f));
      if (cos_out) cos_out[j] = s;
      // device-scope store: written through, so that the compacting workgroup sees it without any
      // cache flush (a release fence per workgroup would write back the whole L2 each time)
      __hip_atomic_store(flag_out + j, (uint8_t)((s < tau) ? 1 : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  // flags of this workgroup are out (thread 0 wrote them); count finished workgroups
  if (threadIdx.x == 0) {
    wait_vmcnt<0>();  // the flag stores have been acknowledged
    const int done = __hip_atomic_fetch_add(co.counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    is_last = (done == (int)gridDim.x - 1);
    if (is_last)  // ready for the next launch on the stream
      __hip_atomic_store(co.counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (is_last) {
    compact_block<FIN_NT>(flag_out, a.rows, n, co.B, co.L, co.idx, co.off, co.cap, co.status, co.overflow_code,
                  true, wave_cnt);
  }
}

}  // namespace

void launch_attn_combine(DType t, const AttnArgs &a, hipStream_t s) {
  int grid = a.rows.cap > 8192 ? 8192 : a.rows.cap;
  if (grid < 1) return;
  if (t == F32) k_attn_combine<float><<<grid, FIN_NT, 0, s>>>(a);
  else k_attn_combine<bf16_t><<<grid, FIN_NT, 0, s>>>(a);
}

void launch_attn_finalize(DType t, const AttnArgs &a, void *c_cache, float tau, float *cos_out,
                          uint8_t *flag_out, int32_t *out_idx, int32_t *out_offsets, int out_cap,
                          int32_t *status, int32_t *counter, hipStream_t s) {
  // an empty list still needs its offsets written: one workgroup runs the (empty) compaction
  int grid = a.rows.cap > 8192 ? 8192 : a.rows.cap;
  if (grid < 1) grid = 1;
  CompactOut co{out_idx, out_offsets, status, counter, out_cap, a.B, a.L, -6};
  if (t == F32)
    k_attn_finalize<float><<<grid, FIN_NT, 0, s>>>(a, (float *)c_cache, tau, cos_out, flag_out, co);
  else
    k_attn_finalize<bf16_t><<<grid, FIN_NT, 0, s>>>(a, (bf16_t *)c_cache, tau, cos_out, flag_out, co);
}

// Query tile and key splits: enough workgroups to cover the chip once when there are few
// (sequence, head, query tile) triples; the splits' partials cost HBM traffic and a merge, so no more
// than that.  Bounded by the partial buffer and by one key tile per split.
void attention_plan(DType t, int B, int L, int H, int dh, int cap, int rows_per_seq, size_t part_elems,
                    AttnArgs *a, int grouped_heads) {
  const int BK = (t == F32) ? 64 : 128;
  const int n_opt = (t == F32) ? 1 : 2;
  const int bq_opt[2] = {(t == F32) ? 16 : 128, 64};
  // Few rows: the kernel is latency-bound and every extra key split costs the merge kernel a read of
  // one more partial result, so half the CUs' worth of workgroups is the aim (measured at 106 rows of
  // one sequence, 32 heads: 64-row tiles x 2 splits 13.2 + 6.0 us for attention + merge, 128-row
  // tiles x 8 splits 13.9 + 8.9 us), and 128-row tiles are taken only when they alone reach it.
  // Once 128-row tiles alone fill the chip (two workgroups per CU) they are taken at any row count:
  // waves without a query skip the products, and the 64-row kernel holds one workgroup per CU only
  // (measured at about 66 rows in each of 16 sequences, 32 heads: 72 us against 116 us).
  // The head_dim-128 bf16 kernel folds the query heads of a KV group into the rows of a tile: its
  // tiles are counted over rows x group per KV head.
  const long target = 128;
  const int Hkv = H / (grouped_heads > 0 ? grouped_heads : 1);
  const bool grouped = (t != F32) && dh == 128 && grouped_heads > 1;
  const long rows_t = grouped ? (long)rows_per_seq * grouped_heads : rows_per_seq;  // packed rows per sequence
  const long heads_t = grouped ? Hkv : H;
  const long tiles128 = ((rows_t + 127) / 128) * B * heads_t;
  const int best_bq = (n_opt == 1) ? bq_opt[0]
                                   : ((rows_t > 80 && tiles128 >= target) || tiles128 >= 2 * 256 ? 128 : 64);
  long tiles = ((rows_t + best_bq - 1) / best_bq) * B * heads_t;
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
