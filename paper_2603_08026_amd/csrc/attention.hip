// Partial attention: dispatch, key-split choice and the merge of split partial results.
#include "attention_common.h"

namespace dy {

namespace {

// One workgroup per query row.  For every head: M = max_s m_s, l = sum_s l_s e^{m_s - M},
// out = sum_s o_s e^{m_s - M} / l  (the usual merge of online-softmax partials).
template <typename T>
__global__ __launch_bounds__(256) void k_attn_combine(AttnArgs a) {
  const int n = a.rows.count ? min(*a.rows.count, a.rows.cap) : a.rows.cap;
  const int D = a.H * a.dh;
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    for (int c = threadIdx.x; c < D; c += 256) {
      const int h = c / a.dh;
      float M = -INFINITY;
      for (int s = 0; s < a.splits; ++s)
        M = fmaxf(M, a.part_ml[(((size_t)s * a.rows.cap + j) * a.H + h) * 2]);
      float l = 0.f, acc = 0.f;
      for (int s = 0; s < a.splits; ++s) {
        const float *ml = a.part_ml + (((size_t)s * a.rows.cap + j) * a.H + h) * 2;
        const float wgt = __expf(ml[0] - M);
        l += ml[1] * wgt;
        acc += a.part_o[((size_t)s * a.rows.cap + j) * D + c] * wgt;
      }
      ((T *)a.out)[(size_t)j * D + c] = from_f<T>(acc / l);
    }
  }
}

}  // namespace

void launch_attn_combine(DType t, const AttnArgs &a, hipStream_t s) {
  int grid = a.rows.cap > 8192 ? 8192 : a.rows.cap;
  if (grid < 1) return;
  if (t == F32) k_attn_combine<float><<<grid, 256, 0, s>>>(a);
  else k_attn_combine<bf16_t><<<grid, 256, 0, s>>>(a);
}

// Splits of the key range: enough workgroups to cover the chip a few times over when there are few
// (sequence, head, query tile) triples, bounded by the partial buffer and by one key tile per split.
void attention_plan(DType t, int B, int L, int H, int dh, int cap, size_t part_elems, int *splits,
                    int *chunk) {
  const int BQ = (t == F32) ? 16 : 64, BK = (t == F32) ? 64 : 128;
  const long tiles = (long)((cap + BQ - 1) / BQ + B) * H;
  int s = (int)((1024 + tiles - 1) / tiles);
  const int max_by_keys = (L + BK - 1) / BK;
  if (s > max_by_keys) s = max_by_keys;
  if (s > 16) s = 16;
  const size_t per_split = (size_t)cap * H * dh;
  if (per_split > 0 && (size_t)s * per_split > part_elems) s = (int)(part_elems / per_split);
  if (s < 1) s = 1;
  const int c = split_chunk(L, s, BK);
  *chunk = c;
  *splits = (L + c - 1) / c;  // drops splits that would be empty
}

void launch_attention(DType t, const AttnArgs &a, hipStream_t s) {
  if (a.rows.cap <= 0) return;
  if (t == F32) launch_attention_f32(t, a, s);
  else launch_attention_bf16(a, s);
  if (a.splits > 1) launch_attn_combine(t, a, s);
}

}  // namespace dy
