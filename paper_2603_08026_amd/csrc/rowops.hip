// Row-wise kernels of the sparse layer step: gather + RMSNorm, rotary embedding + K/V merge,
// cosine saliency (+ context commit), stream compaction.  All are HBM-bound: one workgroup walks
// one token row with 16-byte loads, reductions in fp32.
#include "common.h"
#include "compact.h"
#include "kernels.h"

namespace dy {

namespace {

constexpr int RB = 1024;  // threads per row workgroup: a row of up to 16384 elements in one pass
constexpr int KEEP = 4;   // 16-byte vectors a thread keeps in registers between the two passes of a row

__device__ __forceinline__ int row_count(const Rows &rows) {
  return rows.count ? min(*rows.count, rows.cap) : rows.cap;
}

// ---- gather + RMSNorm  [Alg. 3: layernorm(x) restricted to the salient rows] -------------------
// NT threads per row: 256 when the row fits KEEP vectors per thread (more rows in flight per CU and a
// four-wave reduction), else RB.
template <typename T, int NT>
__global__ __launch_bounds__(NT) void k_gather_rmsnorm(const T *__restrict__ x,
                                                        const T *__restrict__ gain, Rows rows, int d,
                                                        float eps, T *__restrict__ out) {
  __shared__ float red[NT / WAVE];
  constexpr int N = Vec16<T>::N;
  const int n = row_count(rows), nv = d / N;
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    const int r = rows.idx ? rows.idx[j] : j;
    const T *xr = x + (size_t)r * d;
    float ss = 0.f;
    Vec16<T> keep[KEEP];
#pragma unroll
    for (int it = 0; it < KEEP; ++it) {
      const int v = threadIdx.x + it * NT;
      if (v < nv) {
        keep[it] = ld16(xr + v * N);
#pragma unroll
        for (int i = 0; i < N; ++i) ss += keep[it].get(i) * keep[it].get(i);
      }
    }
    ss = block_sum<NT>(ss, red);
    const float sc = 1.0f / sqrtf(ss / (float)d + eps);
    T *orow = out + (size_t)j * d;
#pragma unroll
    for (int it = 0; it < KEEP; ++it) {
      const int v = threadIdx.x + it * NT;
      if (v < nv) {
        Vec16<T> g = ld16(gain + v * N), o;
#pragma unroll
        for (int i = 0; i < N; ++i) o.set(i, keep[it].get(i) * sc * g.get(i));
        st16(orow + v * N, o);
      }
    }
  }
}

// ---- out-projection tail  [Alg. 3: x <- layernorm(out_proj(C)), with the residual] ---------------
// h[j] = x[row_j] + sum_z part[z][j] (kept in fp32 for the second residual), f[j] = RMSNorm(h[j]) * gain
template <typename T>
__global__ __launch_bounds__(RB) void k_oproj_finalize(const float *__restrict__ part, Splits splits_of,
                                                        size_t split_stride, const T *__restrict__ x,
                                                        const T *__restrict__ gain, Rows rows, int d,
                                                        float eps, float *__restrict__ h,
                                                        T *__restrict__ f) {
  __shared__ float red[RB / WAVE];
  const int n = row_count(rows), nv = d / 4;
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    const int r = rows.idx ? rows.idx[j] : j;
    const int splits = splits_of.of(j);
    const T *xr = x + (size_t)r * d;
    float *hr = h + (size_t)j * d;
    float ss = 0.f;
    float4 keep[KEEP];
#pragma unroll
    for (int it = 0; it < KEEP; ++it) {
      const int v = threadIdx.x + it * RB;
      if (v < nv) {
        float4 a = *reinterpret_cast<const float4 *>(part + (size_t)j * d + v * 4);
        for (int z = 1; z < splits; ++z) {
          const float4 b = *reinterpret_cast<const float4 *>(part + z * split_stride + (size_t)j * d + v * 4);
          a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
        }
        a.x += to_f<T>(xr[v * 4 + 0]); a.y += to_f<T>(xr[v * 4 + 1]);
        a.z += to_f<T>(xr[v * 4 + 2]); a.w += to_f<T>(xr[v * 4 + 3]);
        *reinterpret_cast<float4 *>(hr + v * 4) = a;
        ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        keep[it] = a;
      }
    }
    ss = block_sum<RB>(ss, red);
    const float sc = 1.0f / sqrtf(ss / (float)d + eps);
    T *fr = f + (size_t)j * d;
#pragma unroll
    for (int it = 0; it < KEEP; ++it) {
      const int v = threadIdx.x + it * RB;
      if (v < nv) {
        const float4 a = keep[it];
        const T *g = gain + v * 4;
        fr[v * 4 + 0] = from_f<T>(a.x * sc * to_f<T>(g[0]));
        fr[v * 4 + 1] = from_f<T>(a.y * sc * to_f<T>(g[1]));
        fr[v * 4 + 2] = from_f<T>(a.z * sc * to_f<T>(g[2]));
        fr[v * 4 + 3] = from_f<T>(a.w * sc * to_f<T>(g[3]));
      }
    }
  }
}

// ---- down-projection tail after a K split  [Alg. 3: FFN second half + cache commit] ---------------
template <typename T>
__global__ __launch_bounds__(RB) void k_down_finalize(const float *__restrict__ part, Splits splits_of,
                                                       size_t split_stride, const float *__restrict__ h,
                                                       Rows rows, int d, T *__restrict__ out) {
  const int n = row_count(rows), nv = d / 4;
  for (int j = splits_of.done_to + blockIdx.x; j < n; j += gridDim.x) {
    const int r = rows.idx ? rows.idx[j] : j;
    const int splits = splits_of.of(j);
    if (splits == 0) continue;  // the row's result is in place already (its GEMM had no K split)
    T *orow = out + (size_t)r * d;
    for (int v = threadIdx.x; v < nv; v += RB) {
      float4 a = *reinterpret_cast<const float4 *>(h + (size_t)j * d + v * 4);
      for (int z = 0; z < splits; ++z) {
        const float4 b = *reinterpret_cast<const float4 *>(part + z * split_stride + (size_t)j * d + v * 4);
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
      }
      orow[v * 4 + 0] = from_f<T>(a.x); orow[v * 4 + 1] = from_f<T>(a.y);
      orow[v * 4 + 2] = from_f<T>(a.z); orow[v * 4 + 3] = from_f<T>(a.w);
    }
  }
}

// ---- q/k/v tail: bias + rotary embedding + K/V merge  [Alg. 3: K[idx] <- k_proj(x[idx]), same V] --
// Half-split pairing: element p of a head couples with element p + dh/2, rotated by the angle
// pos * theta^(-2p/dh); the table holds (cos, sin) per (pos, p).  A thread handles 4 neighbouring
// pairs of one head (two float4 of the raw result, two float4 of the table).
template <typename T>
__global__ __launch_bounds__(RB) void k_qkv_finalize(const float *__restrict__ part, Splits splits_of,
                                                      size_t split_stride, const float *__restrict__ tab,
                                                      Rows rows, int L, int H, int Hkv, int dh,
                                                      const T *__restrict__ bq, const T *__restrict__ bk,
                                                      const T *__restrict__ bv, T *__restrict__ q_out,
                                                      T *__restrict__ kc, T *__restrict__ vc,
                                                      T *__restrict__ dv_out, int q_by_token,
                                                      T *__restrict__ ksal_out, int dv_by_entry,
                                                      int32_t *__restrict__ entry_of, int entry_lo) {
  const int n = row_count(rows);
  const int half = dh / 2, dq = H * dh, dkv = Hkv * dh, ld = dq + 2 * dkv;
  const int per_head = half / 4;  // items of 4 pairs per head
  const int qk_items = (H + Hkv) * per_head, v_items = dkv / 4;
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    const int r = rows.idx ? rows.idx[j] : j;
    const int splits = splits_of.of(j);
    const int pos = r % L;
    // token -> its list entry (0 = not in the list), for the tokens at positions >= entry_lo only
    if (entry_of && threadIdx.x == 0 && pos >= entry_lo) entry_of[r] = j + 1;
    const float *src = part + (size_t)j * ld;
    const float *t = tab + (size_t)pos * half * 2;
    for (int it = threadIdx.x; it < qk_items + v_items; it += RB) {
      if (it < qk_items) {
        const int head = it / per_head, p4 = (it % per_head) * 4;
        const bool isq = head < H;
        const int hh = isq ? head : head - H;
        const int c0 = hh * dh + p4;              // column inside q or k
        const int s0 = (isq ? 0 : dq) + c0;       // column inside the raw row
        float4 x1 = *reinterpret_cast<const float4 *>(src + s0);
        float4 x2 = *reinterpret_cast<const float4 *>(src + s0 + half);
        for (int z = 1; z < splits; ++z) {
          const float4 y1 = *reinterpret_cast<const float4 *>(src + z * split_stride + s0);
          const float4 y2 = *reinterpret_cast<const float4 *>(src + z * split_stride + s0 + half);
          x1.x += y1.x; x1.y += y1.y; x1.z += y1.z; x1.w += y1.w;
          x2.x += y2.x; x2.y += y2.y; x2.z += y2.z; x2.w += y2.w;
        }
        const T *b = isq ? bq : bk;
        if (b) {
          x1.x += to_f<T>(b[c0]); x1.y += to_f<T>(b[c0 + 1]); x1.z += to_f<T>(b[c0 + 2]); x1.w += to_f<T>(b[c0 + 3]);
          x2.x += to_f<T>(b[c0 + half]); x2.y += to_f<T>(b[c0 + half + 1]);
          x2.z += to_f<T>(b[c0 + half + 2]); x2.w += to_f<T>(b[c0 + half + 3]);
        }
        const float4 t0 = *reinterpret_cast<const float4 *>(t + 2 * p4);      // cos0 sin0 cos1 sin1
        const float4 t1 = *reinterpret_cast<const float4 *>(t + 2 * p4 + 4);  // cos2 sin2 cos3 sin3
        T *dst = isq ? q_out + (size_t)(q_by_token ? r : j) * dq : kc + (size_t)r * dkv;
        const T lo4[4] = {from_f<T>(x1.x * t0.x - x2.x * t0.y), from_f<T>(x1.y * t0.z - x2.y * t0.w),
                          from_f<T>(x1.z * t1.x - x2.z * t1.y), from_f<T>(x1.w * t1.z - x2.w * t1.w)};
        const T hi4[4] = {from_f<T>(x2.x * t0.x + x1.x * t0.y), from_f<T>(x2.y * t0.z + x1.y * t0.w),
                          from_f<T>(x2.z * t1.x + x1.z * t1.y), from_f<T>(x2.w * t1.z + x1.w * t1.w)};
        // (the new key row also goes to a compact copy when the approximate pass scores candidates only)
        T *ks = (!isq && ksal_out) ? ksal_out + (size_t)j * dkv : nullptr;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          dst[c0 + u] = lo4[u];
          dst[c0 + half + u] = hi4[u];
          if (ks) {
            ks[c0 + u] = lo4[u];
            ks[c0 + half + u] = hi4[u];
          }
        }
      } else {
        const int c0 = (it - qk_items) * 4;
        float4 x = *reinterpret_cast<const float4 *>(src + dq + dkv + c0);
        for (int z = 1; z < splits; ++z) {
          const float4 y = *reinterpret_cast<const float4 *>(src + z * split_stride + dq + dkv + c0);
          x.x += y.x; x.y += y.y; x.z += y.z; x.w += y.w;
        }
        if (bv) {
          x.x += to_f<T>(bv[c0]); x.y += to_f<T>(bv[c0 + 1]); x.z += to_f<T>(bv[c0 + 2]); x.w += to_f<T>(bv[c0 + 3]);
        }
        T *vrow = vc + (size_t)r * dkv + c0;
        const T n0 = from_f<T>(x.x), n1 = from_f<T>(x.y), n2 = from_f<T>(x.z), n3 = from_f<T>(x.w);
        if (dv_out) {  // residual of the stored values, before the merge overwrites the cached row
          T *d = dv_out + (size_t)(dv_by_entry ? j : r) * dkv + c0;
          d[0] = from_f<T>(to_f<T>(n0) - to_f<T>(vrow[0])); d[1] = from_f<T>(to_f<T>(n1) - to_f<T>(vrow[1]));
          d[2] = from_f<T>(to_f<T>(n2) - to_f<T>(vrow[2])); d[3] = from_f<T>(to_f<T>(n3) - to_f<T>(vrow[3]));
        }
        vrow[0] = n0; vrow[1] = n1; vrow[2] = n2; vrow[3] = n3;
      }
    }
  }
}

// ---- temporal cosine similarity + salient test (+ commit)  [Sec. 3.1, Sec. 3.2] ----------------
// s = <a,b> / (max(|a|,1e-8) max(|b|,1e-8)), flag = s < tau.  The old cache row b is read before
// the same thread overwrites the same elements with a.
constexpr int SAL_NT = 256;  // a row per workgroup: many small workgroups keep the loads of a CU in flight

template <typename T>
__global__ __launch_bounds__(SAL_NT) void k_saliency(const T *__restrict__ c_new, T *c_cache, Rows rows,
                                                      int D, float tau, float *__restrict__ cos_out,
                                                      uint8_t *__restrict__ flag_out, int commit) {
  __shared__ float red[3 * SAL_NT / WAVE];
  constexpr int N = Vec16<T>::N;
  const int n = row_count(rows), nv = D / N;
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    const int r = rows.idx ? rows.idx[j] : j;
    const T *a = c_new + (size_t)j * D;
    T *b = c_cache + (size_t)r * D;
    float dot = 0.f, na = 0.f, nb = 0.f;
    for (int v = threadIdx.x; v < nv; v += SAL_NT) {
      Vec16<T> va = ld16(a + v * N), vb = ld16(b + v * N);
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const float fa = va.get(i), fb = vb.get(i);
        dot += fa * fb;
        na += fa * fa;
        nb += fb * fb;
      }
      if (commit) st16(b + v * N, va);
    }
    block_sum3<SAL_NT>(dot, na, nb, red);
    if (threadIdx.x == 0) {
      const float s = dot / (fmaxf(sqrtf(na), 1e-8f) * fmaxf(sqrtf(nb), 1e-8f));
      if (cos_out) cos_out[j] = s;
      flag_out[j] = (s < tau) ? 1 : 0;
    }
  }
}

// ---- stream compaction as a kernel of its own ------------------------------------------------------
// Workgroup i takes entries [i*chunk, (i+1)*chunk) of the list.  It counts its flagged entries,
// publishes the count, adds up the counts of the chunks before it, and then places its own entries.
// scan (COMPACT_SCAN_WORDS ints, all zero before and after a launch): [0] a ticket counter that numbers the
// workgroups in the order they start, [1] finished workgroups, [2 + i] 1 + count of chunk i once
// published.  Every workgroup publishes BEFORE it waits, and it only waits for tickets lower than its
// own, whose workgroups are already running: every wait ends.  The workgroup that finishes last puts
// the words back to zero for the next launch.  Launches that share `scan` must not overlap.
// FROM_PARTS: the flags do not exist yet; a thread first takes the cosine of each of its entries from
// the per-head sums the attention kernel left (cos_part [n, H, 4]: <new, old>, |new|^2, |old|^2), writes
// cos_out and the flag, and then counts and places the flags it wrote itself.
struct CosParts {
  const float *part;
  float *cos_out;
  uint8_t *flag_out;
  int H;
  float tau;
};

template <bool FROM_PARTS>
__global__ __launch_bounds__(CB) void k_compact(const uint8_t *__restrict__ flag, Rows rows, int B, int L,
                                                 int chunk, int32_t *out_idx, int32_t *out_off, int out_cap,
                                                 int32_t *status, int overflow_code, int32_t *scan, CosParts cp) {
  __shared__ int wave_cnt[CB / WAVE];
  __shared__ int s_bid, s_last;
  const int tid = threadIdx.x, lane = tid % WAVE, w = tid / WAVE;
  const int n = row_count(rows);
  const int G = gridDim.x;
  if (tid == 0) s_bid = __hip_atomic_fetch_add(scan, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  const int bid = s_bid;
  const int lo = min(n, bid * chunk), hi = min(n, lo + chunk);
  int mine = 0;  // wave-uniform
  for (int start = lo; start < hi; start += CB) {
    const int j = start + tid;
    bool f = false;
    if (j < hi) {
      if constexpr (FROM_PARTS) {
        const float4 *p = reinterpret_cast<const float4 *>(cp.part) + (size_t)j * cp.H;
        float dot = 0.f, na = 0.f, nb = 0.f;
        for (int h = 0; h < cp.H; ++h) {
          const float4 v = p[h];
          dot += v.x; na += v.y; nb += v.z;
        }
        const float c = dot / (fmaxf(sqrtf(na), 1e-8f) * fmaxf(sqrtf(nb), 1e-8f));
        f = c < cp.tau;
        if (cp.cos_out) cp.cos_out[j] = c;
        cp.flag_out[j] = f ? 1 : 0;  // read back in the placement pass (device-scope load, after the store is acknowledged)
      } else {
        f = flag[j] != 0;
      }
    }
    mine += __popcll(__ballot(f));
  }
  if (lane == 0) wave_cnt[w] = mine;
  __syncthreads();
  int own = 0;
#pragma unroll
  for (int i = 0; i < CB / WAVE; ++i) own += wave_cnt[i];
  if (tid == 0) __hip_atomic_store(scan + 2 + bid, own + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  int before = 0;
  if (lo < hi) {  // a chunk past the end places nothing and waits for nobody
    for (int i = tid; i < bid; i += CB) {
      int v;
      do {
        v = __hip_atomic_load(scan + 2 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } while (v == 0);
      before += v - 1;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) before += __shfl_xor(before, o, WAVE);
  __syncthreads();
  if (lane == 0) wave_cnt[w] = before;
  __syncthreads();
  before = 0;
#pragma unroll
  for (int i = 0; i < CB / WAVE; ++i) before += wave_cnt[i];
  __syncthreads();
  if constexpr (FROM_PARTS) wait_vmcnt<0>();  // this thread's flag stores have reached the L2
  const int total = compact_range<CB>(FROM_PARTS ? cp.flag_out : flag, rows, lo, hi, before, B, L, out_idx, out_off,
                                      out_cap, FROM_PARTS, wave_cnt);
  // the workgroup that holds the end of the list (workgroup 0 of an empty one) writes the tail
  if ((lo < hi && hi == n) || (n == 0 && bid == 0))
    compact_tail<CB>(rows, n, total, B, L, out_off, out_cap, status, overflow_code);
  __syncthreads();
  if (tid == 0)
    s_last = __hip_atomic_fetch_add(scan + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == G - 1;
  __syncthreads();
  if (s_last) {
    for (int i = tid; i < G + 2; i += CB)
      __hip_atomic_store(scan + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

__global__ void k_fill_i32(int32_t *p, int32_t v, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

inline int row_grid(int cap) { return cap < 1 ? 1 : (cap > 8192 ? 8192 : cap); }

}  // namespace

void launch_gather_rmsnorm(DType t, const void *x, const void *gain, Rows rows, int d, float eps,
                           void *out, hipStream_t s) {
  if (rows.cap <= 0) return;
  const int grid = rows.cap < 1 ? 1 : (rows.cap > 32768 ? 32768 : rows.cap);
  if (t == F32) {
    if (d / 4 <= 256 * KEEP)
      k_gather_rmsnorm<float, 256><<<grid, 256, 0, s>>>((const float *)x, (const float *)gain, rows, d, eps, (float *)out);
    else
      k_gather_rmsnorm<float, RB><<<row_grid(rows.cap), RB, 0, s>>>((const float *)x, (const float *)gain, rows, d, eps, (float *)out);
  } else {
    if (d / 8 <= 256 * KEEP)
      k_gather_rmsnorm<bf16_t, 256><<<grid, 256, 0, s>>>((const bf16_t *)x, (const bf16_t *)gain, rows, d, eps, (bf16_t *)out);
    else
      k_gather_rmsnorm<bf16_t, RB><<<row_grid(rows.cap), RB, 0, s>>>((const bf16_t *)x, (const bf16_t *)gain, rows, d, eps, (bf16_t *)out);
  }
}

void launch_oproj_finalize(DType t, const float *part, Splits splits, size_t split_stride, const void *x,
                           const void *gain, Rows rows, int d, float eps, float *h, void *f,
                           hipStream_t s) {
  if (rows.cap <= 0) return;
  if (t == F32)
    k_oproj_finalize<float><<<row_grid(rows.cap), RB, 0, s>>>(part, splits, split_stride, (const float *)x,
                                                              (const float *)gain, rows, d, eps, h, (float *)f);
  else
    k_oproj_finalize<bf16_t><<<row_grid(rows.cap), RB, 0, s>>>(part, splits, split_stride, (const bf16_t *)x,
                                                               (const bf16_t *)gain, rows, d, eps, h,
                                                               (bf16_t *)f);
}

void launch_down_finalize(DType t, const float *part, Splits splits, size_t split_stride, const float *h,
                          Rows rows, int d, void *out_cache, hipStream_t s) {
  if (rows.cap <= 0 || splits.done_to >= rows.cap) return;
  const int g = row_grid(rows.cap - splits.done_to);
  if (t == F32)
    k_down_finalize<float><<<g, RB, 0, s>>>(part, splits, split_stride, h, rows, d, (float *)out_cache);
  else
    k_down_finalize<bf16_t><<<g, RB, 0, s>>>(part, splits, split_stride, h, rows, d, (bf16_t *)out_cache);
}

void launch_qkv_finalize(DType t, const float *part, Splits splits, size_t split_stride,
                         const float *rope_tab, Rows rows, int L, int H, int Hkv, int dh,
                         const void *bq, const void *bk, const void *bv, void *q_out, void *k_cache,
                         void *v_cache, void *dv_out, int q_by_token, void *ksal_out, int dv_by_entry,
                         int32_t *entry_of, int entry_lo, hipStream_t s) {
  if (rows.cap <= 0) return;
  if (t == F32)
    k_qkv_finalize<float><<<row_grid(rows.cap), RB, 0, s>>>(
        part, splits, split_stride, rope_tab, rows, L, H, Hkv, dh, (const float *)bq, (const float *)bk,
        (const float *)bv, (float *)q_out, (float *)k_cache, (float *)v_cache, (float *)dv_out, q_by_token,
        (float *)ksal_out, dv_by_entry, entry_of, entry_lo);
  else
    k_qkv_finalize<bf16_t><<<row_grid(rows.cap), RB, 0, s>>>(
        part, splits, split_stride, rope_tab, rows, L, H, Hkv, dh, (const bf16_t *)bq, (const bf16_t *)bk,
        (const bf16_t *)bv, (bf16_t *)q_out, (bf16_t *)k_cache, (bf16_t *)v_cache, (bf16_t *)dv_out, q_by_token,
        (bf16_t *)ksal_out, dv_by_entry, entry_of, entry_lo);
}

inline int sal_grid(int cap) { return cap < 1 ? 1 : (cap > 65536 ? 65536 : cap); }

void launch_saliency(DType t, const void *c_new, void *c_cache, Rows rows, int D, float tau,
                     float *cos_out, uint8_t *flag_out, int commit, hipStream_t s) {
  if (rows.cap <= 0) return;
  if (t == F32)
    k_saliency<float><<<sal_grid(rows.cap), SAL_NT, 0, s>>>((const float *)c_new, (float *)c_cache, rows,
                                                        D, tau, cos_out, flag_out, commit);
  else
    k_saliency<bf16_t><<<sal_grid(rows.cap), SAL_NT, 0, s>>>((const bf16_t *)c_new, (bf16_t *)c_cache,
                                                         rows, D, tau, cos_out, flag_out, commit);
}

void launch_compact(const uint8_t *flag, Rows rows, int B, int L, int32_t *out_idx,
                    int32_t *out_offsets, int out_cap, int32_t *status, int32_t *scan, hipStream_t s) {
  const int cap = rows.cap < 0 ? 0 : rows.cap;
  int G = (cap + CB - 1) / CB;
  G = G < 1 ? 1 : (G > CMAXG ? CMAXG : G);
  int chunk = (cap + G - 1) / G;
  chunk = ((chunk + CB - 1) / CB) * CB;
  if (chunk < CB) chunk = CB;
  k_compact<false><<<G, CB, 0, s>>>(flag, rows, B, L, chunk, out_idx, out_offsets, out_cap, status, -6, scan, CosParts{});
}

void launch_cos_compact(const float *cos_part, int H, float tau, float *cos_out, uint8_t *flag_out, Rows rows,
                        int B, int L, int32_t *out_idx, int32_t *out_offsets, int out_cap, int32_t *status,
                        int32_t *scan, hipStream_t s) {
  const int cap = rows.cap < 0 ? 0 : rows.cap;
  int G = (cap + CB - 1) / CB;
  G = G < 1 ? 1 : (G > CMAXG ? CMAXG : G);
  int chunk = (cap + G - 1) / G;
  chunk = ((chunk + CB - 1) / CB) * CB;
  if (chunk < CB) chunk = CB;
  k_compact<true><<<G, CB, 0, s>>>(flag_out, rows, B, L, chunk, out_idx, out_offsets, out_cap, status, -6, scan,
                                   CosParts{cos_part, cos_out, flag_out, H, tau});
}

// ---- approximate context update of the non-salient rows  [Sec. 3.3; Alg. 3 lines C <- ..., cosine] --
template <typename T>
__global__ __launch_bounds__(256) void k_clear_rows(Rows rows, T *dv, int dkv) {
  const int n = row_count(rows);
  constexpr int N = Vec16<T>::N;
  Vec16<T> zero;
#pragma unroll
  for (int e = 0; e < N; ++e) zero.set(e, 0.f);
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    const int r = rows.idx ? rows.idx[j] : j;
    for (int v = threadIdx.x; v < dkv / N; v += 256) st16(dv + (size_t)r * dkv + v * N, zero);
  }
}

// One workgroup per token of the step (entry j of `win`, token r).  Salient tokens (pos[r] != 0) take
// their exact row, all others the cached row plus the approximate residual; the cosine is taken over
// the stored (rounded) values against the cached row, which is read before it is overwritten.
// cos_out is indexed by token, flag_out by window entry.
// Residual: dc[j] (CACHED = false), or rebuilt from the partials of an attention pass over the compact
// candidate keys with the token's CACHED log-normaliser: sum over the key splits that hold keys of
// the token's sequence of part_o[s][j] * exp(m_s - lse[r, h])  (part_o is relative to the split's own
// running maximum m_s; nothing is renormalised).
struct CachedNorm {
  const float *part_o, *part_ml, *lse;
  const int32_t *key_offsets;
  int cap, H, dh, chunk, splits, L;
};

template <typename T, bool CACHED>
__global__ __launch_bounds__(SAL_NT) void k_saliency_approx(Rows win, int D, const T *__restrict__ c_sal,
                                                             const T *__restrict__ dc,
                                                             int32_t *__restrict__ pos, T *c_cache,
                                                             float tau, float *__restrict__ cos_out,
                                                             uint8_t *__restrict__ flag_out, CachedNorm cn) {
  __shared__ float red[3 * SAL_NT / WAVE];
  constexpr int N = Vec16<T>::N;
  const int nv = D / N;
  const int n = row_count(win);
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    const int r = win.idx ? win.idx[j] : j;
    const int p = pos[r];
    T *b = c_cache + (size_t)r * D;
    const T *src = p ? c_sal + (size_t)(p - 1) * D : dc + (size_t)j * D;
    int ns = 0;  // key splits that hold candidate keys of this token's sequence
    if (CACHED && !p) {
      const int sq = r / cn.L;
      const int lk = cn.key_offsets[sq + 1] - cn.key_offsets[sq];
      ns = (lk + cn.chunk - 1) / cn.chunk;
      ns = ns < cn.splits ? ns : cn.splits;
    }
    float dot = 0.f, na = 0.f, nb = 0.f;
    for (int v = threadIdx.x; v < nv; v += SAL_NT) {
      const Vec16<T> vb = ld16(b + v * N);
      Vec16<T> vn;
      if (CACHED && !p) {
        const int c = v * N, h = c / cn.dh;
        const float ref = cn.lse[(size_t)r * cn.H + h];
        float res[N];
#pragma unroll
        for (int i = 0; i < N; ++i) res[i] = 0.f;
        for (int sp = 0; sp < ns; ++sp) {
          const size_t row = (size_t)sp * cn.cap + j;
          const float wgt = __expf(cn.part_ml[(row * cn.H + h) * 2] - ref);
          const float4 *po = reinterpret_cast<const float4 *>(cn.part_o + row * D + c);
#pragma unroll
          for (int q4 = 0; q4 < N / 4; ++q4) {
            const float4 o = po[q4];
            res[4 * q4] += o.x * wgt; res[4 * q4 + 1] += o.y * wgt;
            res[4 * q4 + 2] += o.z * wgt; res[4 * q4 + 3] += o.w * wgt;
          }
        }
#pragma unroll
        for (int i = 0; i < N; ++i) vn.set(i, vb.get(i) + res[i]);
      } else {
        const Vec16<T> vs = ld16(src + v * N);
#pragma unroll
        for (int i = 0; i < N; ++i) vn.set(i, p ? vs.get(i) : vb.get(i) + vs.get(i));
      }
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const float fa = vn.get(i), fb = vb.get(i);
        dot += fa * fb;
        na += fa * fa;
        nb += fb * fb;
      }
      st16(b + v * N, vn);
    }
    block_sum3<SAL_NT>(dot, na, nb, red);
    if (threadIdx.x == 0) {
      const float s = dot / (fmaxf(sqrtf(na), 1e-8f) * fmaxf(sqrtf(nb), 1e-8f));
      if (cos_out) cos_out[r] = s;
      flag_out[j] = (s < tau) ? 1 : 0;
      // The map goes back to zero as it is consumed: every marked token is a token of the step, this
      // workgroup alone reads its entry, and all its threads did so before the barriers of the sum.
      if (p) pos[r] = 0;
    }
  }
}

// The tokens at positions [lo, L) of every sequence as an index list (a response-only step's rows).
__global__ __launch_bounds__(256) void k_make_window(int B, int L, int lo, int32_t *idx, int32_t *off) {
  const int w = L - lo, n = B * w;
  for (int j = blockIdx.x * 256 + threadIdx.x; j < n; j += gridDim.x * 256) idx[j] = (j / w) * L + lo + j % w;
  if (blockIdx.x == 0)
    for (int b = threadIdx.x; b <= B; b += 256) off[b] = b * w;
}

// flag[r] = 1 for the tokens r of a list at positions >= lo of their sequence (an id outside [0, T)
// is ignored rather than written through)
__global__ __launch_bounds__(256) void k_mark_flags(Rows rows, int T, int L, int lo, uint8_t *flag) {
  const int n = row_count(rows);
  for (int j = blockIdx.x * 256 + threadIdx.x; j < n; j += gridDim.x * 256) {
    const int r = rows.idx[j];
    if ((unsigned)r < (unsigned)T && r % L >= lo) flag[r] = 1;
  }
}

void launch_saliency_approx(DType t, Rows win, int D, const void *c_sal, const void *dc, int32_t *pos,
                            void *c_cache, float tau, float *cos_out, uint8_t *flag_out,
                            const AttnArgs *cached, const float *lse, int L, hipStream_t s) {
  if (win.cap <= 0) return;
  const int grid = win.cap > 65536 ? 65536 : win.cap;
  CachedNorm cn{};
  if (cached)
    cn = CachedNorm{cached->part_o, cached->part_ml, lse, cached->key_offsets, cached->rows.cap,
                    cached->H, cached->dh, cached->chunk, cached->splits, L};
#define DY_SAL_APPROX(TT, C)                                                                        \
  k_saliency_approx<TT, C><<<grid, SAL_NT, 0, s>>>(win, D, (const TT *)c_sal, (const TT *)dc, pos, \
                                                   (TT *)c_cache, tau, cos_out, flag_out, cn)
  if (t == F32) {
    if (cached) DY_SAL_APPROX(float, true);
    else DY_SAL_APPROX(float, false);
  } else {
    if (cached) DY_SAL_APPROX(bf16_t, true);
    else DY_SAL_APPROX(bf16_t, false);
  }
#undef DY_SAL_APPROX
}

void launch_make_window(int B, int L, int lo, int32_t *idx, int32_t *off, hipStream_t s) {
  const int n = B * (L - lo);
  k_make_window<<<n > 0 ? (n + 255) / 256 : 1, 256, 0, s>>>(B, L, lo, idx, off);
}

void launch_mark_flags(Rows rows, int T, int L, int lo, uint8_t *flag, hipStream_t s) {
  if (rows.cap <= 0) return;
  k_mark_flags<<<(rows.cap + 255) / 256, 256, 0, s>>>(rows, T, L, lo, flag);
}

void launch_clear_rows(DType t, Rows rows, void *dv, int dkv, hipStream_t s) {
  if (rows.cap <= 0) return;
  if (t == F32) k_clear_rows<float><<<row_grid(rows.cap), 256, 0, s>>>(rows, (float *)dv, dkv);
  else k_clear_rows<bf16_t><<<row_grid(rows.cap), 256, 0, s>>>(rows, (bf16_t *)dv, dkv);
}

// Row-major [n_out, n_in] matrix of 2-byte elements -> the panel layout the bf16 GEMMs read
// (panels of 32 rows, K-slice-major inside a panel): thread u moves the 16 bytes of destination unit u.
__global__ __launch_bounds__(256) void k_pack_weight(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                     int n_in, size_t units) {
  const int kslices = n_in / 64;
  for (size_t u = (size_t)blockIdx.x * 256 + threadIdx.x; u < units; u += (size_t)gridDim.x * 256) {
    const int c8 = (int)(u % 8), r = (int)((u / 8) % 32);
    const size_t pk = u / 256;  // panel * kslices + slice
    const int kt = (int)(pk % kslices);
    const size_t row = (pk / kslices) * 32 + r;
    dst[u] = src[(row * (size_t)n_in + (size_t)kt * 64) / 8 + c8];
  }
}

void launch_pack_weight(const void *src, int n_out, int n_in, void *dst, hipStream_t s) {
  const size_t units = (size_t)n_out * n_in / 8;
  if (units == 0) return;
  const size_t want = (units + 255) / 256;
  k_pack_weight<<<(unsigned)(want < 65536 ? want : 65536), 256, 0, s>>>((const uint4 *)src, (uint4 *)dst, n_in, units);
}

void launch_fill_i32(int32_t *p, int32_t v, int n, hipStream_t s) {
  if (n <= 0) return;
  k_fill_i32<<<(n + 255) / 256, 256, 0, s>>>(p, v, n);
}

}  // namespace dy
