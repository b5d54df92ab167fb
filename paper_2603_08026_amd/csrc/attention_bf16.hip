// Partial (row-sparse) attention for bf16 storage on the gfx950 matrix cores: exact attention rows
// for the salient queries against all keys/values of their sequence, no mask.
// [Sec. 3.3 salient path; Alg. 3: C_sal]
//
// Everything is computed transposed so that no operand ever has to be re-laid-out between the two
// matrix products:
//   S^T = K Q^T   A = K tile rows (LDS, [key][dh]),   B = Q rows (registers, loaded once)
//                 -> a lane owns ONE query (column l%32) and 16 keys per 32-key block, so the row
//                    maximum / sum of the online softmax are 32 register operations and one
//                    cross-half shuffle, and the rescale of the running output is a plain multiply.
//   O^T = V^T P^T A = V^T (LDS, [dh][key], transposed while it is written), B = P^T straight from
//                    the S^T accumulator registers: element i of the lane's operand is register
//                    8*ks+i, i.e. key 16*ks + 8*(i/4) + 4*(l/32) + i%4 -- the V^T operand is read
//                    with the same key order (two 8-byte LDS reads), and a matrix product does not
//                    care in which order k is summed as long as both operands agree.
// Two kernels.  k_attn_bf16 (head_dim 64): a workgroup of NW waves owns BQ = 32*QB*WQ query rows of
// one (sequence, head): WQ wave rows of QB blocks of 32 queries each; the keys of a tile are split
// over the WK = NW/WQ wave columns (32 keys each), whose partial (max, sum, output) are merged
// through LDS at the end; K/V tiles are double-buffered in LDS with a register-staged prefetch and V
// is transposed while it is written.  k_attn_bf16_dma (head_dim 128, further down): K/V tiles arrive
// by asynchronous global -> LDS copies into four stages, V^T comes from the LDS transpose read, a
// wave holds one block of 32 queries (two waves per SIMD), the loop runs three tiles deep, and the
// query heads of a KV group are folded into the rows of a tile.
// The key range of a sequence can additionally be split over workgroups (few query rows): then
// un-normalised partials go to global memory and k_attn_combine merges them.
#include "attention_common.h"
#include <type_traits>

namespace dy {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

template <int DH, int WQ, int NW, int QB> struct ATile {
  static constexpr int NT = 64 * NW;      // threads per workgroup
  static constexpr int WK = NW / WQ;      // wave columns over the keys of a tile
  static constexpr int BQ = 32 * QB * WQ; // query rows per workgroup
  static constexpr int TK = 32 * WK;      // keys per tile
  static constexpr int KSTR = DH + 8;     // K tile row stride (elements): 16-byte reads conflict-free
  static constexpr int VSTR = TK + 4;     // V^T row stride (elements): 8-byte reads conflict-free
  static constexpr int STAGE = TK * KSTR + DH * VSTR;
  static constexpr int DB = DH / 32, KK = DH / 16;
  static constexpr int K_CH = TK * DH / 8 / NT;       // 16-byte K chunks per thread and tile
  static constexpr int V_CH = TK * DH / 8 / 2 / NT;   // pairs of V chunks per thread and tile
  static constexpr size_t LDS_BYTES = (size_t)2 * STAGE * 2;
  // merge scratch (reuses the tile buffers): (WK-1)*WQ waves x (QB*DB*16 + 2*QB) floats x 64 lanes
  static constexpr int PER_WAVE = (QB * DB * 16 + 2 * QB) * 64;
  static constexpr size_t MERGE_BYTES = (size_t)(WK - 1) * WQ * PER_WAVE * 4;
  static_assert(MERGE_BYTES <= LDS_BYTES, "merge scratch must fit in the tile buffers");
  static_assert(K_CH >= 1 && V_CH >= 1 && K_CH * NT * 8 == TK * DH && V_CH * NT * 16 == TK * DH,
                "the tile is copied in whole 16-byte chunks per thread");
};

// global -> registers: one K/V tile (keys past k_hi are clamped to the last valid key; their scores
// are masked later)
template <typename T, int DH, int KCH, int VCH>
__device__ __forceinline__ void load_kv_tile(uint4 (&rk)[KCH], uint4 (&rv)[VCH][2],
                                             const bf16_t *kc, const bf16_t *vc, size_t kv_stride, int k0,
                                             int k_hi, int tid) {
#pragma unroll
  for (int i = 0; i < T::K_CH; ++i) {
    const int c = tid + T::NT * i;
    int key = k0 + c / (DH / 8);
    key = key < k_hi ? key : k_hi - 1;
    rk[i] = *reinterpret_cast<const uint4 *>(kc + (size_t)key * kv_stride + (c % (DH / 8)) * 8);
  }
#pragma unroll
  for (int i = 0; i < T::V_CH; ++i) {
    const int u = tid + T::NT * i;
    const int rest = u / 64;
    const int ch = (u % 4) + 4 * (rest % (DH / 32));
    const int kp = ((u / 4) % 16) + 16 * (rest / (DH / 32));
    int key0 = k0 + 2 * kp, key1 = key0 + 1;
    key0 = key0 < k_hi ? key0 : k_hi - 1;
    key1 = key1 < k_hi ? key1 : k_hi - 1;
    rv[i][0] = *reinterpret_cast<const uint4 *>(vc + (size_t)key0 * kv_stride + ch * 8);
    rv[i][1] = *reinterpret_cast<const uint4 *>(vc + (size_t)key1 * kv_stride + ch * 8);
  }
}

__device__ __forceinline__ uint32_t half_of(const uint4 &v, int e) {
  const uint32_t w = (e >> 1) == 0 ? v.x : (e >> 1) == 1 ? v.y : (e >> 1) == 2 ? v.z : v.w;
  return (e & 1) ? (w >> 16) : (w & 0xffffu);
}

// registers -> LDS stage: K rows as they are, V transposed ([dh][key]): element e of two
// neighbouring keys forms one 32-bit word, so a wave's 64 stores hit 32 banks twice.
template <typename T, int DH, int KCH, int VCH>
__device__ __forceinline__ void store_kv_tile(const uint4 (&rk)[KCH], const uint4 (&rv)[VCH][2],
                                              bf16_t *stage, int tid) {
  bf16_t *sk = stage, *sv = stage + T::TK * T::KSTR;
#pragma unroll
  for (int i = 0; i < T::K_CH; ++i) {
    const int c = tid + T::NT * i;
    *reinterpret_cast<uint4 *>(sk + (c / (DH / 8)) * T::KSTR + (c % (DH / 8)) * 8) = rk[i];
  }
#pragma unroll
  for (int i = 0; i < T::V_CH; ++i) {
    const int u = tid + T::NT * i;
    const int rest = u / 64;
    const int ch = (u % 4) + 4 * (rest % (DH / 32));
    const int kp = ((u / 4) % 16) + 16 * (rest / (DH / 32));
#pragma unroll
    for (int e = 0; e < 8; ++e)
      *reinterpret_cast<uint32_t *>(sv + (ch * 8 + e) * T::VSTR + 2 * kp) =
          half_of(rv[i][0], e) | (half_of(rv[i][1], e) << 16);
  }
}

template <int DH, int WQ, int NW, int QB>
__global__ __launch_bounds__(64 * NW) void k_attn_bf16(AttnArgs a, int q_tiles) {
  using T = ATile<DH, WQ, NW, QB>;
  constexpr int WK = T::WK, BQ = T::BQ, TK = T::TK, KSTR = T::KSTR, VSTR = T::VSTR, DB = T::DB, KK = T::KK;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *smem = reinterpret_cast<bf16_t *>(smem_raw);
  __shared__ int tile_info[3];

  const int tid = threadIdx.x, lane = tid % WAVE, wave = tid / WAVE;
  const int l32 = lane % 32, lhi = lane / 32;
  const int wq = wave / WK, wk = wave % WK;
  int tile, h, split;
  if (!attn_work_item(a, q_tiles, &tile, &h, &split)) return;  // uniform
  if (tid == 0) find_tile(a, BQ, tile, tile_info);
  __syncthreads();
  const int b = tile_info[0];
  if (b < 0) return;  // uniform: no such tile
  const int j0 = tile_info[1], nq = tile_info[2];
  const int kvh = h / (a.H / a.Hkv);
  const int kbase = a.key_offsets ? a.key_offsets[b] : b * a.L;
  const int Lk = a.key_offsets ? a.key_offsets[b + 1] - kbase : a.L;
  const int k_lo = split * a.chunk, k_hi = min(Lk, k_lo + a.chunk);
  if (k_lo >= k_hi) return;  // uniform

  const size_t kv_stride = (size_t)a.Hkv * DH;
  const bf16_t *kc = (const bf16_t *)a.k + ((size_t)kbase * a.Hkv + kvh) * DH;
  const bf16_t *vc = (const bf16_t *)a.v + ((size_t)kbase * a.Hkv + kvh) * DH;

  // query operands: QB blocks of 32 queries per wave, kept in registers for the whole key sweep
  bf16x8 qf[QB][KK];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int r = wq * (32 * QB) + qb * 32 + l32;
    r = r < nq ? r : nq - 1;  // rows past the end are clamped; their results are never stored
    const size_t qrow = a.q_by_token ? (size_t)a.rows.idx[j0 + r] : (size_t)(j0 + r);
    const bf16_t *qp = (const bf16_t *)a.q + (qrow * a.H + h) * DH + lhi * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[qb][kk] = *reinterpret_cast<const bf16x8 *>(qp + kk * 16);
  }

  floatx16 acc_o[QB][DB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc_o[qb][db][e] = 0.f;
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }
  const float sc = LOG2E / sqrtf((float)DH);  // scores are kept in the log2 domain

  uint4 rk[T::K_CH], rv[T::V_CH][2];
  const int n_tiles = (k_hi - k_lo + TK - 1) / TK;
  load_kv_tile<T, DH, T::K_CH, T::V_CH>(rk, rv, kc, vc, kv_stride, k_lo, k_hi, tid);
  store_kv_tile<T, DH, T::K_CH, T::V_CH>(rk, rv, smem, tid);
  __syncthreads();
  for (int t = 0; t < n_tiles; ++t) {
    const int k0 = k_lo + t * TK;
    const bf16_t *stage = smem + (t & 1) * T::STAGE;
    // prefetch the next tile (the last iteration re-reads its own tile: harmless, keeps the loop uniform)
    load_kv_tile<T, DH, T::K_CH, T::V_CH>(rk, rv, kc, vc, kv_stride, t + 1 < n_tiles ? k0 + TK : k0, k_hi, tid);

    // S^T block of this wave: 32 keys x 64 queries
    floatx16 s[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int e = 0; e < 16; ++e) s[qb][e] = 0.f;
    const bf16_t *skp = stage + (wk * 32 + l32) * KSTR + lhi * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(skp + kk * 16);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) s[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][kk], s[qb], 0, 0, 0);
    }

    // online softmax per query (= per lane), keys of this wave only.  The running reference m_run is
    // only moved when the block maximum exceeds it by more than 2^8: until then exp2(s - m_run) stays
    // below 256, which bf16 probabilities and fp32 sums hold without loss, and the 128-register
    // rescale of the output accumulator is skipped for the whole wave.
    const int key_base = k0 + wk * 32 + 4 * lhi;
    const bool tail = k0 + TK > k_hi;  // wave-uniform: only the last tile can hold keys past the end
    bf16x8 pf[QB][2];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if (tail) {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (key_base + 8 * (e / 4) + (e % 4) >= k_hi) s[qb][e] = -INFINITY;
      }
      float mx = s[qb][0];
#pragma unroll
      for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s[qb][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE)) * sc;
      const bool need = mx > m_run[qb] + 8.0f;
      if (__any(need)) {
        const float corr = need ? __builtin_amdgcn_exp2f(m_run[qb] - mx) : 1.0f;
        m_run[qb] = need ? mx : m_run[qb];
        l_run[qb] *= corr;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc_o[qb][db][e] *= corr;
      }
      const float neg_ref = (m_run[qb] == -INFINITY) ? 0.f : -m_run[qb];
      float ps = 0.f;
      uint32_t pw[8];
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[qb][e], sc, neg_ref));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[qb][e + 1], sc, neg_ref));
        // the sum uses the rounded values that enter the matrix product
        const uint32_t w = pack_bf16(p0, p1);
        ps += __uint_as_float(w << 16) + __uint_as_float(w & 0xffff0000u);
        pw[e >> 1] = w;
      }
      ps += __shfl_xor(ps, 32, WAVE);
      l_run[qb] += ps;
      uint4 v0{pw[0], pw[1], pw[2], pw[3]}, v1{pw[4], pw[5], pw[6], pw[7]};
      pf[qb][0] = __builtin_bit_cast(bf16x8, v0);
      pf[qb][1] = __builtin_bit_cast(bf16x8, v1);
    }

    // O^T += V^T P^T over the wave's 32 keys
    const bf16_t *svp = stage + TK * KSTR + l32 * VSTR + wk * 32 + 4 * lhi;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16_t *p = svp + db * 32 * VSTR + ks * 16;
        const uint2 a0 = *reinterpret_cast<const uint2 *>(p);
        const uint2 a1 = *reinterpret_cast<const uint2 *>(p + 8);
        const uint4 av{a0.x, a0.y, a1.x, a1.y};
        const bf16x8 vf = __builtin_bit_cast(bf16x8, av);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          acc_o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qb][ks], acc_o[qb][db], 0, 0, 0);
      }

    store_kv_tile<T, DH, T::K_CH, T::V_CH>(rk, rv, smem + ((t + 1) & 1) * T::STAGE, tid);
    __syncthreads();
  }

  // merge the WK wave columns of each query block through LDS (tile buffers are free now)
  float *mg = reinterpret_cast<float *>(smem_raw);
  constexpr int PER_WAVE = T::PER_WAVE;
  if (WK > 1) {
    if (wk > 0) {
      float *dst = mg + (size_t)((wk - 1) * WQ + wq) * PER_WAVE + lane;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) dst[((qb * DB + db) * 16 + e) * 64] = acc_o[qb][db][e];
        dst[(QB * DB * 16 + qb) * 64] = m_run[qb];
        dst[(QB * DB * 16 + QB + qb) * 64] = l_run[qb];
      }
    }
    __syncthreads();
    if (wk == 0) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float M = m_run[qb];
#pragma unroll
        for (int w = 1; w < WK; ++w)
          M = fmaxf(M, mg[(size_t)((w - 1) * WQ + wq) * PER_WAVE + (QB * DB * 16 + qb) * 64 + lane]);
        const float Ms = (M == -INFINITY) ? 0.f : M;
        const float c0 = __builtin_amdgcn_exp2f(m_run[qb] - Ms);
        float lsum = l_run[qb] * c0;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc_o[qb][db][e] *= c0;
#pragma unroll
        for (int w = 1; w < WK; ++w) {
          const float *src = mg + (size_t)((w - 1) * WQ + wq) * PER_WAVE + lane;
          const float cw = __builtin_amdgcn_exp2f(src[(QB * DB * 16 + qb) * 64] - Ms);
          lsum += src[(QB * DB * 16 + QB + qb) * 64] * cw;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_o[qb][db][e] += src[((qb * DB + db) * 16 + e) * 64] * cw;
        }
        m_run[qb] = M;
        l_run[qb] = lsum;
      }
    }
  }

  if (wk == 0) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int r = wq * (32 * QB) + qb * 32 + l32;
      if (r < nq) {
        const int j = j0 + r;
        if (a.splits == 1 && !a.partial) {
          bf16_t *out = (bf16_t *)a.out + ((size_t)j * a.H + h) * DH + 4 * lhi;
          const float inv = 1.0f / l_run[qb];
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              uint2 w;
              w.x = pack_bf16(acc_o[qb][db][4 * g] * inv, acc_o[qb][db][4 * g + 1] * inv);
              w.y = pack_bf16(acc_o[qb][db][4 * g + 2] * inv, acc_o[qb][db][4 * g + 3] * inv);
              *reinterpret_cast<uint2 *>(out + db * 32 + 8 * g) = w;
            }
        } else {
          float *po = a.part_o + (((size_t)split * a.rows.cap + j) * a.H + h) * DH + 4 * lhi;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              float4 w{acc_o[qb][db][4 * g], acc_o[qb][db][4 * g + 1], acc_o[qb][db][4 * g + 2],
                       acc_o[qb][db][4 * g + 3]};
              *reinterpret_cast<float4 *>(po + db * 32 + 8 * g) = w;
            }
          if (lhi == 0) {
            float *ml = a.part_ml + (((size_t)split * a.rows.cap + j) * a.H + h) * 2;
            ml[0] = m_run[qb] * LN2;  // partials carry the maximum in natural-log units
            ml[1] = l_run[qb];
          }
        }
      }
    }
  }
}

// ---- head_dim 128: K and V tiles by asynchronous global -> LDS copies -----------------------------
// No register staging: NS LDS stages, so a tile has NS - 1 tile computations to arrive from HBM.
// Both tiles keep the cache layout [key][dh] (256-byte rows, written 4 rows per copy instruction).
//   K rows feed S^T = K Q^T directly (16-byte reads); the 16-byte chunk c of row r sits at chunk
//     position c ^ (r % 16), so the 16 rows a read serves at a time cover all 64 banks once.
//   V^T operands come from the LDS transpose read (ds_read_b64_tr_b16): within 16 lanes, lane j
//     names the 8 bytes of row key0 + j/4 at columns dh0 + 4*(j%4) .. +3 and lane i receives column
//     dh0 + i of the rows key0 .. key0+3 -- four consecutive keys of one dh, which is exactly one half
//     of the operand in the key order the P^T registers have.  The 32-byte pair p of row r sits at
//     pair position p ^ 2*(r % 4).  32 lanes read at a time: two groups of 16 (column pairs 2*db and
//     2*db + 1), each 4 consecutive rows x 32 bytes; a pair position is one octet of the 64 banks, so
//     the even pair lands on the four even-or-odd octets 2*db ^ {0, 2, 4, 6} and the odd pair on the
//     other four -- every bank once (SQ_LDS_BANK_CONFLICT = 0; with p ^ (r % 8) both groups fell on
//     the same four octets and every read took twice its cycles).

// value of the lane 32 away combined with this lane's (v_permlane32_swap: no LDS round trip)
__device__ __forceinline__ float xhalf_max(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
typedef short shortx4 __attribute__((ext_vector_type(4)));

template <int WQ, int WK_> struct DTile {
  static constexpr int DH = 128, WK = WK_;  // wave columns over the keys of a tile
  static constexpr int NW = WQ * WK, NT = 64 * NW;
  static constexpr int BQ = 32 * WQ;      // query rows per workgroup
  static constexpr int TK = 32 * WK;      // keys per tile
  static constexpr int ROWB = DH * 2;     // bytes per key row
  static constexpr int REGION = TK * ROWB;          // K rows, then V rows
  static constexpr int STAGE_BYTES = 2 * REGION;
  static constexpr int NS = 4;                            // LDS stages
  static constexpr int LPW = 2 * (TK / 4) / NW;          // copy instructions per wave and tile
  static constexpr int DB = DH / 32, KK = DH / 16;
  static constexpr int PER_WAVE = (DB * 16 + 2) * 64;    // merge scratch per wave (floats)
  static constexpr size_t LDS_BYTES = (size_t)NS * STAGE_BYTES;
  static_assert(NS >= 3 && (NS - 2) * LPW < 64, "stages (the loop reads two tiles at a time) and vmcnt immediate");
  static_assert((size_t)(WK - 1) * WQ * PER_WAVE * 4 <= LDS_BYTES, "merge scratch must fit in the tile buffers");
  static_assert(LPW >= 2 && LPW % 2 == 0, "every wave copies K and V rows");
};

template <int WQ, int WK_>
__global__ __launch_bounds__(64 * WQ * WK_, 2) void k_attn_bf16_dma(AttnArgs a, int q_tiles) {  // two waves per SIMD: 256 registers, no AGPR shuffling
  using T = DTile<WQ, WK_>;
  constexpr int DH = T::DH, NW = T::NW, WK = T::WK, BQ = T::BQ, TK = T::TK, ROWB = T::ROWB, NS = T::NS,
                DB = T::DB, KK = T::KK, LPW = T::LPW;
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  __shared__ int tile_info[4];

  const int tid = threadIdx.x, lane = tid % WAVE;
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int l32 = lane % 32, lhi = lane / 32;
  const int wq = wave / WK, wk = wave % WK;
  int tile, kvh, split;
  if (!attn_work_item_grouped(a, q_tiles, &tile, &kvh, &split)) return;  // uniform
  if (tid == 0) find_tile_grouped(a, BQ, tile, tile_info);
  __syncthreads();
  const int b = tile_info[0];
  if (b < 0) return;  // uniform: no such tile
  const int nq = tile_info[3];  // (row, head of the group) pairs in this tile
  // this lane's query: packed row p = row * g + head of the group (rows past the end are clamped to
  // the last one; their results are never stored)
  const int grp = a.H / a.Hkv;
  int jq, hq;
  {
    int r = wq * 32 + l32;
    r = r < nq ? r : nq - 1;
    const int p = tile_info[2] + r;
    jq = tile_info[1] + p / grp;
    hq = kvh * grp + p % grp;
  }
  const int kbase = a.key_offsets ? a.key_offsets[b] : b * a.L;
  const int Lk = a.key_offsets ? a.key_offsets[b + 1] - kbase : a.L;
  const int k_lo = split * a.chunk, k_hi = min(Lk, k_lo + a.chunk);
  if (k_lo >= k_hi) return;  // uniform

  const size_t kv_stride = (size_t)a.Hkv * DH;
  const bf16_t *kc = (const bf16_t *)a.k + ((size_t)kbase * a.Hkv + kvh) * DH;
  const bf16_t *vc = (const bf16_t *)a.v + ((size_t)kbase * a.Hkv + kvh) * DH;

  // query operand: the wave's 32 queries, in registers for the whole key sweep
  bf16x8 qf[KK];
  {
    const size_t qrow = a.q_by_token ? (size_t)a.rows.idx[jq] : (size_t)jq;
    const bf16_t *qp = (const bf16_t *)a.q + (qrow * a.H + hq) * DH + lhi * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8 *>(qp + kk * 16);
  }
  floatx16 acc_o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc_o[db][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = LOG2E / sqrtf((float)DH);  // scores are kept in the log2 domain

  const uint32_t lds0 = lds_offset_of(smem_raw);
  const int n_tiles = (k_hi - k_lo + TK - 1) / TK;
  // copy mapping: an instruction fills 4 key rows; this lane holds chunk position cpos of row r4
  const int r4 = lane / 16, cpos = lane % 16;
  auto issue = [&](int t) {  // tile t -> stage t % NS (keys past k_hi re-read the last key; masked later)
    const uint32_t sb = lds0 + (uint32_t)(t % NS) * T::STAGE_BYTES;
    const int kbase = k_lo + t * TK;
#pragma unroll
    for (int i = 0; i < LPW / 2; ++i) {
      const int ii = i * NW + wave;  // rows 4*ii .. 4*ii+3 of the tile
      const int row = ii * 4 + r4;
      int key = kbase + row;
      key = key < k_hi ? key : k_hi - 1;
      const int ck = cpos ^ (row & 15);
      const int cv = (((cpos >> 1) ^ ((row & 3) << 1)) << 1) | (cpos & 1);
      dma16(kc + (size_t)key * kv_stride + ck * 8, sb + (uint32_t)ii * 1024u);
      dma16(vc + (size_t)key * kv_stride + cv * 8, sb + (uint32_t)T::REGION + (uint32_t)ii * 1024u);
    }
  };

  // full tiles: a scalar base per tile and loop-invariant lane offsets (no vector arithmetic per copy)
  uint32_t off_k[LPW / 2], off_v[LPW / 2];
#pragma unroll
  for (int i = 0; i < LPW / 2; ++i) {
    const int ii = i * NW + wave, row = ii * 4 + r4;
    off_k[i] = (uint32_t)(((size_t)row * kv_stride + (cpos ^ (row & 15)) * 8) * 2);
    off_v[i] = (uint32_t)(((size_t)row * kv_stride + (((((cpos >> 1) ^ ((row & 3) << 1)) << 1) | (cpos & 1)) * 8)) * 2);
  }
  auto uniform_ptr = [](const void *p) {
    const uint64_t u = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return (const unsigned char *)(((uint64_t)hi << 32) | lo);
  };
  const unsigned char *kc_u = uniform_ptr(kc + (size_t)k_lo * kv_stride), *vc_u = uniform_ptr(vc + (size_t)k_lo * kv_stride);
  auto issue_full = [&](int t) {  // tile t, all of whose keys exist, -> stage t % NS
    const uint32_t sb = lds0 + (uint32_t)(t % NS) * T::STAGE_BYTES;
    const size_t adv = (size_t)t * TK * kv_stride * 2;
#pragma unroll
    for (int i = 0; i < LPW / 2; ++i) {
      const int ii = i * NW + wave;
      dma16_s(kc_u + adv, off_k[i], sb + (uint32_t)ii * 1024u);
      dma16_s(vc_u + adv, off_v[i], sb + (uint32_t)T::REGION + (uint32_t)ii * 1024u);
    }
  };

  // per-lane constants of the operand reads
  const int krow = wk * 32 + l32, ksw = l32 & 15;
  const int vq = (lane % 16) / 4;                       // row of this lane inside a 4-key group
  const int vrow = wk * 32 + 4 * lhi + vq, vsw = 2 * vq, hb = (lane / 16) & 1;  // (row % 4 = vq)
  const int key_lane = wk * 32 + 4 * lhi;

#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < n_tiles) issue(s);

  // A wave whose 32 query rows all lie past the tile's last row (ragged row counts: a sequence with
  // 70 candidates leaves two of the four waves of a 128-row tile without a query) takes no part in the
  // products: it keeps its share of the copies and meets the same barriers, in a loop of its own so
  // that the schedule of the working waves' loop is untouched.
  if (wq * 32 >= nq) {  // wave-uniform
    if (NS - 2 < n_tiles) wait_vmcnt<(NS - 2) * LPW>();
    else wait_vmcnt<0>();
    __syncthreads();
    for (int t = 0; t < n_tiles; ++t) {
      if (t + NS - 2 < n_tiles) wait_vmcnt<(NS - 3) * LPW>();
      else wait_vmcnt<0>();
      __syncthreads();
      if (t + NS - 1 < n_tiles) issue(t + NS - 1);
    }
  } else {
  // Software pipeline over three tiles: while the vector ALU takes the exponentials of tile t, the
  // matrix pipe works through the P V product of tile t-1 and the score block of tile t+1, so a
  // wave's vector work runs under its own matrix products (the waves of a workgroup move in step,
  // tile by tile, and would otherwise all queue for the same pipe at the same time).
  floatx16 s_cur;
  {
    if (NS - 2 < n_tiles) wait_vmcnt<(NS - 2) * LPW>();  // tile 0 has landed (this wave's part)
    else wait_vmcnt<0>();
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 16; ++e) s_cur[e] = 0.f;
    const unsigned char *skp = smem_raw + krow * ROWB;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(skp + (((2 * kk + lhi) ^ ksw) * 16));
      s_cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s_cur, 0, 0, 0);
    }
  }

  // Loop state carried from one tile to the next: the V^T fragments and the rounded probabilities
  // of the tile whose P V product is still to be issued (zero before the first tile).
  typedef __attribute__((address_space(3))) shortx4 lds_shortx4;
  typedef short shortx8 __attribute__((ext_vector_type(8)));
  bf16x8 vf[2][DB], pf[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
    for (int e = 0; e < 8; ++e) pf[ks][e] = (__bf16)0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) vf[ks][db] = pf[ks];
  }
  auto pv = [&]() {  // O^T += V^T P^T of the tile held in vf / pf
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[ks][db], pf[ks], acc_o[db], 0, 0, 0);
  };
  // One tile.  Order: (1) the first K fragments of tile t+1 are requested from LDS and the maximum
  // of tile t's scores is taken (and, rarely, the reference moved); (2) sixteen matrix instructions
  // follow -- the P V product of tile t-1, then the score product of tile t+1 -- each with its share
  // of tile t's exponentials behind it; the other K fragments are requested in between and the V
  // fragments of tile t at the end, into registers the products have released.  No product waits
  // for an LDS read issued right before it, and the vector ALU works while the matrix pipe does.
  // STEADY: the tile fetched in this iteration is a full one and no key of tile t lies past the end.
  // STAGE: the LDS stage of tile t when the caller knows it at compile time (the loop is unrolled over
  // the stages, so that the operand reads are a loop-invariant lane address plus an immediate), else -1.
  auto body = [&](int t, auto steady_c, auto stage_c) {
    constexpr bool STEADY = decltype(steady_c)::value;
    constexpr int STAGE = decltype(stage_c)::value;
    const int sidx = STAGE >= 0 ? STAGE : t % NS;
    if (STEADY) {
      wait_vmcnt<(NS - 3) * LPW>();
    } else {
      if (t + NS - 2 < n_tiles) wait_vmcnt<(NS - 3) * LPW>();
      else wait_vmcnt<0>();
    }
    __syncthreads();  // tile t+1 is in LDS (all waves' parts); everyone is done with tile t-1's stage
    if (STEADY) issue_full(t + NS - 1);
    else if (t + NS - 1 < n_tiles) issue(t + NS - 1);
    const unsigned char *st = smem_raw + (size_t)sidx * T::STAGE_BYTES;
    const unsigned char *st_next = smem_raw + (size_t)((sidx + 1) % NS) * T::STAGE_BYTES;
    const int k0 = k_lo + t * TK;

    bf16x8 kf[KK];
    {
      const unsigned char *skp = st_next + krow * ROWB;
#pragma unroll
      for (int kk = 0; kk < KK / 2; ++kk)
        kf[kk] = *reinterpret_cast<const bf16x8 *>(skp + (((2 * kk + lhi) ^ ksw) * 16));
    }
    if (!STEADY) {
      const int key_base = k0 + key_lane;
      if (k0 + TK > k_hi) {  // wave-uniform: only the last tile can hold keys past the end
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (key_base + 8 * (e / 4) + (e % 4) >= k_hi) s_cur[e] = -INFINITY;
      }
    }
    // running maximum of tile t (lazily moved reference)
    float mx = s_cur[0];
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s_cur[e]);
    mx = xhalf_max(mx) * sc;
    const bool need = mx > m_run + 8.0f;
    if (__any(need)) {
      // (rare after the first tiles) the accumulator changes its reference; the pending probabilities
      // of tile t-1 belong to the old one and are scaled with it (by 2^-8 at most, or by exactly 1)
      const float corr = need ? __builtin_amdgcn_exp2f(m_run - mx) : 1.0f;
      m_run = need ? mx : m_run;
      l_run *= corr;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_o[db][e] *= corr;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const uint4 w = __builtin_bit_cast(uint4, pf[ks]);
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
        uint32_t o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
          o[q] = pack_bf16(__uint_as_float(ww[q] << 16) * corr, __uint_as_float(ww[q] & 0xffff0000u) * corr);
        pf[ks] = __builtin_bit_cast(bf16x8, uint4{o[0], o[1], o[2], o[3]});
      }
    }
    const float neg_ref = (m_run == -INFINITY) ? 0.f : -m_run;

    // Sixteen matrix instructions -- P V of tile t-1, then the scores of tile t+1 -- each followed by
    // its share of tile t's exponentials; the V fragments of tile t are requested in between, into
    // the registers the first eight have released.
    // (after the last tile the score product reads a stage that holds no tile: the result is dropped)
    float arg[16], pe[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) arg[e] = fmaf(s_cur[e], sc, neg_ref);
    pv();
#pragma unroll
    for (int e = 0; e < 8; ++e) pe[e] = __builtin_amdgcn_exp2f(arg[e]);
    {
      const unsigned char *skp = st_next + krow * ROWB;
#pragma unroll
      for (int kk = KK / 2; kk < KK; ++kk)
        kf[kk] = *reinterpret_cast<const bf16x8 *>(skp + (((2 * kk + lhi) ^ ksw) * 16));
    }
    floatx16 s_next;
#pragma unroll
    for (int e = 0; e < 16; ++e) s_next[e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], s_next, 0, 0, 0);
#pragma unroll
    for (int e = 8; e < 16; ++e) pe[e] = __builtin_amdgcn_exp2f(arg[e]);
    // the row sum is taken over the rounded probabilities, the values the P V product uses
    // (one two-element dot product with (1, 1) per register instead of two additions)
    float ps0 = 0.f, ps1 = 0.f;
    uint32_t pw[8];
    const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3f803f80u);
#pragma unroll
    for (int e = 0; e < 16; e += 4) {
      pw[e >> 1] = pack_bf16(pe[e], pe[e + 1]);
      pw[(e >> 1) + 1] = pack_bf16(pe[e + 2], pe[e + 3]);
      ps0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pw[e >> 1]), ones, ps0, false);
      ps1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pw[(e >> 1) + 1]), ones, ps1, false);
    }
    float ps = ps0 + ps1;
    {
      const unsigned char *svp = st + T::REGION + vrow * ROWB + 8 * (lane % 4);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const unsigned char *p = svp + ks * 16 * ROWB + (((db * 2 + hb) ^ vsw) * 32);
          const shortx4 g0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(p));
          const shortx4 g1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(p + 8 * ROWB));
          const shortx8 av = __builtin_shufflevector(g0, g1, 0, 1, 2, 3, 4, 5, 6, 7);
          vf[ks][db] = __builtin_bit_cast(bf16x8, av);
        }
    }
    // instruction order
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // P V product
      __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);  // scale + shift of two scores
      __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);  // an exponential
      if (i == 3) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);  // the other four K reads
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // score product
      __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);  // an exponential
      __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);  // rounding and sum
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);   // the V reads of tile t
    ps = xhalf_sum(ps);
    l_run += ps;
    {
      const uint4 v0{pw[0], pw[1], pw[2], pw[3]}, v1{pw[4], pw[5], pw[6], pw[7]};
      pf[0] = __builtin_bit_cast(bf16x8, v0);
      pf[1] = __builtin_bit_cast(bf16x8, v1);
    }
    s_cur = s_next;
  };
  {
    int t = 0;
    const int n_steady = n_tiles - NS;  // tiles with a further fetch of a tile that is not the last (so: a full one)
    using dyn = std::integral_constant<int, -1>;
    static_assert(NS == 4, "the unrolled loop names the four stages");
    for (; t + NS <= n_steady; t += NS) {  // t % NS == 0 here
      body(t, std::true_type{}, std::integral_constant<int, 0>{});
      body(t + 1, std::true_type{}, std::integral_constant<int, 1>{});
      body(t + 2, std::true_type{}, std::integral_constant<int, 2>{});
      body(t + 3, std::true_type{}, std::integral_constant<int, 3>{});
    }
    for (; t < n_steady; ++t) body(t, std::true_type{}, dyn{});
    for (; t < n_tiles; ++t) body(t, std::false_type{}, dyn{});
  }
  pv();  // the last tile's
  }
  __syncthreads();  // every wave is done with the last tile: the stages become merge scratch

  // merge the WK wave columns of each query block through LDS
  float *mg = reinterpret_cast<float *>(smem_raw);
  constexpr int PER_WAVE = T::PER_WAVE;
  if (WK > 1 && wk > 0) {
    float *dst = mg + (size_t)((wk - 1) * WQ + wq) * PER_WAVE + lane;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) dst[(db * 16 + e) * 64] = acc_o[db][e];
    dst[(DB * 16) * 64] = m_run;
    dst[(DB * 16 + 1) * 64] = l_run;
  }
  if (WK > 1) __syncthreads();
  if (wk != 0) return;
  if (WK > 1) {
    float M = m_run;
#pragma unroll
    for (int w = 1; w < WK; ++w) M = fmaxf(M, mg[(size_t)((w - 1) * WQ + wq) * PER_WAVE + (DB * 16) * 64 + lane]);
    const float Ms = (M == -INFINITY) ? 0.f : M;
    const float c0 = __builtin_amdgcn_exp2f(m_run - Ms);
    float lsum = l_run * c0;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc_o[db][e] *= c0;
#pragma unroll
    for (int w = 1; w < WK; ++w) {
      const float *src = mg + (size_t)((w - 1) * WQ + wq) * PER_WAVE + lane;
      const float cw = __builtin_amdgcn_exp2f(src[(DB * 16) * 64] - Ms);
      lsum += src[(DB * 16 + 1) * 64] * cw;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_o[db][e] += src[(db * 16 + e) * 64] * cw;
    }
    m_run = M;
    l_run = lsum;
  }

  const int r = wq * 32 + l32;
  if (a.c_commit) {
    // Fused commit  [Alg. 3: cosine line and cache commit]: the row is normalised and rounded to the
    // storage type; this lane holds 64 of the head's 128 columns of its query.  It reads the same
    // columns of the cached context of the query's token, adds up <new, old>, |new|^2, |old|^2 over the
    // stored values, overwrites the cached columns, and the two lanes of a query leave the head's sums.
    float dot = 0.f, na = 0.f, nb = 0.f;
    const bool live = r < nq;  // (lanes past the tile's last row take part in the shuffle only)
    const int j = jq, h = hq;
    if (live) {
      const size_t tok = a.rows.idx ? (size_t)a.rows.idx[j] : (size_t)j;
      bf16_t *crow = (bf16_t *)a.c_commit + (tok * a.H + h) * DH + 4 * lhi;
      const float inv = 1.0f / l_run;
      uint2 old[DB][4];
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) old[db][g] = *reinterpret_cast<const uint2 *>(crow + db * 32 + 8 * g);
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint2 w;
          w.x = pack_bf16(acc_o[db][4 * g] * inv, acc_o[db][4 * g + 1] * inv);
          w.y = pack_bf16(acc_o[db][4 * g + 2] * inv, acc_o[db][4 * g + 3] * inv);
          const uint32_t nw[2] = {w.x, w.y}, ow[2] = {old[db][g].x, old[db][g].y};
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const float f0 = __uint_as_float(nw[q] << 16), f1 = __uint_as_float(nw[q] & 0xffff0000u);
            const float b0 = __uint_as_float(ow[q] << 16), b1 = __uint_as_float(ow[q] & 0xffff0000u);
            dot += f0 * b0 + f1 * b1;
            na += f0 * f0 + f1 * f1;
            nb += b0 * b0 + b1 * b1;
          }
          *reinterpret_cast<uint2 *>(crow + db * 32 + 8 * g) = w;
        }
      if (a.lse_out && lhi == 0) a.lse_out[tok * a.H + h] = m_run * LN2 + __logf(l_run);
    }
    dot += __shfl_xor(dot, 32, WAVE);
    na += __shfl_xor(na, 32, WAVE);
    nb += __shfl_xor(nb, 32, WAVE);
    if (live && lhi == 0)
      *reinterpret_cast<float4 *>(a.cos_part + ((size_t)j * a.H + h) * 4) = float4{dot, na, nb, 0.f};
    return;
  }
  if (r >= nq) return;
  const int j = jq, h = hq;
  if (a.splits == 1 && !a.partial) {
    bf16_t *out = (bf16_t *)a.out + ((size_t)j * a.H + h) * DH + 4 * lhi;
    const float inv = 1.0f / l_run;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack_bf16(acc_o[db][4 * g] * inv, acc_o[db][4 * g + 1] * inv);
        w.y = pack_bf16(acc_o[db][4 * g + 2] * inv, acc_o[db][4 * g + 3] * inv);
        *reinterpret_cast<uint2 *>(out + db * 32 + 8 * g) = w;
      }
  } else {
    float *po = a.part_o + (((size_t)split * a.rows.cap + j) * a.H + h) * DH + 4 * lhi;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 w{acc_o[db][4 * g], acc_o[db][4 * g + 1], acc_o[db][4 * g + 2], acc_o[db][4 * g + 3]};
        *reinterpret_cast<float4 *>(po + db * 32 + 8 * g) = w;
      }
    if (lhi == 0) {
      float *ml = a.part_ml + (((size_t)split * a.rows.cap + j) * a.H + h) * 2;
      ml[0] = m_run * LN2;  // partials carry the maximum in natural-log units
      ml[1] = l_run;
    }
  }
}

template <int WQ, int WK> void launch_dma(const AttnArgs &a, hipStream_t s) {
  using T = DTile<WQ, WK>;
  static bool done = false;
  if (!done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attn_bf16_dma<WQ, WK>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)T::LDS_BYTES);
    done = true;
  }
  const int q_tiles = max_q_tiles_grouped(a, T::BQ);
  k_attn_bf16_dma<WQ, WK><<<attn_grid_grouped(a, q_tiles), T::NT, T::LDS_BYTES, s>>>(a, q_tiles);
}

template <int DH, int WQ, int NW, int QB> void launch_cfg(const AttnArgs &a, hipStream_t s) {
  using T = ATile<DH, WQ, NW, QB>;
  static bool done = false;
  if (!done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attn_bf16<DH, WQ, NW, QB>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)T::LDS_BYTES);
    done = true;
  }
  const int q_tiles = max_q_tiles(a, T::BQ);
  k_attn_bf16<DH, WQ, NW, QB><<<attn_grid(a, q_tiles), T::NT, T::LDS_BYTES, s>>>(a, q_tiles);
}

}  // namespace

void launch_attention_bf16(const AttnArgs &a, hipStream_t s) {
  const bool wide = a.bq == 128;  // 128 or 64 query rows per workgroup
  if (a.dh == 128) {
    // 128 query rows: four waves, each with all keys of a 32-key tile (64 KB of LDS: two workgroups
    // per CU, which drift apart and fill each other's stalls); 64 rows: 2 x 2 waves over 64-key tiles
    if (wide) launch_dma<4, 1>(a, s); else launch_dma<2, 2>(a, s);
  } else {
    if (wide) launch_cfg<64, 2, 4, 2>(a, s); else launch_cfg<64, 1, 4, 2>(a, s);
  }
}

}  // namespace dy
