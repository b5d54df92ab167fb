// bf16 salient-row GEMM for the gfx950 matrix cores with asynchronous global -> LDS copies.
//   C[j,n] = sum_k A[row_j,k] * W[n,k]      (both operands K-contiguous)
//
// Weight layout.  W is stored in panels of 32 output rows, each panel K-slice-major:
//   W[n][k] lives at ((n/32) * (K/64) + k/64) * 2048 + (n%32) * 64 + k%64   (elements).
// The 128 bytes a tile row needs per K slice are then contiguous with those of the 31 other rows of
// its panel (4 KB), and a panel is read front to back while K advances: a workgroup that streams
// weights from HBM reads whole DRAM pages in order instead of one 128-byte piece per 8 KB row
// (measured at 106 rows on a 32-layer stack, whose weights always come from HBM: q/k/v GEMM 25.6 ->
// 23.7 us, gate|up 49.4 -> 46.2 us per layer against the row-major layout; a copy loop without
// products streams 6.0 TB/s from contiguous runs and 4.9-5.3 TB/s from 128-byte pieces).
//
// Data path.  K is cut into slices of 64 elements (128 bytes per tile row).  A slice of the
// (BM + BN) tile rows is copied straight from global memory into LDS by global_load_lds_dwordx4:
// every lane names its own 16-byte global source, the hardware writes lane i's data to
// LDS[M0 + 16*i].  One such instruction therefore fills 8 tile rows x 128 bytes.  No register is
// used for staging, so NS-1 slices can be in flight per workgroup while the MFMAs of the current
// slice run; the only synchronisation is one s_waitcnt vmcnt + one barrier per slice.  The 256-row
// tiles of the large regime use the same copies through buffer descriptors and keep five half
// slices in flight in a ring of LDS slots (gemm_bf16_ring.h).
//
// LDS layout.  Rows are 128 bytes, unpadded (the copy engine writes lanes back to back), with an
// XOR swizzle instead: the 16-byte chunk c of tile row r lives at chunk position c ^ ((r/2) % 8).
// The copy applies it on the global side (the lane that fills position p of row r fetches chunk
// p ^ ((r/2) % 8)), the MFMA operand reads apply it on the LDS side.  The LDS of gfx950 has 64 banks
// (256 bytes per clock) and serves a 16-byte-per-lane read 16 lanes at a time: 16 neighbouring
// lanes (16 rows, same k) then touch 8 different positions in each of the two 128-byte bank halves
// (even rows / odd rows) = all 64 banks once.
//
// MFMA.  v_mfma_f32_32x32x16_bf16: lane l supplies 8 consecutive k of row (l%32) for A and of
// column (l%32) for B at k offset 8*(l/32); the accumulator block holds
//   row = 8*(r/4) + 4*(l/32) + (r%4),  col = l%32   in register r of lane l.
//
// Tile walk.  The row count lives on the device; the grid is sized from the list capacity and each
// workgroup walks the existing tiles in a grouped order, remapped so that neighbouring tiles run on
// one XCD (workgroup i is dispatched to XCD i % 8) and share A / weight tiles in its L2.  A launch
// covers a window of list rows [row_lo, row_hi), so that a launcher can give a short last row tile
// to another tile shape in a launch of its own.
//
// Epilogues.  A wave's loads and stores complete in order, and a wave of the 256-row shapes is alone
// on its SIMD: a load issued behind stores (a residual, a register reloaded from scratch memory)
// returns only after all of them.  The epilogues therefore issue what they read ahead of the stores
// it could wait for, and the raw fp32 store of a K split is a compile-time form of the kernel (SPLIT)
// rather than a run-time branch beside the fused epilogue.
#pragma once
#include <type_traits>
#include "gemm_epilogues.h"
#include "kernels.h"

namespace dy {
namespace mm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int BK = 64;    // K slice (elements)
constexpr int ROWB = 128; // bytes per tile row and slice
constexpr int N_XCD = 8;
constexpr int WPANEL = 32;  // output rows per weight panel

}  // namespace mm
}  // namespace dy
#include "gemm_bf16_ring.h"
namespace dy {
namespace mm {

// Tile shape: BM x BN output tile, WAVES_M x WAVES_N waves, DUAL = two weight matrices per tile (fused
// gate/up), NS LDS stages of one K slice each.
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, bool DUAL_, int NS_> struct Shape {
  static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, NS = NS_;
  static constexpr bool DUAL = DUAL_;
  static constexpr int NMAT = DUAL ? 2 : 1;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int MB = WM / 32, NB = WN / 32;
  static constexpr int NW = WAVES_M * WAVES_N;  // waves per workgroup (4 or 8)
  static constexpr int NT = NW * 64;
  static constexpr int A_LD = BM / (8 * NW);  // copy instructions per wave and slice (8 rows each)
  static constexpr int B_LD = BN / (8 * NW);
  static constexpr int LPS = A_LD + NMAT * B_LD;  // copies per wave and slice
  static constexpr int A_BYTES = BM * ROWB, W_BYTES = NMAT * BN * ROWB;
  // four waves on a 256-row tile with 256 or 128 weight rows: the five-slot ring loop
  static constexpr bool RING = NW == 4 && BM == 256 && (NMAT * BN == 256 || NMAT * BN == 128) && NS == 2;
  static constexpr size_t LDS_BYTES = RING ? (size_t)RING_SLOTS * RING_SLOT : (size_t)NS * (A_BYTES + W_BYTES);
  // shapes with three or more stages (weight streaming) run the loop pipelined over slices
  static constexpr bool PIPE = NS >= 3;
  static_assert(NW == 4 || NW == 8, "four or eight waves per workgroup");
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 blocks");
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile rows are copied in blocks of 8 per wave");
  static_assert(NS >= 2 && NS <= 8, "LDS stages");
  static_assert((NS - 1) * LPS < 64, "vmcnt immediate");
  static_assert(PIPE || MB * NB * NMAT > 2, "two-stage shapes interleave operand reads with enough products");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS of one CU");
};

struct SplitStore {  // part != nullptr: raw fp32 tile part[z][j][n] instead of the fused epilogue
  float *part;
  size_t split_stride;
  int N;
};

// SPLIT: the tile goes to the raw fp32 result part[z][j][n] (split.part) instead of through the
// fused epilogue.  A compile-time switch: with both forms behind a run-time branch the compiler
// moves the accumulators out of the accumulation registers ahead of the branch, where they do not
// fit, and the epilogue's stores each wait for a reload from scratch memory.
template <typename SH, typename Epi, bool SPLIT>
__global__ __launch_bounds__(SH::NT) void k_gemm_bf16(const bf16_t *__restrict__ A,
                                                   const int32_t *__restrict__ gather, int lda,
                                                   Rows rows, int N, WSeg seg,
                                                   const bf16_t *__restrict__ W2, int ldw, int kchunk,
                                                   int group_m, Epi epi, SplitStore split,
                                                   int row_lo, int row_hi) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  constexpr int BM = SH::BM, BN = SH::BN, MB = SH::MB, NB = SH::NB, NMAT = SH::NMAT, NS = SH::NS, NW = SH::NW;

  // rows [row_lo, min(count, row_hi)) of the list are this launch's; row_lo is a multiple of BM
  const int M = min(rows.count ? min(*rows.count, rows.cap) : rows.cap, row_hi);
  const int tm_lo = row_lo / BM;
  const int m_rel = max(M - tm_lo * BM, 0);
  const int tiles_m = (m_rel + BM - 1) / BM, tiles_n = N / BN;
  const int tid = threadIdx.x, lane = tid % WAVE;
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);  // wave-uniform, kept scalar
  const int wm0 = (wave / SH::WAVES_N) * SH::WM, wn0 = (wave % SH::WAVES_N) * SH::WN;
  const int l32 = lane % 32, lhi = lane / 32;
  const int z = blockIdx.y;  // K split
  const int kbeg = z * kchunk;
  const int KT = kchunk / BK;
  const uint32_t lds0 = lds_offset_of(smem_raw);

  // copy mapping of this lane inside an 8-row block: tile row r8, chunk position p, source chunk c
  const int r8 = lane / 8, cpos = lane % 8;
  // tile row of this lane in copy i is (i*NW + wave)*8 + r8, so (row/2) % 8 = ((wave & 1) * 4 + r8 / 2)
  const int csrc = cpos ^ (((wave & 1) << 2) | (r8 >> 1));
  // operand-read swizzle of this lane: chunk position of logical chunk (2*kk + lhi)
  int rd_off[BK / 16];
#pragma unroll
  for (int kk = 0; kk < BK / 16; ++kk) rd_off[kk] = (((2 * kk + lhi) ^ ((l32 >> 1) & 7)) * 16);

  // Tile order.  Workgroup p runs on XCD p % 8, and an XCD takes its workgroups in the order of p.
  // Each XCD gets a contiguous run of the FULL row tiles' tiles (walked in groups of group_m row tiles,
  // so that the tiles it runs at one time share operands in its L2) and, after those, its share of
  // the tiles of a last row tile that holds fewer than BM rows: those cost a fraction of a full tile
  // (see the partial loop below) and fill the end of every XCD's schedule instead of one XCD's.
  const int has_tail = (m_rel % BM != 0) ? 1 : 0;
  const int rows_full = tiles_m - has_tail;
  const int n_full = rows_full * tiles_n, n_part = has_tail * tiles_n;
  const int fx = (n_full + N_XCD - 1) / N_XCD, px = (n_part + N_XCD - 1) / N_XCD;
  const int total_pad = (fx + px) * N_XCD;

  // tile (tm, tn) of position p in that order; false for the padding positions (uniform for the
  // workgroup)
  auto tile_at = [&](int p, int &tm, int &tn) -> bool {
    const int xcd = p % N_XCD, q = p / N_XCD;
    if (q < fx) {
      const int logical = xcd * fx + q;
      if (logical >= n_full) return false;
      const int gsz = group_m * tiles_n;
      const int g = logical / gsz, r = logical % gsz;
      const int gm = min(group_m, rows_full - g * group_m);
      tm = g * group_m + r % gm;
      tn = r / gm;
    } else {
      const int lp = xcd * px + (q - fx);
      if (lp >= n_part) return false;
      tm = tiles_m - 1;
      tn = lp;
    }
    return true;
  };

  // Epilogue of one tile: the accumulators of this wave go through the fused epilogue (or, for a K
  // split, into the raw partial result).
  auto epilogue = [&](floatx16 (&acc)[NMAT][MB][NB], int m0, int n0, int tn) {
    if constexpr (Epi::INTERLEAVE == 48) {
      // 32 x 96 wave tile = columns [0,48) of matrix 0 (gate) and [48,96) of matrix 1 (up): gate
      // column c pairs with tile column c + 48, which lane (c%32) ^ 16 holds one or two blocks on
      static_assert(NB == 3 && SH::WAVES_N == 1 && NMAT == 1, "half-interleaved tiles are 96 columns of one wave");
      const bool hi16 = (l32 & 16) != 0;
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = m0 + wm0 + i * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
          const float a0 = acc[0][i][0][e], a1 = acc[0][i][1][e], a2 = acc[0][i][2][e];
          const float up0 = __shfl_xor(hi16 ? a1 : a2, 16, WAVE);  // up value of gate column l32
          const float up1 = __shfl_xor(a2, 16, WAVE);              // lanes 0..15: up value of gate column 32 + l32
          if (j < M) {
            epi.store(j, tn * 48 + l32, a0, up0);
            if (!hi16) epi.store(j, tn * 48 + 32 + l32, a1, up1);
          }
        }
    } else if constexpr (Epi::INTERLEAVE == 64) {
      // 32 x 128 wave tile = 64 gate + 64 up columns: the partner of a gate column is two blocks on
      // in the same lane
      static_assert(NB == 4 && SH::WAVES_N == 1 && NMAT == 1, "half-interleaved tiles are 128 columns of one wave");
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = m0 + wm0 + i * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
          if (j < M) {
            epi.store(j, tn * 64 + l32, acc[0][i][0][e], acc[0][i][2][e]);
            epi.store(j, tn * 64 + 32 + l32, acc[0][i][1][e], acc[0][i][3][e]);
          }
        }
    } else if (m0 + BM <= M) {
      // Full tile: no row checks, and every address is a wave-uniform base (scalar registers) plus a
      // byte offset per lane that is fixed for the tile.
      const int rbase = m0 + wm0, cbase = n0 + wn0;  // wave-uniform
      if constexpr (SPLIT) {
        float *pz = split.part + (size_t)z * split.split_stride;
        const uint32_t lb = ((uint32_t)(4 * lhi) * split.N + l32) * 4u;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float *r = pz + (size_t)(rbase + i * 32 + 8 * (e / 4) + (e % 4)) * split.N + cbase;
#pragma unroll
            for (int jn = 0; jn < NB; ++jn)
              *reinterpret_cast<float *>(reinterpret_cast<char *>(r + jn * 32) + lb) = acc[0][i][jn][e];
          }
      } else if constexpr (Epi::PRELOAD) {
        // A step of RS rows at a time: what the epilogue reads, then what it writes.  The reads of
        // step u + 1 are issued before the stores of step u: a wave's memory operations complete
        // in order, so a load behind stores would wait for all of them.
        constexpr int RS = NB >= 4 ? 8 : 16, STEPS = MB * 16 / RS;
        struct Pre {
          float v[RS][NB];
          int row[RS];
        };
        const uint32_t lbh = epi.lane_bytes_h(lhi, l32), lbo = epi.lane_bytes(lhi, l32);
        const int ld = epi.ld();
        auto row_of = [&](int u, int x) { return rbase + ((u * RS + x) / 16) * 32 + 8 * (((u * RS + x) % 16) / 4) + (x % 4); };
        auto load = [&](int u, Pre &p) {
#pragma unroll
          for (int x = 0; x < RS; ++x) {
            const int rr = row_of(u, x);
            p.row[x] = rows.idx ? *reinterpret_cast<const int *>(reinterpret_cast<const char *>(rows.idx + rr) + 16 * lhi) : 0;
#pragma unroll
            for (int jn = 0; jn < NB; ++jn) p.v[x][jn] = epi.get((size_t)rr * ld + cbase + jn * 32, lbh);
          }
        };
        Pre cur;
        load(0, cur);
#pragma unroll
        for (int u = 0; u < STEPS; ++u) {
          Pre nxt;
          if (u + 1 < STEPS) load(u + 1, nxt);
#pragma unroll
          for (int x = 0; x < RS; ++x) {
            const int i = (u * RS + x) / 16, e = (u * RS + x) % 16;
            if (rows.idx) {
              auto *o = epi.row_ptr(cur.row[x], cbase + l32);
#pragma unroll
              for (int jn = 0; jn < NB; ++jn) o[jn * 32] = from_f<std::remove_reference_t<decltype(o[0])>>(cur.v[x][jn] + acc[0][i][jn][e]);
            } else {
#pragma unroll
              for (int jn = 0; jn < NB; ++jn) epi.put((size_t)row_of(u, x) * ld + cbase + jn * 32, lbo, acc[0][i][jn][e], cur.v[x][jn]);
            }
          }
          if (u + 1 < STEPS) cur = nxt;
        }
      } else {
        const uint32_t lbo = epi.lane_bytes(lhi, l32);
        const int ld = epi.ld();
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const size_t u = (size_t)(rbase + i * 32 + 8 * (e / 4) + (e % 4)) * ld + cbase;
#pragma unroll
            for (int jn = 0; jn < NB; ++jn) epi.put(u + jn * 32, lbo, acc[0][i][jn][e], acc[NMAT - 1][i][jn][e]);
          }
      }
    } else if constexpr (Epi::PRELOAD) {
      if constexpr (!SPLIT) {
      // a 32-row block at a time: what the epilogue reads, then what it writes (two blocks in
      // flight cost more registers than the four-wave shapes have left: measured slower)
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        float pre[16][NB];
        int rowv[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = m0 + wm0 + i * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
          rowv[e] = (j < M && rows.idx) ? rows.idx[j] : j;
#pragma unroll
          for (int jn = 0; jn < NB; ++jn) pre[e][jn] = j < M ? epi.load(j, n0 + wn0 + jn * 32 + l32) : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = m0 + wm0 + i * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
          if (j < M) {
#pragma unroll
            for (int jn = 0; jn < NB; ++jn) epi.store(rowv[e], n0 + wn0 + jn * 32 + l32, acc[0][i][jn][e], pre[e][jn]);
          }
        }
      }
      } else {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int j = m0 + wm0 + i * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
            if (j < M) {
#pragma unroll
              for (int jn = 0; jn < NB; ++jn)
                split.part[(size_t)z * split.split_stride + (size_t)j * split.N + n0 + wn0 + jn * 32 + l32] =
                    acc[0][i][jn][e];
            }
          }
      }
    } else
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int j = m0 + wm0 + i * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
        if (j < M) {
          if constexpr (SPLIT) {
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
  };

  if constexpr (SH::RING) {
    // Four-wave ring shapes.  The workgroup walks its tiles itself (the launcher starts one per CU),
    // and the ring is refilled for the next tile before the epilogue of the current one, so that
    // the first slices of a tile land while the previous tile's results are written.
    using RingFull = Ring<NMAT, NB, BN, 4>;
    constexpr int NWC = RingFull::NWC;
    static_assert(Epi::INTERLEAVE == 0 && SH::A_LD == 8 && NMAT * SH::B_LD == NWC, "ring shapes");
    auto ring_sources = [&](int tm, int tn, RingSrc &src) {
      const int m0 = (tm_lo + tm) * BM, n0 = tn * BN;
      // Lane offsets are 32 bits.  Without a gather list the descriptor starts at the tile's first
      // row, so the offsets stay below 256 rows; with one they are taken from the start of the
      // operand (the launcher checks that it spans less than 4 GiB).
      src.srd_a = make_srd(gather ? A : A + (size_t)m0 * lda, 0xfffffff0u);
      // (the eight list entries of a gathered operand are loaded back to back, then used)
      int srow[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int j = m0 + (i * NW + wave) * 8 + r8;
        srow[i] = j < M ? j : M - 1;  // rows past the end are clamped; their results are never stored
      }
      if (gather) {
#pragma unroll
        for (int i = 0; i < 8; ++i) srow[i] = gather[srow[i]];
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) srow[i] -= m0;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) src.va[i] = (uint32_t)(((size_t)srow[i] * lda + kbeg + csrc * 8) * 2);
#pragma unroll
      for (int c = 0; c < NWC; ++c) {
        const int t = c / SH::B_LD, i = c % SH::B_LD;
        const int nrow0 = (i * NW + wave) * 8;  // first of the copy's 8 tile rows (wave-uniform)
        const int nu = n0 + nrow0;
        // a copy's rows lie in one matrix: segment ends are multiples of 8
        const bool in1 = nu >= seg.n_end[0], in2 = nu >= seg.n_end[1];
        const void *base = t == 1 ? (const void *)W2 : in2 ? seg.w[2] : in1 ? seg.w[1] : seg.w[0];
        const int nl = nu + r8 - (t == 1 ? 0 : in2 ? seg.n_end[1] : in1 ? seg.n_end[0] : 0);
        src.srd_w[c] = make_srd(base, 0xfffffff0u);
        src.vw[c] = (uint32_t)((((size_t)(nl / WPANEL) * (ldw / BK) + kbeg / BK) * (WPANEL * BK) + (nl % WPANEL) * BK + csrc * 8) * 2);
      }
    };
    int tm = 0, tn = 0, p = blockIdx.x;
    while (p < total_pad && !tile_at(p, tm, tn)) p += gridDim.x;
    if (p >= total_pad) return;
    RingSrc src;
    ring_sources(tm, tn, src);
    RingFull::fill(src, lds0, wave);
    bool all_landed = false;
    const unsigned char *rd_a = smem_raw + (wm0 + l32) * ROWB, *rd_w = smem_raw + (wn0 + l32) * ROWB;
    for (;;) {
      const int m0 = (tm_lo + tm) * BM, n0 = tn * BN;
      floatx16 acc[NMAT][MB][NB];
#pragma unroll
      for (int t = 0; t < NMAT; ++t)
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][i][j][e] = 0.f;
      auto run_ring = [&](auto mbv_c) {
        Ring<NMAT, NB, BN, decltype(mbv_c)::value>::tile(acc, lds0, wave, src, rd_a, rd_w, rd_off, KT, all_landed);
      };
      // 32-row blocks of this wave that hold rows (wave-uniform)
      const int mbv = (M - (m0 + wm0) + 31) / 32;
      if (mbv >= 3) run_ring(std::integral_constant<int, 4>{});
      else if (mbv == 2) run_ring(std::integral_constant<int, 2>{});
      else if (mbv == 1) run_ring(std::integral_constant<int, 1>{});
      else run_ring(std::integral_constant<int, 0>{});
      int pn = p + gridDim.x, tmn = 0, tnn = 0;
      while (pn < total_pad && !tile_at(pn, tmn, tnn)) pn += gridDim.x;
      const bool more = pn < total_pad;
      if (more) {
        ring_sources(tmn, tnn, src);
        RingFull::fill(src, lds0, wave);
      }
      epilogue(acc, m0, n0, tn);
      if (!more) break;
      p = pn; tm = tmn; tn = tnn;
      all_landed = true;
    }
    return;
  }

  for (int p = blockIdx.x; p < total_pad; p += gridDim.x) {
    int tm, tn;
    if (!tile_at(p, tm, tn)) continue;
    const int m0 = (tm_lo + tm) * BM, n0 = tn * BN;

    // per-lane global sources of the copies it issues every slice
    const bf16_t *ap[SH::A_LD];
#pragma unroll
    for (int i = 0; i < SH::A_LD; ++i) {
      int j = m0 + (i * NW + wave) * 8 + r8;
      j = j < M ? j : M - 1;  // rows past the end are clamped; their results are never stored
      const int src = gather ? gather[j] : j;
      ap[i] = A + (size_t)src * lda + kbeg + csrc * 8;
    }
    // a column tile may span two of the stacked weight matrices: the matrix is looked up per row
    const bf16_t *wp[NMAT][SH::B_LD];
#pragma unroll
    for (int i = 0; i < SH::B_LD; ++i) {
      const int nrow = (i * NW + wave) * 8 + r8;
      const int n = n0 + nrow;
      const bf16_t *wbase;
      int nl;  // row inside its matrix
      if constexpr (Epi::INTERLEAVE > 0) {
        // tile tn = HALF rows of matrix 0 followed by the same HALF rows of matrix 1
        constexpr int HALF = Epi::INTERLEAVE;
        static_assert(BN == 2 * HALF, "one half tile per matrix");
        const bool second = nrow >= HALF;
        wbase = (const bf16_t *)(second ? seg.w[1] : seg.w[0]);
        nl = tn * HALF + (second ? nrow - HALF : nrow);
      } else {
        const bool in1 = n >= seg.n_end[0], in2 = n >= seg.n_end[1];
        wbase = (const bf16_t *)(in2 ? seg.w[2] : in1 ? seg.w[1] : seg.w[0]);
        nl = n - (in2 ? seg.n_end[1] : in1 ? seg.n_end[0] : 0);
      }
      // panel layout: slice kt of this row sits kt * (WPANEL * BK) elements further on
      const size_t woff = ((size_t)(nl / WPANEL) * (ldw / BK) + kbeg / BK) * (WPANEL * BK) + (nl % WPANEL) * BK + csrc * 8;
      wp[0][i] = wbase + woff;
      if (SH::DUAL)
        wp[NMAT - 1][i] = W2 + ((size_t)(n / WPANEL) * (ldw / BK) + kbeg / BK) * (WPANEL * BK) + (n % WPANEL) * BK + csrc * 8;
    }

    floatx16 acc[NMAT][MB][NB];
#pragma unroll
    for (int t = 0; t < NMAT; ++t)
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[t][i][j][e] = 0.f;

    // LDS: NS stages of the A tile, then NS stages of the weight tile(s)
    auto issue_a = [&](int kt) {  // A rows of slice kt -> A stage kt % NS
      const uint32_t sb = lds0 + (uint32_t)(kt % NS) * SH::A_BYTES + (uint32_t)wave * 1024u;
      const int ko = kt * BK;
#pragma unroll
      for (int i = 0; i < SH::A_LD; ++i) dma16(ap[i] + ko, sb + i * (NW * 1024u));
    };
    auto issue_w = [&](int kt) {  // weight rows of slice kt -> weight stage kt % NS
      const uint32_t sb = lds0 + (uint32_t)(NS * SH::A_BYTES) + (uint32_t)(kt % NS) * SH::W_BYTES +
                          (uint32_t)wave * 1024u;
      const int ko = kt * (WPANEL * BK);
#pragma unroll
      for (int t = 0; t < NMAT; ++t)
#pragma unroll
        for (int i = 0; i < SH::B_LD; ++i) dma16(wp[t][i] + ko, sb + (uint32_t)(t * BN) * ROWB + i * (NW * 1024u));
    };

    __syncthreads();  // LDS free: the previous tile of this workgroup is fully consumed
    if constexpr (SH::PIPE) {
      // Weight-streaming shapes: one wave per SIMD and few products per slice, so nothing hides the
      // chain wait -> barrier -> operand reads -> products of a slice.  The loop is therefore
      // pipelined over slices: the operands of slice kt+1 are read (into a second register set)
      // while the products of slice kt run, and because a wave holds slice kt in registers when it
      // reaches the barrier of iteration kt, that stage is refilled at once: NS slices are in flight
      // instead of NS-1.
      // Few rows: only the first ALD of a wave's A_LD copies per slice hold rows below M (copy i of
      // wave w fills rows (i*NW + w)*8 ...), the others are left out -- with at most 64 (32) rows that
      // halves (quarters) the activation traffic from L2, which competes with the weight stream.
      // Tile rows that are never filled only feed results that are never stored.
      auto pipe_loop = [&](auto ald_c) {
      constexpr int ALD = decltype(ald_c)::value;
      constexpr int LPS = ALD + NMAT * SH::B_LD;  // copies per wave and slice
      auto issue_a_n = [&](int kt) {
        const uint32_t sb = lds0 + (uint32_t)(kt % NS) * SH::A_BYTES + (uint32_t)wave * 1024u;
        const int ko = kt * BK;
#pragma unroll
        for (int i = 0; i < ALD; ++i) dma16(ap[i] + ko, sb + i * (NW * 1024u));
      };
      constexpr int KS = BK / 16, RD = MB + NMAT * NB, MM = NMAT * MB * NB;
      bf16x8 af[2][KS][MB], bfr[2][KS][NMAT][NB];
      auto read_slice = [&](bf16x8 (&a)[KS][MB], bf16x8 (&b)[KS][NMAT][NB], int kt) {
        const unsigned char *sa = smem_raw + (size_t)(kt % NS) * SH::A_BYTES + (wm0 + l32) * ROWB;
        const unsigned char *sb = smem_raw + (size_t)NS * SH::A_BYTES + (size_t)(kt % NS) * SH::W_BYTES +
                                  (wn0 + l32) * ROWB;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
#pragma unroll
          for (int i = 0; i < MB; ++i) a[kk][i] = *reinterpret_cast<const bf16x8 *>(sa + i * 32 * ROWB + rd_off[kk]);
#pragma unroll
          for (int t = 0; t < NMAT; ++t)
#pragma unroll
            for (int j = 0; j < NB; ++j)
              b[kk][t][j] = *reinterpret_cast<const bf16x8 *>(sb + (t * BN + j * 32) * ROWB + rd_off[kk]);
        }
      };
      auto slice = [&](int kt, auto cur_c) {
        constexpr int CUR = decltype(cur_c)::value;
        // slice kt+1 has landed: the copies issued after it may still be on their way
        if (kt + NS - 1 < KT) wait_vmcnt<(NS - 2) * LPS>();
        else wait_vmcnt<0>();
        wait_lgkmcnt0();  // the operands of slice kt are in registers: its stage is free
        __syncthreads();
        if (kt + NS < KT) { issue_a_n(kt + NS); issue_w(kt + NS); }
        read_slice(af[CUR ^ 1], bfr[CUR ^ 1], kt + 1 < KT ? kt + 1 : kt);  // (past the end: a harmless re-read)
#pragma unroll
        for (int kk = 0; kk < KS; ++kk)
#pragma unroll
          for (int t = 0; t < NMAT; ++t)
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
              for (int j = 0; j < NB; ++j)
                acc[t][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[CUR][kk][i], bfr[CUR][kk][t][j], acc[t][i][j], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, KS * RD, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, KS * MM, 0);
        __builtin_amdgcn_sched_barrier(0);
      };
#pragma unroll
      for (int s = 0; s < NS; ++s)
        if (s < KT) { issue_a_n(s); issue_w(s); }
      if (NS - 1 < KT) wait_vmcnt<(NS - 1) * LPS>();  // slice 0 has landed
      else wait_vmcnt<0>();
      __syncthreads();
      read_slice(af[0], bfr[0], 0);
      int kt = 0;
      for (; kt + 1 < KT; kt += 2) {
        slice(kt, std::integral_constant<int, 0>{});
        slice(kt + 1, std::integral_constant<int, 1>{});
      }
      if (kt < KT) slice(kt, std::integral_constant<int, 0>{});
      };
      const int a_need = (M - m0 + 8 * NW - 1) / (8 * NW);  // copies per wave that hold rows
      if (SH::A_LD >= 4 && a_need <= 1) pipe_loop(std::integral_constant<int, 1>{});
      else if (SH::A_LD >= 2 && a_need <= SH::A_LD / 2) pipe_loop(std::integral_constant<int, (SH::A_LD >= 2 ? SH::A_LD / 2 : 1)>{});
      else pipe_loop(std::integral_constant<int, SH::A_LD>{});
    } else if (NS == 2 && m0 + BM > M) {
      // A row tile that holds fewer than BM rows: copies of 8-row blocks past the end are left out,
      // and a wave multiplies only its 32-row blocks that hold rows (none at all for many waves), so
      // that the tile costs about what its weight copies cost.  Same barriers as the full loop.
      const int mbv_raw = (M - (m0 + wm0) + 31) / 32;
      const int mbv = mbv_raw < 0 ? 0 : (mbv_raw > MB ? MB : mbv_raw);  // wave-uniform
      auto issue_a_part = [&](int kt) {
        const uint32_t sb = lds0 + (uint32_t)(kt % NS) * SH::A_BYTES + (uint32_t)wave * 1024u;
        const int ko = kt * BK;
#pragma unroll
        for (int i = 0; i < SH::A_LD; ++i)
          if (m0 + (i * NW + wave) * 8 < M) dma16(ap[i] + ko, sb + i * (NW * 1024u));
      };
      issue_a_part(0);
      issue_w(0);
      for (int kt = 0; kt < KT; ++kt) {
        wait_vmcnt<0>();
        __syncthreads();
        if (kt + 1 < KT) {
          issue_a_part(kt + 1);
          issue_w(kt + 1);
        }
        if (mbv == 0) continue;  // wave-uniform; the barriers above are all this wave owes the tile
        const unsigned char *sa = smem_raw + (size_t)(kt % NS) * SH::A_BYTES + (wm0 + l32) * ROWB;
        const unsigned char *sb = smem_raw + (size_t)NS * SH::A_BYTES + (size_t)(kt % NS) * SH::W_BYTES +
                                  (wn0 + l32) * ROWB;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
          bf16x8 bfr[NMAT][NB];
#pragma unroll
          for (int t = 0; t < NMAT; ++t)
#pragma unroll
            for (int j = 0; j < NB; ++j)
              bfr[t][j] = *reinterpret_cast<const bf16x8 *>(sb + (t * BN + j * 32) * ROWB + rd_off[kk]);
#pragma unroll
          for (int i = 0; i < MB; ++i) {
            if (i < mbv) {
              const bf16x8 af = *reinterpret_cast<const bf16x8 *>(sa + i * 32 * ROWB + rd_off[kk]);
#pragma unroll
              for (int t = 0; t < NMAT; ++t)
#pragma unroll
                for (int j = 0; j < NB; ++j)
                  acc[t][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr[t][j], acc[t][i][j], 0, 0, 0);
            }
          }
        }
      }
    } else {
    // slice by slice
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
      if (s < KT) { issue_a(s); issue_w(s); }

    for (int kt = 0; kt < KT; ++kt) {
      // slice kt has landed (this wave's part); a wave's copies complete in issue order
      if (kt + NS - 2 < KT) wait_vmcnt<(NS - 2) * SH::LPS>();
      else wait_vmcnt<0>();
      __syncthreads();  // ... all waves' parts; and everyone is done with slice kt-1
      if (kt + NS - 1 < KT) { issue_a(kt + NS - 1); issue_w(kt + NS - 1); }  // into the stage slice kt-1 left

      const unsigned char *sa = smem_raw + (size_t)(kt % NS) * SH::A_BYTES + (wm0 + l32) * ROWB;
      const unsigned char *sb = smem_raw + (size_t)NS * SH::A_BYTES + (size_t)(kt % NS) * SH::W_BYTES +
                                (wn0 + l32) * ROWB;
      // operand fragments of slice step kk+1 are fetched while the MFMAs of step kk run
      bf16x8 af[2][MB], bfr[2][NMAT][NB];
#pragma unroll
      for (int i = 0; i < MB; ++i) af[0][i] = *reinterpret_cast<const bf16x8 *>(sa + i * 32 * ROWB + rd_off[0]);
#pragma unroll
      for (int t = 0; t < NMAT; ++t)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          bfr[0][t][j] = *reinterpret_cast<const bf16x8 *>(sb + (t * BN + j * 32) * ROWB + rd_off[0]);
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        const int c = kk & 1, n = c ^ 1;
        if (kk + 1 < BK / 16) {
#pragma unroll
          for (int i = 0; i < MB; ++i)
            af[n][i] = *reinterpret_cast<const bf16x8 *>(sa + i * 32 * ROWB + rd_off[kk + 1]);
#pragma unroll
          for (int t = 0; t < NMAT; ++t)
#pragma unroll
            for (int j = 0; j < NB; ++j)
              bfr[n][t][j] = *reinterpret_cast<const bf16x8 *>(sb + (t * BN + j * 32) * ROWB + rd_off[kk + 1]);
        }
#pragma unroll
        for (int t = 0; t < NMAT; ++t)
#pragma unroll
          for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
              acc[t][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[c][i], bfr[c][t][j], acc[t][i][j], 0, 0, 0);
      }
      // Instruction order of the slice: the first step's operand reads, then the LDS reads of step
      // kk+1 spread one by one between the MFMAs of step kk (the scheduler alone fetches each
      // operand right before its use and leaves the matrix pipe waiting on the LDS).
      {
        constexpr int RD = MB + NMAT * NB, MM = NMAT * MB * NB;
        __builtin_amdgcn_sched_group_barrier(0x100, RD, 0);
#pragma unroll
        for (int kk = 0; kk + 1 < BK / 16; ++kk) {
#pragma unroll
          for (int q = 0; q < RD; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          }
          if (MM > RD) __builtin_amdgcn_sched_group_barrier(0x008, MM - RD, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, MM, 0);
      }
    }
    }

    epilogue(acc, m0, n0, tn);
  }
}

template <typename SH, typename Epi, bool SPLIT> void set_lds_once() {
  static bool done = false;
  if (!done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_bf16<SH, Epi, SPLIT>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::LDS_BYTES);
    done = true;
  }
}

}  // namespace mm
}  // namespace dy
