// bf16 salient-row GEMMs: tile-shape choice per regime and the four fused launchers.
#include <algorithm>
#include <climits>
#include <cstdlib>
#include "gemm_bf16_dma.h"

namespace dy {

using namespace mm;

namespace {

// Tile shapes per regime (rows = capacity of the row list):
//  xlarge  256 x 256 tile (256 x (128+128) when gate and up are fused), four waves of 128 x 128 over
//          a ring of five LDS slots: a third fewer bytes per flop through the CU's L1 -> LDS path
//          than a 256 x 128 tile and half the LDS operand reads; taken when its coarser tiles still
//          fill the rounds of the chip and every operand can be addressed with 32-bit offsets
//  large   256 x 128 tile (256 x (64+64) when gate and up are fused), the same ring loop with two
//          column blocks per wave; eight waves over two LDS stages when the operand cannot be
//          addressed that way
//  skinny  all rows in one 128-row tile, 64-column tiles, 4 stages in flight and a K split so that
//          about one workgroup per CU streams weights (weight-streaming-bound regime)
typedef Shape<256, 256, 2, 2, false, 2> XLargeS;
typedef Shape<256, 128, 2, 2, true, 2> XLargeD;
typedef Shape<256, 128, 2, 2, false, 2> LargeS;
typedef Shape<256, 64, 2, 2, true, 2> LargeD;
typedef Shape<256, 128, 4, 2, false, 2> LargeS8;  // eight waves, two LDS stages
typedef Shape<256, 64, 4, 2, true, 2> LargeD8;
typedef Shape<128, 64, 4, 2, false, 4> SkinnyS;
// skinny regime, wide column tiles (fewer re-reads of the activation tile): q|k|v raw result, and
// gate|up with half-interleaved tiles (48 + 48 or 64 + 64 columns) and SwiGLU in registers
typedef Shape<128, 96, 4, 1, false, 4> SkinnyW96;
typedef Shape<128, 128, 4, 1, false, 4> SkinnyH128;

constexpr int SKINNY_MAX_ROWS = 128;

int cu_count() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
  }
  return n;
}

// Rounds of the chip (one workgroup per CU at a time) that `cap` rows in 256-row tiles take with
// ncol column tiles and sk K-splits.  The tiles of a last row tile with fewer than 256 rows cost a
// fraction f of a full tile (they still walk all of K with their weight copies: measured at 0.55-0.6 of
// a full tile for a few rows; more with the products of the busiest wave's 32-row blocks); they run
// at the end of every XCD's schedule and first fill the slots the last round of full tiles leaves idle.
double tile_rounds(int cap, long ncol, int sk) {
  const long cu = cu_count(), rows_full = cap / 256;
  const int tail = cap % 256;
  const long full_tiles = rows_full * ncol * sk;
  const long full_rounds = (full_tiles + cu - 1) / cu;
  if (!tail) return (double)full_rounds;
  const double f = std::max(0.55, (double)((tail + 31) / 32) / 8.0);
  const long slack = full_rounds * cu - full_tiles;
  long rest = ncol * sk - slack * (long)(1.0 / f);
  if (rest < 0) rest = 0;
  return (double)full_rounds + (double)((rest + cu - 1) / cu) * f;
}

// 256-row tiles with n_l (large) or n_x (xlarge, twice as wide) column tiles: an xlarge tile takes
// about 1.65 times as long as a large one (measured at many rounds).
constexpr double XLARGE_COST = 1.65;
bool prefer_xlarge(int cap, int n_l, int n_x) {
  return XLARGE_COST * tile_rounds(cap, n_x, 1) < tile_rounds(cap, n_l, 1);
}

// The ring loop addresses its operands with a scalar base and 32-bit byte offsets per lane.  The base
// of the activation operand moves with the tile unless rows are gathered: a gathered operand, and
// each weight matrix, must span less than 4 GiB, and a copy's 8 weight rows must lie in one matrix;
// otherwise the eight-wave 256 x 128 shapes run.  (Every K split of the plans keeps at least 8
// slices; the loop needs 3.)
// DYLLM_GEMM_NO_RING=1 in the environment takes the fallback for every call (diagnostics and tests).
bool ring_ok(const GemmA &A, const Rows &rows, int K, const WSeg &seg, int n_rows_w) {
  (void)rows;
  if (const char *e = getenv("DYLLM_GEMM_NO_RING"))
    if (e[0] == '1') return false;
  const size_t lim = ((size_t)1 << 32) - ((size_t)1 << 20);
  if (A.gather && (A.a_rows == 0 || A.a_rows * (size_t)A.lda * 2 >= lim)) return false;
  if ((size_t)A.lda * 2 * 256 >= lim) return false;
  if ((size_t)n_rows_w * (size_t)K * 2 >= lim) return false;
  if (seg.n_end[0] % 8 || seg.n_end[1] % 8) return false;
  return K / BK >= RING_MIN_SLICES;
}

// Which forms of the kernel an epilogue is launched in: the raw fp32 store (SPLIT), the fused
// epilogue, or either (the down projection, with and without a K split).
template <typename Epi> struct SplitForms { static constexpr bool raw = false, fused = true; };
template <> struct SplitForms<EpiStoreF32> { static constexpr bool raw = true, fused = false; };
template <typename T> struct SplitForms<EpiDown<T>> { static constexpr bool raw = true, fused = true; };

template <typename SH, typename Epi, bool SPLIT>
void launch_tiles(dim3 grid, GemmA A, Rows rows, int K, int N, WSeg seg, const void *w2, Epi epi, int splitk,
                  SplitStore sp, hipStream_t s, int row_lo, int row_hi) {
  set_lds_once<SH, Epi, SPLIT>();
  k_gemm_bf16<SH, Epi, SPLIT><<<grid, SH::NT, SH::LDS_BYTES, s>>>(
      (const bf16_t *)A.a, A.gather, A.lda, rows, N, seg, (const bf16_t *)w2, K, K / splitk,
      /*group_m=*/4, epi, sp, row_lo, row_hi);
}

template <typename SH, typename Epi>
void run_tiles(GemmA A, Rows rows, int K, int N, WSeg seg, const void *w2, Epi epi, int splitk,
               float *part, hipStream_t s, int row_lo = 0, int row_hi = INT_MAX) {
  // one workgroup per tile up to 2048, as the kernel numbers them when the list is full: per XCD its
  // share of the full row tiles' tiles and its share of a partial last row tile's, each rounded up
  // (a shorter list leaves workgroups without a tile, or in rare splits gives a few a second one)
  // (the launch covers rows [row_lo, min(count, row_hi)) of the list)
  const int ncol = N / SH::BN, m_rel = std::max(std::min(rows.cap, row_hi) - row_lo, 0);
  const int n_full = (m_rel / SH::BM) * ncol, n_part = (m_rel % SH::BM) ? ncol : 0;
  int gx = ((n_full + N_XCD - 1) / N_XCD + (n_part + N_XCD - 1) / N_XCD) * N_XCD;
  if (gx < N_XCD) gx = N_XCD;
  if (gx > 2048) gx = 2048;
  // ring shapes: one workgroup per CU walks its tiles and prefetches the next one's first slices
  if (SH::RING && gx > cu_count() / N_XCD * N_XCD) gx = std::max(N_XCD, cu_count() / N_XCD * N_XCD);
  SplitStore sp{part, (size_t)rows.cap * N, N};
  dim3 grid(gx, splitk);
  using F = SplitForms<Epi>;
  if constexpr (F::raw && F::fused) {
    if (part) launch_tiles<SH, Epi, true>(grid, A, rows, K, N, seg, w2, epi, splitk, sp, s, row_lo, row_hi);
    else launch_tiles<SH, Epi, false>(grid, A, rows, K, N, seg, w2, epi, splitk, sp, s, row_lo, row_hi);
  } else {
    launch_tiles<SH, Epi, F::raw>(grid, A, rows, K, N, seg, w2, epi, splitk, sp, s, row_lo, row_hi);
  }
}

// K split for the skinny regime when the column tiles alone cannot fill the chip.
inline int pick_splitk(int N, int K, int bn, size_t part_elems, int cap) {
  const int tiles = N / bn;
  int s = 1;
  while (tiles * s < 192 && s < 8 && (K / (s * 2)) % BK == 0 && K / (s * 2) >= 4 * BK) s *= 2;
  while (s > 1 && (size_t)s * cap * N > part_elems) s /= 2;
  return s;
}

// Large regime: tile shape (256x128 or 256x256) and K split with the least estimated time, in units
// of one 256x128 tile over the whole K: rounds of the chip x tile cost / split, plus the cost of
// writing and re-reading the fp32 partials of a split (dear when N is wide and K short).
struct LargePlan { bool xlarge; int splitk; double cost; };
inline LargePlan plan_large(int cap, int N, int K, size_t part_elems, bool x_ok) {
  LargePlan best{false, 1, 1e30};
  double best_cost = 1e30;
  for (int x = 0; x <= (x_ok ? 1 : 0); ++x) {
    const long ncol = N / (x ? XLargeS::BN : LargeS::BN);
    const double tile_cost = x ? XLARGE_COST : 1.0;
    for (int sk = 1; sk <= 8; ++sk) {
      if ((K / BK) % sk != 0 || K / BK / sk < 8) continue;
      if (sk > 1 && (size_t)sk * cap * N > part_elems) continue;
      const double rounds = tile_rounds(cap, ncol, sk);
      // partials: sk * cap * N floats written and read again (~4 TB/s) against a round of tiles
      // (256 tiles x 2*256*128*K flop at ~1 PFLOP/s)
      const double partials = sk > 1 ? 1.2e-4 * sk * (double)cap * N / K + 0.02 : 0.0;
      const double cost = rounds * tile_cost / sk + partials;
      if (cost < best_cost - 1e-9) { best_cost = cost; best = LargePlan{x == 1, sk, cost}; }
    }
  }
  return best;
}

// Rows of a short last row tile that go to the weight-streaming shapes in a launch of their own
// (0: none).  The column tiles of such a row tile each stream their weight columns alone, on as many
// CUs as there are column tiles, and open a round of their own when the full tiles fill theirs;
// the streaming shapes spread the same bytes over the whole chip.  Estimated times: a partial tile
// 0.55 of a full one (tile flops at ~5 TFLOP/s per CU), the stream all w_elems weight elements once
// at ~5 TB/s plus a launch.  ncol column tiles of tile_cols columns, sk K splits.
int streamed_tail(int cap, double w_elems, int K, int ncol, int tile_cols, int sk) {
  const int tail = cap % 256;
  if (cap < 256 || tail == 0 || tail > SKINNY_MAX_ROWS) return 0;
  const double extra_rounds = tile_rounds(cap, ncol, sk) - tile_rounds(cap - tail, ncol, sk);
  const double t_partial = extra_rounds * (2.0 * 256 * tile_cols * (double)K / sk / 5e12);
  const double t_stream = w_elems * 2 / 5e12 + 5e-6;
  return t_stream < 0.9 * t_partial ? tail : 0;
}

}  // namespace

// raw result part[z][j][n]; returns the numbers of K splits
Splits gemm_bf16_raw(GemmA A, Rows rows, int K, WSeg seg, float *part, size_t part_elems, hipStream_t s) {
  Splits out;
  if (rows.cap <= 0) return out;
  const int N = seg.n_end[2];
  EpiStoreF32 e{part, N};
  // weight streaming for rows [row_lo, ...): wider column tiles where N allows (fewer re-reads of the
  // activation tile)
  auto stream_rows = [&](int row_lo) -> int {
    const bool w96 = N % SkinnyW96::BN == 0;
    const int sk = pick_splitk(N, K, w96 ? SkinnyW96::BN : SkinnyS::BN, part_elems, rows.cap);
    if (w96) run_tiles<SkinnyW96>(A, rows, K, N, seg, nullptr, e, sk, part, s, row_lo);
    else run_tiles<SkinnyS>(A, rows, K, N, seg, nullptr, e, sk, part, s, row_lo);
    return sk;
  };
  if (rows.cap <= SKINNY_MAX_ROWS) {
    out.n = stream_rows(0);
    return out;
  }
  const bool ring = ring_ok(A, rows, K, seg, N);
  const bool x_ok = N % XLargeS::BN == 0 && ring;
  LargePlan pl = plan_large(rows.cap, N, K, part_elems, x_ok);
  int cap_tiles = rows.cap, row_hi = INT_MAX;
  if (ring) {
    const int bn = pl.xlarge ? XLargeS::BN : LargeS::BN;
    if (const int tail = streamed_tail(rows.cap, (double)N * K, K, N / bn, bn, pl.splitk)) {
      cap_tiles = row_hi = rows.cap - tail;  // the 256-row tiles end where the stream begins
      pl = plan_large(cap_tiles, N, K, part_elems, x_ok);
    }
  }
  if (pl.xlarge) run_tiles<XLargeS>(A, rows, K, N, seg, nullptr, e, pl.splitk, part, s, 0, row_hi);
  else if (ring) run_tiles<LargeS>(A, rows, K, N, seg, nullptr, e, pl.splitk, part, s, 0, row_hi);
  else run_tiles<LargeS8>(A, rows, K, N, seg, nullptr, e, pl.splitk, part, s);
  out.n = pl.splitk;
  if (cap_tiles < rows.cap) {
    out.tail_from = cap_tiles;
    out.n_tail = stream_rows(cap_tiles);
  }
  return out;
}

void gemm_bf16_swiglu(GemmA A, Rows rows, int K, int N, const void *wg, const void *wu, void *act,
                      float *, size_t, hipStream_t s) {
  if (rows.cap <= 0) return;
  EpiSwiGLU<bf16_t> e{(bf16_t *)act, N};
  // weight streaming: tiles of HALF gate + HALF up columns, SwiGLU in registers, no raw result
  // (N is a multiple of 64 for every bf16 configuration the library accepts)
  auto stream_rows = [&](int row_lo) {
    WSeg seg;
    seg.w[0] = wg; seg.w[1] = wu; seg.w[2] = wu;
    seg.n_end[0] = N; seg.n_end[1] = 2 * N; seg.n_end[2] = 2 * N;
    if (N % 48 == 0)
      run_tiles<SkinnyW96>(A, rows, K, 2 * N, seg, nullptr, EpiSwiGLUHalves<bf16_t, 48>{(bf16_t *)act, N}, 1, nullptr, s, row_lo);
    else
      run_tiles<SkinnyH128>(A, rows, K, 2 * N, seg, nullptr, EpiSwiGLUHalves<bf16_t, 64>{(bf16_t *)act, N}, 1, nullptr, s, row_lo);
  };
  if (rows.cap <= SKINNY_MAX_ROWS && (N % 48 == 0 || N % 64 == 0)) {
    stream_rows(0);
  } else if (!ring_ok(A, rows, K, wseg_one(wg, N), N)) {
    run_tiles<LargeD8>(A, rows, K, N, wseg_one(wg, N), wu, e, 1, nullptr, s);
  } else {
    bool xl = N % XLargeD::BN == 0 && prefer_xlarge(rows.cap, N / LargeD::BN, N / XLargeD::BN);
    const int bn = xl ? XLargeD::BN : LargeD::BN;
    const int tail = (N % 48 && N % 64) ? 0 : streamed_tail(rows.cap, 2.0 * N * K, K, N / bn, 2 * bn, 1);
    const int row_hi = tail ? rows.cap - tail : INT_MAX;  // the 256-row tiles end where the stream begins
    if (tail) xl = N % XLargeD::BN == 0 && prefer_xlarge(rows.cap - tail, N / LargeD::BN, N / XLargeD::BN);
    if (xl) run_tiles<XLargeD>(A, rows, K, N, wseg_one(wg, N), wu, e, 1, nullptr, s, 0, row_hi);
    else run_tiles<LargeD>(A, rows, K, N, wseg_one(wg, N), wu, e, 1, nullptr, s, 0, row_hi);
    if (tail) stream_rows(rows.cap - tail);
  }
}

void gemm_bf16_down(GemmA A, Rows rows, int K, int N, const void *wd, const float *h, void *out,
                    float *part, size_t part_elems, hipStream_t s) {
  if (rows.cap <= 0) return;
  EpiDown<bf16_t> e{h, (bf16_t *)out, N};
  if (rows.cap <= SKINNY_MAX_ROWS) {
    const int sk = pick_splitk(N, K, SkinnyS::BN, part_elems, rows.cap);
    if (sk > 1) {
      run_tiles<SkinnyS>(A, rows, K, N, wseg_one(wd, N), nullptr, e, sk, part, s);
      Splits sp;
      sp.n = sk;
      launch_down_finalize(BF16, part, sp, (size_t)rows.cap * N, h, rows, N, out, s);
    } else {
      run_tiles<SkinnyS>(A, rows, K, N, wseg_one(wd, N), nullptr, e, 1, nullptr, s);
    }
  } else {
    const bool ring = ring_ok(A, rows, K, wseg_one(wd, N), N), x_ok = N % XLargeS::BN == 0 && ring;
    LargePlan pl = plan_large(rows.cap, N, K, part_elems, x_ok);
    // A last row tile of at most 128 rows goes to the weight-streaming tiles in a launch of its own
    // when the plan for the full row tiles alone plus that stream is estimated well below the plan
    // for all rows (a unit of the plans' cost = one 256 x 128 tile over all of K at ~5 TFLOP/s per
    // CU; the stream: the weights once at ~5 TB/s, a launch, and its rows' share of a sum kernel).
    const int tail = rows.cap % 256;
    int row_hi = INT_MAX, cap_tiles = rows.cap;
    if (ring && rows.cap >= 256 && tail > 0 && tail <= SKINNY_MAX_ROWS) {
      const LargePlan pf = plan_large(rows.cap - tail, N, K, part_elems, x_ok);
      const double unit = 2.0 * 256 * 128 * (double)K / 5e12, t_stream = (double)N * K * 2 / 5e12 + 8e-6;
      if (pf.cost * unit + t_stream < 0.9 * pl.cost * unit) {
        pl = pf;
        row_hi = cap_tiles = rows.cap - tail;
      }
    }
    float *pp = pl.splitk > 1 ? part : nullptr;
    if (pl.xlarge) run_tiles<XLargeS>(A, rows, K, N, wseg_one(wd, N), nullptr, e, pl.splitk, pp, s, 0, row_hi);
    else if (ring) run_tiles<LargeS>(A, rows, K, N, wseg_one(wd, N), nullptr, e, pl.splitk, pp, s, 0, row_hi);
    else run_tiles<LargeS8>(A, rows, K, N, wseg_one(wd, N), nullptr, e, pl.splitk, pp, s);
    Splits sp;
    sp.n = pl.splitk;
    sp.done_to = pl.splitk > 1 ? 0 : cap_tiles;  // rows the fused epilogue has finished
    if (cap_tiles < rows.cap) {
      const int sk = pick_splitk(N, K, SkinnyS::BN, part_elems, rows.cap);
      sp.tail_from = cap_tiles;
      sp.n_tail = sk;
      if (sk > 1) {
        run_tiles<SkinnyS>(A, rows, K, N, wseg_one(wd, N), nullptr, e, sk, part, s, cap_tiles);
      } else {
        run_tiles<SkinnyS>(A, rows, K, N, wseg_one(wd, N), nullptr, e, 1, nullptr, s, cap_tiles);
        if (pl.splitk == 1) sp.done_to = rows.cap;  // nothing left to sum
        // (with a split of the full tiles only, the sum kernel must skip the tail rows: n_tail = 0)
        else sp.n_tail = 0;
      }
    }
    if (sp.done_to < rows.cap && (pl.splitk > 1 || sp.n_tail > 1))
      launch_down_finalize(BF16, part, sp, (size_t)rows.cap * N, h, rows, N, out, s);
  }
}

}  // namespace dy
