// Slice loop of the 256-row bf16 GEMM tiles with four waves (one per SIMD; 128 x 128 outputs each
// for the 256 x 256 tile, 128 x 64 for the 256 x 128 tile; the accumulators in the second register
// file) and a ring of five 32 KB LDS slots.
//
// Why a ring.  A K slice of the tile is 64 KB (A tile 32 KB + weight tile 32 KB), and two whole
// slices are all that fit beside nothing else in the 160 KB of LDS.  With two stages, the copies of
// slice kt+2 can only be issued once slice kt has been read out, and must have landed before slice
// kt+1 is read out: the copy path runs empty before every barrier and is asked for a whole slice in a
// burst after it (measured: 64 KB take about 3000 cycles to land that way, with or without matrix
// work, against 2048 cycles of matrix instructions per slice).  Here the halves of a slice take
// slots of their own, in the order A(0) W(0) A(1) W(1) A(2) ..., slot = position % 5.  There is one
// barrier per slice, in its middle: by then a wave has the operands of the whole slice in registers
// (128 of them), so the two slots of slice kt are free; W(kt+2) is copied into one during the second
// half of slice kt and A(kt+3) into the other during the first half of slice kt+1 -- one copy after
// every fourth matrix instruction, all the time -- and the eight newest copies stay in flight across
// the barrier (s_waitcnt vmcnt(8) and a raw s_barrier: __syncthreads would wait for all of them).
//
// The copies are buffer loads with LDS destination: a scalar descriptor per source matrix, a 32-bit
// byte offset per lane that is fixed for the tile, and the K walk as a scalar offset, so a copy costs
// no vector address arithmetic between the matrix instructions (measured against per-lane 64-bit
// addresses: 2150 against 2340 cycles per slice).  Lane offsets are 32 bits: the activation
// descriptor starts at the tile's first row, and the launcher takes these shapes only when a gathered
// activation operand and every weight matrix span less than 4 GiB.
#pragma once
#include <type_traits>
#include "common.h"

namespace dy {
namespace mm {

typedef __attribute__((address_space(3))) void lds_void_t;

// lane i's 16 bytes at (descriptor base + voff + soff) -> LDS[lds_addr + 16 i]; lds_addr and soff
// are wave-uniform.  Completion is tracked by vmcnt, in issue order.
__device__ __forceinline__ void dma16_buf(__amdgpu_buffer_rsrc_t srd, uint32_t voff, uint32_t soff, uint32_t lds_addr) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(srd, (lds_void_t *)(uintptr_t)lds_addr, 16, voff, soff, 0, 0);
}

// descriptor of a raw byte buffer (no stride, no swizzle, 32-bit data format) that covers `bytes`
// from p; reads past the end return zero instead of faulting
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_srd(const void *p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void *)p, 0, (int)bytes, 0x00020000);
}

constexpr uint32_t RING_SLOT = 32768;
constexpr int RING_SLOTS = 5;
constexpr int RING_MIN_SLICES = 3;

// Sources of a wave's copies for one tile:
//   srd_a / va[i]   descriptor and lane offsets of its 8 A copies (8 tile rows each)
//   srd_w[c] / vw[c] the same for its weight copies (8 for a 256-row weight tile, 4 for a 128-row one;
//                   a copy's 8 rows lie in one weight matrix)
struct RingSrc {
  __amdgpu_buffer_rsrc_t srd_a, srd_w[8];
  uint32_t va[8], vw[8];
};

// The loop for one wave tile of 128 rows x (32 NMAT NB) columns: NMAT x NB column blocks of 32, block
// c = t * NB + j reads weight-tile rows (t * BN + wn0 + 32 j ...).  Four column blocks (a 256-row
// weight tile, 256 x 256 or 256 x (128+128) outputs) or two (128 weight rows: 256 x 128 or
// 256 x (64+64)); the weight half of a slice then fills half of its slot.
// MBV = 32-row blocks of this wave that hold rows (4 in a full tile).  In a row tile with fewer than
// 256 rows a wave multiplies only those, down to none: copies, waits and barriers are the same for
// every wave, so such a tile costs about what its copies cost (leaving out the A copies of the empty
// row groups as well was measured: no faster).
template <int NMAT, int NB, int BN, int MBV> struct Ring {
  static constexpr int NCB = NMAT * NB;  // column blocks per wave
  static constexpr int NWC = 2 * NCB;    // weight copies per wave and slice
  static constexpr int PS = 4 * NCB;     // products per K step
  static constexpr int QH = 2 * PS;      // product slots per half slice
  static constexpr int RD = 4 + NCB;     // operand reads per K step
  static constexpr int RPS = (3 * RD + QH - 1) / QH;  // reads per product slot in the first half
  static_assert(NCB == 4 || NCB == 2, "four or two column blocks per wave");
  static constexpr int ROW = 128, A_STEP = 128, W_STEP = 4096;  // bytes per tile row; K walk per slice

  static __device__ __forceinline__ int w_row(int c) { return ((c / NB) * BN + (c % NB) * 32) * ROW; }
  static __device__ __forceinline__ int nxt(int s, int d) { const int t = s + d; return t >= RING_SLOTS ? t - RING_SLOTS : t; }
  // read x of a K step: A block x (x < 4) or column block x - 4; product p of a K step: row block
  // p / NCB, column block p % NCB
  static __device__ constexpr bool has_read(int x) { return x < 4 ? x < MBV : MBV > 0; }
  static __device__ constexpr bool has_prod(int p) { return p / NCB < MBV; }

  // Fills the ring for a tile: A(0) W(0) A(1) W(1) A(2) into slots 0..4.  The slots must be free
  // (every wave past the middle barrier of the previous tile's last slice).
  static __device__ __forceinline__ void fill(const RingSrc &src, uint32_t lds0, int wave) {
    const uint32_t lds_w = lds0 + (uint32_t)wave * 1024u;
#pragma unroll
    for (int h = 0; h < RING_SLOTS; ++h) {
      const int kt = h / 2;
      if (h % 2 == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) dma16_buf(src.srd_a, src.va[i], (uint32_t)kt * A_STEP, lds_w + h * RING_SLOT + i * 4096u);
      } else {
#pragma unroll
        for (int c = 0; c < NWC; ++c) dma16_buf(src.srd_w[c], src.vw[c], (uint32_t)kt * W_STEP, lds_w + h * RING_SLOT + c * 4096u);
      }
    }
  }

  // One tile: acc += A tile x W tile over KT >= 3 slices; the ring has been filled (fill).
  //   all_landed      wait for everything this wave has in flight (a fill issued before the previous
  //                   tile's epilogue, whose own loads and stores are counted with it) instead of for
  //                   the first slice alone; wave-uniform
  //   rd_a / rd_w     this lane's operand-read addresses inside a slot (slot 0), without the chunk swizzle
  //   rd_off[s]       swizzled chunk offset of K step s
  template <typename Acc>
  static __device__ __forceinline__ void tile(Acc &acc, uint32_t lds0, int wave, const RingSrc &src,
                                              const unsigned char *rd_a, const unsigned char *rd_w,
                                              const int (&rd_off)[4], int KT, bool all_landed) {
    const uint32_t lds_w = lds0 + (uint32_t)wave * 1024u;
    auto copy_a = [&](int i, int kt, int slot) {
      dma16_buf(src.srd_a, src.va[i], (uint32_t)kt * A_STEP, lds_w + (uint32_t)slot * RING_SLOT + i * 4096u);
    };
    auto copy_w = [&](int c, int kt, int slot) {
      dma16_buf(src.srd_w[c], src.vw[c], (uint32_t)kt * W_STEP, lds_w + (uint32_t)slot * RING_SLOT + c * 4096u);
    };
    if (all_landed) wait_vmcnt<0>();
    else wait_vmcnt<16 + NWC>();  // slice 0 has landed (this wave's part); the rest of the fill is behind it
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    bf16x8 af[4][4], bfr[4][NCB];  // [K step][32-row block], [K step][column block]
    auto read = [&](int st, int x, const unsigned char *sa, const unsigned char *sb) {
      if (x < 4) af[st][x] = *reinterpret_cast<const bf16x8 *>(sa + x * 32 * ROW + rd_off[st]);
      else bfr[st][x - 4] = *reinterpret_cast<const bf16x8 *>(sb + w_row(x - 4) + rd_off[st]);
    };
    auto prod = [&](int st, int p) {
      const int i = p / NCB, c = p % NCB;
      acc[c / NB][i][c % NB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[st][i], bfr[st][c], acc[c / NB][i][c % NB], 0, 0, 0);
    };
#pragma unroll
    for (int x = 0; x < RD; ++x)
      if (has_read(x)) read(0, x, rd_a, rd_w + RING_SLOT);

    int slot_a = 0;  // slot of A(kt); W(kt) is in the next one
    auto slice = [&](int kt, auto first_c, auto m1_c, auto m2_c) {
      // FIRST: slice 0 (A(2) is already on its way); M1 / M2: slices kt+1 / kt+2 exist.  The last
      // slice keeps its barrier: past it every wave has read the tile's last operands out of the
      // ring, which the caller may then refill for its next tile.
      constexpr bool FIRST = decltype(first_c)::value, M1 = decltype(m1_c)::value, M2 = decltype(m2_c)::value;
      constexpr bool CA = !FIRST && M2;
      const int slot_w = nxt(slot_a, 1), slot_a1 = nxt(slot_a, 2), slot_w1 = nxt(slot_a, 3), slot_a2 = nxt(slot_a, 4);
      const unsigned char *sa = rd_a + (uint32_t)slot_a * RING_SLOT, *sb = rd_w + (uint32_t)slot_w * RING_SLOT;
      // First half: products of K steps 0 and 1; the operand reads of steps 1..3 behind the first
      // products (RPS per product); the 8 copies of A(kt+2) into the slot W(kt-1) left, evenly.
      // In the instruction order (sched_group_barrier: product, reads, copy) the scheduler left alone
      // would fetch each operand right before its use and bunch the copies.
      auto copy_a_due = [](int q) { return (q + 1) % (QH / 8) == 0; };
#pragma unroll
      for (int q = 0; q < QH; ++q) {
#pragma unroll
        for (int r = q * RPS; r < (q + 1) * RPS && r < 3 * RD; ++r)
          if (has_read(r % RD)) read(1 + r / RD, r % RD, sa, sb);
        if (CA && copy_a_due(q)) copy_a((q + 1) / (QH / 8) - 1, kt + 2, slot_a2);
        if (has_prod(q % PS)) prod(q / PS, q % PS);
      }
#pragma unroll
      for (int q = 0; q < QH; ++q) {
        if (has_prod(q % PS)) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
#pragma unroll
        for (int r = q * RPS; r < (q + 1) * RPS && r < 3 * RD; ++r)
          if (has_read(r % RD)) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        if (CA && copy_a_due(q)) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
      }
      // Middle: slice kt+1 has landed (the copies of A(kt+2) behind it may still be in flight), and
      // with the barrier everyone's part of it; everyone has read slice kt out of its slots.
      if (M1) {
        if (M2) wait_vmcnt<8>();
        else wait_vmcnt<0>();
      }
      wait_lgkmcnt0();
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      // Second half: products of K steps 2 and 3, the copies of W(kt+2) into the slot A(kt) left, the
      // operands of step 0 of slice kt+1 (behind the products of step 3).
      const unsigned char *sa1 = rd_a + (uint32_t)slot_a1 * RING_SLOT, *sb1 = rd_w + (uint32_t)slot_w1 * RING_SLOT;
      auto copy_w_due = [](int q) { return (q + 1) % (QH / NWC) == 0; };
#pragma unroll
      for (int q = 0; q < QH; ++q) {
        if (M1 && q >= PS && q - PS < RD && has_read(q - PS)) read(0, q - PS, sa1, sb1);
        if (M2 && copy_w_due(q)) copy_w((q + 1) / (QH / NWC) - 1, kt + 2, slot_a);
        if (has_prod(q % PS)) prod(2 + q / PS, q % PS);
      }
#pragma unroll
      for (int q = 0; q < QH; ++q) {
        if (has_prod(q % PS)) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (M1 && q >= PS && q - PS < RD && has_read(q - PS)) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        if (M2 && copy_w_due(q)) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
      }
      slot_a = slot_a1;
    };
    slice(0, std::true_type{}, std::true_type{}, std::true_type{});
    int kt = 1;
    for (; kt + 2 < KT; ++kt) slice(kt, std::false_type{}, std::true_type{}, std::true_type{});
    slice(kt, std::false_type{}, std::true_type{}, std::false_type{});
    slice(kt + 1, std::false_type{}, std::false_type{}, std::false_type{});
  }
};

}  // namespace mm
}  // namespace dy
