// Pieces shared by the partial-attention kernels: the mapping from a workgroup's tile number to
// (sequence, first query row, row count) over ragged per-sequence row lists, and the key-range
// split arithmetic.
#pragma once
#include "common.h"
#include "kernels.h"

namespace dy {

// Upper bound (host) of the number of query tiles: sum_b ceil(n_b / BQ) <= cap/BQ + B.
inline int max_q_tiles(const AttnArgs &a, int BQ) {
  if (!a.offsets) return a.B * ((a.L + BQ - 1) / BQ);
  int t = (a.rows.cap + BQ - 1) / BQ + a.B;
  return t < 1 ? 1 : t;
}

// Keys per split, a multiple of the key tile BK.
__host__ __device__ inline int split_chunk(int L, int splits, int BK) {
  int c = (L + splits - 1) / splits;
  return ((c + BK - 1) / BK) * BK;
}

// Tile number -> info[0] = sequence (or -1 if the tile does not exist), info[1] = index of its
// first query row in the row list, info[2] = rows in the tile.  Called by one thread.
__device__ inline void find_tile(const AttnArgs &a, int BQ, int tile, int *info) {
  info[0] = -1;
  info[1] = 0;
  info[2] = 0;
  if (!a.offsets) {
    const int per = (a.L + BQ - 1) / BQ;
    const int b = tile / per, t = tile % per;
    if (b < a.B) {
      info[0] = b;
      info[1] = b * a.L + t * BQ;
      info[2] = min(BQ, a.L - t * BQ);
    }
    return;
  }
  const int total = min(a.offsets[a.B], a.rows.cap);
  int t = tile;
  for (int b = 0; b < a.B; ++b) {
    const int lo = min(a.offsets[b], total), hi = min(a.offsets[b + 1], total);
    const int nt = (hi - lo + BQ - 1) / BQ;
    if (t < nt) {
      info[0] = b;
      info[1] = lo + t * BQ;
      info[2] = min(BQ, hi - lo - t * BQ);
      return;
    }
    t -= nt;
  }
}

// Work item of a workgroup of a 1-D launch over (key split, KV head, query tile, query head of the
// group).  Workgroup p runs on XCD p % 8, and an XCD takes its workgroups in the order of p: every
// XCD gets one contiguous range of the items in the order above, so all query tiles and all query
// heads that read the keys and values of one (sequence, KV head) run on ONE XCD, next to each other
// in time, and that K/V stream crosses the fabric once instead of once per tile and head.
constexpr int ATTN_XCD = 8;
inline int attn_grid(const AttnArgs &a, int q_tiles) {
  const long items = (long)q_tiles * a.H * a.splits;
  return (int)((items + ATTN_XCD - 1) / ATTN_XCD) * ATTN_XCD;
}
// returns false when the workgroup has no item
__device__ __forceinline__ bool attn_work_item(const AttnArgs &a, int q_tiles, int *tile, int *h, int *split) {
  const int items = q_tiles * a.H * a.splits;
  const int per_xcd = (items + ATTN_XCD - 1) / ATTN_XCD;
  const int p = blockIdx.x;
  const int w = (p % ATTN_XCD) * per_xcd + p / ATTN_XCD;
  if (p / ATTN_XCD >= per_xcd || w >= items) return false;
  const int g = a.H / a.Hkv;
  const int gi = w % g;
  int rest = w / g;
  *tile = rest % q_tiles;
  rest /= q_tiles;
  *h = (rest % a.Hkv) * g + gi;
  *split = rest / a.Hkv;
  return true;
}

// ---- grouped form (head_dim 128 kernel): the g = H / Hkv query heads that share a KV head are
// folded into the query rows of a tile.  Per sequence and KV head the "packed rows" are the pairs
// (row of the list, head of the group), numbered p = row * g + head: a tile is BQ consecutive
// packed rows, so a workgroup streams the keys and values of its KV head once for up to BQ
// (row, head) pairs instead of once per head, and ragged row counts leave g times fewer idle waves.
// With g = 1 this is the plain form above.
inline int max_q_tiles_grouped(const AttnArgs &a, int BQ) {
  const int g = a.H / a.Hkv;
  if (!a.offsets) return a.B * ((a.L * g + BQ - 1) / BQ);
  const long t = ((long)a.rows.cap * g + BQ - 1) / BQ + a.B;
  return t < 1 ? 1 : (int)t;
}
inline int attn_grid_grouped(const AttnArgs &a, int q_tiles) {
  const long items = (long)q_tiles * a.Hkv * a.splits;
  return (int)((items + ATTN_XCD - 1) / ATTN_XCD) * ATTN_XCD;
}
// Tile number -> info[0] = sequence (or -1), info[1] = index of the sequence's first row in the row
// list, info[2] = first packed row of the tile, info[3] = packed rows in the tile.  One thread.
__device__ inline void find_tile_grouped(const AttnArgs &a, int BQ, int tile, int *info) {
  const int g = a.H / a.Hkv;
  info[0] = -1;
  info[1] = info[2] = info[3] = 0;
  if (!a.offsets) {
    const int per = (a.L * g + BQ - 1) / BQ;
    const int b = tile / per, t = tile % per;
    if (b < a.B) {
      info[0] = b;
      info[1] = b * a.L;
      info[2] = t * BQ;
      info[3] = min(BQ, a.L * g - t * BQ);
    }
    return;
  }
  const int total = min(a.offsets[a.B], a.rows.cap);
  int t = tile;
  for (int b = 0; b < a.B; ++b) {
    const int lo = min(a.offsets[b], total), hi = min(a.offsets[b + 1], total);
    const int np = (hi - lo) * g;
    const int nt = (np + BQ - 1) / BQ;
    if (t < nt) {
      info[0] = b;
      info[1] = lo;
      info[2] = t * BQ;
      info[3] = min(BQ, np - t * BQ);
      return;
    }
    t -= nt;
  }
}
// Work item of a 1-D launch over (key split, KV head, tile of packed rows), XCD-aware as above.
__device__ __forceinline__ bool attn_work_item_grouped(const AttnArgs &a, int q_tiles, int *tile, int *kvh,
                                                       int *split) {
  const int items = q_tiles * a.Hkv * a.splits;
  const int per_xcd = (items + ATTN_XCD - 1) / ATTN_XCD;
  const int p = blockIdx.x;
  const int w = (p % ATTN_XCD) * per_xcd + p / ATTN_XCD;
  if (p / ATTN_XCD >= per_xcd || w >= items) return false;
  *tile = w % q_tiles;
  const int rest = w / q_tiles;
  *kvh = rest % a.Hkv;
  *split = rest / a.Hkv;
  return true;
}

void launch_attention_f32(DType t, const AttnArgs &a, hipStream_t s);
void launch_attention_bf16(const AttnArgs &a, hipStream_t s);
void launch_attn_combine(DType t, const AttnArgs &a, hipStream_t s);

}  // namespace dy
