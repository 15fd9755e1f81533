// What the prefill FFN kernels share: the launch context and the block -> tile mapping.
#pragma once

#include "common.h"

namespace hmoe {

struct TiledCtx {
  const int32_t* offsets;
  const int32_t* slot_of;
  const char* slots;
  size_t slot_bytes;
  ActiveMask active;
  int n_experts, hidden, ffn;
  int n_tiles_n;  // n-tiles per expert
  int grid_padded;  // blocks launched: an upper bound of the tile count, a multiple of 8
  const int32_t* row_map;  // gate/up only: input row of sorted row p is row_map[p] / map_div
  int map_div;
  int walk_bm = 224;  // blocks that walk through tiles: the most rows an m-tile may have (a multiple of 32)
  // map_div as a multiplication: for 0 <= x < 2^31, x / map_div == umulhi(x, map_mul) >> map_shift (map_div >= 2)
  uint32_t map_mul = 0;
  int map_shift = 0;
};

// Division by the invariant map_div (Granlund and Montgomery's round-up multiplier): with l = ceil(log2 d) and
// m = ceil(2^(31+l) / d), which fits 32 bits, floor(x m / 2^(31+l)) = floor(x / d) for every 0 <= x < 2^31.
static inline void set_map_div(TiledCtx& c) {
  const uint32_t d = (uint32_t)c.map_div;
  if (d < 2) return;
  int l = 0;
  while ((1u << l) < d) ++l;
  c.map_mul = (uint32_t)(((1ull << (31 + l)) + d - 1) / d);
  c.map_shift = l - 1;
}
__device__ __forceinline__ int div_by_map(const TiledCtx& c, int x) {
  return c.map_div < 2 ? x : (int)(__umulhi((uint32_t)x, c.map_mul) >> c.map_shift);
}

// The tile a block works on.  The logical tile list is: for each busy expert in ascending id (rows > 0,
// selected by the mask, resident), for each n-tile, every m-tile of BM rows.  The hardware deals
// consecutive block ids round-robin to the 8 XCDs, so block b takes entry (b / 8) of the (b % 8)-th
// eighth of the list: each XCD works through one contiguous range (blocks that share a weight panel
// share an L2) and the eight ranges differ by at most one tile.  The launch only knows an upper bound
// of the list length; the exact length comes from expert_offsets here, lane-parallel over the
// experts, and every wave of the block computes the same answer.  Returns false for surplus blocks.
struct TileLoc {
  int e, row_first, m_rows, mt, nt;
  int slot;  // cache slot that holds expert e
  int m0, fm;  // TileWalk only: first row of the tile within the expert, and its height in 32-row fragments
};
template <int BM>
__device__ __forceinline__ bool locate_tile(const TiledCtx& c, TileLoc& t) {
  constexpr int CH = HMOE_MAX_EXPERTS / 64;
  const int lane = threadIdx.x % 64;
  int first[CH], rows[CH], incl[CH], slot[CH];
  int total = 0;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    first[j] = rows[j] = 0;
    slot[j] = -1;
    incl[j] = total;
    if (j * 64 < c.n_experts) {  // uniform
      const int i = j * 64 + lane;
      if (i < c.n_experts) slot[j] = c.slot_of[i];
      if (i < c.n_experts && ((c.active.w[j] >> lane) & 1ull) && slot[j] >= 0) {
        first[j] = c.offsets[i];
        rows[j] = c.offsets[i + 1] - first[j];
      }
      int v = (rows[j] + BM - 1) / BM * c.n_tiles_n;
#pragma unroll
      for (int d = 1; d < 64; d *= 2) {
        const int below = __shfl_up(v, d);
        if (lane >= d) v += below;
      }
      incl[j] = total + v;
      total += __shfl(v, 63);
    }
  }
  const int per_xcd = (total + 7) / 8;
  const int idx = blockIdx.x / 8;
  const int tile_id = (blockIdx.x % 8) * per_xcd + idx;
  if (idx >= per_xcd || tile_id >= total) return false;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const unsigned long long past = __ballot(incl[j] > tile_id);  // inclusive prefix sums are monotone
    if (past) {
      const int src = __ffsll((long long)past) - 1;
      // wave-uniform by construction; readfirstlane tells the compiler so (scalar registers, scalar loads)
      t.e = j * 64 + src;
      t.row_first = __builtin_amdgcn_readfirstlane(__shfl(first[j], src));
      t.m_rows = __builtin_amdgcn_readfirstlane(__shfl(rows[j], src));
      t.slot = __builtin_amdgcn_readfirstlane(__shfl(slot[j], src));
      const int mts = (t.m_rows + BM - 1) / BM;
      const int within = __builtin_amdgcn_readfirstlane(tile_id - (__shfl(incl[j], src) - mts * c.n_tiles_n));
      t.nt = within / mts;
      t.mt = within % mts;
      return true;
    }
  }
  return false;
}

// The same tile list for a block that works through several tiles: the per-expert prefix sums are computed once into
// a table in LDS (4 * HMOE_MAX_EXPERTS ints: first row, rows, inclusive tile count, slot), and entry idx of the xcd-th eighth
// of the list is looked up on demand.  Every wave of the block computes and writes the same table.
template <int MIN_FM>
struct TileWalk {
  static constexpr int CH = HMOE_MAX_EXPERTS / 64;
  static constexpr int TABLE_INTS = 4 * HMOE_MAX_EXPERTS;
  int total, per_xcd, n_tiles_n, bm;
  int* tab;
  __device__ __forceinline__ void init(const TiledCtx& c, int* table) {
    const int lane = threadIdx.x % 64;
    tab = table;
    n_tiles_n = c.n_tiles_n;
    bm = c.walk_bm;
    int sum = 0;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      int first = 0, rows = 0, incl = sum, slot = -1;
      if (j * 64 < c.n_experts) {  // uniform
        const int i = j * 64 + lane;
        if (i < c.n_experts) slot = c.slot_of[i];
        if (i < c.n_experts && ((c.active.w[j] >> lane) & 1ull) && slot >= 0) {
          first = c.offsets[i];
          rows = c.offsets[i + 1] - first;
        }
        int v = (rows + bm - 1) / bm * c.n_tiles_n;
#pragma unroll
        for (int d = 1; d < 64; d *= 2) {
          const int below = __shfl_up(v, d);
          if (lane >= d) v += below;
        }
        incl = sum + v;
        sum += __shfl(v, 63);
      }
      tab[j * 64 + lane] = first;
      tab[HMOE_MAX_EXPERTS + j * 64 + lane] = rows;
      tab[2 * HMOE_MAX_EXPERTS + j * 64 + lane] = incl;
      tab[3 * HMOE_MAX_EXPERTS + j * 64 + lane] = slot;
    }
    total = __builtin_amdgcn_readfirstlane(sum);
    per_xcd = (total + 7) / 8;
    __syncthreads();
  }
  __device__ __forceinline__ bool at(int xcd, int idx, TileLoc& t) const {
    const int lane = threadIdx.x % 64;
    const int tile_id = xcd * per_xcd + idx;
    if (idx >= per_xcd || tile_id >= total) return false;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const unsigned long long past = __ballot(tab[2 * HMOE_MAX_EXPERTS + j * 64 + lane] > tile_id);  // monotone
      if (past) {
        const int e = j * 64 + __ffsll((long long)past) - 1;
        t.e = e;
        t.row_first = __builtin_amdgcn_readfirstlane(tab[e]);
        t.m_rows = __builtin_amdgcn_readfirstlane(tab[HMOE_MAX_EXPERTS + e]);
        t.slot = __builtin_amdgcn_readfirstlane(tab[3 * HMOE_MAX_EXPERTS + e]);
        const int mts = (t.m_rows + bm - 1) / bm;
        const int within = tile_id - (__builtin_amdgcn_readfirstlane(tab[2 * HMOE_MAX_EXPERTS + e]) - mts * n_tiles_n);
        t.nt = within / mts;
        t.mt = within % mts;
        // The expert's 32-row fragments are dealt to its m-tiles as evenly as whole fragments allow (heights differ
        // by at most one fragment): at most 31 padded rows per expert.  A lone tile has at least MIN_FM fragments.
        const int frags = (t.m_rows + 31) / 32;
        const int base = frags / mts, rem = frags % mts;
        t.fm = base + (t.mt < rem ? 1 : 0);
        t.m0 = 32 * (t.mt * base + (t.mt < rem ? t.mt : rem));
        if (t.fm < MIN_FM) t.fm = MIN_FM;  // (only when mts == 1)
        return true;
      }
    }
    return false;
  }
};

// upper bound of the tile count of a launch (sum over experts of ceil(rows / BM) is at most this)
static inline long tiles_upper_bound(const TiledCtx& c, int n_rows, int bm) {
  return ((long)n_rows / bm + (c.n_experts < n_rows ? c.n_experts : n_rows)) * c.n_tiles_n;
}

}  // namespace hmoe
