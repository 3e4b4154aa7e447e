// Work decomposition of stage 3 (paper Sec. 3.2 Eq. 3-4) for launches whose query tiles do not fill
// the compute units evenly.
//
// A compute unit runs whole 256-row query tiles, two at a time, and one alone nearly twice as fast, so
// a launch of T tiles on C units takes ceil(T / C) tile times: 400 tiles on 256 units cost as much as
// 512.  The R = T mod C tiles in excess of a multiple of C (the partial last tiles of the heads first,
// then full tiles from the end) are therefore not run whole.  Their work - R tiles x the key tiles of
// their heads, numbered as one line of "units" of (256 queries x 64 keys) - is cut into S equal
// shares, about one or two per compute unit, whatever R is.  A share is one workgroup - equal work
// is what the hardware's dispatch of workgroups to free slots balances - and where it crosses from one
// query tile into the next it is two (or more) segments that the workgroup runs one after the other.
// A segment sees its key range as the whole key sequence and leaves un-normalised fp32 sums (and
// their softmax shift) in a slot of scratch memory; a second kernel adds the segments of a tile in
// key order.  The shares are dispatched behind the whole tiles (workgroups go to the compute units
// one each before any gets a second one, and then to whichever slot frees up): a launch with less
// than one whole tile per compute unit then has a whole tile and shares side by side on every
// unit, and a long launch ends on the small work items.
//
// The functions below are the single statement of that numbering; the host (plan, scratch size,
// tests) and the kernels (which segment am I, which slots belong to my tile) both call them.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace httm {

constexpr int kAttnTileRows = 256;        // query rows of a tile of the kernel instance that splits
constexpr int kAttnKeyTile = 64;          // keys per unit
constexpr int kAttnSplitGroups = 64;      // runs of tiles of one head the excess set may consist of
constexpr int kAttnMaxShares = 512;
constexpr int kAttnMaxExcess = 255;
constexpr int kAttnMinShareUnits = 8;     // a share is at least 512 keys long (pipeline fill and drain)
constexpr int kAttnShareUnits = 64;       // shares of more than 4096 keys are cut finer, down to two per CU
constexpr int kAttnMaxPiecesPerTile = 32; // bounds what one workgroup of the second kernel has to add up
constexpr int64_t kAttnSlotWords = (int64_t)kAttnTileRows * (64 + 2);   // 64 sums of weight * v, sum of weights, shift

// Scratch that covers any launch: a slot per (share, tile) pair that can occur.
constexpr int64_t kAttnScratchBytes = (int64_t)(kAttnMaxShares + kAttnMaxExcess) * kAttnSlotWords * 4;

// `count` consecutive tiles of one head in the excess set: tile e of the set (tile0 <= e < tile0 +
// count) covers the query rows from q0 + (e - tile0) * 256 and the units [cum + (e - tile0) * kt,
// ... + kt), kt = key tiles of the head.
struct SplitGroup {
  int32_t head, q0, tile0, cum, kt;
};

struct SplitPlan {
  int32_t n_tiles;      // tiles that run in pieces (0: none, every tile runs whole)
  int32_t n_groups;
  int32_t units;        // all units of those tiles
  int32_t share_units;  // units per share (the last share may be shorter)
  int32_t shares;
  int32_t span;         // most tiles a share touches
  int32_t slots;        // shares + n_tiles - 1 (a few slots stay unused: a share and a tile that end together)
  SplitGroup grp[kAttnSplitGroups];
};

struct SplitSegment {
  int32_t head, q0;     // the query tile
  int32_t t0, t1;       // its key tiles [t0, t1) of the head's sequence; t0 >= t1: nothing to do
  int32_t slot;         // where its partial results go
};

__host__ __device__ inline int split_group_of_tile(const SplitPlan& p, int e) {
  int g = 0;
  while (g + 1 < p.n_groups && p.grp[g + 1].tile0 <= e) ++g;
  return g;
}

// The tile of the excess set that unit `unit` (0 <= unit < p.units) belongs to.
__host__ __device__ inline int split_tile_of_unit(const SplitPlan& p, int unit) {
  int g = 0;
  while (g + 1 < p.n_groups && p.grp[g + 1].cum <= unit) ++g;
  return p.grp[g].tile0 + (unit - p.grp[g].cum) / p.grp[g].kt;
}

// Slot of the partial results of share s in tile e: consecutive segments differ in s, in e or in
// both, both never decrease, so s + e is unique; the largest is shares + n_tiles - 2.
__host__ __device__ inline int split_slot(int share, int tile) { return share + tile; }

// Share s covers the units [s * share_units, (s + 1) * share_units) (the last one up to p.units): the
// tiles first .. first + count - 1 of the excess set.
__host__ __device__ inline void split_share_tiles(const SplitPlan& p, int share, int* first, int* count) {
  const int u0 = share * p.share_units;
  const int u1 = u0 + p.share_units < p.units ? u0 + p.share_units : p.units;
  *first = split_tile_of_unit(p, u0);
  *count = split_tile_of_unit(p, u1 - 1) - *first + 1;
}

// The part of share s that lies in tile e (one of split_share_tiles).
__host__ __device__ inline SplitSegment split_segment(const SplitPlan& p, int share, int e) {
  const SplitGroup& g = p.grp[split_group_of_tile(p, e)];
  const int tu0 = g.cum + (e - g.tile0) * g.kt;       // first unit of tile e
  const int u0 = share * p.share_units;
  const int u1 = u0 + p.share_units < p.units ? u0 + p.share_units : p.units;
  SplitSegment s;
  s.head = g.head;
  s.q0 = g.q0 + (e - g.tile0) * kAttnTileRows;
  s.t0 = (u0 > tu0 ? u0 : tu0) - tu0;
  s.t1 = (u1 < tu0 + g.kt ? u1 : tu0 + g.kt) - tu0;
  s.slot = split_slot(share, e);
  return s;
}

// Tile e of the excess set for the kernel that adds its segments up: the shares first..last (in key
// order) each left one segment, in slot split_slot(share, e).
struct SplitTile {
  int32_t head, q0, first_share, last_share;
};
__host__ __device__ inline SplitTile split_tile(const SplitPlan& p, int e) {
  const SplitGroup& g = p.grp[split_group_of_tile(p, e)];
  const int tu0 = g.cum + (e - g.tile0) * g.kt;
  return {g.head, g.q0 + (e - g.tile0) * kAttnTileRows, tu0 / p.share_units, (tu0 + g.kt - 1) / p.share_units};
}

// What the host decides for a launch of 256-row tiles on `cus` compute units.  out->n_tiles == 0: no
// split.  *kept_full receives the number of full tiles that stay whole (the first ones, in head
// order), *split_ragged the number of partial tiles (in head order, the first ones) that are split.
// q_off / k_off: H + 1 row offsets each.
inline void plan_attention_split(const int64_t* q_off, const int64_t* k_off, int H, int64_t cus, SplitPlan* out,
                                 int64_t* kept_full, int* split_ragged) {
  SplitPlan& p = *out;
  p.n_tiles = p.n_groups = p.units = p.share_units = p.shares = p.span = p.slots = 0;
  int64_t full = 0, ragged = 0, min_mk = INT64_MAX;
  for (int h = 0; h < H; ++h) {
    const int64_t mq = q_off[h + 1] - q_off[h], mk = k_off[h + 1] - k_off[h];
    full += mq / kAttnTileRows;
    ragged += (mq % kAttnTileRows) != 0;
    if (mq > 0 && mk < min_mk) min_mk = mk;
  }
  *kept_full = full;
  *split_ragged = 0;
  int n_split_ragged = 0;
  if (cus <= 0 || full + ragged == 0) return;
  const int64_t R = (full + ragged) % cus;
  if (R == 0 || R > kAttnMaxExcess || min_mk < (int64_t)kAttnMinShareUnits * kAttnKeyTile) return;
  // the excess set: partial tiles in head order, then the last full tiles, ascending
  int64_t left = R;
  int64_t units = 0;
  int n_groups = 0, n_tiles = 0;
  for (int h = 0; h < H && left > 0; ++h) {
    const int64_t mq = q_off[h + 1] - q_off[h], mk = k_off[h + 1] - k_off[h];
    if (mq % kAttnTileRows == 0) continue;
    if (n_groups == kAttnSplitGroups) return;
    const int32_t kt = (int32_t)((mk + kAttnKeyTile - 1) / kAttnKeyTile);
    p.grp[n_groups++] = {h, (int32_t)(mq / kAttnTileRows) * kAttnTileRows, n_tiles, (int32_t)units, kt};
    n_tiles += 1;
    units += kt;
    --left;
    ++n_split_ragged;
  }
  const int64_t first_split_full = full - left;     // global index (over heads) of the first full tile that is split
  int64_t tile_start = 0;
  for (int h = 0; h < H && left > 0; ++h) {
    const int64_t mq = q_off[h + 1] - q_off[h], mk = k_off[h + 1] - k_off[h];
    const int64_t nf = mq / kAttnTileRows;
    const int64_t lo = first_split_full > tile_start ? first_split_full : tile_start;   // first split tile of this head
    if (lo < tile_start + nf) {
      if (n_groups == kAttnSplitGroups) return;
      const int32_t cnt = (int32_t)(tile_start + nf - lo);
      const int32_t kt = (int32_t)((mk + kAttnKeyTile - 1) / kAttnKeyTile);
      p.grp[n_groups++] = {h, (int32_t)(lo - tile_start) * kAttnTileRows, n_tiles, (int32_t)units, kt};
      n_tiles += cnt;
      units += (int64_t)cnt * kt;
      left -= cnt;
    }
    tile_start += nf;
  }
  if (left != 0 || units >= ((int64_t)1 << 30)) return;
  // It pays when the tile time it saves - the share (1 - R / cus) of an average tile of the excess
  // set, about 0.85 us per unit - outweighs the second kernel and the traffic of the partial results
  // (about 15 us): (cus - R) * units / R >= 20 * cus.
  if ((cus - R) * (units / R) < 20 * cus) return;
  int64_t shares = units / kAttnShareUnits;
  if (shares < cus) shares = cus;
  if (shares > 2 * cus) shares = 2 * cus;
  if (shares > units / kAttnMinShareUnits) shares = units / kAttnMinShareUnits;
  if (shares > kAttnMaxShares) shares = kAttnMaxShares;
  if (shares < 1) return;
  int64_t u = (units + shares - 1) / shares;
  // a tile of kt key tiles is cut into at most kt / u + 2 pieces
  int64_t max_kt = 0;
  for (int g = 0; g < n_groups; ++g) max_kt = p.grp[g].kt > max_kt ? p.grp[g].kt : max_kt;
  const int64_t u_min = (max_kt + kAttnMaxPiecesPerTile - 3) / (kAttnMaxPiecesPerTile - 2);
  if (u < u_min) u = u_min;
  shares = (units + u - 1) / u;
  p.n_groups = n_groups;
  p.units = (int32_t)units;
  p.share_units = (int32_t)u;
  p.shares = (int32_t)shares;
  p.n_tiles = n_tiles;
  int span = 1;
  for (int s = 0; s < p.shares; ++s) {
    const int u0 = s * p.share_units, u1 = u0 + p.share_units < p.units ? u0 + p.share_units : p.units;
    const int d = split_tile_of_unit(p, u1 - 1) - split_tile_of_unit(p, u0) + 1;
    span = d > span ? d : span;
  }
  p.span = span;
  p.slots = p.shares + p.n_tiles - 1;
  *kept_full = first_split_full;
  *split_ragged = n_split_ragged;
}

// Slots of scratch a plan uses (kAttnSlotWords fp32 words each).
inline int64_t split_slots(const SplitPlan& p) { return p.n_tiles ? p.slots : 0; }

}  // namespace httm
