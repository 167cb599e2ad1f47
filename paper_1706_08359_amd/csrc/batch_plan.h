// Tables of a batched histogram launch (several leaves in one grid) and the mapping of a
// block of that grid to its work.  Shared by the kernel and by the host (planning, tests).
#ifndef GBDT_BATCH_PLAN_H_
#define GBDT_BATCH_PLAN_H_

#include <stdint.h>

#include "tile_plan.h"

constexpr int kBatchLeaves = 224;  // leaves per launch: the table travels as kernel arguments (4 KB at most)

struct BatchLeaf {
  uint32_t row_off;   // first entry of the leaf's row list
  uint32_t n;         // its length
  uint32_t first_wg;  // workgroups per tile of all earlier leaves of the launch
  uint32_t wgs_unit;  // workgroups per tile | epochs per unit << 16
};

struct BatchBlock {
  int32_t leaf;  // leaf of the launch
  int32_t tile;  // feature tile
  int32_t wg;    // workgroup of (leaf, tile)
};

// The leaf whose blocks contain block b: the last one that starts at or before it (a
// leaf without rows has no blocks and is never the last such leaf of a live block).
GBDT_HD int32_t batch_leaf_of(const BatchLeaf* leaf, int32_t n_leaves, uint32_t n_tiles, uint32_t b) {
  int32_t lo = 0, hi = n_leaves - 1;
  while (lo < hi) {
    const int32_t mid = (lo + hi + 1) >> 1;
    if (leaf[mid].first_wg * n_tiles <= b) {
      lo = mid;
    } else {
      hi = mid - 1;
    }
  }
  return lo;
}

// Leaf l owns blocks [first_wg * n_tiles, (first_wg + wgs) * n_tiles), in the order of a
// single-leaf launch: consecutive blocks take different main tiles of the same rows, the
// remainder tile's workgroups come last.
GBDT_HD BatchBlock batch_block(const BatchLeaf* leaf, int32_t n_leaves, int32_t n_main, int32_t wr,
                               uint32_t b) {
  const uint32_t n_tiles = (uint32_t)(n_main + (wr ? 1 : 0));
  BatchBlock r;
  r.leaf = batch_leaf_of(leaf, n_leaves, n_tiles, b);
  const int32_t wgs = (int32_t)(leaf[r.leaf].wgs_unit & 0xffffu);
  const int32_t local = (int32_t)(b - leaf[r.leaf].first_wg * n_tiles);
  const int32_t main_blocks = n_main * wgs;
  r.tile = local < main_blocks ? local % n_main : n_main;
  r.wg = local < main_blocks ? local / n_main : local - main_blocks;
  return r;
}

#endif  // GBDT_BATCH_PLAN_H_
