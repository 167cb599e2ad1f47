// Device layout of the binned feature matrix and of the local-memory histograms.
//
// The paper (Sec. 4, "Data Structure") bundles 4 one-byte features of a sample
// into one 4-byte word so that a thread never fetches a single byte, and stores
// those words tuple-major.  Here the bundle is kept (a lane loads 4, 8 or 16 bytes
// = that many features, twice as many with 4-bit bins, App. C.4) but words are laid
// out row-major inside FEATURE TILES of W bytes: tile t holds, for every row, W
// consecutive bytes.  A gathered leaf row then costs one contiguous W-byte
// segment per tile instead of one 4-byte word per cache line.
//
//   packed = [tile 0: n_rows x W_0 bytes][tile 1: n_rows x W_1 bytes] ...
//
// All tiles have the "main" width WM except possibly the last one, which is 16
// or 32 bytes wide when few feature bytes remain (so that padding stays small).
//
// Behind the tiles, and a slack the build kernels may read (and ignore) past the last
// tile, the matrix is stored ONCE MORE, column by column, one byte per value:
//
//   packed = [tiles][slack][column 0: stride bytes][column 1] ...     stride = n_rows rounded up to 256
//
// The row partition after a split looks at ONE feature of every row of a leaf; from the
// tiles that costs a whole 32- or 64-byte tile row per row, from a column one byte.  The
// copy doubles the resident matrix (triples it with 4-bit bins) -- memory this part has.
//
// Inside a tile, a lane loads VEC consecutive bytes of a row (W / 4 with 8-bit bins;
// 4 or 8 with 4-bit bins), so a row is LPR = W / VEC = 4 or 8 lane-chunks.  Byte i of the tile row
// is byte bl = i % VEC of lane-chunk j = i / VEC.  The lane splits its bytes
// into "byte-words" of 4 bin values each: with 8-bit bins byte-word bw is the
// loaded word bl / 4; with 4-bit bins each loaded word gives two byte-words, its
// low nibbles (features 2i) and its high nibbles (features 2i + 1): bw = 2 *
// (bl / 4) + half.  q = bl % 4 is the value's byte inside its byte-word.
//
// Histogram slot of a feature of the tile:  s = j + LPR * q + 4 * LPR * bw.
// The local-memory histogram and each partial block in the workspace are cells
// [page = s / 32][bin][s % 32]; one page row (32 cells of 8 bytes) spans all 32
// banks exactly once.  With this slot order the lanes the LDS serves together,
// which at any step work on pairwise different (j, q), fall into different
// banks whatever the bin values are (see build_tile).
#ifndef GBDT_TILE_PLAN_H_
#define GBDT_TILE_PLAN_H_

#include <stdint.h>

#if defined(__HIPCC__)
#define GBDT_HD __host__ __device__ __forceinline__
#else
#define GBDT_HD inline
#endif

struct TilePlan {
  int32_t cap;        // bin capacity of the kernel variant: 16, 64 or 256
  int32_t nib;        // 1: 4-bit bins, two per byte
  int32_t wm;         // main tile width in bytes (64, or 32 when cap == 256)
  int32_t n_main;     // number of main tiles
  int32_t wr;         // width of the remainder tile in bytes (16 / 32), 0 if none
  int32_t row_bytes;  // n_main * wm + wr: packed bytes per row
  int32_t feat_bytes; // bytes of real feature data per row (before padding)
};

GBDT_HD TilePlan make_tile_plan(int32_t n_features, int32_t n_bins) {
  TilePlan p;
  p.nib = n_bins <= 16 ? 1 : 0;
  p.cap = n_bins <= 16 ? 16 : (n_bins <= 64 ? 64 : 256);
  p.wm = p.cap == 256 ? 32 : 64;
  p.feat_bytes = p.nib ? (n_features + 1) / 2 : n_features;
  p.n_main = p.feat_bytes / p.wm;
  int32_t rem = p.feat_bytes - p.n_main * p.wm;
  p.wr = 0;
  if (rem > p.wm / 2) {
    p.n_main += 1;  // more than half a tile left: pad it to a full tile
  } else if (rem > 0) {
    p.wr = rem <= 16 ? 16 : 32;
  }
  p.row_bytes = p.n_main * p.wm + p.wr;
  return p;
}

// Bytes behind the last tile that the build kernel may read (and ignore): its last epoch
// of a root leaf fetches whole row groups, up to one epoch (512 rows) of the widest tile
// past the end.
constexpr int64_t kPlanSlackBytes = 512 * 64;
GBDT_HD int64_t plan_column_stride(int64_t n_rows) { return (n_rows + 255) / 256 * 256; }
GBDT_HD int64_t plan_columns_base(const TilePlan& p, int64_t n_rows) {
  return (n_rows * (int64_t)p.row_bytes + kPlanSlackBytes + 255) / 256 * 256;
}
GBDT_HD int64_t plan_packed_bytes(const TilePlan& p, int64_t n_rows, int32_t n_features) {
  return plan_columns_base(p, n_rows) + (int64_t)n_features * plan_column_stride(n_rows);
}

GBDT_HD int32_t plan_n_tiles(const TilePlan& p) { return p.n_main + (p.wr ? 1 : 0); }
GBDT_HD int32_t plan_tile_width(const TilePlan& p, int32_t t) { return t < p.n_main ? p.wm : p.wr; }
// features (= slots) held by a tile of width w
GBDT_HD int32_t plan_slots(const TilePlan& p, int32_t w) { return p.nib ? 2 * w : w; }
// bytes a lane loads from a row of a tile of width w: a quarter of the row with 8-bit
// bins; with 4-bit bins at most 8 (16 bin values)
GBDT_HD int32_t plan_vec(const TilePlan& p, int32_t w) { return p.nib ? (w == 16 ? 4 : 8) : w / 4; }
// pages of 32 slots in the histogram of a tile of width w
GBDT_HD int32_t plan_pages(const TilePlan& p, int32_t w) { return (plan_slots(p, w) + 31) / 32; }
// cells ((bin, slot) pairs, padding included) of the histogram of a tile of width w
GBDT_HD int32_t plan_cells(const TilePlan& p, int32_t w) { return plan_pages(p, w) * p.cap * 32; }
// index of cell (bin, slot) inside a histogram / partial block
GBDT_HD int32_t plan_cell(const TilePlan& p, int32_t bin, int32_t slot) {
  return (slot >> 5) * p.cap * 32 + bin * 32 + (slot & 31);
}

struct FeatureSlot {
  int32_t tile;
  int32_t slot;
};

// Where feature f lives: which tile, and which slot of that tile's histogram.
GBDT_HD FeatureSlot plan_locate(const TilePlan& p, int32_t f) {
  int32_t fb = p.nib ? (f >> 1) : f;  // byte of the row holding f
  int32_t t = fb / p.wm;
  if (t >= p.n_main) t = p.n_main;  // remainder tile
  int32_t w = plan_tile_width(p, t);
  int32_t i = fb - t * p.wm;  // byte inside the tile row
  int32_t vec = plan_vec(p, w);
  int32_t lpr = w / vec;
  int32_t j = i / vec;
  int32_t bl = i - j * vec;  // byte inside the lane-chunk
  int32_t bw = p.nib ? (2 * (bl >> 2) + (f & 1)) : (bl >> 2);
  int32_t q = bl & 3;
  FeatureSlot r;
  r.tile = t;
  r.slot = j + lpr * q + 4 * lpr * bw;
  return r;
}

// Inverse of plan_locate: the feature held by `slot` of tile t (may be >= n_features
// for padding slots).
GBDT_HD int32_t plan_feature_of(const TilePlan& p, int32_t t, int32_t slot) {
  int32_t w = plan_tile_width(p, t);
  int32_t vec = plan_vec(p, w);
  int32_t lpr = w / vec;
  int32_t bw = slot / (4 * lpr);
  int32_t rest = slot - bw * 4 * lpr;
  int32_t q = rest / lpr;
  int32_t j = rest - q * lpr;
  if (p.nib) {
    int32_t bl = 4 * (bw >> 1) + q;
    return 2 * (t * p.wm + j * vec + bl) + (bw & 1);
  }
  return t * p.wm + j * vec + 4 * bw + q;
}

// The unit counter of tile t in the head of a scratch buffer (65,536 words): neighbouring tiles'
// counters lie 256 bytes apart, so that the device-scope atomics of a launch's workgroups do not
// all queue at the memory channel of one cache line.
GBDT_HD int32_t plan_counter_slot(int32_t t) { return (t & 1023) * 64 + (t >> 10); }

#endif  // GBDT_TILE_PLAN_H_
