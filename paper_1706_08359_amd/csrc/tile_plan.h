// Device layout of the binned feature matrix and of the local-memory histograms.
//
// The paper (Sec. 4, "Data Structure") bundles 4 one-byte features of a sample
// into one 4-byte word so that a thread never fetches a single byte, and stores
// those words tuple-major.  Here the bundle is kept (a lane still loads one
// 4-byte word = 4 features, or 8 with 4-bit bins, App. C.4) but words are laid
// out row-major inside FEATURE TILES of W bytes: tile t holds, for every row, W
// consecutive bytes.  A gathered leaf row then costs one contiguous W-byte
// segment per tile instead of one 4-byte word per cache line.
//
//   packed = [tile 0: n_rows x W_0 bytes][tile 1: n_rows x W_1 bytes] ...
//
// All tiles have the "main" width WM except possibly the last one, which is 16
// or 32 bytes wide when few feature bytes remain (so that padding stays small).
//
// Inside a tile, a lane loads VEC consecutive bytes of a row: 8 bytes from a
// 64-byte tile, 4 bytes from a 16- or 32-byte tile.  Byte i of the tile row is
// byte i % VEC of lane-chunk j = i / VEC; with 4-bit bins the low nibble of a
// byte is feature 2i, the high nibble 2i + 1.  A lane-chunk so holds NP = VEC
// (or 2 * VEC) features at positions p = 0..NP-1.
//
// Local-memory histogram of one tile: an array of 64-bit (hess:grad) sums and an
// array of 32-bit counts, each [bin][stride] with the feature at slot
// = j + LPR * p, LPR = W / VEC lane-chunks per row.  The stride is the number of
// slots of the tile, except that all tiles of the 64-bin variant use stride 64 so
// that (bin << 8) | (4 * slot) is a byte address a single byte-permute can form.
// With this slot order the lanes the LDS serves together, which at any step work
// on pairwise different (j, p), fall into different banks (see build_tile).
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

GBDT_HD int32_t plan_n_tiles(const TilePlan& p) { return p.n_main + (p.wr ? 1 : 0); }
GBDT_HD int32_t plan_tile_width(const TilePlan& p, int32_t t) { return t < p.n_main ? p.wm : p.wr; }
// features (= slots) held by a tile of width w
GBDT_HD int32_t plan_slots(const TilePlan& p, int32_t w) { return p.nib ? 2 * w : w; }
// bytes a lane loads from a row of a tile of width w
GBDT_HD int32_t plan_vec(int32_t w) { return w == 64 ? 8 : 4; }
// slots per bin row of the LDS / partial-block histogram of a tile of width w
GBDT_HD int32_t plan_stride(const TilePlan& p, int32_t w) { return p.cap == 64 ? 64 : plan_slots(p, w); }

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
  int32_t vec = plan_vec(w);
  int32_t j = i / vec;
  int32_t bl = i - j * vec;  // byte inside the lane-chunk
  int32_t pos = p.nib ? (bl * 2 + (f & 1)) : bl;
  FeatureSlot r;
  r.tile = t;
  r.slot = j + (w / vec) * pos;
  return r;
}

// Inverse of plan_locate: the feature held by `slot` of tile t (may be >= n_features
// for padding slots).
GBDT_HD int32_t plan_feature_of(const TilePlan& p, int32_t t, int32_t slot) {
  int32_t w = plan_tile_width(p, t);
  int32_t vec = plan_vec(w);
  int32_t lpr = w / vec;
  int32_t pos = slot / lpr;
  int32_t j = slot - pos * lpr;
  if (p.nib) return 2 * (t * p.wm + j * vec + (pos >> 1)) + (pos & 1);
  return t * p.wm + j * vec + pos;
}

#endif  // GBDT_TILE_PLAN_H_
