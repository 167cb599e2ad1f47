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
// Inside a tile, byte i of a row sits in word j = i / 4 at position i % 4; with
// 4-bit bins the low nibble of byte i is feature 2i, the high nibble 2i + 1, so
// a word holds NP = 4 (or 8) features at positions p = 0..NP-1.
//
// Local-memory histogram of one tile: three arrays (grad, hess, count), each
// [bin][slot] with slot = j + LPR * p, LPR = W / 4 words per row.  With this
// slot order the lanes of a wavefront, which at any step work on pairwise
// different (j, p), fall into different banks (see hist_build_kernel).
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
  int32_t j = i >> 2;
  int32_t pos = p.nib ? ((i & 3) * 2 + (f & 1)) : (i & 3);
  FeatureSlot r;
  r.tile = t;
  r.slot = j + (w / 4) * pos;
  return r;
}

#endif  // GBDT_TILE_PLAN_H_
