// The reduction pass over the workgroups' partial histograms (Sec. 4, "final reduction
// program") and the sibling histogram by subtraction.  Included by gbdt_hist.hip only, after
// hist_build_kernels.h.
#ifndef GBDT_HIST_REDUCE_KERNELS_H_
#define GBDT_HIST_REDUCE_KERNELS_H_

#include <hip/hip_runtime.h>

#include <stdint.h>
#include <string.h>

#include "../../include/gbdt_hist.h"
#include "tile_plan.h"
#include "batch_plan.h"

namespace {

// ------------------------------------------------------------------ merge kernel

struct MergeArgs {
  const uint32_t* partials;
  gbdt_bin_t* out;
  TilePlan plan;
  int32_t n_features;
  int32_t n_bins;
  int32_t chunks_main;
  int32_t chunks_rem;
  uint32_t* counters;  // the tiles' unit counters, set back to zero here; NULL: not used by the build
};

constexpr int kMergeCells = 64;   // histogram cells per workgroup
constexpr int kMergeLanes = 4;    // threads that share the chunks of one cell ...
constexpr int kMergeLanesWide = 16;  // ... and when there are few cells and many chunks (one or two tiles built
                                     // by hundreds of workgroups): 4 lanes would leave most of the machine idle

// The "final reduction program" of Sec. 4: sums the partial histograms of the
// workgroups that shared a feature tile.  A workgroup takes 64 consecutive (bin,
// slot) pairs of one tile (slot fastest, so reads of a partial block are coalesced
// in runs of 32); 4 threads per pair each sum every 4th chunk in fp64, in chunk
// order, and the 4 sub-sums are added in a fixed order: the result does not depend
// on scheduling.  Counts are summed as integers.  grid.y = tile.  (LANES = 4 or 16 threads per
// pair; which one is a function of the launch's shape only.)
template <int LANES>
__device__ __forceinline__ void merge_cells(const MergeArgs& a) {
  constexpr int kMergeLanes = LANES;
  if (a.counters && blockIdx.x == 0 && threadIdx.x == 0) a.counters[plan_counter_slot((int32_t)blockIdx.y)] = 0u;
  __shared__ double s_g[kMergeLanes][kMergeCells];
  __shared__ double s_h[kMergeLanes][kMergeCells];
  __shared__ uint32_t s_n[kMergeLanes][kMergeCells];
  const int32_t t = blockIdx.y;
  const int32_t w = plan_tile_width(a.plan, t);
  const int32_t slots = plan_slots(a.plan, w);
  const int cell = threadIdx.x % kMergeCells;
  const int part = threadIdx.x / kMergeCells;
  const int32_t e = blockIdx.x * kMergeCells + cell;
  const bool live = e < a.n_bins * slots;
  const int32_t bin = live ? e / slots : 0;
  const int32_t slot = live ? e - bin * slots : 0;
  const size_t hw = (size_t)plan_cells(a.plan, w);
  const size_t main_block = (size_t)3 * plan_cells(a.plan, a.plan.wm);
  const uint32_t* p;
  int32_t chunks;
  if (t < a.plan.n_main) {
    p = a.partials + (size_t)t * a.chunks_main * main_block;
    chunks = a.chunks_main;
  } else {
    p = a.partials + (size_t)a.plan.n_main * a.chunks_main * main_block;
    chunks = a.chunks_rem;
  }
  p += (size_t)plan_cell(a.plan, bin, slot) + (size_t)part * 3 * hw;
  double g = 0.0, h = 0.0;
  uint32_t n = 0;
  if (live) {
    // Same order of additions as a plain loop over the thread's chunks; the loads of 8
    // chunks are issued together (the loop is bound by memory latency, not by bandwidth).
    const size_t step = (size_t)kMergeLanes * 3 * hw;
    int32_t c = part;
    for (; c + 7 * kMergeLanes < chunks; c += 8 * kMergeLanes) {
      uint32_t vg[8], vh[8], vn[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        vg[i] = p[i * step];
        vh[i] = p[i * step + hw];
        vn[i] = p[i * step + 2 * hw];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        g += (double)__uint_as_float(vg[i]);
        h += (double)__uint_as_float(vh[i]);
        n += vn[i];
      }
      p += 8 * step;
    }
    for (; c < chunks; c += kMergeLanes) {
      g += (double)__uint_as_float(p[0]);
      h += (double)__uint_as_float(p[hw]);
      n += p[2 * hw];
      p += step;
    }
  }
  s_g[part][cell] = g;
  s_h[part][cell] = h;
  s_n[part][cell] = n;
  __syncthreads();
  if (part == 0 && live) {
    const int32_t f = plan_feature_of(a.plan, t, slot);
    if (f < a.n_features) {  // else: padding slot
#pragma unroll
      for (int q = 1; q < kMergeLanes; ++q) {
        g += s_g[q][cell];
        h += s_h[q][cell];
        n += s_n[q][cell];
      }
      gbdt_bin_t r;
      r.grad = (float)g;
      r.hess = (float)h;
      r.count = n;
      a.out[(size_t)f * a.n_bins + bin] = r;
    }
  }
}

template <int LANES>
__global__ void __launch_bounds__(kMergeCells * LANES) hist_merge_kernel(MergeArgs a) {
  merge_cells<LANES>(a);
}

// Threads per (bin, slot) pair for a reduction over `blocks` workgroups of 4-lane pairs and up to
// `chunks` partial blocks per pair.
inline int merge_lanes(int64_t blocks, int32_t chunks) {
  return (blocks < 512 && chunks >= 64) ? kMergeLanesWide : kMergeLanes;
}

// The same reduction for a batched launch: grid.z = leaf of the launch; its partial
// blocks start first_wg workgroup columns into the buffer, its histogram is the leaf's
// [n_features][n_bins] slice of the output.  A leaf without rows has no partial blocks
// and gets zeros; a leaf with a single workgroup per tile is skipped.
struct BatchMergeArgs {
  MergeArgs m;            // partials / out of leaf 0 of the launch; chunk counts unused
  uint64_t column_words;  // words of one workgroup column
  int32_t blocks_per_wg;  // partial blocks a workgroup wrote: 1, or 2 with wide accumulation
  BatchLeaf leaf[kBatchLeaves];
};

template <int LANES>
__global__ void __launch_bounds__(kMergeCells * LANES) hist_merge_batch_kernel(BatchMergeArgs a) {
  const BatchLeaf lf = a.leaf[blockIdx.z];
  if ((lf.wgs_unit & 0xffffu) == 1u) return;  // written by the build kernel itself
  MergeArgs m = a.m;
  m.partials += (size_t)lf.first_wg * a.column_words;
  m.out += (size_t)blockIdx.z * m.n_features * m.n_bins;
  m.chunks_main = (int32_t)(lf.wgs_unit & 0xffffu) * a.blocks_per_wg;
  m.chunks_rem = m.plan.wr ? m.chunks_main : 0;
  merge_cells<LANES>(m);
}

// ----------------------------------------------------------------- unfuse kernel

// Marginals of the fused columns' joint histograms (see FusedCol): bin b of feature f is the sum
// of the joint bins v of its column with (v / stride) mod levels == b, v ascending, in fp64;
// bins that do not occur are zero.  One thread per (feature, bin).
__global__ void __launch_bounds__(256)
hist_unfuse_kernel(const gbdt_bin_t* __restrict__ joint, const FusedFeat* __restrict__ feats,
                   int32_t n_features, int32_t n_bins, gbdt_bin_t* __restrict__ out) {
  const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_features * n_bins) return;
  const int32_t f = e / n_bins;
  const int32_t b = e - f * n_bins;
  const FusedFeat ff = feats[f];
  gbdt_bin_t r;
  r.grad = 0.0f;
  r.hess = 0.0f;
  r.count = 0u;
  if (b < (int32_t)ff.levels) {
    const gbdt_bin_t* col = joint + (size_t)ff.col * kFusedCap;
    const int32_t stride = ff.stride, period = stride * (int32_t)ff.levels;
    double g = 0.0, h = 0.0;
    uint32_t n = 0;
    // the joint bins v = hi * period + b * stride + lo (lo < stride) in ascending order, sixteen at a
    // time: their loads are issued together (they do not depend on one another), then summed in order
    int32_t base = b * stride, lo = 0;
    while (base < kFusedCap) {
      gbdt_bin_t c[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int32_t v = base + lo;
        const bool ok = base < kFusedCap && v < kFusedCap;
        c[i].grad = 0.0f;
        c[i].hess = 0.0f;
        c[i].count = 0u;
        if (ok) c[i] = col[v];
        if (++lo == stride) {
          lo = 0;
          base += period;
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        g += (double)c[i].grad;
        h += (double)c[i].hess;
        n += c[i].count;
      }
    }
    r.grad = (float)g;
    r.hess = (float)h;
    r.count = n;
  }
  out[e] = r;
}

// --------------------------------------------------------------- subtract kernel

// sibling = parent - child, element by element over [n_features][n_bins].
__global__ void __launch_bounds__(256)
hist_subtract_kernel(const gbdt_bin_t* parent, const gbdt_bin_t* child, gbdt_bin_t* sibling,
                     int32_t n) {
  const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  const gbdt_bin_t p = parent[e];
  const gbdt_bin_t c = child[e];
  gbdt_bin_t s;
  s.grad = p.grad - c.grad;
  s.hess = p.hess - c.hess;
  s.count = p.count - c.count;
  sibling[e] = s;
}

// Siblings of a tree level: large[j] = parent[parent_slot[j]] - small[j], histograms of n
// (bin, feature) elements; grid.y = j.  The slots travel as kernel arguments.
constexpr int kSiblingTable = 960;
struct SiblingTable {
  int32_t parent_slot[kSiblingTable];
};

__global__ void __launch_bounds__(256)
hist_siblings_kernel(const gbdt_bin_t* __restrict__ parents, const gbdt_bin_t* __restrict__ small,
                     gbdt_bin_t* __restrict__ large, int32_t n, SiblingTable t) {
  const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  const size_t j = blockIdx.y;
  const gbdt_bin_t p = parents[(size_t)t.parent_slot[j] * n + e];
  const gbdt_bin_t c = small[j * n + e];
  gbdt_bin_t s;
  s.grad = p.grad - c.grad;
  s.hess = p.hess - c.hess;
  s.count = p.count - c.count;
  large[j * n + e] = s;
}

// Histogram of an empty leaf: all zero.  (A fill kernel, not a memset node, so the
// call can be captured into a graph.)
__global__ void __launch_bounds__(256) hist_zero_kernel(gbdt_bin_t* hist, int32_t n) {
  const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  gbdt_bin_t z;
  z.grad = 0.0f;
  z.hess = 0.0f;
  z.count = 0;
  hist[e] = z;
}

}  // namespace

#endif  // GBDT_HIST_REDUCE_KERNELS_H_
