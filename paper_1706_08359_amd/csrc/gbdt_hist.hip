// libgbdt_hist: feature-histogram construction, sibling subtraction, best-split scan,
// row partition and leaf-wise tree growth for histogram-based GBDT training on AMD
// gfx950 (MI355X).  This file holds the host side (launch planning, scratch, the C ABI);
// the kernels are in hist_build_kernels.h, hist_reduce_kernels.h, split_kernels.h and
// partition_kernels.h, the layouts in tile_plan.h and batch_plan.h.
// Method: arXiv 1706.08359 -- Alg. 1 (Sec. 3.3) defines the histogram, Sec. 4 /
// Alg. 2 / App. A.1 describe a GPU organisation for older hardware.  What is
// kept from that design: one lane handles a bundle of adjacent features of one
// sample (there 4 bytes, here up to 16); lanes that work in the same step are
// steered to different histogram columns by rotating the feature order per lane;
// work is split by features and by samples with a final reduction pass; small
// bin counts get cheaper variants.
// What is new here is stated at each kernel.
//
// Written for gfx950 only: 64-wide wavefronts, 160 KB LDS per CU, fast integer LDS
// atomics (ds_add_u64 / ds_add_u32; the float form ds_add_f32 is ~35x slower),
// 256 CUs in 8 XCDs.
#include <hip/hip_runtime.h>

#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <mutex>
#include <type_traits>
#include <unordered_map>
#include <utility>
#include <vector>

#include "../../include/gbdt_hist.h"
#include "tile_plan.h"
#include "batch_plan.h"

#include "hist_build_kernels.h"
#include "hist_reduce_kernels.h"
#include "split_kernels.h"
#include "partition_kernels.h"

// Scratch of the no-allocation entry point (gbdt_hist_build_noalloc): the unit counters
// (256 KiB head, as in every scratch buffer of this library) and up to 64 MiB of partial
// histograms.  One copy per GPU the library runs on, held until the process ends.  In host
// code this name is only a stand-in for the symbol: the device address is looked up once
// per device (noalloc_scratch_ptr) and that pointer is what kernels and fills receive.
constexpr size_t kNoAllocPartialBytes = (size_t)64 << 20;
constexpr size_t kNoAllocScratchBytes = (size_t)65536 * sizeof(uint32_t) + kNoAllocPartialBytes;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

namespace {

// ------------------------------------------------------- calibration copy kernel

// Plain copy of n 16-byte words: a kernel of known HBM traffic (n * 16 bytes read, n *
// 16 bytes written) against which the memory counters of a profiler run are scaled.
__global__ void __launch_bounds__(256)
calibration_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// ------------------------------------------------------------------- host state

thread_local char g_hip_err[256] = "";

int hip_fail(hipError_t e, const char* what) {
  snprintf(g_hip_err, sizeof g_hip_err, "%s: %s", what, hipGetErrorString(e));
  return GBDT_EHIP;
}

#define HIP_TRY(expr)                                  \
  do {                                                 \
    hipError_t e_ = (expr);                            \
    if (e_ != hipSuccess) return hip_fail(e_, #expr);  \
  } while (0)

std::atomic<int> g_deterministic{0};
std::atomic<int> g_wide{0};  // wide (fp64-grade) accumulation, see gbdt_set_wide_accumulation

struct Workspace {
  std::mutex mu;
  void* own = nullptr;  // library-owned scratch
  size_t own_bytes = 0;
  int own_device = -1;
  std::vector<void*> retired;  // outgrown library buffers: work enqueued earlier may still use them
  void* user = nullptr;  // caller-registered scratch
  size_t user_bytes = 0;
  void* zeroed = nullptr;  // the buffer whose counter head is known to be all zero
};
Workspace g_ws;

// The head of every scratch buffer holds the build kernels' unit counters (one per
// feature tile, at most 65535 tiles); the scratch handed to a call starts behind it.
constexpr int kCounterSlots = 65536;
constexpr size_t kWsHeadBytes = (size_t)kCounterSlots * sizeof(uint32_t);
static_assert(kNoAllocScratchBytes == kWsHeadBytes + kNoAllocPartialBytes, "head of the fixed scratch");

bool stream_is_capturing(hipStream_t s) {
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &cs) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return cs == hipStreamCaptureStatusActive;
}

// Returns a scratch pointer of at least `bytes` for work enqueued on stream s, growing
// the library-owned buffer when no caller buffer is registered.  Growing allocates a
// new buffer and RETIRES the old one (kernels enqueued earlier may still use it; retired
// buffers are freed by gbdt_reset): no synchronisation, no free inside an enqueuing
// call.  It is refused (GBDT_ENOMEM) while s is being captured into a graph, where an
// allocation is not allowed: run the same call once outside the capture first, or
// register a caller buffer.  counters_out: the counter head of the same buffer;
// *counters_zero_out: whether it is known to be all zero.
int get_workspace(size_t bytes, hipStream_t s, void** out, uint32_t** counters_out = nullptr,
                  bool* counters_zero_out = nullptr) {
  std::lock_guard<std::mutex> lk(g_ws.mu);
  bytes += kWsHeadBytes;
  void* base = nullptr;
  if (g_ws.user) {
    if (bytes > g_ws.user_bytes) {
      snprintf(g_hip_err, sizeof g_hip_err, "caller workspace of %zu bytes, %zu needed", g_ws.user_bytes, bytes);
      return GBDT_ENOMEM;
    }
    base = g_ws.user;
  } else {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (!g_ws.own || g_ws.own_device != dev || g_ws.own_bytes < bytes) {
      if (stream_is_capturing(s)) {
        snprintf(g_hip_err, sizeof g_hip_err,
                 "library scratch must grow to %zu bytes, which is not possible during stream capture", bytes);
        return GBDT_ENOMEM;
      }
      size_t want = bytes < (size_t)(1 << 20) ? (size_t)(1 << 20) : bytes;
      if (g_ws.own && g_ws.own_device == dev && want < 2 * g_ws.own_bytes) want = 2 * g_ws.own_bytes;
      void* fresh = nullptr;
      hipError_t e = hipMalloc(&fresh, want);
      if (e != hipSuccess && want > bytes) e = hipMalloc(&fresh, want = bytes);
      if (e != hipSuccess) {
        hip_fail(e, "hipMalloc(workspace)");
        return GBDT_ENOMEM;
      }
      if (g_ws.own) g_ws.retired.push_back(g_ws.own);
      g_ws.own = fresh;
      g_ws.own_bytes = want;
      g_ws.own_device = dev;
    }
    base = g_ws.own;
  }
  *out = (char*)base + kWsHeadBytes;
  if (counters_out) *counters_out = (uint32_t*)base;
  if (counters_zero_out) *counters_zero_out = g_ws.zeroed == base;
  return GBDT_OK;
}

// Records whether the counter head of the buffer `counters` heads is all zero.
void set_counters_zero(uint32_t* counters, bool zero) {
  std::lock_guard<std::mutex> lk(g_ws.mu);
  if (zero) {
    g_ws.zeroed = counters;
  } else if (g_ws.zeroed == counters) {
    g_ws.zeroed = nullptr;
  }
}

// Device address of `scratch` on the current device, looked up on the first call there
// (every GPU holds its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
int noalloc_scratch_ptr(void** out) {
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return GBDT_EUNSUPPORTED;
  std::lock_guard<std::mutex> lk(mu);
  if (!ptr[dev]) {
    void* q = nullptr;
    HIP_TRY(hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)));
    if (!q) return GBDT_EHIP;
    ptr[dev] = q;
  }
  *out = ptr[dev];
  return GBDT_OK;
}

// ---- fused columns (see FusedCol in hist_build_kernels.h): which packed matrices have a fused
// copy, keyed by the address gbdt_bins_pack wrote them to
struct FusedEntry {
  const uint8_t* tiles = nullptr;     // the fused copy's feature tiles
  const FusedFeat* feats = nullptr;   // [n_features] on the device, inside the fused copy
  int64_t n_rows = 0;
  int32_t n_features = 0, n_bins = 0, n_cols = 0;
};
std::mutex g_fused_mu;
std::unordered_map<const void*, FusedEntry> g_fused;

bool fused_lookup(const void* packed, int64_t n_rows, int32_t n_features, int32_t n_bins, FusedEntry* out) {
  static const bool off = [] {
    const char* e = getenv("GBDT_HIST_NO_FUSE");  // tuning experiments: always build from the plain tiles
    return e && atoi(e) > 0;
  }();
  if (off) return false;
  std::lock_guard<std::mutex> lk(g_fused_mu);
  auto it = g_fused.find(packed);
  if (it == g_fused.end()) return false;
  const FusedEntry& e = it->second;
  if (e.n_rows != n_rows || e.n_features != n_features || e.n_bins != n_bins) return false;
  *out = e;
  return true;
}

// Leaves below this many rows are built from the plain tiles: the extra launch that takes the
// marginals costs more than the atomics the fused columns save.
constexpr int64_t kFusedMinLeafRows = 8192;
// ... and leaves that hold less than a third of the matrix's rows: a gathered row drags its whole
// 128-byte line along, so sparse leaves are bound by HBM traffic, and a fused copy's rows are wider
// than 4-bit rows (measured on 11 M x 700 with 2..16 levels: 0.78x the time at half of the rows and
// more, break-even at a quarter, 1-3 % slower below).
constexpr int64_t kFusedMinLeafFraction = 3;
// A fused copy is made when it has at most this fraction of the features as columns.
constexpr double kFusedMaxColumnRatio = 0.85;

// Packs features into columns of at most kFusedCap joint levels: features in descending order
// of their level counts, each into the fullest column that still takes it (best fit).
void plan_fusion(const std::vector<uint32_t>& levels, std::vector<FusedCol>* cols, std::vector<FusedFeat>* feats) {
  const int32_t F = (int32_t)levels.size();
  std::vector<int32_t> order(F);
  for (int32_t f = 0; f < F; ++f) order[f] = f;
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return levels[a] > levels[b]; });
  std::vector<uint32_t> prod;                          // joint levels of every column so far
  std::vector<std::vector<int32_t>> open(kFusedCap + 1);  // columns by joint levels, with room for another part
  cols->clear();
  feats->assign(F, FusedFeat{});
  for (int32_t f : order) {
    const uint32_t L = levels[f] < 1 ? 1 : levels[f];
    int32_t c = -1;
    for (uint32_t pr = kFusedCap / L; pr >= 1 && c < 0; --pr) {
      if (!open[pr].empty()) {
        c = open[pr].back();
        open[pr].pop_back();
      }
    }
    if (c < 0) {
      c = (int32_t)cols->size();
      FusedCol col;
      for (int k = 0; k < kFusedMaxParts; ++k) {
        col.feature[k] = -1;
        col.stride[k] = 0;
      }
      col.n_parts = 0;
      col.pad = 0;
      cols->push_back(col);
      prod.push_back(1);
    }
    FusedCol& col = (*cols)[c];
    col.feature[col.n_parts] = f;
    col.stride[col.n_parts] = (uint8_t)prod[c];
    FusedFeat& ff = (*feats)[f];
    ff.col = c;
    ff.stride = (uint8_t)prod[c];
    ff.levels = (uint8_t)L;
    ff.pad[0] = ff.pad[1] = 0;
    col.n_parts += 1;
    prod[c] *= L;
    if (col.n_parts < kFusedMaxParts && prod[c] <= kFusedCap) open[prod[c]].push_back(c);
  }
}

// Byte layout of a fused copy with n_cols columns: [feature tiles][slack][FusedFeat x n_features][FusedCol x n_cols]
struct FusedLayout {
  TilePlan plan;
  size_t feats_off, cols_off, total;
};
FusedLayout fused_layout(int64_t n_rows, int32_t n_features, int32_t n_cols) {
  FusedLayout l;
  l.plan = make_tile_plan(n_cols, kFusedCap);
  const size_t tiles = (size_t)n_rows * l.plan.row_bytes + (size_t)kPlanSlackBytes;
  l.feats_off = (tiles + 255) / 256 * 256;
  l.cols_off = (l.feats_off + (size_t)n_features * sizeof(FusedFeat) + 255) / 256 * 256;
  l.total = (l.cols_off + (size_t)n_cols * sizeof(FusedCol) + 255) / 256 * 256;
  return l;
}

// Optional timing of the build kernel alone (it shares its C-ABI call with the merge
// kernel): when enabled, every gbdt_hist_build records a HIP event on the call's
// stream right before and right after the build kernel.
struct Profile {
  std::mutex mu;
  bool on = false;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pairs;
};
Profile g_prof;

int device_cu_count() {
  static int cached_dev = -1, cached_cus = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (dev != cached_dev) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    cached_cus = cus;
    cached_dev = dev;
  }
  return cached_cus;
}

constexpr size_t kLdsPerCu = 160 * 1024;
constexpr int kMinRowsPerChunk = kEpochRows;
static_assert(kPlanSlackBytes == (int64_t)kEpochRows * 64, "slack behind the tiles: one epoch of the widest tile");
constexpr int kBuildThreads = 512;  // threads per workgroup of every build kernel variant

struct BuildGeom {
  TilePlan plan;
  int nt;               // threads per workgroup
  size_t lds_bytes;     // LDS per workgroup
  int wgs;              // workgroups per tile
  int unit_epochs;      // epochs per unit
  bool one_unit_each;   // short leaf: every workgroup has exactly one unit, no counter
  int blocks_per_wg;    // partial blocks a workgroup writes: 1, or 2 with wide accumulation
  size_t partial_words;  // total words of all partial blocks
};

// Leaves of at most this many epochs get ONE workgroup per tile, which writes the
// finished histogram itself: a second launch (the reduction pass) would cost more than
// the few epochs a second workgroup could take over.
constexpr int kDirectEpochs = 4;

// When an index-list build gathers grad / hess into leaf order first: with several feature
// tiles (each would gather the same scattered values again), a leaf that is sparse in the
// matrix (scattered 4-byte reads cost a memory sector each) and big enough for the saving
// to exceed one more small launch.  While the two arrays fit an XCD's L2 (4 MB) the tiles'
// gathers mostly hit there and only leaves below a fifth of the rows gain; beyond that,
// leaves up to half of the rows do.  Measured: 10-45 % off the build kernel of such leaves
// on the 137-, 500- and 700-feature matrices.
constexpr int kStatsGatherMinTiles = 4;
constexpr int64_t kStatsGatherMinRows = 8192;
bool stats_gather_pays(int n_tiles, int64_t list_rows, int64_t rows_per_leaf, int64_t n_rows) {
  const int64_t dense_limit = n_rows >= (1 << 20) ? 2 : 5;  // leaf holds at most 1/2 or 1/5 of the rows
  return n_tiles >= kStatsGatherMinTiles && list_rows >= kStatsGatherMinRows &&
         rows_per_leaf * dense_limit <= n_rows;
}

// Workgroups per tile and epochs per unit for a leaf of n_epochs epochs that may use
// `budget` workgroups per tile: units of kUnitEpochs handed out at run time when every
// workgroup gets more than kEvenSplitUnits of them; otherwise (short leaf) the epochs are
// split evenly, one unit per workgroup, and the unit counter is not needed
// (*one_unit_each_out).  With only a few units each, what the run-time hand-out gains in
// balance is less than what whole units lose: a workgroup with 2 units of 4 epochs waits
// for one with 3, while 10 or 11 epochs each end together (measured: 4-19 % on leaves of
// 10-25 % of the rows, nothing lost elsewhere).
constexpr int kEvenSplitUnits = 3;
void plan_leaf_units(int64_t n_epochs, int64_t budget, int* wgs_out, int* unit_epochs_out,
                     bool* one_unit_each_out) {
  int64_t wgs = budget;
  if (wgs > n_epochs) wgs = n_epochs;
  if (n_epochs <= kDirectEpochs) wgs = 1;
  if (wgs < 1) wgs = 1;
  int unit_epochs = kUnitEpochs;
  bool one_each = false;
  if (wgs * kUnitEpochs * kEvenSplitUnits >= n_epochs) {
    unit_epochs = (int)((n_epochs + wgs - 1) / wgs);
    if (unit_epochs < 1) unit_epochs = 1;
    const int64_t n_units = (n_epochs + unit_epochs - 1) / unit_epochs;
    if (n_units >= 1 && wgs > n_units) wgs = n_units;  // no workgroup without a unit
    one_each = true;
  }
  *wgs_out = (int)wgs;
  *unit_epochs_out = unit_epochs;
  *one_unit_each_out = one_each;
}

// Chooses the grid: as many workgroups per tile as fit the machine at once (they stay
// until their tile's units are used up), and the unit size.  wg_per_cu: resident
// workgroups per CU of the kernel variant as reported by the runtime (<= 0: estimate
// from the LDS footprint alone).
BuildGeom make_geom(int32_t n_features, int32_t n_bins, int64_t n_leaf, int cus,
                    int wg_per_cu_hint, bool wide = false, int64_t max_wgs = (int64_t)1 << 40) {
  BuildGeom g;
  g.plan = make_tile_plan(n_features, n_bins);
  const TilePlan& p = g.plan;
  g.nt = kBuildThreads;
  g.blocks_per_wg = wide ? 2 : 1;
  const size_t main_block = (size_t)3 * plan_cells(p, p.wm);
  g.lds_bytes = (size_t)plan_cells(p, p.wm) * 8 * g.blocks_per_wg + 4 * (g.nt / 64) * sizeof(float) + 8;
  int wg_per_cu = wg_per_cu_hint;
  if (wg_per_cu <= 0) {
    wg_per_cu = (int)(kLdsPerCu / g.lds_bytes);
    const int by_threads = 2048 / g.nt;
    if (wg_per_cu > by_threads) wg_per_cu = by_threads;
  }
  if (wg_per_cu < 1) wg_per_cu = 1;
  const int64_t resident = (int64_t)cus * wg_per_cu;
  const int n_tiles = plan_n_tiles(p);
  const int64_t n_epochs = (n_leaf + kEpochRows - 1) / kEpochRows;
  // (A narrow tile's epochs are cheaper, but not by much: the per-epoch overhead does
  // not shrink with the tile.  It gets as many workgroups as a main tile.)
  int64_t budget = resident / n_tiles;
  if (budget > max_wgs) budget = max_wgs;
  plan_leaf_units(n_epochs, budget, &g.wgs, &g.unit_epochs, &g.one_unit_each);
  g.partial_words = ((size_t)p.n_main * g.wgs * main_block +
                     (size_t)(p.wr ? g.wgs : 0) * 3 * (p.wr ? plan_cells(p, p.wr) : 0)) *
                    g.blocks_per_wg;
  return g;
}

// Kernel variants: bin capacity -> (main tile width, 4-bit, waves per SIMD the
// register budget is set for).
#define GBDT_VARIANT_16 16, 64, true, kBuildThreads, 8, double
#define GBDT_VARIANT_64 64, 64, false, kBuildThreads, 6, float
#define GBDT_VARIANT_256 256, 32, false, kBuildThreads, 4, float
// The same with wide accumulation: twice the LDS, fp64 accumulators.
#define GBDT_VARIANT_16W 16, 64, true, kBuildThreads, 6, double
#define GBDT_VARIANT_64W 64, 64, false, kBuildThreads, 4, double
#define GBDT_VARIANT_256W 256, 32, false, kBuildThreads, 2, double

template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC, bool INDEXED, bool WIDE = false>
int query_occupancy() {
  int n = 0;
  hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(
      &n, reinterpret_cast<const void*>(hist_build_kernel<CAP, WM, NIB, NT, WPE, ACC, INDEXED, WIDE>), NT, 0);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return n;
}

// Resident workgroups per CU of the build kernel variant for this bin capacity
// (registers, LDS and wave slots taken into account by the runtime); cached.
int build_wg_per_cu(int cap, bool indexed, bool wide = false) {
  // GBDT_HIST_WG_PER_CU overrides the runtime's answer (tuning experiments only)
  if (const char* e = getenv("GBDT_HIST_WG_PER_CU")) {
    const int v = atoi(e);
    if (v > 0) return v;
  }
  static int cache[6][2] = {{-1, -1}, {-1, -1}, {-1, -1}, {-1, -1}, {-1, -1}, {-1, -1}};
  const int ci = cap == 16 ? 0 : (cap == 64 ? 1 : 2);
  int& c = cache[ci + (wide ? 3 : 0)][indexed ? 1 : 0];
  if (c < 0 && wide) {
    if (cap == 16) c = indexed ? query_occupancy<GBDT_VARIANT_16W, true, true>() : query_occupancy<GBDT_VARIANT_16W, false, true>();
    else if (cap == 64) c = indexed ? query_occupancy<GBDT_VARIANT_64W, true, true>() : query_occupancy<GBDT_VARIANT_64W, false, true>();
    else c = indexed ? query_occupancy<GBDT_VARIANT_256W, true, true>() : query_occupancy<GBDT_VARIANT_256W, false, true>();
  }
  if (c < 0) {
    if (cap == 16) c = indexed ? query_occupancy<GBDT_VARIANT_16, true>() : query_occupancy<GBDT_VARIANT_16, false>();
    else if (cap == 64) c = indexed ? query_occupancy<GBDT_VARIANT_64, true>() : query_occupancy<GBDT_VARIANT_64, false>();
    else c = indexed ? query_occupancy<GBDT_VARIANT_256, true>() : query_occupancy<GBDT_VARIANT_256, false>();
  }
  return c;
}

// Work split of split_gain_kernel over the n_hists histograms of a launch.  group: features a
// workgroup holds in local memory at a time; passes: groups it takes one after the other; n_wg:
// workgroups, and candidates, per histogram.  A workgroup's time is a chain of latencies (loads,
// the serial fp64 prefix, the candidate's hand-off) that hardly depends on the group, so a lone
// histogram is spread over about 256 workgroups, and a launch with many histograms gets larger
// groups (up to 16 features: more leave too few workgroups per CU to hide those latencies), then
// up to 4 passes, aiming at 500-1000 workgroups in all.  (2,000 features x 63 bins, 64
// histograms: 188 us with 8 features per workgroup as for a lone histogram, 85 us with 16 x 4;
// 137 x 255, 64 histograms: 113 us with one feature per workgroup, 40 us with 7 x 2.)
struct SplitGrouping {
  int group, passes, n_wg;
};
SplitGrouping split_grouping(int32_t n_features, int32_t n_bins, int32_t n_hists) {
  SplitGrouping g;
  int cap = kSplitLdsBudget / split_feature_bytes(n_bins);
  if (cap > 16) cap = 16;
  if (cap < 1) cap = 1;
  const int spread = (n_features + 255) / 256;  // a lone histogram: about 256 groups
  const int64_t total = (int64_t)n_features * (n_hists > 0 ? n_hists : 1);
  const int64_t shared = (total + 511) / 512;   // many histograms: about 512 groups in all
  g.group = (int)(shared > spread ? shared : spread);
  if (g.group > cap) g.group = cap;
  if (g.group < 1) g.group = 1;
  const int n_groups = (n_features + g.group - 1) / g.group;
  const int64_t wgs = (int64_t)n_groups * (n_hists > 0 ? n_hists : 1);
  g.passes = (int)((wgs + 1023) / 1024);
  if (g.passes > 4) g.passes = 4;
  if (g.passes > n_groups) g.passes = n_groups;
  if (g.passes < 1) g.passes = 1;
  g.n_wg = (n_groups + g.passes - 1) / g.passes;
  return g;
}

// GBDT_HIST_CHECK_INPUTS=1 (debugging): every call that takes a row list first counts its
// out-of-range entries on the device, WAITS for the stream and fails with GBDT_EINVAL if
// there are any, instead of the undefined behaviour of the unchecked path.
bool check_inputs_enabled() {
  static const bool on = [] {
    const char* e = getenv("GBDT_HIST_CHECK_INPUTS");
    return e && atoi(e) > 0;
  }();
  return on;
}

int check_row_ids(const int32_t* idx, int64_t n, int64_t n_rows, hipStream_t s) {
  if (!check_inputs_enabled() || !idx || n <= 0) return GBDT_OK;
  void* ws = nullptr;
  int rc = get_workspace(256, s, &ws);
  if (rc != GBDT_OK) return rc;
  unsigned long long* n_bad = (unsigned long long*)ws;
  hipLaunchKernelGGL(counters_zero_kernel, dim3(1), dim3(256), 0, s, (uint32_t*)ws, 2);
  HIP_TRY(hipGetLastError());
  const int64_t blocks = (n + 255) / 256;
  hipLaunchKernelGGL(row_ids_check_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s, idx,
                     n, n_rows, n_bad);
  HIP_TRY(hipGetLastError());
  unsigned long long bad = 0;
  HIP_TRY(hipMemcpyAsync(&bad, n_bad, sizeof bad, hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  if (bad) {
    snprintf(g_hip_err, sizeof g_hip_err, "%llu row ids outside [0, n_rows)", bad);
    return GBDT_EINVAL;
  }
  return GBDT_OK;
}

bool valid_shape(int64_t n_rows, int32_t n_features, int32_t n_bins) {
  return n_rows >= 0 && n_features > 0 && n_bins >= 2 && n_bins <= 256;
}

// Brackets the build kernel with events while profiling is enabled.
struct BuildTimer {
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  bool on = false;
  int begin(hipStream_t s) {
    {
      std::lock_guard<std::mutex> lk(g_prof.mu);
      on = g_prof.on;
    }
    if (on) {
      HIP_TRY(hipEventCreate(&ev0));
      HIP_TRY(hipEventCreate(&ev1));
      HIP_TRY(hipEventRecord(ev0, s));
    }
    return GBDT_OK;
  }
  int end(hipStream_t s) {
    if (on) {
      HIP_TRY(hipEventRecord(ev1, s));
      std::lock_guard<std::mutex> lk(g_prof.mu);
      g_prof.pairs.emplace_back(ev0, ev1);
    }
    return GBDT_OK;
  }
};

template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC, bool WIDE = false>
int launch_build(const BuildArgs& a, int blocks, hipStream_t s, bool timed = true) {
  BuildTimer timer;
  int rc = timed ? timer.begin(s) : GBDT_OK;
  if (rc != GBDT_OK) return rc;
  if (a.idx) {
    hipLaunchKernelGGL((hist_build_kernel<CAP, WM, NIB, NT, WPE, ACC, true, WIDE>), dim3(blocks), dim3(NT), 0, s,
                       a);
  } else {
    hipLaunchKernelGGL((hist_build_kernel<CAP, WM, NIB, NT, WPE, ACC, false, WIDE>), dim3(blocks), dim3(NT), 0, s,
                       a);
  }
  HIP_TRY(hipGetLastError());
  return timer.end(s);
}

template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC, bool WIDE = false>
int launch_build_batch(const BatchArgs& a, int blocks, hipStream_t s) {
  BuildTimer timer;
  int rc = timer.begin(s);
  if (rc != GBDT_OK) return rc;
  hipLaunchKernelGGL((hist_build_batch_kernel<CAP, WM, NIB, NT, WPE, ACC, WIDE>), dim3(blocks), dim3(NT), 0, s, a);
  HIP_TRY(hipGetLastError());
  return timer.end(s);
}

template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC>
size_t variant_column_words(const TilePlan& p) {
  return column_words<CAP, WM, NIB, NT>(p.n_main, p.wr);
}

// Plan of one batched launch: leaves [l0, l0 + n) of the call share the machine in
// proportion to their epochs, at least one workgroup per tile each.
struct BatchPlan {
  BatchLeaf leaf[kBatchLeaves];
  int n = 0;
  uint32_t total_wgs = 0;  // workgroups per tile over all leaves
};

BatchPlan plan_batch(const int64_t* leaf_offsets, int32_t l0, int32_t n, int64_t resident,
                     int n_tiles) {
  BatchPlan b;
  b.n = n;
  int64_t total_epochs = 0;
  for (int i = 0; i < n; ++i)
    total_epochs += (leaf_offsets[l0 + i + 1] - leaf_offsets[l0 + i] + kEpochRows - 1) / kEpochRows;
  int64_t budget = resident / n_tiles;
  if (budget < 1) budget = 1;
  uint32_t first = 0;
  for (int i = 0; i < n; ++i) {
    const int64_t rows = leaf_offsets[l0 + i + 1] - leaf_offsets[l0 + i];
    const int64_t n_epochs = (rows + kEpochRows - 1) / kEpochRows;
    int wgs = 0, unit_epochs = 1;
    bool one_each = false;
    if (n_epochs > 0) plan_leaf_units(n_epochs, budget * n_epochs / total_epochs, &wgs, &unit_epochs, &one_each);
    b.leaf[i].row_off = (uint32_t)(leaf_offsets[l0 + i] - leaf_offsets[l0]);
    b.leaf[i].n = (uint32_t)rows;
    b.leaf[i].first_wg = first;
    b.leaf[i].wgs_unit = (uint32_t)wgs | ((uint32_t)unit_epochs << 16);
    first += (uint32_t)wgs;
  }
  b.total_wgs = first;
  return b;
}

// Split search of n_hists (<= kSplitMaxHists) histograms, hist_stride bins apart, in one
// launch; splits_out[i] receives the record of histogram i.
int launch_split(const gbdt_bin_t* hists, int64_t hist_stride, int32_t n_hists, float lambda,
                 float min_child_hess, gbdt_split_t* splits_out, int32_t n_features, int32_t n_bins,
                 hipStream_t s, gbdt_split_t* host_mirror = nullptr, const SplitSiblings* siblings = nullptr) {
  const SplitGrouping sg = split_grouping(n_features, n_bins, n_hists);
  void* ws = nullptr;
  int rc = get_workspace((size_t)n_hists * sg.n_wg * sizeof(SplitCand), s, &ws);
  if (rc != GBDT_OK) return rc;
  const size_t lds = (size_t)sg.group * split_feature_bytes(n_bins);
  SplitSiblings sib;
  if (siblings) {
    sib = *siblings;
  } else {
    memset(&sib, 0, sizeof sib);
  }
  // (only with siblings does the kernel write to the histograms)
  hipLaunchKernelGGL(split_gain_kernel, dim3(sg.n_wg, n_hists), dim3(kSplitThreads), lds, s,
                     const_cast<gbdt_bin_t*>(hists), hist_stride, n_features, n_bins, sg.group, sg.passes,
                     (double)lambda, (double)min_child_hess, (SplitCand*)ws, splits_out, host_mirror, sib);
  HIP_TRY(hipGetLastError());
  return GBDT_OK;
}

// Scratch of gbdt_grow_tree.
size_t align256(size_t b) { return (b + 255) / 256 * 256; }

// gbdt_grow_tree expands up to kGrowRound open leaves per round (one wait for the stream per
// round instead of one per split) and may expand leaves that best-first growth never gets to
// before the leaf budget is used up; the histogram pool is sized for the splits of the tree plus
// that many speculative ones.
constexpr int kGrowRound = 32;
static_assert(kGrowRound <= kSplitSiblings, "a round's siblings travel as one kernel argument");
int32_t grow_speculative_budget(int32_t max_leaves) { return (max_leaves - 1) / 2 + 16; }
int32_t grow_max_expansions(int32_t max_leaves) { return (max_leaves - 1) + grow_speculative_budget(max_leaves); }

struct TreeScratch {
  size_t rows_a, rows_b, rows_small, hists, recs, total;  // byte offsets
  size_t row_elems;   // int32 entries between the two row buffers
  int32_t n_slots;    // histograms in the pool
};

TreeScratch tree_scratch_layout(int64_t n_rows, int32_t n_features, int32_t n_bins, int32_t max_leaves) {
  TreeScratch t;
  const size_t rows = align256((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(int32_t));
  t.row_elems = rows / sizeof(int32_t);
  t.n_slots = 1 + 2 * grow_max_expansions(max_leaves);
  t.rows_a = 0;
  t.rows_b = rows;
  t.rows_small = 2 * rows;  // the smaller children of a round: at most half of the rows
  t.hists = t.rows_small + align256(((size_t)(n_rows > 0 ? n_rows : 1) / 2 + 1) * sizeof(int32_t));
  t.recs = t.hists + align256((size_t)t.n_slots * n_features * n_bins * sizeof(gbdt_bin_t));
  t.total = t.recs + align256((size_t)t.n_slots * sizeof(gbdt_split_t));
  return t;
}

// Page-locked host memory of gbdt_grow_tree (one block per process, never freed): the split
// records of a round, which the split search writes there as well as to device memory (the
// host reads them after waiting for the stream, without a copy).  *dev_out: the address the
// device uses for it.
constexpr int kGrowPinnedRecs = 2 * kGrowRound;
gbdt_split_t* pinned_records(gbdt_split_t** dev_out) {
  static gbdt_split_t* p = nullptr;
  static gbdt_split_t* d = nullptr;
  static std::mutex mu;
  std::lock_guard<std::mutex> lk(mu);
  if (!p) {
    void* q = nullptr;
    if (hipHostMalloc(&q, kGrowPinnedRecs * sizeof(gbdt_split_t), hipHostMallocMapped) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    void* dq = nullptr;
    if (hipHostGetDevicePointer(&dq, q, 0) != hipSuccess) {
      (void)hipGetLastError();
      (void)hipHostFree(q);
      return nullptr;
    }
    p = (gbdt_split_t*)q;
    d = (gbdt_split_t*)dq;
  }
  *dev_out = d;
  return p;
}


// Scratch of gbdt_grow_tree_depthwise: two row buffers, the smaller children's rows, two
// levels of histograms, the split records of a level and the records its partition uses.
constexpr int kMaxTreeDepth = 16;
struct LevelScratch {
  size_t rows_a, rows_b, rows_small, hists_a, hists_b, recs, part_recs, total;
};

LevelScratch level_scratch_layout(int64_t n_rows, int32_t n_features, int32_t n_bins, int32_t max_depth) {
  LevelScratch t;
  const size_t rows = align256((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(int32_t));
  const size_t width = (size_t)1 << max_depth;
  const size_t hists = align256(width * n_features * n_bins * sizeof(gbdt_bin_t));
  const size_t recs = align256(width * sizeof(gbdt_split_t));
  t.rows_a = 0;
  t.rows_b = rows;
  t.rows_small = 2 * rows;
  t.hists_a = 3 * rows;
  t.hists_b = t.hists_a + hists;
  t.recs = t.hists_b + hists;
  t.part_recs = t.recs + recs;
  t.total = t.part_recs + recs;
  return t;
}

// Page-locked host memory for the split records of a level (grows, never freed).
gbdt_split_t* pinned_level_records(size_t n) {
  static gbdt_split_t* p = nullptr;
  static size_t cap = 0;
  static std::mutex mu;
  std::lock_guard<std::mutex> lk(mu);
  if (cap < n) {
    if (p) (void)hipHostFree(p);
    p = nullptr;
    cap = 0;
    void* q = nullptr;
    if (hipHostMalloc(&q, n * sizeof(gbdt_split_t), hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    p = (gbdt_split_t*)q;
    cap = n;
  }
  return p;
}

// gbdt_hist_build, with the scratch either the library's workspace (fixed_base == NULL) or a
// fixed buffer of fixed_bytes whose head holds the unit counters (the no-allocation entry
// point): then nothing is allocated, the grid shrinks until its partial blocks fit, and
// the counters are zeroed by every call that uses them.
int hist_build_impl(const void* bin_matrix, int64_t n_rows, int32_t n_features, int32_t n_bins,
                    const int32_t* leaf_row_idx, int64_t n_leaf_rows, const float* grad,
                    const float* hess, gbdt_bin_t* hist_out, void* stream, void* fixed_base,
                    size_t fixed_bytes) {
  g_hip_err[0] = 0;
  if (!valid_shape(n_rows, n_features, n_bins)) return GBDT_EINVAL;
  if (!hist_out) return GBDT_EINVAL;
  if (n_leaf_rows < 0) return GBDT_EINVAL;
  if (!leaf_row_idx && n_leaf_rows > n_rows) return GBDT_EINVAL;
  if (n_rows >= ((int64_t)1 << 30) || n_leaf_rows >= ((int64_t)1 << 31)) return GBDT_EUNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (n_leaf_rows == 0) {
    const int32_t n = n_features * n_bins;
    hipLaunchKernelGGL(hist_zero_kernel, dim3((n + 255) / 256), dim3(256), 0, s, hist_out, n);
    HIP_TRY(hipGetLastError());
    return GBDT_OK;
  }
  if (!bin_matrix || !grad || !hess) return GBDT_EINVAL;
  if (!fixed_base) {  // (the checking kernel's counter lives in the library's workspace)
    const int rc_ids = check_row_ids(leaf_row_idx, n_leaf_rows, n_rows, s);
    if (rc_ids != GBDT_OK) return rc_ids;
  }

  const bool wide = g_wide.load() != 0;
  // A fused copy of the matrix (few-level features sharing columns): the build kernel then sees
  // build_f one-byte columns of kFusedCap joint bins, and the marginals are taken at the end.
  FusedEntry fe;
  // (not with wide accumulation: the joint histograms are rounded to fp32 before the marginals are
  // taken, which would break that mode's promise of the exact sum rounded once)
  const bool fused = !wide && n_leaf_rows >= kFusedMinLeafRows && n_leaf_rows * kFusedMinLeafFraction >= n_rows &&
                     fused_lookup(bin_matrix, n_rows, n_features, n_bins, &fe);
  const int32_t real_features = n_features, real_bins = n_bins;
  if (fused) {
    n_features = fe.n_cols;
    n_bins = kFusedCap;
  }
  const size_t joint_words = fused ? (size_t)n_features * n_bins * 3 : 0;
  const int wg_per_cu = build_wg_per_cu(make_tile_plan(n_features, n_bins).cap, leaf_row_idx != nullptr, wide);
  BuildGeom g = make_geom(n_features, n_bins, n_leaf_rows, device_cu_count(), wg_per_cu, wide);
  if (fixed_base) {
    // fewer workgroups per tile until the partial blocks fit the fixed buffer
    size_t avail_words = fixed_bytes > kWsHeadBytes ? (fixed_bytes - kWsHeadBytes) / 4 : 0;
    avail_words = avail_words > joint_words ? avail_words - joint_words : 0;
    if (g.partial_words > avail_words) {
      const size_t per_wg = g.partial_words / (size_t)g.wgs;  // words of one workgroup of every tile
      const int64_t fit = (int64_t)(avail_words / per_wg);
      if (fit < 1) {
        snprintf(g_hip_err, sizeof g_hip_err,
                 "%d features x %d bins need %zu bytes of partial histograms, the fixed scratch holds %zu",
                 n_features, n_bins, per_wg * 4, avail_words * 4);
        return GBDT_EUNSUPPORTED;
      }
      g = make_geom(n_features, n_bins, n_leaf_rows, device_cu_count(), wg_per_cu, wide, fit);
    }
  }
  const TilePlan& p = g.plan;
  if (plan_n_tiles(p) > 65535) return GBDT_EUNSUPPORTED;
  // byte offsets inside a tile (slack included) are formed in 32 bits
  if ((n_rows + kEpochRows) * (int64_t)p.wm >= ((int64_t)1 << 32)) return GBDT_EUNSUPPORTED;
  void* ws = nullptr;
  uint32_t* counters = nullptr;
  bool counters_zero = false;
  // With an index list and several feature tiles, gather grad / hess into leaf order once
  // instead of letting every tile's workgroups gather them from scattered rows.
  bool by_pos = leaf_row_idx != nullptr && stats_gather_pays(plan_n_tiles(p), n_leaf_rows, n_leaf_rows, n_rows);
  size_t stats_words = by_pos ? 2 * (((size_t)n_leaf_rows + 63) / 64 * 64) : 0;
  int rc = GBDT_OK;
  if (fixed_base) {
    if (kWsHeadBytes + (g.partial_words + joint_words + stats_words) * 4 > fixed_bytes) {  // the gather is optional
      by_pos = false;
      stats_words = 0;
    }
    counters = (uint32_t*)fixed_base;
    ws = (char*)fixed_base + kWsHeadBytes;
    counters_zero = false;
  } else {
    rc = get_workspace((g.partial_words + joint_words + stats_words) * 4, s, &ws, &counters, &counters_zero);
    if (rc == GBDT_ENOMEM && by_pos) {  // a caller's workspace sized for the partial blocks alone: no gather
      by_pos = false;
      stats_words = 0;
      rc = get_workspace((g.partial_words + joint_words) * 4, s, &ws, &counters, &counters_zero);
    }
  }
  if (rc != GBDT_OK) return rc;

  // scratch: [partial blocks][joint histograms of the fused columns][grad / hess in leaf order]
  gbdt_bin_t* joint = (gbdt_bin_t*)((uint32_t*)ws + g.partial_words);
  BuildArgs a;
  a.packed = fused ? fe.tiles : (const uint8_t*)bin_matrix;
  a.idx = leaf_row_idx;
  a.grad = grad;
  a.hess = hess;
  a.stats_by_pos = 0;
  if (by_pos) {
    float* g_leaf = (float*)ws + g.partial_words + joint_words;
    float* h_leaf = g_leaf + stats_words / 2;
    hipLaunchKernelGGL(stats_gather_kernel, dim3((unsigned)((n_leaf_rows + 255) / 256)), dim3(256), 0, s,
                       leaf_row_idx, grad, hess, n_leaf_rows, g_leaf, h_leaf);
    HIP_TRY(hipGetLastError());
    a.grad = g_leaf;
    a.hess = h_leaf;
    a.stats_by_pos = 1;
  }
  a.partials = (uint32_t*)ws;
  a.counters = counters;
  a.n_rows = n_rows;
  a.n_leaf = n_leaf_rows;
  a.n_main = p.n_main;
  a.wr = p.wr;
  a.wgs = g.wgs;
  a.chunks = g.wgs * g.blocks_per_wg;
  a.unit_epochs = g.unit_epochs;
  // no counter when every workgroup has one unit anyway, or when the split must be fixed
  a.fixed_stride = (g.one_unit_each || g_deterministic.load()) ? g.wgs : 0;
  a.direct_out = (g.wgs == 1 && !fused) ? hist_out : nullptr;  // (joint histograms always take the reduction pass)
  a.n_features = n_features;
  a.n_bins = n_bins;
  const int n_tiles = plan_n_tiles(p);
  const int blocks = n_tiles * g.wgs;
  const bool uses_counters = a.fixed_stride == 0;
  // While the stream is being captured nothing runs now, so what is known about the
  // counters must not change: the captured sequence zeroes them itself, before and (if
  // no reduction pass follows) after the build, and leaves them zero on every replay.
  // (the fixed buffer is treated the same way: what is known about it is not tracked)
  const bool capturing = fixed_base != nullptr || stream_is_capturing(s);
  auto zero_counters = [&]() -> int {
    hipLaunchKernelGGL(counters_zero_kernel, dim3(kCounterSlots / 256), dim3(256), 0, s, counters,
                       kCounterSlots);
    HIP_TRY(hipGetLastError());
    return GBDT_OK;
  };
  if (uses_counters && (capturing || !counters_zero)) {  // e.g. a new scratch buffer
    rc = zero_counters();
    if (rc != GBDT_OK) return rc;
  }
  // From here until the reduction pass has been enqueued the counters are in use.
  if (uses_counters && !capturing) set_counters_zero(counters, false);

  const bool timed = fixed_base == nullptr;  // the profiling events are created on the fly: an allocation
  if (wide) {
    if (p.cap == 16) {
      rc = launch_build<GBDT_VARIANT_16W, true>(a, blocks, s, timed);
    } else if (p.cap == 64) {
      rc = launch_build<GBDT_VARIANT_64W, true>(a, blocks, s, timed);
    } else {
      rc = launch_build<GBDT_VARIANT_256W, true>(a, blocks, s, timed);
    }
  } else if (p.cap == 16) {
    rc = launch_build<GBDT_VARIANT_16>(a, blocks, s, timed);
  } else if (p.cap == 64) {
    rc = launch_build<GBDT_VARIANT_64>(a, blocks, s, timed);
  } else {
    rc = launch_build<GBDT_VARIANT_256>(a, blocks, s, timed);
  }
  if (rc != GBDT_OK) return rc;
  if (a.direct_out) {  // one workgroup per tile: the histogram is written
    if (uses_counters && capturing) return zero_counters();
    return GBDT_OK;
  }

  MergeArgs m;
  m.partials = (const uint32_t*)ws;
  m.out = fused ? joint : hist_out;
  m.plan = p;
  m.n_features = n_features;
  m.n_bins = n_bins;
  m.chunks_main = a.chunks;
  m.chunks_rem = p.wr ? a.chunks : 0;
  m.counters = uses_counters ? counters : nullptr;
  const int max_slots = plan_slots(p, p.wm);
  const int mx = (n_bins * max_slots + kMergeCells - 1) / kMergeCells;
  if (merge_lanes((int64_t)mx * plan_n_tiles(p), a.chunks) == kMergeLanesWide) {
    hipLaunchKernelGGL(hist_merge_kernel<kMergeLanesWide>, dim3(mx, plan_n_tiles(p)),
                       dim3(kMergeCells * kMergeLanesWide), 0, s, m);
  } else {
    hipLaunchKernelGGL(hist_merge_kernel<kMergeLanes>, dim3(mx, plan_n_tiles(p)), dim3(kMergeCells * kMergeLanes),
                       0, s, m);
  }
  HIP_TRY(hipGetLastError());
  if (uses_counters && !capturing) set_counters_zero(counters, true);  // the reduction pass leaves them zero
  if (fused) {
    const int32_t n = real_features * real_bins;
    hipLaunchKernelGGL(hist_unfuse_kernel, dim3((n + 255) / 256), dim3(256), 0, s, (const gbdt_bin_t*)joint, fe.feats,
                       real_features, real_bins, hist_out);
    HIP_TRY(hipGetLastError());
  }
  return GBDT_OK;
}


}  // namespace

// ----------------------------------------------------------------------- C ABI

extern "C" {

size_t gbdt_bins_packed_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins) {
  if (!valid_shape(n_rows, n_features, n_bins)) return 0;
  const TilePlan p = make_tile_plan(n_features, n_bins);
  return (size_t)plan_packed_bytes(p, n_rows, n_features);
}

int gbdt_bins_pack(const uint8_t* bins_rowmajor, int64_t n_rows, int32_t n_features,
                   int32_t n_bins, void* packed_out, void* stream) {
  if (!valid_shape(n_rows, n_features, n_bins)) return GBDT_EINVAL;
  if (packed_out) (void)gbdt_bins_unfuse(packed_out);  // a fused copy registered for this address is stale now
  if (n_rows == 0) return GBDT_OK;
  if (!bins_rowmajor || !packed_out) return GBDT_EINVAL;
  if (((uintptr_t)packed_out & 15u) != 0) return GBDT_EINVAL;
  if (n_rows >= ((int64_t)1 << 31)) return GBDT_EUNSUPPORTED;
  const TilePlan p = make_tile_plan(n_features, n_bins);
  const int tiles = plan_n_tiles(p);
  if (tiles > 65535) return GBDT_EUNSUPPORTED;
  const int64_t max_words = n_rows * (p.wm / 4);
  const int64_t bx = (max_words + 255) / 256;
  if (bx >= ((int64_t)1 << 31)) return GBDT_EUNSUPPORTED;
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)bx, (unsigned)tiles), dim3(256), 0,
                     (hipStream_t)stream, bins_rowmajor, n_rows, n_features, p,
                     (uint8_t*)packed_out);
  HIP_TRY(hipGetLastError());
  // the column-major copy behind the tiles
  const int64_t rb = (n_rows + 63) / 64;
  const int32_t fb = (n_features + 63) / 64;
  if (fb > 65535) return GBDT_EUNSUPPORTED;
  hipLaunchKernelGGL(pack_columns_kernel, dim3((unsigned)rb, (unsigned)fb), dim3(256), 0, (hipStream_t)stream,
                     bins_rowmajor, n_rows, n_features, p.nib ? 15u : (uint32_t)(p.cap - 1),
                     (uint8_t*)packed_out + plan_columns_base(p, n_rows), plan_column_stride(n_rows));
  HIP_TRY(hipGetLastError());
  return GBDT_OK;
}

size_t gbdt_bins_fused_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins) {
  if (!valid_shape(n_rows, n_features, n_bins) || n_bins > kFusedCap || n_rows == 0) return 0;
  const int32_t max_cols = (int32_t)(kFusedMaxColumnRatio * n_features);
  if (max_cols < 1) return 0;
  return fused_layout(n_rows, n_features, max_cols).total;
}

int gbdt_bins_unfuse(const void* packed) {
  std::lock_guard<std::mutex> lk(g_fused_mu);
  g_fused.erase(packed);
  return GBDT_OK;
}

int gbdt_bins_fuse(const uint8_t* bins_rowmajor, int64_t n_rows, int32_t n_features, int32_t n_bins,
                   const void* packed, void* fused_out, size_t fused_bytes, int32_t* n_columns_out,
                   void* stream) {
  g_hip_err[0] = 0;
  if (!valid_shape(n_rows, n_features, n_bins) || !n_columns_out || !packed) return GBDT_EINVAL;
  *n_columns_out = 0;
  (void)gbdt_bins_unfuse(packed);
  if (n_bins > kFusedCap || n_rows == 0) return GBDT_OK;  // never fused
  if (!bins_rowmajor || !fused_out) return GBDT_EINVAL;
  if (((uintptr_t)fused_out & 255u) != 0) return GBDT_EINVAL;
  if (fused_bytes < (size_t)n_features * sizeof(uint32_t)) return GBDT_ENOMEM;
  if (n_rows >= ((int64_t)1 << 30)) return GBDT_EUNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (stream_is_capturing(s)) return GBDT_EUNSUPPORTED;  // this call reads results on the host
  // 1. the largest bin value of every feature (the head of fused_out serves as scratch)
  uint32_t* max_dev = (uint32_t*)fused_out;
  hipLaunchKernelGGL(counters_zero_kernel, dim3((n_features + 255) / 256), dim3(256), 0, s, max_dev, n_features);
  HIP_TRY(hipGetLastError());
  const int64_t row_blocks = (n_rows + 255) / 256;
  if (row_blocks >= ((int64_t)1 << 31)) return GBDT_EUNSUPPORTED;
  hipLaunchKernelGGL(feature_max_kernel, dim3((unsigned)row_blocks), dim3(256), 0, s, bins_rowmajor, n_rows,
                     n_features, max_dev);
  HIP_TRY(hipGetLastError());
  std::vector<uint32_t> levels((size_t)n_features);
  HIP_TRY(hipMemcpyAsync(levels.data(), max_dev, levels.size() * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  for (uint32_t& l : levels) {
    l = l + 1;                       // bins 0 .. max occur (at most)
    if (l > (uint32_t)n_bins) l = (uint32_t)n_bins;  // the build masks stray values to the capacity anyway
  }
  // 2. the plan; does it pay?
  std::vector<FusedCol> cols;
  std::vector<FusedFeat> feats;
  plan_fusion(levels, &cols, &feats);
  const int32_t n_cols = (int32_t)cols.size();
  if ((double)n_cols > kFusedMaxColumnRatio * n_features) return GBDT_OK;
  const FusedLayout lay = fused_layout(n_rows, n_features, n_cols);
  if (lay.total > fused_bytes) {
    snprintf(g_hip_err, sizeof g_hip_err, "fused copy needs %zu bytes, %zu given", lay.total, fused_bytes);
    return GBDT_ENOMEM;
  }
  if (plan_n_tiles(lay.plan) > 65535) return GBDT_OK;
  // 3. tables, then the tiles
  char* base = (char*)fused_out;
  HIP_TRY(hipMemcpyAsync(base + lay.feats_off, feats.data(), feats.size() * sizeof(FusedFeat), hipMemcpyHostToDevice, s));
  HIP_TRY(hipMemcpyAsync(base + lay.cols_off, cols.data(), cols.size() * sizeof(FusedCol), hipMemcpyHostToDevice, s));
  const int tiles = plan_n_tiles(lay.plan);
  const int64_t max_words = n_rows * (lay.plan.wm / 4);
  const int64_t bx = (max_words + 255) / 256;
  if (bx >= ((int64_t)1 << 31)) return GBDT_EUNSUPPORTED;
  hipLaunchKernelGGL(pack_fused_kernel, dim3((unsigned)bx, (unsigned)tiles), dim3(256), 0, s, bins_rowmajor, n_rows,
                     n_features, lay.plan, (const FusedCol*)(base + lay.cols_off), n_cols, (uint8_t*)base);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(s));  // the host tables must outlive their copies
  FusedEntry e;
  e.tiles = (const uint8_t*)base;
  e.feats = (const FusedFeat*)(base + lay.feats_off);
  e.n_rows = n_rows;
  e.n_features = n_features;
  e.n_bins = n_bins;
  e.n_cols = n_cols;
  {
    std::lock_guard<std::mutex> lk(g_fused_mu);
    g_fused[packed] = e;
  }
  *n_columns_out = n_cols;
  return GBDT_OK;
}

size_t gbdt_workspace_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins) {
  if (!valid_shape(n_rows, n_features, n_bins)) return 0;
  const int cap = make_tile_plan(n_features, n_bins).cap;
  const bool wide = g_wide.load() != 0;
  const BuildGeom g0 =
      make_geom(n_features, n_bins, n_rows, device_cu_count(), build_wg_per_cu(cap, false, wide), wide);
  const BuildGeom g1 =
      make_geom(n_features, n_bins, n_rows, device_cu_count(), build_wg_per_cu(cap, true, wide), wide);
  size_t b = (g0.partial_words > g1.partial_words ? g0.partial_words : g1.partial_words) * 4 +
             2 * (((size_t)n_rows + 63) / 64 * 64) * 4;  // + grad / hess of a leaf in leaf order
  // + the joint histograms of a fused copy (at most one column per feature)
  if (n_bins <= kFusedCap) b += (size_t)n_features * kFusedCap * sizeof(gbdt_bin_t);
  // gbdt_grow_tree searches the children of a round in one launch
  const size_t cand = (size_t)2 * kGrowRound * split_grouping(n_features, n_bins, 1).n_wg * sizeof(SplitCand);
  if (cand > b) b = cand;
  const size_t part = make_part_geom(n_rows > 0 ? n_rows : 1).bytes;
  if (part > b) b = part;
  return (b + 255) / 256 * 256 + kWsHeadBytes;
}

int gbdt_set_workspace(void* dev_ptr, size_t bytes) {
  if ((dev_ptr == nullptr) != (bytes == 0)) return GBDT_EINVAL;
  if (((uintptr_t)dev_ptr & 255u) != 0) return GBDT_EINVAL;
  std::lock_guard<std::mutex> lk(g_ws.mu);
  g_ws.user = dev_ptr;
  g_ws.user_bytes = bytes;
  g_ws.zeroed = g_ws.zeroed == dev_ptr ? nullptr : g_ws.zeroed;  // a caller buffer starts with unknown contents
  return GBDT_OK;
}

int gbdt_hist_build(const void* bin_matrix, int64_t n_rows, int32_t n_features, int32_t n_bins,
                    const int32_t* leaf_row_idx, int64_t n_leaf_rows, const float* grad,
                    const float* hess, gbdt_bin_t* hist_out, void* stream) {
  return hist_build_impl(bin_matrix, n_rows, n_features, n_bins, leaf_row_idx, n_leaf_rows, grad, hess, hist_out,
                         stream, nullptr, 0);
}

int gbdt_hist_build_noalloc(const void* bin_matrix, int64_t n_rows, int32_t n_features, int32_t n_bins,
                            const int32_t* leaf_row_idx, int64_t n_leaf_rows, const float* grad,
                            const float* hess, gbdt_bin_t* hist_out, void* stream) {
  void* base = nullptr;
  const int rc = noalloc_scratch_ptr(&base);
  if (rc != GBDT_OK) return rc;
  return hist_build_impl(bin_matrix, n_rows, n_features, n_bins, leaf_row_idx, n_leaf_rows, grad, hess, hist_out,
                         stream, base, kNoAllocScratchBytes);
}

size_t gbdt_hist_build_noalloc_max_partial_bytes(void) { return kNoAllocPartialBytes; }

// gbdt_hist_build_batch; with seg_off (gbdt_grow_tree: the leaves of a round are segments of its
// row buffers, not one list back to back) leaf l's rows are row_idx[seg_off[l] .. seg_off[l] + its
// length by leaf_offsets), and grad / hess are always read by row id.
static int hist_build_batch_impl(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                          int32_t n_bins, const int32_t* row_idx, const int64_t* leaf_offsets,
                          int32_t n_leaves, const float* grad, const float* hess,
                          gbdt_bin_t* hist_out, void* stream, const uint32_t* seg_off) {
  if (!valid_shape(n_rows, n_features, n_bins)) return GBDT_EINVAL;
  if (n_leaves < 0) return GBDT_EINVAL;
  if (n_leaves == 0) return GBDT_OK;
  if (!leaf_offsets || !hist_out) return GBDT_EINVAL;
  if (leaf_offsets[0] < 0) return GBDT_EINVAL;
  for (int32_t l = 0; l < n_leaves; ++l)
    if (leaf_offsets[l + 1] < leaf_offsets[l]) return GBDT_EINVAL;
  const int64_t total_rows = leaf_offsets[n_leaves] - leaf_offsets[0];
  if (total_rows > 0 && (!bin_matrix || !row_idx || !grad || !hess)) return GBDT_EINVAL;
  if (total_rows > 0 && n_rows == 0) return GBDT_EINVAL;
  if (n_rows >= ((int64_t)1 << 30)) return GBDT_EUNSUPPORTED;
  // (always from the plain tiles: the leaves of a batch are sparse in the matrix, where a fused copy's
  // wider rows cost more HBM traffic than its fewer columns save in atomics)
  const TilePlan p = make_tile_plan(n_features, n_bins);
  const int n_tiles = plan_n_tiles(p);
  if (n_tiles > 65535) return GBDT_EUNSUPPORTED;
  if ((n_rows + kEpochRows) * (int64_t)p.wm >= ((int64_t)1 << 32)) return GBDT_EUNSUPPORTED;
  const bool wide = g_wide.load() != 0;
  const int64_t resident = (int64_t)device_cu_count() * build_wg_per_cu(p.cap, true, wide);
  // words of the partial blocks of one workgroup column (two blocks each with wide accumulation)
  const size_t col = (p.cap == 16 ? variant_column_words<GBDT_VARIANT_16>(p)
                                  : (p.cap == 64 ? variant_column_words<GBDT_VARIANT_64>(p)
                                                 : variant_column_words<GBDT_VARIANT_256>(p))) *
                     (wide ? 2 : 1);
  // one scratch buffer serves the launches one after the other: size it for the largest
  size_t need_words = 0;
  for (int32_t l0 = 0; l0 < n_leaves; l0 += kBatchLeaves) {
    const int32_t n = n_leaves - l0 < kBatchLeaves ? n_leaves - l0 : kBatchLeaves;
    for (int32_t i = 0; i < n; ++i)
      if (leaf_offsets[l0 + i + 1] - leaf_offsets[l0 + i] >= ((int64_t)1 << 31)) return GBDT_EUNSUPPORTED;
    if (leaf_offsets[l0 + n] - leaf_offsets[l0] >= ((int64_t)1 << 32)) return GBDT_EUNSUPPORTED;
    const BatchPlan b = plan_batch(leaf_offsets, l0, n, resident, n_tiles);
    if ((int64_t)b.total_wgs * n_tiles >= ((int64_t)1 << 31)) return GBDT_EUNSUPPORTED;
    const size_t w = (size_t)b.total_wgs * col;
    if (w > need_words) need_words = w;
  }
  hipStream_t s = (hipStream_t)stream;
  if (total_rows > 0 && !seg_off) {
    const int rc_ids = check_row_ids(row_idx + leaf_offsets[0], total_rows, n_rows, s);
    if (rc_ids != GBDT_OK) return rc_ids;
  }
  // grad / hess of the whole concatenated list in list order, gathered once (see stats_gather_pays)
  bool by_pos = !seg_off && total_rows > 0 && stats_gather_pays(n_tiles, total_rows, total_rows / n_leaves, n_rows);
  size_t stats_words = by_pos ? 2 * (((size_t)total_rows + 63) / 64 * 64) : 0;
  void* ws = nullptr;
  int rc = get_workspace((need_words + stats_words) * 4 + 256, s, &ws);
  if (rc == GBDT_ENOMEM && by_pos) {  // a caller's workspace sized for the partial blocks alone: no gather
    by_pos = false;
    stats_words = 0;
    rc = get_workspace(need_words * 4 + 256, s, &ws);
  }
  if (rc != GBDT_OK) return rc;
  float* g_list = (float*)ws + need_words;
  float* h_list = g_list + stats_words / 2;
  if (by_pos) {
    hipLaunchKernelGGL(stats_gather_kernel, dim3((unsigned)((total_rows + 255) / 256)), dim3(256), 0, s,
                       row_idx + leaf_offsets[0], grad, hess, total_rows, g_list, h_list);
    HIP_TRY(hipGetLastError());
  }
  for (int32_t l0 = 0; l0 < n_leaves; l0 += kBatchLeaves) {
    const int32_t n = n_leaves - l0 < kBatchLeaves ? n_leaves - l0 : kBatchLeaves;
    BatchPlan b = plan_batch(leaf_offsets, l0, n, resident, n_tiles);
    if (seg_off)
      for (int32_t i = 0; i < n; ++i) b.leaf[i].row_off = seg_off[l0 + i];
    BatchMergeArgs m;
    m.m.partials = (const uint32_t*)ws;
    m.m.out = hist_out + (size_t)l0 * n_features * n_bins;
    m.m.plan = p;
    m.m.n_features = n_features;
    m.m.n_bins = n_bins;
    m.m.chunks_main = 0;
    m.m.chunks_rem = 0;
    m.m.counters = nullptr;
    m.column_words = col;
    m.blocks_per_wg = wide ? 2 : 1;
    memcpy(m.leaf, b.leaf, sizeof m.leaf);
    if (b.total_wgs > 0) {
      BatchArgs a;
      a.packed = (const uint8_t*)bin_matrix;
      a.idx = seg_off ? row_idx : row_idx + leaf_offsets[l0];
      a.grad = by_pos ? g_list + (leaf_offsets[l0] - leaf_offsets[0]) : grad;
      a.hess = by_pos ? h_list + (leaf_offsets[l0] - leaf_offsets[0]) : hess;
      a.stats_by_pos = by_pos ? 1 : 0;
      a.partials = (uint32_t*)ws;
      a.n_rows = n_rows;
      a.n_main = p.n_main;
      a.wr = p.wr;
      a.n_leaves = n;
      a.hist_out = hist_out + (size_t)l0 * n_features * n_bins;
      a.n_features = n_features;
      a.n_bins = n_bins;
      memcpy(a.leaf, b.leaf, sizeof a.leaf);
      const int blocks = (int)b.total_wgs * n_tiles;
      if (wide) {
        if (p.cap == 16) {
          rc = launch_build_batch<GBDT_VARIANT_16W, true>(a, blocks, s);
        } else if (p.cap == 64) {
          rc = launch_build_batch<GBDT_VARIANT_64W, true>(a, blocks, s);
        } else {
          rc = launch_build_batch<GBDT_VARIANT_256W, true>(a, blocks, s);
        }
      } else if (p.cap == 16) {
        rc = launch_build_batch<GBDT_VARIANT_16>(a, blocks, s);
      } else if (p.cap == 64) {
        rc = launch_build_batch<GBDT_VARIANT_64>(a, blocks, s);
      } else {
        rc = launch_build_batch<GBDT_VARIANT_256>(a, blocks, s);
      }
      if (rc != GBDT_OK) return rc;
    }
    bool any_to_merge = false;  // empty leaves (zeros) or leaves of several workgroups per tile
    for (int32_t i = 0; i < n; ++i) any_to_merge |= (b.leaf[i].wgs_unit & 0xffffu) != 1u;
    if (!any_to_merge) continue;
    const int max_slots = plan_slots(p, p.wm);
    const int mx = (n_bins * max_slots + kMergeCells - 1) / kMergeCells;
    int32_t most_chunks = 0;
    for (int32_t i = 0; i < n; ++i) {
      const int32_t c = (int32_t)(b.leaf[i].wgs_unit & 0xffffu) * (wide ? 2 : 1);
      most_chunks = c > most_chunks ? c : most_chunks;
    }
    if (merge_lanes((int64_t)mx * n_tiles * n, most_chunks) == kMergeLanesWide) {
      hipLaunchKernelGGL(hist_merge_batch_kernel<kMergeLanesWide>, dim3(mx, n_tiles, n),
                         dim3(kMergeCells * kMergeLanesWide), 0, s, m);
    } else {
      hipLaunchKernelGGL(hist_merge_batch_kernel<kMergeLanes>, dim3(mx, n_tiles, n),
                         dim3(kMergeCells * kMergeLanes), 0, s, m);
    }
    HIP_TRY(hipGetLastError());
  }
  return GBDT_OK;
}

int gbdt_hist_build_batch(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                          int32_t n_bins, const int32_t* row_idx, const int64_t* leaf_offsets,
                          int32_t n_leaves, const float* grad, const float* hess,
                          gbdt_bin_t* hist_out, void* stream) {
  return hist_build_batch_impl(bin_matrix, n_rows, n_features, n_bins, row_idx, leaf_offsets, n_leaves, grad, hess,
                               hist_out, stream, nullptr);
}

size_t gbdt_hist_build_batch_workspace_bytes(int32_t n_features, int32_t n_bins, int32_t n_leaves) {
  if (n_features <= 0 || n_bins < 2 || n_bins > 256 || n_leaves < 0) return 0;
  const TilePlan p = make_tile_plan(n_features, n_bins);
  const int n_tiles = plan_n_tiles(p);
  const bool wide = g_wide.load() != 0;
  const int64_t resident = (int64_t)device_cu_count() * build_wg_per_cu(p.cap, true, wide);
  const size_t col = (p.cap == 16 ? variant_column_words<GBDT_VARIANT_16>(p)
                                  : (p.cap == 64 ? variant_column_words<GBDT_VARIANT_64>(p)
                                                 : variant_column_words<GBDT_VARIANT_256>(p))) *
                     (wide ? 2 : 1);
  // every leaf of a launch gets its share of the resident workgroups, rounded down, but
  // at least one workgroup per tile
  int64_t budget = resident / n_tiles;
  if (budget < 1) budget = 1;
  const int64_t per_launch = n_leaves < kBatchLeaves ? n_leaves : kBatchLeaves;
  // (the call gathers grad / hess into list order only when the scratch has 8 more bytes per listed
  // row to spare; with a caller buffer of exactly this size it reads them by row id)
  const size_t b = (size_t)(budget + per_launch) * col * 4 + 256;
  return (b + 255) / 256 * 256 + kWsHeadBytes;
}

int gbdt_hist_subtract(const gbdt_bin_t* parent, const gbdt_bin_t* child, gbdt_bin_t* sibling_out,
                       int32_t n_features, int32_t n_bins, void* stream) {
  if (!parent || !child || !sibling_out) return GBDT_EINVAL;
  if (n_features <= 0 || n_bins < 2 || n_bins > 256) return GBDT_EINVAL;
  const int32_t n = n_features * n_bins;
  hipLaunchKernelGGL(hist_subtract_kernel, dim3((n + 255) / 256), dim3(256), 0,
                     (hipStream_t)stream, parent, child, sibling_out, n);
  HIP_TRY(hipGetLastError());
  return GBDT_OK;
}

int gbdt_best_split_batch(const gbdt_bin_t* hists, int32_t n_hists, float lambda,
                          float min_child_hess, gbdt_split_t* splits_out, int32_t n_features,
                          int32_t n_bins, void* stream) {
  if (n_hists < 0) return GBDT_EINVAL;
  if (n_features <= 0 || n_bins < 2 || n_bins > 256) return GBDT_EINVAL;
  if (!(lambda >= 0.0f)) return GBDT_EINVAL;
  if (n_hists == 0) return GBDT_OK;
  if (!hists || !splits_out) return GBDT_EINVAL;
  const int64_t stride = (int64_t)n_features * n_bins;
  for (int32_t h0 = 0; h0 < n_hists; h0 += kSplitMaxHists) {
    const int32_t nh = n_hists - h0 < kSplitMaxHists ? n_hists - h0 : kSplitMaxHists;
    const int rc = launch_split(hists + (size_t)h0 * stride, stride, nh, lambda, min_child_hess,
                                splits_out + h0, n_features, n_bins, (hipStream_t)stream);
    if (rc != GBDT_OK) return rc;
  }
  return GBDT_OK;
}

int gbdt_best_split(const gbdt_bin_t* hist, float lambda, float min_child_hess,
                    gbdt_split_t* split_out, int32_t n_features, int32_t n_bins, void* stream) {
  if (!hist || !split_out) return GBDT_EINVAL;
  return gbdt_best_split_batch(hist, 1, lambda, min_child_hess, split_out, n_features, n_bins,
                               stream);
}

int gbdt_partition_rows(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                        int32_t n_bins, const int32_t* leaf_row_idx, int64_t n_leaf_rows,
                        const gbdt_split_t* split, int32_t* children_out, int64_t* n_left_out,
                        void* stream) {
  if (!valid_shape(n_rows, n_features, n_bins)) return GBDT_EINVAL;
  if (!bin_matrix || !split || !children_out) return GBDT_EINVAL;
  if (n_leaf_rows < 0) return GBDT_EINVAL;
  if (!leaf_row_idx && n_leaf_rows > n_rows) return GBDT_EINVAL;
  if (n_rows == 0 && n_leaf_rows > 0) return GBDT_EINVAL;
  if (n_rows >= ((int64_t)1 << 30) || n_leaf_rows >= ((int64_t)1 << 31)) return GBDT_EUNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    const int rc_ids = check_row_ids(leaf_row_idx, n_leaf_rows, n_rows, s);
    if (rc_ids != GBDT_OK) return rc_ids;
  }
  const TilePlan p = make_tile_plan(n_features, n_bins);
  if (n_leaf_rows <= (int64_t)kPartThreads * kPartOneSteps) {  // small leaf: one workgroup, one launch
    hipLaunchKernelGGL(partition_one_kernel, dim3(1), dim3(kPartThreads), 0, s, (const uint8_t*)bin_matrix,
                       n_rows, n_features, p, leaf_row_idx, (int32_t)n_leaf_rows, split, children_out,
                       n_left_out);
    HIP_TRY(hipGetLastError());
    return GBDT_OK;
  }
  const PartGeom g = make_part_geom(n_leaf_rows > 0 ? n_leaf_rows : 1);
  void* ws = nullptr;
  int rc = get_workspace(g.bytes, s, &ws);
  if (rc != GBDT_OK) return rc;
  uint64_t* flags = (uint64_t*)ws;
  uint32_t* chunk_left = (uint32_t*)(flags + g.flag_words);
  hipLaunchKernelGGL(partition_flag_kernel, dim3(g.n_chunks), dim3(kPartThreads), 0, s,
                     (const uint8_t*)bin_matrix, n_rows, n_features, p, leaf_row_idx, n_leaf_rows,
                     split, g.rows_per_thread, flags, chunk_left);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(partition_scatter_kernel, dim3(g.n_chunks), dim3(kPartThreads), 0, s,
                     leaf_row_idx, n_leaf_rows, g.rows_per_thread, (const uint64_t*)flags,
                     (const uint32_t*)chunk_left, g.n_chunks, children_out, n_left_out);
  HIP_TRY(hipGetLastError());
  return GBDT_OK;
}

int gbdt_partition_rows_batch(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                              int32_t n_bins, const int32_t* row_idx, const int64_t* leaf_offsets,
                              int32_t n_leaves, const gbdt_split_t* splits, int32_t* children_out,
                              int64_t* n_left_out, void* stream) {
  if (!valid_shape(n_rows, n_features, n_bins)) return GBDT_EINVAL;
  if (n_leaves < 0) return GBDT_EINVAL;
  if (n_leaves == 0) return GBDT_OK;
  if (!leaf_offsets || !splits) return GBDT_EINVAL;
  if (leaf_offsets[0] < 0) return GBDT_EINVAL;
  int64_t longest = 0;
  for (int32_t l = 0; l < n_leaves; ++l) {
    const int64_t n = leaf_offsets[l + 1] - leaf_offsets[l];
    if (n < 0) return GBDT_EINVAL;
    if (n >= ((int64_t)1 << 31)) return GBDT_EUNSUPPORTED;
    if (n > longest) longest = n;
  }
  const int64_t total_rows = leaf_offsets[n_leaves] - leaf_offsets[0];
  if (total_rows > 0 && (!bin_matrix || !row_idx || !children_out)) return GBDT_EINVAL;
  if (total_rows > 0 && n_rows == 0) return GBDT_EINVAL;
  if (n_rows >= ((int64_t)1 << 30)) return GBDT_EUNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (total_rows > 0) {
    const int rc_ids = check_row_ids(row_idx + leaf_offsets[0], total_rows, n_rows, s);
    if (rc_ids != GBDT_OK) return rc_ids;
  }
  // chunks of 256 * rows_per_thread positions, at most kPartMaxChunks per leaf
  const int32_t rpt = make_part_geom(longest > 0 ? longest : 1).rows_per_thread;
  const int64_t chunk_rows = (int64_t)kPartThreads * rpt;
  // scratch for the launch with the most chunks
  int64_t max_chunks = 0;
  for (int32_t l0 = 0; l0 < n_leaves; l0 += kPartBatchLeaves) {
    const int32_t n = n_leaves - l0 < kPartBatchLeaves ? n_leaves - l0 : kPartBatchLeaves;
    if (leaf_offsets[l0 + n] - leaf_offsets[l0] >= ((int64_t)1 << 32)) return GBDT_EUNSUPPORTED;
    int64_t chunks = 0;
    for (int32_t i = 0; i < n; ++i)
      chunks += (leaf_offsets[l0 + i + 1] - leaf_offsets[l0 + i] + chunk_rows - 1) / chunk_rows;
    if (chunks > max_chunks) max_chunks = chunks;
  }
  if (max_chunks >= ((int64_t)1 << 31)) return GBDT_EUNSUPPORTED;
  const size_t flag_words = (size_t)max_chunks * rpt * kPartWaves;
  void* ws = nullptr;
  int rc = get_workspace(flag_words * 8 + (size_t)max_chunks * 4 + 256, s, &ws);
  if (rc != GBDT_OK) return rc;
  const TilePlan p = make_tile_plan(n_features, n_bins);
  for (int32_t l0 = 0; l0 < n_leaves; l0 += kPartBatchLeaves) {
    const int32_t n = n_leaves - l0 < kPartBatchLeaves ? n_leaves - l0 : kPartBatchLeaves;
    PartBatchArgs a;
    a.packed = (const uint8_t*)bin_matrix;
    a.idx = row_idx + leaf_offsets[l0];
    a.split = splits + l0;
    a.out = children_out + leaf_offsets[l0];
    a.n_left_out = n_left_out ? n_left_out + l0 : nullptr;
    a.flags = (uint64_t*)ws;
    a.chunk_left = (uint32_t*)(a.flags + flag_words);
    a.n_rows = n_rows;
    a.plan = p;
    a.n_features = n_features;
    a.rows_per_thread = rpt;
    a.n_leaves = n;
    uint32_t chunks = 0;
    for (int32_t i = 0; i < kPartBatchLeaves; ++i) {
      PartLeaf& lf = a.leaf[i];
      if (i < n) {
        lf.row_off = lf.out_off = (uint32_t)(leaf_offsets[l0 + i] - leaf_offsets[l0]);
        lf.n = (uint32_t)(leaf_offsets[l0 + i + 1] - leaf_offsets[l0 + i]);
        lf.split_idx = (uint32_t)i;
        lf.first_chunk = chunks;
        chunks += (uint32_t)(((int64_t)lf.n + chunk_rows - 1) / chunk_rows);
      } else {
        lf.row_off = lf.out_off = lf.n = lf.split_idx = 0;
        lf.first_chunk = chunks;
      }
    }
    a.n_chunks = chunks;
    if (n_left_out) {
      hipLaunchKernelGGL(partition_empty_counts_kernel, dim3((n + 255) / 256), dim3(256), 0, s, a);
      HIP_TRY(hipGetLastError());
    }
    if (chunks == 0) continue;
    hipLaunchKernelGGL(partition_flag_batch_kernel, dim3(chunks), dim3(kPartThreads), 0, s, a);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(partition_scatter_batch_kernel, dim3(chunks), dim3(kPartThreads), 0, s, a);
    HIP_TRY(hipGetLastError());
  }
  return GBDT_OK;
}

// --- leaf-wise tree growth -------------------------------------------------------------

size_t gbdt_grow_tree_scratch_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins,
                                    int32_t max_leaves) {
  if (!valid_shape(n_rows, n_features, n_bins) || max_leaves < 1) return 0;
  return tree_scratch_layout(n_rows, n_features, n_bins, max_leaves).total;
}

int gbdt_grow_tree(const void* bin_matrix, int64_t n_rows, int32_t n_features, int32_t n_bins,
                   const float* grad, const float* hess, int32_t max_leaves, float lambda,
                   float min_child_hess, float min_split_gain, void* scratch, size_t scratch_bytes,
                   gbdt_tree_node_t* nodes_out, int32_t* n_nodes_out, int32_t* row_order_out,
                   void* stream) {
  if (!valid_shape(n_rows, n_features, n_bins)) return GBDT_EINVAL;
  if (max_leaves < 1 || !nodes_out || !n_nodes_out || !scratch) return GBDT_EINVAL;
  if (!(lambda >= 0.0f) || min_split_gain != min_split_gain) return GBDT_EINVAL;
  if (n_rows > 0 && (!bin_matrix || !grad || !hess)) return GBDT_EINVAL;
  if (((uintptr_t)scratch & 255u) != 0) return GBDT_EINVAL;
  if (n_rows >= ((int64_t)1 << 30)) return GBDT_EUNSUPPORTED;
  const TreeScratch lay = tree_scratch_layout(n_rows, n_features, n_bins, max_leaves);
  if (scratch_bytes < lay.total) return GBDT_ENOMEM;
  gbdt_split_t* pinned_dev = nullptr;
  gbdt_split_t* pinned = pinned_records(&pinned_dev);
  if (!pinned) return GBDT_ENOMEM;
  hipStream_t s = (hipStream_t)stream;
  char* base = (char*)scratch;
  int32_t* rows_base = (int32_t*)(base + lay.rows_a);   // row buffer b starts b * row_elems entries in
  int32_t* small_rows = (int32_t*)(base + lay.rows_small);
  gbdt_bin_t* pool = (gbdt_bin_t*)(base + lay.hists);
  gbdt_split_t* recs = (gbdt_split_t*)(base + lay.recs);            // record of the histogram in slot i
  const size_t hist_elems = (size_t)n_features * n_bins;
  const TilePlan plan = make_tile_plan(n_features, n_bins);

  // Best-first growth is sequential by definition: the open leaf with the largest gain is split,
  // its children join the open leaves, and so on (the older leaf on equal gains).  To wait for
  // the device once per ROUND instead of once per split, a round expands (partitions, builds,
  // searches) the best few open leaves at once; the host then replays the sequential rule on
  // what it knows and stops at the first leaf whose children it has not seen yet.  Every node
  // the replay splits is one the sequential rule splits, in the same order, so the tree is the
  // sequential one; an expansion the replay never reaches before the leaf budget is used up is
  // dropped (its leaf keeps its rows: children are written to the other row buffer).
  struct Cand {            // a node whose histogram exists on the device
    int64_t begin;         // its rows: positions [begin, begin + count) of row buffer `buf`
    uint32_t count;
    int buf;
    int slot;              // histogram slot in the pool
    gbdt_split_t rec;      // its best split
    float sum_grad, sum_hess;
    int kid[2];            // children once expanded (-1: not yet)
    int id;                // node id once it belongs to the tree
  };
  std::vector<Cand> cands;
  cands.reserve(1 + 2 * (size_t)grow_max_expansions(max_leaves));
  auto fill_node = [&](int k, int parent, const Cand& c) {
    gbdt_tree_node_t& nd = nodes_out[k];
    nd.parent = parent;
    nd.left = nd.right = -1;
    nd.feature = c.rec.feature;
    nd.bin = c.rec.bin;
    nd.gain = c.rec.gain;
    nd.sum_grad = c.sum_grad;
    nd.sum_hess = c.sum_hess;
    nd.count = c.count;
    nd.reserved = 0;
    nd.row_begin = c.begin;
  };

  // root: histogram without an index list, its row list 0..n-1 for the first partition
  int rc = gbdt_hist_build(bin_matrix, n_rows, n_features, n_bins, nullptr, n_rows, grad, hess, pool, s);
  if (rc != GBDT_OK) return rc;
  rc = launch_split(pool, 0, 1, lambda, min_child_hess, recs, n_features, n_bins, s, pinned_dev);
  if (rc != GBDT_OK) return rc;
  if (n_rows > 0 && max_leaves > 1) {
    hipLaunchKernelGGL(row_iota_kernel, dim3((unsigned)((n_rows + 255) / 256)), dim3(256), 0, s, rows_base, n_rows);
    HIP_TRY(hipGetLastError());
  }
  HIP_TRY(hipStreamSynchronize(s));
  {
    Cand root;
    root.begin = 0;
    root.count = (uint32_t)n_rows;
    root.buf = 0;
    root.slot = 0;
    root.rec = pinned[0];
    root.kid[0] = root.kid[1] = -1;
    root.id = 0;
    root.sum_grad = root.rec.left_grad + root.rec.right_grad;
    root.sum_hess = root.rec.left_hess + root.rec.right_hess;
    if (root.rec.feature < 0 && n_rows > 0) {
      // no split record carries the totals: sum feature 0's bins on the host
      std::vector<gbdt_bin_t> row((size_t)n_bins);
      HIP_TRY(hipMemcpyAsync(row.data(), pool, (size_t)n_bins * sizeof(gbdt_bin_t), hipMemcpyDeviceToHost, s));
      HIP_TRY(hipStreamSynchronize(s));
      double g = 0.0, h = 0.0;
      for (const gbdt_bin_t& b : row) {
        g += b.grad;
        h += b.hess;
      }
      root.sum_grad = (float)g;
      root.sum_hess = (float)h;
    }
    cands.push_back(root);
    fill_node(0, -1, root);
  }
  auto eligible = [&](const Cand& c) { return c.rec.feature >= 0 && c.rec.gain > min_split_gain; };
  std::vector<int> open = {0};  // candidates that are leaves of the tree so far
  int n_nodes = 1, n_leaves = 1, next_slot = 1;
  int expansions = 0, splits = 0, rounds = 0;
  const int spec_budget = grow_speculative_budget(max_leaves);
  // (host clock, for the trace line: all rounds, and the part of them spent waiting for the stream)
  double wait_us = 0, rounds_us = 0;
  auto last_round_end = std::chrono::steady_clock::now();
  for (;;) {
    // ---- replay the sequential rule as far as the expansions seen so far carry it
    int blocked = -1;
    while (n_leaves < max_leaves) {
      int m = -1;
      for (int h : open) {  // larger gain, then smaller node id
        const Cand& c = cands[h];
        if (!eligible(c)) continue;
        if (m < 0 || c.rec.gain > cands[m].rec.gain || (c.rec.gain == cands[m].rec.gain && c.id < cands[m].id)) m = h;
      }
      if (m < 0) break;
      if (cands[m].kid[0] < 0) {
        blocked = m;
        break;
      }
      const int left = n_nodes, right = n_nodes + 1;
      nodes_out[cands[m].id].left = left;
      nodes_out[cands[m].id].right = right;
      for (int side = 0; side < 2; ++side) {
        Cand& k = cands[cands[m].kid[side]];
        k.id = side == 0 ? left : right;
        fill_node(k.id, cands[m].id, k);
        open.push_back(cands[m].kid[side]);
      }
      open.erase(std::find(open.begin(), open.end(), m));
      n_nodes += 2;
      n_leaves += 1;
      splits += 1;
    }
    if (blocked < 0) break;  // leaf budget used up, or nothing left to split
    // ---- this round: the blocking leaf and the next best open leaves without children
    // (A width that follows the number of splits the last round made possible was tried: fewer
    // leaves expanded in vain on deep, chain-like trees, but more rounds, and rounds cost more.)
    int extra = kGrowRound - 1;
    if (extra > max_leaves - n_leaves - 1) extra = max_leaves - n_leaves - 1;
    if (extra > spec_budget - (expansions - splits)) extra = spec_budget - (expansions - splits);
    if (extra < 0) extra = 0;
    std::vector<int> batch = {blocked};
    if (extra > 0) {
      std::vector<int> more;
      for (int h : open)
        if (h != blocked && cands[h].kid[0] < 0 && eligible(cands[h])) more.push_back(h);
      std::sort(more.begin(), more.end(), [&](int x, int y) {
        return cands[x].rec.gain > cands[y].rec.gain || (cands[x].rec.gain == cands[y].rec.gain && cands[x].id < cands[y].id);
      });
      if ((int)more.size() > extra) more.resize(extra);
      batch.insert(batch.end(), more.begin(), more.end());
    }
    const int k = (int)batch.size();
    if (next_slot + 2 * k > lay.n_slots) return GBDT_ENOMEM;  // (cannot happen: the budget above bounds it)

    // ---- partition the k leaves: children into the other row buffer, same positions; every leaf's
    // split record is read on the device, from the records by histogram slot
    {
      uint32_t longest = 1;
      for (int j = 0; j < k; ++j) longest = cands[batch[j]].count > longest ? cands[batch[j]].count : longest;
      const int32_t rpt = make_part_geom(longest).rows_per_thread;
      const int64_t chunk_rows = (int64_t)kPartThreads * rpt;
      PartBatchArgs a;
      a.packed = (const uint8_t*)bin_matrix;
      a.idx = rows_base;
      a.split = recs;
      a.out = rows_base;
      a.n_left_out = nullptr;
      a.n_rows = n_rows;
      a.plan = plan;
      a.n_features = n_features;
      a.rows_per_thread = rpt;
      a.n_leaves = k;
      uint32_t chunks = 0;
      for (int j = 0; j < kPartBatchLeaves; ++j) {
        PartLeaf& lf = a.leaf[j];
        lf.row_off = lf.out_off = lf.n = lf.split_idx = 0;
        lf.first_chunk = chunks;
        if (j < k) {
          const Cand& c = cands[batch[j]];
          lf.row_off = (uint32_t)(c.begin + (int64_t)c.buf * (int64_t)lay.row_elems);
          lf.out_off = (uint32_t)(c.begin + (int64_t)(1 - c.buf) * (int64_t)lay.row_elems);
          lf.n = c.count;
          lf.split_idx = (uint32_t)c.slot;
          chunks += (uint32_t)(((int64_t)lf.n + chunk_rows - 1) / chunk_rows);
        }
      }
      a.n_chunks = chunks;
      const size_t flag_words = (size_t)chunks * rpt * kPartWaves;
      void* ws = nullptr;
      rc = get_workspace(flag_words * 8 + (size_t)chunks * 4 + 256, s, &ws);
      if (rc != GBDT_OK) return rc;
      a.flags = (uint64_t*)ws;
      a.chunk_left = (uint32_t*)(a.flags + flag_words);
      if (chunks > 0) {
        hipLaunchKernelGGL(partition_flag_batch_kernel, dim3(chunks), dim3(kPartThreads), 0, s, a);
        HIP_TRY(hipGetLastError());
        hipLaunchKernelGGL(partition_scatter_batch_kernel, dim3(chunks), dim3(kPartThreads), 0, s, a);
        HIP_TRY(hipGetLastError());
      }
    }
    // ---- the smaller children's histograms in one batched build, straight from their segments of
    // the row buffers -- or, where gathering grad / hess into list order pays (sparse leaves of a
    // matrix of many tiles), from a copy of their rows back to back
    std::vector<int64_t> small_offs = {0};
    std::vector<uint32_t> small_seg((size_t)k);
    std::vector<int> left_small((size_t)k);
    for (int j = 0; j < k; ++j) {
      const Cand& c = cands[batch[j]];
      const uint32_t nl = c.rec.left_count, nr = c.rec.right_count;
      left_small[j] = nl <= nr;
      const int64_t kid_base = c.begin + (int64_t)(1 - c.buf) * (int64_t)lay.row_elems;
      small_seg[j] = (uint32_t)(left_small[j] ? kid_base : kid_base + nl);
      small_offs.push_back(small_offs.back() + (left_small[j] ? nl : nr));
    }
    gbdt_bin_t* h_small = pool + (size_t)next_slot * hist_elems;  // k slots: the built children; then k: their siblings
    const int64_t small_total = small_offs.back();
    if (small_total > 0 && stats_gather_pays(plan_n_tiles(plan), small_total, small_total / k, n_rows)) {
      CompactTable t;
      for (int j = 0; j < k; ++j) {
        t.src_begin[j] = small_seg[j];
        t.dst_begin[j] = (uint32_t)small_offs[j];
      }
      t.dst_begin[k] = (uint32_t)small_total;
      t.n_seg = k;
      hipLaunchKernelGGL(segments_compact_kernel, dim3((unsigned)((small_total + 255) / 256)), dim3(256), 0, s,
                         (const int32_t*)rows_base, t, small_rows);
      HIP_TRY(hipGetLastError());
      rc = hist_build_batch_impl(bin_matrix, n_rows, n_features, n_bins, small_rows, small_offs.data(), k, grad,
                                 hess, h_small, s, nullptr);
    } else {
      rc = hist_build_batch_impl(bin_matrix, n_rows, n_features, n_bins, rows_base, small_offs.data(), k, grad,
                                 hess, h_small, s, small_seg.data());
    }
    if (rc != GBDT_OK) return rc;
    // ---- best splits of the 2k children, one launch, which first forms the k siblings as parent -
    // built child; the records also land in `pinned`
    {
      SplitSiblings sib;
      sib.pool = pool;
      sib.first = k;
      sib.n = k;
      for (int j = 0; j < kSplitSiblings; ++j) sib.parent_slot[j] = j < k ? cands[batch[j]].slot : 0;
      rc = launch_split(h_small, (int64_t)hist_elems, 2 * k, lambda, min_child_hess, recs + next_slot, n_features,
                        n_bins, s, pinned_dev, &sib);
      if (rc != GBDT_OK) return rc;
    }
    {
      auto t0 = std::chrono::steady_clock::now();
      HIP_TRY(hipStreamSynchronize(s));
      auto t1 = std::chrono::steady_clock::now();
      wait_us += std::chrono::duration<double, std::micro>(t1 - t0).count();
      rounds_us += std::chrono::duration<double, std::micro>(t1 - last_round_end).count();
      last_round_end = t1;
    }
    for (int j = 0; j < k; ++j) {
      const int par = batch[j];
      const Cand pc = cands[par];
      const uint32_t nl = pc.rec.left_count, nr = pc.rec.right_count;
      for (int side = 0; side < 2; ++side) {
        const bool is_small = (side == 0) == (left_small[j] != 0);
        Cand c;
        c.begin = side == 0 ? pc.begin : pc.begin + nl;
        c.count = side == 0 ? nl : nr;
        c.buf = 1 - pc.buf;
        c.slot = is_small ? next_slot + j : next_slot + k + j;
        c.rec = pinned[is_small ? j : k + j];
        c.sum_grad = side == 0 ? pc.rec.left_grad : pc.rec.right_grad;
        c.sum_hess = side == 0 ? pc.rec.left_hess : pc.rec.right_hess;
        c.kid[0] = c.kid[1] = -1;
        c.id = -1;
        cands[par].kid[side] = (int)cands.size();
        cands.push_back(c);
      }
    }
    next_slot += 2 * k;
    expansions += k;
    rounds += 1;
  }
  *n_nodes_out = n_nodes;
  {
    static const bool trace = [] {
      const char* e = getenv("GBDT_HIST_TRACE_TREE");  // tuning aid: one line per tree on stderr
      return e && atoi(e) > 0;
    }();
    if (trace)
      fprintf(stderr, "gbdt_grow_tree: %d leaves, %d rounds, %d leaves expanded, %d of them never split; rounds %.0f us, "
              "of which %.0f us waiting for the stream\n", n_leaves,
              rounds, expansions, expansions - splits, rounds_us, wait_us);
  }
  if (row_order_out && n_rows > 0) {
    if (n_nodes == 1) {  // never split: the rows in their own order
      hipLaunchKernelGGL(row_iota_kernel, dim3((unsigned)((n_rows + 255) / 256)), dim3(256), 0, s,
                         row_order_out, n_rows);
      HIP_TRY(hipGetLastError());
    } else {
      // the leaves' segments in position order, a table-full per launch
      std::vector<std::pair<uint32_t, int>> segs;  // (begin, buffer)
      for (int h : open) segs.emplace_back((uint32_t)cands[h].begin, cands[h].buf);
      std::sort(segs.begin(), segs.end());
      for (size_t s0 = 0; s0 < segs.size(); s0 += kSegTable) {
        SegTable t;
        const size_t ns = segs.size() - s0 < (size_t)kSegTable ? segs.size() - s0 : (size_t)kSegTable;
        for (size_t j = 0; j < ns; ++j)
          t.start[j] = segs[s0 + j].first | ((uint32_t)segs[s0 + j].second << 31);
        t.n_seg = (int32_t)ns;
        t.end = s0 + ns < segs.size() ? segs[s0 + ns].first : (uint32_t)n_rows;
        const uint32_t span = t.end - segs[s0].first;
        hipLaunchKernelGGL(leaf_rows_gather_kernel, dim3((span + 255) / 256), dim3(256), 0, s,
                           (const int32_t*)rows_base, (const int32_t*)(rows_base + lay.row_elems), t, row_order_out);
        HIP_TRY(hipGetLastError());
      }
    }
  }
  return GBDT_OK;
}

// --- level-wise tree growth ------------------------------------------------------------

size_t gbdt_grow_tree_depthwise_scratch_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins,
                                              int32_t max_depth) {
  if (!valid_shape(n_rows, n_features, n_bins) || max_depth < 0 || max_depth > kMaxTreeDepth) return 0;
  return level_scratch_layout(n_rows, n_features, n_bins, max_depth).total;
}

int gbdt_grow_tree_depthwise(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                             int32_t n_bins, const float* grad, const float* hess, int32_t max_depth,
                             float lambda, float min_child_hess, float min_split_gain, void* scratch,
                             size_t scratch_bytes, gbdt_tree_node_t* nodes_out, int32_t* n_nodes_out,
                             int32_t* row_order_out, void* stream) {
  if (!valid_shape(n_rows, n_features, n_bins)) return GBDT_EINVAL;
  if (max_depth < 0 || max_depth > kMaxTreeDepth || !nodes_out || !n_nodes_out || !scratch) return GBDT_EINVAL;
  if (!(lambda >= 0.0f) || min_split_gain != min_split_gain) return GBDT_EINVAL;
  if (n_rows > 0 && (!bin_matrix || !grad || !hess)) return GBDT_EINVAL;
  if (((uintptr_t)scratch & 255u) != 0) return GBDT_EINVAL;
  if (n_rows >= ((int64_t)1 << 30)) return GBDT_EUNSUPPORTED;
  const LevelScratch lay = level_scratch_layout(n_rows, n_features, n_bins, max_depth);
  if (scratch_bytes < lay.total) return GBDT_ENOMEM;
  const size_t width = (size_t)1 << max_depth;  // most nodes a level can hold
  gbdt_split_t* pinned = pinned_level_records(2 * width);
  if (!pinned) return GBDT_ENOMEM;
  gbdt_split_t* pinned_part = pinned + width;  // records the partition of a level is driven by
  hipStream_t s = (hipStream_t)stream;
  char* base = (char*)scratch;
  int32_t* rows_buf[2] = {(int32_t*)(base + lay.rows_a), (int32_t*)(base + lay.rows_b)};
  int32_t* small_rows = (int32_t*)(base + lay.rows_small);
  gbdt_bin_t* hist_buf[2] = {(gbdt_bin_t*)(base + lay.hists_a), (gbdt_bin_t*)(base + lay.hists_b)};
  gbdt_split_t* recs = (gbdt_split_t*)(base + lay.recs);
  gbdt_split_t* part_recs = (gbdt_split_t*)(base + lay.part_recs);
  const size_t hist_elems = (size_t)n_features * n_bins;

  auto fill_node = [&](int k, int parent, const gbdt_split_t& r, float sg, float sh, uint32_t cnt,
                       int64_t begin) {
    gbdt_tree_node_t& nd = nodes_out[k];
    nd.parent = parent;
    nd.left = nd.right = -1;
    nd.feature = r.feature;
    nd.bin = r.bin;
    nd.gain = r.gain;
    nd.sum_grad = sg;
    nd.sum_hess = sh;
    nd.count = cnt;
    nd.reserved = 0;
    nd.row_begin = begin;
  };

  // root: its histogram without an index list; the row list 0..n-1 for the first partition
  int cur = 0;  // row buffer and histogram buffer of the current level
  int rc = gbdt_hist_build(bin_matrix, n_rows, n_features, n_bins, nullptr, n_rows, grad, hess, hist_buf[cur], s);
  if (rc != GBDT_OK) return rc;
  if (n_rows > 0) {
    hipLaunchKernelGGL(row_iota_kernel, dim3((unsigned)((n_rows + 255) / 256)), dim3(256), 0, s, rows_buf[cur],
                       n_rows);
    HIP_TRY(hipGetLastError());
  }
  // the level: its nodes in position order with their histogram slots; `frontier` also holds
  // the finished leaves, whose rows every later partition copies through unchanged
  struct Entry {
    int node;   // node id
    int slot;   // histogram slot in hist_buf[cur]; -1: a finished leaf
  };
  std::vector<Entry> frontier = {{0, 0}};
  int n_nodes = 1;
  bool root_done = false;
  for (int depth = 0;; ++depth) {
    // ---- best split of every open node of the level, one launch, one read-back
    std::vector<int> open;  // indices into frontier, in histogram slot order
    for (size_t i = 0; i < frontier.size(); ++i)
      if (frontier[i].slot >= 0) open.push_back((int)i);
    std::sort(open.begin(), open.end(), [&](int a, int b) { return frontier[a].slot < frontier[b].slot; });
    const int n_open = (int)open.size();
    if (n_open == 0) break;
    rc = gbdt_best_split_batch(hist_buf[cur], n_open, lambda, min_child_hess, recs, n_features, n_bins, s);
    if (rc != GBDT_OK) return rc;
    HIP_TRY(hipMemcpyAsync(pinned, recs, (size_t)n_open * sizeof(gbdt_split_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (!root_done) {
      const gbdt_split_t r = pinned[0];
      float sg = r.left_grad + r.right_grad, sh = r.left_hess + r.right_hess;
      if (r.feature < 0 && n_rows > 0) {  // no record carries the totals: sum feature 0's bins here
        std::vector<gbdt_bin_t> row((size_t)n_bins);
        HIP_TRY(hipMemcpyAsync(row.data(), hist_buf[cur], (size_t)n_bins * sizeof(gbdt_bin_t),
                               hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        double g = 0.0, h = 0.0;
        for (const gbdt_bin_t& b : row) {
          g += b.grad;
          h += b.hess;
        }
        sg = (float)g;
        sh = (float)h;
      }
      fill_node(0, -1, r, sg, sh, (uint32_t)n_rows, 0);
      root_done = true;
    }
    // the records of the level's nodes (slot order = order of `open`)
    std::vector<gbdt_split_t> rec_of(frontier.size());
    for (int j = 0; j < n_open; ++j) {
      const gbdt_split_t& r = pinned[frontier[open[j]].slot];
      rec_of[open[j]] = r;
      gbdt_tree_node_t& nd = nodes_out[frontier[open[j]].node];
      nd.feature = r.feature;
      nd.bin = r.bin;
      nd.gain = r.gain;
    }
    if (depth == max_depth) break;
    // ---- which nodes split; the partition records of ALL entries (others: no split)
    std::vector<Entry> next;
    std::vector<int64_t> offs;          // positions of the entries of this level
    std::vector<int> splitting;         // indices into frontier
    for (size_t i = 0; i < frontier.size(); ++i) {
      const gbdt_tree_node_t& nd = nodes_out[frontier[i].node];
      offs.push_back(nd.row_begin);
      gbdt_split_t pr;
      memset(&pr, 0, sizeof pr);
      pr.feature = pr.bin = -1;
      if (frontier[i].slot >= 0 && rec_of[i].feature >= 0 && rec_of[i].gain > min_split_gain) {
        pr = rec_of[i];
        splitting.push_back((int)i);
      }
      pinned_part[i] = pr;
    }
    offs.push_back(n_rows);
    if (splitting.empty()) break;
    HIP_TRY(hipMemcpyAsync(part_recs, pinned_part, frontier.size() * sizeof(gbdt_split_t),
                           hipMemcpyHostToDevice, s));
    const int nxt = cur ^ 1;
    rc = gbdt_partition_rows_batch(bin_matrix, n_rows, n_features, n_bins, rows_buf[cur], offs.data(),
                                   (int32_t)frontier.size(), part_recs, rows_buf[nxt], nullptr, s);
    if (rc != GBDT_OK) return rc;
    // ---- children: node ids in the order of their parents' ids (the level's numbering),
    // histogram slots: the smaller children first (built), then the larger (by subtraction)
    std::vector<int> by_node = splitting;
    std::sort(by_node.begin(), by_node.end(), [&](int a, int b) { return frontier[a].node < frontier[b].node; });
    const int k = (int)by_node.size();
    std::vector<int64_t> small_offs = {0};
    std::vector<int> parent_slot((size_t)k);
    std::vector<std::pair<uint32_t, uint32_t>> small_seg((size_t)k);  // (begin in the row buffer, length)
    std::vector<std::pair<Entry, Entry>> kids(frontier.size());
    for (int j = 0; j < k; ++j) {
      const int i = by_node[j];
      const int parent = frontier[i].node;
      const gbdt_split_t& r = rec_of[i];
      const int64_t begin = nodes_out[parent].row_begin;
      const int left = n_nodes, right = n_nodes + 1;
      n_nodes += 2;
      nodes_out[parent].left = left;
      nodes_out[parent].right = right;
      gbdt_split_t none;
      memset(&none, 0, sizeof none);
      none.feature = none.bin = -1;
      fill_node(left, parent, none, r.left_grad, r.left_hess, r.left_count, begin);
      fill_node(right, parent, none, r.right_grad, r.right_hess, r.right_count, begin + r.left_count);
      const bool left_small = r.left_count <= r.right_count;
      small_seg[j] = left_small ? std::make_pair((uint32_t)begin, r.left_count)
                                : std::make_pair((uint32_t)(begin + r.left_count), r.right_count);
      small_offs.push_back(small_offs.back() + small_seg[j].second);
      parent_slot[j] = frontier[i].slot;
      kids[i] = left_small ? std::make_pair(Entry{left, j}, Entry{right, k + j})
                           : std::make_pair(Entry{left, k + j}, Entry{right, j});
    }
    for (size_t i = 0; i < frontier.size(); ++i) {
      if (nodes_out[frontier[i].node].left >= 0) {
        next.push_back(kids[i].first);
        next.push_back(kids[i].second);
      } else {
        next.push_back(Entry{frontier[i].node, -1});  // a leaf from now on
      }
    }
    // ---- the smaller children's rows back to back, their histograms in one batched build
    for (int j0 = 0; j0 < k; j0 += kCompactSegs) {
      CompactTable t;
      const int ns = k - j0 < kCompactSegs ? k - j0 : kCompactSegs;
      for (int j = 0; j < ns; ++j) {
        t.src_begin[j] = small_seg[j0 + j].first;
        t.dst_begin[j] = (uint32_t)small_offs[j0 + j];
      }
      t.dst_begin[ns] = (uint32_t)small_offs[j0 + ns];
      t.n_seg = ns;
      const uint32_t span = t.dst_begin[ns] - t.dst_begin[0];
      if (span == 0) continue;
      hipLaunchKernelGGL(segments_compact_kernel, dim3((span + 255) / 256), dim3(256), 0, s,
                         (const int32_t*)rows_buf[nxt], t, small_rows);
      HIP_TRY(hipGetLastError());
    }
    rc = gbdt_hist_build_batch(bin_matrix, n_rows, n_features, n_bins, small_rows, small_offs.data(), k, grad,
                               hess, hist_buf[nxt], s);
    if (rc != GBDT_OK) return rc;
    for (int j0 = 0; j0 < k; j0 += kSiblingTable) {
      SiblingTable t;
      const int ns = k - j0 < kSiblingTable ? k - j0 : kSiblingTable;
      for (int j = 0; j < ns; ++j) t.parent_slot[j] = parent_slot[j0 + j];
      hipLaunchKernelGGL(hist_siblings_kernel, dim3((unsigned)((hist_elems + 255) / 256), ns), dim3(256), 0, s,
                         (const gbdt_bin_t*)hist_buf[cur], (const gbdt_bin_t*)(hist_buf[nxt] + (size_t)j0 * hist_elems),
                         hist_buf[nxt] + (size_t)(k + j0) * hist_elems, (int32_t)hist_elems, t);
      HIP_TRY(hipGetLastError());
    }
    frontier.swap(next);
    cur = nxt;
  }
  *n_nodes_out = n_nodes;
  if (row_order_out && n_rows > 0)
    HIP_TRY(hipMemcpyAsync(row_order_out, rows_buf[cur], (size_t)n_rows * sizeof(int32_t),
                           hipMemcpyDeviceToDevice, s));
  return GBDT_OK;
}

int gbdt_debug_geometry(int32_t n_features, int32_t n_bins, int64_t n_leaf_rows, int32_t n_cus,
                        int64_t* out, int32_t n_out) {
  if (!out || n_out < 16 || n_features <= 0 || n_bins < 2 || n_bins > 256 || n_leaf_rows < 0)
    return GBDT_EINVAL;
  const BuildGeom g = make_geom(n_features, n_bins, n_leaf_rows, n_cus > 0 ? n_cus : 256, 0);
  const TilePlan& p = g.plan;
  const int64_t v[16] = {p.cap,         p.nib,          p.wm,          p.n_main,
                         p.wr,          p.row_bytes,    p.feat_bytes,  g.nt,
                         (int64_t)g.lds_bytes, g.wgs, g.unit_epochs, (int64_t)g.partial_words,
                         0,             0, 0, 0};
  for (int i = 0; i < 16; ++i) out[i] = v[i];
  return GBDT_OK;
}

int gbdt_debug_batch_plan(int32_t n_features, int32_t n_bins, const int64_t* leaf_offsets,
                          int32_t n_leaves, int32_t n_cus, int32_t wg_per_cu, int32_t* leaf_wgs_out,
                          int32_t* leaf_unit_epochs_out, int32_t* block_out, int32_t max_blocks) {
  if (n_features <= 0 || n_bins < 2 || n_bins > 256 || !leaf_offsets || n_leaves < 1 ||
      n_leaves > kBatchLeaves || n_cus <= 0 || wg_per_cu <= 0 || !leaf_wgs_out ||
      !leaf_unit_epochs_out || (!block_out && max_blocks > 0))
    return GBDT_EINVAL;
  for (int32_t l = 0; l < n_leaves; ++l)
    if (leaf_offsets[l + 1] < leaf_offsets[l]) return GBDT_EINVAL;
  const TilePlan p = make_tile_plan(n_features, n_bins);
  const int n_tiles = plan_n_tiles(p);
  const BatchPlan b = plan_batch(leaf_offsets, 0, n_leaves, (int64_t)n_cus * wg_per_cu, n_tiles);
  for (int32_t l = 0; l < n_leaves; ++l) {
    leaf_wgs_out[l] = (int32_t)(b.leaf[l].wgs_unit & 0xffffu);
    leaf_unit_epochs_out[l] = (int32_t)(b.leaf[l].wgs_unit >> 16);
  }
  const int64_t blocks = (int64_t)b.total_wgs * n_tiles;
  for (int64_t i = 0; i < blocks && i < max_blocks; ++i) {
    const BatchBlock k = batch_block(b.leaf, n_leaves, p.n_main, p.wr, (uint32_t)i);
    block_out[3 * i] = k.leaf;
    block_out[3 * i + 1] = k.tile;
    block_out[3 * i + 2] = k.wg;
  }
  return (int)blocks;
}

int gbdt_debug_fusion_plan(const uint32_t* levels, int32_t n_features, int32_t* col_out, int32_t* stride_out,
                           int32_t* n_cols_out) {
  if (!levels || n_features <= 0 || !col_out || !stride_out || !n_cols_out) return GBDT_EINVAL;
  std::vector<uint32_t> lv(levels, levels + n_features);
  for (uint32_t l : lv)
    if (l < 1 || l > (uint32_t)kFusedCap) return GBDT_EINVAL;
  std::vector<FusedCol> cols;
  std::vector<FusedFeat> feats;
  plan_fusion(lv, &cols, &feats);
  for (int32_t f = 0; f < n_features; ++f) {
    col_out[f] = feats[f].col;
    stride_out[f] = feats[f].stride;
  }
  *n_cols_out = (int32_t)cols.size();
  return GBDT_OK;
}

int gbdt_debug_occupancy(int32_t n_bins, int32_t indexed) {
  if (n_bins < 2 || n_bins > 256) return GBDT_EINVAL;
  return build_wg_per_cu(n_bins <= 16 ? 16 : (n_bins <= 64 ? 64 : 256), indexed != 0);
}

int gbdt_debug_split_plan(int32_t n_features, int32_t n_bins, int32_t n_hists, int64_t* out, int32_t n_out) {
  if (!out || n_out < 4 || n_features <= 0 || n_bins < 2 || n_bins > 256 || n_hists < 1) return GBDT_EINVAL;
  const SplitGrouping g = split_grouping(n_features, n_bins, n_hists);
  out[0] = g.group;
  out[1] = g.passes;
  out[2] = g.n_wg;
  out[3] = (int64_t)g.group * split_feature_bytes(n_bins);
  return GBDT_OK;
}

int gbdt_debug_partition_plan(int64_t n_leaf_rows, int64_t* out, int32_t n_out) {
  if (!out || n_out < 3 || n_leaf_rows < 1 || n_leaf_rows >= ((int64_t)1 << 32)) return GBDT_EINVAL;
  const PartGeom g = make_part_geom(n_leaf_rows);
  out[0] = g.rows_per_thread;
  out[1] = g.n_chunks;
  out[2] = (int64_t)g.bytes;
  return GBDT_OK;
}

int gbdt_debug_locate(int32_t n_features, int32_t n_bins, int32_t feature, int32_t* tile_out,
                      int32_t* slot_out) {
  if (!tile_out || !slot_out || n_features <= 0 || n_bins < 2 || n_bins > 256 || feature < 0 ||
      feature >= n_features)
    return GBDT_EINVAL;
  const TilePlan p = make_tile_plan(n_features, n_bins);
  const FeatureSlot fs = plan_locate(p, feature);
  *tile_out = fs.tile;
  *slot_out = fs.slot;
  return GBDT_OK;
}

int gbdt_set_deterministic(int enable) {
  g_deterministic.store(enable != 0);
  return GBDT_OK;
}

int gbdt_set_wide_accumulation(int enable) {
  g_wide.store(enable != 0);
  return GBDT_OK;
}

int gbdt_calibration_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || bytes == 0 || (bytes & 15u) != 0) return GBDT_EINVAL;
  if ((((uintptr_t)src) | ((uintptr_t)dst)) & 15u) return GBDT_EINVAL;
  hipLaunchKernelGGL(calibration_copy_kernel, dim3(device_cu_count() * 8), dim3(256), 0,
                     (hipStream_t)stream, (const uint4*)src, (uint4*)dst, bytes / 16);
  HIP_TRY(hipGetLastError());
  return GBDT_OK;
}

int gbdt_profile_enable(int enable) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  g_prof.on = enable != 0;
  return GBDT_OK;
}

int gbdt_profile_collect(double* build_kernel_ms_total, int64_t* n_launches) {
  if (!build_kernel_ms_total || !n_launches) return GBDT_EINVAL;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pairs;
  {
    std::lock_guard<std::mutex> lk(g_prof.mu);
    pairs.swap(g_prof.pairs);
  }
  double total = 0.0;
  int rc = GBDT_OK;
  for (auto& pr : pairs) {
    float ms = 0.0f;
    hipError_t e = hipEventSynchronize(pr.second);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, pr.first, pr.second);
    if (e != hipSuccess && rc == GBDT_OK) rc = hip_fail(e, "hipEventElapsedTime");
    total += ms;
    (void)hipEventDestroy(pr.first);
    (void)hipEventDestroy(pr.second);
  }
  *build_kernel_ms_total = total;
  *n_launches = (int64_t)pairs.size();
  return rc;
}

int gbdt_profile_durations(double* ms_out, int64_t capacity, int64_t* n_launches) {
  if (!n_launches || capacity < 0 || (capacity > 0 && !ms_out)) return GBDT_EINVAL;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pairs;
  {
    std::lock_guard<std::mutex> lk(g_prof.mu);
    pairs.swap(g_prof.pairs);
  }
  int rc = GBDT_OK;
  int64_t i = 0;
  for (auto& pr : pairs) {
    float ms = 0.0f;
    hipError_t e = hipEventSynchronize(pr.second);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, pr.first, pr.second);
    if (e != hipSuccess && rc == GBDT_OK) rc = hip_fail(e, "hipEventElapsedTime");
    if (i < capacity) ms_out[i] = ms;
    ++i;
    (void)hipEventDestroy(pr.first);
    (void)hipEventDestroy(pr.second);
  }
  *n_launches = i;
  return rc;
}

int gbdt_reset(void) {
  // everything enqueued so far must be done before buffers go away and counters are cleared
  HIP_TRY(hipDeviceSynchronize());
  {
    std::lock_guard<std::mutex> lk(g_ws.mu);
    for (void* q : g_ws.retired) (void)hipFree(q);
    g_ws.retired.clear();
    if (g_ws.own) (void)hipFree(g_ws.own);
    g_ws.own = nullptr;
    g_ws.own_bytes = 0;
    g_ws.own_device = -1;
    g_ws.zeroed = nullptr;  // a caller's buffer stays registered; its counters are zeroed by the next build
  }
  {
    std::lock_guard<std::mutex> lk(g_prof.mu);
    for (auto& pr : g_prof.pairs) {
      (void)hipEventDestroy(pr.first);
      (void)hipEventDestroy(pr.second);
    }
    g_prof.pairs.clear();
  }
  (void)hipGetLastError();
  // the split search's tickets: a launch that failed half-way may have left some counted
  hipLaunchKernelGGL(split_tickets_zero_kernel, dim3(kSplitMaxHists / 256), dim3(256), 0, nullptr);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipDeviceSynchronize());
  g_hip_err[0] = 0;
  return GBDT_OK;
}

const char* gbdt_strerror(int code) {
  switch (code) {
    case GBDT_OK: return "ok";
    case GBDT_EINVAL: return "invalid argument";
    case GBDT_EUNSUPPORTED: return "unsupported problem size";
    case GBDT_EHIP: return "HIP runtime error";
    case GBDT_ENOMEM: return "workspace allocation failed or too small";
    default: return "unknown error code";
  }
}

const char* gbdt_last_hip_error(void) { return g_hip_err; }

}  // extern "C"
