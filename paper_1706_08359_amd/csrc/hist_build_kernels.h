// Re-layout of the bin matrix and the histogram build kernels (single leaf and batched):
// Alg. 1 / Sec. 4 / App. A.1 of arXiv 1706.08359 for gfx950.  Included by gbdt_hist.hip only.
#ifndef GBDT_HIST_BUILD_KERNELS_H_
#define GBDT_HIST_BUILD_KERNELS_H_

#include <hip/hip_runtime.h>

#include <stdint.h>
#include <string.h>

#include <type_traits>
#include <utility>

#include "../../include/gbdt_hist.h"
#include "tile_plan.h"
#include "batch_plan.h"

namespace {

// ------------------------------------------------------------------ pack kernel

// One thread writes one 4-byte word of the packed layout (see tile_plan.h).
// grid.y = tile, grid.x covers n_rows * (W / 4) words of that tile.
__global__ void __launch_bounds__(256)
pack_kernel(const uint8_t* __restrict__ src, int64_t n_rows, int32_t n_features, TilePlan plan,
            uint8_t* __restrict__ dst) {
  const int32_t t = blockIdx.y;
  const int32_t w = plan_tile_width(plan, t);
  const int32_t lpr = w >> 2;
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= n_rows * lpr) return;
  const int64_t r = q / lpr;
  const int32_t j = (int32_t)(q - r * lpr);
  const int64_t tile_off = n_rows * ((int64_t)t * plan.wm);  // t <= n_main, all earlier tiles are main
  const uint8_t* row = src + r * (int64_t)n_features;
  uint32_t word = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int32_t fb = t * plan.wm + 4 * j + i;  // byte of the (virtual, unpadded) packed row
    uint32_t v;
    if (plan.nib) {
      const int32_t f0 = 2 * fb, f1 = 2 * fb + 1;
      const uint32_t lo = f0 < n_features ? (row[f0] & 15u) : 0u;
      const uint32_t hi = f1 < n_features ? (row[f1] & 15u) : 0u;
      v = lo | (hi << 4);
    } else {
      v = fb < n_features ? (row[fb] & (uint32_t)(plan.cap - 1)) : 0u;
    }
    word |= v << (8 * i);
  }
  *reinterpret_cast<uint32_t*>(dst + tile_off + r * w + 4 * j) = word;
}

// The column-major copy behind the tiles: a 64 x 64 block of the row-major matrix is read a
// row at a time (a wavefront = 64 consecutive features of one row), turned in local memory,
// and written a column at a time, four rows per thread.  grid = (row blocks, feature blocks).
__global__ void __launch_bounds__(256)
pack_columns_kernel(const uint8_t* __restrict__ src, int64_t n_rows, int32_t n_features, uint32_t mask,
                    uint8_t* __restrict__ cols, int64_t stride) {
  __shared__ uint8_t t[64][64 + 4];  // [feature][row]
  const int tid = threadIdx.x;
  const int64_t r0 = (int64_t)blockIdx.x * 64;
  const int32_t f0 = (int32_t)blockIdx.y * 64;
#pragma unroll 4
  for (int i = 0; i < 16; ++i) {
    const int rl = (tid >> 6) + 4 * i, fl = tid & 63;
    const int64_t r = r0 + rl;
    const int32_t f = f0 + fl;
    uint32_t v = 0;
    if (r < n_rows && f < n_features) v = src[r * n_features + f] & mask;
    t[fl][rl] = (uint8_t)v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int fl = (tid >> 4) + 16 * i, rq = (tid & 15) * 4;
    const int32_t f = f0 + fl;
    if (f < n_features) {  // rows past n_rows fall into the column's padding (stride >= r0 + 64)
      const uint32_t w = (uint32_t)t[fl][rq] | ((uint32_t)t[fl][rq + 1] << 8) |
                         ((uint32_t)t[fl][rq + 2] << 16) | ((uint32_t)t[fl][rq + 3] << 24);
      *reinterpret_cast<uint32_t*>(cols + (int64_t)f * stride + r0 + rq) = w;
    }
  }
}

// ------------------------------------------------------------- fused columns
//
// Features with few distinct bins can share one histogram column: the bins b_1 .. b_m of m
// features with L_1 .. L_m levels (L_1 * ... * L_m <= 64) are stored as ONE byte
// v = b_1 + L_1 * (b_2 + L_2 * (...)), the build kernel accumulates the column's joint
// histogram over v with ONE local-memory atomic per row, and each feature's histogram is a
// marginal of it (hist_unfuse_kernel).  The paper stores features of at most 16 bins in 4 bits
// to halve the bytes (App. C.4) and spreads features that use few bins over MORE counters to
// cut atomic conflicts (Alg. 3, App. A.3); on this part conflicts cost nothing and the number
// of atomic instructions is what bounds the build, so few-level features are merged into FEWER
// counters instead.  A constant feature (one level) rides along for free.
constexpr int kFusedCap = 64;      // joint levels per column: the bin capacity of the kernel variant used
constexpr int kFusedMaxParts = 6;  // features per column: 2^6 = 64

struct FusedCol {  // one column of the fused layout
  int32_t feature[kFusedMaxParts];  // -1: unused
  uint8_t stride[kFusedMaxParts];   // L_1 * ... * L_(k-1)
  uint8_t n_parts;
  uint8_t pad;
};
struct FusedFeat {  // where a feature went
  int32_t col;
  uint8_t stride;
  uint8_t levels;  // bins 0 .. levels - 1 occur
  uint8_t pad[2];
};

// Largest bin value of every feature of a row-major matrix (maxima start at zero).  A block
// takes 256 rows; a thread walks down the columns tid, tid + 256, ...
__global__ void __launch_bounds__(256)
feature_max_kernel(const uint8_t* __restrict__ src, int64_t n_rows, int32_t n_features,
                   uint32_t* __restrict__ max_out) {
  const int64_t r0 = (int64_t)blockIdx.x * 256;
  const int64_t r1 = r0 + 256 < n_rows ? r0 + 256 : n_rows;
  for (int32_t f = threadIdx.x; f < n_features; f += 256) {
    uint32_t m = 0;
    for (int64_t r = r0; r < r1; ++r) {
      const uint32_t v = src[r * n_features + f];
      m = v > m ? v : m;
    }
    if (m) atomicMax(max_out + f, m);
  }
}

// The fused layout: feature tiles exactly as pack_kernel writes them for a matrix of n_cols
// one-byte features, a byte being the joint value of its column.  One thread per 4-byte word.
__global__ void __launch_bounds__(256)
pack_fused_kernel(const uint8_t* __restrict__ src, int64_t n_rows, int32_t n_features, TilePlan plan,
                  const FusedCol* __restrict__ cols, int32_t n_cols, uint8_t* __restrict__ dst) {
  const int32_t t = blockIdx.y;
  const int32_t w = plan_tile_width(plan, t);
  const int32_t lpr = w >> 2;
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= n_rows * lpr) return;
  const int64_t r = q / lpr;
  const int32_t j = (int32_t)(q - r * lpr);
  const int64_t tile_off = n_rows * ((int64_t)t * plan.wm);
  const uint8_t* row = src + r * (int64_t)n_features;
  uint32_t word = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int32_t c = t * plan.wm + 4 * j + i;
    uint32_t v = 0;
    if (c < n_cols) {
      const FusedCol col = cols[c];
      for (int k = 0; k < col.n_parts; ++k) v += (uint32_t)row[col.feature[k]] * col.stride[k];
      v &= (uint32_t)(kFusedCap - 1);
    }
    word |= v << (8 * i);
  }
  *reinterpret_cast<uint32_t*>(dst + tile_off + r * w + 4 * j) = word;
}

// ----------------------------------------------------------- histogram build kernel

struct BuildArgs {
  const uint8_t* packed;
  const int32_t* idx;  // NULL: rows 0..n_leaf-1
  const float* grad;
  const float* hess;
  int32_t stats_by_pos;  // grad / hess are indexed by leaf position (gathered beforehand), not by row id
  uint32_t* partials;  // one [3][cells] block of words per workgroup
  uint32_t* counters;  // per tile: the next unit of work to hand out
  int64_t n_rows;
  int64_t n_leaf;
  int32_t n_main;       // main tiles
  int32_t wr;           // remainder tile width, 0 if none
  int32_t wgs;          // workgroups per tile
  int32_t chunks;       // partial blocks per tile: wgs, or 2 * wgs with wide accumulation
  int32_t unit_epochs;  // consecutive epochs a workgroup takes at a time
  int32_t fixed_stride; // 0: units from the tile's counter; else unit u is followed by u + this
  gbdt_bin_t* direct_out;  // wgs == 1 only: the histogram itself, written by the build kernel
  int32_t n_features;
  int32_t n_bins;
};

// A histogram cell is ONE 64-bit integer that carries, from the low bits up, the
// count (10 bits), the quantised gradient sum (27 bits, signed) and the quantised
// hessian sum (27 bits, signed).  A workgroup drains its cells after every epoch
// of kEpochRows rows, so a cell receives at most 512 additions between drains.
constexpr int kEpochRows = 512;
constexpr int kUnitEpochs = 4;  // consecutive epochs a workgroup takes from its group's counter (>= 3)
constexpr int kCountBits = 10;
constexpr int kSumBits = 27;
static_assert(kEpochRows < (1 << kCountBits), "an epoch's count must fit its field");
static_assert(kCountBits + 2 * kSumBits == 64, "the three fields fill the cell");

// Power-of-two scale 2^k for quantising the values of one epoch to integers: the
// largest k with 2^k * m + kEpochRows / 2 (rounding slack) < 2^26, so that no cell's
// signed 27-bit field can overflow whatever the bins are.  m_bits: the bit pattern of
// m = 1.002 * (fp32 sum of |v| over the epoch) (the factor covers the rounding of the
// sum itself).  Integer arithmetic only: on a wave-uniform value it runs on the
// scalar unit.  A zero (or denormal) sum gives k = 0; k is kept in [-126, 126] so
// that 2^k and 2^-k are normal floats.
__device__ __forceinline__ int epoch_scale_exp(uint32_t m_bits) {
  const int e = (int)((m_bits >> 23) & 0xffu);
  const uint32_t mant = m_bits & 0x7fffffu;
  if (e == 0) return 0;
  int k = (kSumBits - 2) + 127 - e;  // 2^k * m in [2^25, 2^26)
  // 2^k * m = (1 + mant / 2^23) * 2^25 > 2^26 - kEpochRows  <=>  mant > 2^23 - kEpochRows / 4
  if (mant > (1u << 23) - (uint32_t)(kEpochRows >> (kSumBits - 25))) k -= 1;
  if (k > 126) k = 126;
  if (k < -126) k = -126;
  return k;
}
__device__ __forceinline__ float pow2f(int k) { return __uint_as_float((uint32_t)(k + 127) << 23); }

// Wide accumulation (the double precision switch of App. A.6): a (bin, feature) pair owns TWO
// 64-bit cells, gradient and hessian, each a signed 54-bit sum above the 10-bit count field (the
// count is kept in the gradient cell).  Values are scaled by 2^(k + kWideShift), k the exponent
// of the narrow format, so an epoch's sum of magnitudes stays below 2^50 and a value is rounded
// at 2^-50 of it at worst -- a fp32 value that is not 2^26 times smaller than the epoch's sum is
// taken exactly.  Cells are drained into fp64 accumulators.  Twice the LDS atomics and twice the
// LDS space of the default format.
constexpr int kWideShift = 24;
__device__ __forceinline__ double pow2d(int k) {
  return __longlong_as_double((long long)(k + 1023) << 52);
}
// round-to-nearest-even of |v| < 2^51 to a 64-bit integer (the sum's low mantissa bits)
__device__ __forceinline__ long long rint_to_i64(double v) {
  return __double_as_longlong(v + 6755399441055744.0) - 0x4338000000000000LL;
}

// Sum over the lanes of a wavefront with DPP moves (no LDS traffic); the total
// arrives in lane 63.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
  const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false);
  return v + __int_as_float(t);
}
__device__ __forceinline__ float sum_in_8(float v) {  // every lane: sum of its aligned group of 8
  v = dpp_add<0xb1, 0xf>(v);   // quad_perm [1,0,3,2]
  v = dpp_add<0x4e, 0xf>(v);   // quad_perm [2,3,0,1]
  v = dpp_add<0x141, 0xf>(v);  // row_half_mirror
  return v;
}
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
  v = sum_in_8(v);
  v = dpp_add<0x140, 0xf>(v);  // row_mirror: every lane holds the sum of its row of 16
  v = dpp_add<0x142, 0xa>(v);  // row_bcast15: rows 1 and 3 add the row before
  v = dpp_add<0x143, 0xc>(v);  // row_bcast31: rows 2 and 3 add lane 31 (rows 0 + 1)
  return v;
}

// Where a workgroup that is the only one of its (leaf, tile) writes the finished
// histogram itself instead of a partial block for the reduction pass (hist == NULL:
// partial block).
struct DirectOut {
  gbdt_bin_t* hist;  // [n_features][n_bins] of the leaf
  int32_t tile, wm, n_main, wr;
  int32_t n_features, n_bins;
};

// Compile-time shape of the work of one wavefront on a tile of width W.
template <int CAP, int W, bool NIB, int NT>
struct TileShape {
  static constexpr int VEC = NIB ? (W == 16 ? 4 : 8) : W / 4;  // bytes a lane loads: 4, 8 or 16
  static constexpr int NWORD = VEC / 4;             // 32-bit words a lane loads
  static constexpr int LPR = W / VEC;               // lanes per row
  static constexpr int RPW = 64 / LPR;              // rows per wavefront load
  static constexpr int NBW = NWORD * (NIB ? 2 : 1); // byte-words (4 bin values each) per lane
  static constexpr int SLOTS = 4 * LPR * NBW;       // features of the tile
  static constexpr int PAGES = (SLOTS + 31) / 32;
  static constexpr int CELLS = PAGES * CAP * 32;
  static constexpr int NW = NT / 64;
  static constexpr int PP = CELLS / NT;             // cells drained by one thread
  static constexpr int GPE = 64 / RPW;              // row groups per wavefront per epoch
  static_assert(NT == kEpochRows, "an epoch gives every lane one row of its own");
  static_assert(CELLS % NT == 0, "every thread drains the same number of cells");
  static_assert(LPR == 4 || LPR == 8, "a row is shared by a quad or by two quads");
};

// This workgroup's share of the histogram of leaf positions [0, end) for one feature
// tile, accumulated in its local memory and then written out as one partial block.
//
// Lane mapping.  A lane loads VEC bytes of a tile row, so a row is LPR = W / VEC
// lane-chunks and a wavefront load covers RPW = 64 / LPR rows: lane = rho * LPR + j
// loads chunk j of row rho.  The chunk's bin values are then handled in steps, 4 per
// byte-word, and the order of the 4 steps is rotated by the lane's row: in step k
// the lane takes byte q = (rho + k) mod 4.  This is the rotation of Alg. 2 (p = (l +
// s) mod 4 there) used for a stronger purpose: with slot = j + LPR * q (+ a
// compile-time term per byte-word) and cells laid out [page][bin][32 slots], the 16
// lanes whose 64-bit atomics the LDS serves together address 16 different,
// 16-aligned consecutive slots, and a row of 32 cells covers all 32 banks once, so
// the bank pair is fixed by the slot whatever the bin values are: the atomics of a
// step are free of bank conflicts by construction, not by chance as with the paper's
// 8-way interleave or its banked counters (App. A.1).  What skewed bin distributions
// (App. A.3) still cause is lanes of ONE instruction on the same address: the four rows
// of a wavefront that share a slot, when they share the bin too.  The LDS merges those
// at little cost (all 64 lanes on one cell: 8.5 instead of 6.4 cycles per instruction);
// measured on the whole kernel, a constant feature is 5 % and 60 % of the values in one
// bin 10 % slower than uniform bins at 64 bins, nothing at 256 bins -- against the 4x
// the paper reports for its hardware.  Switching the lanes of a frequent bin off does
// not help: an LDS atomic costs the same with 1 or 64 active lanes.
//
// Addressing.  The byte address of a cell inside its page is (bin << 8) | (8 *
// slot): one byte-permute builds it from the loaded bins and a per-lane table of
// the four values 8 * slot; the page is an immediate offset of the instruction.
//
// Arithmetic.  The paper adds floats with a compare-and-swap loop in local memory
// (App. B.3).  gfx950 has a native LDS float add, but it retires about 0.33
// lanes/clock/CU against about 10 for a 64-bit integer add, so values are
// accumulated as integers instead: rows are taken in epochs of kEpochRows = one row
// per thread.  A lane fetches the gradient and hessian of ITS row of the next epoch
// while the current epoch is accumulated; the workgroup sums their magnitudes, picks
// the largest power-of-two scales that cannot overflow a 27-bit field, and each lane
// quantises its own row once into a 64-bit addend that carries count, gradient and
// hessian.  The lanes that then work on a row fetch its addend with DPP moves, and
// every (row, feature) costs ONE 64-bit integer atomic.  After each epoch the cells
// are drained into accumulators held in registers (each thread owns PP cells) and
// cleared.
// Error: each value is rounded once, by at most half a quantum; the quantum is at
// most sum|g|_epoch / (2^25 - 256), so a bin is off by at most 512 / (2^26 - 512) =
// 7.7e-6 of the leaf's sum |g| (likewise for h), and integer addition is
// order-independent.  (The accumulators add one fp32 rounding per epoch on top.)
//
// Memory.  The bins of a wavefront's 64 rows of an epoch sit in one register set of
// GPE row groups; as soon as a group has been added, the same group of the next
// epoch is requested into its registers; gradients / hessians are requested one
// epoch and row ids two epochs ahead, so that requests stay in flight across the
// epoch barriers and across the hand-out of work.
//
// All wavefronts of a workgroup share ONE histogram; no replica has to be reduced.
template <int CAP, int W, bool NIB, int NT, typename ACC, bool INDEXED, bool WIDE = false>
__device__ __forceinline__ void build_tile(const uint8_t* __restrict__ tile,
                                           const int32_t* __restrict__ idx,
                                           const float* __restrict__ grad,
                                           const float* __restrict__ hess, bool stats_by_pos,
                                           uint32_t end,
                                           uint32_t first_unit, uint32_t unit_epochs,
                                           uint32_t fixed_stride, uint32_t* counter,
                                           uint32_t counter_base, unsigned long long* lds,
                                           uint32_t* __restrict__ out, const DirectOut& direct,
                                           uint32_t* __restrict__ out_lo = nullptr) {
  static_assert(!WIDE || sizeof(ACC) == 8, "wide cells are drained into fp64 accumulators");
  using S = TileShape<CAP, W, NIB, NT>;
  constexpr int VEC = S::VEC, NWORD = S::NWORD, LPR = S::LPR, RPW = S::RPW, NBW = S::NBW;
  constexpr int CELLS = S::CELLS, PP = S::PP, NW = S::NW;
  constexpr int NTBL = LPR == 8 ? 1 : 2;  // LPR 4: two byte-words share a page of 32 slots

  char* cells = reinterpret_cast<char*>(lds);
  constexpr int NCELLARR = WIDE ? 2 : 1;  // wide: gradient cells, then hessian cells
  float* red = reinterpret_cast<float*>(lds + NCELLARR * CELLS);  // [2 parities][2 stats][NW]
  uint32_t* unit_box = reinterpret_cast<uint32_t*>(red + 4 * NW);  // the unit just taken from the counter

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept scalar
  const int j = lane % LPR;
  const int rho = lane / LPR;

  // Per-lane constants of the rotated step order.
  uint32_t sel[4];     // byte-permute selectors: byte 1 = bins byte q, byte 0 = table byte q
  uint32_t tbl[NTBL];  // 8 * slot-in-page of bytes q = 0..3
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint32_t q = (uint32_t)(rho + k) & 3u;
    sel[k] = 0x0c0c0000u | ((4u + q) << 8) | q;
  }
#pragma unroll
  for (int v = 0; v < NTBL; ++v) {
    uint32_t t = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) t |= (uint32_t)(8 * (16 * v + j + LPR * q)) << (8 * q);
    tbl[v] = t;
  }

#pragma unroll
  for (int m = 0; m < PP * NCELLARR; ++m) lds[tid + m * NT] = 0ull;
  ACC acc_g[PP], acc_h[PP];
  uint32_t acc_c[PP];
#pragma unroll
  for (int m = 0; m < PP; ++m) {
    acc_g[m] = (ACC)0;
    acc_h[m] = (ACC)0;
    acc_c[m] = 0u;
  }

  static_assert(NW == 8, "the wave sums of one statistic fill one group of 8 lanes");
  auto reduce_abs = [&](float ag, float ah, int parity) {
    ag = wave_sum_to_lane63(ag);
    ah = wave_sum_to_lane63(ah);
    if (lane == 63) {
      red[parity * 2 * NW + wave] = ag;
      red[parity * 2 * NW + NW + wave] = ah;
    }
  };
  // lanes 0..7 fetch the wave sums of |g|, lanes 8..15 those of |h|; the two totals are
  // moved to scalar registers and turned into exponents there
  auto read_scales = [&](int parity, int& kg, int& kh) {
    float v = red[parity * 2 * NW + (lane & (2 * NW - 1))];
    v = sum_in_8(v) * 1.001953125f;
    kg = epoch_scale_exp(__builtin_amdgcn_readlane(__float_as_uint(v), 0));
    kh = epoch_scale_exp(__builtin_amdgcn_readlane(__float_as_uint(v), 8));
  };

  // Row ownership.  In every epoch the wavefront takes 64 consecutive leaf positions,
  // as GPE row groups of RPW rows; lane (rho, j) works on row rho of every group and
  // OWNS (fetches the row id, gradient and hessian of, and quantises) row rho of
  // group j.  The owner of a row therefore sits among the LPR lanes that work on it,
  // and its values reach them with DPP broadcasts, without LDS traffic.
  static_assert(S::GPE == LPR, "one owner lane per (row, group)");
  const uint32_t own = (uint32_t)wave * 64u + (uint32_t)(j * RPW + rho);
  // leaf position (clamped to the chunk's last row, so that every load stays in
  // range), validity and row id of the row this lane owns in the epoch starting at e0
  auto own_pos = [&](uint32_t e0) {
    const uint32_t i = e0 + own;
    return i < end ? i : end - 1;
  };
  auto own_valid = [&](uint32_t e0) { return e0 + own < end; };
  auto load_row_id = [&](uint32_t e0) -> uint32_t {
    const uint32_t i = own_pos(e0);
    return INDEXED ? (uint32_t)*reinterpret_cast<const int32_t*>(
                         reinterpret_cast<const char*>(idx) + (i << 2))
                   : i;
  };
  auto load_stat = [&](const float* a, uint32_t r) {
    return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(a) + (r << 2));
  };
  // value of `v` held by the owner of this lane's row of group gi: lane j = gi of the
  // LPR lanes that share the row
  auto from_owner = [&](uint32_t v, auto gi_tag) -> uint32_t {
    constexpr int gi = decltype(gi_tag)::value;
    if (LPR == 4) {  // quad broadcast: every lane of a quad takes lane gi of the quad
      return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, gi * 0x55, 0xf, 0xf, false);
    }
    // LPR 8: lanes 0..7 of each row of 16 take lane gi, lanes 8..15 take lane 8 + gi
    const int lo8 = __builtin_amdgcn_update_dpp(0, (int)v, 0x150 + gi, 0xf, 0x3, false);
    return (uint32_t)__builtin_amdgcn_update_dpp(lo8, (int)v, 0x158 + gi, 0xf, 0xc, false);
  };

  // Bins of one row group.  Without an index list the rows of an epoch are
  // consecutive, so group gi sits gi * RPW * W bytes behind group 0 (an immediate
  // offset of the load) and rows past the chunk end are simply read: they lie inside
  // the matrix or its slack and their addend is zero.  With an index list the row id
  // comes from the row's owner.
  constexpr int GPE = S::GPE;
  auto load_group = [&](uint4& w, uint32_t rows, uint32_t off0, auto gi_tag) {
    constexpr int gi = decltype(gi_tag)::value;
    uint32_t off;  // 32-bit byte offsets ((n_rows + slack) * W < 2^32)
    if (INDEXED) {
      off = from_owner(rows, gi_tag) * (uint32_t)W + (uint32_t)(VEC * j);
    } else {
      off = off0 + (uint32_t)(gi * RPW * W);
    }
    if (NWORD == 4) {
      w = *reinterpret_cast<const uint4*>(tile + off);
    } else if (NWORD == 2) {
      const uint2 v = *reinterpret_cast<const uint2*>(tile + off);
      w.x = v.x;
      w.y = v.y;
    } else {
      w.x = *reinterpret_cast<const uint32_t*>(tile + off);
    }
  };
  // lo, hi: the addend of the row this lane owns (zero for a row past the chunk end); wide:
  // the gradient cell's addend, and lo2, hi2 the hessian cell's
  auto add_group = [&](const uint4& w, uint32_t lo, uint32_t hi, uint32_t lo2, uint32_t hi2, auto gi_tag) {
    const unsigned long long add =
        ((unsigned long long)from_owner(hi, gi_tag) << 32) | from_owner(lo, gi_tag);
    unsigned long long add2 = 0ull;
    if (WIDE) add2 = ((unsigned long long)from_owner(hi2, gi_tag) << 32) | from_owner(lo2, gi_tag);
    uint32_t bword[NBW];
#pragma unroll
    for (int x = 0; x < NWORD; ++x) {
      const uint32_t word = x == 0 ? w.x : (x == 1 ? w.y : (x == 2 ? w.z : w.w));
      if (NIB) {
        bword[2 * x] = word & 0x0f0f0f0fu;
        bword[2 * x + 1] = (word >> 4) & 0x0f0f0f0fu;
      } else {
        bword[x] = word;  // the pack kernel keeps every bin value below CAP
      }
    }
#pragma unroll
    for (int bw = 0; bw < NBW; ++bw) {
      const int page = LPR == 8 ? bw : (bw >> 1);
      const int tv = LPR == 8 ? 0 : (bw & 1);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t a = __builtin_amdgcn_perm(bword[bw], tbl[tv], sel[k]);
        __hip_atomic_fetch_add(
            reinterpret_cast<unsigned long long*>(cells + a + page * (CAP * 256)), add,
            __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (WIDE) {
          __hip_atomic_fetch_add(
              reinterpret_cast<unsigned long long*>(cells + a + page * (CAP * 256) + CELLS * 8), add2,
              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
      }
    }
  };
  static_assert(GPE == 4 || GPE == 8, "row groups per epoch");
  // (an epoch past the leaf is read at the leaf's last epoch: in range, and ignored)
  const uint32_t n_epochs_leaf = (end + kEpochRows - 1) / kEpochRows;
  const uint32_t past = n_epochs_leaf * (uint32_t)kEpochRows;  // position of "no epoch"
  auto group_offset0 = [&](uint32_t e0) {
    const uint32_t e = e0 < past ? e0 : past - (uint32_t)kEpochRows;
    return (e + (uint32_t)wave * 64u + (uint32_t)rho) * (uint32_t)W + (uint32_t)(VEC * j);
  };
  // The bins of all row groups of one epoch, requested in group order.  (The scheduling
  // barriers keep that order: the epoch loop waits for group gi with "at most GPE + 1
  // younger requests outstanding", which is only right when the first epoch's requests were
  // issued in the order the loop re-issues them.)
  auto load_epoch = [&](uint4 (&w)[GPE], uint32_t rows, uint32_t e0) {
    const uint32_t off0 = group_offset0(e0);
    auto step = [&](auto gi_tag) {
      constexpr int gi = decltype(gi_tag)::value;
      load_group(w[gi], rows, off0, gi_tag);
      __builtin_amdgcn_sched_barrier(0);
    };
    step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{});
    step(std::integral_constant<int, 3>{});
    if constexpr (GPE == 8) {
      step(std::integral_constant<int, 4>{});
      step(std::integral_constant<int, 5>{});
      step(std::integral_constant<int, 6>{});
      step(std::integral_constant<int, 7>{});
    }
  };
  // Moves the sums of cell m into this thread's accumulators and clears it.
  auto drain_cell = [&](int m, float inv_g, float inv_h, double inv_gw, double inv_hw) {
    if constexpr (WIDE) {
      const unsigned long long tg = __hip_atomic_exchange(&lds[tid + m * NT], 0ull, __ATOMIC_RELAXED,
                                                          __HIP_MEMORY_SCOPE_WORKGROUP);
      const unsigned long long th = __hip_atomic_exchange(&lds[CELLS + tid + m * NT], 0ull, __ATOMIC_RELAXED,
                                                          __HIP_MEMORY_SCOPE_WORKGROUP);
      // the count sits below the gradient sum; an arithmetic shift drops it whatever the sign
      acc_c[m] += (uint32_t)tg & ((1u << kCountBits) - 1u);
      acc_g[m] = (ACC)fma((double)((long long)tg >> kCountBits), inv_gw, (double)acc_g[m]);
      acc_h[m] = (ACC)fma((double)((long long)th >> kCountBits), inv_hw, (double)acc_h[m]);
      return;
    }
    // read and clear in one LDS operation
    const unsigned long long t = __hip_atomic_exchange(&lds[tid + m * NT], 0ull, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_WORKGROUP);
    const uint32_t tlo = (uint32_t)t, thi = (uint32_t)(t >> 32);
    const uint32_t c = tlo & ((1u << kCountBits) - 1u);
    // bits 10..36: the gradient sum, sign-extended; the hessian sum sits above a
    // borrow of one when the gradient sum is negative
    const uint32_t mid = (thi << (32 - kCountBits)) | (tlo >> kCountBits);
    const int32_t gs = (int32_t)(mid << (32 - kSumBits)) >> (32 - kSumBits);
    const int32_t hs = ((int32_t)thi >> (kCountBits + kSumBits - 32)) + (int32_t)((mid >> (kSumBits - 1)) & 1u);
    // integer * power of two + accumulator, rounded once
    if (sizeof(ACC) == 8) {
      acc_g[m] = (ACC)fma((double)gs, (double)inv_g, (double)acc_g[m]);
      acc_h[m] = (ACC)fma((double)hs, (double)inv_h, (double)acc_h[m]);
    } else {
      acc_g[m] = (ACC)__fmaf_rn((float)gs, inv_g, (float)acc_g[m]);
      acc_h[m] = (ACC)__fmaf_rn((float)hs, inv_h, (float)acc_h[m]);
    }
    acc_c[m] += c;
  };
  // Adds the row groups of one epoch and, as soon as a group's registers are free,
  // requests the same group of the next epoch into them: every request has a whole
  // epoch to complete, requests are spread evenly over the epoch, and one register set
  // serves both epochs.
  auto add_and_reload = [&](uint4 (&w)[GPE], uint32_t lo, uint32_t hi, uint32_t lo2, uint32_t hi2,
                            uint32_t rows_nxt, uint32_t e0_nxt) {
    const uint32_t off0 = group_offset0(e0_nxt);
    auto step = [&](auto gi_tag) {
      constexpr int gi = decltype(gi_tag)::value;
      add_group(w[gi], lo, hi, lo2, hi2, gi_tag);
      load_group(w[gi], rows_nxt, off0, gi_tag);
    };
    step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{});
    step(std::integral_constant<int, 3>{});
    if constexpr (GPE == 8) {
      step(std::integral_constant<int, 4>{});
      step(std::integral_constant<int, 5>{});
      step(std::integral_constant<int, 6>{});
      step(std::integral_constant<int, 7>{});
    }
  };

  // Work distribution.  The workgroups of a tile share out the n_epochs epochs of the
  // leaf in units of unit_epochs consecutive epochs.  Workgroup c of the tile starts
  // with unit c; when it enters a unit, one lane takes the next one from the tile's
  // counter (a global atomic that starts at zero: the take is counter_base + its old
  // value, counter_base = the units the workgroups started with), and the pipeline of
  // requests (row ids two epochs ahead, gradients / hessians and bins one epoch ahead)
  // runs on from the last epoch of a unit into the first epoch of the next.  Fast and
  // slow workgroups (the CU issues the instructions of its oldest workgroup first) so
  // end within a unit of each other, and one partial block per workgroup suffices.
  // Looking two epochs ahead needs the next unit from a unit's second-last epoch on:
  // the counter is only used with units of at least 3 epochs; shorter units (short
  // leaves) are handed out one per workgroup, and every take from the counter fails.
  // (Units also keep a workgroup's rows together.)
  // With fixed_stride != 0 the counter is not used: after unit u a workgroup takes unit
  // u + fixed_stride.  The grouping of epochs into partial sums is then the same in
  // every run, and so is every bit of the result.
  struct Pos {
    uint32_t row;  // first leaf position of the epoch; `past`: no epoch
    uint32_t idx;  // its number inside its unit
  };
  const uint32_t n_units = (n_epochs_leaf + unit_epochs - 1) / unit_epochs;
  uint32_t next_unit = n_units;  // the unit taken from the counter (n_units or more: none)
  auto unit_first = [&](uint32_t u) {
    Pos r;
    r.row = u < n_units ? u * unit_epochs * (uint32_t)kEpochRows : past;
    r.idx = 0;
    return r;
  };
  auto after = [&](Pos x) {  // the epoch after x in this workgroup's sequence
    if (x.row >= past) return x;
    Pos r;
    r.row = x.row + kEpochRows;
    r.idx = x.idx + 1;
    // the leaf may end inside its last unit
    if (r.idx == unit_epochs || r.row >= past) {
      // The taken unit is used up: until the next take arrives there is no further unit
      // (only the leaf's short last unit can end before that, and nothing follows it).
      r = unit_first(next_unit);
      next_unit = n_units;
    }
    return r;
  };
  Pos p0 = unit_first(first_unit), p1 = after(p0), p2 = after(p1);

  int kg, kh;
  // rows the lane owns in the current epoch and the next one; the current row's stats
  uint32_t row_cur = load_row_id(p0.row);
  uint32_t row_nxt = load_row_id(p1.row);
  // gradients / hessians are indexed by row id, or (stats_by_pos) by leaf position when the
  // call has gathered them into leaf order beforehand
  float g_cur = load_stat(grad, stats_by_pos ? own_pos(p0.row) : row_cur);
  float h_cur = load_stat(hess, stats_by_pos ? own_pos(p0.row) : row_cur);
  uint4 w[GPE];
  load_epoch(w, row_cur, p0.row);
  {
    const bool ok = own_valid(p0.row);
    reduce_abs(ok ? fabsf(g_cur) : 0.0f, ok ? fabsf(h_cur) : 0.0f, 0);
  }
  __syncthreads();  // also orders the LDS clearing before the first atomics
  read_scales(0, kg, kh);

  uint32_t parity = 0;
  while (p0.row < end) {  // uniform over the workgroup
    const bool enters_unit = p0.idx == 0;
    uint32_t taken = 0;
    if (enters_unit) {
      if (fixed_stride) {
        taken = p0.row / (unit_epochs * (uint32_t)kEpochRows) + fixed_stride;
      } else if (tid == 0) {
        taken = counter_base + __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    // ---- requests for later epochs
    const uint32_t row_nn = load_row_id(p2.row);
    const uint32_t stat_nxt = stats_by_pos ? own_pos(p1.row) : row_nxt;
    const float g_nxt = load_stat(grad, stat_nxt);
    const float h_nxt = load_stat(hess, stat_nxt);
    // ---- this lane's row -> 64-bit addend 1 + gq * 2^10 + hq * 2^37 (two's complement)
    //      (wide: 1 + gq * 2^10 into the gradient cell, hq * 2^10 into the hessian cell)
    uint32_t lo, hi, lo2 = 0u, hi2 = 0u;
    if constexpr (WIDE) {
      const long long gq = rint_to_i64((double)g_cur * pow2d(kg + kWideShift));
      const long long hq = rint_to_i64((double)h_cur * pow2d(kh + kWideShift));
      const unsigned long long ag = ((unsigned long long)gq << kCountBits) + 1ull;
      const unsigned long long ah = (unsigned long long)hq << kCountBits;
      const bool ok = own_valid(p0.row);
      lo = ok ? (uint32_t)ag : 0u;
      hi = ok ? (uint32_t)(ag >> 32) : 0u;
      lo2 = ok ? (uint32_t)ah : 0u;
      hi2 = ok ? (uint32_t)(ah >> 32) : 0u;
    } else {
      const int32_t gq = __float2int_rn(g_cur * pow2f(kg));
      const int32_t hq = __float2int_rn(h_cur * pow2f(kh));
      lo = ((uint32_t)gq << kCountBits) + 1u;
      hi = (uint32_t)(gq >> (32 - kCountBits)) + ((uint32_t)hq << (kCountBits + kSumBits - 32));
      const bool ok = own_valid(p0.row);
      lo = ok ? lo : 0u;
      hi = ok ? hi : 0u;
    }
    // The atomics are what the kernel is bound by; the drain of a co-resident workgroup is
    // mostly VALU work.  Raised priority lets the waves that feed the LDS pipe issue first,
    // and the other workgroup's drain fills the gaps (8-12 % on the 256-bin variants).
    __builtin_amdgcn_s_setprio(1);
    add_and_reload(w, lo, hi, lo2, hi2, row_nxt, p1.row);
    __builtin_amdgcn_s_setprio(0);

    parity ^= 1u;
    {
      const bool ok = own_valid(p1.row);
      reduce_abs(ok ? fabsf(g_nxt) : 0.0f, ok ? fabsf(h_nxt) : 0.0f, (int)parity);
    }
    if (enters_unit && !fixed_stride && tid == 0) unit_box[0] = taken;
    __syncthreads();  // all atomics of the epoch have landed

    // ---- drain: integer sums -> registers, clear the cells for the next epoch
    const float inv_g = pow2f(-kg), inv_h = pow2f(-kh);
    const double inv_gw = pow2d(-kg - kWideShift), inv_hw = pow2d(-kh - kWideShift);
    // The next epoch's scales are requested from local memory BEFORE the cells: results come
    // back in order, so the cells can then be decoded one by one as they arrive, instead of
    // all of them being waited for because the youngest request is needed first.
    read_scales((int)parity, kg, kh);
    if (enters_unit) next_unit = __builtin_amdgcn_readfirstlane(fixed_stride ? taken : unit_box[0]);
#pragma unroll
    for (int m = 0; m < PP; ++m) drain_cell(m, inv_g, inv_h, inv_gw, inv_hw);
    p0 = p1;
    p1 = p2;
    p2 = after(p2);
    row_cur = row_nxt;
    row_nxt = row_nn;
    g_cur = g_nxt;
    h_cur = h_nxt;
    __syncthreads();  // cells are clear, `red` and the unit box are read, before reuse
  }

  if (direct.hist) {
    // The tile's only workgroup: its sums are the histogram.  Cell -> (bin, slot) ->
    // feature, as the reduction pass would do it.
    TilePlan plan;
    plan.cap = CAP;
    plan.nib = NIB ? 1 : 0;
    plan.wm = direct.wm;
    plan.n_main = direct.n_main;
    plan.wr = direct.wr;
    plan.row_bytes = plan.feat_bytes = 0;  // not used by the slot -> feature map
#pragma unroll
    for (int m = 0; m < PP; ++m) {
      const int cell = tid + m * NT;
      const int bin = (cell >> 5) % CAP;
      const int slot = (cell / (CAP * 32)) * 32 + (cell & 31);
      const int32_t f = plan_feature_of(plan, direct.tile, slot);
      if (slot < S::SLOTS && bin < direct.n_bins && f < direct.n_features) {
        gbdt_bin_t r;
        r.grad = (float)acc_g[m];
        r.hess = (float)acc_h[m];
        r.count = acc_c[m];
        direct.hist[(size_t)f * direct.n_bins + bin] = r;
      }
    }
    return;
  }
  // partial block layout: [stat][cell] words
#pragma unroll
  for (int m = 0; m < PP; ++m) {
    out[tid + m * NT] = __float_as_uint((float)acc_g[m]);
    out[CELLS + tid + m * NT] = __float_as_uint((float)acc_h[m]);
    out[2 * CELLS + tid + m * NT] = acc_c[m];
  }
  if constexpr (WIDE) {
    // what fp32 cannot hold of the fp64 sums goes into a second block of the same layout (count
    // 0), which the reduction pass adds like any other workgroup's
#pragma unroll
    for (int m = 0; m < PP; ++m) {
      const double g = (double)acc_g[m], h = (double)acc_h[m];
      out_lo[tid + m * NT] = __float_as_uint((float)(g - (double)(float)g));
      out_lo[CELLS + tid + m * NT] = __float_as_uint((float)(h - (double)(float)h));
      out_lo[2 * CELLS + tid + m * NT] = 0u;
    }
  }
}

// Words of one partial block of a tile of width W.
template <int CAP, int W, bool NIB, int NT>
__device__ __host__ constexpr int block_words() {
  return 3 * TileShape<CAP, W, NIB, NT>::CELLS;
}

// Work is split by feature tiles and by samples (Sec. 4, "Parallel By Features and
// Data"): every tile has a fixed set of workgroups that share out its epochs.  Block
// -> (tile, workgroup of the tile); consecutive blocks take different tiles, so the
// row ids / gradients / hessians of an epoch are fetched from HBM once and served to
// the other tiles from cache.
template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC, bool INDEXED, bool WIDE = false>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
hist_build_kernel(BuildArgs a) {
  // one histogram of the main tile width (8 bytes per cell; two with wide accumulation), the
  // reduction scratch and the unit box
  constexpr int kCells = (WIDE ? 2 : 1) * TileShape<CAP, WM, NIB, NT>::CELLS;
  __shared__ __align__(16) unsigned long long lds[kCells + (4 * (NT / 64) * 4 + 7) / 8 + 1];
  const int32_t main_blocks = a.n_main * a.wgs;
  const int32_t b = blockIdx.x;
  const uint32_t n_leaf = (uint32_t)a.n_leaf;
  const int32_t t = b < main_blocks ? b % a.n_main : a.n_main;         // tile
  const int32_t c = b < main_blocks ? b / a.n_main : b - main_blocks;  // workgroup of the tile
  uint32_t* counter = a.counters + plan_counter_slot(t);
  const uint8_t* tile = a.packed + a.n_rows * ((int64_t)t * WM);
  const DirectOut direct = {a.direct_out, t, WM, a.n_main, a.wr, a.n_features, a.n_bins};
  // wide accumulation: the workgroup's second block lies a.wgs blocks behind its first
  if (b < main_blocks) {
    constexpr size_t kBlock = (size_t)block_words<CAP, WM, NIB, NT>();
    uint32_t* out = a.partials + ((size_t)t * a.chunks + c) * kBlock;
    build_tile<CAP, WM, NIB, NT, ACC, INDEXED, WIDE>(tile, a.idx, a.grad, a.hess, a.stats_by_pos != 0, n_leaf,
                                                     (uint32_t)c, (uint32_t)a.unit_epochs,
                                                     (uint32_t)a.fixed_stride, counter, (uint32_t)a.wgs, lds,
                                                     out, direct, out + (size_t)a.wgs * kBlock);
  } else {
    uint32_t* rem_base =
        a.partials + (size_t)a.n_main * a.chunks * (size_t)block_words<CAP, WM, NIB, NT>();
    if (a.wr == 16) {
      constexpr size_t kBlock = (size_t)block_words<CAP, 16, NIB, NT>();
      build_tile<CAP, 16, NIB, NT, ACC, INDEXED, WIDE>(
          tile, a.idx, a.grad, a.hess, a.stats_by_pos != 0, n_leaf, (uint32_t)c, (uint32_t)a.unit_epochs,
          (uint32_t)a.fixed_stride, counter, (uint32_t)a.wgs, lds, rem_base + (size_t)c * kBlock, direct,
          rem_base + (size_t)(a.wgs + c) * kBlock);
    } else if constexpr (WM > 32) {
      constexpr size_t kBlock = (size_t)block_words<CAP, 32, NIB, NT>();
      build_tile<CAP, 32, NIB, NT, ACC, INDEXED, WIDE>(
          tile, a.idx, a.grad, a.hess, a.stats_by_pos != 0, n_leaf, (uint32_t)c, (uint32_t)a.unit_epochs,
          (uint32_t)a.fixed_stride, counter, (uint32_t)a.wgs, lds, rem_base + (size_t)c * kBlock, direct,
          rem_base + (size_t)(a.wgs + c) * kBlock);
    }
  }
}

// Gradients and hessians of a row list, in list order: g_out[i] = grad[idx[i]].  The paper
// has the CPU prepare these "ordered" arrays for every leaf (App. A.5, App. C.1); here they pay
// when many feature tiles would each gather the same scattered 4-byte values again.
__global__ void __launch_bounds__(256)
stats_gather_kernel(const int32_t* __restrict__ idx, const float* __restrict__ grad,
                    const float* __restrict__ hess, int64_t n, float* __restrict__ g_out,
                    float* __restrict__ h_out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint32_t r = (uint32_t)idx[i];
  g_out[i] = grad[r];
  h_out[i] = hess[r];
}

// The unit counters of all tiles live at the head of the scratch workspace and are zero
// between calls: a workgroup's take is (workgroups per tile) + (old counter value), and
// the reduction pass, which follows every build that used them, sets them back to zero.
// This kernel zeroes them when a workspace is new.  (A fill kernel, not a memset node, so
// the call can be captured into a graph.)
__global__ void __launch_bounds__(256) counters_zero_kernel(uint32_t* counters, int32_t n_counters) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_counters) counters[i] = 0u;
}

// Several leaves in one launch.  Small leaves cannot fill the machine on their own (the
// synthetic benchmark of App. C.2 shows the rate falling with the leaf size); a level of
// a tree, or both children of a split, can.  The launch carries a table of up to
// kBatchLeaves leaves as kernel arguments -- nothing is staged through memory.  Leaf l
// (batch_plan.h) owns the row list idx[row_off .. row_off + n) and wgs workgroups per tile, which take
// its units of unit_epochs epochs in a fixed stride (no counters): a workgroup of leaf l
// runs build_tile exactly as a single-leaf launch in its fixed-split mode would, and the
// leaves' partial blocks lie back to back, each leaf's in the single-leaf order.  A leaf
// with one workgroup per tile writes its histogram itself and skips the reduction pass.
struct BatchArgs {
  const uint8_t* packed;
  const int32_t* idx;
  const float* grad;
  const float* hess;
  int32_t stats_by_pos;
  uint32_t* partials;
  int64_t n_rows;
  int32_t n_main;
  int32_t wr;
  int32_t n_leaves;
  gbdt_bin_t* hist_out;  // [n_leaves][n_features][n_bins]: written directly by leaves of one workgroup per tile
  int32_t n_features;
  int32_t n_bins;
  BatchLeaf leaf[kBatchLeaves];
};

// Words of the partial blocks one workgroup column (one workgroup of every tile) writes.
template <int CAP, int WM, bool NIB, int NT>
__device__ __host__ inline size_t column_words(int32_t n_main, int32_t wr) {
  size_t w = (size_t)n_main * block_words<CAP, WM, NIB, NT>();
  if (wr == 16) w += block_words<CAP, 16, NIB, NT>();
  if (wr == 32) w += block_words<CAP, 32, NIB, NT>();
  return w;
}

template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC, bool WIDE = false>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
hist_build_batch_kernel(BatchArgs a) {
  constexpr int kCells = (WIDE ? 2 : 1) * TileShape<CAP, WM, NIB, NT>::CELLS;
  __shared__ __align__(16) unsigned long long lds[kCells + (4 * (NT / 64) * 4 + 7) / 8 + 1];
  const BatchBlock blk = batch_block(a.leaf, a.n_leaves, a.n_main, a.wr, blockIdx.x);
  const BatchLeaf lf = a.leaf[blk.leaf];
  const int32_t wgs = (int32_t)(lf.wgs_unit & 0xffffu);
  const uint32_t unit_epochs = lf.wgs_unit >> 16;
  constexpr int kPerWg = WIDE ? 2 : 1;  // partial blocks per workgroup
  const int32_t chunks = kPerWg * wgs;
  const int32_t t = blk.tile, c = blk.wg;
  const bool is_main = t < a.n_main;
  const uint8_t* tile = a.packed + a.n_rows * ((int64_t)t * WM);
  const int32_t* idx = a.idx + lf.row_off;
  const bool by_pos = a.stats_by_pos != 0;  // then grad / hess follow the concatenated row lists
  const float* grad = by_pos ? a.grad + lf.row_off : a.grad;
  const float* hess = by_pos ? a.hess + lf.row_off : a.hess;
  uint32_t* leaf_out =
      a.partials + (size_t)lf.first_wg * kPerWg * column_words<CAP, WM, NIB, NT>(a.n_main, a.wr);
  const DirectOut direct = {
      wgs == 1 ? a.hist_out + (size_t)blk.leaf * a.n_features * a.n_bins : nullptr,
      t, WM, a.n_main, a.wr, a.n_features, a.n_bins};
  if (is_main) {
    constexpr size_t kBlock = (size_t)block_words<CAP, WM, NIB, NT>();
    uint32_t* out = leaf_out + ((size_t)t * chunks + c) * kBlock;
    build_tile<CAP, WM, NIB, NT, ACC, true, WIDE>(tile, idx, grad, hess, by_pos, lf.n, (uint32_t)c, unit_epochs,
                                                  (uint32_t)wgs, nullptr, 0u, lds, out, direct,
                                                  out + (size_t)wgs * kBlock);
  } else {
    uint32_t* rem_base = leaf_out + (size_t)a.n_main * chunks * (size_t)block_words<CAP, WM, NIB, NT>();
    if (a.wr == 16) {
      constexpr size_t kBlock = (size_t)block_words<CAP, 16, NIB, NT>();
      build_tile<CAP, 16, NIB, NT, ACC, true, WIDE>(tile, idx, grad, hess, by_pos, lf.n, (uint32_t)c, unit_epochs,
                                                    (uint32_t)wgs, nullptr, 0u, lds, rem_base + (size_t)c * kBlock,
                                                    direct, rem_base + (size_t)(wgs + c) * kBlock);
    } else if constexpr (WM > 32) {
      constexpr size_t kBlock = (size_t)block_words<CAP, 32, NIB, NT>();
      build_tile<CAP, 32, NIB, NT, ACC, true, WIDE>(tile, idx, grad, hess, by_pos, lf.n, (uint32_t)c, unit_epochs,
                                                    (uint32_t)wgs, nullptr, 0u, lds, rem_base + (size_t)c * kBlock,
                                                    direct, rem_base + (size_t)(wgs + c) * kBlock);
    }
  }
}

}  // namespace

#endif  // GBDT_HIST_BUILD_KERNELS_H_
