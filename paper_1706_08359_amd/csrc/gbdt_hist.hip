// libgbdt_hist: feature-histogram construction, sibling subtraction and best-split
// scan for histogram-based GBDT training on AMD gfx950 (MI355X).
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
#include <mutex>
#include <type_traits>
#include <utility>
#include <vector>

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

// ----------------------------------------------------------- histogram build kernel

struct BuildArgs {
  const uint8_t* packed;
  const int32_t* idx;  // NULL: rows 0..n_leaf-1
  const float* grad;
  const float* hess;
  uint32_t* partials;  // one [3][cells] block of words per workgroup
  uint32_t* counters;  // per tile: the next unit of work to hand out
  int64_t n_rows;
  int64_t n_leaf;
  int32_t n_main;       // main tiles
  int32_t wr;           // remainder tile width, 0 if none
  int32_t wgs;          // workgroups per tile
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
// step are free of bank conflicts and of same-address collisions by construction,
// not by chance as with the paper's 8-way interleave or its banked counters
// (App. A.1).  Skewed bin distributions (App. A.3) cost nothing extra.
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
template <int CAP, int W, bool NIB, int NT, typename ACC, bool INDEXED>
__device__ __forceinline__ void build_tile(const uint8_t* __restrict__ tile,
                                           const int32_t* __restrict__ idx,
                                           const float* __restrict__ grad,
                                           const float* __restrict__ hess, uint32_t end,
                                           uint32_t first_unit, uint32_t unit_epochs,
                                           uint32_t fixed_stride, uint32_t* counter,
                                           unsigned long long* lds,
                                           uint32_t* __restrict__ out, const DirectOut& direct) {
  using S = TileShape<CAP, W, NIB, NT>;
  constexpr int VEC = S::VEC, NWORD = S::NWORD, LPR = S::LPR, RPW = S::RPW, NBW = S::NBW;
  constexpr int CELLS = S::CELLS, PP = S::PP, NW = S::NW;
  constexpr int NTBL = LPR == 8 ? 1 : 2;  // LPR 4: two byte-words share a page of 32 slots

  char* cells = reinterpret_cast<char*>(lds);
  float* red = reinterpret_cast<float*>(lds + CELLS);  // [2 parities][2 stats][NW]
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
  for (int m = 0; m < PP; ++m) lds[tid + m * NT] = 0ull;
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
  // lo, hi: the addend of the row this lane owns (zero for a row past the chunk end)
  auto add_group = [&](const uint4& w, uint32_t lo, uint32_t hi, auto gi_tag) {
    const unsigned long long add =
        ((unsigned long long)from_owner(hi, gi_tag) << 32) | from_owner(lo, gi_tag);
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
  auto drain_cell = [&](int m, float inv_g, float inv_h) {
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
  auto add_and_reload = [&](uint4 (&w)[GPE], uint32_t lo, uint32_t hi, uint32_t rows_nxt,
                            uint32_t e0_nxt) {
    const uint32_t off0 = group_offset0(e0_nxt);
    auto step = [&](auto gi_tag) {
      constexpr int gi = decltype(gi_tag)::value;
      add_group(w[gi], lo, hi, gi_tag);
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
  // counter (a global atomic), and the pipeline of
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
  float g_cur = load_stat(grad, row_cur);
  float h_cur = load_stat(hess, row_cur);
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
        taken = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    // ---- requests for later epochs
    const uint32_t row_nn = load_row_id(p2.row);
    const float g_nxt = load_stat(grad, row_nxt);
    const float h_nxt = load_stat(hess, row_nxt);
    // ---- this lane's row -> 64-bit addend 1 + gq * 2^10 + hq * 2^37 (two's complement)
    uint32_t lo, hi;
    {
      const int32_t gq = __float2int_rn(g_cur * pow2f(kg));
      const int32_t hq = __float2int_rn(h_cur * pow2f(kh));
      lo = ((uint32_t)gq << kCountBits) + 1u;
      hi = (uint32_t)(gq >> (32 - kCountBits)) + ((uint32_t)hq << (kCountBits + kSumBits - 32));
      const bool ok = own_valid(p0.row);
      lo = ok ? lo : 0u;
      hi = ok ? hi : 0u;
    }
    add_and_reload(w, lo, hi, row_nxt, p1.row);

    parity ^= 1u;
    {
      const bool ok = own_valid(p1.row);
      reduce_abs(ok ? fabsf(g_nxt) : 0.0f, ok ? fabsf(h_nxt) : 0.0f, (int)parity);
    }
    if (enters_unit && !fixed_stride && tid == 0) unit_box[0] = taken;
    __syncthreads();  // all atomics of the epoch have landed

    // ---- drain: integer sums -> registers, clear the cells for the next epoch
    const float inv_g = pow2f(-kg), inv_h = pow2f(-kh);
#pragma unroll
    for (int m = 0; m < PP; ++m) drain_cell(m, inv_g, inv_h);
    read_scales((int)parity, kg, kh);
    if (enters_unit) next_unit = __builtin_amdgcn_readfirstlane(fixed_stride ? taken : unit_box[0]);
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
template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC, bool INDEXED>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
hist_build_kernel(BuildArgs a) {
  // one histogram of the main tile width (8 bytes per cell), the reduction scratch and
  // the unit box
  constexpr int kCells = TileShape<CAP, WM, NIB, NT>::CELLS;
  __shared__ __align__(16) unsigned long long lds[kCells + (4 * (NT / 64) * 4 + 7) / 8 + 1];
  const int32_t main_blocks = a.n_main * a.wgs;
  const int32_t b = blockIdx.x;
  const uint32_t n_leaf = (uint32_t)a.n_leaf;
  const int32_t t = b < main_blocks ? b % a.n_main : a.n_main;         // tile
  const int32_t c = b < main_blocks ? b / a.n_main : b - main_blocks;  // workgroup of the tile
  uint32_t* counter = a.counters + t;
  const uint8_t* tile = a.packed + a.n_rows * ((int64_t)t * WM);
  const DirectOut direct = {a.direct_out, t, WM, a.n_main, a.wr, a.n_features, a.n_bins};
  if (b < main_blocks) {
    uint32_t* out = a.partials + ((size_t)t * a.wgs + c) * (size_t)block_words<CAP, WM, NIB, NT>();
    build_tile<CAP, WM, NIB, NT, ACC, INDEXED>(tile, a.idx, a.grad, a.hess, n_leaf, (uint32_t)c,
                                               (uint32_t)a.unit_epochs, (uint32_t)a.fixed_stride, counter,
                                               lds, out, direct);
  } else {
    uint32_t* rem_base = a.partials + (size_t)main_blocks * (size_t)block_words<CAP, WM, NIB, NT>();
    if (a.wr == 16) {
      build_tile<CAP, 16, NIB, NT, ACC, INDEXED>(
          tile, a.idx, a.grad, a.hess, n_leaf, (uint32_t)c, (uint32_t)a.unit_epochs,
          (uint32_t)a.fixed_stride, counter, lds,
          rem_base + (size_t)c * (size_t)block_words<CAP, 16, NIB, NT>(), direct);
    } else if constexpr (WM > 32) {
      build_tile<CAP, 32, NIB, NT, ACC, INDEXED>(
          tile, a.idx, a.grad, a.hess, n_leaf, (uint32_t)c, (uint32_t)a.unit_epochs,
          (uint32_t)a.fixed_stride, counter, lds,
          rem_base + (size_t)c * (size_t)block_words<CAP, 32, NIB, NT>(), direct);
    }
  }
}

// Sets every tile's unit counter to the number of units its workgroups start with
// (one each).  (A fill kernel, not a memset node, so the call can be captured into a
// graph.)
__global__ void __launch_bounds__(256)
counters_init_kernel(uint32_t* counters, int32_t wgs, int32_t n_counters) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_counters) counters[i] = (uint32_t)wgs;
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

template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
hist_build_batch_kernel(BatchArgs a) {
  constexpr int kCells = TileShape<CAP, WM, NIB, NT>::CELLS;
  __shared__ __align__(16) unsigned long long lds[kCells + (4 * (NT / 64) * 4 + 7) / 8 + 1];
  const BatchBlock blk = batch_block(a.leaf, a.n_leaves, a.n_main, a.wr, blockIdx.x);
  const BatchLeaf lf = a.leaf[blk.leaf];
  const int32_t wgs = (int32_t)(lf.wgs_unit & 0xffffu);
  const uint32_t unit_epochs = lf.wgs_unit >> 16;
  const int32_t main_blocks = a.n_main * wgs;
  const int32_t t = blk.tile, c = blk.wg;
  const bool is_main = t < a.n_main;
  const uint8_t* tile = a.packed + a.n_rows * ((int64_t)t * WM);
  const int32_t* idx = a.idx + lf.row_off;
  uint32_t* leaf_out = a.partials + (size_t)lf.first_wg * column_words<CAP, WM, NIB, NT>(a.n_main, a.wr);
  const DirectOut direct = {
      wgs == 1 ? a.hist_out + (size_t)blk.leaf * a.n_features * a.n_bins : nullptr,
      t, WM, a.n_main, a.wr, a.n_features, a.n_bins};
  if (is_main) {
    build_tile<CAP, WM, NIB, NT, ACC, true>(
        tile, idx, a.grad, a.hess, lf.n, (uint32_t)c, unit_epochs, (uint32_t)wgs, nullptr, lds,
        leaf_out + ((size_t)t * wgs + c) * (size_t)block_words<CAP, WM, NIB, NT>(), direct);
  } else {
    uint32_t* rem_base = leaf_out + (size_t)main_blocks * (size_t)block_words<CAP, WM, NIB, NT>();
    if (a.wr == 16) {
      build_tile<CAP, 16, NIB, NT, ACC, true>(tile, idx, a.grad, a.hess, lf.n, (uint32_t)c, unit_epochs,
                                              (uint32_t)wgs, nullptr, lds,
                                              rem_base + (size_t)c * (size_t)block_words<CAP, 16, NIB, NT>(),
                                              direct);
    } else if constexpr (WM > 32) {
      build_tile<CAP, 32, NIB, NT, ACC, true>(tile, idx, a.grad, a.hess, lf.n, (uint32_t)c, unit_epochs,
                                              (uint32_t)wgs, nullptr, lds,
                                              rem_base + (size_t)c * (size_t)block_words<CAP, 32, NIB, NT>(),
                                              direct);
    }
  }
}

// ------------------------------------------------------------------ merge kernel

struct MergeArgs {
  const uint32_t* partials;
  gbdt_bin_t* out;
  TilePlan plan;
  int32_t n_features;
  int32_t n_bins;
  int32_t chunks_main;
  int32_t chunks_rem;
};

constexpr int kMergeCells = 64;   // histogram cells per workgroup
constexpr int kMergeLanes = 4;    // threads that share the chunks of one cell

// The "final reduction program" of Sec. 4: sums the partial histograms of the
// workgroups that shared a feature tile.  A workgroup takes 64 consecutive (bin,
// slot) pairs of one tile (slot fastest, so reads of a partial block are coalesced
// in runs of 32); 4 threads per pair each sum every 4th chunk in fp64, in chunk
// order, and the 4 sub-sums are added in a fixed order: the result does not depend
// on scheduling.  Counts are summed as integers.  grid.y = tile.
__device__ __forceinline__ void merge_cells(const MergeArgs& a) {
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
    for (int32_t c = part; c < chunks; c += kMergeLanes) {
      g += (double)__uint_as_float(p[0]);
      h += (double)__uint_as_float(p[hw]);
      n += p[2 * hw];
      p += (size_t)kMergeLanes * 3 * hw;
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

__global__ void __launch_bounds__(kMergeCells * kMergeLanes) hist_merge_kernel(MergeArgs a) {
  merge_cells(a);
}

// The same reduction for a batched launch: grid.z = leaf of the launch; its partial
// blocks start first_wg workgroup columns into the buffer, its histogram is the leaf's
// [n_features][n_bins] slice of the output.  A leaf without rows has no partial blocks
// and gets zeros; a leaf with a single workgroup per tile is skipped.
struct BatchMergeArgs {
  MergeArgs m;            // partials / out of leaf 0 of the launch; chunk counts unused
  uint64_t column_words;  // words of one workgroup column
  BatchLeaf leaf[kBatchLeaves];
};

__global__ void __launch_bounds__(kMergeCells * kMergeLanes) hist_merge_batch_kernel(BatchMergeArgs a) {
  const BatchLeaf lf = a.leaf[blockIdx.z];
  if ((lf.wgs_unit & 0xffffu) == 1u) return;  // written by the build kernel itself
  MergeArgs m = a.m;
  m.partials += (size_t)lf.first_wg * a.column_words;
  m.out += (size_t)blockIdx.z * m.n_features * m.n_bins;
  m.chunks_main = (int32_t)(lf.wgs_unit & 0xffffu);
  m.chunks_rem = m.plan.wr ? m.chunks_main : 0;
  merge_cells(m);
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

// ------------------------------------------------------------------ split kernels

struct SplitCand {
  double gain;
  double gl, hl, gr, hr;
  uint32_t nl, nr;
  int32_t feature;  // -1: no admissible threshold among this workgroup's features
  int32_t bin;
};

static_assert(sizeof(SplitCand) == 7 * 8, "a candidate is moved as 7 64-bit words");

constexpr int kSplitThreads = 256;
constexpr int kSplitLdsBudget = 48 * 1024;
constexpr int kSplitMaxHists = 32768;  // histograms per launch (grid.y)

// One ticket counter per histogram of a launch: the workgroups of a histogram count
// themselves off, and the last of them sets the counter back to zero, so the counters
// need no resetting between launches (zero when the module is loaded).
__device__ unsigned int g_split_ticket[kSplitMaxHists];

// Candidates cross from the workgroups that write them to the one that reduces them,
// possibly on another XCD with its own L2: they are moved with device-scope atomic
// accesses (which bypass the caches that are not coherent across XCDs), inside the
// release / acquire fences around the ticket.
__device__ __forceinline__ void store_cand(SplitCand* dst, const SplitCand& c) {
  unsigned long long w[7];
  memcpy(w, &c, sizeof c);
  unsigned long long* d = reinterpret_cast<unsigned long long*>(dst);
#pragma unroll
  for (int i = 0; i < 7; ++i) __hip_atomic_store(d + i, w[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ SplitCand load_cand(const SplitCand* src) {
  unsigned long long w[7];
  const unsigned long long* p = reinterpret_cast<const unsigned long long*>(src);
#pragma unroll
  for (int i = 0; i < 7; ++i)
    w[i] = __hip_atomic_load(const_cast<unsigned long long*>(p) + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  SplitCand c;
  memcpy(&c, w, sizeof c);
  return c;
}
__device__ __forceinline__ double load_cand_gain(const SplitCand* src) {
  const unsigned long long w = __hip_atomic_load(
      const_cast<unsigned long long*>(reinterpret_cast<const unsigned long long*>(src)), __ATOMIC_RELAXED,
      __HIP_MEMORY_SCOPE_AGENT);
  double g;
  memcpy(&g, &w, sizeof g);
  return g;
}
__device__ __forceinline__ int32_t load_cand_feature(const SplitCand* src) {
  // word 6 = (feature, bin)
  const unsigned long long w = __hip_atomic_load(
      const_cast<unsigned long long*>(reinterpret_cast<const unsigned long long*>(src)) + 6, __ATOMIC_RELAXED,
      __HIP_MEMORY_SCOPE_AGENT);
  return (int32_t)(uint32_t)(w & 0xffffffffull);
}

// LDS bytes one feature needs in split_gain_kernel: fp64 running sums of gradient,
// hessian and count per bin (bins padded to a multiple of 8), + the feature's parent term.
__host__ __device__ inline int split_padded_bins(int n_bins) { return (n_bins + 7) & ~7; }
__host__ __device__ inline int split_feature_bytes(int n_bins) { return 24 * split_padded_bins(n_bins) + 8; }

// Gain scan of Sec. 3.3.  A workgroup takes a group of consecutive features.
//  1. Their histogram rows are copied into local memory as doubles.
//  2. One lane per (feature, statistic) runs the left-to-right prefix sum of grad, hess
//     or count in fp64, bins ascending (this fixes the rounding order).
//  3. All lanes then evaluate the gain of every (feature, threshold) pair from those
//     prefixes -- the divisions, the expensive part -- and keep the best pair under
//     the order "larger gain, then smaller feature, then smaller bin".
// Feature totals are the prefix at the last bin, right = total - left, a threshold is
// admissible when both sides hold >= 1 sample and >= min_child_hess of hessian.
//  4. The workgroup that finishes last for its histogram (a ticket taken after its own
//     candidate is written and fenced; nobody waits) reduces the candidates of all
//     workgroups to the histogram's split record: workgroups hold ascending feature
//     groups, so "smaller candidate index" is "smaller feature".
// grid.y = histogram of the call; histogram y starts hist_stride bins after histogram
// y - 1 (the stride may be negative: any two histograms of a pool can be searched in
// one launch).
__global__ void __launch_bounds__(kSplitThreads)
split_gain_kernel(const gbdt_bin_t* __restrict__ hist, int64_t hist_stride, int32_t n_features,
                  int32_t n_bins, int32_t group, double lambda, double min_child_hess,
                  SplitCand* __restrict__ cand, gbdt_split_t* __restrict__ out) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ double s_gain[kSplitThreads];
  __shared__ int32_t s_pair[kSplitThreads];
  __shared__ int s_last;
  const int tid = threadIdx.x;
  hist += (int64_t)blockIdx.y * hist_stride;
  cand += (size_t)blockIdx.y * gridDim.x;
  out += blockIdx.y;
  const int32_t f0 = blockIdx.x * group;
  const int32_t nf = (n_features - f0 < group) ? (n_features - f0) : group;
  const int B = n_bins;
  const int Bp = split_padded_bins(B);
  // layout (doubles): pg[group][Bp] | ph[group][Bp] | pn[group][Bp] | parent[group]
  double* pg = reinterpret_cast<double*>(smem);
  double* ph = pg + (size_t)group * Bp;
  double* pn = ph + (size_t)group * Bp;
  double* parent = pn + (size_t)group * Bp;

  // 1. every bin's (gradient, hessian, count) as doubles (all exact), zeros in the padding
  for (int e = tid; e < nf * Bp; e += kSplitThreads) {
    const int fl = e / Bp;
    const int b = e - fl * Bp;
    gbdt_bin_t v = {0.0f, 0.0f, 0u};
    if (b < B) v = hist[(size_t)(f0 + fl) * B + b];
    pg[e] = (double)v.grad;
    ph[e] = (double)v.hess;
    pn[e] = (double)v.count;
  }
  __syncthreads();

  // 2. running sums in place, strictly left to right, one lane per (statistic, feature).
  // The loop is bound by LDS latency: the next 8 values are requested before the current
  // 8 are added and written back.
  if (tid < 3 * nf) {
    const int st = tid / nf;
    const int fl = tid - st * nf;
    double* p = pg + ((size_t)st * group + fl) * Bp;
    double cur[8], nxt[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) cur[i] = p[i];
    double acc = 0.0;
    for (int b0 = 0; b0 < Bp; b0 += 8) {
      if (b0 + 8 < Bp) {
#pragma unroll
        for (int i = 0; i < 8; ++i) nxt[i] = p[b0 + 8 + i];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        acc = acc + cur[i];
        p[b0 + i] = acc;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) cur[i] = nxt[i];
    }
  }
  __syncthreads();
  if (tid < nf) {
    const double G = pg[tid * Bp + B - 1], H = ph[tid * Bp + B - 1];
    parent[tid] = __ddiv_rn(__dmul_rn(G, G), H + lambda);
  }
  __syncthreads();

  double best_gain = 0.0;
  int32_t best_pair = -1;  // fl * (B - 1) + t, ascending in (feature, bin)
  const int n_pairs = nf * (B - 1);
  for (int e = tid; e < n_pairs; e += kSplitThreads) {
    const int fl = e / (B - 1);
    const int t = e - fl * (B - 1);
    const double GL = pg[fl * Bp + t], HL = ph[fl * Bp + t], NL = pn[fl * Bp + t];
    const double GR = pg[fl * Bp + B - 1] - GL, HR = ph[fl * Bp + B - 1] - HL;
    const double NR = pn[fl * Bp + B - 1] - NL;  // counts are exact in fp64
    const bool ok = NL >= 1.0 && NR >= 1.0 && HL >= min_child_hess && HR >= min_child_hess;
    if (ok) {
      const double lt = __ddiv_rn(__dmul_rn(GL, GL), HL + lambda);
      const double rt = __ddiv_rn(__dmul_rn(GR, GR), HR + lambda);
      const double gain = __dsub_rn(__dadd_rn(lt, rt), parent[fl]);
      if (best_pair < 0 || gain > best_gain) {  // e ascends: ties keep the earlier pair
        best_gain = gain;
        best_pair = e;
      }
    }
  }
  s_gain[tid] = best_gain;
  s_pair[tid] = best_pair;
  __syncthreads();
  for (int s = kSplitThreads / 2; s > 0; s >>= 1) {
    if (tid < s) {
      const double g2 = s_gain[tid + s];
      const int32_t p2 = s_pair[tid + s];
      const double g1 = s_gain[tid];
      const int32_t p1 = s_pair[tid];
      const bool take = p2 >= 0 && (p1 < 0 || g2 > g1 || (g2 == g1 && p2 < p1));
      if (take) {
        s_gain[tid] = g2;
        s_pair[tid] = p2;
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    SplitCand c;
    const int32_t e = s_pair[0];
    if (e < 0) {
      c.gain = 0.0;
      c.gl = c.hl = c.gr = c.hr = 0.0;
      c.nl = c.nr = 0;
      c.feature = -1;
      c.bin = -1;
    } else {
      const int fl = e / (B - 1);
      const int t = e - fl * (B - 1);
      c.gain = s_gain[0];
      c.gl = pg[fl * Bp + t];
      c.hl = ph[fl * Bp + t];
      c.nl = (uint32_t)pn[fl * Bp + t];
      c.gr = pg[fl * Bp + B - 1] - c.gl;
      c.hr = ph[fl * Bp + B - 1] - c.hl;
      c.nr = (uint32_t)(pn[fl * Bp + B - 1] - pn[fl * Bp + t]);
      c.feature = f0 + fl;
      c.bin = t;
    }
    store_cand(cand + blockIdx.x, c);
    // The candidate's stores are device-scope atomics (written through, not left dirty in
    // this XCD's L2): once they are acknowledged they are visible device-wide, so waiting
    // for them (vmcnt(0)) is all the release the ticket needs -- a full fence would also
    // write back every dirty line of the L2, which costs tens of microseconds here.
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0); expcnt, lgkmcnt untouched
    const unsigned int old = __hip_atomic_fetch_add(&g_split_ticket[blockIdx.y], 1u, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
    const bool last = old == gridDim.x - 1;
    if (last)  // back to zero for the next launch
      __hip_atomic_store(&g_split_ticket[blockIdx.y], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = last;
  }
  __syncthreads();
  if (!s_last) return;
  // The ticket's value has arrived, so every other workgroup's candidate was acknowledged
  // before its ticket; the loads below are device-scope atomics and bypass stale caches.

  // ---- the histogram's last workgroup: arg-max over all candidates.  Each thread folds
  // a strided subset in ascending order, then a tree reduction.
  const int32_t n_cand = (int32_t)gridDim.x;
  double bg = 0.0;
  int32_t bi = -1;
  for (int32_t i = tid; i < n_cand; i += kSplitThreads) {
    if (load_cand_feature(cand + i) >= 0) {
      const double g = load_cand_gain(cand + i);
      if (bi < 0 || g > bg) {  // i ascends, so ties keep the smaller feature
        bg = g;
        bi = i;
      }
    }
  }
  s_gain[tid] = bg;
  s_pair[tid] = bi;
  __syncthreads();
  for (int s = kSplitThreads / 2; s > 0; s >>= 1) {
    if (tid < s) {
      const double g2 = s_gain[tid + s];
      const int32_t i2 = s_pair[tid + s];
      const double g1 = s_gain[tid];
      const int32_t i1 = s_pair[tid];
      const bool take = i2 >= 0 && (i1 < 0 || g2 > g1 || (g2 == g1 && i2 < i1));
      if (take) {
        s_gain[tid] = g2;
        s_pair[tid] = i2;
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    gbdt_split_t r;
    const int32_t i = s_pair[0];
    if (i < 0) {
      r.feature = -1;
      r.bin = -1;
      r.gain = 0.0f;
      r.left_grad = r.left_hess = r.right_grad = r.right_hess = 0.0f;
      r.left_count = r.right_count = 0;
    } else {
      const SplitCand c = load_cand(cand + i);
      r.feature = c.feature;
      r.bin = c.bin;
      r.gain = (float)c.gain;
      r.left_grad = (float)c.gl;
      r.left_hess = (float)c.hl;
      r.left_count = c.nl;
      r.right_grad = (float)c.gr;
      r.right_hess = (float)c.hr;
      r.right_count = c.nr;
    }
    *out = r;
  }
}

// ------------------------------------------------------------- partition kernels

// Split() of App. C.1 on the device: the rows of a leaf are handed to its two children
// by the bin of one feature, left rows (bin <= threshold) first, each side in the
// parent's order.  The paper leaves this step on the CPU and copies the new index list to
// the GPU after every split (App. A.5); with the list kept in HBM nothing is copied.
//
// Two passes over chunks of kPartThreads * rows_per_thread consecutive leaf positions,
// one workgroup per chunk, no waiting between workgroups:
//   1. flag pass: fetch each row's bin, ballot "goes left" into one 64-bit word per
//      (wavefront, step) and count the chunk's left rows;
//   2. scatter pass: every workgroup sums the chunk counts before its own (at most
//      kPartMaxChunks of them) to find where its rows start on either side, then ranks
//      its rows inside the chunk from the flag words and writes the row ids.
// The flag words save the second pass the scattered read of the bin matrix, which is
// by far the larger part of the traffic (one 32- or 64-byte tile row per leaf row).
constexpr int kPartThreads = 256;
constexpr int kPartWaves = kPartThreads / 64;
constexpr int kPartMaxChunks = 8192;

struct PartGeom {
  int32_t rows_per_thread;  // steps of kPartThreads rows a workgroup takes
  int32_t n_chunks;
  size_t flag_words;        // 64-bit words
  size_t bytes;             // flags, then one 32-bit count per chunk
};

PartGeom make_part_geom(int64_t n_leaf) {
  PartGeom g;
  g.rows_per_thread = 8;
  while ((n_leaf + (int64_t)kPartThreads * g.rows_per_thread - 1) /
             ((int64_t)kPartThreads * g.rows_per_thread) > kPartMaxChunks)
    g.rows_per_thread *= 2;
  const int64_t chunk_rows = (int64_t)kPartThreads * g.rows_per_thread;
  g.n_chunks = (int32_t)((n_leaf + chunk_rows - 1) / chunk_rows);
  g.flag_words = (size_t)g.n_chunks * g.rows_per_thread * kPartWaves;
  g.bytes = g.flag_words * 8 + (size_t)g.n_chunks * 4;
  return g;
}

// Where the bin of the split feature sits in a row of the packed matrix, and the test
// "this leaf position goes left".
struct SplitColumn {
  bool has_split;    // false: the record holds no split, every row goes left
  int64_t tile_off;  // byte offset of the feature's tile
  int32_t w, col;    // tile width; byte of the tile row
  int32_t shift;     // 4-bit bins: the nibble
  uint32_t mask;
  int32_t thr;
};

__device__ __forceinline__ SplitColumn split_column(const gbdt_split_t* __restrict__ split,
                                                    const TilePlan& plan, int64_t n_rows,
                                                    int32_t n_features) {
  SplitColumn c;
  const int32_t f = split->feature;
  c.thr = split->bin;
  c.has_split = f >= 0 && f < n_features;
  c.tile_off = 0;
  c.w = plan.wm;
  c.col = 0;
  c.shift = 0;
  c.mask = 0xffu;
  if (c.has_split) {
    const int32_t fb = plan.nib ? (f >> 1) : f;
    int32_t t = fb / plan.wm;
    if (t > plan.n_main) t = plan.n_main;
    c.w = plan_tile_width(plan, t);
    c.col = fb - t * plan.wm;
    c.tile_off = n_rows * ((int64_t)t * plan.wm);
    if (plan.nib) {
      c.shift = (f & 1) ? 4 : 0;
      c.mask = 15u;
    }
  }
  return c;
}

__device__ __forceinline__ bool goes_left(const SplitColumn& c, const uint8_t* __restrict__ packed,
                                          int64_t n_rows, const int32_t* __restrict__ idx, int64_t e,
                                          int64_t n_leaf) {
  if (e >= n_leaf) return false;
  if (!c.has_split) return true;
  int64_t r = idx ? (int64_t)idx[e] : e;
  r = r < 0 ? 0 : (r >= n_rows ? n_rows - 1 : r);  // a bad row id must not fault
  const uint32_t b = ((uint32_t)packed[c.tile_off + r * c.w + c.col] >> c.shift) & c.mask;
  return (int32_t)b <= c.thr;
}

__global__ void __launch_bounds__(kPartThreads)
partition_flag_kernel(const uint8_t* __restrict__ packed, int64_t n_rows, int32_t n_features,
                      TilePlan plan, const int32_t* __restrict__ idx, int64_t n_leaf,
                      const gbdt_split_t* __restrict__ split, int32_t rows_per_thread,
                      uint64_t* __restrict__ flags, uint32_t* __restrict__ chunk_left) {
  __shared__ uint32_t s_left[kPartWaves];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const SplitColumn sc = split_column(split, plan, n_rows, n_features);
  const int64_t chunk_base = (int64_t)blockIdx.x * kPartThreads * rows_per_thread;
  uint64_t* my_flags = flags + (size_t)blockIdx.x * rows_per_thread * kPartWaves;
  uint32_t wave_left = 0;
  for (int32_t k = 0; k < rows_per_thread; ++k) {
    const int64_t e = chunk_base + (int64_t)k * kPartThreads + tid;
    const uint64_t m = __ballot(goes_left(sc, packed, n_rows, idx, e, n_leaf));
    if (lane == 0) my_flags[k * kPartWaves + wave] = m;
    wave_left += (uint32_t)__popcll(m);
  }
  if (lane == 0) s_left[wave] = wave_left;
  __syncthreads();
  if (tid == 0) {
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < kPartWaves; ++i) c += s_left[i];
    chunk_left[blockIdx.x] = c;
  }
}

__global__ void __launch_bounds__(kPartThreads)
partition_scatter_kernel(const int32_t* __restrict__ idx, int64_t n_leaf, int32_t rows_per_thread,
                         const uint64_t* __restrict__ flags, const uint32_t* __restrict__ chunk_left,
                         int32_t n_chunks, int32_t* __restrict__ out, int64_t* __restrict__ n_left_out) {
  __shared__ int64_t s_before[kPartWaves], s_total[kPartWaves];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t chunk = blockIdx.x;
  // left rows in the chunks before this one, and in the whole leaf
  int64_t before = 0, total = 0;
  for (int32_t c = tid; c < n_chunks; c += kPartThreads) {
    const int64_t v = chunk_left[c];
    total += v;
    if (c < chunk) before += v;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    before += __shfl_xor(before, o);
    total += __shfl_xor(total, o);
  }
  if (lane == 0) {
    s_before[wave] = before;
    s_total[wave] = total;
  }
  __syncthreads();
  before = 0;
  total = 0;
#pragma unroll
  for (int i = 0; i < kPartWaves; ++i) {
    before += s_before[i];
    total += s_total[i];
  }
  if (chunk == 0 && tid == 0 && n_left_out) *n_left_out = total;

  const int64_t chunk_base = (int64_t)chunk * kPartThreads * rows_per_thread;
  const uint64_t* my_flags = flags + (size_t)chunk * rows_per_thread * kPartWaves;
  const uint64_t below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  int64_t left_pos = before;  // left rows before the current step
  for (int32_t k = 0; k < rows_per_thread; ++k) {
    uint64_t m = 0;
    int64_t wave_base = left_pos;
#pragma unroll
    for (int i = 0; i < kPartWaves; ++i) {
      const uint64_t mi = my_flags[k * kPartWaves + i];
      const int64_t ci = __popcll(mi);
      if (i < wave) wave_base += ci;
      if (i == wave) m = mi;
      left_pos += ci;
    }
    const int64_t e = chunk_base + (int64_t)k * kPartThreads + tid;
    if (e < n_leaf) {
      const int32_t r = idx ? idx[e] : (int32_t)e;
      const int64_t lefts_before_e = wave_base + __popcll(m & below);
      const bool left = (m >> lane) & 1ull;
      out[left ? lefts_before_e : total + (e - lefts_before_e)] = r;
    }
  }
}

// A leaf of at most kPartThreads * kPartOneSteps rows: both passes in one workgroup, the
// flag words in local memory, one launch.
constexpr int kPartOneSteps = 32;

__global__ void __launch_bounds__(kPartThreads)
partition_one_kernel(const uint8_t* __restrict__ packed, int64_t n_rows, int32_t n_features,
                     TilePlan plan, const int32_t* __restrict__ idx, int32_t n_leaf,
                     const gbdt_split_t* __restrict__ split, int32_t* __restrict__ out,
                     int64_t* __restrict__ n_left_out) {
  __shared__ uint64_t s_flags[kPartOneSteps * kPartWaves];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const SplitColumn sc = split_column(split, plan, n_rows, n_features);
  const int32_t steps = (n_leaf + kPartThreads - 1) / kPartThreads;
  for (int32_t k = 0; k < steps; ++k) {
    const uint64_t m = __ballot(goes_left(sc, packed, n_rows, idx, (int64_t)k * kPartThreads + tid, n_leaf));
    if (lane == 0) s_flags[k * kPartWaves + wave] = m;
  }
  __syncthreads();
  int32_t total = 0;
  for (int32_t i = 0; i < steps * kPartWaves; ++i) total += __popcll(s_flags[i]);
  if (tid == 0 && n_left_out) *n_left_out = total;
  const uint64_t below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  int32_t left_pos = 0;  // left rows before the current step
  for (int32_t k = 0; k < steps; ++k) {
    uint64_t m = 0;
    int32_t wave_base = left_pos;
#pragma unroll
    for (int i = 0; i < kPartWaves; ++i) {
      const uint64_t mi = s_flags[k * kPartWaves + i];
      const int32_t ci = __popcll(mi);
      if (i < wave) wave_base += ci;
      if (i == wave) m = mi;
      left_pos += ci;
    }
    const int32_t e = k * kPartThreads + tid;
    if (e < n_leaf) {
      const int32_t r = idx ? idx[e] : e;
      const int32_t lefts_before_e = wave_base + __popcll(m & below);
      const bool left = (m >> lane) & 1ull;
      out[left ? lefts_before_e : total + (e - lefts_before_e)] = r;
    }
  }
}

// out[i] = i: the row list of the root, for a tree that never splits.
__global__ void __launch_bounds__(256) row_iota_kernel(int32_t* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = (int32_t)i;
}

// The leaves of a grown tree tile the positions 0..n-1 with segments, each held by one of
// two row buffers.  out[i] = (buffer of i's segment)[i] for the positions of up to
// kSegTable consecutive segments, whose starts (ascending; bit 31 = buffer) travel as
// kernel arguments.
constexpr int kSegTable = 960;
struct SegTable {
  uint32_t start[kSegTable];
  uint32_t end;     // one past the last position of the last segment
  int32_t n_seg;
};

__global__ void __launch_bounds__(256)
leaf_rows_gather_kernel(const int32_t* __restrict__ buf0, const int32_t* __restrict__ buf1, SegTable t,
                        int32_t* __restrict__ out) {
  const uint32_t first = t.start[0] & 0x7fffffffu;
  const uint32_t i = first + blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= t.end) return;
  int32_t lo = 0, hi = t.n_seg - 1;  // last segment that starts at or before i
  while (lo < hi) {
    const int32_t mid = (lo + hi + 1) >> 1;
    if ((t.start[mid] & 0x7fffffffu) <= i) {
      lo = mid;
    } else {
      hi = mid - 1;
    }
  }
  out[i] = (t.start[lo] >> 31) ? buf1[i] : buf0[i];
}

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

struct Workspace {
  std::mutex mu;
  void* own = nullptr;  // library-owned scratch
  size_t own_bytes = 0;
  int own_device = -1;
  void* user = nullptr;  // caller-registered scratch
  size_t user_bytes = 0;
};
Workspace g_ws;

// Returns a scratch pointer of at least `bytes`, growing the library-owned buffer
// when no caller buffer is registered.
int get_workspace(size_t bytes, void** out) {
  std::lock_guard<std::mutex> lk(g_ws.mu);
  if (g_ws.user) {
    if (bytes > g_ws.user_bytes) return GBDT_ENOMEM;
    *out = g_ws.user;
    return GBDT_OK;
  }
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (g_ws.own && (g_ws.own_device != dev || g_ws.own_bytes < bytes)) {
    HIP_TRY(hipDeviceSynchronize());  // earlier work may still use the old buffer
    HIP_TRY(hipFree(g_ws.own));
    g_ws.own = nullptr;
    g_ws.own_bytes = 0;
  }
  if (!g_ws.own) {
    size_t want = bytes < (size_t)(1 << 20) ? (size_t)(1 << 20) : bytes;
    hipError_t e = hipMalloc(&g_ws.own, want);
    if (e != hipSuccess) {
      g_ws.own = nullptr;
      hip_fail(e, "hipMalloc(workspace)");
      return GBDT_ENOMEM;
    }
    g_ws.own_bytes = want;
    g_ws.own_device = dev;
  }
  *out = g_ws.own;
  return GBDT_OK;
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
// Bytes behind the last tile that the build kernel may read (and ignore): its last
// epoch of a root leaf fetches whole row groups, up to one epoch of rows of the widest
// tile past the end.
constexpr size_t kPackSlackBytes = (size_t)kEpochRows * 64;
constexpr int kBuildThreads = 512;  // threads per workgroup of every build kernel variant

struct BuildGeom {
  TilePlan plan;
  int nt;               // threads per workgroup
  size_t lds_bytes;     // LDS per workgroup
  int wgs;              // workgroups per tile
  int unit_epochs;      // epochs per unit
  bool one_unit_each;   // short leaf: every workgroup has exactly one unit, no counter
  size_t partial_words;  // total words of all partial blocks
  size_t counter_words;  // one unit counter per tile
};

// Leaves of at most this many epochs get ONE workgroup per tile, which writes the
// finished histogram itself: a second launch (the reduction pass) would cost more than
// the few epochs a second workgroup could take over.
constexpr int kDirectEpochs = 4;

// Workgroups per tile and epochs per unit for a leaf of n_epochs epochs that may use
// `budget` workgroups per tile: units of kUnitEpochs when every workgroup gets at least
// one of them; otherwise (short leaf) one shorter unit per workgroup, and the unit
// counter is not needed (*one_unit_each_out).
void plan_leaf_units(int64_t n_epochs, int64_t budget, int* wgs_out, int* unit_epochs_out,
                     bool* one_unit_each_out) {
  int64_t wgs = budget;
  if (wgs > n_epochs) wgs = n_epochs;
  if (n_epochs <= kDirectEpochs) wgs = 1;
  if (wgs < 1) wgs = 1;
  int unit_epochs = kUnitEpochs;
  bool one_each = false;
  if (wgs * kUnitEpochs >= n_epochs) {
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
                    int wg_per_cu_hint) {
  BuildGeom g;
  g.plan = make_tile_plan(n_features, n_bins);
  const TilePlan& p = g.plan;
  g.nt = kBuildThreads;
  const size_t main_block = (size_t)3 * plan_cells(p, p.wm);
  g.lds_bytes = (size_t)plan_cells(p, p.wm) * 8 + 4 * (g.nt / 64) * sizeof(float) + 8;
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
  plan_leaf_units(n_epochs, resident / n_tiles, &g.wgs, &g.unit_epochs, &g.one_unit_each);
  g.partial_words = (size_t)p.n_main * g.wgs * main_block +
                    (size_t)(p.wr ? g.wgs : 0) * 3 * (p.wr ? plan_cells(p, p.wr) : 0);
  g.counter_words = (size_t)n_tiles;
  return g;
}

// Kernel variants: bin capacity -> (main tile width, 4-bit, waves per SIMD the
// register budget is set for).
#define GBDT_VARIANT_16 16, 64, true, kBuildThreads, 8, double
#define GBDT_VARIANT_64 64, 64, false, kBuildThreads, 6, float
#define GBDT_VARIANT_256 256, 32, false, kBuildThreads, 4, float

template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC, bool INDEXED>
int query_occupancy() {
  int n = 0;
  hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(
      &n, reinterpret_cast<const void*>(hist_build_kernel<CAP, WM, NIB, NT, WPE, ACC, INDEXED>), NT, 0);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return n;
}

// Resident workgroups per CU of the build kernel variant for this bin capacity
// (registers, LDS and wave slots taken into account by the runtime); cached.
int build_wg_per_cu(int cap, bool indexed) {
  // GBDT_HIST_WG_PER_CU overrides the runtime's answer (tuning experiments only)
  if (const char* e = getenv("GBDT_HIST_WG_PER_CU")) {
    const int v = atoi(e);
    if (v > 0) return v;
  }
  static int cache[3][2] = {{-1, -1}, {-1, -1}, {-1, -1}};
  const int ci = cap == 16 ? 0 : (cap == 64 ? 1 : 2);
  int& c = cache[ci][indexed ? 1 : 0];
  if (c < 0) {
    if (cap == 16) c = indexed ? query_occupancy<GBDT_VARIANT_16, true>() : query_occupancy<GBDT_VARIANT_16, false>();
    else if (cap == 64) c = indexed ? query_occupancy<GBDT_VARIANT_64, true>() : query_occupancy<GBDT_VARIANT_64, false>();
    else c = indexed ? query_occupancy<GBDT_VARIANT_256, true>() : query_occupancy<GBDT_VARIANT_256, false>();
  }
  return c;
}

// Features per workgroup of split_gain_kernel: as many as fit its LDS budget, at most
// 32, but fewer when that leaves the machine short of workgroups.
void split_grouping(int32_t n_features, int32_t n_bins, int* group_out, int* n_groups_out) {
  int group = kSplitLdsBudget / split_feature_bytes(n_bins);
  if (group > 32) group = 32;
  const int spread = (n_features + 255) / 256;  // features per group that gives ~256 groups
  if (spread < group) group = spread;
  if (group < 1) group = 1;
  *group_out = group;
  *n_groups_out = (n_features + group - 1) / group;
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

template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC>
int launch_build(const BuildArgs& a, int blocks, hipStream_t s) {
  BuildTimer timer;
  int rc = timer.begin(s);
  if (rc != GBDT_OK) return rc;
  if (a.idx) {
    hipLaunchKernelGGL((hist_build_kernel<CAP, WM, NIB, NT, WPE, ACC, true>), dim3(blocks), dim3(NT), 0, s, a);
  } else {
    hipLaunchKernelGGL((hist_build_kernel<CAP, WM, NIB, NT, WPE, ACC, false>), dim3(blocks), dim3(NT), 0, s, a);
  }
  HIP_TRY(hipGetLastError());
  return timer.end(s);
}

template <int CAP, int WM, bool NIB, int NT, int WPE, typename ACC>
int launch_build_batch(const BatchArgs& a, int blocks, hipStream_t s) {
  BuildTimer timer;
  int rc = timer.begin(s);
  if (rc != GBDT_OK) return rc;
  hipLaunchKernelGGL((hist_build_batch_kernel<CAP, WM, NIB, NT, WPE, ACC>), dim3(blocks), dim3(NT), 0, s, a);
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
                 hipStream_t s) {
  int group = 0, n_groups = 0;
  split_grouping(n_features, n_bins, &group, &n_groups);
  void* ws = nullptr;
  int rc = get_workspace((size_t)n_hists * n_groups * sizeof(SplitCand), &ws);
  if (rc != GBDT_OK) return rc;
  const size_t lds = (size_t)group * split_feature_bytes(n_bins);
  hipLaunchKernelGGL(split_gain_kernel, dim3(n_groups, n_hists), dim3(kSplitThreads), lds, s, hists,
                     hist_stride, n_features, n_bins, group, (double)lambda, (double)min_child_hess,
                     (SplitCand*)ws, splits_out);
  HIP_TRY(hipGetLastError());
  return GBDT_OK;
}

// Scratch of gbdt_grow_tree.
size_t align256(size_t b) { return (b + 255) / 256 * 256; }

struct TreeScratch {
  size_t rows_a, rows_b, hists, recs, total;  // byte offsets
};

TreeScratch tree_scratch_layout(int64_t n_rows, int32_t n_features, int32_t n_bins, int32_t max_leaves) {
  TreeScratch t;
  const size_t rows = align256((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(int32_t));
  t.rows_a = 0;
  t.rows_b = rows;
  t.hists = 2 * rows;
  t.recs = t.hists + align256((size_t)max_leaves * n_features * n_bins * sizeof(gbdt_bin_t));
  t.total = t.recs + align256((size_t)2 * max_leaves * sizeof(gbdt_split_t));
  return t;
}

// Two split records in page-locked host memory, the landing place of the per-split
// device-to-host copy (one per process, never freed).
gbdt_split_t* pinned_records() {
  static gbdt_split_t* p = nullptr;
  static std::mutex mu;
  std::lock_guard<std::mutex> lk(mu);
  if (!p) {
    void* q = nullptr;
    if (hipHostMalloc(&q, 2 * sizeof(gbdt_split_t), hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    p = (gbdt_split_t*)q;
  }
  return p;
}


}  // namespace

// ----------------------------------------------------------------------- C ABI

extern "C" {

size_t gbdt_bins_packed_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins) {
  if (!valid_shape(n_rows, n_features, n_bins)) return 0;
  const TilePlan p = make_tile_plan(n_features, n_bins);
  return (size_t)n_rows * (size_t)p.row_bytes + kPackSlackBytes;
}

int gbdt_bins_pack(const uint8_t* bins_rowmajor, int64_t n_rows, int32_t n_features,
                   int32_t n_bins, void* packed_out, void* stream) {
  if (!valid_shape(n_rows, n_features, n_bins)) return GBDT_EINVAL;
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
  return GBDT_OK;
}

size_t gbdt_workspace_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins) {
  if (!valid_shape(n_rows, n_features, n_bins)) return 0;
  const int cap = make_tile_plan(n_features, n_bins).cap;
  const BuildGeom g0 = make_geom(n_features, n_bins, n_rows, device_cu_count(), build_wg_per_cu(cap, false));
  const BuildGeom g1 = make_geom(n_features, n_bins, n_rows, device_cu_count(), build_wg_per_cu(cap, true));
  size_t b = (g0.partial_words > g1.partial_words ? g0.partial_words : g1.partial_words) * 4 +
             g0.counter_words * 4;
  int sg = 0, sn = 0;
  split_grouping(n_features, n_bins, &sg, &sn);
  const size_t cand = (size_t)2 * sn * sizeof(SplitCand);  // gbdt_grow_tree searches two histograms at once
  if (cand > b) b = cand;
  const size_t part = make_part_geom(n_rows > 0 ? n_rows : 1).bytes;
  if (part > b) b = part;
  return (b + 255) / 256 * 256;
}

int gbdt_set_workspace(void* dev_ptr, size_t bytes) {
  if ((dev_ptr == nullptr) != (bytes == 0)) return GBDT_EINVAL;
  if (((uintptr_t)dev_ptr & 255u) != 0) return GBDT_EINVAL;
  std::lock_guard<std::mutex> lk(g_ws.mu);
  g_ws.user = dev_ptr;
  g_ws.user_bytes = bytes;
  return GBDT_OK;
}

int gbdt_hist_build(const void* bin_matrix, int64_t n_rows, int32_t n_features, int32_t n_bins,
                    const int32_t* leaf_row_idx, int64_t n_leaf_rows, const float* grad,
                    const float* hess, gbdt_bin_t* hist_out, void* stream) {
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

  const BuildGeom g =
      make_geom(n_features, n_bins, n_leaf_rows, device_cu_count(),
                build_wg_per_cu(make_tile_plan(n_features, n_bins).cap, leaf_row_idx != nullptr));
  const TilePlan& p = g.plan;
  if (plan_n_tiles(p) > 65535) return GBDT_EUNSUPPORTED;
  // byte offsets inside a tile (slack included) are formed in 32 bits
  if ((n_rows + kEpochRows) * (int64_t)p.wm >= ((int64_t)1 << 32)) return GBDT_EUNSUPPORTED;
  void* ws = nullptr;
  int rc = get_workspace((g.partial_words + g.counter_words) * 4, &ws);
  if (rc != GBDT_OK) return rc;

  BuildArgs a;
  a.packed = (const uint8_t*)bin_matrix;
  a.idx = leaf_row_idx;
  a.grad = grad;
  a.hess = hess;
  a.partials = (uint32_t*)ws;
  a.counters = (uint32_t*)ws + g.partial_words;
  a.n_rows = n_rows;
  a.n_leaf = n_leaf_rows;
  a.n_main = p.n_main;
  a.wr = p.wr;
  a.wgs = g.wgs;
  a.unit_epochs = g.unit_epochs;
  // no counter when every workgroup has one unit anyway, or when the split must be fixed
  a.fixed_stride = (g.one_unit_each || g_deterministic.load()) ? g.wgs : 0;
  a.direct_out = g.wgs == 1 ? hist_out : nullptr;
  a.n_features = n_features;
  a.n_bins = n_bins;
  const int n_tiles = plan_n_tiles(p);
  const int blocks = n_tiles * g.wgs;
  if (a.fixed_stride == 0) {
    const int n_counters = (int)g.counter_words;
    hipLaunchKernelGGL(counters_init_kernel, dim3((n_counters + 255) / 256), dim3(256), 0, s,
                       a.counters, g.wgs, n_counters);
    HIP_TRY(hipGetLastError());
  }

  if (p.cap == 16) {
    rc = launch_build<GBDT_VARIANT_16>(a, blocks, s);
  } else if (p.cap == 64) {
    rc = launch_build<GBDT_VARIANT_64>(a, blocks, s);
  } else {
    rc = launch_build<GBDT_VARIANT_256>(a, blocks, s);
  }
  if (rc != GBDT_OK) return rc;
  if (a.direct_out) return GBDT_OK;  // one workgroup per tile: the histogram is written

  MergeArgs m;
  m.partials = (const uint32_t*)ws;
  m.out = hist_out;
  m.plan = p;
  m.n_features = n_features;
  m.n_bins = n_bins;
  m.chunks_main = g.wgs;
  m.chunks_rem = p.wr ? g.wgs : 0;
  const int max_slots = plan_slots(p, p.wm);
  const int mx = (n_bins * max_slots + kMergeCells - 1) / kMergeCells;
  hipLaunchKernelGGL(hist_merge_kernel, dim3(mx, plan_n_tiles(p)), dim3(kMergeCells * kMergeLanes),
                     0, s, m);
  HIP_TRY(hipGetLastError());
  return GBDT_OK;
}

int gbdt_hist_build_batch(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                          int32_t n_bins, const int32_t* row_idx, const int64_t* leaf_offsets,
                          int32_t n_leaves, const float* grad, const float* hess,
                          gbdt_bin_t* hist_out, void* stream) {
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
  const TilePlan p = make_tile_plan(n_features, n_bins);
  const int n_tiles = plan_n_tiles(p);
  if (n_tiles > 65535) return GBDT_EUNSUPPORTED;
  if ((n_rows + kEpochRows) * (int64_t)p.wm >= ((int64_t)1 << 32)) return GBDT_EUNSUPPORTED;
  const int64_t resident = (int64_t)device_cu_count() * build_wg_per_cu(p.cap, true);
  const size_t col = p.cap == 16 ? variant_column_words<GBDT_VARIANT_16>(p)
                                 : (p.cap == 64 ? variant_column_words<GBDT_VARIANT_64>(p)
                                                : variant_column_words<GBDT_VARIANT_256>(p));
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
  void* ws = nullptr;
  int rc = get_workspace(need_words * 4 + 256, &ws);
  if (rc != GBDT_OK) return rc;
  hipStream_t s = (hipStream_t)stream;
  for (int32_t l0 = 0; l0 < n_leaves; l0 += kBatchLeaves) {
    const int32_t n = n_leaves - l0 < kBatchLeaves ? n_leaves - l0 : kBatchLeaves;
    const BatchPlan b = plan_batch(leaf_offsets, l0, n, resident, n_tiles);
    BatchMergeArgs m;
    m.m.partials = (const uint32_t*)ws;
    m.m.out = hist_out + (size_t)l0 * n_features * n_bins;
    m.m.plan = p;
    m.m.n_features = n_features;
    m.m.n_bins = n_bins;
    m.m.chunks_main = 0;
    m.m.chunks_rem = 0;
    m.column_words = col;
    memcpy(m.leaf, b.leaf, sizeof m.leaf);
    if (b.total_wgs > 0) {
      BatchArgs a;
      a.packed = (const uint8_t*)bin_matrix;
      a.idx = row_idx + leaf_offsets[l0];
      a.grad = grad;
      a.hess = hess;
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
      if (p.cap == 16) {
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
    hipLaunchKernelGGL(hist_merge_batch_kernel, dim3(mx, n_tiles, n), dim3(kMergeCells * kMergeLanes), 0,
                       s, m);
    HIP_TRY(hipGetLastError());
  }
  return GBDT_OK;
}

size_t gbdt_hist_build_batch_workspace_bytes(int32_t n_features, int32_t n_bins, int32_t n_leaves) {
  if (n_features <= 0 || n_bins < 2 || n_bins > 256 || n_leaves < 0) return 0;
  const TilePlan p = make_tile_plan(n_features, n_bins);
  const int n_tiles = plan_n_tiles(p);
  const int64_t resident = (int64_t)device_cu_count() * build_wg_per_cu(p.cap, true);
  const size_t col = p.cap == 16 ? variant_column_words<GBDT_VARIANT_16>(p)
                                 : (p.cap == 64 ? variant_column_words<GBDT_VARIANT_64>(p)
                                                : variant_column_words<GBDT_VARIANT_256>(p));
  // every leaf of a launch gets its share of the resident workgroups, rounded down, but
  // at least one workgroup per tile
  int64_t budget = resident / n_tiles;
  if (budget < 1) budget = 1;
  const int64_t per_launch = n_leaves < kBatchLeaves ? n_leaves : kBatchLeaves;
  const size_t b = (size_t)(budget + per_launch) * col * 4 + 256;
  return (b + 255) / 256 * 256;
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
  int rc = get_workspace(g.bytes, &ws);
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
  gbdt_split_t* pinned = pinned_records();
  if (!pinned) return GBDT_ENOMEM;
  hipStream_t s = (hipStream_t)stream;
  char* base = (char*)scratch;
  int32_t* rows_buf[2] = {(int32_t*)(base + lay.rows_a), (int32_t*)(base + lay.rows_b)};
  gbdt_bin_t* pool = (gbdt_bin_t*)(base + lay.hists);
  gbdt_split_t* recs = (gbdt_split_t*)(base + lay.recs);
  const size_t hist_elems = (size_t)n_features * n_bins;

  struct Leaf {
    int slot;  // histogram slot in the pool
    int buf;   // row buffer that holds the node's rows; -1: rows 0..n-1, nowhere stored
  };
  std::vector<Leaf> state(2 * (size_t)max_leaves);
  std::vector<gbdt_split_t> host_recs(2 * (size_t)max_leaves);  // every node's record, as read back
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

  // root
  int rc = gbdt_hist_build(bin_matrix, n_rows, n_features, n_bins, nullptr, n_rows, grad, hess, pool, s);
  if (rc != GBDT_OK) return rc;
  rc = gbdt_best_split(pool, lambda, min_child_hess, recs, n_features, n_bins, s);
  if (rc != GBDT_OK) return rc;
  HIP_TRY(hipMemcpyAsync(pinned, recs, sizeof(gbdt_split_t), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  {
    const gbdt_split_t r = pinned[0];
    float sg = r.left_grad + r.right_grad, sh = r.left_hess + r.right_hess;
    if (r.feature < 0 && n_rows > 0) {
      // no split record carries the totals: sum feature 0's bins on the host
      std::vector<gbdt_bin_t> row((size_t)n_bins);
      HIP_TRY(hipMemcpyAsync(row.data(), pool, (size_t)n_bins * sizeof(gbdt_bin_t), hipMemcpyDeviceToHost, s));
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
    state[0] = {0, -1};
    host_recs[0] = r;
  }
  int n_nodes = 1, n_leaves = 1, next_slot = 1;
  while (n_leaves < max_leaves) {
    int k = -1;
    for (int i = 0; i < n_nodes; ++i) {  // ascending id: equal gains go to the older leaf
      const gbdt_tree_node_t& nd = nodes_out[i];
      if (nd.left >= 0 || nd.feature < 0 || !(nd.gain > min_split_gain)) continue;
      if (k < 0 || nd.gain > nodes_out[k].gain) k = i;
    }
    if (k < 0) break;
    gbdt_tree_node_t& par = nodes_out[k];
    const int64_t begin = par.row_begin;
    const int src_buf = state[k].buf;
    const int dst_buf = src_buf == 0 ? 1 : 0;
    const int32_t* src = src_buf < 0 ? nullptr : rows_buf[src_buf] + begin;
    int32_t* dst = rows_buf[dst_buf] + begin;
    rc = gbdt_partition_rows(bin_matrix, n_rows, n_features, n_bins, src, par.count, recs + k, dst,
                             nullptr, s);
    if (rc != GBDT_OK) return rc;
    const gbdt_split_t prec = host_recs[k];  // the same record the device partitions by
    const uint32_t nl = prec.left_count, nr = prec.right_count;
    const int left = n_nodes, right = n_nodes + 1;
    const bool left_small = nl <= nr;
    const int small = left_small ? left : right, large = left_small ? right : left;
    const int64_t small_begin = left_small ? begin : begin + nl;
    const uint32_t small_n = left_small ? nl : nr;
    state[small] = {next_slot++, dst_buf};
    state[large] = {state[k].slot, dst_buf};  // the sibling takes over the parent's histogram slot
    gbdt_bin_t* h_small = pool + (size_t)state[small].slot * hist_elems;
    gbdt_bin_t* h_large = pool + (size_t)state[large].slot * hist_elems;
    rc = gbdt_hist_build(bin_matrix, n_rows, n_features, n_bins, rows_buf[dst_buf] + small_begin, small_n,
                         grad, hess, h_small, s);
    if (rc != GBDT_OK) return rc;
    rc = gbdt_hist_subtract(h_large, h_small, h_large, n_features, n_bins, s);
    if (rc != GBDT_OK) return rc;
    // both children in one launch: their histograms sit in two slots of the pool
    rc = launch_split(pool + (size_t)state[left].slot * hist_elems,
                      ((int64_t)state[right].slot - state[left].slot) * (int64_t)hist_elems, 2, lambda,
                      min_child_hess, recs + left, n_features, n_bins, s);
    if (rc != GBDT_OK) return rc;
    HIP_TRY(hipMemcpyAsync(pinned, recs + left, 2 * sizeof(gbdt_split_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    par.left = left;
    par.right = right;
    host_recs[left] = pinned[0];
    host_recs[right] = pinned[1];
    fill_node(left, k, pinned[0], prec.left_grad, prec.left_hess, nl, begin);
    fill_node(right, k, pinned[1], prec.right_grad, prec.right_hess, nr, begin + nl);
    n_nodes += 2;
    n_leaves += 1;
  }
  *n_nodes_out = n_nodes;
  if (row_order_out && n_rows > 0) {
    if (n_nodes == 1) {  // never split: the rows in their own order
      hipLaunchKernelGGL(row_iota_kernel, dim3((unsigned)((n_rows + 255) / 256)), dim3(256), 0, s,
                         row_order_out, n_rows);
      HIP_TRY(hipGetLastError());
    } else {
      // the leaves' segments in position order, a table-full per launch
      std::vector<std::pair<uint32_t, int>> segs;  // (begin, buffer)
      for (int i = 0; i < n_nodes; ++i)
        if (nodes_out[i].left < 0) segs.emplace_back((uint32_t)nodes_out[i].row_begin, state[i].buf);
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
                           (const int32_t*)rows_buf[0], (const int32_t*)rows_buf[1], t, row_order_out);
        HIP_TRY(hipGetLastError());
      }
    }
  }
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

int gbdt_debug_occupancy(int32_t n_bins, int32_t indexed) {
  if (n_bins < 2 || n_bins > 256) return GBDT_EINVAL;
  return build_wg_per_cu(n_bins <= 16 ? 16 : (n_bins <= 64 ? 64 : 256), indexed != 0);
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
