// Row partition of a leaf after a split (App. C.1, Split()) and the row-list helpers of
// tree growth.  Included by gbdt_hist.hip only.
#ifndef GBDT_PARTITION_KERNELS_H_
#define GBDT_PARTITION_KERNELS_H_

#include <hip/hip_runtime.h>

#include <stdint.h>
#include <string.h>

#include "../../include/gbdt_hist.h"
#include "tile_plan.h"

namespace {

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
// The split feature's bins come from the column-major copy of the matrix (tile_plan.h): one
// byte per leaf row instead of a 32- or 64-byte tile row.  The flag words save the second
// pass even that read.  (Leaves small enough for partition_one_kernel read the tiles instead:
// their tile rows were fetched a moment ago, by the histogram build of the same leaf, and
// are still in cache, while the column bytes would come from HBM.)
constexpr int kPartThreads = 256;
constexpr int kPartWaves = kPartThreads / 64;
// (every workgroup of the scatter pass reads the counts of all chunks of its list: long lists
// get longer chunks rather than more of them)
constexpr int kPartMaxChunks = 2048;

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

// Where the bins of the split feature sit in the packed matrix -- in the column-major copy,
// or in the feature's tile -- and the test "this leaf position goes left".
struct SplitColumn {
  bool has_split;    // false: the record holds no split, every row goes left
  bool from_tiles;
  int64_t col_off;   // byte offset of the feature's column
  int64_t tile_off;  // byte offset of the feature's tile
  int32_t w, col;    // tile width; byte of the tile row
  int32_t shift;     // 4-bit bins: the nibble
  uint32_t mask;
  int32_t thr;
};

__device__ __forceinline__ SplitColumn split_column(const gbdt_split_t* __restrict__ split,
                                                    const TilePlan& plan, int64_t n_rows,
                                                    int32_t n_features, bool from_tiles = false) {
  SplitColumn c;
  const int32_t f = split->feature;
  c.thr = split->bin;
  c.has_split = f >= 0 && f < n_features;
  c.from_tiles = from_tiles;
  c.col_off = 0;
  c.tile_off = 0;
  c.w = plan.wm;
  c.col = 0;
  c.shift = 0;
  c.mask = 0xffu;
  if (c.has_split) {
    c.col_off = plan_columns_base(plan, n_rows) + (int64_t)f * plan_column_stride(n_rows);
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
  if (!c.from_tiles) return (int32_t)packed[c.col_off + r] <= c.thr;
  const uint32_t b = ((uint32_t)packed[c.tile_off + r * c.w + c.col] >> c.shift) & c.mask;
  return (int32_t)b <= c.thr;
}

// Both passes are chains of dependent memory round trips (row id -> bin -> flag word; flag words
// and row id -> store) around a little integer arithmetic per row, and that arithmetic is what
// bounds them once enough requests are in flight (with the stores taken out, the first scatter pass
// of a 10 M-row list ran 10 % faster, no more).  So: a thread takes S = min(rows_per_thread, 16) steps of
// its chunk at a time, all S requests of a kind leaving before the first answer is used, and
// everything per row is 32-bit and relative to the chunk (lists hold fewer than 2^32 positions,
// matrices fewer than 2^30 rows).  (rows_per_thread is 8 or a multiple of 16.)
constexpr int kPartMaxBlock = 16;

// What a workgroup knows about its chunk: positions [base, base + n_valid) of the list.
struct PartChunk {
  int64_t base;
  uint32_t n_valid;  // >= 1
};
__device__ __forceinline__ PartChunk part_chunk(int64_t n_leaf, int32_t chunk, int32_t rows_per_thread) {
  PartChunk c;
  const uint32_t chunk_rows = (uint32_t)kPartThreads * (uint32_t)rows_per_thread;
  c.base = (int64_t)chunk * chunk_rows;
  const int64_t rest = n_leaf - c.base;
  c.n_valid = rest < (int64_t)chunk_rows ? (uint32_t)rest : chunk_rows;
  return c;
}

// Row ids of S steps of a thread, from chunk position p0 on in strides of kPartThreads.
// Positions past the end repeat the last one: a valid address, and the callers mask them.
template <int S>
__device__ __forceinline__ void part_request_rows(const int32_t* __restrict__ idx, const PartChunk& c, uint32_t p0,
                                                  int32_t (&r)[S]) {
  const uint32_t last = c.n_valid - 1;
  if (idx) {
    const int32_t* __restrict__ idx_c = idx + c.base;
#pragma unroll
    for (int j = 0; j < S; ++j) {
      const uint32_t p = p0 + (uint32_t)j * kPartThreads;
      r[j] = idx_c[p < last ? p : last];
    }
  } else {
    const int32_t first_row = (int32_t)c.base;  // the list is 0, 1, 2, ...: fewer than 2^30 of them
#pragma unroll
    for (int j = 0; j < S; ++j) {
      const uint32_t p = p0 + (uint32_t)j * kPartThreads;
      r[j] = first_row + (int32_t)(p < last ? p : last);
    }
  }
}

// Flag pass of one chunk of the list idx[0..n_leaf), n_leaf >= 1.
template <int S>
__device__ __forceinline__ void partition_flag_chunk(const SplitColumn& sc, const uint8_t* __restrict__ packed,
                                                     int64_t n_rows, const int32_t* __restrict__ idx,
                                                     int64_t n_leaf, int32_t chunk, int32_t rows_per_thread,
                                                     uint64_t* __restrict__ my_flags,
                                                     uint32_t* __restrict__ my_chunk_left) {
  __shared__ uint32_t s_left[kPartWaves];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const PartChunk c = part_chunk(n_leaf, chunk, rows_per_thread);
  // the column of the split feature, or (no split: every row goes left) any readable bytes
  const uint8_t* __restrict__ column = packed + sc.col_off;
  const int32_t thr = sc.has_split ? sc.thr : 0x7fffffff;
  const int32_t last_row = (int32_t)(n_rows - 1);
  uint32_t wave_left = 0;
  for (int32_t k0 = 0; k0 < rows_per_thread; k0 += S) {
    const uint32_t p0 = (uint32_t)k0 * kPartThreads + tid;
    int32_t r[S];
    part_request_rows<S>(idx, c, p0, r);
    int32_t b[S];
#pragma unroll
    for (int j = 0; j < S; ++j) {
      const int32_t rr = r[j] < 0 ? 0 : (r[j] > last_row ? last_row : r[j]);  // a bad row id must not fault
      b[j] = (int32_t)column[(uint32_t)rr];
    }
#pragma unroll
    for (int j = 0; j < S; ++j) {
      const uint32_t p = p0 + (uint32_t)j * kPartThreads;
      const uint64_t m = __ballot(p < c.n_valid && b[j] <= thr);
      if (lane == 0) my_flags[(k0 + j) * kPartWaves + wave] = m;
      wave_left += (uint32_t)__popcll(m);
    }
  }
  if (lane == 0) s_left[wave] = wave_left;
  __syncthreads();
  if (tid == 0) {
    uint32_t n = 0;
#pragma unroll
    for (int i = 0; i < kPartWaves; ++i) n += s_left[i];
    *my_chunk_left = n;
  }
}

// Scatter pass of one chunk of a list with n_chunks chunks whose left counts are
// chunk_left[0..n_chunks) and whose flag words start at `flags`.
template <int S>
__device__ __forceinline__ void partition_scatter_chunk(const int32_t* __restrict__ idx, int64_t n_leaf,
                                                        int32_t chunk, int32_t n_chunks,
                                                        int32_t rows_per_thread,
                                                        const uint64_t* __restrict__ flags,
                                                        const uint32_t* __restrict__ chunk_left,
                                                        int32_t* __restrict__ out,
                                                        int64_t* __restrict__ n_left_out) {
  static_assert(S * kPartWaves / 2 <= 64, "one wavefront fetches the flag words of S steps, two per lane");
  __shared__ uint32_t s_before[kPartWaves], s_total[kPartWaves];
  // per (step, wavefront) of the S steps in hand: the flag word, the left rows of these steps
  // before it; and the left rows of all S steps
  __shared__ uint64_t s_flag[S * kPartWaves];
  __shared__ uint32_t s_base[S * kPartWaves];
  __shared__ uint32_t s_steps_left;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const PartChunk c = part_chunk(n_leaf, chunk, rows_per_thread);
  const uint64_t* my_flags = flags + (size_t)chunk * rows_per_thread * kPartWaves;
  const uint32_t below_lo = lane >= 32 ? ~0u : ((1u << lane) - 1u);
  const uint32_t below_hi = lane > 32 ? ((1u << (lane - 32)) - 1u) : 0u;
  const uint32_t own_lo = lane < 32 ? (1u << lane) : 0u, own_hi = lane >= 32 ? (1u << (lane - 32)) : 0u;
  uint32_t before = 0, total = 0;
  // where the chunk's left and right rows start, and its left rows before the current steps
  int32_t* __restrict__ out_left = out;
  int32_t* __restrict__ out_right = out;
  uint32_t left_in_chunk = 0;
  for (int32_t k0 = 0; k0 < rows_per_thread; k0 += S) {
    if (k0 > 0) __syncthreads();  // everybody has read the words of the steps before
    // requests: the row ids of S steps, ...
    const uint32_t p0 = (uint32_t)k0 * kPartThreads + tid;
    int32_t r[S];
    part_request_rows<S>(idx, c, p0, r);
    // ... their flag words (the first wavefront: two per lane, ranked with a scan over the lanes) ...
    if (wave == 0) {
      uint64_t m0 = 0, m1 = 0;
      if (lane < S * kPartWaves / 2) {
        m0 = my_flags[k0 * kPartWaves + 2 * lane];
        m1 = my_flags[k0 * kPartWaves + 2 * lane + 1];
      }
      const uint32_t n0 = (uint32_t)__popcll(m0), n1 = (uint32_t)__popcll(m1);
      uint32_t inc = n0 + n1;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(inc, o);
        if (lane >= (uint32_t)o) inc += up;
      }
      if (lane < S * kPartWaves / 2) {
        const uint32_t ex = inc - n0 - n1;
        s_flag[2 * lane] = m0;
        s_flag[2 * lane + 1] = m1;
        s_base[2 * lane] = ex;
        s_base[2 * lane + 1] = ex + n0;
      }
      if (lane == 63) s_steps_left = inc;
    }
    if (k0 == 0) {
      // ... and the left rows in the chunks before this one, and in the whole list
      for (int32_t i = tid; i < n_chunks; i += kPartThreads) {
        const uint32_t v = chunk_left[i];
        total += v;
        if (i < chunk) before += v;
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
    }
    __syncthreads();
    if (k0 == 0) {
      before = 0;
      total = 0;
#pragma unroll
      for (int i = 0; i < kPartWaves; ++i) {
        before += s_before[i];
        total += s_total[i];
      }
      if (chunk == 0 && tid == 0 && n_left_out) *n_left_out = (int64_t)total;
      out_left = out + before;
      out_right = out + ((int64_t)total + (c.base - (int64_t)before));
    }
#pragma unroll
    for (int j = 0; j < S; ++j) {
      const uint64_t m = s_flag[j * kPartWaves + wave];
      const uint32_t m_lo = (uint32_t)m, m_hi = (uint32_t)(m >> 32);
      // left rows of the chunk before this position
      const uint32_t lefts = left_in_chunk + s_base[j * kPartWaves + wave] + __popc(m_lo & below_lo) +
                             __popc(m_hi & below_hi);
      const uint32_t p = p0 + (uint32_t)j * kPartThreads;
      if (p < c.n_valid) {
        // (ordinary stores: a wavefront's ids go to two runs that end inside cache lines which the
        // next wavefront completes; marked as streaming they took a third longer on an even split)
        if ((m_lo & own_lo) | (m_hi & own_hi)) {
          out_left[lefts] = r[j];
        } else {
          out_right[p - lefts] = r[j];
        }
      }
    }
    left_in_chunk += s_steps_left;
  }
}

// The two passes with the number of steps in flight chosen from rows_per_thread.
#define GBDT_PART_DISPATCH(rows_per_thread, CALL) \
  do {                                            \
    if ((rows_per_thread) == 8) {                 \
      constexpr int S = 8;                        \
      CALL;                                       \
    } else {                                      \
      constexpr int S = kPartMaxBlock;            \
      CALL;                                       \
    }                                             \
  } while (0)

__global__ void __launch_bounds__(kPartThreads)
partition_flag_kernel(const uint8_t* __restrict__ packed, int64_t n_rows, int32_t n_features,
                      TilePlan plan, const int32_t* __restrict__ idx, int64_t n_leaf,
                      const gbdt_split_t* __restrict__ split, int32_t rows_per_thread,
                      uint64_t* __restrict__ flags, uint32_t* __restrict__ chunk_left) {
  const SplitColumn sc = split_column(split, plan, n_rows, n_features);
  GBDT_PART_DISPATCH(rows_per_thread,
                     partition_flag_chunk<S>(sc, packed, n_rows, idx, n_leaf, (int32_t)blockIdx.x, rows_per_thread,
                                             flags + (size_t)blockIdx.x * rows_per_thread * kPartWaves,
                                             chunk_left + blockIdx.x));
}

__global__ void __launch_bounds__(kPartThreads)
partition_scatter_kernel(const int32_t* __restrict__ idx, int64_t n_leaf, int32_t rows_per_thread,
                         const uint64_t* __restrict__ flags, const uint32_t* __restrict__ chunk_left,
                         int32_t n_chunks, int32_t* __restrict__ out, int64_t* __restrict__ n_left_out) {
  GBDT_PART_DISPATCH(rows_per_thread,
                     partition_scatter_chunk<S>(idx, n_leaf, (int32_t)blockIdx.x, n_chunks, rows_per_thread, flags,
                                                chunk_left, out, n_left_out));
}

// Several leaves per launch (a level of a tree): leaf l of the launch owns the row list
// idx[row_off .. row_off + n), chunks first_chunk .. of the
// launch's flag / count arrays, the split record split[split_idx], and writes its children to
// out[out_off .. out_off + n).  The table travels as kernel arguments.
constexpr int kPartBatchLeaves = 192;
struct PartLeaf {
  uint32_t row_off, out_off, n, first_chunk, split_idx;
};
struct PartBatchArgs {
  const uint8_t* packed;
  const int32_t* idx;
  const gbdt_split_t* split;
  int32_t* out;
  int64_t* n_left_out;  // [n_leaves] or NULL
  uint64_t* flags;
  uint32_t* chunk_left;
  int64_t n_rows;
  TilePlan plan;
  int32_t n_features;
  int32_t rows_per_thread;
  int32_t n_leaves;
  uint32_t n_chunks;  // of the whole launch
  PartLeaf leaf[kPartBatchLeaves];
};

// the leaf that owns chunk `b` of the launch (leaves without rows own no chunk)
__device__ __forceinline__ int32_t part_leaf_of(const PartLeaf* leaf, int32_t n_leaves, uint32_t b) {
  int32_t lo = 0, hi = n_leaves - 1;
  while (lo < hi) {
    const int32_t mid = (lo + hi + 1) >> 1;
    if (leaf[mid].first_chunk <= b) {
      lo = mid;
    } else {
      hi = mid - 1;
    }
  }
  return lo;
}

__global__ void __launch_bounds__(kPartThreads) partition_flag_batch_kernel(PartBatchArgs a) {
  const int32_t l = part_leaf_of(a.leaf, a.n_leaves, blockIdx.x);
  const PartLeaf lf = a.leaf[l];
  const SplitColumn sc = split_column(a.split + lf.split_idx, a.plan, a.n_rows, a.n_features);
  GBDT_PART_DISPATCH(a.rows_per_thread,
                     partition_flag_chunk<S>(sc, a.packed, a.n_rows, a.idx + lf.row_off, lf.n,
                                             (int32_t)(blockIdx.x - lf.first_chunk), a.rows_per_thread,
                                             a.flags + (size_t)blockIdx.x * a.rows_per_thread * kPartWaves,
                                             a.chunk_left + blockIdx.x));
}

__global__ void __launch_bounds__(kPartThreads) partition_scatter_batch_kernel(PartBatchArgs a) {
  const int32_t l = part_leaf_of(a.leaf, a.n_leaves, blockIdx.x);
  const PartLeaf lf = a.leaf[l];
  const uint32_t next_first = l + 1 < a.n_leaves ? a.leaf[l + 1].first_chunk : a.n_chunks;
  // (a later leaf without rows shares its first chunk with the next one: this leaf's
  // chunks end where the next leaf WITH rows begins, which is what first_chunk gives)
  GBDT_PART_DISPATCH(a.rows_per_thread,
                     partition_scatter_chunk<S>(a.idx + lf.row_off, lf.n, (int32_t)(blockIdx.x - lf.first_chunk),
                                                (int32_t)(next_first - lf.first_chunk), a.rows_per_thread,
                                                a.flags + (size_t)lf.first_chunk * a.rows_per_thread * kPartWaves,
                                                a.chunk_left + lf.first_chunk, a.out + lf.out_off,
                                                a.n_left_out ? a.n_left_out + l : nullptr));
}

// n_left_out[l] = 0 for the leaves of a batched partition that have no rows (they own no
// chunk, so no workgroup of the scatter pass writes their count).
__global__ void __launch_bounds__(256) partition_empty_counts_kernel(PartBatchArgs a) {
  const int32_t l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l < a.n_leaves && a.leaf[l].n == 0 && a.n_left_out) a.n_left_out[l] = 0;
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
  const SplitColumn sc = split_column(split, plan, n_rows, n_features, /*from_tiles=*/true);
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

// Copies up to kCompactSegs segments of a row buffer back to back into another list:
// segment j = src[src_begin[j] .. src_begin[j] + len_j) goes to dst[dst_begin[j] ..), the
// dst_begin ascending with dst_begin[n_seg] = total.  (The smaller children of a tree
// level, gathered for one batched histogram build.)
constexpr int kCompactSegs = 448;
struct CompactTable {
  uint32_t src_begin[kCompactSegs];
  uint32_t dst_begin[kCompactSegs + 1];
  int32_t n_seg;
};

__global__ void __launch_bounds__(256)
segments_compact_kernel(const int32_t* __restrict__ src, CompactTable t, int32_t* __restrict__ dst) {
  const uint32_t i = t.dst_begin[0] + blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= t.dst_begin[t.n_seg]) return;
  int32_t lo = 0, hi = t.n_seg - 1;  // last segment that starts at or before i
  while (lo < hi) {
    const int32_t mid = (lo + hi + 1) >> 1;
    if (t.dst_begin[mid] <= i) {
      lo = mid;
    } else {
      hi = mid - 1;
    }
  }
  dst[i] = src[t.src_begin[lo] + (i - t.dst_begin[lo])];
}

// Debug aid: counts the entries of a row list that are not row ids of the matrix.
__global__ void __launch_bounds__(256)
row_ids_check_kernel(const int32_t* __restrict__ idx, int64_t n, int64_t n_rows,
                     unsigned long long* __restrict__ n_bad) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  unsigned long long bad = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const int64_t r = idx[i];
    bad += (r < 0 || r >= n_rows) ? 1ull : 0ull;
  }
  if (bad) atomicAdd(n_bad, bad);
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

}  // namespace

#endif  // GBDT_PARTITION_KERNELS_H_
