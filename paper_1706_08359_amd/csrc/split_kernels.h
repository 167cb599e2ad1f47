// Best-split search over bin boundaries (Sec. 3.3).  Included by gbdt_hist.hip only.
#ifndef GBDT_SPLIT_KERNELS_H_
#define GBDT_SPLIT_KERNELS_H_

#include <hip/hip_runtime.h>

#include <stdint.h>
#include <string.h>

#include "../../include/gbdt_hist.h"

namespace {

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
// The counters of neighbouring histograms lie kSplitTicketStride words apart: every workgroup of a
// launch adds to one of them with a device-scope atomic, those are carried out one after the
// other where the word's memory channel is, and with the counters of a launch side by side the
// whole launch queued at one channel (measured: 14 ns per workgroup, 28 us for 8 x 250 of them).
constexpr int kSplitTicketStride = 64;
__device__ __forceinline__ unsigned int* split_ticket(unsigned int y) {
  constexpr unsigned int lines = kSplitMaxHists / kSplitTicketStride;
  return &g_split_ticket[(y % lines) * kSplitTicketStride + y / lines];
}

// Sets every ticket counter back to zero (gbdt_reset: after a launch that did not complete).
__global__ void __launch_bounds__(256) split_tickets_zero_kernel() {
  g_split_ticket[blockIdx.x * 256 + threadIdx.x] = 0u;
}

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
// hessian and count per bin (bins padded to a multiple of kSplitBlock), + the feature's parent term.
constexpr int kSplitBlock = 16;  // bins the prefix loop adds per register block
__host__ __device__ inline int split_padded_bins(int n_bins) { return (n_bins + kSplitBlock - 1) & ~(kSplitBlock - 1); }
__host__ __device__ inline int split_feature_bytes(int n_bins) { return 24 * split_padded_bins(n_bins) + 8; }

// Arg-max over the threads of a workgroup under the order "larger gain, then smaller index"
// (index < 0: no candidate): exchanges inside each wavefront, then the four wavefront
// results through local memory.  The order is total, so the result does not depend on how
// the comparisons are arranged.  Every thread returns with the winner in (gain, idx).
__device__ __forceinline__ void block_argmax(double& gain, int32_t& idx, double* s_gain, int32_t* s_idx) {
  auto better = [](double g2, int32_t i2, double g1, int32_t i1) {
    return i2 >= 0 && (i1 < 0 || g2 > g1 || (g2 == g1 && i2 < i1));
  };
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const double g2 = __shfl_xor(gain, o);
    const int32_t i2 = __shfl_xor(idx, o);
    if (better(g2, i2, gain, idx)) {
      gain = g2;
      idx = i2;
    }
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    s_gain[wave] = gain;
    s_idx[wave] = idx;
  }
  __syncthreads();
  gain = s_gain[0];
  idx = s_idx[0];
#pragma unroll
  for (int w = 1; w < kSplitThreads / 64; ++w) {
    const double g2 = s_gain[w];
    const int32_t i2 = s_idx[w];
    if (better(g2, i2, gain, idx)) {
      gain = g2;
      idx = i2;
    }
  }
  __syncthreads();  // the scratch may be reused
}

// Gain scan of Sec. 3.3.  A workgroup takes `passes` groups of `group` consecutive features, one
// group at a time:
//  1. Their histogram rows are copied into local memory as doubles.
//  2. One lane per (feature, statistic) runs the left-to-right prefix sum of grad, hess
//     or count in fp64, bins ascending (this fixes the rounding order).
//  3. All lanes then evaluate the gain of every (feature, threshold) pair from those
//     prefixes -- the divisions, the expensive part -- and keep the best pair under
//     the order "larger gain, then smaller feature, then smaller bin".
// Feature totals are the prefix at the last bin, right = total - left, a threshold is
// admissible when both sides hold >= 1 sample and >= min_child_hess of hessian.
// and keeps the best pair over its groups in registers.
//  4. The workgroup that finishes last for its histogram (a ticket taken after its own
//     candidate is written and fenced; nobody waits) reduces the candidates of all
//     workgroups to the histogram's split record: workgroups hold ascending feature
//     groups, so "smaller candidate index" is "smaller feature".
// grid.y = histogram of the call; histogram y starts hist_stride bins after histogram
// y - 1 (the stride may be negative: any two histograms of a pool can be searched in
// one launch).  mirror (may be NULL): a second place for the records, page-locked host
// memory that the device can write, so that a caller who must look at them on the host
// needs no copy after the kernel, only to wait for it.
// sib (sib.n may be 0): histograms sib.first .. sib.first + sib.n - 1 of the call are siblings
// by subtraction that do not exist yet: histogram sib.first + j is first formed, element by
// element as hist_subtract_kernel does it, as (pool histogram parent_slot[j]) - (histogram j of
// the call, the built child), written to its place and searched in the same pass: every
// (feature, bin) is read by exactly one workgroup, which also writes the difference.
constexpr int kSplitSiblings = 32;
struct SplitSiblings {
  const gbdt_bin_t* pool;  // histograms of hist_elems bins each
  int32_t first, n;
  int32_t parent_slot[kSplitSiblings];
};

__global__ void __launch_bounds__(kSplitThreads)
split_gain_kernel(gbdt_bin_t* hist, int64_t hist_stride, int32_t n_features,
                  int32_t n_bins, int32_t group, int32_t passes, double lambda, double min_child_hess,
                  SplitCand* __restrict__ cand, gbdt_split_t* __restrict__ out,
                  gbdt_split_t* __restrict__ mirror, SplitSiblings sib) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ double s_gain[kSplitThreads / 64];
  __shared__ int32_t s_pair[kSplitThreads / 64];
  __shared__ int s_last;
  const int tid = threadIdx.x;
  const int32_t sib_j = (int32_t)blockIdx.y - sib.first;
  const bool is_sib = sib_j >= 0 && sib_j < sib.n;
  const gbdt_bin_t* built = hist + (int64_t)(is_sib ? sib_j : 0) * hist_stride;  // the sibling's built twin
  const gbdt_bin_t* sib_parent = is_sib ? sib.pool + (int64_t)sib.parent_slot[sib_j] * hist_stride : nullptr;
  hist += (int64_t)blockIdx.y * hist_stride;
  cand += (size_t)blockIdx.y * gridDim.x;
  out += blockIdx.y;
  const int B = n_bins;
  const int Bp = split_padded_bins(B);
  // layout (doubles): pg[group][Bp] | ph[group][Bp] | pn[group][Bp] | parent[group]
  double* pg = reinterpret_cast<double*>(smem);
  double* ph = pg + (size_t)group * Bp;
  double* pn = ph + (size_t)group * Bp;
  double* parent = pn + (size_t)group * Bp;

  // The workgroup takes `passes` groups of `group` consecutive features one after the other and
  // keeps, per thread, the best pair seen so far with everything the record needs: one
  // candidate and one ticket per workgroup, however many features it looked at.
  const int32_t f_first = (int32_t)blockIdx.x * passes * group;
  double best_gain = 0.0;
  int32_t best_pair = -1;  // (feature - f_first) * (B - 1) + bin, ascending in (feature, bin)
  double best_gl = 0.0, best_hl = 0.0, best_nl = 0.0, best_g = 0.0, best_h = 0.0, best_n = 0.0;
  for (int32_t pass = 0; pass < passes; ++pass) {
    const int32_t f0 = f_first + pass * group;
    if (f0 >= n_features) break;  // (the same for every thread)
    const int32_t nf = (n_features - f0 < group) ? (n_features - f0) : group;
    if (pass > 0) __syncthreads();  // the sums of the group before are no longer needed

    // 1. every bin's (gradient, hessian, count) as doubles (all exact), zeros in the padding
    for (int e = tid; e < nf * Bp; e += kSplitThreads) {
      const int fl = e / Bp;
      const int b = e - fl * Bp;
      gbdt_bin_t v = {0.0f, 0.0f, 0u};
      if (b < B) {
        const size_t at = (size_t)(f0 + fl) * B + b;
        if (is_sib) {
          const gbdt_bin_t pv = sib_parent[at];
          const gbdt_bin_t c = built[at];
          v.grad = pv.grad - c.grad;
          v.hess = pv.hess - c.hess;
          v.count = pv.count - c.count;
          hist[at] = v;
        } else {
          v = hist[at];
        }
      }
      pg[e] = (double)v.grad;
      ph[e] = (double)v.hess;
      pn[e] = (double)v.count;
    }
    __syncthreads();

    // 2. running sums in place, strictly left to right, one lane per (statistic, feature).
    // The chain of dependent fp64 adds is the critical path (about 30 cycles a link).  Two
    // register blocks of kSplitBlock bins are used in turn, without copies: while one is added
    // and written back, the other one's values are on their way from local memory.
    if (tid < 3 * nf) {
      const int st = tid / nf;
      const int fl = tid - st * nf;
      double* p = pg + ((size_t)st * group + fl) * Bp;
      double va[kSplitBlock], vb[kSplitBlock];
#pragma unroll
      for (int i = 0; i < kSplitBlock; ++i) va[i] = p[i];
      double acc = 0.0;
      for (int b0 = 0; b0 < Bp; b0 += 2 * kSplitBlock) {
        const bool has_b = b0 + kSplitBlock < Bp;
        if (has_b) {
#pragma unroll
          for (int i = 0; i < kSplitBlock; ++i) vb[i] = p[b0 + kSplitBlock + i];
        }
#pragma unroll
        for (int i = 0; i < kSplitBlock; ++i) {
          acc = acc + va[i];
          va[i] = acc;
        }
#pragma unroll
        for (int i = 0; i < kSplitBlock; ++i) p[b0 + i] = va[i];
        if (b0 + 2 * kSplitBlock < Bp) {
#pragma unroll
          for (int i = 0; i < kSplitBlock; ++i) va[i] = p[b0 + 2 * kSplitBlock + i];
        }
        if (has_b) {
#pragma unroll
          for (int i = 0; i < kSplitBlock; ++i) {
            acc = acc + vb[i];
            vb[i] = acc;
          }
#pragma unroll
          for (int i = 0; i < kSplitBlock; ++i) p[b0 + kSplitBlock + i] = vb[i];
        }
      }
    }
    __syncthreads();
    if (tid < nf) {
      const double G = pg[tid * Bp + B - 1], H = ph[tid * Bp + B - 1];
      parent[tid] = __ddiv_rn(__dmul_rn(G, G), H + lambda);
    }
    __syncthreads();

    // 3. the gains of this group's (feature, threshold) pairs
    const int n_pairs = nf * (B - 1);
    for (int e = tid; e < n_pairs; e += kSplitThreads) {
      const int fl = e / (B - 1);
      const int t = e - fl * (B - 1);
      const double GL = pg[fl * Bp + t], HL = ph[fl * Bp + t], NL = pn[fl * Bp + t];
      const double G = pg[fl * Bp + B - 1], H = ph[fl * Bp + B - 1], N = pn[fl * Bp + B - 1];
      const double GR = G - GL, HR = H - HL;
      const double NR = N - NL;  // counts are exact in fp64
      const bool ok = NL >= 1.0 && NR >= 1.0 && HL >= min_child_hess && HR >= min_child_hess;
      if (ok) {
        const double lt = __ddiv_rn(__dmul_rn(GL, GL), HL + lambda);
        const double rt = __ddiv_rn(__dmul_rn(GR, GR), HR + lambda);
        const double gain = __dsub_rn(__dadd_rn(lt, rt), parent[fl]);
        if (best_pair < 0 || gain > best_gain) {  // pairs ascend: ties keep the earlier pair
          best_gain = gain;
          best_pair = (f0 - f_first + fl) * (B - 1) + t;
          best_gl = GL;
          best_hl = HL;
          best_nl = NL;
          best_g = G;
          best_h = H;
          best_n = N;
        }
      }
    }
  }
  const int32_t my_pair = best_pair;
  block_argmax(best_gain, best_pair, s_gain, s_pair);
  // the thread that holds the winning pair (thread 0 when there is none) hands the candidate over
  const bool writer = best_pair < 0 ? tid == 0 : my_pair == best_pair;
  if (writer) {
    SplitCand c;
    const int32_t e = best_pair;
    if (e < 0) {
      c.gain = 0.0;
      c.gl = c.hl = c.gr = c.hr = 0.0;
      c.nl = c.nr = 0;
      c.feature = -1;
      c.bin = -1;
    } else {
      const int fl = e / (B - 1);
      const int t = e - fl * (B - 1);
      c.gain = best_gain;
      c.gl = best_gl;
      c.hl = best_hl;
      c.nl = (uint32_t)best_nl;
      c.gr = best_g - best_gl;
      c.hr = best_h - best_hl;
      c.nr = (uint32_t)(best_n - best_nl);
      c.feature = f_first + fl;
      c.bin = t;
    }
    store_cand(cand + blockIdx.x, c);
    // HARDWARE ASSUMPTION (gfx942 / gfx950, not the language's memory model): a device-scope
    // atomic store is written through to the point where the other XCDs' device-scope atomic
    // loads read it, and is acknowledged (vmcnt) only then.  Waiting for the candidate's
    // stores (vmcnt(0)) before taking the ticket is therefore all the release this hand-off
    // needs, and the reader needs no acquire because it reads the candidates with device-scope
    // atomic loads only.  A release / acquire pair in the language's sense would also write back
    // and invalidate every line of the L2, which costs tens of microseconds here -- several
    // times the whole kernel.  tests/test_gpu_robustness.py runs 64 x 250 workgroups of this
    // hand-off 20 times and every split test goes through it; on a part where the assumption
    // did not hold those tests would show stale candidates.
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0); expcnt, lgkmcnt untouched
    unsigned int* ticket = split_ticket(blockIdx.y);
    const unsigned int old = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool last = old == gridDim.x - 1;
    if (last)  // back to zero for the next launch
      __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
  block_argmax(bg, bi, s_gain, s_pair);
  if (tid == 0) {
    gbdt_split_t r;
    const int32_t i = bi;
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
    if (mirror) mirror[blockIdx.y] = r;
  }
}

}  // namespace

#endif  // GBDT_SPLIT_KERNELS_H_
