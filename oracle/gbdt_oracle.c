/*
 * gbdt_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, obviously-correct CPU statement (fp64 sums, 64-bit counts)
 * of what the histogram hot path of "GPU-acceleration for Large-scale Tree
 * Boosting" (arXiv 1706.08359) computes.  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table
 * or helper with the HIP library and reads only the caller's plain row-major
 * uint8 bin matrix, never the device layout.
 *
 * Pins (all in tests/, CPU only): numpy.bincount per feature, the per-feature
 * sum invariant, a closed form for constant hessians, parent = left + right,
 * brute-force enumeration of every (feature, threshold) from raw rows, the
 * square-loss special case of Eq. (4), and a planted split; for the row
 * partition a per-row loop over raw values, the disjoint-ordered-cover
 * invariant and agreement of its child sizes with the counts the split search
 * derived from the histogram.  Nothing here is "parity unpinned".
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC gbdt_oracle.c
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  double grad;    /* o[b][1] of Alg. 1 */
  double hess;    /* o[b][2] */
  uint64_t count; /* o[b][3] */
} oracle_bin_t;

typedef struct {
  int32_t feature; /* -1 when no threshold is admissible */
  int32_t bin;     /* threshold t: left = rows with bin <= t */
  double gain;
  double left_grad, left_hess;
  uint64_t left_count;
  double right_grad, right_hess;
  uint64_t right_count;
} oracle_split_t;

/* Number of threads the feature loop will use (1 without OpenMP). */
int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/*
 * Alg. 1 (Sec. 3.3), run once per feature j: walk the leaf's samples in order,
 * look up the sample's bin of feature j and add its gradient, its hessian and
 * one to that bin.  Statistics are indexed by row id (g_{d_ri} in Alg. 1).
 * Bins are 0-based here (the paper writes 1..k).  leaf_row_idx == NULL means
 * the leaf is rows 0..n_leaf_rows-1.
 * Returns 0, or -1 on a bad argument / out-of-range bin or row id.
 */
int oracle_hist_build(const uint8_t *bins, int64_t n_rows, int32_t n_features,
                      int32_t n_bins, const int32_t *leaf_row_idx,
                      int64_t n_leaf_rows, const float *grad,
                      const float *hess, oracle_bin_t *hist_out) {
  if (!bins || !grad || !hess || !hist_out) return -1;
  if (n_rows < 0 || n_features <= 0 || n_bins < 1 || n_bins > 256) return -1;
  if (n_leaf_rows < 0) return -1;
  if (!leaf_row_idx && n_leaf_rows > n_rows) return -1;
  int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
  for (int32_t j = 0; j < n_features; ++j) {
    oracle_bin_t *o = hist_out + (size_t)j * (size_t)n_bins;
    for (int32_t b = 0; b < n_bins; ++b) {
      o[b].grad = 0.0;
      o[b].hess = 0.0;
      o[b].count = 0;
    }
    for (int64_t i = 0; i < n_leaf_rows; ++i) {
      int64_t d = leaf_row_idx ? (int64_t)leaf_row_idx[i] : i;
      if (d < 0 || d >= n_rows) {
        bad |= 1;
        continue;
      }
      int32_t b = bins[(size_t)d * (size_t)n_features + (size_t)j];
      if (b >= n_bins) {
        bad |= 1;
        continue;
      }
      o[b].grad = o[b].grad + (double)grad[d];
      o[b].hess = o[b].hess + (double)hess[d];
      o[b].count = o[b].count + 1;
    }
  }
  return bad ? -1 : 0;
}

/*
 * Sibling histogram as parent minus the child that was built.  The paper does
 * not describe this step; this is the only definition under which the parent
 * equals the sum of its two children bin by bin (every parent sample falls in
 * exactly one child and, by Alg. 1, in exactly one bin of each feature).
 */
int oracle_hist_subtract(const oracle_bin_t *parent, const oracle_bin_t *child,
                         oracle_bin_t *sibling_out, int32_t n_features,
                         int32_t n_bins) {
  if (!parent || !child || !sibling_out || n_features <= 0 || n_bins < 1)
    return -1;
  size_t n = (size_t)n_features * (size_t)n_bins;
  for (size_t e = 0; e < n; ++e) {
    if (child[e].count > parent[e].count) return -1;
    oracle_bin_t s;
    s.grad = parent[e].grad - child[e].grad;
    s.hess = parent[e].hess - child[e].hess;
    s.count = parent[e].count - child[e].count;
    sibling_out[e] = s;
  }
  return 0;
}

/*
 * Histogram-based split search (Sec. 3.3: the split objective is evaluated
 * only at the k bin boundaries, from the gradient and hessian histograms).
 *
 * For a sample set V with G = sum g, H = sum h, the second-order objective
 * Eq. (9) with a constant leaf value w is minimised at w = -G/(H+lambda) and
 * drops by G^2/(2(H+lambda)); splitting V into L and R therefore gains
 *     G_L^2/(H_L+lambda) + G_R^2/(H_R+lambda) - G^2/(H+lambda)
 * (factor 1/2 dropped).  This is what plugging Eq. (3) into Eq. (2) to get
 * Eq. (4) becomes for the weighted problem; lambda is the L2 term the paper
 * leaves out of its exposition.
 *
 * Threshold t in 0..n_bins-2 sends bins <= t left.  A threshold is admissible
 * when both sides hold at least one sample and at least min_child_hess of
 * hessian.  Among admissible thresholds the largest gain wins; equal gains go
 * to the smaller feature, then the smaller bin.  Per-feature totals are the
 * sums of that feature's own bins; left sums are a running left-to-right
 * prefix; right = total - left.
 */
int oracle_best_split(const oracle_bin_t *hist, int32_t n_features,
                      int32_t n_bins, double lambda, double min_child_hess,
                      oracle_split_t *split_out, double *gain_table) {
  if (!hist || !split_out || n_features <= 0 || n_bins < 1 || lambda < 0.0)
    return -1;
  oracle_split_t best;
  memset(&best, 0, sizeof best);
  best.feature = -1;
  best.bin = -1;
  best.gain = 0.0;
  int have = 0;
  for (int32_t j = 0; j < n_features; ++j) {
    const oracle_bin_t *o = hist + (size_t)j * (size_t)n_bins;
    double G = 0.0, H = 0.0;
    uint64_t N = 0;
    for (int32_t b = 0; b < n_bins; ++b) {
      G = G + o[b].grad;
      H = H + o[b].hess;
      N = N + o[b].count;
    }
    double parent_term = (G * G) / (H + lambda);
    double GL = 0.0, HL = 0.0;
    uint64_t NL = 0;
    for (int32_t t = 0; t + 1 < n_bins; ++t) {
      GL = GL + o[t].grad;
      HL = HL + o[t].hess;
      NL = NL + o[t].count;
      double GR = G - GL, HR = H - HL;
      uint64_t NR = N - NL;
      int ok = (NL >= 1) && (NR >= 1) && (HL >= min_child_hess) &&
               (HR >= min_child_hess);
      double gain = 0.0;
      if (ok) {
        double left_term = (GL * GL) / (HL + lambda);
        double right_term = (GR * GR) / (HR + lambda);
        gain = (left_term + right_term) - parent_term;
      }
      if (gain_table) {
        /* NaN marks an inadmissible threshold; t = n_bins-1 is never one. */
        gain_table[(size_t)j * (size_t)n_bins + (size_t)t] =
            ok ? gain : (0.0 / 0.0);
      }
      if (ok && (!have || gain > best.gain)) {
        have = 1;
        best.feature = j;
        best.bin = t;
        best.gain = gain;
        best.left_grad = GL;
        best.left_hess = HL;
        best.left_count = NL;
        best.right_grad = GR;
        best.right_hess = HR;
        best.right_count = NR;
      }
    }
    if (gain_table)
      gain_table[(size_t)j * (size_t)n_bins + (size_t)(n_bins - 1)] =
          (0.0 / 0.0);
  }
  *split_out = best;
  return 0;
}

/*
 * Split() of App. C.1: hand the samples of a node to its two children, given
 * the feature and the threshold bin the split search chose.  A sample goes left
 * when its bin of that feature is <= the threshold (the convention of
 * oracle_best_split) and right otherwise; each child keeps the samples in the
 * order the parent listed them, so sorted index lists stay sorted.  This is the
 * per-leaf index list the CPU maintains and ships after every split in
 * App. A.5.  leaf_row_idx == NULL means the node is rows 0..n_leaf_rows-1.
 * left_out and right_out each have room for n_leaf_rows entries.
 * Returns 0, or -1 on a bad argument or an out-of-range row id.
 */
int oracle_partition_rows(const uint8_t *bins, int64_t n_rows,
                          int32_t n_features, const int32_t *leaf_row_idx,
                          int64_t n_leaf_rows, int32_t feature,
                          int32_t threshold_bin, int32_t *left_out,
                          int64_t *n_left_out, int32_t *right_out,
                          int64_t *n_right_out) {
  if (!bins || !left_out || !right_out || !n_left_out || !n_right_out)
    return -1;
  if (n_rows < 0 || n_features <= 0 || n_leaf_rows < 0) return -1;
  if (feature < 0 || feature >= n_features) return -1;
  if (!leaf_row_idx && n_leaf_rows > n_rows) return -1;
  int64_t nl = 0, nr = 0;
  for (int64_t i = 0; i < n_leaf_rows; ++i) {
    int64_t d = leaf_row_idx ? (int64_t)leaf_row_idx[i] : i;
    if (d < 0 || d >= n_rows) return -1;
    int32_t b = bins[(size_t)d * (size_t)n_features + (size_t)feature];
    if (b <= threshold_bin) {
      left_out[nl] = (int32_t)d;
      nl = nl + 1;
    } else {
      right_out[nr] = (int32_t)d;
      nr = nr + 1;
    }
  }
  *n_left_out = nl;
  *n_right_out = nr;
  return 0;
}
