/*
 * gbdt_hist.h -- C ABI of libgbdt_hist: feature-histogram construction for the
 * leaves of a histogram-based gradient-boosted decision tree, the sibling
 * histogram by subtraction, the best-split gain scan and the row partition that
 * follows a split, on one AMD gfx950 (MI355X) GPU.  Method: "GPU-acceleration for Large-scale Tree Boosting"
 * (arXiv 1706.08359), Sec. 3.3 / Alg. 1 (what a feature histogram is), Sec. 4
 * (building many of them at once on a GPU), App. C.4 (4-bit bins).
 *
 * Conventions shared by every call
 *  - Pointers marked DEVICE are device (HBM) addresses owned by the caller;
 *    the library neither frees nor keeps them after the call's work on
 *    `stream` has finished.  All data is passed by device pointer; the only
 *    HOST pointers are small descriptors marked as such (the leaf offsets of
 *    gbdt_hist_build_batch, the node array gbdt_grow_tree returns), which are
 *    read or written before the call returns.
 *  - `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *    Calls enqueue kernels and return; they do not synchronise and never read
 *    device data on the host (gbdt_grow_tree, which drives the others, is the one
 *    exception and says so).
 *  - Return value: GBDT_OK (0) or a negative gbdt_status code.  Argument
 *    errors are detected before anything is enqueued.  Contents of device
 *    buffers (bin values < n_bins, row ids < n_rows) are NOT checked;
 *    violating them is undefined behaviour.  Debugging aid: with the environment
 *    variable GBDT_HIST_CHECK_INPUTS=1 every call that takes a row list first counts
 *    its out-of-range entries on the device, waits for the stream, and returns
 *    GBDT_EINVAL if there are any.
 *  - Bins are 0-based: a binned value b satisfies 0 <= b < n_bins (the paper
 *    writes 1..k).  2 <= n_bins <= 256.
 *  - The library keeps one scratch workspace per process (partial histograms,
 *    split candidates, partition flags) and a few process-wide counters in device
 *    memory.  Calls that use them (gbdt_hist_build[_batch], gbdt_best_split[_batch],
 *    gbdt_partition_rows[_batch], the tree growers) must be issued on ONE stream at a
 *    time: two such calls in flight on different streams, or from two threads, race.
 *    When the library owns the scratch it grows it on demand: a call that needs more
 *    allocates a larger buffer (hipMalloc) and keeps the old one until gbdt_reset; it never
 *    frees or synchronises inside an enqueuing call.  During stream capture growing is
 *    refused (GBDT_ENOMEM): issue the same call once outside the capture first, or register
 *    a caller buffer (gbdt_set_workspace), or use gbdt_hist_build_noalloc.
 *  - Size limits: n_rows < 2^30, and byte offsets inside a feature tile are 32-bit:
 *    (n_rows + 512) x tile width < 2^32, i.e. n_rows < 67,108,352 with up to 64 bins
 *    (64-byte tiles) and n_rows < 134,217,216 with more (32-byte tiles); at most 65,535
 *    feature tiles.  Beyond that: GBDT_EUNSUPPORTED.
 */
#ifndef GBDT_HIST_H_
#define GBDT_HIST_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GBDT_OK = 0,
  GBDT_EINVAL = -1,       /* NULL required pointer, size out of range, lambda < 0 */
  GBDT_EUNSUPPORTED = -2, /* valid request the library cannot serve (e.g. n_rows >= 2^30) */
  GBDT_EHIP = -3,         /* a HIP runtime call or kernel launch failed */
  GBDT_ENOMEM = -4        /* workspace allocation failed or caller workspace too small */
} gbdt_status;

/* One histogram bin: o[b][1..3] of Alg. 1 -- summed gradient, summed hessian,
 * sample count.  12 bytes, no padding. */
typedef struct {
  float grad;
  float hess;
  uint32_t count;
} gbdt_bin_t;

/* Result of the split search.  A split is [feature id, threshold] (Sec. 3.1);
 * the threshold is a bin index t: rows with bin <= t go left, the others right.
 * feature = bin = -1 and gain = 0 when no threshold is admissible. */
typedef struct {
  int32_t feature;
  int32_t bin;
  float gain; /* G_L^2/(H_L+lambda) + G_R^2/(H_R+lambda) - G^2/(H+lambda), no 1/2 factor */
  float left_grad;
  float left_hess;
  uint32_t left_count;
  float right_grad;
  float right_hess;
  uint32_t right_count;
} gbdt_split_t;

/*
 * Size in bytes of the device layout of an n_rows x n_features binned matrix
 * (App. C.4: n_bins <= 16 stores two 4-bit values per byte, otherwise one byte
 * per value; Sec. 4 "Data Structure": features are bundled so that one thread
 * loads a 4-byte group of one sample).  Rows are kept contiguous inside
 * feature tiles of 16, 32 or 64 bytes; 32 KiB of slack follow the last tile (the
 * build kernel may read, and ignore, whole row groups past the last row).  Behind
 * them the matrix is stored once more column by column, one byte per value
 * (columns padded to a multiple of 256 rows): the row partition after a split reads
 * one feature of every leaf row from there, a byte instead of a tile row.  The layout
 * therefore takes about twice the bytes of the row-major matrix (three times with
 * 4-bit bins).  Returns 0 on invalid arguments.
 */
size_t gbdt_bins_packed_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins);

/*
 * Re-lay a row-major matrix of binned values into the device layout.  Done
 * once before training (App. A.5: feature data is copied once and then stays
 * unchanged).
 *   bins_rowmajor  DEVICE, uint8 [n_rows][n_features], every value < n_bins
 *   packed_out     DEVICE, gbdt_bins_packed_bytes(...) bytes, 16-byte aligned;
 *                  the tiles and columns are fully overwritten (padding is written
 *                  as 0, bin values are reduced modulo the kernel's bin capacity
 *                  16 / 64 / 256), the slack is left as it is
 */
int gbdt_bins_pack(const uint8_t* bins_rowmajor, int64_t n_rows, int32_t n_features,
                   int32_t n_bins, void* packed_out, void* stream);

/*
 * Fused columns for features with few distinct bins (optional, n_bins <= 64 only).  The paper
 * stores features of at most 16 bins in 4 bits (App. C.4) and spreads a feature that uses few
 * of its bins over MORE counters to cut atomic conflicts (Alg. 3, App. A.3).  On this part
 * conflicts cost nothing and the number of local-memory atomic instructions bounds the build,
 * so features with few levels are merged into FEWER counters: features whose level counts
 * multiply to at most 64 share one byte per row (a mixed-radix number of their bins), the
 * build accumulates that column's joint histogram with ONE atomic per row, and every
 * feature's histogram is a marginal of it (exact for counts; one more fp64 sum of at most 64
 * fp32 terms for gradients and hessians).  Constant features ride along for free.
 * gbdt_bins_fuse finds each feature's largest bin value on the device, plans the columns on
 * the host and, if at most 85 % as many columns as features result, writes the fused copy
 * into fused_out and remembers it for `packed`: later gbdt_hist_build /
 * gbdt_hist_build_noalloc calls with that bin_matrix address and shape build leaves that hold
 * at least 8192 rows and a third of the matrix's rows from the fused copy (sparser leaves are
 * bound by HBM traffic, where the plain tiles' narrower rows win; also not with wide
 * accumulation, whose stored sums are exact sums rounded once).  Results and error bound are those of the plain path.  Unlike the
 * other calls it WAITS for the stream (it reads the maxima on the host).
 *   bins_rowmajor   DEVICE, the matrix gbdt_bins_pack packed
 *   packed          DEVICE address gbdt_bins_pack wrote to (used as a key only; a buffer
 *                   copied elsewhere is simply built from its plain tiles)
 *   fused_out       DEVICE, 256-byte aligned, fused_bytes >= gbdt_bins_fused_bytes(...) (0:
 *                   this shape is never fused); owned by the caller, to be kept as long as
 *                   `packed` is used or until gbdt_bins_unfuse(packed) / a new gbdt_bins_pack
 *                   to that address
 *   n_columns_out   HOST: the number of fused columns, 0 when fusing does not pay (nothing
 *                   is remembered then and fused_out may be freed)
 */
size_t gbdt_bins_fused_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins);
int gbdt_bins_fuse(const uint8_t* bins_rowmajor, int64_t n_rows, int32_t n_features, int32_t n_bins,
                   const void* packed, void* fused_out, size_t fused_bytes, int32_t* n_columns_out,
                   void* stream);
int gbdt_bins_unfuse(const void* packed);

/*
 * Feature histograms of one leaf (Alg. 1 for every feature; Sec. 4 and
 * App. A.1 for the GPU organisation: work split by features and by samples,
 * per-workgroup histograms in local memory, a final reduction pass).
 * For every leaf sample i with row id d = leaf_row_idx[i] and every feature j:
 *   hist_out[j][bin(d, j)] += (grad[d], hess[d], 1).
 *   bin_matrix     DEVICE, layout written by gbdt_bins_pack with the same
 *                  n_rows, n_features, n_bins
 *   leaf_row_idx   DEVICE int32 [n_leaf_rows], row ids in [0, n_rows); NULL
 *                  means rows 0..n_leaf_rows-1 (the root when n_leaf_rows ==
 *                  n_rows).  Any order and repeats are legal (each occurrence
 *                  counts); ascending order reads memory best.
 *   n_leaf_rows    0 <= n_leaf_rows; with NULL index also <= n_rows
 *   grad, hess     DEVICE float [n_rows], indexed by ROW ID (g_{d_ri}, h_{d_ri}
 *                  in Alg. 1), not by position in the leaf
 *   hist_out       DEVICE gbdt_bin_t [n_features][n_bins], fully overwritten;
 *                  all zero when n_leaf_rows == 0
 * Arithmetic: a workgroup takes its rows in epochs of 512.  Per epoch it sums |grad|
 * and |hess| over the epoch's rows, derives the largest power-of-two scales for
 * which no signed 27-bit bin sum can overflow, rounds every gradient and hessian
 * once to that grid and accumulates count, gradient and hessian as the three fields
 * of one 64-bit integer per (feature, bin) (App. A.6 discusses the precision of this
 * accumulation; gfx950's local-memory float add is ~30x slower than its integer
 * add).  Epoch sums are rescaled and accumulated in fp32 (fp64 for n_bins <= 16),
 * the partial histograms of the workgroups are combined in fp64 in a fixed order
 * and rounded to fp32.  Consequences:
 *   - counts are exact;
 *   - every gradient (hessian) bin sum is within 512 / (2^26 - 512) = 7.7e-6 of the
 *     sum of |grad| (|hess|) over the leaf, plus the fp32 roundings named above, for
 *     any input values and any bin distribution;
 *   - values that are multiples of a power of two well above the quantum (e.g.
 *     +-0.5, 0.25) are accumulated exactly;
 *   - the split of a leaf's rows among workgroups is decided at run time, so the
 *     last bits of gradient / hessian sums may differ between runs.
 * grad / hess must be finite.
 */
int gbdt_hist_build(const void* bin_matrix, int64_t n_rows, int32_t n_features, int32_t n_bins,
                    const int32_t* leaf_row_idx, int64_t n_leaf_rows, const float* grad,
                    const float* hess, gbdt_bin_t* hist_out, void* stream);

/*
 * gbdt_hist_build for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same results and error
 * bound as gbdt_hist_build, but the scratch (unit counters and the workgroups' partial
 * histograms) is a fixed array inside the library's device code -- 64 MiB of partial
 * histograms plus a 256 KiB head, one copy per GPU the library runs on, held until the
 * process ends -- and the call neither allocates, frees nor synchronises (no hipMalloc /
 * hipFree, no profiling events, no row-id checking pass; it ignores gbdt_set_workspace and
 * gbdt_profile_enable).  A leaf whose usual grid would write more partial histograms than
 * the array holds is built with fewer workgroups per feature tile (slower, same result up
 * to the summation order); if even one workgroup per tile does not fit (roughly n_features
 * x bin capacity x 12 bytes > 64 MiB, e.g. more than 21,800 features at 256 bins) the call
 * returns GBDT_EUNSUPPORTED and gbdt_last_hip_error() says so.  The array keeps the last
 * call's contents; every call clears the counters it uses itself.  All calls on one GPU
 * share the array: calls that overlap on one GPU (two streams, two threads) race.
 * gbdt_hist_build_noalloc_max_partial_bytes: the capacity for partial histograms.
 */
int gbdt_hist_build_noalloc(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                            int32_t n_bins, const int32_t* leaf_row_idx, int64_t n_leaf_rows,
                            const float* grad, const float* hess, gbdt_bin_t* hist_out, void* stream);
size_t gbdt_hist_build_noalloc_max_partial_bytes(void);

/*
 * Feature histograms of several leaves in one call: hist_out[l] is what gbdt_hist_build
 * writes for the leaf whose row list is row_idx[leaf_offsets[l] .. leaf_offsets[l + 1]).
 * The paper builds one leaf at a time, and its kernel benchmark (App. C.2) shows the
 * rate falling as leaves get small, because a small leaf cannot fill the GPU; a level of
 * a depth-wise tree, or the small children of several splits, can when they share a
 * launch.  Up to 224 leaves go into one kernel launch (plus one reduction launch);
 * longer batches are cut into such launches.
 *   row_idx        DEVICE int32: the leaves' row lists back to back (e.g. the
 *                  children_out segments gbdt_partition_rows wrote), row ids in
 *                  [0, n_rows); may be NULL when every leaf is empty
 *   leaf_offsets   HOST int64 [n_leaves + 1], non-decreasing, leaf_offsets[0] >= 0;
 *                  read before the call returns.  Leaves may be empty; each holds fewer
 *                  than 2^31 rows and each launch of 224 leaves fewer than 2^32.
 *   grad, hess     DEVICE float [n_rows], indexed by row id
 *   hist_out       DEVICE gbdt_bin_t [n_leaves][n_features][n_bins], fully overwritten
 * Arithmetic and error bound per leaf as for gbdt_hist_build; the split of a leaf's rows
 * among workgroups is fixed by the batch's shape and the device, so the same call gives
 * the same bits every time.  Scratch: see gbdt_hist_build_batch_workspace_bytes.
 */
int gbdt_hist_build_batch(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                          int32_t n_bins, const int32_t* row_idx, const int64_t* leaf_offsets,
                          int32_t n_leaves, const float* grad, const float* hess,
                          gbdt_bin_t* hist_out, void* stream);

/* Upper bound on the scratch gbdt_hist_build_batch needs for batches of at most n_leaves
 * leaves of this shape on the current device (0 on invalid arguments); to be covered by
 * the buffer given to gbdt_set_workspace when the caller owns the scratch.  (With 8 more
 * bytes per listed row to spare the call first gathers grad / hess of sparse leaves into list
 * order, which is faster on matrices of many feature tiles; a buffer of exactly this size
 * makes it read them by row id instead.) */
size_t gbdt_hist_build_batch_workspace_bytes(int32_t n_features, int32_t n_bins, int32_t n_leaves);

/*
 * Bit-reproducible histograms (App. A.6 weighs precision against speed; this switch
 * weighs run-to-run reproducibility against speed).  By default the workgroups of
 * gbdt_hist_build share out a leaf's rows at run time, which balances them best but
 * lets the last bits of gradient / hessian sums vary between runs.  With enable != 0
 * (process-wide, affects later gbdt_hist_build calls) the split is fixed by the
 * problem shape and the device: the same call then gives the same bits every time.
 * Counts are identical in both modes.
 */
int gbdt_set_deterministic(int enable);

/*
 * Wide accumulation: the double precision switch of App. A.6 (the paper's GPU code sums
 * in fp32 by default and offers fp64 for precision and reproducibility; the CPU trainer
 * it extends stores fp32 and accumulates in fp64).  With enable != 0 (process-wide,
 * affects later gbdt_hist_build / gbdt_hist_build_batch calls and the tree growers,
 * which build through them) a workgroup sums gradients and hessians in 54-bit fixed
 * point and fp64 instead of 27-bit fixed point and fp32: a stored sum is the exact sum
 * rounded to fp32, up to 5e-13 of the leaf's sum of magnitudes.  1.6-2.0x the build
 * time; twice the LDS and twice the scratch for partial results, so query
 * gbdt_workspace_bytes / gbdt_hist_build_batch_workspace_bytes AFTER setting the mode
 * when the caller owns the scratch.  Together with gbdt_set_deterministic the sums are
 * bit-reproducible as well.  Counts are identical in all modes.
 */
int gbdt_set_wide_accumulation(int enable);

/*
 * Sibling histogram: sibling_out[j][b] = parent[j][b] - child[j][b] for the
 * gradient sum, hessian sum and count.  Not described in the paper; it is the
 * complement of Alg. 1 over the parent's samples that are not in the child.
 * All three are DEVICE gbdt_bin_t [n_features][n_bins]; sibling_out may alias
 * parent or child.  child counts must not exceed parent counts.
 * (n_features, n_bins: sizes the short form of the call leaves implicit.)
 */
int gbdt_hist_subtract(const gbdt_bin_t* parent, const gbdt_bin_t* child, gbdt_bin_t* sibling_out,
                       int32_t n_features, int32_t n_bins, void* stream);

/*
 * Best split of a leaf from its histograms (Sec. 3.3: the split objective of
 * Eq. (4), in its gradient/hessian form from Eq. (9), is evaluated only at the
 * bin boundaries).  For every feature j and threshold t in 0..n_bins-2, left =
 * bins <= t (running prefix), right = feature total - left.  A threshold is
 * admissible when both sides have count >= 1 and hessian sum >= min_child_hess.
 * The admissible threshold with the largest gain wins; equal gains go to the
 * smaller feature, then the smaller bin.  Prefix sums and gains are computed in
 * fp64 from the fp32 histogram, bins in ascending order.
 *   hist        DEVICE gbdt_bin_t [n_features][n_bins]
 *   lambda      L2 regularisation added to each hessian sum, >= 0
 *   split_out   DEVICE, one gbdt_split_t, overwritten
 */
int gbdt_best_split(const gbdt_bin_t* hist, float lambda, float min_child_hess,
                    gbdt_split_t* split_out, int32_t n_features, int32_t n_bins, void* stream);

/*
 * gbdt_best_split for n_hists histograms at once: splits_out[i] is the best split of
 * hists[i] (e.g. the two children of a split, or a level of a tree), same rule, same
 * arithmetic, one kernel launch for up to 32768 histograms.
 *   hists       DEVICE gbdt_bin_t [n_hists][n_features][n_bins]
 *   splits_out  DEVICE gbdt_split_t [n_hists], overwritten
 * n_hists == 0 is a no-op.  Scratch: 56 bytes per histogram and workgroup of the launch (never
 * more workgroups per histogram than a lone histogram gets, see gbdt_debug_split_plan; a
 * caller-owned workspace sized by gbdt_workspace_bytes covers 64 histograms).
 */
int gbdt_best_split_batch(const gbdt_bin_t* hists, int32_t n_hists, float lambda,
                          float min_child_hess, gbdt_split_t* splits_out, int32_t n_features,
                          int32_t n_bins, void* stream);

/*
 * Row partition of a leaf into its two children (the Split() step of App. C.1; it
 * produces the per-leaf sample index list that App. A.5 has the CPU rebuild and copy
 * to the GPU after every split -- here the list never leaves the device).
 * A leaf row with row id d goes left when bin(d, split->feature) <= split->bin, right
 * otherwise -- the convention of gbdt_split_t.  children_out receives the left rows,
 * then the right rows, each side in the order the parent listed them (ascending lists
 * stay ascending), so the children are children_out[0 .. n_left) and
 * children_out[n_left .. n_leaf_rows) and both can be passed to gbdt_hist_build as
 * leaf_row_idx.  n_left equals split->left_count when the record came from the leaf's own
 * histogram.
 *   bin_matrix     DEVICE, layout written by gbdt_bins_pack with the same n_rows,
 *                  n_features, n_bins
 *   leaf_row_idx   DEVICE int32 [n_leaf_rows] or NULL (rows 0..n_leaf_rows-1), as in
 *                  gbdt_hist_build
 *   split          DEVICE, one gbdt_split_t (e.g. as written by gbdt_best_split); only
 *                  feature and bin are read, on the device.  A feature outside
 *                  [0, n_features) -- such as the -1 of "no admissible split" -- sends
 *                  every row left.
 *   children_out   DEVICE int32 [n_leaf_rows], fully overwritten; must not overlap
 *                  leaf_row_idx
 *   n_left_out     DEVICE int64 [1], receives the number of left rows; may be NULL
 * Uses the scratch workspace (n_leaf_rows / 8 bytes of flags plus a few KiB).  Exact
 * integer work: the result is unique and reproducible.
 */
int gbdt_partition_rows(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                        int32_t n_bins, const int32_t* leaf_row_idx, int64_t n_leaf_rows,
                        const gbdt_split_t* split, int32_t* children_out, int64_t* n_left_out,
                        void* stream);

/*
 * gbdt_partition_rows for several leaves at once (a level of a tree): leaf l has the row list
 * row_idx[leaf_offsets[l] .. leaf_offsets[l + 1]) and the split record splits[l]; its children
 * are written to the same positions of children_out (left rows, then right rows, order
 * kept), so the children of a whole level again lie back to back and can go straight into
 * gbdt_hist_build_batch.  Two kernel launches per 192 leaves.
 *   row_idx        DEVICE int32, row ids in [0, n_rows)
 *   leaf_offsets   HOST int64 [n_leaves + 1], non-decreasing, read before the call returns
 *   splits         DEVICE gbdt_split_t [n_leaves]; a record without a split keeps all rows left
 *   children_out   DEVICE int32, as long as row_idx; must not overlap it
 *   n_left_out     DEVICE int64 [n_leaves] or NULL
 */
int gbdt_partition_rows_batch(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                              int32_t n_bins, const int32_t* row_idx, const int64_t* leaf_offsets,
                              int32_t n_leaves, const gbdt_split_t* splits, int32_t* children_out,
                              int64_t* n_left_out, void* stream);

/*
 * One node of a tree grown by gbdt_grow_tree (a HOST struct).  Node 0 is the root; the two
 * children of a split get the next two ids, left first, so parents precede children.
 */
typedef struct {
  int32_t parent;  /* -1 for the root */
  int32_t left;    /* children; -1 for a leaf */
  int32_t right;
  int32_t feature; /* the node's best split as gbdt_best_split found it (applied when left >= 0); */
  int32_t bin;     /* feature = bin = -1 when no threshold is admissible */
  float gain;
  float sum_grad;  /* sums over the node's rows (for a leaf value such as -G / (H + lambda)) */
  float sum_hess;
  uint32_t count;
  int32_t reserved;
  int64_t row_begin; /* the node's rows are row_order_out[row_begin .. row_begin + count) */
} gbdt_tree_node_t;

/*
 * Grows one regression tree leaf-wise, entirely from the calls above, with row lists and
 * histograms resident on the device (Sec. 3.1: start from the root and keep splitting
 * leaves; Sec. 5: stop at a fixed number of leaves, 255 in the experiments, at least one
 * sample per leaf; App. A.5 / App. C.1: what the CPU does around the histogram kernel --
 * rebuild and copy the index list after each split -- is done here on the device, so
 * nothing but 36-byte split records crosses the bus).  The paper does not say which leaf is
 * split next; this takes the open leaf whose best split has the largest gain (it must exceed
 * min_split_gain), the older leaf on equal gains.  Per split: partition the leaf's rows,
 * build the histogram of the smaller child, subtract it from the parent's for the sibling,
 * search both for their best split.  That rule is sequential; to wait for the device once
 * per ROUND rather than once per split, a round does this work for up to 32 open leaves at
 * once (batched calls), and the host then applies the rule to what it knows, stopping at the
 * first leaf whose children it has not seen.  The tree is exactly the sequential rule's; work
 * on a leaf the rule never reaches before max_leaves is used up is dropped.
 *   grad, hess       DEVICE float [n_rows]
 *   max_leaves       >= 1; growth also stops when no open leaf has an admissible split
 *   scratch          DEVICE, 256-byte aligned, gbdt_grow_tree_scratch_bytes(...) bytes
 *                    (two row lists, half a row list for the smaller children of a round,
 *                    about 3 x max_leaves histograms, the split records); the calls inside
 *                    also use the library's scratch workspace
 *   nodes_out        HOST gbdt_tree_node_t [2 * max_leaves - 1]
 *   n_nodes_out      HOST, receives the number of nodes written (always odd)
 *   row_order_out    DEVICE int32 [n_rows] or NULL: all row ids, grouped by leaf, ascending
 *                    inside each node's segment (see row_begin)
 * Unlike the other calls this one WAITS for `stream` (once per round, to read the new split
 * records) and allocates a few KB of page-locked host memory on first use.  The histograms
 * of a round are built by gbdt_hist_build_batch, whose split of rows among workgroups is
 * fixed: the same call gives the same tree, bit for bit, every time.
 */
int gbdt_grow_tree(const void* bin_matrix, int64_t n_rows, int32_t n_features, int32_t n_bins,
                   const float* grad, const float* hess, int32_t max_leaves, float lambda,
                   float min_child_hess, float min_split_gain, void* scratch, size_t scratch_bytes,
                   gbdt_tree_node_t* nodes_out, int32_t* n_nodes_out, int32_t* row_order_out,
                   void* stream);
size_t gbdt_grow_tree_scratch_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins,
                                    int32_t max_leaves);

/*
 * The same tree, grown level by level to a maximum depth instead of leaf by leaf to a
 * number of leaves (Sec. 5 runs its comparison trainers with a maximum depth of 8): every
 * node of the current level whose best split is admissible and gains more than
 * min_split_gain is split.  A whole level costs a handful of launches whatever its width:
 * one batched split search and one read-back of the level's records, one batched
 * partition, one batched histogram build of all the smaller children, one subtraction
 * kernel for their siblings.  Nodes are numbered level by level, the children of a level
 * in the order of their parents, left first (parents precede children).
 *   max_depth        0 .. 16; at most 2^max_depth leaves
 *   scratch          DEVICE, 256-byte aligned, gbdt_grow_tree_depthwise_scratch_bytes(...)
 *   nodes_out        HOST gbdt_tree_node_t [2^(max_depth + 1) - 1]
 *   other arguments, waiting and allocation as for gbdt_grow_tree (one wait per level).
 */
int gbdt_grow_tree_depthwise(const void* bin_matrix, int64_t n_rows, int32_t n_features,
                             int32_t n_bins, const float* grad, const float* hess, int32_t max_depth,
                             float lambda, float min_child_hess, float min_split_gain, void* scratch,
                             size_t scratch_bytes, gbdt_tree_node_t* nodes_out, int32_t* n_nodes_out,
                             int32_t* row_order_out, void* stream);
size_t gbdt_grow_tree_depthwise_scratch_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins,
                                              int32_t max_depth);

/*
 * Scratch workspace.  By default the library allocates device scratch itself
 * on first use and grows it when a larger problem arrives (hipMalloc inside
 * gbdt_hist_build / gbdt_best_split / gbdt_partition_rows).  A caller that wants no allocation in
 * those calls registers its own buffer:
 *   gbdt_workspace_bytes  upper bound on scratch needed by gbdt_hist_build,
 *                         gbdt_best_split and gbdt_partition_rows (leaves of at
 *                         most n_rows entries) for this problem shape on the
 *                         current device (0 on invalid arguments)
 *   gbdt_set_workspace    DEVICE buffer, 256-byte aligned, kept until replaced;
 *                         (NULL, 0) returns to library-owned scratch.  With a
 *                         caller buffer, a call that needs more returns
 *                         GBDT_ENOMEM.
 */
size_t gbdt_workspace_bytes(int64_t n_rows, int32_t n_features, int32_t n_bins);
int gbdt_set_workspace(void* dev_ptr, size_t bytes);

/* Static, human-readable text for a gbdt_status code. */
const char* gbdt_strerror(int code);

/* Text of the last HIP error seen by this thread's failing call ("" if none). */
const char* gbdt_last_hip_error(void);

/*
 * Timing of the histogram build kernel by itself (gbdt_hist_build also launches
 * the reduction pass in the same call).  While enabled, every gbdt_hist_build
 * records a HIP event on its stream before and after the build kernel.
 * gbdt_profile_collect waits for the recorded events, returns the summed kernel
 * time in milliseconds and the number of launches, and forgets them.
 */
int gbdt_profile_enable(int enable);
int gbdt_profile_collect(double* build_kernel_ms_total, int64_t* n_launches);
/* The same, launch by launch: ms_out[i] receives the duration of the i-th recorded build
 * kernel (the first `capacity` of them), *n_launches their number; the events are forgotten. */
int gbdt_profile_durations(double* ms_out, int64_t capacity, int64_t* n_launches);

/*
 * Back to a clean state after a failure: WAITS for the device, frees the library-owned
 * scratch (including buffers it outgrew: growing never frees, so that an enqueuing call
 * never synchronises) and forgets pending profiling events, then sets the split search's
 * ticket counters and what is known about the unit counters back to "unknown", so that the
 * next call clears what it uses.  A caller-registered workspace stays registered.  Needed
 * only after a call failed half-way (GBDT_EHIP, or GBDT_ENOMEM from a too-small caller
 * workspace between the kernels of one call): a build whose reduction pass never ran leaves
 * unit counters counted up, and later histograms would silently miss rows.  The modes set by
 * gbdt_set_deterministic / gbdt_set_wide_accumulation are kept.
 */
int gbdt_reset(void);

/*
 * A plain copy kernel of known HBM traffic (bytes read + bytes written), used to scale
 * the memory counters of a profiler run.  src, dst: DEVICE, 16-byte aligned, bytes a
 * multiple of 16, not overlapping.
 */
int gbdt_calibration_copy(const void* src, void* dst, size_t bytes, void* stream);

/*
 * Introspection of the host-side launch planning (no GPU needed; used by tests).
 * gbdt_debug_geometry fills out[0..15] with: bin capacity, 4-bit flag, main tile
 * width, number of main tiles, remainder tile width, packed bytes per row, feature
 * bytes per row, threads per workgroup, LDS bytes per workgroup, workgroups per
 * tile, epochs (of 512 rows) per unit of work, total 4-byte words of partial
 * histograms, 0, 0, 0, 0 -- as planned for a device with n_cus compute units (<= 0:
 * 256).  n_out must be >= 16.
 * gbdt_debug_locate reports the tile and the local-memory slot of a feature.
 */
int gbdt_debug_geometry(int32_t n_features, int32_t n_bins, int64_t n_leaf_rows, int32_t n_cus,
                        int64_t* out, int32_t n_out);
/* Launch plan of the first (at most 224-leaf) launch of gbdt_hist_build_batch on a device
 * with n_cus compute units holding wg_per_cu workgroups each: per leaf the workgroups per
 * tile and the epochs per unit; for block i < max_blocks of the grid, block_out[3 i ..
 * 3 i + 2] = (leaf, tile, workgroup of that leaf and tile), computed by the function the
 * kernel uses.  Returns the number of blocks, or a negative gbdt_status. */
int gbdt_debug_batch_plan(int32_t n_features, int32_t n_bins, const int64_t* leaf_offsets,
                          int32_t n_leaves, int32_t n_cus, int32_t wg_per_cu, int32_t* leaf_wgs_out,
                          int32_t* leaf_unit_epochs_out, int32_t* block_out, int32_t max_blocks);
/* The column plan gbdt_bins_fuse makes for features with the given numbers of levels (1..64
 * each): col_out[f] / stride_out[f] = the column of feature f and the weight of its bin in the
 * column's joint value; *n_cols_out the number of columns.  Host only. */
int gbdt_debug_fusion_plan(const uint32_t* levels, int32_t n_features, int32_t* col_out, int32_t* stride_out,
                           int32_t* n_cols_out);
/* Resident workgroups per compute unit of the build kernel variant that serves
 * n_bins (indexed != 0: the variant that gathers through leaf_row_idx), as the HIP
 * runtime reports it on the current device; 0 if the query is not possible. */
int gbdt_debug_occupancy(int32_t n_bins, int32_t indexed);
/* How gbdt_best_split_batch splits a launch over n_hists histograms of n_features x n_bins:
 * out[0] = features a workgroup holds in local memory at a time, out[1] = such groups it takes
 * one after the other, out[2] = workgroups (and candidates) per histogram, out[3] = bytes of
 * local memory per workgroup.  Host only. */
int gbdt_debug_split_plan(int32_t n_features, int32_t n_bins, int32_t n_hists, int64_t* out, int32_t n_out);
/* How gbdt_partition_rows cuts a list of n_leaf_rows positions into chunks: out[0] = steps of
 * 256 positions a workgroup takes (positions per chunk / 256), out[1] = chunks, out[2] = bytes of
 * scratch (flag words and chunk counts).  Host only. */
int gbdt_debug_partition_plan(int64_t n_leaf_rows, int64_t* out, int32_t n_out);
int gbdt_debug_locate(int32_t n_features, int32_t n_bins, int32_t feature, int32_t* tile_out,
                      int32_t* slot_out);

#ifdef __cplusplus
}
#endif
#endif /* GBDT_HIST_H_ */
