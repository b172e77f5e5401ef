/*
 * gbt.h -- C ABI of libgbt: quantised-histogram decision-tree construction
 * (the data-parallel hot path of arXiv 1806.11248) for AMD MI355X (gfx950).
 *
 * Conventions
 * -----------
 *  - Plain C, no exceptions.  Every call returns an int32_t status:
 *      GBT_OK, GBT_EINVAL (null pointer / bad shape / value out of range),
 *      GBT_ENOMEM (caller's workspace too small), GBT_EHIP (a HIP runtime call
 *      failed; text in gbt_last_error), GBT_EUNSUPPORTED (e.g. bits > 16).
 *    On an argument error nothing has been enqueued and outputs are untouched.
 *  - Pointers marked [dev] are device (HBM) addresses, [host] are host
 *    addresses.  The caller owns every buffer, including workspaces: the
 *    library allocates no device memory after gbt_create (which takes a few KB
 *    of pinned host staging).  Pointers are borrowed for the call only.
 *  - Work is enqueued on the stream given to gbt_create.  A call that returns
 *    a host value (a count, split records, a tree) synchronises that stream
 *    before returning; every other call is asynchronous.
 *  - One gbt_ctx must not be used from two threads at once.
 *
 * Data layout
 * -----------
 *  - Symbols: sym(r,f) in [0, nb[f]) is the quantile bin of feature f in row r;
 *    a missing value has the one global symbol missing_sym = max_f nb[f].
 *  - Packed matrix (Sec. 2.2): element e = r*F + f occupies bits
 *    [e*bits, (e+1)*bits) of a little-endian bit stream stored in uint32 words,
 *    rows back to back without padding, unused tail bits zero, followed by one
 *    zero word (so an 8-byte read at the last element stays in bounds).
 *    bits = number of bits of the largest symbol present, 1..16.
 *  - Gradient pairs: float2 (g, h) per row, h >= 0.  Histograms are summed in
 *    64-bit fixed point: each g is rounded once to an int32 multiple of
 *    1/scale_g and each h to a multiple of 1/scale_h (scales are powers of two
 *    with |g*scale_g| <= 2^26 and h*scale_h <= 2^22 for every row), and all
 *    later sums are exact integers, so a histogram does not depend on the order
 *    of accumulation and "parent - child" is exactly the sibling.
 *  - Histogram of one node: int64 hist[F][B][2] (g then h), B = max_bins.
 */
#ifndef GBT_H
#define GBT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GBT_API __attribute__((visibility("default")))

#define GBT_OK 0
#define GBT_EINVAL (-1)
#define GBT_ENOMEM (-2)
#define GBT_EHIP (-3)
#define GBT_EUNSUPPORTED (-4)

#define GBT_OBJ_SQUARED 0
#define GBT_OBJ_LOGISTIC 1

#define GBT_MAX_BITS 16
#define GBT_GAIN_FLOOR 1e-6 /* a node is split only if gain > max(gamma, GBT_GAIN_FLOOR) */

typedef struct gbt_ctx gbt_ctx;

typedef struct gbt_params {
    int32_t max_depth;       /* edges from the root to the deepest leaf, 0..16 */
    int32_t max_bins;        /* B: stride of the bin axis, >= every nb[f], 2..4096 */
    double lambda;           /* L2 term in gain and leaf weight, >= 0 */
    double gamma;            /* minimum gain of a split */
    double min_child_weight; /* minimum hessian mass of a child */
    double eta;              /* learning rate used by gbt_predict callers */
    int32_t objective;       /* GBT_OBJ_* */
    float base_margin;
} gbt_params;

/* One split candidate (the best of a node), Alg. 1 "EvaluateSplit". */
typedef struct gbt_split {
    int32_t feature;      /* -1: no valid candidate */
    int32_t bin;          /* rows with symbol <= bin go left */
    int32_t default_left; /* 1: rows with the missing symbol go left */
    int32_t valid;
    double gain;          /* GL^2/(HL+l) + GR^2/(HR+l) - G^2/(H+l); a term with denominator 0 counts 0 */
    double GL, HL, GR, HR;
    int64_t GLq, HLq;     /* left sums in fixed point (exact) */
} gbt_split;

/* A tree as caller-allocated host arrays of `capacity` >= 2^(max_depth+1)-1
 * entries each.  Node 0 is the root; children are numbered in creation order,
 * level by level, left to right. */
typedef struct gbt_tree {
    int32_t capacity;
    int32_t n_nodes;       /* out */
    int32_t *feature;      /* -1 = leaf */
    int32_t *bin;
    int32_t *default_left;
    int32_t *left, *right; /* child ids, -1 for a leaf */
    float *threshold;      /* raw-value form of the split: left iff x < threshold
                              (= cuts[feature][bin]; +inf when bin is the last bin) */
    double *weight;        /* -G/(H+lambda) of every node; 0 where H+lambda = 0 */
    double *gain;          /* gain of the node's split, 0 for a leaf */
    double *sumG, *sumH;
    int64_t *n_rows;
} gbt_tree;

/* ---- context ----------------------------------------------------------- */

/* Creates a context on HIP device `device`; `stream` is a hipStream_t (NULL =
 * the default stream).  Loads nothing lazily: a missing or wrong-architecture
 * GPU makes this call fail with GBT_EHIP.
 *
 * Environment switches, read here once per context.  None changes a result (every
 * tree, histogram and partition is the same under all of them, which the tests
 * check by creating contexts under them); they choose between kernels and launch
 * shapes, for measurements and for covering the alternative code paths.  Unset =
 * the default in brackets; values outside the stated range are ignored.
 *   GBT_TUNE_PART_HIST          [1] 0: never fuse the partition with a child's histogram (grow path 2 off)
 *   GBT_TUNE_PART_FUSED         [1] 0: no one-launch unordered partition (paths 1 and 2 off)
 *   GBT_TUNE_PART_IDS           [1] 0: wide rows are moved as whole records instead of partitioning id lists (path 3 off)
 *   GBT_TUNE_MOVE_MAX_WORDS     [8] 1..64: rows of more 32-bit words than this are listed (path 3), not moved
 *   GBT_TUNE_ORDER_ROWS         [1] 0: row ids travel with the rows (path 0) instead of the order being rebuilt from the tree
 *   GBT_TUNE_PART_NOMOVE        [2] 0..2: how many of the last levels of a depth-wise tree leave their rows in place (path 2)
 *   GBT_TUNE_PART_CYCLE         [1] 0: above those levels rows are moved at every level instead of every third (two levels in place, then one move over three levels of splits; path 2)
 *   GBT_TUNE_HIST_FIX           [1] 0: gradient pairs are rounded to fixed point in a pass of their own, not in the root histogram launch
 *   GBT_TUNE_HIST8              [1] 0: the root histogram of byte symbols by the general byte-symbol kernel
 *   GBT_TUNE_HIST8_STAGGER      [64] 0..128: in 1/1024 of a job's length, how unequal the jobs of that launch are
 *   GBT_TUNE_HIST_RUNTIME_BITS  [0] 1: histogram kernel with a run-time symbol width instead of the compile-time ones
 *   GBT_TUNE_HIST_BLOCK         [512] 256, 512, 1024: threads per histogram workgroup
 *   GBT_TUNE_HIST_LDS_KB        [64] 8..128: cap on a workgroup's LDS histogram (smaller feature tiles, more workgroups per CU); unset, a shape
 *                                    that needs two to four feature tiles takes twice the cap where that saves a tile
 *   GBT_TUNE_HIST_JOBS          [8] 1..64: histogram workgroups to aim for per compute unit and launch
 *   GBT_TUNE_HIST_MERGE_RATIO   [96] 1..100000: LDS additions a bin should receive per value a job merges into HBM (longer row pieces)
 *   GBT_TUNE_LOSSGUIDE_BATCH    [16] 1..64: open leaves expanded per round of loss-guided growth
 *   GBT_TUNE_SPARSE_JOBS        [1] 1..64: sparse-row histogram workgroups per compute unit
 *   GBT_TUNE_SPARSE_TILED       [0] 1: sparse-row histogram in id-range tiles even where all ids fit one workgroup's LDS */
GBT_API int32_t gbt_create(gbt_ctx **ctx_out, int32_t device, void *stream);
GBT_API int32_t gbt_destroy(gbt_ctx *ctx);
/* Text of the last error of this context ("" if none).  [host], owned by ctx. */
GBT_API const char *gbt_last_error(const gbt_ctx *ctx);
GBT_API const char *gbt_version(void);

/* ---- Sec. 2.1 feature quantile generation ------------------------------ */

/* Bytes of workspace gbt_quantise needs. n_values = n*F for dense input, the
 * number of stored values for CSR. */
GBT_API size_t gbt_quantise_workspace_bytes(int64_t n, int32_t F, int64_t n_values, int32_t max_bins);

/*
 * Per-feature quantile cuts and binning.  Input is EITHER dense row-major
 * X[n][F] [dev] with NaN = missing (indptr = indices = values = NULL) OR CSR
 * (X = NULL; indptr int64[n+1], indices int32[nnz] column ids, values
 * float[nnz], all [dev]; absent entries are missing; with nnz = indptr[n] = 0
 * indices and values may be NULL).
 *   cuts_out  [dev] float[F][max_bins-1], strictly increasing, +inf padded.
 *             With m present values v[0..m) sorted and d distinct ones:
 *             d <= max_bins: every distinct value but the smallest is a cut;
 *             else the distinct values among v[floor(k*m/max_bins)], k=1..B-1,
 *             without any equal to v[0].  Cuts are data values.
 *   nb_out    [dev] int32[F]   bins per feature = cuts + 1 (1 if nothing present)
 *   sym_out   [dev] uint16[n][F]  sym = #{cuts <= x}; missing -> missing_sym
 *   max_value_out, missing_sym_out  [host] largest symbol written; max_f nb[f]
 * Synchronises the stream.
 */
GBT_API int32_t gbt_quantise(gbt_ctx *ctx, const float *X, const int64_t *indptr, const int32_t *indices,
                     const float *values, int64_t n, int32_t F, int32_t max_bins, float *cuts_out,
                     int32_t *nb_out, uint16_t *sym_out, int32_t *max_value_out,
                     int32_t *missing_sym_out, void *workspace, size_t workspace_bytes);

/*
 * gbt_quantise and gbt_compress in one call (Sec. 2.1 -> Sec. 2.2): the same cuts, and the same bit stream as
 * packing the symbols gbt_quantise would write, but the symbols go from the binning straight into the stream and
 * the uint16 matrix is never stored.
 *   packed_out [dev] uint32[packed_capacity_words].  The width is only known once the cuts are (the largest symbol
 *             is max_f nb[f] if any element is missing, one less otherwise), and it never exceeds
 *             gbt_bits(max_bins): capacity gbt_packed_words(n, F, gbt_bits(max_bins)) always suffices.  Too small
 *             for the width found: GBT_ENOMEM, nothing packed.
 *   bits_out  [host] the width; max_value_out, missing_sym_out, cuts_out, nb_out, the inputs and the workspace
 *             (gbt_quantise_workspace_bytes) as for gbt_quantise.
 * CSR input whose rows have too many features for 32 of them to fit the packing tile in LDS (F above ~760) is
 * refused with GBT_EUNSUPPORTED: take the two calls.  Synchronises the stream.
 */
GBT_API int32_t gbt_quantise_packed(gbt_ctx *ctx, const float *X, const int64_t *indptr, const int32_t *indices,
                                    const float *values, int64_t n, int32_t F, int32_t max_bins, float *cuts_out,
                                    int32_t *nb_out, uint32_t *packed_out, int64_t packed_capacity_words,
                                    int32_t *bits_out, int32_t *max_value_out, int32_t *missing_sym_out,
                                    void *workspace, size_t workspace_bytes);

/* ---- Sec. 2.2 data compression ----------------------------------------- */

/* Bits per element for a largest symbol max_value: its bit length, at least 1. */
GBT_API int32_t gbt_bits(uint32_t max_value);
/* uint32 words of the packed matrix, including the trailing zero word. */
GBT_API int64_t gbt_packed_words(int64_t n, int32_t F, int32_t bits);
/* Packs sym[n][F] [dev] into packed_out [dev] (gbt_packed_words words) at
 * bits = gbt_bits(max_value), returned in *bits_out [host].  Asynchronous. */
GBT_API int32_t gbt_compress(gbt_ctx *ctx, const uint16_t *sym, int64_t n, int32_t F, uint32_t max_value,
                     uint32_t *packed_out, int32_t *bits_out);

/* ---- sparse rows: Sec. 1 (sparse input), Sec. 2.2 (compressed storage) ---- */

/*
 * A second storage form of the quantised matrix for mostly-empty data: row r
 * keeps only its present elements (sym != missing_sym), each as the global bin
 * id  gid = f * max_bins + sym, ascending, in ent[rowptr[r] .. rowptr[r+1]).
 * An entry is a uint16 where F * max_bins <= 65536 and a uint32 in a wider
 * matrix: gbt_sparse_entry_bytes(F, max_bins) = 2 or 4 (0: not a valid shape;
 * more than 2^28 ids are refused with GBT_EUNSUPPORTED), and every `ent`
 * argument below is an array of that type.  2*gid is the
 * element's place in a [F][max_bins][2] histogram.  Two calls, because the
 * caller allocates the entry stream:
 *   gbt_compress_sparse_count  sym [dev] uint16[n][F] -> rowptr_out [dev]
 *                              uint32[n+1], *nnz_out [host] = rowptr[n].
 *                              Synchronises the stream.
 *   gbt_compress_sparse        fills ent_out [dev, 4-byte aligned]; it must hold
 *                              gbt_sparse_capacity(nnz) entries: the kernels read
 *                              the stream as whole words, up to 32 entries past
 *                              the end.  Asynchronous.
 */
GBT_API int32_t gbt_sparse_entry_bytes(int32_t F, int32_t max_bins);
GBT_API int64_t gbt_sparse_capacity(int64_t nnz);
GBT_API size_t gbt_compress_sparse_workspace_bytes(int64_t n);
GBT_API int32_t gbt_compress_sparse_count(gbt_ctx *ctx, const uint16_t *sym, int64_t n, int32_t F,
                      int32_t missing_sym, uint32_t *rowptr_out, int64_t *nnz_out, void *workspace,
                      size_t workspace_bytes);
GBT_API int32_t gbt_compress_sparse(gbt_ctx *ctx, const uint16_t *sym, int64_t n, int32_t F, int32_t max_bins,
                      int32_t missing_sym, const uint32_t *rowptr, int64_t nnz, void *ent_out,
                      int64_t ent_capacity);

/* ---- Sec. 2.5 gradient evaluation (Eq. 1, Eq. 2) ------------------------ */

/* gpair_out[i] = (g, h) of margin[i], label[i]: logistic g = s - y, h = s(1-s)
 * with s = sigmoid(margin); squared error g = margin - y, h = 1.  All [dev],
 * n entries.  Asynchronous. */
GBT_API int32_t gbt_gradients(gbt_ctx *ctx, int32_t objective, const float *margin, const float *label,
                      int64_t n, float *gpair_out);

/* ---- Alg. 1 BuildPartialHistograms ------------------------------------- */

/* Rounds gpair[n] [dev] to fixed point: gq_out [dev] int32[n][2] =
 * (rint(g*scale[0]), rint(h*scale[1])), scale_out [host] double[2] the two
 * powers of two (chosen from max|g|, max h over the n rows).  A non-finite
 * value or a negative h is refused with GBT_EINVAL.
 * workspace [dev] >= 4096 bytes.  Synchronises the stream. */
GBT_API int32_t gbt_gpair_fixed(gbt_ctx *ctx, const float *gpair, int64_t n, int32_t *gq_out,
                        double *scale_out, void *workspace, size_t workspace_bytes);

/* Exact sums of gq over the node's rows -> sums_out [host] int64[2].
 * row_idx NULL = rows 0..n_rows-1.  workspace [dev] >= 4096 bytes.  Synchronises. */
GBT_API int32_t gbt_sum_gpair(gbt_ctx *ctx, const int32_t *gq, const uint32_t *row_idx, int64_t n_rows,
                      int64_t *sums_out, void *workspace, size_t workspace_bytes);

/*
 * hist_out[f][b] = (sum gq_g, sum gq_h) over the node's rows r with
 * sym(r,f) = b; the missing symbol is not accumulated (Sec. 2.1; Alg. 1
 * BuildPartialHistograms).
 *   packed, bits, n, F : the packed matrix [dev]
 *   B                  : bin stride (max_bins); every non-missing symbol < B
 *   row_idx [dev]      : the node's rows (uint32 ids < n), NULL = all n rows
 *   n_node_rows        : length of row_idx (ignored when NULL)
 *   gq [dev]           : int32[n][2] from gbt_gpair_fixed (|g| <= 2^26, 0 <= h <= 2^22)
 *   hist_out [dev]     : int64[F][B][2], overwritten
 * Asynchronous.
 */
GBT_API int32_t gbt_build_hist(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                       int32_t B, int32_t missing_sym, const uint32_t *row_idx, int64_t n_node_rows,
                       const int32_t *gq, int64_t *hist_out);

/* gbt_build_hist over sparse rows (gbt_compress_sparse): the node's rows are the
 * contiguous range [row_begin, row_begin + n_node_rows) of the n rows; absent
 * elements are missing and accumulate nowhere.  hist_out [dev] int64[F][B][2],
 * overwritten.  Asynchronous. */
GBT_API int32_t gbt_build_hist_sparse(gbt_ctx *ctx, const uint32_t *rowptr, const void *ent, int64_t n,
                       int32_t F, int32_t B, int64_t row_begin, int64_t n_node_rows, const int32_t *gq,
                       int64_t *hist_out);

/* out = parent - child, elementwise over `count` int64 values [dev] (the
 * sibling-subtraction trick: the larger child's histogram).  Asynchronous. */
GBT_API int32_t gbt_hist_subtract(gbt_ctx *ctx, const int64_t *parent, const int64_t *child, int64_t *out,
                          int64_t count);

/* out[f][b][c] = hist[f][b][c] / scale[c] as fp64 [dev].  Asynchronous. */
GBT_API int32_t gbt_hist_export_f64(gbt_ctx *ctx, const int64_t *hist, int32_t F, int32_t B,
                            const double *scale /* [host] double[2] */, double *out);

/* ---- Alg. 1 EvaluateSplit ---------------------------------------------- */

/*
 * Best split of one node from its histogram: an inclusive prefix scan over the
 * bins of every feature gives (GL, HL) of each candidate (Sec. 2.3), gain in
 * fp64.  The node's missing mass for feature f is (Gq, Hq) - sum_b hist[f][b];
 * it is tried on the right and, when non-zero, on the left.  Candidates are
 * ordered (feature, bin, right-before-left); a later one wins only with a
 * strictly larger gain.  A candidate needs HL, HR >= min_child_weight.  (Rows
 * are not counted here: a side without rows has mass exactly (0, 0), so such
 * a candidate can only come back with a gain <= 0, below what any grower of
 * this library accepts.)
 *   hist [dev], nb [dev] int32[F], Gq/Hq node totals (gbt_sum_gpair),
 *   scale [host] double[2], split_out [host].  workspace [dev] >= 4096 bytes.
 * Synchronises the stream.
 */
GBT_API int32_t gbt_eval_split(gbt_ctx *ctx, const int64_t *hist, const int32_t *nb, int32_t F, int32_t B,
                       int64_t Gq, int64_t Hq, const double *scale, const gbt_params *params,
                       gbt_split *split_out, void *workspace, size_t workspace_bytes);

/* ---- Alg. 1 RepartitionInstances --------------------------------------- */

GBT_API size_t gbt_partition_workspace_bytes(int64_t n_rows);

/*
 * Stable partition of row_idx[begin, end) [dev, in place]: first the rows with
 * sym(r, feature) <= bin (or the missing symbol when default_left), then the
 * others, both in their previous order.  *n_left_out [host] = size of the first
 * part.  Synchronises the stream.
 */
GBT_API int32_t gbt_partition(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                      uint32_t *row_idx, int64_t begin, int64_t end, int32_t feature, int32_t bin,
                      int32_t default_left, int32_t missing_sym, void *workspace,
                      size_t workspace_bytes, int64_t *n_left_out);

/*
 * gbt_partition for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments (without the workspace), same result, same
 * kernels; the scratch memory is a static device array inside the library, sized
 * for segments of at most GBT_PARTITION_STATIC_MAX_ROWS rows (about 17 MB, held
 * by every GPU the library runs on until the process ends).  A longer segment
 * is refused with GBT_EUNSUPPORTED and nothing is enqueued.  The call allocates
 * nothing.  Every call on one GPU uses that GPU's one array: calls that overlap
 * on one GPU (two contexts, two streams) race and must be serialised by the
 * caller.  The array keeps the last call's contents; no call depends on them.
 * Synchronises the stream.
 */
#define GBT_PARTITION_STATIC_MAX_ROWS (1 << 22)
GBT_API int32_t gbt_partition_static(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                      uint32_t *row_idx, int64_t begin, int64_t end, int32_t feature, int32_t bin,
                      int32_t default_left, int32_t missing_sym, int64_t *n_left_out);

/* ---- Alg. 1 as a whole -------------------------------------------------- */

GBT_API size_t gbt_grow_tree_workspace_bytes(int64_t n, int32_t F, int32_t bits, int32_t max_bins,
                                             int32_t max_depth);

/*
 * How gbt_grow_tree moves the rows of splitting nodes for this shape (for
 * profiling and tests; the result of gbt_grow_tree does not depend on it):
 *   0  three launches per level (flags, offsets, move); row ids travel with the
 *      rows and every node's rows keep their order
 *   1  one launch per level, order inside a node not kept, no ids (rows of at
 *      most 64 words)
 *   2  as 1, and the launch also builds one child's histogram of every split
 *      node (8-bit symbols, at most 16 features).  Depth-wise, most levels
 *      then leave the rows where they are (a pass reads them in place and
 *      adds up the rows of the children to be built, for up to two levels in
 *      a row) and every third level moves them over three levels of splits
 *      at once; see GBT_TUNE_PART_NOMOVE and GBT_TUNE_PART_CYCLE
 *   3  rows wider than 64 words are never moved: the nodes' row-id lists are
 *      partitioned (stable, three launches) and the histogram kernel gathers
 *      the rows by id from the packed matrix
 * track_rows: whether the caller passes row_idx_out.  It does not change the
 * answer unless the library was told (GBT_TUNE_ORDER_ROWS=0 in the environment
 * when the context was created) to produce row_idx_out by carrying the ids,
 * which needs form 0.
 * Negative: a GBT_E* code.
 */
GBT_API int32_t gbt_grow_tree_path(gbt_ctx *ctx, int32_t F, int32_t bits, int32_t max_bins, int32_t track_rows);

/*
 * Grows one tree depth-wise (Alg. 1 with the "closest to the root first"
 * policy): root histogram; per level evaluate the open nodes, partition the
 * rows of those that split (whole records -- symbols, gradient pair, row id --
 * move inside the workspace so that each node's rows stay contiguous), build
 * the histogram of one child of each split from its rows (the one with fewer
 * rows, tie -> left; where partition and histogram run as one pass, the one
 * with the smaller hessian sum) and get the other one by subtraction; sums are
 * exact integers, so the choice changes no value.  A node is
 * split iff it has a valid candidate with gain > max(gamma, GBT_GAIN_FLOOR) and
 * depth < max_depth.  Leaf weight = -G/(H+lambda), 0 where H+lambda = 0.
 *   packed, bits, n, F, missing_sym : packed matrix [dev]
 *   nb [dev] int32[F]; cuts [dev] float[F][max_bins-1] (for thresholds)
 *   gpair [dev] float2[n]
 *   tree_out [host]              caller-allocated arrays, see gbt_tree
 *   row_idx_out [dev] uint32[n]  final row order (may be NULL): what the stable
 *                                partitions of Alg. 1 leave of the list 0..n-1;
 *                                each node's rows are one ascending run, the
 *                                left child's run first.  Where the rows move
 *                                without ids (forms 1 and 2 above) the list is
 *                                made at the end: the rows sorted stably by
 *                                their leaf's place in left-to-right order
 *   leaf_of_row_out [dev] int32[n] leaf id per row (may be NULL).  In forms 1
 *                                and 2 it comes from one walk of the finished
 *                                tree over the packed matrix
 * Synchronises the stream.
 */
GBT_API int32_t gbt_grow_tree(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                      int32_t missing_sym, const int32_t *nb, const float *cuts, const float *gpair,
                      const gbt_params *params, gbt_tree *tree_out, uint32_t *row_idx_out,
                      int32_t *leaf_of_row_out, void *workspace, size_t workspace_bytes);

/*
 * Alg. 1 with the loss-guided policy of Sec. 2.3 ("highest gain first"): the open
 * leaf whose best split has the largest gain is expanded next (the smaller node id
 * on equal gains) until the tree has max_leaves leaves or no leaf is open.  A leaf is
 * open iff it has a valid candidate with gain > max(gamma, GBT_GAIN_FLOOR) and its
 * depth is below params->max_depth (any value >= 0 here).  Children get the next
 * two node ids at the moment of the expansion, so the k-th expansion creates nodes
 * 2k+1 and 2k+2.  Arguments, outputs, the NULL row_idx_out form and error behaviour
 * as for gbt_grow_tree; tree_out needs capacity >= 2*max_leaves - 1.
 * The kernels are those of the depth-wise loop.  Work is issued in rounds: the
 * leaf whose turn it is and a few more open leaves in gain order are expanded
 * together (a leaf's best split does not depend on when it is found), and the
 * tree follows the sequential rule over what is known, numbering children when
 * their parent's turn comes; expansions the budget never reaches are discarded.
 * The workspace holds histograms for those extra nodes (max_leaves/4, at least
 * 32 and at most 4096 expansions).
 */
GBT_API size_t gbt_grow_tree_lossguide_workspace_bytes(int64_t n, int32_t F, int32_t bits, int32_t max_bins,
                                                       int32_t max_leaves);
GBT_API int32_t gbt_grow_tree_lossguide(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                      int32_t missing_sym, const int32_t *nb, const float *cuts, const float *gpair,
                      const gbt_params *params, int32_t max_leaves, gbt_tree *tree_out, uint32_t *row_idx_out,
                      int32_t *leaf_of_row_out, void *workspace, size_t workspace_bytes);

/*
 * gbt_grow_tree (depth-wise) over sparse rows (gbt_compress_sparse): the same
 * tree as on the packed matrix of the same symbols -- an absent element is a
 * missing value.  Rows move without ids through one-launch unordered
 * partitions; leaf_of_row_out comes from a walk of the finished tree,
 * row_idx_out from a stable sort of the rows by leaf (both may be NULL).
 * nnz = rowptr[n].  Other arguments, outputs and errors as for gbt_grow_tree.
 * Synchronises the stream.
 */
GBT_API size_t gbt_grow_tree_sparse_workspace_bytes(int64_t n, int64_t nnz, int32_t F, int32_t max_bins,
                                                    int32_t max_depth);
GBT_API int32_t gbt_grow_tree_sparse(gbt_ctx *ctx, const uint32_t *rowptr, const void *ent, int64_t n,
                      int64_t nnz, int32_t F, const int32_t *nb, const float *cuts, const float *gpair,
                      const gbt_params *params, gbt_tree *tree_out, uint32_t *row_idx_out,
                      int32_t *leaf_of_row_out, void *workspace, size_t workspace_bytes);

/*
 * gbt_grow_tree_lossguide over sparse rows: the loss-guided policy of Sec. 2.3 with the
 * kernels of gbt_grow_tree_sparse; the same tree as gbt_grow_tree_lossguide grows on
 * the packed matrix of the same symbols.  Arguments as for gbt_grow_tree_sparse plus
 * max_leaves; tree_out needs capacity >= 2*max_leaves - 1.  Synchronises the stream.
 */
GBT_API size_t gbt_grow_tree_sparse_lossguide_workspace_bytes(int64_t n, int64_t nnz, int32_t F, int32_t max_bins,
                                                              int32_t max_leaves);
GBT_API int32_t gbt_grow_tree_sparse_lossguide(gbt_ctx *ctx, const uint32_t *rowptr, const void *ent, int64_t n,
                      int64_t nnz, int32_t F, const int32_t *nb, const float *cuts, const float *gpair,
                      const gbt_params *params, int32_t max_leaves, gbt_tree *tree_out, uint32_t *row_idx_out,
                      int32_t *leaf_of_row_out, void *workspace, size_t workspace_bytes);

/*
 * One boosting iteration as the loop of Fig. 1 runs it (Sec. 2.5, Alg. 1, Sec. 2.4 in
 * one call): gpair[r] = gradient pair of (margin_in[r], label[r]) under
 * params->objective (as gbt_gradients), one depth-wise tree on those pairs (as
 * gbt_grow_tree with row_idx_out = leaf_of_row_out = NULL), and
 * margin_out[r] = margin_in[r] + params->eta * weight[leaf(r)] (as gbt_predict with
 * that one tree on the packed matrix).  Results are those of the three calls, bit
 * for bit; done together they share two passes: the gradient kernel also finds the
 * bounds the fixed-point scales are chosen from, and the walk that updates the
 * margins also counts the rows of the last level's children (tree_out->n_rows).
 *   label, margin_in [dev] float[n]; margin_out [dev] float[n], may be margin_in
 *   gpair [dev] float2[n]  receives the iteration's gradient pairs
 *   workspace              gbt_grow_tree_workspace_bytes(n, F, bits, max_bins, max_depth)
 * Other arguments and errors as for gbt_grow_tree.  Synchronises the stream.
 */
GBT_API int32_t gbt_boost_round(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                      int32_t missing_sym, const int32_t *nb, const float *cuts, const float *label,
                      const float *margin_in, float *margin_out, float *gpair, const gbt_params *params,
                      gbt_tree *tree_out, void *workspace, size_t workspace_bytes);

/* ---- Sec. 2.4 prediction ------------------------------------------------ */

GBT_API size_t gbt_predict_workspace_bytes(const gbt_tree *trees, int32_t n_trees);

/*
 * margin[r] += eta * weight[leaf_t(r)] for t = 0..n_trees-1 in order, one row
 * per thread walking each tree from its root.  Rows come EITHER as the packed
 * symbols (packed != NULL: left iff sym <= bin, missing symbol -> default
 * child) OR as raw floats X[n][F] [dev] (packed == NULL: left iff
 * x < threshold, NaN -> default child); both give the same leaves on the
 * training matrix.  trees [host].  Synchronises the stream (the trees are
 * staged through the workspace).
 */
GBT_API int32_t gbt_predict(gbt_ctx *ctx, const gbt_tree *trees, int32_t n_trees, const uint32_t *packed,
                    int32_t bits, int32_t missing_sym, const float *X, int64_t n, int32_t F,
                    double eta, float *margin_inout, void *workspace, size_t workspace_bytes);

/* gbt_predict over sparse rows: left iff the row's symbol of the node's feature
 * is <= bin, an absent element -> default child.  workspace as for gbt_predict.
 * Synchronises the stream. */
GBT_API int32_t gbt_predict_sparse(gbt_ctx *ctx, const gbt_tree *trees, int32_t n_trees, const uint32_t *rowptr,
                      const void *ent, int64_t n, int32_t F, int32_t max_bins, double eta, float *margin,
                      void *workspace, size_t workspace_bytes);

/* ---- measurement -------------------------------------------------------- */

/* Kernel classes timed by the optional profiler. */
#define GBT_PROF_HIST_ROOT 0 /* histogram of all rows (no row-id list) */
#define GBT_PROF_HIST_NODE 1 /* histograms of levels >= 1 (the partition + histogram pass where that runs) */
#define GBT_PROF_PARTITION 2 /* moving or counting rows without a histogram */
#define GBT_PROF_EVAL 3      /* split evaluation, sibling subtraction included */
#define GBT_PROF_CLEAR 4     /* zero-fill of the children's histograms */
#define GBT_PROF_OTHER 5     /* scale search, fixed-point conversion, tree walks (leaf ids, prediction), row order */
/* The partition + histogram pass has four kernels; GBT_PROF_HIST_NODE holds the one that reads and writes
 * records (the levels that move rows, except the first), these two classes the others: */
#define GBT_PROF_HIST_FIRST 6   /* its first level, whose source is the caller's packed matrix */
#define GBT_PROF_HIST_INPLACE 7 /* its last one or two levels, whose records stay in place (one, then two histograms per workgroup) */
#define GBT_PROF_CLASSES 8

#define GBT_PROF_LEVELS 18 /* depths 0..16 of the nodes a launch builds histograms for, one spare */
typedef struct gbt_profile {
    double ms[GBT_PROF_CLASSES];        /* device time between HIP events around the launches */
    double bytes[GBT_PROF_CLASSES];     /* HBM bytes this library's design moves in those launches (whole records
                                           read and written where rows move) */
    int64_t launches[GBT_PROF_CLASSES]; /* timed launch groups */
    /* Bytes the method itself needs, whatever the design does: a histogram rows_built * (F*bits/8 + 8) for the
     * symbols and the gradient pair, + 4 per row where the node is a subset of the rows (its row id); a
     * repartition 4 + 4 + bits/8 per row of the split nodes (row id read and written, one symbol); a launch
     * that does both, the sum; a launch that only counts rows, bits/8 per row. */
    double alg_bytes[GBT_PROF_CLASSES];
    /* The histogram-building launches once more, by the depth of the nodes built (0 = the root): time, method
     * bytes, rows * features accumulated, launch groups. */
    double level_ms[GBT_PROF_LEVELS];
    double level_alg_bytes[GBT_PROF_LEVELS];
    double level_row_features[GBT_PROF_LEVELS];
    int64_t level_launches[GBT_PROF_LEVELS];
} gbt_profile;

/* Turns per-class device timing on or off (off by default).  While on, every
 * launch group of gbt_build_hist and gbt_grow_tree is bracketed by HIP events on
 * the context's stream.  gbt_profile_read synchronises the stream, adds up what
 * was recorded since the last reset into *out [host] and resets. */
GBT_API int32_t gbt_profile_enable(gbt_ctx *ctx, int32_t on);
GBT_API int32_t gbt_profile_read(gbt_ctx *ctx, gbt_profile *out);

/* The streaming-read ceiling of this GPU, measured here and now: a kernel that only reads `bytes` bytes of buf
 * [dev, 16-byte aligned] (whole 16-byte pieces, every byte once, nothing written) is launched `reps` >= 1
 * times on the context's stream between HIP events; *gbps_out [host] receives the best bytes / time in
 * GB/s.  The figure to hold beside a histogram kernel's achieved bandwidth: what HBM gives a kernel that does
 * nothing else.  workspace [dev] >= 4096 bytes.  Synchronises the stream. */
GBT_API int32_t gbt_measure_stream_read(gbt_ctx *ctx, const void *buf, size_t bytes, int32_t reps,
                                        double *gbps_out, void *workspace, size_t workspace_bytes);

#ifdef __cplusplus
}
#endif
#endif /* GBT_H */
