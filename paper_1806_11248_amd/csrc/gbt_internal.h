// Internal declarations shared by the translation units of libgbt.
// Not part of the ABI; include/gbt.h is.
#pragma once

#include <hip/hip_runtime.h>
#include <mutex>
#include <stdint.h>
#include <stdio.h>

#include <vector>

#include "gbt.h"

struct ProfSpan {
    int cls;
    double bytes;       // HBM bytes this library's design moves in the launch
    double alg_bytes;   // bytes the method itself needs (see gbt_profile); < 0: the same as `bytes`
    int level;          // depth of the nodes whose histograms the launch builds, -1: not a histogram launch
    double row_features;   // rows * features accumulated into those histograms
    hipEvent_t start, stop;
};

struct gbt_ctx {
    int device;
    hipStream_t stream;
    int num_cu;
    size_t lds_per_block;   // largest dynamic LDS a workgroup may ask for
    size_t lds_max;         // the most LDS one workgroup can be given (a kernel with one workgroup per CU and no static LDS)
    char *pinned;           // host staging for job tables and small read-backs
    size_t pinned_bytes;
    int hist_block;         // threads per histogram workgroup
    int hist_runtime_bits;  // 1: unpack with run-time shifts even where a compile-time kernel exists
    int part_fused;         // 1: one-launch record partition where it applies
    int lossguide_batch;    // open leaves a round of loss-guided growth expands at once (1: only the one whose turn it is)
    int part_nomove;        // partition + histogram path, depth-wise: 1: the last histogram level is built without moving rows; 2: the last two
    int part_cycle;         // same path: above the last two levels, rows are moved every third level only (keep, keep with two histograms, move three levels)
    int part_ids;           // 1: rows wider than 64 words are not moved: id lists are partitioned and the histogram kernel gathers
    int order_rows;         // 1: a caller's row order is made from the finished tree, so that it does not restrict the partition form
    int hist_fix;           // 1: the root histogram kernel also converts the gradient pairs where that applies
    int part_hist;          // 1: and the children's histograms in the same pass where that applies
    int hist_lds_kb;        // 0, or a cap on the LDS histogram of one workgroup (more workgroups per CU)
    int hist_lds_auto;      // 1: hist_lds_kb is the default, which a shape of two to four feature tiles may double to save a tile
    int hist_jobs_per_cu;   // histogram workgroups to aim for per compute unit and launch
    int move_max_words;     // rows of more 32-bit words than this are never moved: only their ids are partitioned
    int hist_merge_ratio;   // LDS additions a bin should receive, on average, per value a job merges into HBM
    int hist8;              // 1: the root histogram of 8-bit symbols with at most 16 features takes kernels_hist8.hip
    int hist8_stagger;      // its workgroups on one compute unit get unequal shares of rows: spread in 1/256ths
    int sparse_jobs_per_cu; // row pieces per compute unit and launch of the sparse-row histogram kernel
    int sparse_tiled;       // 1: keep the sparse-row LDS histogram under hist_lds_kb even where all ids would fit
    char *part_static;      // this device's copy of the static partition scratch (gbt_partition_static), or NULL
    size_t up_off;          // next free byte of the upload ring (first half of `pinned`)
    char err[512];
    bool profiling;
    std::vector<ProfSpan> *spans;       // recorded, not yet read
    std::vector<hipEvent_t> *free_events;
};

// Brackets a launch group with events when profiling is on (no-ops otherwise).
// bytes: what the design moves; alg_bytes: what the method needs (< 0: the same); level, row_features: for
// launches that build histograms (see ProfSpan).  Returns the span's index for gbt_prof_patch, -1 when off.
int gbt_prof_begin(gbt_ctx *ctx, int cls, double bytes, double alg_bytes = -1.0, int level = -1,
                   double row_features = 0.0);
void gbt_prof_end(gbt_ctx *ctx);
// Figures of a span that are only known after its launch has been waited for (rows of the built children).
void gbt_prof_patch(gbt_ctx *ctx, int span, double alg_bytes, double row_features);

#define GBT_STAGING_BYTES (8u << 20)

// ---- error plumbing -------------------------------------------------------
int32_t gbt_fail(gbt_ctx *ctx, int32_t code, const char *fmt, ...);

#define GBT_HIP(ctx, call)                                                                  \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return gbt_fail((ctx), GBT_EHIP, "%s: %s (%s:%d)", #call, hipGetErrorString(e_), \
                            __FILE__, __LINE__);                                            \
    } while (0)

#define GBT_REQUIRE(ctx, cond, code, ...) \
    do {                                  \
        if (!(cond)) return gbt_fail((ctx), (code), __VA_ARGS__); \
    } while (0)

static constexpr inline size_t gbt_align(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// ---- job descriptors (host-built, read by kernels) --------------------------
// One workgroup of the histogram kernel: rows [row_begin, row_begin+n_rows) of
// the level's row-id buffer (or of the matrix itself when there is no row-id
// buffer), features [f0, f0+ft), accumulated into the histogram at hist_off.
struct HistJob {
    uint64_t hist_off;   // offset of the node's histogram in int64 units
    uint32_t row_begin;
    uint32_t n_rows;
    uint32_t f0, ft;
    uint32_t pad0;   // 1: this is the only job of its (node, feature tile): it may store its bins instead of adding them
    uint32_t pad1;
};

// One node for the split kernel.
struct EvalNode {
    uint64_t hist_off;
    int64_t Gq, Hq;
    // sibling subtraction folded into the evaluation: when parent_off != GBT_NO_HIST the node's histogram
    // does not exist yet; the kernel makes it as parent - built (int64 units, like hist_off), stores it
    // at hist_off and evaluates it in the same pass
    uint64_t parent_off, built_off;
};
#define GBT_NO_HIST (~0ull)

// One segment for the partition kernels.
struct PartJob {
    uint32_t seg_begin, seg_len;
    uint32_t feature, bin;
    uint32_t default_left;
    uint32_t tile_begin;   // index of the segment's first tile in the level's tile arrays
    uint32_t n_tiles;
    uint32_t pad;          // partition + histogram pass: the child to build (1 left, 0 right, 2 none)
    uint64_t hist_off;     // same pass: that child's histogram in the pool (int64 units)
};

// One parent segment for the two-level row count: the rows still lie in the parent's order, its split
// (index 0) tells each row's child, and the children's splits (1: left child, 2: right child; has[] = 0
// for a child that is not split) tell the row's side there.
struct CountJob {
    uint32_t seg_begin, seg_len;
    uint32_t tile_begin, n_tiles;
    // the splits below the segment in heap order: 0 the segment's own, 1 and 2 its left / right child's,
    // 3..6 the grandchildren's (left to right); has[p]: node p splits (0 always does)
    uint32_t feature[7], bin[7], default_left[7];
    uint32_t has[7];
    uint32_t pad;
};

// One segment for the histogram pass over rows that were not moved at the segment's own split: the
// split tells each row's child (0 left, 1 right), the child's split (if it has one) the row's side there.
// Of each splitting child's two children one histogram is built (build[c]: 1 the left, 0 the right)
// into hist_off[c]; cursor word 2 * job + c counts the child's left rows.
struct Hist2Job {
    uint32_t seg_begin, seg_len;
    uint32_t tile_begin, n_tiles;   // in spans of rows_per_span rows
    uint32_t feature[3], bin[3], default_left[3];
    uint32_t has[2], build[2];
    uint32_t pad;
    uint64_t hist_off[2];
};

// One segment for the pass that puts rows in order again after two levels in place (gbt_launch_move3): the splits
// below the segment in heap order as in CountJob (0 the segment's own, 1 and 2 its children's, 3..6 the
// grandchildren's; has[p] = 0: node p does not split and its rows are dropped), and the row range of each
// grandchild in the destination, inside which its left rows are stored from the front and its right rows from the
// back.  Cursor word 4 * job + g counts grandchild g's left (low half) and right (high half) rows.
struct Move3Job {
    uint32_t seg_begin, seg_len;
    uint32_t tile_begin, n_tiles;   // in spans of rows_per_span rows
    uint32_t feature[7], bin[7], default_left[7];
    uint32_t has[7];
    uint32_t node_begin[4], node_len[4];
};
static_assert(sizeof(Move3Job) % 4 == 0 && sizeof(Move3Job) / 4 <= 64, "staged into LDS by the first wave");

// One leaf segment for the final gather.
struct LeafSeg {
    uint32_t seg_begin;
    uint32_t node;
    uint32_t buf;   // which of the two row-id buffers holds the segment
    uint32_t len;
};

#define GBT_PART_TILE 2048   // rows per partition workgroup
#define GBT_PART_BLOCK 256

// ---- kernel launchers (each returns the hipGetLastError of its launches) ---
hipError_t gbt_launch_fill_u64(hipStream_t s, uint64_t *p, uint64_t v, int64_t count);
hipError_t gbt_launch_iota_u32(hipStream_t s, uint32_t *p, int64_t count);
hipError_t gbt_launch_stream_read(hipStream_t s, const void *buf, int64_t bytes, uint32_t *sink);
// out2 [dev] uint32[4]: bits of the largest |g|, of the largest |h|, 1 if some h < 0, ~(bits of the smallest |h|)
hipError_t gbt_launch_absmax(hipStream_t s, const float *gpair, int64_t n, uint32_t *out2);
// sums_out (may be NULL): int64[2] [dev] receiving the exact totals of gq (zeroed by the launcher).
hipError_t gbt_launch_to_fixed(hipStream_t s, const float *gpair, int64_t n, double sg, double sh,
                               int32_t *gq, int64_t *sums_out);
hipError_t gbt_launch_sum_gq(hipStream_t s, const int32_t *gq, const uint32_t *row_idx, int64_t n_rows,
                             int64_t *out2 /* zeroed by the launcher */);
// bounds (may be NULL): 4 * kBoundsStride words, cleared here; word k * kBoundsStride receives what word k of
// gbt_launch_absmax's output holds for these pairs
constexpr int kBoundsStride = 32;
hipError_t gbt_launch_gradients(hipStream_t s, int objective, const float *margin, const float *label,
                                int64_t n, float *gpair, uint32_t *bounds = nullptr);
hipError_t gbt_launch_subtract_one(hipStream_t s, const int64_t *parent, const int64_t *child,
                                   int64_t *out, int64_t count);
hipError_t gbt_launch_export(hipStream_t s, const int64_t *hist, int64_t count, double inv_sg,
                             double inv_sh, double *out);

// packed: a bit stream whose row r starts at bit r*stride_bits (the canonical packed matrix has
// stride_bits = F*bits; the word-aligned working copy of the grow loop 32*ceil(F*bits/32));
// n_words: readable 32-bit words of `packed`; row_idx NULL: job rows are matrix rows.
hipError_t gbt_launch_hist(gbt_ctx *ctx, const uint32_t *packed, int bits, int64_t stride_bits, int64_t n_words,
                           int64_t n, int B, uint32_t missing, const uint32_t *row_idx, const int32_t *gq,
                           int64_t *hist_pool, const HistJob *jobs, int n_jobs, int max_ft,
                           // every row's rounded h equals hq_uniform: kernels that have a form for it (symbol widths
                           // other than 8 bits) count rows instead of summing h; jobs then hold at most
                           // gbt_histw_max_rows(true) rows
                           bool uniform_h = false, int32_t hq_uniform = 0);
int gbt_histw_max_rows(bool uniform_h);
hipError_t gbt_launch_histw(gbt_ctx *ctx, const uint32_t *packed, int bits, int64_t stride_bits, int64_t n_words,
                            int64_t n, int B, uint32_t missing, const uint32_t *row_idx, const int32_t *gq,
                            int64_t *hist_pool, const HistJob *jobs, int n_jobs, int max_ft, bool uniform_h,
                            int32_t hq_uniform);
// Largest feature tile whose LDS histogram fits, and the per-job row count to aim for.
int gbt_hist_feature_tile(const gbt_ctx *ctx, int F, int B, int64_t n_rows = 0);   // n_rows: rows of the matrix the tiles are for (0: unknown)

// out receives n_nodes * n_chunks records (node-major); gbt_eval_chunks picks n_chunks.
int gbt_eval_chunks(int F, int n_nodes, size_t record_budget_bytes);
// `out` may be host memory the device can address (the pinned staging): the records are then where the
// host reads them when the launch has finished, without a copy.  tail: n 64-bit words copied from src to
// dst (again possibly such host memory) by the same launch, and src cleared behind the copy if `clear`
// (the row cursors of the partition that ran before, returned and made ready for the next one).
// clear_slot >= 0: the launch also zeroes the histograms that the evaluated nodes' children would
// accumulate into if their parents split: pool slots clear_slot + 2 i and clear_slot + 2 i + 1 for node
// i, as far as they lie below clear_slot_end (a slot is F * B * 2 values).
struct EvalTail {
    unsigned long long *src, *dst;
    int n, clear;
    int64_t clear_slot, clear_slot_end;
    int src_stride = 1;   // word i is src[i * src_stride]
    int skip_store = 0;   // 1: a histogram made by subtraction is evaluated but not stored (nothing below these nodes
                          // will subtract from it: their children are leaves)
};
// The cursors of the passes that partition and build histograms in one launch lie one per 128-byte line
// (index * kCursorStride): atomics on words of one line take turns as if they were one address.
constexpr int kCursorStride = 16;
hipError_t gbt_launch_eval(hipStream_t s, int64_t *hist_pool, const EvalNode *nodes, int n_nodes,
                           const int32_t *nb, int F, int B, int n_chunks, double inv_sg, double inv_sh,
                           double lambda, double mcw, gbt_split *out, EvalTail tail = EvalTail{nullptr, nullptr, 0, 0, -1, 0});

hipError_t gbt_launch_partition(hipStream_t s, const uint32_t *packed, int bits, int64_t stride_bits, int64_t n,
                                uint32_t missing, const uint32_t *src, uint32_t *dst,
                                const PartJob *jobs, int n_jobs, int total_tiles, uint64_t *masks,
                                uint32_t *tile_left, uint32_t *n_left_out);

// A set of rows in some order: symbols (row p starts at bit p*stride_bits), fixed-point gradient
// pairs and original row ids (NULL: the id of position p is p).  The *_rw members are the same
// addresses for a set that may be written.
struct GbtRows {
    const uint32_t *sym;
    int64_t stride_bits, n_words;
    const int32_t *gq;
    const uint32_t *id;
    uint32_t *sym_rw;
    int32_t *gq_rw;
    uint32_t *id_rw;
};
// Stable partition of the jobs' segments of `src` into `dst` (records move, see kernels_partition.hip).
// ids_only: move the row ids alone (the segments' children will not be read again).
hipError_t gbt_launch_partition_records(hipStream_t s, const GbtRows &src, const GbtRows &dst, int bits, int row_bits,
                                        int64_t n, uint32_t missing, int what, const PartJob *jobs,
                                        int n_jobs, int total_tiles, uint64_t *masks, uint32_t *tile_left,
                                        uint32_t *n_left_out);
// `what` above: move whole records, move only the ids, or only count the left rows of every job
enum { GBT_PART_RECORDS = 0, GBT_PART_IDS = 1, GBT_PART_COUNT = 2 };
// The same move of whole records in one launch for a caller that does not need the row order
// (and no ids): rows narrow enough (gbt_partition_fused_ok), tiles of gbt_partition_fused_tile(dst)
// rows (PartJob.tile_begin / n_tiles count those).  cursor: one word per job, cleared by the
// launcher; after the launch its low half is the job's n_left.  Inside a child the rows of one
// tile keep their order, the tiles' order is arbitrary.
bool gbt_partition_fused_ok(const GbtRows &dst);
int gbt_partition_fused_tile(const GbtRows &dst);
hipError_t gbt_launch_partition_fused(hipStream_t s, const GbtRows &src, const GbtRows &dst, int bits, int row_bits,
                                      uint32_t missing, const PartJob *jobs, int n_jobs, int total_tiles,
                                      unsigned long long *cursor);
// The root histogram straight from the fp32 gradient pairs (8-bit symbols, one feature tile of at
// most 16 features, jobs that cover rows [0, n) exactly once: gbt_hist_fix_ok): rounds each pair to
// fixed point with the given scales, stores it to gq_out and adds the totals into sums_out[2].
bool gbt_hist_fix_ok(int bits, int64_t stride_bits, int max_ft, int n_ftiles);
hipError_t gbt_launch_hist_fix(gbt_ctx *ctx, const uint32_t *packed, int64_t stride_bits, int64_t n_words, int64_t n,
                               int B, uint32_t missing, const float *gpair, double sg, double sh, int32_t *gq_out,
                               int64_t *sums_out, int64_t *hist_pool, const HistJob *jobs, int n_jobs, int max_ft);
// The histogram of ALL n rows of a packed matrix with 8-bit symbols and F <= 16 features (kernels_hist8.hip).
// The pairs come as fixed-point gq (gpair == NULL), or as fp32 gpair, which the kernel rounds itself:
// mode 1 through fp64, mode 2 in fp32 (only where gbt_fix32_ok(sg, sh)); gq_out (may be NULL) receives the
// rounded pairs; sums (may be NULL) int64[gbt_hist8_max_jobs()][2] receives one pair of partial totals per
// workgroup ([0, *n_jobs_out) are written; their sum is the total of all rows).  uniform_h: every
// row's rounded h equals hq_uniform (the caller has checked that all fp32 h are equal).  hist_out must be zero.
// A launch that asks for more dynamic LDS than the default limit of a launch first raises the kernel's limit.
// That limit is one value per kernel for the whole process, so the raise and the launch it serves happen under
// one process-wide lock: a concurrent launch of the same kernel from another context cannot lower it in between.
// Declare the guard before the attribute call and keep it alive until the kernel has been launched.
std::recursive_mutex &gbt_lds_mutex();
struct GbtLdsGuard {
    bool needed;
    std::unique_lock<std::recursive_mutex> lock;
    explicit GbtLdsGuard(size_t lds) : needed(lds > 64u * 1024u) {
        if (needed) lock = std::unique_lock<std::recursive_mutex>(gbt_lds_mutex());
    }
};

struct Hist8Pairs {
    const float *gpair;
    const int32_t *gq;
    int32_t *gq_out;
    double sg, sh;
    int mode;
    int uniform_h;
    int32_t hq_uniform;
    int64_t *sums;
};
bool gbt_hist8_ok(int bits, int F, int n_ftiles, int64_t n, int64_t n_words);
bool gbt_fix32_ok(double sg, double sh);
int gbt_hist8_max_jobs();
// filter (may be NULL): only the rows on one side of a split are added -- the histogram of one child of the root
// with the rows staying in the matrix; hist_out must have been cleared; *lefts (device, cleared by the caller)
// receives the number of rows that go left.  Pairs as fixed point (p.gq) or fp32 with mode 2.
struct Hist8Filter {
    int feature, bin, default_left;
    int take_left;               // 1: the left rows are added, 0: the right rows
    unsigned long long *lefts;
};
hipError_t gbt_launch_hist8(gbt_ctx *ctx, const uint32_t *packed, int64_t n, int F, int B, uint32_t missing,
                            const Hist8Pairs &p, int64_t *hist_out, int *n_jobs_out = nullptr,
                            const Hist8Filter *filter = nullptr);
hipError_t gbt_launch_hist8_records(gbt_ctx *ctx, const uint32_t *records, int F, int B, uint32_t missing,
                                    const PartJob *jobs, int n_jobs, int n_spans, uint32_t rows_per_span, int64_t *pool,
                                    int32_t hq_uniform);
// Partition and the histogram of one child of every job in one pass (8-bit symbols, at most 16
// features, the bins of all features in one LDS tile: gbt_part_hist_ok).  No ids, order inside a
// child not kept.  Rows travel as records of gbt_part_hist_record_words(F) words (symbols, padding,
// the fixed-point pair in the last 7 bytes); src_records == NULL: the source is the packed matrix
// (rows of F bytes) with the pairs in gq.  PartJob.tile_begin / n_tiles count spans of rows_per_span
// rows (a multiple of gbt_part_hist_tile()); PartJob.pad / hist_off name the child to build, whose
// histogram must have been cleared.
// dst_records == NULL: nothing is moved (the children's rows stay interleaved in the parent's segment);
// the histogram is built and the low word of each cursor counts the left rows.
// The cursors (one 64-bit word per job) are cleared here unless the caller says they are zero already.
bool gbt_part_hist_ok(const gbt_ctx *ctx, int bits, int F, int B);
// Rows of 8-bit symbols, row p at byte p * stride_bytes of `rows`.  levels = 1: counts[2 * j + c] = rows
// of job j's child c that go left at that child's split; levels = 2: counts[4 * j + t] the same for
// grandchild t (heap position 3 + t).  Rows that reach a node without a split on their way are not
// counted.  counts is cleared here.
int gbt_count2_tile();
hipError_t gbt_launch_count2(hipStream_t s, const uint8_t *rows, int64_t stride_bytes, uint32_t missing,
                             const CountJob *jobs, int n_jobs, int n_tiles, uint32_t *counts, int levels = 1,
                             bool records_ok = false);   // records_ok: rows are records of the partition + histogram pass
// The histogram pass over record segments that stay in place for a second level (Hist2Job); 8-bit symbols,
// at most 16 features, two LDS histograms per workgroup (gbt_hist2_ok).  cursor: 2 words per job, cleared
// here unless the caller says they are zero; the built children's histograms must have been cleared.
bool gbt_hist2_ok(const gbt_ctx *ctx, int F, int B);
hipError_t gbt_launch_hist2(gbt_ctx *ctx, const uint32_t *records, int F, int B, uint32_t missing,
                            const Hist2Job *jobs, int n_jobs, int n_spans, uint32_t rows_per_span,
                            unsigned long long *cursor, int64_t *hist_pool, bool cursors_are_zero = false,
                            int hq_uniform = -1);   // >= 0: every row has this hessian (fixed point): bins count rows
// The pass that moves the records of segments whose rows stayed in place for two levels to their grandchildren's
// children (Move3Job); records of at most 16 byte symbols.  dst_rows: rows the destination holds (a store past it
// is skipped).  cursor: 4 words per job, cleared here unless the caller says they are zero.
int gbt_move3_tile();
hipError_t gbt_launch_move3(gbt_ctx *ctx, const uint32_t *src_records, uint32_t *dst_records, int64_t dst_rows, int F,
                            uint32_t missing, const Move3Job *jobs, int n_jobs, int n_spans, uint32_t rows_per_span,
                            unsigned long long *cursor, bool cursors_are_zero = false);
// The same over two levels of splits (the segment's own and its children's: Move3Job entries 0..2, targets 0 and 1)
// with the rows taken from the caller's packed matrix and pair array (gq, or fp32 pairs rounded with sg, sh as in
// gbt_launch_part_hist) and written as records: for a segment whose rows stayed in the matrix at its split.
hipError_t gbt_launch_move2_first(gbt_ctx *ctx, const uint32_t *packed, int64_t packed_words, const int32_t *gq,
                                  const float *gpair_fp32, double sg, double sh, uint32_t *dst_records, int64_t dst_rows, int F,
                                  uint32_t missing, const Move3Job *jobs, int n_jobs, int n_spans, uint32_t rows_per_span,
                                  unsigned long long *cursor, bool cursors_are_zero = false);
int gbt_part_hist_tile();
int gbt_part_hist_record_words(int F);
hipError_t gbt_launch_part_hist(gbt_ctx *ctx, const uint32_t *packed, int64_t packed_words, const int32_t *gq,
                                const uint32_t *src_records, uint32_t *dst_records, int F, int B, uint32_t missing,
                                const PartJob *jobs, int n_jobs, int n_spans, uint32_t rows_per_span,
                                unsigned long long *cursor, int64_t *hist_pool, bool cursors_are_zero = false,
                                // first level only: the pairs are these fp32 pairs (not gq), rounded in the pass with
                                // the scales sg, sh, for which gbt_fix32_ok must hold
                                const float *gpair_fp32 = nullptr, double sg = 1.0, double sh = 1.0,
                                // >= 0: every row has this hessian (fixed point): bins count rows instead of adding hessians
                                int hq_uniform = -1);
// LeafSeg.buf: 0/1 = id buffers buf0/buf1, 2 = the id of position p is p.
hipError_t gbt_launch_leaf_gather(hipStream_t s, const uint32_t *buf0, const uint32_t *buf1,
                                  const LeafSeg *segs, int n_segs, int64_t n, uint32_t *row_idx_out,
                                  int32_t *leaf_of_row);

// Row ids in leaf order from each row's leaf: a stable sort of the positions 0..n-1 by
// rank_tbl[leaf[row]] (n_nodes table entries, ranks below n_ranks).  key_tmp / val_tmp: two buffers of
// n words each, touched only when n_ranks > 256; ws: gbt_order_ws(n) bytes.
size_t gbt_order_ws(int64_t n);
hipError_t gbt_launch_order_rows(hipStream_t s, const int32_t *leaf, const uint32_t *rank_tbl, uint32_t n_nodes,
                                 uint32_t n_ranks, int64_t n, uint32_t *key_tmp[2], uint32_t *val_tmp[2], char *ws,
                                 uint32_t *row_idx_out);

// sparse rows (kernels_sparse.hip): rowptr + global bin ids of ent_bytes = 2 or 4 bytes each, see there
int64_t gbt_sparse_scan_tiles(int64_t n);
hipError_t gbt_launch_sparse_rowptr(hipStream_t s, const uint16_t *sym, int64_t n, int F, uint32_t missing,
                                    uint32_t *rowptr, uint64_t *tile_ws, uint64_t *total_dev);
hipError_t gbt_launch_sparse_fill(hipStream_t s, const uint16_t *sym, int64_t n, int F, int B, uint32_t missing,
                                  const uint32_t *rowptr, void *ent, int ent_bytes, int64_t nnz, int64_t capacity);
int gbt_sparse_hist_tile(const gbt_ctx *ctx, int64_t bins);
// HistJob.f0 / ft: the job's range of global bin ids
hipError_t gbt_launch_sparse_hist(gbt_ctx *ctx, const uint32_t *rowptr, const void *ent, int ent_bytes, const int32_t *gq,
                                  int64_t *pool, const HistJob *jobs, int n_jobs, int max_glen, bool tiled);

// Unordered partition of sparse rows, one launch per level (PartJob as for the dense forms; tiles of
// gbt_sparse_part_tile() rows).  cursor: two 64-bit words per job, cleared here; afterwards the low
// word of cursor[2 * j] is job j's number of left rows.  move == false: only that count.
int gbt_sparse_part_tile();
hipError_t gbt_launch_sparse_partition(hipStream_t s, const uint32_t *src_rowptr, const void *src_ent, int ent_bytes,
                                       const int32_t *src_gq, uint32_t *dst_rowptr, void *dst_ent,
                                       int32_t *dst_gq, int B, bool move, const PartJob *jobs, int n_jobs,
                                       int n_tiles, unsigned long long *cursor);
struct DevTree;
hipError_t gbt_launch_sparse_walk(hipStream_t s, const char *ws, const DevTree *trees, int n_trees,
                                  const uint32_t *rowptr, const void *ent, int ent_bytes, int64_t n, int B, double eta,
                                  float *margin, int32_t *leaf_out, int max_nodes);

hipError_t gbt_launch_compress(hipStream_t s, const uint16_t *sym, int64_t n_elems, int bits,
                               uint32_t *packed, int64_t n_words);

struct DevTree {   // one tree's arrays inside the predict workspace (offsets in bytes)
    int32_t n_nodes;
    int32_t pad;   // the tree's depth (steps of its longest root-to-leaf walk)
    uint64_t feature, bin, default_left, left, right, threshold, weight;
};
hipError_t gbt_launch_predict(hipStream_t s, const char *ws, const DevTree *trees, int n_trees,
                              const uint32_t *packed, int bits, uint32_t missing, const float *X,
                              int64_t n, int F, double eta, float *margin, int32_t *leaf_out, int max_nodes,
                              bool compact_ok, uint32_t *node_rows = nullptr,
                              const float *margin_src = nullptr);   // leaf_out != NULL: store each row's leaf id instead of updating margin
// node_rows, margin_src (one tree, and only where gbt_predict_counts_ok): count the rows that end in every node into
// node_rows[node * kNodeRowsStride] (zeroed by the caller); margin[r] = margin_src[r] + eta * weight
constexpr int kNodeRowsStride = 32;   // words between two nodes' row counters (gbt_launch_predict's node_rows)
bool gbt_predict_counts_ok(bool packed, int bits, int F, int max_nodes, bool compact_ok);
// compact_ok: every split node has right == left + 1, feature < 2^20 and bin < 4096

// Many trees on raw floats in one pass over the rows (kernels_misc.hip).  A node is 8 bytes:
// meta = left child's id inside its tree (15 bits) | default_left << 15 | step << 16 | feature << 17,
// next = left + (go left ? 0 : step); a leaf has step 0 and left = its own id.  tree_off[t] = first
// node of tree t in nodes / wts (tree_off[n_trees] = total); group_end[g] = one past the last tree of
// group g; no group has more than cap_nodes nodes.
struct gbt_batch_node {
    float thr;
    uint32_t meta;
};
int gbt_predict_batch_max_features();
hipError_t gbt_launch_predict_raw_batched(hipStream_t s, const gbt_batch_node *nodes, const double *wts,
                                          const int32_t *tree_off, const int32_t *tree_depth,
                                          const int32_t *group_end, int n_groups, int cap_nodes, const float *X,
                                          int64_t n, int F, double eta, float *margin);

// Four consecutive words with ONE load instruction at 4-byte alignment (rows of packed symbols start at any byte).
typedef uint32_t gbt_u32x4 __attribute__((ext_vector_type(4), aligned(4)));
template <int N>
__device__ __forceinline__ void load_words(uint32_t (&x)[N], const uint32_t *p) {
    static_assert(N >= 1 && N <= 5, "a 16-byte window and the word behind it");
    if (N >= 4) {
        const gbt_u32x4 v = *(const gbt_u32x4 *)p;
        x[0] = v.x;
        x[1] = v.y;
        x[2] = v.z;
        x[3] = v.w;
        if (N == 5) x[N - 1] = p[4];
    } else {
#pragma unroll
        for (int k = 0; k < N; ++k) x[k] = p[k];
    }
}
constexpr int kHShift = 30;                        // width of the h field
constexpr uint32_t kHMask = (1u << kHShift) - 1u;


// quantise
hipError_t gbt_quantise_run(gbt_ctx *ctx, const float *X, const int64_t *indptr, const int32_t *indices,
                            const float *values, int64_t n, int F, int64_t n_values, int B, float *cuts,
                            int32_t *nb, uint16_t *sym, int32_t *max_value, int32_t *missing_sym,
                            char *ws, size_t ws_bytes, int32_t *status, uint32_t *packed = nullptr,
                            int64_t packed_cap_words = 0, int32_t *bits_out = nullptr);
size_t gbt_quantise_ws(int64_t n, int F, int64_t n_values, int B);
