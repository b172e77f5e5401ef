// RepartitionInstances (Alg. 1: "sort training instances into leaf nodes based
// on previous split") as a stable partition of row-id segments.
//
// All splitting nodes of a level are handled by the same three launches:
//   1. flag   : one workgroup per 2048-row tile gathers the split feature's
//               symbol of each row from the packed matrix, decides left/right,
//               stores the decision as wave ballots (one bit per row) and the
//               tile's count of left rows;
//   2. scan   : one workgroup per segment turns its tile counts into exclusive
//               offsets and the segment's n_left;
//   3. scatter: each tile recomputes every row's rank from the ballots
//               (popcounts below the lane + an LDS scan over the tile's 32
//               ballot words) and writes it to its place in the other buffer.
// Ranks are taken in row order, so both halves keep their order (stable).
// No workgroup waits on another one.
//
// Two scatter flavours share the flag and scan kernels:
//   * ids only  (gbt_partition): row ids move, the matrix stays where it is;
//   * records   (the grow loop): each row's symbols, fixed-point gradient pair
//     and id move together into a second set of buffers, so that every node's
//     rows stay physically contiguous and the next level's histogram and flag
//     passes stream through HBM instead of gathering 64-byte sectors per row.
//     Destination rows start on 32-bit word boundaries.
#include "gbt_internal.h"

namespace {

constexpr int kTile = GBT_PART_TILE;
constexpr int kBlock = GBT_PART_BLOCK;
constexpr int kWordsPerTile = kTile / 64;       // 32 ballot words
constexpr int kRowsPerThread = kTile / kBlock;  // 8
static_assert(kBlock == 256 && kTile == 2048, "index arithmetic below assumes 4 waves x 8 steps");

// the job whose tile range contains `tile` (jobs are sorted by tile_begin)
__device__ inline int find_job(const PartJob *jobs, int n_jobs, uint32_t tile) {
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].tile_begin <= tile) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ inline uint32_t load_symbol(const uint32_t *packed, uint64_t bp, int bits, uint32_t mask) {
    const uint32_t *w = packed + (bp >> 5);
    const uint32_t sh = (uint32_t)(bp & 31);
    uint32_t v = w[0] >> sh;
    if (sh + (uint32_t)bits > 32u) v |= w[1] << (32u - sh);   // the element straddles into the next word
    return v & mask;
}

// src == NULL: the segment's rows are matrix rows seg_begin .. seg_begin+seg_len-1
__global__ __launch_bounds__(kBlock) void part_flag_kernel(
    const uint32_t *__restrict__ packed, int bits, int64_t stride_bits, int64_t n, uint32_t missing,
    const uint32_t *__restrict__ src, const PartJob *__restrict__ jobs, int n_jobs,
    uint64_t *__restrict__ masks, uint32_t *__restrict__ tile_left) {
    const uint32_t tile = blockIdx.x;
    const PartJob job = jobs[find_job(jobs, n_jobs, tile)];
    const uint32_t t_in_seg = tile - job.tile_begin;
    const uint32_t base = t_in_seg * kTile;   // first row of the tile inside the segment
    const uint32_t mask = (1u << bits) - 1u;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t count = 0;
#pragma unroll
    for (int j = 0; j < kRowsPerThread; ++j) {
        const uint32_t off = base + (uint32_t)j * kBlock + threadIdx.x;
        bool left = false;
        if (off < job.seg_len) {
            const uint64_t p = (uint64_t)job.seg_begin + off;
            const uint64_t r = src ? (uint64_t)src[p] : p;
            if (r < (uint64_t)n) {
                const uint32_t s = load_symbol(packed, r * (uint64_t)stride_bits + (uint64_t)job.feature * bits, bits, mask);
                left = (s == missing) ? (job.default_left != 0) : (s <= job.bin);
            }
        }
        const uint64_t ballot = __ballot(left);
        if (lane == 0) masks[(uint64_t)tile * kWordsPerTile + (j * (kBlock / 64) + wave)] = ballot;
        count += (uint32_t)__popcll(ballot);   // same value in every lane of the wave
    }
    __shared__ uint32_t wsum[kBlock / 64];
    if (lane == 0) wsum[wave] = count;
    __syncthreads();
    if (threadIdx.x == 0) tile_left[tile] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

__global__ __launch_bounds__(kBlock) void part_scan_kernel(const PartJob *__restrict__ jobs,
                                                           uint32_t *__restrict__ tile_left,
                                                           uint32_t *__restrict__ n_left_out) {
    const PartJob job = jobs[blockIdx.x];
    __shared__ uint32_t wtot[kBlock / 64];
    __shared__ uint32_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint32_t t0 = 0; t0 < job.n_tiles; t0 += kBlock) {
        const uint32_t t = t0 + threadIdx.x;
        const uint32_t v = t < job.n_tiles ? tile_left[job.tile_begin + t] : 0;
        uint32_t x = v;
        for (int d = 1; d < 64; d <<= 1) {
            uint32_t y = (uint32_t)__shfl_up((int)x, d);
            if (lane >= d) x += y;
        }
        if (lane == 63) wtot[wave] = x;
        __syncthreads();
        uint32_t before = carry_s;
        for (int w = 0; w < wave; ++w) before += wtot[w];
        if (t < job.n_tiles) tile_left[job.tile_begin + t] = before + x - v;   // exclusive
        __syncthreads();
        if (threadIdx.x == 0) carry_s += wtot[0] + wtot[1] + wtot[2] + wtot[3];
        __syncthreads();
    }
    if (threadIdx.x == 0) n_left_out[blockIdx.x] = carry_s;
}

__global__ __launch_bounds__(kBlock) void part_scatter_kernel(
    const uint32_t *__restrict__ src, uint32_t *__restrict__ dst, const PartJob *__restrict__ jobs,
    int n_jobs, const uint64_t *__restrict__ masks, const uint32_t *__restrict__ tile_left_off,
    const uint32_t *__restrict__ n_left) {
    const uint32_t tile = blockIdx.x;
    const int ji = find_job(jobs, n_jobs, tile);
    const PartJob job = jobs[ji];
    const uint32_t base = (tile - job.tile_begin) * kTile;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    __shared__ uint64_t words[kWordsPerTile];
    __shared__ uint32_t lefts_before[kWordsPerTile];
    if (threadIdx.x < kWordsPerTile) words[threadIdx.x] = masks[(uint64_t)tile * kWordsPerTile + threadIdx.x];
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t acc = 0;
        for (int w = 0; w < kWordsPerTile; ++w) {
            lefts_before[w] = acc;
            acc += (uint32_t)__popcll(words[w]);
        }
    }
    __syncthreads();

    const uint32_t left_base = tile_left_off[tile];   // lefts of this segment before this tile
    const uint32_t right_base = base - left_base;     // rights of this segment before this tile
    const uint32_t seg_n_left = n_left[ji];
#pragma unroll
    for (int j = 0; j < kRowsPerThread; ++j) {
        const int w = j * (kBlock / 64) + wave;
        const uint32_t off = base + (uint32_t)w * 64u + (uint32_t)lane;
        if (off < job.seg_len) {
            const uint64_t m = words[w];
            const uint32_t below = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            const uint32_t r = src[(uint64_t)job.seg_begin + off];
            uint32_t pos;
            if ((m >> lane) & 1ull) {
                pos = left_base + lefts_before[w] + below;
            } else {
                const uint32_t rights_before_word = (uint32_t)w * 64u - lefts_before[w];
                pos = seg_n_left + right_base + rights_before_word + ((uint32_t)lane - below);
            }
            dst[(uint64_t)job.seg_begin + pos] = r;
        }
    }
}

// Scatter of whole records.  dst rows are SW words each; src rows start at bit
// p*src_stride_bits (any alignment).  src_id == NULL: the id of the row at
// position p is p itself.  Long rows are cut into slices of `slice_words` words,
// one workgroup per (tile, slice) (blockIdx.y); slice 0 also moves ids and pairs.
__global__ __launch_bounds__(kBlock) void part_move_kernel(
    const uint32_t *__restrict__ src_sym, int64_t src_stride_bits, int64_t src_words,
    uint32_t *__restrict__ dst_sym, int SW, int row_bits, const int2 *__restrict__ src_gq,
    int2 *__restrict__ dst_gq, const uint32_t *__restrict__ src_id, uint32_t *__restrict__ dst_id,
    const PartJob *__restrict__ jobs, int n_jobs, const uint64_t *__restrict__ masks,
    const uint32_t *__restrict__ tile_left_off, const uint32_t *__restrict__ n_left, int slice_words,
    bool vec_rows) {
    const uint32_t tile = blockIdx.x;
    const int ji = find_job(jobs, n_jobs, tile);
    const PartJob job = jobs[ji];
    const uint32_t base = (tile - job.tile_begin) * kTile;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k_begin = (int)blockIdx.y * slice_words;
    const int k_end = k_begin + slice_words < SW ? k_begin + slice_words : SW;

    __shared__ uint64_t words[kWordsPerTile];
    __shared__ uint32_t lefts_before[kWordsPerTile];
    __shared__ uint32_t dstpos[kTile];   // destination position of each row of the tile
    if (threadIdx.x < kWordsPerTile) words[threadIdx.x] = masks[(uint64_t)tile * kWordsPerTile + threadIdx.x];
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t acc = 0;
        for (int w = 0; w < kWordsPerTile; ++w) {
            lefts_before[w] = acc;
            acc += (uint32_t)__popcll(words[w]);
        }
    }
    __syncthreads();
    const uint32_t left_base = tile_left_off[tile];
    const uint32_t right_base = base - left_base;
    const uint32_t seg_n_left = n_left[ji];
    const uint32_t tile_rows = job.seg_len - base < (uint32_t)kTile ? job.seg_len - base : (uint32_t)kTile;
#pragma unroll
    for (int j = 0; j < kRowsPerThread; ++j) {
        const int w = j * (kBlock / 64) + wave;
        const uint32_t in_tile = (uint32_t)w * 64u + (uint32_t)lane;
        if (in_tile < tile_rows) {
            const uint64_t m = words[w];
            const uint32_t below = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            uint32_t pos;
            if ((m >> lane) & 1ull) {
                pos = left_base + lefts_before[w] + below;
            } else {
                const uint32_t rights_before_word = (uint32_t)w * 64u - lefts_before[w];
                pos = seg_n_left + right_base + rights_before_word + ((uint32_t)lane - below);
            }
            const uint32_t q = job.seg_begin + pos;
            dstpos[in_tile] = q;
            if (blockIdx.y == 0) {
                const uint64_t p = (uint64_t)job.seg_begin + base + in_tile;
                dst_id[q] = src_id ? src_id[p] : (uint32_t)p;
                dst_gq[q] = src_gq[p];
            }
        }
    }
    __syncthreads();
    const uint32_t tail_bits = (uint32_t)(row_bits - 32 * (SW - 1));   // valid bits of a row's last word, 1..32
    const uint32_t tail_mask = tail_bits >= 32 ? 0xffffffffu : ((1u << tail_bits) - 1u);
    const uint64_t p0 = (uint64_t)job.seg_begin + base;
    if (vec_rows) {
        // 16-byte rows on both sides, both bases 16-byte aligned: one 128-bit load and store per row
        const uint4 *s4 = (const uint4 *)src_sym;
        uint4 *d4 = (uint4 *)dst_sym;
        for (uint32_t in_tile = threadIdx.x; in_tile < tile_rows; in_tile += kBlock)
            d4[dstpos[in_tile]] = s4[p0 + in_tile];
    } else {
        // a group of lanes (the next power of two >= SW, at most 64) copies one row, one word per
        // lane and step: the words of a row, and the rows of a run, are written side by side
        const int nk = k_end - k_begin;
        int lpr = 1;
        while (lpr < nk && lpr < 64) lpr <<= 1;
        const int rows_per_wave = 64 / lpr;
        const int sub = lane / lpr, k0 = lane % lpr;
        for (uint32_t row0 = (uint32_t)wave * rows_per_wave; row0 < tile_rows; row0 += (kBlock / 64) * rows_per_wave) {
            const uint32_t in_tile = row0 + (uint32_t)sub;
            if (in_tile >= tile_rows) continue;
            const uint64_t sb = (p0 + in_tile) * (uint64_t)src_stride_bits;
            const int64_t s0 = (int64_t)(sb >> 5);
            const uint32_t sh = (uint32_t)(sb & 31);
            uint32_t *d = dst_sym + (uint64_t)dstpos[in_tile] * (uint64_t)SW;
            for (int k = k_begin + k0; k < k_end; k += lpr) {
                const int64_t si = s0 + k;
                const uint32_t lo = src_sym[si < src_words ? si : src_words - 1];
                const uint32_t hi = src_sym[si + 1 < src_words ? si + 1 : src_words - 1];
                uint32_t v = __builtin_amdgcn_alignbit(hi, lo, sh);
                if (k == SW - 1) v &= tail_mask;
                d[k] = v;
            }
        }
    }
}

// Same ranks as part_move_kernel, but only the ids move (the children are leaves: nobody will
// read their symbols or gradient pairs again).
__global__ __launch_bounds__(kBlock) void part_move_ids_kernel(
    const uint32_t *__restrict__ src_id, uint32_t *__restrict__ dst_id, const PartJob *__restrict__ jobs,
    int n_jobs, const uint64_t *__restrict__ masks, const uint32_t *__restrict__ tile_left_off,
    const uint32_t *__restrict__ n_left) {
    const uint32_t tile = blockIdx.x;
    const int ji = find_job(jobs, n_jobs, tile);
    const PartJob job = jobs[ji];
    const uint32_t base = (tile - job.tile_begin) * kTile;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __shared__ uint64_t words[kWordsPerTile];
    __shared__ uint32_t lefts_before[kWordsPerTile];
    if (threadIdx.x < kWordsPerTile) words[threadIdx.x] = masks[(uint64_t)tile * kWordsPerTile + threadIdx.x];
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t acc = 0;
        for (int w = 0; w < kWordsPerTile; ++w) {
            lefts_before[w] = acc;
            acc += (uint32_t)__popcll(words[w]);
        }
    }
    __syncthreads();
    const uint32_t left_base = tile_left_off[tile];
    const uint32_t right_base = base - left_base;
    const uint32_t seg_n_left = n_left[ji];
#pragma unroll
    for (int j = 0; j < kRowsPerThread; ++j) {
        const int w = j * (kBlock / 64) + wave;
        const uint32_t off = base + (uint32_t)w * 64u + (uint32_t)lane;
        if (off < job.seg_len) {
            const uint64_t m = words[w];
            const uint32_t below = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            const uint64_t p = (uint64_t)job.seg_begin + off;
            uint32_t pos;
            if ((m >> lane) & 1ull) {
                pos = left_base + lefts_before[w] + below;
            } else {
                const uint32_t rights_before_word = (uint32_t)w * 64u - lefts_before[w];
                pos = seg_n_left + right_base + rights_before_word + ((uint32_t)lane - below);
            }
            dst_id[(uint64_t)job.seg_begin + pos] = src_id ? src_id[p] : (uint32_t)p;
        }
    }
}

// ---------------------------------------------------------------------------
// One-launch partition of whole records for a caller that does not need the row
// order kept (the grow loop when row ids are not tracked: histograms are exact
// integer sums, so the order of a node's rows does not change any result).
//
// A tile decides its rows' sides from the rows it has just loaded, then reserves
// room for both halves with ONE 64-bit atomic add on its segment's cursor (low
// word: left rows handed out so far, high word: right rows).  Left rows fill the
// segment from its start, right rows from its end backwards; inside a tile both
// halves keep their order, tiles land in the order their atomics arrive.  Compared
// with the three-launch form the matrix is read once instead of twice, no ballots
// go through HBM and no workgroup waits for another.  The cursor's low word ends
// as the segment's n_left.
// ---------------------------------------------------------------------------
constexpr int kFBlock = 512;
constexpr int kFTile = kFBlock * kRowsPerThread;   // 4096 rows
constexpr int kFWords = kFTile / 64;               // 64 ballot words: one per lane of a wave
static_assert(kFWords == 64, "the ballot words are ranked by one wave");

__device__ inline uint32_t pick_word(const uint4 &v, int k) { return k == 0 ? v.x : k == 1 ? v.y : k == 2 ? v.z : v.w; }

// Rows of four words in the destination and at most 128 bits in the source: a thread keeps its eight
// rows in registers between the load and the store.  (Other widths: part_staged_kernel below.)
__global__ __launch_bounds__(kFBlock) void part_fused_kernel(
    const uint32_t *__restrict__ src_sym, int64_t src_stride_bits, int64_t src_words, bool aligned_src,
    uint32_t *__restrict__ dst_sym, int SW, int row_bits, int bits, uint32_t missing,
    const int2 *__restrict__ src_gq, int2 *__restrict__ dst_gq, const PartJob *__restrict__ jobs, int n_jobs,
    unsigned long long *__restrict__ cursor) {
    __shared__ uint32_t left_base_s, right_base_s;
    __shared__ uint64_t words[kFWords];
    __shared__ uint32_t lefts_before[kFWords];
    const uint32_t tile = blockIdx.x;
    const int ji = find_job(jobs, n_jobs, tile);
    const PartJob job = jobs[ji];
    const uint32_t base = (tile - job.tile_begin) * kFTile;
    const uint32_t tile_rows = job.seg_len - base < (uint32_t)kFTile ? job.seg_len - base : (uint32_t)kFTile;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t p0 = (uint64_t)job.seg_begin + base;
    const uint32_t sym_mask = (1u << bits) - 1u;
    const uint32_t tail_bits = (uint32_t)(row_bits - 32 * (SW - 1));   // valid bits of a row's last word, 1..32
    const uint32_t tail_mask = tail_bits >= 32 ? 0xffffffffu : ((1u << tail_bits) - 1u);
    const uint32_t fbit = job.feature * (uint32_t)bits;   // the split feature's first bit inside a row

    // ---- load, decide
    uint4 row[kRowsPerThread];
    int2 pair[kRowsPerThread];
#pragma unroll
    for (int j = 0; j < kRowsPerThread; ++j) {
        const int w = j * (kFBlock / 64) + wave;
        const uint32_t in_tile = (uint32_t)w * 64u + (uint32_t)lane;
        bool left = false;
        if (in_tile < tile_rows) {
            const uint64_t p = p0 + in_tile;
            uint32_t sy;
            {
                uint4 v;
                if (aligned_src) {   // 16-byte rows on a 16-byte aligned base
                    v = ((const uint4 *)src_sym)[p];
                } else {
                    const uint64_t sb = p * (uint64_t)src_stride_bits;
                    const int64_t s0 = (int64_t)(sb >> 5);
                    const uint32_t sh = (uint32_t)(sb & 31);
                    uint32_t x[5];
#pragma unroll
                    for (int k = 0; k < 5; ++k) x[k] = src_sym[s0 + k < src_words ? s0 + k : src_words - 1];
                    v.x = __builtin_amdgcn_alignbit(x[1], x[0], sh);
                    v.y = __builtin_amdgcn_alignbit(x[2], x[1], sh);
                    v.z = __builtin_amdgcn_alignbit(x[3], x[2], sh);
                    v.w = __builtin_amdgcn_alignbit(x[4], x[3], sh) & tail_mask;
                }
                row[j] = v;
                pair[j] = src_gq[p];
                const int k = (int)(fbit >> 5);
                const uint32_t lo = pick_word(v, k), hi = k < 3 ? pick_word(v, k + 1) : 0u;
                sy = __builtin_amdgcn_alignbit(hi, lo, fbit & 31u) & sym_mask;
            }
            left = (sy == missing) ? (job.default_left != 0) : (sy <= job.bin);
        }
        const uint64_t ballot = __ballot(left);
        if (lane == 0) words[w] = ballot;
    }
    __syncthreads();

    // ---- wave 0 ranks the ballot words (one per lane) and reserves the tile's room
    if (wave == 0) {
        const uint32_t c = (uint32_t)__popcll(words[lane]);
        uint32_t x = c;
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t y = (uint32_t)__shfl_up((int)x, d);
            if (lane >= d) x += y;
        }
        lefts_before[lane] = x - c;
        if (lane == 63) {
            const uint32_t cnt = x;
            const unsigned long long old =
                atomicAdd(&cursor[ji], (unsigned long long)cnt | ((unsigned long long)(tile_rows - cnt) << 32));
            left_base_s = (uint32_t)(old & 0xffffffffull);
            right_base_s = (uint32_t)(old >> 32);
        }
    }
    __syncthreads();
    const uint32_t left_base = left_base_s;     // left rows of this segment placed before this tile's
    const uint32_t right_base = right_base_s;   // right rows likewise
    const uint32_t seg_last = job.seg_begin + job.seg_len - 1u;

    // ---- write
#pragma unroll
    for (int j = 0; j < kRowsPerThread; ++j) {
        const int w = j * (kFBlock / 64) + wave;
        const uint32_t in_tile = (uint32_t)w * 64u + (uint32_t)lane;
        if (in_tile < tile_rows) {
            const uint64_t m = words[w];
            const uint32_t below = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            uint32_t q;
            if ((m >> lane) & 1ull) {
                q = job.seg_begin + left_base + lefts_before[w] + below;
            } else {
                const uint32_t rights_before_word = (uint32_t)w * 64u - lefts_before[w];
                q = seg_last - (right_base + rights_before_word + ((uint32_t)lane - below));
            }
            ((uint4 *)dst_sym)[q] = row[j];
            dst_gq[q] = pair[j];
        }
    }
}

// The same one-launch partition for rows of any width up to 64 words: the tile's rows are one
// contiguous piece of the source bit stream, which is read linearly into LDS (every lane busy, whole
// lines, each byte fetched once); the split symbols are then cut out of LDS, and every row is copied
// from LDS to its new place by a group of lanes, one word per lane.  The tile holds as many rows as
// fit kStageBytes (at most kFTile).
constexpr int kStageBytes = 48 * 1024;
__host__ __device__ inline int staged_tile_rows(int64_t dst_stride_bits) {
    int64_t r = (int64_t)kStageBytes * 8 / dst_stride_bits;   // the source stride is never larger
    r = r / 64 * 64;
    return (int)(r > kFTile ? kFTile : (r < 64 ? 64 : r));
}

__global__ __launch_bounds__(kFBlock) void part_staged_kernel(
    const uint32_t *__restrict__ src_sym, int64_t src_stride_bits, int64_t src_words,
    uint32_t *__restrict__ dst_sym, int SW, int row_bits, int bits, uint32_t missing,
    const int2 *__restrict__ src_gq, int2 *__restrict__ dst_gq, const PartJob *__restrict__ jobs, int n_jobs,
    int tile_cap, unsigned long long *__restrict__ cursor) {
    extern __shared__ uint32_t stage[];                 // the tile's words, then one destination per row
    __shared__ uint32_t left_base_s, right_base_s;
    __shared__ uint64_t words[kFWords];
    __shared__ uint32_t lefts_before[kFWords];
    const uint32_t tile = blockIdx.x;
    const int ji = find_job(jobs, n_jobs, tile);
    const PartJob job = jobs[ji];
    const uint32_t base = (tile - job.tile_begin) * (uint32_t)tile_cap;
    const uint32_t tile_rows = job.seg_len - base < (uint32_t)tile_cap ? job.seg_len - base : (uint32_t)tile_cap;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t p0 = (uint64_t)job.seg_begin + base;
    const uint64_t bit0 = p0 * (uint64_t)src_stride_bits;      // first bit of the tile in the source
    const int64_t w_lo = (int64_t)(bit0 >> 5);
    const uint32_t sh0 = (uint32_t)(bit0 & 31);
    const uint32_t n_stage = (uint32_t)((sh0 + (uint64_t)tile_rows * (uint64_t)src_stride_bits + 31) >> 5) + 1u;
    uint32_t *dstpos = stage + (((uint64_t)tile_cap * (uint64_t)src_stride_bits + 31) >> 5) + 2;
    for (uint32_t i = threadIdx.x; i < n_stage; i += kFBlock)
        stage[i] = src_sym[w_lo + i < src_words ? w_lo + i : src_words - 1];
    __syncthreads();

    const uint32_t sym_mask = (1u << bits) - 1u;
    const uint32_t fbit = job.feature * (uint32_t)bits;
    const int n_words_tile = (tile_cap + 63) / 64;             // ballot words in use, <= kFWords
    for (int w = wave; w < n_words_tile; w += kFBlock / 64) {
        const uint32_t in_tile = (uint32_t)w * 64u + (uint32_t)lane;
        bool left = false;
        if (in_tile < tile_rows) {
            const uint64_t b = sh0 + (uint64_t)in_tile * (uint64_t)src_stride_bits + fbit;   // inside the staged words
            const uint32_t lo = stage[b >> 5], hi = stage[(b >> 5) + 1];
            const uint32_t sy = __builtin_amdgcn_alignbit(hi, lo, (uint32_t)(b & 31)) & sym_mask;
            left = (sy == missing) ? (job.default_left != 0) : (sy <= job.bin);
        }
        const uint64_t ballot = __ballot(left);
        if (lane == 0) words[w] = ballot;
    }
    __syncthreads();
    if (wave == 0) {
        const uint32_t c = lane < n_words_tile ? (uint32_t)__popcll(words[lane]) : 0u;
        uint32_t x = c;
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t y = (uint32_t)__shfl_up((int)x, d);
            if (lane >= d) x += y;
        }
        if (lane < n_words_tile) lefts_before[lane] = x - c;
        if (lane == 63) {
            const unsigned long long old =
                atomicAdd(&cursor[ji], (unsigned long long)x | ((unsigned long long)(tile_rows - x) << 32));
            left_base_s = (uint32_t)(old & 0xffffffffull);
            right_base_s = (uint32_t)(old >> 32);
        }
    }
    __syncthreads();
    const uint32_t left_base = left_base_s, right_base = right_base_s;
    const uint32_t seg_last = job.seg_begin + job.seg_len - 1u;
    for (int w = wave; w < n_words_tile; w += kFBlock / 64) {
        const uint32_t in_tile = (uint32_t)w * 64u + (uint32_t)lane;
        if (in_tile < tile_rows) {
            const uint64_t m = words[w];
            const uint32_t below = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            uint32_t q;
            if ((m >> lane) & 1ull) {
                q = job.seg_begin + left_base + lefts_before[w] + below;
            } else {
                const uint32_t rights_before_word = (uint32_t)w * 64u - lefts_before[w];
                q = seg_last - (right_base + rights_before_word + ((uint32_t)lane - below));
            }
            dstpos[in_tile] = q;
            dst_gq[q] = src_gq[p0 + in_tile];
        }
    }
    __syncthreads();
    const uint32_t tail_bits = (uint32_t)(row_bits - 32 * (SW - 1));
    const uint32_t tail_mask = tail_bits >= 32 ? 0xffffffffu : ((1u << tail_bits) - 1u);
    int lpr = 1;   // lanes per row: the next power of two >= SW, at most 64
    while (lpr < SW && lpr < 64) lpr <<= 1;
    const int rows_per_wave = 64 / lpr;
    const int sub = lane / lpr, k0 = lane % lpr;
    for (uint32_t row0 = (uint32_t)wave * rows_per_wave; row0 < tile_rows; row0 += (kFBlock / 64) * rows_per_wave) {
        const uint32_t in_tile = row0 + (uint32_t)sub;
        if (in_tile >= tile_rows) continue;
        const uint64_t b = sh0 + (uint64_t)in_tile * (uint64_t)src_stride_bits;
        const uint32_t s0 = (uint32_t)(b >> 5), sh = (uint32_t)(b & 31);
        uint32_t *d = dst_sym + (uint64_t)dstpos[in_tile] * (uint64_t)SW;
        for (int k = k0; k < SW; k += lpr) {
            uint32_t v = __builtin_amdgcn_alignbit(stage[s0 + k + 1], stage[s0 + k], sh);   // s0 + k + 1 < n_stage
            if (k == SW - 1) v &= tail_mask;
            d[k] = v;
        }
    }
}

}  // namespace

hipError_t gbt_launch_partition(hipStream_t s, const uint32_t *packed, int bits, int64_t stride_bits, int64_t n,
                                uint32_t missing, const uint32_t *src, uint32_t *dst,
                                const PartJob *jobs, int n_jobs, int total_tiles, uint64_t *masks,
                                uint32_t *tile_left, uint32_t *n_left_out) {
    if (n_jobs <= 0 || total_tiles <= 0) return hipSuccess;
    part_flag_kernel<<<total_tiles, kBlock, 0, s>>>(packed, bits, stride_bits, n, missing, src, jobs, n_jobs, masks,
                                                    tile_left);
    part_scan_kernel<<<n_jobs, kBlock, 0, s>>>(jobs, tile_left, n_left_out);
    part_scatter_kernel<<<total_tiles, kBlock, 0, s>>>(src, dst, jobs, n_jobs, masks, tile_left, n_left_out);
    return hipGetLastError();
}

hipError_t gbt_launch_partition_records(hipStream_t s, const GbtRows &src, const GbtRows &dst, int bits, int row_bits,
                                        int64_t n, uint32_t missing, int what, const PartJob *jobs,
                                        int n_jobs, int total_tiles, uint64_t *masks, uint32_t *tile_left,
                                        uint32_t *n_left_out) {
    if (n_jobs <= 0 || total_tiles <= 0) return hipSuccess;
    part_flag_kernel<<<total_tiles, kBlock, 0, s>>>(src.sym, bits, src.stride_bits, n, missing, nullptr, jobs, n_jobs,
                                                    masks, tile_left);
    part_scan_kernel<<<n_jobs, kBlock, 0, s>>>(jobs, tile_left, n_left_out);
    if (what == GBT_PART_COUNT) return hipGetLastError();
    if (what == GBT_PART_IDS) {
        part_move_ids_kernel<<<total_tiles, kBlock, 0, s>>>(src.id, dst.id_rw, jobs, n_jobs, masks, tile_left,
                                                            n_left_out);
        return hipGetLastError();
    }
    const int SW = (int)(dst.stride_bits >> 5);
    const int slice_words = SW <= 64 ? SW : 64;   // a wave copies 256 contiguous bytes of a row per step
    dim3 grid((unsigned)total_tiles, (unsigned)((SW + slice_words - 1) / slice_words));
    part_move_kernel<<<grid, kBlock, 0, s>>>(src.sym, src.stride_bits, src.n_words, dst.sym_rw, SW, row_bits,
                                             (const int2 *)src.gq, (int2 *)dst.gq_rw, src.id, dst.id_rw, jobs,
                                             n_jobs, masks, tile_left, n_left_out, slice_words,
                                             SW == 4 && src.stride_bits == 128 && ((uintptr_t)src.sym & 15u) == 0);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Row counts two levels down, for the children of nodes whose rows were not moved at their own
// split (the last level that needs histograms: its children's histograms come out of the pass that
// would have moved the rows, and below them only row counts are wanted).  One byte per level and row
// is needed; the rows come in by whole sectors.
// ---------------------------------------------------------------------------
namespace {
constexpr int kC2Block = 512, kC2Rows = 8, kC2Tile = kC2Block * kC2Rows;

// LEVELS splits lie between the segment and the nodes whose left rows are counted: a row is taken down
// from the segment's own split and counted at the node it reaches if that node splits.
// RECORDS: the rows are records of whole words whose first 16 bytes hold every symbol: they are loaded
// once (all of a thread's rows before the first is used) and a split's byte is cut out with v_perm;
// otherwise (rows of the packed matrix, any byte stride) one dependent byte load per level.
template <int LEVELS, bool RECORDS>
__global__ __launch_bounds__(kC2Block) void count2_kernel(const uint8_t *__restrict__ rows, int64_t stride_bytes,
                                                          uint32_t missing, const CountJob *__restrict__ jobs,
                                                          int n_jobs, uint32_t *__restrict__ counts) {
    constexpr int NT = 1 << LEVELS;          // target nodes per job
    constexpr int FIRST_T = NT - 1;          // heap position of the first target
    __shared__ uint32_t acc[NT];
    __shared__ CountJob sjob;
    int lo = 0, hi = n_jobs;   // last job with tile_begin <= this tile
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (jobs[mid].tile_begin <= blockIdx.x) lo = mid; else hi = mid;
    }
    if (threadIdx.x < (int)(sizeof(CountJob) / 4)) ((uint32_t *)&sjob)[threadIdx.x] = ((const uint32_t *)&jobs[lo])[threadIdx.x];
    if (threadIdx.x < NT) acc[threadIdx.x] = 0;
    __syncthreads();
    const CountJob &job = sjob;
    const uint32_t t0 = (blockIdx.x - job.tile_begin) * (uint32_t)kC2Tile;
    const uint8_t *rp[kC2Rows];
    uint4 rec[RECORDS ? kC2Rows : 1];
    uint32_t pos[kC2Rows];     // heap position of the node the row has reached; 0xff: out of the count
    uint32_t sy[kC2Rows];
    auto symbol = [&](int j, uint32_t f) __attribute__((always_inline)) -> uint32_t {
        if (RECORDS) {
            const uint32_t sa = 0x0C0C0C00u | (f < 8u ? f : 0x0Cu), sb = 0x0C0C0C00u | (f >= 8u ? f - 8u : 0x0Cu);
            return __builtin_amdgcn_perm(rec[RECORDS ? j : 0].y, rec[RECORDS ? j : 0].x, sa) |
                   __builtin_amdgcn_perm(rec[RECORDS ? j : 0].w, rec[RECORDS ? j : 0].z, sb);
        }
        return rp[j][f];
    };
#pragma unroll
    for (int j = 0; j < kC2Rows; ++j) {   // every load of the tile (of a level) is issued before the first is used
        const uint32_t i = t0 + (uint32_t)j * kC2Block + threadIdx.x;
        const uint32_t ic = i < job.seg_len ? i : job.seg_len - 1;
        rp[j] = rows + ((uint64_t)job.seg_begin + ic) * (uint64_t)stride_bytes;
        pos[j] = i < job.seg_len ? 0u : 0xffu;
        if (RECORDS) {
            const uint32_t *w = (const uint32_t *)rp[j];
            rec[RECORDS ? j : 0] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
#pragma unroll
    for (int j = 0; j < kC2Rows; ++j) sy[j] = symbol(j, job.feature[0]);
    unsigned long long mine = 0;   // 16 bits per target: rows of this thread counted there
#pragma unroll
    for (int l = 0; l <= LEVELS; ++l) {
#pragma unroll
        for (int j = 0; j < kC2Rows; ++j) {
            if (pos[j] != 0xffu) {
                const uint32_t p = pos[j];
                const bool left = sy[j] == missing ? job.default_left[p] != 0 : sy[j] <= job.bin[p];
                if (l == LEVELS) {
                    if (left) mine += 1ull << (16 * (p - FIRST_T));
                } else {
                    const uint32_t q = 2u * p + (left ? 1u : 2u);
                    pos[j] = job.has[q] ? q : 0xffu;
                }
            }
        }
        if (l < LEVELS) {
#pragma unroll
            for (int j = 0; j < kC2Rows; ++j) sy[j] = pos[j] != 0xffu ? symbol(j, job.feature[pos[j]]) : 0u;
        }
    }
    for (int o = 32; o > 0; o >>= 1) {   // a field holds at most 64 * kC2Rows
        const uint32_t a = (uint32_t)__shfl_xor((int)(uint32_t)mine, o), b = (uint32_t)__shfl_xor((int)(uint32_t)(mine >> 32), o);
        mine += ((unsigned long long)b << 32) | a;
    }
    static_assert(64 * kC2Rows < 65536, "16-bit fields");
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint32_t c = (uint32_t)(mine >> (16 * t)) & 0xffffu;
            if (c) atomicAdd(&acc[t], c);
        }
    }
    __syncthreads();
    if (threadIdx.x < NT && acc[threadIdx.x]) atomicAdd(&counts[NT * lo + threadIdx.x], acc[threadIdx.x]);
}
}  // namespace

int gbt_count2_tile() { return kC2Tile; }
hipError_t gbt_launch_count2(hipStream_t s, const uint8_t *rows, int64_t stride_bytes, uint32_t missing,
                             const CountJob *jobs, int n_jobs, int n_tiles, uint32_t *counts, int levels, bool records_ok) {
    if (n_jobs <= 0) return hipSuccess;
    if (levels != 1 && levels != 2) return hipErrorInvalidValue;
    hipError_t e = gbt_launch_fill_u64(s, (uint64_t *)counts, 0, (int64_t)n_jobs * levels);   // 2 or 4 32-bit counts per job
    if (e != hipSuccess || n_tiles <= 0) return e;
    // records: whole words per row, 4-byte aligned, at least 16 readable bytes from every row's start (the
    // working copies end in spare words), every feature index below 16
    const bool records = (stride_bytes & 3) == 0 && ((uintptr_t)rows & 3u) == 0 && records_ok;
    if (levels == 1 && records)
        count2_kernel<1, true><<<n_tiles, kC2Block, 0, s>>>(rows, stride_bytes, missing, jobs, n_jobs, counts);
    else if (levels == 1)
        count2_kernel<1, false><<<n_tiles, kC2Block, 0, s>>>(rows, stride_bytes, missing, jobs, n_jobs, counts);
    else if (records)
        count2_kernel<2, true><<<n_tiles, kC2Block, 0, s>>>(rows, stride_bytes, missing, jobs, n_jobs, counts);
    else
        count2_kernel<2, false><<<n_tiles, kC2Block, 0, s>>>(rows, stride_bytes, missing, jobs, n_jobs, counts);
    return hipGetLastError();
}

bool gbt_partition_fused_ok(const GbtRows &dst) { return (dst.stride_bits >> 5) <= 64; }
int gbt_partition_fused_tile(const GbtRows &dst) {
    return (dst.stride_bits >> 5) == 4 ? kFTile : staged_tile_rows(dst.stride_bits);
}

hipError_t gbt_launch_partition_fused(hipStream_t s, const GbtRows &src, const GbtRows &dst, int bits, int row_bits,
                                      uint32_t missing, const PartJob *jobs, int n_jobs, int total_tiles,
                                      unsigned long long *cursor) {
    if (n_jobs <= 0 || total_tiles <= 0) return hipSuccess;
    hipError_t e = gbt_launch_fill_u64(s, (uint64_t *)cursor, 0, n_jobs);
    if (e != hipSuccess) return e;
    const int SW = (int)(dst.stride_bits >> 5);
    const bool aligned_src = src.stride_bits == 128 && ((uintptr_t)src.sym & 15u) == 0;
    if (SW == 4 && src.stride_bits <= 128)
        part_fused_kernel<<<total_tiles, kFBlock, 0, s>>>(src.sym, src.stride_bits, src.n_words, aligned_src,
                                                                dst.sym_rw, SW, row_bits, bits, missing,
                                                                (const int2 *)src.gq, (int2 *)dst.gq_rw, jobs, n_jobs,
                                                                cursor);
    else {
        const int cap = staged_tile_rows(dst.stride_bits);
        const size_t lds = ((((size_t)cap * (size_t)src.stride_bits + 31) >> 5) + 2 + (size_t)cap) * 4;
        GbtLdsGuard lds_guard(lds);
        if (lds_guard.needed) {
            e = hipFuncSetAttribute((const void *)part_staged_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds);
            if (e != hipSuccess) return e;
        }
        part_staged_kernel<<<total_tiles, kFBlock, lds, s>>>(src.sym, src.stride_bits, src.n_words, dst.sym_rw, SW,
                                                             row_bits, bits, missing, (const int2 *)src.gq,
                                                             (int2 *)dst.gq_rw, jobs, n_jobs, cap, cursor);
    }
    return hipGetLastError();
}
