// Feature quantile generation (Sec. 2.1) on the GPU: exact per-feature order
// statistics by a segmented LSD radix sort of the order-preserving integer
// image of the fp32 values, then cuts, then binning.
//
//   1. keys: every feature's values become one contiguous segment of uint32
//      keys (dense input: an LDS-tiled transpose, a missing value becomes the
//      largest key; CSR input: counted, offset and scattered by column);
//   2. sort: four 8-bit passes; per pass a per-tile digit histogram, one
//      workgroup per segment turning the tile histograms into offsets, and a
//      stable scatter (ranks from wave ballots, tiles and waves in order);
//   3. cuts: one thread per feature walks the sorted segment (distinct values
//      by upper-bound jumps, else the order statistics v[floor(k*m/B)]);
//   4. bin: symbol = number of cuts <= x by bisection over the feature's cuts.
#include "gbt_internal.h"

#include <string.h>

#include <vector>

namespace {

constexpr int kSortBlock = 256;
constexpr int kSortTile = 4096;                       // keys per workgroup and pass
constexpr int kKeysPerWave = kSortTile / (kSortBlock / 64);   // 1024
constexpr int kRounds = kKeysPerWave / 64;            // 16
constexpr uint32_t kMissingKey = 0xffffffffu;

__device__ inline uint32_t float_key(float x) {
    if (x != x) return kMissingKey;
    x = x + 0.0f;   // -0.0 -> +0.0: the two compare equal and must share a key
    uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float key_float(uint32_t k) {
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

// ---- 1a. dense input: transpose into per-feature key segments -------------
constexpr int kTrRows = 64, kTrCols = 64;
__global__ __launch_bounds__(256) void dense_keys_kernel(const float *__restrict__ X, int64_t n, int F,
                                                         uint32_t *__restrict__ keys) {
    __shared__ uint32_t tile[kTrRows][kTrCols + 1];
    const int64_t r0 = (int64_t)blockIdx.x * kTrRows;
    const int f0 = blockIdx.y * kTrCols;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;   // 64 x 4
    for (int i = ty; i < kTrRows; i += 4) {
        const int64_t r = r0 + i;
        const int f = f0 + tx;
        tile[i][tx] = (r < n && f < F) ? float_key(X[r * F + f]) : kMissingKey;
    }
    __syncthreads();
    for (int j = ty; j < kTrCols; j += 4) {
        const int f = f0 + j;
        const int64_t r = r0 + tx;
        if (f < F && r < n) keys[(int64_t)f * n + r] = tile[tx][j];
    }
}

// Few features (F <= 64): a tile of 256 whole rows is one contiguous piece of X; it is read linearly
// (every lane busy, whole lines), kept in LDS with an odd row stride, and written out column by column.
constexpr int kTrNarrowRows = 256;
__global__ __launch_bounds__(256) void dense_keys_narrow_kernel(const float *__restrict__ X, int64_t n, int F,
                                                                uint32_t *__restrict__ keys) {
    extern __shared__ uint32_t ntile[];   // [kTrNarrowRows][F | 1]
    const int stride = F | 1;
    const int64_t r0 = (int64_t)blockIdx.x * kTrNarrowRows;
    const int rows = n - r0 < kTrNarrowRows ? (int)(n - r0) : kTrNarrowRows;
    const float *src = X + r0 * F;
    for (int i = threadIdx.x; i < rows * F; i += 256) {
        const int r = i / F, f = i - r * F;
        ntile[r * stride + f] = float_key(src[i]);
    }
    __syncthreads();
    for (int f = 0; f < F; ++f)
        if ((int)threadIdx.x < rows) keys[(int64_t)f * n + r0 + threadIdx.x] = ntile[threadIdx.x * stride + f];
}

// ---- 1b. CSR input: count, offset, scatter by column -----------------------
// Workgroups take chunks of kCsrChunk stored values and count columns in LDS first, so that
// HBM sees one atomic per (chunk, column) instead of one per value.  Columns beyond
// kCsrLdsCols use the direct form.
constexpr int kCsrChunk = 8192;
constexpr int kCsrLdsCols = 4096;

__global__ __launch_bounds__(256) void csr_count_kernel(const int32_t *__restrict__ indices, int64_t nnz, int F,
                                                        uint32_t *__restrict__ counts) {
    __shared__ uint32_t lc[kCsrLdsCols];
    const bool use_lds = F <= kCsrLdsCols;
    if (use_lds) {
        for (int i = threadIdx.x; i < F; i += 256) lc[i] = 0;
        __syncthreads();
    }
    const int64_t i0 = (int64_t)blockIdx.x * kCsrChunk;
    const int64_t i1 = i0 + kCsrChunk < nnz ? i0 + kCsrChunk : nnz;
    for (int64_t i = i0 + threadIdx.x; i < i1; i += 256) {
        const int f = indices[i];
        if (f < 0 || f >= F) continue;
        if (use_lds) atomicAdd(&lc[f], 1u); else atomicAdd(&counts[f], 1u);
    }
    if (use_lds) {
        __syncthreads();
        for (int i = threadIdx.x; i < F; i += 256)
            if (lc[i]) atomicAdd(&counts[i], lc[i]);
    }
}

__global__ __launch_bounds__(256) void csr_scatter_kernel(const int32_t *__restrict__ indices,
                                                          const float *__restrict__ values, int64_t nnz, int F,
                                                          const uint64_t *__restrict__ seg_off,
                                                          uint32_t *__restrict__ cursor,
                                                          uint32_t *__restrict__ keys) {
    __shared__ uint32_t lc[kCsrLdsCols];     // count, then the chunk's first slot, per column
    const bool use_lds = F <= kCsrLdsCols;
    const int64_t i0 = (int64_t)blockIdx.x * kCsrChunk;
    const int64_t i1 = i0 + kCsrChunk < nnz ? i0 + kCsrChunk : nnz;
    if (!use_lds) {
        for (int64_t i = i0 + threadIdx.x; i < i1; i += 256) {
            const int f = indices[i];
            if (f < 0 || f >= F) continue;
            const uint32_t slot = atomicAdd(&cursor[f], 1u);   // order inside a segment is irrelevant before the sort
            keys[seg_off[f] + slot] = float_key(values[i]);
        }
        return;
    }
    for (int i = threadIdx.x; i < F; i += 256) lc[i] = 0;
    __syncthreads();
    // rank of every value among the chunk's values of its column (kCsrChunk / 256 = 32 per thread)
    uint32_t rank[kCsrChunk / 256];
#pragma unroll
    for (int k = 0; k < kCsrChunk / 256; ++k) {
        const int64_t i = i0 + (int64_t)k * 256 + threadIdx.x;
        rank[k] = 0;
        if (i < i1) {
            const int f = indices[i];
            if (f >= 0 && f < F) rank[k] = atomicAdd(&lc[f], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < F; i += 256) {
        const uint32_t c = lc[i];
        lc[i] = c ? atomicAdd(&cursor[i], c) : 0u;   // the chunk's slots in column i start here
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kCsrChunk / 256; ++k) {
        const int64_t i = i0 + (int64_t)k * 256 + threadIdx.x;
        if (i < i1) {
            const int f = indices[i];
            if (f >= 0 && f < F) keys[seg_off[f] + lc[f] + rank[k]] = float_key(values[i]);
        }
    }
}

// chk_off[f] = exclusive prefix of the segments' scan chunks (kScanChunk tiles each)
__global__ void offsets_kernel(const uint32_t *counts, int F, int64_t fixed_len, uint64_t *seg_off,
                               uint32_t *blk_off, uint32_t *chk_off, int scan_chunk) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    uint64_t o = 0;
    uint32_t b = 0, c = 0;
    for (int f = 0; f < F; ++f) {
        seg_off[f] = o;
        blk_off[f] = b;
        chk_off[f] = c;
        const uint64_t len = counts ? (uint64_t)counts[f] : (uint64_t)fixed_len;
        const uint32_t tiles = (uint32_t)((len + kSortTile - 1) / kSortTile);
        o += len;
        b += tiles;
        c += (tiles + (uint32_t)scan_chunk - 1) / (uint32_t)scan_chunk;
    }
    seg_off[F] = o;
    blk_off[F] = b;
    chk_off[F] = c;
}

// ---- 2. segmented radix sort ----------------------------------------------
// One count per key into a 256-bin LDS histogram.  Sorted or low-cardinality data gives a whole wave
// the same digit, which as 64 atomics on one address would take 64 turns: that case is one add.
__device__ inline void count_digit(uint32_t *h, uint32_t d, bool live) {
    const uint64_t act = __ballot(live);
    if (act == 0) return;
    const uint32_t lead = (uint32_t)__builtin_amdgcn_readlane((int)d, (int)__builtin_ctzll(act));
    if (__ballot(live && d == lead) == act) {
        if ((threadIdx.x & 63) == (uint32_t)__builtin_ctzll(act)) atomicAdd(&h[lead], (uint32_t)__popcll(act));
    } else if (live) {
        atomicAdd(&h[d], 1u);
    }
}

__device__ inline int find_segment(const uint32_t *blk_off, int F, uint32_t blk) {
    int lo = 0, hi = F;   // last f with blk_off[f] <= blk and a non-empty tile range
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (blk_off[mid] <= blk) lo = mid; else hi = mid;
    }
    return lo;
}

// A segment's keys sit in one of the two key buffers (bit 0 of its flag word: 0 = keys_a); a pass in which all keys
// of a segment have the same digit is the identity for it and moves nothing (bit 1, set by scan_chunks_kernel, read
// by sort_scatter_kernel), so after the pass the segment is still where it was (flip_kernel).
constexpr uint32_t kSegInB = 1u, kSegSkip = 2u;

__global__ __launch_bounds__(kSortBlock) void sort_hist_kernel(const uint32_t *__restrict__ keys_a,
                                                               const uint32_t *__restrict__ keys_b,
                                                               const uint32_t *__restrict__ seg_flags,
                                                               const uint64_t *__restrict__ seg_off,
                                                               const uint32_t *__restrict__ blk_off, int F,
                                                               int shift, uint32_t *__restrict__ tile_hist) {
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t blk = blockIdx.x;
    const int f = find_segment(blk_off, F, blk);
    const uint32_t *__restrict__ keys = (seg_flags[f] & kSegInB) ? keys_b : keys_a;
    const uint64_t base = seg_off[f], len = seg_off[f + 1] - base;
    const uint64_t t0 = (uint64_t)(blk - blk_off[f]) * kSortTile;
    if (t0 + kSortTile <= len) {   // a whole tile: all loads are issued before the first count
        uint32_t k[kSortTile / kSortBlock];
#pragma unroll
        for (int j = 0; j < kSortTile / kSortBlock; ++j) k[j] = keys[base + t0 + (uint64_t)j * kSortBlock + threadIdx.x];
#pragma unroll
        for (int j = 0; j < kSortTile / kSortBlock; ++j) count_digit(h, (k[j] >> shift) & 255u, true);
    } else {
        for (int i0 = 0; i0 < kSortTile; i0 += kSortBlock) {   // uniform trip count: count_digit uses ballots
            const uint64_t p = t0 + i0 + threadIdx.x;
            const bool live = p < len;
            count_digit(h, live ? (keys[base + p] >> shift) & 255u : 0u, live);
        }
    }
    __syncthreads();
    tile_hist[(uint64_t)blk * 256 + threadIdx.x] = h[threadIdx.x];
}

// tile_hist[blk][d] becomes the position (inside the segment) of the first key of tile blk
// with digit d.  Three launches, thread d owns digit d everywhere:
//   partial : one workgroup per chunk of kScanChunk tiles adds up the chunk's counts;
//   chunks  : one workgroup per segment turns the chunk totals into chunk start positions
//             (exclusive over chunks, then offset by the exclusive scan over the digits);
//   apply   : one workgroup per chunk walks its tiles from the chunk's start position.
constexpr int kScanChunk = 128;

__global__ __launch_bounds__(256) void scan_partial_kernel(const uint32_t *__restrict__ blk_off,
                                                           const uint32_t *__restrict__ chk_off, int F,
                                                           const uint32_t *__restrict__ tile_hist,
                                                           uint32_t *__restrict__ chunk_tot) {
    const uint32_t chunk = blockIdx.x;
    const int f = find_segment(chk_off, F, chunk), d = threadIdx.x;
    const uint32_t b0 = blk_off[f] + (chunk - chk_off[f]) * kScanChunk;
    const uint32_t b1 = b0 + kScanChunk < blk_off[f + 1] ? b0 + kScanChunk : blk_off[f + 1];
    uint32_t run = 0;
    for (uint32_t b = b0; b < b1; ++b) run += tile_hist[(uint64_t)b * 256 + d];
    chunk_tot[(uint64_t)chunk * 256 + d] = run;
}

__global__ __launch_bounds__(256) void scan_chunks_kernel(const uint32_t *__restrict__ chk_off,
                                                          const uint64_t *__restrict__ seg_off,
                                                          uint32_t *__restrict__ seg_flags,
                                                          uint32_t *__restrict__ chunk_tot) {
    const int f = blockIdx.x, d = threadIdx.x;
    const uint32_t c0 = chk_off[f], c1 = chk_off[f + 1];
    uint32_t run = 0;
    for (uint32_t c = c0; c < c1; ++c) {
        const uint32_t v = chunk_tot[(uint64_t)c * 256 + d];
        chunk_tot[(uint64_t)c * 256 + d] = run;
        run += v;
    }
    __shared__ uint32_t tot[256];
    tot[d] = run;
    if (d == 0) seg_flags[f] &= ~kSegSkip;
    __syncthreads();
    // every key of the segment has digit d: at most one thread sees that
    if (run > 0 && (uint64_t)run == seg_off[f + 1] - seg_off[f]) seg_flags[f] |= kSegSkip;
    for (int o = 1; o < 256; o <<= 1) {
        uint32_t v = d >= o ? tot[d - o] : 0;
        __syncthreads();
        tot[d] += v;
        __syncthreads();
    }
    const uint32_t base = tot[d] - run;   // keys of this segment with a smaller digit
    for (uint32_t c = c0; c < c1; ++c) chunk_tot[(uint64_t)c * 256 + d] += base;
}

__global__ __launch_bounds__(256) void scan_apply_kernel(const uint32_t *__restrict__ blk_off,
                                                         const uint32_t *__restrict__ chk_off, int F,
                                                         uint32_t *__restrict__ tile_hist,
                                                         const uint32_t *__restrict__ chunk_tot) {
    const uint32_t chunk = blockIdx.x;
    const int f = find_segment(chk_off, F, chunk), d = threadIdx.x;
    const uint32_t b0 = blk_off[f] + (chunk - chk_off[f]) * kScanChunk;
    const uint32_t b1 = b0 + kScanChunk < blk_off[f + 1] ? b0 + kScanChunk : blk_off[f + 1];
    uint32_t run = chunk_tot[(uint64_t)chunk * 256 + d];
    for (uint32_t b = b0; b < b1; ++b) {
        const uint32_t c = tile_hist[(uint64_t)b * 256 + d];
        tile_hist[(uint64_t)b * 256 + d] = run;
        run += c;
    }
}

// Stable scatter of one tile.  The tile's keys are first put in digit order inside LDS (ranks from
// per-wave digit counts and, inside a round of 64 keys, from ballots), then copied out: consecutive
// threads hold consecutive keys of a digit's run, so the run goes to HBM as whole lines instead of
// 64 separate 4-byte stores per wave instruction.
__global__ __launch_bounds__(kSortBlock) void sort_scatter_kernel(uint32_t *__restrict__ keys_a,
                                                                  uint32_t *__restrict__ keys_b,
                                                                  const uint32_t *__restrict__ seg_flags,
                                                                  const uint64_t *__restrict__ seg_off,
                                                                  const uint32_t *__restrict__ blk_off, int F,
                                                                  int shift,
                                                                  const uint32_t *__restrict__ tile_hist) {
    __shared__ uint32_t cnt[kSortBlock / 64][256];   // per wave: running local position per digit
    __shared__ uint32_t local_start[256];            // first local position of each digit's run
    __shared__ uint32_t run_base[256];               // position in the segment of each digit's run
    __shared__ uint32_t stage[kSortTile];
    static_assert(kSortBlock == 256, "one thread per digit below");
    const uint32_t blk = blockIdx.x;
    const int f = find_segment(blk_off, F, blk);
    const uint32_t flags = seg_flags[f];
    if (flags & kSegSkip) return;   // (the whole workgroup: one segment per tile)
    const uint32_t *__restrict__ src = (flags & kSegInB) ? keys_b : keys_a;
    uint32_t *__restrict__ dst = (flags & kSegInB) ? keys_a : keys_b;
    const uint64_t base = seg_off[f], len = seg_off[f + 1] - base;
    const uint64_t t0 = (uint64_t)(blk - blk_off[f]) * kSortTile;
    const uint32_t tile_keys = len - t0 < (uint64_t)kSortTile ? (uint32_t)(len - t0) : (uint32_t)kSortTile;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < (kSortBlock / 64) * 256; i += kSortBlock) (&cnt[0][0])[i] = 0;
    __syncthreads();

    // the wave's 1024 keys, 64 per round, kept in registers
    uint32_t key[kRounds];
    const uint64_t w0 = t0 + (uint64_t)wave * kKeysPerWave;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const uint64_t p = w0 + (uint64_t)r * 64 + lane;
        key[r] = p < len ? src[base + p] : 0;
        if (p < len) atomicAdd(&cnt[wave][(key[r] >> shift) & 255u], 1u);
    }
    __syncthreads();
    // thread d: the tile's digit-d keys are [local_start[d], local_start[d] + total) inside the tile,
    // wave w's share of them starts at cnt[w][d]
    {
        const int d = threadIdx.x;
        uint32_t total = 0;
        for (int w = 0; w < kSortBlock / 64; ++w) total += cnt[w][d];
        // exclusive scan of the totals over the 256 digits
        uint32_t x = total;
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t y = (uint32_t)__shfl_up((int)x, o);
            if (lane >= o) x += y;
        }
        __shared__ uint32_t wave_tot[kSortBlock / 64];
        if (lane == 63) wave_tot[wave] = x;
        __syncthreads();
        uint32_t before = 0;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        const uint32_t start = before + x - total;
        local_start[d] = start;
        run_base[d] = tile_hist[(uint64_t)blk * 256 + d];
        uint32_t run = start;
        for (int w = 0; w < kSortBlock / 64; ++w) {
            const uint32_t c = cnt[w][d];
            cnt[w][d] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const uint64_t p = w0 + (uint64_t)r * 64 + lane;
        const bool live = p < len;
        const uint32_t dgt = (key[r] >> shift) & 255u;
        // lanes of this round with the same digit
        uint64_t peers = __ballot(live);
        for (int b = 0; b < 8; ++b) {
            const uint64_t m = __ballot((dgt >> b) & 1u);
            peers &= ((dgt >> b) & 1u) ? m : ~m;
        }
        volatile uint32_t *wc = cnt[wave];   // touched by this wave only from here on
        const uint32_t below = (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
        uint32_t first = 0;
        if (live) first = wc[dgt];            // every peer reads the same count ...
        __builtin_amdgcn_wave_barrier();
        if (live && below == 0) wc[dgt] = first + (uint32_t)__popcll(peers);   // ... before the leader bumps it
        __builtin_amdgcn_wave_barrier();
        if (live) stage[first + below] = key[r];   // first + below < tile_keys
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < tile_keys; i += kSortBlock) {
        const uint32_t k = stage[i];
        const uint32_t d = (k >> shift) & 255u;
        dst[base + run_base[d] + (i - local_start[d])] = k;
    }
}

// after a pass: the segments that were scattered have changed buffers
__global__ void flip_kernel(uint32_t *seg_flags, int F) {
    const int f = blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= F) return;
    const uint32_t fl = seg_flags[f];
    seg_flags[f] = (fl & kSegSkip) ? (fl & kSegInB) : ((fl & kSegInB) ^ kSegInB);
}

// ---- 3. cuts ----------------------------------------------------------------
// First index in [lo, hi) with a[i] > v (hi if there is none), found by a whole wave: 64 probes per step cut the
// range by 65, so 1.15e8 keys take five dependent rounds of loads instead of 27.  Every lane passes the same
// arguments and gets the same result.
__device__ inline uint64_t upper_bound_wave(const uint32_t *a, uint64_t lo, uint64_t hi, uint32_t v, int lane) {
    while (hi - lo > 64) {
        const uint64_t span = hi - lo;   // probes lo + span * (l + 1) / 65 are distinct and inside [lo, hi)
        const bool gt = a[lo + span * (uint64_t)(lane + 1) / 65] > v;
        const uint64_t m = __ballot(gt);
        if (m == 0) {
            lo = lo + span * 64 / 65 + 1;   // the last probe is still <= v
        } else {
            const int first = __builtin_ctzll(m);
            const uint64_t new_hi = lo + span * (uint64_t)(first + 1) / 65;   // > v: the answer is at or before it
            if (first > 0) lo = lo + span * (uint64_t)first / 65 + 1;         // the probe before it is <= v
            hi = new_hi;
        }
    }
    const bool gt = lo + (uint64_t)lane < hi && a[lo + (uint64_t)lane] > v;
    const uint64_t m = __ballot(gt);
    return m ? lo + (uint64_t)__builtin_ctzll(m) : hi;
}

// One wave per feature.  Wave-uniform control flow throughout; lane 0 writes.
__global__ __launch_bounds__(64) void cuts_kernel(const uint32_t *__restrict__ keys_a, const uint32_t *__restrict__ keys_b,
                                                  const uint32_t *__restrict__ seg_flags,
                                                  const uint64_t *__restrict__ seg_off, int F, int B,
                                                  float *__restrict__ cuts, int32_t *__restrict__ nb,
                                                  uint32_t *__restrict__ present) {
    const int f = blockIdx.x, lane = threadIdx.x;
    if (f >= F) return;
    const uint32_t *v = ((seg_flags[f] & kSegInB) ? keys_b : keys_a) + seg_off[f];
    const uint64_t len = seg_off[f + 1] - seg_off[f];
    float *c = cuts + (int64_t)f * (B - 1);
    for (int k = lane; k < B - 1; k += 64) c[k] = __uint_as_float(0x7f800000u);   // +inf
    // present values = keys below the missing key
    const uint64_t m = len == 0 ? 0 : upper_bound_wave(v, 0, len, kMissingKey - 1u, lane);
    if (lane == 0) present[f] = (uint32_t)m;
    if (m == 0) {
        if (lane == 0) nb[f] = 1;
        return;
    }
    // distinct values, counted up to B+1; the first B-1 after the smallest are
    // written as tentative cuts
    int d = 0, nc = 0;
    uint64_t pos = 0;
    while (pos < m && d <= B) {
        const uint32_t key = v[pos];
        if (d >= 1 && d <= B - 1 && lane == 0) c[d - 1] = key_float(key);
        ++d;
        pos = upper_bound_wave(v, pos + 1, m, key, lane);
    }
    if (d <= B) {
        nc = d - 1;
    } else {
        // the B-1 order statistics, fetched 64 at a time, then thinned by lane 0 in order
        __shared__ uint32_t pick[4096];
        const uint32_t vmin = v[0];
        uint32_t prev = 0;
        for (int k0 = 1; k0 < B; k0 += 4096) {
            const int cnt = B - k0 < 4096 ? B - k0 : 4096;
            for (int j = lane; j < cnt; j += 64) pick[j] = v[(uint64_t)(k0 + j) * m / (uint64_t)B];
            __syncthreads();
            if (lane == 0) {
                for (int j = 0; j < cnt; ++j) {
                    const uint32_t key = pick[j];
                    if (key == vmin) continue;
                    if (nc > 0 && key == prev) continue;
                    c[nc++] = key_float(key);
                    prev = key;
                }
            }
            __syncthreads();
        }
        nc = __shfl(nc, 0);
        for (int k = nc + lane; k < B - 1; k += 64) c[k] = __uint_as_float(0x7f800000u);
    }
    if (lane == 0) nb[f] = nc + 1;
}

// ---- 4. binning -------------------------------------------------------------
__device__ inline uint32_t bin_of(const float *c, int ncut, float x) {
    int lo = 0, hi = ncut;   // number of cuts <= x
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (c[mid] <= x) lo = mid + 1; else hi = mid;
    }
    return (uint32_t)lo;
}

// LDS_CUTS: the cut table (F * (B-1) floats) and nb are staged in LDS first, so the bisection's
// dependent reads stay on the CU (the table is 13 KB for 13 x 256 bins).  The feature of an element
// is carried along instead of a 64-bit modulo per element.
template <bool LDS_CUTS>
__global__ __launch_bounds__(256) void bin_dense_kernel(const float *__restrict__ X, int64_t n_elems, int F, int B,
                                                        const float *__restrict__ cuts, const int32_t *__restrict__ nb,
                                                        uint32_t missing, uint16_t *__restrict__ sym,
                                                        uint32_t *__restrict__ max_out) {
    extern __shared__ float lcuts[];
    int32_t *lnb = (int32_t *)(lcuts + (LDS_CUTS ? F * (B - 1) : 0));
    if (LDS_CUTS) {
        for (int i = threadIdx.x; i < F * (B - 1); i += 256) lcuts[i] = cuts[i];
        for (int i = threadIdx.x; i < F; i += 256) lnb[i] = nb[i];
        __syncthreads();
    }
    const float *ct = LDS_CUTS ? lcuts : cuts;
    const int32_t *nbt = LDS_CUTS ? lnb : nb;
    uint32_t mx = 0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int step_f = (int)(stride % F);
    int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int f = (int)(e % F);
    for (; e < n_elems; e += stride) {
        const float x = X[e];
        const uint32_t s = (x != x) ? missing : bin_of(ct + f * (B - 1), nbt[f] - 1, x);
        sym[e] = (uint16_t)s;
        mx = s > mx ? s : mx;
        f += step_f;
        f = f >= F ? f - F : f;
    }
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t t = (uint32_t)__shfl_xor((int)mx, o);
        mx = t > mx ? t : mx;
    }
    __shared__ uint32_t wmax[4];
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) atomicMax(max_out, max(max(wmax[0], wmax[1]), max(wmax[2], wmax[3])));
}

__global__ void fill_u16_kernel(uint16_t *p, uint16_t v, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

__global__ void bin_csr_kernel(const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                               const float *__restrict__ values, int64_t n, int64_t nnz, int F, int B,
                               const float *__restrict__ cuts, const int32_t *__restrict__ nb, uint32_t missing,
                               uint16_t *__restrict__ sym, uint32_t *__restrict__ max_out) {
    uint32_t mx = 0;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n;
         r += (int64_t)gridDim.x * blockDim.x) {
        int64_t a = indptr[r], b = indptr[r + 1];
        if (a < 0) a = 0;
        if (b > nnz) b = nnz;
        bool any_missing = (b - a) < F;
        for (int64_t i = a; i < b; ++i) {
            const int f = indices[i];
            if (f < 0 || f >= F) continue;
            const float x = values[i];
            const uint32_t s = (x != x) ? missing : bin_of(cuts + (int64_t)f * (B - 1), nb[f] - 1, x);
            sym[r * F + f] = (uint16_t)s;
            mx = s > mx ? s : mx;
        }
        if (any_missing) mx = missing > mx ? missing : mx;
    }
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t t = (uint32_t)__shfl_xor((int)mx, o);
        mx = t > mx ? t : mx;
    }
    if ((threadIdx.x & 63) == 0) atomicMax(max_out, mx);
}

// ---- 4b. binning and packing in one pass (Sec. 2.1 -> Sec. 2.2) ------------------
// The symbols of a tile of elements are binned into LDS and leave as words of the bit stream: the uint16 symbol
// matrix never exists.  A tile holds a multiple of 32 elements, so it starts on a word boundary whatever the width;
// one thread assembles one word from the LDS symbols that overlap it.
constexpr int kPackTile = 4096;   // elements per tile of the dense form

__device__ inline void pack_tile(const uint16_t *lsym, int tile_elems, int bits, uint32_t *out) {
    const int nw = (tile_elems * bits + 31) >> 5;
    for (int w = threadIdx.x; w < nw; w += 256) {
        const int bit0 = w * 32;
        uint32_t word = 0;
        for (int e = bit0 / bits; e < tile_elems; ++e) {
            const int pos = e * bits - bit0;   // may be negative for the first element
            if (pos >= 32) break;
            const uint32_t sv = lsym[e];
            word |= pos >= 0 ? (sv << pos) : (sv >> (-pos));
        }
        out[w] = word;
    }
}

template <bool LDS_CUTS>
__global__ __launch_bounds__(256) void bin_pack_dense_kernel(const float *__restrict__ X, int64_t n_elems, int F, int B,
                                                             const float *__restrict__ cuts,
                                                             const int32_t *__restrict__ nb, uint32_t missing, int bits,
                                                             uint32_t *__restrict__ packed, int64_t n_words) {
    extern __shared__ float lcuts[];
    int32_t *lnb = (int32_t *)(lcuts + (LDS_CUTS ? F * (B - 1) : 0));
    __shared__ uint16_t lsym[kPackTile];
    if (LDS_CUTS) {
        for (int i = threadIdx.x; i < F * (B - 1); i += 256) lcuts[i] = cuts[i];
        for (int i = threadIdx.x; i < F; i += 256) lnb[i] = nb[i];
        __syncthreads();
    }
    const float *ct = LDS_CUTS ? lcuts : cuts;
    const int32_t *nbt = LDS_CUTS ? lnb : nb;
    const int64_t n_tiles = (n_elems + kPackTile - 1) / kPackTile;
    const int step_f = 256 % F;
    for (int64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const int64_t e0 = t * kPackTile;
        const int tile_elems = n_elems - e0 < kPackTile ? (int)(n_elems - e0) : kPackTile;
        int f = (int)((e0 + threadIdx.x) % F);
        float x[kPackTile / 256];
#pragma unroll
        for (int j = 0; j < kPackTile / 256; ++j) {
            const int i = j * 256 + (int)threadIdx.x;
            x[j] = i < tile_elems ? X[e0 + i] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < kPackTile / 256; ++j) {
            const int i = j * 256 + (int)threadIdx.x;
            if (i < tile_elems)
                lsym[i] = (uint16_t)((x[j] != x[j]) ? missing : bin_of(ct + f * (B - 1), nbt[f] - 1, x[j]));
            f += step_f;
            f = f >= F ? f - F : f;
        }
        __syncthreads();
        pack_tile(lsym, tile_elems, bits, packed + e0 / 32 * bits);   // kPackTile * bits / 32 words per tile
        __syncthreads();
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) packed[n_words - 1] = 0;   // the pad word (Sec. 2.2 layout)
}

// CSR input: a tile of rows (a multiple of 32) is laid out in LDS as missing symbols, the stored values of those
// rows (one contiguous piece of the CSR arrays) are binned into their places, and the tile is packed.
__global__ __launch_bounds__(256) void bin_pack_csr_kernel(const int64_t *__restrict__ indptr,
                                                           const int32_t *__restrict__ indices,
                                                           const float *__restrict__ values, int64_t n, int64_t nnz,
                                                           int F, int B, const float *__restrict__ cuts,
                                                           const int32_t *__restrict__ nb, uint32_t missing, int bits,
                                                           int tile_rows, uint32_t *__restrict__ packed,
                                                           int64_t n_words) {
    extern __shared__ uint16_t lrow[];                       // tile_rows * F symbols
    int64_t *lptr = (int64_t *)(lrow + (((size_t)tile_rows * F + 3) & ~(size_t)3));   // tile_rows + 1 row pointers
    const int64_t n_tiles = (n + tile_rows - 1) / tile_rows;
    for (int64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const int64_t r0 = t * tile_rows;
        const int rows = n - r0 < tile_rows ? (int)(n - r0) : tile_rows;
        for (int i = threadIdx.x; i < rows * F; i += 256) lrow[i] = (uint16_t)missing;
        for (int i = threadIdx.x; i <= rows; i += 256) {
            int64_t p = indptr[r0 + i];
            p = p < 0 ? 0 : p;
            lptr[i] = p > nnz ? nnz : p;
        }
        __syncthreads();
        const int64_t a0 = lptr[0], b0 = lptr[rows];
        for (int64_t i = a0 + threadIdx.x; i < b0; i += 256) {
            int lo = 0, hi = rows;   // last row whose first entry is at or before i
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (lptr[mid] <= i) lo = mid; else hi = mid;
            }
            const int f = indices[i];
            if (f < 0 || f >= F) continue;
            const float x = values[i];
            lrow[lo * F + f] = (uint16_t)((x != x) ? missing : bin_of(cuts + (int64_t)f * (B - 1), nb[f] - 1, x));
        }
        __syncthreads();
        pack_tile(lrow, rows * F, bits, packed + (r0 * F) / 32 * bits);   // r0 * F is a multiple of 32
        __syncthreads();
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) packed[n_words - 1] = 0;
}

// Does any element lack a value?  A row with fewer than F stored entries, or a stored NaN.
__global__ void csr_any_missing_kernel(const int64_t *__restrict__ indptr, const float *__restrict__ values, int64_t n,
                                       int64_t nnz, int F, uint32_t *__restrict__ flag) {
    bool any = false;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x, i0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t r = i0; r < n; r += stride) {
        int64_t a = indptr[r], b = indptr[r + 1];
        a = a < 0 ? 0 : a;
        b = b > nnz ? nnz : b;
        any |= (b - a) < F;
    }
    for (int64_t i = i0; i < nnz; i += stride) {
        const float x = values[i];
        any |= x != x;
    }
    if (__ballot(any) != 0 && (threadIdx.x & 63) == 0) atomicOr(flag, 1u);
}

struct QLayout {
    size_t keys_a, keys_b, tile_hist, chunk_tot, seg_off, blk_off, chk_off, counts, cursor, seg_flags, present, misc, total;
    int64_t max_tiles, max_chunks;
};
QLayout q_layout(int64_t n, int F, int64_t n_values) {
    (void)n;
    QLayout L;
    L.max_tiles = n_values / kSortTile + F + 1;
    size_t o = 0;
    L.keys_a = o;    o += gbt_align((size_t)n_values * 4 + 4);
    L.keys_b = o;    o += gbt_align((size_t)n_values * 4 + 4);
    L.tile_hist = o; o += gbt_align((size_t)L.max_tiles * 256 * 4);
    L.max_chunks = L.max_tiles / 128 + F + 1;
    L.chunk_tot = o; o += gbt_align((size_t)L.max_chunks * 256 * 4);
    L.seg_off = o;   o += gbt_align((size_t)(F + 1) * 8);
    L.blk_off = o;   o += gbt_align((size_t)(F + 1) * 4);
    L.chk_off = o;   o += gbt_align((size_t)(F + 1) * 4);
    L.counts = o;    o += gbt_align((size_t)F * 4);
    L.cursor = o;    o += gbt_align((size_t)F * 4);
    L.seg_flags = o; o += gbt_align((size_t)F * 4);
    L.present = o;   o += gbt_align((size_t)F * 4);
    L.misc = o;      o += 256;
    L.total = o;
    return L;
}

inline int grid_for(int64_t count, int per_block, int cap) {
    int64_t g = (count + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace

size_t gbt_quantise_ws(int64_t n, int F, int64_t n_values, int B) {
    (void)B;
    return q_layout(n, F, n_values).total;
}

#define Q_HIP(call)                        \
    do {                                   \
        hipError_t e_ = (call);            \
        if (e_ != hipSuccess) return e_;   \
    } while (0)

hipError_t gbt_quantise_run(gbt_ctx *ctx, const float *X, const int64_t *indptr, const int32_t *indices,
                            const float *values, int64_t n, int F, int64_t n_values, int B, float *cuts,
                            int32_t *nb, uint16_t *sym, int32_t *max_value, int32_t *missing_sym, char *ws,
                            size_t ws_bytes, int32_t *status, uint32_t *packed, int64_t packed_cap_words,
                            int32_t *bits_out) {
    (void)ws_bytes;
    *status = GBT_OK;
    hipStream_t s = ctx->stream;
    const QLayout L = q_layout(n, F, n_values);
    uint32_t *keys_a = (uint32_t *)(ws + L.keys_a), *keys_b = (uint32_t *)(ws + L.keys_b);
    uint32_t *tile_hist = (uint32_t *)(ws + L.tile_hist);
    uint64_t *seg_off = (uint64_t *)(ws + L.seg_off);
    uint32_t *blk_off = (uint32_t *)(ws + L.blk_off);
    uint32_t *chk_off = (uint32_t *)(ws + L.chk_off);
    uint32_t *chunk_tot = (uint32_t *)(ws + L.chunk_tot);
    uint32_t *counts = (uint32_t *)(ws + L.counts), *cursor = (uint32_t *)(ws + L.cursor);
    uint32_t *misc = (uint32_t *)(ws + L.misc);
    uint32_t *seg_flags = (uint32_t *)(ws + L.seg_flags);
    uint32_t *present = (uint32_t *)(ws + L.present);
    const bool dense = X != nullptr;

    // 1. key segments
    if (dense) {
        offsets_kernel<<<1, 1, 0, s>>>(nullptr, F, n, seg_off, blk_off, chk_off, kScanChunk);
        if (n > 0 && F <= 64) {
            const size_t lds = (size_t)kTrNarrowRows * (F | 1) * 4;   // at most 65 KB
            GbtLdsGuard lds_guard(lds);
            if (lds_guard.needed) {
                Q_HIP(hipFuncSetAttribute((const void *)dense_keys_narrow_kernel,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            }
            dense_keys_narrow_kernel<<<(unsigned)((n + kTrNarrowRows - 1) / kTrNarrowRows), 256, lds, s>>>(X, n, F,
                                                                                                           keys_a);
        } else if (n > 0) {
            dim3 grid((unsigned)((n + kTrRows - 1) / kTrRows), (unsigned)((F + kTrCols - 1) / kTrCols));
            dense_keys_kernel<<<grid, 256, 0, s>>>(X, n, F, keys_a);
        }
    } else {
        Q_HIP(gbt_launch_fill_u64(s, (uint64_t *)counts, 0, (int64_t)(gbt_align((size_t)F * 4) / 8)));
        Q_HIP(gbt_launch_fill_u64(s, (uint64_t *)cursor, 0, (int64_t)(gbt_align((size_t)F * 4) / 8)));
        const int csr_grid = (int)((n_values + kCsrChunk - 1) / kCsrChunk);
        if (n_values > 0) csr_count_kernel<<<csr_grid, 256, 0, s>>>(indices, n_values, F, counts);
        offsets_kernel<<<1, 1, 0, s>>>(counts, F, 0, seg_off, blk_off, chk_off, kScanChunk);
        if (n_values > 0)
            csr_scatter_kernel<<<csr_grid, 256, 0, s>>>(indices, values, n_values, F, seg_off, cursor, keys_a);
    }
    Q_HIP(hipGetLastError());
    // number of sort tiles
    Q_HIP(hipMemcpyAsync(ctx->pinned + GBT_STAGING_BYTES / 2, blk_off + F, 4, hipMemcpyDeviceToHost, s));
    Q_HIP(hipMemcpyAsync(ctx->pinned + GBT_STAGING_BYTES / 2 + 4, chk_off + F, 4, hipMemcpyDeviceToHost, s));
    Q_HIP(hipStreamSynchronize(s));
    uint32_t n_tiles, n_chunks;
    memcpy(&n_tiles, ctx->pinned + GBT_STAGING_BYTES / 2, 4);
    memcpy(&n_chunks, ctx->pinned + GBT_STAGING_BYTES / 2 + 4, 4);
    if ((int64_t)n_tiles > L.max_tiles || (int64_t)n_chunks > L.max_chunks) {
        *status = gbt_fail(ctx, GBT_EINVAL, "gbt_quantise: inconsistent input (tile count)");
        return hipSuccess;
    }

    // 2. four stable 8-bit passes between the two key buffers; a segment skips the passes whose digit is the same
    //    for all its keys (small integers stored as floats: the low mantissa bytes) and stays where it is
    Q_HIP(gbt_launch_fill_u64(s, (uint64_t *)seg_flags, 0, (int64_t)(gbt_align((size_t)F * 4) / 8)));
    for (int pass = 0; pass < 4 && n_tiles > 0; ++pass) {
        const int shift = pass * 8;
        sort_hist_kernel<<<n_tiles, kSortBlock, 0, s>>>(keys_a, keys_b, seg_flags, seg_off, blk_off, F, shift, tile_hist);
        scan_partial_kernel<<<n_chunks, 256, 0, s>>>(blk_off, chk_off, F, tile_hist, chunk_tot);
        scan_chunks_kernel<<<F, 256, 0, s>>>(chk_off, seg_off, seg_flags, chunk_tot);
        scan_apply_kernel<<<n_chunks, 256, 0, s>>>(blk_off, chk_off, F, tile_hist, chunk_tot);
        sort_scatter_kernel<<<n_tiles, kSortBlock, 0, s>>>(keys_a, keys_b, seg_flags, seg_off, blk_off, F, shift, tile_hist);
        flip_kernel<<<(F + 255) / 256, 256, 0, s>>>(seg_flags, F);
    }
    Q_HIP(hipGetLastError());

    // 3. cuts
    cuts_kernel<<<F, 64, 0, s>>>(keys_a, keys_b, seg_flags, seg_off, F, B, cuts, nb, present);
    Q_HIP(hipGetLastError());
    std::vector<int32_t> hnb((size_t)F);
    Q_HIP(hipMemcpyAsync(hnb.data(), nb, (size_t)F * 4, hipMemcpyDeviceToHost, s));
    Q_HIP(hipStreamSynchronize(s));
    int32_t miss = 1;
    for (int f = 0; f < F; ++f) miss = hnb[f] > miss ? hnb[f] : miss;
    if (miss > 65535) {
        *status = gbt_fail(ctx, GBT_EUNSUPPORTED, "gbt_quantise: %d bins do not fit a 16-bit symbol", miss);
        return hipSuccess;
    }

    if (packed) {
        // 4b. symbols straight into the bit stream.  Its width follows from the largest symbol, which is known
        //     without binning: the largest present value of a feature falls into its last bin, and the missing
        //     symbol (max_f nb[f]) occurs iff some element has no value.
        bool any_missing;
        if (dense) {
            std::vector<uint32_t> hp((size_t)F);
            Q_HIP(hipMemcpyAsync(hp.data(), present, (size_t)F * 4, hipMemcpyDeviceToHost, s));
            Q_HIP(hipStreamSynchronize(s));
            uint64_t tot = 0;
            for (int f = 0; f < F; ++f) tot += hp[f];
            any_missing = tot < (uint64_t)n * (uint64_t)F;
        } else {
            Q_HIP(gbt_launch_fill_u64(s, (uint64_t *)misc, 0, 1));
            if (n > 0)
                csr_any_missing_kernel<<<grid_for(n > n_values ? n : n_values, 256 * 8, 4096), 256, 0, s>>>(
                    indptr, values, n, n_values, F, misc);
            Q_HIP(hipGetLastError());
            Q_HIP(hipMemcpyAsync(ctx->pinned + GBT_STAGING_BYTES / 2, misc, 4, hipMemcpyDeviceToHost, s));
            Q_HIP(hipStreamSynchronize(s));
            uint32_t fl;
            memcpy(&fl, ctx->pinned + GBT_STAGING_BYTES / 2, 4);
            any_missing = fl != 0;
        }
        const int32_t mx = n == 0 ? 0 : (any_missing ? miss : miss - 1);
        const int bits = gbt_bits((uint32_t)mx);
        if (bits > GBT_MAX_BITS) {
            *status = gbt_fail(ctx, GBT_EUNSUPPORTED, "gbt_quantise_packed: symbols need %d bits", bits);
            return hipSuccess;
        }
        const int64_t n_words = gbt_packed_words(n, F, bits);
        if (n_words > packed_cap_words) {
            *status = gbt_fail(ctx, GBT_ENOMEM, "gbt_quantise_packed: %lld words needed for %d-bit symbols, %lld given",
                               (long long)n_words, bits, (long long)packed_cap_words);
            return hipSuccess;
        }
        const int64_t n_elems = n * (int64_t)F;
        if (dense) {
            const size_t cut_bytes = ((size_t)F * (B - 1) + (size_t)F) * 4;
            const int grid = grid_for(n_elems, kPackTile, 8192);
            if (cut_bytes <= 48u * 1024u)
                bin_pack_dense_kernel<true><<<grid, 256, cut_bytes, s>>>(X, n_elems, F, B, cuts, nb, (uint32_t)miss, bits,
                                                                         packed, n_words);
            else
                bin_pack_dense_kernel<false><<<grid, 256, 0, s>>>(X, n_elems, F, B, cuts, nb, (uint32_t)miss, bits,
                                                                  packed, n_words);
        } else {
            int tile_rows = 256;
            while (tile_rows >= 32 && (size_t)tile_rows * F * 2 + 8 + ((size_t)tile_rows + 1) * 8 > 48u * 1024u) tile_rows -= 32;
            if (tile_rows < 32) {
                *status = gbt_fail(ctx, GBT_EUNSUPPORTED, "gbt_quantise_packed: CSR rows of %d features do not fit the "
                                   "packing tile; use gbt_quantise and gbt_compress", F);
                return hipSuccess;
            }
            const size_t lds = (((size_t)tile_rows * F + 3) & ~(size_t)3) * 2 + ((size_t)tile_rows + 1) * 8;
            bin_pack_csr_kernel<<<grid_for(n, tile_rows, 8192), 256, lds, s>>>(indptr, indices, values, n, n_values, F, B,
                                                                             cuts, nb, (uint32_t)miss, bits, tile_rows,
                                                                             packed, n_words);
        }
        Q_HIP(hipGetLastError());
        Q_HIP(hipStreamSynchronize(s));
        *max_value = mx;
        *missing_sym = miss;
        *bits_out = bits;
        return hipSuccess;
    }

    // 4. symbols
    Q_HIP(gbt_launch_fill_u64(s, (uint64_t *)misc, 0, 1));
    if (n > 0) {
        if (dense) {
            const size_t cut_bytes = ((size_t)F * (B - 1) + (size_t)F) * 4;
            if (cut_bytes <= 60u * 1024u) {
                GbtLdsGuard lds_guard(cut_bytes);
                if (lds_guard.needed) {
                    Q_HIP(hipFuncSetAttribute((const void *)bin_dense_kernel<true>,
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)cut_bytes));
                }
                bin_dense_kernel<true><<<grid_for(n * (int64_t)F, 4096, 8192), 256, cut_bytes, s>>>(
                    X, n * (int64_t)F, F, B, cuts, nb, (uint32_t)miss, sym, misc);
            } else {
                bin_dense_kernel<false><<<grid_for(n * (int64_t)F, 1024, 16384), 256, 0, s>>>(
                    X, n * (int64_t)F, F, B, cuts, nb, (uint32_t)miss, sym, misc);
            }
        } else {
            fill_u16_kernel<<<grid_for(n * (int64_t)F, 2048, 16384), 256, 0, s>>>(sym, (uint16_t)miss,
                                                                                   n * (int64_t)F);
            bin_csr_kernel<<<grid_for(n, 256, 16384), 256, 0, s>>>(indptr, indices, values, n, n_values, F, B, cuts,
                                                                   nb, (uint32_t)miss, sym, misc);
        }
    }
    Q_HIP(hipGetLastError());
    Q_HIP(hipMemcpyAsync(ctx->pinned + GBT_STAGING_BYTES / 2, misc, 4, hipMemcpyDeviceToHost, s));
    Q_HIP(hipStreamSynchronize(s));
    uint32_t mx;
    memcpy(&mx, ctx->pinned + GBT_STAGING_BYTES / 2, 4);
    *max_value = (int32_t)mx;
    *missing_sym = miss;
    return hipSuccess;
}
