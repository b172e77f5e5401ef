// Row ids in leaf order for a tree that was grown without following the rows.
//
// RepartitionInstances of Alg. 1, applied level after level as a stable filter to the id list
// 0..n-1, ends with the rows grouped by leaf, the leaves in left-to-right order of the tree and the
// ids ascending inside each leaf.  That final list is a stable sort of the row ids by the rank of
// each row's leaf in left-to-right order, so it can be made after the fact from one walk of the
// finished tree (which names each row's leaf) instead of carrying ids through every level:
// an LSD radix sort of (rank, row) pairs with 8-bit digits, one pass per 8 bits of the largest rank.
// The first pass takes its keys from the leaf ids through a rank table and its values from the row
// positions; the last pass writes only the values.
//
// Per pass: a digit histogram per tile of 8192 rows, offsets from a scan over the tiles (thread d
// owns digit d), then a stable scatter that first orders the tile inside LDS so that each digit's
// run leaves as consecutive words.
#include "gbt_internal.h"

namespace {

constexpr int kOrdBlock = 512;
constexpr int kOrdWaves = kOrdBlock / 64;
constexpr int kOrdTile = 8192;
constexpr int kOrdPerThread = kOrdTile / kOrdBlock;          // 16
constexpr int kOrdPerWave = kOrdTile / kOrdWaves;            // 1024
constexpr int kOrdRounds = kOrdPerWave / 64;                 // 16
constexpr int kOrdChunk = 128;                               // tiles per scan chunk

// the key of position p: pass 0 reads the row's leaf and looks its rank up
template <bool FIRST>
__device__ inline uint32_t order_key(const int32_t *__restrict__ leaf, const uint32_t *__restrict__ rank_tbl,
                                     uint32_t n_nodes, const uint32_t *__restrict__ key_in, int64_t p) {
    if (FIRST) {
        uint32_t id = (uint32_t)leaf[p];
        id = id < n_nodes ? id : n_nodes - 1;   // the table has n_nodes entries
        return rank_tbl[id];
    }
    return key_in[p];
}

template <bool FIRST>
__global__ __launch_bounds__(kOrdBlock) void order_count_kernel(const int32_t *__restrict__ leaf,
                                                                const uint32_t *__restrict__ rank_tbl,
                                                                uint32_t n_nodes,
                                                                const uint32_t *__restrict__ key_in, int64_t n,
                                                                int shift, uint32_t *__restrict__ tile_hist) {
    __shared__ uint32_t h[256];
    if (threadIdx.x < 256) h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t t0 = (int64_t)blockIdx.x * kOrdTile;
    if (t0 + kOrdTile <= n) {   // a whole tile: every load is issued before the first count
        uint32_t k[kOrdPerThread];
#pragma unroll
        for (int j = 0; j < kOrdPerThread; ++j)
            k[j] = order_key<FIRST>(leaf, rank_tbl, n_nodes, key_in, t0 + (int64_t)j * kOrdBlock + threadIdx.x);
#pragma unroll
        for (int j = 0; j < kOrdPerThread; ++j) atomicAdd(&h[(k[j] >> shift) & 255u], 1u);
    } else {
        for (int64_t p = t0 + threadIdx.x; p < n; p += kOrdBlock)
            atomicAdd(&h[(order_key<FIRST>(leaf, rank_tbl, n_nodes, key_in, p) >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (threadIdx.x < 256) tile_hist[(int64_t)blockIdx.x * 256 + threadIdx.x] = h[threadIdx.x];
}

// tile_hist[t][d] becomes the output position of the first digit-d element of tile t:
//   partial: one workgroup per chunk of kOrdChunk tiles adds up the chunk's counts per digit;
//   chunks : one workgroup makes the chunk totals exclusive over the chunks and adds the number of
//            elements with a smaller digit;
//   apply  : one workgroup per chunk walks its tiles from the chunk's start.
__global__ __launch_bounds__(256) void order_scan_partial_kernel(const uint32_t *__restrict__ tile_hist,
                                                                 int n_tiles, uint32_t *__restrict__ chunk_tot) {
    const int d = threadIdx.x;
    const int b0 = blockIdx.x * kOrdChunk, b1 = b0 + kOrdChunk < n_tiles ? b0 + kOrdChunk : n_tiles;
    uint32_t run = 0;
    for (int b = b0; b < b1; ++b) run += tile_hist[(int64_t)b * 256 + d];
    chunk_tot[(int64_t)blockIdx.x * 256 + d] = run;
}

__global__ __launch_bounds__(256) void order_scan_chunks_kernel(uint32_t *__restrict__ chunk_tot, int n_chunks) {
    const int d = threadIdx.x;
    uint32_t run = 0;
    for (int c = 0; c < n_chunks; ++c) {
        const uint32_t v = chunk_tot[(int64_t)c * 256 + d];
        chunk_tot[(int64_t)c * 256 + d] = run;
        run += v;
    }
    __shared__ uint32_t tot[256];
    tot[d] = run;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
        const uint32_t v = d >= o ? tot[d - o] : 0;
        __syncthreads();
        tot[d] += v;
        __syncthreads();
    }
    const uint32_t base = tot[d] - run;   // elements with a smaller digit
    for (int c = 0; c < n_chunks; ++c) chunk_tot[(int64_t)c * 256 + d] += base;
}

__global__ __launch_bounds__(256) void order_scan_apply_kernel(uint32_t *__restrict__ tile_hist, int n_tiles,
                                                               const uint32_t *__restrict__ chunk_tot) {
    const int d = threadIdx.x;
    const int b0 = blockIdx.x * kOrdChunk, b1 = b0 + kOrdChunk < n_tiles ? b0 + kOrdChunk : n_tiles;
    uint32_t run = chunk_tot[(int64_t)blockIdx.x * 256 + d];
    for (int b = b0; b < b1; ++b) {
        const uint32_t c = tile_hist[(int64_t)b * 256 + d];
        tile_hist[(int64_t)b * 256 + d] = run;
        run += c;
    }
}

// Stable scatter of one tile.  Wave w holds positions [w * 1024, (w + 1) * 1024) of the tile, 64 per
// round, so that (wave, round, lane) order is position order.  Ranks inside the tile come from
// per-wave digit counts (made exclusive over digits and waves) and, inside a round, from ballots.
template <bool FIRST, bool LAST>
__global__ __launch_bounds__(kOrdBlock) void order_scatter_kernel(const int32_t *__restrict__ leaf,
                                                                  const uint32_t *__restrict__ rank_tbl,
                                                                  uint32_t n_nodes,
                                                                  const uint32_t *__restrict__ key_in,
                                                                  const uint32_t *__restrict__ val_in, int64_t n,
                                                                  int shift, int digit_bits,
                                                                  const uint32_t *__restrict__ tile_hist,
                                                                  uint32_t *__restrict__ key_out,
                                                                  uint32_t *__restrict__ val_out) {
    __shared__ uint32_t cnt[kOrdWaves][256];   // per wave: running local position per digit
    __shared__ uint32_t local_start[256];      // first local position of each digit's run
    __shared__ uint32_t run_base[256];         // output position of each digit's run
    __shared__ uint32_t wave_tot[4];
    __shared__ uint32_t stage[kOrdTile];       // the tile in output order: values first, then keys
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t t0 = (int64_t)blockIdx.x * kOrdTile;
    const uint32_t tile_rows = n - t0 < (int64_t)kOrdTile ? (uint32_t)(n - t0) : (uint32_t)kOrdTile;
    for (int i = threadIdx.x; i < kOrdWaves * 256; i += kOrdBlock) (&cnt[0][0])[i] = 0;
    __syncthreads();

    uint32_t key[kOrdRounds], val[kOrdRounds], pos[kOrdRounds];
    const uint32_t w0 = (uint32_t)wave * kOrdPerWave;
    if (tile_rows == (uint32_t)kOrdTile) {
#pragma unroll
        for (int r = 0; r < kOrdRounds; ++r) {
            const uint32_t q = w0 + (uint32_t)r * 64 + lane;
            key[r] = order_key<FIRST>(leaf, rank_tbl, n_nodes, key_in, t0 + q);
            val[r] = FIRST ? 0u : val_in[t0 + q];
        }
    } else {
#pragma unroll
        for (int r = 0; r < kOrdRounds; ++r) {
            const uint32_t q = w0 + (uint32_t)r * 64 + lane;
            key[r] = q < tile_rows ? order_key<FIRST>(leaf, rank_tbl, n_nodes, key_in, t0 + q) : 0u;
            val[r] = (FIRST || q >= tile_rows) ? 0u : val_in[t0 + q];
        }
    }
#pragma unroll
    for (int r = 0; r < kOrdRounds; ++r) {
        const uint32_t q = w0 + (uint32_t)r * 64 + lane;
        if (q < tile_rows) atomicAdd(&cnt[wave][(key[r] >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (threadIdx.x < 256) {   // thread d: digit d's run inside the tile, and each wave's share of it
        const int d = threadIdx.x;
        uint32_t total = 0;
        for (int w = 0; w < kOrdWaves; ++w) total += cnt[w][d];
        uint32_t x = total;
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t y = (uint32_t)__shfl_up((int)x, o);
            if (lane >= o) x += y;
        }
        if (lane == 63) wave_tot[wave] = x;
        // (the four waves of this branch meet at the barrier below)
        local_start[d] = x - total;   // so far exclusive inside the wave's 64 digits
        run_base[d] = tile_hist[(int64_t)blockIdx.x * 256 + d];
    }
    __syncthreads();
    if (threadIdx.x < 256) {
        const int d = threadIdx.x;
        uint32_t before = 0;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        const uint32_t start = local_start[d] + before;
        local_start[d] = start;
        uint32_t run = start;
        for (int w = 0; w < kOrdWaves; ++w) {
            const uint32_t c = cnt[w][d];
            cnt[w][d] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kOrdRounds; ++r) {
        const uint32_t q = w0 + (uint32_t)r * 64 + lane;
        const bool live = q < tile_rows;
        const uint32_t dgt = (key[r] >> shift) & 255u;
        uint64_t peers = __ballot(live);   // lanes of this round with the same digit
        for (int b = 0; b < digit_bits; ++b) {
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
        pos[r] = first + below;   // < tile_rows for a live lane
        if (live) stage[pos[r]] = FIRST ? (q | (dgt << 16)) : val[r];   // FIRST: the value of a row is its position
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < tile_rows; i += kOrdBlock) {
        const uint32_t v = stage[i];
        uint32_t d;
        if (FIRST) {
            d = v >> 16;
        } else {   // the last run that starts at or before i
            int lo = 0, hi = 256;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (local_start[mid] <= i) lo = mid; else hi = mid;
            }
            d = (uint32_t)lo;
        }
        val_out[run_base[d] + (i - local_start[d])] = FIRST ? (uint32_t)t0 + (v & 0xffffu) : v;
    }
    if (!LAST) {   // the keys travel with the values into the next pass
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kOrdRounds; ++r)
            if (w0 + (uint32_t)r * 64 + lane < tile_rows) stage[pos[r]] = key[r];
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < tile_rows; i += kOrdBlock) {
            const uint32_t k = stage[i], d = (k >> shift) & 255u;
            key_out[run_base[d] + (i - local_start[d])] = k;
        }
    }
}


}  // namespace

int gbt_order_tile() { return kOrdTile; }


size_t gbt_order_ws(int64_t n) {
    const int64_t tiles = (n + kOrdTile - 1) / kOrdTile, chunks = (tiles + kOrdChunk - 1) / kOrdChunk;
    return gbt_align((size_t)(tiles + 1) * 1024) + gbt_align((size_t)(chunks + 1) * 1024);
}

hipError_t gbt_launch_order_rows(hipStream_t s, const int32_t *leaf, const uint32_t *rank_tbl, uint32_t n_nodes,
                                 uint32_t n_ranks, int64_t n, uint32_t *key_tmp[2], uint32_t *val_tmp[2], char *ws,
                                 uint32_t *row_idx_out) {
    if (n <= 0) return hipSuccess;
    if (n_ranks <= 1) return gbt_launch_iota_u32(s, row_idx_out, n);   // one leaf: the ids in order
    int rank_bits = 1;
    while (rank_bits < 32 && (1ull << rank_bits) < (unsigned long long)n_ranks) ++rank_bits;
    const int passes = (rank_bits + 7) / 8;
    const int n_tiles = (int)((n + kOrdTile - 1) / kOrdTile), n_chunks = (n_tiles + kOrdChunk - 1) / kOrdChunk;
    uint32_t *tile_hist = (uint32_t *)ws;
    uint32_t *chunk_tot = (uint32_t *)(ws + gbt_align((size_t)(n_tiles + 1) * 1024));
    const uint32_t *kin = nullptr, *vin = nullptr;
    for (int p = 0; p < passes; ++p) {
        const bool first = p == 0, last = p == passes - 1;
        const int shift = 8 * p;
        const int digit_bits = rank_bits - shift < 8 ? rank_bits - shift : 8;
        if (first)
            order_count_kernel<true><<<n_tiles, kOrdBlock, 0, s>>>(leaf, rank_tbl, n_nodes, nullptr, n, shift, tile_hist);
        else
            order_count_kernel<false><<<n_tiles, kOrdBlock, 0, s>>>(nullptr, nullptr, 0, kin, n, shift, tile_hist);
        order_scan_partial_kernel<<<n_chunks, 256, 0, s>>>(tile_hist, n_tiles, chunk_tot);
        order_scan_chunks_kernel<<<1, 256, 0, s>>>(chunk_tot, n_chunks);
        order_scan_apply_kernel<<<n_chunks, 256, 0, s>>>(tile_hist, n_tiles, chunk_tot);
        uint32_t *kout = last ? nullptr : key_tmp[p & 1], *vout = last ? row_idx_out : val_tmp[p & 1];
        if (first && last)
            order_scatter_kernel<true, true><<<n_tiles, kOrdBlock, 0, s>>>(leaf, rank_tbl, n_nodes, nullptr, nullptr, n,
                                                                          shift, digit_bits, tile_hist, kout, vout);
        else if (first)
            order_scatter_kernel<true, false><<<n_tiles, kOrdBlock, 0, s>>>(leaf, rank_tbl, n_nodes, nullptr, nullptr, n,
                                                                           shift, digit_bits, tile_hist, kout, vout);
        else if (last)
            order_scatter_kernel<false, true><<<n_tiles, kOrdBlock, 0, s>>>(nullptr, nullptr, 0, kin, vin, n, shift,
                                                                           digit_bits, tile_hist, kout, vout);
        else
            order_scatter_kernel<false, false><<<n_tiles, kOrdBlock, 0, s>>>(nullptr, nullptr, 0, kin, vin, n, shift,
                                                                            digit_bits, tile_hist, kout, vout);
        kin = kout;
        vin = vout;
    }
    return hipGetLastError();
}
