// Sparse-native row layout (Sec. 1: sparse input is supported; Sec. 2.2: the quantised matrix is
// stored compressed).  A row keeps only its present elements, each as a global bin id
//     gid = feature * B + symbol            (B = max_bins),
// ascending inside the row; rowptr[r] .. rowptr[r+1] delimit row r in the entry stream.  An id takes 16 bits
// where F * B <= 65536 and 32 bits in a wider matrix (gbt_sparse_entry_bytes; the kernels are templates over the
// entry type E, the 16-bit histogram kernel is a form of its own).  A missing
// element costs nothing instead of one symbol, so a matrix that is 80% empty moves about a third
// of the bytes of its dense packing, and the histogram kernel issues atomics for present elements
// only.  gid * 2 is also the element's place in the node's [F][B][2] histogram.
//
// The entry stream is read as aligned 32-bit words, up to nine words per row and step, so the buffer
// must extend 32 entries past the last one (gbt_sparse_capacity).
#include "gbt_internal.h"
#include "wave_scan.h"

namespace {

constexpr int kHShift = 30;                        // [ g : 34 bits signed | h : 30 bits ] as in the dense kernels
constexpr uint32_t kHMask = (1u << kHShift) - 1u;

__device__ __forceinline__ unsigned long long sp_pack_pair(int2 q) {
    return ((unsigned long long)(long long)q.x << kHShift) + (unsigned long long)(uint32_t)q.y;
}

// The rare events that the packed add cannot hold -- a carry out of the h field (it lands in the g
// field as +1), a wrap of the g field -- are seen by the lane whose add caused them in the returned
// word.  It corrects the node's histogram in HBM right away (integer adds commute with the merge of
// the LDS words), so the LDS histogram needs no side counters: 8 bytes per bin.
__device__ __forceinline__ void sp_check(int64_t *out2, uint32_t idx, unsigned long long old,
                                         unsigned long long addv, uint32_t hq) {
    uint32_t olo = (uint32_t)old, ohi = (uint32_t)(old >> 32);
    const bool danger = ((olo & 0x3FC00000u) == 0x3FC00000u) | ((ohi + 0x82000000u) < 0x04000000u);
    if (danger) {
        asm volatile("" : "+v"(olo), "+v"(ohi));
        const uint32_t carry = ((olo & kHMask) + hq) >> kHShift;
        const uint32_t alo = (uint32_t)addv, ahi = (uint32_t)(addv >> 32);
        const uint32_t nlo = olo + alo;
        const uint32_t nhi = ohi + ahi + (nlo < olo ? 1u : 0u);
        const int32_t ovf = (int32_t)((ohi ^ nhi) & (ahi ^ nhi));
        const int64_t wraps = ovf < 0 ? ((int32_t)nhi < 0 ? 1 : -1) : 0;
        if (carry != 0 || wraps != 0) {
            const int64_t dg = wraps * ((int64_t)1 << (64 - kHShift)) - (int64_t)carry;
            atomicAdd((unsigned long long *)(out2 + 2 * (int64_t)idx), (unsigned long long)dg);
            if (carry) atomicAdd((unsigned long long *)(out2 + 2 * (int64_t)idx + 1), (unsigned long long)carry << kHShift);
        }
    }
}

// ---- layout conversion -----------------------------------------------------
constexpr int kScanTile = 4096;   // counts per workgroup of the scan kernels (256 threads x 16)

// len[r] = present elements of row r (sym != missing); len[n] = 0
__global__ __launch_bounds__(256) void sparse_count_kernel(const uint16_t *__restrict__ sym, int64_t n, int F,
                                                           uint32_t missing, uint32_t *__restrict__ len) {
    for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r <= n; r += (int64_t)gridDim.x * 256) {
        uint32_t c = 0;
        if (r < n) {
            const uint16_t *row = sym + r * F;
            for (int f = 0; f < F; ++f) c += row[f] != missing;
        }
        len[r] = c;
    }
}

// exclusive scan of v[0..m) in place, three launches; total (64-bit) to *total_out
__global__ __launch_bounds__(256) void scan_tile_sums_kernel(const uint32_t *__restrict__ v, int64_t m,
                                                             uint64_t *__restrict__ tile_sum) {
    __shared__ uint64_t red[4];
    const int64_t t0 = (int64_t)blockIdx.x * kScanTile;
    uint64_t s = 0;
    for (int k = 0; k < kScanTile / 256; ++k) {
        const int64_t i = t0 + (int64_t)k * 256 + threadIdx.x;
        if (i < m) s += v[i];
    }
    for (int o = 32; o > 0; o >>= 1)
        s += ((uint64_t)(uint32_t)__shfl_xor((int)(s >> 32), o) << 32) | (uint32_t)__shfl_xor((int)(uint32_t)s, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(256) void scan_tile_offsets_kernel(uint64_t *__restrict__ tile_sum, int64_t n_tiles,
                                                                uint64_t *__restrict__ total_out) {
    __shared__ uint64_t buf[256];
    uint64_t carry = 0;
    for (int64_t b0 = 0; b0 < n_tiles; b0 += 256) {
        const int64_t i = b0 + threadIdx.x;
        const uint64_t x = i < n_tiles ? tile_sum[i] : 0;
        buf[threadIdx.x] = x;
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {
            const uint64_t y = (int)threadIdx.x >= o ? buf[threadIdx.x - o] : 0;
            __syncthreads();
            buf[threadIdx.x] += y;
            __syncthreads();
        }
        if (i < n_tiles) tile_sum[i] = carry + buf[threadIdx.x] - x;
        carry += buf[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) *total_out = carry;
}

__global__ __launch_bounds__(256) void scan_apply_u32_kernel(uint32_t *__restrict__ v, int64_t m,
                                                             const uint64_t *__restrict__ tile_off) {
    // thread t owns 16 consecutive counts of the tile
    __shared__ uint32_t part[256];
    const int64_t i0 = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * 16;
    uint32_t x[16], s = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        x[k] = i0 + k < m ? v[i0 + k] : 0;
        s += x[k];
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
        const uint32_t y = (int)threadIdx.x >= o ? part[threadIdx.x - o] : 0;
        __syncthreads();
        part[threadIdx.x] += y;
        __syncthreads();
    }
    uint32_t run = (uint32_t)tile_off[blockIdx.x] + part[threadIdx.x] - s;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        if (i0 + k < m) v[i0 + k] = run;
        run += x[k];
    }
}

template <typename E>
__global__ __launch_bounds__(256) void sparse_fill_kernel(const uint16_t *__restrict__ sym, int64_t n, int F, int B,
                                                          uint32_t missing, const uint32_t *__restrict__ rowptr,
                                                          E *__restrict__ ent) {
    for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < n; r += (int64_t)gridDim.x * 256) {
        const uint16_t *row = sym + r * F;
        uint32_t o = rowptr[r];
        for (int f = 0; f < F; ++f) {
            const uint32_t s = row[f];
            if (s != missing) ent[o++] = (E)((uint32_t)f * (uint32_t)B + s);
        }
    }
}

template <typename E>
__global__ __launch_bounds__(256) void fill_tail_kernel(E *p, int count) {
    if ((int)threadIdx.x < count) p[threadIdx.x] = 0;
}

// ---- BuildPartialHistograms over sparse rows --------------------------------
// One workgroup: rows [row_begin, row_begin + n_rows), global bin ids [f0, f0 + ft) (HistJob's
// fields, reused), a private LDS histogram of that id range.  lane = one row: its entries are
// fetched 16 at a time as eight aligned words (all loads of a step in flight together) and cut out
// of registers; an entry outside the job's id range or outside the row is skipped, a step that no
// lane of the wave needs is skipped by the whole wave.
constexpr int kSpBlock = 512;
struct __attribute__((packed, aligned(4))) Words4 {   // four words at a 4-byte aligned address
    uint32_t x, y, z, w;
};

// BLOCK: 512, or 1024 for an id range whose LDS histogram leaves room for one workgroup per compute
// unit only.  TILED: the job covers part of the ids, entries outside it are skipped.
template <int BLOCK, bool TILED>
__global__ __launch_bounds__(BLOCK) void sparse_hist_kernel(const uint32_t *__restrict__ rowptr,
                                                            const uint32_t *__restrict__ ent_words,
                                                            const int2 *__restrict__ gq,
                                                            int64_t *__restrict__ pool,
                                                            const HistJob *__restrict__ jobs) {
    extern __shared__ unsigned long long lds[];
    const HistJob job = jobs[blockIdx.x];
    const uint32_t g0 = job.f0, glen = job.ft;
    int64_t *out = pool + job.hist_off + 2 * (int64_t)g0;
    for (uint32_t i = threadIdx.x; i < glen; i += BLOCK) lds[i] = 0;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < job.n_rows; i += BLOCK) {
        const uint64_t r = (uint64_t)job.row_begin + i;
        const uint32_t s = rowptr[r], len = rowptr[r + 1] - s;
        const int2 q = gq[r];
        const unsigned long long addv = sp_pack_pair(q);
        const uint32_t hq = (uint32_t)q.y;
        const uint32_t sh = (s & 1u) * 16u;               // the row starts in the upper half of its first word
        const uint32_t *wp = ent_words + (s >> 1);
        for (uint32_t k0 = 0; k0 < len; k0 += 16) {
            // nine words hold the step's 16 entries whatever the row's alignment; shifted so that
            // entry k0 + k sits at halfword k
            const Words4 lo = *(const Words4 *)(wp + (k0 >> 1));
            const Words4 hi = *(const Words4 *)(wp + (k0 >> 1) + 4);
            const uint32_t w8 = wp[(k0 >> 1) + 8];
            const uint32_t w[9] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w, w8};
            uint32_t W[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) W[k] = __builtin_amdgcn_alignbit(w[k + 1], w[k], sh);
            const uint32_t rem = len - k0;
            uint32_t rel[16];
            unsigned long long old[16];
            uint32_t live = 0;
            // all atomics of the step are issued before the first returned word is looked at
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const uint32_t gid = (k & 1) ? (W[k >> 1] >> 16) : (W[k >> 1] & 0xffffu);
                rel[k] = gid - g0;
                bool in = (uint32_t)k < rem;
                if (TILED) in = in && rel[k] < glen;
                if (in) {
                    live |= 1u << k;
                    old[k] = atomicAdd(&lds[rel[k]], addv);
                }
            }
#pragma unroll
            for (int k = 0; k < 16; ++k)
                if (live & (1u << k)) sp_check(out, rel[k], old[k], addv, hq);
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < glen; i += BLOCK) {
        const unsigned long long w = lds[i];
        if (w == 0) continue;
        const int64_t g = (int64_t)w >> kHShift;
        const int64_t h = (int64_t)(w & kHMask);
        if (g != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i), (unsigned long long)g);
        if (h != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i + 1), (unsigned long long)h);
    }
}

// The same over 32-bit ids (a matrix of more than 65536 global bin ids, whose histogram never fits one LDS tile):
// eight entries per step as two aligned four-word loads.  The ids of a row ascend, so a job that covers part of
// the ids starts at the row's first entry inside its range (bisection) and leaves the row at the first step that
// ends beyond it: a row's entries are visited about once over all the tiles, not once per tile.
template <int BLOCK, bool TILED>
__global__ __launch_bounds__(BLOCK) void sparse_hist32_kernel(const uint32_t *__restrict__ rowptr,
                                                              const uint32_t *__restrict__ ent,
                                                              const int2 *__restrict__ gq,
                                                              int64_t *__restrict__ pool,
                                                              const HistJob *__restrict__ jobs) {
    extern __shared__ unsigned long long lds[];
    const HistJob job = jobs[blockIdx.x];
    const uint32_t g0 = job.f0, glen = job.ft;
    int64_t *out = pool + job.hist_off + 2 * (int64_t)g0;
    for (uint32_t i = threadIdx.x; i < glen; i += BLOCK) lds[i] = 0;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < job.n_rows; i += BLOCK) {
        const uint64_t r = (uint64_t)job.row_begin + i;
        const uint32_t s = rowptr[r], len = rowptr[r + 1] - s;
        const int2 q = gq[r];
        const unsigned long long addv = sp_pack_pair(q);
        const uint32_t hq = (uint32_t)q.y;
        const uint32_t *wp = ent + s;
        uint32_t first = 0;
        if (TILED) {   // first entry with an id >= g0
            uint32_t b = len;
            while (first < b) {
                const uint32_t mid = first + ((b - first) >> 1);
                if (wp[mid] < g0) first = mid + 1; else b = mid;
            }
        }
        for (uint32_t k0 = first; k0 < len; k0 += 8) {
            const Words4 lo = *(const Words4 *)(wp + k0);
            const Words4 hi = *(const Words4 *)(wp + k0 + 4);
            const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            const uint32_t rem = len - k0;
            uint32_t rel[8];
            unsigned long long old[8];
            uint32_t live = 0;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                rel[k] = w[k] - g0;
                bool in = (uint32_t)k < rem;
                if (TILED) in = in && rel[k] < glen;
                if (in) {
                    live |= 1u << k;
                    old[k] = atomicAdd(&lds[rel[k]], addv);
                }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (live & (1u << k)) sp_check(out, rel[k], old[k], addv, hq);
            if (TILED && rem > 7u && rel[7] >= glen) break;   // (rel >= 0 from `first` on: ascending ids)
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < glen; i += BLOCK) {
        const unsigned long long w = lds[i];
        if (w == 0) continue;
        const int64_t g = (int64_t)w >> kHShift;
        const int64_t h = (int64_t)(w & kHMask);
        if (g != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i), (unsigned long long)g);
        if (h != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i + 1), (unsigned long long)h);
    }
}

// ---- RepartitionInstances over sparse rows ----------------------------------
// One launch per level, order inside a child not kept.  A tile of kSpTile rows finds each row's
// side (the row's entry of the split feature is looked up among its ascending ids; a row without
// one is missing and takes the default side), ranks rows and entries per side inside the tile and
// reserves room in both children with two 64-bit atomics on the node's cursors
// [ entries : high word | rows : low word ], one for each side.  Left rows and their entries fill
// the node's row range and entry range from the front, right rows from the back, so both children
// stay contiguous in rows AND in entries, and rowptr[r + 1] - rowptr[r] stays a row's length.
// move == 0: only the left rows are counted (the last level).
constexpr int kSpTile = 1024;
constexpr int kSpRowsPerThread = kSpTile / kSpBlock;   // 2
constexpr int kSpGroups = kSpRowsPerThread * (kSpBlock / 64);   // (k, wave) groups of 64 rows: 16

__device__ inline int find_part_job(const PartJob *jobs, int n_jobs, uint32_t tile) {
    int lo = 0, hi = n_jobs;   // last job with tile_begin <= tile
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (jobs[mid].tile_begin <= tile) lo = mid; else hi = mid;
    }
    return lo;
}

// the entry with an id in [lo, lo + B) among the ascending ids ent[s .. e), or 0xffffffff
template <typename P>
__device__ __forceinline__ uint32_t find_feature_entry(P ent, uint32_t s, uint32_t e, uint32_t lo, uint32_t B) {
    uint32_t a = s, b = e;   // first entry >= lo by bisection
    while (a < b) {
        const uint32_t mid = a + ((b - a) >> 1);
        if ((uint32_t)ent[mid] < lo) a = mid + 1; else b = mid;
    }
    if (a < e) {
        const uint32_t g = ent[a];
        if (g - lo < B) return g;
    }
    return 0xffffffffu;
}

// The entries of a tile's rows are one contiguous piece of the stream: it is fetched once, linearly,
// into LDS (kSpStage / 2 words; a tile with more reads the stream in place and copies it row by row, a wave
// at a time), and the feature look-ups read it there.  The tile's left rows land in one contiguous piece of
// the destination stream and its right rows in another: both are put together inside LDS (a second
// window, halfword-aligned like the destination) and leave as whole 32-bit words -- sub-word stores
// retire about one lane per clock and compute unit, whatever their addresses.
constexpr int kSpStage = 12288;

template <typename E>
__global__ __launch_bounds__(kSpBlock) void sparse_part_kernel(const uint32_t *__restrict__ src_rowptr,
                                                               const E *__restrict__ src_ent,
                                                               const int2 *__restrict__ src_gq,
                                                               uint32_t *__restrict__ dst_rowptr,
                                                               E *__restrict__ dst_ent,
                                                               int2 *__restrict__ dst_gq, uint32_t B, int move,
                                                               const PartJob *__restrict__ jobs, int n_jobs,
                                                               unsigned long long *__restrict__ cursor) {
    __shared__ uint32_t stage_w[kSpStage / 2];
    __shared__ uint32_t out_w[kSpStage / 2 + 4];
    __shared__ uint32_t grp_rows[2][kSpGroups];   // [side][group]: rows, then their exclusive offsets
    __shared__ uint32_t grp_ent[2][kSpGroups];
    __shared__ unsigned long long base[2];        // what the cursors returned
    __shared__ uint32_t tot[4];                   // rows L, rows R, entries L, entries R of the tile
    constexpr uint32_t EPW = 4 / sizeof(E), SH = EPW == 2 ? 1 : 0;   // entries per word, and its log2
    const E *stage = (const E *)stage_w;
    const int j = find_part_job(jobs, n_jobs, blockIdx.x);
    const PartJob job = jobs[j];
    const uint32_t t_local = blockIdx.x - job.tile_begin;
    const uint32_t seg_end = job.seg_begin + job.seg_len;
    const uint32_t r0 = job.seg_begin + t_local * (uint32_t)kSpTile;
    const uint32_t r1 = r0 + (uint32_t)kSpTile < seg_end ? r0 + (uint32_t)kSpTile : seg_end;
    const uint32_t lo = job.feature * B, thr = lo + job.bin;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // the tile's piece of the stream, from the word that holds its first entry
    const uint32_t e0 = src_rowptr[r0], e1 = src_rowptr[r1];
    const uint32_t w0 = e0 >> SH, n_words = ((e1 + EPW - 1) >> SH) - w0;
    const bool staged = n_words <= (uint32_t)(kSpStage / 2);
    if (staged) {
        const uint32_t *src_w = (const uint32_t *)src_ent + w0;
        for (uint32_t w = threadIdx.x; w < n_words; w += kSpBlock) stage_w[w] = src_w[w];
    }
    const uint32_t sbase = w0 << SH;   // stream index of stage[0]

    uint32_t rs[kSpRowsPerThread], rlen[kSpRowsPerThread], within_rows[kSpRowsPerThread], within_ent[kSpRowsPerThread];
    bool live[kSpRowsPerThread], left[kSpRowsPerThread];
    int2 pair[kSpRowsPerThread];
#pragma unroll
    for (int k = 0; k < kSpRowsPerThread; ++k) {
        const uint32_t r = r0 + (uint32_t)k * kSpBlock + threadIdx.x;
        live[k] = r < r1;
        rs[k] = 0;
        rlen[k] = 0;
        left[k] = false;
        pair[k] = make_int2(0, 0);
        if (live[k]) {
            rs[k] = src_rowptr[r];
            rlen[k] = src_rowptr[r + 1] - rs[k];
            if (move) pair[k] = src_gq[r];
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kSpRowsPerThread; ++k) {
        if (live[k]) {
            const uint32_t g = staged ? find_feature_entry(stage, rs[k] - sbase, rs[k] - sbase + rlen[k], lo, B)
                                      : find_feature_entry(src_ent, rs[k], rs[k] + rlen[k], lo, B);
            left[k] = g == 0xffffffffu ? job.default_left != 0 : g <= thr;
        }
    }
    // ranks inside each group of 64 rows: rows by ballot, entries by a 64-bit scan holding both sides
#pragma unroll
    for (int k = 0; k < kSpRowsPerThread; ++k) {
        const uint64_t bl = __ballot(live[k] && left[k]), br = __ballot(live[k] && !left[k]);
        const uint64_t below = (1ull << lane) - 1ull;
        within_rows[k] = (uint32_t)__popcll((left[k] ? bl : br) & below);
        unsigned long long x = !live[k] ? 0ull : left[k] ? (unsigned long long)rlen[k] : ((unsigned long long)rlen[k] << 32);
        const unsigned long long incl = (unsigned long long)wave_scan_i64((int64_t)x);
        const unsigned long long excl = incl - x;
        within_ent[k] = left[k] ? (uint32_t)excl : (uint32_t)(excl >> 32);
        if (lane == 63) {
            const int grp = k * (kSpBlock / 64) + wave;
            grp_rows[0][grp] = (uint32_t)__popcll(bl);
            grp_rows[1][grp] = (uint32_t)__popcll(br);
            grp_ent[0][grp] = (uint32_t)incl;
            grp_ent[1][grp] = (uint32_t)(incl >> 32);
        }
    }
    __syncthreads();
    if (wave == 0 && lane < 2 * kSpGroups) {   // exclusive offsets over the groups: first G lanes rows, next G entries
        static_assert(kSpGroups <= 32 && (kSpGroups & (kSpGroups - 1)) == 0, "two tables inside one wave");
        const int grp = lane & (kSpGroups - 1);
        const bool rows_tab = lane < kSpGroups;
        for (int side = 0; side < 2; ++side) {
            uint32_t *tab = rows_tab ? grp_rows[side] : grp_ent[side];
            const uint32_t v = tab[grp];
            uint32_t incl = v;
            for (int o = 1; o < kSpGroups; o <<= 1) {
                const uint32_t y = (uint32_t)__shfl_up((int)incl, o);
                if (grp >= o) incl += y;
            }
            tab[grp] = incl - v;
            if (grp == kSpGroups - 1) tot[(rows_tab ? 0 : 2) + side] = incl;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        base[0] = atomicAdd(&cursor[2 * j], ((unsigned long long)tot[2] << 32) | tot[0]);
        if (move) base[1] = atomicAdd(&cursor[2 * j + 1], ((unsigned long long)tot[3] << 32) | tot[1]);
    }
    if (!move) return;
    __syncthreads();
    const uint32_t ent_begin = src_rowptr[job.seg_begin], ent_end = src_rowptr[seg_end];
    const uint32_t row_l = job.seg_begin + (uint32_t)base[0], ent_l = ent_begin + (uint32_t)(base[0] >> 32);
    const uint32_t row_r = seg_end - (uint32_t)base[1] - tot[1], ent_r = ent_end - (uint32_t)(base[1] >> 32) - tot[3];
    if (t_local == 0 && threadIdx.x == 0) dst_rowptr[seg_end] = ent_end;   // the segment's closing row pointer
    // where the two pieces sit in the output window: at the place inside a word that they have in the stream
    const uint32_t lds_l = ent_l & (EPW - 1u);
    const uint32_t lds_r = ((lds_l + tot[2] + EPW - 1u) & ~(EPW - 1u)) + (ent_r & (EPW - 1u));
    E *outE = (E *)out_w;
#pragma unroll
    for (int k = 0; k < kSpRowsPerThread; ++k) {
        const int grp = k * (kSpBlock / 64) + wave;
        const int side = left[k] ? 0 : 1;
        const uint32_t in_piece = grp_ent[side][grp] + within_ent[k];   // the row's place inside its side's piece
        const uint32_t drow = (left[k] ? row_l : row_r) + grp_rows[side][grp] + within_rows[k];
        const uint32_t dent = (left[k] ? ent_l : ent_r) + in_piece;
        if (live[k]) {
            dst_rowptr[drow] = dent;
            dst_gq[drow] = pair[k];
            if (staged) {
                const E *from = stage + (rs[k] - sbase);
                E *to = outE + (left[k] ? lds_l : lds_r) + in_piece;
                for (uint32_t q = 0; q < rlen[k]; ++q) to[q] = from[q];
            }
        }
        if (!staged) {   // the wave copies its rows one after the other, 64 entries at a time (rlen is 0 off the tile)
            for (int l = 0; l < 64; ++l) {
                const uint32_t len_l = (uint32_t)__builtin_amdgcn_readlane((int)rlen[k], l);
                if (len_l == 0) continue;
                const uint32_t src_l = (uint32_t)__builtin_amdgcn_readlane((int)rs[k], l);
                const uint32_t dst_l = (uint32_t)__builtin_amdgcn_readlane((int)dent, l);
                for (uint32_t q = lane; q < len_l; q += 64) dst_ent[dst_l + q] = src_ent[src_l + q];
            }
        }
    }
    if (!staged) return;
    __syncthreads();
    for (int side = 0; side < 2; ++side) {
        const uint32_t gs = side == 0 ? ent_l : ent_r, ge = gs + tot[2 + side];   // the piece in the stream
        const uint32_t ls = side == 0 ? lds_l : lds_r;                             // and in the window
        if (gs == ge) continue;
        const uint32_t wfirst = (gs + EPW - 1u) >> SH, wend = ge >> SH;            // whole words [wfirst, wend)
        const uint32_t lw = (ls + (gs & (EPW - 1u))) >> SH;                        // window word of stream word wfirst
        uint32_t *dst_words = (uint32_t *)dst_ent;
        for (uint32_t w = threadIdx.x; wfirst + w < wend; w += kSpBlock) dst_words[wfirst + w] = out_w[lw + w];
        // (16-bit ids: a piece may begin and end in the middle of a word)
        if (threadIdx.x == 0 && (gs & (EPW - 1u))) dst_ent[gs] = outE[ls];
        if (threadIdx.x == 64 && (ge & (EPW - 1u)) && (ge - 1 >= gs)) dst_ent[ge - 1] = outE[ls + (ge - 1 - gs)];
    }
}

// ---- Sec. 2.4 prediction over sparse rows -----------------------------------
// One row per thread, trees in order, nodes staged in LDS as in the dense kernels; the row's entry of
// a node's feature is found by bisection over the row's ascending ids.
struct SpNode {
    int32_t feature, bin, left, right;
    int32_t dl, pad;
    double weight;
};
// A wave's 64 consecutive rows own one contiguous piece of the entry stream: the wave fetches it
// linearly into its own LDS window (kWalkWords words; a longer piece is read from the stream
// directly) and every level's look-up bisects there.
constexpr int kWalkWords = 1024;
template <typename E>
__global__ __launch_bounds__(256) void sparse_walk_kernel(const char *ws, const DevTree *trees, int n_trees,
                                                          const uint32_t *__restrict__ rowptr,
                                                          const E *__restrict__ ent, int64_t n, uint32_t B,
                                                          double eta, float *margin, int32_t *leaf_out,
                                                          int rows_per_block, int max_nodes) {
    // max_nodes == 0: the trees are too large for LDS, their nodes are read from the staged arrays
    const bool lds_nodes = max_nodes > 0;
    extern __shared__ SpNode sp_nodes[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t *st = (uint32_t *)(sp_nodes + max_nodes) + wave * kWalkWords;
    constexpr uint32_t EPW = 4 / sizeof(E), SH = EPW == 2 ? 1 : 0;
    const E *stE = (const E *)st;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
    for (int t = 0; t < n_trees; ++t) {
        const DevTree T = trees[t];
        __syncthreads();
        for (int i = threadIdx.x; lds_nodes && i < T.n_nodes; i += 256) {
            SpNode nd;
            nd.feature = ((const int32_t *)(ws + T.feature))[i];
            nd.bin = ((const int32_t *)(ws + T.bin))[i];
            nd.left = ((const int32_t *)(ws + T.left))[i];
            nd.right = ((const int32_t *)(ws + T.right))[i];
            nd.dl = ((const int32_t *)(ws + T.default_left))[i];
            nd.pad = 0;
            nd.weight = ((const double *)(ws + T.weight))[i];
            sp_nodes[i] = nd;
        }
        __syncthreads();
        for (int64_t rw = r0 + wave * 64; rw < r1; rw += 256) {   // rw: the wave's first row
            const int64_t r = rw + lane;
            const bool live = r < r1;
            const uint32_t s = live ? rowptr[r] : 0u, e = live ? rowptr[r + 1] : 0u;
            const int last = 63 - (int)__builtin_clzll(__ballot(live));   // lane 0 is live
            const uint32_t ws0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)s);
            const uint32_t we = (uint32_t)__builtin_amdgcn_readlane((int)e, last);
            const uint32_t word0 = ws0 >> SH, n_words = ((we + EPW - 1) >> SH) - word0;
            const bool fits = n_words <= (uint32_t)kWalkWords;
            if (fits) {
                const uint32_t *src_w = (const uint32_t *)ent + word0;
                for (uint32_t w = lane; w < n_words; w += 64) st[w] = src_w[w];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (live) {
                const uint32_t sb = word0 << SH;
                int node = 0;
                for (int step = 0; step < T.n_nodes; ++step) {
                    SpNode nd;
                    if (lds_nodes) {
                        nd = sp_nodes[node];
                    } else {
                        nd.feature = ((const int32_t *)(ws + T.feature))[node];
                        nd.bin = ((const int32_t *)(ws + T.bin))[node];
                        nd.left = ((const int32_t *)(ws + T.left))[node];
                        nd.right = ((const int32_t *)(ws + T.right))[node];
                        nd.dl = ((const int32_t *)(ws + T.default_left))[node];
                    }
                    if (nd.feature < 0) break;
                    const uint32_t lo = (uint32_t)nd.feature * B;
                    const uint32_t g = fits ? find_feature_entry(stE, s - sb, e - sb, lo, B)
                                            : find_feature_entry(ent, s, e, lo, B);
                    const bool go_left = g == 0xffffffffu ? nd.dl != 0 : g <= lo + (uint32_t)nd.bin;
                    node = go_left ? nd.left : nd.right;
                }
                if (leaf_out) leaf_out[r] = node;
                else margin[r] = (float)((double)margin[r] +
                                         eta * (lds_nodes ? sp_nodes[node].weight : ((const double *)(ws + T.weight))[node]));
            }
            __builtin_amdgcn_wave_barrier();   // the window is refilled only after every lane has left it
        }
    }
}

int grid_rows(int64_t n) {
    int64_t g = (n + 255) / 256;
    if (g < 1) g = 1;
    if (g > 65536) g = 65536;
    return (int)g;
}

}  // namespace

int64_t gbt_sparse_scan_tiles(int64_t n) { return (n + 1 + kScanTile - 1) / kScanTile; }

// rowptr[0..n] = exclusive scan of the rows' present counts; *total_dev (device) = number of entries
hipError_t gbt_launch_sparse_rowptr(hipStream_t s, const uint16_t *sym, int64_t n, int F, uint32_t missing,
                                    uint32_t *rowptr, uint64_t *tile_ws, uint64_t *total_dev) {
    const int64_t m = n + 1, tiles = gbt_sparse_scan_tiles(n);
    sparse_count_kernel<<<grid_rows(m), 256, 0, s>>>(sym, n, F, missing, rowptr);
    scan_tile_sums_kernel<<<(unsigned)tiles, 256, 0, s>>>(rowptr, m, tile_ws);
    scan_tile_offsets_kernel<<<1, 256, 0, s>>>(tile_ws, tiles, total_dev);
    scan_apply_u32_kernel<<<(unsigned)tiles, 256, 0, s>>>(rowptr, m, tile_ws);
    return hipGetLastError();
}

hipError_t gbt_launch_sparse_fill(hipStream_t s, const uint16_t *sym, int64_t n, int F, int B, uint32_t missing,
                                  const uint32_t *rowptr, void *ent, int ent_bytes, int64_t nnz, int64_t capacity) {
    const int64_t tail = capacity - nnz;   // the slack that word-wise readers may touch: defined values
    const int tail_n = (int)(tail < 256 ? tail : 256);
    if (ent_bytes == 2) {
        if (n > 0) sparse_fill_kernel<uint16_t><<<grid_rows(n), 256, 0, s>>>(sym, n, F, B, missing, rowptr, (uint16_t *)ent);
        if (tail > 0) fill_tail_kernel<uint16_t><<<1, 256, 0, s>>>((uint16_t *)ent + nnz, tail_n);
    } else {
        if (n > 0) sparse_fill_kernel<uint32_t><<<grid_rows(n), 256, 0, s>>>(sym, n, F, B, missing, rowptr, (uint32_t *)ent);
        if (tail > 0) fill_tail_kernel<uint32_t><<<1, 256, 0, s>>>((uint32_t *)ent + nnz, tail_n);
    }
    return hipGetLastError();
}

// ids per LDS tile for a total of `bins` global bin ids (8 bytes of LDS per id): all of them when they
// fit one workgroup's LDS at all (one pass over a row's entries then serves every id), else equal
// parts under the cap that lets several workgroups share a compute unit
int gbt_sparse_hist_tile(const gbt_ctx *ctx, int64_t bins) {
    if ((size_t)bins * 8 <= ctx->lds_per_block && !ctx->sparse_tiled) return (int)bins;
    size_t limit = ctx->lds_per_block;
    if (ctx->hist_lds_kb > 0 && (size_t)ctx->hist_lds_kb * 1024 < limit) limit = (size_t)ctx->hist_lds_kb * 1024;
    const int64_t cap = (int64_t)(limit / 8);
    const int64_t tiles = (bins + cap - 1) / cap;
    return (int)((bins + tiles - 1) / tiles);
}

// tiled: the jobs cover parts of the id range [0, bins)
hipError_t gbt_launch_sparse_hist(gbt_ctx *ctx, const uint32_t *rowptr, const void *ent, int ent_bytes, const int32_t *gq,
                                  int64_t *pool, const HistJob *jobs, int n_jobs, int max_glen, bool tiled) {
    if (n_jobs <= 0) return hipSuccess;
    const size_t lds = (size_t)max_glen * 8;
    const bool big = lds > 64u * 1024u;   // one workgroup per compute unit: make it a large one
    if (ent_bytes == 4) {
        const void *fn32 = big ? (tiled ? (const void *)sparse_hist32_kernel<1024, true> : (const void *)sparse_hist32_kernel<1024, false>)
                               : (tiled ? (const void *)sparse_hist32_kernel<512, true> : (const void *)sparse_hist32_kernel<512, false>);
        GbtLdsGuard lds_guard(lds);
        if (lds_guard.needed) {
            hipError_t e = hipFuncSetAttribute(fn32, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        const uint32_t *e32 = (const uint32_t *)ent;
        const int2 *g2 = (const int2 *)gq;
        if (big && tiled) sparse_hist32_kernel<1024, true><<<n_jobs, 1024, lds, ctx->stream>>>(rowptr, e32, g2, pool, jobs);
        else if (big) sparse_hist32_kernel<1024, false><<<n_jobs, 1024, lds, ctx->stream>>>(rowptr, e32, g2, pool, jobs);
        else if (tiled) sparse_hist32_kernel<512, true><<<n_jobs, 512, lds, ctx->stream>>>(rowptr, e32, g2, pool, jobs);
        else sparse_hist32_kernel<512, false><<<n_jobs, 512, lds, ctx->stream>>>(rowptr, e32, g2, pool, jobs);
        return hipGetLastError();
    }
    const void *fn = big ? (tiled ? (const void *)sparse_hist_kernel<1024, true> : (const void *)sparse_hist_kernel<1024, false>)
                         : (tiled ? (const void *)sparse_hist_kernel<512, true> : (const void *)sparse_hist_kernel<512, false>);
    GbtLdsGuard lds_guard(lds);
    if (lds_guard.needed) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const uint32_t *words = (const uint32_t *)ent;
    const int2 *gq2 = (const int2 *)gq;
    if (big && tiled) sparse_hist_kernel<1024, true><<<n_jobs, 1024, lds, ctx->stream>>>(rowptr, words, gq2, pool, jobs);
    else if (big) sparse_hist_kernel<1024, false><<<n_jobs, 1024, lds, ctx->stream>>>(rowptr, words, gq2, pool, jobs);
    else if (tiled) sparse_hist_kernel<512, true><<<n_jobs, 512, lds, ctx->stream>>>(rowptr, words, gq2, pool, jobs);
    else sparse_hist_kernel<512, false><<<n_jobs, 512, lds, ctx->stream>>>(rowptr, words, gq2, pool, jobs);
    return hipGetLastError();
}

int gbt_sparse_part_tile() { return kSpTile; }

hipError_t gbt_launch_sparse_partition(hipStream_t s, const uint32_t *src_rowptr, const void *src_ent, int ent_bytes,
                                       const int32_t *src_gq, uint32_t *dst_rowptr, void *dst_ent,
                                       int32_t *dst_gq, int B, bool move, const PartJob *jobs, int n_jobs,
                                       int n_tiles, unsigned long long *cursor) {
    if (n_jobs <= 0 || n_tiles <= 0) return hipSuccess;
    hipError_t e = gbt_launch_fill_u64(s, (uint64_t *)cursor, 0, 2 * (int64_t)n_jobs);
    if (e != hipSuccess) return e;
    if (ent_bytes == 2)
        sparse_part_kernel<uint16_t><<<n_tiles, kSpBlock, 0, s>>>(src_rowptr, (const uint16_t *)src_ent, (const int2 *)src_gq,
                                                                  dst_rowptr, (uint16_t *)dst_ent, (int2 *)dst_gq, (uint32_t)B,
                                                                  move ? 1 : 0, jobs, n_jobs, cursor);
    else
        sparse_part_kernel<uint32_t><<<n_tiles, kSpBlock, 0, s>>>(src_rowptr, (const uint32_t *)src_ent, (const int2 *)src_gq,
                                                                  dst_rowptr, (uint32_t *)dst_ent, (int2 *)dst_gq, (uint32_t)B,
                                                                  move ? 1 : 0, jobs, n_jobs, cursor);
    return hipGetLastError();
}

// the trees staged as for gbt_launch_predict; a tree's nodes go through LDS (32 bytes each) when they fit
hipError_t gbt_launch_sparse_walk(hipStream_t s, const char *ws, const DevTree *trees, int n_trees,
                                  const uint32_t *rowptr, const void *ent, int ent_bytes, int64_t n, int B, double eta,
                                  float *margin, int32_t *leaf_out, int max_nodes) {
    if (n <= 0 || n_trees <= 0) return hipSuccess;
    if ((size_t)max_nodes * sizeof(SpNode) + 4 * kWalkWords * 4 > 120u * 1024u) max_nodes = 0;   // nodes stay in HBM / L2
    const size_t lds = (size_t)max_nodes * sizeof(SpNode) + 4 * kWalkWords * 4;
    const void *fn = ent_bytes == 2 ? (const void *)sparse_walk_kernel<uint16_t> : (const void *)sparse_walk_kernel<uint32_t>;
    GbtLdsGuard lds_guard(lds);
    if (lds_guard.needed) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const int rows_per_block = 2048;
    const int64_t grid = (n + rows_per_block - 1) / rows_per_block;
    if (ent_bytes == 2)
        sparse_walk_kernel<uint16_t><<<(unsigned)grid, 256, lds, s>>>(ws, trees, n_trees, rowptr, (const uint16_t *)ent, n,
                                                                      (uint32_t)B, eta, margin, leaf_out, rows_per_block, max_nodes);
    else
        sparse_walk_kernel<uint32_t><<<(unsigned)grid, 256, lds, s>>>(ws, trees, n_trees, rowptr, (const uint32_t *)ent, n,
                                                                      (uint32_t)B, eta, margin, leaf_out, rows_per_block, max_nodes);
    return hipGetLastError();
}
