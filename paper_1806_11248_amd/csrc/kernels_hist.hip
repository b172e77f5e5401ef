// BuildPartialHistograms (Alg. 1; Sec. 2.1) for gfx950: the pairs of a node's rows are added up per
// (feature, bin).
//
// Each workgroup owns a private histogram of one feature tile in LDS, streams
// its share of the node's rows and merges the non-zero bins into the node's
// int64 histogram in HBM with 64-bit global atomics.  All sums are integers, so
// the result does not depend on the order in which lanes and workgroups arrive.
//
// The LDS atomic unit of a CDNA4 compute unit retires only a handful of
// 64-bit lane-atomics per clock, so the kernels issue ONE atomic per (row,
// feature) instead of one for g and one for h: the pair travels as a single
// 64-bit word  [ g : 34 bits, signed | h : 30 bits, unsigned ]  (|g| <= 2^26,
// 0 <= h <= 2^22 per row).  Added as a plain 64-bit integer the word stays exact
// as long as two events are counted: a carry out of the h field (it lands in the
// g field as +1) and a wrap of the g field.  The atomic returns the old word;
// the lane whose add caused an event records it in a small side counter
// [ wraps : int16 | carries : uint16 ] of the same bin.  A bin sees an event only
// every few hundred adds (at least 256 adds between carries, 128 same-sign extreme
// adds between wraps), and a two-compare test on the returned word, exact for the
// carry and tight for the wrap, skips the bookkeeping otherwise.
//
// The bin axis of the LDS histogram is padded to an odd stride so that equal bin
// indices of different features (e.g. the most frequent category of several
// skewed columns) fall into different LDS banks.
#include "gbt_internal.h"
#include "hist_common.h"

namespace {

// ---------------------------------------------------------------------------
// Any bit width (run-time), any feature tile, optional row-id list.
// lane = one row.  The row's slice of the bit stream is consumed in windows of
// four 32-bit words held in registers (five are loaded: an element may straddle
// into the next word); lanes start at different windows of a multi-window row.
// ---------------------------------------------------------------------------
template <bool LIST>
__global__ __launch_bounds__(kHistBlock) void hist_generic_kernel(
    const uint32_t *__restrict__ packed, int64_t n_words, int bits, uint32_t inv_bits, int64_t stride_bits,
    int64_t n, int B, int Bp, uint32_t missing, const uint32_t *__restrict__ row_idx,
    const int2 *__restrict__ gq, int64_t *__restrict__ pool, const HistJob *__restrict__ jobs) {
    extern __shared__ unsigned long long lds[];
    const HistJob job = jobs[blockIdx.x];
    const int ft = (int)job.ft;
    unsigned long long *main_ = lds;
    uint32_t *side = (uint32_t *)(lds + ft * Bp + 256);   // same layout as the 8-bit kernels (trash row unused)
    for (int i = threadIdx.x; i < ft * Bp; i += (int)blockDim.x) {
        main_[i] = 0;
        side[i] = 0;
    }
    __syncthreads();

    const uint32_t mask = (1u << bits) - 1u;
    const int nbits = ft * bits;
    const int lane = threadIdx.x & 63;
    for (uint32_t i = threadIdx.x; i < job.n_rows; i += blockDim.x) {
        const uint64_t pos_in = (uint64_t)job.row_begin + i;
        const uint64_t r = LIST ? (uint64_t)row_idx[pos_in] : pos_in;
        if (r >= (uint64_t)n) continue;   // a malformed row id is skipped, never dereferenced
        const int2 q = gq[r];
        const unsigned long long addv = pack_pair(q);
        const uint32_t hq = (uint32_t)q.y;
        const uint64_t bit0 = r * (uint64_t)stride_bits + (uint64_t)job.f0 * (uint64_t)bits;
        const int64_t w0 = (int64_t)(bit0 >> 5);
        const int sh = (int)(bit0 & 31);
        const int nchunks = (sh + nbits + 127) >> 7;
        int c = (lane * nchunks) >> 6;   // lanes of a wave start at different windows
        for (int cc = 0; cc < nchunks; ++cc) {
            // words past the end of the buffer hold no bit of this row: read the last word instead
            uint32_t w[5];
#pragma unroll
            for (int k = 0; k < 5; ++k) {
                const int64_t wi = w0 + 4 * c + k;
                w[k] = packed[wi < n_words ? wi : n_words - 1];
            }
            // elements whose first bit lies in this window: t in [t_lo, t_hi)
            const int lo_bits = 128 * c - sh;   // window start relative to the slice
            // floor(x / bits) for x < 2^24 as a multiply-high by ceil(2^32 / bits) (bits = 1: identity)
            int t = lo_bits <= 0 ? 0 : (bits == 1 ? lo_bits : (int)__umulhi((uint32_t)(lo_bits + bits - 1), inv_bits));
            int t_hi = bits == 1 ? lo_bits + 128 : (int)__umulhi((uint32_t)(lo_bits + 128 + bits - 1), inv_bits);
            t_hi = t_hi < ft ? t_hi : ft;
            int pos = t * bits - lo_bits;       // first bit of element t inside the window, 0..127
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint64_t pair = (uint64_t)w[k] | ((uint64_t)w[k + 1] << 32);
                while (pos < 32 * (k + 1) && t < t_hi) {
                    const uint32_t s = (uint32_t)(pair >> (pos - 32 * k)) & mask;
                    if (s != missing && s < (uint32_t)B) pk_add(main_, side, t * Bp + (int)s, addv, hq);
                    pos += bits;
                    ++t;
                }
            }
            ++c;
            if (c == nchunks) c = 0;
        }
    }
    __syncthreads();
    flush_tile(main_, side, ft, B, Bp, pool + job.hist_off + (uint64_t)job.f0 * (uint64_t)B * 2u, (int)blockDim.x, job.pad0 == 1u);
}

// ---------------------------------------------------------------------------
// 8-bit symbols (one byte per element).  lane = one row; the row's bytes are
// loaded once into a 16-byte register window and realigned to the row's first
// byte with byte-funnel shifts.
//
// SINGLE (the tile has at most 16 features, one window per row): the window is
// then PERMUTED per lane with v_perm_b32 so that unrolled slot j of lane l holds
// feature (j + l) mod ft.  The lanes of a wave therefore work on different
// features in the same instruction, and rows that share the heavy bin of a
// skewed column do not meet at one LDS address.  The byte selectors and the
// slots' LDS offsets depend on the lane only and live in registers.
// Wider tiles are walked window by window, lanes starting at different windows.
//
// All atomics of a window are issued before the first returned word is examined,
// so their latencies overlap.  A missing symbol, a symbol >= B or a slot past the
// tile's last feature is sent to a spare "trash" row behind the histogram instead
// of being predicated: word `lane` of it, so that no two lanes of an instruction
// meet on one address (same-address atomics take turns).
//   NS  : unrolled slots per window.  0: wide tile (16 slots, no permutation);
//         otherwise the tile has at most NS <= 16 features (slots past the last
//         feature fall into the trash row)
//   CHK : a symbol may be the missing symbol, or >= B (B < 256)
//   FIX : (the root of a tree: every row is visited by exactly one workgroup) the
//         gradient pairs are still fp32: the kernel rounds them to fixed point
//         itself, stores them for the later levels and adds up the root's totals,
//         which saves the separate conversion pass over all rows
// ---------------------------------------------------------------------------
struct FixArgs {   // FIX only
    const float2 *gpair;
    double sg, sh;
    int2 *gq_out;
    int64_t *sums;   // [2], cleared by the launcher
};

template <bool LIST, int NS, bool CHK, bool FIX>
__global__ __launch_bounds__(kHistBlock) void hist_b8_kernel(
    const uint32_t *__restrict__ packed, int64_t n_words, int64_t stride_bytes, int64_t n, int B, int Bp,
    uint32_t missing, const uint32_t *__restrict__ row_idx, const int2 *__restrict__ gq,
    int64_t *__restrict__ pool, const HistJob *__restrict__ jobs, FixArgs fix) {
    extern __shared__ unsigned long long lds[];
    const HistJob job = jobs[blockIdx.x];
    const int ft = (int)job.ft;
    const int trash = ft * Bp;                       // first word of the trash row
    const int n_acc = trash + 256;
    unsigned long long *main_ = lds;
    uint32_t *side = (uint32_t *)(lds + n_acc);
    for (int i = threadIdx.x; i < n_acc; i += (int)blockDim.x) {
        main_[i] = 0;
        side[i] = 0;
    }
    __syncthreads();

    constexpr bool SINGLE = NS != 0;
    constexpr int SLOTS = SINGLE ? NS : 16;
    static_assert(!FIX || (SINGLE && !LIST), "the conversion needs every row visited once, in matrix order");
    int64_t sum_g = 0, sum_h = 0;              // FIX: this thread's share of the root's totals
    const int lane = threadIdx.x & 63;
    const int nchunks = (ft + 15) >> 4;        // 16-byte windows per row slice (same for every lane)
    // SINGLE: slot j of this lane handles feature (j + lane) mod ft
    uint32_t selA[4], selB[4];                 // v_perm selectors for window words (1:0) and (3:2)
    int pre[16];                               // word offset of the slot's feature in the LDS histogram
    if (SINGLE) {
        const int l0 = lane % ft;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            selA[k] = 0;
            selB[k] = 0;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            int t = j + l0;
            t = t >= ft ? t - ft : t;          // (j + lane) mod ft for j < ft
            const bool live = j < ft;
            pre[j] = live ? t * Bp : trash + lane;   // a slot past the last feature: this lane's own trash word
            const uint32_t a = (live && t < 8) ? (uint32_t)t : 0x0Cu;           // 0x0C selects a zero byte
            const uint32_t b = (live && t >= 8) ? (uint32_t)(t - 8) : 0x0Cu;
            selA[j >> 2] |= a << (8 * (j & 3));
            selB[j >> 2] |= b << (8 * (j & 3));
        }
    }
    for (uint32_t i = threadIdx.x; i < job.n_rows; i += blockDim.x) {
        const uint64_t pos_in = (uint64_t)job.row_begin + i;
        const uint64_t r = LIST ? (uint64_t)row_idx[pos_in] : pos_in;
        if (r >= (uint64_t)n) continue;
        int2 q;
        if (FIX) {
            const float2 v = fix.gpair[r];
            q.x = __double2int_rn((double)v.x * fix.sg);
            q.y = __double2int_rn((double)v.y * fix.sh);
            fix.gq_out[r] = q;
            sum_g += q.x;
            sum_h += q.y;
        } else {
            q = gq[r];
        }
        const unsigned long long addv = pack_pair(q);
        const uint32_t hq = (uint32_t)q.y;
        const uint64_t byte0 = r * (uint64_t)stride_bytes + job.f0;
        const int64_t w0 = (int64_t)(byte0 >> 2);
        const uint32_t a = (uint32_t)(byte0 & 3);
        int c = SINGLE ? 0 : (lane * nchunks) >> 6;
        for (int cc = 0; cc < (SINGLE ? 1 : nchunks); ++cc) {
            // words past the end of the buffer hold no bit of this row: read the last word instead
            uint32_t w[5];   // (five single-word loads: one 16-byte load, with or without a test for the buffer's end, measured slower in this kernel)
#pragma unroll
            for (int k = 0; k < 5; ++k) {
                const int64_t wi = w0 + 4 * c + k;
                w[k] = packed[wi < n_words ? wi : n_words - 1];
            }
            // realign: W = bytes [16c, 16c+16) of the row slice
            uint32_t W[4], V[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) W[k] = __builtin_amdgcn_alignbyte(w[k + 1], w[k], a);
            if (SINGLE) {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    V[k] = __builtin_amdgcn_perm(W[1], W[0], selA[k]) | __builtin_amdgcn_perm(W[3], W[2], selB[k]);
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) V[k] = W[k];
            }
            const int nv = ft - 16 * c;              // wide tile: features left from this window on
            int idx[SLOTS];
            unsigned long long old[SLOTS];
#pragma unroll
            for (int j = 0; j < SLOTS; ++j) {
                const uint32_t s = (V[j >> 2] >> (8 * (j & 3))) & 0xffu;
                const bool dead = !SINGLE && j >= nv;   // wide tile: a slot past the tile's last feature
                const int base = SINGLE ? pre[j] : (16 * c + j) * Bp;
                bool bad = dead;
                if (CHK) bad |= (s == missing) | (s >= (uint32_t)B);
                idx[j] = bad ? trash + lane : base + (int)s;   // trash: one word per lane, no two lanes collide
                old[j] = atomicAdd(&main_[idx[j]], addv);
            }
            if (SINGLE) {   // measured: here the word-by-word test is the faster one (0.85 against 0.97 ms on 115M x 13)
#pragma unroll
                for (int j = 0; j < SLOTS; ++j) pk_check(side, idx[j], old[j], addv, hq);
            } else {
                pk_check_group<SLOTS>(side, idx, old, SLOTS, addv, hq);
            }
            ++c;
            if (c == nchunks) c = 0;
        }
    }
    __syncthreads();
    flush_tile(main_, side, ft, B, Bp, pool + job.hist_off + (uint64_t)job.f0 * (uint64_t)B * 2u, (int)blockDim.x, job.pad0 == 1u);
    if (FIX) {   // one pair of global atomics per workgroup
        __shared__ int64_t red[2][kHistBlock / 64];
        for (int o = 32; o > 0; o >>= 1) {
            sum_g += (int64_t)(((uint64_t)(uint32_t)__shfl_xor((int)(sum_g >> 32), o) << 32) |
                               (uint32_t)__shfl_xor((int)(sum_g & 0xffffffff), o));
            sum_h += (int64_t)(((uint64_t)(uint32_t)__shfl_xor((int)(sum_h >> 32), o) << 32) |
                               (uint32_t)__shfl_xor((int)(sum_h & 0xffffffff), o));
        }
        if (lane == 0) {
            red[0][threadIdx.x >> 6] = sum_g;
            red[1][threadIdx.x >> 6] = sum_h;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int w = 1; w < (int)(blockDim.x >> 6); ++w) {
                sum_g += red[0][w];
                sum_h += red[1][w];
            }
            atomicAdd((unsigned long long *)&fix.sums[0], (unsigned long long)sum_g);
            atomicAdd((unsigned long long *)&fix.sums[1], (unsigned long long)sum_h);
        }
    }
}

// ---------------------------------------------------------------------------
// RepartitionInstances and the children's BuildPartialHistograms in ONE pass
// (8-bit symbols, at most 16 features, row order not needed).
//
// Moving a node's records to its children is bound by HBM, the histogram of a
// child by the LDS atomic unit; run one after the other the two leave each other's
// resource idle.  Here a workgroup takes a span of one splitting node's rows, tile
// by tile: every thread loads its rows into registers, decides their side, adds
// the rows of the side to be built into the workgroup's LDS histogram (exactly as
// hist_b8_kernel does) while the tile's room in the children is being reserved
// with one 64-bit atomic on the node's cursor, and then stores the rows at their
// new place.  The span's histogram is merged into the child's histogram at the end.
// Left rows fill the node's segment from its start, right rows from its end
// backwards; tiles land in the order their atomics arrive (see part_fused_kernel
// for the same scheme without a histogram).
//
// Records.  The pass is bound by the bytes it moves, so a row travels as ONE record
// of RW = ceil((NS + 7) / 4) words: the symbols from byte 0, zero padding, and in the
// last 7 bytes the fixed-point pair as a 56-bit little-endian number
// [ h : 24 bits | g : 28 bits, two's complement ] (|g| <= 2^26, 0 <= h <= 2^22).
// 13 features: 20 bytes instead of a 16-byte padded row plus an 8-byte pair.  The
// pair always sits in bytes 1..3 of word RW-2 and in word RW-1.
// part_hist_first_kernel (level 0): the source is the caller's packed matrix (rows of
// `ft` bytes at any byte alignment) with the pairs in their own array;
// part_hist_kernel (every later level): records.
//
// PartJob: tile_begin / n_tiles count SPANS of `rows_per_span` rows here; pad is
// the side to build (1 left, 0 right, 2 none), hist_off that child's histogram.
// ---------------------------------------------------------------------------
constexpr int kPHBlock = 512;
constexpr int kPHRows = 8;                       // rows per thread and tile: what is in flight while the tile loads
constexpr int kPHTile = kPHBlock * kPHRows;      // 4096
constexpr int kPFRows = 4;                       // records kernel: rows per thread and tile, twice (current and next tile)
static_assert(kPHTile % (kPHBlock * kPFRows) == 0, "spans are whole tiles of either kernel");
constexpr int kPHWords = kPHTile / 64;           // 64 ballot words
static_assert(kPHWords == 64, "the ballot words are ranked by one wave");
constexpr int kPHGroup = 7;                      // atomics of a row in flight together (registers for their results)
constexpr int record_words(int ns) { return (ns + 7 + 3) / 4; }
constexpr int slots_for(int ft) { return ft <= 4 ? 4 : ft <= 8 ? 8 : ft <= 12 ? 12 : ft == 13 ? 13 : 16; }

__device__ inline int find_span_job(const PartJob *jobs, int n_jobs, uint32_t span) {
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (jobs[mid].tile_begin <= span) lo = mid; else hi = mid;
    }
    return lo;
}

// Adds one record's pair to the LDS histogram at the bins of its NS symbol slots (slot j of a lane
// is feature (j + lane) mod ft; pre[] / selA / selB are the lane's slot tables).  The atomics go out
// in groups; a group's returned words are tested together for an event (a carry out of the h field,
// a wrap of the g field): the smallest distance of any of them from one decides whether the
// per-word bookkeeping runs at all.
// UNI: every row of the tree has the same hessian.  A bin's word is then [ sum of g : 46 bits | rows : 18 bits ],
// added to with an atomic whose result nobody waits for, and nothing is tested; the bin's H is rows times that
// hessian (flush_tile_uniform).  A workgroup may add at most kUniRowsMax rows to one histogram.
constexpr int kUniRowsShift = 18;
constexpr uint32_t kUniRowsMax = (1u << kUniRowsShift) - 1u;
template <int NS, bool CHK, int RW, int GROUP = kPHGroup, bool UNI = false>
__device__ __forceinline__ void ph_add_row(const uint32_t (&row)[RW], unsigned long long *main_, uint32_t *side,
                                           const int (&pre)[NS], const uint32_t (&selA)[4], const uint32_t (&selB)[4],
                                           int trash, int lane, uint32_t missing, int B) {
    constexpr int SW = (NS + 3) / 4;
    // the pair: bytes 1..3 of word RW-2 and word RW-1
    const uint32_t qlo = (row[RW - 2] >> 8) | (row[RW - 1] << 24);   // bits 0..31 of the 56
    const uint32_t qhi = row[RW - 1] >> 8;                           // bits 32..55
    int2 q;
    q.x = (int32_t)(qlo << 4) >> 4;                                  // 28 bits, sign-extended
    q.y = (int32_t)((qlo >> 28) | (qhi << 4));                       // 24 bits
    const unsigned long long addv = UNI ? ((unsigned long long)(long long)q.x << kUniRowsShift) + 1ull : pack_pair(q);
    const uint32_t hq = (uint32_t)q.y;
    uint32_t W[4], V[(NS + 3) / 4];
#pragma unroll
    for (int k = 0; k < 4; ++k) W[k] = k < SW ? row[k < SW ? k : 0] : 0u;   // words past the symbols are never selected
#pragma unroll
    for (int k = 0; k < (NS + 3) / 4; ++k)
        V[k] = __builtin_amdgcn_perm(W[1], W[0], selA[k]) | __builtin_amdgcn_perm(W[3], W[2], selB[k]);
    if (UNI) {
#pragma unroll
        for (int t = 0; t < NS; ++t) {
            const uint32_t sv = (V[t >> 2] >> (8 * (t & 3))) & 0xffu;
            bool bad = false;
            if (CHK) bad = (sv == missing) | (sv >= (uint32_t)B);
            (void)__hip_atomic_fetch_add(&main_[bad ? trash + lane : pre[t] + (int)sv], addv, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        return;
    }
#pragma unroll
    for (int t0 = 0; t0 < NS; t0 += GROUP) {
        int idx[GROUP];
        unsigned long long old[GROUP];
#pragma unroll
        for (int tt = 0; tt < GROUP; ++tt) {
            const int t = t0 + tt;
            if (t < NS) {
                const uint32_t sv = (V[t >> 2] >> (8 * (t & 3))) & 0xffu;
                bool bad = false;
                if (CHK) bad = (sv == missing) | (sv >= (uint32_t)B);
                idx[tt] = bad ? trash + lane : pre[t] + (int)sv;
                old[tt] = atomicAdd(&main_[idx[tt]], addv);
            }
        }
        pk_check_group<GROUP>(side, idx, old, NS - t0, addv, hq);
    }
}

// The merge of a histogram kept in the uniform-hessian form (see ph_add_row) into the node's histogram in HBM.
__device__ __forceinline__ void flush_tile_uniform(const unsigned long long *main_, int ft, int B, int Bp, int64_t *out,
                                                   int block, int64_t hq_uniform) {
    for (int i = threadIdx.x; i < ft * B; i += block) {
        const int t = i / B, b = i - t * B;
        const unsigned long long w = main_[t * Bp + b];
        if (w == 0) continue;
        const int64_t rows = (int64_t)(w & kUniRowsMax);
        const int64_t g = ((int64_t)w - rows) >> kUniRowsShift, h = rows * hq_uniform;
        if (g != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i), (unsigned long long)g);
        if (h != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i + 1), (unsigned long long)h);
    }
}

// Where rows stay in place only some lanes of a wave hold a row whose pair is added, and a wave's LDS atomic
// costs about the same with 25 active lanes as with 64.  Such rows are therefore first packed: a wave appends
// the records it takes to a ring of its own in LDS (ranks from the ballot), and as soon as 64 are waiting it
// reads them back one per lane and adds them with every lane busy.  TAG: one more word travels with a record.
// The ring is private to the wave, whose LDS instructions execute in program order: no barrier is involved.
constexpr int kQueueSlots = 128;   // >= 63 waiting + 64 appended
template <int RW, bool TAG>
struct WaveQueue {
    static constexpr int kWords = RW + (TAG ? 1 : 0);
    uint32_t *q;           // kWords * kQueueSlots words, word-major: the lanes of a wave touch consecutive words
    uint32_t head, tail;   // wave-uniform
    __device__ __forceinline__ void push(bool take, const uint32_t (&row)[RW], uint32_t tag) {
        const uint64_t m = __ballot(take);
        if (take) {
            const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
            const uint32_t s = (tail + rank) & (kQueueSlots - 1);
#pragma unroll
            for (int k = 0; k < RW; ++k) q[k * kQueueSlots + s] = row[k];
            if (TAG) q[RW * kQueueSlots + s] = tag;
        }
        tail += (uint32_t)__popcll(m);
        __builtin_amdgcn_wave_barrier();
    }
    __device__ __forceinline__ uint32_t waiting() const { return tail - head; }
    // the record `lane` places after the head (the caller has checked that it exists); advance with drop()
    __device__ __forceinline__ void peek(int lane, uint32_t (&row)[RW], uint32_t &tag) const {
        const uint32_t s = (head + (uint32_t)lane) & (kQueueSlots - 1);
#pragma unroll
        for (int k = 0; k < RW; ++k) row[k] = q[k * kQueueSlots + s];
        tag = TAG ? q[RW * kQueueSlots + s] : 0u;
    }
    __device__ __forceinline__ void drop(uint32_t n) {
        head += n;
        __builtin_amdgcn_wave_barrier();
    }
};

// F32: the pairs are still fp32 (src_gq then points at float2): each is rounded to fixed point here, in fp32
// arithmetic, which is exact for the power-of-two scales sgf, shf the launcher accepts (gbt_fix32_ok)
template <int NS, bool CHK, bool F32, bool UNI>
__global__ __launch_bounds__(kPHBlock, 4) void part_hist_first_kernel(
    const uint32_t *__restrict__ src, int64_t src_stride_bytes, int64_t src_words, const int2 *__restrict__ src_gq,
    float sgf, float shf, uint32_t *__restrict__ dst, int ft, int B, int Bp, uint32_t missing, const PartJob *__restrict__ jobs,
    int n_jobs, uint32_t rows_per_span, unsigned long long *__restrict__ cursor, int64_t *__restrict__ pool, int hq_uniform) {
    constexpr int SW = (NS + 3) / 4;        // words that hold symbols
    constexpr int RW = record_words(NS);    // words of a record
    extern __shared__ unsigned long long lds[];
    __shared__ uint64_t words[2][kPHWords];
    __shared__ uint32_t lefts_before[2][kPHWords];
    __shared__ uint32_t base_s[2][2];
    const int ji = find_span_job(jobs, n_jobs, blockIdx.x);
    const PartJob job = jobs[ji];
    const uint32_t span_begin = (blockIdx.x - job.tile_begin) * rows_per_span;
    const uint32_t span_rows = job.seg_len - span_begin < rows_per_span ? job.seg_len - span_begin : rows_per_span;
    const bool build = job.pad != 2u, build_left = job.pad == 1u;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    const int trash = ft * Bp;
    const int n_acc = trash + 256;
    unsigned long long *main_ = lds;
    uint32_t *side = (uint32_t *)(lds + n_acc);
    for (int i = threadIdx.x; i < n_acc; i += kPHBlock) {
        main_[i] = 0;
        side[i] = 0;
    }
    // slot j of this lane handles feature (j + lane) mod ft (see hist_b8_kernel)
    uint32_t selA[4], selB[4];
    int pre[NS];
    {
        const int l0 = lane % ft;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            selA[k] = 0;
            selB[k] = 0;
        }
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            int t = j + l0;
            t = t >= ft ? t - ft : t;
            const bool live = j < ft;
            pre[j] = live ? t * Bp : trash + lane;   // a slot past the last feature: this lane's own trash word
            const uint32_t a = (live && t < 8) ? (uint32_t)t : 0x0Cu;
            const uint32_t b = (live && t >= 8) ? (uint32_t)(t - 8) : 0x0Cu;
            selA[j >> 2] |= a << (8 * (j & 3));
            selB[j >> 2] |= b << (8 * (j & 3));
        }
    }
    const int fword = (int)(job.feature >> 2);              // the split feature's word and shift inside a row
    const uint32_t fshift = (job.feature & 3u) * 8u;
    const uint32_t tail_bits = (uint32_t)(ft * 8 - 32 * (SW - 1));   // valid bits of the last symbol word, 1..32
    const uint32_t tail_mask = tail_bits >= 32 ? 0xffffffffu : ((1u << tail_bits) - 1u);
    const uint32_t seg_last = job.seg_begin + job.seg_len - 1u;
    __syncthreads();

    const bool nomove = dst == nullptr;   // the rows stay where they are: no ranks, no room to reserve, no barriers
    uint32_t my_lefts = 0;                // nomove, lane 0 of every wave: left rows seen
    int par = 0;
    for (uint32_t done = 0; done < span_rows; done += kPHTile, par ^= 1) {
        const uint32_t tile_rows = span_rows - done < (uint32_t)kPHTile ? span_rows - done : (uint32_t)kPHTile;
        const uint64_t p0 = (uint64_t)job.seg_begin + span_begin + done;
        // every word an unaligned row load of this tile can touch lies inside the source buffer
        const bool tile_inside = (int64_t)(((p0 + tile_rows) * (uint64_t)src_stride_bytes) >> 2) + SW + 1 <= src_words;
        uint32_t row[kPHRows][RW];
        uint32_t takebits = 0;
        // ---- load, decide
#pragma unroll
        for (int j = 0; j < kPHRows; ++j) {
            const int w = j * (kPHBlock / 64) + wave;
            const uint32_t in_tile = (uint32_t)w * 64u + (uint32_t)lane;
            bool left = false;
            if (in_tile < tile_rows) {
                const uint64_t p = p0 + in_tile;
                {
                    const uint64_t sb = p * (uint64_t)src_stride_bytes;
                    const int64_t s0 = (int64_t)(sb >> 2);
                    const uint32_t sh = (uint32_t)(sb & 3);
                    uint32_t x[SW + 1];
                    if (tile_inside) {
                        load_words(x, src + s0);
                    } else {   // the matrix ends inside this tile's last window: read the last word instead
#pragma unroll
                        for (int k = 0; k <= SW; ++k) x[k] = src[s0 + k < src_words ? s0 + k : src_words - 1];
                    }
#pragma unroll
                    for (int k = 0; k < RW; ++k) row[j][k] = k < SW ? __builtin_amdgcn_alignbyte(x[k < SW ? k + 1 : 0], x[k < SW ? k : 0], sh) : 0u;
                    row[j][SW - 1] &= tail_mask;
                    int2 q;
                    if (F32) {
                        const float2 v = ((const float2 *)src_gq)[p];
                        q.x = (int)rintf(v.x * sgf);
                        q.y = (int)rintf(v.y * shf);
                    } else {
                        q = src_gq[p];
                    }
                    const unsigned long long v56 = ((unsigned long long)(uint32_t)q.x & 0x0fffffffull) |
                                                   ((unsigned long long)(uint32_t)q.y << 28);
                    row[j][RW - 2] |= (uint32_t)(v56 << 8);          // bytes 1..3
                    row[j][RW - 1] = (uint32_t)(v56 >> 24);
                }
                uint32_t fw = row[j][0];
#pragma unroll
                for (int k = 1; k < SW; ++k) fw = fword == k ? row[j][k] : fw;
                const uint32_t sy = (fw >> fshift) & 0xffu;
                left = (sy == missing) ? (job.default_left != 0) : (sy <= job.bin);
                takebits |= (build && left == build_left) ? (1u << j) : 0u;
            }
            const uint64_t ballot = __ballot(left);
            if (nomove) my_lefts += (uint32_t)__popcll(ballot);
            else if (lane == 0) words[par][w] = ballot;
        }
        if (!nomove) __syncthreads();

        // ---- wave 0 ranks the ballot words and reserves the tile's room (the answer is awaited after
        //      the histogram work below)
        unsigned long long reserved = 0;
        if (wave == 0 && !nomove) {
            const uint32_t c = (uint32_t)__popcll(words[par][lane]);   // kPHWords == 64: one word per lane
            uint32_t x = c;
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t y = (uint32_t)__shfl_up((int)x, d);
                if (lane >= d) x += y;
            }
            lefts_before[par][lane] = x - c;
            if (lane == 63)
                reserved = atomicAdd(&cursor[(size_t)ji * kCursorStride], (unsigned long long)x | ((unsigned long long)(tile_rows - x) << 32));
        }

        // ---- histogram of the rows on the side to be built
#pragma unroll
        for (int j = 0; j < kPHRows; ++j) {
            // (groups of 5 atomics here: with 8 rows of raw words per thread, 7 results in flight spill registers)
            if ((takebits >> j) & 1u) ph_add_row<NS, CHK, RW, 5, UNI>(row[j], main_, side, pre, selA, selB, trash, lane, missing, B);
        }
        if (nomove) continue;
        if (wave == 0 && lane == 63) {
            base_s[par][0] = (uint32_t)(reserved & 0xffffffffull);
            base_s[par][1] = (uint32_t)(reserved >> 32);
        }
        __syncthreads();

        // ---- store
        const uint32_t left_base = base_s[par][0], right_base = base_s[par][1];
#pragma unroll
        for (int j = 0; j < kPHRows; ++j) {
            const int w = j * (kPHBlock / 64) + wave;
            const uint32_t in_tile = (uint32_t)w * 64u + (uint32_t)lane;
            if (in_tile < tile_rows) {
                const uint64_t m = words[par][w];
                const uint32_t below = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
                uint32_t q;
                if ((m >> lane) & 1ull) {
                    q = job.seg_begin + left_base + lefts_before[par][w] + below;
                } else {
                    const uint32_t rights_before_word = (uint32_t)w * 64u - lefts_before[par][w];
                    q = seg_last - (right_base + rights_before_word + ((uint32_t)lane - below));
                }
                uint32_t *dp = dst + (uint64_t)q * RW;
#pragma unroll
                for (int k = 0; k < RW; ++k) dp[k] = row[j][k];
            }
        }
        // words[par] is rewritten two tiles from now, after two more barriers: no third barrier needed
    }
    if (nomove && lane == 0 && my_lefts) atomicAdd(&cursor[(size_t)ji * kCursorStride], (unsigned long long)my_lefts);
    __syncthreads();
    if (build) {
        if (UNI) flush_tile_uniform(main_, ft, B, Bp, pool + job.hist_off, kPHBlock, (int64_t)hq_uniform);
        else flush_tile(main_, side, ft, B, Bp, pool + job.hist_off, kPHBlock);
    }
}

// Levels below the first: the source is records.  A thread holds two sets of kPFRows records, one
// being ranked, added to the histogram and stored, the other (the next tile) on its way from HBM
// meanwhile, so that the loads never start from an empty pipe behind a tile's barriers.
// (The wave queue of the passes that keep rows in place does not pay here: its LDS leaves room for two workgroups
// per CU instead of four, and the barriers of a moving tile then cost more than the packed atomics save.)
template <int NS, bool CHK, bool UNI>
__global__ __launch_bounds__(kPHBlock, 4) void part_hist_kernel(
    const uint32_t *__restrict__ src, uint32_t *__restrict__ dst, int ft, int B, int Bp, uint32_t missing,
    const PartJob *__restrict__ jobs, int n_jobs, uint32_t rows_per_span, unsigned long long *__restrict__ cursor,
    int64_t *__restrict__ pool, int hq_uniform) {
    constexpr int SW = (NS + 3) / 4;
    constexpr int RW = record_words(NS);
    constexpr int BLK = kPHBlock, ROWS = kPFRows;
    constexpr int TILE = BLK * ROWS;
    constexpr int NW = TILE / 64;          // ballot words of a tile
    constexpr int WAVES = BLK / 64;
    static_assert(NW <= 64 && TILE % 64 == 0, "the ballot words are ranked by one wave");
    extern __shared__ unsigned long long lds[];
    __shared__ uint64_t words[2][NW];
    __shared__ uint32_t lefts_before[2][NW];
    __shared__ uint32_t base_s[2][2];
    const int ji = find_span_job(jobs, n_jobs, blockIdx.x);
    const PartJob job = jobs[ji];
    const uint32_t span_begin = (blockIdx.x - job.tile_begin) * rows_per_span;
    const uint32_t span_rows = job.seg_len - span_begin < rows_per_span ? job.seg_len - span_begin : rows_per_span;
    const bool build = job.pad != 2u, build_left = job.pad == 1u;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    const int trash = ft * Bp;
    const int n_acc = trash + 256;
    unsigned long long *main_ = lds;
    uint32_t *side = (uint32_t *)(lds + n_acc);
    for (int i = threadIdx.x; i < n_acc; i += BLK) {
        main_[i] = 0;
        side[i] = 0;
    }
    uint32_t selA[4], selB[4];
    int pre[NS];
    {
        const int l0 = lane % ft;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            selA[k] = 0;
            selB[k] = 0;
        }
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            int t = j + l0;
            t = t >= ft ? t - ft : t;
            const bool live = j < ft;
            pre[j] = live ? t * Bp : trash + lane;
            const uint32_t a = (live && t < 8) ? (uint32_t)t : 0x0Cu;
            const uint32_t b = (live && t >= 8) ? (uint32_t)(t - 8) : 0x0Cu;
            selA[j >> 2] |= a << (8 * (j & 3));
            selB[j >> 2] |= b << (8 * (j & 3));
        }
    }
    // byte `feature` of a record, picked without indexing the register array by a run-time value
    const uint32_t fselA = 0x0C0C0C00u | (job.feature < 8u ? job.feature : 0x0Cu);
    const uint32_t fselB = 0x0C0C0C00u | (job.feature >= 8u ? job.feature - 8u : 0x0Cu);
    const uint32_t seg_last = job.seg_begin + job.seg_len - 1u;
    const bool nomove = dst == nullptr;
    uint32_t my_lefts = 0;
    const uint64_t span_first = (uint64_t)job.seg_begin + span_begin;
    __syncthreads();

    auto load_tile = [&](uint32_t (&row)[ROWS][RW], uint32_t done) __attribute__((always_inline)) {
        const uint32_t tile_rows = span_rows - done < (uint32_t)TILE ? span_rows - done : (uint32_t)TILE;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const uint32_t in_tile = (uint32_t)(j * WAVES + wave) * 64u + (uint32_t)lane;
            if (in_tile < tile_rows) {
                const uint32_t *rp = src + (span_first + done + in_tile) * RW;
#pragma unroll
                for (int k = 0; k < RW; ++k) row[j][k] = rp[k];
            }
        }
    };
    auto process = [&](uint32_t (&row)[ROWS][RW], uint32_t done, int par) __attribute__((always_inline)) {
        const uint32_t tile_rows = span_rows - done < (uint32_t)TILE ? span_rows - done : (uint32_t)TILE;
        uint32_t takebits = 0;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const int w = j * WAVES + wave;
            const uint32_t in_tile = (uint32_t)w * 64u + (uint32_t)lane;
            bool left = false;
            if (in_tile < tile_rows) {
                const uint32_t sy = __builtin_amdgcn_perm(SW > 1 ? row[j][SW > 1 ? 1 : 0] : 0u, row[j][0], fselA) |
                                    __builtin_amdgcn_perm(SW > 3 ? row[j][SW > 3 ? 3 : 0] : 0u,
                                                          SW > 2 ? row[j][SW > 2 ? 2 : 0] : 0u, fselB);
                left = (sy == missing) ? (job.default_left != 0) : (sy <= job.bin);
                takebits |= (build && left == build_left) ? (1u << j) : 0u;
            }
            const uint64_t ballot = __ballot(left);
            if (nomove) my_lefts += (uint32_t)__popcll(ballot);
            else if (lane == 0) words[par][w] = ballot;
        }
        if (!nomove) __syncthreads();
        unsigned long long reserved = 0;
        if (wave == 0 && !nomove) {
            const uint32_t c = lane < NW ? (uint32_t)__popcll(words[par][lane < NW ? lane : 0]) : 0u;
            uint32_t x = c;
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t y = (uint32_t)__shfl_up((int)x, d);
                if (lane >= d) x += y;
            }
            if (lane < NW) lefts_before[par][lane] = x - c;
            if (lane == 63)
                reserved = atomicAdd(&cursor[(size_t)ji * kCursorStride], (unsigned long long)x | ((unsigned long long)(tile_rows - x) << 32));
        }
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            if ((takebits >> j) & 1u) ph_add_row<NS, CHK, RW, kPHGroup, UNI>(row[j], main_, side, pre, selA, selB, trash, lane, missing, B);
        }
        if (nomove) return;
        if (wave == 0 && lane == 63) {
            base_s[par][0] = (uint32_t)(reserved & 0xffffffffull);
            base_s[par][1] = (uint32_t)(reserved >> 32);
        }
        __syncthreads();
        const uint32_t left_base = base_s[par][0], right_base = base_s[par][1];
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const int w = j * WAVES + wave;
            const uint32_t in_tile = (uint32_t)w * 64u + (uint32_t)lane;
            if (in_tile < tile_rows) {
                const uint64_t m = words[par][w];
                const uint32_t below = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
                uint32_t q;
                if ((m >> lane) & 1ull) {
                    q = job.seg_begin + left_base + lefts_before[par][w] + below;
                } else {
                    const uint32_t rights_before_word = (uint32_t)w * 64u - lefts_before[par][w];
                    q = seg_last - (right_base + rights_before_word + ((uint32_t)lane - below));
                }
                uint32_t *dp = dst + (uint64_t)q * RW;
#pragma unroll
                for (int k = 0; k < RW; ++k) dp[k] = row[j][k];
            }
        }
        // words[par] is rewritten two tiles from now, after two more barriers
    };

    uint32_t rowA[ROWS][RW], rowB[ROWS][RW];
    load_tile(rowA, 0);
    for (uint32_t done = 0; done < span_rows;) {
        if (done + TILE < span_rows) load_tile(rowB, done + TILE);
        process(rowA, done, 0);
        done += TILE;
        if (done >= span_rows) break;
        if (done + TILE < span_rows) load_tile(rowA, done + TILE);
        process(rowB, done, 1);
        done += TILE;
    }
    if (nomove && lane == 0 && my_lefts) atomicAdd(&cursor[(size_t)ji * kCursorStride], (unsigned long long)my_lefts);
    __syncthreads();
    if (build) {
        if (UNI) flush_tile_uniform(main_, ft, B, Bp, pool + job.hist_off, BLK, (int64_t)hq_uniform);
        else flush_tile(main_, side, ft, B, Bp, pool + job.hist_off, BLK);
    }
}

// Rows still in the caller's packed matrix (byte symbols, row p at byte p * stride_bytes) with their pairs in an
// array of their own: how the passes below that usually read records take them instead.
struct MoveFirst {
    int64_t stride_bytes, src_words;
    const int2 *gq;   // or float2 pairs (F32), rounded with sgf, shf as in part_hist_first_kernel
    float sgf, shf;
    int ft;
};
// Row p as a record.  inside: every word the unaligned load can touch lies in the buffer (else the last word is read
// instead); tail_mask: valid bits of the last symbol word.
template <int NS, bool F32>
__device__ __forceinline__ void load_first_row(uint32_t (&row)[record_words(NS)], const uint32_t *__restrict__ src, uint64_t p,
                                               const MoveFirst &first, bool inside, uint32_t tail_mask) {
    constexpr int SW = (NS + 3) / 4, RW = record_words(NS);
    const uint64_t sb = p * (uint64_t)first.stride_bytes;
    const int64_t s0 = (int64_t)(sb >> 2);
    const uint32_t sh = (uint32_t)(sb & 3);
    uint32_t x[SW + 1];
    if (inside) {
        load_words(x, src + s0);
    } else {
#pragma unroll
        for (int k = 0; k <= SW; ++k) x[k] = src[s0 + k < first.src_words ? s0 + k : first.src_words - 1];
    }
#pragma unroll
    for (int k = 0; k < RW; ++k) row[k] = k < SW ? __builtin_amdgcn_alignbyte(x[k < SW ? k + 1 : 0], x[k < SW ? k : 0], sh) : 0u;
    row[SW - 1] &= tail_mask;
    int2 q;
    if (F32) {
        const float2 v = ((const float2 *)first.gq)[p];
        q.x = (int)rintf(v.x * first.sgf);
        q.y = (int)rintf(v.y * first.shf);
    } else {
        q = first.gq[p];
    }
    const unsigned long long v56 = ((unsigned long long)(uint32_t)q.x & 0x0fffffffull) | ((unsigned long long)(uint32_t)q.y << 28);
    row[RW - 2] |= (uint32_t)(v56 << 8);          // bytes 1..3
    row[RW - 1] = (uint32_t)(v56 >> 24);
}

// One split per segment, rows stay where they are (the last level but one that needs histograms, see
// gbt_launch_part_hist): every record is read once, its side decided and counted, and the records of the side
// to be built are added to the LDS histogram through the wave's queue.  No ranks, no stores, no barriers inside a
// span; the next tile's records are on their way while the current one is handled.
constexpr int kKeepBlock = 512;
// FIRST: the rows are read from the caller's matrix and pair array (load_first_row) instead of records.
// UNI: the uniform-hessian form of the LDS histogram (ph_add_row), hq_uniform that hessian in fixed point; a span
// then has at most kUniRowsMax rows.
template <int NS, bool CHK, bool FIRST, bool F32, bool UNI>
__global__ __launch_bounds__(kKeepBlock, 2) void hist_keep_kernel(
    const uint32_t *__restrict__ src, int ft, int B, int Bp, uint32_t missing, const PartJob *__restrict__ jobs, int n_jobs,
    uint32_t rows_per_span, unsigned long long *__restrict__ cursor, int64_t *__restrict__ pool, MoveFirst first,
    int hq_uniform) {
    constexpr int SW = (NS + 3) / 4;
    constexpr int RW = record_words(NS);
    constexpr int BLK = kKeepBlock, ROWS = kPFRows, TILE = BLK * ROWS, WAVES = BLK / 64;
    extern __shared__ unsigned long long lds[];
    const int ji = find_span_job(jobs, n_jobs, blockIdx.x);
    const PartJob job = jobs[ji];
    const uint32_t span_begin = (blockIdx.x - job.tile_begin) * rows_per_span;
    const uint32_t span_rows = job.seg_len - span_begin < rows_per_span ? job.seg_len - span_begin : rows_per_span;
    const bool build = job.pad != 2u, build_left = job.pad == 1u;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    const int trash = ft * Bp;
    const int n_acc = trash + 256;
    unsigned long long *main_ = lds;
    uint32_t *side = (uint32_t *)(lds + n_acc);
    for (int i = threadIdx.x; i < n_acc; i += BLK) {
        main_[i] = 0;
        side[i] = 0;
    }
    WaveQueue<RW, false> queue{side + n_acc + wave * (RW * kQueueSlots), 0u, 0u};
    uint32_t selA[4], selB[4];
    int pre[NS];
    {
        const int l0 = lane % ft;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            selA[k] = 0;
            selB[k] = 0;
        }
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            int t = j + l0;
            t = t >= ft ? t - ft : t;
            const bool live = j < ft;
            pre[j] = live ? t * Bp : trash + lane;
            const uint32_t a = (live && t < 8) ? (uint32_t)t : 0x0Cu;
            const uint32_t b = (live && t >= 8) ? (uint32_t)(t - 8) : 0x0Cu;
            selA[j >> 2] |= a << (8 * (j & 3));
            selB[j >> 2] |= b << (8 * (j & 3));
        }
    }
    const uint32_t fselA = 0x0C0C0C00u | (job.feature < 8u ? job.feature : 0x0Cu);
    const uint32_t fselB = 0x0C0C0C00u | (job.feature >= 8u ? job.feature - 8u : 0x0Cu);
    uint32_t my_lefts = 0;
    const uint64_t span_first = (uint64_t)job.seg_begin + span_begin;
    const uint32_t tail_bits = FIRST ? (uint32_t)(first.ft * 8 - 32 * (SW - 1)) : 32u;
    const uint32_t tail_mask = tail_bits >= 32 ? 0xffffffffu : ((1u << tail_bits) - 1u);
    __syncthreads();

    auto load_tile = [&](uint32_t (&row)[ROWS][RW], uint32_t done) __attribute__((always_inline)) {
        const uint32_t tile_rows = span_rows - done < (uint32_t)TILE ? span_rows - done : (uint32_t)TILE;
        const bool tile_inside = FIRST && (int64_t)(((span_first + done + tile_rows) * (uint64_t)first.stride_bytes) >> 2) + SW + 1 <= first.src_words;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const uint32_t in_tile = (uint32_t)(j * WAVES + wave) * 64u + (uint32_t)lane;
            if (in_tile < tile_rows) {
                if (FIRST) {
                    load_first_row<NS, F32>(row[j], src, span_first + done + in_tile, first, tile_inside, tail_mask);
                } else {
                    const uint32_t *rp = src + (span_first + done + in_tile) * RW;
#pragma unroll
                    for (int k = 0; k < RW; ++k) row[j][k] = rp[k];
                }
            }
        }
    };
    auto add_waiting = [&](uint32_t n) __attribute__((always_inline)) {   // n <= 64 records from the head of the queue
        uint32_t rec[RW], tag;
        if ((uint32_t)lane < n) {
            queue.peek(lane, rec, tag);
            ph_add_row<NS, CHK, RW, kPHGroup, UNI>(rec, main_, side, pre, selA, selB, trash, lane, missing, B);
        }
        queue.drop(n);
    };
    auto process = [&](uint32_t (&row)[ROWS][RW], uint32_t done) __attribute__((always_inline)) {
        const uint32_t tile_rows = span_rows - done < (uint32_t)TILE ? span_rows - done : (uint32_t)TILE;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const uint32_t in_tile = (uint32_t)(j * WAVES + wave) * 64u + (uint32_t)lane;
            bool left = false, take = false;
            if (in_tile < tile_rows) {
                const uint32_t sy = __builtin_amdgcn_perm(SW > 1 ? row[j][SW > 1 ? 1 : 0] : 0u, row[j][0], fselA) |
                                    __builtin_amdgcn_perm(SW > 3 ? row[j][SW > 3 ? 3 : 0] : 0u,
                                                          SW > 2 ? row[j][SW > 2 ? 2 : 0] : 0u, fselB);
                left = (sy == missing) ? (job.default_left != 0) : (sy <= job.bin);
                take = build && left == build_left;
            }
            my_lefts += (uint32_t)__popcll(__ballot(left));
            queue.push(take, row[j], 0u);
            if (queue.waiting() >= 64u) add_waiting(64u);
        }
    };

    uint32_t rowA[ROWS][RW], rowB[ROWS][RW];
    load_tile(rowA, 0);
    for (uint32_t done = 0; done < span_rows;) {
        if (done + TILE < span_rows) load_tile(rowB, done + TILE);
        process(rowA, done);
        done += TILE;
        if (done >= span_rows) break;
        if (done + TILE < span_rows) load_tile(rowA, done + TILE);
        process(rowB, done);
        done += TILE;
    }
    if (queue.waiting()) add_waiting(queue.waiting());
    if (lane == 0 && my_lefts) atomicAdd(&cursor[(size_t)ji * kCursorStride], (unsigned long long)my_lefts);
    __syncthreads();
    if (build) {
        if (UNI) flush_tile_uniform(main_, ft, B, Bp, pool + job.hist_off, BLK, (int64_t)hq_uniform);
        else flush_tile(main_, side, ft, B, Bp, pool + job.hist_off, BLK);
    }
}

// Rows that were not moved at their segment's split and are not moved now: every row belongs to one
// of the segment's two children, whose split (if it has one) sends it left or right; of each splitting
// child's two children one histogram is built.  A workgroup keeps BOTH histograms in LDS and takes a
// span of the segment tile by tile, the next tile's records on their way while the current one is
// added (through the wave's queue, tagged with the histogram a record goes to); no ranks, no stores, no
// barriers inside the span.  Left rows of the children are counted in the cursor words 2 * job and 2 * job + 1.
constexpr int kH2Block = 1024;
template <int NS, bool CHK, bool UNI>
__global__ __launch_bounds__(kH2Block) void hist2_kernel(
    const uint32_t *__restrict__ src, int ft, int B, int Bp, uint32_t missing, const Hist2Job *__restrict__ jobs,
    int n_jobs, uint32_t rows_per_span, unsigned long long *__restrict__ cursor, int64_t *__restrict__ pool, int hq_uniform) {
    constexpr int SW = (NS + 3) / 4;
    constexpr int RW = record_words(NS);
    constexpr int ROWS = kPFRows, TILE = kH2Block * ROWS, WAVES = kH2Block / 64;
    extern __shared__ unsigned long long lds[];
    int lo = 0, hi = n_jobs;   // last job with tile_begin <= this span
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (jobs[mid].tile_begin <= blockIdx.x) lo = mid; else hi = mid;
    }
    const int ji = lo;
    const Hist2Job job = jobs[ji];
    const uint32_t span_begin = (blockIdx.x - job.tile_begin) * rows_per_span;
    const uint32_t span_rows = job.seg_len - span_begin < rows_per_span ? job.seg_len - span_begin : rows_per_span;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    const int trash = ft * Bp;
    const int n_acc = trash + 256;
    // histogram c: words [c * n_acc, (c + 1) * n_acc) of the accumulators, then of the side counters
    unsigned long long *main0 = lds;
    uint32_t *side0 = (uint32_t *)(lds + 2 * n_acc);
    for (int i = threadIdx.x; i < 2 * n_acc; i += kH2Block) {
        main0[i] = 0;
        side0[i] = 0;
    }
    WaveQueue<RW, true> queue{side0 + 2 * n_acc + wave * ((RW + 1) * kQueueSlots), 0u, 0u};
    uint32_t selA[4], selB[4];
    int pre[NS];
    {
        const int l0 = lane % ft;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            selA[k] = 0;
            selB[k] = 0;
        }
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            int t = j + l0;
            t = t >= ft ? t - ft : t;
            const bool live = j < ft;
            pre[j] = live ? t * Bp : trash + lane;
            const uint32_t a = (live && t < 8) ? (uint32_t)t : 0x0Cu;
            const uint32_t b = (live && t >= 8) ? (uint32_t)(t - 8) : 0x0Cu;
            selA[j >> 2] |= a << (8 * (j & 3));
            selB[j >> 2] |= b << (8 * (j & 3));
        }
    }
    // byte `feature` of a record for the three splits (see part_hist_kernel)
    uint32_t fselA[3], fselB[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        fselA[k] = 0x0C0C0C00u | (job.feature[k] < 8u ? job.feature[k] : 0x0Cu);
        fselB[k] = 0x0C0C0C00u | (job.feature[k] >= 8u ? job.feature[k] - 8u : 0x0Cu);
    }
    uint32_t my_lefts[2] = {0, 0};
    const uint64_t span_first = (uint64_t)job.seg_begin + span_begin;
    __syncthreads();

    auto byte_of = [&](const uint32_t (&row)[RW], uint32_t sa, uint32_t sb) __attribute__((always_inline)) {
        return __builtin_amdgcn_perm(SW > 1 ? row[SW > 1 ? 1 : 0] : 0u, row[0], sa) |
               __builtin_amdgcn_perm(SW > 3 ? row[SW > 3 ? 3 : 0] : 0u, SW > 2 ? row[SW > 2 ? 2 : 0] : 0u, sb);
    };
    auto load_tile = [&](uint32_t (&row)[ROWS][RW], uint32_t done) __attribute__((always_inline)) {
        const uint32_t tile_rows = span_rows - done < (uint32_t)TILE ? span_rows - done : (uint32_t)TILE;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const uint32_t in_tile = (uint32_t)(j * WAVES + wave) * 64u + (uint32_t)lane;
            if (in_tile < tile_rows) {
                const uint32_t *rp = src + (span_first + done + in_tile) * RW;
#pragma unroll
                for (int k = 0; k < RW; ++k) row[j][k] = rp[k];
            }
        }
    };
    auto add_waiting = [&](uint32_t n) __attribute__((always_inline)) {   // n <= 64 records from the head of the queue
        uint32_t rec[RW], c;
        if ((uint32_t)lane < n) {
            queue.peek(lane, rec, c);
            ph_add_row<NS, CHK, RW, kPHGroup, UNI>(rec, main0 + c * n_acc, side0 + c * n_acc, pre, selA, selB, trash, lane, missing, B);
        }
        queue.drop(n);
    };
    auto process = [&](uint32_t (&row)[ROWS][RW], uint32_t done) __attribute__((always_inline)) {
        const uint32_t tile_rows = span_rows - done < (uint32_t)TILE ? span_rows - done : (uint32_t)TILE;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const uint32_t in_tile = (uint32_t)(j * WAVES + wave) * 64u + (uint32_t)lane;
            bool left1 = false, counted = false;
            int c = 0;
            if (in_tile < tile_rows) {
                const uint32_t s0 = byte_of(row[j], fselA[0], fselB[0]);
                const bool left0 = (s0 == missing) ? (job.default_left[0] != 0) : (s0 <= job.bin[0]);
                c = left0 ? 0 : 1;
                const uint32_t s1 = byte_of(row[j], left0 ? fselA[1] : fselA[2], left0 ? fselB[1] : fselB[2]);
                const uint32_t bin1 = left0 ? job.bin[1] : job.bin[2];
                const uint32_t dl1 = left0 ? job.default_left[1] : job.default_left[2];
                left1 = (s1 == missing) ? (dl1 != 0) : (s1 <= bin1);
                counted = (left0 ? job.has[0] : job.has[1]) != 0;
            }
            const uint64_t b0 = __ballot(counted && c == 0 && left1), b1 = __ballot(counted && c == 1 && left1);
            my_lefts[0] += (uint32_t)__popcll(b0);
            my_lefts[1] += (uint32_t)__popcll(b1);
            const bool take = counted && (left1 == ((c == 0 ? job.build[0] : job.build[1]) == 1u));
            queue.push(take, row[j], (uint32_t)c);
            if (queue.waiting() >= 64u) add_waiting(64u);
        }
    };

    uint32_t rowA[ROWS][RW], rowB[ROWS][RW];
    load_tile(rowA, 0);
    for (uint32_t done = 0; done < span_rows;) {
        if (done + TILE < span_rows) load_tile(rowB, done + TILE);
        process(rowA, done);
        done += TILE;
        if (done >= span_rows) break;
        if (done + TILE < span_rows) load_tile(rowA, done + TILE);
        process(rowB, done);
        done += TILE;
    }
    if (queue.waiting()) add_waiting(queue.waiting());
    if (lane == 0) {
        if (my_lefts[0]) atomicAdd(&cursor[(size_t)(2 * ji) * kCursorStride], (unsigned long long)my_lefts[0]);
        if (my_lefts[1]) atomicAdd(&cursor[(size_t)(2 * ji + 1) * kCursorStride], (unsigned long long)my_lefts[1]);
    }
    __syncthreads();
    if (UNI) {
        if (job.has[0]) flush_tile_uniform(main0, ft, B, Bp, pool + job.hist_off[0], kH2Block, (int64_t)hq_uniform);
        if (job.has[1]) flush_tile_uniform(main0 + n_acc, ft, B, Bp, pool + job.hist_off[1], kH2Block, (int64_t)hq_uniform);
    } else {
        if (job.has[0]) flush_tile(main0, side0, ft, B, Bp, pool + job.hist_off[0], kH2Block);
        if (job.has[1]) flush_tile(main0 + n_acc, side0 + n_acc, ft, B, Bp, pool + job.hist_off[1], kH2Block);
    }
}

// Rows that stayed in place below their segment's own split are put in order again, LEVELS levels at once: a row
// is taken down from the segment's split through those of the nodes below (heap positions 0; 1, 2; 3..6) to a
// target node -- a child (LEVELS = 2) or a grandchild (LEVELS = 3) of the segment -- and stored on the left or
// right side of the target's range, left rows from the front, right rows from the back, room reserved per tile
// with one 64-bit atomic per target on its cursor ((4 * job + target) * kCursorStride: low word left rows handed
// out, high word right rows).  A row that reaches a node without a split is dropped: nothing reads the rows of a
// leaf again.  No histogram here: several targets would need as many of them in LDS; the built children are added
// up afterwards from their (then contiguous) records.  Two tiles are in flight as in part_hist_kernel; a row's
// category is 2 * target + (0 left, 1 right).
// FIRST: the rows come from the caller's packed matrix and the pair array (fp32 pairs where F32, rounded here as
// in part_hist_first_kernel) and leave as records; else they are records already.
constexpr int kM3Block = 512;
template <int NS, int LEVELS, bool FIRST, bool F32>
__global__ __launch_bounds__(kM3Block, 2) void move_levels_kernel(
    const uint32_t *__restrict__ src, uint32_t *__restrict__ dst, uint64_t dst_rows, uint32_t missing,
    const Move3Job *__restrict__ jobs, int n_jobs, uint32_t rows_per_span, unsigned long long *__restrict__ cursor,
    MoveFirst first) {
    constexpr int SW = (NS + 3) / 4;
    constexpr int RW = record_words(NS);
    constexpr int BLK = kM3Block, ROWS = kPFRows, TILE = BLK * ROWS, WAVES = BLK / 64, NW = TILE / 64;
    constexpr int NT = 1 << (LEVELS - 1);   // targets per segment
    constexpr int NC = 2 * NT;              // categories
    static_assert(LEVELS == 2 || LEVELS == 3, "two or three levels of splits");
    static_assert(WAVES >= NT, "one wave per target");
    static_assert(NW == 32, "a category's tile counts are scanned by half a wave");
    __shared__ Move3Job sjob;
    __shared__ uint32_t cnt[2][NW][NC];
    __shared__ uint32_t base_s[2][NC];
    int lo = 0, hi = n_jobs;   // last job with tile_begin <= this span
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (jobs[mid].tile_begin <= blockIdx.x) lo = mid; else hi = mid;
    }
    const int ji = lo;
    if (threadIdx.x < (int)(sizeof(Move3Job) / 4)) ((uint32_t *)&sjob)[threadIdx.x] = ((const uint32_t *)&jobs[ji])[threadIdx.x];
    __syncthreads();
    const Move3Job &job = sjob;
    const uint32_t span_begin = (blockIdx.x - job.tile_begin) * rows_per_span;
    if (span_begin >= job.seg_len) return;   // (uniform: a span past its segment has nothing to do)
    const uint32_t span_rows = job.seg_len - span_begin < rows_per_span ? job.seg_len - span_begin : rows_per_span;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t span_first = (uint64_t)job.seg_begin + span_begin;
    const uint64_t below_me = (1ull << lane) - 1ull;
    // FIRST: valid bits of the last symbol word of a row
    const uint32_t tail_bits = FIRST ? (uint32_t)(first.ft * 8 - 32 * (SW - 1)) : 32u;
    const uint32_t tail_mask = tail_bits >= 32 ? 0xffffffffu : ((1u << tail_bits) - 1u);

    auto symbol = [&](const uint32_t (&row)[RW], uint32_t f) __attribute__((always_inline)) -> uint32_t {
        const uint32_t sa = 0x0C0C0C00u | (f < 8u ? f : 0x0Cu), sb = 0x0C0C0C00u | (f >= 8u ? f - 8u : 0x0Cu);
        return __builtin_amdgcn_perm(SW > 1 ? row[SW > 1 ? 1 : 0] : 0u, row[0], sa) |
               __builtin_amdgcn_perm(SW > 3 ? row[SW > 3 ? 3 : 0] : 0u, SW > 2 ? row[SW > 2 ? 2 : 0] : 0u, sb);
    };
    auto goes_left = [&](const uint32_t (&row)[RW], uint32_t p) __attribute__((always_inline)) -> bool {
        const uint32_t sy = symbol(row, job.feature[p]);
        return sy == missing ? job.default_left[p] != 0 : sy <= job.bin[p];
    };
    auto load_tile = [&](uint32_t (&row)[ROWS][RW], uint32_t done) __attribute__((always_inline)) {
        const uint32_t tile_rows = span_rows - done < (uint32_t)TILE ? span_rows - done : (uint32_t)TILE;
        // FIRST: every word an unaligned row load of this tile can touch lies inside the source buffer
        const bool tile_inside = FIRST && (int64_t)(((span_first + done + tile_rows) * (uint64_t)first.stride_bytes) >> 2) + SW + 1 <= first.src_words;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const uint32_t in_tile = (uint32_t)(j * WAVES + wave) * 64u + (uint32_t)lane;
            if (in_tile < tile_rows) {
                const uint64_t p = span_first + done + in_tile;
                if (FIRST) {
                    load_first_row<NS, F32>(row[j], src, p, first, tile_inside, tail_mask);
                } else {
                    const uint32_t *rp = src + p * RW;
#pragma unroll
                    for (int k = 0; k < RW; ++k) row[j][k] = rp[k];
                }
            }
        }
    };
    auto process = [&](uint32_t (&row)[ROWS][RW], uint32_t done, int par) __attribute__((always_inline)) {
        const uint32_t tile_rows = span_rows - done < (uint32_t)TILE ? span_rows - done : (uint32_t)TILE;
        uint32_t cat[ROWS], rank[ROWS];
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const int w = j * WAVES + wave;
            const uint32_t in_tile = (uint32_t)w * 64u + (uint32_t)lane;
            uint32_t c = (uint32_t)NC;   // dropped
            if (in_tile < tile_rows) {
                const uint32_t p1 = goes_left(row[j], 0u) ? 1u : 2u;
                if (job.has[p1]) {
                    if (LEVELS == 2) {
                        c = 2u * (p1 - 1u) + (goes_left(row[j], p1) ? 0u : 1u);
                    } else {
                        const uint32_t p2 = 2u * p1 + (goes_left(row[j], p1) ? 1u : 2u);
                        if (job.has[p2]) c = 2u * (p2 - 3u) + (goes_left(row[j], p2) ? 0u : 1u);
                    }
                }
            }
            uint32_t r = 0;
#pragma unroll
            for (uint32_t k = 0; k < (uint32_t)NC; ++k) {
                const uint64_t b = __ballot(c == k);
                if (c == k) r = (uint32_t)__popcll(b & below_me);
                if (lane == 0) cnt[par][w][k] = (uint32_t)__popcll(b);
            }
            cat[j] = c;
            rank[j] = r;
        }
        __syncthreads();
        if (wave < NT) {   // wave g: places of target g's left rows (lanes 0..31) and right rows (lanes 32..63)
                           // inside the tile, and the tile's room in the target's range: one atomic for both sides
            const int half = lane >> 5, wl = lane & 31;
            const uint32_t v = cnt[par][wl][2 * wave + half];
            uint32_t x = v;
            for (int d = 1; d < 32; d <<= 1) {
                const uint32_t y = (uint32_t)__shfl_up((int)x, d);
                if (wl >= d) x += y;
            }
            cnt[par][wl][2 * wave + half] = x - v;
            const uint32_t lefts = (uint32_t)__shfl((int)x, 31), rights = (uint32_t)__shfl((int)x, 63);
            if (lane == 63) {
                unsigned long long old = 0;
                if (lefts | rights)
                    old = atomicAdd(&cursor[(size_t)(4 * ji + wave) * kCursorStride], (unsigned long long)lefts | ((unsigned long long)rights << 32));
                base_s[par][2 * wave] = (uint32_t)(old & 0xffffffffull);
                base_s[par][2 * wave + 1] = (uint32_t)(old >> 32);
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const int w = j * WAVES + wave;
            const uint32_t c = cat[j];
            if (c < (uint32_t)NC) {
                const uint32_t g = c >> 1;
                const uint32_t off = base_s[par][c] + cnt[par][w][c] + rank[j];
                const uint64_t q = (c & 1u) ? (uint64_t)job.node_begin[g] + job.node_len[g] - 1u - off : (uint64_t)job.node_begin[g] + off;
                if (off < job.node_len[g] && q < dst_rows) {   // (always, when the ranges are the counts of these very splits)
                    uint32_t *dp = dst + q * RW;
#pragma unroll
                    for (int k = 0; k < RW; ++k) dp[k] = row[j][k];
                }
            }
        }
        // cnt[par] and base_s[par] are rewritten two tiles from now, after two more barriers
    };

    uint32_t rowA[ROWS][RW], rowB[ROWS][RW];
    load_tile(rowA, 0);
    for (uint32_t done = 0; done < span_rows;) {
        if (done + TILE < span_rows) load_tile(rowB, done + TILE);
        process(rowA, done, 0);
        done += TILE;
        if (done >= span_rows) break;
        if (done + TILE < span_rows) load_tile(rowA, done + TILE);
        process(rowB, done, 1);
        done += TILE;
    }
}

}  // namespace

constexpr int64_t kAutoTileMinRows = 4000000;
int gbt_hist_feature_tile(const gbt_ctx *ctx, int F, int B, int64_t n_rows) {
    const size_t per_feature = (size_t)padded_bins(B) * 12;   // 8-byte word + 4-byte side counter per bin
    size_t limit = ctx->lds_per_block;
    if (ctx->hist_lds_kb > 0 && (size_t)ctx->hist_lds_kb * 1024 < limit) limit = (size_t)ctx->hist_lds_kb * 1024;
    if (limit < per_feature + 256 * 12) limit = ctx->lds_per_block;   // one feature must fit
    const size_t budget = limit - 256 * 12;                    // the trash row
    int ft = (int)(budget / per_feature);
    if (ft > F) ft = F;
    // A matrix that needs two to four tiles under the default cap pays for every tile with another pass over its rows
    // and pairs: where twice the LDS saves a tile, that is worth the halved occupancy (10M x 50 x 257 bins: three tiles
    // of 17 features -> two of 25, root 0.44 -> 0.35 ms, node histograms 1.21 -> 1.04 ms per tree).  With many tiles
    // the atomics of a tile's features outweigh the row fetch and the smaller tile wins (2000 features: 25 tiles of
    // 80 at 0.64 ms against 13 of 160 at 0.87 ms), and so it does on few rows, where workgroups are what is short
    // (1M x 28: two tiles 0.056 ms, one 0.082 ms).
    if (ctx->hist_lds_auto && ft >= 1 && n_rows >= kAutoTileMinRows) {
        const int nt = (F + ft - 1) / ft;
        const size_t limit2 = std::min<size_t>(ctx->lds_per_block, 2 * limit);
        if (nt >= 2 && nt <= 4 && limit2 > limit) {
            int ft2 = (int)((limit2 - 256 * 12) / per_feature);
            if (ft2 > F) ft2 = F;
            if (ft2 >= 1 && (F + ft2 - 1) / ft2 < nt) ft = ft2;
        }
    }
    return ft;   // 0: one feature's bins do not fit in LDS
}

namespace {
struct B8Args {
    hipStream_t s;
    int n_jobs, block;
    size_t lds;
    const uint32_t *packed;
    int64_t n_words, stride_bytes, n;
    int B, Bp;
    uint32_t missing;
    const uint32_t *row_idx;
    const int2 *gq;
    int64_t *pool;
    const HistJob *jobs;
    FixArgs fix;
};
template <bool LIST, int NS, bool CHK, bool FIX>
hipError_t launch_b8(const B8Args &a) {
    GbtLdsGuard lds_guard(a.lds);
    if (lds_guard.needed) {
        hipError_t e = hipFuncSetAttribute((const void *)hist_b8_kernel<LIST, NS, CHK, FIX>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds);
        if (e != hipSuccess) return e;
    }
    hist_b8_kernel<LIST, NS, CHK, FIX><<<a.n_jobs, a.block, a.lds, a.s>>>(a.packed, a.n_words, a.stride_bytes, a.n,
                                                                              a.B, a.Bp, a.missing, a.row_idx, a.gq,
                                                                              a.pool, a.jobs, a.fix);
    return hipGetLastError();
}
template <bool LIST, bool CHK, bool FIX>
hipError_t pick_slots_single(int max_ft, const B8Args &a) {
    if (max_ft <= 4) return launch_b8<LIST, 4, CHK, FIX>(a);
    if (max_ft <= 8) return launch_b8<LIST, 8, CHK, FIX>(a);
    if (max_ft <= 12) return launch_b8<LIST, 12, CHK, FIX>(a);
    if (max_ft == 13) return launch_b8<LIST, 13, CHK, FIX>(a);
    return launch_b8<LIST, 16, CHK, FIX>(a);
}
template <bool LIST, bool CHK>
hipError_t pick_slots(int max_ft, const B8Args &a) {
    if (max_ft > 16) return launch_b8<LIST, 0, CHK, false>(a);
    return pick_slots_single<LIST, CHK, false>(max_ft, a);
}
template <bool LIST>
hipError_t launch_generic(hipStream_t s, int n_jobs, int block, size_t lds, const uint32_t *packed, int64_t n_words, int bits,
                          int64_t stride_bits, int64_t n, int B, int Bp, uint32_t missing,
                          const uint32_t *row_idx, const int2 *gq, int64_t *pool, const HistJob *jobs) {
    GbtLdsGuard lds_guard(lds);
    if (lds_guard.needed) {
        hipError_t e = hipFuncSetAttribute((const void *)hist_generic_kernel<LIST>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const uint32_t inv_bits = (uint32_t)((((uint64_t)1 << 32) + (uint32_t)bits - 1) / (uint32_t)bits);
    hist_generic_kernel<LIST><<<n_jobs, block, lds, s>>>(packed, n_words, bits, inv_bits, stride_bits, n, B, Bp,
                                                               missing, row_idx, gq, pool, jobs);
    return hipGetLastError();
}
}  // namespace

hipError_t gbt_launch_hist(gbt_ctx *ctx, const uint32_t *packed, int bits, int64_t stride_bits, int64_t n_words,
                           int64_t n, int B, uint32_t missing, const uint32_t *row_idx, const int32_t *gq,
                           int64_t *hist_pool, const HistJob *jobs, int n_jobs, int max_ft, bool uniform_h,
                           int32_t hq_uniform) {
    if (n_jobs <= 0) return hipSuccess;
    if (!ctx->hist_runtime_bits && bits != 8)
        return gbt_launch_histw(ctx, packed, bits, stride_bits, n_words, n, B, missing, row_idx, gq, hist_pool, jobs,
                                n_jobs, max_ft, uniform_h, hq_uniform);
    const int Bp = padded_bins(B);
    const size_t lds = ((size_t)max_ft * Bp + 256) * 12;
    const int2 *g2 = (const int2 *)gq;
    hipStream_t s = ctx->stream;
    if (bits == 8 && (stride_bits & 7) == 0) {
        const bool chk = missing < 256u || B < 256;
        const B8Args a{s, n_jobs, ctx->hist_block, lds, packed, n_words, stride_bits >> 3, n, B, Bp, missing, row_idx, g2, hist_pool, jobs, FixArgs{}};
        if (row_idx) return chk ? pick_slots<true, true>(max_ft, a) : pick_slots<true, false>(max_ft, a);
        return chk ? pick_slots<false, true>(max_ft, a) : pick_slots<false, false>(max_ft, a);
    }
    if (row_idx)
        return launch_generic<true>(s, n_jobs, ctx->hist_block, lds, packed, n_words, bits, stride_bits, n, B, Bp, missing, row_idx, g2, hist_pool, jobs);
    return launch_generic<false>(s, n_jobs, ctx->hist_block, lds, packed, n_words, bits, stride_bits, n, B, Bp, missing, row_idx, g2, hist_pool, jobs);
}

bool gbt_hist_fix_ok(int bits, int64_t stride_bits, int max_ft, int n_ftiles) {
    return bits == 8 && (stride_bits & 7) == 0 && n_ftiles == 1 && max_ft <= 16;
}

hipError_t gbt_launch_hist_fix(gbt_ctx *ctx, const uint32_t *packed, int64_t stride_bits, int64_t n_words, int64_t n,
                               int B, uint32_t missing, const float *gpair, double sg, double sh, int32_t *gq_out,
                               int64_t *sums_out, int64_t *hist_pool, const HistJob *jobs, int n_jobs, int max_ft) {
    hipError_t e = gbt_launch_fill_u64(ctx->stream, (uint64_t *)sums_out, 0, 2);
    if (e != hipSuccess || n_jobs <= 0) return e;
    const int Bp = padded_bins(B);
    const size_t lds = ((size_t)max_ft * Bp + 256) * 12;
    const B8Args a{ctx->stream, n_jobs, ctx->hist_block, lds, packed, n_words, stride_bits >> 3, n, B, Bp, missing,
                   nullptr, nullptr, hist_pool, jobs,
                   FixArgs{(const float2 *)gpair, sg, sh, (int2 *)gq_out, sums_out}};
    const bool chk = missing < 256u || B < 256;
    return chk ? pick_slots_single<false, true, true>(max_ft, a) : pick_slots_single<false, false, true>(max_ft, a);
}

// ---- partition + histogram in one pass --------------------------------------
namespace {
struct PHArgs {
    hipStream_t s;
    int n_spans;
    size_t lds;
    const uint32_t *src;
    int64_t src_stride_bytes, src_words;
    const int2 *src_gq;
    bool src_fp32;     // first level: src_gq holds fp32 pairs, to be rounded with sgf, shf
    float sgf, shf;
    uint32_t *dst;
    int ft, B, Bp;
    uint32_t missing;
    const PartJob *jobs;
    int n_jobs;
    uint32_t rows_per_span;
    unsigned long long *cursor;
    int64_t *pool;
    int hq_uniform = -1;   // >= 0: every row has this hessian (the passes that keep rows in place then count rows instead)
};
template <int NS, bool CHK, bool F32, bool UNI>
hipError_t launch_ph_first_as(const PHArgs &a) {
    GbtLdsGuard lds_guard(a.lds);
    if (lds_guard.needed) {
        hipError_t e = hipFuncSetAttribute((const void *)part_hist_first_kernel<NS, CHK, F32, UNI>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds);
        if (e != hipSuccess) return e;
    }
    part_hist_first_kernel<NS, CHK, F32, UNI><<<a.n_spans, kPHBlock, a.lds, a.s>>>(a.src, a.src_stride_bytes, a.src_words, a.src_gq,
                                                                                   a.sgf, a.shf, a.dst, a.ft, a.B, a.Bp, a.missing,
                                                                                   a.jobs, a.n_jobs, a.rows_per_span, a.cursor, a.pool,
                                                                                   a.hq_uniform);
    return hipGetLastError();
}
template <int NS, bool CHK>
hipError_t launch_ph_first(const PHArgs &a) {
    const bool uni = a.hq_uniform >= 0 && a.rows_per_span <= kUniRowsMax;   // (a bin's row count has 18 bits)
    if (uni) return a.src_fp32 ? launch_ph_first_as<NS, CHK, true, true>(a) : launch_ph_first_as<NS, CHK, false, true>(a);
    return a.src_fp32 ? launch_ph_first_as<NS, CHK, true, false>(a) : launch_ph_first_as<NS, CHK, false, false>(a);
}
template <int NS, bool CHK, bool UNI>
hipError_t launch_ph_u(const PHArgs &a) {
    GbtLdsGuard lds_guard(a.lds);
    if (lds_guard.needed) {
        hipError_t e = hipFuncSetAttribute((const void *)part_hist_kernel<NS, CHK, UNI>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds);
        if (e != hipSuccess) return e;
    }
    part_hist_kernel<NS, CHK, UNI><<<a.n_spans, kPHBlock, a.lds, a.s>>>(a.src, a.dst, a.ft, a.B, a.Bp, a.missing, a.jobs, a.n_jobs,
                                                                        a.rows_per_span, a.cursor, a.pool, a.hq_uniform);
    return hipGetLastError();
}
template <int NS, bool CHK>
hipError_t launch_ph(const PHArgs &a) {
    if (a.hq_uniform >= 0 && a.rows_per_span <= kUniRowsMax) return launch_ph_u<NS, CHK, true>(a);
    return launch_ph_u<NS, CHK, false>(a);
}
template <int NS, bool CHK, bool FIRST, bool F32, bool UNI>
hipError_t launch_keep_as(const PHArgs &a) {
    GbtLdsGuard lds_guard(a.lds);
    if (lds_guard.needed) {
        hipError_t e = hipFuncSetAttribute((const void *)hist_keep_kernel<NS, CHK, FIRST, F32, UNI>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds);
        if (e != hipSuccess) return e;
    }
    const MoveFirst mf{a.src_stride_bytes, a.src_words, a.src_gq, a.sgf, a.shf, a.ft};
    hist_keep_kernel<NS, CHK, FIRST, F32, UNI><<<a.n_spans, kKeepBlock, a.lds, a.s>>>(a.src, a.ft, a.B, a.Bp, a.missing, a.jobs,
                                                                                      a.n_jobs, a.rows_per_span, a.cursor, a.pool,
                                                                                      mf, a.hq_uniform);
    return hipGetLastError();
}
template <int NS, bool CHK, bool UNI>
hipError_t launch_keep_u(const PHArgs &a, bool first) {
    if (!first) return launch_keep_as<NS, CHK, false, false, UNI>(a);
    return a.src_fp32 ? launch_keep_as<NS, CHK, true, true, UNI>(a) : launch_keep_as<NS, CHK, true, false, UNI>(a);
}
template <int NS, bool CHK>
hipError_t launch_keep(const PHArgs &a, bool first) {
    // (the row count of a bin has 18 bits: longer spans take the general form)
    if (a.hq_uniform >= 0 && a.rows_per_span <= kUniRowsMax) return launch_keep_u<NS, CHK, true>(a, first);
    return launch_keep_u<NS, CHK, false>(a, first);
}
template <bool CHK>
hipError_t pick_keep(int ft, const PHArgs &a, bool first) {
    if (ft <= 4) return launch_keep<4, CHK>(a, first);
    if (ft <= 8) return launch_keep<8, CHK>(a, first);
    if (ft <= 12) return launch_keep<12, CHK>(a, first);
    if (ft == 13) return launch_keep<13, CHK>(a, first);
    return launch_keep<16, CHK>(a, first);
}
template <bool CHK, bool FIRST>
hipError_t pick_ph(int ft, const PHArgs &a) {
    if (FIRST) {
        if (ft <= 4) return launch_ph_first<4, CHK>(a);
        if (ft <= 8) return launch_ph_first<8, CHK>(a);
        if (ft <= 12) return launch_ph_first<12, CHK>(a);
        if (ft == 13) return launch_ph_first<13, CHK>(a);
        return launch_ph_first<16, CHK>(a);
    }
    if (ft <= 4) return launch_ph<4, CHK>(a);
    if (ft <= 8) return launch_ph<8, CHK>(a);
    if (ft <= 12) return launch_ph<12, CHK>(a);
    if (ft == 13) return launch_ph<13, CHK>(a);
    return launch_ph<16, CHK>(a);
}
}  // namespace

bool gbt_part_hist_ok(const gbt_ctx *ctx, int bits, int F, int B) {
    if (bits != 8 || F > 16 || B > 256) return false;
    const size_t lds = ((size_t)F * padded_bins(B) + 256) * 12;
    const size_t cap = ctx->hist_lds_kb > 0 ? (size_t)ctx->hist_lds_kb * 1024 : ctx->lds_per_block;
    return lds <= cap && lds <= ctx->lds_per_block;
}
int gbt_part_hist_tile() { return kPHTile; }

namespace {
// LDS of the two-histogram pass: both histograms, then a tagged queue per wave
size_t hist2_lds(int F, int B) {
    return 2 * ((size_t)F * padded_bins(B) + 256) * 12 +
           (size_t)(kH2Block / 64) * (record_words(slots_for(F)) + 1) * kQueueSlots * 4;
}
// ... of the one-histogram pass over rows that stay
size_t keep_lds(int F, int B) {
    return ((size_t)F * padded_bins(B) + 256) * 12 + (size_t)(kKeepBlock / 64) * record_words(slots_for(F)) * kQueueSlots * 4;
}
}  // namespace
bool gbt_hist2_ok(const gbt_ctx *ctx, int F, int B) {
    if (F > 16 || B > 256) return false;
    return hist2_lds(F, B) <= ctx->lds_max;   // one workgroup per CU, no static LDS
}
namespace {
template <int NS, bool CHK, bool UNI>
hipError_t launch_hist2_u(gbt_ctx *ctx, size_t lds, const uint32_t *records, int ft, int B, int Bp, uint32_t missing,
                          const Hist2Job *jobs, int n_jobs, int n_spans, uint32_t rows_per_span,
                          unsigned long long *cursor, int64_t *pool, int hq_uniform) {
    GbtLdsGuard lds_guard(lds);
    if (lds_guard.needed) {
        hipError_t e = hipFuncSetAttribute((const void *)hist2_kernel<NS, CHK, UNI>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds);
        if (e != hipSuccess) return e;
    }
    hist2_kernel<NS, CHK, UNI><<<n_spans, kH2Block, lds, ctx->stream>>>(records, ft, B, Bp, missing, jobs, n_jobs, rows_per_span,
                                                                        cursor, pool, hq_uniform);
    return hipGetLastError();
}
template <int NS, bool CHK>
hipError_t launch_hist2(gbt_ctx *ctx, size_t lds, const uint32_t *records, int ft, int B, int Bp, uint32_t missing,
                        const Hist2Job *jobs, int n_jobs, int n_spans, uint32_t rows_per_span,
                        unsigned long long *cursor, int64_t *pool, int hq_uniform) {
    if (hq_uniform >= 0 && rows_per_span <= kUniRowsMax)
        return launch_hist2_u<NS, CHK, true>(ctx, lds, records, ft, B, Bp, missing, jobs, n_jobs, n_spans, rows_per_span, cursor, pool, hq_uniform);
    return launch_hist2_u<NS, CHK, false>(ctx, lds, records, ft, B, Bp, missing, jobs, n_jobs, n_spans, rows_per_span, cursor, pool, hq_uniform);
}
template <bool CHK>
hipError_t pick_hist2(int ft, gbt_ctx *ctx, size_t lds, const uint32_t *records, int B, int Bp, uint32_t missing,
                      const Hist2Job *jobs, int n_jobs, int n_spans, uint32_t rows_per_span, unsigned long long *cursor,
                      int64_t *pool, int hq) {
    if (ft <= 4) return launch_hist2<4, CHK>(ctx, lds, records, ft, B, Bp, missing, jobs, n_jobs, n_spans, rows_per_span, cursor, pool, hq);
    if (ft <= 8) return launch_hist2<8, CHK>(ctx, lds, records, ft, B, Bp, missing, jobs, n_jobs, n_spans, rows_per_span, cursor, pool, hq);
    if (ft <= 12) return launch_hist2<12, CHK>(ctx, lds, records, ft, B, Bp, missing, jobs, n_jobs, n_spans, rows_per_span, cursor, pool, hq);
    if (ft == 13) return launch_hist2<13, CHK>(ctx, lds, records, ft, B, Bp, missing, jobs, n_jobs, n_spans, rows_per_span, cursor, pool, hq);
    return launch_hist2<16, CHK>(ctx, lds, records, ft, B, Bp, missing, jobs, n_jobs, n_spans, rows_per_span, cursor, pool, hq);
}
}  // namespace

hipError_t gbt_launch_hist2(gbt_ctx *ctx, const uint32_t *records, int F, int B, uint32_t missing,
                            const Hist2Job *jobs, int n_jobs, int n_spans, uint32_t rows_per_span,
                            unsigned long long *cursor, int64_t *hist_pool, bool cursors_are_zero, int hq_uniform) {
    if (n_jobs <= 0 || n_spans <= 0) return hipSuccess;
    if (!cursors_are_zero) {
        hipError_t e = gbt_launch_fill_u64(ctx->stream, (uint64_t *)cursor, 0, 2 * (int64_t)n_jobs * kCursorStride);
        if (e != hipSuccess) return e;
    }
    const int Bp = padded_bins(B);
    const size_t lds = hist2_lds(F, B);
    const bool chk = missing < 256u || B < 256;
    return chk ? pick_hist2<true>(F, ctx, lds, records, B, Bp, missing, jobs, n_jobs, n_spans, rows_per_span, cursor, hist_pool, hq_uniform)
               : pick_hist2<false>(F, ctx, lds, records, B, Bp, missing, jobs, n_jobs, n_spans, rows_per_span, cursor, hist_pool, hq_uniform);
}
int gbt_move3_tile() { return kM3Block * kPFRows; }
namespace {
template <int LEVELS, bool FIRST, bool F32>
hipError_t launch_move(hipStream_t s, int ns, int n_spans, const uint32_t *src, uint32_t *dst, uint64_t dst_rows, uint32_t missing,
                       const Move3Job *jobs, int n_jobs, uint32_t rows_per_span, unsigned long long *cursor, const MoveFirst &mf) {
#define GBT_MV(NS_) move_levels_kernel<NS_, LEVELS, FIRST, F32><<<n_spans, kM3Block, 0, s>>>(src, dst, dst_rows, missing, jobs, n_jobs, \
                                                                                             rows_per_span, cursor, mf)
    if (ns == 4) GBT_MV(4);
    else if (ns == 8) GBT_MV(8);
    else if (ns == 12) GBT_MV(12);
    else if (ns == 13) GBT_MV(13);
    else GBT_MV(16);
#undef GBT_MV
    return hipGetLastError();
}
}  // namespace
hipError_t gbt_launch_move3(gbt_ctx *ctx, const uint32_t *src_records, uint32_t *dst_records, int64_t dst_rows, int F,
                            uint32_t missing, const Move3Job *jobs, int n_jobs, int n_spans, uint32_t rows_per_span,
                            unsigned long long *cursor, bool cursors_are_zero) {
    if (n_jobs <= 0 || n_spans <= 0) return hipSuccess;
    if (F < 1 || F > 16 || rows_per_span == 0 || dst_rows < 0) return hipErrorInvalidValue;
    if (!cursors_are_zero) {
        hipError_t e = gbt_launch_fill_u64(ctx->stream, (uint64_t *)cursor, 0, 4 * (int64_t)n_jobs * kCursorStride);
        if (e != hipSuccess) return e;
    }
    return launch_move<3, false, false>(ctx->stream, slots_for(F), n_spans, src_records, dst_records, (uint64_t)dst_rows, missing,
                                        jobs, n_jobs, rows_per_span, cursor, MoveFirst{});
}
hipError_t gbt_launch_move2_first(gbt_ctx *ctx, const uint32_t *packed, int64_t packed_words, const int32_t *gq,
                                  const float *gpair_fp32, double sg, double sh, uint32_t *dst_records, int64_t dst_rows, int F,
                                  uint32_t missing, const Move3Job *jobs, int n_jobs, int n_spans, uint32_t rows_per_span,
                                  unsigned long long *cursor, bool cursors_are_zero) {
    if (n_jobs <= 0 || n_spans <= 0) return hipSuccess;
    if (F < 1 || F > 16 || rows_per_span == 0 || dst_rows < 0 || (!gq && !gpair_fp32)) return hipErrorInvalidValue;
    if (!cursors_are_zero) {
        hipError_t e = gbt_launch_fill_u64(ctx->stream, (uint64_t *)cursor, 0, 4 * (int64_t)n_jobs * kCursorStride);
        if (e != hipSuccess) return e;
    }
    const MoveFirst mf{(int64_t)F, packed_words, gpair_fp32 ? (const int2 *)gpair_fp32 : (const int2 *)gq, (float)sg, (float)sh, F};
    if (gpair_fp32)
        return launch_move<2, true, true>(ctx->stream, slots_for(F), n_spans, packed, dst_records, (uint64_t)dst_rows, missing, jobs,
                                          n_jobs, rows_per_span, cursor, mf);
    return launch_move<2, true, false>(ctx->stream, slots_for(F), n_spans, packed, dst_records, (uint64_t)dst_rows, missing, jobs,
                                       n_jobs, rows_per_span, cursor, mf);
}

int gbt_part_hist_record_words(int F) { return record_words(slots_for(F)); }

hipError_t gbt_launch_part_hist(gbt_ctx *ctx, const uint32_t *packed, int64_t packed_words, const int32_t *gq,
                                const uint32_t *src_records, uint32_t *dst_records, int F, int B, uint32_t missing,
                                const PartJob *jobs, int n_jobs, int n_spans, uint32_t rows_per_span,
                                unsigned long long *cursor, int64_t *hist_pool, bool cursors_are_zero,
                                const float *gpair_fp32, double sg, double sh, int hq_uniform) {
    if (n_jobs <= 0 || n_spans <= 0) return hipSuccess;
    if (!cursors_are_zero) {
        hipError_t e = gbt_launch_fill_u64(ctx->stream, (uint64_t *)cursor, 0, (int64_t)n_jobs * kCursorStride);
        if (e != hipSuccess) return e;
    }
    const int Bp = padded_bins(B);
    const bool first = src_records == nullptr;
    const bool fp32 = first && gpair_fp32 != nullptr;
    const PHArgs a{ctx->stream, n_spans, ((size_t)F * Bp + 256) * 12, first ? packed : src_records, first ? (int64_t)F : 0,
                   packed_words, fp32 ? (const int2 *)gpair_fp32 : (const int2 *)gq, fp32, (float)sg, (float)sh, dst_records,
                   F, B, Bp, missing, jobs, n_jobs, rows_per_span, cursor, hist_pool, hq_uniform};
    const bool chk = missing < 256u || B < 256;
    if (dst_records == nullptr && keep_lds(F, B) <= ctx->lds_per_block) {   // rows that stay in place
        PHArgs k = a;
        k.lds = keep_lds(F, B);
        return chk ? pick_keep<true>(F, k, first) : pick_keep<false>(F, k, first);
    }
    if (first) return chk ? pick_ph<true, true>(F, a) : pick_ph<false, true>(F, a);
    return chk ? pick_ph<true, false>(F, a) : pick_ph<false, false>(F, a);
}
