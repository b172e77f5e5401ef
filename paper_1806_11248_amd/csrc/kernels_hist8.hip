// BuildPartialHistograms (Alg. 1) of ALL rows of the matrix -- the root of a tree -- for 8-bit symbols
// and at most 16 features (one LDS tile), gfx950.
//
// The launch is bound by the stream of rows from HBM, so everything else is arranged to stay out of its
// way:
//  * lane = row.  A row's bytes are loaded as whole words at immediate offsets from one address (the
//    compiler merges them into one wide load), realigned with byte funnel shifts, and permuted per lane
//    so that unrolled slot j of lane l holds feature (j + l) mod ft: the lanes of an instruction work on
//    different features.  The loads of the rows a few iterations ahead are issued before a row is
//    processed (software prefetch), so a wave never waits a whole memory latency per row.
//  * LDS word of (feature t, symbol s) = s * 16 + t: a feature owns one LDS bank pair, so the lanes of an
//    instruction meet in a bank only if they work on the same feature (five lanes at thirteen features),
//    whatever the symbols are.  All 256 symbol values have a word: a missing or out-of-range symbol needs
//    no test in the loop, its word is simply never merged.
//  * two forms of the accumulated word:
//      general   [ g : 34 bits signed | h : 30 bits ], added with a returning 64-bit atomic; the lane whose
//                add carried out of the h field or wrapped the g field sees it in the returned word and
//                counts it in a side counter of the bin (see kernels_hist.hip for the tests);
//      uniform h (every row of the tree has the same hessian: squared error always, the first tree of a
//                logistic model)  [ g : 46 bits signed | rows : 18 bits ], added with a non-returning
//                atomic: with at most 2^18 - 1 rows per workgroup neither field can overflow, so nothing
//                is tested, and sum h = rows * h.
//  * few, long jobs: workgroup (c, k) takes slice k of column c of the rows, about one column per compute
//    unit.  Every workgroup merges its whole LDS histogram into HBM with 64-bit global atomics at its end
//    and the chip retires those slowly, so the slices of a column have UNEQUAL lengths: the workgroups
//    that share a compute unit finish, and merge, one after the other while the others still stream.
//  * the gradient pairs may still be fp32 (the first launch of a tree): the kernel rounds them to fixed
//    point itself -- in fp32 arithmetic where that is exact (power-of-two scales of moderate size), else
//    through fp64 --, stores them only if asked to, and adds up the totals of all rows.
#include "gbt_internal.h"

#include <math.h>

#include <algorithm>

namespace {

typedef unsigned long long __attribute__((address_space(3))) lds_u64;
__device__ __forceinline__ unsigned long long lds_add_rtn(uint32_t addr, unsigned long long v) {
    return __hip_atomic_fetch_add((lds_u64 *)(uintptr_t)addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void lds_add(uint32_t addr, unsigned long long v) {
    (void)__hip_atomic_fetch_add((lds_u64 *)(uintptr_t)addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

constexpr int kRowsShift = 18;                                  // uniform h: width of the row-count field
constexpr uint32_t kUniformMaxRows = (1u << kRowsShift) - 1u;   // rows of one workgroup
constexpr uint32_t kGeneralMaxRows = 1u << 21;                  // the side counters are 16 bits wide
constexpr int kLdsWords = 256 * 16;

struct Hist8Args {
    const uint32_t *packed;
    int64_t n;
    int ft, B;
    uint32_t missing;
    const float2 *gpair;
    const int2 *gq;
    int2 *gq_out;
    double sg, sh;
    float sgf, shf;
    int32_t hq_uniform;
    int64_t *sums, *out;
    uint32_t cols, slots, stagger;   // job geometry: see job_rows()
    // FILT: only the rows on one side of a split are added (the histogram of one child of the root, the rows
    // staying where they are); the rows that go left are counted into *lefts
    uint32_t split_feature, split_bin, split_default_left, take_left;
    unsigned long long *lefts;
    // FIX == 3: the rows are records (symbols, padding, 7 bytes of fixed-point pair) of several nodes, each node's
    // contiguous: workgroup = one span of rows_per_span rows of a job (PartJob: seg_begin, seg_len, tile_begin = its
    // first span, hist_off = the node's histogram inside pool)
    const uint32_t *records;
    const PartJob *jobs;
    int n_jobs;
    uint32_t rows_per_span;
    int64_t *pool;
};

// Rows of workgroup (column c, slice k): the n rows are cut into `cols` equal columns, a column into
// `slots` slices whose lengths fall linearly from (1 + stagger/256 * (slots-1)/slots) / slots of the column to
// (1 - ...) / slots.
__host__ __device__ inline uint64_t slice_edge(uint64_t len, uint32_t k, uint32_t slots, uint32_t stagger) {
    const uint64_t num = (uint64_t)k * 256u * slots + (uint64_t)stagger * k * (slots - k);
    return len * num / (256ull * slots * slots);   // len < 2^32, num < 2^22
}

// The two quick tests on a returned word and the bookkeeping behind them: as in kernels_hist.hip.
__device__ __forceinline__ void pk_check8(uint32_t side_addr, unsigned long long old, unsigned long long addv, uint32_t hq,
                                          uint32_t kind, uint32_t reach) {
    uint32_t olo = (uint32_t)old, ohi = (uint32_t)(old >> 32);
    const bool danger = ((~olo & kHMask) < hq) | ((ohi ^ kind) < reach);
    if (danger) {
        asm volatile("" : "+v"(olo), "+v"(ohi));   // keep the rare bookkeeping inside the branch
        const uint32_t carry = ((olo & kHMask) + hq) >> kHShift;
        const uint32_t alo = (uint32_t)addv, ahi = (uint32_t)(addv >> 32);
        const uint32_t nlo = olo + alo;
        const uint32_t nhi = ohi + ahi + (nlo < olo ? 1u : 0u);
        const int32_t ovf = (int32_t)((ohi ^ nhi) & (ahi ^ nhi));   // sign bit set: the g field wrapped
        const int32_t delta = ovf < 0 ? ((int32_t)nhi < 0 ? 1 : -1) : 0;
        if (carry != 0 || delta != 0)
            (void)__hip_atomic_fetch_add((uint32_t __attribute__((address_space(3))) *)(uintptr_t)side_addr,
                                         (uint32_t)(delta * 65536 + (int32_t)carry), __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

// NS  : unrolled slots = features of the tile rounded up to 4, 8, 12, 13, 16 (ft > NS - 4, or NS - 1 for 13)
// UNI : the uniform-h word
// FIX : 0 fixed-point pairs are read; 1 fp32 pairs rounded through fp64; 2 rounded in fp32; 3 the rows are records
//       that carry their pair (Hist8Args)
// FILT: see Hist8Args
template <int NS, bool UNI, int FIX, int BLOCK, int MINWG, int PF, bool FILT>
__global__ __launch_bounds__(BLOCK, MINWG) void hist8_kernel(const Hist8Args a) {
    constexpr bool REC = FIX == 3;
    constexpr int RW = (NS + 7 + 3) / 4;                // words of a record
    constexpr int NW = REC ? RW : (NS + 6) / 4;         // words a row of NS - 3 .. NS bytes can touch at any alignment
    constexpr int SW = (NS + 3) / 4;                    // words of symbols after realignment
    extern __shared__ unsigned long long lds[];
    unsigned long long *main_ = lds;
    uint32_t *side = (uint32_t *)(lds + kLdsWords);
    for (int i = threadIdx.x; i < kLdsWords; i += BLOCK) {
        main_[i] = 0;
        if (!UNI) side[i] = 0;
    }
    const int lane = threadIdx.x & 63;
    const int ft = a.ft;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_u64 *)main_;
    // slot j of this lane handles feature (j + lane) mod ft
    uint32_t selA[4] = {0, 0, 0, 0}, selB[4] = {0, 0, 0, 0};
    uint32_t pre[NS];   // LDS byte address of word (feature of slot j, symbol 0)
    {
        const int l0 = lane % ft;
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            int t = j + l0;
            t = t >= ft ? t - ft : t;
            const bool live = j < ft;
            pre[j] = (uint32_t)t * 8u + lds_base;
            const uint32_t sa = (live && t < 8) ? (uint32_t)t : 0x0Cu;           // 0x0C selects a zero byte
            const uint32_t sb = (live && t >= 8) ? (uint32_t)(t - 8) : 0x0Cu;
            selA[j >> 2] |= sa << (8 * (j & 3));
            selB[j >> 2] |= sb << (8 * (j & 3));
        }
    }
    __syncthreads();

    // this workgroup's rows
    uint64_t job_row0;
    uint32_t job_rows;
    int64_t *__restrict__ out = a.out;
    if (REC) {
        int lo = 0, hi = a.n_jobs;   // last job whose first span is <= this one
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (a.jobs[mid].tile_begin <= blockIdx.x) lo = mid; else hi = mid;
        }
        const PartJob job = a.jobs[lo];
        const uint32_t span_begin = (blockIdx.x - job.tile_begin) * a.rows_per_span;
        job_rows = job.seg_len - span_begin < a.rows_per_span ? job.seg_len - span_begin : a.rows_per_span;
        job_row0 = (uint64_t)job.seg_begin + span_begin;
        out = a.pool + job.hist_off;
    } else {
        const uint32_t c = blockIdx.x % a.cols, sl = blockIdx.x / a.cols;
        const uint64_t col = ((uint64_t)a.n + a.cols - 1) / a.cols;
        const uint64_t c0 = (uint64_t)c * col < (uint64_t)a.n ? (uint64_t)c * col : (uint64_t)a.n;
        const uint64_t c1 = c0 + col < (uint64_t)a.n ? c0 + col : (uint64_t)a.n;
        const uint64_t e0 = slice_edge(c1 - c0, sl, a.slots, a.stagger), e1 = slice_edge(c1 - c0, sl + 1, a.slots, a.stagger);
        job_row0 = c0 + e0;
        job_rows = (uint32_t)(e1 - e0);
    }
    const uint64_t job_byte0 = REC ? 0 : job_row0 * (uint64_t)ft;
    const char *__restrict__ pb = (const char *)(a.packed + (job_byte0 >> 2));
    const uint32_t a0 = (uint32_t)(job_byte0 & 3);
    const float2 *__restrict__ gp = a.gpair + (REC ? 0 : job_row0);
    const int2 *__restrict__ gq = a.gq + (REC ? 0 : job_row0);
    int2 *__restrict__ gqo = (!REC && a.gq_out) ? a.gq_out + job_row0 : nullptr;
    const uint32_t *__restrict__ recs = REC ? a.records + job_row0 * RW : nullptr;

    long long sum_g = 0, sum_h = 0;   // UNI: sum_g holds the sum of the packed words (G * 2^18 + rows)
    // FILT: byte `split_feature` of the realigned row, and the rows seen going left
    const uint32_t fselA = 0x0C0C0C00u | (a.split_feature < 8u ? a.split_feature : 0x0Cu);
    const uint32_t fselB = 0x0C0C0C00u | (a.split_feature >= 8u ? a.split_feature - 8u : 0x0Cu);
    uint32_t my_lefts = 0;
    // the words and the pair of the row PF iterations ahead are on their way while a row is processed
    uint32_t wq[PF + 1][NW];
    float2 vq[PF + 1];
    int2 gqq[PF + 1];
    auto issue = [&](int slot, uint32_t i) __attribute__((always_inline)) {
        if (i < job_rows) {
            if (REC) {
#pragma unroll
                for (int k = 0; k < NW; ++k) wq[slot][k] = recs[(size_t)i * RW + k];
            } else {
                const uint32_t b4 = (a0 + i * (uint32_t)ft) & ~3u;
#pragma unroll
                for (int k = 0; k < NW; ++k) wq[slot][k] = *(const uint32_t *)(pb + b4 + 4 * k);
                if (FIX != 0) vq[slot] = gp[i];
                else gqq[slot] = gq[i];
            }
        }
    };
#pragma unroll
    for (int d = 0; d < PF; ++d) issue(d, threadIdx.x + d * BLOCK);
    for (uint32_t i = threadIdx.x; i < job_rows; i += BLOCK) {
        issue(PF, i + PF * BLOCK);
        uint32_t w[NW];
#pragma unroll
        for (int k = 0; k < NW; ++k) w[k] = wq[0][k];
        const float2 v = vq[0];
        int2 q = gqq[0];
#pragma unroll
        for (int d = 0; d < PF; ++d) {
#pragma unroll
            for (int k = 0; k < NW; ++k) wq[d][k] = wq[d + 1][k];
            vq[d] = vq[d + 1];
            gqq[d] = gqq[d + 1];
        }
        if (FIX == 1) {
            q.x = __double2int_rn((double)v.x * a.sg);
            q.y = __double2int_rn((double)v.y * a.sh);
        } else if (FIX == 2) {
            q.x = (int)rintf(v.x * a.sgf);
            q.y = (int)rintf(v.y * a.shf);
        } else if (REC) {   // the pair: bytes 1..3 of word RW - 2 and word RW - 1 (28 bits of g, signed, then 24 of h)
            const uint32_t qlo = (w[RW - 2] >> 8) | (w[RW - 1] << 24), qhi = w[RW - 1] >> 8;
            q.x = (int32_t)(qlo << 4) >> 4;
            q.y = (int32_t)((qlo >> 28) | (qhi << 4));
        }
        if (FIX != 0 && !REC && gqo) gqo[i] = q;
        const uint32_t al = REC ? 0u : (a0 + i * (uint32_t)ft) & 3u;
        uint32_t W[4] = {0, 0, 0, 0}, V[SW];
#pragma unroll
        for (int k = 0; k < SW; ++k) W[k] = __builtin_amdgcn_alignbyte(w[k + 1 < NW ? k + 1 : NW - 1], w[k], al);
#pragma unroll
        for (int k = 0; k < SW; ++k)
            V[k] = __builtin_amdgcn_perm(W[1], W[0], selA[k]) | __builtin_amdgcn_perm(W[3], W[2], selB[k]);
        if (FILT) {
            const uint32_t sy = __builtin_amdgcn_perm(W[1], W[0], fselA) | __builtin_amdgcn_perm(W[3], W[2], fselB);
            const bool left = sy == a.missing ? a.split_default_left != 0 : sy <= a.split_bin;
            my_lefts += left ? 1u : 0u;
            if (left != (a.take_left != 0)) continue;
        }
        if (!UNI) {
            const unsigned long long addv = ((unsigned long long)(long long)q.x << kHShift) + (unsigned long long)(uint32_t)q.y;
            const uint32_t hq = (uint32_t)q.y;
            sum_g += q.x;
            sum_h += hq;
            const uint32_t ahi = (uint32_t)(addv >> 32);                       // floor(g / 4), signed
            const uint32_t down = (uint32_t)((int32_t)ahi >> 31);              // 0 going up, all ones going down
            const uint32_t kind = down ^ 0x7FFFFFFFu, reach = (ahi ^ down) + 2u;
            unsigned long long old[NS];
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                const uint32_t s = (V[j >> 2] >> (8 * (j & 3))) & 0xffu;
                if (j < NS - 3 || j < ft) old[j] = lds_add_rtn((s << 7) + pre[j], addv);
            }
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                const uint32_t s = (V[j >> 2] >> (8 * (j & 3))) & 0xffu;
                // the side counter of word x (byte address lds_base + 8 x) is at lds_base + 8 * kLdsWords + 4 x
                if (j < NS - 3 || j < ft)
                    pk_check8(lds_base + 8u * kLdsWords + ((((s << 7) + pre[j]) - lds_base) >> 1), old[j], addv, hq, kind, reach);
            }
        } else {
            const unsigned long long addv = ((unsigned long long)(long long)q.x << kRowsShift) + 1ull;
            sum_g += (long long)addv;
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                const uint32_t s = (V[j >> 2] >> (8 * (j & 3))) & 0xffu;
                if (j < NS - 3 || j < ft) lds_add((s << 7) + pre[j], addv);
            }
        }
    }
    if (FILT) {   // one atomic per workgroup on a counter that has a line of its own
        __shared__ uint32_t lred[BLOCK / 64];
        for (int o = 32; o > 0; o >>= 1) my_lefts += (uint32_t)__shfl_xor((int)my_lefts, o);
        if (lane == 0) lred[threadIdx.x >> 6] = my_lefts;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t t = 0;
            for (int w = 0; w < BLOCK / 64; ++w) t += lred[w];
            if (t) atomicAdd(a.lefts, (unsigned long long)t);
        }
    }
    __syncthreads();
    // merge the bins into the node's histogram
    const int B = a.B;
    for (int i = threadIdx.x; i < ft * B; i += BLOCK) {
        const int t = i / B, b = i - t * B;
        if (b > 255 || (uint32_t)b == a.missing) continue;
        const int idx = b * 16 + t;
        const unsigned long long wv = main_[idx];
        int64_t g, h;
        if (!UNI) {
            const uint32_t sc = side[idx];
            if (wv == 0 && sc == 0) continue;
            const int64_t carry = (int64_t)(sc & 0xffffu), wraps = (int64_t)((int32_t)sc >> 16);
            g = ((int64_t)wv >> kHShift) + wraps * ((int64_t)1 << (64 - kHShift)) - carry;
            h = (int64_t)(wv & kHMask) + (carry << kHShift);
        } else {
            if (wv == 0) continue;
            const int64_t rows = (int64_t)(wv & kUniformMaxRows);
            g = ((int64_t)wv - rows) >> kRowsShift;
            h = rows * a.hq_uniform;
        }
        if (g != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i), (unsigned long long)g);
        if (h != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i + 1), (unsigned long long)h);
    }
    if (!REC && a.sums) {   // totals of this workgroup's rows into its own slot: same-address global atomics take turns
        long long G = sum_g, H = sum_h;
        if (UNI) {
            const long long rows = sum_g & (long long)kUniformMaxRows;
            G = (sum_g - rows) >> kRowsShift;
            H = rows * a.hq_uniform;
        }
        for (int o = 32; o > 0; o >>= 1) {
            G += __shfl_xor(G, o);
            H += __shfl_xor(H, o);
        }
        __shared__ long long red[2][BLOCK / 64];
        if (lane == 0) {
            red[0][threadIdx.x >> 6] = G;
            red[1][threadIdx.x >> 6] = H;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int w = 1; w < BLOCK / 64; ++w) {
                G += red[0][w];
                H += red[1][w];
            }
            a.sums[2 * blockIdx.x] = G;
            a.sums[2 * blockIdx.x + 1] = H;
        }
    }
}

template <int NS, bool UNI, int FIX, bool FILT>
hipError_t launch8(hipStream_t s, const Hist8Args &a, int grid) {
    constexpr int BLOCK = UNI ? 256 : 512, MINWG = UNI ? 4 : 2, PF = UNI ? 3 : 1;
    const size_t lds = (size_t)kLdsWords * (UNI ? 8 : 12);   // 32 or 48 KB: within the default limit of a launch
    hist8_kernel<NS, UNI, FIX, BLOCK, MINWG, PF, FILT><<<grid, BLOCK, lds, s>>>(a);
    return hipGetLastError();
}
template <bool UNI, int FIX, bool FILT>
hipError_t pick8f(hipStream_t s, const Hist8Args &a, int grid) {
    if (a.ft <= 4) return launch8<4, UNI, FIX, FILT>(s, a, grid);
    if (a.ft <= 8) return launch8<8, UNI, FIX, FILT>(s, a, grid);
    if (a.ft <= 12) return launch8<12, UNI, FIX, FILT>(s, a, grid);
    if (a.ft == 13) return launch8<13, UNI, FIX, FILT>(s, a, grid);
    return launch8<16, UNI, FIX, FILT>(s, a, grid);
}
template <bool UNI, int FIX>
hipError_t pick8(hipStream_t s, const Hist8Args &a, int grid) {
    // (the filtered form reads fixed-point pairs or rounds fp32 pairs in fp32: the two ways its callers have them)
    if constexpr (FIX == 0 || FIX == 2) {
        if (a.lefts != nullptr) return pick8f<UNI, FIX, true>(s, a, grid);
    }
    if (a.lefts != nullptr) return hipErrorInvalidValue;
    return pick8f<UNI, FIX, false>(s, a, grid);
}
int slots_of(int ft) { return ft <= 4 ? 4 : ft <= 8 ? 8 : ft <= 12 ? 12 : ft == 13 ? 13 : 16; }
}  // namespace

bool gbt_hist8_ok(int bits, int F, int n_ftiles, int64_t n, int64_t n_words) {
    if (bits != 8 || n_ftiles != 1 || F < 1 || F > 16 || n < 1) return false;
    // the last row's window of whole words lies inside the buffer (true for a matrix of gbt_packed_words words)
    const int NW = (slots_of(F) + 6) / 4;
    return (((n - 1) * (int64_t)F) >> 2) + NW <= n_words;
}

bool gbt_fix32_ok(double sg, double sh) {
    // v * scale is exact in fp32 and rounds like the fp64 product: a power-of-two scale of moderate size
    auto ok = [](double s) {
        int e;
        return s > 0.0 && frexp(s, &e) == 0.5 && e - 1 >= -60 && e - 1 <= 60;
    };
    return ok(sg) && ok(sh);
}

int gbt_hist8_max_jobs() { return 1 << 14; }

hipError_t gbt_launch_hist8(gbt_ctx *ctx, const uint32_t *packed, int64_t n, int F, int B, uint32_t missing,
                            const Hist8Pairs &p, int64_t *hist_out, int *n_jobs_out, const Hist8Filter *filter) {
    if (n_jobs_out) *n_jobs_out = 0;
    if (n <= 0) return hipSuccess;
    if (filter && (filter->lefts == nullptr || filter->feature < 0 || filter->feature >= F || (p.gpair && p.mode == 1)))
        return hipErrorInvalidValue;
    const bool uni = p.uniform_h != 0;
    Hist8Args a;
    a.packed = packed;
    a.n = n;
    a.ft = F;
    a.B = B;
    a.missing = missing;
    a.gpair = (const float2 *)p.gpair;
    a.gq = (const int2 *)p.gq;
    a.gq_out = (int2 *)p.gq_out;
    a.sg = p.sg;
    a.sh = p.sh;
    a.sgf = (float)p.sg;
    a.shf = (float)p.sh;
    a.hq_uniform = p.hq_uniform;
    a.sums = p.sums;
    a.out = hist_out;
    a.split_feature = filter ? (uint32_t)filter->feature : 0u;
    a.split_bin = filter ? (uint32_t)filter->bin : 0u;
    a.split_default_left = filter ? (uint32_t)filter->default_left : 0u;
    a.take_left = filter ? (uint32_t)filter->take_left : 0u;
    a.lefts = filter ? filter->lefts : nullptr;
    // about one column of rows per compute unit, cut into as many slices as workgroups share a unit; short
    // inputs take fewer, equal jobs; long ones more slices, so that no workgroup exceeds its row limit
    const int64_t block = uni ? 256 : 512;
    const int64_t resident = uni ? 4 : 2;
    const uint64_t max_rows = uni ? kUniformMaxRows : kGeneralMaxRows;
    int64_t cols = std::min<int64_t>(ctx->num_cu, (n + 4 * block - 1) / (4 * block));
    int64_t slots = (n / cols) >= resident * 8 * block ? resident : 1;
    uint32_t stagger = slots > 1 ? (uint32_t)ctx->hist8_stagger : 0u;
    const uint64_t col = ((uint64_t)n + cols - 1) / cols;
    while (slice_edge(col, 1, (uint32_t)slots, stagger) > max_rows) slots += resident;   // the first slice is the longest
    a.cols = (uint32_t)cols;
    a.slots = (uint32_t)slots;
    a.stagger = stagger;
    const int grid = (int)(cols * slots);
    if (grid > gbt_hist8_max_jobs()) return hipErrorInvalidValue;
    if (n_jobs_out) *n_jobs_out = grid;
    const int mode = p.gpair ? p.mode : 0;
    if (uni) {
        if (mode == 0) return pick8<true, 0>(ctx->stream, a, grid);
        if (mode == 1) return pick8<true, 1>(ctx->stream, a, grid);
        return pick8<true, 2>(ctx->stream, a, grid);
    }
    if (mode == 0) return pick8<false, 0>(ctx->stream, a, grid);
    if (mode == 1) return pick8<false, 1>(ctx->stream, a, grid);
    return pick8<false, 2>(ctx->stream, a, grid);
}

// The same kernel over records: the histograms of several nodes, each from its contiguous records (every row of a
// job's segment is added).  jobs [dev]: PartJob with seg_begin, seg_len, tile_begin (first span), hist_off; spans of
// rows_per_span rows; the histograms (pool + hist_off) must have been cleared.  hq_uniform >= 0: every row has that
// hessian (the row-count form, where a span is short enough for it).
hipError_t gbt_launch_hist8_records(gbt_ctx *ctx, const uint32_t *records, int F, int B, uint32_t missing,
                                    const PartJob *jobs, int n_jobs, int n_spans, uint32_t rows_per_span, int64_t *pool,
                                    int32_t hq_uniform) {
    if (n_jobs <= 0 || n_spans <= 0) return hipSuccess;
    if (F < 1 || F > 16 || rows_per_span == 0 || rows_per_span > kGeneralMaxRows) return hipErrorInvalidValue;
    Hist8Args a{};
    a.ft = F;
    a.B = B;
    a.missing = missing;
    a.hq_uniform = hq_uniform >= 0 ? hq_uniform : 0;
    a.records = records;
    a.jobs = jobs;
    a.n_jobs = n_jobs;
    a.rows_per_span = rows_per_span;
    a.pool = pool;
    if (hq_uniform >= 0 && rows_per_span <= kUniformMaxRows) return pick8<true, 3>(ctx->stream, a, n_spans);
    return pick8<false, 3>(ctx->stream, a, n_spans);
}
