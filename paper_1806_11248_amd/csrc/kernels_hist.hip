// BuildPartialHistograms (Alg. 1; Sec. 2.1 "gradient summation into
// histograms") for gfx950.
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
// [ wraps : int16 | carries : uint16 ] of the same bin.  Events are rare (at
// least 256 adds between carries, 128 same-sign extreme adds between wraps), a
// two-compare test on the returned word skips the bookkeeping otherwise.
//
// The bin axis of the LDS histogram is padded to an odd stride so that equal bin
// indices of different features (e.g. the most frequent category of several
// skewed columns) fall into different LDS banks.
#include "gbt_internal.h"

namespace {

constexpr int kHistBlock = 1024;
constexpr int kHShift = 30;                        // width of the h field
constexpr uint32_t kHMask = (1u << kHShift) - 1u;

__device__ __forceinline__ void pk_add(unsigned long long *main_, uint32_t *side, int idx,
                                       unsigned long long addv, uint32_t hq) {
    const unsigned long long old = atomicAdd(&main_[idx], addv);
    const uint32_t olo = (uint32_t)old, ohi = (uint32_t)(old >> 32);
    // carry possible only if h-field bits 22..29 are all ones; wrap possible only if the
    // g field is within 2^27 of +-2^33 (top seven bits of the word are 0111111 or 1000000)
    const bool danger = ((olo & 0x3FC00000u) == 0x3FC00000u) | ((ohi + 0x82000000u) < 0x04000000u);
    if (danger) {
        const uint32_t carry = ((olo & kHMask) + hq) >> kHShift;
        const unsigned long long nw = old + addv;
        const uint32_t nhi = (uint32_t)(nw >> 32), ahi = (uint32_t)(addv >> 32);
        const int32_t ovf = (int32_t)((ohi ^ nhi) & (ahi ^ nhi));   // sign bit set: the g field wrapped
        const int32_t delta = ovf < 0 ? ((int32_t)nhi < 0 ? 1 : -1) : 0;
        if (carry != 0 || delta != 0) atomicAdd(&side[idx], (uint32_t)(delta * 65536 + (int32_t)carry));
    }
}

__device__ __forceinline__ unsigned long long pack_pair(int2 q) {
    return ((unsigned long long)(long long)q.x << kHShift) + (unsigned long long)(uint32_t)q.y;
}

// Merge the workgroup's LDS histogram into the node's histogram in HBM.
__device__ __forceinline__ void flush_tile(const unsigned long long *main_, const uint32_t *side, int ft, int B,
                                           int Bp, int64_t *out, int block) {
    for (int i = threadIdx.x; i < ft * B; i += block) {
        const int t = i / B, b = i - t * B;
        const int idx = t * Bp + b;
        const unsigned long long w = main_[idx];
        const uint32_t sc = side[idx];
        if (w == 0 && sc == 0) continue;
        const int64_t carry = (int64_t)(sc & 0xffffu);
        const int64_t wraps = (int64_t)((int32_t)sc >> 16);
        const int64_t g = ((int64_t)w >> kHShift) + wraps * ((int64_t)1 << (64 - kHShift)) - carry;
        const int64_t h = (int64_t)(w & kHMask) + (carry << kHShift);
        if (g != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i), (unsigned long long)g);
        if (h != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i + 1), (unsigned long long)h);
    }
}

// ---------------------------------------------------------------------------
// Any bit width (run-time), any feature tile, optional row-id list.
// lane = one row.  The row's slice of the bit stream is consumed in windows of
// four 32-bit words held in registers (five are loaded: an element may straddle
// into the next word); lanes start at different windows of a multi-window row.
// ---------------------------------------------------------------------------
template <bool LIST>
__global__ __launch_bounds__(kHistBlock) void hist_generic_kernel(
    const uint32_t *__restrict__ packed, int64_t n_words, int bits, uint32_t inv_bits, int64_t n, int F, int B,
    int Bp, uint32_t missing, const uint32_t *__restrict__ row_idx, const int2 *__restrict__ gq,
    int64_t *__restrict__ pool, const HistJob *__restrict__ jobs) {
    extern __shared__ unsigned long long lds[];
    const HistJob job = jobs[blockIdx.x];
    const int ft = (int)job.ft;
    unsigned long long *main_ = lds;
    uint32_t *side = (uint32_t *)(lds + ft * Bp);
    for (int i = threadIdx.x; i < ft * Bp; i += kHistBlock) {
        main_[i] = 0;
        side[i] = 0;
    }
    __syncthreads();

    const uint32_t mask = (1u << bits) - 1u;
    const int nbits = ft * bits;
    const int lane = threadIdx.x & 63;
    for (uint32_t i = threadIdx.x; i < job.n_rows; i += kHistBlock) {
        const uint64_t pos_in = (uint64_t)job.row_begin + i;
        const uint64_t r = LIST ? (uint64_t)row_idx[pos_in] : pos_in;
        if (r >= (uint64_t)n) continue;   // a malformed row id is skipped, never dereferenced
        const int2 q = gq[r];
        const unsigned long long addv = pack_pair(q);
        const uint32_t hq = (uint32_t)q.y;
        const uint64_t bit0 = (r * (uint64_t)F + job.f0) * (uint64_t)bits;
        const int64_t w0 = (int64_t)(bit0 >> 5);
        const int sh = (int)(bit0 & 31);
        const int nchunks = (sh + nbits + 127) >> 7;
        int c = (lane * nchunks) >> 6;   // lanes of a wave start at different windows
        for (int cc = 0; cc < nchunks; ++cc) {
            uint32_t w[5];
#pragma unroll
            for (int k = 0; k < 5; ++k) {
                const int64_t wi = w0 + 4 * c + k;
                w[k] = wi < n_words ? packed[wi] : 0u;
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
    flush_tile(main_, side, ft, B, Bp, pool + job.hist_off + (uint64_t)job.f0 * (uint64_t)B * 2u, kHistBlock);
}

// ---------------------------------------------------------------------------
// 8-bit symbols (one byte per element).  lane = one row; the row's bytes are
// loaded once into a 16-byte register window, realigned to the row's first byte
// with byte-funnel shifts, and ROTATED by a lane-dependent number of bytes, so
// that the sixteen unrolled extraction slots of a wave touch sixteen different
// features at the same time: rows that share the heavy bin of a skewed column do
// not meet at one LDS address in the same instruction.
// ---------------------------------------------------------------------------
template <bool LIST>
__global__ __launch_bounds__(kHistBlock) void hist_b8_kernel(
    const uint32_t *__restrict__ packed, int64_t n_words, int64_t n, int F, int B, int Bp, uint32_t missing,
    const uint32_t *__restrict__ row_idx, const int2 *__restrict__ gq, int64_t *__restrict__ pool,
    const HistJob *__restrict__ jobs) {
    extern __shared__ unsigned long long lds[];
    const HistJob job = jobs[blockIdx.x];
    const int ft = (int)job.ft;
    unsigned long long *main_ = lds;
    uint32_t *side = (uint32_t *)(lds + ft * Bp);
    for (int i = threadIdx.x; i < ft * Bp; i += kHistBlock) {
        main_[i] = 0;
        side[i] = 0;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int rot = lane & 15;                 // bytes this lane's window is rotated by
    const int nchunks = (ft + 15) >> 4;        // 16-byte windows per row slice (same for every lane)
    for (uint32_t i = threadIdx.x; i < job.n_rows; i += kHistBlock) {
        const uint64_t pos_in = (uint64_t)job.row_begin + i;
        const uint64_t r = LIST ? (uint64_t)row_idx[pos_in] : pos_in;
        if (r >= (uint64_t)n) continue;
        const int2 q = gq[r];
        const unsigned long long addv = pack_pair(q);
        const uint32_t hq = (uint32_t)q.y;
        const uint64_t byte0 = r * (uint64_t)F + job.f0;
        const int64_t w0 = (int64_t)(byte0 >> 2);
        const uint32_t a = (uint32_t)(byte0 & 3);
        int c = (lane * nchunks) >> 6;
        for (int cc = 0; cc < nchunks; ++cc) {
            uint32_t w[5];
#pragma unroll
            for (int k = 0; k < 5; ++k) {
                const int64_t wi = w0 + 4 * c + k;
                w[k] = wi < n_words ? packed[wi] : 0u;
            }
            // realign: W = bytes [16c, 16c+16) of the row slice
            uint32_t W[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) W[k] = __builtin_amdgcn_alignbyte(w[k + 1], w[k], a);
            // rotate the window by `rot` bytes: whole words first, then a byte funnel
            uint32_t X[4], Y[4], V[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) X[k] = (rot & 4) ? W[(k + 1) & 3] : W[k];
#pragma unroll
            for (int k = 0; k < 4; ++k) Y[k] = (rot & 8) ? X[(k + 2) & 3] : X[k];
#pragma unroll
            for (int k = 0; k < 4; ++k) V[k] = __builtin_amdgcn_alignbyte(Y[(k + 1) & 3], Y[k], (uint32_t)(rot & 3));
            const int nv = ft - 16 * c < 16 ? ft - 16 * c : 16;   // valid bytes in this window
            const int tbase = 16 * c;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int tt = (j + rot) & 15;   // slot j holds byte tt of the window
                const uint32_t s = (V[j >> 2] >> (8 * (j & 3))) & 0xffu;
                if (tt < nv && s != missing && s < (uint32_t)B)
                    pk_add(main_, side, (tbase + tt) * Bp + (int)s, addv, hq);
            }
            ++c;
            if (c == nchunks) c = 0;
        }
    }
    __syncthreads();
    flush_tile(main_, side, ft, B, Bp, pool + job.hist_off + (uint64_t)job.f0 * (uint64_t)B * 2u, kHistBlock);
}

inline int padded_bins(int B) { return B | 1; }   // odd stride: see the note on LDS banks above

}  // namespace

int gbt_hist_feature_tile(const gbt_ctx *ctx, int F, int B) {
    const size_t per_feature = (size_t)padded_bins(B) * 12;   // 8-byte word + 4-byte side counter per bin
    int ft = (int)(ctx->lds_per_block / per_feature);
    if (ft > F) ft = F;
    return ft;   // 0: one feature's bins do not fit in LDS
}

hipError_t gbt_launch_hist(gbt_ctx *ctx, const uint32_t *packed, int bits, int64_t n, int F, int B,
                           uint32_t missing, const uint32_t *row_idx, const int32_t *gq,
                           int64_t *hist_pool, const HistJob *jobs, int n_jobs, int max_ft) {
    if (n_jobs <= 0) return hipSuccess;
    const int Bp = padded_bins(B);
    const size_t lds = (size_t)max_ft * Bp * 12;
    const int64_t n_words = (n * (int64_t)F * bits + 31) / 32 + 1;
    const void *fn[4] = {(const void *)hist_generic_kernel<false>, (const void *)hist_generic_kernel<true>,
                         (const void *)hist_b8_kernel<false>, (const void *)hist_b8_kernel<true>};
    static size_t configured[4] = {0, 0, 0, 0};
    const int which = (bits == 8 ? 2 : 0) + (row_idx ? 1 : 0);
    if (lds > configured[which]) {
        hipError_t e = hipFuncSetAttribute(fn[which], hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured[which] = lds;
    }
    const int2 *g2 = (const int2 *)gq;
    if (bits == 8) {
        if (row_idx)
            hist_b8_kernel<true><<<n_jobs, kHistBlock, lds, ctx->stream>>>(packed, n_words, n, F, B, Bp, missing,
                                                                            row_idx, g2, hist_pool, jobs);
        else
            hist_b8_kernel<false><<<n_jobs, kHistBlock, lds, ctx->stream>>>(packed, n_words, n, F, B, Bp, missing,
                                                                             row_idx, g2, hist_pool, jobs);
    } else {
        const uint32_t inv_bits = (uint32_t)((((uint64_t)1 << 32) + (uint32_t)bits - 1) / (uint32_t)bits);
        if (row_idx)
            hist_generic_kernel<true><<<n_jobs, kHistBlock, lds, ctx->stream>>>(
                packed, n_words, bits, inv_bits, n, F, B, Bp, missing, row_idx, g2, hist_pool, jobs);
        else
            hist_generic_kernel<false><<<n_jobs, kHistBlock, lds, ctx->stream>>>(
                packed, n_words, bits, inv_bits, n, F, B, Bp, missing, row_idx, g2, hist_pool, jobs);
    }
    return hipGetLastError();
}
