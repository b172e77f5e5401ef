// BuildPartialHistograms (Alg. 1) for symbol widths other than 8 bits (compile-time width), any feature tile,
// rows given as a range or as a list of row ids.
//
// lane = one row.  A row's slice of the bit stream is consumed in register windows of E = min(128 / BITS, 32)
// whole elements: five words are loaded, funnel-shifted (v_alignbit) so that the window starts at bit 0, and
// every element is then cut out at a compile-time position.  The lanes of a wave start at different windows of
// a multi-window row, so that they work on different features.  What keeps the launch off the memory latency:
// the words of the NEXT window (of this row, or the first of the lane's next row) are requested before the
// current window is processed, the next row's gradient pair one row ahead, a listed row's id two rows ahead.
// A slot without a live feature, a missing symbol or a symbol >= B goes to a spare LDS word of the lane's own
// (conflict-free) instead of being predicated.
//
// Two forms of the accumulated LDS word, as in kernels_hist8.hip:
//   general     [ g : 34 | h : 30 ], returning atomics in groups of up to 16 whose returned words are tested
//               together for a carry out of h or a wrap of g, side counter per bin;
//   uniform h   [ g : 46 | rows : 18 ], non-returning atomics, nothing tested (at most 2^18 - 1 rows per job),
//               8 bytes of LDS per bin instead of 12.
#include "gbt_internal.h"
#include "hist_common.h"

namespace {

typedef unsigned long long __attribute__((address_space(3))) ldsw_u64;
typedef uint32_t __attribute__((address_space(3))) ldsw_u32;
__device__ __forceinline__ unsigned long long ldsw_add_rtn(uint32_t addr, unsigned long long v) {
    return __hip_atomic_fetch_add((ldsw_u64 *)(uintptr_t)addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void ldsw_add(uint32_t addr, unsigned long long v) {
    (void)__hip_atomic_fetch_add((ldsw_u64 *)(uintptr_t)addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

constexpr int kWRowsShift = 18;
constexpr uint32_t kWRowsMask = (1u << kWRowsShift) - 1u;

// One returned word: the exact carry test and the tight wrap test, then the bookkeeping (see hist_common.h).
// side_addr: LDS byte address of the bin's side counter.
__device__ __forceinline__ void pkw_check(uint32_t side_addr, unsigned long long old, unsigned long long addv, uint32_t hq) {
    uint32_t olo = (uint32_t)old, ohi = (uint32_t)(old >> 32);
    if ((pk_near_carry(old) < hq) | (pk_near_wrap(old, addv) < pk_reach(addv))) {
        asm volatile("" : "+v"(olo), "+v"(ohi));
        const uint32_t carry = ((olo & kHMask) + hq) >> kHShift;
        const uint32_t alo = (uint32_t)addv, ahi = (uint32_t)(addv >> 32);
        const uint32_t nlo = olo + alo;
        const uint32_t nhi = ohi + ahi + (nlo < olo ? 1u : 0u);
        const int32_t ovf = (int32_t)((ohi ^ nhi) & (ahi ^ nhi));
        const int32_t delta = ovf < 0 ? ((int32_t)nhi < 0 ? 1 : -1) : 0;
        if (carry != 0 || delta != 0)
            (void)__hip_atomic_fetch_add((ldsw_u32 *)(uintptr_t)side_addr, (uint32_t)(delta * 65536 + (int32_t)carry),
                                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

// CHK = false: every value the BITS can hold is a bin (B > 2^BITS - 1 and no missing symbol among them), so a
// symbol is only tested for lying in a live slot of the window.
template <int BITS, bool LIST, bool UNI, bool CHK>
__global__ __launch_bounds__(kHistBlock) void hist_bits_kernel(
    const uint32_t *__restrict__ packed, int64_t n_words, int64_t stride_bits, int64_t n, int B, int Bp,
    uint32_t missing, const uint32_t *__restrict__ row_idx, const int2 *__restrict__ gq,
    int64_t *__restrict__ pool, const HistJob *__restrict__ jobs, int32_t hq_uniform) {
    constexpr int E = (128 / BITS) < 32 ? (128 / BITS) : 32;   // elements per window
    constexpr int G = E < 16 ? E : 16;                         // atomics in flight per lane
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    extern __shared__ unsigned long long lds[];
    const HistJob job = jobs[blockIdx.x];
    const int ft = (int)job.ft;
    const int trash = ft * Bp;
    const int n_acc = trash + 64;   // + one spare word per lane
    unsigned long long *main_ = lds;
    uint32_t *side = (uint32_t *)(lds + n_acc);
    for (int i = threadIdx.x; i < n_acc; i += (int)blockDim.x) {
        main_[i] = 0;
        if (!UNI) side[i] = 0;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(ldsw_u64 *)main_;
    const uint32_t side_base = lds_base + 8u * (uint32_t)n_acc;
    const uint32_t my_trash = lds_base + 8u * (uint32_t)(trash + lane);
    const int nwin = (ft + E - 1) / E;
    const int c0 = (lane * nwin) >> 6;   // lanes of a wave start at different windows
    const uint32_t nrows = job.n_rows, step = blockDim.x;
    const uint64_t f0_bits = (uint64_t)job.f0 * BITS;

    auto row_id = [&](uint32_t i) __attribute__((always_inline)) -> uint64_t {
        const uint64_t pos = (uint64_t)job.row_begin + i;
        return LIST ? (uint64_t)row_idx[pos] : pos;
    };
    uint32_t wn[5], shn = 0;   // the window on its way
    auto issue = [&](uint64_t r, int c) __attribute__((always_inline)) {
        const uint64_t wb = r * (uint64_t)stride_bits + f0_bits + (uint64_t)(c * (E * BITS));
        const int64_t w0 = (int64_t)(wb >> 5);
        shn = (uint32_t)(wb & 31);
        // words past the end of the buffer hold no bit of this row: the last word is read instead
        const int64_t room = n_words - 1 - w0;
        const uint32_t room32 = room >= 4 ? 4u : (uint32_t)room;
        const uint32_t *p = packed + w0;
#pragma unroll
        for (int k = 0; k < 5; ++k) wn[k] = p[min((uint32_t)k, room32)];
    };

    uint32_t i = threadIdx.x;
    if (i < nrows) {
        uint64_t r = row_id(i);
        uint64_t r1 = i + step < nrows ? row_id(i + step) : 0;
        bool ok_row = r < (uint64_t)n;   // a malformed row id is skipped, never dereferenced
        int2 q = ok_row ? gq[r] : make_int2(0, 0);
        if (ok_row) issue(r, c0);
        for (;;) {
            const bool more = i + step < nrows;
            const uint64_t r2 = i + 2 * step < nrows ? row_id(i + 2 * step) : 0;
            const bool ok_next = more && r1 < (uint64_t)n;
            const int2 q1 = ok_next ? gq[r1] : make_int2(0, 0);
            const unsigned long long addv =
                UNI ? ((unsigned long long)(long long)q.x << kWRowsShift) + 1ull : pack_pair(q);
            const uint32_t hq = (uint32_t)q.y;
            int c = c0;
            for (int cc = 0; cc < nwin; ++cc) {
                uint32_t w[5];
#pragma unroll
                for (int k = 0; k < 5; ++k) w[k] = wn[k];
                const uint32_t sh = shn;
                const int c_next = c + 1 == nwin ? 0 : c + 1;
                if (cc + 1 < nwin) {
                    if (ok_row) issue(r, c_next);
                } else if (ok_next) {
                    issue(r1, c0);
                }
                if (ok_row) {
                    uint32_t W[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) W[k] = __builtin_amdgcn_alignbit(w[k + 1], w[k], sh);
                    const int tbase = c * E;
                    const uint32_t tb8 = lds_base + 8u * (uint32_t)(tbase * Bp);
#pragma unroll
                    for (int g0 = 0; g0 < E; g0 += G) {
                        uint32_t addr[G];
                        unsigned long long old[G];
#pragma unroll
                        for (int jj = 0; jj < G; ++jj) {
                            const int j = g0 + jj;
                            if (j < E) {
                                const int pos = j * BITS, wd = pos >> 5, off = pos & 31;
                                uint32_t sv;
                                if (off + BITS <= 32)
                                    sv = (W[wd] >> off) & MASK;
                                else
                                    sv = __builtin_amdgcn_alignbit(W[wd < 3 ? wd + 1 : 3], W[wd], (uint32_t)off) & MASK;
                                const bool ok = CHK ? (tbase + j < ft) & (sv != missing) & (sv < (uint32_t)B) : (tbase + j < ft);
                                addr[jj] = ok ? tb8 + 8u * (uint32_t)(j * Bp) + (sv << 3) : my_trash;
                                if (UNI) ldsw_add(addr[jj], addv);
                                else old[jj] = ldsw_add_rtn(addr[jj], addv);
                            }
                        }
                        if (!UNI) {
                            // the returned words of the group tested together: the smallest distance of any of them
                            // from an event decides whether the per-word bookkeeping runs at all
                            uint32_t near_carry = 0xffffffffu, near_wrap = 0xffffffffu;
#pragma unroll
                            for (int jj = 0; jj < G; ++jj)
                                if (g0 + jj < E) {
                                    near_carry = min(near_carry, pk_near_carry(old[jj]));
                                    near_wrap = min(near_wrap, pk_near_wrap(old[jj], addv));
                                }
                            if (near_carry < hq || near_wrap < pk_reach(addv)) {
#pragma unroll
                                for (int jj = 0; jj < G; ++jj)
                                    if (g0 + jj < E) pkw_check(side_base + ((addr[jj] - lds_base) >> 1), old[jj], addv, hq);
                            }
                        }
                    }
                }
                c = c_next;
            }
            if (!more) break;
            i += step;
            r = r1;
            r1 = r2;
            q = q1;
            ok_row = ok_next;
        }
    }
    __syncthreads();
    int64_t *out = pool + job.hist_off + (uint64_t)job.f0 * (uint64_t)B * 2u;
    const bool exclusive = job.pad0 == 1u;   // the only job of its (node, tile): plain stores, zeros included
    if (!UNI) {
        flush_tile(main_, side, ft, B, Bp, out, (int)blockDim.x, exclusive);
    } else {
        for (int k = threadIdx.x; k < ft * B; k += (int)blockDim.x) {
            const int t = k / B, b = k - t * B;
            const unsigned long long wv = main_[t * Bp + b];
            if (!exclusive && wv == 0) continue;
            const int64_t rows = (int64_t)(wv & kWRowsMask);
            const int64_t g = ((int64_t)wv - rows) >> kWRowsShift;
            const int64_t h = rows * hq_uniform;
            if (exclusive) {
                *(longlong2 *)(out + 2 * (int64_t)k) = make_longlong2(g, h);
            } else {
                if (g != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)k), (unsigned long long)g);
                if (h != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)k + 1), (unsigned long long)h);
            }
        }
    }
}

struct WArgs {
    hipStream_t s;
    int n_jobs, block;
    size_t lds;
    const uint32_t *packed;
    int64_t n_words, stride_bits, n;
    int B, Bp;
    uint32_t missing;
    const uint32_t *row_idx;
    const int2 *gq;
    int64_t *pool;
    const HistJob *jobs;
    int32_t hq_uniform;
};
template <int BITS, bool LIST, bool UNI, bool CHK>
hipError_t launch_w(const WArgs &a) {
    GbtLdsGuard lds_guard(a.lds);
    if (lds_guard.needed) {
        hipError_t e = hipFuncSetAttribute((const void *)hist_bits_kernel<BITS, LIST, UNI, CHK>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds);
        if (e != hipSuccess) return e;
    }
    hist_bits_kernel<BITS, LIST, UNI, CHK><<<a.n_jobs, a.block, a.lds, a.s>>>(a.packed, a.n_words, a.stride_bits, a.n, a.B, a.Bp,
                                                                          a.missing, a.row_idx, a.gq, a.pool, a.jobs,
                                                                          a.hq_uniform);
    return hipGetLastError();
}
template <int BITS, bool CHK>
hipError_t pick_w2(const WArgs &a, bool uni) {
    if (a.row_idx) return uni ? launch_w<BITS, true, true, CHK>(a) : launch_w<BITS, true, false, CHK>(a);
    return uni ? launch_w<BITS, false, true, CHK>(a) : launch_w<BITS, false, false, CHK>(a);
}
template <int BITS>
hipError_t pick_w(const WArgs &a, bool uni) {
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    const bool chk = a.missing <= MASK || (uint32_t)a.B <= MASK;   // some value of the field is not a bin
    return chk ? pick_w2<BITS, true>(a, uni) : pick_w2<BITS, false>(a, uni);
}
}  // namespace

int gbt_histw_max_rows(bool uniform_h) { return uniform_h ? (int)kWRowsMask : 1 << 21; }

hipError_t gbt_launch_histw(gbt_ctx *ctx, const uint32_t *packed, int bits, int64_t stride_bits, int64_t n_words,
                            int64_t n, int B, uint32_t missing, const uint32_t *row_idx, const int32_t *gq,
                            int64_t *hist_pool, const HistJob *jobs, int n_jobs, int max_ft, bool uniform_h,
                            int32_t hq_uniform) {
    if (n_jobs <= 0) return hipSuccess;
    const int Bp = padded_bins(B);
    const size_t lds = ((size_t)max_ft * Bp + 64) * (uniform_h ? 8 : 12);
    const WArgs a{ctx->stream, n_jobs, ctx->hist_block, lds, packed, n_words, stride_bits, n, B, Bp, missing, row_idx,
                  (const int2 *)gq, hist_pool, jobs, hq_uniform};
    switch (bits) {
        case 1: return pick_w<1>(a, uniform_h);
        case 2: return pick_w<2>(a, uniform_h);
        case 3: return pick_w<3>(a, uniform_h);
        case 4: return pick_w<4>(a, uniform_h);
        case 5: return pick_w<5>(a, uniform_h);
        case 6: return pick_w<6>(a, uniform_h);
        case 7: return pick_w<7>(a, uniform_h);
        case 9: return pick_w<9>(a, uniform_h);
        case 10: return pick_w<10>(a, uniform_h);
        case 11: return pick_w<11>(a, uniform_h);
        case 12: return pick_w<12>(a, uniform_h);
        case 13: return pick_w<13>(a, uniform_h);
        case 14: return pick_w<14>(a, uniform_h);
        case 15: return pick_w<15>(a, uniform_h);
        case 16: return pick_w<16>(a, uniform_h);
        default: return hipErrorInvalidValue;
    }
}
