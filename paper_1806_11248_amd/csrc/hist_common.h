// Pieces shared by the histogram kernels (kernels_hist.hip, kernels_histw.hip): the packed (g, h) LDS word, the
// tests on the word an atomic returns, and the merge of a workgroup's LDS histogram into HBM.
#ifndef GBT_HIST_COMMON_H
#define GBT_HIST_COMMON_H
#include "gbt_internal.h"

namespace {

inline int padded_bins(int B) { return B | 1; }   // odd bin stride: equal bins of different features fall into different LDS banks

constexpr int kHistBlock = 1024;
__device__ __forceinline__ void pk_check(uint32_t *side, int idx, unsigned long long old,
                                         unsigned long long addv, uint32_t hq);

__device__ __forceinline__ void pk_add(unsigned long long *main_, uint32_t *side, int idx,
                                       unsigned long long addv, uint32_t hq) {
    const unsigned long long old = atomicAdd(&main_[idx], addv);
    pk_check(side, idx, old, addv, hq);
}

__device__ __forceinline__ unsigned long long pack_pair(int2 q) {
    return ((unsigned long long)(long long)q.x << kHShift) + (unsigned long long)(uint32_t)q.y;
}

// Merge the workgroup's LDS histogram into the node's histogram in HBM: two 64-bit global atomics per non-zero
// bin -- or, when this job is the only one of its (node, feature tile) (`exclusive`), plain 16-byte stores of
// every bin, zeros included: no atomics (the chip retires them slowly) and nothing to clear beforehand.
__device__ __forceinline__ void flush_tile(const unsigned long long *main_, const uint32_t *side, int ft, int B,
                                           int Bp, int64_t *out, int block, bool exclusive = false) {
    for (int i = threadIdx.x; i < ft * B; i += block) {
        const int t = i / B, b = i - t * B;
        const int idx = t * Bp + b;
        const unsigned long long w = main_[idx];
        const uint32_t sc = side[idx];
        if (!exclusive && w == 0 && sc == 0) continue;
        const int64_t carry = (int64_t)(sc & 0xffffu);
        const int64_t wraps = (int64_t)((int32_t)sc >> 16);
        const int64_t g = ((int64_t)w >> kHShift) + wraps * ((int64_t)1 << (64 - kHShift)) - carry;
        const int64_t h = (int64_t)(w & kHMask) + (carry << kHShift);
        if (exclusive) {
            *(longlong2 *)(out + 2 * (int64_t)i) = make_longlong2(g, h);
        } else {
            if (g != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i), (unsigned long long)g);
            if (h != 0) atomicAdd((unsigned long long *)(out + 2 * (int64_t)i + 1), (unsigned long long)h);
        }
    }
}

// The two quick tests on a returned word, as tight as the row's own pair allows (events are not
// rare enough for loose ones: a heavy bin sees a carry every few hundred adds, and with 64 lanes
// and 13 features some lane is near one most of the time):
//   carry  iff  h field + hq >= 2^30        iff  (~low word & 2^30-1) < hq          (exact)
//   wrap   only if the g field lies within |g| + 1 of the end it is moving towards.  In units of
//          four (the high word is the g field >> 2, signed): its distance from that end is
//          high ^ kind, kind = 0x7FFFFFFF going up, 0x80000000 going down, and the test is
//          distance < reach, reach = |g| / 4 rounded up, plus one for the carry that may come along.
// (everything is derived from the pair's own word where it is used, so that no register is held for it)
__device__ __forceinline__ uint32_t pk_near_carry(unsigned long long old) { return ~(uint32_t)old & kHMask; }
__device__ __forceinline__ uint32_t pk_near_wrap(unsigned long long old, unsigned long long addv) {
    const uint32_t down = (uint32_t)((int32_t)(addv >> 32) >> 31);   // 0 going up, all ones going down
    return (uint32_t)(old >> 32) ^ down ^ 0x7FFFFFFFu;
}
__device__ __forceinline__ uint32_t pk_reach(unsigned long long addv) {
    const uint32_t ahi = (uint32_t)(addv >> 32);   // floor(g / 4), signed
    return (ahi ^ (uint32_t)((int32_t)ahi >> 31)) + 2u;
}

__device__ __forceinline__ void pk_check(uint32_t *side, int idx, unsigned long long old,
                                         unsigned long long addv, uint32_t hq) {
    uint32_t olo = (uint32_t)old, ohi = (uint32_t)(old >> 32);
    const bool danger = (pk_near_carry(old) < hq) | (pk_near_wrap(old, addv) < pk_reach(addv));
    if (danger) {
        asm volatile("" : "+v"(olo), "+v"(ohi));   // keep the rare bookkeeping inside the branch
        const uint32_t carry = ((olo & kHMask) + hq) >> kHShift;
        const uint32_t alo = (uint32_t)addv, ahi = (uint32_t)(addv >> 32);
        const uint32_t nlo = olo + alo;
        const uint32_t nhi = ohi + ahi + (nlo < olo ? 1u : 0u);
        const int32_t ovf = (int32_t)((ohi ^ nhi) & (ahi ^ nhi));   // sign bit set: the g field wrapped
        const int32_t delta = ovf < 0 ? ((int32_t)nhi < 0 ? 1 : -1) : 0;
        if (carry != 0 || delta != 0) atomicAdd(&side[idx], (uint32_t)(delta * 65536 + (int32_t)carry));
    }
}

// The returned words of a group of atomics (the first `live` of G) tested together: the smallest
// distance of any of them from an event decides whether the per-word bookkeeping runs at all.
template <int G>
__device__ __forceinline__ void pk_check_group(uint32_t *side, const int (&idx)[G], const unsigned long long (&old)[G],
                                               int live, unsigned long long addv, uint32_t hq) {
    uint32_t near_carry = 0xffffffffu, near_wrap = 0xffffffffu;   // see pk_check for the two conditions
#pragma unroll
    for (int j = 0; j < G; ++j)
        if (j < live) {
            near_carry = min(near_carry, pk_near_carry(old[j]));
            near_wrap = min(near_wrap, pk_near_wrap(old[j], addv));
        }
    if (near_carry < hq || near_wrap < pk_reach(addv)) {
#pragma unroll
        for (int j = 0; j < G; ++j)
            if (j < live) pk_check(side, idx[j], old[j], addv, hq);
    }
}

}  // namespace
#endif
