// BuildPartialHistograms (Alg. 1; Sec. 2.1 "gradient summation into
// histograms") for gfx950.
//
// Each workgroup owns a private histogram of one feature tile in LDS
// (int64 fixed point, ds_add_u64), streams its share of the node's rows,
// and merges the non-zero bins into the node's histogram in HBM with 64-bit
// global atomics.  Integer sums make the result independent of the order in
// which workgroups and lanes arrive.
#include "gbt_internal.h"

namespace {

constexpr int kHistBlock = 1024;

__device__ inline void lds_add(int64_t *p, int64_t v) {
    atomicAdd((unsigned long long *)p, (unsigned long long)v);
}

// Generic kernel: any bit width, any feature tile, optional row-id list.
// lane = one row; the lane walks the tile's features starting at a
// lane-dependent rotation so that the 64 lanes of a wave are spread over the
// features (rows that share a heavy bin of one feature then do not all hit the
// same LDS address in the same instruction).
__global__ __launch_bounds__(kHistBlock) void hist_generic_kernel(
    const uint32_t *__restrict__ packed, int bits, int64_t n, int F, int B, uint32_t missing,
    const uint32_t *__restrict__ row_idx, const int2 *__restrict__ gq, int64_t *__restrict__ pool,
    const HistJob *__restrict__ jobs) {
    extern __shared__ int64_t lds[];
    const HistJob job = jobs[blockIdx.x];
    const int ft = (int)job.ft;
    const int n_acc = ft * B * 2;
    for (int i = threadIdx.x; i < n_acc; i += kHistBlock) lds[i] = 0;
    __syncthreads();

    const uint32_t mask = (1u << bits) - 1u;
    const int rot = (int)(threadIdx.x % (unsigned)ft);
    for (uint32_t i = threadIdx.x; i < job.n_rows; i += kHistBlock) {
        const uint64_t pos = (uint64_t)job.row_begin + i;
        const uint64_t r = row_idx ? (uint64_t)row_idx[pos] : pos;
        if (r >= (uint64_t)n) continue;   // a malformed row id is skipped, never dereferenced
        const int2 q = gq[r];
        const int64_t g = q.x, h = q.y;
        const uint64_t e0 = r * (uint64_t)F + job.f0;
        int t = rot;
        for (int k = 0; k < ft; ++k) {
            const uint64_t bp = (e0 + (uint64_t)t) * (uint64_t)bits;
            const uint32_t *w = packed + (bp >> 5);
            const uint64_t v = (uint64_t)w[0] | ((uint64_t)w[1] << 32);
            const uint32_t s = (uint32_t)(v >> (bp & 31)) & mask;
            if (s != missing && s < (uint32_t)B) {
                int64_t *a = lds + ((t * B + (int)s) << 1);
                lds_add(a, g);
                lds_add(a + 1, h);
            }
            ++t;
            if (t == ft) t = 0;
        }
    }
    __syncthreads();

    int64_t *out = pool + job.hist_off + (uint64_t)job.f0 * (uint64_t)B * 2u;
    for (int i = threadIdx.x; i < n_acc; i += kHistBlock) {
        const int64_t v = lds[i];
        if (v != 0) atomicAdd((unsigned long long *)(out + i), (unsigned long long)v);
    }
}

}  // namespace

int gbt_hist_feature_tile(const gbt_ctx *ctx, int F, int B) {
    size_t per_feature = (size_t)B * 16;
    int ft = (int)(ctx->lds_per_block / per_feature);
    if (ft > F) ft = F;
    return ft;   // 0: one feature's bins do not fit in LDS
}

hipError_t gbt_launch_hist(gbt_ctx *ctx, const uint32_t *packed, int bits, int64_t n, int F, int B,
                           uint32_t missing, const uint32_t *row_idx, const int32_t *gq,
                           int64_t *hist_pool, const HistJob *jobs, int n_jobs, int max_ft) {
    if (n_jobs <= 0) return hipSuccess;
    size_t lds = (size_t)max_ft * B * 16;
    static size_t configured = 0;
    if (lds > configured) {
        hipError_t e = hipFuncSetAttribute((const void *)hist_generic_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = lds;
    }
    hist_generic_kernel<<<n_jobs, kHistBlock, lds, ctx->stream>>>(packed, bits, n, F, B, missing, row_idx,
                                                                   (const int2 *)gq, hist_pool, jobs);
    return hipGetLastError();
}
