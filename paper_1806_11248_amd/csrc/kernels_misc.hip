// Small streaming kernels around the tree builder: fills, fixed-point
// conversion of the gradient pairs, node totals, gradients (Eq. 1-2), sibling
// subtraction, export, bit packing (Sec. 2.2), prediction (Sec. 2.4) and the
// final leaf gather.  All are bandwidth-trivial next to the histogram kernel.
#include "gbt_internal.h"

namespace {

constexpr int kBlock = 256;

inline int grid_for(int64_t count, int per_block, int cap = 1 << 20) {
    int64_t g = (count + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

__global__ void fill_u64_kernel(uint64_t *p, uint64_t v, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

__global__ void iota_u32_kernel(uint32_t *p, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = (uint32_t)i;
}

// max |g| and max |h| as raw float bits (non-negative floats order like their
// bit patterns; NaN sorts above +inf, so a non-finite input is detected).
// out2[2] becomes non-zero if any h is negative.
// A thread takes kStreamBatch 16-byte loads (two pairs each) that are all issued before the
// first is used, so that enough bytes are in flight to cover the HBM latency.
constexpr int kStreamBatch = 4;
// The pointers must be 16-byte aligned; `head` pairs (0 or 1) in front of them are taken singly,
// which is how a caller's pointer that is only 8-byte aligned is served.
// out2[3] receives ~(smallest |h| as bits), so that a zero-filled word is the neutral start of an atomicMax
__global__ __launch_bounds__(kBlock) void absmax_kernel(const float2 *gp, int64_t n, int head, uint32_t *out2) {
    uint32_t mg = 0, mh = 0, neg = 0, lh = 0xffffffffu;
    if (head && blockIdx.x == 0 && threadIdx.x == 1) {
        const float2 v = gp[-1];
        mg = __float_as_uint(v.x) & 0x7fffffffu;
        mh = __float_as_uint(v.y) & 0x7fffffffu;
        lh = mh;
        neg = v.y < 0.0f ? 1u : 0u;
    }
    const float4 *gp4 = (const float4 *)gp;
    const int64_t n4 = n >> 1;   // whole 16-byte pieces
    auto take = [&](const float4 &v) {
        const uint32_t a0 = __float_as_uint(v.x) & 0x7fffffffu, b0 = __float_as_uint(v.y) & 0x7fffffffu;
        const uint32_t a1 = __float_as_uint(v.z) & 0x7fffffffu, b1 = __float_as_uint(v.w) & 0x7fffffffu;
        mg = max(mg, max(a0, a1));
        mh = max(mh, max(b0, b1));
        lh = min(lh, min(b0, b1));
        neg |= (v.y < 0.0f || v.w < 0.0f) ? 1u : 0u;
    };
    // a workgroup takes contiguous chunks of kStreamBatch * kBlock pieces; whole chunks need no conditional load
    const int64_t chunk = (int64_t)kStreamBatch * kBlock, n_whole = n4 / chunk;
    for (int64_t c = blockIdx.x; c < n_whole; c += gridDim.x) {
        float4 v[kStreamBatch];
#pragma unroll
        for (int k = 0; k < kStreamBatch; ++k) v[k] = gp4[c * chunk + k * kBlock + threadIdx.x];
#pragma unroll
        for (int k = 0; k < kStreamBatch; ++k) take(v[k]);
    }
    for (int64_t i = n_whole * chunk + (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (int64_t)gridDim.x * kBlock)
        take(gp4[i]);
    if ((n & 1) && blockIdx.x == 0 && threadIdx.x == 0) {   // the odd last pair
        const float2 v = gp[n - 1];
        mg = max(mg, __float_as_uint(v.x) & 0x7fffffffu);
        mh = max(mh, __float_as_uint(v.y) & 0x7fffffffu);
        lh = min(lh, __float_as_uint(v.y) & 0x7fffffffu);
        neg |= v.y < 0.0f ? 1u : 0u;
    }
    for (int o = 32; o > 0; o >>= 1) {
        uint32_t a = __shfl_xor(mg, o), b = __shfl_xor(mh, o), c = __shfl_xor(lh, o);
        mg = a > mg ? a : mg;
        mh = b > mh ? b : mh;
        lh = c < lh ? c : lh;
        neg |= __shfl_xor(neg, o);
    }
    // one set of atomics per workgroup: atomics on one address run one after the other
    __shared__ uint32_t red[4][kBlock / 64];
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = mg;
        red[1][threadIdx.x >> 6] = mh;
        red[2][threadIdx.x >> 6] = neg;
        red[3][threadIdx.x >> 6] = lh;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / 64; ++w) {
            mg = max(mg, red[0][w]);
            mh = max(mh, red[1][w]);
            neg |= red[2][w];
            lh = min(lh, red[3][w]);
        }
        atomicMax(&out2[0], mg);
        atomicMax(&out2[1], mh);
        if (neg) atomicOr(&out2[2], 1u);
        atomicMax(&out2[3], ~lh);
    }
}

// Adds the workgroup's (g, h) to sums[0..1] with one pair of atomics (every thread must call).
__device__ inline void block_add_i64x2(int64_t g, int64_t h, int64_t *sums);

__device__ inline int64_t wave_sum_i64(int64_t v) {
    for (int o = 32; o > 0; o >>= 1) {
        int lo = __shfl_xor((int)(v & 0xffffffff), o);
        int hi = __shfl_xor((int)(v >> 32), o);
        v += (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
    }
    return v;
}

// gp and gq must be 16-byte aligned; `head` pairs (0 or 1) in front of BOTH are taken singly.
__device__ inline void block_add_i64x2(int64_t g, int64_t h, int64_t *sums) {
    __shared__ int64_t red[2][kBlock / 64];
    g = wave_sum_i64(g);
    h = wave_sum_i64(h);
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = g;
        red[1][threadIdx.x >> 6] = h;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w) {
            g += red[0][w];
            h += red[1][w];
        }
        atomicAdd((unsigned long long *)&sums[0], (unsigned long long)g);
        atomicAdd((unsigned long long *)&sums[1], (unsigned long long)h);
    }
}

__global__ __launch_bounds__(kBlock) void to_fixed_kernel(const float2 *gp, int64_t n, int head, double sg, double sh,
                                                          int2 *gq, int64_t *sums) {
    int64_t g = 0, h = 0;
    if (head && blockIdx.x == 0 && threadIdx.x == 1) {
        const float2 v = gp[-1];
        int2 q;
        q.x = __double2int_rn((double)v.x * sg);
        q.y = __double2int_rn((double)v.y * sh);
        gq[-1] = q;
        g = q.x;
        h = q.y;
    }
    const float4 *gp4 = (const float4 *)gp;
    int4 *gq4 = (int4 *)gq;
    const int64_t n4 = n >> 1;   // whole 16-byte pieces (two pairs)
    auto take = [&](int64_t at, const float4 &v) {
        int4 q;
        q.x = __double2int_rn((double)v.x * sg);
        q.y = __double2int_rn((double)v.y * sh);
        q.z = __double2int_rn((double)v.z * sg);
        q.w = __double2int_rn((double)v.w * sh);
        gq4[at] = q;
        g += (int64_t)q.x + q.z;
        h += (int64_t)q.y + q.w;
    };
    const int64_t chunk = (int64_t)kStreamBatch * kBlock, n_whole = n4 / chunk;
    for (int64_t c = blockIdx.x; c < n_whole; c += gridDim.x) {
        float4 v[kStreamBatch];
#pragma unroll
        for (int k = 0; k < kStreamBatch; ++k) v[k] = gp4[c * chunk + k * kBlock + threadIdx.x];
#pragma unroll
        for (int k = 0; k < kStreamBatch; ++k) take(c * chunk + k * kBlock + threadIdx.x, v[k]);
    }
    for (int64_t i = n_whole * chunk + (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (int64_t)gridDim.x * kBlock)
        take(i, gp4[i]);
    if ((n & 1) && blockIdx.x == 0 && threadIdx.x == 0) {   // the odd last pair
        const float2 v = gp[n - 1];
        int2 q;
        q.x = __double2int_rn((double)v.x * sg);
        q.y = __double2int_rn((double)v.y * sh);
        gq[n - 1] = q;
        g += q.x;
        h += q.y;
    }
    if (sums) {
        block_add_i64x2(g, h, sums);
    }
}

// One pair per load: for a source and a destination whose 16-byte alignments differ.
__global__ __launch_bounds__(kBlock) void to_fixed_pairs_kernel(const float2 *gp, int64_t n, double sg, double sh,
                                                                int2 *gq, int64_t *sums) {
    int64_t g = 0, h = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const float2 v = gp[i];
        int2 q;
        q.x = __double2int_rn((double)v.x * sg);
        q.y = __double2int_rn((double)v.y * sh);
        gq[i] = q;
        g += q.x;
        h += q.y;
    }
    if (sums) {
        block_add_i64x2(g, h, sums);
    }
}

__global__ __launch_bounds__(kBlock) void sum_gq_kernel(const int2 *gq, const uint32_t *row_idx, int64_t n_rows, int64_t *out2) {
    int64_t g = 0, h = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_rows;
         i += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = row_idx ? (int64_t)row_idx[i] : i;
        int2 q = gq[r];
        g += q.x;
        h += q.y;
    }
    block_add_i64x2(g, h, out2);
}

// Eq. 1 and Eq. 2 (logistic) and the squared-error pair, one instance per
// thread.  Evaluated in fp64 and rounded once so that the fp32 pair does not
// depend on a fast-math exp.
__device__ __forceinline__ float2 gradient_pair(int objective, float margin, float label) {
    double m = margin, y = label, g, h;
    if (objective == GBT_OBJ_LOGISTIC) {
        double p = 1.0 / (1.0 + exp(-m));
        g = p - y;
        h = p * (1.0 - p);
    } else {
        g = m - y;
        h = 1.0;
    }
    return make_float2((float)g, (float)h);
}
// A thread takes four consecutive instances at a time (16-byte loads, two 16-byte stores) where the three
// arrays are 16-byte aligned; the launcher says so.  The last n mod 4 instances are taken singly.
// bounds (may be NULL): the four words absmax_kernel leaves for these pairs (largest |g| and |h| as bits, a flag for a
// negative h, ~smallest |h|), reduced on the way so that the pairs need not be read again for them.
__global__ __launch_bounds__(kBlock) void gradients_kernel(int objective, const float *__restrict__ margin,
                                                           const float *__restrict__ label, int64_t n,
                                                           float2 *__restrict__ gp, int vec, uint32_t *bounds, int nt) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, nthreads = (int64_t)gridDim.x * blockDim.x;
    uint32_t mg = 0, mh = 0, neg = 0, lh = 0xffffffffu;
    auto note = [&](const float2 &v) {
        const uint32_t a = __float_as_uint(v.x) & 0x7fffffffu, b = __float_as_uint(v.y) & 0x7fffffffu;
        mg = max(mg, a);
        mh = max(mh, b);
        lh = min(lh, b);
        neg |= v.y < 0.0f ? 1u : 0u;
    };
    int64_t done = 0;
    if (vec) {
        const int64_t n4 = n >> 2;
        const float4 *m4 = (const float4 *)margin, *y4 = (const float4 *)label;
        float4 *o4 = (float4 *)gp;
        for (int64_t i = tid; i < n4; i += nthreads) {
            typedef float f4v __attribute__((ext_vector_type(4)));
            const float4 m = m4[i], y = y4[i];
            const float2 a = gradient_pair(objective, m.x, y.x), b = gradient_pair(objective, m.y, y.y);
            const float2 c = gradient_pair(objective, m.z, y.z), d = gradient_pair(objective, m.w, y.w);
            // nt: non-temporal stores.  Written the ordinary way, the last few hundred MB of an array much larger than
            // the memory-side cache are still waiting there when the kernel ends, and their write-back then competes
            // with whatever streams next (measured: the root histogram launch right behind takes 0.52 ms instead of
            // 0.48 on 115M rows).  Pairs that fit the cache are better left in it for the launch that reads them.
            if (nt) {
                const f4v s0 = {a.x, a.y, b.x, b.y}, s1 = {c.x, c.y, d.x, d.y};
                __builtin_nontemporal_store(s0, (f4v *)&o4[2 * i]);
                __builtin_nontemporal_store(s1, (f4v *)&o4[2 * i + 1]);
            } else {
                o4[2 * i] = make_float4(a.x, a.y, b.x, b.y);
                o4[2 * i + 1] = make_float4(c.x, c.y, d.x, d.y);
            }
            note(a);
            note(b);
            note(c);
            note(d);
        }
        done = n4 << 2;
    }
    for (int64_t i = done + tid; i < n; i += nthreads) {
        const float2 v = gradient_pair(objective, margin[i], label[i]);
        gp[i] = v;
        note(v);
    }
    if (!bounds) return;
    for (int o = 32; o > 0; o >>= 1) {
        uint32_t a = __shfl_xor(mg, o), b = __shfl_xor(mh, o), c = __shfl_xor(lh, o);
        mg = a > mg ? a : mg;
        mh = b > mh ? b : mh;
        lh = c < lh ? c : lh;
        neg |= __shfl_xor(neg, o);
    }
    __shared__ uint32_t red[4][kBlock / 64];   // one set of atomics per workgroup
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = mg;
        red[1][threadIdx.x >> 6] = mh;
        red[2][threadIdx.x >> 6] = neg;
        red[3][threadIdx.x >> 6] = lh;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / 64; ++w) {
            mg = max(mg, red[0][w]);
            mh = max(mh, red[1][w]);
            neg |= red[2][w];
            lh = min(lh, red[3][w]);
        }
        // (a word per 128-byte line: atomics on words of one line take turns like atomics on one address)
        atomicMax(&bounds[0 * kBoundsStride], mg);
        atomicMax(&bounds[1 * kBoundsStride], mh);
        if (neg) atomicOr(&bounds[2 * kBoundsStride], 1u);
        atomicMax(&bounds[3 * kBoundsStride], ~lh);
    }
}


__global__ void subtract_one_kernel(const int64_t *p, const int64_t *c, int64_t *o, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)gridDim.x * blockDim.x)
        o[i] = p[i] - c[i];
}

__global__ void export_kernel(const int64_t *hist, int64_t count, double inv_sg, double inv_sh,
                              double *out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)gridDim.x * blockDim.x)
        out[i] = (double)hist[i] * ((i & 1) ? inv_sh : inv_sg);
}

// Sec. 2.2: one thread assembles one 32-bit word of the bit stream from the
// elements that overlap it (no atomics; the trailing pad word comes out zero).
__global__ void compress_kernel(const uint16_t *sym, int64_t n_elems, int bits, uint32_t *packed,
                                int64_t n_words) {
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < n_words;
         w += (int64_t)gridDim.x * blockDim.x) {
        int64_t bit0 = w * 32;
        int64_t e = bit0 / bits;
        uint32_t word = 0;
        for (; e < n_elems; ++e) {
            int64_t pos = e * bits - bit0;   // may be negative for the first element
            if (pos >= 32) break;
            uint32_t s = sym[e];
            word |= pos >= 0 ? (s << pos) : (s >> (-pos));
        }
        packed[w] = word;
    }
}

__device__ inline uint32_t load_symbol(const uint32_t *packed, uint64_t elem, int bits, uint32_t mask) {
    uint64_t bp = elem * (uint64_t)bits;
    const uint32_t *w = packed + (bp >> 5);
    uint64_t v = (uint64_t)w[0] | ((uint64_t)w[1] << 32);
    return (uint32_t)(v >> (bp & 31)) & mask;
}

// Sec. 2.4: one instance per thread, trees in order, walking from the root.
__global__ void predict_kernel(const char *ws, const DevTree *trees, int n_trees,
                               const uint32_t *packed, int bits, uint32_t missing, const float *X,
                               int64_t n, int F, double eta, float *margin, int32_t *leaf_out) {
    const uint32_t mask = (1u << bits) - 1u;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n;
         r += (int64_t)gridDim.x * blockDim.x) {
        double m = margin ? margin[r] : 0.0;
        for (int t = 0; t < n_trees; ++t) {
            DevTree T = trees[t];
            const int32_t *feature = (const int32_t *)(ws + T.feature);
            const int32_t *bin = (const int32_t *)(ws + T.bin);
            const int32_t *dl = (const int32_t *)(ws + T.default_left);
            const int32_t *left = (const int32_t *)(ws + T.left);
            const int32_t *right = (const int32_t *)(ws + T.right);
            const float *thr = (const float *)(ws + T.threshold);
            const double *weight = (const double *)(ws + T.weight);
            int node = 0;
            // a well-formed tree ends in fewer than n_nodes steps; the bound keeps a
            // malformed one from spinning
            for (int step = 0; step < T.n_nodes; ++step) {
                int f = feature[node];
                if (f < 0) break;
                bool go_left;
                if (packed) {
                    uint32_t s = load_symbol(packed, (uint64_t)r * F + f, bits, mask);
                    go_left = (s == missing) ? (dl[node] != 0) : ((int)s <= bin[node]);
                } else {
                    float x = X[r * F + f];
                    go_left = (x != x) ? (dl[node] != 0) : (x < thr[node]);
                }
                node = go_left ? left[node] : right[node];
            }
            m = (double)(float)(m + eta * weight[node]);
            if (leaf_out) leaf_out[r] = node;   // leaf mode: the caller passes one tree
        }
        if (margin) margin[r] = (float)m;
    }
}

// Same walk with the tree's nodes staged in LDS (32 bytes per node): the per-level
// node fetches then cost an LDS read instead of a dependent global load.
struct LdsNode {
    int32_t feature, bin, left, right;
    float thr;
    int32_t dl;
    double weight;
};
__global__ __launch_bounds__(256) void predict_lds_kernel(const char *ws, const DevTree *trees, int n_trees,
                                                          const uint32_t *packed, int bits, uint32_t missing,
                                                          const float *X, int64_t n, int F, double eta,
                                                          float *margin, int rows_per_block, int32_t *leaf_out) {
    extern __shared__ LdsNode nodes[];
    const uint32_t mask = (1u << bits) - 1u;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
    for (int t = 0; t < n_trees; ++t) {
        const DevTree T = trees[t];
        __syncthreads();   // the previous tree's walks are done
        for (int i = threadIdx.x; i < T.n_nodes; i += 256) {
            LdsNode nd;
            nd.feature = ((const int32_t *)(ws + T.feature))[i];
            nd.bin = ((const int32_t *)(ws + T.bin))[i];
            nd.left = ((const int32_t *)(ws + T.left))[i];
            nd.right = ((const int32_t *)(ws + T.right))[i];
            nd.thr = ((const float *)(ws + T.threshold))[i];
            nd.dl = ((const int32_t *)(ws + T.default_left))[i];
            nd.weight = ((const double *)(ws + T.weight))[i];
            nodes[i] = nd;
        }
        __syncthreads();
        for (int64_t r = r0 + threadIdx.x; r < r1; r += 256) {
            const uint64_t rowbit = (uint64_t)r * (uint64_t)F * (uint64_t)bits;
            int node = 0;
            for (int step = 0; step < T.n_nodes; ++step) {
                const LdsNode nd = nodes[node];
                if (nd.feature < 0) break;
                bool go_left;
                if (packed) {
                    const uint64_t bp = rowbit + (uint64_t)nd.feature * (uint64_t)bits;
                    const uint32_t *w = packed + (bp >> 5);
                    const uint32_t sh = (uint32_t)(bp & 31);
                    uint32_t v = w[0] >> sh;
                    if (sh + (uint32_t)bits > 32u) v |= w[1] << (32u - sh);
                    const uint32_t s = v & mask;
                    go_left = (s == missing) ? (nd.dl != 0) : ((int)s <= nd.bin);
                } else {
                    const float x = X[r * F + nd.feature];
                    go_left = (x != x) ? (nd.dl != 0) : (x < nd.thr);
                }
                node = go_left ? nd.left : nd.right;
            }
            if (leaf_out) leaf_out[r] = node;
            else margin[r] = (float)((double)margin[r] + eta * nodes[node].weight);
        }
    }
}

// Rows of at most 128 bits: the whole row is fetched once (five words, funnel-shifted to the
// row's first bit) and every level's symbol is cut out of registers, so a tree walk costs one
// row fetch instead of one dependent gather per level.
__device__ __forceinline__ uint32_t pick4(const uint32_t (&W)[4], int i) {
    return i == 0 ? W[0] : (i == 1 ? W[1] : (i == 2 ? W[2] : W[3]));
}
// Nodes are staged as 8 bytes: x = left child id | default_left << 31 (the right child is
// left + 1, which the caller has checked), y = feature << 12 | bin.  A leaf is staged as a
// node that sends every row to itself (left = own id, default left, bin 0xfff >= any symbol),
// so every row takes exactly T.pad steps (the tree's depth) and the walks of the kPredRows rows
// a thread handles at once run side by side instead of one divergent loop after the other.
constexpr int kPredRows = 4;
__global__ __launch_bounds__(256) void predict_window_kernel(const char *ws, const DevTree *trees, int n_trees,
                                                             const uint32_t *packed, int64_t n_words, int bits,
                                                             uint32_t missing, int64_t n, int F, double eta,
                                                             float *margin, int rows_per_block, int max_nodes,
                                                             int32_t *leaf_out) {
    extern __shared__ uint2 cnodes[];
    double *lweight = (double *)(cnodes + max_nodes);
    const uint32_t mask = (1u << bits) - 1u;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
    for (int t = 0; t < n_trees; ++t) {
        const DevTree T = trees[t];
        __syncthreads();
        for (int i = threadIdx.x; i < T.n_nodes; i += 256) {
            const int32_t f = ((const int32_t *)(ws + T.feature))[i];
            uint2 c;
            if (f < 0) {
                c.x = (uint32_t)i | 0x80000000u;
                c.y = 0xfffu;
            } else {
                c.x = (uint32_t)((const int32_t *)(ws + T.left))[i] |
                      (((const int32_t *)(ws + T.default_left))[i] ? 0x80000000u : 0u);
                c.y = ((uint32_t)f << 12) | (uint32_t)((const int32_t *)(ws + T.bin))[i];
            }
            cnodes[i] = c;
            lweight[i] = ((const double *)(ws + T.weight))[i];
        }
        __syncthreads();
        const int depth = T.pad;
        for (int64_t rb = r0 + threadIdx.x; rb < r1; rb += 256 * kPredRows) {
            uint32_t W[kPredRows][4];
            float m[kPredRows];
#pragma unroll
            for (int q = 0; q < kPredRows; ++q) {
                // rows past the end repeat the last row (their result is dropped)
                const int64_t r = rb + 256 * q < r1 ? rb + 256 * q : r1 - 1;
                const uint64_t rowbit = (uint64_t)r * (uint64_t)F * (uint64_t)bits;
                const int64_t w0 = (int64_t)(rowbit >> 5);
                const uint32_t sh = (uint32_t)(rowbit & 31);
                uint32_t w[5];
#pragma unroll
                for (int k = 0; k < 5; ++k) w[k] = packed[w0 + k < n_words ? w0 + k : n_words - 1];
#pragma unroll
                for (int k = 0; k < 4; ++k) W[q][k] = __builtin_amdgcn_alignbit(w[k + 1], w[k], sh);
                m[q] = leaf_out ? 0.f : margin[r];
            }
            uint32_t node[kPredRows];
#pragma unroll
            for (int q = 0; q < kPredRows; ++q) node[q] = 0;
            for (int step = 0; step < depth; ++step) {
#pragma unroll
                for (int q = 0; q < kPredRows; ++q) {
                    const uint2 c = cnodes[node[q]];
                    const int pos = (int)(c.y >> 12) * bits, wd = pos >> 5;
                    const uint32_t lo = pick4(W[q], wd), hi = wd < 3 ? pick4(W[q], wd + 1) : 0u;
                    const uint32_t s = __builtin_amdgcn_alignbit(hi, lo, (uint32_t)(pos & 31)) & mask;
                    const bool go_left = (s == missing) ? (c.x >> 31) != 0 : (s <= (c.y & 0xfffu));
                    node[q] = (c.x & 0x7fffffffu) + (go_left ? 0u : 1u);
                }
            }
#pragma unroll
            for (int q = 0; q < kPredRows; ++q) {
                const int64_t r = rb + 256 * q;
                if (r < r1) {
                    if (leaf_out) leaf_out[r] = (int32_t)node[q];
                    else margin[r] = (float)((double)m[q] + eta * lweight[node[q]]);
                }
            }
        }
    }
}

// Rows wider than the register window, up to kStagedRowBits bits: a wave's 64 consecutive rows are one contiguous
// piece of the bit stream, which the wave fetches linearly into an LDS window of its own; every level's symbol is
// then cut out of LDS instead of being gathered from memory, one dependent access per level.  Nodes as in
// predict_window_kernel.  wave_words: words of a wave's window (64 rows and one word of slack).
constexpr int kStagedRowBits = 1024;
__global__ __launch_bounds__(256) void predict_staged_kernel(const char *ws, const DevTree *trees, int n_trees,
                                                             const uint32_t *packed, int64_t n_words, int bits,
                                                             uint32_t missing, int64_t n, int F, double eta,
                                                             float *margin, int rows_per_block, int max_nodes,
                                                             int32_t *leaf_out, int wave_words) {
    extern __shared__ uint2 cnodes[];
    double *lweight = (double *)(cnodes + max_nodes);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t *st = (uint32_t *)(lweight + max_nodes) + (size_t)wave * wave_words;
    const uint32_t mask = (1u << bits) - 1u;
    const uint64_t stride_bits = (uint64_t)F * (uint64_t)bits;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
    for (int t = 0; t < n_trees; ++t) {
        const DevTree T = trees[t];
        __syncthreads();
        for (int i = threadIdx.x; i < T.n_nodes; i += 256) {
            const int32_t f = ((const int32_t *)(ws + T.feature))[i];
            uint2 c;
            if (f < 0) {
                c.x = (uint32_t)i | 0x80000000u;
                c.y = 0xfffu;
            } else {
                c.x = (uint32_t)((const int32_t *)(ws + T.left))[i] |
                      (((const int32_t *)(ws + T.default_left))[i] ? 0x80000000u : 0u);
                c.y = ((uint32_t)f << 12) | (uint32_t)((const int32_t *)(ws + T.bin))[i];
            }
            cnodes[i] = c;
            lweight[i] = ((const double *)(ws + T.weight))[i];
        }
        __syncthreads();
        const int depth = T.pad;
        for (int64_t rw = r0 + (int64_t)wave * 64; rw < r1; rw += 256) {   // rw: the wave's first row
            const int64_t rend = rw + 64 < r1 ? rw + 64 : r1;
            const uint64_t bit0 = (uint64_t)rw * stride_bits, bit1 = (uint64_t)rend * stride_bits;
            const int64_t word0 = (int64_t)(bit0 >> 5);
            const uint32_t nw = (uint32_t)(((bit1 + 31) >> 5) - (uint64_t)word0) + 1u;   // + the word a last symbol may reach into
            for (uint32_t w = lane; w < nw; w += 64) st[w] = packed[word0 + w < n_words ? word0 + w : n_words - 1];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int64_t r = rw + lane;
            if (r < r1) {
                const uint32_t rowbit = (uint32_t)((uint64_t)r * stride_bits - ((uint64_t)word0 << 5));
                uint32_t node = 0;
                for (int step = 0; step < depth; ++step) {
                    const uint2 c = cnodes[node];
                    const uint32_t pos = rowbit + (c.y >> 12) * (uint32_t)bits;
                    const uint32_t lo = st[pos >> 5], hi = st[(pos >> 5) + 1];
                    const uint32_t sy = __builtin_amdgcn_alignbit(hi, lo, pos & 31u) & mask;
                    const bool go_left = (sy == missing) ? (c.x >> 31) != 0 : (sy <= (c.y & 0xfffu));
                    node = (c.x & 0x7fffffffu) + (go_left ? 0u : 1u);
                }
                if (leaf_out) leaf_out[r] = (int32_t)node;
                else margin[r] = (float)((double)margin[r] + eta * lweight[node]);
            }
            __builtin_amdgcn_wave_barrier();   // the window is refilled only after every lane has left it
        }
    }
}

// The same walk for 8-bit symbols (rows of at most 16 bytes, any byte alignment): a node is staged
// as a v_perm selector that cuts its feature's byte out of one half of the row, so a step is two
// permutes and a handful of compares.
//   y = 0x0C0C0C00 | (feature & 7)                       (selector: byte -> bits 0..7, zeros above)
//   x = left child id (20 bits) | bin << 20 | (feature >= 8) << 28 | default_left << 29
// A leaf is staged as (own id, bin 255, feature 0, default left): every row stays on it.
// MISS: the matrix has a missing symbol (it is < 256).
// A workgroup takes blocks of rows_per_block rows, blockIdx.x, blockIdx.x + gridDim.x, ...
// node_rows (may be NULL; one tree only): the rows that end in each node are counted, per workgroup in LDS and
// then into node_rows[node * kNodeRowsStride] (one counter per 128-byte line: atomics on one line take turns).
// margin_src: where a row's margin is read from (margin itself, or with one tree another array: out = src + step).
template <bool MISS>
__global__ __launch_bounds__(256) void predict_b8_kernel(const char *ws, const DevTree *trees, int n_trees,
                                                         const uint32_t *packed, int64_t n_words, uint32_t missing,
                                                         int64_t n, int F, double eta, float *margin,
                                                         int rows_per_block, int max_nodes, int32_t *leaf_out,
                                                         uint32_t *node_rows, const float *margin_src) {
    extern __shared__ uint2 cnodes[];
    double *lweight = (double *)(cnodes + max_nodes);
    uint32_t *lcount = (uint32_t *)(lweight + max_nodes);   // only there when node_rows is given
    if (node_rows)
        for (int i = threadIdx.x; i < max_nodes; i += 256) lcount[i] = 0;
    const int64_t n_blocks = (n + rows_per_block - 1) / rows_per_block;
    for (int t = 0; t < n_trees; ++t) {
        const DevTree T = trees[t];
        __syncthreads();
        for (int i = threadIdx.x; i < T.n_nodes; i += 256) {
            const int32_t f = ((const int32_t *)(ws + T.feature))[i];
            uint2 c;
            if (f < 0) {
                c.x = (uint32_t)i | (255u << 20) | (1u << 29);
                c.y = 0x0C0C0C00u;
            } else {
                const int32_t bin = ((const int32_t *)(ws + T.bin))[i];   // a bin >= 255 admits every symbol
                c.x = (uint32_t)((const int32_t *)(ws + T.left))[i] |
                      ((uint32_t)(bin < 255 ? bin : 255) << 20) | ((uint32_t)((f >> 3) & 1) << 28) |
                      (((const int32_t *)(ws + T.default_left))[i] ? (1u << 29) : 0u);
                c.y = 0x0C0C0C00u | (uint32_t)(f & 7);
            }
            cnodes[i] = c;
            lweight[i] = ((const double *)(ws + T.weight))[i];
        }
        __syncthreads();
        const int depth = T.pad;
        for (int64_t blk = blockIdx.x; blk < n_blocks; blk += gridDim.x) {
        const int64_t r0 = blk * rows_per_block;
        const int64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
        for (int64_t rb = r0 + threadIdx.x; rb < r1; rb += 256 * kPredRows) {
            uint32_t W[kPredRows][4];
            float m[kPredRows];
#pragma unroll
            for (int q = 0; q < kPredRows; ++q) {
                const int64_t r = rb + 256 * q < r1 ? rb + 256 * q : r1 - 1;   // past the end: the last row again
                const uint64_t byte0 = (uint64_t)r * (uint64_t)F;
                const int64_t w0 = (int64_t)(byte0 >> 2);
                const uint32_t a = (uint32_t)(byte0 & 3);
                uint32_t w[5];
                if (w0 + 4 < n_words) {   // (all but the last rows of the matrix) one 16-byte load and one word
                    load_words(w, packed + w0);
                } else {
#pragma unroll
                    for (int k = 0; k < 5; ++k) w[k] = packed[w0 + k < n_words ? w0 + k : n_words - 1];
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) W[q][k] = __builtin_amdgcn_alignbyte(w[k + 1], w[k], a);
                m[q] = leaf_out ? 0.f : margin_src[r];
            }
            uint32_t node[kPredRows];
#pragma unroll
            for (int q = 0; q < kPredRows; ++q) node[q] = 0;
            for (int step = 0; step < depth; ++step) {
#pragma unroll
                for (int q = 0; q < kPredRows; ++q) {
                    const uint2 c = cnodes[node[q]];
                    const uint32_t lo = __builtin_amdgcn_perm(W[q][1], W[q][0], c.y);
                    const uint32_t hi = __builtin_amdgcn_perm(W[q][3], W[q][2], c.y);
                    const uint32_t sy = (c.x & (1u << 28)) ? hi : lo;
                    bool go_left = sy <= ((c.x >> 20) & 0xffu);
                    if (MISS) go_left = (sy == missing) ? (c.x & (1u << 29)) != 0 : go_left;
                    node[q] = (c.x & 0xfffffu) + (go_left ? 0u : 1u);
                }
            }
#pragma unroll
            for (int q = 0; q < kPredRows; ++q) {
                const int64_t r = rb + 256 * q;
                if (r < r1) {
                    if (leaf_out) leaf_out[r] = (int32_t)node[q];
                    else margin[r] = (float)((double)m[q] + eta * lweight[node[q]]);
                    if (node_rows) atomicAdd(&lcount[node[q]], 1u);
                }
            }
        }
        }
    }
    if (node_rows) {
        __syncthreads();
        for (int i = threadIdx.x; i < max_nodes; i += 256) {
            const uint32_t c = lcount[i];
            if (c) atomicAdd(&node_rows[(size_t)i * kNodeRowsStride], c);
        }
    }
}

// Final row order and leaf ids: every position of [0, n) lies in exactly one
// leaf segment; segments are sorted by seg_begin.
// Each workgroup takes a chunk of positions; the search starts from the segment of the chunk's
// first position (found once) and only walks forward.
constexpr int kGatherChunk = 256 * 16;
__global__ __launch_bounds__(256) void leaf_gather_kernel(const uint32_t *buf0, const uint32_t *buf1,
                                                          const LeafSeg *segs, int n_segs, int64_t n,
                                                          uint32_t *row_idx_out, int32_t *leaf_of_row) {
    const int64_t p0 = (int64_t)blockIdx.x * kGatherChunk;
    __shared__ int first_seg;
    if (threadIdx.x == 0) {
        int lo = 0, hi = n_segs;   // last segment with seg_begin <= p0
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if ((int64_t)segs[mid].seg_begin <= p0) lo = mid; else hi = mid;
        }
        first_seg = lo;
    }
    __syncthreads();
    int cur = first_seg;
    for (int k = 0; k < kGatherChunk / 256; ++k) {
        const int64_t p = p0 + (int64_t)k * 256 + threadIdx.x;
        if (p >= n) break;
        while (cur + 1 < n_segs && (int64_t)segs[cur + 1].seg_begin <= p) ++cur;
        const LeafSeg s = segs[cur];
        const uint32_t r = s.buf == 2 ? (uint32_t)p : (s.buf ? buf1 : buf0)[p];
        row_idx_out[p] = r;
        if (leaf_of_row && (int64_t)r < n) leaf_of_row[r] = (int32_t)s.node;
    }
}

}  // namespace

hipError_t gbt_launch_fill_u64(hipStream_t s, uint64_t *p, uint64_t v, int64_t count) {
    if (count <= 0) return hipSuccess;
    fill_u64_kernel<<<grid_for(count, kBlock * 4, 4096), kBlock, 0, s>>>(p, v, count);
    return hipGetLastError();
}
hipError_t gbt_launch_iota_u32(hipStream_t s, uint32_t *p, int64_t count) {
    if (count <= 0) return hipSuccess;
    iota_u32_kernel<<<grid_for(count, kBlock * 4, 8192), kBlock, 0, s>>>(p, count);
    return hipGetLastError();
}
// A plain streaming read of `n16` 16-byte pieces: what HBM delivers to a kernel that only reads (the yardstick
// beside the histogram kernels' achieved bandwidth).  sink is written only if the xor of everything read
// equals a magic word, which keeps the loads alive.
namespace {
__global__ __launch_bounds__(kBlock) void stream_read_kernel(const uint4 *__restrict__ p, int64_t n16, uint32_t *sink) {
    uint32_t acc = 0;
    const int64_t chunk = (int64_t)kStreamBatch * kBlock, n_whole = n16 / chunk;
    for (int64_t c = blockIdx.x; c < n_whole; c += gridDim.x) {
        uint4 v[kStreamBatch];
#pragma unroll
        for (int k = 0; k < kStreamBatch; ++k) v[k] = p[c * chunk + k * kBlock + threadIdx.x];
#pragma unroll
        for (int k = 0; k < kStreamBatch; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    }
    for (int64_t i = n_whole * chunk + (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n16; i += (int64_t)gridDim.x * kBlock) {
        const uint4 v = p[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9E3779B9u) *sink = acc;
}
}  // namespace
hipError_t gbt_launch_stream_read(hipStream_t s, const void *buf, int64_t bytes, uint32_t *sink) {
    const int64_t n16 = bytes / 16;
    if (n16 <= 0) return hipSuccess;
    stream_read_kernel<<<grid_for(n16, kBlock * kStreamBatch, 4096), kBlock, 0, s>>>((const uint4 *)buf, n16, sink);
    return hipGetLastError();
}

hipError_t gbt_launch_absmax(hipStream_t s, const float *gpair, int64_t n, uint32_t *out2) {
    hipError_t e = gbt_launch_fill_u64(s, (uint64_t *)out2, 0, 2);
    if (e != hipSuccess || n <= 0) return e;
    const int head = (int)(((uintptr_t)gpair >> 3) & 1u);   // pairs before the first 16-byte boundary
    absmax_kernel<<<grid_for(n, kBlock * 2 * kStreamBatch, 2048), kBlock, 0, s>>>((const float2 *)gpair + head,
                                                                                  n - head, head, out2);
    return hipGetLastError();
}
hipError_t gbt_launch_to_fixed(hipStream_t s, const float *gpair, int64_t n, double sg, double sh,
                               int32_t *gq, int64_t *sums_out) {
    if (sums_out) {
        hipError_t e = gbt_launch_fill_u64(s, (uint64_t *)sums_out, 0, 2);
        if (e != hipSuccess) return e;
    }
    if (n <= 0) return hipSuccess;
    const int head = (int)(((uintptr_t)gpair >> 3) & 1u);
    if (head != (int)(((uintptr_t)gq >> 3) & 1u)) {
        to_fixed_pairs_kernel<<<grid_for(n, kBlock * 4, 2048), kBlock, 0, s>>>((const float2 *)gpair, n, sg, sh,
                                                                               (int2 *)gq, sums_out);
        return hipGetLastError();
    }
    to_fixed_kernel<<<grid_for(n, kBlock * 2 * kStreamBatch, 2048), kBlock, 0, s>>>(
        (const float2 *)gpair + head, n - head, head, sg, sh, (int2 *)gq + head, sums_out);
    return hipGetLastError();
}
hipError_t gbt_launch_sum_gq(hipStream_t s, const int32_t *gq, const uint32_t *row_idx, int64_t n_rows,
                             int64_t *out2) {
    hipError_t e = gbt_launch_fill_u64(s, (uint64_t *)out2, 0, 2);
    if (e != hipSuccess || n_rows <= 0) return e;
    sum_gq_kernel<<<grid_for(n_rows, kBlock * 8, 2048), kBlock, 0, s>>>((const int2 *)gq, row_idx, n_rows,
                                                                        out2);
    return hipGetLastError();
}
hipError_t gbt_launch_gradients(hipStream_t s, int objective, const float *margin, const float *label,
                                int64_t n, float *gpair, uint32_t *bounds) {
    if (bounds) {
        hipError_t e = gbt_launch_fill_u64(s, (uint64_t *)bounds, 0, 2 * kBoundsStride);
        if (e != hipSuccess) return e;
    }
    if (n <= 0) return hipSuccess;
    const int vec = ((((uintptr_t)margin | (uintptr_t)label | (uintptr_t)gpair) & 15u) == 0) ? 1 : 0;
    // with bounds: no more workgroups than are resident at once, each ends with one set of atomics
    gradients_kernel<<<grid_for(n, kBlock * 4, bounds ? 2048 : 8192), kBlock, 0, s>>>(objective, margin, label, n,
                                                                      (float2 *)gpair, vec, bounds,
                                                                      (size_t)n * sizeof(float2) > ((size_t)192 << 20) ? 1 : 0);
    return hipGetLastError();
}
hipError_t gbt_launch_subtract_one(hipStream_t s, const int64_t *parent, const int64_t *child,
                                   int64_t *out, int64_t count) {
    if (count <= 0) return hipSuccess;
    subtract_one_kernel<<<grid_for(count, kBlock * 4, 4096), kBlock, 0, s>>>(parent, child, out, count);
    return hipGetLastError();
}
hipError_t gbt_launch_export(hipStream_t s, const int64_t *hist, int64_t count, double inv_sg,
                             double inv_sh, double *out) {
    if (count <= 0) return hipSuccess;
    export_kernel<<<grid_for(count, kBlock * 4, 4096), kBlock, 0, s>>>(hist, count, inv_sg, inv_sh, out);
    return hipGetLastError();
}
hipError_t gbt_launch_compress(hipStream_t s, const uint16_t *sym, int64_t n_elems, int bits,
                               uint32_t *packed, int64_t n_words) {
    if (n_words <= 0) return hipSuccess;
    compress_kernel<<<grid_for(n_words, kBlock * 4, 16384), kBlock, 0, s>>>(sym, n_elems, bits, packed,
                                                                            n_words);
    return hipGetLastError();
}
// ---------------------------------------------------------------------------
// Sec. 2.4 for many trees on raw floats: the rows are read from HBM once.  A workgroup stages a
// tile of 256 rows in LDS (odd row stride), then takes the trees in groups that fit LDS beside it
// (8-byte nodes + 8-byte weights, converted on the host): one row per thread, four trees of a group
// walked side by side (independent chains hide the LDS latency), every walk a fixed number of steps
// (the tree's depth) because a leaf is staged as a node that leads to itself.  The margin stays in a
// register and is rounded to fp32 after every tree, in tree order, like the one-tree kernels.
// ---------------------------------------------------------------------------
namespace {
constexpr int kBatchRows = 256;
constexpr int kBatchTrees = 4;

__global__ __launch_bounds__(kBatchRows) void predict_raw_batched_kernel(
    const gbt_batch_node *__restrict__ nodes_g, const double *__restrict__ wts_g,
    const int32_t *__restrict__ tree_off, const int32_t *__restrict__ tree_depth,
    const int32_t *__restrict__ group_end, int n_groups, const float *__restrict__ X, int64_t n, int F, int XS,
    double eta, float *__restrict__ margin, int cap_nodes) {
    extern __shared__ char smem[];
    float *xs = (float *)smem;
    gbt_batch_node *nd = (gbt_batch_node *)(smem + (((size_t)kBatchRows * XS * 4 + 15) & ~(size_t)15));
    double *wt = (double *)(nd + cap_nodes);
    const int64_t r0 = (int64_t)blockIdx.x * kBatchRows;
    const int rows = n - r0 < kBatchRows ? (int)(n - r0) : kBatchRows;
    {   // the tile is one contiguous piece of X: element tid + 256 k is loaded by thread tid in step k,
        // eight loads in flight per thread; (row, feature) of an element advance without divisions
        const int total = rows * F;
        const float *src = X + r0 * F;
        const int dq = kBatchRows / F, dr = kBatchRows % F;
        int row = (int)threadIdx.x / F, f = (int)threadIdx.x % F;
        for (int i0 = threadIdx.x; i0 < total; i0 += 8 * kBatchRows) {
            float v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = i0 + k * kBatchRows < total ? src[i0 + k * kBatchRows] : 0.0f;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (i0 + k * kBatchRows < total) xs[row * XS + f] = v[k];
                row += dq;
                f += dr;
                if (f >= F) {
                    f -= F;
                    ++row;
                }
            }
        }
    }
    const bool live = (int)threadIdx.x < rows;
    float m = live ? margin[r0 + threadIdx.x] : 0.0f;
    const float *xrow = xs + (live ? (int)threadIdx.x : 0) * XS;
    int t_begin = 0;
    for (int g = 0; g < n_groups; ++g) {
        const int t_end = group_end[g];
        const int n0 = tree_off[t_begin], n1 = tree_off[t_end];
        __syncthreads();   // the row tile is complete; the previous group's walks are done
        for (int i0 = threadIdx.x; i0 < n1 - n0; i0 += 4 * kBatchRows) {   // eight loads in flight per thread
            gbt_batch_node a[4];
            double w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = i0 + k * kBatchRows;
                const int ic = i < n1 - n0 ? i : n1 - n0 - 1;
                a[k] = nodes_g[n0 + ic];
                w[k] = wts_g[n0 + ic];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = i0 + k * kBatchRows;
                if (i < n1 - n0) {
                    nd[i] = a[k];
                    wt[i] = w[k];
                }
            }
        }
        __syncthreads();
        for (int t = t_begin; t < t_end; t += kBatchTrees) {
            int base[kBatchTrees], id[kBatchTrees], depth = 0;
#pragma unroll
            for (int k = 0; k < kBatchTrees; ++k) {
                const int tk = t + k < t_end ? t + k : t_end - 1;   // past the group: the last tree again, unused
                base[k] = tree_off[tk] - n0;
                id[k] = 0;
                const int dk = tree_depth[tk];
                depth = dk > depth ? dk : depth;
            }
            for (int d = 0; d < depth; ++d) {
                // the four walks' LDS reads are issued together: first the nodes, then the values
                uint2 q[kBatchTrees];
                float x[kBatchTrees];
#pragma unroll
                for (int k = 0; k < kBatchTrees; ++k) q[k] = *(const uint2 *)&nd[base[k] + id[k]];   // x: thr, y: meta
#pragma unroll
                for (int k = 0; k < kBatchTrees; ++k) x[k] = xrow[q[k].y >> 17];
#pragma unroll
                for (int k = 0; k < kBatchTrees; ++k) {
                    const uint32_t lt = x[k] < __uint_as_float(q[k].x) ? 1u : 0u;      // false for NaN
                    const uint32_t nan = x[k] != x[k] ? 1u : 0u;
                    const uint32_t go_left = (nan & (q[k].y >> 15)) | lt;
                    id[k] = (int)((q[k].y & 0x7fffu) + ((go_left ^ 1u) & (q[k].y >> 16) & 1u));
                }
            }
#pragma unroll
            for (int k = 0; k < kBatchTrees; ++k)
                if (t + k < t_end) m = (float)((double)m + eta * wt[base[k] + id[k]]);
        }
        t_begin = t_end;
    }
    if (live) margin[r0 + threadIdx.x] = m;
}
}  // namespace

int gbt_predict_batch_max_features() { return 95; }   // 256 rows x 96 words = 96 KB of LDS for the row tile

hipError_t gbt_launch_predict_raw_batched(hipStream_t s, const gbt_batch_node *nodes, const double *wts,
                                          const int32_t *tree_off, const int32_t *tree_depth,
                                          const int32_t *group_end, int n_groups, int cap_nodes, const float *X,
                                          int64_t n, int F, double eta, float *margin) {
    if (n <= 0 || n_groups <= 0) return hipSuccess;
    const int XS = F | 1;
    const size_t lds = (((size_t)kBatchRows * XS * 4 + 15) & ~(size_t)15) + (size_t)cap_nodes * 16;
    GbtLdsGuard lds_guard(lds);
    if (lds_guard.needed) {
        hipError_t e = hipFuncSetAttribute((const void *)predict_raw_batched_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const int64_t grid = (n + kBatchRows - 1) / kBatchRows;
    predict_raw_batched_kernel<<<(unsigned)grid, kBatchRows, lds, s>>>(nodes, wts, tree_off, tree_depth, group_end,
                                                                      n_groups, X, n, F, XS, eta, margin, cap_nodes);
    return hipGetLastError();
}

// Can the walk also count the rows per node, or read the margins from another array?  Only the byte-symbol kernel does.
bool gbt_predict_counts_ok(bool packed, int bits, int F, int max_nodes, bool compact_ok) {
    return packed && compact_ok && bits == 8 && F <= 16 && max_nodes <= (1 << 20) &&
           (size_t)max_nodes * (sizeof(LdsNode) + 4) <= 96u * 1024u;
}

hipError_t gbt_launch_predict(hipStream_t s, const char *ws, const DevTree *trees, int n_trees,
                              const uint32_t *packed, int bits, uint32_t missing, const float *X,
                              int64_t n, int F, double eta, float *margin, int32_t *leaf_out, int max_nodes,
                              bool compact_ok, uint32_t *node_rows, const float *margin_src) {
    if (n <= 0) return hipSuccess;
    if (margin_src == margin) margin_src = nullptr;
    if ((node_rows || margin_src) && !(n_trees == 1 && gbt_predict_counts_ok(packed != nullptr, bits, F, max_nodes, compact_ok)))
        return hipErrorInvalidValue;   // (the caller asks gbt_predict_counts_ok first)
    const size_t lds = (size_t)max_nodes * (sizeof(LdsNode) + (node_rows ? 4 : 0));
    static_assert(sizeof(LdsNode) >= 16, "the register-window kernel stages 16 bytes per node");
    if (lds <= 96u * 1024u) {
        GbtLdsGuard lds_guard(lds);
        if (lds_guard.needed) {
            hipError_t e = hipFuncSetAttribute((const void *)predict_lds_kernel,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        const int rows_per_block = 256 * 16;
        const int64_t grid = (n + rows_per_block - 1) / rows_per_block;
        if (packed && compact_ok && (int64_t)F * bits <= 128) {
            GbtLdsGuard lds_guard_w(lds);
            if (lds_guard_w.needed) {
                hipError_t e = hipFuncSetAttribute((const void *)predict_window_kernel,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                if (e != hipSuccess) return e;
            }
            const int64_t n_words = (n * (int64_t)F * bits + 31) / 32 + 1;
            if (bits == 8 && F <= 16 && max_nodes <= (1 << 20)) {   // node ids fit the 20-bit field
                GbtLdsGuard lds_guard_b(lds);
                if (lds_guard_b.needed) {
                    hipError_t e = hipFuncSetAttribute((const void *)predict_b8_kernel<true>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                    if (e == hipSuccess)
                        e = hipFuncSetAttribute((const void *)predict_b8_kernel<false>,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                    if (e != hipSuccess) return e;
                }
                // counting: few enough workgroups that their counts meet rarely in HBM, each taking many blocks
                const int64_t grid_b = node_rows && grid > 2048 ? 2048 : grid;
                if (missing < 256u)
                    predict_b8_kernel<true><<<(unsigned)grid_b, 256, lds, s>>>(ws, trees, n_trees, packed, n_words, missing,
                                                                              n, F, eta, margin, rows_per_block, max_nodes,
                                                                              leaf_out, node_rows, margin_src ? margin_src : margin);
                else
                    predict_b8_kernel<false><<<(unsigned)grid_b, 256, lds, s>>>(ws, trees, n_trees, packed, n_words, missing,
                                                                               n, F, eta, margin, rows_per_block, max_nodes,
                                                                               leaf_out, node_rows, margin_src ? margin_src : margin);
                return hipGetLastError();
            }
            predict_window_kernel<<<(unsigned)grid, 256, lds, s>>>(ws, trees, n_trees, packed, n_words, bits, missing,
                                                                   n, F, eta, margin, rows_per_block, max_nodes, leaf_out);
            return hipGetLastError();
        }
        // rows staged through LDS, a wave's 64 at a time (a row of up to 32 bytes lies in one cache line that the
        // gathers of its levels all hit: 1M x 28 bytes measured 0.107 ms gathered against 0.121 ms staged; 10M x 57
        // bytes 0.39 against 0.30 ms)
        if (packed && compact_ok && (int64_t)F * bits > 256 && (int64_t)F * bits <= kStagedRowBits) {
            const int wave_words = (int)((64 * (int64_t)F * bits + 31) / 32) + 2;
            const size_t lds_s = lds + (size_t)4 * wave_words * 4;
            if (lds_s <= 96u * 1024u) {
                GbtLdsGuard lds_guard_s(lds_s);
                if (lds_guard_s.needed) {
                    hipError_t e = hipFuncSetAttribute((const void *)predict_staged_kernel,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_s);
                    if (e != hipSuccess) return e;
                }
                const int64_t n_words = (n * (int64_t)F * bits + 31) / 32 + 1;
                predict_staged_kernel<<<(unsigned)grid, 256, lds_s, s>>>(ws, trees, n_trees, packed, n_words, bits, missing, n, F,
                                                                         eta, margin, rows_per_block, max_nodes, leaf_out,
                                                                         wave_words);
                return hipGetLastError();
            }
        }
        predict_lds_kernel<<<(unsigned)grid, 256, lds, s>>>(ws, trees, n_trees, packed, bits, missing, X, n, F, eta,
                                                            margin, rows_per_block, leaf_out);
        return hipGetLastError();
    }
    predict_kernel<<<grid_for(n, kBlock, 1 << 16), kBlock, 0, s>>>(ws, trees, n_trees, packed, bits,
                                                                    missing, X, n, F, eta, margin, leaf_out);
    return hipGetLastError();
}
hipError_t gbt_launch_leaf_gather(hipStream_t s, const uint32_t *buf0, const uint32_t *buf1,
                                  const LeafSeg *segs, int n_segs, int64_t n, uint32_t *row_idx_out,
                                  int32_t *leaf_of_row) {
    if (n <= 0 || n_segs <= 0) return hipSuccess;
    const int64_t grid = (n + kGatherChunk - 1) / kGatherChunk;
    leaf_gather_kernel<<<(unsigned)grid, 256, 0, s>>>(buf0, buf1, segs, n_segs, n, row_idx_out, leaf_of_row);
    return hipGetLastError();
}
