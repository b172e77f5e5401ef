// EvaluateSplit (Alg. 1; Sec. 2.3): every (feature, bin) candidate of a node is priced from running
// sums over the node's histogram, which a wave forms with a prefix scan.
//
// One workgroup per (node, feature chunk); each wave takes whole features.  With several
// chunks per node the caller merges the chunks' records (largest gain, first chunk on ties:
// chunks are in feature order, so that is the candidate order).  For a feature the
// wave first reduces the bins to get the node's missing mass for that feature,
// then runs an inclusive wave-level prefix scan (64 bins per step, carry between
// steps) over the exact int64 sums and prices every (bin, direction) candidate
// in fp64.  The best candidate is kept per lane in candidate order, so a strict
// '>' keeps the first of equal gains; lanes and waves are then merged with
// (gain descending, candidate index ascending).
//
// Compiled with -ffp-contract=off: the gain must be the same sequence of
// rounded fp64 operations a plain C compiler produces.
#include "gbt_internal.h"
#include "wave_scan.h"

#include <math.h>

namespace {

constexpr int kEvalBlock = 256;
constexpr int kEvalWaves = kEvalBlock / 64;
constexpr int kEvalGroups = 8192;

__device__ inline int64_t shfl_xor_i64(int64_t v, int m) {
    int lo = __shfl_xor((int)(v & 0xffffffff), m);
    int hi = __shfl_xor((int)(v >> 32), m);
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}
__device__ inline double shfl_xor_f64(double v, int m) {
    return __longlong_as_double(shfl_xor_i64(__double_as_longlong(v), m));
}

struct Best {
    double gain;
    uint32_t key;   // (feature * B + bin) * 2 + direction; 0xffffffff = none
    int64_t GLq, HLq;
};

__device__ inline bool better(double ga, uint32_t ka, double gb, uint32_t kb) {
    return ga > gb || (ga == gb && ka < kb);
}

// G^2/(H + lambda): what the best step of a set of rows gains.  Without curvature (denominator 0: lambda = 0 and
// no hessian mass) there is no best step; the leaf weight is then defined as 0 and, to match, so is the gain.
__device__ __forceinline__ double gain_term(double G, double denom) { return denom > 0.0 ? G * G / denom : 0.0; }

__global__ __launch_bounds__(kEvalBlock) void eval_kernel(
    int64_t *__restrict__ pool, const EvalNode *__restrict__ nodes, const int32_t *__restrict__ nb,
    int F, int B, int f_per_chunk, double inv_sg, double inv_sh, double lambda, double mcw,
    gbt_split *__restrict__ out, EvalTail tail) {
    if (blockIdx.x == 0 && blockIdx.y == 0) {   // the words handed back with the records (see gbt_launch_eval)
        for (int i = threadIdx.x; i < tail.n; i += kEvalBlock) {
            tail.dst[i] = tail.src[(size_t)i * tail.src_stride];
            if (tail.clear) tail.src[(size_t)i * tail.src_stride] = 0ull;
        }
    }
    const EvalNode nd = nodes[blockIdx.x];
    const int f_begin = blockIdx.y * f_per_chunk;
    const int f_end = f_begin + f_per_chunk < F ? f_begin + f_per_chunk : F;
    if (tail.clear_slot >= 0 && f_begin < f_end) {   // this chunk's features of the two histograms below node blockIdx.x
        const int64_t per = (int64_t)F * B * 2, span = (int64_t)(f_end - f_begin) * B * 2;
        for (int c = 0; c < 2; ++c) {
            const int64_t slot = tail.clear_slot + 2 * (int64_t)blockIdx.x + c;
            if (slot >= tail.clear_slot_end) break;
            int64_t *z = pool + slot * per + (int64_t)f_begin * B * 2;
            for (int64_t i = threadIdx.x; i < span; i += kEvalBlock) z[i] = 0;
        }
    }
    int64_t *hist = pool + nd.hist_off;
    // the larger sibling: its histogram is made here, as parent - built (exact: integers), and kept
    const bool subtract = nd.parent_off != GBT_NO_HIST;
    const bool store = subtract && !tail.skip_store;
    const int64_t *hpar = pool + (subtract ? nd.parent_off : 0), *hblt = pool + (subtract ? nd.built_off : 0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t Gq = nd.Gq, Hq = nd.Hq;
    const double G = (double)Gq * inv_sg, H = (double)Hq * inv_sh;
    const double parent = gain_term(G, H + lambda);

    Best best;
    best.gain = -INFINITY;
    best.key = 0xffffffffu;
    best.GLq = 0;
    best.HLq = 0;

    // one 64-bin piece of a feature's scan: the inclusive prefix over the piece's bins (carried in from cg, ch) ...
    auto scan = [&](int64_t &pg, int64_t &ph, int64_t &cg, int64_t &ch) __attribute__((always_inline)) {
        pg = wave_scan_i64(pg) + cg;
        ph = wave_scan_i64(ph) + ch;
        cg = last_lane_i64(pg);
        ch = last_lane_i64(ph);
    };
    // ... then the gain of every (bin, direction) of the piece; pg, ph: the inclusive sums of bin b0 + lane
    auto score = [&](int f, int nbf, int b0, int64_t pg, int64_t ph, int64_t Gm, int64_t Hm, bool has_missing)
                     __attribute__((always_inline)) {
        const int b = b0 + lane;
        if (b < nbf) {
            for (int dir = 0; dir <= (has_missing ? 1 : 0); ++dir) {
                if (b == nbf - 1 && (dir == 1 || !has_missing)) continue;   // right side empty
                const int64_t GLq = pg + (dir ? Gm : 0), HLq = ph + (dir ? Hm : 0);
                const double GL = (double)GLq * inv_sg, HL = (double)HLq * inv_sh;
                const double GR = (double)(Gq - GLq) * inv_sg, HR = (double)(Hq - HLq) * inv_sh;
                if (!(HL >= mcw) || !(HR >= mcw)) continue;
                const double a = gain_term(GL, HL + lambda);
                const double c = gain_term(GR, HR + lambda);
                const double gain = (a + c) - parent;
                if (gain > best.gain) {
                    best.gain = gain;
                    best.key = ((uint32_t)f * (uint32_t)B + (uint32_t)b) * 2u + (uint32_t)dir;
                    best.GLq = GLq;
                    best.HLq = HLq;
                }
            }
        }
    };

    if (B <= 64) {
        // Every feature's bins fit one per lane: a lane's bin stays in registers between the reduction and the scan,
        // and the NEXT feature's words are asked for before this one's are worked on (a wave otherwise has one
        // kilobyte in flight at a time, too little to keep HBM busy at a few waves per SIMD).  (Two features ahead, or
        // one 16-byte load per bin instead of two of 8, measured the same.)
        auto fetch = [&](int f, int64_t &g, int64_t &h) __attribute__((always_inline)) {
            g = 0;
            h = 0;
            if (f < f_end) {
                int nbf = nb[f];
                if (nbf > B) nbf = B;
                if (lane < nbf) {
                    const int64_t o = (int64_t)f * B * 2 + 2 * lane;
                    if (subtract) {
                        g = hpar[o] - hblt[o];
                        h = hpar[o + 1] - hblt[o + 1];
                    } else {
                        g = hist[o];
                        h = hist[o + 1];
                    }
                }
            }
        };
        int64_t g0, h0;
        fetch(f_begin + wave, g0, h0);
        for (int f = f_begin + wave; f < f_end; f += kEvalWaves) {
            int64_t g1, h1;
            fetch(f + kEvalWaves, g1, h1);
            int nbf = nb[f];
            if (nbf > B) nbf = B;
            if (store && lane < nbf) {
                int64_t *hf = hist + (int64_t)f * B * 2;
                hf[2 * lane] = g0;
                hf[2 * lane + 1] = h0;
            }
            // the scan's last lane holds the feature's present mass (lanes past nbf hold zeros): no reduction of its own
            int64_t cg = 0, ch = 0;
            scan(g0, h0, cg, ch);
            const int64_t Gm = Gq - cg, Hm = Hq - ch;
            if (nbf > 0) score(f, nbf, 0, g0, h0, Gm, Hm, (Gm != 0) || (Hm != 0));
            g0 = g1;
            h0 = h1;
        }
    } else
    for (int f = f_begin + wave; f < f_end; f += kEvalWaves) {
        int nbf = nb[f];
        if (nbf > B) nbf = B;
        int64_t *hf = hist + (int64_t)f * B * 2;
        // pass 1: the feature's present mass -> the node's missing mass
        int64_t sg = 0, sh = 0;
        const int64_t *pf = hpar + (int64_t)f * B * 2, *bf = hblt + (int64_t)f * B * 2;
        if (subtract) {   // (the lane that stores bin b is the lane that reads it again in pass 2)
            for (int b = lane; b < nbf; b += 64) {
                const int64_t g = pf[2 * b] - bf[2 * b], h = pf[2 * b + 1] - bf[2 * b + 1];
                if (store) {
                    hf[2 * b] = g;
                    hf[2 * b + 1] = h;
                }
                sg += g;
                sh += h;
            }
        } else {
            for (int b = lane; b < nbf; b += 64) {
                sg += hf[2 * b];
                sh += hf[2 * b + 1];
            }
        }
        sg = last_lane_i64(wave_scan_i64(sg));
        sh = last_lane_i64(wave_scan_i64(sh));
        const int64_t Gm = Gq - sg, Hm = Hq - sh;
        const bool has_missing = (Gm != 0) || (Hm != 0);
        // pass 2: inclusive scan over bins, 64 at a time
        int64_t cg = 0, ch = 0;
        for (int b0 = 0; b0 < nbf; b0 += 64) {
            const int b = b0 + lane;
            int64_t pg = 0, ph = 0;
            if (b < nbf) {
                if (subtract && !store) {   // nothing was stored: the difference once more (the words are cached)
                    pg = pf[2 * b] - bf[2 * b];
                    ph = pf[2 * b + 1] - bf[2 * b + 1];
                } else {
                    pg = hf[2 * b];
                    ph = hf[2 * b + 1];
                }
            }
            scan(pg, ph, cg, ch);
            score(f, nbf, b0, pg, ph, Gm, Hm, has_missing);
        }
    }

    // merge lanes, then waves
    for (int o = 32; o > 0; o >>= 1) {
        double g2 = shfl_xor_f64(best.gain, o);
        uint32_t k2 = (uint32_t)__shfl_xor((int)best.key, o);
        int64_t gl2 = shfl_xor_i64(best.GLq, o), hl2 = shfl_xor_i64(best.HLq, o);
        if (better(g2, k2, best.gain, best.key)) {
            best.gain = g2;
            best.key = k2;
            best.GLq = gl2;
            best.HLq = hl2;
        }
    }
    __shared__ Best wb[kEvalWaves];
    if (lane == 0) wb[wave] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        Best r = wb[0];
        for (int w = 1; w < kEvalWaves; ++w)
            if (better(wb[w].gain, wb[w].key, r.gain, r.key)) r = wb[w];
        gbt_split s;
        if (r.key == 0xffffffffu) {
            s.feature = -1;
            s.bin = 0;
            s.default_left = 0;
            s.valid = 0;
            s.gain = -INFINITY;
            s.GL = s.HL = s.GR = s.HR = 0.0;
            s.GLq = s.HLq = 0;
        } else {
            const uint32_t fb = r.key >> 1;
            s.feature = (int32_t)(fb / (uint32_t)B);
            s.bin = (int32_t)(fb % (uint32_t)B);
            s.default_left = (int32_t)(r.key & 1u);
            s.valid = 1;
            s.gain = r.gain;
            s.GLq = r.GLq;
            s.HLq = r.HLq;
            s.GL = (double)r.GLq * inv_sg;
            s.HL = (double)r.HLq * inv_sh;
            s.GR = (double)(Gq - r.GLq) * inv_sg;
            s.HR = (double)(Hq - r.HLq) * inv_sh;
        }
        out[(size_t)blockIdx.x * gridDim.y + blockIdx.y] = s;
    }
}

}  // namespace

int gbt_eval_chunks(int F, int n_nodes, size_t record_budget_bytes) {
    int chunks = (F + 3) / 4;     // one feature per wave while that keeps the number of records small
    if (chunks > 64) chunks = 64;
    // a level of many nodes fills the chip without chunks: about kEvalGroups workgroups per launch are enough, and
    // every chunk more is a record the host reads back and merges
    const int by_nodes = (kEvalGroups + n_nodes - 1) / (n_nodes > 0 ? n_nodes : 1);
    if (chunks > by_nodes) chunks = by_nodes;
    while (chunks > 1 && (size_t)n_nodes * chunks * sizeof(gbt_split) > record_budget_bytes) --chunks;
    return chunks < 1 ? 1 : chunks;
}

hipError_t gbt_launch_eval(hipStream_t s, int64_t *hist_pool, const EvalNode *nodes, int n_nodes,
                           const int32_t *nb, int F, int B, int n_chunks, double inv_sg, double inv_sh,
                           double lambda, double mcw, gbt_split *out, EvalTail tail) {
    if (n_nodes <= 0) return hipSuccess;   // (the callers have no tail without nodes)
    const int f_per_chunk = (F + n_chunks - 1) / n_chunks;
    dim3 grid((unsigned)n_nodes, (unsigned)n_chunks);
    eval_kernel<<<grid, kEvalBlock, 0, s>>>(hist_pool, nodes, nb, F, B, f_per_chunk, inv_sg, inv_sh, lambda, mcw, out, tail);
    return hipGetLastError();
}
