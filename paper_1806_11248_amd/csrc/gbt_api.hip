// The C ABI of libgbt (see include/gbt.h) and the host side of Alg. 1.
#include "gbt_internal.h"

#include <math.h>
#include <stdarg.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <set>
#include <vector>

// ---------------------------------------------------------------- plumbing --
int32_t gbt_fail(gbt_ctx *ctx, int32_t code, const char *fmt, ...) {
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof ctx->err, fmt, ap);
        va_end(ap);
    }
    return code;
}

std::recursive_mutex &gbt_lds_mutex() {
    static std::recursive_mutex m;
    return m;
}

namespace {

hipError_t part_static_address(int device, char **out);   // gbt_partition_static's scratch array, below

constexpr size_t kUploadBytes = GBT_STAGING_BYTES / 2;   // first half of the pinned staging
constexpr size_t kReadbackOff = GBT_STAGING_BYTES / 2;   // second half
constexpr int kMaxDepth = 16;

inline char *up(gbt_ctx *c) { return c->pinned; }
inline char *rb(gbt_ctx *c) { return c->pinned + kReadbackOff; }

int32_t check_matrix(gbt_ctx *ctx, const void *packed, int32_t bits, int64_t n, int32_t F) {
    GBT_REQUIRE(ctx, packed != nullptr, GBT_EINVAL, "packed is NULL");
    GBT_REQUIRE(ctx, bits >= 1, GBT_EINVAL, "bits = %d < 1", bits);
    GBT_REQUIRE(ctx, bits <= GBT_MAX_BITS, GBT_EUNSUPPORTED, "bits = %d > %d", bits, GBT_MAX_BITS);
    GBT_REQUIRE(ctx, n >= 0 && n < ((int64_t)1 << 32), GBT_EINVAL, "n = %lld out of range", (long long)n);
    GBT_REQUIRE(ctx, F >= 1 && F <= (1 << 20), GBT_EINVAL, "F = %d out of range", F);
    return GBT_OK;
}

int32_t check_bins(gbt_ctx *ctx, int32_t F, int32_t B) {
    GBT_REQUIRE(ctx, B >= 2 && B <= 4096, GBT_EINVAL, "max_bins = %d outside 2..4096", B);
    GBT_REQUIRE(ctx, (int64_t)F * B < ((int64_t)1 << 31), GBT_EINVAL, "F*max_bins too large");
    return GBT_OK;
}

// Power-of-two scale s with |x|*s <= 2^top for every |x| <= vmax.
constexpr int kGBits = 26, kHBits = 22;   // |g*scale_g| <= 2^26, h*scale_h <= 2^22: the packed LDS word's fields
double fixed_scale(float vmax, int top) {
    if (!(vmax > 0.0f)) return 1.0;
    int e;
    frexp((double)vmax, &e);   // vmax = m * 2^e, m in [0.5, 1)
    return ldexp(1.0, top - e);
}

// Uniform job split of a dense or listed row range for the histogram kernel.
struct HistPlan {
    int ft_max, n_ftiles, ft;
};
// The kernels consume a row slice in register windows of E whole elements and issue an atomic for
// every slot of a window, used or not.  More tiles than the LDS budget demands cost a pass over the
// gradient pairs each, so they are taken only when they save at least a fifth of the slots.
bool plan_tiles(const gbt_ctx *ctx, int F, int B, int bits, HistPlan *p, int64_t n_rows = 0) {
    p->ft_max = gbt_hist_feature_tile(ctx, F, B, n_rows);
    if (p->ft_max < 1) return false;
    const int E = bits == 8 ? 16 : std::min(128 / std::max(bits, 1), 32);
    const int nt_min = (F + p->ft_max - 1) / p->ft_max;
    int64_t best_slots = -1;
    for (int nt = nt_min; nt <= nt_min + 8 && nt <= F; ++nt) {
        const int ft = (F + nt - 1) / nt;
        const int64_t slots = (int64_t)nt * ((ft + E - 1) / E) * E;
        if (best_slots < 0 || slots * 5 <= best_slots * 4) {
            best_slots = slots;
            p->n_ftiles = nt;
            p->ft = ft;
        }
    }
    return true;
}

// Appends the jobs of one node; rows_per_job > 0.
// A node covered by ONE row piece has exclusive jobs (HistJob.pad0 = 1: their bins are stored, not added); set
// may_store = false where the histogram is not 16-byte aligned.
void add_hist_jobs(std::vector<HistJob> &jobs, uint64_t hist_off, uint32_t begin, uint32_t len, int F,
                   const HistPlan &pl, uint32_t rows_per_job, bool may_store = true) {
    const bool exclusive = may_store && len <= rows_per_job;
    for (uint32_t r0 = 0; r0 < len; r0 += rows_per_job) {
        uint32_t nr = std::min(rows_per_job, len - r0);
        for (int t = 0; t < pl.n_ftiles; ++t) {
            HistJob j;
            j.hist_off = hist_off;
            j.row_begin = begin + r0;
            j.n_rows = nr;
            j.f0 = (uint32_t)(t * pl.ft);
            j.ft = (uint32_t)std::min(pl.ft, F - t * pl.ft);
            j.pad0 = exclusive ? 1u : 0u;
            j.pad1 = 0;
            if (j.ft > 0) jobs.push_back(j);
        }
    }
}

// max_rows: what a job of the kernel may hold (2^21: its per-bin event counters are 16 bits wide; fewer where
// it counts rows in a narrow field, gbt_histw_max_rows)
// Every job of a launch merges the bins of its feature tile into HBM with two 64-bit global atomics per non-zero
// bin, and the chip retires only ~1e11 of those per second, some forty times fewer than LDS atomics: a row piece
// is therefore long enough that a bin receives hist_merge_ratio LDS additions on average per value merged
// (rows >= ratio * 2 * B), unless that would leave fewer than about one workgroup per compute unit.
uint32_t pick_rows_per_job(const gbt_ctx *ctx, int64_t total_rows, int64_t max_rows = 1 << 21, int n_tiles = 1,
                           int B = 0) {
    int64_t pieces = std::max<int64_t>(1, (int64_t)ctx->num_cu * ctx->hist_jobs_per_cu / std::max(1, n_tiles));
    if (B > 0) {
        const int64_t by_merge = std::max<int64_t>(total_rows / ((int64_t)ctx->hist_merge_ratio * 2 * B),
                                                   ((int64_t)ctx->num_cu + n_tiles - 1) / n_tiles);
        pieces = std::min(pieces, std::max<int64_t>(1, by_merge));
    }
    int64_t rpj = (total_rows + pieces - 1) / pieces;
    if (rpj < 4096) rpj = 4096;
    if (rpj > max_rows) rpj = max_rows;
    return (uint32_t)rpj;
}

// Best of one node's per-chunk split records: largest gain, earliest chunk on ties.
gbt_split merge_chunks(const gbt_split *rec, int n_chunks) {
    gbt_split best = rec[0];
    for (int c = 1; c < n_chunks; ++c)
        if (rec[c].valid && (!best.valid || rec[c].gain > best.gain)) best = rec[c];
    return best;
}

// The first half of the pinned staging is a ring of upload slots: a slot may be
// overwritten only after the copy (or kernel) that reads it has finished, which
// a stream synchronisation guarantees; wrapping therefore synchronises first.
int32_t sync(gbt_ctx *ctx) {
    GBT_HIP(ctx, hipStreamSynchronize(ctx->stream));
    ctx->up_off = 0;
    return GBT_OK;
}

int32_t stage(gbt_ctx *ctx, const void *host, size_t bytes, char **slot) {
    GBT_REQUIRE(ctx, bytes <= kUploadBytes, GBT_EUNSUPPORTED, "job table of %zu bytes exceeds staging", bytes);
    const size_t need = gbt_align(bytes ? bytes : 1);
    if (ctx->up_off + need > kUploadBytes) {
        int32_t st = sync(ctx);
        if (st != GBT_OK) return st;
    }
    *slot = up(ctx) + ctx->up_off;
    memcpy(*slot, host, bytes);
    ctx->up_off += need;
    return GBT_OK;
}

#define GBT_SYNC(ctx)                      \
    do {                                   \
        int32_t st_ = sync(ctx);           \
        if (st_ != GBT_OK) return st_;     \
    } while (0)

// Uploads `bytes` of job descriptors through the pinned staging into `dev`.
int32_t upload(gbt_ctx *ctx, const void *host, size_t bytes, void *dev) {
    char *slot;
    int32_t st = stage(ctx, host, bytes, &slot);
    if (st != GBT_OK) return st;
    GBT_HIP(ctx, hipMemcpyAsync(dev, slot, bytes, hipMemcpyHostToDevice, ctx->stream));
    return GBT_OK;
}

// Two tables with one copy: `b` lands behind `a` at the next aligned offset, which is returned.
int32_t upload2(gbt_ctx *ctx, const void *a, size_t a_bytes, const void *b, size_t b_bytes, void *dev, size_t *b_off) {
    const size_t off = gbt_align(a_bytes ? a_bytes : 1);
    GBT_REQUIRE(ctx, off + b_bytes <= kUploadBytes, GBT_EUNSUPPORTED, "job tables of %zu bytes exceed staging", off + b_bytes);
    const size_t need = gbt_align(off + (b_bytes ? b_bytes : 1));
    if (ctx->up_off + need > kUploadBytes) {
        int32_t st = sync(ctx);
        if (st != GBT_OK) return st;
    }
    char *slot = up(ctx) + ctx->up_off;
    memcpy(slot, a, a_bytes);
    memcpy(slot + off, b, b_bytes);
    ctx->up_off += need;
    GBT_HIP(ctx, hipMemcpyAsync(dev, slot, off + b_bytes, hipMemcpyHostToDevice, ctx->stream));
    *b_off = off;
    return GBT_OK;
}

}  // namespace

// ------------------------------------------------------------------ context --
extern "C" const char *gbt_version(void) { return "libgbt 0.1 (gfx950)"; }

extern "C" int32_t gbt_create(gbt_ctx **ctx_out, int32_t device, void *stream) {
    if (!ctx_out) return GBT_EINVAL;
    *ctx_out = nullptr;
    gbt_ctx *c = new (std::nothrow) gbt_ctx();
    if (!c) return GBT_ENOMEM;
    memset(c, 0, sizeof *c);
    c->spans = new std::vector<ProfSpan>();
    c->free_events = new std::vector<hipEvent_t>();
    c->device = device;
    c->stream = (hipStream_t)stream;
    hipError_t e = hipSetDevice(device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
    if (e == hipSuccess && strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
        fprintf(stderr, "libgbt: device %d is %s, this library is built for gfx950 only\n", device,
                prop.gcnArchName);
        delete c->spans;
        delete c->free_events;
        delete c;
        return GBT_EHIP;
    }
    if (e == hipSuccess) {
        c->num_cu = prop.multiProcessorCount;
        c->hist_block = 512;
        c->hist_jobs_per_cu = 8;
        c->hist_merge_ratio = 96;
        c->move_max_words = 8;    // measured: 15-word rows (10M x 50 x 9 bits) grow 18 % faster by id lists than moved; 7-word rows stay moved
        if (const char *e20 = getenv("GBT_TUNE_MOVE_MAX_WORDS")) { int v = atoi(e20); if (v >= 1 && v <= 64) c->move_max_words = v; }
        c->hist_lds_kb = 64;   // two resident workgroups per CU hide the row-fetch latency better than one big tile
        if (const char *e1 = getenv("GBT_TUNE_HIST_BLOCK")) { int v = atoi(e1); if (v == 256 || v == 512 || v == 1024) c->hist_block = v; }
        if (const char *e3 = getenv("GBT_TUNE_HIST_RUNTIME_BITS")) c->hist_runtime_bits = atoi(e3) != 0;
        c->part_fused = 1;
        c->part_hist = 1;
        c->hist_fix = 1;
        c->hist8 = 1;
        c->hist8_stagger = 64;
        if (const char *e17 = getenv("GBT_TUNE_HIST8")) c->hist8 = atoi(e17) != 0;
        if (const char *e18 = getenv("GBT_TUNE_HIST8_STAGGER")) { int v = atoi(e18); if (v >= 0 && v <= 128) c->hist8_stagger = v; }
        c->sparse_jobs_per_cu = 1;
        if (const char *e12 = getenv("GBT_TUNE_SPARSE_JOBS")) { int v = atoi(e12); if (v >= 1 && v <= 64) c->sparse_jobs_per_cu = v; }
        if (const char *e13 = getenv("GBT_TUNE_SPARSE_TILED")) c->sparse_tiled = atoi(e13) != 0;
        c->lossguide_batch = 16;
        if (const char *e16 = getenv("GBT_TUNE_LOSSGUIDE_BATCH")) { int v = atoi(e16); if (v >= 1 && v <= 64) c->lossguide_batch = v; }
        c->part_nomove = 2;
        if (const char *e15 = getenv("GBT_TUNE_PART_NOMOVE")) { int v = atoi(e15); if (v >= 0 && v <= 2) c->part_nomove = v; }
        c->part_cycle = 1;
        if (const char *e17 = getenv("GBT_TUNE_PART_CYCLE")) c->part_cycle = atoi(e17) != 0;
        c->part_ids = 1;
        if (const char *e14 = getenv("GBT_TUNE_PART_IDS")) c->part_ids = atoi(e14) != 0;
        c->order_rows = 1;
        if (const char *e11 = getenv("GBT_TUNE_ORDER_ROWS")) c->order_rows = atoi(e11) != 0;
        if (const char *e10 = getenv("GBT_TUNE_HIST_FIX")) c->hist_fix = atoi(e10) != 0;
        if (const char *e8 = getenv("GBT_TUNE_PART_HIST")) c->part_hist = atoi(e8) != 0;
        if (const char *e6 = getenv("GBT_TUNE_PART_FUSED")) c->part_fused = atoi(e6) != 0;
        c->hist_lds_auto = 1;
        if (const char *e5 = getenv("GBT_TUNE_HIST_LDS_KB")) { int v = atoi(e5); if (v >= 8 && v <= 128) { c->hist_lds_kb = v; c->hist_lds_auto = 0; } }
        if (const char *e19 = getenv("GBT_TUNE_HIST_MERGE_RATIO")) { int v = atoi(e19); if (v >= 1 && v <= 100000) c->hist_merge_ratio = v; }
        if (const char *e2 = getenv("GBT_TUNE_HIST_JOBS")) { int v = atoi(e2); if (v >= 1 && v <= 64) c->hist_jobs_per_cu = v; }
        size_t lds = prop.sharedMemPerBlock;
        int optin = 0;
        if (hipDeviceGetAttribute(&optin, hipDeviceAttributeSharedMemPerBlockOptin, device) == hipSuccess &&
            (size_t)optin > lds)
            lds = (size_t)optin;
        c->lds_max = lds;
        if (lds > 128u * 1024u) lds = 128u * 1024u;   // leave room for a second resident workgroup's statics
        c->lds_per_block = lds;
        e = hipHostMalloc((void **)&c->pinned, GBT_STAGING_BYTES, hipHostMallocDefault);
        c->pinned_bytes = GBT_STAGING_BYTES;
        if (e == hipSuccess) e = part_static_address(device, &c->part_static);
    }
    if (e != hipSuccess) {
        fprintf(stderr, "libgbt: gbt_create failed: %s\n", hipGetErrorString(e));
        (void)hipGetLastError();
        if (c->pinned) (void)hipHostFree(c->pinned);
        delete c->spans;
        delete c->free_events;
        delete c;
        return GBT_EHIP;
    }
    *ctx_out = c;
    return GBT_OK;
}

extern "C" int32_t gbt_destroy(gbt_ctx *ctx) {
    if (!ctx) return GBT_EINVAL;
    if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    for (ProfSpan &sp : *ctx->spans) {
        (void)hipEventDestroy(sp.start);
        (void)hipEventDestroy(sp.stop);
    }
    for (hipEvent_t e : *ctx->free_events) (void)hipEventDestroy(e);
    delete ctx->spans;
    delete ctx->free_events;
    delete ctx;
    return GBT_OK;
}

extern "C" const char *gbt_last_error(const gbt_ctx *ctx) { return ctx ? ctx->err : "null context"; }

// --------------------------------------------------------------- profiling --
static hipEvent_t prof_event(gbt_ctx *ctx) {
    if (!ctx->free_events->empty()) {
        hipEvent_t e = ctx->free_events->back();
        ctx->free_events->pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

int gbt_prof_begin(gbt_ctx *ctx, int cls, double bytes, double alg_bytes, int level, double row_features) {
    if (!ctx->profiling) return -1;
    ProfSpan sp;
    sp.cls = cls;
    sp.bytes = bytes;
    sp.alg_bytes = alg_bytes;
    sp.level = level;
    sp.row_features = row_features;
    sp.start = prof_event(ctx);
    sp.stop = prof_event(ctx);
    if (!sp.start || !sp.stop) return -1;
    (void)hipEventRecord(sp.start, ctx->stream);
    ctx->spans->push_back(sp);
    return (int)ctx->spans->size() - 1;
}

void gbt_prof_patch(gbt_ctx *ctx, int span, double alg_bytes, double row_features) {
    if (!ctx->profiling || span < 0 || span >= (int)ctx->spans->size()) return;
    (*ctx->spans)[(size_t)span].alg_bytes = alg_bytes;
    (*ctx->spans)[(size_t)span].row_features = row_features;
}

void gbt_prof_end(gbt_ctx *ctx) {
    if (!ctx->profiling || ctx->spans->empty()) return;
    (void)hipEventRecord(ctx->spans->back().stop, ctx->stream);
}

extern "C" int32_t gbt_profile_enable(gbt_ctx *ctx, int32_t on) {
    if (!ctx) return GBT_EINVAL;
    ctx->profiling = on != 0;
    return GBT_OK;
}

extern "C" int32_t gbt_profile_read(gbt_ctx *ctx, gbt_profile *out) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, out != nullptr, GBT_EINVAL, "NULL argument");
    GBT_SYNC(ctx);
    memset(out, 0, sizeof *out);
    for (ProfSpan &sp : *ctx->spans) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sp.start, sp.stop) == hipSuccess && sp.cls >= 0 && sp.cls < GBT_PROF_CLASSES) {
            out->ms[sp.cls] += ms;
            out->bytes[sp.cls] += sp.bytes;
            out->alg_bytes[sp.cls] += sp.alg_bytes < 0.0 ? sp.bytes : sp.alg_bytes;
            out->launches[sp.cls] += 1;
            if (sp.level >= 0 && sp.level < GBT_PROF_LEVELS) {
                out->level_ms[sp.level] += ms;
                out->level_alg_bytes[sp.level] += sp.alg_bytes < 0.0 ? sp.bytes : sp.alg_bytes;
                out->level_row_features[sp.level] += sp.row_features;
                out->level_launches[sp.level] += 1;
            }
        }
        ctx->free_events->push_back(sp.start);
        ctx->free_events->push_back(sp.stop);
    }
    (void)hipGetLastError();
    ctx->spans->clear();
    return GBT_OK;
}

extern "C" int32_t gbt_measure_stream_read(gbt_ctx *ctx, const void *buf, size_t bytes, int32_t reps, double *gbps_out,
                                           void *workspace, size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, buf && gbps_out && workspace, GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, ((uintptr_t)buf & 15u) == 0, GBT_EINVAL, "buf must be 16-byte aligned");
    GBT_REQUIRE(ctx, bytes >= 16 && reps >= 1, GBT_EINVAL, "nothing to read");
    GBT_REQUIRE(ctx, workspace_bytes >= 4096, GBT_ENOMEM, "workspace < 4096 bytes");
    hipEvent_t e0 = prof_event(ctx), e1 = prof_event(ctx);
    GBT_REQUIRE(ctx, e0 && e1, GBT_EHIP, "hipEventCreate failed");
    double best_ms = 0.0;
    int32_t st = GBT_OK;
    for (int32_t r = 0; r <= reps && st == GBT_OK; ++r) {   // the first launch warms up and is not counted
        hipError_t e = hipEventRecord(e0, ctx->stream);
        if (e == hipSuccess) e = gbt_launch_stream_read(ctx->stream, buf, (int64_t)bytes, (uint32_t *)workspace);
        if (e == hipSuccess) e = hipEventRecord(e1, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) st = gbt_fail(ctx, GBT_EHIP, "gbt_measure_stream_read: %s", hipGetErrorString(e));
        else if (r > 0 && (best_ms == 0.0 || ms < best_ms)) best_ms = ms;
    }
    ctx->free_events->push_back(e0);
    ctx->free_events->push_back(e1);
    if (st != GBT_OK) return st;
    *gbps_out = best_ms > 0.0 ? (double)(bytes / 16 * 16) / (best_ms * 1e-3) / 1e9 : 0.0;
    return GBT_OK;
}

// ------------------------------------------------------------- compression --
extern "C" int32_t gbt_bits(uint32_t max_value) {
    int32_t b = 1;
    while (b < 32 && (max_value >> b) != 0) ++b;
    return b;
}

extern "C" int64_t gbt_packed_words(int64_t n, int32_t F, int32_t bits) {
    if (n < 0 || F < 0 || bits < 1) return -1;
    return (n * (int64_t)F * bits + 31) / 32 + 1;
}

extern "C" int32_t gbt_compress(gbt_ctx *ctx, const uint16_t *sym, int64_t n, int32_t F, uint32_t max_value,
                                uint32_t *packed_out, int32_t *bits_out) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, n >= 0 && F >= 1, GBT_EINVAL, "bad shape");
    GBT_REQUIRE(ctx, (sym || n == 0) && packed_out && bits_out, GBT_EINVAL, "NULL argument");
    int32_t bits = gbt_bits(max_value);
    GBT_REQUIRE(ctx, bits <= GBT_MAX_BITS, GBT_EUNSUPPORTED, "max_value %u needs %d bits", max_value, bits);
    GBT_HIP(ctx, gbt_launch_compress(ctx->stream, sym, n * (int64_t)F, bits, packed_out,
                                     gbt_packed_words(n, F, bits)));
    *bits_out = bits;
    return GBT_OK;
}

// --------------------------------------------------------------- gradients --
extern "C" int32_t gbt_gradients(gbt_ctx *ctx, int32_t objective, const float *margin, const float *label,
                                 int64_t n, float *gpair_out) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, n >= 0, GBT_EINVAL, "n < 0");
    GBT_REQUIRE(ctx, n == 0 || (margin && label && gpair_out), GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, objective == GBT_OBJ_SQUARED || objective == GBT_OBJ_LOGISTIC, GBT_EINVAL,
                "unknown objective %d", objective);
    GBT_HIP(ctx, gbt_launch_gradients(ctx->stream, objective, margin, label, n, gpair_out));
    return GBT_OK;
}

// ------------------------------------------------------- fixed-point gpair --
// The scales alone (one pass for the largest |g| and h; synchronises).
// uniform_h (may be NULL): receives 1 and the common value when every row has the same |h| (n >= 1), else 0.
// bounds_dev (may be NULL): the four words gbt_launch_absmax would find, already on the device (left there by
// gbt_launch_gradients when the same call made the pairs)
static int32_t gpair_scale_impl(gbt_ctx *ctx, const float *gpair, int64_t n, double *scale, void *ws,
                                int *uniform_h = nullptr, float *h_value = nullptr, const uint32_t *bounds_dev = nullptr) {
    if (!bounds_dev) GBT_HIP(ctx, gbt_launch_absmax(ctx->stream, gpair, n, (uint32_t *)ws));
    const int stride = bounds_dev ? kBoundsStride : 1;   // (gbt_launch_gradients keeps its four words on lines of their own)
    GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), bounds_dev ? (const void *)bounds_dev : (const void *)ws, (3 * stride + 1) * 4,
                                hipMemcpyDeviceToHost, ctx->stream));
    GBT_SYNC(ctx);
    uint32_t bits2[4];
    for (int k = 0; k < 4; ++k) memcpy(&bits2[k], rb(ctx) + (size_t)k * stride * 4, 4);
    GBT_REQUIRE(ctx, bits2[0] < 0x7f800000u && bits2[1] < 0x7f800000u, GBT_EINVAL,
                "gradient pairs contain a non-finite value");
    GBT_REQUIRE(ctx, bits2[2] == 0, GBT_EINVAL, "gradient pairs contain a negative hessian");
    float mg, mh;
    memcpy(&mg, &bits2[0], 4);
    memcpy(&mh, &bits2[1], 4);
    scale[0] = fixed_scale(mg, kGBits);
    scale[1] = fixed_scale(mh, kHBits);
    if (uniform_h) {
        *uniform_h = n >= 1 && ~bits2[3] == bits2[1];   // smallest |h| == largest |h| (and none is negative)
        if (h_value) *h_value = mh;
    }
    return GBT_OK;
}

static int32_t gpair_fixed_impl(gbt_ctx *ctx, const float *gpair, int64_t n, int32_t *gq, double *scale,
                                void *ws, int64_t *sums_dev /* may be NULL */) {
    int32_t st = gpair_scale_impl(ctx, gpair, n, scale, ws);
    if (st != GBT_OK) return st;
    GBT_HIP(ctx, gbt_launch_to_fixed(ctx->stream, gpair, n, scale[0], scale[1], gq, sums_dev));
    return GBT_OK;
}

extern "C" int32_t gbt_gpair_fixed(gbt_ctx *ctx, const float *gpair, int64_t n, int32_t *gq_out,
                                   double *scale_out, void *workspace, size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, gpair && gq_out && scale_out && workspace, GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, n >= 0, GBT_EINVAL, "n < 0");
    GBT_REQUIRE(ctx, workspace_bytes >= 4096, GBT_ENOMEM, "workspace < 4096 bytes");
    int32_t st = gpair_fixed_impl(ctx, gpair, n, gq_out, scale_out, workspace, nullptr);
    if (st != GBT_OK) return st;
    GBT_SYNC(ctx);
    return GBT_OK;
}

extern "C" int32_t gbt_sum_gpair(gbt_ctx *ctx, const int32_t *gq, const uint32_t *row_idx, int64_t n_rows,
                                 int64_t *sums_out, void *workspace, size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, gq && sums_out && workspace, GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, n_rows >= 0, GBT_EINVAL, "n_rows < 0");
    GBT_REQUIRE(ctx, workspace_bytes >= 4096, GBT_ENOMEM, "workspace < 4096 bytes");
    GBT_HIP(ctx, gbt_launch_sum_gq(ctx->stream, gq, row_idx, n_rows, (int64_t *)workspace));
    GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), workspace, 16, hipMemcpyDeviceToHost, ctx->stream));
    GBT_SYNC(ctx);
    memcpy(sums_out, rb(ctx), 16);
    return GBT_OK;
}

// --------------------------------------------------------------- histogram --
// Enqueues the histogram of one row range split uniformly into jobs that the
// kernel derives from its block index (no job table).
struct RootFix {   // the root histogram converts the fp32 pairs itself (gbt_launch_hist_fix, gbt_launch_hist8)
    const float *gpair;
    double sg, sh;
    int32_t *gq_out;      // where the rounded pairs go (gbt_launch_hist8: may be NULL)
    int64_t *sums_dev;
    int uniform_h;        // every row has the same hessian ...
    int32_t hq_uniform;   // ... this one, rounded
    // gbt_launch_hist8 leaves the totals as one pair per workgroup: where (room for gbt_hist8_max_jobs() pairs), and,
    // on return, how many (0: the totals are in sums_dev as one pair)
    int64_t *slot_sums;
    int n_slots;
};
static int32_t hist_uniform(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                            int32_t B, int32_t missing_sym, const uint32_t *row_idx, int64_t n_rows,
                            const int32_t *gq, int64_t *hist_out, HistJob *dev_jobs /* may be NULL */,
                            RootFix *fix = nullptr, bool uniform_h = false, int32_t hq_uniform = 0);

extern "C" int32_t gbt_build_hist(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                                  int32_t B, int32_t missing_sym, const uint32_t *row_idx,
                                  int64_t n_node_rows, const int32_t *gq, int64_t *hist_out) {
    if (!ctx) return GBT_EINVAL;
    int32_t st = check_matrix(ctx, packed, bits, n, F);
    if (st != GBT_OK) return st;
    st = check_bins(ctx, F, B);
    if (st != GBT_OK) return st;
    GBT_REQUIRE(ctx, gq && hist_out, GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, missing_sym >= 0, GBT_EINVAL, "missing_sym < 0");
    int64_t rows = row_idx ? n_node_rows : n;
    GBT_REQUIRE(ctx, rows >= 0 && rows <= n, GBT_EINVAL, "n_node_rows = %lld out of range", (long long)rows);
    return hist_uniform(ctx, packed, bits, n, F, B, missing_sym, row_idx, rows, gq, hist_out, nullptr);
}

extern "C" int32_t gbt_hist_subtract(gbt_ctx *ctx, const int64_t *parent, const int64_t *child, int64_t *out,
                                     int64_t count) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, parent && child && out, GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, count >= 0, GBT_EINVAL, "count < 0");
    GBT_HIP(ctx, gbt_launch_subtract_one(ctx->stream, parent, child, out, count));
    return GBT_OK;
}

extern "C" int32_t gbt_hist_export_f64(gbt_ctx *ctx, const int64_t *hist, int32_t F, int32_t B,
                                       const double *scale, double *out) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, hist && scale && out, GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, F >= 1 && B >= 1, GBT_EINVAL, "bad shape");
    GBT_REQUIRE(ctx, scale[0] > 0 && scale[1] > 0, GBT_EINVAL, "scale must be positive");
    GBT_HIP(ctx, gbt_launch_export(ctx->stream, hist, (int64_t)F * B * 2, 1.0 / scale[0], 1.0 / scale[1], out));
    return GBT_OK;
}

// ------------------------------------------------------------------- split --
extern "C" int32_t gbt_eval_split(gbt_ctx *ctx, const int64_t *hist, const int32_t *nb, int32_t F, int32_t B,
                                  int64_t Gq, int64_t Hq, const double *scale, const gbt_params *params,
                                  gbt_split *split_out, void *workspace, size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, hist && nb && scale && params && split_out && workspace, GBT_EINVAL, "NULL argument");
    int32_t st = check_bins(ctx, F, B);
    if (st != GBT_OK) return st;
    GBT_REQUIRE(ctx, F >= 1, GBT_EINVAL, "F < 1");
    GBT_REQUIRE(ctx, workspace_bytes >= 4096, GBT_ENOMEM, "workspace < 4096 bytes");
    GBT_REQUIRE(ctx, scale[0] > 0 && scale[1] > 0, GBT_EINVAL, "scale must be positive");
    EvalNode nd;
    nd.hist_off = 0;
    nd.Gq = Gq;
    nd.Hq = Hq;
    nd.parent_off = nd.built_off = GBT_NO_HIST;
    char *ws = (char *)workspace;
    st = upload(ctx, &nd, sizeof nd, ws);
    if (st != GBT_OK) return st;
    gbt_split *dsplit = (gbt_split *)(ws + 256);
    const int chunks = gbt_eval_chunks(F, 1, workspace_bytes - 256);
    GBT_HIP(ctx, gbt_launch_eval(ctx->stream, const_cast<int64_t *>(hist), (const EvalNode *)ws, 1, nb, F, B, chunks, 1.0 / scale[0],
                                 1.0 / scale[1], params->lambda, params->min_child_weight, dsplit));
    GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), dsplit, chunks * sizeof(gbt_split), hipMemcpyDeviceToHost, ctx->stream));
    GBT_SYNC(ctx);
    *split_out = merge_chunks((const gbt_split *)rb(ctx), chunks);
    return GBT_OK;
}

// --------------------------------------------------------------- partition --
namespace {
struct PartLayout {
    size_t dst, masks, tile_left, jobs, n_left, total;
};
constexpr PartLayout part_layout(int64_t n_rows) {
    PartLayout L{};
    int64_t tiles = (n_rows + GBT_PART_TILE - 1) / GBT_PART_TILE + 1;
    size_t o = 0;
    L.dst = o;       o += gbt_align((size_t)n_rows * 4);
    L.masks = o;     o += gbt_align((size_t)tiles * (GBT_PART_TILE / 64) * 8);
    L.tile_left = o; o += gbt_align((size_t)tiles * 4);
    L.jobs = o;      o += gbt_align(sizeof(PartJob));
    L.n_left = o;    o += gbt_align(4);
    L.total = o;
    return L;
}

// The stable three-launch partition of one segment over the scratch memory `ws` (part_layout(len).total
// bytes, none of which has to hold anything on entry: every word a launch reads, an earlier launch of the
// same call has written).
int32_t partition_impl(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F, uint32_t *row_idx,
                       int64_t begin, int64_t end, int32_t feature, int32_t bin, int32_t default_left,
                       int32_t missing_sym, char *ws, int64_t *n_left_out) {
    const int64_t len = end - begin;
    const PartLayout L = part_layout(len);
    PartJob job;
    job.seg_begin = 0;
    job.seg_len = (uint32_t)len;
    job.feature = (uint32_t)feature;
    job.bin = (uint32_t)bin;
    job.default_left = default_left ? 1u : 0u;
    job.tile_begin = 0;
    job.n_tiles = (uint32_t)((len + GBT_PART_TILE - 1) / GBT_PART_TILE);
    job.pad = 0;
    int32_t st = upload(ctx, &job, sizeof job, ws + L.jobs);
    if (st != GBT_OK) return st;
    uint32_t *seg = row_idx + begin;
    GBT_HIP(ctx, gbt_launch_partition(ctx->stream, packed, bits, (int64_t)F * bits, n, (uint32_t)missing_sym, seg,
                                      (uint32_t *)(ws + L.dst), (const PartJob *)(ws + L.jobs), 1,
                                      (int)job.n_tiles, (uint64_t *)(ws + L.masks),
                                      (uint32_t *)(ws + L.tile_left), (uint32_t *)(ws + L.n_left)));
    GBT_HIP(ctx, hipMemcpyAsync(seg, ws + L.dst, (size_t)len * 4, hipMemcpyDeviceToDevice, ctx->stream));
    GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), ws + L.n_left, 4, hipMemcpyDeviceToHost, ctx->stream));
    GBT_SYNC(ctx);
    uint32_t nl;
    memcpy(&nl, rb(ctx), 4);
    *n_left_out = nl;
    return GBT_OK;
}

int32_t check_partition_args(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                             const uint32_t *row_idx, int64_t begin, int64_t end, int32_t feature, int32_t bin,
                             int32_t missing_sym, const int64_t *n_left_out) {
    int32_t st = check_matrix(ctx, packed, bits, n, F);
    if (st != GBT_OK) return st;
    GBT_REQUIRE(ctx, row_idx && n_left_out, GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, 0 <= begin && begin <= end && end - begin <= n, GBT_EINVAL, "bad segment [%lld, %lld)",
                (long long)begin, (long long)end);
    GBT_REQUIRE(ctx, feature >= 0 && feature < F, GBT_EINVAL, "feature %d outside [0, %d)", feature, F);
    GBT_REQUIRE(ctx, bin >= 0 && missing_sym >= 0, GBT_EINVAL, "negative bin or missing symbol");
    return GBT_OK;
}
}  // namespace

extern "C" size_t gbt_partition_workspace_bytes(int64_t n_rows) {
    return n_rows < 0 ? 0 : part_layout(n_rows).total;
}

extern "C" int32_t gbt_partition(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                                 uint32_t *row_idx, int64_t begin, int64_t end, int32_t feature, int32_t bin,
                                 int32_t default_left, int32_t missing_sym, void *workspace,
                                 size_t workspace_bytes, int64_t *n_left_out) {
    if (!ctx) return GBT_EINVAL;
    int32_t st = check_partition_args(ctx, packed, bits, n, F, row_idx, begin, end, feature, bin, missing_sym, n_left_out);
    if (st != GBT_OK) return st;
    GBT_REQUIRE(ctx, workspace != nullptr, GBT_EINVAL, "NULL argument");
    const size_t need = part_layout(end - begin).total;
    GBT_REQUIRE(ctx, workspace_bytes >= need, GBT_ENOMEM, "workspace %zu < %zu bytes", workspace_bytes, need);
    if (end == begin) {
        *n_left_out = 0;
        return GBT_OK;
    }
    return partition_impl(ctx, packed, bits, n, F, row_idx, begin, end, feature, bin, default_left, missing_sym,
                          (char *)workspace, n_left_out);
}

// ---- the same partition for callers that cannot allocate ------------------------------------------
// Its scratch memory (ballot masks, tile counts, the reordered ids) is a static device array instead of
// a caller workspace.  In host code the array's name is only a stand-in: the address a kernel can use
// is asked for once per device, with that device current (gbt_create does it), and kept.
namespace {
constexpr size_t kPartStaticBytes = part_layout(GBT_PARTITION_STATIC_MAX_ROWS).total;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kPartStaticBytes];
namespace {
char *g_part_static[kMaxDevices];   // per device: the address of its copy of `scratch`
std::mutex g_part_static_mu;

// Called with `device` current.  Returns hipSuccess and the device's address of the array.
hipError_t part_static_address(int device, char **out) {
    *out = nullptr;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_part_static_mu);
    if (!g_part_static[device]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_part_static[device] = (char *)p;
    }
    *out = g_part_static[device];
    return hipSuccess;
}
}  // namespace

extern "C" int32_t gbt_partition_static(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                                        uint32_t *row_idx, int64_t begin, int64_t end, int32_t feature,
                                        int32_t bin, int32_t default_left, int32_t missing_sym,
                                        int64_t *n_left_out) {
    if (!ctx) return GBT_EINVAL;
    int32_t st = check_partition_args(ctx, packed, bits, n, F, row_idx, begin, end, feature, bin, missing_sym, n_left_out);
    if (st != GBT_OK) return st;
    GBT_REQUIRE(ctx, end - begin <= (int64_t)GBT_PARTITION_STATIC_MAX_ROWS, GBT_EUNSUPPORTED,
                "segment of %lld rows exceeds the static scratch of gbt_partition_static (%lld rows): use gbt_partition",
                (long long)(end - begin), (long long)GBT_PARTITION_STATIC_MAX_ROWS);
    GBT_REQUIRE(ctx, ctx->part_static != nullptr, GBT_EHIP, "the static scratch array has no address on device %d",
                ctx->device);
    if (end == begin) {
        *n_left_out = 0;
        return GBT_OK;
    }
    return partition_impl(ctx, packed, bits, n, F, row_idx, begin, end, feature, bin, default_left, missing_sym,
                          ctx->part_static, n_left_out);
}

// ------------------------------------------------------------ histogram job --
static int32_t hist_uniform(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                            int32_t B, int32_t missing_sym, const uint32_t *row_idx, int64_t n_rows,
                            const int32_t *gq, int64_t *hist_out, HistJob *dev_jobs, RootFix *fix, bool uniform_h,
                            int32_t hq_uniform) {
    HistPlan pl;
    GBT_REQUIRE(ctx, plan_tiles(ctx, F, B, bits, &pl, n_rows), GBT_EUNSUPPORTED,
                "max_bins = %d: one feature's bins (%d bytes) exceed the LDS budget", B, B * 16);
    GBT_HIP(ctx, gbt_launch_fill_u64(ctx->stream, (uint64_t *)hist_out, 0, (int64_t)F * B * 2));
    if (n_rows == 0) return GBT_OK;
    if (ctx->hist8 && !row_idx && n_rows == n && gbt_hist8_ok(bits, F, pl.n_ftiles, n, gbt_packed_words(n, F, bits))) {
        Hist8Pairs p{};
        if (fix) {
            p.gpair = fix->gpair;
            p.gq_out = fix->gq_out;
            p.sg = fix->sg;
            p.sh = fix->sh;
            p.mode = gbt_fix32_ok(fix->sg, fix->sh) ? 2 : 1;
            p.uniform_h = fix->uniform_h;
            p.hq_uniform = fix->hq_uniform;
            p.sums = fix->slot_sums;
        } else {
            p.gq = gq;
        }
        int n_jobs8 = 0;
        gbt_prof_begin(ctx, GBT_PROF_HIST_ROOT, (double)n_rows * ((double)F * bits / 8.0 + 8.0), -1.0, 0, (double)n_rows * F);
        GBT_HIP(ctx, gbt_launch_hist8(ctx, packed, n, F, B, (uint32_t)missing_sym, p, hist_out, &n_jobs8));
        gbt_prof_end(ctx);
        if (fix) fix->n_slots = n_jobs8;
        return GBT_OK;
    }
    std::vector<HistJob> jobs;
    const bool uni_w = uniform_h && bits != 8 && !ctx->hist_runtime_bits;   // the kernels with a row-count form
    add_hist_jobs(jobs, 0, 0, (uint32_t)n_rows, F, pl,
                  pick_rows_per_job(ctx, n_rows, gbt_histw_max_rows(uni_w), pl.n_ftiles, B),
                  ((uintptr_t)hist_out & 15u) == 0);
    // Without a caller workspace the job table is read straight from the pinned
    // staging, which the device can address; it is small (a few KB).
    size_t bytes = jobs.size() * sizeof(HistJob);
    if (dev_jobs) {
        int32_t st = upload(ctx, jobs.data(), bytes, dev_jobs);
        if (st != GBT_OK) return st;
    } else {
        char *slot;
        int32_t st = stage(ctx, jobs.data(), bytes, &slot);
        if (st != GBT_OK) return st;
        dev_jobs = (HistJob *)slot;
    }
    gbt_prof_begin(ctx, row_idx ? GBT_PROF_HIST_NODE : GBT_PROF_HIST_ROOT,
                   (double)n_rows * ((double)F * bits / 8.0 + 8.0 + (row_idx ? 4.0 : 0.0)), -1.0, row_idx ? -1 : 0,
                   (double)n_rows * F);
    if (fix)
        GBT_HIP(ctx, gbt_launch_hist_fix(ctx, packed, (int64_t)F * bits, gbt_packed_words(n, F, bits), n, B,
                                         (uint32_t)missing_sym, fix->gpair, fix->sg, fix->sh, fix->gq_out,
                                         fix->sums_dev, hist_out, dev_jobs, (int)jobs.size(), pl.ft));
    else
        GBT_HIP(ctx, gbt_launch_hist(ctx, packed, bits, (int64_t)F * bits, gbt_packed_words(n, F, bits), n, B,
                                     (uint32_t)missing_sym, row_idx, gq, hist_out, dev_jobs, (int)jobs.size(), pl.ft,
                                     uni_w, hq_uniform));
    gbt_prof_end(ctx);
    return GBT_OK;
}

// -------------------------------------------------------------------- grow --
namespace {

struct GrowLayout {
    size_t tree_stage, tree_stage_bytes, gq, wsym[2], wgq[2], wid[2], masks, tile_left, n_left, state, pool, eval_nodes, jobs, scratch, order, rank_tbl, node_rows, total;
    int64_t hist_nodes, level_nodes, tiles, w_words;
    int sw;   // 32-bit words per row of the working copies
};

// hist_nodes: nodes that may own a histogram (ids below it); level_nodes: most nodes split in one round
GrowLayout grow_layout_nodes(int64_t n, int F, int bits, int B, int64_t hist_nodes, int64_t level_nodes);
GrowLayout grow_layout(int64_t n, int F, int bits, int B, int max_depth) {
    return grow_layout_nodes(n, F, bits, B, max_depth == 0 ? 1 : (((int64_t)1 << max_depth) - 1),
                             (int64_t)1 << (max_depth > 0 ? max_depth - 1 : 0));
}
GrowLayout grow_layout_nodes(int64_t n, int F, int bits, int B, int64_t hist_nodes, int64_t level_nodes) {
    GrowLayout L;
    L.hist_nodes = hist_nodes;
    L.level_nodes = level_nodes;
    L.tiles = n / GBT_PART_TILE + L.level_nodes + 1;
    L.sw = (int)(((int64_t)F * bits + 31) / 32);
    // the partition + histogram pass keeps symbols and gradient pair in one record per row
    const int rw = (bits == 8 && F <= 16) ? gbt_part_hist_record_words(F) : 0;
    L.w_words = n * std::max(L.sw, rw) + 4;
    size_t o = 0;
    L.gq = o;         o += gbt_align((size_t)n * 8);
    for (int k = 0; k < 2; ++k) {
        L.wsym[k] = o; o += gbt_align((size_t)L.w_words * 4);
        L.wgq[k] = o;  o += gbt_align((size_t)n * 8);
        L.wid[k] = o;  o += gbt_align((size_t)n * 4);
    }
    L.masks = o;      o += gbt_align((size_t)L.tiles * (GBT_PART_TILE / 64) * 8);
    L.tile_left = o;  o += gbt_align((size_t)L.tiles * 4);
    L.n_left = o;     o += gbt_align((size_t)L.level_nodes * 4 + 4);
    L.state = o;      o += gbt_align((size_t)L.level_nodes * 8 * kCursorStride);
    L.pool = o;       o += gbt_align((size_t)L.hist_nodes * F * B * 16);
    L.eval_nodes = o; o += gbt_align((size_t)L.level_nodes * 2 * sizeof(EvalNode));
    L.jobs = o;       o += gbt_align(kUploadBytes);
    L.scratch = o;    o += 4096;
    // room to stage the finished tree for a walk (as gbt_predict_workspace_bytes counts it); a tree has
    // at most 2 * hist_nodes + 1 nodes under either policy
    const size_t cap_nodes = (size_t)(2 * hist_nodes + 1);
    L.tree_stage_bytes = gbt_align(64) + gbt_align(cap_nodes * 4) * 6 + gbt_align(cap_nodes * 8) + 256;
    L.tree_stage = o; o += gbt_align(L.tree_stage_bytes);
    // row ids in leaf order after a growth that did not follow the rows
    L.order = o;      o += gbt_order_ws(n);
    L.rank_tbl = o;   o += gbt_align(cap_nodes * 4);
    // one row counter per node, a 128-byte line each, for the walk that also counts (trees small enough for it)
    L.node_rows = o;  o += gbt_align(std::min<size_t>(cap_nodes, 8192) * kNodeRowsStride * 4);
    L.total = o;
    return L;
}

struct HNode {
    int32_t id;
    uint32_t begin, len;
    int64_t Gq, Hq;
    int32_t depth;
    int32_t buf;   // where the node's rows are: 0/1 = working copy, 2 = the caller's matrix (the root)
    // virt >= 0: the node's rows were not moved when it was made: they lie interleaved with other nodes' rows
    // in segment `virt` of the table of such segments, where the node has heap position vpos below the
    // segment's own split (1, 2: its children; 3..6: its grandchildren)
    int32_t virt = -1, vpos = 0;
    // >= 0: the node's histogram is still to be made as parent - built (pool slots) when it is evaluated
    int32_t sub_parent = -1, sub_built = -1;
};
struct UnmovedSeg {   // a segment whose rows stay in place below its own split, and the splits made there since
    uint32_t begin, len;
    int32_t buf;
    uint32_t feature[7], bin[7], default_left[7], has[7];   // heap order, as in CountJob
    void set(int p, const gbt_split &sp) {
        feature[p] = (uint32_t)sp.feature;
        bin[p] = (uint32_t)sp.bin;
        default_left[p] = (uint32_t)sp.default_left;
        has[p] = 1;
    }
};
enum { GBT_POLICY_DEPTHWISE = 0, GBT_POLICY_LOSSGUIDE = 1 };
constexpr int32_t kMaxLeaves = 1 << 20;
// Loss-guided growth expands a few open leaves per round ahead of their turn (see grow_impl): nodes
// created that way need histogram slots even if the leaf budget ends before they are reached.
constexpr int kLossguideBatchMax = 32;
int64_t lossguide_phys_nodes(int32_t max_leaves) {
    const int64_t slack = std::min<int64_t>(std::max<int64_t>(max_leaves / 4, 32), 4096);   // expansions that may go unused
    return 2 * (int64_t)max_leaves - 1 + 2 * slack;
}

}  // namespace

extern "C" size_t gbt_grow_tree_workspace_bytes(int64_t n, int32_t F, int32_t bits, int32_t max_bins,
                                                int32_t max_depth) {
    if (n < 0 || F < 1 || bits < 1 || bits > GBT_MAX_BITS || max_bins < 2 || max_depth < 0 || max_depth > kMaxDepth)
        return 0;
    return grow_layout(n, F, bits, max_bins, max_depth).total;
}

namespace {
// the working copies' row stride for a shape (rows start on 32-bit word boundaries)
GbtRows working_rows_shape(int F, int bits) {
    GbtRows r{};
    r.stride_bits = 32 * (((int64_t)F * bits + 31) / 32);
    return r;
}
int grow_path(const gbt_ctx *ctx, int F, int bits, int B, bool tracked, int n_ftiles) {
    const GbtRows w = working_rows_shape(F, bits);
    // rows too wide to be worth moving: they stay where they are and only their ids are partitioned
    if (!gbt_partition_fused_ok(w) || (w.stride_bits >> 5) > ctx->move_max_words) return ctx->part_ids ? 3 : 0;
    if ((tracked && !ctx->order_rows) || !ctx->part_fused) return 0;
    if (ctx->part_hist && n_ftiles == 1 && gbt_part_hist_ok(ctx, bits, F, B)) return 2;
    return 1;
}
}  // namespace

extern "C" int32_t gbt_grow_tree_path(gbt_ctx *ctx, int32_t F, int32_t bits, int32_t max_bins, int32_t track_rows) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, F >= 1 && bits >= 1 && bits <= GBT_MAX_BITS && max_bins >= 2, GBT_EINVAL, "bad shape");
    HistPlan pl;
    GBT_REQUIRE(ctx, plan_tiles(ctx, F, max_bins, bits, &pl), GBT_EUNSUPPORTED,
                "max_bins = %d: one feature's bins exceed the LDS budget", max_bins);
    return grow_path(ctx, F, bits, max_bins, track_rows != 0, pl.n_ftiles);
}

struct SparseRowsArg {   // rows in the sparse form instead of packed / X
    const uint32_t *rowptr;
    const void *ent;
    int32_t ent_bytes;
    int32_t B;
};
static int32_t predict_impl(gbt_ctx *ctx, const gbt_tree *trees, int32_t n_trees, const uint32_t *packed,
                            int32_t bits, int32_t missing_sym, const float *X, int64_t n, int32_t F, double eta,
                            float *margin, int32_t *leaf_out, void *workspace, size_t workspace_bytes,
                            const SparseRowsArg *sparse = nullptr, bool own_span = false, uint32_t *node_rows = nullptr,
                            const float *margin_src = nullptr);

// Alg. 1 under either policy of Sec. 2.3.  Growth proceeds in rounds: the nodes created by the round
// before are evaluated; depth-wise then splits every one of them that may split, loss-guided only
// the open leaf with the largest gain (smaller id on equal gains), however long ago it was created.
static int32_t grow_impl(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                         int32_t missing_sym, const int32_t *nb, const float *cuts, const float *gpair,
                         const gbt_params *params, int policy, int32_t max_leaves, gbt_tree *tree,
                         uint32_t *row_idx_out, int32_t *leaf_of_row_out, void *workspace, size_t workspace_bytes,
                         float *margin_update = nullptr, const float *margin_src = nullptr,
                         const uint32_t *bounds_dev = nullptr) {
    // margin_update (may be NULL): margin_update[r] = margin_src[r] + eta * (weight of r's leaf), by a walk of the
    // finished tree (margin_src NULL: margin_update itself)
    // bounds_dev (may be NULL): see gpair_scale_impl
    if (!ctx) return GBT_EINVAL;
    int32_t st = check_matrix(ctx, packed, bits, n, F);
    if (st != GBT_OK) return st;
    GBT_REQUIRE(ctx, nb && cuts && gpair && params && tree && workspace, GBT_EINVAL, "NULL argument");
    const bool tracked = row_idx_out != nullptr;   // else row ids are not carried along
    const int B = params->max_bins, max_depth = params->max_depth;
    st = check_bins(ctx, F, B);
    if (st != GBT_OK) return st;
    const bool lossguide = policy == GBT_POLICY_LOSSGUIDE;
    GBT_REQUIRE(ctx, max_depth >= 0, GBT_EINVAL, "max_depth < 0");
    GBT_REQUIRE(ctx, lossguide || max_depth <= kMaxDepth, GBT_EUNSUPPORTED, "max_depth %d > %d", max_depth, kMaxDepth);
    GBT_REQUIRE(ctx, !lossguide || (max_leaves >= 1 && max_leaves <= kMaxLeaves), lossguide && max_leaves >= 1 ? GBT_EUNSUPPORTED : GBT_EINVAL,
                "max_leaves %d outside 1..%d", max_leaves, kMaxLeaves);
    GBT_REQUIRE(ctx, n >= 1, GBT_EINVAL, "n < 1");
    GBT_REQUIRE(ctx, missing_sym >= 0, GBT_EINVAL, "missing_sym < 0");
    GBT_REQUIRE(ctx, params->lambda >= 0.0, GBT_EINVAL, "lambda < 0");
    const int64_t cap = lossguide ? 2 * (int64_t)max_leaves - 1 : ((int64_t)1 << (max_depth + 1)) - 1;
    GBT_REQUIRE(ctx, tree->capacity >= cap, GBT_EINVAL, "tree capacity %d < %lld", tree->capacity, (long long)cap);
    GBT_REQUIRE(ctx, tree->feature && tree->bin && tree->default_left && tree->left && tree->right &&
                         tree->threshold && tree->weight && tree->gain && tree->sumG && tree->sumH && tree->n_rows,
                GBT_EINVAL, "tree arrays must be allocated");
    const int64_t cap_phys = lossguide ? lossguide_phys_nodes(max_leaves) : cap;
    const GrowLayout L = lossguide ? grow_layout_nodes(n, F, bits, B, cap_phys, kLossguideBatchMax)
                                   : grow_layout(n, F, bits, B, max_depth);
    GBT_REQUIRE(ctx, workspace_bytes >= L.total, GBT_ENOMEM, "workspace %zu < %zu bytes", workspace_bytes, L.total);
    HistPlan pl;
    GBT_REQUIRE(ctx, plan_tiles(ctx, F, B, bits, &pl, n), GBT_EUNSUPPORTED,
                "max_bins = %d: one feature's bins exceed the LDS budget", B);

    char *ws = (char *)workspace;
    int32_t *gq = (int32_t *)(ws + L.gq);
    int64_t *pool = (int64_t *)(ws + L.pool);
    const int64_t hist_len = (int64_t)F * B * 2;
    const int row_bits = F * bits;
    hipStream_t s = ctx->stream;

    // The rows in their current order.  Level 0 reads the caller's packed matrix; every
    // partition then moves whole records (symbols, gradient pair, id) into the other of two
    // word-aligned working copies, so that each node's rows stay contiguous.
    const int path = grow_path(ctx, F, bits, B, tracked, pl.n_ftiles);
    GbtRows W[2];
    for (int k = 0; k < 2; ++k) {
        W[k].sym_rw = (uint32_t *)(ws + L.wsym[k]);
        W[k].gq_rw = (int32_t *)(ws + L.wgq[k]);
        W[k].id_rw = (uint32_t *)(ws + L.wid[k]);
        W[k].sym = W[k].sym_rw;
        W[k].gq = W[k].gq_rw;
        W[k].id = W[k].id_rw;
        W[k].stride_bits = 32 * (int64_t)L.sw;
        W[k].n_words = L.w_words;
        if (path == 2) {   // records: the pair travels inside the row (only symbols are read from outside)
            W[k].stride_bits = 32 * (int64_t)gbt_part_hist_record_words(F);
            W[k].gq = nullptr;
            W[k].gq_rw = nullptr;
        }
    }
    GbtRows matrix;   // the caller's matrix seen as "buffer 2": rows in matrix order, ids = positions
    matrix.sym = packed;
    matrix.stride_bits = row_bits;
    matrix.n_words = gbt_packed_words(n, F, bits);
    matrix.gq = gq;
    matrix.id = nullptr;
    matrix.sym_rw = nullptr;
    matrix.gq_rw = nullptr;
    matrix.id_rw = nullptr;

    // thresholds come from the cut table: it travels through the part of the pinned read-back buffer that
    // the split records use later, and is picked up behind the first wait below (a copy into pageable
    // memory would be a wait of its own); a table too large for that is copied directly
    std::vector<float> hcuts((size_t)F * (B - 1));
    constexpr size_t kCutsRb = 512u << 10;   // (= where the split records go, see kSplitRb)
    const bool cuts_via_pinned = hcuts.size() * sizeof(float) <= GBT_STAGING_BYTES - kReadbackOff - kCutsRb;
    GBT_HIP(ctx, hipMemcpyAsync(cuts_via_pinned ? (void *)(rb(ctx) + kCutsRb) : (void *)hcuts.data(), cuts,
                                hcuts.size() * sizeof(float), hipMemcpyDeviceToHost, s));

    // Fixed-point gradient pairs and the root's totals: the scales need one pass over the pairs;
    // the conversion is a pass of its own, or part of the root histogram kernel where that can do it.
    double scale[2];
    int64_t *sums_dev = (int64_t *)(ws + L.scratch + 256);
    const bool root_may_split = max_depth > 0 && (!lossguide || max_leaves > 1);
    // With a margin to update the finished tree is walked over all rows anyway; that walk can count the rows of
    // every node, so the children of the last level (leaves, of which only the row counts are wanted) need no
    // counting pass of their own.
    const bool defer_counts = margin_update && !tracked && !leaf_of_row_out && !lossguide && (path == 1 || path == 2) &&
                              cap <= 8192 && gbt_predict_counts_ok(true, bits, F, (int)cap, true);
    std::vector<int32_t> deferred_children;
    const bool fix_in_hist = ctx->hist_fix && root_may_split && gbt_hist_fix_ok(bits, row_bits, pl.ft, pl.n_ftiles);
    int uniform_h = 0;
    float h_value = 0.0f;
    gbt_prof_begin(ctx, GBT_PROF_OTHER, (double)n * (fix_in_hist ? 8.0 : 24.0));
    st = gpair_scale_impl(ctx, gpair, n, scale, ws + L.scratch, &uniform_h, &h_value, bounds_dev);
    if (st == GBT_OK && !fix_in_hist) {
        hipError_t e = gbt_launch_to_fixed(s, gpair, n, scale[0], scale[1], gq, sums_dev);
        if (e != hipSuccess) st = gbt_fail(ctx, GBT_EHIP, "gbt_launch_to_fixed: %s", hipGetErrorString(e));
    }
    gbt_prof_end(ctx);
    if (st != GBT_OK) return st;
    const double inv_sg = 1.0 / scale[0], inv_sh = 1.0 / scale[1];
    const double lambda = params->lambda;
    const double min_gain = std::max(params->gamma, (double)GBT_GAIN_FLOOR);
    // every row has the same hessian (squared error always, the first tree of a logistic model): the passes over rows
    // that stay in place then keep a row count per bin instead of a hessian sum (>= 0: that hessian in fixed point)
    const int hq_uni = uniform_h ? (int)llrint((double)h_value * scale[1]) : -1;
    if (path == 3 && root_may_split)   // the root's id list, read by the first partition
        GBT_HIP(ctx, gbt_launch_iota_u32(s, W[1].id_rw, n));
    // Where the partition + histogram pass follows (path 2) and rounding in fp32 is exact, the fixed-point pairs
    // are never stored: the root histogram and the first pass each round the fp32 pairs themselves, and from
    // then on a row's pair travels inside its record.
    const bool pairs_stay_fp32 = fix_in_hist && path == 2 && ctx->hist8 && gbt_fix32_ok(scale[0], scale[1]) &&
                                 gbt_hist8_ok(bits, F, pl.n_ftiles, n, gbt_packed_words(n, F, bits));
    int sum_slots = 0;   // > 0: the root's totals come as this many partial pairs (gbt_launch_hist8), in the job area
    static_assert(kUploadBytes >= ((size_t)1 << 14) * 16, "room for the partial totals of gbt_launch_hist8");
    if (root_may_split) {
        RootFix fix{gpair, scale[0], scale[1], pairs_stay_fp32 ? nullptr : gq, sums_dev, uniform_h,
                    (int32_t)llrint((double)h_value * scale[1]), (int64_t *)(ws + L.jobs), 0};
        st = hist_uniform(ctx, packed, bits, n, F, B, missing_sym, nullptr, n, gq, pool,
                          (HistJob *)(ws + L.jobs), fix_in_hist ? &fix : nullptr, uniform_h != 0, fix.hq_uniform);
        if (st != GBT_OK) return st;
        sum_slots = fix_in_hist ? fix.n_slots : 0;
    }
    GBT_REQUIRE(ctx, sum_slots <= gbt_hist8_max_jobs() && (size_t)sum_slots * 16 <= kCutsRb, GBT_EHIP, "internal: partial totals");
    GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), sum_slots ? (const void *)(ws + L.jobs) : (const void *)sums_dev,
                                sum_slots ? (size_t)sum_slots * 16 : 16, hipMemcpyDeviceToHost, s));
    GBT_SYNC(ctx);
    int64_t root_sums[2] = {0, 0};
    if (sum_slots) {
        const int64_t *ps = (const int64_t *)rb(ctx);
        for (int j = 0; j < sum_slots; ++j) {
            root_sums[0] += ps[2 * j];
            root_sums[1] += ps[2 * j + 1];
        }
    } else {
        memcpy(root_sums, rb(ctx), 16);
    }
    if (cuts_via_pinned) memcpy(hcuts.data(), rb(ctx) + kCutsRb, hcuts.size() * sizeof(float));

    auto set_node_at = [&](int32_t at, const HNode &nd) {
        const double G = (double)nd.Gq * inv_sg, H = (double)nd.Hq * inv_sh;
        tree->feature[at] = -1;
        tree->bin[at] = 0;
        tree->default_left[at] = 0;
        tree->left[at] = tree->right[at] = -1;
        tree->threshold[at] = INFINITY;
        tree->gain[at] = 0.0;
        tree->sumG[at] = G;
        tree->sumH[at] = H;
        tree->weight[at] = H + lambda > 0.0 ? -G / (H + lambda) : 0.0;   // no curvature, no step
        tree->n_rows[at] = nd.len;
    };
    auto set_node = [&](const HNode &nd) { set_node_at(nd.id, nd); };

    std::vector<HNode> level, next;   // the nodes created by the last round: to be evaluated
    std::vector<LeafSeg> leaves;
    HNode root{0, 0, (uint32_t)n, root_sums[0], root_sums[1], 0, 2};
    set_node(root);
    if (root_may_split)
        level.push_back(root);
    else
        leaves.push_back(LeafSeg{0, 0, 2, (uint32_t)n});
    int32_t n_nodes = 1, n_leaves = 1;
    // Loss-guided growth.  The tree is defined by a strictly sequential rule (expand the open leaf with
    // the largest gain, then look again), but a step per expansion leaves the chip idle between small
    // launches.  So growth runs in two layers.  PHYSICAL nodes are created in rounds: the leaf whose turn it
    // is plus a few more open leaves in gain order (they are likely to have their turn soon; a leaf's best
    // split does not depend on when it is found).  A physical node's id is its slot in the histogram pool.
    // The LOGICAL tree -- the caller's -- follows the sequential rule over what is known: it pops the best
    // open leaf as long as that leaf has been expanded physically, numbering children at that moment, and
    // asks for a round when it has not.  Expansions the budget never reaches are simply not part of the
    // tree; leaf ids and row order come from the finished logical tree (walk + sort), never from where
    // the rows physically ended up.
    struct Phys {
        HNode nd;
        gbt_split sp;
        int32_t lc, rc;        // physical children, -1: not expanded
        int32_t logical;       // id in the caller's tree, -1: not (yet) part of it
        bool open;             // has a split that may be taken
    };
    std::vector<Phys> phys;             // by physical id
    struct OpenKey {   // order of turns: larger gain first, smaller logical id on equal gains
        double gain;
        int32_t logical, pid;
        bool operator<(const OpenKey &o) const { return gain > o.gain || (gain == o.gain && logical < o.logical); }
    };
    std::set<OpenKey> sim_open;         // the logical tree's open leaves
    int32_t n_logical = 1;
    if (lossguide) phys.push_back(Phys{root, gbt_split{}, -1, -1, 0, false});
    const int batch_max = std::max(1, std::min(ctx->lossguide_batch, kLossguideBatchMax));
    std::vector<UnmovedSeg> unmoved;
    std::vector<CountJob> cjobs;
    std::vector<Hist2Job> h2jobs;
    std::vector<Move3Job> m3jobs;
    std::vector<PartJob> kjobs;        // histogram jobs over the built children's records behind a three-level move
    std::vector<int> job_of;           // sel node -> its segment's job (count and two-histogram passes)
    uint32_t h2_spans = 0;
    int64_t h2_rows = 0;
    std::vector<uint32_t> nl_of;       // left rows of each node this round splits
    std::vector<HNode> sel_nodes;      // the nodes this round splits ...
    std::vector<gbt_split> sel_splits; // ... and how

    std::vector<EvalNode> enodes;
    std::vector<PartJob> pjobs;
    std::vector<HistJob> hjobs;
    std::vector<gbt_split> splits;

    // Split records come back in the read-back half of the staging behind the partition's row counts.
    constexpr size_t kSplitRb = 512u << 10;
    int chunks = 1;
    bool pre_eval = false;   // the level's split records are already in the read-back buffer
    // The kernel writes the records straight into the pinned read-back buffer (the device can address it):
    // no copy launch between the evaluation and the host's wait.  dev_nodes: the node table is on the
    // device already; tail: words the same launch hands back (see gbt_launch_eval).
    auto enqueue_eval = [&](const std::vector<EvalNode> &en, int *n_chunks, const EvalNode *dev_nodes = nullptr,
                            EvalTail tail = EvalTail{nullptr, nullptr, 0, 0, -1, 0}) -> int32_t {
        if (dev_nodes == nullptr) {
            int32_t st2 = upload(ctx, en.data(), en.size() * sizeof(EvalNode), ws + L.eval_nodes);
            if (st2 != GBT_OK) return st2;
            dev_nodes = (const EvalNode *)(ws + L.eval_nodes);
        }
        const size_t budget = GBT_STAGING_BYTES - kReadbackOff - kSplitRb;
        *n_chunks = gbt_eval_chunks(F, (int)en.size(), budget);
        const size_t sbytes = en.size() * (size_t)*n_chunks * sizeof(gbt_split);
        GBT_REQUIRE(ctx, sbytes <= budget, GBT_EUNSUPPORTED, "level too wide");
        gbt_prof_begin(ctx, GBT_PROF_EVAL, (double)en.size() * (double)hist_len * 8.0);
        GBT_HIP(ctx, gbt_launch_eval(s, pool, dev_nodes, (int)en.size(), nb, F, B, *n_chunks, inv_sg, inv_sh, lambda,
                                     params->min_child_weight, (gbt_split *)(rb(ctx) + kSplitRb), tail));
        gbt_prof_end(ctx);
        return GBT_OK;
    };
    int64_t pool_zero_end = 0;   // pool slots [n_nodes, pool_zero_end) were zeroed by the last evaluation launch
    bool cursors_zero = false;   // the partition + histogram pass's cursors (L.state) were cleared by the evaluation behind the last pass

    while (!level.empty() || !sim_open.empty()) {
        // ---- EvaluateSplit for every open node of the level (already enqueued, and waited for, by
        //      the level before when that ran the partition + histogram pass)
        if (!pre_eval && !level.empty()) {
            enodes.resize(level.size());
            for (size_t i = 0; i < level.size(); ++i)
                enodes[i] = EvalNode{(uint64_t)level[i].id * (uint64_t)hist_len, level[i].Gq, level[i].Hq,
                                     level[i].sub_parent >= 0 ? (uint64_t)level[i].sub_parent * (uint64_t)hist_len : GBT_NO_HIST,
                                     level[i].sub_parent >= 0 ? (uint64_t)level[i].sub_built * (uint64_t)hist_len : GBT_NO_HIST};
            // (depth-wise, the children of the deepest nodes that are evaluated are leaves: a histogram made by
            // subtraction there is priced and forgotten)
            EvalTail plain{nullptr, nullptr, 0, 0, -1, 0};
            plain.skip_store = !lossguide && level[0].depth >= max_depth - 1 ? 1 : 0;
            st = enqueue_eval(enodes, &chunks, nullptr, plain);
            if (st != GBT_OK) return st;
            GBT_SYNC(ctx);
        }
        pre_eval = false;
        splits.resize(level.size());
        for (size_t i = 0; i < level.size(); ++i)
            splits[i] = merge_chunks((const gbt_split *)(rb(ctx) + kSplitRb) + i * chunks, chunks);

        // ---- which nodes split; RepartitionInstances for those.
        // Children that are split again get their whole records moved: by the one-launch form
        // when nobody needs the row order and the rows are narrow enough (and then, where the
        // histogram kernel's 8-bit single-tile case applies, one child's histogram is built in
        // the same pass), else by the three-launch form.  Leaves only need their ids moved, or
        // just the row counts when no ids travel with the rows.
        sel_nodes.clear();
        sel_splits.clear();
        for (size_t i = 0; i < level.size(); ++i) {
            const gbt_split &sp = splits[i];
            const HNode &nd = level[i];
            const bool ok = sp.valid && sp.gain > min_gain && sp.feature >= 0 && sp.feature < F &&
                            sp.bin >= 0 && sp.bin < B && nd.len > 0;
            if (lossguide) {
                Phys &ph = phys[(size_t)nd.id];
                ph.sp = sp;
                ph.open = ok;
                if (ok && ph.logical >= 0) sim_open.insert(OpenKey{sp.gain, ph.logical, nd.id});   // the root
            } else if (!ok) {
                leaves.push_back(LeafSeg{nd.begin, (uint32_t)nd.id, (uint32_t)nd.buf, nd.len});
            } else {
                sel_nodes.push_back(nd);
                sel_splits.push_back(sp);
            }
        }
        level.clear();
        if (lossguide) {
            // the logical tree advances as far as the physical expansions reach
            while (n_leaves < max_leaves && !sim_open.empty()) {
                const int32_t pid = sim_open.begin()->pid;
                Phys &ph = phys[(size_t)pid];
                if (ph.lc < 0) break;   // its turn, but not expanded yet: a round is needed
                sim_open.erase(sim_open.begin());
                const int32_t at = ph.logical, lcl = n_logical, rcl = n_logical + 1;
                GBT_REQUIRE(ctx, rcl < tree->capacity, GBT_EHIP, "internal: logical tree overflow");
                n_logical += 2;
                n_leaves += 1;
                tree->feature[at] = ph.sp.feature;
                tree->bin[at] = ph.sp.bin;
                tree->default_left[at] = ph.sp.default_left;
                tree->left[at] = lcl;
                tree->right[at] = rcl;
                tree->gain[at] = ph.sp.gain;
                tree->threshold[at] =
                    ph.sp.bin < B - 1 ? hcuts[(size_t)ph.sp.feature * (B - 1) + ph.sp.bin] : INFINITY;
                for (int side = 0; side < 2; ++side) {
                    const int32_t cid = side == 0 ? ph.lc : ph.rc;
                    Phys &ch = phys[(size_t)cid];
                    ch.logical = side == 0 ? lcl : rcl;
                    set_node_at(ch.logical, ch.nd);
                    if (ch.open) sim_open.insert(OpenKey{ch.sp.gain, ch.logical, cid});
                }
            }
            if (n_leaves < max_leaves && !sim_open.empty()) {
                // the leaf whose turn it is, and the next ones in gain order that live in the same working
                // copy and agree with it on whether their children can still split; every expansion takes two
                // physical slots, of which enough stay reserved for the expansions the budget still allows
                const int64_t room = (cap_phys - n_nodes) / 2, budget = (int64_t)max_leaves - n_leaves;
                const int64_t k_max = std::max<int64_t>(1, std::min<int64_t>({(int64_t)batch_max, budget, room - budget + 1}));
                const HNode first = phys[(size_t)sim_open.begin()->pid].nd;
                int looked = 0;
                for (const OpenKey &key : sim_open) {
                    if (++looked > 8 * kLossguideBatchMax) break;   // far down the order a leaf's turn is unlikely to come
                    const Phys &ph = phys[(size_t)key.pid];
                    if (ph.lc >= 0) continue;   // expanded ahead of its turn already
                    if (ph.nd.buf != first.buf || (ph.nd.depth + 1 < max_depth) != (first.depth + 1 < max_depth)) continue;
                    sel_nodes.push_back(ph.nd);
                    sel_splits.push_back(ph.sp);
                    if ((int64_t)sel_nodes.size() >= k_max) break;
                }
            }
        }
        if (sel_nodes.empty()) break;   // nothing splits any more: what is still open stays a leaf
        // all nodes of a round lie in the same buffer (a whole level, or a single node)
        const int wcur = sel_nodes[0].buf;
        const GbtRows &cur = wcur == 2 ? matrix : W[wcur];
        const int wnext = wcur == 0 ? 1 : 0;
        const int child_depth = sel_nodes[0].depth + 1;   // loss-guided: of the first node; the others agree on "< max_depth"
        const bool children_need_hist =
            child_depth < max_depth && (!lossguide || n_leaves + 1 < max_leaves);
        const bool unordered = path == 1 || path == 2;
        const bool fused = children_need_hist && unordered;
        const bool in_place = sel_nodes[0].virt >= 0;   // this level's nodes were not moved when they were made
        // Rows that have stayed in place for two levels (their nodes are grandchildren of the segment they lie in) are
        // put in order again by a pass of its own, without a histogram: one child of each is then built from its
        // contiguous records
        // (likewise rows that stayed in the caller's matrix at the root's split: two levels at once, into records)
        const bool move3 = children_need_hist && path == 2 && in_place && (sel_nodes[0].vpos >= 3 || wcur == 2);
        const int move_levels = sel_nodes[0].vpos >= 3 ? 3 : 2;
        const bool with_hist = children_need_hist && path == 2 && !move3;
        // Depth-wise, the last level that needs histograms: its children's children are leaves, of which only
        // the row counts are wanted.  The pass then builds the histograms and counts without moving a row,
        // and the counts one level down come from a two-level count over the parents' segments.
        // One level earlier the same again where that level's rows are records that can serve a second pass with
        // TWO histograms per workgroup (one for each of a segment's two children): the nodes of depth
        // max_depth - 3 are then the last whose rows were moved into place, and the leaves are counted over
        // three levels of splits.
        // Further up the same three passes repeat (GBT_TUNE_PART_CYCLE): keep, keep again with two histograms, move
        // three levels at once -- 20 + 20 + 40 (+ the built children's 20 * 1/2) bytes per row and three levels
        // instead of 3 * 40 -- timed so that a cycle ends where the last two in-place levels begin.
        const int levels_after = (max_depth - 1) - child_depth;   // histogram levels below this one
        const bool cycle_start = ctx->part_cycle && ctx->part_nomove >= 2 && levels_after >= 4 && levels_after % 3 == 1 &&
                                 sel_nodes.size() <= 512;   // (each becomes a segment with four cursors to read back)
        // At the root's split the rows stay in the matrix where the level below would otherwise move them a second
        // time: the children's histogram is built in place (21 bytes per row instead of 41) and the next level moves
        // the rows from the matrix straight to the grandchildren (41 + the built children's 10 instead of 40).
        const int levels_after_next = levels_after - 1;
        const bool first_keep = ctx->part_cycle && ctx->part_nomove >= 2 && wcur == 2 && child_depth == 1 &&
                                levels_after_next >= 2 && !(levels_after_next >= 4 && levels_after_next % 3 == 1);
        const bool nomove = with_hist && !lossguide && !in_place && ctx->part_nomove &&
                            (child_depth == max_depth - 1 || first_keep ||
                             (ctx->part_nomove >= 2 && (child_depth == max_depth - 2 || cycle_start) && wcur != 2 &&
                              gbt_hist2_ok(ctx, F, B)));
        const bool nomove2 = with_hist && in_place;     // (their heap positions are 1 and 2)
        const bool two_level = !children_need_hist && in_place;
        const int count_levels = two_level && sel_nodes[0].vpos >= 3 ? 2 : 1;
        double part_rows = 0;
        for (const HNode &nd : sel_nodes) part_rows += nd.len;
        // rows per partition workgroup: a tile, or (with the histogram) a span of tiles long enough
        // to be worth merging an LDS histogram into HBM for
        uint32_t part_tile = fused ? (uint32_t)gbt_partition_fused_tile(W[wnext]) : (uint32_t)GBT_PART_TILE;
        if (with_hist) {
            // Every span merges a whole histogram (two in the two-histogram pass, which has one workgroup per CU) into
            // HBM at its end, 64-bit global atomics that the chip retires slowly: a pass that moves nothing has little
            // else to wait for, so it takes half the spans -- and the two-histogram pass, while the level has few
            // segments to balance, three eighths (measured per level on 115M x 13: 0.50 -> 0.45, 0.57 -> 0.53 ms; with
            // 32 segments of unequal length fewer spans lose more to imbalance than they save: 0.51 -> 0.59 ms).
            const uint32_t t = (uint32_t)gbt_part_hist_tile();
            const int J = ctx->hist_jobs_per_cu;
            const int per_cu = in_place ? std::max(1, sel_nodes.size() < 32 ? 3 * J / 8 : J / 2) : nomove ? std::max(1, J / 2) : J;
            const double want = part_rows / ((double)ctx->num_cu * per_cu);
            part_tile = (uint32_t)std::min<double>(std::max<double>(std::ceil(want / t), 4.0), (double)((1u << 21) / t)) * t;
        }
        pjobs.clear();
        uint32_t tile_cursor = 0;
        for (size_t k = 0; k < sel_nodes.size(); ++k) {
            const gbt_split &sp = sel_splits[k];
            const HNode &nd = sel_nodes[k];
            PartJob j;
            j.seg_begin = nd.begin;
            j.seg_len = nd.len;
            j.feature = (uint32_t)sp.feature;
            j.bin = (uint32_t)sp.bin;
            j.default_left = (uint32_t)sp.default_left;
            j.tile_begin = tile_cursor;
            j.n_tiles = (nd.len + part_tile - 1) / part_tile;
            // with the histogram: build the child with the smaller hessian sum (a stand-in for "fewer
            // rows", which is only known after the partition); children are numbered in job order
            const bool build_left = sp.HLq <= nd.Hq - sp.HLq;
            j.pad = build_left ? 1u : 0u;
            j.hist_off = (uint64_t)(n_nodes + 2 * (int64_t)k + (build_left ? 0 : 1)) * (uint64_t)hist_len;
            tile_cursor += j.n_tiles;
            pjobs.push_back(j);
        }
        next.clear();
        nl_of.assign(sel_nodes.size(), 0u);
        int pass_span_of_round = -1;      // the profiler's span of this round's partition (+ histogram) pass ...
        double pass_alg_of_round = 0.0;   // ... and the method bytes of its partition part
        const int what = path == 3            ? GBT_PART_IDS
                         : children_need_hist ? GBT_PART_RECORDS
                         : (tracked && path == 0) ? GBT_PART_IDS
                                                  : GBT_PART_COUNT;
        // the segments this level's nodes live in, one job each (nodes of a segment are adjacent in sel_nodes)
        job_of.assign(sel_nodes.size(), -1);
        if (in_place) {
            int n_seg_jobs = 0;
            for (size_t k = 0; k < sel_nodes.size(); ++k) {
                if (k == 0 || sel_nodes[k - 1].virt != sel_nodes[k].virt) ++n_seg_jobs;
                job_of[k] = n_seg_jobs - 1;
                unmoved[(size_t)sel_nodes[k].virt].set(sel_nodes[k].vpos, sel_splits[k]);
            }
        }
        const bool deferred = defer_counts && !children_need_hist;   // nl_of stays 0: see the walk at the end
        if (deferred) {
            // nothing is launched for these nodes
        } else if (two_level) {
            cjobs.clear();
            uint32_t ctiles = 0;
            const uint32_t ct = (uint32_t)gbt_count2_tile();
            for (size_t k = 0; k < sel_nodes.size(); ++k) {
                if (k > 0 && job_of[k] == job_of[k - 1]) continue;
                const UnmovedSeg &u = unmoved[(size_t)sel_nodes[k].virt];
                CountJob cj{};
                cj.seg_begin = u.begin;
                cj.seg_len = u.len;
                cj.tile_begin = ctiles;
                cj.n_tiles = (u.len + ct - 1) / ct;
                ctiles += cj.n_tiles;
                cjobs.push_back(cj);
            }
            for (size_t k = 0; k < sel_nodes.size(); ++k) {   // (after every split of the level has been noted in its segment)
                const UnmovedSeg &u = unmoved[(size_t)sel_nodes[k].virt];
                CountJob &cj = cjobs[(size_t)job_of[k]];
                memcpy(cj.feature, u.feature, sizeof cj.feature);
                memcpy(cj.bin, u.bin, sizeof cj.bin);
                memcpy(cj.default_left, u.default_left, sizeof cj.default_left);
                memcpy(cj.has, u.has, sizeof cj.has);
            }
            const size_t cnt_bytes = cjobs.size() * (count_levels == 2 ? 16 : 8);
            GBT_REQUIRE(ctx, cjobs.size() * sizeof(CountJob) <= kUploadBytes && cnt_bytes <= (size_t)L.level_nodes * 8,
                        GBT_EUNSUPPORTED, "level too wide");
            st = upload(ctx, cjobs.data(), cjobs.size() * sizeof(CountJob), ws + L.jobs);
            if (st != GBT_OK) return st;
            const UnmovedSeg &u0 = unmoved[(size_t)sel_nodes[0].virt];
            const bool from_matrix = u0.buf == 2;
            const uint8_t *rows8 = from_matrix ? (const uint8_t *)packed : (const uint8_t *)W[u0.buf].sym;
            const int64_t stride8 = from_matrix ? (int64_t)F : 4 * (int64_t)gbt_part_hist_record_words(F);
            double crow = 0;
            for (const CountJob &cj : cjobs) crow += cj.seg_len;
            gbt_prof_begin(ctx, GBT_PROF_PARTITION, crow * (double)stride8, crow * count_levels * (bits / 8.0));
            GBT_HIP(ctx, gbt_launch_count2(s, rows8, stride8, (uint32_t)missing_sym, (const CountJob *)(ws + L.jobs),
                                           (int)cjobs.size(), (int)ctiles, (uint32_t *)(ws + L.state), count_levels,
                                           !from_matrix));
            GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), ws + L.state, cnt_bytes, hipMemcpyDeviceToHost, s));
            cursors_zero = false;
            gbt_prof_end(ctx);
            GBT_SYNC(ctx);
            const uint32_t *cnt = (const uint32_t *)rb(ctx);
            for (size_t k = 0; k < sel_nodes.size(); ++k)
                nl_of[k] = count_levels == 2 ? cnt[4 * job_of[k] + (sel_nodes[k].vpos - 3)]
                                             : cnt[2 * job_of[k] + (sel_nodes[k].vpos - 1)];
        } else if (move3) {
            // one job per segment: the three levels of splits below it and where its grandchildren's rows go
            GBT_REQUIRE(ctx, (move_levels == 2) == (wcur == 2), GBT_EHIP, "internal: %d levels of rows kept in buffer %d", move_levels, wcur);
            m3jobs.clear();
            uint32_t m3_spans = 0;
            double m3_rows = 0;
            const uint32_t m3_span_rows = 4u * (uint32_t)gbt_move3_tile();
            for (size_t k = 0; k < sel_nodes.size(); ++k) {
                if (k > 0 && job_of[k] == job_of[k - 1]) continue;
                const UnmovedSeg &u = unmoved[(size_t)sel_nodes[k].virt];
                Move3Job mj{};
                mj.seg_begin = u.begin;
                mj.seg_len = u.len;
                mj.tile_begin = m3_spans;
                mj.n_tiles = (u.len + m3_span_rows - 1) / m3_span_rows;
                m3_spans += mj.n_tiles;
                m3_rows += u.len;
                m3jobs.push_back(mj);
            }
            for (size_t k = 0; k < sel_nodes.size(); ++k) {   // (after every split of the level has been noted in its segment)
                const UnmovedSeg &u = unmoved[(size_t)sel_nodes[k].virt];
                Move3Job &mj = m3jobs[(size_t)job_of[k]];
                memcpy(mj.feature, u.feature, sizeof mj.feature);
                memcpy(mj.bin, u.bin, sizeof mj.bin);
                memcpy(mj.default_left, u.default_left, sizeof mj.default_left);
                memcpy(mj.has, u.has, sizeof mj.has);
                const int gch = sel_nodes[k].vpos - (move_levels == 3 ? 3 : 1);
                GBT_REQUIRE(ctx, gch >= 0 && gch < (move_levels == 3 ? 4 : 2), GBT_EHIP, "internal: heap position %d", sel_nodes[k].vpos);
                mj.node_begin[gch] = sel_nodes[k].begin;
                mj.node_len[gch] = sel_nodes[k].len;
            }
            GBT_REQUIRE(ctx, m3jobs.size() * sizeof(Move3Job) <= kUploadBytes && 4 * (int64_t)m3jobs.size() <= L.level_nodes &&
                                 m3jobs.size() * 32 * kCursorStride <= kSplitRb,
                        GBT_EUNSUPPORTED, "level too wide");
            st = upload(ctx, m3jobs.data(), m3jobs.size() * sizeof(Move3Job), ws + L.jobs);
            if (st != GBT_OK) return st;
            const double rec_bytes3 = 4.0 * gbt_part_hist_record_words(F);
            // What the method needs for this: it repartitions at every level, 4 bytes of row id read and 4 written per
            // row, plus the symbol that decides.  A move over `move_levels` levels of splits is the repartition of that
            // many levels (the passes that left the rows in place were credited with their symbol only).
            gbt_prof_begin(ctx, GBT_PROF_PARTITION, m3_rows * (rec_bytes3 + (wcur == 2 ? row_bits / 8.0 + 8.0 : rec_bytes3)),
                           m3_rows * (8.0 * move_levels + bits / 8.0));
            if (wcur == 2)
                GBT_HIP(ctx, gbt_launch_move2_first(ctx, packed, gbt_packed_words(n, F, bits), gq, pairs_stay_fp32 ? gpair : nullptr,
                                                    scale[0], scale[1], W[wnext].sym_rw, n, F, (uint32_t)missing_sym,
                                                    (const Move3Job *)(ws + L.jobs), (int)m3jobs.size(), (int)m3_spans,
                                                    m3_span_rows, (unsigned long long *)(ws + L.state), cursors_zero));
            else
                GBT_HIP(ctx, gbt_launch_move3(ctx, W[wcur].sym, W[wnext].sym_rw, n, F, (uint32_t)missing_sym,
                                              (const Move3Job *)(ws + L.jobs), (int)m3jobs.size(), (int)m3_spans, m3_span_rows,
                                              (unsigned long long *)(ws + L.state), cursors_zero));
            GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), ws + L.state, m3jobs.size() * 32 * kCursorStride, hipMemcpyDeviceToHost, s));
            cursors_zero = false;
            gbt_prof_end(ctx);
            GBT_SYNC(ctx);
            const unsigned long long *cur64 = (const unsigned long long *)rb(ctx);
            for (size_t k = 0; k < sel_nodes.size(); ++k) {
                const unsigned long long c = cur64[(4 * (size_t)job_of[k] + (size_t)(sel_nodes[k].vpos - (move_levels == 3 ? 3 : 1))) * kCursorStride];
                const uint32_t lefts = (uint32_t)(c & 0xffffffffull), rights = (uint32_t)(c >> 32);
                GBT_REQUIRE(ctx, (uint64_t)lefts + rights == sel_nodes[k].len, GBT_EHIP,
                            "internal: node %d holds %u rows, %u + %u were moved", sel_nodes[k].id, sel_nodes[k].len, lefts, rights);
                nl_of[k] = lefts;
            }
        } else {
            // the three-launch form keeps ballots and counts per tile in the workspace
            GBT_REQUIRE(ctx, fused || (int64_t)tile_cursor <= L.tiles, GBT_ENOMEM, "internal: tile count");
            GBT_REQUIRE(ctx, pjobs.size() * sizeof(PartJob) <= kUploadBytes, GBT_EUNSUPPORTED, "level too wide");
            const EvalNode *children_dev = nullptr;   // with_hist: the children's evaluation table, uploaded with the jobs
            if (with_hist) {
                // Everything the children's evaluation needs is known before the rows are counted (ids,
                // sums, which child was built): it is enqueued behind the pass (and makes the other child's
                // histogram by subtraction on the way), so that the host waits once per level, not twice.
                enodes.clear();
                for (size_t k = 0; k < pjobs.size(); ++k) {
                    const HNode &nd = sel_nodes[k];
                    const gbt_split &sp = sel_splits[k];
                    const int64_t lid = n_nodes + 2 * (int64_t)k, rid = lid + 1;
                    const bool left_built = pjobs[k].pad == 1u;
                    const uint64_t par = (uint64_t)nd.id * (uint64_t)hist_len;
                    const uint64_t blt = (uint64_t)(left_built ? lid : rid) * (uint64_t)hist_len;
                    enodes.push_back(EvalNode{(uint64_t)lid * (uint64_t)hist_len, sp.GLq, sp.HLq,
                                              left_built ? GBT_NO_HIST : par, left_built ? GBT_NO_HIST : blt});
                    enodes.push_back(EvalNode{(uint64_t)rid * (uint64_t)hist_len, nd.Gq - sp.GLq, nd.Hq - sp.HLq,
                                              left_built ? par : GBT_NO_HIST, left_built ? blt : GBT_NO_HIST});
                }
                const void *jobs_host = pjobs.data();
                size_t pj_bytes = pjobs.size() * sizeof(PartJob);
                if (nomove2) {   // one job per segment: its own split, and what its (one or two) splitting children do
                    h2jobs.clear();
                    h2_spans = 0;
                    h2_rows = 0;
                    for (size_t k = 0; k < sel_nodes.size(); ++k) {
                        const UnmovedSeg &u = unmoved[(size_t)sel_nodes[k].virt];
                        if (k == 0 || job_of[k] != job_of[k - 1]) {
                            Hist2Job hj{};
                            hj.seg_begin = u.begin;
                            hj.seg_len = u.len;
                            hj.tile_begin = h2_spans;
                            hj.n_tiles = (u.len + part_tile - 1) / part_tile;
                            hj.feature[0] = u.feature[0];
                            hj.bin[0] = u.bin[0];
                            hj.default_left[0] = u.default_left[0];
                            hj.build[0] = hj.build[1] = 2u;
                            h2_spans += hj.n_tiles;
                            h2_rows += u.len;
                            h2jobs.push_back(hj);
                        }
                        Hist2Job &hj = h2jobs.back();
                        const int c = sel_nodes[k].vpos - 1;
                        hj.feature[1 + c] = (uint32_t)sel_splits[k].feature;
                        hj.bin[1 + c] = (uint32_t)sel_splits[k].bin;
                        hj.default_left[1 + c] = (uint32_t)sel_splits[k].default_left;
                        hj.has[c] = 1;
                        hj.build[c] = pjobs[k].pad;
                        hj.hist_off[c] = pjobs[k].hist_off;
                    }
                    jobs_host = h2jobs.data();
                    pj_bytes = h2jobs.size() * sizeof(Hist2Job);
                }
                const size_t en_bytes = enodes.size() * sizeof(EvalNode);
                if (gbt_align(pj_bytes) + en_bytes <= kUploadBytes) {   // both tables with one copy
                    size_t en_off = 0;
                    st = upload2(ctx, jobs_host, pj_bytes, enodes.data(), en_bytes, ws + L.jobs, &en_off);
                    children_dev = (const EvalNode *)(ws + L.jobs + en_off);
                } else {
                    st = upload(ctx, jobs_host, pj_bytes, ws + L.jobs);
                }
            } else {
                st = upload(ctx, pjobs.data(), pjobs.size() * sizeof(PartJob), ws + L.jobs);
            }
            if (st != GBT_OK) return st;
            if (with_hist && (int64_t)n_nodes + 2 * (int64_t)pjobs.size() > pool_zero_end) {
                // the children's histograms are accumulated into: clear them first (unless the evaluation
                // launch of the level before has done so, as it does for every child its nodes can have)
                const int64_t n_children = 2 * (int64_t)pjobs.size();
                gbt_prof_begin(ctx, GBT_PROF_CLEAR, (double)n_children * (double)hist_len * 8.0);
                GBT_HIP(ctx, gbt_launch_fill_u64(s, (uint64_t *)(pool + (int64_t)n_nodes * hist_len), 0,
                                                 n_children * hist_len));
                gbt_prof_end(ctx);
            }
            const double rec_bytes = row_bits / 8.0 + 8.0;
            // what the method needs: a repartition is 4 + 4 + bits/8 bytes per row (where rows are only counted, the
            // symbol alone); the histogram part of a pass is added below, once the built children's rows are known
            const double part_alg = part_rows * ((nomove || nomove2 || what == GBT_PART_COUNT) ? bits / 8.0 : 8.0 + bits / 8.0);
            const bool keeps_records = nomove2 || (nomove && with_hist && wcur != 2);   // a pass over records that stay in place
            const int pass_span = gbt_prof_begin(ctx, keeps_records ? GBT_PROF_HIST_INPLACE : with_hist ? (wcur == 2 ? GBT_PROF_HIST_FIRST : GBT_PROF_HIST_NODE)
                                                                            : GBT_PROF_PARTITION,
                           nomove2 ? (double)h2_rows * rec_bytes :
                           part_rows * (path == 3 ? 8.0 + 32.0   // ids read and written, one sector of symbols per row
                                        : nomove  ? rec_bytes
                                    : fused   ? 2.0 * rec_bytes
                                        : what == GBT_PART_RECORDS ? row_bits / 8.0 + 2.0 * (rec_bytes + 4.0)
                                        : what == GBT_PART_IDS     ? row_bits / 8.0 + 8.0
                                                                   : row_bits / 8.0),
                           part_alg, with_hist ? child_depth : -1);
            pass_span_of_round = pass_span;
            pass_alg_of_round = part_alg;
            if (with_hist) {
                GBT_REQUIRE(ctx, pjobs.size() * 8 <= kSplitRb, GBT_EUNSUPPORTED, "level too wide");
                if (!cursors_zero) {   // every cursor a level can have; from then on the evaluation launch keeps them clear
                    GBT_HIP(ctx, gbt_launch_fill_u64(s, (uint64_t *)(ws + L.state), 0, L.level_nodes * kCursorStride));
                    cursors_zero = true;
                }
                if (nomove2)   // the segments' records once more, two histograms per workgroup
                    GBT_HIP(ctx, gbt_launch_hist2(ctx, W[wcur].sym, F, B, (uint32_t)missing_sym, (const Hist2Job *)(ws + L.jobs),
                                                  (int)h2jobs.size(), (int)h2_spans, part_tile,
                                                  (unsigned long long *)(ws + L.state), pool, true, hq_uni));
                else if (nomove && wcur == 2 && pjobs.size() == 1 && ctx->hist8 && pjobs[0].seg_begin == 0 &&
                         (int64_t)pjobs[0].seg_len == n && gbt_hist8_ok(bits, F, pl.n_ftiles, n, gbt_packed_words(n, F, bits))) {
                    // the root's rows stay in the matrix: the root histogram kernel once more, adding only the rows of
                    // the child to be built and counting the rows that go left
                    Hist8Pairs hp{};
                    if (pairs_stay_fp32) {
                        hp.gpair = gpair;
                        hp.sg = scale[0];
                        hp.sh = scale[1];
                        hp.mode = 2;
                    } else {
                        hp.gq = gq;
                    }
                    hp.uniform_h = hq_uni >= 0;
                    hp.hq_uniform = hq_uni >= 0 ? hq_uni : 0;
                    const Hist8Filter flt{(int)pjobs[0].feature, (int)pjobs[0].bin, (int)pjobs[0].default_left,
                                          pjobs[0].pad == 1u ? 1 : 0, (unsigned long long *)(ws + L.state)};
                    GBT_HIP(ctx, gbt_launch_hist8(ctx, packed, n, F, B, (uint32_t)missing_sym, hp, pool + pjobs[0].hist_off,
                                                  nullptr, &flt));
                } else   // level 0 reads the caller's matrix and the pairs, later levels the records of the level before
                    GBT_HIP(ctx, gbt_launch_part_hist(ctx, packed, gbt_packed_words(n, F, bits), gq,
                                                      wcur == 2 ? nullptr : W[wcur].sym, nomove ? nullptr : W[wnext].sym_rw, F, B,
                                                      (uint32_t)missing_sym, (const PartJob *)(ws + L.jobs),
                                                      (int)pjobs.size(), (int)tile_cursor, part_tile,
                                                      (unsigned long long *)(ws + L.state), pool, true,
                                                      pairs_stay_fp32 ? gpair : nullptr, scale[0], scale[1], hq_uni));
                gbt_prof_end(ctx);
                // the evaluation launch also hands the cursors (the left counts) to the host and clears them
                // for the next pass: no copy and no fill launch of their own
                // ... and zeroes the histograms of the children's children where those will be built
                const int64_t after = (int64_t)n_nodes + 2 * (int64_t)pjobs.size();
                const bool more = child_depth + 1 < max_depth;
                const int64_t zero_end = more ? std::min<int64_t>(after + 2 * (int64_t)enodes.size(), L.hist_nodes) : 0;
                st = enqueue_eval(enodes, &chunks, children_dev,
                                  EvalTail{(unsigned long long *)(ws + L.state), (unsigned long long *)rb(ctx),
                                           nomove2 ? 2 * (int)h2jobs.size() : (int)pjobs.size(), 1, more ? after : -1, zero_end,
                                           kCursorStride, !lossguide && child_depth >= max_depth - 1 ? 1 : 0});
                if (st != GBT_OK) return st;
                pool_zero_end = zero_end;
                pre_eval = true;
            } else if (fused) {
                GBT_HIP(ctx, gbt_launch_partition_fused(s, cur, W[wnext], bits, row_bits, (uint32_t)missing_sym,
                                                        (const PartJob *)(ws + L.jobs), (int)pjobs.size(),
                                                        (int)tile_cursor, (unsigned long long *)(ws + L.state)));
                cursors_zero = false;
                GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), ws + L.state, pjobs.size() * 8, hipMemcpyDeviceToHost, s));
                gbt_prof_end(ctx);
            } else if (path == 3) {
                // stable partition of the nodes' id lists; the symbols are gathered from the caller's matrix
                GBT_HIP(ctx, gbt_launch_partition(s, packed, bits, row_bits, n, (uint32_t)missing_sym,
                                                  wcur == 2 ? W[1].id : W[wcur].id, W[wnext].id_rw,
                                                  (const PartJob *)(ws + L.jobs), (int)pjobs.size(), (int)tile_cursor,
                                                  (uint64_t *)(ws + L.masks), (uint32_t *)(ws + L.tile_left),
                                                  (uint32_t *)(ws + L.n_left)));
                GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), ws + L.n_left, pjobs.size() * 4, hipMemcpyDeviceToHost, s));
                gbt_prof_end(ctx);
            } else {
                GBT_HIP(ctx, gbt_launch_partition_records(s, cur, W[wnext], bits, row_bits, n, (uint32_t)missing_sym, what,
                                                          (const PartJob *)(ws + L.jobs), (int)pjobs.size(),
                                                          (int)tile_cursor, (uint64_t *)(ws + L.masks),
                                                          (uint32_t *)(ws + L.tile_left), (uint32_t *)(ws + L.n_left)));
                GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), ws + L.n_left, pjobs.size() * 4, hipMemcpyDeviceToHost, s));
                gbt_prof_end(ctx);
            }
            GBT_SYNC(ctx);
            const int nl_stride = fused ? 2 : 1;   // the one-launch form returns 64-bit cursors, n_left in the low half
            const uint32_t *n_left = (const uint32_t *)rb(ctx);
            for (size_t k = 0; k < pjobs.size(); ++k)   // (two-histogram pass: cursor 2 * job + child, 64 bits each)
                nl_of[k] = nomove2 ? n_left[2 * (2 * job_of[k] + (sel_nodes[k].vpos - 1))] : n_left[k * nl_stride];
        }
        const int child_buf = (nomove || nomove2 || two_level || what == GBT_PART_COUNT) ? wcur : wnext;   // a count moves nothing

        // ---- children, in creation order
        hjobs.clear();
        int64_t built_rows = 0;
        struct Built { uint64_t off; uint32_t begin, len; };
        std::vector<Built> built;
        const int32_t first_child = n_nodes;
        for (size_t k = 0; k < pjobs.size(); ++k) {
            const HNode &nd = sel_nodes[k];
            const gbt_split &sp = sel_splits[k];
            const uint32_t nl = nl_of[k];
            GBT_REQUIRE(ctx, nl <= nd.len, GBT_EHIP, "internal: n_left %u > %u", nl, nd.len);
            HNode lc{n_nodes, nd.begin, nl, sp.GLq, sp.HLq, nd.depth + 1, child_buf};
            HNode rc{n_nodes + 1, nd.begin + nl, nd.len - nl, nd.Gq - sp.GLq, nd.Hq - sp.HLq, nd.depth + 1, child_buf};
            if (deferred) {   // their row counts (0 and everything, for now) come from the walk at the end
                deferred_children.push_back(lc.id);
                deferred_children.push_back(rc.id);
            }
            if (nomove) {   // a new segment of rows that stay in place: the children are its heap positions 1 and 2
                UnmovedSeg u{};
                u.begin = nd.begin;
                u.len = nd.len;
                u.buf = wcur;
                u.set(0, sp);
                lc.virt = rc.virt = (int32_t)unmoved.size();
                lc.vpos = 1;
                rc.vpos = 2;
                unmoved.push_back(u);
            } else if (nomove2) {   // one level further down in the same segment
                lc.virt = rc.virt = nd.virt;
                lc.vpos = 2 * nd.vpos + 1;
                rc.vpos = 2 * nd.vpos + 2;
            }
            n_nodes += 2;
            if (lossguide) {   // physical children; the caller's tree learns of them when their parent is popped
                GBT_REQUIRE(ctx, n_nodes <= cap_phys, GBT_EHIP, "internal: physical node overflow");
                phys[(size_t)nd.id].lc = lc.id;
                phys[(size_t)nd.id].rc = rc.id;
                phys.push_back(Phys{lc, gbt_split{}, -1, -1, -1, false});
                phys.push_back(Phys{rc, gbt_split{}, -1, -1, -1, false});
            } else {
                n_leaves += 1;
                tree->feature[nd.id] = sp.feature;
                tree->bin[nd.id] = sp.bin;
                tree->default_left[nd.id] = sp.default_left;
                tree->left[nd.id] = lc.id;
                tree->right[nd.id] = rc.id;
                tree->gain[nd.id] = sp.gain;
                tree->threshold[nd.id] = sp.bin < B - 1 ? hcuts[(size_t)sp.feature * (B - 1) + sp.bin] : INFINITY;
                set_node(lc);
                set_node(rc);
            }
            if (children_need_hist) {
                // the child whose histogram is built from rows: the one the partition pass has already
                // built, else the one with fewer rows; its sibling comes by subtraction
                const bool left_small = with_hist ? pjobs[k].pad == 1u : lc.len <= rc.len;
                const HNode &sm = left_small ? lc : rc;
                built.push_back(Built{(uint64_t)sm.id * (uint64_t)hist_len, sm.begin, sm.len});
                built_rows += sm.len;
                HNode &other = left_small ? rc : lc;   // its histogram: parent - built, made when it is evaluated
                other.sub_parent = nd.id;
                other.sub_built = sm.id;
                next.push_back(lc);
                next.push_back(rc);
            } else {
                leaves.push_back(LeafSeg{lc.begin, (uint32_t)lc.id, (uint32_t)child_buf, lc.len});
                leaves.push_back(LeafSeg{rc.begin, (uint32_t)rc.id, (uint32_t)child_buf, rc.len});
            }
        }
        if (with_hist)   // the pass also built these children's histograms: rows * (symbols + pair + row id)
            gbt_prof_patch(ctx, pass_span_of_round, pass_alg_of_round + (double)built_rows * ((double)row_bits / 8.0 + 12.0),
                           (double)built_rows * F);
        if (move3) {
            // ---- BuildPartialHistograms for the smaller children from their records, now contiguous: the pass
            //      that keeps rows in place, under a split that takes every row
            if ((int64_t)n_nodes > pool_zero_end) {
                const int32_t n_children = n_nodes - first_child;
                gbt_prof_begin(ctx, GBT_PROF_CLEAR, (double)n_children * (double)hist_len * 8.0);
                GBT_HIP(ctx, gbt_launch_fill_u64(s, (uint64_t *)(pool + (int64_t)first_child * hist_len), 0,
                                                 (int64_t)n_children * hist_len));
                gbt_prof_end(ctx);
            }
            const uint32_t t = (uint32_t)gbt_part_hist_tile();
            // (the root kernel's loop over records: as many spans as workgroups are resident, four per compute unit --
            // every span merges a whole histogram into HBM at its end, and those atomics are what such a launch waits for)
            const bool rec8 = ctx->hist8 && bits == 8 && F <= 16 && pl.n_ftiles == 1;
            const double want = (double)built_rows / ((double)ctx->num_cu * (rec8 ? 4 : ctx->hist_jobs_per_cu));
            const uint32_t ktile = (uint32_t)std::min<double>(std::max<double>(std::ceil(want / t), 4.0), (double)((1u << 21) / t)) * t;
            kjobs.clear();
            uint32_t kspans = 0;
            for (const Built &b : built) {
                if (b.len == 0) continue;   // its histogram stays zero
                PartJob j{};
                j.seg_begin = b.begin;
                j.seg_len = b.len;
                j.feature = 0;
                j.bin = 255u;             // every byte symbol goes left,
                j.default_left = 1u;      // a missing one as well,
                j.pad = 1u;               // and the left side is the one added up
                j.tile_begin = kspans;
                j.n_tiles = (b.len + ktile - 1) / ktile;
                j.hist_off = b.off;
                kspans += j.n_tiles;
                kjobs.push_back(j);
            }
            GBT_REQUIRE(ctx, kjobs.size() * sizeof(PartJob) <= kUploadBytes && (int64_t)kjobs.size() <= L.level_nodes,
                        GBT_EUNSUPPORTED, "level too wide");
            if (!kjobs.empty()) {
                st = upload(ctx, kjobs.data(), kjobs.size() * sizeof(PartJob), ws + L.jobs);
                if (st != GBT_OK) return st;
                gbt_prof_begin(ctx, GBT_PROF_HIST_NODE, (double)built_rows * 4.0 * gbt_part_hist_record_words(F),
                               (double)built_rows * ((double)row_bits / 8.0 + 8.0), child_depth, (double)built_rows * F);
                if (rec8)   // every row is added: the root kernel's loop, over records
                    GBT_HIP(ctx, gbt_launch_hist8_records(ctx, W[wnext].sym, F, B, (uint32_t)missing_sym,
                                                          (const PartJob *)(ws + L.jobs), (int)kjobs.size(), (int)kspans, ktile,
                                                          pool, hq_uni));
                else
                    GBT_HIP(ctx, gbt_launch_part_hist(ctx, packed, gbt_packed_words(n, F, bits), gq, W[wnext].sym, nullptr, F, B,
                                                      (uint32_t)missing_sym, (const PartJob *)(ws + L.jobs), (int)kjobs.size(),
                                                      (int)kspans, ktile, (unsigned long long *)(ws + L.state), pool, false,
                                                      nullptr, 1.0, 1.0, hq_uni));
                gbt_prof_end(ctx);
            }
        } else if (children_need_hist && !with_hist) {
            // ---- BuildPartialHistograms for the smaller children (their rows are now one
            //      contiguous run of the working copy)
            const int32_t n_children = n_nodes - first_child;
            const bool uni_w = uniform_h && bits != 8 && !ctx->hist_runtime_bits;   // the kernels with a row-count form
            const int32_t hq_uniform = (int32_t)llrint((double)h_value * scale[1]);
            const uint32_t rpj = pick_rows_per_job(ctx, built_rows, gbt_histw_max_rows(uni_w), pl.n_ftiles, B);
            // Jobs add into a histogram that must start at zero, except where a node is one row piece: its jobs
            // store every bin of their tile.  (The sibling's histogram is stored bin by bin by the evaluation's
            // subtraction.)  Deep levels consist of such nodes only, and there the fill is the larger part of the
            // level: 2 MB per node for 2000 features x 64 bins.
            bool all_stored = true;
            for (const Built &b : built) all_stored = all_stored && b.len > 0 && b.len <= rpj;
            if (!all_stored) {
                gbt_prof_begin(ctx, GBT_PROF_CLEAR, (double)n_children * (double)hist_len * 8.0);
                GBT_HIP(ctx, gbt_launch_fill_u64(s, (uint64_t *)(pool + (int64_t)first_child * hist_len), 0,
                                                 (int64_t)n_children * hist_len));
                gbt_prof_end(ctx);
            }
            for (const Built &b : built) add_hist_jobs(hjobs, b.off, b.begin, b.len, F, pl, rpj);
            const size_t per_launch = kUploadBytes / sizeof(HistJob);
            for (size_t j0 = 0; j0 < hjobs.size(); j0 += per_launch) {
                const size_t nj = std::min(per_launch, hjobs.size() - j0);
                st = upload(ctx, hjobs.data() + j0, nj * sizeof(HistJob), ws + L.jobs);
                if (st != GBT_OK) return st;
                gbt_prof_begin(ctx, GBT_PROF_HIST_NODE,
                               j0 == 0 ? (double)built_rows * ((double)row_bits / 8.0 + 8.0 + (path == 3 ? 4.0 : 0.0)) : 0.0,
                               j0 == 0 ? (double)built_rows * ((double)row_bits / 8.0 + 12.0) : 0.0, child_depth,
                               j0 == 0 ? (double)built_rows * F : 0.0);
                if (path == 3)   // the rows by id from the caller's matrix, the pairs by id
                    GBT_HIP(ctx, gbt_launch_hist(ctx, packed, bits, row_bits, gbt_packed_words(n, F, bits), n, B,
                                                 (uint32_t)missing_sym, W[wnext].id, gq, pool,
                                                 (const HistJob *)(ws + L.jobs), (int)nj, pl.ft, uni_w, hq_uniform));
                else
                    GBT_HIP(ctx, gbt_launch_hist(ctx, W[wnext].sym, bits, W[wnext].stride_bits, W[wnext].n_words, n, B,
                                                 (uint32_t)missing_sym, nullptr, W[wnext].gq, pool,
                                                 (const HistJob *)(ws + L.jobs), (int)nj, pl.ft, uni_w, hq_uniform));
                gbt_prof_end(ctx);
            }
        }
        level.swap(next);
    }
    // whatever is still waiting when nothing splits any more is a leaf
    for (const HNode &nd : level) leaves.push_back(LeafSeg{nd.begin, (uint32_t)nd.id, (uint32_t)nd.buf, nd.len});
    const int32_t n_tree = lossguide ? n_logical : n_nodes;   // nodes of the caller's tree
    // margin_update: one walk of the finished tree over the packed matrix adds eta * leaf weight to every row's
    // margin, and counts the rows of the nodes whose counting was left to it
    auto update_margin = [&]() -> int32_t {
        if (!margin_update) return GBT_OK;
        tree->n_nodes = n_tree;
        uint32_t *node_rows = deferred_children.empty() ? nullptr : (uint32_t *)(ws + L.node_rows);
        if (node_rows) GBT_HIP(ctx, gbt_launch_fill_u64(s, (uint64_t *)node_rows, 0, (int64_t)n_tree * kNodeRowsStride / 2));
        gbt_prof_begin(ctx, GBT_PROF_OTHER, (double)n * (row_bits / 8.0 + 8.0));
        const int32_t st2 = predict_impl(ctx, tree, 1, packed, bits, missing_sym, nullptr, n, F, params->eta, margin_update,
                                         nullptr, ws + L.tree_stage, L.tree_stage_bytes, nullptr, false, node_rows, margin_src);
        gbt_prof_end(ctx);
        if (st2 != GBT_OK || !node_rows) return st2;
        std::vector<uint32_t> counts((size_t)n_tree * kNodeRowsStride);
        GBT_HIP(ctx, hipMemcpyAsync(counts.data(), node_rows, counts.size() * 4, hipMemcpyDeviceToHost, s));
        GBT_SYNC(ctx);
        for (const int32_t id : deferred_children) tree->n_rows[id] = (int64_t)counts[(size_t)id * kNodeRowsStride];
        return GBT_OK;
    };
    if (!tracked || path == 1 || path == 2 || lossguide) {
        tree->n_nodes = n_tree;
        st = update_margin();
        if (st != GBT_OK) return st;
        // the rows were not followed: one walk of the finished tree over the matrix names each row's leaf
        int32_t *leaf_ids = leaf_of_row_out ? leaf_of_row_out : (int32_t *)W[0].id_rw;
        if (leaf_of_row_out || tracked) {
            gbt_prof_begin(ctx, GBT_PROF_OTHER, (double)n * (row_bits / 8.0 + 4.0));
            st = predict_impl(ctx, tree, 1, packed, bits, missing_sym, nullptr, n, F, 0.0, nullptr, leaf_ids,
                              ws + L.tree_stage, L.tree_stage_bytes);
            gbt_prof_end(ctx);
            if (st != GBT_OK) return st;
        }
        if (tracked) {
            // ... and the stable partitions' final id list is the rows sorted by their leaf's place in
            // the tree's left-to-right order, ids ascending inside a leaf
            std::vector<uint32_t> rank((size_t)n_tree, 0u);
            std::vector<int32_t> stack{0};
            uint32_t n_ranks = 0;
            while (!stack.empty()) {
                const int32_t id = stack.back();
                stack.pop_back();
                if (tree->feature[id] < 0) {
                    rank[(size_t)id] = n_ranks++;
                } else {
                    stack.push_back(tree->right[id]);
                    stack.push_back(tree->left[id]);
                }
            }
            const size_t per_upload = kUploadBytes / 4;
            for (size_t i0 = 0; i0 < rank.size(); i0 += per_upload) {
                st = upload(ctx, rank.data() + i0, std::min(per_upload, rank.size() - i0) * 4, ws + L.rank_tbl + i0 * 4);
                if (st != GBT_OK) return st;
            }
            uint32_t *key_tmp[2] = {W[1].id_rw, (uint32_t *)(ws + L.wgq[0]) + n};
            uint32_t *val_tmp[2] = {(uint32_t *)(ws + L.wgq[0]), (uint32_t *)(ws + L.wgq[1])};
            gbt_prof_begin(ctx, GBT_PROF_OTHER, (double)n * 12.0);
            GBT_HIP(ctx, gbt_launch_order_rows(s, leaf_ids, (const uint32_t *)(ws + L.rank_tbl), (uint32_t)n_tree,
                                               n_ranks, n, key_tmp, val_tmp, ws + L.order, row_idx_out));
            gbt_prof_end(ctx);
        }
        GBT_SYNC(ctx);
        return GBT_OK;
    }

    std::sort(leaves.begin(), leaves.end(),
              [](const LeafSeg &a, const LeafSeg &b) {   // an empty segment sorts before the one that starts at the same place
                  return a.seg_begin != b.seg_begin ? a.seg_begin < b.seg_begin : (a.len != 0) < (b.len != 0);
              });
    st = upload(ctx, leaves.data(), leaves.size() * sizeof(LeafSeg), ws + L.jobs);
    if (st != GBT_OK) return st;
    gbt_prof_begin(ctx, GBT_PROF_OTHER, (double)n * 12.0);
    GBT_HIP(ctx, gbt_launch_leaf_gather(s, W[0].id, W[1].id, (const LeafSeg *)(ws + L.jobs), (int)leaves.size(), n,
                                        row_idx_out, leaf_of_row_out));
    gbt_prof_end(ctx);
    GBT_SYNC(ctx);
    tree->n_nodes = n_nodes;
    return update_margin();
}

extern "C" int32_t gbt_grow_tree(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                                 int32_t missing_sym, const int32_t *nb, const float *cuts, const float *gpair,
                                 const gbt_params *params, gbt_tree *tree, uint32_t *row_idx_out,
                                 int32_t *leaf_of_row_out, void *workspace, size_t workspace_bytes) {
    return grow_impl(ctx, packed, bits, n, F, missing_sym, nb, cuts, gpair, params, GBT_POLICY_DEPTHWISE, 0, tree,
                     row_idx_out, leaf_of_row_out, workspace, workspace_bytes);
}

// One boosting iteration (Fig. 1): gradient pairs of the current margins, one depth-wise tree, margins updated.
// The three steps share what each of them finds on its way: the gradient kernel leaves the bounds the scale search
// needs, and the walk that updates the margins counts the rows of the last level's children.
extern "C" int32_t gbt_boost_round(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                                   int32_t missing_sym, const int32_t *nb, const float *cuts, const float *label,
                                   const float *margin_in, float *margin_out, float *gpair, const gbt_params *params,
                                   gbt_tree *tree, void *workspace, size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, params && label && margin_in && margin_out && gpair && workspace, GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, params->objective == GBT_OBJ_SQUARED || params->objective == GBT_OBJ_LOGISTIC, GBT_EINVAL,
                "unknown objective %d", params->objective);
    GBT_REQUIRE(ctx, n >= 1 && F >= 1 && bits >= 1 && bits <= GBT_MAX_BITS && params->max_bins >= 2 &&
                         params->max_depth >= 0 && params->max_depth <= kMaxDepth, GBT_EINVAL, "bad shape");
    const GrowLayout L = grow_layout(n, F, bits, params->max_bins, params->max_depth);
    GBT_REQUIRE(ctx, workspace_bytes >= L.total, GBT_ENOMEM, "workspace %zu < %zu bytes", workspace_bytes, L.total);
    uint32_t *bounds = (uint32_t *)((char *)workspace + L.scratch + 1024);
    gbt_prof_begin(ctx, GBT_PROF_OTHER, (double)n * 16.0);
    GBT_HIP(ctx, gbt_launch_gradients(ctx->stream, params->objective, margin_in, label, n, gpair, bounds));
    gbt_prof_end(ctx);
    return grow_impl(ctx, packed, bits, n, F, missing_sym, nb, cuts, gpair, params, GBT_POLICY_DEPTHWISE, 0, tree,
                     nullptr, nullptr, workspace, workspace_bytes, margin_out, margin_in, bounds);
}

extern "C" size_t gbt_grow_tree_lossguide_workspace_bytes(int64_t n, int32_t F, int32_t bits, int32_t max_bins,
                                                          int32_t max_leaves) {
    if (n < 0 || F < 1 || bits < 1 || bits > GBT_MAX_BITS || max_bins < 2 || max_leaves < 1 || max_leaves > kMaxLeaves)
        return 0;
    return grow_layout_nodes(n, F, bits, max_bins, lossguide_phys_nodes(max_leaves), kLossguideBatchMax).total;
}

extern "C" int32_t gbt_grow_tree_lossguide(gbt_ctx *ctx, const uint32_t *packed, int32_t bits, int64_t n, int32_t F,
                                           int32_t missing_sym, const int32_t *nb, const float *cuts,
                                           const float *gpair, const gbt_params *params, int32_t max_leaves,
                                           gbt_tree *tree, uint32_t *row_idx_out, int32_t *leaf_of_row_out,
                                           void *workspace, size_t workspace_bytes) {
    return grow_impl(ctx, packed, bits, n, F, missing_sym, nb, cuts, gpair, params, GBT_POLICY_LOSSGUIDE, max_leaves,
                     tree, row_idx_out, leaf_of_row_out, workspace, workspace_bytes);
}

// ----------------------------------------------------------------- predict --
namespace {
size_t tree_bytes(int32_t n_nodes) { return gbt_align((size_t)n_nodes * 4) * 6 + gbt_align((size_t)n_nodes * 8); }
}

namespace {
// the plain staging (table of DevTree, then every tree's arrays) ...
size_t predict_plain_bytes(const gbt_tree *trees, int32_t n_trees) {
    size_t o = gbt_align((size_t)n_trees * sizeof(DevTree));
    for (int t = 0; t < n_trees; ++t) o += tree_bytes(trees[t].n_nodes);
    return o + 256;
}
// ... and behind it the form of the many-trees kernel: 8-byte nodes, weights, three small tables
struct BatchLayout {
    size_t nodes, wts, tree_off, tree_depth, group_end, total;
};
BatchLayout batch_layout(size_t base, int64_t total_nodes, int32_t n_trees) {
    BatchLayout L;
    size_t o = base;
    L.nodes = o;      o += gbt_align((size_t)total_nodes * 8);
    L.wts = o;        o += gbt_align((size_t)total_nodes * 8);
    L.tree_off = o;   o += gbt_align((size_t)(n_trees + 1) * 4);
    L.tree_depth = o; o += gbt_align((size_t)(n_trees + 1) * 4);
    L.group_end = o;  o += gbt_align((size_t)(n_trees + 1) * 4);
    L.total = o;
    return L;
}
int64_t total_nodes_of(const gbt_tree *trees, int32_t n_trees) {
    int64_t s = 0;
    for (int t = 0; t < n_trees; ++t) s += std::max(trees[t].n_nodes, 0);
    return s;
}
}  // namespace

extern "C" size_t gbt_predict_workspace_bytes(const gbt_tree *trees, int32_t n_trees) {
    if (!trees || n_trees < 0) return 0;
    return batch_layout(predict_plain_bytes(trees, n_trees), total_nodes_of(trees, n_trees), n_trees).total;
}

// Stages the trees in `workspace` and walks them: margin += eta * leaf weight per tree, or (leaf_out,
// one tree) the id of each row's leaf.  Does not synchronise.
static int32_t predict_impl(gbt_ctx *ctx, const gbt_tree *trees, int32_t n_trees, const uint32_t *packed,
                            int32_t bits, int32_t missing_sym, const float *X, int64_t n, int32_t F, double eta,
                            float *margin, int32_t *leaf_out, void *workspace, size_t workspace_bytes,
                            const SparseRowsArg *sparse, bool own_span, uint32_t *node_rows, const float *margin_src) {
    // node_rows: one tree over packed symbols; the walk also counts the rows per node (gbt_launch_predict)
    // margin_src (one tree, margin != NULL): margin[r] = margin_src[r] + eta * weight instead of margin[r] += ...
    // own_span: the walk is a profile span of its own (class "other"); callers inside a span pass false
    GBT_REQUIRE(ctx, trees && (margin || leaf_out) && workspace, GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, sparse || (packed != nullptr) != (X != nullptr), GBT_EINVAL, "give exactly one of packed and X");
    GBT_REQUIRE(ctx, n >= 0 && F >= 1 && n_trees >= 0, GBT_EINVAL, "bad shape");
    if (sparse) {
        bits = 1;
    } else if (packed) {
        int32_t st = check_matrix(ctx, packed, bits, n, F);
        if (st != GBT_OK) return st;
    } else {
        bits = 1;
    }
    const bool may_batch = X && margin && !leaf_out && n_trees >= 2;   // then the workspace also holds the batched form
    GBT_REQUIRE(ctx, workspace_bytes >= (may_batch ? gbt_predict_workspace_bytes(trees, n_trees)
                                                   : predict_plain_bytes(trees, n_trees)),
                GBT_ENOMEM, "workspace too small");
    bool compact_ok = true;   // the 8-byte node form of the register-window kernel applies
    // stage the trees: table of offsets, then each tree's arrays
    std::vector<char> host(predict_plain_bytes(trees, n_trees), 0);
    std::vector<int> depths((size_t)n_trees, 0);
    bool ordered = true;      // every child comes after its parent, in every tree
    DevTree *tab = (DevTree *)host.data();
    size_t o = gbt_align((size_t)n_trees * sizeof(DevTree));
    for (int t = 0; t < n_trees; ++t) {
        const gbt_tree &T = trees[t];
        GBT_REQUIRE(ctx, T.n_nodes >= 1 && T.n_nodes <= T.capacity, GBT_EINVAL, "tree %d: bad n_nodes", t);
        for (int i = 0; i < T.n_nodes; ++i) {
            if (T.feature[i] < 0) continue;
            if (T.right[i] != T.left[i] + 1 || T.feature[i] >= (1 << 20) || T.bin[i] < 0 || T.bin[i] >= 4096)
                compact_ok = false;
            GBT_REQUIRE(ctx, T.feature[i] < F && T.left[i] >= 0 && T.left[i] < T.n_nodes && T.right[i] >= 0 &&
                                 T.right[i] < T.n_nodes,
                        GBT_EINVAL, "tree %d node %d: bad feature or child id", t, i);
        }
        // the tree's depth (steps of its longest walk), if every child comes after its parent
        std::vector<int> depth_of((size_t)T.n_nodes, 0);
        int tree_depth = 0;
        for (int i = 0; i < T.n_nodes; ++i) {
            if (T.feature[i] < 0) continue;
            if (T.left[i] <= i || T.right[i] <= i) {
                compact_ok = false;
                ordered = false;
                break;
            }
            depth_of[T.left[i]] = depth_of[T.right[i]] = depth_of[i] + 1;
            tree_depth = std::max(tree_depth, depth_of[i] + 1);
        }
        const size_t a4 = gbt_align((size_t)T.n_nodes * 4);
        tab[t].n_nodes = T.n_nodes;
        tab[t].pad = tree_depth;
        depths[(size_t)t] = tree_depth;
        const void *src4[6] = {T.feature, T.bin, T.default_left, T.left, T.right, T.threshold};
        uint64_t *dst4[6] = {&tab[t].feature, &tab[t].bin, &tab[t].default_left, &tab[t].left, &tab[t].right,
                             &tab[t].threshold};
        for (int k = 0; k < 6; ++k) {
            memcpy(host.data() + o, src4[k], (size_t)T.n_nodes * 4);
            *dst4[k] = o;
            o += a4;
        }
        memcpy(host.data() + o, T.weight, (size_t)T.n_nodes * 8);
        tab[t].weight = o;
        o += gbt_align((size_t)T.n_nodes * 8);
    }
    GBT_HIP(ctx, hipMemcpyAsync(workspace, host.data(), o, hipMemcpyHostToDevice, ctx->stream));
    int max_nodes = 1;
    for (int t = 0; t < n_trees; ++t) max_nodes = std::max(max_nodes, trees[t].n_nodes);
    // Several trees on raw floats: one pass over the rows with the trees taken through LDS in groups
    // (needs right == left + 1 and children after parents, which grown trees have).
    if (may_batch && compact_ok && ordered && F <= gbt_predict_batch_max_features() && max_nodes <= 32767) {
        const size_t tile = (((size_t)256 * (size_t)(F | 1) * 4) + 15) & ~(size_t)15;
        int cap_nodes = std::max(2048, max_nodes);
        if (tile + (size_t)cap_nodes * 16 > ctx->lds_per_block) cap_nodes = max_nodes;
        if (tile + (size_t)cap_nodes * 16 <= ctx->lds_per_block) {
            const int64_t total_nodes = total_nodes_of(trees, n_trees);
            const BatchLayout BL = batch_layout(predict_plain_bytes(trees, n_trees), total_nodes, n_trees);
            std::vector<gbt_batch_node> bn((size_t)total_nodes);
            std::vector<double> bw((size_t)total_nodes);
            std::vector<int32_t> off((size_t)n_trees + 1), grp;
            int64_t run = 0;
            int in_group = 0;
            for (int t = 0; t < n_trees; ++t) {
                const gbt_tree &T = trees[t];
                if (in_group + T.n_nodes > cap_nodes) {   // the group is full: it ends before this tree
                    grp.push_back(t);
                    in_group = 0;
                }
                in_group += T.n_nodes;
                off[(size_t)t] = (int32_t)run;
                for (int i = 0; i < T.n_nodes; ++i) {
                    gbt_batch_node q;
                    if (T.feature[i] < 0) {
                        q.thr = INFINITY;
                        q.meta = (uint32_t)i | (1u << 15);
                    } else {
                        q.thr = T.threshold[i];
                        q.meta = (uint32_t)T.left[i] | ((T.default_left[i] ? 1u : 0u) << 15) | (1u << 16) |
                                 ((uint32_t)T.feature[i] << 17);
                    }
                    bn[(size_t)(run + i)] = q;
                    bw[(size_t)(run + i)] = T.weight[i];
                }
                run += T.n_nodes;
            }
            off[(size_t)n_trees] = (int32_t)run;
            grp.push_back(n_trees);
            char *wsb = (char *)workspace;
            const size_t per_upload = kUploadBytes;
            auto put = [&](const void *src, size_t bytes, size_t at) -> int32_t {
                for (size_t o2 = 0; o2 < bytes; o2 += per_upload) {
                    int32_t st2 = upload(ctx, (const char *)src + o2, std::min(per_upload, bytes - o2), wsb + at + o2);
                    if (st2 != GBT_OK) return st2;
                }
                return GBT_OK;
            };
            int32_t st = put(bn.data(), bn.size() * 8, BL.nodes);
            if (st == GBT_OK) st = put(bw.data(), bw.size() * 8, BL.wts);
            if (st == GBT_OK) st = put(off.data(), off.size() * 4, BL.tree_off);
            if (st == GBT_OK) st = put(depths.data(), depths.size() * 4, BL.tree_depth);
            if (st == GBT_OK) st = put(grp.data(), grp.size() * 4, BL.group_end);
            if (st != GBT_OK) return st;
            if (own_span) gbt_prof_begin(ctx, GBT_PROF_OTHER, (double)n * ((double)F * 4.0 + 8.0));
            GBT_HIP(ctx, gbt_launch_predict_raw_batched(ctx->stream, (const gbt_batch_node *)(wsb + BL.nodes),
                                                        (const double *)(wsb + BL.wts), (const int32_t *)(wsb + BL.tree_off),
                                                        (const int32_t *)(wsb + BL.tree_depth),
                                                        (const int32_t *)(wsb + BL.group_end), (int)grp.size(), cap_nodes,
                                                        X, n, F, eta, margin));
            if (own_span) gbt_prof_end(ctx);
            return GBT_OK;
        }
    }
    if (sparse) {
        if (own_span) gbt_prof_begin(ctx, GBT_PROF_OTHER, 0.0);
        GBT_HIP(ctx, gbt_launch_sparse_walk(ctx->stream, (const char *)workspace, (const DevTree *)workspace, n_trees,
                                            sparse->rowptr, sparse->ent, sparse->ent_bytes, n, sparse->B, eta, margin, leaf_out, max_nodes));
        if (own_span) gbt_prof_end(ctx);
        return GBT_OK;
    }
    if (margin_src == margin) margin_src = nullptr;
    if (margin_src) {
        GBT_REQUIRE(ctx, n_trees == 1 && margin && !leaf_out && !sparse, GBT_EINVAL, "internal: margin_src");
        if (!gbt_predict_counts_ok(packed != nullptr, bits, F, max_nodes, compact_ok)) {   // no kernel form reads it: copy first
            GBT_HIP(ctx, hipMemcpyAsync(margin, margin_src, (size_t)n * sizeof(float), hipMemcpyDeviceToDevice, ctx->stream));
            margin_src = nullptr;
        }
    }
    if (own_span) gbt_prof_begin(ctx, GBT_PROF_OTHER, 0.0);
    GBT_HIP(ctx, gbt_launch_predict(ctx->stream, (const char *)workspace, (const DevTree *)workspace, n_trees, packed,
                                    bits, (uint32_t)missing_sym, X, n, F, eta, margin, leaf_out, max_nodes,
                                    compact_ok, node_rows, margin_src));
    if (own_span) gbt_prof_end(ctx);
    return GBT_OK;
}

extern "C" int32_t gbt_predict(gbt_ctx *ctx, const gbt_tree *trees, int32_t n_trees, const uint32_t *packed,
                               int32_t bits, int32_t missing_sym, const float *X, int64_t n, int32_t F, double eta,
                               float *margin, void *workspace, size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, margin != nullptr, GBT_EINVAL, "NULL argument");
    int32_t st = predict_impl(ctx, trees, n_trees, packed, bits, missing_sym, X, n, F, eta, margin, nullptr, workspace,
                              workspace_bytes, nullptr, true);
    if (st != GBT_OK) return st;
    GBT_SYNC(ctx);
    return GBT_OK;
}

// ------------------------------------------------------------- sparse rows --
namespace {
constexpr int64_t kSparseSlack = 32;   // entries past the last one that word-wise readers may touch
constexpr int64_t kSparseMaxIds = (int64_t)1 << 28;

int32_t check_sparse_shape(gbt_ctx *ctx, int64_t n, int32_t F, int32_t B) {
    GBT_REQUIRE(ctx, n >= 0 && n < ((int64_t)1 << 32) - 1, GBT_EINVAL, "n = %lld out of range", (long long)n);
    GBT_REQUIRE(ctx, F >= 1 && B >= 2, GBT_EINVAL, "bad shape");
    GBT_REQUIRE(ctx, (int64_t)F * B <= kSparseMaxIds, GBT_EUNSUPPORTED,
                "F * max_bins = %lld global bin ids, at most %lld", (long long)F * B, (long long)kSparseMaxIds);
    return GBT_OK;
}
// bytes of an entry: 16-bit ids where all of them fit, else 32-bit
int sparse_ent_bytes(int64_t F, int64_t B) { return F * B <= 65536 ? 2 : 4; }

// Rows per workgroup: every workgroup merges its whole id tile into HBM at the end with 64-bit global
// atomics (about 10^11 of them per second, all compute units together), so a launch aims at few, long
// jobs: the rows are cut into about one piece per compute unit, whatever the number of id tiles.
uint32_t sparse_rows_per_job(const gbt_ctx *ctx, int64_t total_rows, int64_t bins, int glen) {
    (void)bins;
    (void)glen;
    int64_t per_tile = std::max<int64_t>(1, (int64_t)ctx->num_cu * ctx->sparse_jobs_per_cu);
    int64_t rpj = (total_rows + per_tile - 1) / per_tile;
    if (rpj < 2048) rpj = 2048;
    if (rpj > ((int64_t)1 << 24)) rpj = (int64_t)1 << 24;
    return (uint32_t)rpj;
}

// jobs over rows [begin, begin + len) for every id tile of a node
void add_sparse_hist_jobs(std::vector<HistJob> &jobs, uint64_t hist_off, uint32_t begin, uint32_t len, int64_t bins,
                          int glen, uint32_t rows_per_job) {
    for (uint32_t r0 = 0; r0 < len; r0 += rows_per_job) {
        const uint32_t nr = std::min(rows_per_job, len - r0);
        for (int64_t g0 = 0; g0 < bins; g0 += glen) {
            HistJob j;
            j.hist_off = hist_off;
            j.row_begin = begin + r0;
            j.n_rows = nr;
            j.f0 = (uint32_t)g0;
            j.ft = (uint32_t)std::min<int64_t>(glen, bins - g0);
            j.pad0 = j.pad1 = 0;
            jobs.push_back(j);
        }
    }
}
}  // namespace

extern "C" int32_t gbt_sparse_entry_bytes(int32_t F, int32_t max_bins) {
    if (F < 1 || max_bins < 2 || (int64_t)F * max_bins > kSparseMaxIds) return 0;
    return sparse_ent_bytes(F, max_bins);
}

extern "C" int64_t gbt_sparse_capacity(int64_t nnz) {
    if (nnz < 0) return 0;
    return ((nnz + 1) & ~(int64_t)1) + kSparseSlack;
}

extern "C" size_t gbt_compress_sparse_workspace_bytes(int64_t n) {
    if (n < 0) return 0;
    return gbt_align((size_t)gbt_sparse_scan_tiles(n) * 8) + 256;
}

extern "C" int32_t gbt_compress_sparse_count(gbt_ctx *ctx, const uint16_t *sym, int64_t n, int32_t F,
                                             int32_t missing_sym, uint32_t *rowptr_out, int64_t *nnz_out,
                                             void *workspace, size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, sym && rowptr_out && nnz_out && workspace, GBT_EINVAL, "NULL argument");
    GBT_REQUIRE(ctx, n >= 0 && n < ((int64_t)1 << 32) - 1 && F >= 1, GBT_EINVAL, "bad shape");
    GBT_REQUIRE(ctx, missing_sym >= 0 && missing_sym <= 65535, GBT_EINVAL, "missing_sym out of range");
    GBT_REQUIRE(ctx, workspace_bytes >= gbt_compress_sparse_workspace_bytes(n), GBT_ENOMEM, "workspace too small");
    char *ws = (char *)workspace;
    uint64_t *total = (uint64_t *)ws;
    uint64_t *tile_ws = (uint64_t *)(ws + 256);
    GBT_HIP(ctx, gbt_launch_sparse_rowptr(ctx->stream, sym, n, F, (uint32_t)missing_sym, rowptr_out, tile_ws, total));
    GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), total, 8, hipMemcpyDeviceToHost, ctx->stream));
    GBT_SYNC(ctx);
    uint64_t nnz;
    memcpy(&nnz, rb(ctx), 8);
    GBT_REQUIRE(ctx, nnz < ((uint64_t)1 << 32) - 64, GBT_EUNSUPPORTED, "%llu present elements exceed 32-bit row pointers",
                (unsigned long long)nnz);
    *nnz_out = (int64_t)nnz;
    return GBT_OK;
}

extern "C" int32_t gbt_compress_sparse(gbt_ctx *ctx, const uint16_t *sym, int64_t n, int32_t F, int32_t max_bins,
                                       int32_t missing_sym, const uint32_t *rowptr, int64_t nnz, void *ent_out,
                                       int64_t ent_capacity) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, sym && rowptr && ent_out, GBT_EINVAL, "NULL argument");
    int32_t st = check_sparse_shape(ctx, n, F, max_bins);
    if (st != GBT_OK) return st;
    GBT_REQUIRE(ctx, missing_sym >= 0 && missing_sym <= 65535, GBT_EINVAL, "missing_sym out of range");
    GBT_REQUIRE(ctx, nnz >= 0 && ent_capacity >= gbt_sparse_capacity(nnz), GBT_ENOMEM,
                "ent_out holds %lld entries, %lld needed", (long long)ent_capacity, (long long)gbt_sparse_capacity(nnz));
    GBT_REQUIRE(ctx, ((uintptr_t)ent_out & 3) == 0, GBT_EINVAL, "ent_out must be 4-byte aligned");
    GBT_HIP(ctx, gbt_launch_sparse_fill(ctx->stream, sym, n, F, max_bins, (uint32_t)missing_sym, rowptr, ent_out,
                                        sparse_ent_bytes(F, max_bins), nnz, gbt_sparse_capacity(nnz)));
    return GBT_OK;
}

extern "C" int32_t gbt_build_hist_sparse(gbt_ctx *ctx, const uint32_t *rowptr, const void *ent, int64_t n,
                                         int32_t F, int32_t B, int64_t row_begin, int64_t n_node_rows,
                                         const int32_t *gq, int64_t *hist_out) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, rowptr && ent && gq && hist_out, GBT_EINVAL, "NULL argument");
    int32_t st = check_sparse_shape(ctx, n, F, B);
    if (st != GBT_OK) return st;
    GBT_REQUIRE(ctx, ((uintptr_t)ent & 3) == 0, GBT_EINVAL, "ent must be 4-byte aligned");
    GBT_REQUIRE(ctx, row_begin >= 0 && n_node_rows >= 0 && row_begin + n_node_rows <= n, GBT_EINVAL,
                "rows [%lld, +%lld) outside the matrix", (long long)row_begin, (long long)n_node_rows);
    const int64_t bins = (int64_t)F * B;
    GBT_HIP(ctx, gbt_launch_fill_u64(ctx->stream, (uint64_t *)hist_out, 0, bins * 2));
    if (n_node_rows == 0) return GBT_OK;
    const int glen = gbt_sparse_hist_tile(ctx, bins);
    std::vector<HistJob> jobs;
    add_sparse_hist_jobs(jobs, 0, (uint32_t)row_begin, (uint32_t)n_node_rows, bins, glen,
                         sparse_rows_per_job(ctx, n_node_rows, bins, glen));
    char *slot;
    st = stage(ctx, jobs.data(), jobs.size() * sizeof(HistJob), &slot);
    if (st != GBT_OK) return st;
    gbt_prof_begin(ctx, row_begin == 0 && n_node_rows == n ? GBT_PROF_HIST_ROOT : GBT_PROF_HIST_NODE, 0.0);
    GBT_HIP(ctx, gbt_launch_sparse_hist(ctx, rowptr, ent, sparse_ent_bytes(F, B), gq, hist_out, (const HistJob *)slot,
                                        (int)jobs.size(), glen, glen < bins));
    gbt_prof_end(ctx);
    return GBT_OK;
}

namespace {
struct SparseGrowLayout {
    size_t gq, rowptr[2], ent[2], wgq[2], state, pool, eval_nodes, jobs, scratch, tree_stage, tree_stage_bytes,
        order, rank_tbl, total;
    int64_t hist_nodes, level_nodes;
};
// hist_nodes: nodes that may own a histogram (ids below it); level_nodes: most nodes split in one round
SparseGrowLayout sparse_grow_layout_nodes(int64_t n, int64_t nnz, int F, int B, int64_t hist_nodes, int64_t level_nodes) {
    SparseGrowLayout L;
    L.hist_nodes = hist_nodes;
    L.level_nodes = level_nodes;
    size_t o = 0;
    L.gq = o; o += gbt_align((size_t)n * 8);
    for (int k = 0; k < 2; ++k) {
        L.rowptr[k] = o; o += gbt_align((size_t)(n + 1) * 4);
        L.ent[k] = o;    o += gbt_align((size_t)gbt_sparse_capacity(nnz) * sparse_ent_bytes(F, B));
        L.wgq[k] = o;    o += gbt_align((size_t)n * 8);
    }
    L.state = o;      o += gbt_align((size_t)L.level_nodes * 16);
    L.pool = o;       o += gbt_align((size_t)L.hist_nodes * F * B * 16);
    L.eval_nodes = o; o += gbt_align((size_t)L.level_nodes * 2 * sizeof(EvalNode));
    L.jobs = o;       o += gbt_align(kUploadBytes);
    L.scratch = o;    o += 4096;
    const size_t cap_nodes = (size_t)(2 * L.hist_nodes + 1);
    L.tree_stage_bytes = gbt_align(64) + gbt_align(cap_nodes * 4) * 6 + gbt_align(cap_nodes * 8) + 256;
    L.tree_stage = o; o += gbt_align(L.tree_stage_bytes);
    L.order = o;      o += gbt_order_ws(n);
    L.rank_tbl = o;   o += gbt_align(cap_nodes * 4);
    L.total = o;
    return L;
}
SparseGrowLayout sparse_grow_layout(int64_t n, int64_t nnz, int F, int B, int max_depth) {
    return sparse_grow_layout_nodes(n, nnz, F, B, max_depth == 0 ? 1 : (((int64_t)1 << max_depth) - 1),
                                    (int64_t)1 << (max_depth > 0 ? max_depth - 1 : 0));
}
}  // namespace

extern "C" size_t gbt_grow_tree_sparse_workspace_bytes(int64_t n, int64_t nnz, int32_t F, int32_t max_bins,
                                                       int32_t max_depth) {
    if (n < 0 || nnz < 0 || F < 1 || max_bins < 2 || (int64_t)F * max_bins > kSparseMaxIds || max_depth < 0 ||
        max_depth > kMaxDepth)
        return 0;
    return sparse_grow_layout(n, nnz, F, max_bins, max_depth).total;
}

// Alg. 1 over sparse rows under either policy of Sec. 2.3: the loop of grow_impl with the sparse-row kernels (rounds,
// and for loss-guided growth the physical and the logical tree, exactly as there).  Rows move without ids through
// one-launch unordered partitions; leaf ids come from a walk of the finished tree, the row order from a stable sort
// by leaf rank.
static int32_t sparse_grow_impl(gbt_ctx *ctx, const uint32_t *rowptr, const void *ent, int64_t n,
                                int64_t nnz, int32_t F, const int32_t *nb, const float *cuts,
                                const float *gpair, const gbt_params *params, int policy, int32_t max_leaves, gbt_tree *tree,
                                uint32_t *row_idx_out, int32_t *leaf_of_row_out, void *workspace,
                                size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, rowptr && ent && nb && cuts && gpair && params && tree && workspace, GBT_EINVAL, "NULL argument");
    const int B = params->max_bins, max_depth = params->max_depth;
    int32_t st = check_sparse_shape(ctx, n, F, B);
    if (st != GBT_OK) return st;
    st = check_bins(ctx, F, B);
    if (st != GBT_OK) return st;
    GBT_REQUIRE(ctx, ((uintptr_t)ent & 3) == 0, GBT_EINVAL, "ent must be 4-byte aligned");
    GBT_REQUIRE(ctx, n >= 1 && nnz >= 0 && nnz < ((int64_t)1 << 32) - 64, GBT_EINVAL, "bad n or nnz");
    const bool lossguide = policy == GBT_POLICY_LOSSGUIDE;
    GBT_REQUIRE(ctx, max_depth >= 0, GBT_EINVAL, "max_depth < 0");
    GBT_REQUIRE(ctx, lossguide || max_depth <= kMaxDepth, GBT_EUNSUPPORTED, "max_depth %d > %d", max_depth, kMaxDepth);
    GBT_REQUIRE(ctx, !lossguide || (max_leaves >= 1 && max_leaves <= kMaxLeaves), lossguide && max_leaves >= 1 ? GBT_EUNSUPPORTED : GBT_EINVAL,
                "max_leaves %d outside 1..%d", max_leaves, kMaxLeaves);
    GBT_REQUIRE(ctx, params->lambda >= 0.0, GBT_EINVAL, "lambda < 0");
    const int64_t cap = lossguide ? 2 * (int64_t)max_leaves - 1 : ((int64_t)1 << (max_depth + 1)) - 1;
    GBT_REQUIRE(ctx, tree->capacity >= cap, GBT_EINVAL, "tree capacity %d < %lld", tree->capacity, (long long)cap);
    GBT_REQUIRE(ctx, tree->feature && tree->bin && tree->default_left && tree->left && tree->right &&
                         tree->threshold && tree->weight && tree->gain && tree->sumG && tree->sumH && tree->n_rows,
                GBT_EINVAL, "tree arrays must be allocated");
    const int64_t cap_phys = lossguide ? lossguide_phys_nodes(max_leaves) : cap;
    const SparseGrowLayout L = lossguide ? sparse_grow_layout_nodes(n, nnz, F, B, cap_phys, kLossguideBatchMax)
                                         : sparse_grow_layout(n, nnz, F, B, max_depth);
    GBT_REQUIRE(ctx, workspace_bytes >= L.total, GBT_ENOMEM, "workspace %zu < %zu bytes", workspace_bytes, L.total);

    char *ws = (char *)workspace;
    hipStream_t s = ctx->stream;
    int32_t *gq = (int32_t *)(ws + L.gq);
    int64_t *pool = (int64_t *)(ws + L.pool);
    const int64_t bins = (int64_t)F * B, hist_len = bins * 2;
    const int glen = gbt_sparse_hist_tile(ctx, bins);
    const int ent_bytes = sparse_ent_bytes(F, B);
    struct Rows { const uint32_t *rowptr; const void *ent; const int32_t *gq; };
    const Rows canon{rowptr, ent, gq};
    uint32_t *w_rowptr[2] = {(uint32_t *)(ws + L.rowptr[0]), (uint32_t *)(ws + L.rowptr[1])};
    void *w_ent[2] = {(void *)(ws + L.ent[0]), (void *)(ws + L.ent[1])};
    int32_t *w_gq[2] = {(int32_t *)(ws + L.wgq[0]), (int32_t *)(ws + L.wgq[1])};
    auto rows_of = [&](int buf) { return buf == 2 ? canon : Rows{w_rowptr[buf], w_ent[buf], w_gq[buf]}; };
    std::vector<float> hcuts((size_t)F * (B - 1));
    GBT_HIP(ctx, hipMemcpyAsync(hcuts.data(), cuts, hcuts.size() * sizeof(float), hipMemcpyDeviceToHost, s));

    double scale[2];
    int64_t *sums_dev = (int64_t *)(ws + L.scratch + 256);
    gbt_prof_begin(ctx, GBT_PROF_OTHER, (double)n * 24.0);
    st = gpair_scale_impl(ctx, gpair, n, scale, ws + L.scratch);
    if (st == GBT_OK) {
        hipError_t e = gbt_launch_to_fixed(s, gpair, n, scale[0], scale[1], gq, sums_dev);
        if (e != hipSuccess) st = gbt_fail(ctx, GBT_EHIP, "gbt_launch_to_fixed: %s", hipGetErrorString(e));
    }
    gbt_prof_end(ctx);
    if (st != GBT_OK) return st;
    const double inv_sg = 1.0 / scale[0], inv_sh = 1.0 / scale[1];
    const double lambda = params->lambda;
    const double min_gain = std::max(params->gamma, (double)GBT_GAIN_FLOOR);
    const double row_bytes = 12.0 + (double)ent_bytes * (double)nnz / (double)n;   // row pointer, pair, the average row's entries

    std::vector<HistJob> hjobs;
    auto launch_hist = [&](const Rows &R, int cls, double bytes) -> int32_t {
        const size_t per_launch = kUploadBytes / sizeof(HistJob);
        for (size_t j0 = 0; j0 < hjobs.size(); j0 += per_launch) {
            const size_t nj = std::min(per_launch, hjobs.size() - j0);
            int32_t st2 = upload(ctx, hjobs.data() + j0, nj * sizeof(HistJob), ws + L.jobs);
            if (st2 != GBT_OK) return st2;
            gbt_prof_begin(ctx, cls, j0 == 0 ? bytes : 0.0);
            GBT_HIP(ctx, gbt_launch_sparse_hist(ctx, R.rowptr, R.ent, ent_bytes, R.gq, pool, (const HistJob *)(ws + L.jobs), (int)nj,
                                                glen, glen < bins));
            gbt_prof_end(ctx);
        }
        return GBT_OK;
    };

    const bool root_may_split = max_depth > 0 && (!lossguide || max_leaves > 1);
    if (root_may_split) {
        GBT_HIP(ctx, gbt_launch_fill_u64(s, (uint64_t *)pool, 0, hist_len));
        hjobs.clear();
        add_sparse_hist_jobs(hjobs, 0, 0, (uint32_t)n, bins, glen, sparse_rows_per_job(ctx, n, bins, glen));
        st = launch_hist(canon, GBT_PROF_HIST_ROOT, (double)n * row_bytes);
        if (st != GBT_OK) return st;
    }
    GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), sums_dev, 16, hipMemcpyDeviceToHost, s));
    GBT_SYNC(ctx);
    int64_t root_sums[2];
    memcpy(root_sums, rb(ctx), 16);

    auto set_node_at = [&](int32_t at, const HNode &nd) {
        const double G = (double)nd.Gq * inv_sg, H = (double)nd.Hq * inv_sh;
        tree->feature[at] = -1;
        tree->bin[at] = 0;
        tree->default_left[at] = 0;
        tree->left[at] = tree->right[at] = -1;
        tree->threshold[at] = INFINITY;
        tree->gain[at] = 0.0;
        tree->sumG[at] = G;
        tree->sumH[at] = H;
        tree->weight[at] = H + lambda > 0.0 ? -G / (H + lambda) : 0.0;   // no curvature, no step
        tree->n_rows[at] = nd.len;
    };
    auto set_node = [&](const HNode &nd) { set_node_at(nd.id, nd); };
    std::vector<HNode> level, next, sel_nodes;
    std::vector<gbt_split> splits, sel_splits;
    std::vector<EvalNode> enodes;
    std::vector<PartJob> pjobs;
    HNode root{0, 0, (uint32_t)n, root_sums[0], root_sums[1], 0, 2};
    set_node(root);
    if (root_may_split) level.push_back(root);
    int32_t n_nodes = 1, n_leaves = 1;
    constexpr size_t kSplitRb = 512u << 10;
    // loss-guided growth: physical nodes are made in rounds, the caller's tree follows the sequential rule over
    // what is known (see grow_impl)
    struct Phys {
        HNode nd;
        gbt_split sp;
        int32_t lc, rc;        // physical children, -1: not expanded
        int32_t logical;       // id in the caller's tree, -1: not (yet) part of it
        bool open;             // has a split that may be taken
    };
    std::vector<Phys> phys;
    struct OpenKey {   // order of turns: larger gain first, smaller logical id on equal gains
        double gain;
        int32_t logical, pid;
        bool operator<(const OpenKey &o) const { return gain > o.gain || (gain == o.gain && logical < o.logical); }
    };
    std::set<OpenKey> sim_open;
    int32_t n_logical = 1;
    if (lossguide) phys.push_back(Phys{root, gbt_split{}, -1, -1, 0, false});
    const int batch_max = std::max(1, std::min(ctx->lossguide_batch, kLossguideBatchMax));

    while (!level.empty() || !sim_open.empty()) {
        if (!level.empty()) {
            // ---- EvaluateSplit for the level's nodes
            enodes.resize(level.size());
            for (size_t i = 0; i < level.size(); ++i)
                enodes[i] = EvalNode{(uint64_t)level[i].id * (uint64_t)hist_len, level[i].Gq, level[i].Hq,
                                     level[i].sub_parent >= 0 ? (uint64_t)level[i].sub_parent * (uint64_t)hist_len : GBT_NO_HIST,
                                     level[i].sub_parent >= 0 ? (uint64_t)level[i].sub_built * (uint64_t)hist_len : GBT_NO_HIST};
            st = upload(ctx, enodes.data(), enodes.size() * sizeof(EvalNode), ws + L.eval_nodes);
            if (st != GBT_OK) return st;
            const size_t budget = GBT_STAGING_BYTES - kReadbackOff - kSplitRb;
            const int chunks = gbt_eval_chunks(F, (int)enodes.size(), budget);
            const size_t sbytes = enodes.size() * (size_t)chunks * sizeof(gbt_split);
            GBT_REQUIRE(ctx, sbytes <= budget, GBT_EUNSUPPORTED, "level too wide");
            gbt_prof_begin(ctx, GBT_PROF_EVAL, (double)enodes.size() * (double)hist_len * 8.0);
            // (the records go straight into the pinned read-back buffer: no copy launch before the wait)
            EvalTail plain{nullptr, nullptr, 0, 0, -1, 0};
            plain.skip_store = !lossguide && level[0].depth >= max_depth - 1 ? 1 : 0;   // (their children are leaves)
            GBT_HIP(ctx, gbt_launch_eval(s, pool, (const EvalNode *)(ws + L.eval_nodes), (int)enodes.size(), nb, F, B, chunks,
                                         inv_sg, inv_sh, lambda, params->min_child_weight, (gbt_split *)(rb(ctx) + kSplitRb),
                                         plain));
            gbt_prof_end(ctx);
            GBT_SYNC(ctx);
            sel_nodes.clear();
            sel_splits.clear();
            for (size_t i = 0; i < level.size(); ++i) {
                const gbt_split sp = merge_chunks((const gbt_split *)(rb(ctx) + kSplitRb) + i * chunks, chunks);
                const HNode &nd = level[i];
                const bool ok = sp.valid && sp.gain > min_gain && sp.feature >= 0 && sp.feature < F && sp.bin >= 0 &&
                                sp.bin < B && nd.len > 0;
                if (lossguide) {
                    Phys &ph = phys[(size_t)nd.id];
                    ph.sp = sp;
                    ph.open = ok;
                    if (ok && ph.logical >= 0) sim_open.insert(OpenKey{sp.gain, ph.logical, nd.id});   // the root
                } else if (ok) {
                    sel_nodes.push_back(nd);
                    sel_splits.push_back(sp);
                }
            }
            level.clear();
        } else {
            sel_nodes.clear();
            sel_splits.clear();
        }
        if (lossguide) {
            // the logical tree advances as far as the physical expansions reach
            while (n_leaves < max_leaves && !sim_open.empty()) {
                const int32_t pid = sim_open.begin()->pid;
                Phys &ph = phys[(size_t)pid];
                if (ph.lc < 0) break;   // its turn, but not expanded yet: a round is needed
                sim_open.erase(sim_open.begin());
                const int32_t at = ph.logical, lcl = n_logical, rcl = n_logical + 1;
                GBT_REQUIRE(ctx, rcl < tree->capacity, GBT_EHIP, "internal: logical tree overflow");
                n_logical += 2;
                n_leaves += 1;
                tree->feature[at] = ph.sp.feature;
                tree->bin[at] = ph.sp.bin;
                tree->default_left[at] = ph.sp.default_left;
                tree->left[at] = lcl;
                tree->right[at] = rcl;
                tree->gain[at] = ph.sp.gain;
                tree->threshold[at] = ph.sp.bin < B - 1 ? hcuts[(size_t)ph.sp.feature * (B - 1) + ph.sp.bin] : INFINITY;
                for (int side = 0; side < 2; ++side) {
                    const int32_t cid = side == 0 ? ph.lc : ph.rc;
                    Phys &ch = phys[(size_t)cid];
                    ch.logical = side == 0 ? lcl : rcl;
                    set_node_at(ch.logical, ch.nd);
                    if (ch.open) sim_open.insert(OpenKey{ch.sp.gain, ch.logical, cid});
                }
            }
            if (n_leaves < max_leaves && !sim_open.empty()) {
                // the leaf whose turn it is and the next ones in gain order that live in the same working copy and
                // agree with it on whether their children can still split (see grow_impl)
                const int64_t room = (cap_phys - n_nodes) / 2, budget = (int64_t)max_leaves - n_leaves;
                const int64_t k_max = std::max<int64_t>(1, std::min<int64_t>({(int64_t)batch_max, budget, room - budget + 1}));
                const HNode first = phys[(size_t)sim_open.begin()->pid].nd;
                int looked = 0;
                for (const OpenKey &key : sim_open) {
                    if (++looked > 8 * kLossguideBatchMax) break;
                    const Phys &ph = phys[(size_t)key.pid];
                    if (ph.lc >= 0) continue;   // expanded ahead of its turn already
                    if (ph.nd.buf != first.buf || (ph.nd.depth + 1 < max_depth) != (first.depth + 1 < max_depth)) continue;
                    sel_nodes.push_back(ph.nd);
                    sel_splits.push_back(ph.sp);
                    if ((int64_t)sel_nodes.size() >= k_max) break;
                }
            }
        }
        if (sel_nodes.empty()) break;

        // ---- RepartitionInstances: the whole level in one launch
        const int wcur = sel_nodes[0].buf, wnext = wcur == 0 ? 1 : 0;
        const Rows cur = rows_of(wcur);
        const int child_depth = sel_nodes[0].depth + 1;   // loss-guided: of the first node; the others agree on "< max_depth"
        const bool children_need_hist = child_depth < max_depth && (!lossguide || n_leaves + 1 < max_leaves);
        const uint32_t tile = (uint32_t)gbt_sparse_part_tile();
        pjobs.clear();
        uint32_t tile_cursor = 0;
        double part_rows = 0;
        for (size_t k = 0; k < sel_nodes.size(); ++k) {
            PartJob j;
            j.seg_begin = sel_nodes[k].begin;
            j.seg_len = sel_nodes[k].len;
            j.feature = (uint32_t)sel_splits[k].feature;
            j.bin = (uint32_t)sel_splits[k].bin;
            j.default_left = (uint32_t)sel_splits[k].default_left;
            j.tile_begin = tile_cursor;
            j.n_tiles = (j.seg_len + tile - 1) / tile;
            j.pad = 2;
            j.hist_off = 0;
            tile_cursor += j.n_tiles;
            part_rows += j.seg_len;
            pjobs.push_back(j);
        }
        GBT_REQUIRE(ctx, pjobs.size() * sizeof(PartJob) <= kUploadBytes && pjobs.size() * 16 <= kSplitRb, GBT_EUNSUPPORTED,
                    "level too wide");
        st = upload(ctx, pjobs.data(), pjobs.size() * sizeof(PartJob), ws + L.jobs);
        if (st != GBT_OK) return st;
        gbt_prof_begin(ctx, GBT_PROF_PARTITION, part_rows * (children_need_hist ? 2.0 * row_bytes : row_bytes - 8.0));
        GBT_HIP(ctx, gbt_launch_sparse_partition(s, cur.rowptr, cur.ent, ent_bytes, cur.gq, w_rowptr[wnext], w_ent[wnext], w_gq[wnext],
                                                 B, children_need_hist, (const PartJob *)(ws + L.jobs), (int)pjobs.size(),
                                                 (int)tile_cursor, (unsigned long long *)(ws + L.state)));
        GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), ws + L.state, pjobs.size() * 16, hipMemcpyDeviceToHost, s));
        gbt_prof_end(ctx);
        GBT_SYNC(ctx);
        const uint32_t *cur_words = (const uint32_t *)rb(ctx);   // four words per job; the first: left rows

        // ---- children, in creation order; the child with fewer rows is built from rows
        hjobs.clear();
        next.clear();
        int64_t built_rows = 0;
        const int32_t first_child = n_nodes;
        const int child_buf = children_need_hist ? wnext : wcur;
        struct Built { uint64_t off; uint32_t begin, len; };
        std::vector<Built> built;
        for (size_t k = 0; k < pjobs.size(); ++k) {
            const HNode &nd = sel_nodes[k];
            const gbt_split &sp = sel_splits[k];
            const uint32_t nl = cur_words[4 * k];
            GBT_REQUIRE(ctx, nl <= nd.len, GBT_EHIP, "internal: n_left %u > %u", nl, nd.len);
            HNode lc{n_nodes, nd.begin, nl, sp.GLq, sp.HLq, nd.depth + 1, child_buf};
            HNode rc{n_nodes + 1, nd.begin + nl, nd.len - nl, nd.Gq - sp.GLq, nd.Hq - sp.HLq, nd.depth + 1, child_buf};
            n_nodes += 2;
            if (lossguide) {   // physical children; the caller's tree learns of them when their parent is popped
                GBT_REQUIRE(ctx, n_nodes <= cap_phys, GBT_EHIP, "internal: physical node overflow");
                phys[(size_t)nd.id].lc = lc.id;
                phys[(size_t)nd.id].rc = rc.id;
                phys.push_back(Phys{lc, gbt_split{}, -1, -1, -1, false});
                phys.push_back(Phys{rc, gbt_split{}, -1, -1, -1, false});
            } else {
                tree->feature[nd.id] = sp.feature;
                tree->bin[nd.id] = sp.bin;
                tree->default_left[nd.id] = sp.default_left;
                tree->left[nd.id] = lc.id;
                tree->right[nd.id] = rc.id;
                tree->gain[nd.id] = sp.gain;
                tree->threshold[nd.id] = sp.bin < B - 1 ? hcuts[(size_t)sp.feature * (B - 1) + sp.bin] : INFINITY;
                set_node(lc);
                set_node(rc);
            }
            if (children_need_hist) {
                const bool left_small = lc.len <= rc.len;
                const HNode &sm = left_small ? lc : rc;
                built.push_back(Built{(uint64_t)sm.id * (uint64_t)hist_len, sm.begin, sm.len});
                built_rows += sm.len;
                HNode &other = left_small ? rc : lc;   // its histogram: parent - built, made when it is evaluated
                other.sub_parent = nd.id;
                other.sub_built = sm.id;
                next.push_back(lc);
                next.push_back(rc);
            }
        }
        if (children_need_hist) {
            const int32_t n_children = n_nodes - first_child;
            gbt_prof_begin(ctx, GBT_PROF_CLEAR, (double)n_children * (double)hist_len * 8.0);
            GBT_HIP(ctx, gbt_launch_fill_u64(s, (uint64_t *)(pool + (int64_t)first_child * hist_len), 0,
                                             (int64_t)n_children * hist_len));
            gbt_prof_end(ctx);
            const uint32_t rpj = sparse_rows_per_job(ctx, built_rows, bins, glen);
            for (const Built &b : built) add_sparse_hist_jobs(hjobs, b.off, b.begin, b.len, bins, glen, rpj);
            st = launch_hist(rows_of(wnext), GBT_PROF_HIST_NODE, (double)built_rows * row_bytes);
            if (st != GBT_OK) return st;
        }
        level.swap(next);
    }
    const int32_t n_tree = lossguide ? n_logical : n_nodes;   // nodes of the caller's tree
    tree->n_nodes = n_tree;

    // ---- each row's leaf by a walk of the finished tree; the row order by a stable sort on leaf rank
    int32_t *leaf_ids = leaf_of_row_out ? leaf_of_row_out : (int32_t *)w_rowptr[0];
    if (leaf_of_row_out || row_idx_out) {
        const SparseRowsArg sr{rowptr, ent, ent_bytes, B};
        gbt_prof_begin(ctx, GBT_PROF_OTHER, (double)n * (row_bytes - 8.0 + 4.0));
        st = predict_impl(ctx, tree, 1, nullptr, 1, 0, nullptr, n, F, 0.0, nullptr, leaf_ids, ws + L.tree_stage,
                          L.tree_stage_bytes, &sr);
        gbt_prof_end(ctx);
        if (st != GBT_OK) return st;
    }
    if (row_idx_out) {
        std::vector<uint32_t> rank((size_t)n_tree, 0u);
        std::vector<int32_t> stack{0};
        uint32_t n_ranks = 0;
        while (!stack.empty()) {
            const int32_t id = stack.back();
            stack.pop_back();
            if (tree->feature[id] < 0) {
                rank[(size_t)id] = n_ranks++;
            } else {
                stack.push_back(tree->right[id]);
                stack.push_back(tree->left[id]);
            }
        }
        const size_t per_upload = kUploadBytes / 4;
        for (size_t i0 = 0; i0 < rank.size(); i0 += per_upload) {
            st = upload(ctx, rank.data() + i0, std::min(per_upload, rank.size() - i0) * 4, ws + L.rank_tbl + i0 * 4);
            if (st != GBT_OK) return st;
        }
        uint32_t *key_tmp[2] = {w_rowptr[1], (uint32_t *)w_gq[0] + n};
        uint32_t *val_tmp[2] = {(uint32_t *)w_gq[0], (uint32_t *)w_gq[1]};
        gbt_prof_begin(ctx, GBT_PROF_OTHER, (double)n * 12.0);
        GBT_HIP(ctx, gbt_launch_order_rows(s, leaf_ids, (const uint32_t *)(ws + L.rank_tbl), (uint32_t)n_tree, n_ranks, n,
                                           key_tmp, val_tmp, ws + L.order, row_idx_out));
        gbt_prof_end(ctx);
    }
    GBT_SYNC(ctx);
    return GBT_OK;
}

extern "C" int32_t gbt_grow_tree_sparse(gbt_ctx *ctx, const uint32_t *rowptr, const void *ent, int64_t n,
                                        int64_t nnz, int32_t F, const int32_t *nb, const float *cuts,
                                        const float *gpair, const gbt_params *params, gbt_tree *tree,
                                        uint32_t *row_idx_out, int32_t *leaf_of_row_out, void *workspace,
                                        size_t workspace_bytes) {
    return sparse_grow_impl(ctx, rowptr, ent, n, nnz, F, nb, cuts, gpair, params, GBT_POLICY_DEPTHWISE, 0, tree, row_idx_out,
                            leaf_of_row_out, workspace, workspace_bytes);
}

extern "C" size_t gbt_grow_tree_sparse_lossguide_workspace_bytes(int64_t n, int64_t nnz, int32_t F, int32_t max_bins,
                                                                 int32_t max_leaves) {
    if (n < 0 || nnz < 0 || F < 1 || max_bins < 2 || (int64_t)F * max_bins > kSparseMaxIds || max_leaves < 1 || max_leaves > kMaxLeaves)
        return 0;
    return sparse_grow_layout_nodes(n, nnz, F, max_bins, lossguide_phys_nodes(max_leaves), kLossguideBatchMax).total;
}

extern "C" int32_t gbt_grow_tree_sparse_lossguide(gbt_ctx *ctx, const uint32_t *rowptr, const void *ent, int64_t n,
                                                  int64_t nnz, int32_t F, const int32_t *nb, const float *cuts,
                                                  const float *gpair, const gbt_params *params, int32_t max_leaves,
                                                  gbt_tree *tree, uint32_t *row_idx_out, int32_t *leaf_of_row_out,
                                                  void *workspace, size_t workspace_bytes) {
    return sparse_grow_impl(ctx, rowptr, ent, n, nnz, F, nb, cuts, gpair, params, GBT_POLICY_LOSSGUIDE, max_leaves, tree,
                            row_idx_out, leaf_of_row_out, workspace, workspace_bytes);
}

extern "C" int32_t gbt_predict_sparse(gbt_ctx *ctx, const gbt_tree *trees, int32_t n_trees, const uint32_t *rowptr,
                                      const void *ent, int64_t n, int32_t F, int32_t max_bins, double eta,
                                      float *margin, void *workspace, size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, rowptr && ent && margin, GBT_EINVAL, "NULL argument");
    int32_t st = check_sparse_shape(ctx, n, F, max_bins);
    if (st != GBT_OK) return st;
    const SparseRowsArg sr{rowptr, ent, sparse_ent_bytes(F, max_bins), max_bins};
    st = predict_impl(ctx, trees, n_trees, nullptr, 1, 0, nullptr, n, F, eta, margin, nullptr, workspace, workspace_bytes,
                      &sr, true);
    if (st != GBT_OK) return st;
    GBT_SYNC(ctx);
    return GBT_OK;
}

// ---------------------------------------------------------------- quantise --
extern "C" size_t gbt_quantise_workspace_bytes(int64_t n, int32_t F, int64_t n_values, int32_t max_bins) {
    if (n < 0 || F < 1 || n_values < 0 || max_bins < 2) return 0;
    return gbt_quantise_ws(n, F, n_values, max_bins);
}

namespace {
int32_t quantise_impl(gbt_ctx *ctx, const char *who, const float *X, const int64_t *indptr, const int32_t *indices,
                      const float *values, int64_t n, int32_t F, int32_t max_bins, float *cuts_out, int32_t *nb_out,
                      uint16_t *sym_out, uint32_t *packed_out, int64_t packed_capacity_words, int32_t *bits_out,
                      int32_t *max_value_out, int32_t *missing_sym_out, void *workspace, size_t workspace_bytes) {
    const bool dense = X != nullptr;
    GBT_REQUIRE(ctx, dense != (indptr != nullptr), GBT_EINVAL, "%s: give exactly one of X and (indptr, indices, values)", who);
    GBT_REQUIRE(ctx, cuts_out && nb_out && (sym_out || (packed_out && bits_out)) && max_value_out && missing_sym_out &&
                         workspace, GBT_EINVAL, "%s: NULL argument", who);
    GBT_REQUIRE(ctx, n >= 0 && n < ((int64_t)1 << 32) && F >= 1 && F <= (1 << 20), GBT_EINVAL, "%s: bad shape", who);
    GBT_REQUIRE(ctx, max_bins >= 2 && max_bins <= 4096, GBT_EINVAL, "%s: max_bins = %d outside 2..4096", who, max_bins);
    GBT_REQUIRE(ctx, packed_capacity_words >= 0, GBT_EINVAL, "%s: negative capacity", who);
    int64_t n_values = n * (int64_t)F;
    if (!dense) {
        // the number of stored values is the last row pointer
        GBT_HIP(ctx, hipMemcpyAsync(rb(ctx), indptr + n, 8, hipMemcpyDeviceToHost, ctx->stream));
        GBT_SYNC(ctx);
        memcpy(&n_values, rb(ctx), 8);
        GBT_REQUIRE(ctx, n_values >= 0 && n_values <= n * (int64_t)F, GBT_EINVAL, "%s: indptr[n] = %lld out of range", who,
                    (long long)n_values);
        // (a matrix with nothing stored has nothing to point at: every value is missing)
        GBT_REQUIRE(ctx, n_values == 0 || (indices && values), GBT_EINVAL, "%s: CSR input needs indices and values", who);
    }
    GBT_REQUIRE(ctx, workspace_bytes >= gbt_quantise_ws(n, F, n_values, max_bins), GBT_ENOMEM,
                "%s: workspace %zu < %zu bytes", who, workspace_bytes, gbt_quantise_ws(n, F, n_values, max_bins));
    int32_t status = GBT_OK;
    hipError_t e = gbt_quantise_run(ctx, X, indptr, indices, values, n, F, n_values, max_bins, cuts_out, nb_out,
                                    sym_out, max_value_out, missing_sym_out, (char *)workspace, workspace_bytes,
                                    &status, packed_out, packed_capacity_words, bits_out);
    if (e != hipSuccess) return gbt_fail(ctx, GBT_EHIP, "%s: %s", who, hipGetErrorString(e));
    return status;
}
}  // namespace

extern "C" int32_t gbt_quantise(gbt_ctx *ctx, const float *X, const int64_t *indptr, const int32_t *indices,
                                const float *values, int64_t n, int32_t F, int32_t max_bins, float *cuts_out,
                                int32_t *nb_out, uint16_t *sym_out, int32_t *max_value_out,
                                int32_t *missing_sym_out, void *workspace, size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, sym_out, GBT_EINVAL, "gbt_quantise: NULL argument");
    return quantise_impl(ctx, "gbt_quantise", X, indptr, indices, values, n, F, max_bins, cuts_out, nb_out, sym_out,
                         nullptr, 0, nullptr, max_value_out, missing_sym_out, workspace, workspace_bytes);
}

extern "C" int32_t gbt_quantise_packed(gbt_ctx *ctx, const float *X, const int64_t *indptr, const int32_t *indices,
                                       const float *values, int64_t n, int32_t F, int32_t max_bins, float *cuts_out,
                                       int32_t *nb_out, uint32_t *packed_out, int64_t packed_capacity_words,
                                       int32_t *bits_out, int32_t *max_value_out, int32_t *missing_sym_out,
                                       void *workspace, size_t workspace_bytes) {
    if (!ctx) return GBT_EINVAL;
    GBT_REQUIRE(ctx, packed_out && bits_out, GBT_EINVAL, "gbt_quantise_packed: NULL argument");
    return quantise_impl(ctx, "gbt_quantise_packed", X, indptr, indices, values, n, F, max_bins, cuts_out, nb_out,
                         nullptr, packed_out, packed_capacity_words, bits_out, max_value_out, missing_sym_out,
                         workspace, workspace_bytes);
}
