/*
 * CPU oracle for quantised-histogram decision-tree construction.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the GPU library has to compute.  It shares no code with the GPU path
 * and must never be called from it; only the tests, the smoke check and the
 * benchmark's CPU-baseline leg may use it.
 *
 * What each function follows (paper = arXiv 1806.11248):
 *   gbto_cuts, gbto_bin      Sec. 2.1  (feature quantile generation: every
 *                            feature value is replaced by its quantile bin)
 *   gbto_bits, gbto_pack,    Sec. 2.2  (matrix values stored in
 *   gbto_unpack              log2(max_value) bits, packed with bitwise ops)
 *   gbto_gradients           Sec. 2.5, Eq. 1 and Eq. 2 (logistic g and h) and
 *                            the linear-regression objective named there
 *   gbto_hist                Sec. 2.1 / Alg. 1 BuildPartialHistograms: per
 *                            (feature, bin), the sums of g and of h over the
 *                            node's rows
 *   gbto_eval_split          Alg. 1 EvaluateSplit / Sec. 2.3: running sums
 *                            over a feature's bins price every candidate
 *   gbto_partition           Alg. 1 "RepartitionInstances"
 *   gbto_predict_*           Sec. 2.4 (one instance at a time, trees in order)
 *
 * The paper does not print the gain formula, the treatment of missing values,
 * tie-breaks or the bin-boundary convention.  The readings taken here:
 *   - symbol of a value x in feature f  = number of cuts of f that are <= x;
 *     a split (f, b) sends left the rows whose symbol is <= b;
 *   - cuts are data values: exact order statistics v[floor(k*m/B)], k=1..B-1,
 *     of the m present values (or every distinct value when there are <= B);
 *   - gain = GL^2/(HL+lambda) + GR^2/(HR+lambda) - G^2/(H+lambda), where a term
 *     whose denominator is 0 (lambda = 0, no hessian mass) counts 0; a candidate
 *     is valid iff both sides hold at least one row (counted, not inferred from
 *     the sums: with lambda = 0 and min_child_weight = 0 the term of a side
 *     without rows is 0/0, and rounding noise in G - GL must not turn it into
 *     a winner) and HL >= min_child_weight and HR >= min_child_weight;
 *   - the missing rows' mass is tried on the right, then on the left (only if
 *     the node really has missing rows in that feature);
 *   - best = first candidate, in (feature, bin, right-before-left) order,
 *     with a strictly larger gain.
 *
 * No blocking, no sibling subtraction, no fused steps: every function is the
 * definition written out.  The only parallelism is an OpenMP loop over
 * features where the features are independent.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ cuts -- */

static int cmp_float(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

/*
 * Quantile cuts of one feature (Sec. 2.1).
 *   col, n, stride : the feature's values col[i*stride], NaN = missing
 *   B              : maximum number of bins
 *   cuts_out[B-1]  : strictly increasing cuts, padded with +inf
 * Returns nb = number of bins = number of cuts + 1 (1 when no value is present).
 */
int32_t gbto_cuts(const float *col, int64_t n, int64_t stride, int32_t B, float *cuts_out)
{
    for (int32_t k = 0; k < B - 1; ++k) cuts_out[k] = INFINITY;
    float *v = (float *)malloc((size_t)(n > 0 ? n : 1) * sizeof(float));
    int64_t m = 0;
    for (int64_t i = 0; i < n; ++i) {
        float x = col[i * stride];
        if (!isnan(x)) v[m++] = x;
    }
    if (m == 0) { free(v); return 1; }
    qsort(v, (size_t)m, sizeof(float), cmp_float);

    /* number of distinct values, counted up to B+1 */
    int64_t d = 1;
    for (int64_t i = 1; i < m && d <= B; ++i) if (v[i] != v[i - 1]) ++d;

    int32_t nc = 0;
    if (d <= B) {
        /* every distinct value gets a bin of its own: cuts = u[1..d) */
        for (int64_t i = 1; i < m; ++i) if (v[i] != v[i - 1]) cuts_out[nc++] = v[i];
    } else {
        for (int32_t k = 1; k < B; ++k) {
            float c = v[(int64_t)(((__int128)k * m) / B)];
            if (c == v[0]) continue;                  /* bin 0 must not be empty */
            if (nc > 0 && cuts_out[nc - 1] == c) continue;  /* unique */
            cuts_out[nc++] = c;
        }
    }
    free(v);
    return nc + 1;
}

/* Cuts of every feature of a dense row-major matrix X[n][F]; the features are
 * independent, so they are handled by separate threads.
 *   cuts_out[F][B-1], nb_out[F] */
void gbto_cuts_matrix(const float *X, int64_t n, int32_t F, int32_t B, float *cuts_out,
                      int32_t *nb_out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t f = 0; f < F; ++f)
        nb_out[f] = gbto_cuts(X + f, n, F, B, cuts_out + (int64_t)f * (B - 1));
}

/* --------------------------------------------------------------- binning -- */

/*
 * Symbols of a dense row-major matrix X[n][F] (NaN = missing), Sec. 2.1.
 *   cuts[F][B-1], nb[F] : from gbto_cuts
 *   missing_sym         : the symbol written for a missing value
 * sym(r,f) = #{k < nb[f]-1 : cuts[f][k] <= x}.  The cuts are strictly
 * increasing, so that count is the index of the first cut greater than x,
 * found here by bisection.
 */
void gbto_bin(const float *X, int64_t n, int32_t F, const float *cuts, const int32_t *nb,
              int32_t B, int32_t missing_sym, uint16_t *sym_out)
{
#pragma omp parallel for schedule(static)
    for (int32_t f = 0; f < F; ++f) {
        const float *c = cuts + (int64_t)f * (B - 1);
        int32_t ncut = nb[f] - 1;
        for (int64_t r = 0; r < n; ++r) {
            float x = X[r * F + f];
            int32_t s;
            if (isnan(x)) {
                s = missing_sym;
            } else {
                int32_t lo = 0, hi = ncut; /* invariant: c[k] <= x for k < lo, c[k] > x for k >= hi */
                while (lo < hi) {
                    int32_t mid = (lo + hi) / 2;
                    if (c[mid] <= x) lo = mid + 1; else hi = mid;
                }
                s = lo;
            }
            sym_out[r * F + f] = (uint16_t)s;
        }
    }
}

/* --------------------------------------------------------------- packing -- */

/* Bits per element for a largest symbol max_value (Sec. 2.2): the smallest
 * width that can hold max_value, at least 1. */
int32_t gbto_bits(uint32_t max_value)
{
    int32_t bits = 1;
    while (bits < 32 && (max_value >> bits) != 0) ++bits;
    return bits;
}

/* Number of 32-bit words of the packed stream, including one zero pad word. */
int64_t gbto_packed_words(int64_t n_elems, int32_t bits)
{
    return (n_elems * bits + 31) / 32 + 1;
}

/*
 * Element e occupies bits [e*bits, (e+1)*bits) of a little-endian bit stream
 * held in little-endian 32-bit words; unused bits are zero.  Written bit by bit.
 */
void gbto_pack(const uint16_t *sym, int64_t n_elems, int32_t bits, uint32_t *words_out)
{
    int64_t nw = gbto_packed_words(n_elems, bits);
    memset(words_out, 0, (size_t)nw * sizeof(uint32_t));
    for (int64_t e = 0; e < n_elems; ++e)
        for (int32_t j = 0; j < bits; ++j)
            if ((sym[e] >> j) & 1u) {
                int64_t p = e * bits + j;
                words_out[p >> 5] |= (uint32_t)1 << (p & 31);
            }
}

void gbto_unpack(const uint32_t *words, int64_t n_elems, int32_t bits, uint16_t *sym_out)
{
    for (int64_t e = 0; e < n_elems; ++e) {
        uint32_t s = 0;
        for (int32_t j = 0; j < bits; ++j) {
            int64_t p = e * bits + j;
            s |= ((words[p >> 5] >> (p & 31)) & 1u) << j;
        }
        sym_out[e] = (uint16_t)s;
    }
}

/* ------------------------------------------------------------- gradients -- */

/*
 * objective 0: squared error   g = margin - label,        h = 1
 * objective 1: logistic        g = sigmoid(margin) - y    (Eq. 1)
 *                              h = sigmoid(margin) * (1 - sigmoid(margin))  (Eq. 2)
 * Evaluated in fp64 and rounded once to the fp32 pair the tree builder reads.
 */
void gbto_gradients(int32_t objective, const float *margin, const float *label, int64_t n,
                    float *gpair_out)
{
    for (int64_t i = 0; i < n; ++i) {
        double m = margin[i], y = label[i], g, h;
        if (objective == 1) {
            double p = 1.0 / (1.0 + exp(-m));
            g = p - y;
            h = p * (1.0 - p);
        } else {
            g = m - y;
            h = 1.0;
        }
        gpair_out[2 * i] = (float)g;
        gpair_out[2 * i + 1] = (float)h;
    }
}

/* ------------------------------------------------------------- histogram -- */

/*
 * hist[f][b] = (sum g_r, sum h_r) over the node's rows r with sym(r,f) = b,
 * cnt[f][b] = how many such rows; the missing symbol is not a bin and is not
 * accumulated (B is the stride of the bin axis, every other symbol is < B).  GH_out = (sum g_r, sum h_r) over all the node's rows.
 *   rows == NULL : the node holds rows 0..n_rows-1.
 */
void gbto_hist(const uint16_t *sym, int32_t F, int32_t B, int32_t missing_sym, const uint32_t *rows,
               int64_t n_rows, const float *gpair, double *hist_out, int64_t *cnt_out, double *GH_out)
{
#pragma omp parallel for schedule(static)
    for (int32_t f = 0; f < F; ++f) {
        double *hf = hist_out + (int64_t)f * B * 2;
        int64_t *cf = cnt_out + (int64_t)f * B;
        for (int32_t b = 0; b < B; ++b) { hf[2 * b] = 0.0; hf[2 * b + 1] = 0.0; cf[b] = 0; }
        for (int64_t i = 0; i < n_rows; ++i) {
            int64_t r = rows ? (int64_t)rows[i] : i;
            uint32_t s = sym[r * F + f];
            if (s != (uint32_t)missing_sym && s < (uint32_t)B) {
                hf[2 * s] += (double)gpair[2 * r];
                hf[2 * s + 1] += (double)gpair[2 * r + 1];
                cf[s] += 1;
            }
        }
    }
    double G = 0.0, H = 0.0;
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t r = rows ? (int64_t)rows[i] : i;
        G += (double)gpair[2 * r];
        H += (double)gpair[2 * r + 1];
    }
    GH_out[0] = G;
    GH_out[1] = H;
}

/* ----------------------------------------------------------------- split -- */

typedef struct {
    int32_t feature;      /* -1 when no valid candidate exists */
    int32_t bin;          /* rows with symbol <= bin go left */
    int32_t default_left; /* 1: missing rows go left */
    int32_t valid;
    double gain, GL, HL, GR, HR;
} gbto_split;

/* What the best step w = -G/(H+lambda) of a set of rows gains (twice over): G^2/(H+lambda).  Without
 * curvature, H + lambda = 0, there is no best step: the weight is defined as 0 and so, to match, is this. */
static double term(double G, double H, double lambda)
{
    double d = H + lambda;
    return d > 0.0 ? G * G / d : 0.0;
}

static double split_gain(double GL, double HL, double GR, double HR, double G, double H,
                         double lambda)
{
    double a = term(GL, HL, lambda);
    double b = term(GR, HR, lambda);
    double c = term(G, H, lambda);
    return (a + b) - c;
}

/*
 * Gain of one named candidate (feature f, bin b, direction) from a node's
 * histogram and bin counts; NaN when the candidate is not valid.  The rule is
 * the one of the exhaustive search below: both sides hold at least one row and
 * both have H >= min_child_weight.  Used to price a split that somebody else
 * chose.
 */
double gbto_candidate_gain(const double *hist, const int64_t *cnt, int32_t B, int64_t n_rows, int32_t f,
                           int32_t b, int32_t default_left, double G, double H, double lambda,
                           double min_child_weight, double *sides_out /* GL HL GR HR, may be NULL */)
{
    const double *hf = hist + (int64_t)f * B * 2;
    const int64_t *cf = cnt + (int64_t)f * B;
    double sg = 0.0, sh = 0.0;
    int64_t present = 0;
    for (int32_t k = 0; k < B; ++k) { sg += hf[2 * k]; sh += hf[2 * k + 1]; present += cf[k]; }
    double Gm = G - sg, Hm = H - sh;
    double GL = 0.0, HL = 0.0;
    int64_t n_left = 0;
    for (int32_t k = 0; k <= b; ++k) { GL += hf[2 * k]; HL += hf[2 * k + 1]; n_left += cf[k]; }
    if (default_left) { GL += Gm; HL += Hm; n_left += n_rows - present; }
    double GR = G - GL, HR = H - HL;
    if (sides_out) { sides_out[0] = GL; sides_out[1] = HL; sides_out[2] = GR; sides_out[3] = HR; }
    if (n_left == 0 || n_left == n_rows) return NAN; /* a side without rows is no split */
    if (!(HL >= min_child_weight) || !(HR >= min_child_weight)) return NAN;
    return split_gain(GL, HL, GR, HR, G, H, lambda);
}

/*
 * Exhaustive search over every (feature, bin, direction).
 *   hist[F][B][2], cnt[F][B] : from gbto_hist;  nb[F] : bins per feature
 *   G, H, n_rows             : node totals
 * Order of candidates: feature ascending, bin ascending, missing-right before
 * missing-left; a later candidate wins only with a strictly larger gain.
 */
void gbto_eval_split(const double *hist, const int64_t *cnt, const int32_t *nb, int32_t F, int32_t B,
                     double G, double H, int64_t n_rows, double lambda, double min_child_weight,
                     gbto_split *out)
{
    gbto_split best;
    memset(&best, 0, sizeof best);
    best.feature = -1;
    best.gain = -INFINITY;
    for (int32_t f = 0; f < F; ++f) {
        const double *hf = hist + (int64_t)f * B * 2;
        const int64_t *cf = cnt + (int64_t)f * B;
        double sg = 0.0, sh = 0.0;
        int64_t present = 0;
        for (int32_t k = 0; k < nb[f]; ++k) { sg += hf[2 * k]; sh += hf[2 * k + 1]; present += cf[k]; }
        int has_missing = present < n_rows;
        double Gm = G - sg, Hm = H - sh;
        double pg = 0.0, ph = 0.0;
        int64_t pc = 0;
        for (int32_t b = 0; b < nb[f]; ++b) {
            pg += hf[2 * b];
            ph += hf[2 * b + 1];
            pc += cf[b];
            for (int32_t dir = 0; dir <= has_missing; ++dir) {
                int64_t n_left = pc + (dir == 1 ? n_rows - present : 0);
                if (n_left == 0 || n_left == n_rows) continue; /* a side without rows is no split */
                double GL = pg, HL = ph;
                if (dir == 1) { GL += Gm; HL += Hm; }
                double GR = G - GL, HR = H - HL;
                if (!(HL >= min_child_weight) || !(HR >= min_child_weight)) continue;
                double gain = split_gain(GL, HL, GR, HR, G, H, lambda);
                if (gain > best.gain) {
                    best.feature = f; best.bin = b; best.default_left = dir; best.valid = 1;
                    best.gain = gain; best.GL = GL; best.HL = HL; best.GR = GR; best.HR = HR;
                }
            }
        }
    }
    *out = best;
}

/* ------------------------------------------------------------- partition -- */

/*
 * Stable partition of a node's row list: left = rows with sym(r,f) <= bin, or
 * missing with default_left; right = the rest; both keep their order.
 * rows_out receives [left..., right...]; returns the size of the left part.
 */
int64_t gbto_partition(const uint16_t *sym, int32_t F, const uint32_t *rows, int64_t n_rows,
                       int32_t f, int32_t bin, int32_t default_left, int32_t missing_sym,
                       uint32_t *rows_out)
{
    int64_t nl = 0;
    for (int64_t i = 0; i < n_rows; ++i) {
        int32_t s = sym[(int64_t)rows[i] * F + f];
        int left = (s == missing_sym) ? default_left : (s <= bin);
        if (left) rows_out[nl++] = rows[i];
    }
    int64_t k = nl;
    for (int64_t i = 0; i < n_rows; ++i) {
        int32_t s = sym[(int64_t)rows[i] * F + f];
        int left = (s == missing_sym) ? default_left : (s <= bin);
        if (!left) rows_out[k++] = rows[i];
    }
    return nl;
}

/* --------------------------------------------------------------- predict -- */

/*
 * One tree stored as arrays indexed by node id: feature (-1 = leaf), bin,
 * threshold (= cuts[feature][bin], +inf when bin is the feature's last bin),
 * default_left, left, right, weight.  margin[r] += eta * weight[leaf(r)].
 * Sec. 2.4: one instance at a time, walking the tree from the root.
 */
void gbto_predict_sym(const int32_t *feature, const int32_t *bin, const int32_t *default_left,
                      const int32_t *left, const int32_t *right, const double *weight,
                      const uint16_t *sym, int64_t n, int32_t F, int32_t missing_sym, double eta,
                      float *margin_inout, int32_t *leaf_out /* may be NULL */)
{
    for (int64_t r = 0; r < n; ++r) {
        int32_t node = 0;
        while (feature[node] >= 0) {
            int32_t s = sym[r * F + feature[node]];
            int go_left = (s == missing_sym) ? default_left[node] : (s <= bin[node]);
            node = go_left ? left[node] : right[node];
        }
        if (leaf_out) leaf_out[r] = node;
        margin_inout[r] = (float)((double)margin_inout[r] + eta * weight[node]);
    }
}

void gbto_predict_raw(const int32_t *feature, const float *threshold, const int32_t *default_left,
                      const int32_t *left, const int32_t *right, const double *weight,
                      const float *X, int64_t n, int32_t F, double eta, float *margin_inout,
                      int32_t *leaf_out /* may be NULL */)
{
    for (int64_t r = 0; r < n; ++r) {
        int32_t node = 0;
        while (feature[node] >= 0) {
            float x = X[r * F + feature[node]];
            int go_left = isnan(x) ? default_left[node] : (x < threshold[node]);
            node = go_left ? left[node] : right[node];
        }
        if (leaf_out) leaf_out[r] = node;
        margin_inout[r] = (float)((double)margin_inout[r] + eta * weight[node]);
    }
}
