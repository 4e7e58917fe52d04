/*
 * krul_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, fp64 CPU statement of what the cross-layer attention-similarity
 * estimator and the layer-pair selector of Krul (arxiv 2507.08045) compute.  It
 * exists so that tests, the smoke check and the benchmark's cpu_baseline leg have
 * something independent to compare the GPU library with.  Nothing in the product
 * path may include, link or call this file, and this file shares no code, header
 * or table with the GPU library.
 *
 * What is computed, and from which passage:
 *   - attention weights  softmax(Q K^T / sqrt(d_K))            (Sec. 2.1, the
 *     attention equation), one full Tq x S matrix per (layer, head), stored;
 *   - per query row, the similarity of the two rows that two adjacent layers
 *     give the same token: cosine (the measure named in the caption of the
 *     layer-similarity figure, Fig. 3) and the Euclidean distance (Alg. 1,
 *     "Euclidean_Distance", and Sec. 4.2), the latter as a plain difference,
 *     never through the a^2+b^2-2ab expansion of Sec. 7;
 *   - token-wise aggregation (Sec. 5; Sec. 7 "adds up"): mean over query rows,
 *     then the average over heads (Sec. 4.2 "average distance");
 *   - the greedy disjoint pair choice of Alg. 1 (sort by similarity, skip a pair
 *     if either layer is already shared, stop at the budget) (Sec. 4.2);
 *   - the input-insensitive ("I-R") layer test of Sec. 4.2 / Alg. 1, first loop:
 *     mean attention mass on the first and last tenth of the history;
 *   - the same similarities and the same greedy choice over EVERY two layers
 *     i > j, as Alg. 1 is printed (krul_oracle_all_pairs,
 *     krul_oracle_select_pairs_all).
 *
 * Readings taken where the paper leaves a choice (adjacent pairs only, row-wise
 * similarity then mean, grouped-query head mapping h -> h / (Hq/Hkv), no mask
 * between query tokens unless the causal reading is asked for, stable tie-break on
 * the lower layer index) are listed in
 * the design notes of the repository; each is marked below where it is applied.
 *
 * Every function here is pinned by tests that do not re-use this code: closed
 * forms (uniform keys, S = 1, S = 2, one-hot limit), invariants (identical
 * layers, shift, permutation, pair symmetry, GQA == repeated MHA), library
 * routines (scipy softmax / cdist) on small inputs, the Gaussian large-S limit,
 * and exhaustive simulation of Alg. 1 for the selector.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };

typedef struct {
    int32_t batch, n_layers, n_q_heads, n_kv_heads, head_dim, n_hist, n_query;
    int32_t dtype;   /* ORACLE_F32, ORACLE_BF16 or ORACLE_F16 (raw 16-bit patterns: bfloat16, IEEE binary16) */
    double scale;    /* <= 0 means 1/sqrt(head_dim)  (Sec. 2.1) */
    int32_t causal;  /* 0: every query row sees all n_hist keys.  1: the n_query rows are the last
                        n_query tokens of the n_hist-token sequence and row t sees the keys up to
                        and including its own position, j <= n_hist - n_query + t (decode, Sec. 5:
                        a generated token attends to all previous tokens; chunked prefill) */
} oracle_shape_t;

/* Exact widening of one stored element to double. */
static double elem(const void *p, int dtype, size_t i)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)p)[i];
    if (dtype == ORACLE_F16) {   /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
        const uint16_t h = ((const uint16_t *)p)[i];
        const int sign = h >> 15, ex = (h >> 10) & 31, frac = h & 1023;
        double v;
        if (ex == 0)
            v = ldexp((double)frac, -24);                 /* zero and subnormals: frac * 2^-24 */
        else if (ex == 31)
            v = frac ? NAN : INFINITY;
        else
            v = ldexp((double)(1024 + frac), ex - 25);    /* (1 + frac/1024) * 2^(ex-15) */
        return sign ? -v : v;
    }
    uint32_t bits = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static double eff_scale(const oracle_shape_t *s)
{
    return s->scale > 0.0 ? s->scale : 1.0 / sqrt((double)s->head_dim);
}

/*
 * Attention weights of layer l, query head h of conversation b: P[t*S + j],
 * t < Tq, j < S.  Sec. 2.1: softmax over the keys of (q . k) / sqrt(d_K).
 * Query head h reads kv head h / (Hq/Hkv) (grouped-query reading).  Without the
 * causal reading every query row sees all S keys; with it row t sees keys
 * j <= S - Tq + t and the weights of the later keys are exactly 0.
 */
static void attention_weights(const oracle_shape_t *s, const void *q, const void *k,
                              int b, int l, int h, double *P)
{
    const int d = s->head_dim, S = s->n_hist, Tq = s->n_query;
    const int g = s->n_q_heads / s->n_kv_heads;
    const int hk = h / g;
    const double sc = eff_scale(s);
    const size_t qbase = ((((size_t)b * s->n_layers + l) * s->n_q_heads + h) * (size_t)Tq) * d;
    const size_t kbase = ((((size_t)b * s->n_layers + l) * s->n_kv_heads + hk) * (size_t)S) * d;
    double *qrow = (double *)malloc(sizeof(double) * (size_t)d);
    for (int t = 0; t < Tq; ++t) {
        double *row = P + (size_t)t * S;
        for (int i = 0; i < d; ++i)
            qrow[i] = elem(q, s->dtype, qbase + (size_t)t * d + i);
        const int vis = s->causal ? S - Tq + t + 1 : S;   /* keys 0 .. vis-1 are visible */
        double mx = -INFINITY;
        for (int j = 0; j < vis; ++j) {
            double acc = 0.0;
            for (int i = 0; i < d; ++i)
                acc += qrow[i] * elem(k, s->dtype, kbase + (size_t)j * d + i);
            row[j] = acc * sc;
            if (row[j] > mx) mx = row[j];
        }
        double z = 0.0;
        for (int j = 0; j < vis; ++j) {
            row[j] = exp(row[j] - mx);
            z += row[j];
        }
        for (int j = 0; j < vis; ++j)
            row[j] /= z;
        for (int j = vis; j < S; ++j)
            row[j] = 0.0;
    }
    free(qrow);
}

/*
 * One (conversation b, pair l -> (l, l+1), query head h) unit: mean over the
 * query rows of the cosine similarity and of the Euclidean distance between
 * the two layers' attention rows.
 */
static void unit_scores(const oracle_shape_t *s, const void *q, const void *k,
                        int b, int l, int h, double *cos_mean, double *dist_mean)
{
    const int S = s->n_hist, Tq = s->n_query;
    double *Pa = (double *)malloc(sizeof(double) * (size_t)Tq * S);
    double *Pb = (double *)malloc(sizeof(double) * (size_t)Tq * S);
    attention_weights(s, q, k, b, l, h, Pa);
    attention_weights(s, q, k, b, l + 1, h, Pb);
    double csum = 0.0, dsum = 0.0;
    for (int t = 0; t < Tq; ++t) {
        const double *a = Pa + (size_t)t * S, *c = Pb + (size_t)t * S;
        double ab = 0.0, aa = 0.0, bb = 0.0, dd = 0.0;
        for (int j = 0; j < S; ++j) {
            ab += a[j] * c[j];
            aa += a[j] * a[j];
            bb += c[j] * c[j];
            const double df = a[j] - c[j];
            dd += df * df;
        }
        csum += ab / (sqrt(aa) * sqrt(bb));
        dsum += sqrt(dd);
    }
    *cos_mean = csum / Tq;
    *dist_mean = dsum / Tq;
    free(Pa);
    free(Pb);
}

static int shape_ok(const oracle_shape_t *s)
{
    return s && s->batch > 0 && s->n_layers >= 2 && s->n_q_heads > 0 && s->n_kv_heads > 0 &&
           s->n_q_heads % s->n_kv_heads == 0 && s->head_dim > 0 && s->n_hist > 0 &&
           s->n_query > 0 && (s->dtype == ORACLE_F32 || s->dtype == ORACLE_BF16 || s->dtype == ORACLE_F16) &&
           (s->causal == 0 || (s->causal == 1 && s->n_hist >= s->n_query));
}

/*
 * Scores of a chosen list of units.  units[3*u + {0,1,2}] = (b, l, h).
 * head_cos[u], head_dist[u] receive the token means.  Returns 0, or -1 on a bad
 * argument.  Units are independent; they are spread over the host threads.
 */
int krul_oracle_units(const oracle_shape_t *s, const void *q, const void *k,
                      int n_units, const int32_t *units, double *head_cos, double *head_dist)
{
    if (!shape_ok(s) || !q || !k || n_units < 0 || (n_units && (!units || !head_cos || !head_dist)))
        return -1;
    for (int u = 0; u < n_units; ++u) {
        const int b = units[3 * u], l = units[3 * u + 1], h = units[3 * u + 2];
        if (b < 0 || b >= s->batch || l < 0 || l >= s->n_layers - 1 || h < 0 || h >= s->n_q_heads)
            return -1;
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < n_units; ++u)
        unit_scores(s, q, k, units[3 * u], units[3 * u + 1], units[3 * u + 2],
                    &head_cos[u], &head_dist[u]);
    return 0;
}

/*
 * All scores.  head_cos / head_dist: [B][L-1][Hq]; pair_cos / pair_dist: [B][L-1]
 * (mean over the Hq query heads; each query head counts once).  Any output may
 * be NULL except that the head arrays are always computed internally.
 */
int krul_oracle_pair_similarity(const oracle_shape_t *s, const void *q, const void *k,
                                double *pair_cos, double *head_cos,
                                double *pair_dist, double *head_dist)
{
    if (!shape_ok(s) || !q || !k)
        return -1;
    const int B = s->batch, NP = s->n_layers - 1, H = s->n_q_heads;
    const int n_units = B * NP * H;
    int32_t *units = (int32_t *)malloc(sizeof(int32_t) * 3 * (size_t)n_units);
    double *hc = (double *)malloc(sizeof(double) * (size_t)n_units);
    double *hd = (double *)malloc(sizeof(double) * (size_t)n_units);
    int u = 0;
    for (int b = 0; b < B; ++b)
        for (int l = 0; l < NP; ++l)
            for (int h = 0; h < H; ++h, ++u) {
                units[3 * u] = b;
                units[3 * u + 1] = l;
                units[3 * u + 2] = h;
            }
    int rc = krul_oracle_units(s, q, k, n_units, units, hc, hd);
    if (rc == 0) {
        for (int bl = 0; bl < B * NP; ++bl) {
            double cs = 0.0, ds = 0.0;
            for (int h = 0; h < H; ++h) {
                cs += hc[(size_t)bl * H + h];
                ds += hd[(size_t)bl * H + h];
            }
            if (pair_cos) pair_cos[bl] = cs / H;
            if (pair_dist) pair_dist[bl] = ds / H;
        }
        if (head_cos) memcpy(head_cos, hc, sizeof(double) * (size_t)n_units);
        if (head_dist) memcpy(head_dist, hd, sizeof(double) * (size_t)n_units);
    }
    free(units);
    free(hc);
    free(hd);
    return rc;
}

/*
 * Alg. 1, second half (Sec. 4.2), for adjacent pairs.  pair_score[b][l] is the
 * similarity of (l, l+1); larger means more alike, so "ascending distance" is
 * descending score.  A pair is a candidate only if both its layers are eligible
 * (eligible == NULL: all are).  Candidates are stably ordered by score (equal
 * scores: lower layer index first) and scanned once; a pair is taken iff neither
 * of its layers has been taken; the scan stops once n_select pairs are held.
 * A pair whose score is NaN has no place in the order and is never a candidate
 * (the paper is silent on non-finite scores).
 * out_pairs[b][n_select] gets the lower layer index of each chosen pair in the
 * order chosen, -1 beyond out_count[b].
 */
int krul_oracle_select_pairs(const double *pair_score, const uint8_t *eligible,
                             int batch, int n_layers, int n_select,
                             int32_t *out_pairs, int32_t *out_count)
{
    if (!pair_score || batch <= 0 || n_layers < 2 || n_select < 0 || !out_count ||
        (n_select > 0 && !out_pairs))
        return -1;
    const int NP = n_layers - 1;
    int *order = (int *)malloc(sizeof(int) * (size_t)NP);
    uint8_t *shared = (uint8_t *)malloc((size_t)n_layers);
    for (int b = 0; b < batch; ++b) {
        const double *sc = pair_score + (size_t)b * NP;
        const uint8_t *el = eligible ? eligible + (size_t)b * n_layers : NULL;
        int n = 0;
        for (int l = 0; l < NP; ++l)
            if ((!el || (el[l] && el[l + 1])) && sc[l] == sc[l])   /* a pair whose score is NaN is no candidate */
                order[n++] = l;
        /* stable insertion sort, descending score */
        for (int i = 1; i < n; ++i) {
            int cur = order[i], j = i - 1;
            while (j >= 0 && sc[order[j]] < sc[cur]) {
                order[j + 1] = order[j];
                --j;
            }
            order[j + 1] = cur;
        }
        memset(shared, 0, (size_t)n_layers);
        int cnt = 0;
        for (int i = 0; i < n && cnt < n_select; ++i) {
            const int l = order[i];
            if (shared[l] || shared[l + 1])
                continue;
            shared[l] = shared[l + 1] = 1;
            out_pairs[(size_t)b * n_select + cnt++] = l;
        }
        out_count[b] = cnt;
        for (int i = cnt; i < n_select; ++i)
            out_pairs[(size_t)b * n_select + i] = -1;
    }
    free(order);
    free(shared);
    return 0;
}

/*
 * Sec. 4.2, "Non-I-R Layer Extraction" / Alg. 1 first loop: for every layer, the
 * attention mass that lands on the first tenth and on the last tenth of the
 * history, averaged over all query heads and query rows.  Initial region: keys
 * [0, floor(0.1*S)); recent region: keys [floor(0.9*S), S).  mass[b][l] is that
 * mean; eligible[b][l] = (mass >= gamma), i.e. a layer whose mass stays below
 * gamma is set aside as not input-insensitive.  Either output may be NULL.
 */
int krul_oracle_ir_mass(const oracle_shape_t *s, const void *q, const void *k,
                        double gamma, double *mass, uint8_t *eligible)
{
    if (!shape_ok(s) || !q || !k || s->causal)   /* the test is stated for whole-sequence attention */
        return -1;
    const int B = s->batch, L = s->n_layers, H = s->n_q_heads, S = s->n_hist, Tq = s->n_query;
    const int n_init = (int)floor(0.1 * (double)S);
    const int recent0 = (int)floor(0.9 * (double)S);
    const int n_units = B * L * H;
    double *unit_mass = (double *)malloc(sizeof(double) * (size_t)n_units);
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < n_units; ++u) {
        const int h = u % H, l = (u / H) % L, b = u / (H * L);
        double *P = (double *)malloc(sizeof(double) * (size_t)Tq * S);
        attention_weights(s, q, k, b, l, h, P);
        double acc = 0.0;
        for (int t = 0; t < Tq; ++t) {
            const double *row = P + (size_t)t * S;
            double m = 0.0;
            for (int j = 0; j < n_init; ++j) m += row[j];
            for (int j = recent0; j < S; ++j) m += row[j];
            acc += m;
        }
        unit_mass[u] = acc / Tq;
        free(P);
    }
    for (int bl = 0; bl < B * L; ++bl) {
        double m = 0.0;
        for (int h = 0; h < H; ++h) m += unit_mass[(size_t)bl * H + h];
        m /= H;
        if (mass) mass[bl] = m;
        if (eligible) eligible[bl] = (uint8_t)(m >= gamma);
    }
    free(unit_mass);
    return 0;
}

/*
 * Alg. 1 as printed scores EVERY two layers i > j, not only neighbours (its second loop runs
 * over all two-layer combinations of the remaining layers, Sec. 4.2; the similarity figure of
 * Sec. 2.3 shows the full layer-by-layer map).  For every conversation b, query head h and layers i != j: the mean over the query rows
 * of the cosine similarity and of the Euclidean distance between the rows that layers i and j
 * give the same token; then the average over heads.
 *   head_cos / head_dist : [B][Hq][L][L]   (may be NULL)
 *   pair_cos / pair_dist : [B][L][L]       (may be NULL)
 * All are symmetric; the diagonal holds cos 1 and distance 0 (a row against itself).
 */
/* One (conversation b, query head h): c_out, d_out [L][L] as described above. */
static void head_all_pairs(const oracle_shape_t *s, const void *q, const void *k, int b, int h,
                           double *c_out, double *d_out)
{
    const int L = s->n_layers, S = s->n_hist, Tq = s->n_query;
    /* the attention weights of all layers for this head, stored: P[l][t][j] */
    double *P = (double *)malloc(sizeof(double) * (size_t)L * Tq * S);
    for (int l = 0; l < L; ++l)
        attention_weights(s, q, k, b, l, h, P + (size_t)l * Tq * S);
    for (int i = 0; i < L; ++i) {
        c_out[(size_t)i * L + i] = 1.0;
        d_out[(size_t)i * L + i] = 0.0;
        for (int j = 0; j < i; ++j) {
            double csum = 0.0, dsum = 0.0;
            for (int t = 0; t < Tq; ++t) {
                const double *a = P + ((size_t)i * Tq + t) * S;
                const double *c = P + ((size_t)j * Tq + t) * S;
                double ab = 0.0, aa = 0.0, bb = 0.0, dd = 0.0;
                for (int x = 0; x < S; ++x) {
                    ab += a[x] * c[x];
                    aa += a[x] * a[x];
                    bb += c[x] * c[x];
                    const double df = a[x] - c[x];
                    dd += df * df;
                }
                csum += ab / (sqrt(aa) * sqrt(bb));
                dsum += sqrt(dd);
            }
            c_out[(size_t)i * L + j] = c_out[(size_t)j * L + i] = csum / Tq;
            d_out[(size_t)i * L + j] = d_out[(size_t)j * L + i] = dsum / Tq;
        }
    }
    free(P);
}

/*
 * The same for a chosen list of heads only: heads[2*u + {0,1}] = (b, h); head_cos / head_dist
 * [n_heads][L][L].  Returns 0, or -1 on a bad argument.
 */
int krul_oracle_all_pairs_heads(const oracle_shape_t *s, const void *q, const void *k, int n_heads,
                                const int32_t *heads, double *head_cos, double *head_dist)
{
    if (!shape_ok(s) || !q || !k || n_heads < 0 || (n_heads && (!heads || !head_cos || !head_dist)))
        return -1;
    for (int u = 0; u < n_heads; ++u)
        if (heads[2 * u] < 0 || heads[2 * u] >= s->batch || heads[2 * u + 1] < 0 || heads[2 * u + 1] >= s->n_q_heads)
            return -1;
    const size_t LL = (size_t)s->n_layers * s->n_layers;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < n_heads; ++u)
        head_all_pairs(s, q, k, heads[2 * u], heads[2 * u + 1], head_cos + (size_t)u * LL, head_dist + (size_t)u * LL);
    return 0;
}

int krul_oracle_all_pairs(const oracle_shape_t *s, const void *q, const void *k,
                          double *pair_cos, double *pair_dist, double *head_cos, double *head_dist)
{
    if (!shape_ok(s) || !q || !k)
        return -1;
    const int B = s->batch, L = s->n_layers, H = s->n_q_heads;
    const size_t LL = (size_t)L * L;
    double *hc = (double *)malloc(sizeof(double) * (size_t)B * H * LL);
    double *hd = (double *)malloc(sizeof(double) * (size_t)B * H * LL);
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh)
        head_all_pairs(s, q, k, bh / H, bh % H, hc + (size_t)bh * LL, hd + (size_t)bh * LL);
    for (int b = 0; b < B; ++b)
        for (size_t e = 0; e < LL; ++e) {
            double cs = 0.0, ds = 0.0;
            for (int h = 0; h < H; ++h) {
                cs += hc[((size_t)b * H + h) * LL + e];
                ds += hd[((size_t)b * H + h) * LL + e];
            }
            if (pair_cos) pair_cos[(size_t)b * LL + e] = cs / H;
            if (pair_dist) pair_dist[(size_t)b * LL + e] = ds / H;
        }
    if (head_cos) memcpy(head_cos, hc, sizeof(double) * (size_t)B * H * LL);
    if (head_dist) memcpy(head_dist, hd, sizeof(double) * (size_t)B * H * LL);
    free(hc);
    free(hd);
    return 0;
}

/*
 * Alg. 1, second half (Sec. 4.2), over every two layers i > j.  score[b][i][j] (the lower
 * triangle of an [L][L] matrix is read) measures the two layers: a distance (closer_is_smaller
 * != 0: Alg. 1's "Euclidean_Distance", taken in ascending order) or a similarity
 * (closer_is_smaller == 0: taken in descending order).  A pair is a candidate only if both its
 * layers are eligible (eligible == NULL: all are).  Candidates are listed with j ascending,
 * then i ascending, stably ordered by score and scanned once; a pair is taken iff neither of its
 * layers has been taken; the scan stops once n_select pairs are held.
 * out_pairs[b][n][2] = (j, i) with j < i, in the order chosen; (-1, -1) beyond out_count[b].
 */
int krul_oracle_select_pairs_all(const double *score, int closer_is_smaller, const uint8_t *eligible,
                                 int batch, int n_layers, int n_select,
                                 int32_t *out_pairs, int32_t *out_count)
{
    if (!score || batch <= 0 || n_layers < 2 || n_select < 0 || !out_count ||
        (n_select > 0 && !out_pairs))
        return -1;
    const int L = n_layers;
    const int NC = L * (L - 1) / 2;
    int *cj = (int *)malloc(sizeof(int) * (size_t)NC), *ci = (int *)malloc(sizeof(int) * (size_t)NC);
    double *key = (double *)malloc(sizeof(double) * (size_t)NC);
    uint8_t *shared = (uint8_t *)malloc((size_t)L);
    for (int b = 0; b < batch; ++b) {
        const double *sc = score + (size_t)b * L * L;
        const uint8_t *el = eligible ? eligible + (size_t)b * L : NULL;
        int n = 0;
        for (int j = 0; j < L; ++j)
            for (int i = j + 1; i < L; ++i)
                if ((!el || (el[i] && el[j])) && sc[(size_t)i * L + j] == sc[(size_t)i * L + j]) {   /* (NaN: no candidate) */
                    cj[n] = j;
                    ci[n] = i;
                    /* one ordering for both readings: ascending key */
                    key[n] = closer_is_smaller ? sc[(size_t)i * L + j] : -sc[(size_t)i * L + j];
                    ++n;
                }
        /* stable insertion sort, ascending key */
        for (int a = 1; a < n; ++a) {
            const int tj = cj[a], ti = ci[a];
            const double tk = key[a];
            int p = a - 1;
            while (p >= 0 && key[p] > tk) {
                cj[p + 1] = cj[p];
                ci[p + 1] = ci[p];
                key[p + 1] = key[p];
                --p;
            }
            cj[p + 1] = tj;
            ci[p + 1] = ti;
            key[p + 1] = tk;
        }
        memset(shared, 0, (size_t)L);
        int cnt = 0;
        for (int a = 0; a < n && cnt < n_select; ++a) {
            if (shared[ci[a]] || shared[cj[a]])
                continue;
            shared[ci[a]] = shared[cj[a]] = 1;
            out_pairs[((size_t)b * n_select + cnt) * 2] = cj[a];
            out_pairs[((size_t)b * n_select + cnt) * 2 + 1] = ci[a];
            ++cnt;
        }
        out_count[b] = cnt;
        for (int a = cnt; a < n_select; ++a)
            out_pairs[((size_t)b * n_select + a) * 2] = out_pairs[((size_t)b * n_select + a) * 2 + 1] = -1;
    }
    free(cj);
    free(ci);
    free(key);
    free(shared);
    return 0;
}

int krul_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
