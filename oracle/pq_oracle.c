/*
 * pq_oracle.c -- reference CPU implementation of product-quantization ADC search.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the GPU path, and the GPU path never calls it.  Only the test-suite, the
 * smoke check and the benchmark's CPU-baseline leg may load it.
 *
 * Everything is written straight from the thesis (F. Andre, "Exploiting Modern
 * Hardware for High-Dimensional Nearest Neighbor Search"):
 *   - vector / product quantizer and encoder : Section 2.3.1 "Vector Encoding"
 *   - inverted index with residuals (IVFADC)  : Section 2.3.2 "Inverted Indexes"
 *   - lookup tables                           : Section 2.3.3, Eq. (tables)
 *   - ADC distance                            : Section 2.3.3, Eq. (adc1); Alg. 1 (adc)
 *   - scan with a binary heap of size r       : Alg. 1 (scan) and the heap paragraph
 *   - 4-bit sub-codes, two per byte           : Section 5.2.2, Alg. 3 (Quick ADC)
 *   - 8-bit table quantisation                : Section 4.2.4 "Quantization of Distances",
 *                                               Section 5.2.1, Section 6.2.3 Step 1.2
 *   - two-pass search (candidates + rerank)   : Section 6.2.3, Alg. 5
 *   - rotation of optimized product quantization : Section 2.3.4 (OPQ paragraph)
 *
 * Arithmetic: floating-point sums are accumulated in double and rounded once to
 * float, except the table quantiser, whose float operation sequence is fixed
 * below so that integer results are reproducible bit for bit.  Compile without
 * -ffast-math and with -ffp-contract=off.
 *
 * Parity status: every function here is pinned by tests that do not call it to
 * produce their expected values (worked example of Fig. "ADC", brute force,
 * Eq. (adc2) invariant, full sort, closed forms).  Recall against true
 * neighbours of the thesis's datasets: parity unpinned (datasets unavailable).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_CODES_U8 0        /* one byte per sub-quantizer index                      */
#define ORC_CODES_U4_PACKED 1 /* byte r holds index 2r in bits 0-3, index 2r+1 in 4-7 */

static int code_bytes(int m, int fmt) { return fmt == ORC_CODES_U4_PACKED ? m / 2 : m; }

/* j-th sub-quantizer index of a stored code.  Alg. 3 masks with 0x0f for the
 * even component and shifts right by 4 for the odd one (unsigned byte). */
static int code_index(const uint8_t *code, int j, int fmt)
{
    if (fmt == ORC_CODES_U4_PACKED) {
        uint8_t byte = code[j / 2];
        return (j % 2 == 0) ? (byte & 0x0f) : (byte >> 4);
    }
    return code[j];
}

/* ------------------------------------------------------------------------- */
/* squared Euclidean distance between two float vectors, in double           */
static double sqdist(const float *a, const float *b, int len)
{
    double s = 0.0;
    for (int t = 0; t < len; t++) {
        double diff = (double)a[t] - (double)b[t];
        s += diff * diff;
    }
    return s;
}

/* ------------------------------------------------------------------------- */
/* Lloyd k-means on n points of dimension dsub (row stride `stride` floats).
 * Section 2.3.1: a quantizer maps x to its closest centroid (Lloyd condition);
 * centroids are the means of their cells.  Initial centroids are the points
 * init_idx[0..k-1] (chosen by the caller's seeded generator).  A cell that
 * becomes empty is re-seeded with the point currently farthest from its own
 * centroid (the thesis is silent on this).  Ties in assignment go to the
 * smallest centroid index. */
int orc_kmeans(const float *x, int64_t n, int dsub, int64_t stride, int k, int iters,
               const int64_t *init_idx, float *centroids /* [k][dsub] */)
{
    if (n <= 0 || k <= 0 || dsub <= 0) return -1;
    for (int i = 0; i < k; i++)
        memcpy(centroids + (size_t)i * dsub, x + init_idx[i] * stride, sizeof(float) * dsub);
    int32_t *assign = (int32_t *)malloc(sizeof(int32_t) * n);
    double *dist = (double *)malloc(sizeof(double) * n);
    double *sum = (double *)malloc(sizeof(double) * (size_t)k * dsub);
    int64_t *count = (int64_t *)malloc(sizeof(int64_t) * k);
    if (!assign || !dist || !sum || !count) return -2;
    for (int it = 0; it < iters; it++) {
        for (int64_t p = 0; p < n; p++) {
            int best = 0;
            double bestd = sqdist(x + p * stride, centroids, dsub);
            for (int i = 1; i < k; i++) {
                double dd = sqdist(x + p * stride, centroids + (size_t)i * dsub, dsub);
                if (dd < bestd) { bestd = dd; best = i; }
            }
            assign[p] = best;
            dist[p] = bestd;
        }
        memset(sum, 0, sizeof(double) * (size_t)k * dsub);
        memset(count, 0, sizeof(int64_t) * k);
        for (int64_t p = 0; p < n; p++) {
            count[assign[p]]++;
            for (int t = 0; t < dsub; t++) sum[(size_t)assign[p] * dsub + t] += (double)x[p * stride + t];
        }
        for (int i = 0; i < k; i++) {
            if (count[i] > 0) {
                for (int t = 0; t < dsub; t++)
                    centroids[(size_t)i * dsub + t] = (float)(sum[(size_t)i * dsub + t] / (double)count[i]);
            } else {
                int64_t far = 0;
                for (int64_t p = 1; p < n; p++)
                    if (dist[p] > dist[far]) far = p;
                memcpy(centroids + (size_t)i * dsub, x + far * stride, sizeof(float) * dsub);
                dist[far] = 0.0; /* do not pick the same point for another empty cell */
            }
        }
    }
    free(assign); free(dist); free(sum); free(count);
    return 0;
}

/* Train the m codebooks of a product quantizer: sub-space j covers dimensions
 * j*d/m .. (j+1)*d/m - 1 (Section 2.3.1, "Product Quantizer"). */
int orc_pq_train(const float *x, int64_t n, int d, int m, int k, int iters,
                 const int64_t *init_idx /* [m][k] */, float *codebooks /* [m][k][d/m] */)
{
    if (m <= 0 || d % m != 0) return -1;
    int dsub = d / m;
    for (int j = 0; j < m; j++) {
        int rc = orc_kmeans(x + j * dsub, n, dsub, d, k, iters, init_idx + (size_t)j * k,
                            codebooks + (size_t)j * k * dsub);
        if (rc) return rc;
    }
    return 0;
}

/* enc(x) = (i_0 .. i_{m-1}), i_j = index of the centroid of codebook j closest
 * to sub-vector x^j (Section 2.3.1).  Output: one byte per index, [n][m]. */
int orc_pq_encode(const float *x, int64_t n, int d, int m, int k, const float *codebooks,
                  uint8_t *codes /* [n][m] */)
{
    if (m <= 0 || d % m != 0 || k > 256) return -1;
    int dsub = d / m;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < n; p++) {
        for (int j = 0; j < m; j++) {
            const float *cb = codebooks + (size_t)j * k * dsub;
            int best = 0;
            double bestd = sqdist(x + p * d + j * dsub, cb, dsub);
            for (int i = 1; i < k; i++) {
                double dd = sqdist(x + p * d + j * dsub, cb + (size_t)i * dsub, dsub);
                if (dd < bestd) { bestd = dd; best = i; }
            }
            codes[p * m + j] = (uint8_t)best;
        }
    }
    return 0;
}

/* Pack [n][m] 4-bit indexes (each < 16) two per byte: even component in the
 * low nibble, odd component in the high nibble (Section 5.2.2). */
int orc_pack_u4(const uint8_t *codes, int64_t n, int m, uint8_t *packed /* [n][m/2] */)
{
    if (m % 2 != 0) return -1;
    for (int64_t p = 0; p < n; p++)
        for (int r = 0; r < m / 2; r++) {
            uint8_t lo = codes[p * m + 2 * r], hi = codes[p * m + 2 * r + 1];
            if (lo > 15 || hi > 15) return -2;
            packed[p * (m / 2) + r] = (uint8_t)(lo | (hi << 4));
        }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Rotation of optimized product quantization (Section 2.3.4, paragraph OPQ):
 * opq(x) = pq(R x) with R a d x d orthogonal matrix; this is the product R x,
 * out[p][r] = sum_t R[r][t] * x[p][t], accumulated in double in index order and
 * rounded once.  (R is data: learning it is outside the search path.) */
int orc_rotate(const float *x, int64_t n, int d, const float *R /* [d][d] */, float *out /* [n][d] */)
{
    if (d <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < n; p++)
        for (int r = 0; r < d; r++) {
            double acc = 0.0;
            for (int t = 0; t < d; t++) acc += (double)R[(size_t)r * d + t] * (double)x[p * d + t];
            out[p * d + r] = (float)acc;
        }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Tables step, Eq. (tables): D^j[i] = || y^j - C^j[i] ||^2.                  */
int orc_build_luts(const float *queries, int nq, int d, int m, int k, const float *codebooks,
                   float *luts /* [nq][m][k] */)
{
    if (m <= 0 || d % m != 0) return -1;
    int dsub = d / m;
    for (int q = 0; q < nq; q++)
        for (int j = 0; j < m; j++)
            for (int i = 0; i < k; i++)
                luts[((size_t)q * m + j) * k + i] =
                    (float)sqdist(queries + (size_t)q * d + j * dsub,
                                  codebooks + ((size_t)j * k + i) * dsub, dsub);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* 8-bit quantisation of the tables of each query (Sections 4.2.4, 5.2.1, 6.3
 * Step 1.2).  qmin is the smallest entry over all m tables of the query; the
 * interval [qmin, qmax) is cut into 255 equal bins numbered 0..254 and every
 * value at or above qmax becomes 255 (the unsigned-byte reading; the thesis's
 * SSE variant keeps 127 bins because SSE lacks an unsigned compare).  The
 * float operation sequence is fixed:
 *     range = qmax - qmin                       (float subtract)
 *     scale = range > 0 and finite ? 255.0f / range : 0   (float divide)
 *     t     = (D - qmin) * scale                (float subtract, float multiply)
 *     Q     = t >= 255 ? 255 : (uint8) floorf(t)
 */
int orc_quantize_luts(const float *luts, int nq, int m, int k, const float *qmax,
                      uint8_t *qluts /* [nq][m][k] */, float *qmin_out, float *scale_out)
{
    size_t per = (size_t)m * k;
    for (int q = 0; q < nq; q++) {
        const float *D = luts + q * per;
        float qmin = D[0];
        for (size_t e = 1; e < per; e++)
            if (D[e] < qmin) qmin = D[e];
        volatile float range = qmax[q] - qmin;
        volatile float scale = 0.0f;
        if (range > 0.0f && isfinite(range)) scale = 255.0f / range;
        for (size_t e = 0; e < per; e++) {
            volatile float shifted = D[e] - qmin;
            volatile float t = shifted * scale;
            qluts[q * per + e] = (t >= 255.0f) ? 255 : (uint8_t)floorf(t);
        }
        if (qmin_out) qmin_out[q] = qmin;
        if (scale_out) scale_out[q] = scale;
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* ADC, Eq. (adc1): adc(y, c) = sum_{j=0}^{m-1} D^j[c[j]].                    */
static float adc_f32(const uint8_t *code, int fmt, const float *lut, int m, int k)
{
    double dist = 0.0;
    for (int j = 0; j < m; j++) dist += (double)lut[(size_t)j * k + code_index(code, j, fmt)];
    return (float)dist;
}

/* same with quantised tables; plain integer sum, no saturation */
static uint32_t adc_u8(const uint8_t *code, int fmt, const uint8_t *qlut, int m, int k)
{
    uint32_t s = 0;
    for (int j = 0; j < m; j++) s += qlut[(size_t)j * k + code_index(code, j, fmt)];
    return s;
}

/* all n distances of one query (for tests) */
int orc_adc_all_f32(const uint8_t *codes, int64_t n, int fmt, const float *lut, int m, int k,
                    float *dist /* [n] */)
{
    int cb = code_bytes(m, fmt);
    for (int64_t i = 0; i < n; i++) dist[i] = adc_f32(codes + i * cb, fmt, lut, m, k);
    return 0;
}

int orc_adc_all_u8(const uint8_t *codes, int64_t n, int fmt, const uint8_t *qlut, int m, int k,
                   uint32_t *sum /* [n] */)
{
    int cb = code_bytes(m, fmt);
    for (int64_t i = 0; i < n; i++) sum[i] = adc_u8(codes + i * cb, fmt, qlut, m, k);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Binary max-heap of (value, id) pairs, capacity r (Alg. 1 `binheap(r)` and the
 * paragraph on the heap).  The pair order is (value, then id): the root is the
 * largest pair.  `value` is a double so that one heap serves float distances
 * and integer sums exactly.  A new pair enters a full heap only if it is
 * smaller than the root, which is then removed. */
typedef struct { double v; int64_t id; } pair_t;
typedef struct { pair_t *a; int size, cap; } heap_t;

static int pair_less(pair_t x, pair_t y) { return x.v < y.v || (x.v == y.v && x.id < y.id); }

static void heap_sift_up(heap_t *h, int pos)
{
    while (pos > 0) {
        int parent = (pos - 1) / 2;
        if (!pair_less(h->a[parent], h->a[pos])) break;
        pair_t tmp = h->a[parent]; h->a[parent] = h->a[pos]; h->a[pos] = tmp;
        pos = parent;
    }
}

static void heap_sift_down(heap_t *h, int pos)
{
    for (;;) {
        int l = 2 * pos + 1, r = l + 1, big = pos;
        if (l < h->size && pair_less(h->a[big], h->a[l])) big = l;
        if (r < h->size && pair_less(h->a[big], h->a[r])) big = r;
        if (big == pos) break;
        pair_t tmp = h->a[big]; h->a[big] = h->a[pos]; h->a[pos] = tmp;
        pos = big;
    }
}

static void heap_add(heap_t *h, double v, int64_t id)
{
    pair_t p = { v, id };
    if (h->size < h->cap) {
        h->a[h->size] = p;
        h->size++;
        heap_sift_up(h, h->size - 1);
    } else if (h->cap > 0 && pair_less(p, h->a[0])) {
        h->a[0] = p;
        heap_sift_down(h, 0);
    }
}

/* pop everything: fills out[0..size-1] in ascending pair order, returns size */
static int heap_drain_sorted(heap_t *h, pair_t *out)
{
    int total = h->size;
    for (int pos = total - 1; pos >= 0; pos--) {
        out[pos] = h->a[0];
        h->size--;
        h->a[0] = h->a[h->size];
        heap_sift_down(h, 0);
    }
    return total;
}

/* ------------------------------------------------------------------------- */
/* Scan step with float tables (Alg. 1 `scan`): ids are list positions.  Output
 * per query: the topk smallest (distance, id) pairs in ascending order; if
 * n < topk the tail is (+inf, -1). */
int orc_adc_scan_topk_f32(const uint8_t *codes, int64_t n, int fmt, const float *luts, int nq,
                          int m, int k, int topk, float *out_dist, int64_t *out_ids)
{
    int cb = code_bytes(m, fmt);
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; q++) {
        heap_t h = { (pair_t *)malloc(sizeof(pair_t) * (topk > 0 ? topk : 1)), 0, topk };
        pair_t *sorted = (pair_t *)malloc(sizeof(pair_t) * (topk > 0 ? topk : 1));
        if (!h.a || !sorted) { err = -2; free(h.a); free(sorted); continue; }
        const float *lut = luts + (size_t)q * m * k;
        for (int64_t i = 0; i < n; i++) heap_add(&h, (double)adc_f32(codes + i * cb, fmt, lut, m, k), i);
        int got = heap_drain_sorted(&h, sorted);
        for (int t = 0; t < topk; t++) {
            out_dist[(size_t)q * topk + t] = t < got ? (float)sorted[t].v : INFINITY;
            out_ids[(size_t)q * topk + t] = t < got ? sorted[t].id : -1;
        }
        free(h.a); free(sorted);
    }
    return err;
}

/* Scan step with quantised tables and integer sums (Alg. 3 `quick_adc_scan`
 * without the SIMD block layout, Alg. 5 `scan`/`adc_low_bits`): topk smallest
 * (sum, id) pairs ascending; tail (UINT32_MAX, -1) if n < topk. */
int orc_adc_scan_topk_u8(const uint8_t *codes, int64_t n, int fmt, const uint8_t *qluts, int nq,
                         int m, int k, int topk, uint32_t *out_sum, int64_t *out_ids)
{
    int cb = code_bytes(m, fmt);
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; q++) {
        heap_t h = { (pair_t *)malloc(sizeof(pair_t) * (topk > 0 ? topk : 1)), 0, topk };
        pair_t *sorted = (pair_t *)malloc(sizeof(pair_t) * (topk > 0 ? topk : 1));
        if (!h.a || !sorted) { err = -2; free(h.a); free(sorted); continue; }
        const uint8_t *qlut = qluts + (size_t)q * m * k;
        for (int64_t i = 0; i < n; i++) heap_add(&h, (double)adc_u8(codes + i * cb, fmt, qlut, m, k), i);
        int got = heap_drain_sorted(&h, sorted);
        for (int t = 0; t < topk; t++) {
            out_sum[(size_t)q * topk + t] = t < got ? (uint32_t)sorted[t].v : UINT32_MAX;
            out_ids[(size_t)q * topk + t] = t < got ? sorted[t].id : -1;
        }
        free(h.a); free(sorted);
    }
    return err;
}

/* Second pass of the two-pass search (Alg. 5 `rerank`): float ADC of the given
 * candidates (positions into `codes`; negative entries are skipped), then the
 * topk smallest (distance, id). */
int orc_rerank_f32(const uint8_t *codes, int fmt, const float *luts, int nq, int m, int k,
                   const int64_t *cand_ids /* [nq][ncand] */, int ncand, int topk,
                   float *out_dist, int64_t *out_ids)
{
    int cb = code_bytes(m, fmt);
    for (int q = 0; q < nq; q++) {
        heap_t h = { (pair_t *)malloc(sizeof(pair_t) * (topk > 0 ? topk : 1)), 0, topk };
        pair_t *sorted = (pair_t *)malloc(sizeof(pair_t) * (topk > 0 ? topk : 1));
        if (!h.a || !sorted) return -2;
        const float *lut = luts + (size_t)q * m * k;
        for (int c = 0; c < ncand; c++) {
            int64_t id = cand_ids[(size_t)q * ncand + c];
            if (id < 0) continue;
            heap_add(&h, (double)adc_f32(codes + id * cb, fmt, lut, m, k), id);
        }
        int got = heap_drain_sorted(&h, sorted);
        for (int t = 0; t < topk; t++) {
            out_dist[(size_t)q * topk + t] = t < got ? (float)sorted[t].v : INFINITY;
            out_ids[(size_t)q * topk + t] = t < got ? sorted[t].id : -1;
        }
        free(h.a); free(sorted);
    }
    return 0;
}

/* Upper quantisation bound (Sections 4.2.4 / 5.2.1 / 6.3 Step 1.2): float ADC
 * over the first min(init, n) codes; qmax is the kq-th smallest of those
 * distances (kq clipped to the number scanned).  kq = 1 is the thesis's
 * "temporary nearest neighbour"; kq = init is Step 1.2's "greatest distance". */
int orc_qmax_prescan(const uint8_t *codes, int64_t n, int fmt, const float *luts, int nq, int m,
                     int k, int64_t init, int kq, float *qmax_out)
{
    int cb = code_bytes(m, fmt);
    int64_t cnt = init < n ? init : n;
    if (cnt <= 0 || kq <= 0) return -1;
    if (kq > cnt) kq = (int)cnt;
    for (int q = 0; q < nq; q++) {
        heap_t h = { (pair_t *)malloc(sizeof(pair_t) * kq), 0, kq };
        if (!h.a) return -2;
        const float *lut = luts + (size_t)q * m * k;
        for (int64_t i = 0; i < cnt; i++) heap_add(&h, (double)adc_f32(codes + i * cb, fmt, lut, m, k), i);
        qmax_out[q] = (float)h.a[0].v; /* root = kq-th smallest */
        free(h.a);
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* IVFADC (Section 2.3.2 and the Index step of Section 2.3.3).
 * Index step: distances from the query to the nlist coarse centroids, the
 * nprobe smallest by (distance, list id). */
int orc_ivf_probe(const float *queries, int nq, int d, const float *coarse, int nlist, int nprobe,
                  int32_t *probe_out /* [nq][nprobe] */, float *probe_dist_out /* may be NULL */)
{
    if (nprobe > nlist || nprobe <= 0) return -1;
    for (int q = 0; q < nq; q++) {
        heap_t h = { (pair_t *)malloc(sizeof(pair_t) * nprobe), 0, nprobe };
        pair_t *sorted = (pair_t *)malloc(sizeof(pair_t) * nprobe);
        if (!h.a || !sorted) return -2;
        for (int l = 0; l < nlist; l++)
            heap_add(&h, (double)(float)sqdist(queries + (size_t)q * d, coarse + (size_t)l * d, d), l);
        heap_drain_sorted(&h, sorted);
        for (int p = 0; p < nprobe; p++) {
            probe_out[(size_t)q * nprobe + p] = (int32_t)sorted[p].id;
            if (probe_dist_out) probe_dist_out[(size_t)q * nprobe + p] = (float)sorted[p].v;
        }
        free(h.a); free(sorted);
    }
    return 0;
}

/* Tables + Scan over the probed lists: for each probed list l the query
 * residual y' = y - centroid_l (float), its tables by Eq. (tables), ADC of every
 * code of the list; one heap over all probed lists.  The id of a code is
 * ids[pos] if ids != NULL, else its position pos in the grouped code array.
 * `probes` = lists to scan per query (from orc_ivf_probe or supplied). */
int orc_ivf_scan(const float *queries, int nq, int d, const float *coarse, int nlist,
                 const int64_t *list_offsets /* [nlist+1] */, const uint8_t *codes, const int64_t *ids,
                 const float *codebooks, int m, int k, int fmt, const int32_t *probes, int nprobe,
                 int topk, float *out_dist, int64_t *out_ids)
{
    if (m <= 0 || d % m != 0) return -1;
    int cb = code_bytes(m, fmt);
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; q++) {
        heap_t h = { (pair_t *)malloc(sizeof(pair_t) * (topk > 0 ? topk : 1)), 0, topk };
        pair_t *sorted = (pair_t *)malloc(sizeof(pair_t) * (topk > 0 ? topk : 1));
        float *resid = (float *)malloc(sizeof(float) * d);
        float *lut = (float *)malloc(sizeof(float) * (size_t)m * k);
        if (!h.a || !sorted || !resid || !lut) { err = -2; free(h.a); free(sorted); free(resid); free(lut); continue; }
        for (int p = 0; p < nprobe; p++) {
            int l = probes[(size_t)q * nprobe + p];
            if (l < 0 || l >= nlist) continue;
            for (int t = 0; t < d; t++) resid[t] = queries[(size_t)q * d + t] - coarse[(size_t)l * d + t];
            orc_build_luts(resid, 1, d, m, k, codebooks, lut);
            for (int64_t pos = list_offsets[l]; pos < list_offsets[l + 1]; pos++)
                heap_add(&h, (double)adc_f32(codes + pos * cb, fmt, lut, m, k), ids ? ids[pos] : pos);
        }
        int got = heap_drain_sorted(&h, sorted);
        for (int t = 0; t < topk; t++) {
            out_dist[(size_t)q * topk + t] = t < got ? (float)sorted[t].v : INFINITY;
            out_ids[(size_t)q * topk + t] = t < got ? sorted[t].id : -1;
        }
        free(h.a); free(sorted); free(resid); free(lut);
    }
    return err;
}

/* IVFADC search with Quick ADC in the Scan step (chapter 5: 4-bit sub-quantizers and tables
 * quantised to 8 bits, Section 5.2; Section 5.3 measures it inside the inverted index of
 * Section 2.3.2).  Per query, with the probed lists in probe order:
 *   Tables   float tables of the residual y - centroid_l for every probed list (as orc_ivf_scan);
 *   qmax     float ADC (each code with the tables of its own list) of the first `init` codes met
 *            when the probed lists are walked in probe order; qmax = the topk-th smallest of these
 *            distances (the distance to the temporary topk-th neighbour; rank clipped to the number
 *            of codes met; +inf if the probed lists are empty);
 *   8 bits   the tables of each (query, list) pair quantised by orc_quantize_luts with the pair's
 *            own qmin and the query's qmax;
 *   Scan     plain integer sums of the quantised entries (Alg. 3 without saturation) for every code
 *            of the list; the kprime smallest (sum, position) of each pair are its candidates;
 *   Rerank   float ADC of the candidates with the pair's float tables; the topk smallest
 *            (distance, position) over all pairs of the query; positions mapped through ids.
 * Integer sums of different pairs are not comparable (each pair has its own qmin and scale), which
 * is why candidates are chosen per pair and ranked by float distance. */
int orc_ivf_quick_scan(const float *queries, int nq, int d, const float *coarse, int nlist,
                       const int64_t *list_offsets, const uint8_t *codes, const int64_t *ids,
                       const float *codebooks, int m, int k, int fmt, const int32_t *probes, int nprobe,
                       int64_t init, int kprime, int topk, float *out_dist, int64_t *out_ids)
{
    if (m <= 0 || d % m != 0 || kprime <= 0 || topk <= 0 || init < 0) return -1;
    int cb = code_bytes(m, fmt);
    size_t per = (size_t)m * k;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; q++) {
        float *resid = (float *)malloc(sizeof(float) * d);
        float *luts = (float *)malloc(sizeof(float) * per * nprobe);
        uint8_t *qluts = (uint8_t *)malloc(per * nprobe);
        float *qmax = (float *)malloc(sizeof(float) * nprobe);
        heap_t temp = { (pair_t *)malloc(sizeof(pair_t) * topk), 0, topk };
        heap_t cand = { (pair_t *)malloc(sizeof(pair_t) * kprime), 0, kprime };
        heap_t best = { (pair_t *)malloc(sizeof(pair_t) * topk), 0, topk };
        pair_t *sorted = (pair_t *)malloc(sizeof(pair_t) * (topk > kprime ? topk : kprime));
        if (!resid || !luts || !qluts || !qmax || !temp.a || !cand.a || !best.a || !sorted) {
            err = -2;
        } else {
            const int32_t *pr = probes + (size_t)q * nprobe;
            /* Tables */
            for (int p = 0; p < nprobe; p++) {
                int l = pr[p];
                if (l < 0 || l >= nlist) { for (size_t e = 0; e < per; e++) luts[p * per + e] = 0.0f; continue; }
                for (int t = 0; t < d; t++) resid[t] = queries[(size_t)q * d + t] - coarse[(size_t)l * d + t];
                orc_build_luts(resid, 1, d, m, k, codebooks, luts + p * per);
            }
            /* qmax */
            int64_t met = 0, total = 0;
            for (int p = 0; p < nprobe; p++) {
                int l = pr[p];
                if (l >= 0 && l < nlist) total += list_offsets[l + 1] - list_offsets[l];
            }
            int64_t want = init < total ? init : total;
            temp.cap = (int64_t)topk < want ? topk : (int)want;
            for (int p = 0; p < nprobe && met < want; p++) {
                int l = pr[p];
                if (l < 0 || l >= nlist) continue;
                for (int64_t pos = list_offsets[l]; pos < list_offsets[l + 1] && met < want; pos++, met++)
                    heap_add(&temp, (double)adc_f32(codes + pos * cb, fmt, luts + p * per, m, k), pos);
            }
            float bound = temp.size > 0 ? (float)temp.a[0].v : INFINITY;
            for (int p = 0; p < nprobe; p++) qmax[p] = bound;
            /* 8 bits */
            orc_quantize_luts(luts, nprobe, m, k, qmax, qluts, NULL, NULL);
            /* Scan and Rerank */
            for (int p = 0; p < nprobe; p++) {
                int l = pr[p];
                if (l < 0 || l >= nlist) continue;
                cand.size = 0;
                for (int64_t pos = list_offsets[l]; pos < list_offsets[l + 1]; pos++)
                    heap_add(&cand, (double)adc_u8(codes + pos * cb, fmt, qluts + p * per, m, k), pos);
                int nc = heap_drain_sorted(&cand, sorted);
                for (int c = 0; c < nc; c++) {
                    int64_t pos = sorted[c].id;
                    heap_add(&best, (double)adc_f32(codes + pos * cb, fmt, luts + p * per, m, k), pos);
                }
            }
            int got = heap_drain_sorted(&best, sorted);
            for (int t = 0; t < topk; t++) {
                out_dist[(size_t)q * topk + t] = t < got ? (float)sorted[t].v : INFINITY;
                out_ids[(size_t)q * topk + t] = t < got ? (ids ? ids[sorted[t].id] : sorted[t].id) : -1;
            }
        }
        free(resid); free(luts); free(qluts); free(qmax); free(temp.a); free(cand.a); free(best.a); free(sorted);
    }
    return err;
}
