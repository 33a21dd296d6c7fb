/*
 * pq_adc.h -- C ABI of libpqadc: product-quantization ADC search on one MI355X (gfx950).
 *
 * The entry points follow the three-step search of the thesis (Section 2.3.3 "ANN
 * Search", Alg. 1): Index (ivf_adc_search), Tables (pq_build_luts, optionally followed
 * by pq_quantize_luts) and Scan (pq_adc_scan_topk), plus the second pass of the
 * two-pass search of Section 6.2.3 / Alg. 5 (pq_rerank_f32) and, on the database side, the
 * encoder of Section 2.3.1 (pq_encode).
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers owned by the caller (for instance the
 *     storage of torch tensors).  The library reads inputs, writes outputs and keeps
 *     no pointer past the call.  Arrays are dense, row-major, in the shapes given.
 *   - Work is enqueued on the HIP stream the context was created with and is
 *     asynchronous: results are valid after that stream is synchronised.
 *   - The context owns a device workspace that grows on demand (hipMalloc inside the
 *     call when a larger one is needed, otherwise no allocation).  One context must
 *     not be used from two host threads at once.
 *   - Return value: PQ_OK (0) or a negative pq_status.  Arguments are validated before
 *     anything is enqueued (a PQ_EINVAL / PQ_ESHAPE / PQ_EUNSUPPORTED leaves the outputs
 *     untouched); a PQ_EHIP or PQ_ENOMEM, and the PQ_ESHAPE of pq_derived_search for a
 *     candidate buffer that turns out too small, can arrive after some of the call's
 *     kernels were enqueued: the outputs are then unspecified.  pq_last_error() gives a
 *     message owned by the context (valid until the next call on it).  No exception
 *     crosses the ABI.
 *   - Codes: a code is m sub-quantizer indexes (Section 2.3.1).  PQ_CODES_U8 stores
 *     one index per byte, component 0 first (m bytes per code).  PQ_CODES_U4_PACKED
 *     stores two 4-bit indexes per byte, component 2r in bits 0-3 and component 2r+1
 *     in bits 4-7 of byte r (m/2 bytes per code; Section 5.2.2, Alg. 3).
 *   - Ids returned by the flat scan are positions in the code array (Alg. 1 keeps
 *     (i, d) pairs with i the list position).
 *   - Top-k order: ascending by (value, id); among equal values the smaller id wins,
 *     which is what Alg. 1's heap with strict "<" replacement yields when the list is
 *     scanned in order.  If fewer than topk codes exist the tail is padded with
 *     (+inf or UINT32_MAX, -1).
 */
#ifndef PQ_ADC_H
#define PQ_ADC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PQ_OK = 0,
    PQ_EINVAL = -1,       /* null pointer, non-positive size, bad enum            */
    PQ_ESHAPE = -2,       /* sizes inconsistent with each other (d % m, nprobe..) */
    PQ_EUNSUPPORTED = -3, /* valid request outside what the kernels cover         */
    PQ_EHIP = -4,         /* a HIP runtime call failed                            */
    PQ_ENOMEM = -5        /* workspace allocation failed                          */
} pq_status;

typedef enum { PQ_CODES_U8 = 0, PQ_CODES_U4_PACKED = 1 } pq_code_fmt;
typedef enum { PQ_LUT_F32 = 0, PQ_LUT_U8 = 1 } pq_lut_fmt;

typedef struct pq_ctx pq_ctx;

/* Create a context on `device` using `hip_stream` (a hipStream_t, borrowed; NULL = the
 * default stream).  *out is set on success. */
int pq_create(pq_ctx **out, int device, void *hip_stream);
/* Free the context and its workspace (synchronises the stream first). */
int pq_destroy(pq_ctx *ctx);
const char *pq_last_error(const pq_ctx *ctx);
/* Library version string, static storage. */
const char *pq_version(void);

/* Switches for tests and tuning, kept in the context.  pq_create reads each one once from the
 * environment variable "PQ_" + NAME IN UPPER CASE (unset = the default below); pq_set_option changes
 * it for the calls that follow, pq_unset_option returns it to its default.  Unknown name: PQ_EINVAL.
 *   scan_prune (1)            0: float scans without lower-bound pruning
 *   scan_q8 (1)               0: no 8-bit lower bounds (16 queries per pass), whatever the number of queries
 *   scan_force_general (0)    1: the general scan kernel for every shape
 *   scan_blocks (number of compute units), scan_items_per_block (4, or 6 with 16 queries per pass),
 *   scan_head (4)             launch shape of the flat scans: persistent blocks, work items per block, block
 *                             tiles per chunk of the first round of short items that long result lists
 *                             start with (0: none)
 *   lut_mfma (1)              0: pq_build_luts without the matrix cores
 *   ivf_prune (unset)         1 / 0: the inverted lists that the kernel for short lists does not take are scanned
 *                             by the loop on 16-bit lower bounds / by the plain float loop (unset: the former
 *                             where short lists have their kernel, else the latter)
 *   ivf_ws_gib (24)           workspace limit of ivf_adc_search in GiB (1 ... 128)
 *   ivf_block_waves (8)       16: inverted lists scanned by blocks of 16 waves
 *   scan_wide_seed (1)        0: first bounds of flat scans of few queries from the small sample only
 *   ivf_short_max (12288)     inverted lists of fewer codes take the kernel for short lists (0: none)
 *   ivf_coarse_f32 (1)        0: Index step of ivf_adc_search from exact distances to every list (default: lists
 *                             ranked by matrix-core distances, the nearest measured exactly; same lists)
 *   ivf_coarse_f16 (1)        0: the ranking pass over all lists on the fp32 matrix cores (default: on the fp16 ones,
 *                             every operand as the sum of two halves: the accuracy of fp32, a third of the time)
 *   ivf_quick_chunk_rows (1048576)  ivf_quick_adc_search: rows per work item at most (1024 ... 2^20); a list longer than
 *                             this is scanned in chunks, and a query's result lists (one per chunk of each of its
 *                             lists, at most nprobe + ntotal / this value) are part of the workspace */
int pq_set_option(pq_ctx *ctx, const char *name, int value);
int pq_unset_option(pq_ctx *ctx, const char *name);

/* Tables step, Eq. (tables) of Section 2.3.3:  luts[q][j][i] = || y_q^j - C^j[i] ||^2,
 * sub-space j = dimensions j*d/m .. (j+1)*d/m-1.
 *   queries   [nq][d] f32, codebooks [m][k][d/m] f32  ->  luts [nq][m][k] f32.
 * Requires d % m == 0, 1 <= k <= 65536.  Sub-vectors of 8 dimensions and more are handled in
 * double precision on the matrix cores (expanded form, entries rounded once to f32); shorter
 * ones by differences, squared and added in double in the order of the dimensions, rounded once. */
int pq_build_luts(pq_ctx *ctx, const float *queries, const float *codebooks, int nq, int d, int m, int k,
                  float *luts);

/* Rotation of optimized product quantization (Section 2.3.4, paragraph on OPQ:
 * opq(x) = pq(R x) with R orthogonal): out[p] = R * vectors[p], to be applied to database
 * vectors before pq_encode and to queries before pq_build_luts.
 *   vectors [n][d] f32, rot [d][d] f32 row-major  ->  out [n][d] f32 (must not overlap vectors).
 * Sums in double precision, rounded once.  At most 2^28 vectors per call. */
int pq_rotate(pq_ctx *ctx, const float *vectors, const float *rot, int64_t n, int d, float *out);

/* Encoder of the product quantizer (Section 2.3.1, "Vector Encoding"): sub-vector j of every
 * vector is replaced by the index of the closest centroid of codebook j,
 *   code_j(x) = argmin_i || x^j - C^j[i] ||^2, ties to the smallest i,
 * decided on distances computed in double precision.
 *   vectors [n][d] f32, codebooks [m][k][d/m] f32  ->  codes [n][code_bytes] u8
 * (PQ_CODES_U8: m bytes, k <= 256; PQ_CODES_U4_PACKED: m/2 bytes, k <= 16, m even).
 * Requires d % m == 0. */
int pq_encode(pq_ctx *ctx, const float *vectors, const float *codebooks, int64_t n, int d, int m, int k,
              pq_code_fmt cf, uint8_t *codes);

/* 8-bit quantisation of each query's tables (Sections 4.2.4, 5.2.1; Section 6.2.3 Step 1.2
 * for the unsigned 0..254 + 255 range).  Per query q:
 *   qmin  = min over all m*k entries;  range = qmax[q] - qmin;
 *   scale = (range > 0 and finite) ? 255 / range : 0;
 *   qluts = t >= 255 ? 255 : floor(t),  t = (luts - qmin) * scale      (all in f32)
 *   luts [nq][m][k] f32, qmax [nq] f32 -> qluts [nq][m][k] u8, qmin_out [nq], scale_out [nq]
 * (the last two may be NULL). */
int pq_quantize_luts(pq_ctx *ctx, const float *luts, int nq, int m, int k, const float *qmax, uint8_t *qluts,
                     float *qmin_out, float *scale_out);

/* Upper quantisation bound (Sections 4.2.4 / 5.2.1: distance to a temporary neighbour
 * found by a float ADC scan of the first `init` codes; Section 6.2.3 Step 1.2: greatest
 * distance among the first r2 codes).  qmax_out[q] = kq-th smallest float ADC distance
 * among the first min(init, n) codes (kq clipped to that count).  Requires init <= 4096. */
int pq_qmax_prescan(pq_ctx *ctx, const uint8_t *codes, int64_t n, pq_code_fmt cf, const float *luts, int nq,
                    int m, int k, int init, int kq, float *qmax_out);

/* Scan step (Alg. 1 `scan` + `adc`, Eq. (adc1); Alg. 3 `quick_adc_scan` for packed
 * 4-bit codes with quantised tables):  value[q][i] = sum_j luts[q][j][code_i[j]], and the
 * topk smallest (value, i) per query.
 *   codes [n][code_bytes] u8; luts [nq][m][k] f32 (PQ_LUT_F32) or u8 (PQ_LUT_U8);
 *   out_val [nq][topk] f32 (float tables) or u32 (u8 tables, plain integer sums, no
 *   saturation); out_ids [nq][topk] i64.
 * Covered: (U8 codes, F32 tables, k = 256, m = 8 or 16), (U4 codes, U8 tables, k = 16,
 * m = 16), and any (U8 | U4 codes, F32 | U8 tables) with m*k <= 8192 through a slower
 * general kernel.  1 <= topk <= 1024, 0 <= n < 2^32; `codes` 16-byte aligned.
 * Float sums add the m entries in fp32, in table order or in a rotation of it (the result
 * differs from the exact sum by at most (m-1) * 2^-24 relative either way).  For k = 256,
 * m = 8 or 16 and n >= 65536 the kernel first dismisses codes by integer lower bounds of their
 * distances (the pruning idea of Section 4.2: small quantised tables, exact distances only
 * for the codes they cannot rule out) and forms float sums only for the rest; the result is
 * that of the plain definition.  The bounds are 16-bit sums for 8 queries per pass over the
 * codes, or, for m = 8 and 249 queries and more, 8-bit sums for 16 queries per pass.
 * Integer sums are exact; with 249 queries and more and n >= 65536 the integer scan also
 * runs on 8-bit lower bounds of its sums (16 queries per pass) and adds up the exact sums
 * only for the codes that pass.
 * (Switches: pq_set_option.) */
int pq_adc_scan_topk(pq_ctx *ctx, const uint8_t *codes, int64_t n, pq_code_fmt cf, const void *luts,
                     pq_lut_fmt lf, int nq, int m, int k, int topk, void *out_val, int64_t *out_ids);

/* pq_adc_scan_topk for callers that cannot allocate device memory: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * the same results as pq_adc_scan_topk; where that call uses the context's growable workspace
 * (shared bounds, candidate histograms, per-wave candidate lists, per-chunk result lists, first-bound
 * tables), this one uses a fixed scratch array of PQ_NOALLOC_SCRATCH_MIB MiB that is part of the
 * library image: every GPU the library runs on holds its own copy until the process ends, and its
 * address is looked up once per device by pq_create.  The call itself makes no hipMalloc / hipFree
 * and calls no allocating routine; inputs and outputs are the caller's.
 * Limit: the scratch the scan needs must fit.  That holds for the tuned shapes with topk <= 128 and
 * fewer than 249 queries, whatever n is (about 120 MiB on 256 compute units), and for calls of the
 * general kernel with few (chunk, query) blocks; a request that does not fit returns PQ_ENOMEM with a
 * message naming both sizes, and nothing has been enqueued.
 * Every call on a GPU shares that GPU's array (whatever the context or stream): calls that overlap
 * in time on one GPU race.  The array keeps the last call's contents; everything that must start
 * from a known value (work counter, bounds, histograms, candidate counters) is cleared by the call's
 * first kernel, as in pq_adc_scan_topk. */
#define PQ_NOALLOC_SCRATCH_MIB 128
int pq_adc_scan_topk_noalloc(pq_ctx *ctx, const uint8_t *codes, int64_t n, pq_code_fmt cf, const void *luts,
                             pq_lut_fmt lf, int nq, int m, int k, int topk, void *out_val, int64_t *out_ids);

/* Second pass of the two-pass search (Alg. 5 `rerank`): float ADC of the given
 * candidates and the topk smallest (distance, id).
 *   cand_ids [nq][ncand] i64, positions into codes; negative entries are skipped.
 *   out_dist [nq][topk] f32, out_ids [nq][topk] i64.  1 <= topk <= ncand <= 4096. */
int pq_rerank_f32(pq_ctx *ctx, const uint8_t *codes, int64_t n, pq_code_fmt cf, const float *luts, int nq,
                  int m, int k, const int64_t *cand_ids, int ncand, int topk, float *out_dist,
                  int64_t *out_ids);

/* Search with derived quantizers (chapter 6; Section 6.2.3, Alg. 5 nns_derived) over 64-bit codes
 * of m = 4 sub-quantizer indexes of 16 bits each.  The codebooks obey property P1 of Section
 * 6.2.2: the low 8 bits of a centroid's index name the centroid of the derived 8-bit quantizer
 * it belongs to, so the derived quantizer needs no codes of its own.
 *   Step 1.1  compact tables of the derived codebooks (as pq_build_luts);
 *   Step 1.2  qmin = smallest entry of the query's compact tables, qmax = greatest compact
 *             distance among the first min(r2, n) codes (entries added in double in table
 *             order, rounded once), 8-bit tables as pq_quantize_luts;
 *   Step 1.3  integer distance of every code = sum of the 8-bit entries at the low bytes of
 *             its indexes (plain sums, no saturation), which is the index of its bucket;
 *   Step 2    the buckets are taken in increasing order until r2 vectors are in; the bucket
 *             of the r2-th vector is finished, so the candidates of a query are all codes up
 *             to that bucket b* (all codes if n < r2).  Their precise distances
 *             sum_j || y^j - C^j[c[j]] ||^2 come from the full codebooks (each term summed in
 *             double and rounded to f32 like a table entry, the four terms added in double,
 *             rounded once); the topk smallest (distance, row) are returned, padded with
 *             (+inf, -1).
 *   codes [n][4] u16 (device, 16-byte aligned; index c[j] < k), derived_codebooks [4][256][d/4],
 *   codebooks [4][k][d/4], queries [nq][d]  ->  out_dist [nq][topk] f32, out_ids [nq][topk] i64.
 * Optional outputs (device, may be NULL): bucket_out [nq] u32 = b*; ncand_out [nq] i64 = number
 * of candidates; cand_ids_out [nq][cand_cap] i64 = their rows in no particular order, padded
 * with -1 (PQ_ESHAPE if a query has more than cand_cap candidates).
 * The capped-buckets lists of the thesis are replaced by two passes over the codes (bucket
 * counts, then the ids of the buckets 0..b*); between them the call waits for the stream and
 * reads the nq list sizes back to size its workspace.  With 640 queries and more the second pass
 * takes 16 queries per pass over the codes (lower bounds of the integer sums in the loop, exact
 * sums for the codes that pass; option scan_q8 = 0: 8 queries per pass as for fewer queries).
 * Covered: m = 4, d % 4 == 0, d <= 4096, 256 <= k <= 65536, 1 <= topk <= 128, r2 >= 1,
 * nq <= 65535, 0 <= n < 2^32. */
int pq_derived_search(pq_ctx *ctx, const uint16_t *codes, int64_t n, const float *derived_codebooks,
                      const float *codebooks, int k, const float *queries, int nq, int d, int m, int r2, int topk,
                      float *out_dist, int64_t *out_ids, uint32_t *bucket_out, int64_t *ncand_out,
                      int64_t *cand_ids_out, int64_t cand_cap);

/* Inverted lists of an IVFADC index (Section 2.3.2): nlist coarse centroids; the codes
 * of list l are rows list_offsets[l] .. list_offsets[l+1]-1 of `codes`, which encode the
 * residuals x - centroid_l.  ids may be NULL (id = row number). */
typedef struct {
    const float *coarse_centroids; /* [nlist][d] f32, device */
    const int64_t *list_offsets;   /* [nlist+1] i64, device, non-decreasing, [0] = 0 */
    const uint8_t *codes;          /* [ntotal][code_bytes], device, grouped by list */
    const int64_t *ids;            /* [ntotal] i64, device, or NULL */
    int nlist;
    int d;
    int64_t ntotal;
} ivf_lists;

/* Index + Tables + Scan of Section 2.3.3 with an inverted index: for each query the
 * nprobe lists with the closest centroids (ties: smaller list id), tables of the query
 * residual y - centroid_l per probed list, ADC over the codes of those lists, topk
 * smallest (distance, row) overall, rows then mapped through `ids` (equal distances are
 * ordered by their position in the grouped code array, not by the mapped id).  probe_out [nq][nprobe] i32 may be NULL; when given
 * it receives the probed lists in ascending (distance, list id) order.
 * Covered: U8 codes, k = 256, m = 8 or 16; 1 <= nprobe <= min(nlist, 1024);
 * 1 <= topk <= 128; ntotal < 2^32.
 * Queries are served in batches whose workspace (coarse distances, residual tables of
 * every (query, list) pair, result lists) stays within ivf_ws_gib GiB of device
 * memory (pq_set_option, default 24, 1 ... 128); one batch is fastest because a list's
 * codes are then scanned once for all the queries that probe it.
 * With m = 8, lists of fewer than ivf_short_max codes are scanned by a kernel of their own (the whole list for
 * four pairs per pass); the longer lists by the loop on 16-bit lower bounds with exact float distances only for
 * the codes whose bound passes (as in pq_adc_scan_topk), eight (query, list) pairs per work item, in blocks of
 * 8 waves, two per compute unit.  Option ivf_prune = 0 selects the plain float loop, four pairs per item (also
 * the default with m = 16 and with ivf_block_waves = 16: one block of 16 waves per compute unit, no kernel
 * for short lists).
 * The probed lists are those with the smallest (distance from the plain definition, summed in double and
 * rounded to fp32 once; list id).  With many lists and queries they are found through approximate distances:
 * the lists are ranked on the matrix cores (operands split into two fp16 halves each, fp32 accumulation; magnitudes of
 * 2^-40 .. 2^40), the nprobe + 16 nearest are measured exactly, and a query whose nprobe-th exact distance is not
 * provably below that of every other list gets first all the lists that the ranking pass kept for it (some hundreds)
 * and then, if that does not settle it either, all its distances computed exactly (option ivf_coarse_f32 = 0: exact
 * distances to every list for every query). */
int ivf_adc_search(pq_ctx *ctx, const ivf_lists *lists, const float *codebooks, int m, int k, pq_code_fmt cf,
                   const float *queries, int nq, int nprobe, int topk, float *out_dist, int64_t *out_ids,
                   int32_t *probe_out);

/* The same search with Quick ADC in the Scan step (chapter 5; Section 5.2: 4-bit sub-quantizers and tables
 * quantised to 8 bits; Section 5.3 evaluates Quick ADC inside the inverted index of Section 2.3.2).
 * lists->codes holds PQ_CODES_U4_PACKED codes of m = 16 indexes (8 bytes per code), codebooks [16][16][d/16].
 * Index and Tables steps as ivf_adc_search.  Then, per query:
 *   qmax    float ADC of the first `init` codes met when the probed lists are walked in probe order, each code
 *           with the float tables of its own (query, list) pair; qmax = the topk-th smallest of these distances
 *           (rank clipped to the number of codes met; +inf if the probed lists are empty) - the distance to a
 *           temporary topk-th neighbour (Section 5.2.1);
 *   8 bits  the tables of every (query, list) pair quantised as by pq_quantize_luts, with the pair's own qmin
 *           and the query's qmax;
 *   Scan    plain integer sums of the 8-bit entries (Alg. 3) for every code of the list; the kprime smallest
 *           (sum, row) of each pair are its candidates (sums of different pairs have different scales and are
 *           never compared);
 *   Rerank  float ADC of the candidates with the pair's float tables; the topk smallest (distance, row) over
 *           the pairs of the query, rows mapped through `ids`.  Fewer than topk candidates: (+inf, -1) behind.
 * Float sums are formed in double in table order and rounded to fp32 once.
 * Covered: m = 16, k = 16; 1 <= nprobe <= min(nlist, 1024); 1 <= topk, kprime <= 128; 1 <= init <= 4096;
 * ntotal < 2^32; codes 16-byte aligned.  Workspace and batching as ivf_adc_search. */
int ivf_quick_adc_search(pq_ctx *ctx, const ivf_lists *lists, const float *codebooks, int m, int k, const float *queries,
                         int nq, int nprobe, int init, int kprime, int topk, float *out_dist, int64_t *out_ids,
                         int32_t *probe_out);

#ifdef __cplusplus
}
#endif
#endif /* PQ_ADC_H */
