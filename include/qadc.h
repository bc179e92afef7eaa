/*
 * qadc.h -- C ABI of the MI355X (gfx950) asymmetric-distance scan over
 * product-quantized codes with quantized distance tables.
 *
 * The calls follow the paper's statement of the search problem (Section 2.1.3:
 * query z, codebooks, short codes, R -> the R nearest codes) and its distance
 * quantizer (Section 3.4) and scan loop (Section 3.5).
 *
 * General conventions
 *   - Pointers marked [dev] are device pointers owned by the caller (hipMalloc /
 *     PyTorch); pointers marked [host] are ordinary host memory.  The library
 *     never frees or keeps caller memory beyond a call, except that an index
 *     handle keeps the codebook pointer it was given (the caller keeps that
 *     buffer alive for the life of the handle).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Every call only enqueues work on that stream; it never synchronises and
 *     never allocates device memory (pq_index_create excepted).
 *   - Return value: PQ_OK (0) or a negative code; pq_last_error() then gives a
 *     thread-local description.  Nothing throws or aborts.
 *   - Row-major, densely packed arrays throughout.  Inputs are assumed finite
 *     (no NaN / Inf in queries, codebooks or tables).
 *   - Sub-code layout (Section 3.3, packing paragraph): a code is a
 *     little-endian bit stream of code_size = ceil(sum(nbits)/8) bytes;
 *     sub-code j occupies bits [off_j, off_j + nbits[j]), off_j = sum of the
 *     earlier widths, bit 0 = least significant bit of byte 0.  For m x 4
 *     layouts byte i holds sub-code 2i in its low nibble and 2i+1 in its high
 *     nibble.
 *   - Results are sorted ascending by (key, id); ties go to the lowest id.
 *     When fewer than R codes exist the tail is padded with id = -1,
 *     key = q_max, dist = +inf.
 */
#ifndef QADC_H
#define QADC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PQ_OK 0
#define PQ_EINVAL (-1) /* bad argument: null pointer, bad shape, unsupported size, misalignment */
#define PQ_ENOMEM (-2) /* caller-supplied workspace too small */
#define PQ_EHIP (-3)   /* a HIP runtime call failed (message holds hipGetErrorString) */

/* limits of this build */
#define PQ_MAX_M 64           /* sub-quantizers per code */
#define PQ_MAX_TABLE_LEN 4096 /* sum_j 2^nbits[j] */
#define PQ_MAX_R 2048         /* results per query */
#define PQ_MAX_T_EFF 8192     /* calibration codes: max(t, 4R) must not exceed this */
#define PQ_MAX_DIM 4096
#define PQ_MAX_NQ 65535       /* queries per call */

/* Immutable description of a product quantizer; opaque. */
typedef struct pq_index pq_index_t;

/*
 * Per-query state of the distance quantizer (Section 3.4).  One per query for
 * the exhaustive calls.  24 bytes, no padding.
 *   d_min     sum over sub-quantizers of the smallest table entry (fp64 sum)
 *   delta     bin width (d_max - d_min)/q_max; 0 when d_max <= d_min or when
 *             there was no code to calibrate on (all table entries are then 0)
 *   d_max     R-th smallest float ADC among the first t_eff codes
 *   key_bound an inclusive upper bound on the R-th best quantized key of the
 *             list.  Output of pq_quantize_tables (the R-th smallest key among
 *             the first few ten thousand codes, a superset of the calibration
 *             codes) and INPUT of pq_adc_scan_topk, which keeps only codes with
 *             key <= key_bound.  A caller who writes this record by hand either
 *             supplies a valid bound or PQ_KEY_BOUND_UNKNOWN (any value >= q_max
 *             means the same): every code is then a candidate and the selection
 *             takes its slow exact path.  A bound that is too small loses
 *             results without an error.
 */
typedef struct pq_qparams {
    double d_min;
    double delta;
    float d_max;
    uint32_t key_bound;
} pq_qparams_t;
#define PQ_KEY_BOUND_UNKNOWN 0xffffffffu

/*
 * Create an index handle.  Section 2.1.2 (product quantizer = m codebooks) and
 * Section 3.1 (irregular product quantizers: sub-quantizers of different widths
 * over sub-vectors of different dimension).
 *   d          vector dimension, 1..PQ_MAX_DIM
 *   m          number of sub-quantizers, 1..PQ_MAX_M
 *   nbits      [host][m] bits of each sub-quantizer, each 1..8
 *   dsub       [host][m] dimensions of each sub-vector, each >= 1, sum == d
 *   codebooks  [dev] concatenation over j of [2^nbits[j]][dsub[j]] float32
 *   acc_bits   8 or 16: width of quantized table entries and of the
 *              saturating accumulator (q_max = 2^acc_bits - 1)
 * Allocates a few KB of device memory for the layout description on the
 * current device.  Returns PQ_EINVAL for bad shapes.
 */
int pq_index_create(pq_index_t **out, int d, int m, const int32_t *nbits, const int32_t *dsub,
                    const float *codebooks, int acc_bits);
void pq_index_destroy(pq_index_t *idx);

size_t pq_code_size(const pq_index_t *idx); /* bytes per code */
size_t pq_table_len(const pq_index_t *idx); /* T = sum_j 2^nbits[j] */

/* Bytes of workspace pq_adc_scan_topk needs for (nq queries, n codes, R). */
size_t pq_workspace_bytes(const pq_index_t *idx, int nq, int64_t n, int R);
/* Bytes of workspace ivf_adc_scan_topk needs for (nq queries, nprobe probes, R). */
size_t ivf_workspace_bytes(const pq_index_t *idx, int nq, int nprobe, int R);
/* The same plus room to order the (query, probe) pairs by probed cell (K cells): given that
 * much, and at least K/4 pairs, ivf_adc_scan_topk scans the pairs of one cell close together
 * in time, so that a list probed by several queries of the call is read from memory once;
 * with at least 1.5 pairs per cell, 16 x 4-bit codes over equal sub-spaces of 4, 6 or 8
 * dimensions and 8-bit tables, one pass over a list then serves up to four of the queries that
 * probe it (PQ_OPT_IVF_SHARED_LISTS).  Results are the same. */
size_t ivf_sorted_workspace_bytes(const pq_index_t *idx, int nq, int nprobe, int R, int K);

/*
 * Distance tables, eq. (1): tables[q][toff_j + i] = || z_q^j - C^j[i] ||^2.
 * fp32, dimensions accumulated in ascending order with separate subtract,
 * multiply and add (no fused multiply-add), so the result is reproducible bit
 * for bit.
 *   queries [dev][nq][d] float32      tables [dev][nq][T] float32 (out)
 * nq == 0 is a no-op.
 */
int pq_compute_tables(const pq_index_t *idx, const float *queries, int nq, float *tables,
                      void *stream);

/*
 * Distance quantizer, Section 3.4.  For every query:
 *   t_eff = min(n, max(t, 4R)); d_max = min(R,t_eff)-th smallest float ADC
 *   (eq. (2), fp32, sub-quantizers in ascending order) among codes 0..t_eff-1;
 *   p_min(j) = smallest entry of table j; d_min = sum_j p_min(j) (fp64);
 *   delta = (d_max - d_min)/q_max (fp64);
 *   q = min(q_max, floor((p - p_min(j))/delta)) (fp64), all 0 if delta is not a
 *   positive finite number (delta is then stored as 0).
 *   tables  [dev][nq][T] float32       codes [dev][n][code_size] uint8
 *   qtables [dev][nq][T] uint8 (acc_bits 8) or uint16 (acc_bits 16)   (out)
 *   qparams [dev][nq]                                                   (out)
 * Requires 1 <= R <= PQ_MAX_R, t >= 1, max(t,4R) <= PQ_MAX_T_EFF, n >= 0.
 */
int pq_quantize_tables(const pq_index_t *idx, const float *tables, int nq, const uint8_t *codes,
                       int64_t n, int t, int R, void *qtables, pq_qparams_t *qparams,
                       void *stream);

/*
 * Scan, eq. (2) with quantized tables and saturating unsigned sums at the
 * accumulator width (Section 3.4 last paragraph, Section 3.5), then the R
 * smallest (key, id) per query, id = position of the code in `codes`.
 *   qtables, qparams  as written by pq_quantize_tables, or by the caller (then see
 *             pq_qparams_t.key_bound, an input here); nq <= PQ_MAX_NQ, R <= PQ_MAX_R
 *   codes     [dev][n][code_size], n < 2^31; must be 16-byte aligned
 *   out_ids   [dev][nq][R] int32       out_keys [dev][nq][R] uint16
 *   out_dist  [dev][nq][R] float32 = fmaf(key, (float)delta, (float)d_min)
 *   workspace [dev] >= pq_workspace_bytes(idx, nq, n, R) bytes, 256-byte
 *             aligned, any content; private to this call until the stream has
 *             finished it (concurrent calls need distinct workspaces)
 * nq == 0 is a no-op; n == 0 writes padding only.
 */
int pq_adc_scan_topk(const pq_index_t *idx, const void *qtables, const pq_qparams_t *qparams,
                     int nq, const uint8_t *codes, int64_t n, int R, int32_t *out_ids,
                     uint16_t *out_keys, float *out_dist, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * pq_adc_scan_topk for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and error rules, minus the workspace: the scan's scratch memory is an
 * array of PQ_STATIC_SCRATCH_BYTES bytes inside the library, one copy per GPU, held from the
 * time the library is loaded until the process ends.  The call allocates nothing and frees
 * nothing.  PQ_ENOMEM when pq_workspace_bytes(idx, nq, n, R) exceeds PQ_STATIC_SCRATCH_BYTES
 * (the message says how much was needed).  All calls on one GPU share that GPU's array: two
 * calls that overlap in time on one GPU (different streams, different threads) race and give
 * undefined results; calls on one stream, or otherwise ordered, are fine.  Nothing in the array
 * has to be cleared between calls.
 */
#define PQ_STATIC_SCRATCH_BYTES (16u << 20)
int pq_adc_scan_topk_static(const pq_index_t *idx, const void *qtables, const pq_qparams_t *qparams,
                            int nq, const uint8_t *codes, int64_t n, int R, int32_t *out_ids,
                            uint16_t *out_keys, float *out_dist, void *stream);

/*
 * The two halves of pq_adc_scan_topk as calls of their own (same arguments, same
 * workspace): pq_adc_scan_candidates prepares the query's lookup tables in the
 * workspace, streams the codes and leaves, per query, the codes whose key is
 * within qparams.key_bound in the workspace; pq_select_topk turns those
 * candidates into the sorted top-R.  Calling the two in this order on one stream
 * is exactly pq_adc_scan_topk.
 */
int pq_adc_scan_candidates(const pq_index_t *idx, const void *qtables,
                           const pq_qparams_t *qparams, int nq, const uint8_t *codes, int64_t n,
                           int R, void *workspace, size_t workspace_bytes, void *stream);
int pq_select_topk(const pq_index_t *idx, const void *qtables, const pq_qparams_t *qparams, int nq,
                   const uint8_t *codes, int64_t n, int R, int32_t *out_ids, uint16_t *out_keys,
                   float *out_dist, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The three calls above in one: tables (eq. (1)), distance quantizer (Section
 * 3.4) and scan + top-R (eq. (2), Section 3.5) for nq queries against one list
 * of codes, with the float tables kept on chip.  Same arithmetic, same results
 * and same argument rules as pq_compute_tables -> pq_quantize_tables ->
 * pq_adc_scan_topk; it saves two kernel launches per batch, which matters
 * when a batch is a single query.
 *   workspace >= pq_search_workspace_bytes(idx, nq, n, R), 256-byte aligned, any
 *   content; it also holds the quantized tables and quantizer parameters.
 */
size_t pq_search_workspace_bytes(const pq_index_t *idx, int nq, int64_t n, int R);
int pq_search_topk(const pq_index_t *idx, const float *queries, int nq, const uint8_t *codes,
                   int64_t n, int t, int R, int32_t *out_ids, uint16_t *out_keys, float *out_dist,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Inverted-list search (Section 2.1.1: residuals are what is encoded;
 * Section 2.1.3: one table set per probed cell from z' = z - centroid).
 * For every query: d_max from the float ADC of the first t_eff probed codes
 * (probe order, list order, each with its own cell's tables); per probed list
 * its own p_min / d_min / delta from that shared d_max; lists whose d_min
 * is not below d_max are skipped (nothing in them is closer than d_max); every code of the other probed lists gets
 * dist = fmaf(key, (float)delta_l, (float)d_min_l); the R smallest
 * (dist, stored id) are returned.
 *   coarse       [dev][K][d] float32 cell centroids
 *   list_offsets [dev][K+1] int64, list l = codes [off[l], off[l+1])
 *   list_codes   [dev][off[K]][code_size]; 16-byte aligned base
 *   list_ids     [dev][off[K]] int32 stored ids
 *   queries      [dev][nq][d]
 *   probe_ids    [dev][nq][nprobe] int32, nearest cell first, distinct;
 *                negative entries are ignored
 *   out_ids      [dev][nq][R] int32     out_dist [dev][nq][R] float32
 *   workspace    >= ivf_workspace_bytes(idx, nq, nprobe, R), 256-byte aligned
 *                (ivf_sorted_workspace_bytes for the cell-ordered scan)
 * Requires 1 <= nprobe <= 1024 and the limits of pq_quantize_tables.
 */
int ivf_adc_scan_topk(const pq_index_t *idx, const float *coarse_centroids, int K,
                      const int64_t *list_offsets, const uint8_t *list_codes,
                      const int32_t *list_ids, const float *queries, int nq,
                      const int32_t *probe_ids, int nprobe, int t, int R, int32_t *out_ids,
                      float *out_dist, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Inverted-list search with a bound that tightens from list to list (optional
 * mode).  Section 3.5: a scanned vector is kept when it is closer than the worst
 * of the R candidates held; Section 3.4: that worst distance is the largest
 * distance the quantizer has to represent.  For every query the probed lists are
 * visited in probe order, and list l is quantized against
 *     cur_l = min(d_max, R-th smallest dist among the candidates of the lists
 *                        visited before l)     (the second term once R are held)
 * with d_max the calibration bound of ivf_adc_scan_topk: p_min / d_min as there,
 * delta_l = (cur_l - d_min_l) / q_max; a list with d_min_l >= cur_l is skipped;
 * a code whose sum saturates (key = q_max) is no candidate; every other code
 * gets dist = fmaf(key, (float)delta_l, (float)d_min_l).  The R smallest
 * (dist, stored id) are returned, fewer (ids -1, dist +inf) if fewer codes stayed
 * below their bounds.  Later lists are quantized more finely than with the fixed
 * bound; the result depends on the probe order by construction.
 * Arguments, workspace size (ivf_workspace_bytes), limits and errors as for
 * ivf_adc_scan_topk.  One block of 256 threads serves a query: the call needs a
 * few hundred queries to fill the chip.
 */
int ivf_adc_scan_topk_tightening(const pq_index_t *idx, const float *coarse_centroids, int K,
                                 const int64_t *list_offsets, const uint8_t *list_codes,
                                 const int32_t *list_ids, const float *queries, int nq,
                                 const int32_t *probe_ids, int nprobe, int t, int R,
                                 int32_t *out_ids, float *out_dist, void *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * Encode vectors (Section 2.1.2: every sub-vector is replaced by the index of its
 * nearest centroid; Section 2.1.1: behind an inverted index the residual
 * x - centroid is encoded; Section 3.3: sub-codes are packed as a little-endian
 * bit stream, sub-code j in bits [off_j, off_j + nbits[j])).  The distance of
 * sub-vector j to centroid i is eq. (1) with z = x (fp32, dimensions ascending,
 * separate subtract / multiply / add); sub-code j is the index of the smallest,
 * the lowest index among equals.
 *   vectors     [dev][n][d] float32
 *   shift_rows  [dev][K][d] float32 and shift_ids [dev][n] int32 (each in 0..K-1):
 *               vector v is encoded as vectors[v] - shift_rows[shift_ids[v]]; both
 *               NULL: vectors are encoded as they are
 *   codes       [dev][n][pq_code_size(idx)], every byte written
 * Needs 64 * ((d | 1) * 4 + m) bytes of LDS per block (d up to about 630).
 * Errors: PQ_EINVAL (null, only one of the shift arguments, d too large), PQ_EHIP.
 */
int pq_encode(const pq_index_t *idx, const float *vectors, int64_t n, const float *shift_rows,
              const int32_t *shift_ids, uint8_t *codes, void *stream);

/*
 * Coarse-quantizer search (Section 2.1.1: a query is routed to the cells of the
 * inverted index whose centroids are nearest).  For every query the nprobe
 * cells with the smallest (score, id), score = ||c||^2 - 2 z.c, i.e. the
 * squared distance minus the query's own norm, are returned in that order.
 * Arithmetic (fp32): z.c and ||c||^2 are chains of fused multiply-adds over the
 * dimensions in ascending order, score = fma(-2, z.c, ||c||^2).  The output is
 * what ivf_adc_scan_topk takes as probe_ids.
 *   queries      [dev][nq][d] float32     centroids [dev][K][d] float32
 *   nprobe       1..1024; when nprobe > K the tail is padded with id -1, score +inf
 *   probe_ids    [dev][nq][nprobe] int32
 *   probe_scores [dev][nq][nprobe] float32, or NULL
 *   workspace    >= ivf_coarse_workspace_bytes(nq, K), 256-byte aligned, any content
 * Queries are processed in passes whose score matrix stays within 256 MB.
 * Errors: PQ_EINVAL (shape, null, alignment), PQ_ENOMEM (workspace), PQ_EHIP.
 */
size_t ivf_coarse_workspace_bytes(int nq, int K);
int ivf_coarse_search(const float *queries, int nq, const float *centroids, int K, int d, int nprobe,
                      int32_t *probe_ids, float *probe_scores, void *workspace,
                      size_t workspace_bytes, void *stream);

/* Description of the last error on this thread ("" if none). */
const char *pq_last_error(void);

/*
 * Tuning options.  Process-wide; none changes a result.  Workspace sizes depend on
 * PQ_OPT_SCAN_BLOCKS and PQ_OPT_PILOT_BLOCKS: set those before asking for sizes, and do not
 * change them between a size query and the call that uses the workspace.
 * pq_set_option returns PQ_EINVAL for an unknown option or a value outside its range
 * (pq_last_error says which); pq_get_option returns -1 for an unknown option.
 */
enum {
    PQ_OPT_SCAN_BLOCKS = 0,        /* scan blocks per query for one or a few queries: 1..4096 (2048) */
    PQ_OPT_PILOT_CODES = 1,        /* codes the fused search samples for its pruning bound when
                                      several blocks share them: 0..2^24 (524288) */
    PQ_OPT_PILOT_CODES_SINGLE = 2, /* ... when one block per query counts them: 0..2^24 (65536) */
    PQ_OPT_PILOT_BLOCKS = 3,       /* most blocks per query that share that sample: 1..128 (128) */
    PQ_OPT_IVF_THREADS = 4,        /* threads per (query, list) block of the inverted-list scan:
                                      64, 128 or 256 (128) */
    PQ_OPT_SHARED_PASSES = 5,      /* 1: four queries of a batch share each pass over the codes;
                                      0: one pass per query (1) */
    PQ_OPT_COARSE_FILTER = 6,      /* 1: the coarse search keeps only scores within a sampled bound;
                                      0: it always writes the full score matrix (1) */
    PQ_OPT_IVF_SHARED_LISTS = 7,   /* inverted-list search, 16 x 4-bit codes with 8-bit tables: one pass
                                      over a list serves up to four of the queries that probe it.
                                      0: never; 1: when the call has at least 1.5 (query, probe)
                                      pairs per cell and the workspace is the larger one; 2: whenever
                                      the workspace is the larger one (1) */
    PQ_OPT_COUNT = 8
};
int pq_set_option(int option, int64_t value);
int64_t pq_get_option(int option);

#ifdef __cplusplus
}
#endif
#endif /* QADC_H */
