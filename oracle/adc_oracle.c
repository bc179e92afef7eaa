/*
 * CPU oracle for the ADC scan over product-quantized codes.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU path must compute;
 * it is called by the tests, by the smoke check and by the benchmark's
 * cpu_baseline leg, never by the product path.  It shares no code with the HIP
 * kernels.  Plain scalar C, one step after the other in the paper's order:
 *
 *   O1  distance tables            Section 2.1.3, eq. (1)
 *   O2  calibration (p_min, d_min, d_max from the first t codes)
 *                                  Section 3.4, second and third paragraphs;
 *                                  t = 400 in Section 4.1
 *   O3  table quantization         Section 3.4, Delta and q formulas
 *   O4  scan with saturating sums  eq. (2); Section 3.4 (saturated arithmetic);
 *                                  Section 3.5
 *   O5  top-R and unquantization   Section 3.5 (candidates kept when smaller);
 *                                  Section 3.4, d = (sum q) Delta + d_min
 *   O6  inverted-list search       Section 2.1.1 (residuals), Section 2.1.3
 *                                  (one table set per probed cell)
 *   O6b the same with a bound that tightens from list to list (optional mode)
 *                                  Sections 3.4, 3.5
 *   O7  coarse-quantizer search    Section 2.1.1 (the cells a query is routed to)
 *   O8  encoding and packing       Sections 2.1.2, 2.1.1, 3.3
 *
 * Precision: the paper stores tables as 32-bit floats (Section 3.4, first
 * paragraph), so table entries and float ADC sums are fp32, evaluated in a
 * fixed order with separate subtract / multiply / add (build with
 * -ffp-contract=off).  The few scalar operations of the distance quantizer
 * are fp64.
 *
 * Readings where the paper is silent (each listed in the design notes):
 *   - q is rounded down (floor), then clamped to q_max;
 *   - t_eff = min(n, max(t, 4R));
 *   - all n codes, the calibration prefix included, are scored with the
 *     quantized tables;
 *   - q_max is an ordinary (largest) key, so min(R, n) results always return;
 *   - Delta <= 0 or not finite: every q is 0 and Delta is reported as 0;
 *   - ties are broken by lowest id;
 *   - IVF: one d_max per query from the first t_eff probed codes, per-list
 *     p_min / d_min / Delta, lists with d_min >= d_max skipped (Section 3.4:
 *     later candidates have to be closer than d_max), candidates from
 *     different lists compared on the unquantized float.
 *
 * Sub-code extraction: a code is a little-endian bit stream; sub-code j sits in
 * bits [off_j, off_j + nbits[j]), off_j = sum_{i<j} nbits[i], bit 0 being the
 * least significant bit of byte 0 (Section 3.3, packing paragraph).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int d, m;
    const int32_t *nbits; /* [m] */
    const int32_t *dsub;  /* [m] */
    int acc_bits;         /* 8 or 16 */
} layout_t;

static int code_bits(const layout_t *L) {
    int b = 0;
    for (int j = 0; j < L->m; ++j) b += L->nbits[j];
    return b;
}
static int code_size(const layout_t *L) { return (code_bits(L) + 7) / 8; }
static int table_len(const layout_t *L) {
    int t = 0;
    for (int j = 0; j < L->m; ++j) t += 1 << L->nbits[j];
    return t;
}
static uint32_t q_max_of(const layout_t *L) { return (1u << L->acc_bits) - 1u; }

/* sub-code j of one packed code, read bit by bit */
static unsigned subcode(const uint8_t *code, int off, int b) {
    unsigned v = 0;
    for (int k = 0; k < b; ++k) {
        int pos = off + k;
        unsigned bit = (code[pos >> 3] >> (pos & 7)) & 1u;
        v |= bit << k;
    }
    return v;
}

int oracle_code_size(int m, const int32_t *nbits) {
    layout_t L = {0, m, nbits, NULL, 8};
    return code_size(&L);
}
int oracle_table_len(int m, const int32_t *nbits) {
    layout_t L = {0, m, nbits, NULL, 8};
    return table_len(&L);
}

/* [n,cs] packed codes -> [n,m] sub-codes */
void oracle_unpack(int m, const int32_t *nbits, const uint8_t *codes, int64_t n, uint8_t *sub) {
    layout_t L = {0, m, nbits, NULL, 8};
    int cs = code_size(&L);
    for (int64_t p = 0; p < n; ++p) {
        int off = 0;
        for (int j = 0; j < m; ++j) {
            sub[p * m + j] = (uint8_t)subcode(codes + p * cs, off, nbits[j]);
            off += nbits[j];
        }
    }
}

/* O1: D^j[i] = || z'^j - C^j[i] ||^2, z' = z - shift (shift may be NULL). eq. (1) */
void oracle_tables(int d, int m, const int32_t *nbits, const int32_t *dsub, const float *codebooks,
                   const float *z, const float *shift, float *table) {
    float *zr = (float *)malloc(sizeof(float) * (size_t)(d > 0 ? d : 1));
    for (int i = 0; i < d; ++i) zr[i] = shift ? (z[i] - shift[i]) : z[i];
    int o = 0;
    size_t cb = 0, t = 0;
    for (int j = 0; j < m; ++j) {
        int k = 1 << nbits[j];
        for (int i = 0; i < k; ++i) {
            float acc = 0.0f;
            for (int l = 0; l < dsub[j]; ++l) {
                float diff = zr[o + l] - codebooks[cb + (size_t)i * dsub[j] + l];
                float sq = diff * diff;
                acc = acc + sq;
            }
            table[t + i] = acc;
        }
        o += dsub[j];
        cb += (size_t)k * dsub[j];
        t += k;
    }
    free(zr);
}

/* float ADC of one code, eq. (2): fp32, j ascending */
static float adc_float(const layout_t *L, const float *table, const uint8_t *code) {
    float s = 0.0f;
    int off = 0, t = 0;
    for (int j = 0; j < L->m; ++j) {
        s = s + table[t + subcode(code, off, L->nbits[j])];
        off += L->nbits[j];
        t += 1 << L->nbits[j];
    }
    return s;
}

void oracle_adc_float(int m, const int32_t *nbits, const float *table, const uint8_t *codes,
                      int64_t n, float *out) {
    layout_t L = {0, m, nbits, NULL, 8};
    int cs = code_size(&L);
    for (int64_t p = 0; p < n; ++p) out[p] = adc_float(&L, table, codes + p * cs);
}

int64_t oracle_t_eff(int64_t n, int t, int R) {
    int64_t want = t > 4 * (int64_t)R ? t : 4 * (int64_t)R;
    return n < want ? n : want;
}

static int cmp_float(const void *a, const void *b) {
    float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

/* k-th smallest (1-based) of s[0..cnt) by a full sort of a copy */
static float kth_smallest(const float *s, int64_t cnt, int64_t k) {
    float *tmp = (float *)malloc(sizeof(float) * (size_t)cnt);
    memcpy(tmp, s, sizeof(float) * (size_t)cnt);
    qsort(tmp, (size_t)cnt, sizeof(float), cmp_float);
    float v = tmp[k - 1];
    free(tmp);
    return v;
}

/* p_min(j) and d_min = sum_j p_min(j) in fp64, j ascending (Section 3.4) */
static double table_minima(const layout_t *L, const float *table, float *pmin) {
    double dmin = 0.0;
    int t = 0;
    for (int j = 0; j < L->m; ++j) {
        int k = 1 << L->nbits[j];
        float mn = table[t];
        for (int i = 1; i < k; ++i)
            if (table[t + i] < mn) mn = table[t + i];
        pmin[j] = mn;
        dmin = dmin + (double)mn;
        t += k;
    }
    return dmin;
}

/* O3 given (table, pmin, d_min, d_max): Delta and the quantized table (stored as u16) */
static double quantize_table(const layout_t *L, const float *table, const float *pmin, double dmin,
                             float dmax, uint16_t *qtable) {
    uint32_t qmax = q_max_of(L);
    double delta = ((double)dmax - dmin) / (double)qmax;
    int ok = (delta > 0.0) && isfinite(delta);
    int t = 0;
    for (int j = 0; j < L->m; ++j) {
        int k = 1 << L->nbits[j];
        for (int i = 0; i < k; ++i) {
            uint32_t q = 0;
            if (ok) {
                double x = floor(((double)table[t + i] - (double)pmin[j]) / delta);
                q = (x >= (double)qmax) ? qmax : (uint32_t)x;
            }
            qtable[t + i] = (uint16_t)q;
        }
        t += k;
    }
    return ok ? delta : 0.0;
}

/*
 * O2 + O3 for one query over one list of codes.
 * out_params = { d_min, delta, d_max } as doubles (d_max exactly representable as float).
 */
void oracle_quantize(int m, const int32_t *nbits, int acc_bits, const float *table,
                     const uint8_t *codes, int64_t n, int t, int R, uint16_t *qtable,
                     double *out_params) {
    layout_t L = {0, m, nbits, NULL, acc_bits};
    int cs = code_size(&L);
    float *pmin = (float *)malloc(sizeof(float) * (size_t)m);
    double dmin = table_minima(&L, table, pmin);
    int64_t te = oracle_t_eff(n, t, R);
    float dmax = INFINITY; /* no code to calibrate on: Delta is not finite, every q is 0 */
    if (te > 0) {
        float *s = (float *)malloc(sizeof(float) * (size_t)te);
        for (int64_t p = 0; p < te; ++p) s[p] = adc_float(&L, table, codes + p * cs);
        dmax = kth_smallest(s, te, R < te ? R : te);
        free(s);
    }
    double delta = quantize_table(&L, table, pmin, dmin, dmax, qtable);
    out_params[0] = dmin;
    out_params[1] = delta;
    out_params[2] = (double)dmax;
    free(pmin);
}

/* saturating unsigned add at the accumulator width (Section 3.4, last paragraph) */
static uint32_t sat_add(uint32_t a, uint32_t b, uint32_t qmax) {
    uint32_t s = a + b;
    return s > qmax ? qmax : s;
}

static uint32_t adc_key(const layout_t *L, const uint16_t *qtable, const uint8_t *code) {
    uint32_t qmax = q_max_of(L), acc = 0;
    int off = 0, t = 0;
    for (int j = 0; j < L->m; ++j) {
        acc = sat_add(acc, qtable[t + subcode(code, off, L->nbits[j])], qmax);
        off += L->nbits[j];
        t += 1 << L->nbits[j];
    }
    return acc;
}

/* O4: key of every code */
void oracle_scan_keys(int m, const int32_t *nbits, int acc_bits, const uint16_t *qtable,
                      const uint8_t *codes, int64_t n, uint16_t *keys) {
    layout_t L = {0, m, nbits, NULL, acc_bits};
    int cs = code_size(&L);
    for (int64_t p = 0; p < n; ++p) keys[p] = (uint16_t)adc_key(&L, qtable, codes + p * cs);
}

typedef struct {
    uint32_t key;
    int64_t id;
} kid_t;
static int cmp_kid(const void *a, const void *b) {
    const kid_t *x = (const kid_t *)a, *y = (const kid_t *)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

/* O5: full sort by (key, id); first min(R,n); pad with id -1, key q_max, dist +inf */
void oracle_topk(int acc_bits, const uint16_t *keys, int64_t n, int R, double dmin, double delta,
                 int32_t *out_ids, uint16_t *out_keys, float *out_dist) {
    uint32_t qmax = (1u << acc_bits) - 1u;
    kid_t *a = (kid_t *)malloc(sizeof(kid_t) * (size_t)(n > 0 ? n : 1));
    for (int64_t p = 0; p < n; ++p) {
        a[p].key = keys[p];
        a[p].id = p;
    }
    qsort(a, (size_t)n, sizeof(kid_t), cmp_kid);
    for (int r = 0; r < R; ++r) {
        if (r < n) {
            out_ids[r] = (int32_t)a[r].id;
            out_keys[r] = (uint16_t)a[r].key;
            out_dist[r] = fmaf((float)a[r].key, (float)delta, (float)dmin);
        } else {
            out_ids[r] = -1;
            out_keys[r] = (uint16_t)qmax;
            out_dist[r] = INFINITY;
        }
    }
    free(a);
}

/* O1..O5 for one query: exhaustive search over one list */
void oracle_search(int d, int m, const int32_t *nbits, const int32_t *dsub, int acc_bits,
                   const float *codebooks, const float *z, const uint8_t *codes, int64_t n, int t,
                   int R, int32_t *out_ids, uint16_t *out_keys, float *out_dist) {
    layout_t L = {d, m, nbits, dsub, acc_bits};
    int T = table_len(&L);
    float *table = (float *)malloc(sizeof(float) * (size_t)T);
    uint16_t *qtable = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)T);
    uint16_t *keys = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)(n > 0 ? n : 1));
    double prm[3];
    oracle_tables(d, m, nbits, dsub, codebooks, z, NULL, table);
    oracle_quantize(m, nbits, acc_bits, table, codes, n, t, R, qtable, prm);
    oracle_scan_keys(m, nbits, acc_bits, qtable, codes, n, keys);
    oracle_topk(acc_bits, keys, n, R, prm[0], prm[1], out_ids, out_keys, out_dist);
    free(table);
    free(qtable);
    free(keys);
}

typedef struct {
    float dist;
    int32_t id;
} fid_t;
static int cmp_fid(const void *a, const void *b) {
    const fid_t *x = (const fid_t *)a, *y = (const fid_t *)b;
    if (x->dist != y->dist) return x->dist < y->dist ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

/*
 * O6 for one query.  probe[] lists the cells to visit, nearest first; negative
 * entries are ignored.  out_dmax receives the calibration bound (+inf when the
 * probed lists are empty).
 */
void oracle_search_ivf(int d, int m, const int32_t *nbits, const int32_t *dsub, int acc_bits,
                       const float *codebooks, const float *coarse, const int64_t *list_offsets,
                       const uint8_t *list_codes, const int32_t *list_ids, const float *z,
                       const int32_t *probe, int nprobe, int t, int R, int32_t *out_ids,
                       float *out_dist, float *out_dmax) {
    layout_t L = {d, m, nbits, dsub, acc_bits};
    int T = table_len(&L), cs = code_size(&L);
    float *table = (float *)malloc(sizeof(float) * (size_t)T);
    uint16_t *qtable = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)T);
    float *pmin = (float *)malloc(sizeof(float) * (size_t)m);

    int64_t nprobed = 0;
    for (int a = 0; a < nprobe; ++a)
        if (probe[a] >= 0) nprobed += list_offsets[probe[a] + 1] - list_offsets[probe[a]];
    int64_t te = oracle_t_eff(nprobed, t, R);

    /* calibration: float ADC of the first t_eff probed codes, each with its own list's tables */
    float dmax = INFINITY;
    if (te > 0) {
        float *s = (float *)malloc(sizeof(float) * (size_t)te);
        int64_t seen = 0;
        for (int a = 0; a < nprobe && seen < te; ++a) {
            if (probe[a] < 0) continue;
            int64_t lo = list_offsets[probe[a]], hi = list_offsets[probe[a] + 1];
            if (hi == lo) continue;
            oracle_tables(d, m, nbits, dsub, codebooks, z, coarse + (size_t)probe[a] * d, table);
            for (int64_t p = lo; p < hi && seen < te; ++p)
                s[seen++] = adc_float(&L, table, list_codes + p * cs);
        }
        dmax = kth_smallest(s, te, R < te ? R : te);
        free(s);
    }
    *out_dmax = dmax;

    fid_t *cand = (fid_t *)malloc(sizeof(fid_t) * (size_t)(nprobed > 0 ? nprobed : 1));
    int64_t nc = 0;
    for (int a = 0; a < nprobe; ++a) {
        if (probe[a] < 0) continue;
        int64_t lo = list_offsets[probe[a]], hi = list_offsets[probe[a] + 1];
        if (hi == lo) continue;
        oracle_tables(d, m, nbits, dsub, codebooks, z, coarse + (size_t)probe[a] * d, table);
        double dmin = table_minima(&L, table, pmin);
        /* Section 3.4: every candidate after calibration has to be closer than d_max, and no
         * code of this list can be closer than the list's d_min */
        if (dmin >= (double)dmax) continue;
        double delta = quantize_table(&L, table, pmin, dmin, dmax, qtable);
        for (int64_t p = lo; p < hi; ++p) {
            uint32_t key = adc_key(&L, qtable, list_codes + p * cs);
            cand[nc].dist = fmaf((float)key, (float)delta, (float)dmin);
            cand[nc].id = list_ids[p];
            ++nc;
        }
    }
    qsort(cand, (size_t)nc, sizeof(fid_t), cmp_fid);
    for (int r = 0; r < R; ++r) {
        if (r < nc) {
            out_ids[r] = cand[r].id;
            out_dist[r] = cand[r].dist;
        } else {
            out_ids[r] = -1;
            out_dist[r] = INFINITY;
        }
    }
    free(cand);
    free(table);
    free(qtable);
    free(pmin);
}

/*
 * O6b: the inverted-list search with a bound that tightens from list to list (optional mode).
 * Section 3.5: a scanned vector is compared with the worst of the R candidates held and kept
 * when it is closer; Section 3.4: the distance of the R-th candidate is the largest distance
 * the quantizer has to represent.  Read together for several lists visited one after the
 * other: the lists are scanned in probe order, and list l is quantized against
 *     cur_l = min(d_max, R-th smallest unquantized distance among all codes of the unskipped
 *                        lists before l)           (the second term only once R codes were seen)
 * with d_max the calibration bound of O6.  A list with d_min >= cur_l is skipped.  A code of
 * the other lists whose sum saturates (key = q_max, the value Section 3.4 reserves for a
 * distance that is too large) is not a candidate: unlike in O6, where the bound is fixed and
 * generous, a saturated code here is one that is not closer than the worst candidate held.
 * Every other code gets dist = fmaf(key, (float)Delta_l, (float)d_min_l) with the list's own
 * Delta_l = (cur_l - d_min_l)/q_max; the R smallest (dist, stored id) are returned, fewer (the
 * rest padded) if fewer codes stayed below their bounds.  cur_l never grows, so later lists
 * are quantized more finely than in O6; the result depends on the probe order by construction.
 * out_bounds[a] receives cur for probe a (the value its list was, or would have been,
 * quantized against); may be NULL.
 */
void oracle_search_ivf_tightening(int d, int m, const int32_t *nbits, const int32_t *dsub, int acc_bits,
                                  const float *codebooks, const float *coarse,
                                  const int64_t *list_offsets, const uint8_t *list_codes,
                                  const int32_t *list_ids, const float *z, const int32_t *probe,
                                  int nprobe, int t, int R, int32_t *out_ids, float *out_dist,
                                  float *out_dmax, float *out_bounds) {
    layout_t L = {d, m, nbits, dsub, acc_bits};
    int T = table_len(&L), cs = code_size(&L);
    float *table = (float *)malloc(sizeof(float) * (size_t)T);
    uint16_t *qtable = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)T);
    float *pmin = (float *)malloc(sizeof(float) * (size_t)m);

    int64_t nprobed = 0;
    for (int a = 0; a < nprobe; ++a)
        if (probe[a] >= 0) nprobed += list_offsets[probe[a] + 1] - list_offsets[probe[a]];
    int64_t te = oracle_t_eff(nprobed, t, R);

    /* calibration exactly as in O6 */
    float dmax = INFINITY;
    if (te > 0) {
        float *s = (float *)malloc(sizeof(float) * (size_t)te);
        int64_t seen = 0;
        for (int a = 0; a < nprobe && seen < te; ++a) {
            if (probe[a] < 0) continue;
            int64_t lo = list_offsets[probe[a]], hi = list_offsets[probe[a] + 1];
            if (hi == lo) continue;
            oracle_tables(d, m, nbits, dsub, codebooks, z, coarse + (size_t)probe[a] * d, table);
            for (int64_t p = lo; p < hi && seen < te; ++p)
                s[seen++] = adc_float(&L, table, list_codes + p * cs);
        }
        dmax = kth_smallest(s, te, R < te ? R : te);
        free(s);
    }
    *out_dmax = dmax;

    fid_t *cand = (fid_t *)malloc(sizeof(fid_t) * (size_t)(nprobed > 0 ? nprobed : 1));
    float *dists = (float *)malloc(sizeof(float) * (size_t)(nprobed > 0 ? nprobed : 1));
    int64_t nc = 0;
    float cur = dmax;
    for (int a = 0; a < nprobe; ++a) {
        if (out_bounds) out_bounds[a] = cur;
        if (probe[a] < 0) continue;
        int64_t lo = list_offsets[probe[a]], hi = list_offsets[probe[a] + 1];
        if (hi == lo) continue;
        oracle_tables(d, m, nbits, dsub, codebooks, z, coarse + (size_t)probe[a] * d, table);
        double dmin = table_minima(&L, table, pmin);
        if (dmin >= (double)cur) continue; /* nothing in this list is closer than the bound */
        double delta = quantize_table(&L, table, pmin, dmin, cur, qtable);
        for (int64_t p = lo; p < hi; ++p) {
            uint32_t key = adc_key(&L, qtable, list_codes + p * cs);
            if (key == q_max_of(&L)) continue; /* saturated: not closer than the bound */
            cand[nc].dist = fmaf((float)key, (float)delta, (float)dmin);
            cand[nc].id = list_ids[p];
            dists[nc] = cand[nc].dist;
            ++nc;
        }
        if (nc >= R) { /* the worst of the R best seen so far */
            float worst = kth_smallest(dists, nc, R);
            if (worst < cur) cur = worst;
        }
    }
    qsort(cand, (size_t)nc, sizeof(fid_t), cmp_fid);
    for (int r = 0; r < R; ++r) {
        if (r < nc) {
            out_ids[r] = cand[r].id;
            out_dist[r] = cand[r].dist;
        } else {
            out_ids[r] = -1;
            out_dist[r] = INFINITY;
        }
    }
    free(cand);
    free(dists);
    free(table);
    free(qtable);
    free(pmin);
}

/*
 * O7: coarse-quantizer search (Section 2.1.1: a query is routed to the cells whose centroids
 * are nearest).  Cells are ranked by  score(c) = ||c||^2 - 2 z.c , the squared distance minus
 * ||z||^2, which is the same for every cell.  fp32 throughout:
 *   z.c     acc = fma(z[l], c[l], acc), l ascending from 0
 *   ||c||^2 acc = fma(c[l], c[l], acc), l ascending from 0
 *   score   = fma(-2, z.c, ||c||^2)
 * The nprobe cells with the smallest (score, id) are returned in that order; when nprobe > K
 * the rest is padded with id -1 and score +inf.
 */
void oracle_coarse_search(int d, int64_t K, const float *centroids, const float *z, int nprobe,
                          int32_t *out_ids, float *out_scores) {
    fid_t *cand = (fid_t *)malloc(sizeof(fid_t) * (size_t)(K > 0 ? K : 1));
    for (int64_t c = 0; c < K; ++c) {
        const float *cen = centroids + (size_t)c * d;
        float dot = 0.0f, nrm = 0.0f;
        for (int l = 0; l < d; ++l) dot = fmaf(z[l], cen[l], dot);
        for (int l = 0; l < d; ++l) nrm = fmaf(cen[l], cen[l], nrm);
        cand[c].dist = fmaf(-2.0f, dot, nrm);
        cand[c].id = (int32_t)c;
    }
    qsort(cand, (size_t)K, sizeof(fid_t), cmp_fid);
    for (int r = 0; r < nprobe; ++r) {
        if (r < K) {
            out_ids[r] = cand[r].id;
            out_scores[r] = cand[r].dist;
        } else {
            out_ids[r] = -1;
            out_scores[r] = INFINITY;
        }
    }
    free(cand);
}

/*
 * O8: encoding (Section 2.1.2: a vector is encoded by the index of the nearest centroid in each
 * sub-space; Section 2.1.1: with an inverted index the residual x - centroid is what is
 * encoded; Section 3.3, packing paragraph: the sub-codes form a little-endian bit stream).
 * For vector x (minus shift, if given) the distances to the centroids of sub-quantizer j are
 * exactly the table entries of eq. (1) for z = x; sub-code j is the index of the smallest, the
 * lowest index among equals.
 *   x      [n][d]            shift  [n][d] or NULL
 *   codes  [n][code_size], every byte written (unused high bits zero)
 */
void oracle_encode(int d, int m, const int32_t *nbits, const int32_t *dsub, const float *codebooks,
                   const float *x, const float *shift, int64_t n, uint8_t *codes) {
    layout_t L = {d, m, nbits, dsub, 8};
    int T = table_len(&L), cs = code_size(&L);
    float *table = (float *)malloc(sizeof(float) * (size_t)T);
    for (int64_t v = 0; v < n; ++v) {
        oracle_tables(d, m, nbits, dsub, codebooks, x + v * d, shift ? shift + v * d : NULL, table);
        uint8_t *code = codes + v * cs;
        memset(code, 0, (size_t)cs);
        int off = 0, t = 0;
        for (int j = 0; j < m; ++j) {
            int k = 1 << nbits[j], best = 0;
            for (int i = 1; i < k; ++i)
                if (table[t + i] < table[t + best]) best = i;
            for (int b = 0; b < nbits[j]; ++b) {
                int pos = off + b;
                code[pos >> 3] |= (uint8_t)(((best >> b) & 1) << (pos & 7));
            }
            off += nbits[j];
            t += k;
        }
    }
    free(table);
}
