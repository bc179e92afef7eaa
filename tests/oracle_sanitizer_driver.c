/* Drives every entry point of the CPU oracle over small seeded inputs (regular and irregular
 * layouts, empty and short lists, more results than codes, empty and invalid inverted lists).
 * Built with -fsanitize=address,undefined by tests/test_oracle_pins.py: any out-of-bounds
 * access, leak, overflow or misaligned access in the oracle ends it with a non-zero status. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_code_size(int m, const int32_t *nbits);
int oracle_table_len(int m, const int32_t *nbits);
void oracle_unpack(int m, const int32_t *nbits, const uint8_t *codes, int64_t n, uint8_t *sub);
void oracle_tables(int d, int m, const int32_t *nbits, const int32_t *dsub, const float *codebooks,
                   const float *z, const float *shift, float *table);
void oracle_adc_float(int m, const int32_t *nbits, const float *table, const uint8_t *codes,
                      int64_t n, float *out);
int64_t oracle_t_eff(int64_t n, int t, int R);
void oracle_quantize(int m, const int32_t *nbits, int acc_bits, const float *table,
                     const uint8_t *codes, int64_t n, int t, int R, uint16_t *qtable,
                     double *out_params);
void oracle_scan_keys(int m, const int32_t *nbits, int acc_bits, const uint16_t *qtable,
                      const uint8_t *codes, int64_t n, uint16_t *keys);
void oracle_topk(int acc_bits, const uint16_t *keys, int64_t n, int R, double dmin, double delta,
                 int32_t *out_ids, uint16_t *out_keys, float *out_dist);
void oracle_search(int d, int m, const int32_t *nbits, const int32_t *dsub, int acc_bits,
                   const float *codebooks, const float *z, const uint8_t *codes, int64_t n, int t,
                   int R, int32_t *out_ids, uint16_t *out_keys, float *out_dist);
void oracle_search_ivf(int d, int m, const int32_t *nbits, const int32_t *dsub, int acc_bits,
                       const float *codebooks, const float *coarse, const int64_t *list_offsets,
                       const uint8_t *list_codes, const int32_t *list_ids, const float *z,
                       const int32_t *probe, int nprobe, int t, int R, int32_t *out_ids,
                       float *out_dist, float *out_dmax);
void oracle_coarse_search(int d, int64_t K, const float *centroids, const float *z, int nprobe,
                          int32_t *out_ids, float *out_scores);
void oracle_encode(int d, int m, const int32_t *nbits, const int32_t *dsub, const float *codebooks,
                   const float *x, const float *shift, int64_t n, uint8_t *codes);

static uint64_t rng = 0x9E3779B97F4A7C15ull;
static float frand(void) {
    rng = rng * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((rng >> 40) & 0xffff) / 65536.0f - 0.5f;
}
static float *fvec(size_t n) {
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = frand();
    return p;
}

static void one_layout(int m, const int32_t *nbits, const int32_t *dsub, int acc_bits) {
    int d = 0;
    size_t cbn = 0;
    for (int j = 0; j < m; ++j) {
        d += dsub[j];
        cbn += ((size_t)1 << nbits[j]) * (size_t)dsub[j];
    }
    const int T = oracle_table_len(m, nbits), cs = oracle_code_size(m, nbits);
    float *cb = fvec(cbn), *z = fvec((size_t)d);
    float *table = (float *)malloc(sizeof(float) * (size_t)T);
    uint16_t *qt = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)T);
    const int64_t ns[] = {0, 1, 37, 1000};
    const int Rs[] = {1, 10, 100};
    for (unsigned a = 0; a < sizeof(ns) / sizeof(ns[0]); ++a) {
        const int64_t n = ns[a];
        float *x = fvec((size_t)n * (size_t)d);
        uint8_t *codes = (uint8_t *)malloc((size_t)(n ? n : 1) * (size_t)cs);
        uint8_t *sub = (uint8_t *)malloc((size_t)(n ? n : 1) * (size_t)m);
        float *fl = (float *)malloc(sizeof(float) * (size_t)(n ? n : 1));
        uint16_t *keys = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)(n ? n : 1));
        oracle_encode(d, m, nbits, dsub, cb, x, NULL, n, codes);
        oracle_unpack(m, nbits, codes, n, sub);
        oracle_tables(d, m, nbits, dsub, cb, z, NULL, table);
        oracle_adc_float(m, nbits, table, codes, n, fl);
        for (unsigned b = 0; b < sizeof(Rs) / sizeof(Rs[0]); ++b) {
            const int R = Rs[b];
            double prm[3];
            int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)R);
            uint16_t *ok = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)R);
            float *od = (float *)malloc(sizeof(float) * (size_t)R);
            oracle_quantize(m, nbits, acc_bits, table, codes, n, 40, R, qt, prm);
            oracle_scan_keys(m, nbits, acc_bits, qt, codes, n, keys);
            oracle_topk(acc_bits, keys, n, R, prm[0], prm[1], ids, ok, od);
            oracle_search(d, m, nbits, dsub, acc_bits, cb, z, codes, n, 40, R, ids, ok, od);
            (void)oracle_t_eff(n, 40, R);
            free(ids); free(ok); free(od);
        }
        /* inverted lists over the same codes: 6 cells, cell 2 empty, probes with an invalid id */
        if (n >= 37) {
            const int K = 6, nprobe = 4, R = 10;
            float *coarse = fvec((size_t)K * (size_t)d);
            int64_t off[7] = {0, n / 8, n / 4, n / 4, n / 2, (3 * n) / 4, n};
            int32_t *lids = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
            for (int64_t p = 0; p < n; ++p) lids[p] = (int32_t)(n - 1 - p);
            const int32_t probe[4] = {2, -1, 5, 0};
            int32_t ids[10], cid[4];
            float od[10], dmax, csc[4];
            oracle_search_ivf(d, m, nbits, dsub, acc_bits, cb, coarse, off, codes, lids, z, probe, nprobe,
                              40, R, ids, od, &dmax);
            oracle_coarse_search(d, K, coarse, z, nprobe, cid, csc);
            float *shift = fvec((size_t)n * (size_t)d);
            oracle_encode(d, m, nbits, dsub, cb, x, shift, n, codes);
            free(coarse); free(lids); free(shift);
        }
        free(x); free(codes); free(sub); free(fl); free(keys);
    }
    free(cb); free(z); free(table); free(qt);
}

int main(void) {
    const int32_t b4[16] = {4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4};
    const int32_t d4[16] = {2, 2, 2, 2, 2, 2, 2, 2, 2, 2, 2, 2, 2, 2, 2, 2};
    const int32_t b3[8] = {6, 5, 5, 6, 5, 5, 4, 4};
    const int32_t d3[8] = {3, 2, 2, 3, 2, 2, 1, 1};
    const int32_t b8[2] = {8, 8};
    const int32_t d8[2] = {3, 4};
    const int32_t b1[3] = {1, 7, 3};
    const int32_t d1[3] = {1, 2, 1};
    one_layout(16, b4, d4, 8);
    one_layout(8, b3, d3, 16);
    one_layout(2, b8, d8, 16);
    one_layout(2, b8, d8, 8);
    one_layout(3, b1, d1, 8);
    puts("oracle sanitizer driver: ok");
    return 0;
}
