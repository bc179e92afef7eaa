// pq_quantize_tables: the query-time distance quantizer of Section 3.4.
#include <math.h>
#include <stdlib.h>


#include "scan_device.h"

// P blocks per query (grid = nq * P, block q*P + p).  Every block of a query computes
//   0. (fused form only) the float table from the query, eq. (1)
//   1. p_min(j), d_min = sum_j p_min(j) (fp64, ascending j)
//   2. float ADC (eq. (2), fp32, ascending j) of the first t_eff codes; d_max is
//      the k-th smallest of them, k = min(R, t_eff)
//   3. delta = (d_max - d_min)/q_max; q = min(q_max, floor((p - p_min)/delta))
// (a few thousand operations, cheaper to repeat than to hand over between kernels) and then
// its share of
//   4. key_bound: an upper bound of the k-th smallest quantized key among the first `pilot`
//      codes (pilot >= t_eff), from a 256-bin histogram of the keys (of their high bytes for
//      16-bit keys).  It bounds the R-th best key of the whole list from above and lets the
//      scan drop almost every code with one compare.
// Block p counts the codes [p*slice, (p+1)*slice) of the pilot.  With P == 1 the block selects
// the bound itself and stores it in the query's parameters.  With P > 1 no block waits for
// another: each leaves a record of 64 cumulative counts (how many of its codes have a key in
// coarse bin t or below, a coarse bin being four bins of the 256-bin histogram) in `bound_rec`,
// and the scan kernel adds the P records up (scan_bound_from_records); the parameters then
// carry q_max as the bound.  Block 0 of a query stores the tables and the parameters.
// `queries` non-null: tables are computed here (and stored to tables_out if
// that is non-null); otherwise they are read from tables_in.
#ifndef QUANT_THREADS
#define QUANT_THREADS 256
#endif
// The few layout numbers the kernel needs before anything else, as kernel arguments (reading
// them through the layout pointer would be a memory round trip ahead of every other load).
struct QuantShape {
    int T, m, cs, qmax, d;
    int ubits, uds;  // bits and dimensions of every sub-quantizer if they are all alike, else 0
};
// NIB8 pilot codes a thread holds in registers per batch
#define PILOT_PER_THREAD 8
template <int KIND, typename QT>
__global__ void __launch_bounds__(QUANT_THREADS)
k_quantize(const DevLayout *__restrict__ L, const QuantShape shape, const EntryDesc *__restrict__ edesc,
           const float *__restrict__ cb,
           const float *__restrict__ queries, const float *__restrict__ tables_in,
           float *__restrict__ tables_out, const uint8_t *__restrict__ codes, int t_eff, int k,
           int pilot, int slice, int P, void *__restrict__ qtables,
           pq_qparams_t *__restrict__ qparams, char *__restrict__ gtab_out, size_t gtab_stride,
           char *__restrict__ hdr_out, uint16_t *__restrict__ bound_rec) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int T = shape.T, m = shape.m, cs = shape.cs, qmax = shape.qmax, d = shape.d;
    float *tab = (float *)smem;
    uint32_t *ord = (uint32_t *)(tab + T);                    // max(t_eff, d) words
    const int nord = (t_eff > d ? t_eff : d) > 0 ? (t_eff > d ? t_eff : d) : 1;
    float *pmin = (float *)(ord + nord);
    uint16_t *qt = (uint16_t *)(pmin + PQ_MAX_M);
    uint8_t *esub = (uint8_t *)(qt + T);
    QT *gtab = (QT *)(smem + (((size_t)T * 4 + (size_t)nord * 4 + PQ_MAX_M * 4 + (size_t)T * 3 + 15) &
                              ~(size_t)15));
    __shared__ __align__(16) uint32_t hist[256];
    __shared__ uint32_t sel[8];
    __shared__ uint32_t kmem[QADC_KTH_MEM];
    __shared__ double s_dmin, s_delta;
    __shared__ float s_dmax;
    __shared__ uint32_t sdesc[PQ_MAX_M];  // table offset | bit offset << 12 | bits << 24 of each sub-quantizer
    __shared__ uint32_t pmin_ord[PQ_MAX_M];  // table minima as ordered words (qadc_f2ord), by LDS atomic min
    if ((int)threadIdx.x < m) {  // (read after the barriers of the table set-up)
        sdesc[threadIdx.x] = (uint32_t)L->toff[threadIdx.x] | ((uint32_t)L->bitoff[threadIdx.x] << 12) |
                             ((uint32_t)L->nbits[threadIdx.x] << 24);
        pmin_ord[threadIdx.x] = 0xffffffffu;
    }

    const size_t q = blockIdx.x / (unsigned)P;
    const int p = (int)(blockIdx.x % (unsigned)P);
    const bool first = p == 0;
    const int lo = (int64_t)p * slice < pilot ? p * slice : pilot;
    const int hi = (int64_t)lo + slice < pilot ? lo + slice : pilot;
    constexpr int PPT = KIND == SCAN_NIB8 ? PILOT_PER_THREAD : 8;  // pilot codes per thread and batch
    const int step = PPT * (int)blockDim.x;

    // The first batch of this block's pilot codes is requested now and used at the very end.
    uint2 pc[PPT];
    if (KIND == SCAN_NIB8 && hi > lo) {
#pragma unroll
        for (int u = 0; u < PPT; ++u) {
            int id = lo + u * (int)blockDim.x + (int)threadIdx.x;
            id = id < hi ? id : hi - 1;
            pc[u] = *(const uint2 *)(codes + (size_t)id * 8);
        }
    }

    // The calibration code of this thread (at most one per thread in the common case) and the
    // descriptor of its table entry are requested now as well: they do not depend on anything.
    const bool cal_pre = t_eff <= 2 * (int)blockDim.x && cs <= 16;  // up to two per thread
    uint32_t cw[2][4] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
    if (cal_pre) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int pp = r * (int)blockDim.x + (int)threadIdx.x;
            if (pp < t_eff) qadc_load_code16(codes + (size_t)pp * cs, cs, cw[r]);
        }
    }
    EntryDesc ed0 = {0, 0, 0, 0};
    if ((int)threadIdx.x < T) ed0 = edesc[threadIdx.x];

    if (queries && shape.ubits > 0 && shape.uds > 0 && T > (int)blockDim.x) {
        // long tables of sub-quantizers that are all alike (m x 8 bits): entry e is centroid
        // e mod 2^bits of sub-quantizer e >> bits at codebook offset e * ds, so nothing has to
        // be looked up before the codebook values are requested, and the loop over the
        // dimensions has the same length in every lane
        float *zs = (float *)ord;
        for (int i = threadIdx.x; i < d; i += blockDim.x) zs[i] = queries[q * d + i];
        __syncthreads();
        const int ub = shape.ubits, ds = shape.uds;
        for (int e = threadIdx.x; e < T; e += blockDim.x) {
            const int j = e >> ub;
            const float *c = cb + (size_t)e * ds;
            const float *z = zs + j * ds;
            float acc = 0.0f;
            for (int l = 0; l < ds; ++l) {
                float diff = __fsub_rn(z[l], c[l]);
                acc = __fadd_rn(acc, __fmul_rn(diff, diff));
            }
            tab[e] = acc;
            esub[e] = (uint8_t)j;
            atomicMin(&pmin_ord[j], qadc_f2ord(acc));
            if (tables_out && first) tables_out[q * T + e] = acc;
        }
        __syncthreads();
    } else if (queries) {
        float *zs = (float *)ord;  // the query lives where the ADC sums go later
        for (int i = threadIdx.x; i < d; i += blockDim.x) zs[i] = queries[q * d + i];
        for (int e = threadIdx.x; e < T; e += blockDim.x)
            esub[e] = (uint8_t)(e == (int)threadIdx.x ? ed0.j : edesc[e].j);
        // the first eight codebook values of this thread's own entry: requested before the
        // barrier, so that they travel while the query settles in LDS
        float c0[8];
#pragma unroll
        for (int l = 0; l < 8; ++l) c0[l] = ((int)threadIdx.x < T && l < ed0.ds) ? cb[ed0.cb_off + l] : 0.0f;
        __syncthreads();
        for (int e = threadIdx.x; e < T; e += blockDim.x) {
            const bool own = e == (int)threadIdx.x;
            const EntryDesc ed = own ? ed0 : edesc[e];
            const int ds = ed.ds;
            const float *c = cb + ed.cb_off;
            const float *z = zs + ed.dim_off;
            float acc = 0.0f;
            if (own) {
#pragma unroll
                for (int l = 0; l < 8; ++l)
                    if (l < ds) {
                        float diff = __fsub_rn(z[l], c0[l]);
                        acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                    }
            }
            for (int l = own ? 8 : 0; l < ds; ++l) {
                float diff = __fsub_rn(z[l], c[l]);
                acc = __fadd_rn(acc, __fmul_rn(diff, diff));
            }
            tab[e] = acc;
            atomicMin(&pmin_ord[ed.j], qadc_f2ord(acc));
            if (tables_out && first) tables_out[q * T + e] = acc;
        }
        __syncthreads();
    } else {
        __syncthreads();  // pmin_ord is set up
        for (int e = threadIdx.x; e < T; e += blockDim.x) {
            const float v = tables_in[q * T + e];
            const int j = e == (int)threadIdx.x ? ed0.j : edesc[e].j;
            tab[e] = v;
            esub[e] = (uint8_t)j;
            atomicMin(&pmin_ord[j], qadc_f2ord(v));
        }
        __syncthreads();
    }
    if ((int)threadIdx.x < m) pmin[threadIdx.x] = qadc_ord2f(pmin_ord[threadIdx.x]);
    // float ADC of the calibration codes
    for (int pp = threadIdx.x, r = 0; pp < t_eff; pp += blockDim.x, ++r) {
        const uint8_t *code = codes + (size_t)pp * cs;
        float s = 0.0f;
        const uint32_t *cwr = cw[r & 1];  // (r < 2 whenever cal_pre)
        if (KIND == SCAN_NIB8) {  // sub-code j is nibble j of the 8-byte code
            const uint2 v = cal_pre ? make_uint2(cwr[0], cwr[1]) : *(const uint2 *)code;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                s = __fadd_rn(s, tab[16 * j + (((j < 8 ? v.x : v.y) >> (4 * (j & 7))) & 15u)]);
        } else if (KIND == SCAN_NIB16) {  // ... of the 16-byte code
            const uint4 v = cal_pre ? make_uint4(cwr[0], cwr[1], cwr[2], cwr[3]) : *(const uint4 *)code;
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 32; ++j)
                s = __fadd_rn(s, tab[16 * j + ((w[j >> 3] >> (4 * (j & 7))) & 15u)]);
        } else if (cs <= 16) {  // the code in registers, the sub-quantizers' fields from LDS
            uint32_t w[4];
            if (cal_pre) {
                w[0] = cwr[0]; w[1] = cwr[1]; w[2] = cwr[2]; w[3] = cwr[3];
            } else {
                qadc_load_code16(code, cs, w);
            }
            for (int j = 0; j < m; ++j) {
                const uint32_t ds = sdesc[j];
                s = __fadd_rn(s, tab[(ds & 0xfffu) + qadc_extract_sub16(w, (ds >> 12) & 0xfffu, ds >> 24)]);
            }
        } else {
            for (int j = 0; j < m; ++j)
                s = __fadd_rn(s, tab[L->toff[j] + qadc_extract_sub(code, L->bitoff[j], L->nbits[j])]);
        }
        ord[pp] = qadc_f2ord(s);
    }
    __syncthreads();
    if (threadIdx.x < QADC_WAVE) {  // d_min = sum of the minima in fp64, ascending j (m <= 64: one per lane)
        const double mine = (int)threadIdx.x < m ? (double)pmin[threadIdx.x] : 0.0;
        const unsigned long long bits = (unsigned long long)__double_as_longlong(mine);
        double dm = 0.0;
        for (int j = 0; j < m; ++j) {  // (lane reads: no memory involved)
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bits, j);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(bits >> 32), j);
            dm = dm + __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
        }
        if (threadIdx.x == 0) s_dmin = dm;
    }
    float dmax = INFINITY;
    if (t_eff > 0) dmax = qadc_ord2f(qadc_block_kth_f32(ord, t_eff, k, hist, sel, kmem));
    __syncthreads();
    if (threadIdx.x == 0) {
        double delta = ((double)dmax - s_dmin) / (double)qmax;
        bool ok = (delta > 0.0) && isfinite(delta);
        s_delta = ok ? delta : 0.0;
        s_dmax = dmax;
    }
    __syncthreads();
    const double delta = s_delta;
    for (int e = threadIdx.x; e < T; e += blockDim.x) {
        const int j = esub[e];
        uint32_t qv = 0;
        if (delta > 0.0) {
            double x = floor(((double)tab[e] - (double)pmin[j]) / delta);
            qv = (x >= (double)qmax) ? (uint32_t)qmax : (uint32_t)x;
        }
        qt[e] = (uint16_t)qv;
        if (first) {
            if (sizeof(QT) == 1)
                ((uint8_t *)qtables)[q * T + e] = (uint8_t)qv;
            else
                ((uint16_t *)qtables)[q * T + e] = (uint16_t)qv;
        }
    }
    __syncthreads();
    uint32_t bound = (uint32_t)qmax;
    if (pilot > 0 || gtab_out) {
        build_gtab<KIND, QT>(L, qt, gtab);
        if (gtab_out && first) {  // hand the prepared group tables to the scan kernel
            QT *dst = (QT *)(gtab_out + q * gtab_stride);
            for (int e = threadIdx.x; e < L->gtab_len; e += blockDim.x) dst[e] = gtab[e];
        }
    }
    if (hdr_out && first) scan_hdr_clear((ScanHdr *)(hdr_out + q * gtab_stride));  // empty candidate lists
    if (pilot > 0) {
        const int shift = sizeof(QT) == 1 ? 0 : 8;
        for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
        __syncthreads();
        // count one key (0xffffffff = none); the top bin collects every saturated key and
        // is counted once per wave
        auto count_key = [&](uint32_t key) {
            const uint32_t bin = key == 0xffffffffu ? 0xffffffffu : key >> shift;
            const uint64_t top = __ballot(bin == 255u);
            if (top != 0 && __lane_id() == 0) atomicAdd(&hist[255], (uint32_t)__popcll(top));
            if (bin < 255u) atomicAdd(&hist[bin], 1u);
        };
        if (KIND == SCAN_NIB8) {
            for (int base = lo; base < hi; base += step) {
                if (base != lo) {
#pragma unroll
                    for (int u = 0; u < PPT; ++u) {
                        int id = base + u * (int)blockDim.x + (int)threadIdx.x;
                        id = id < hi ? id : hi - 1;
                        pc[u] = *(const uint2 *)(codes + (size_t)id * 8);
                    }
                }
#pragma unroll
                for (int u = 0; u < PPT; ++u) {
                    const int id = base + u * (int)blockDim.x + (int)threadIdx.x;
                    const uint32_t sm = sum8(gtab, pc[u].x, pc[u].y);
                    count_key(id < hi ? (sm > (uint32_t)qmax ? (uint32_t)qmax : sm) : 0xffffffffu);
                }
            }
        } else if ((KIND == SCAN_W64 || KIND == SCAN_C5) && L->g32ok != 0 && L->ng <= QADC_MAXG_FAST) {
            // group descriptors in registers; 8-byte codes one per load, 5-byte codes four per
            // 20-byte chunk of five dwords (slices start on multiples of 1024 codes)
            const GroupDesc gd = load_group_desc(L);
            for (int base = lo; base < hi; base += step) {
                if (KIND == SCAN_W64) {
                    uint2 w[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        int id = base + u * (int)blockDim.x + (int)threadIdx.x;
                        id = id < hi ? id : hi - 1;
                        w[u] = *(const uint2 *)(codes + (size_t)id * 8);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int id = base + u * (int)blockDim.x + (int)threadIdx.x;
                        const uint32_t sm = sum_groups_rt(gd, gtab, w[u].x, w[u].y);
                        count_key(id < hi ? (sm > (uint32_t)qmax ? (uint32_t)qmax : sm) : 0xffffffffu);
                    }
                } else {
                    uint32_t c5[2][5];
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int id = base + 4 * (u * (int)blockDim.x + (int)threadIdx.x);
#pragma unroll
                        for (int i = 0; i < 5; ++i)  // a chunk not wholly inside is handled code by code
                            c5[u][i] = id + 3 < hi ? ((const uint32_t *)(codes + (size_t)id * 5))[i] : 0u;
                    }
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int id = base + 4 * (u * (int)blockDim.x + (int)threadIdx.x);
                        uint32_t k4[4];
                        if (id + 3 < hi) {
                            // code v = bits [40v, 40v+40) of the chunk, as (low dword, high byte)
                            const uint32_t l4[4] = {c5[u][0], __builtin_amdgcn_alignbit(c5[u][2], c5[u][1], 8),
                                                    __builtin_amdgcn_alignbit(c5[u][3], c5[u][2], 16),
                                                    __builtin_amdgcn_alignbit(c5[u][4], c5[u][3], 24)};
                            const uint32_t h4[4] = {c5[u][1] & 0xffu, (c5[u][2] >> 8) & 0xffu,
                                                    (c5[u][3] >> 16) & 0xffu, c5[u][4] >> 24};
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                const uint32_t sm = sum_groups_rt(gd, gtab, l4[v], h4[v]);
                                k4[v] = sm > (uint32_t)qmax ? (uint32_t)qmax : sm;
                            }
                        } else {
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                k4[v] = id + v < hi ? key_at<KIND, QT>(L, gtab, codes, id + v) : 0xffffffffu;
                        }
                        // (count_key holds wave-wide operations: every lane calls it)
#pragma unroll
                        for (int v = 0; v < 4; ++v) count_key(k4[v]);
                    }
                }
            }
        } else {
            for (int base = lo; base < hi; base += step) {
                uint32_t key[8];
                keys_batch<KIND, QT, 8>(L, gtab, codes, (int64_t)base + threadIdx.x, blockDim.x,
                                        (int64_t)hi, key);
#pragma unroll
                for (int u = 0; u < 8; ++u) count_key(key[u]);
            }
        }
        __syncthreads();
        if (P > 1) {
            // this block's record: cumulative counts over 64 coarse bins, one lane per bin
            if (threadIdx.x < QADC_WAVE) {
                const uint4 h4 = *(const uint4 *)&hist[4 * threadIdx.x];
                const uint32_t c4 = h4.x + h4.y + h4.z + h4.w;
                const uint32_t cum = qadc_wave_incl_scan(c4);
                bound_rec[((size_t)q * QADC_REC_BINS + threadIdx.x) * QADC_REC_SLOTS + p] =
                    (uint16_t)(cum > 65535u ? 65535u : cum);
            }
        } else {
            if (threadIdx.x < QADC_WAVE) qadc_wave_select_bin(hist, (uint32_t)k, 0u, sel);
            __syncthreads();
            bound = sizeof(QT) == 1 ? sel[0] : ((sel[0] << 8) | 255u);
        }
    }
    if (!first) return;
    if (threadIdx.x == 0) {
        pq_qparams_t prm;
        prm.d_min = s_dmin;
        prm.delta = s_delta;
        prm.d_max = s_dmax;
        prm.key_bound = bound;
        qparams[q] = prm;
    }
}

// Codes one pilot block counts per batch (eight per thread) and at most in total.
#define PILOT_BATCH (8 * QUANT_THREADS)
#define PILOT_BLOCK_MAX 65536

int qadc_pilot_blocks_max(int nq) {
    const int64_t cap = qadc_option(PQ_OPT_PILOT_BLOCKS);
    int pmax = 2048 / (nq > 0 ? nq : 1);  // (blocks of 256 threads: a few thousand fill the chip)
    pmax = pmax < 1 ? 1 : (pmax > QADC_REC_SLOTS ? QADC_REC_SLOTS : pmax);
    return cap >= 1 && cap < pmax ? (int)cap : pmax;
}

size_t qadc_pilot_scratch_bytes(int nq) {
    return (size_t)(nq > 0 ? nq : 0) * QADC_REC_BINS * QADC_REC_SLOTS * sizeof(uint16_t);
}

// The pilot of a call: how many codes, split over how many blocks per query.  With scratch
// memory (the fused search) a small batch of queries spreads a large pilot over many
// blocks; without it every query has one block and the pilot stays small.
PilotPlan qadc_pilot_plan(int nq, int64_t n, int t_eff, int R, bool have_scratch, bool cheap_lookups) {
    int64_t multi = qadc_option(PQ_OPT_PILOT_CODES);
    const int64_t single = qadc_option(PQ_OPT_PILOT_CODES_SINGLE);
    PilotPlan pp;
    const int pmax = have_scratch ? qadc_pilot_blocks_max(nq) : 1;
    // The whole sample pays when many blocks share it and a look-up is cheap (m x 4 codes, one
    // query per call: 4096 codes per block; fewer candidates then shorten the scan's appends and
    // the selection by more than the sample costs).  Otherwise half of it, as long as that is
    // not below 262144.
    const int64_t per_block = cheap_lookups ? 4096 : 2048;
    if (multi > 262144 && multi > per_block * pmax) multi = per_block * pmax > 262144 ? per_block * pmax : 262144;
    int64_t want = pmax > 1 ? multi : single;
    // the candidates the scan keeps grow with R / pilot: long result lists get a longer pilot
    if (pmax > 1 && want < 512 * (int64_t)R) want = 512 * (int64_t)R;
    if (want > (int64_t)pmax * PILOT_BLOCK_MAX) want = (int64_t)pmax * PILOT_BLOCK_MAX;
    if (want < 64 * (int64_t)R) want = 64 * (int64_t)R;
    if (want < t_eff) want = t_eff;
    if (want > n) want = n;
    int64_t P = (want + PILOT_BATCH - 1) / PILOT_BATCH;
    if (P > pmax) P = pmax;
    if (P < 1) P = 1;
    int64_t slice = (want + P - 1) / P;
    slice = (slice + 1023) / 1024 * 1024;
    if (slice < 1024) slice = 1024;
    pp.pilot = (int)want;
    pp.P = (int)P;
    pp.slice = (int)slice;
    return pp;
}

static size_t quantize_lds(const DevLayout &h, int t_eff, size_t esz) {
    const size_t nord = (size_t)((t_eff > h.d ? t_eff : h.d) > 0 ? (t_eff > h.d ? t_eff : h.d) : 1);
    return (((size_t)h.T * 4 + nord * 4 + PQ_MAX_M * 4 + (size_t)h.T * 3 + 15) & ~(size_t)15) +
           (size_t)h.gtab_len * esz;
}

template <int KIND, typename QT>
static int launch_quantize(const pq_index *idx, const float *queries, const float *tables_in,
                           float *tables_out, int nq, const uint8_t *codes, int t_eff, int k,
                           const PilotPlan &pp, void *qtables, pq_qparams_t *qparams, char *gtab_out,
                           size_t gtab_stride, char *hdr_out, uint16_t *bound_rec, hipStream_t s) {
    const size_t lds = quantize_lds(idx->h, t_eff, sizeof(QT));
    if (lds > 48 * 1024)
        QADC_HIP_TRY(hipFuncSetAttribute((const void *)k_quantize<KIND, QT>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    int ubits = idx->h.nbits[0], uds = idx->h.dsub[0];
    for (int j = 1; j < idx->h.m; ++j) {
        if (idx->h.nbits[j] != ubits) ubits = 0;
        if (idx->h.dsub[j] != uds) uds = 0;
    }
    hipLaunchKernelGGL((k_quantize<KIND, QT>), dim3((unsigned)nq * (unsigned)pp.P), dim3(QUANT_THREADS), lds, s,
                       idx->dev, QuantShape{idx->h.T, idx->h.m, idx->h.cs, idx->h.qmax, idx->h.d, ubits, uds}, idx->edesc,
                       idx->codebooks, queries, tables_in, tables_out, codes, t_eff, k,
                       pp.pilot, pp.slice, pp.P, qtables, qparams, gtab_out, gtab_stride, hdr_out, bound_rec);
    QADC_LAUNCH_CHECK("k_quantize");
    return PQ_OK;
}

// Shared by pq_quantize_tables (queries == null) and the fused search call.  `scratch`
// (qadc_pilot_scratch_bytes(nq) bytes, 256-byte aligned, any contents) lets several blocks
// share a query's pilot; null keeps one block per query.
int qadc_quantize_launch(const pq_index *idx, const float *queries, const float *tables_in,
                         float *tables_out, int nq, const uint8_t *codes, int64_t n, int t, int R,
                         void *qtables, pq_qparams_t *qparams, char *gtab_out, size_t gtab_stride,
                         char *hdr_out, char *scratch, PilotPlan *plan_used, hipStream_t s) {
    const int64_t want = t > 4 * (int64_t)R ? t : 4 * (int64_t)R;
    const int t_eff = (int)(n < want ? n : want);
    const int k = R < t_eff ? R : t_eff;
    const PilotPlan pp = qadc_pilot_plan(nq, n, t_eff, R, scratch != nullptr,
                                         idx->h.kind == SCAN_NIB8 || idx->h.kind == SCAN_NIB16);
    if (plan_used) *plan_used = pp;
    uint16_t *bound_rec = (uint16_t *)scratch;
    const bool u8 = idx->h.acc_bits == 8;
#define QADC_GO(KIND, QT)                                                                       \
    return launch_quantize<KIND, QT>(idx, queries, tables_in, tables_out, nq, codes, t_eff, k, \
                                     pp, qtables, qparams, gtab_out, gtab_stride, hdr_out, bound_rec, s)
    switch (idx->h.kind) {
        case SCAN_NIB8:
            if (u8) QADC_GO(SCAN_NIB8, uint8_t); else QADC_GO(SCAN_NIB8, uint16_t);
        case SCAN_NIB16:
            if (u8) QADC_GO(SCAN_NIB16, uint8_t); else QADC_GO(SCAN_NIB16, uint16_t);
        case SCAN_W64:
            if (u8) QADC_GO(SCAN_W64, uint8_t); else QADC_GO(SCAN_W64, uint16_t);
        case SCAN_C5:
            if (u8) QADC_GO(SCAN_C5, uint8_t); else QADC_GO(SCAN_C5, uint16_t);
        case SCAN_W128:
            if (u8) QADC_GO(SCAN_W128, uint8_t); else QADC_GO(SCAN_W128, uint16_t);
        default:
            if (u8) QADC_GO(SCAN_GENERIC, uint8_t); else QADC_GO(SCAN_GENERIC, uint16_t);
    }
#undef QADC_GO
}

extern "C" int pq_quantize_tables(const pq_index_t *idx, const float *tables, int nq,
                                  const uint8_t *codes, int64_t n, int t, int R, void *qtables,
                                  pq_qparams_t *qparams, void *stream) {
    if (!idx || nq < 0 || n < 0) {
        qadc_set_error("pq_quantize_tables: bad handle, nq or n");
        return PQ_EINVAL;
    }
    if (R < 1 || R > PQ_MAX_R || t < 1) {
        qadc_set_error("pq_quantize_tables: need 1<=R<=%d and t>=1 (got R=%d t=%d)", PQ_MAX_R, R, t);
        return PQ_EINVAL;
    }
    const int64_t want = t > 4 * (int64_t)R ? t : 4 * (int64_t)R;
    if (want > PQ_MAX_T_EFF) {
        qadc_set_error("pq_quantize_tables: max(t,4R)=%lld exceeds %d", (long long)want, PQ_MAX_T_EFF);
        return PQ_EINVAL;
    }
    if (nq == 0) return PQ_OK;
    if (!tables || !qtables || !qparams || (n > 0 && !codes)) {
        qadc_set_error("pq_quantize_tables: null pointer");
        return PQ_EINVAL;
    }
    if (n > 0 && ((uintptr_t)codes & 15u) != 0) {
        qadc_set_error("pq_quantize_tables: codes must be 16-byte aligned");
        return PQ_EINVAL;
    }
    return qadc_quantize_launch(idx, nullptr, tables, nullptr, nq, codes, n, t, R, qtables, qparams,
                                nullptr, 0, nullptr, nullptr, nullptr, (hipStream_t)stream);
}
