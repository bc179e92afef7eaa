// ivf_adc_scan_topk: ADC over the inverted lists of the probed cells.
// Section 2.1.1 (residuals are encoded), Section 2.1.3 (one table set per probed
// cell from z' = z - centroid), Section 3.4 (distance quantizer).
//
//   k_ivf_calib  one block per query: float ADC of the first t_eff probed codes
//                (each with its own cell's tables) -> d_max; then the quantized
//                distances of the first few thousand probed codes -> thr0, the
//                R-th smallest of them, an upper bound on the R-th best distance
//                of the query, and a monotone 256-bin map of [lo, thr0].
//   k_ivf_scan   one block per (query, probed cell): residual tables, the
//                cell's p_min / d_min / delta from the shared d_max, quantized
//                group tables in LDS, scan of the list; codes with distance
//                <= thr0 go to the block's slot list as
//                (ordered float distance << 32 | stored id).
//   k_ivf_final  one block per query: gather the candidates, find the bin of the
//                R-th, rank the few up to it; exact multi-pass selection over
//                all probed codes if a slot list overflowed.
#include "scan_device.h"

struct IvfLds {
    float *zres;   // [d]
    float *tab;    // [T]
    float *pmin;   // [PQ_MAX_M]
    uint16_t *qt;  // [T]
    void *gtab;    // [gtab_len] of QT
    double *sc;    // {d_min, delta}
    int *flag;     // skip flag
};

__device__ inline size_t ivf_lds_bytes_dev(const DevLayout *L, size_t esz) {
    return (size_t)L->d * 4 + (size_t)L->T * 4 + PQ_MAX_M * 4 + (size_t)L->T * 4 +
           (((size_t)L->gtab_len * esz + 15) & ~(size_t)15) + 32;
}
static size_t ivf_lds_bytes(const DevLayout &L, size_t esz) {
    return (size_t)L.d * 4 + (size_t)L.T * 4 + PQ_MAX_M * 4 + (size_t)L.T * 4 +
           (((size_t)L.gtab_len * esz + 15) & ~(size_t)15) + 32;
}

// carve the per-list LDS arrays out of `base` (16-byte aligned)
__device__ inline unsigned char *ivf_carve(const DevLayout *L, unsigned char *base, size_t esz,
                                           IvfLds &l) {
    unsigned char *p = base;
    l.sc = (double *)p;      p += 16;
    l.flag = (int *)p;       p += 16;
    l.zres = (float *)p;     p += (size_t)L->d * 4;
    l.tab = (float *)p;      p += (size_t)L->T * 4;
    l.pmin = (float *)p;     p += PQ_MAX_M * 4;
    l.gtab = (void *)p;      p += (((size_t)L->gtab_len * esz + 15) & ~(size_t)15);
    l.qt = (uint16_t *)p;    p += (size_t)L->T * 2;
    p += (size_t)L->T * 2;  // spare; keeps what follows 4-byte aligned
    return p;
}

// Block-wide: residual, float tables (eq. (1)), p_min, d_min; with `quantize`
// also delta from dmax, the quantized table and (with `groups`) the group
// tables.  Returns false when the list is skipped (d_min >= d_max: Section 3.4, later
// candidates have to be closer than d_max).
template <int KIND, typename QT>
__device__ inline bool ivf_setup(const DevLayout *L, const EntryDesc *__restrict__ edesc,
                                 const float *__restrict__ cb, const float *__restrict__ z,
                                 const float *__restrict__ cen, float dmax, bool quantize,
                                 bool groups, const IvfLds &l) {
    const int d = L->d, m = L->m, T = L->T, qmax = L->qmax;
    for (int i = threadIdx.x; i < d; i += blockDim.x) l.zres[i] = __fsub_rn(z[i], cen[i]);
    __syncthreads();
    for (int e = threadIdx.x; e < T; e += blockDim.x) {
        const EntryDesc ed = edesc[e];
        const int ds = ed.ds;
        const float *c = cb + ed.cb_off;
        const float *zz = l.zres + ed.dim_off;
        float acc = 0.0f;
        for (int k = 0; k < ds; ++k) {
            float diff = __fsub_rn(zz[k], c[k]);
            acc = __fadd_rn(acc, __fmul_rn(diff, diff));
        }
        l.tab[e] = acc;
    }
    __syncthreads();
    if ((int)threadIdx.x < m) {
        const int j = threadIdx.x;
        const int kj = 1 << L->nbits[j];
        const float *tj = l.tab + L->toff[j];
        float mn = tj[0];
        for (int i = 1; i < kj; ++i) mn = tj[i] < mn ? tj[i] : mn;
        l.pmin[j] = mn;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double dm = 0.0;
        for (int j = 0; j < m; ++j) dm = dm + (double)l.pmin[j];
        l.sc[0] = dm;
        int skip = 0;
        double delta = 0.0;
        if (quantize) {
            skip = dm >= (double)dmax;
            delta = ((double)dmax - dm) / (double)qmax;
            if (!((delta > 0.0) && isfinite(delta))) delta = 0.0;
        }
        l.sc[1] = delta;
        *l.flag = skip;
    }
    __syncthreads();
    if (!quantize) return true;
    if (*l.flag) return false;
    const double delta = l.sc[1];
    for (int e = threadIdx.x; e < T; e += blockDim.x) {
        const int j = edesc[e].j;
        uint32_t qv = 0;
        if (delta > 0.0) {
            double x = floor(((double)l.tab[e] - (double)l.pmin[j]) / delta);
            qv = (x >= (double)qmax) ? (uint32_t)qmax : (uint32_t)x;
        }
        l.qt[e] = (uint16_t)qv;
    }
    __syncthreads();
    if (groups) build_gtab<KIND, QT>(L, l.qt, (QT *)l.gtab);
    return true;
}

// The same for the fixed shape 16 x 4 bits over sub-spaces of DS dimensions each (T = 256,
// d = 16 DS) by a block of 256 threads: thread e holds table entry e = centroid e % 16 of
// sub-quantizer e / 16 at codebook offset e * DS, so nothing is looked up, the minima come
// from lane exchanges, and the codebook values travel while the residual settles in LDS.
template <int DS>
__device__ inline bool ivf_setup_fix(const float *__restrict__ cb, const float *__restrict__ z,
                                     const float *__restrict__ cen, float dmax, bool quantize,
                                     uint32_t qmax, const IvfLds &l) {
    constexpr int d = 16 * DS;
    const int e = threadIdx.x;
    float cv[DS];
#pragma unroll
    for (int t = 0; t < DS; ++t) cv[t] = cb[e * DS + t];
    if (e < d) l.zres[e] = __fsub_rn(z[e], cen[e]);
    __syncthreads();
    const float *zz = l.zres + (e >> 4) * DS;
    float acc = 0.0f;
#pragma unroll
    for (int t = 0; t < DS; ++t) {
        const float diff = __fsub_rn(zz[t], cv[t]);
        acc = __fadd_rn(acc, __fmul_rn(diff, diff));
    }
    l.tab[e] = acc;
    float mn = acc;
#pragma unroll
    for (int sft = 1; sft < 16; sft <<= 1) {
        const float o = __shfl_xor(mn, sft, QADC_WAVE);
        mn = o < mn ? o : mn;
    }
    if ((e & 15) == 0) l.pmin[e >> 4] = mn;
    __syncthreads();
    if (e == 0) {
        double dm = 0.0;
        for (int j = 0; j < 16; ++j) dm = dm + (double)l.pmin[j];
        l.sc[0] = dm;
        int skip = 0;
        double delta = 0.0;
        if (quantize) {
            skip = dm >= (double)dmax;
            delta = ((double)dmax - dm) / (double)qmax;
            if (!((delta > 0.0) && isfinite(delta))) delta = 0.0;
        }
        l.sc[1] = delta;
        *l.flag = skip;
    }
    __syncthreads();
    if (!quantize) return true;
    if (*l.flag) return false;
    const double delta = l.sc[1];
    uint32_t qv = 0;
    if (delta > 0.0) {
        const double x = floor(((double)acc - (double)l.pmin[e >> 4]) / delta);
        qv = (x >= (double)qmax) ? qmax : (uint32_t)x;
    }
    l.qt[e] = (uint16_t)qv;
    __syncthreads();
    return true;
}

__device__ __forceinline__ uint32_t dist_bin(float dist, float lo, float scale) {
    float x = (dist - lo) * scale;
    return x <= 0.0f ? 0u : (x >= 255.0f ? 255u : (uint32_t)x);
}

// ------------------------------------------------------------ k_ivf_calib ---
#define CALIB_PC 64      // probes whose cell and list bounds the block keeps in LDS
#define CALIB_EARLY1 2   // codes per thread requested before the set-up, calibration pass
#define CALIB_EARLY2 4   // the same, pilot pass

// cell and list bounds of probe a: from the block's table, or from memory beyond it
__device__ __forceinline__ void calib_list(int a, const int32_t *__restrict__ probes,
                                           const int64_t *__restrict__ list_offsets, int K,
                                           const int32_t *s_pcell, const int64_t *s_plo, const int32_t *s_plen,
                                           int &c, int64_t &lo, int64_t &hi) {
    if (a < CALIB_PC) {
        c = s_pcell[a];
        lo = s_plo[a];
        hi = lo + s_plen[a];
    } else {
        c = probes[a];
        const bool valid = c >= 0 && c < K;
        lo = valid ? list_offsets[c] : 0;
        hi = valid ? list_offsets[c + 1] : 0;
    }
}

// NIB: 64-bit m x 4 codes (sub-code j is nibble j of the code).  Other layouts take the
// sub-quantizers' table offset, bit offset and width from a small LDS array.
// pair_cnt (or null): bucket counts of the pairs' sort by cell, pair_nb buckets and one more
// for pairs without a list, zero on entry; the block adds its query's pairs.
template <bool NIB, int DS = 0>
__global__ void __launch_bounds__(256)
k_ivf_calib(const DevLayout *__restrict__ L, const EntryDesc *__restrict__ edesc,
            const float *__restrict__ cb,
            const float *__restrict__ coarse, const int64_t *__restrict__ list_offsets,
            const uint8_t *__restrict__ list_codes, const float *__restrict__ queries,
            const int32_t *__restrict__ probe_ids, int nprobe, int K, int want, int pilot_want,
            int R, char *__restrict__ ws, size_t per_query, uint32_t *__restrict__ pair_cnt, int pair_nb) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sel[8];
    __shared__ uint32_t kmem[QADC_KTH_MEM];
    __shared__ unsigned long long s_np;
    __shared__ uint32_t sdesc[PQ_MAX_M];  // table offset | bit offset << 12 | bits << 24
    // cell, first code and length of the lists of the first CALIB_PC probes (length 0: no list):
    // the loops below walk a few lists one after the other and would otherwise wait for the
    // probe id and then the bounds of each
    __shared__ int64_t s_plo[CALIB_PC];
    __shared__ int32_t s_plen[CALIB_PC], s_pcell[CALIB_PC];
    IvfLds l;
    unsigned char *rest = ivf_carve(L, smem, 2, l);
    uint32_t *ord = (uint32_t *)rest;  // [max(want, pilot_want)]
    if (!NIB && (int)threadIdx.x < L->m)
        sdesc[threadIdx.x] = (uint32_t)L->toff[threadIdx.x] | ((uint32_t)L->bitoff[threadIdx.x] << 12) |
                             ((uint32_t)L->nbits[threadIdx.x] << 24);
    const size_t q = blockIdx.x;
    IvfState *st = (IvfState *)(ws + q * per_query);
    const int32_t *probes = probe_ids + q * nprobe;
    const float *z = queries + q * L->d;
    const int m = L->m, cs = L->cs, qmax = L->qmax;

    // number of probed codes: one probe per thread (independent loads), then a block sum
    if (threadIdx.x == 0) s_np = 0;
    __syncthreads();
    {
        long long np = 0;
        for (int a = threadIdx.x; a < nprobe; a += blockDim.x) {
            const int c = probes[a];
            const bool valid = c >= 0 && c < K;
            const int64_t lo = valid ? list_offsets[c] : 0, hi = valid ? list_offsets[c + 1] : 0;
            np += hi - lo;
            // the count of the sort of the (query, probe) pairs by cell (ivf_pair_bucket), for
            // which this loop has the cell and the bounds at hand
            if (pair_cnt) atomicAdd(&pair_cnt[hi > lo ? (int)(((int64_t)c * pair_nb) / K) : pair_nb], 1u);
            if (a < CALIB_PC) {
                s_pcell[a] = c;
                s_plo[a] = lo;
                s_plen[a] = (int32_t)(hi - lo);  // a list is shorter than 2^31 codes
            }
        }
        for (int sft = QADC_WAVE / 2; sft > 0; sft >>= 1) np += __shfl_xor(np, sft, QADC_WAVE);
        if (threadIdx.x % QADC_WAVE == 0 && np != 0)
            atomicAdd((unsigned long long *)&s_np, (unsigned long long)np);
    }
    __syncthreads();
    const int t_eff = (int)((long long)s_np < (long long)want ? (long long)s_np : (long long)want);
    const int pilot = (int)((long long)s_np < (long long)pilot_want ? (long long)s_np : (long long)pilot_want);
    const int k = R < t_eff ? R : t_eff;
    if (t_eff == 0) {
        if (threadIdx.x == 0) {
            st->dmax = INFINITY;
            st->thr0 = INFINITY;
            st->lo = 0.f;
            st->scale = 0.f;
        }
        return;
    }
    // pass 1: float ADC of the calibration codes
    int seen = 0;
    for (int a = 0; a < nprobe && seen < t_eff; ++a) {
        int c;
        int64_t lo, hi;
        calib_list(a, probes, list_offsets, K, s_pcell, s_plo, s_plen, c, lo, hi);
        if (hi == lo) continue;
        const int take = (int)((hi - lo) < (int64_t)(t_eff - seen) ? (hi - lo) : (int64_t)(t_eff - seen));
        // the first codes are requested before the set-up (their sub-codes index its tables)
        uint2 early[CALIB_EARLY1];
        if (NIB) {
#pragma unroll
            for (int u = 0; u < CALIB_EARLY1; ++u) {
                const int p = (int)threadIdx.x + u * 256;
                early[u] = *(const uint2 *)(list_codes + (size_t)(lo + (p < take ? p : take - 1)) * 8);
            }
        }
        if constexpr (DS > 0)
            ivf_setup_fix<DS>(cb, z, coarse + (size_t)c * (16 * DS), 0.f, false, (uint32_t)qmax, l);
        else
            ivf_setup<SCAN_GENERIC, uint16_t>(L, edesc, cb, z, coarse + (size_t)c * L->d, 0.f, false, false, l);
        auto adc = [&](int p, bool have, uint2 v) {  // have: v holds the code already (NIB)
            const uint8_t *code = list_codes + (size_t)(lo + p) * cs;
            float s = 0.0f;
            if (NIB) {
                if (!have) v = *(const uint2 *)code;
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    s = __fadd_rn(s, l.tab[16 * j + (((j < 8 ? v.x : v.y) >> (4 * (j & 7))) & 15u)]);
            } else if (cs <= 16) {
                uint32_t w[4];
                qadc_load_code16(code, cs, w);
                for (int j = 0; j < m; ++j) {
                    const uint32_t ds = sdesc[j];
                    s = __fadd_rn(s, l.tab[(ds & 0xfffu) + qadc_extract_sub16(w, (ds >> 12) & 0xfffu, ds >> 24)]);
                }
            } else {
                for (int j = 0; j < m; ++j)
                    s = __fadd_rn(s, l.tab[L->toff[j] + qadc_extract_sub(code, L->bitoff[j], L->nbits[j])]);
            }
            ord[seen + p] = qadc_f2ord(s);
        };
        int p = threadIdx.x;
        if (NIB) {
#pragma unroll
            for (int u = 0; u < CALIB_EARLY1; ++u, p += 256)
                if (p < take) adc(p, true, early[u]);
        }
        for (; p < take; p += blockDim.x) adc(p, false, make_uint2(0u, 0u));
        seen += take;
        __syncthreads();
    }
    const float dmax = qadc_ord2f(qadc_block_kth_f32(ord, t_eff, k, hist, sel, kmem));
    // pass 2: quantized distances of the first `pilot` probed codes -> thr0 and the binning
    seen = 0;
    for (int a = 0; a < nprobe && seen < pilot; ++a) {
        int c;
        int64_t lo, hi;
        calib_list(a, probes, list_offsets, K, s_pcell, s_plo, s_plen, c, lo, hi);
        if (hi == lo) continue;
        const int take = (int)((hi - lo) < (int64_t)(pilot - seen) ? (hi - lo) : (int64_t)(pilot - seen));
        uint2 early[CALIB_EARLY2];
        if (NIB) {
#pragma unroll
            for (int u = 0; u < CALIB_EARLY2; ++u) {
                const int p = (int)threadIdx.x + u * 256;
                early[u] = *(const uint2 *)(list_codes + (size_t)(lo + (p < take ? p : take - 1)) * 8);
            }
        }
        bool ok;
        if constexpr (DS > 0)
            ok = ivf_setup_fix<DS>(cb, z, coarse + (size_t)c * (16 * DS), dmax, true, (uint32_t)qmax, l);
        else
            ok = ivf_setup<SCAN_GENERIC, uint16_t>(L, edesc, cb, z, coarse + (size_t)c * L->d, dmax, true, false, l);
        const float fdelta = (float)l.sc[1], fdmin = (float)l.sc[0];
        auto qadc_of = [&](int p, bool have, uint2 v) {
            uint32_t o = 0xffffffffu;
            if (ok) {
                const uint8_t *code = list_codes + (size_t)(lo + p) * cs;
                uint32_t acc = 0;
                if (NIB) {
                    if (!have) v = *(const uint2 *)code;
#pragma unroll
                    for (int j = 0; j < 16; ++j)
                        acc += l.qt[16 * j + (((j < 8 ? v.x : v.y) >> (4 * (j & 7))) & 15u)];
                } else if (cs <= 16) {
                    uint32_t w[4];
                    qadc_load_code16(code, cs, w);
                    for (int j = 0; j < m; ++j) {
                        const uint32_t ds = sdesc[j];
                        acc += l.qt[(ds & 0xfffu) + qadc_extract_sub16(w, (ds >> 12) & 0xfffu, ds >> 24)];
                    }
                } else {
                    for (int j = 0; j < m; ++j)
                        acc += l.qt[L->toff[j] + qadc_extract_sub(code, L->bitoff[j], L->nbits[j])];
                }
                if (acc > (uint32_t)qmax) acc = (uint32_t)qmax;
                o = qadc_f2ord(fmaf((float)acc, fdelta, fdmin));
            }
            ord[seen + p] = o;
        };
        int p = threadIdx.x;
        if (NIB) {
            // rounds of CALIB_EARLY2 codes per thread; the next round is requested before the
            // current one is looked up
            while (p < take) {
                uint2 cur[CALIB_EARLY2];
#pragma unroll
                for (int u = 0; u < CALIB_EARLY2; ++u) cur[u] = early[u];
                const int pn = p + CALIB_EARLY2 * 256;
                if (pn < take) {
#pragma unroll
                    for (int u = 0; u < CALIB_EARLY2; ++u) {
                        const int pp = pn + u * 256;
                        early[u] = *(const uint2 *)(list_codes + (size_t)(lo + (pp < take ? pp : take - 1)) * 8);
                    }
                }
#pragma unroll
                for (int u = 0; u < CALIB_EARLY2; ++u)
                    if (p + u * 256 < take) qadc_of(p + u * 256, true, cur[u]);
                p = pn;
            }
        }
        for (; p < take; p += blockDim.x) qadc_of(p, false, make_uint2(0u, 0u));
        seen += take;
        __syncthreads();
    }
    const uint32_t inf_o = qadc_f2ord(INFINITY);
    uint32_t t0 = qadc_block_kth_u32(ord, pilot, k, 4, hist, sel);
    // smallest pilot distance: block minimum
    uint32_t l0 = 0xffffffffu;
    for (int p = threadIdx.x; p < pilot; p += blockDim.x) l0 = ord[p] < l0 ? ord[p] : l0;
    l0 = qadc_wave_min(l0);
    __syncthreads();
    if (threadIdx.x == 0) sel[0] = 0xffffffffu;
    __syncthreads();
    if (threadIdx.x % QADC_WAVE == 0) atomicMin(&sel[0], l0);
    __syncthreads();
    l0 = sel[0];
    if (threadIdx.x == 0) {
        const float thr0 = t0 > inf_o ? INFINITY : qadc_ord2f(t0);
        const float lo = l0 > inf_o ? 0.f : qadc_ord2f(l0);
        const float span = thr0 - lo;
        st->dmax = dmax;
        st->thr0 = thr0;
        st->lo = lo;
        st->scale = (span > 0.f && isfinite(span)) ? 256.0f / span : 0.f;
    }
}

// ------------------------------------------------- (query, probe) pairs by cell ---
// The scan kernel's blocks are handed out in the order of the probed cell, so that the blocks
// that read one inverted list run close together and all but the first find it in the L2 /
// last-level cache: a counting sort of the pair indices p = q * nprobe + a into NB <= 4096
// buckets of consecutive cells (a bucket's few dozen blocks run within one filling of the chip,
// which is close enough, and its lists are neighbours in memory).  Pairs without a list
// (negative or out-of-range id, empty list) go to a bucket of their own at the end.  The order
// within a bucket depends on timing; results do not (every pair owns its slots).
#define IVF_SORT_BUCKETS 4096
__global__ void __launch_bounds__(256)
k_pair_zero(uint32_t *__restrict__ cnt, int nwords) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nwords) cnt[i] = 0;
}

__device__ __forceinline__ int ivf_pair_bucket(const int32_t *__restrict__ probe_ids,
                                               const int64_t *__restrict__ list_offsets, int64_t p, int K,
                                               int NB) {
    const int c = probe_ids[p];
    if (c < 0 || c >= K) return NB;
    return list_offsets[c + 1] > list_offsets[c] ? (int)(((int64_t)c * NB) / K) : NB;
}

// one block: start[b] = number of pairs in buckets before b (b = 0 .. NB), and cnt cleared to
// serve as the buckets' fill cursors
__global__ void __launch_bounds__(1024)
k_pair_scan(uint32_t *__restrict__ cnt, uint32_t *__restrict__ start, int nb) {
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    const int wave = threadIdx.x / QADC_WAVE, lane = threadIdx.x % QADC_WAVE;
    for (int base = 0; base < nb; base += 1024) {
        const int i = base + (int)threadIdx.x;
        const uint32_t v = i < nb ? cnt[i] : 0u;
        const uint32_t incl = qadc_wave_incl_scan(v);
        if (lane == QADC_WAVE - 1) wsum[wave] = incl;
        __syncthreads();
        uint32_t before = carry;
        for (int w = 0; w < wave; ++w) before += wsum[w];
        if (i < nb) {
            start[i] = before + incl - v;
            cnt[i] = 0;
        }
        __syncthreads();
        if (threadIdx.x == 1023) carry = before + incl;
        __syncthreads();
    }
}

__global__ void __launch_bounds__(256)
k_pair_fill(const int32_t *__restrict__ probe_ids, const int64_t *__restrict__ list_offsets,
            int64_t npairs, int K, int NB, const uint32_t *__restrict__ start,
            uint32_t *__restrict__ fill, uint32_t *__restrict__ order) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= npairs) return;
    const int b = ivf_pair_bucket(probe_ids, list_offsets, p, K, NB);
    order[start[b] + atomicAdd(&fill[b], 1u)] = (uint32_t)p;
}

// ------------------------------------------------------------- k_ivf_scan ---
// One block per (query, probed cell).  A block is short (a few thousand codes behind a chain
// of small dependent steps) and the kernel as a whole streams lists that are not cached, so
// many blocks per CU matter (few registers) and the set-up is ordered for few round trips:
//   A  probe id, query state, query, entry descriptors      (independent loads)
//   B  list bounds, centroid, codebook values of the entries (need A)
//   C  the first codes of the list                           (need B; used after the set-up)
// NE = table entries per thread (1, 2 or 4; 0 = the general set-up routine, no early loads).
// DS > 0 fixes the shape at compile time: 16 sub-quantizers of 16 centroids over DS dimensions
// each (T = 256, d = 16 DS) and blocks of 256 / NE threads, so that table entry e = thread +
// k * threads is centroid e % 16 of sub-quantizer e / 16 at codebook offset e * DS, and the
// set-up needs neither descriptors nor bounds tests.
#ifndef QADC_IVF_PF
#define QADC_IVF_PF 2
#endif
template <int KIND, typename QT, int NE, int DS = 0>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(8, 8)))
k_ivf_scan(const DevLayout *__restrict__ L, const EntryDesc *__restrict__ edesc,
           const float *__restrict__ cb, const float *__restrict__ coarse,
           const int64_t *__restrict__ list_offsets, const uint8_t *__restrict__ list_codes,
           const int32_t *__restrict__ list_ids, const float *__restrict__ queries,
           const int32_t *__restrict__ probe_ids, int nprobe, int K, int R, char *__restrict__ ws,
           size_t per_query, size_t counts_off, size_t slots_off, int cap_b,
           const uint32_t *__restrict__ order) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ uint32_t s_count;
    IvfLds l;
    ivf_carve(L, smem, sizeof(QT), l);
    // block -> (query, probe): in grid order, or in the order of the probed cells
    const uint32_t lin = blockIdx.y * gridDim.x + blockIdx.x;
    const uint32_t pair = order ? order[lin] : lin;
    const size_t q = pair / (uint32_t)nprobe;
    const int a = (int)(pair % (uint32_t)nprobe);
    constexpr bool FIX = DS > 0;
    static_assert(!FIX || (KIND == SCAN_NIB8 && NE > 0 && DS <= 8 && 256 % NE == 0), "fixed shape");
    const int bd = FIX ? 256 / (NE > 0 ? NE : 1) : (int)blockDim.x;
    char *wq = ws + q * per_query;
    const IvfState *st = (const IvfState *)wq;
    uint32_t *counts = (uint32_t *)(wq + counts_off);
    constexpr int MAXDS = 8;  // codebook values per entry held in registers
    const int d = FIX ? 16 * DS : L->d, T = FIX ? 256 : L->T, m = FIX ? 16 : L->m, qmax = L->qmax;

    // A
    const int c = probe_ids[q * nprobe + a];
    const float dmax = st->dmax, thr0 = st->thr0;
    EntryDesc ed[NE > 0 ? NE : 1];
    if (NE > 0) {
#pragma unroll
        for (int k = 0; k < NE; ++k) {
            const int e = (int)threadIdx.x + k * bd;
            if (FIX) {
                ed[k].j = e >> 4;
                ed[k].cb_off = e * DS;
                ed[k].dim_off = (e >> 4) * DS;
                ed[k].ds = DS;
            } else {
                ed[k] = edesc[e < T ? e : T - 1];
            }
        }
        for (int i = threadIdx.x; i < d; i += bd) l.zres[i] = queries[q * d + i];
    }
    int64_t lo = 0, hi = 0;
    if (c >= 0 && c < K) {
        lo = list_offsets[c];
        hi = list_offsets[c + 1];
    }
    if (hi == lo) {
        if (threadIdx.x == 0) counts[a] = 0;
        return;
    }
    if (threadIdx.x == 0) s_count = 0;
    bool ok;
    // 64-bit m x 4 codes are read two at a time: the list from its first even position
    constexpr int PF = QADC_IVF_PF;  // 16-byte loads per lane in flight
    const int64_t lo2 = (lo + 1) & ~(int64_t)1;
    const int64_t npair = hi > lo2 ? (hi - lo2) >> 1 : 0;
    const uint4 *__restrict__ pairs = (const uint4 *)(list_codes + lo2 * 8);
    uint4 pp[PF];
    if (NE > 0) {
        // B
        // sub-space width if all sub-quantizers share one (then a scalar, and nothing below
        // needs per-lane predicates), else 0
        const int dsu = FIX ? DS : L->ds_uniform;
        float cv[NE > 0 ? NE : 1][MAXDS];
#pragma unroll
        for (int k = 0; k < NE; ++k)
#pragma unroll
            for (int t = 0; t < MAXDS; ++t) {
                if (dsu > 0) {
                    if (t < dsu) cv[k][t] = cb[ed[k].cb_off + t];
                } else {
                    cv[k][t] = t < ed[k].ds ? cb[ed[k].cb_off + t] : 0.0f;
                }
            }
        __syncthreads();  // the query is in LDS
        for (int i = threadIdx.x; i < d; i += bd)
            l.zres[i] = __fsub_rn(l.zres[i], coarse[(size_t)c * d + i]);
        // C: the first PF 16-byte pairs of codes per lane, from the first even position on
        if (KIND == SCAN_NIB8 && npair > 0) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                int64_t pi = (int64_t)u * bd + threadIdx.x;
                pi = pi < npair ? pi : npair - 1;
                pp[u] = pairs[pi];
            }
        }
        __syncthreads();  // the residual is in LDS
        // eq. (1), terms in ascending dimension order
#pragma unroll
        for (int k = 0; k < NE; ++k) {
            const int e = (int)threadIdx.x + k * bd;
            if (FIX || e < T) {
                const float *zz = l.zres + ed[k].dim_off;
                float acc = 0.0f;
#pragma unroll
                for (int t = 0; t < MAXDS; ++t) {
                    if (dsu > 0 ? t < dsu : t < ed[k].ds) {
                        const float diff = __fsub_rn(zz[t], cv[k][t]);
                        acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                    }
                }
                for (int t = MAXDS; !FIX && t < ed[k].ds; ++t) {  // wider sub-spaces: the rest from memory
                    const float diff = __fsub_rn(zz[t], cb[ed[k].cb_off + t]);
                    acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                }
                l.tab[e] = acc;
            }
        }
        if (KIND == SCAN_NIB8 || KIND == SCAN_NIB16) {
            // 16 entries per sub-quantizer, held by 16 adjacent lanes: minimum by exchange
#pragma unroll
            for (int k = 0; k < NE; ++k) {
                const int e = (int)threadIdx.x + k * bd;
                float mn = (FIX || e < T) ? l.tab[e] : INFINITY;  // own entry, just written by this thread
#pragma unroll
                for (int sft = 1; sft < 16; sft <<= 1) {
                    const float o = __shfl_xor(mn, sft, QADC_WAVE);
                    mn = o < mn ? o : mn;
                }
                if ((FIX || e < T) && (e & 15) == 0) l.pmin[e >> 4] = mn;
            }
        } else {
            __syncthreads();
            if ((int)threadIdx.x < m) {
                const int j = threadIdx.x;
                const int kj = 1 << L->nbits[j];
                const float *tj = l.tab + L->toff[j];
                float mn = tj[0];
                for (int i = 1; i < kj; ++i) mn = tj[i] < mn ? tj[i] : mn;
                l.pmin[j] = mn;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            double dm = 0.0;
            for (int j = 0; j < m; ++j) dm = dm + (double)l.pmin[j];
            l.sc[0] = dm;
            double delta = ((double)dmax - dm) / (double)qmax;
            if (!((delta > 0.0) && isfinite(delta))) delta = 0.0;
            l.sc[1] = delta;
            *l.flag = dm >= (double)dmax;
        }
        __syncthreads();
        ok = *l.flag == 0;
        if (ok) {
            const double delta = l.sc[1];
#pragma unroll
            for (int k = 0; k < NE; ++k) {
                const int e = (int)threadIdx.x + k * bd;
                if (FIX || e < T) {
                    uint32_t qv = 0;
                    if (delta > 0.0) {
                        double x = floor(((double)l.tab[e] - (double)l.pmin[ed[k].j]) / delta);
                        qv = (x >= (double)qmax) ? (uint32_t)qmax : (uint32_t)x;
                    }
                    l.qt[e] = (uint16_t)qv;
                }
            }
            __syncthreads();
            build_gtab<KIND, QT>(L, l.qt, (QT *)l.gtab);
        }
    } else {
        ok = ivf_setup<KIND, QT>(L, edesc, cb, queries + q * d, coarse + (size_t)c * d, dmax, true, true, l);
    }
    if (!ok) {
        if (threadIdx.x == 0) counts[a] = 0;
        return;
    }
    const QT *gtab = (const QT *)l.gtab;
    const float fdelta = (float)l.sc[1], fdmin = (float)l.sc[0];
    uint64_t *slot = (uint64_t *)(wq + slots_off) + (size_t)a * cap_b;
    if (NE > 0 && KIND == SCAN_NIB8) {
        for (int64_t pb = 0; pb < npair; pb += (int64_t)PF * bd) {
            if (pb != 0) {
#pragma unroll
                for (int u = 0; u < PF; ++u) {
                    int64_t pi = pb + (int64_t)u * bd + threadIdx.x;
                    pi = pi < npair ? pi : npair - 1;
                    pp[u] = pairs[pi];
                }
            }
            uint32_t ord[2 * PF], id[2 * PF];
            bool pass[2 * PF], any = false;
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                const int64_t pi = pb + (int64_t)u * bd + threadIdx.x;
                const uint32_t k0 = sum8(gtab, pp[u].x, pp[u].y), k1 = sum8(gtab, pp[u].z, pp[u].w);
                const float d0 = fmaf((float)(k0 > (uint32_t)qmax ? (uint32_t)qmax : k0), fdelta, fdmin);
                const float d1 = fmaf((float)(k1 > (uint32_t)qmax ? (uint32_t)qmax : k1), fdelta, fdmin);
                ord[2 * u] = qadc_f2ord(d0);
                ord[2 * u + 1] = qadc_f2ord(d1);
                pass[2 * u] = pi < npair && d0 <= thr0;
                pass[2 * u + 1] = pi < npair && d1 <= thr0;
                any = any || pass[2 * u] || pass[2 * u + 1];
            }
            if (__ballot(any) != 0) {
#pragma unroll
                for (int u = 0; u < 2 * PF; ++u) {
                    const int64_t pos = lo2 + 2 * (pb + (int64_t)(u >> 1) * bd + threadIdx.x) + (u & 1);
                    id[u] = pass[u] ? (uint32_t)list_ids[pos] : 0u;
                }
                slot_append_multi<2 * PF>(pass, ord, id, slot, (uint32_t)cap_b, &s_count);
            }
        }
        // the codes outside the pairs: position lo if it is odd, position hi-1 if one is left over
        if (threadIdx.x < QADC_WAVE) {
            int64_t pos = -1;
            if (threadIdx.x == 0 && lo2 != lo) pos = lo;
            if (threadIdx.x == 1 && lo2 + 2 * npair < hi) pos = hi - 1;
            uint32_t o = 0, idv = 0;
            bool ps = false;
            if (pos >= 0) {
                const uint32_t key = key_at<KIND, QT>(L, gtab, list_codes, pos);
                const float dist = fmaf((float)key, fdelta, fdmin);
                o = qadc_f2ord(dist);
                ps = dist <= thr0;
                idv = ps ? (uint32_t)list_ids[pos] : 0u;
            }
            slot_append(ps, o, idv, slot, (uint32_t)cap_b, &s_count);
        }
    } else {
        for (int64_t base = lo; base < hi; base += 4 * bd) {
            uint32_t key[4], ord[4], id[4];
            bool pass[4], any = false;
            keys_batch<KIND, QT, 4>(L, gtab, list_codes, base + threadIdx.x, bd, hi, key);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float dist = fmaf((float)(key[u] == 0xffffffffu ? 0u : key[u]), fdelta, fdmin);
                ord[u] = qadc_f2ord(dist);
                pass[u] = key[u] != 0xffffffffu && dist <= thr0;
                any = any || pass[u];
            }
            if (__ballot(any) != 0) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t p = base + u * bd + threadIdx.x;
                    id[u] = pass[u] ? (uint32_t)list_ids[p] : 0u;
                }
                slot_append_multi<4>(pass, ord, id, slot, (uint32_t)cap_b, &s_count);
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) counts[a] = s_count;  // uncapped: > cap_b tells k_ivf_final about the overflow
}

// --------------------------------------------------------- k_ivf_scan_mq ---
// One pass over a list for up to four of the queries that probe it (Section 2.1.3: every
// (query, cell) pair has its own tables, but the codes of the cell are the same for all).
// For calls with several (query, probe) pairs per cell, 16 x 4-bit codes over equal sub-spaces
// and 8-bit tables.  The pairs are sorted by cell exactly (one bucket per cell), the pairs of a
// cell are cut into groups of at most four, and a block of four waves serves one group: wave w
// builds the residual tables and the quantizer of the group's w-th pair exactly as k_ivf_scan
// does, writes its byte-indexed group tables as field w of 8-byte entries {u16 q0..q3} in LDS,
// and then all four waves scan the list once: one 8-byte read per code byte serves the four
// pairs.  Every pair keeps its own slot list and count, so the selection is unchanged.
#define IVF_MQ 4
// A group: up to four (query, probe) pairs of one cell, in one 32-byte record so that a block's
// loads depend on one another two deep (record; then queries, list bounds and so on).
struct __align__(16) IvfGroup {
    uint32_t pair[IVF_MQ];  // q * nprobe + a; entries beyond k repeat the first
    int32_t cell;
    int32_t k;
    int32_t pad[2];
};
struct IvfMqLds {                      // behind the interleaved tables (which start at LDS address 0)
    float zres[IVF_MQ][128];
    float pmin[IVF_MQ][16];
    uint16_t qt[IVF_MQ][256];
    double sc[IVF_MQ][2];              // d_min, delta
    unsigned long long slot[IVF_MQ];   // slot list of the pair
    float thr[IVF_MQ];                 // pruning bound; -inf: nothing passes (no pair, or list skipped)
    uint32_t count[IVF_MQ];
    uint32_t *counts_out[IVF_MQ];
    int flag[IVF_MQ];
};
#define IVF_MQ_TAB_BYTES (8 * 256 * 8)

// the four packed sums of one 64-bit code: lo = {q0, q1}, hi = {q2, q3} (16 bits each; eight
// addends of at most 510 cannot carry)
__device__ __forceinline__ void ivf_mq_sums(uint32_t w0, uint32_t w1, uint32_t three, uint32_t &lo, uint32_t &hi) {
    const uint2 e0 = mq_entry<0>(0, w0, three), e1 = mq_entry<1>(1, w0, three);
    const uint2 e2 = mq_entry<2>(2, w0, three), e3 = mq_entry<3>(3, w0, three);
    const uint2 e4 = mq_entry<0>(4, w1, three), e5 = mq_entry<1>(5, w1, three);
    const uint2 e6 = mq_entry<2>(6, w1, three), e7 = mq_entry<3>(7, w1, three);
    lo = e0.x + e1.x + e2.x + e3.x + e4.x + e5.x + e6.x + e7.x;
    hi = e0.y + e1.y + e2.y + e3.y + e4.y + e5.y + e6.y + e7.y;
}

template <int DS>
__global__ void __launch_bounds__(256)
k_ivf_scan_mq(const float *__restrict__ cb, const float *__restrict__ coarse,
              const int64_t *__restrict__ list_offsets, const uint8_t *__restrict__ list_codes,
              const int32_t *__restrict__ list_ids, const float *__restrict__ queries, int nprobe,
              char *__restrict__ ws, size_t per_query, size_t counts_off, size_t slots_off, int cap_b,
              const IvfGroup *__restrict__ gdesc, const uint32_t *__restrict__ ngroups) {
    extern __shared__ __align__(16) unsigned char smem[];  // tables at LDS address 0 (no static LDS here)
    IvfMqLds &S = *(IvfMqLds *)(smem + IVF_MQ_TAB_BYTES);
    if (blockIdx.x >= *ngroups) return;
    constexpr int d = 16 * DS;
    constexpr uint32_t qmax = 255;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const IvfGroup *gp = gdesc + blockIdx.x;
    const int k = gp->k;  // 1..4 pairs, all of cell c, whose list is not empty
    const int c = gp->cell;
    const bool act = w < k;
    const uint32_t pair = gp->pair[w];  // (idle waves mirror pair 0, store nothing)
    const int64_t lo = list_offsets[c], hi = list_offsets[c + 1];
    const size_t q = pair / (uint32_t)nprobe;
    const int a = (int)(pair % (uint32_t)nprobe);
    char *wq = ws + q * per_query;
    const IvfState *st = (const IvfState *)wq;
    const float dmax = st->dmax, thr0 = st->thr0;
    // the first codes of the list, requested now and used after the set-up
    constexpr int PF = 2;
    const int64_t lo2 = (lo + 1) & ~(int64_t)1;
    const int64_t npair = hi > lo2 ? (hi - lo2) >> 1 : 0;
    const uint4 *__restrict__ pairs = (const uint4 *)(list_codes + lo2 * 8);
    uint4 pp[PF];
    if (npair > 0) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            int64_t pi = (int64_t)u * 256 + threadIdx.x;
            pi = pi < npair ? pi : npair - 1;
            pp[u] = pairs[pi];
        }
    }
    // codebook values of this lane's four table entries e = lane + 64 i
    float cv[4][DS];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int t = 0; t < DS; ++t) cv[i][t] = cb[(lane + 64 * i) * DS + t];
    for (int i = lane; i < d; i += 64) S.zres[w][i] = __fsub_rn(queries[q * d + i], coarse[(size_t)c * d + i]);
    if (lane == 0) {
        S.count[w] = 0;
        S.slot[w] = (unsigned long long)((uint64_t *)(wq + slots_off) + (size_t)a * cap_b);
        S.counts_out[w] = (uint32_t *)(wq + counts_off) + a;
    }
    __syncthreads();
    // eq. (1), terms in ascending dimension order; 16 adjacent lanes hold one sub-quantizer
    float tv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = lane + 64 * i;
        const float *zz = S.zres[w] + (e >> 4) * DS;
        float acc = 0.0f;
#pragma unroll
        for (int t = 0; t < DS; ++t) {
            const float diff = __fsub_rn(zz[t], cv[i][t]);
            acc = __fadd_rn(acc, __fmul_rn(diff, diff));
        }
        tv[i] = acc;
        float mn = acc;
#pragma unroll
        for (int sft = 1; sft < 16; sft <<= 1) {
            const float o = __shfl_xor(mn, sft, QADC_WAVE);
            mn = o < mn ? o : mn;
        }
        if ((lane & 15) == 0) S.pmin[w][e >> 4] = mn;
    }
    __syncthreads();
    if (lane == 0) {
        double dm = 0.0;
        for (int j = 0; j < 16; ++j) dm = dm + (double)S.pmin[w][j];
        double delta = ((double)dmax - dm) / (double)qmax;
        if (!((delta > 0.0) && isfinite(delta))) delta = 0.0;
        const int skip = dm >= (double)dmax;  // Section 3.4: nothing in this list is closer than d_max
        S.sc[w][0] = dm;
        S.sc[w][1] = delta;
        S.flag[w] = skip;
        S.thr[w] = (act && !skip) ? thr0 : -INFINITY;
    }
    __syncthreads();
    {
        const double delta = S.sc[w][1];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = lane + 64 * i;
            uint32_t qv = 0;
            if (delta > 0.0) {
                const double x = floor(((double)tv[i] - (double)S.pmin[w][e >> 4]) / delta);
                qv = (x >= (double)qmax) ? qmax : (uint32_t)x;
            }
            S.qt[w][e] = (uint16_t)qv;
        }
    }
    __syncthreads();
    // the interleaved tables: entry (g, byte) holds, for each of the four pairs, low-nibble entry +
    // high-nibble entry; a thread writes whole 8-byte entries
    {
        uint2 *tab = (uint2 *)smem;
        for (int x = threadIdx.x; x < 8 * 256; x += 256) {
            const int g = x >> 8, byte = x & 255;
            const int il = 32 * g + (byte & 15), ih = 32 * g + 16 + (byte >> 4);
            uint32_t v[IVF_MQ];
#pragma unroll
            for (int j = 0; j < IVF_MQ; ++j) v[j] = (uint32_t)S.qt[j][il] + (uint32_t)S.qt[j][ih];
            tab[x] = make_uint2(v[0] | (v[1] << 16), v[2] | (v[3] << 16));
        }
    }
    __syncthreads();
    // ---- one pass over the list for the four pairs
    float fdelta[IVF_MQ], fdmin[IVF_MQ], thr[IVF_MQ];
#pragma unroll
    for (int j = 0; j < IVF_MQ; ++j) {
        fdelta[j] = (float)S.sc[j][1];
        fdmin[j] = (float)S.sc[j][0];
        thr[j] = S.thr[j];
    }
    const uint32_t three = 3;
    for (int64_t pb = 0; pb < npair; pb += (int64_t)PF * 256) {
        // the next round of codes is requested before this one is looked up
        uint4 cur[PF];
#pragma unroll
        for (int u = 0; u < PF; ++u) cur[u] = pp[u];
        if (pb + (int64_t)PF * 256 < npair) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                int64_t pi = pb + (int64_t)(PF + u) * 256 + threadIdx.x;
                pi = pi < npair ? pi : npair - 1;
                pp[u] = pairs[pi];
            }
        }
        uint32_t slo[2 * PF], shi[2 * PF];
        bool valid[PF];
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            valid[u] = pb + (int64_t)u * 256 + threadIdx.x < npair;
            ivf_mq_sums(cur[u].x, cur[u].y, three, slo[2 * u], shi[2 * u]);
            ivf_mq_sums(cur[u].z, cur[u].w, three, slo[2 * u + 1], shi[2 * u + 1]);
        }
        uint32_t ord[IVF_MQ][2 * PF];
        bool pass[IVF_MQ][2 * PF], any = false;
#pragma unroll
        for (int j = 0; j < IVF_MQ; ++j)
#pragma unroll
            for (int u = 0; u < 2 * PF; ++u) {
                const uint32_t sum = j == 0 ? (slo[u] & 0xffffu) : (j == 1 ? (slo[u] >> 16) : (j == 2 ? (shi[u] & 0xffffu) : (shi[u] >> 16)));
                const float dist = fmaf((float)(sum > qmax ? qmax : sum), fdelta[j], fdmin[j]);
                ord[j][u] = qadc_f2ord(dist);
                pass[j][u] = valid[u >> 1] && dist <= thr[j];
                any = any || pass[j][u];
            }
        if (__ballot(any) != 0) {
            uint32_t id[2 * PF];
#pragma unroll
            for (int u = 0; u < 2 * PF; ++u) {
                const int64_t pos = lo2 + 2 * (pb + (int64_t)(u >> 1) * 256 + threadIdx.x) + (u & 1);
                bool need = false;
#pragma unroll
                for (int j = 0; j < IVF_MQ; ++j) need = need || pass[j][u];
                id[u] = need ? (uint32_t)list_ids[pos] : 0u;
            }
#pragma unroll
            for (int j = 0; j < IVF_MQ; ++j)
                slot_append_multi<2 * PF>(pass[j], ord[j], id, (uint64_t *)S.slot[j], (uint32_t)cap_b, &S.count[j]);
        }
    }
    // the codes outside the 16-byte pairs: position lo if it is odd, position hi-1 if one is left over
    if (threadIdx.x < QADC_WAVE) {
        int64_t pos = -1;
        if (threadIdx.x == 0 && lo2 != lo) pos = lo;
        if (threadIdx.x == 1 && lo2 + 2 * npair < hi) pos = hi - 1;
        uint32_t l2 = 0, h2 = 0, idv = 0;
        if (pos >= 0) {
            const uint2 cw = *(const uint2 *)(list_codes + pos * 8);
            ivf_mq_sums(cw.x, cw.y, three, l2, h2);
            idv = (uint32_t)list_ids[pos];
        }
#pragma unroll
        for (int j = 0; j < IVF_MQ; ++j) {
            const uint32_t sum = j == 0 ? (l2 & 0xffffu) : (j == 1 ? (l2 >> 16) : (j == 2 ? (h2 & 0xffffu) : (h2 >> 16)));
            const float dist = fmaf((float)(sum > qmax ? qmax : sum), fdelta[j], fdmin[j]);
            slot_append(pos >= 0 && dist <= thr[j], qadc_f2ord(dist), idv, (uint64_t *)S.slot[j], (uint32_t)cap_b, &S.count[j]);
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < k) *S.counts_out[threadIdx.x] = S.count[threadIdx.x];  // uncapped, as in k_ivf_scan
}

// Sorting the pairs by cell exactly, and cutting each cell's pairs into groups of IVF_MQ.
// start[c] / gstart[c] = pairs / groups in cells before c (c = 0 .. nb, nb = K + 1 buckets: the
// last holds the pairs without a list, which get no groups); cnt is cleared to serve as fill
// cursors.  Two launches of nb / 1024 blocks: sums per block of 1024 buckets, then every block
// adds up the sums before it and scans its own buckets.
__device__ __forceinline__ uint32_t ivf_groups_of(uint32_t pairs, int bucket, int nb) {
    return bucket < nb - 1 ? (pairs + IVF_MQ - 1) / IVF_MQ : 0u;
}
// block-wide sums of two values (1024 threads); the result reaches every thread
__device__ __forceinline__ void ivf_block_sum2(uint32_t &a, uint32_t &b, uint32_t (*wsum)[16]) {
    for (int sft = QADC_WAVE / 2; sft > 0; sft >>= 1) {
        a += __shfl_xor(a, sft, QADC_WAVE);
        b += __shfl_xor(b, sft, QADC_WAVE);
    }
    if (threadIdx.x % QADC_WAVE == 0) {
        wsum[0][threadIdx.x / QADC_WAVE] = a;
        wsum[1][threadIdx.x / QADC_WAVE] = b;
    }
    __syncthreads();
    a = 0, b = 0;
    for (int w = 0; w < 16; ++w) {
        a += wsum[0][w];
        b += wsum[1][w];
    }
    __syncthreads();
}
__global__ void __launch_bounds__(1024)
k_pair_block_sums(const uint32_t *__restrict__ cnt, int nb, uint32_t *__restrict__ bsum) {
    __shared__ uint32_t wsum[2][16];
    const int i = blockIdx.x * 1024 + threadIdx.x;
    uint32_t s = i < nb ? cnt[i] : 0u;
    uint32_t g = i < nb ? ivf_groups_of(s, i, nb) : 0u;
    ivf_block_sum2(s, g, wsum);
    if (threadIdx.x == 0) {
        bsum[2 * blockIdx.x] = s;
        bsum[2 * blockIdx.x + 1] = g;
    }
}
__global__ void __launch_bounds__(1024)
k_pair_scan_groups(uint32_t *__restrict__ cnt, uint32_t *__restrict__ start, uint32_t *__restrict__ gstart, int nb,
                   const uint32_t *__restrict__ bsum) {
    __shared__ uint32_t wsum[2][16];
    // pairs and groups in the blocks before this one (gridDim.x <= 1024 blocks: K < 2^20)
    uint32_t ps = (int)threadIdx.x < (int)blockIdx.x ? bsum[2 * threadIdx.x] : 0u;
    uint32_t pg = (int)threadIdx.x < (int)blockIdx.x ? bsum[2 * threadIdx.x + 1] : 0u;
    ivf_block_sum2(ps, pg, wsum);
    const int i = blockIdx.x * 1024 + threadIdx.x;
    const uint32_t v = i < nb ? cnt[i] : 0u;
    const uint32_t gv = i < nb ? ivf_groups_of(v, i, nb) : 0u;
    const int wave = threadIdx.x / QADC_WAVE, lane = threadIdx.x % QADC_WAVE;
    const uint32_t is = qadc_wave_incl_scan(v), ig = qadc_wave_incl_scan(gv);
    if (lane == QADC_WAVE - 1) {
        wsum[0][wave] = is;
        wsum[1][wave] = ig;
    }
    __syncthreads();
    uint32_t bs = ps + is - v, bg = pg + ig - gv;
    for (int w = 0; w < wave; ++w) {
        bs += wsum[0][w];
        bg += wsum[1][w];
    }
    if (i < nb) {
        start[i] = bs;
        gstart[i] = bg;
        cnt[i] = 0;
    }
    if (i == nb - 1) {
        start[nb] = bs + v;
        gstart[nb] = bg + gv;  // number of groups
    }
}

// One thread per cell writes the cell's group records; the pairs
// without a list get their slot counts cleared (no block will visit them).  cnt holds the
// cells' pair counts again after k_pair_fill.
__global__ void __launch_bounds__(256)
k_group_fill(const uint32_t *__restrict__ cnt, const uint32_t *__restrict__ start,
             const uint32_t *__restrict__ gstart, const uint32_t *__restrict__ order, int K, int nprobe,
             char *__restrict__ ws, size_t per_query, size_t counts_off, IvfGroup *__restrict__ gdesc) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c < K) {
        const uint32_t n = cnt[c], s0 = start[c];
        uint32_t g = gstart[c];
        for (uint32_t i = 0; i < n; i += IVF_MQ, ++g) {
            IvfGroup gr;
            gr.k = (int32_t)(n - i < IVF_MQ ? n - i : (uint32_t)IVF_MQ);
            gr.cell = c;
            gr.pad[0] = gr.pad[1] = 0;
#pragma unroll
            for (int j = 0; j < IVF_MQ; ++j) gr.pair[j] = order[s0 + i + (j < gr.k ? (uint32_t)j : 0u)];
            gdesc[g] = gr;
        }
    }
    const uint32_t nodd = cnt[K], sodd = start[K];
    for (uint32_t i = blockIdx.x * 256 + threadIdx.x; i < nodd; i += gridDim.x * 256) {
        const uint32_t pair = order[sodd + i];
        ((uint32_t *)(ws + (size_t)(pair / (uint32_t)nprobe) * per_query + counts_off))[pair % (uint32_t)nprobe] = 0;
    }
}

// ------------------------------------------------------------ k_ivf_final ---
// Rank candidates (ordered-float distance << 32 | id) and write the first R.
__device__ inline void ivf_rank_and_write(const uint64_t *A, int na, int R, int32_t *ids,
                                          float *dist) {
    for (int i = threadIdx.x; i < na; i += blockDim.x) {
        const uint64_t mine = A[i];
        int rank = 0;
        for (int j = 0; j < na; ++j) rank += (A[j] < mine) ? 1 : 0;
        if (rank < R) {
            ids[rank] = (int32_t)(uint32_t)mine;
            dist[rank] = qadc_ord2f((uint32_t)(mine >> 32));
        }
    }
    for (int r = (na < R ? na : R) + threadIdx.x; r < R; r += blockDim.x) {
        ids[r] = -1;
        dist[r] = INFINITY;
    }
}

// Exact selection by one block over every code of the probed, unskipped lists:
// byte-wise radix selection of the R-th smallest 64-bit (distance, id) word,
// regenerating the stream once per byte, then one collecting pass.
template <int KIND, typename QT>
__device__ inline int ivf_exact_select(const DevLayout *L, const EntryDesc *edesc, const float *cb,
                                       const float *coarse,
                                       const int64_t *list_offsets, const uint8_t *list_codes,
                                       const int32_t *list_ids, const float *z,
                                       const int32_t *probes, int nprobe, int K, float dmax, int R,
                                       const IvfLds &l, uint64_t *A, uint32_t *hist, uint32_t *sh) {
    uint64_t prefix = 0, mask = 0;
    uint32_t kk = 0;
    // pass 8 counts the stream, passes 7..0 select a byte each, pass -1 collects
    for (int pass = 8; pass >= -1; --pass) {
        for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
        if (threadIdx.x == 0) sh[2] = 0;
        __syncthreads();
        for (int a = 0; a < nprobe; ++a) {
            const int c = probes[a];
            if (c < 0 || c >= K) continue;
            const int64_t lo = list_offsets[c], hi = list_offsets[c + 1];
            if (hi == lo) continue;
            if (!ivf_setup<KIND, QT>(L, edesc, cb, z, coarse + (size_t)c * L->d, dmax, true, true, l)) continue;
            const QT *gtab = (const QT *)l.gtab;
            const float fdelta = (float)l.sc[1], fdmin = (float)l.sc[0];
            for (int64_t p = lo + threadIdx.x; p < hi; p += blockDim.x) {
                const uint32_t key = key_at<KIND, QT>(L, gtab, list_codes, p);
                const uint64_t item = ((uint64_t)qadc_f2ord(fmaf((float)key, fdelta, fdmin)) << 32) |
                                      (uint64_t)(uint32_t)list_ids[p];
                if (pass == 8) {
                    atomicAdd(&hist[0], 1u);
                } else if (pass >= 0) {
                    if ((item & mask) == prefix) atomicAdd(&hist[(item >> (8 * pass)) & 255u], 1u);
                } else if (item <= prefix) {
                    uint32_t pos = atomicAdd(&sh[2], 1u);
                    if (pos < (uint32_t)R) A[pos] = item;
                }
            }
            __syncthreads();
        }
        __syncthreads();
        if (pass == 8) {
            const uint32_t total = hist[0];
            kk = total < (uint32_t)R ? total : (uint32_t)R;
            if (kk == 0) return 0;
        } else if (pass >= 0) {
            if (threadIdx.x == 0) {
                uint32_t run = 0;
                int b = 0;
                for (; b < 255; ++b) {
                    if (run + hist[b] >= kk) break;
                    run += hist[b];
                }
                sh[0] = (uint32_t)b;
                sh[1] = kk - run;
            }
            __syncthreads();
            prefix |= (uint64_t)sh[0] << (8 * pass);
            mask |= (uint64_t)255u << (8 * pass);
            kk = sh[1];
        }
        __syncthreads();
    }
    const uint32_t got = sh[2];
    return (int)(got < (uint32_t)R ? got : (uint32_t)R);
}

// SMALL: blocks of 256 threads that can rank IVF_SMALL_CAP candidates (short result lists):
// a quarter of the LDS and of the wave slots, so that several queries share a CU.
#define IVF_SMALL_CAP 2048
template <int KIND, typename QT, bool SMALL>
__global__ void __launch_bounds__(SMALL ? 256 : 1024)
k_ivf_final(const DevLayout *__restrict__ L, const EntryDesc *__restrict__ edesc,
            const float *__restrict__ cb,
            const float *__restrict__ coarse, const int64_t *__restrict__ list_offsets,
            const uint8_t *__restrict__ list_codes, const int32_t *__restrict__ list_ids,
            const float *__restrict__ queries, const int32_t *__restrict__ probe_ids, int nprobe,
            int K, int R, char *__restrict__ ws, size_t per_query, size_t counts_off, size_t slots_off,
            int cap_b, int32_t *__restrict__ out_ids, float *__restrict__ out_dist) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int CAP = SMALL ? IVF_SMALL_CAP : FINAL_CAP;
    __shared__ uint32_t hist[256];
    __shared__ uint32_t whist[SMALL ? 4 : 16][256];  // one histogram per wave
    __shared__ uint32_t sh[32];
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t off[1024 + 1];  // one slot list per probed cell, nprobe <= 1024
    uint64_t *A = (uint64_t *)smem;  // CAP entries
    const size_t q = blockIdx.x;
    char *wq = ws + q * per_query;
    IvfState *st = (IvfState *)wq;
    const uint32_t *counts = (const uint32_t *)(wq + counts_off);
    const uint64_t *slots = (const uint64_t *)(wq + slots_off);
    const float blo = st->lo, bscale = st->scale;
    FinalShared S;
    S.hist = hist;
    S.whist = whist;
    S.sh = sh;
    S.wsum = wsum;
    S.off = off;
    int na = 0;
    const bool slow = gather_select(
        counts, slots, nprobe, cap_b, R,
        [blo, bscale](uint64_t c) { return dist_bin(qadc_ord2f((uint32_t)(c >> 32)), blo, bscale); }, A,
        CAP, S, na);
    if (slow) {
        IvfLds l;
        ivf_carve(L, smem + CAP * 8, sizeof(QT), l);
        na = ivf_exact_select<KIND, QT>(L, edesc, cb, coarse, list_offsets, list_codes, list_ids,
                                        queries + q * L->d, probe_ids + q * nprobe, nprobe, K,
                                        st->dmax, R, l, A, hist, sh);
        __syncthreads();
    }
    ivf_rank_and_write(A, na, R, out_ids + q * R, out_dist + q * R);
}

// ------------------------------------------------------------ k_ivf_tight ---
// The search with a bound that tightens from list to list (Section 3.5: a scanned vector is
// kept when it is closer than the worst of the R candidates held; Section 3.4: that worst
// distance is the largest the quantizer has to represent).  One block per query walks the
// probed lists in probe order; list l is quantized against
//     cur = min(d_max, R-th smallest distance among the candidates of the lists before l),
// a list whose d_min is not below cur is skipped, and a code whose sum saturates is no
// candidate.  The block holds the candidates as (ordered float distance << 32 | stored id) in
// LDS; whenever the buffer runs full, and at the end of every list that added to it, the R
// smallest are kept and the rest dropped: a dropped word is above R held ones, so it can
// neither be a result nor move a later R-th smallest.
#define TIGHT_CAP 4096       // words of the candidate buffer ...
#define TIGHT_CAP_SMALL 2048 // ... and for R <= TIGHT_CAP_SMALL - TIGHT_U * 256: half the LDS, more blocks per CU
#define TIGHT_U 4  // codes per thread between two looks at the fill level
#define TIGHT_PC 64  // probes whose cells and list bounds are fetched together

// k-th smallest (k = 1..na) of the different 64-bit words A[0..na), byte by byte from the top.
__device__ inline uint64_t tight_kth(const uint64_t *A, int na, int k, uint32_t *hist, uint32_t *sh) {
    uint64_t prefix = 0, mask = 0;
    uint32_t kk = (uint32_t)k;
    for (int pass = 7; pass >= 0; --pass) {
        for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < na; i += blockDim.x) {
            const uint64_t w = A[i];
            if ((w & mask) == prefix) atomicAdd(&hist[(uint32_t)(w >> (8 * pass)) & 255u], 1u);
        }
        __syncthreads();
        if (threadIdx.x < QADC_WAVE) {
            // lane l owns bins 4l .. 4l+3; the bin of the kk-th lies in the first lane whose
            // running total reaches kk (the total over all lanes is at least kk)
            const uint4 h = *(const uint4 *)&hist[4 * threadIdx.x];
            const uint32_t sum = h.x + h.y + h.z + h.w;
            const uint32_t incl = qadc_wave_incl_scan(sum);
            const unsigned long long reach = __ballot(incl >= kk);
            if (reach != 0 && (int)threadIdx.x == __ffsll(reach) - 1) {
                uint32_t run = incl - sum, b = 4 * threadIdx.x;
                if (run + h.x < kk) {
                    run += h.x, ++b;
                    if (run + h.y < kk) {
                        run += h.y, ++b;
                        if (run + h.z < kk) run += h.z, ++b;
                    }
                }
                sh[0] = b;
                sh[1] = kk - run;
            }
        }
        __syncthreads();
        prefix |= (uint64_t)sh[0] << (8 * pass);
        mask |= (uint64_t)255u << (8 * pass);
        kk = sh[1];
        __syncthreads();
    }
    return prefix;
}

// Keep the R smallest of A[0..na), na > R; returns the R-th smallest.  *count becomes R.
template <int CAP>
__device__ inline uint64_t tight_keep(uint64_t *A, int na, int R, uint32_t *hist, uint32_t *sh,
                                      uint32_t *count) {
    const uint64_t thr = tight_kth(A, na, R, hist, sh);
    constexpr int PER = CAP / 256;
    uint64_t mine[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int i = (int)threadIdx.x + u * 256;
        mine[u] = i < na ? A[i] : ~0ull;
    }
    if (threadIdx.x == 0) *count = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PER; ++u)
        if (mine[u] <= thr) {
            const uint32_t pos = atomicAdd(count, 1u);
            if (pos < CAP) A[pos] = mine[u];
        }
    __syncthreads();
    return thr;
}

// The same for na <= 256 (one word per thread), R <= na: every thread counts the words below its
// own (equal words, which only repeated stored ids give, count by position: the counts are
// the ranks), the R smallest go to A[rank], in order, and the word of rank R - 1 is returned.
// nsorted: A[0..nsorted) are in order already (the R words this function left), so that only
// the words added since are compared one by one: an old word's rank is its position plus the
// new words below it, a new word's the old words not above it (binary search) plus the new
// words below it.  With R = 100 nearly every list adds a few candidates to the R held.
__device__ inline uint64_t tight_keep_small(uint64_t *A, int na, int R, int nsorted, uint32_t *sh,
                                            uint32_t *count) {
    const bool have = (int)threadIdx.x < na;
    const uint64_t mine = have ? A[threadIdx.x] : ~0ull;
    int rank = 0;
    if (nsorted > 0) {
        if ((int)threadIdx.x < nsorted) {
            rank = (int)threadIdx.x;
        } else if (have) {
            int lo = 0, hi = nsorted;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (A[mid] <= mine) lo = mid + 1; else hi = mid;
            }
            rank = lo;
        }
#pragma unroll 4
        for (int j = nsorted; j < na; ++j) {
            const uint64_t o = A[j];
            rank += (o < mine || (o == mine && j < (int)threadIdx.x)) ? 1 : 0;
        }
    } else {
        // four words per step as two 16-byte reads (every lane reads the same address), two steps
        // in flight; words past na (stale, inside the buffer) count as the largest value
#pragma unroll 2
        for (int j = 0; j < na; j += 4) {
            const uint4 p0 = *(const uint4 *)&A[j], p1 = *(const uint4 *)&A[j + 2];
            const uint64_t other[4] = {((uint64_t)p0.y << 32) | p0.x, ((uint64_t)p0.w << 32) | p0.z,
                                       ((uint64_t)p1.y << 32) | p1.x, ((uint64_t)p1.w << 32) | p1.z};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint64_t o = j + k < na ? other[k] : ~0ull;
                rank += (o < mine || (o == mine && j + k < (int)threadIdx.x)) ? 1 : 0;
            }
        }
    }
    __syncthreads();  // every thread has read A
    if (have && rank < R) A[rank] = mine;
    if (have && rank == R - 1) {
        sh[2] = (uint32_t)mine;
        sh[3] = (uint32_t)(mine >> 32);
    }
    if (threadIdx.x == 0) *count = (uint32_t)R;
    __syncthreads();
    return ((uint64_t)sh[3] << 32) | sh[2];
}

template <int KIND, typename QT, int CAP, int DS = 0>
__global__ void __launch_bounds__(256)
k_ivf_tight(const DevLayout *__restrict__ L, const EntryDesc *__restrict__ edesc,
            const float *__restrict__ cb, const float *__restrict__ coarse,
            const int64_t *__restrict__ list_offsets, const uint8_t *__restrict__ list_codes,
            const int32_t *__restrict__ list_ids, const float *__restrict__ queries,
            const int32_t *__restrict__ probe_ids, int nprobe, int K, int R,
            const char *__restrict__ ws, size_t per_query, int32_t *__restrict__ out_ids,
            float *__restrict__ out_dist) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ __align__(16) uint32_t hist[256];
    __shared__ uint32_t sh[8];
    __shared__ uint32_t s_na;
    __shared__ int64_t s_plo[TIGHT_PC];
    __shared__ int32_t s_plen[TIGHT_PC], s_pcell[TIGHT_PC];
    uint64_t *A = (uint64_t *)smem;  // CAP words
    IvfLds l;
    ivf_carve(L, smem + CAP * 8, sizeof(QT), l);
    const size_t q = blockIdx.x;
    const IvfState *st = (const IvfState *)(ws + q * per_query);
    const int32_t *probes = probe_ids + q * nprobe;
    const int bd = 256;
    const uint32_t qmax = (uint32_t)L->qmax;
    float cur = st->dmax;
    uint64_t pthr = ~0ull;  // words above it are beyond R held candidates
    int na = 0;
    int nsorted = 0;  // A[0..nsorted) are in ascending order
    if (threadIdx.x == 0) s_na = 0;
    __syncthreads();
    // The block's time is a chain of memory round trips, so as few as possible are left in it:
    // cells and list bounds of TIGHT_PC probes are fetched at once, and (64-bit codes of
    // nibbles) a list's first codes are requested before its set-up and every further batch
    // before the previous one is looked up.
    for (int a0 = 0; a0 < nprobe; a0 += TIGHT_PC) {
        __syncthreads();  // the previous chunk's entries have been used
        if (threadIdx.x < TIGHT_PC) {
            const int a = a0 + (int)threadIdx.x;
            const int c = a < nprobe ? probes[a] : -1;
            const bool valid = c >= 0 && c < K;
            const int64_t lo = valid ? list_offsets[c] : 0, hi = valid ? list_offsets[c + 1] : 0;
            s_pcell[threadIdx.x] = c;
            s_plo[threadIdx.x] = lo;
            s_plen[threadIdx.x] = (int32_t)(hi - lo);  // a list is shorter than 2^31 codes
        }
        __syncthreads();
        const int a1 = nprobe - a0 < TIGHT_PC ? nprobe - a0 : TIGHT_PC;
        for (int ai = 0; ai < a1; ++ai) {
            if (s_plen[ai] <= 0) continue;
            const int c = s_pcell[ai];
            const int64_t lo = s_plo[ai], hi = lo + s_plen[ai];
            uint2 wnext[TIGHT_U];
            auto request = [&](int64_t base) {  // codes past the end: the last one again
#pragma unroll
                for (int u = 0; u < TIGHT_U; ++u) {
                    int64_t id = base + (int64_t)u * bd + threadIdx.x;
                    id = id < hi ? id : hi - 1;
                    wnext[u] = *(const uint2 *)(list_codes + id * 8);
                }
            };
            if constexpr (KIND == SCAN_NIB8) request(lo);
            bool ok;
            if constexpr (DS > 0) {
                ok = ivf_setup_fix<DS>(cb, queries + q * (16 * DS), coarse + (size_t)c * (16 * DS), cur, true, qmax, l);
                if (ok) build_gtab<KIND, QT>(L, l.qt, (QT *)l.gtab);
            } else {
                ok = ivf_setup<KIND, QT>(L, edesc, cb, queries + q * L->d, coarse + (size_t)c * L->d, cur, true, true, l);
            }
            if (!ok) continue;
            const QT *gtab = (const QT *)l.gtab;
            const float fdelta = (float)l.sc[1], fdmin = (float)l.sc[0];
            bool added = false;  // the list has added to the buffer (also if a full buffer was cut back since)
            for (int64_t base = lo; base < hi; base += TIGHT_U * bd) {
                if (na + TIGHT_U * bd > CAP) {  // na > R here: R <= CAP - TIGHT_U * 256
                    pthr = tight_keep<CAP>(A, na, R, hist, sh, &s_na);
                    na = R;
                    nsorted = 0;
                }
                const int na_old = na;
                uint32_t key[TIGHT_U];
                if constexpr (KIND == SCAN_NIB8) {
                    uint2 w[TIGHT_U];
#pragma unroll
                    for (int u = 0; u < TIGHT_U; ++u) w[u] = wnext[u];
                    if (base + TIGHT_U * bd < hi) request(base + TIGHT_U * bd);
#pragma unroll
                    for (int u = 0; u < TIGHT_U; ++u) {
                        const uint32_t sum = sum8(gtab, w[u].x, w[u].y);
                        key[u] = base + (int64_t)u * bd + threadIdx.x < hi ? (sum > qmax ? qmax : sum) : 0xffffffffu;
                    }
                } else {
                    keys_batch<KIND, QT, TIGHT_U>(L, gtab, list_codes, base + threadIdx.x, bd, hi, key);
                }
#pragma unroll
                for (int u = 0; u < TIGHT_U; ++u) {
                    if (key[u] == 0xffffffffu || key[u] >= qmax) continue;  // past the end, or saturated
                    const uint32_t o = qadc_f2ord(fmaf((float)key[u], fdelta, fdmin));
                    if (o > (uint32_t)(pthr >> 32)) continue;
                    const int64_t p = base + (int64_t)u * bd + threadIdx.x;
                    const uint64_t w = ((uint64_t)o << 32) | (uint64_t)(uint32_t)list_ids[p];
                    if (w <= pthr) {
                        const uint32_t pos = atomicAdd(&s_na, 1u);
                        if (pos < CAP) A[pos] = w;  // always, unless stored ids repeat
                    }
                }
                __syncthreads();
                na = (int)(s_na < CAP ? s_na : CAP);
                added = added || na != na_old;
                __syncthreads();  // every thread has read the fill level before the next batch adds to it
            }
            if (added && na >= R) {
                if (na <= 256) {
                    pthr = tight_keep_small(A, na, R, nsorted, sh, &s_na);
                    na = R;
                    nsorted = R;
                } else if (na > R) {
                    pthr = tight_keep<CAP>(A, na, R, hist, sh, &s_na);
                    na = R;
                    nsorted = 0;
                } else {
                    pthr = tight_kth(A, na, R, hist, sh);
                }
                const float worst = qadc_ord2f((uint32_t)(pthr >> 32));
                cur = worst < cur ? worst : cur;
            }
        }
    }
    ivf_rank_and_write(A, na, R, out_ids + q * R, out_dist + q * R);
}

// ------------------------------------------------------------------ host ---
template <typename K>
static int allow_lds(K kernel, size_t bytes) {
    if (bytes <= 48 * 1024) return PQ_OK;
    QADC_HIP_TRY(hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)bytes));
    return PQ_OK;
}

// 16 x 4 bits over equal sub-spaces of 4, 6 or 8 dimensions with 8-bit tables: that width, else 0
static int ivf_fixed_shape(const pq_index *idx) {
    const DevLayout &h = idx->h;
    const bool ok = h.kind == SCAN_NIB8 && h.acc_bits == 8 && h.m == 16 && h.T == 256 && h.ds_uniform > 0 &&
                    h.d == 16 * h.ds_uniform && (h.ds_uniform == 4 || h.ds_uniform == 6 || h.ds_uniform == 8);
    return ok ? h.ds_uniform : 0;
}

template <int KIND, typename QT>
static int launch_ivf(const pq_index *idx, const float *coarse, const int64_t *list_offsets,
                      const uint8_t *list_codes, const int32_t *list_ids, const float *queries,
                      int nq, const int32_t *probe_ids, int nprobe, int K, int want, int R,
                      int32_t *out_ids, float *out_dist, char *ws, const IvfPlan &p, uint32_t *sortws,
                      bool shared_lists, bool tighten, hipStream_t s) {
    // blocks in the order of the probed cells (see ivf_pair_bucket):
    // sortws = cnt[NB+1] | start[NB+1] | order[pairs]
    const uint32_t *order = nullptr;
    // fixed shape of k_ivf_scan's fast set-up and of k_ivf_scan_mq: 16 x 4 bits over equal
    // sub-spaces of 4, 6 or 8 dimensions, 8-bit tables
    const int dsf = (KIND == SCAN_NIB8 && sizeof(QT) == 1) ? ivf_fixed_shape(idx) : 0;
    const IvfGroup *gdesc = nullptr;
    const uint32_t *ngroups = nullptr;
    size_t max_groups = 0;
    // The sort's bucket counts are taken by k_ivf_calib (its blocks walk their probes anyway);
    // the counters are cleared before it and the rest of the sort follows it.
    uint32_t *pair_cnt = nullptr;
    int pair_nb = 0;
    const int64_t npairs = (int64_t)nq * nprobe;
    const int sort_kind = tighten || !sortws ? 0 : (shared_lists && dsf != 0 ? 2 : 1);
    if (sort_kind == 2) {
        // pairs sorted by cell exactly and cut into groups of four (see k_ivf_scan_mq):
        // sortws = cnt[K+2] | start[K+2] | gstart[K+2] | bsum[2 * 1024] | order[pairs] | (16-byte aligned) gdesc[pairs/4 + K + 1]
        const size_t nbw = (size_t)K + 2;
        hipLaunchKernelGGL(k_pair_zero, dim3((unsigned)((nbw + 255) / 256)), dim3(256), 0, s, sortws, (int)nbw);
        QADC_LAUNCH_CHECK("k_pair_zero");
        pair_cnt = sortws;
        pair_nb = K;
    } else if (sort_kind == 1) {
        const int NB = K < IVF_SORT_BUCKETS ? K : IVF_SORT_BUCKETS;
        hipLaunchKernelGGL(k_pair_zero, dim3((NB + 1 + 255) / 256), dim3(256), 0, s, sortws, NB + 1);
        QADC_LAUNCH_CHECK("k_pair_zero");
        pair_cnt = sortws;
        pair_nb = NB;
    }
    // pilot: as many codes as fit the calibration block's LDS next to its tables (the kernel's
    // own static arrays stay under 12 KB of the 160 KB), never fewer than the calibration codes;
    // a shorter pilot only gives a weaker (still valid) pruning bound
    int pilot_want = 4096 > 32 * R ? 4096 : 32 * R;
    const size_t lds_room = (size_t)(160 - 12) * 1024;
    const size_t lds_tabs = ivf_lds_bytes(idx->h, 2);
    if (lds_tabs + (size_t)want * 4 > lds_room) {
        qadc_set_error("ivf_adc_scan_topk: tables of %zu bytes and %d calibration codes exceed the "
                       "%zu bytes of LDS of the calibration kernel", lds_tabs, want, lds_room);
        return PQ_EINVAL;
    }
    if ((size_t)pilot_want > (lds_room - lds_tabs) / 4) pilot_want = (int)((lds_room - lds_tabs) / 4);
    if (pilot_want < want) pilot_want = want;
    const size_t lds_calib = lds_tabs + (size_t)pilot_want * 4;
    const size_t lds_scan = ivf_lds_bytes(idx->h, sizeof(QT));
    // short result lists: the small selection kernel (four lists per thread: nprobe <= 1024)
    const bool small_final = R <= IVF_SMALL_CAP / 8;
    const size_t lds_final = (small_final ? IVF_SMALL_CAP : FINAL_CAP) * 8 + lds_scan;
    int rc;
    constexpr bool NIB = KIND == SCAN_NIB8;
    if ((rc = allow_lds(k_ivf_scan<KIND, QT, 0>, lds_scan)) != PQ_OK) return rc;
    if ((rc = allow_lds(k_ivf_scan<KIND, QT, 1>, lds_scan)) != PQ_OK) return rc;
    if ((rc = allow_lds(k_ivf_scan<KIND, QT, 2>, lds_scan)) != PQ_OK) return rc;
    if ((rc = allow_lds(k_ivf_scan<KIND, QT, 4>, lds_scan)) != PQ_OK) return rc;
    if (small_final) {
        if ((rc = allow_lds(k_ivf_final<KIND, QT, true>, lds_final)) != PQ_OK) return rc;
    } else {
        if ((rc = allow_lds(k_ivf_final<KIND, QT, false>, lds_final)) != PQ_OK) return rc;
    }
#define QADC_IVF_CALIB(...)                                                                          \
    do {                                                                                             \
        if ((rc = allow_lds(k_ivf_calib<__VA_ARGS__>, lds_calib)) != PQ_OK) return rc;               \
        hipLaunchKernelGGL((k_ivf_calib<__VA_ARGS__>), dim3(nq), dim3(256), lds_calib, s, idx->dev,  \
                           idx->edesc, idx->codebooks, coarse, list_offsets, list_codes, queries,    \
                           probe_ids, nprobe, K, want, pilot_want, R, ws, p.per_query, pair_cnt,     \
                           pair_nb);                                                                 \
    } while (0)
    // (the fixed 16 x 4-bit shape has a set-up of its own)
    if (dsf == 4) QADC_IVF_CALIB(true, 4);
    else if (dsf == 6) QADC_IVF_CALIB(true, 6);
    else if (dsf == 8) QADC_IVF_CALIB(true, 8);
    else QADC_IVF_CALIB(NIB);
#undef QADC_IVF_CALIB
    QADC_LAUNCH_CHECK("k_ivf_calib");
    if (tighten) {
        static_assert(PQ_MAX_R + TIGHT_U * 256 <= TIGHT_CAP, "room for one batch above R candidates");
        const bool small_cap = R + TIGHT_U * 256 <= TIGHT_CAP_SMALL;
        const size_t lds_tight = (size_t)(small_cap ? TIGHT_CAP_SMALL : TIGHT_CAP) * 8 + lds_scan;
#define QADC_IVF_TIGHT1(...)                                                                         \
    do {                                                                                             \
        if ((rc = allow_lds(k_ivf_tight<__VA_ARGS__>, lds_tight)) != PQ_OK) return rc;               \
        hipLaunchKernelGGL((k_ivf_tight<__VA_ARGS__>), dim3(nq), dim3(256), lds_tight, s, idx->dev,  \
                           idx->edesc, idx->codebooks, coarse, list_offsets, list_codes, list_ids,   \
                           queries, probe_ids, nprobe, K, R, (const char *)ws, p.per_query, out_ids, \
                           out_dist);                                                                \
    } while (0)
#define QADC_IVF_TIGHT(KINDV, QTV, DSV)                                                              \
    do {                                                                                             \
        if (small_cap) QADC_IVF_TIGHT1(KINDV, QTV, TIGHT_CAP_SMALL, DSV);                            \
        else QADC_IVF_TIGHT1(KINDV, QTV, TIGHT_CAP, DSV);                                            \
    } while (0)
        if (KIND == SCAN_NIB8 && sizeof(QT) == 1 && dsf != 0) {
            if (dsf == 4) QADC_IVF_TIGHT(SCAN_NIB8, uint8_t, 4);
            else if (dsf == 6) QADC_IVF_TIGHT(SCAN_NIB8, uint8_t, 6);
            else QADC_IVF_TIGHT(SCAN_NIB8, uint8_t, 8);
        } else {
            QADC_IVF_TIGHT(KIND, QT, 0);
        }
#undef QADC_IVF_TIGHT1
#undef QADC_IVF_TIGHT
        QADC_LAUNCH_CHECK("k_ivf_tight");
        return PQ_OK;
    }
    if (sort_kind == 2) {
        const size_t nbw = (size_t)K + 2;
        uint32_t *cnt = sortws, *start = sortws + nbw, *gstart = sortws + 2 * nbw, *bsum = sortws + 3 * nbw;
        uint32_t *ord = bsum + 2048;
        IvfGroup *gd = (IvfGroup *)(((uintptr_t)(ord + npairs) + 15) & ~(uintptr_t)15);
        max_groups = (size_t)(npairs / IVF_MQ) + (size_t)K + 1;
        const unsigned scan_blocks = (unsigned)((K + 1 + 1023) / 1024);  // <= 1024: K < 2^20 is checked by the caller
        hipLaunchKernelGGL(k_pair_block_sums, dim3(scan_blocks), dim3(1024), 0, s, (const uint32_t *)cnt, K + 1, bsum);
        QADC_LAUNCH_CHECK("k_pair_block_sums");
        hipLaunchKernelGGL(k_pair_scan_groups, dim3(scan_blocks), dim3(1024), 0, s, cnt, start, gstart, K + 1,
                           (const uint32_t *)bsum);
        QADC_LAUNCH_CHECK("k_pair_scan_groups");
        hipLaunchKernelGGL(k_pair_fill, dim3((unsigned)((npairs + 255) / 256)), dim3(256), 0, s, probe_ids,
                           list_offsets, npairs, K, K, (const uint32_t *)start, cnt, ord);
        QADC_LAUNCH_CHECK("k_pair_fill");
        hipLaunchKernelGGL(k_group_fill, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, s, (const uint32_t *)cnt,
                           (const uint32_t *)start, (const uint32_t *)gstart, (const uint32_t *)ord, K, nprobe,
                           ws, p.per_query, p.counts_off, gd);
        QADC_LAUNCH_CHECK("k_group_fill");
        order = ord;
        gdesc = gd;
        ngroups = gstart + (K + 1);
    } else if (sort_kind == 1) {
        const int NB = pair_nb;
        uint32_t *cnt = sortws, *start = sortws + (NB + 1), *ord = sortws + 2 * (size_t)(NB + 1);
        hipLaunchKernelGGL(k_pair_scan, dim3(1), dim3(1024), 0, s, cnt, start, NB + 1);
        QADC_LAUNCH_CHECK("k_pair_scan");
        hipLaunchKernelGGL(k_pair_fill, dim3((unsigned)((npairs + 255) / 256)), dim3(256), 0, s, probe_ids,
                           list_offsets, npairs, K, NB, (const uint32_t *)start, cnt, ord);
        QADC_LAUNCH_CHECK("k_pair_fill");
        order = ord;
    }
    if (gdesc) {
        const size_t lds_mq = IVF_MQ_TAB_BYTES + sizeof(IvfMqLds);
        static int mq_static_lds = -1;  // k_ivf_scan_mq addresses its tables from LDS address 0
        if (mq_static_lds < 0) {
            hipFuncAttributes a4, a6, a8;
            if (hipFuncGetAttributes(&a4, (const void *)k_ivf_scan_mq<4>) != hipSuccess ||
                hipFuncGetAttributes(&a6, (const void *)k_ivf_scan_mq<6>) != hipSuccess ||
                hipFuncGetAttributes(&a8, (const void *)k_ivf_scan_mq<8>) != hipSuccess) {
                qadc_set_error("k_ivf_scan_mq: hipFuncGetAttributes failed");
                return PQ_EHIP;
            }
            mq_static_lds = (int)(a4.sharedSizeBytes + a6.sharedSizeBytes + a8.sharedSizeBytes);
        }
        if (mq_static_lds != 0) {
            qadc_set_error("k_ivf_scan_mq: static LDS of %d bytes (its tables must start at LDS address 0)", mq_static_lds);
            return PQ_EHIP;
        }
#define QADC_IVF_MQ(DSV)                                                                             \
    hipLaunchKernelGGL((k_ivf_scan_mq<DSV>), dim3((unsigned)max_groups), dim3(256), lds_mq, s,       \
                       idx->codebooks, coarse, list_offsets, list_codes, list_ids, queries, nprobe,  \
                       ws, p.per_query, p.counts_off, p.slots_off, p.cap_b, gdesc, ngroups)
        if (dsf == 4) QADC_IVF_MQ(4); else if (dsf == 6) QADC_IVF_MQ(6); else QADC_IVF_MQ(8);
#undef QADC_IVF_MQ
        QADC_LAUNCH_CHECK("k_ivf_scan_mq");
    } else {
    const int scan_threads = (int)qadc_option(PQ_OPT_IVF_THREADS);
    // table entries per thread: the low-latency set-up holds up to four in registers
    const int ne = idx->h.T <= scan_threads ? 1 : (idx->h.T <= 2 * scan_threads ? 2 : (idx->h.T <= 4 * scan_threads ? 4 : 0));
#define QADC_IVF_SCAN(NEV)                                                                          \
    hipLaunchKernelGGL((k_ivf_scan<KIND, QT, NEV>), dim3(nprobe, nq), dim3(scan_threads), lds_scan, s, \
                       idx->dev, idx->edesc, idx->codebooks, coarse, list_offsets, list_codes,     \
                       list_ids, queries, probe_ids, nprobe, K, R, ws, p.per_query, p.counts_off,  \
                       p.slots_off, p.cap_b, order)
    // 16 x 4 bits over equal sub-spaces with 8-bit tables, at the default block size: the
    // fixed-shape set-up
    const int dsfix = scan_threads == 128 ? dsf : 0;
#define QADC_IVF_SCAN_FIX(DSV)                                                                      \
    hipLaunchKernelGGL((k_ivf_scan<SCAN_NIB8, uint8_t, 2, DSV>), dim3(nprobe, nq), dim3(128), lds_scan, s, \
                       idx->dev, idx->edesc, idx->codebooks, coarse, list_offsets, list_codes,     \
                       list_ids, queries, probe_ids, nprobe, K, R, ws, p.per_query, p.counts_off,  \
                       p.slots_off, p.cap_b, order)
    if (dsfix != 0) {
        if (KIND == SCAN_NIB8 && sizeof(QT) == 1) {  // (the macro names the types itself)
            if (dsfix == 4) QADC_IVF_SCAN_FIX(4); else if (dsfix == 6) QADC_IVF_SCAN_FIX(6); else QADC_IVF_SCAN_FIX(8);
        }
    } else if (ne == 1) QADC_IVF_SCAN(1); else if (ne == 2) QADC_IVF_SCAN(2); else if (ne == 4) QADC_IVF_SCAN(4); else QADC_IVF_SCAN(0);
#undef QADC_IVF_SCAN_FIX
#undef QADC_IVF_SCAN
    QADC_LAUNCH_CHECK("k_ivf_scan");
    }
    if (small_final)
        hipLaunchKernelGGL((k_ivf_final<KIND, QT, true>), dim3(nq), dim3(256), lds_final, s, idx->dev,
                           idx->edesc, idx->codebooks, coarse, list_offsets, list_codes, list_ids, queries,
                           probe_ids, nprobe, K, R, ws, p.per_query, p.counts_off, p.slots_off, p.cap_b,
                           out_ids, out_dist);
    else
        hipLaunchKernelGGL((k_ivf_final<KIND, QT, false>), dim3(nq), dim3(1024), lds_final, s, idx->dev,
                           idx->edesc, idx->codebooks, coarse, list_offsets, list_codes, list_ids, queries,
                           probe_ids, nprobe, K, R, ws, p.per_query, p.counts_off, p.slots_off, p.cap_b,
                           out_ids, out_dist);
    QADC_LAUNCH_CHECK("k_ivf_final");
    return PQ_OK;
}

static size_t ivf_sort_bytes(int nq, int nprobe, int K) {
    const size_t nb = K < IVF_SORT_BUCKETS ? (size_t)K : (size_t)IVF_SORT_BUCKETS;
    return ((2 * (nb + 1) + (size_t)nq * (size_t)nprobe) * sizeof(uint32_t) + 255) & ~(size_t)255;
}
// the sort by cell and the groups of k_ivf_scan_mq
static size_t ivf_group_bytes(int nq, int nprobe, int K) {
    const size_t pairs = (size_t)nq * (size_t)nprobe;
    return ((3 * ((size_t)K + 2) + 2048 + pairs) * sizeof(uint32_t) + 16 +
            (pairs / IVF_MQ + (size_t)K + 1) * sizeof(IvfGroup) + 255) & ~(size_t)255;
}
// Half-pairs per cell from which one pass per list for four pairs beats a block per pair
// (C4 shape, measured: 1 pair per cell -7 %, 2 pairs +9 %, 3.9 pairs +22 %, 9.8 pairs +32 %)
#define IVF_SHARED_MIN_HALF_PAIRS_PER_CELL 3

extern "C" size_t ivf_sorted_workspace_bytes(const pq_index_t *idx, int nq, int nprobe, int R, int K) {
    if (!idx || nq < 0 || nprobe < 1 || R < 1 || K < 1) return 0;
    const size_t base = (qadc_ivf_plan(idx, nq, nprobe, R).total + 255) & ~(size_t)255;
    const size_t a = ivf_sort_bytes(nq, nprobe, K), b = ivf_group_bytes(nq, nprobe, K);
    return base + (a > b ? a : b) + 256;
}

static int ivf_search(const char *name, bool tighten, const pq_index_t *idx, const float *coarse_centroids,
                      int K, const int64_t *list_offsets, const uint8_t *list_codes,
                      const int32_t *list_ids, const float *queries, int nq, const int32_t *probe_ids,
                      int nprobe, int t, int R, int32_t *out_ids, float *out_dist, void *workspace,
                      size_t workspace_bytes, void *stream) {
    if (!idx || nq < 0 || K < 1 || nprobe < 1 || nprobe > 1024) {
        qadc_set_error("%s: bad handle, nq, K or nprobe (1..1024)", name);
        return PQ_EINVAL;
    }
    if (R < 1 || R > PQ_MAX_R || t < 1) {
        qadc_set_error("%s: need 1<=R<=%d and t>=1 (got R=%d t=%d)", name, PQ_MAX_R, R, t);
        return PQ_EINVAL;
    }
    const int64_t want = t > 4 * (int64_t)R ? t : 4 * (int64_t)R;
    if (want > PQ_MAX_T_EFF) {
        qadc_set_error("%s: max(t,4R)=%lld exceeds %d", name, (long long)want, PQ_MAX_T_EFF);
        return PQ_EINVAL;
    }
    if (nq == 0) return PQ_OK;
    if (nq > 65535) {
        qadc_set_error("%s: at most 65535 queries per call (got %d)", name, nq);
        return PQ_EINVAL;
    }
    if (!coarse_centroids || !list_offsets || !list_codes || !list_ids || !queries || !probe_ids ||
        !out_ids || !out_dist || !workspace) {
        qadc_set_error("%s: null pointer", name);
        return PQ_EINVAL;
    }
    if (((uintptr_t)list_codes & 15u) != 0 || ((uintptr_t)workspace & 255u) != 0) {
        qadc_set_error("%s: list_codes must be 16-byte and workspace 256-byte aligned", name);
        return PQ_EINVAL;
    }
    const IvfPlan p = qadc_ivf_plan(idx, nq, nprobe, R);
    if (workspace_bytes < p.total) {
        qadc_set_error("%s: workspace of %zu bytes, need %zu", name, workspace_bytes, p.total);
        return PQ_ENOMEM;
    }
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    // With the larger workspace of ivf_sorted_workspace_bytes, and enough (query, probe) pairs
    // for cells to be probed more than once, the scan runs in the order of the probed cells.
    const size_t base_bytes = (p.total + 255) & ~(size_t)255;
    uint32_t *sortws = nullptr;
    if (!tighten && (int64_t)nq * nprobe * 4 >= (int64_t)K &&
        workspace_bytes >= base_bytes + ivf_sort_bytes(nq, nprobe, K))
        sortws = (uint32_t *)(ws + base_bytes);
    // many pairs per cell (or the option says always): one pass over a list serves four pairs
    const int64_t shared_opt = qadc_option(PQ_OPT_IVF_SHARED_LISTS);
    const bool shared_lists = !tighten && shared_opt != 0 && ivf_fixed_shape(idx) != 0 && K < (1 << 20) &&
                              workspace_bytes >= base_bytes + ivf_group_bytes(nq, nprobe, K) &&
                              (shared_opt == 2 || 2 * (int64_t)nq * nprobe >= (int64_t)IVF_SHARED_MIN_HALF_PAIRS_PER_CELL * K);
    if (shared_lists) sortws = (uint32_t *)(ws + base_bytes);
    const bool u8 = idx->h.acc_bits == 8;
#define QADC_GO(KIND, QT)                                                                          \
    return launch_ivf<KIND, QT>(idx, coarse_centroids, list_offsets, list_codes, list_ids, queries, \
                                nq, probe_ids, nprobe, K, (int)want, R, out_ids, out_dist, ws, p, sortws, shared_lists, tighten, s)
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

extern "C" int ivf_adc_scan_topk(const pq_index_t *idx, const float *coarse_centroids, int K,
                                 const int64_t *list_offsets, const uint8_t *list_codes,
                                 const int32_t *list_ids, const float *queries, int nq,
                                 const int32_t *probe_ids, int nprobe, int t, int R,
                                 int32_t *out_ids, float *out_dist, void *workspace,
                                 size_t workspace_bytes, void *stream) {
    return ivf_search("ivf_adc_scan_topk", false, idx, coarse_centroids, K, list_offsets, list_codes,
                      list_ids, queries, nq, probe_ids, nprobe, t, R, out_ids, out_dist, workspace,
                      workspace_bytes, stream);
}

extern "C" int ivf_adc_scan_topk_tightening(const pq_index_t *idx, const float *coarse_centroids, int K,
                                            const int64_t *list_offsets, const uint8_t *list_codes,
                                            const int32_t *list_ids, const float *queries, int nq,
                                            const int32_t *probe_ids, int nprobe, int t, int R,
                                            int32_t *out_ids, float *out_dist, void *workspace,
                                            size_t workspace_bytes, void *stream) {
    return ivf_search("ivf_adc_scan_topk_tightening", true, idx, coarse_centroids, K, list_offsets,
                      list_codes, list_ids, queries, nq, probe_ids, nprobe, t, R, out_ids, out_dist,
                      workspace, workspace_bytes, stream);
}
