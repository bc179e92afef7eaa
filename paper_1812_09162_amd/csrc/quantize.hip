// pq_quantize_tables: the query-time distance quantizer of Section 3.4.
#include <math.h>
#include <stdlib.h>

#include "scan_device.h"

// One block per query.
//   0. (fused form only) the float table from the query, eq. (1)
//   1. p_min(j), d_min = sum_j p_min(j) (fp64, ascending j)
//   2. float ADC (eq. (2), fp32, ascending j) of the first t_eff codes; d_max is
//      the k-th smallest of them, k = min(R, t_eff)
//   3. delta = (d_max - d_min)/q_max; q = min(q_max, floor((p - p_min)/delta))
//   4. key_bound: the k-th smallest quantized key among the first `pilot` codes
//      (pilot >= t_eff).  It bounds the R-th best key of the whole list from
//      above and lets the scan drop almost every code with one compare.
// `queries` non-null: tables are computed here (and stored to tables_out if
// that is non-null); otherwise they are read from tables_in.
template <int KIND, typename QT>
__global__ void __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(4, 4)))
k_quantize(const DevLayout *__restrict__ L, const float *__restrict__ cb,
           const float *__restrict__ queries, const float *__restrict__ tables_in,
           float *__restrict__ tables_out, const uint8_t *__restrict__ codes, int t_eff, int k,
           int pilot, void *__restrict__ qtables, pq_qparams_t *__restrict__ qparams,
           char *__restrict__ gtab_out, size_t gtab_stride) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int T = L->T, m = L->m, cs = L->cs, qmax = L->qmax, d = L->d;
    float *tab = (float *)smem;
    uint32_t *ord = (uint32_t *)(tab + T);                    // max(t_eff, d) words
    const int nord = (t_eff > d ? t_eff : d) > 0 ? (t_eff > d ? t_eff : d) : 1;
    float *pmin = (float *)(ord + nord);
    uint16_t *qt = (uint16_t *)(pmin + PQ_MAX_M);
    uint8_t *esub = (uint8_t *)(qt + T);
    QT *gtab = (QT *)(smem + (((size_t)T * 4 + (size_t)nord * 4 + PQ_MAX_M * 4 + (size_t)T * 3 + 15) &
                              ~(size_t)15));
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sel[2];
    __shared__ double s_dmin, s_delta;
    __shared__ float s_dmax;

    const size_t q = blockIdx.x;
    if (queries) {
        float *zs = (float *)ord;  // the query lives where the ADC sums go later
        for (int i = threadIdx.x; i < d; i += blockDim.x) zs[i] = queries[q * d + i];
        qadc_build_entry_map(L, esub);
        for (int e = threadIdx.x; e < T; e += blockDim.x) {
            const int j = esub[e];
            const int i = e - L->toff[j];
            const int ds = L->dsub[j];
            const float *c = cb + L->cboff[j] + (size_t)i * ds;
            const float *z = zs + L->dimoff[j];
            float acc = 0.0f;
            for (int l = 0; l < ds; ++l) {
                float diff = __fsub_rn(z[l], c[l]);
                acc = __fadd_rn(acc, __fmul_rn(diff, diff));
            }
            tab[e] = acc;
            if (tables_out) tables_out[q * T + e] = acc;
        }
        __syncthreads();
    } else {
        for (int e = threadIdx.x; e < T; e += blockDim.x) tab[e] = tables_in[q * T + e];
        qadc_build_entry_map(L, esub);
    }
    if ((int)threadIdx.x < m) {
        const int j = threadIdx.x;
        const int kj = 1 << L->nbits[j];
        const float *tj = tab + L->toff[j];
        float mn = tj[0];
        for (int i = 1; i < kj; ++i) mn = tj[i] < mn ? tj[i] : mn;
        pmin[j] = mn;
    }
    // float ADC of the calibration codes
    for (int p = threadIdx.x; p < t_eff; p += blockDim.x) {
        const uint8_t *code = codes + (size_t)p * cs;
        float s = 0.0f;
        for (int j = 0; j < m; ++j)
            s = __fadd_rn(s, tab[L->toff[j] + qadc_extract_sub(code, L->bitoff[j], L->nbits[j])]);
        ord[p] = qadc_f2ord(s);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double dm = 0.0;
        for (int j = 0; j < m; ++j) dm = dm + (double)pmin[j];
        s_dmin = dm;
    }
    float dmax = INFINITY;
    if (t_eff > 0) dmax = qadc_ord2f(qadc_block_kth_u32(ord, t_eff, k, 4, hist, sel));
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
        if (sizeof(QT) == 1)
            ((uint8_t *)qtables)[q * T + e] = (uint8_t)qv;
        else
            ((uint16_t *)qtables)[q * T + e] = (uint16_t)qv;
    }
    __syncthreads();
    // Pilot: the k-th smallest quantized key of the first `pilot` codes by histogram
    // selection.  The bound is tightened in stages (1/8 of the codes, then the rest)
    // and only keys within the current bound are counted, so that the histogram
    // atomics stay few and spread out.  16-bit keys: high byte first, then the low
    // byte among the keys that share the selected high byte.
    uint32_t bound = (uint32_t)qmax;
    if (pilot > 0 || gtab_out) {
        build_gtab<KIND, QT>(L, qt, gtab);
        if (gtab_out) {  // hand the prepared group tables to the scan kernel
            QT *dst = (QT *)(gtab_out + q * gtab_stride);
            for (int e = threadIdx.x; e < L->gtab_len; e += blockDim.x) dst[e] = gtab[e];
        }
    }
    if (pilot > 0) {
        const bool wide = sizeof(QT) != 1;
        const int stage1 = pilot / 8 > 4 * k ? pilot / 8 : pilot;
        uint32_t kstar = 0, below = 0;
        for (int level = 0; level < (wide ? 2 : 1); ++level) {
            for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
            uint32_t cut = 255;  // bins above `cut` cannot hold the k-th key and are not counted
            __syncthreads();
            int lo = 0;
            for (int stage = 0; stage < 2 && lo < pilot; ++stage) {
                const int hi = stage == 0 ? stage1 : pilot;
                // count one key (0xffffffff = none) in the histogram of this level
                auto count_key = [&](uint32_t key) {
                    uint32_t bin = 0xffffffffu;  // not counted
                    if (key != 0xffffffffu) {
                        if (!wide)
                            bin = key;
                        else if (level == 0)
                            bin = key >> 8;
                        else if ((key >> 8) == kstar)
                            bin = key & 255u;
                    }
                    // the top bin collects every saturated key: count it once per wave
                    const uint64_t top = __ballot(bin == 255u);
                    if (top != 0 && cut == 255u && __lane_id() == 0)
                        atomicAdd(&hist[255], (uint32_t)__popcll(top));
                    if (bin < 255u && bin <= cut) atomicAdd(&hist[bin], 1u);
                };
                if (KIND == SCAN_NIB8) {
                    // double-buffered: the loads of the next batch fly while this one is looked up
                    const int step = 8 * (int)blockDim.x;
                    uint2 cur[8], nxt[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        int id = lo + u * (int)blockDim.x + (int)threadIdx.x;
                        id = id < hi ? id : hi - 1;
                        cur[u] = *(const uint2 *)(codes + (size_t)id * 8);
                    }
                    for (int base = lo; base < hi; base += step) {
                        if (base + step < hi) {
#pragma unroll
                            for (int u = 0; u < 8; ++u) {
                                int id = base + step + u * (int)blockDim.x + (int)threadIdx.x;
                                id = id < hi ? id : hi - 1;
                                nxt[u] = *(const uint2 *)(codes + (size_t)id * 8);
                            }
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const int id = base + u * (int)blockDim.x + (int)threadIdx.x;
                            const uint32_t sm = sum8(gtab, cur[u].x, cur[u].y);
                            count_key(id < hi ? (sm > (uint32_t)qmax ? (uint32_t)qmax : sm) : 0xffffffffu);
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) cur[u] = nxt[u];
                    }
                } else {
                    for (int base = lo; base < hi; base += 8 * (int)blockDim.x) {
                        uint32_t key[8];
                        keys_batch<KIND, QT, 8>(L, gtab, codes, (int64_t)base + threadIdx.x,
                                                blockDim.x, (int64_t)hi, key);
#pragma unroll
                        for (int u = 0; u < 8; ++u) count_key(key[u]);
                    }
                }
                __syncthreads();
                if (threadIdx.x < QADC_WAVE) qadc_wave_select_bin(hist, (uint32_t)k, below, sel);
                __syncthreads();
                cut = sel[0];
                lo = hi;
                __syncthreads();
            }
            kstar = (level == 0) ? sel[0] : ((kstar << 8) | sel[0]);
            below = sel[1];
            __syncthreads();
        }
        bound = kstar;
    }
    if (threadIdx.x == 0) {
        pq_qparams_t prm;
        prm.d_min = s_dmin;
        prm.delta = s_delta;
        prm.d_max = s_dmax;
        prm.key_bound = bound;
        qparams[q] = prm;
    }
}

static int64_t pilot_default() {
    static int64_t v = -1;
    if (v < 0) {
        const char *e = getenv("QADC_PILOT");
        v = e ? atoll(e) : 65536;
        if (v < 0) v = 0;
    }
    return v;
}

static size_t quantize_lds(const DevLayout &h, int t_eff, size_t esz) {
    const size_t nord = (size_t)((t_eff > h.d ? t_eff : h.d) > 0 ? (t_eff > h.d ? t_eff : h.d) : 1);
    return (((size_t)h.T * 4 + nord * 4 + PQ_MAX_M * 4 + (size_t)h.T * 3 + 15) & ~(size_t)15) +
           (size_t)h.gtab_len * esz;
}

template <int KIND, typename QT>
static int launch_quantize(const pq_index *idx, const float *queries, const float *tables_in,
                           float *tables_out, int nq, const uint8_t *codes, int t_eff, int k,
                           int pilot, void *qtables, pq_qparams_t *qparams, char *gtab_out,
                           size_t gtab_stride, hipStream_t s) {
    const size_t lds = quantize_lds(idx->h, t_eff, sizeof(QT));
    if (lds > 48 * 1024)
        QADC_HIP_TRY(hipFuncSetAttribute((const void *)k_quantize<KIND, QT>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL((k_quantize<KIND, QT>), dim3(nq), dim3(1024), lds, s, idx->dev,
                       idx->codebooks, queries, tables_in, tables_out, codes, t_eff, k, pilot,
                       qtables, qparams, gtab_out, gtab_stride);
    QADC_LAUNCH_CHECK("k_quantize");
    return PQ_OK;
}

// Shared by pq_quantize_tables (queries == null) and the fused search call.
int qadc_quantize_launch(const pq_index *idx, const float *queries, const float *tables_in,
                         float *tables_out, int nq, const uint8_t *codes, int64_t n, int t, int R,
                         void *qtables, pq_qparams_t *qparams, char *gtab_out, size_t gtab_stride,
                         hipStream_t s) {
    const int64_t want = t > 4 * (int64_t)R ? t : 4 * (int64_t)R;
    const int t_eff = (int)(n < want ? n : want);
    const int k = R < t_eff ? R : t_eff;
    int64_t pil = pilot_default();
    if (pil < 64 * (int64_t)R) pil = 64 * (int64_t)R;
    if (pil < t_eff) pil = t_eff;
    if (pil > n) pil = n;
    const int pilot = (int)pil;
    const bool u8 = idx->h.acc_bits == 8;
#define QADC_GO(KIND, QT)                                                                        \
    return launch_quantize<KIND, QT>(idx, queries, tables_in, tables_out, nq, codes, t_eff, k, \
                                     pilot, qtables, qparams, gtab_out, gtab_stride, s)
    switch (idx->h.kind) {
        case SCAN_NIB8:
            if (u8) QADC_GO(SCAN_NIB8, uint8_t); else QADC_GO(SCAN_NIB8, uint16_t);
        case SCAN_NIB16:
            if (u8) QADC_GO(SCAN_NIB16, uint8_t); else QADC_GO(SCAN_NIB16, uint16_t);
        case SCAN_W64:
            if (u8) QADC_GO(SCAN_W64, uint8_t); else QADC_GO(SCAN_W64, uint16_t);
        case SCAN_C5:
            if (u8) QADC_GO(SCAN_C5, uint8_t); else QADC_GO(SCAN_C5, uint16_t);
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
                                nullptr, 0, (hipStream_t)stream);
}
