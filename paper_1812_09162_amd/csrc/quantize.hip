// pq_quantize_tables: the query-time distance quantizer of Section 3.4.
#include <math.h>

#include "qadc_device.h"

// One block per query.
//   1. p_min(j), d_min = sum_j p_min(j) (fp64, ascending j)
//   2. float ADC (eq. (2), fp32, ascending j) of the first t_eff codes; d_max is
//      the k-th smallest of them, k = min(R, t_eff)
//   3. delta = (d_max - d_min)/q_max; q = min(q_max, floor((p - p_min)/delta))
//   4. key_bound: k-th smallest quantized key of the same t_eff codes
__global__ void __launch_bounds__(256)
k_quantize(const DevLayout *__restrict__ L, const float *__restrict__ tables,
           const uint8_t *__restrict__ codes, int t_eff, int k, void *__restrict__ qtables,
           pq_qparams_t *__restrict__ qparams) {
    extern __shared__ unsigned char smem[];
    const int T = L->T, m = L->m, cs = L->cs, qmax = L->qmax;
    float *tab = (float *)smem;
    uint32_t *ord = (uint32_t *)(tab + T);
    uint32_t *hist = ord + (t_eff > 0 ? t_eff : 1);
    uint32_t *sel = hist + 256;
    float *pmin = (float *)(sel + 2);
    uint16_t *qt = (uint16_t *)(pmin + PQ_MAX_M);
    __shared__ double s_dmin, s_delta;
    __shared__ float s_dmax;

    const size_t q = blockIdx.x;
    for (int e = threadIdx.x; e < T; e += blockDim.x) tab[e] = tables[q * T + e];
    __syncthreads();
    if ((int)threadIdx.x < m) {
        const int j = threadIdx.x;
        const int kj = 1 << L->nbits[j];
        const float *tj = tab + L->toff[j];
        float mn = tj[0];
        for (int i = 1; i < kj; ++i) mn = tj[i] < mn ? tj[i] : mn;
        pmin[j] = mn;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double dm = 0.0;
        for (int j = 0; j < m; ++j) dm = dm + (double)pmin[j];
        s_dmin = dm;
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
    float dmax = INFINITY;
    if (t_eff > 0) dmax = qadc_ord2f(qadc_block_kth_u32(ord, t_eff, k, 4, hist, sel));
    if (threadIdx.x == 0) {
        double delta = ((double)dmax - s_dmin) / (double)qmax;
        bool ok = (delta > 0.0) && isfinite(delta);
        s_delta = ok ? delta : 0.0;
        s_dmax = dmax;
    }
    __syncthreads();
    const double delta = s_delta;
    for (int e = threadIdx.x; e < T; e += blockDim.x) {
        int j = 0;
        while (j + 1 < m && (int)L->toff[j + 1] <= e) ++j;
        uint32_t qv = 0;
        if (delta > 0.0) {
            double x = floor(((double)tab[e] - (double)pmin[j]) / delta);
            qv = (x >= (double)qmax) ? (uint32_t)qmax : (uint32_t)x;
        }
        qt[e] = (uint16_t)qv;
        if (L->acc_bits == 8)
            ((uint8_t *)qtables)[q * T + e] = (uint8_t)qv;
        else
            ((uint16_t *)qtables)[q * T + e] = (uint16_t)qv;
    }
    __syncthreads();
    // quantized keys of the calibration codes -> inclusive bound on the R-th best key
    for (int p = threadIdx.x; p < t_eff; p += blockDim.x) {
        const uint8_t *code = codes + (size_t)p * cs;
        uint32_t acc = 0;
        for (int j = 0; j < m; ++j)
            acc += qt[L->toff[j] + qadc_extract_sub(code, L->bitoff[j], L->nbits[j])];
        ord[p] = acc > (uint32_t)qmax ? (uint32_t)qmax : acc;
    }
    __syncthreads();
    uint32_t bound = (uint32_t)qmax;
    if (t_eff > 0 && k <= t_eff) bound = qadc_block_kth_u32(ord, t_eff, k, 2, hist, sel);
    if (threadIdx.x == 0) {
        pq_qparams_t prm;
        prm.d_min = s_dmin;
        prm.delta = s_delta;
        prm.d_max = s_dmax;
        prm.key_bound = bound;
        qparams[q] = prm;
    }
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
    int64_t want = t > 4 * (int64_t)R ? t : 4 * (int64_t)R;
    if (want > PQ_MAX_T_EFF) {
        qadc_set_error("pq_quantize_tables: max(t,4R)=%lld exceeds %d", (long long)want, PQ_MAX_T_EFF);
        return PQ_EINVAL;
    }
    if (nq == 0) return PQ_OK;
    if (!tables || !qtables || !qparams || (n > 0 && !codes)) {
        qadc_set_error("pq_quantize_tables: null pointer");
        return PQ_EINVAL;
    }
    // a code with fewer than R predecessors can never be displaced: calibrate on min(n, want)
    int t_eff = (int)(n < want ? n : want);
    int k = R < t_eff ? R : t_eff;
    size_t lds = (size_t)idx->h.T * 4 + (size_t)(t_eff > 0 ? t_eff : 1) * 4 + 256 * 4 + 2 * 4 +
                 PQ_MAX_M * 4 + (size_t)idx->h.T * 2 + 16;
    hipLaunchKernelGGL(k_quantize, dim3(nq), dim3(256), lds, (hipStream_t)stream, idx->dev, tables,
                       codes, t_eff, k, qtables, qparams);
    QADC_LAUNCH_CHECK("k_quantize");
    return PQ_OK;
}
