// pq_compute_tables: float distance tables, eq. (1) of Section 2.1.3.
#include "qadc_device.h"

// One block per query.  Entry (j, i) = sum over the dims of sub-vector j of
// (z - c)^2, fp32, ascending dimension, separate subtract / multiply / add so
// that the result does not depend on FMA contraction.
__global__ void __launch_bounds__(256)
k_tables(const DevLayout *__restrict__ L, const float *__restrict__ cb,
         const float *__restrict__ queries, float *__restrict__ tables) {
    extern __shared__ float zs[];
    const int d = L->d, T = L->T;
    uint8_t *esub = (uint8_t *)(zs + d);
    const size_t q = blockIdx.x;
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
        tables[q * T + e] = acc;
    }
}

extern "C" int pq_compute_tables(const pq_index_t *idx, const float *queries, int nq, float *tables,
                                 void *stream) {
    if (!idx || nq < 0) {
        qadc_set_error("pq_compute_tables: bad handle or nq");
        return PQ_EINVAL;
    }
    if (nq == 0) return PQ_OK;
    if (!queries || !tables) {
        qadc_set_error("pq_compute_tables: null pointer");
        return PQ_EINVAL;
    }
    hipLaunchKernelGGL(k_tables, dim3(nq), dim3(256), idx->h.d * sizeof(float) + idx->h.T, (hipStream_t)stream,
                       idx->dev, idx->codebooks, queries, tables);
    QADC_LAUNCH_CHECK("k_tables");
    return PQ_OK;
}
