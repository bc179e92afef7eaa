// pq_encode: vectors -> packed codes (Section 2.1.2: each sub-vector is replaced by the index of
// its nearest centroid; Section 2.1.1: behind an inverted index the residual x - centroid is
// encoded; Section 3.3: the sub-codes are packed as a little-endian bit stream).
//
// The distance of sub-vector j to centroid i is the table entry D^j[i] of eq. (1) for z = x:
// fp32, dimensions ascending, separate subtract / multiply / add.  Sub-code j is the index of
// the smallest distance, the lowest index among equals.
//
// One block of 256 threads encodes 64 vectors, staged (minus the shift) in LDS; wave w takes the
// sub-quantizers w, w+4, ... and lane v the vector v, so that centroid values are uniform across
// a wave: codebooks of up to 16 KB are read from memory with scalar loads (they stay in the
// scalar cache), larger ones are staged in LDS when they fit (one word broadcast to 64 lanes).
// Sub-spaces of up to 8 dimensions are unrolled.  A second step packs the sub-codes.
#include "qadc_device.h"

#define ENC_VB 64  // vectors per block

// Nearest of kj centroids of DS dimensions (rows of c) to the sub-vector xv: eq. (1) term by
// term, the lowest index among equal distances.
template <int DS>
__device__ __forceinline__ void enc_nearest(const float *xv, const float *c, int kj, float &best,
                                            int &besti) {
    float xr[DS];
#pragma unroll
    for (int l = 0; l < DS; ++l) xr[l] = xv[l];
#pragma unroll 4
    for (int i = 0; i < kj; ++i) {
        float acc = 0.0f;
#pragma unroll
        for (int l = 0; l < DS; ++l) {
            const float diff = __fsub_rn(xr[l], c[i * DS + l]);
            acc = __fadd_rn(acc, __fmul_rn(diff, diff));
        }
        if (i == 0 || acc < best) {
            best = acc;
            besti = i;
        }
    }
}

__global__ void __launch_bounds__(256)
k_encode(const DevLayout *__restrict__ L, const float *__restrict__ cb,
         const float *__restrict__ x, int64_t n, const float *__restrict__ shift_rows,
         const int32_t *__restrict__ shift_ids, uint8_t *__restrict__ codes, int cb_floats) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int d = L->d, m = L->m, cs = L->cs;
    const int ldx = d | 1;  // odd row stride: lanes of a wave (consecutive vectors) hit distinct banks
    float *xs = (float *)smem;                             // [ENC_VB][ldx]
    float *cbs = xs + (size_t)ENC_VB * ldx;                 // [cb_floats] (0 if they do not fit)
    uint8_t *sub = (uint8_t *)(cbs + cb_floats);            // [ENC_VB][m]
    const int64_t v0 = (int64_t)blockIdx.x * ENC_VB;
    const int nv = n - v0 < ENC_VB ? (int)(n - v0) : ENC_VB;

    for (int e = threadIdx.x; e < nv * d; e += blockDim.x) {
        const int v = e / d, l = e - v * d;
        float val = x[(size_t)v0 * d + e];
        if (shift_rows) val = __fsub_rn(val, shift_rows[(size_t)shift_ids[v0 + v] * d + l]);
        xs[v * ldx + l] = val;
    }
    for (int e = threadIdx.x; e < cb_floats; e += blockDim.x) cbs[e] = cb[e];
    __syncthreads();

    // the wave index as a scalar: sub-quantizer, widths and codebook addresses are then uniform
    // values, and codebook entries read from memory come through the scalar cache
    const int v = threadIdx.x % ENC_VB, w = __builtin_amdgcn_readfirstlane(threadIdx.x / ENC_VB);
    // `c0` = the codebooks, in LDS or in memory: one instance of the loop for each, so that the
    // reads are plain LDS reads or (uniform addresses) scalar loads, not generic-pointer loads
    auto assign = [&](const float *c0) {
        for (int j = w; j < m; j += 4) {
            const int ds = L->dsub[j], kj = 1 << L->nbits[j];
            const float *c = c0 + L->cboff[j];
            const float *xv = xs + v * ldx + L->dimoff[j];
            float best = INFINITY;
            int besti = 0;
            switch (ds) {  // uniform over the wave; widths up to 8 are unrolled without predicates
                case 1: enc_nearest<1>(xv, c, kj, best, besti); break;
                case 2: enc_nearest<2>(xv, c, kj, best, besti); break;
                case 3: enc_nearest<3>(xv, c, kj, best, besti); break;
                case 4: enc_nearest<4>(xv, c, kj, best, besti); break;
                case 5: enc_nearest<5>(xv, c, kj, best, besti); break;
                case 6: enc_nearest<6>(xv, c, kj, best, besti); break;
                case 7: enc_nearest<7>(xv, c, kj, best, besti); break;
                case 8: enc_nearest<8>(xv, c, kj, best, besti); break;
                default:
                    for (int i = 0; i < kj; ++i) {
                        float acc = 0.0f;
                        for (int l = 0; l < ds; ++l) {
                            const float diff = __fsub_rn(xv[l], c[i * ds + l]);
                            acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                        }
                        if (i == 0 || acc < best) {
                            best = acc;
                            besti = i;
                        }
                    }
            }
            if (v < nv) sub[v * m + j] = (uint8_t)besti;
        }
    };
    if (cb_floats)
        assign(cbs);
    else
        assign(cb);
    __syncthreads();

    // pack: one output byte per thread and round
    for (int e = threadIdx.x; e < nv * cs; e += blockDim.x) {
        const int vv = e / cs, b = e - vv * cs;
        uint32_t byte = 0;
        for (int j = 0; j < m; ++j) {
            const int off = L->bitoff[j], nb = L->nbits[j];
            if (off + nb <= 8 * b || off >= 8 * b + 8) continue;
            const uint32_t val = sub[vv * m + j];
            const int rel = off - 8 * b;  // position of the sub-code's bit 0 relative to this byte
            byte |= rel >= 0 ? (val << rel) : (val >> (-rel));
        }
        codes[(size_t)v0 * cs + e] = (uint8_t)(byte & 255u);
    }
}

extern "C" int pq_encode(const pq_index_t *idx, const float *vectors, int64_t n,
                         const float *shift_rows, const int32_t *shift_ids, uint8_t *codes,
                         void *stream) {
    if (!idx || n < 0) {
        qadc_set_error("pq_encode: bad handle or n");
        return PQ_EINVAL;
    }
    if (n == 0) return PQ_OK;
    if (!vectors || !codes || ((shift_rows == nullptr) != (shift_ids == nullptr))) {
        qadc_set_error("pq_encode: null pointer (shift_rows and shift_ids go together)");
        return PQ_EINVAL;
    }
    const DevLayout &h = idx->h;
    size_t cbf = 0;  // codebook floats
    for (int j = 0; j < h.m; ++j) cbf += ((size_t)1 << h.nbits[j]) * (size_t)h.dsub[j];
    const size_t base_lds = (size_t)ENC_VB * (size_t)(h.d | 1) * sizeof(float) + (size_t)ENC_VB * (size_t)h.m;
    if (cbf * sizeof(float) > 48 * 1024 || base_lds + cbf * sizeof(float) > 96 * 1024) cbf = 0;
    // small codebooks are read through the scalar cache instead (faster than LDS reads)
    if (cbf * sizeof(float) <= 16 * 1024) cbf = 0;
    const size_t lds = base_lds + cbf * sizeof(float);
    if (lds > 160 * 1024) {
        qadc_set_error("pq_encode: d=%d needs %zu bytes of LDS per block, more than 163840", h.d, lds);
        return PQ_EINVAL;
    }
    if (lds > 48 * 1024)
        QADC_HIP_TRY(hipFuncSetAttribute((const void *)k_encode, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)lds));
    const int64_t blocks = (n + ENC_VB - 1) / ENC_VB;
    if (blocks > 0x7fffffffLL) {
        qadc_set_error("pq_encode: n=%lld too large for one call", (long long)n);
        return PQ_EINVAL;
    }
    hipLaunchKernelGGL(k_encode, dim3((unsigned)blocks), dim3(256), lds, (hipStream_t)stream, idx->dev,
                       idx->codebooks, vectors, n, shift_rows, shift_ids, codes, (int)cbf);
    QADC_LAUNCH_CHECK("k_encode");
    return PQ_OK;
}
