// pq_adc_scan_topk: scan of packed codes with quantized tables (eq. (2),
// Section 3.4 saturating sums, Section 3.5) and exact top-R by (key, id).
//
// Three kernels per call:
//   k_pilot  one block per query: clears the per-query state and derives a first
//            inclusive key threshold from the first few thousand codes;
//   k_scan   G blocks per query stream the codes once; a code whose key bin is
//            within the current threshold is appended to the block's private
//            slot array and counted in a per-query histogram, from which any
//            wave that appended tightens the shared threshold;
//   k_final  one block per query gathers the surviving candidates, ranks them
//            by (key, id) and writes the R best.  If any slot array overflowed
//            (degenerate inputs with huge tie classes) it instead runs an exact
//            two-pass selection over all codes.
//
// Why the threshold is safe: it is only ever lowered to a bin x for which at
// least R codes of the data set are known to have bin <= x, so the R-th best
// key lies in a bin <= x and no code in a higher bin can be a result.  The
// result is defined as a sort by (key, id) and therefore does not depend on
// the order in which blocks run.
#include <math.h>

#include "scan_device.h"

// --------------------------------------------------------------- k_pilot ---
template <int KIND, typename QT>
__global__ void __launch_bounds__(1024)
k_pilot(const DevLayout *__restrict__ L, const void *__restrict__ qtables,
        const pq_qparams_t *__restrict__ qparams, const uint8_t *__restrict__ codes,
        int64_t pilot_codes, int R, char *__restrict__ ws, size_t per_query) {
    extern __shared__ unsigned char smem[];
    QT *gtab = (QT *)smem;
    __shared__ uint32_t hist[256];
    const size_t q = blockIdx.x;
    ScanState *st = (ScanState *)(ws + q * per_query);
    const int shift = L->acc_bits == 8 ? 0 : 8;
    for (int i = threadIdx.x; i < 256; i += blockDim.x) {
        hist[i] = 0;
        st->hist[i] = 0;
    }
    if (threadIdx.x == 0) st->overflow = 0;
    build_gtab<QT>(L, (const QT *)qtables + q * L->T, gtab);
    for (int64_t id = threadIdx.x; id < pilot_codes; id += blockDim.x)
        atomicAdd(&hist[key_at<KIND, QT>(L, gtab, codes, id) >> shift], 1u);
    __syncthreads();
    if (threadIdx.x < QADC_WAVE) {
        uint32_t b = wave_bound_from_hist(hist, (uint32_t)R);
        uint32_t kb = qparams[q].key_bound;
        if (kb > (uint32_t)L->qmax) kb = (uint32_t)L->qmax;
        kb >>= shift;
        if (b > 255u) b = 255u;
        if (threadIdx.x == 0) st->thr = b < kb ? b : kb;
    }
}

// ---------------------------------------------------------------- k_scan ---
template <int KIND, typename QT>
__global__ void __launch_bounds__(256)
k_scan(const DevLayout *__restrict__ L, const void *__restrict__ qtables,
       const uint8_t *__restrict__ codes, int64_t n, int R, char *__restrict__ ws,
       size_t per_query, size_t counts_off, size_t slots_off, int cap_b) {
    extern __shared__ unsigned char smem[];
    QT *gtab = (QT *)smem;
    __shared__ uint32_t s_count;
    const size_t q = blockIdx.y;
    const int b = blockIdx.x, G = gridDim.x;
    char *wq = ws + q * per_query;
    ScanState *st = (ScanState *)wq;
    uint32_t *counts = (uint32_t *)(wq + counts_off);
    SlotRef ref;
    ref.slot = (uint64_t *)(wq + slots_off) + (size_t)b * cap_b;
    ref.cap = (uint32_t)cap_b;
    ref.lds_count = &s_count;
    ref.st = st;
    if (threadIdx.x == 0) s_count = 0;
    build_gtab<QT>(L, (const QT *)qtables + q * L->T, gtab);
    const int shift = L->acc_bits == 8 ? 0 : 8;
    const uint32_t qmax = (uint32_t)L->qmax;
    const int64_t ntiles = (n + 1023) / 1024;  // 1024 codes per tile, 4 per thread

    for (int64_t tile = b; tile < ntiles; tile += G) {
        const uint32_t thr = __hip_atomic_load(&st->thr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t key[4], id[4];
        bool ok[4];
        if (KIND == SCAN_NIB8) {
            // two 16-byte chunks per thread, two codes per chunk
            const int64_t nchunks = (n + 1) >> 1;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int64_t c = tile * 512 + u * 256 + threadIdx.x;
                uint4 w = make_uint4(0, 0, 0, 0);
                const bool c_ok = c < nchunks;
                const bool second = c_ok && (2 * c + 1 < n);
                if (second)
                    w = *(const uint4 *)(codes + c * 16);
                else if (c_ok) {
                    uint2 h = *(const uint2 *)(codes + c * 16);
                    w.x = h.x;
                    w.y = h.y;
                }
                uint32_t s0 = sum8(gtab, w.x, w.y), s1 = sum8(gtab, w.z, w.w);
                key[2 * u] = s0 > qmax ? qmax : s0;
                key[2 * u + 1] = s1 > qmax ? qmax : s1;
                id[2 * u] = (uint32_t)(2 * c);
                id[2 * u + 1] = (uint32_t)(2 * c + 1);
                ok[2 * u] = c_ok;
                ok[2 * u + 1] = second;
            }
        } else if (KIND == SCAN_NIB16) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t c = tile * 1024 + u * 256 + threadIdx.x;
                uint4 w = make_uint4(0, 0, 0, 0);
                ok[u] = c < n;
                if (ok[u]) w = *(const uint4 *)(codes + c * 16);
                uint32_t s = sum8(gtab, w.x, w.y) + sum8(gtab + 2048, w.z, w.w);
                key[u] = s > qmax ? qmax : s;
                id[u] = (uint32_t)c;
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t c = tile * 1024 + u * 256 + threadIdx.x;
                ok[u] = c < n;
                key[u] = ok[u] ? key_generic(L, gtab, codes + c * L->cs) : qmax;
                id[u] = (uint32_t)c;
            }
        }
        bool pass[4], any = false;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            pass[u] = ok[u] && ((key[u] >> shift) <= thr);
            any = any || pass[u];
        }
        if (__ballot(any) != 0) {  // rare once the threshold has tightened
#pragma unroll
            for (int u = 0; u < 4; ++u) wave_append(pass[u], key[u], id[u], key[u] >> shift, ref);
            uint32_t nb = wave_bound_from_hist(st->hist, (uint32_t)R);
            if (__lane_id() == 0 && nb < thr) atomicMin(&st->thr, nb);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) counts[b] = s_count < (uint32_t)cap_b ? s_count : (uint32_t)cap_b;
}

// --------------------------------------------------------------- k_final ---
struct FinalOut {
    int32_t *ids;
    uint16_t *keys;
    float *dist;
};

// Rank the na candidates of A by (key, id) and write the first R, padding the rest.
__device__ inline void rank_and_write(const uint64_t *A, int na, int R, const pq_qparams_t &prm,
                                      uint32_t qmax, const FinalOut &o) {
    const float fdelta = (float)prm.delta, fdmin = (float)prm.d_min;
    for (int i = threadIdx.x; i < na; i += blockDim.x) {
        const uint64_t mine = A[i];
        int rank = 0;
        for (int j = 0; j < na; ++j) rank += (A[j] < mine) ? 1 : 0;
        if (rank < R) {
            const uint32_t key = (uint32_t)(mine >> 32);
            o.ids[rank] = (int32_t)(uint32_t)mine;
            o.keys[rank] = (uint16_t)key;
            o.dist[rank] = fmaf((float)key, fdelta, fdmin);
        }
    }
    for (int r = (na < R ? na : R) + threadIdx.x; r < R; r += blockDim.x) {
        o.ids[r] = -1;
        o.keys[r] = (uint16_t)qmax;
        o.dist[r] = INFINITY;
    }
}

// Exact selection over all n codes by one block: histogram of key bins (two
// levels for 16-bit keys) gives the R-th key k*; a second pass in id order keeps
// every code below k* and the first (R - count_below) codes equal to k*.
template <int KIND, typename QT>
__device__ inline void exact_select(const DevLayout *L, const QT *gtab,
                                    const uint8_t *__restrict__ codes, int64_t n, int R,
                                    uint64_t *A, uint32_t *hist, uint32_t *sh) {
    const int Rn = (int64_t)R < n ? R : (int)n;
    const bool wide = L->acc_bits != 8;
    uint32_t kstar = 0, below = 0;
    for (int level = 0; level < (wide ? 2 : 1); ++level) {
        for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
        __syncthreads();
        for (int64_t id = threadIdx.x; id < n; id += blockDim.x) {
            uint32_t key = key_at<KIND, QT>(L, gtab, codes, id);
            if (!wide)
                atomicAdd(&hist[key], 1u);
            else if (level == 0)
                atomicAdd(&hist[key >> 8], 1u);
            else if ((key >> 8) == kstar)
                atomicAdd(&hist[key & 255u], 1u);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t run = below;
            int bsel = 0;
            for (; bsel < 255; ++bsel) {
                if (run + hist[bsel] >= (uint32_t)Rn) break;
                run += hist[bsel];
            }
            sh[0] = (uint32_t)bsel;
            sh[1] = run;
        }
        __syncthreads();
        kstar = (level == 0) ? sh[0] : ((kstar << 8) | sh[0]);
        below = sh[1];
        __syncthreads();
    }
    const uint32_t need = (uint32_t)Rn - below;  // ties to keep, lowest ids first
    if (threadIdx.x == 0) sh[2] = 0;             // entries written to A
    uint32_t tie_base = 0;
    const int wave = threadIdx.x / QADC_WAVE, lane = threadIdx.x % QADC_WAVE;
    const int nwaves = blockDim.x / QADC_WAVE;
    uint32_t *wtot = sh + 8;  // nwaves words
    __syncthreads();
    for (int64_t base = 0; base < n; base += blockDim.x) {
        const int64_t id = base + threadIdx.x;
        const bool valid = id < n;
        const uint32_t key = valid ? key_at<KIND, QT>(L, gtab, codes, id) : 0xffffffffu;
        const bool lt = valid && key < kstar, eq = valid && key == kstar;
        const uint64_t m = __ballot(eq);
        if (lane == 0) wtot[wave] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t woff = 0, tot = 0;
        for (int w = 0; w < nwaves; ++w) {
            uint32_t c = wtot[w];
            woff += (w < wave) ? c : 0;
            tot += c;
        }
        const uint32_t tie_rank = tie_base + woff + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
        if (lt || (eq && tie_rank < need)) {
            uint32_t pos = atomicAdd(&sh[2], 1u);
            A[pos] = ((uint64_t)key << 32) | (uint64_t)(uint32_t)id;
        }
        tie_base += tot;
        __syncthreads();
    }
}

template <int KIND, typename QT>
__global__ void __launch_bounds__(1024)
k_final(const DevLayout *__restrict__ L, const void *__restrict__ qtables,
        const pq_qparams_t *__restrict__ qparams, const uint8_t *__restrict__ codes, int64_t n,
        int R, char *__restrict__ ws, size_t per_query, size_t counts_off, size_t slots_off,
        int cap_b, int G, int32_t *__restrict__ out_ids, uint16_t *__restrict__ out_keys,
        float *__restrict__ out_dist) {
    extern __shared__ unsigned char smem[];
    uint64_t *A = (uint64_t *)smem;                // FINAL_CAP entries
    QT *gtab = (QT *)(smem + FINAL_CAP * 8);       // only built on the slow path
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh[32];
    const size_t q = blockIdx.x;
    char *wq = ws + q * per_query;
    ScanState *st = (ScanState *)wq;
    const uint32_t *counts = (const uint32_t *)(wq + counts_off);
    const uint64_t *slots = (const uint64_t *)(wq + slots_off);
    const int shift = L->acc_bits == 8 ? 0 : 8;
    const uint32_t qmax = (uint32_t)L->qmax;
    FinalOut o;
    o.ids = out_ids + q * R;
    o.keys = out_keys + q * R;
    o.dist = out_dist + q * R;
    const pq_qparams_t prm = qparams[q];

    if (threadIdx.x == 0) {
        sh[0] = 0;  // na
        sh[1] = st->overflow;
    }
    __syncthreads();
    const uint32_t thr = st->thr;
    const int wave = threadIdx.x / QADC_WAVE, lane = threadIdx.x % QADC_WAVE;
    const int nwaves = blockDim.x / QADC_WAVE;
    for (int b = wave; b < G; b += nwaves) {
        const uint32_t cnt = counts[b];
        for (uint32_t i = lane; i < cnt; i += QADC_WAVE) {
            const uint64_t c = slots[(size_t)b * cap_b + i];
            if ((((uint32_t)(c >> 32)) >> shift) <= thr) {
                uint32_t pos = atomicAdd(&sh[0], 1u);
                if (pos < FINAL_CAP)
                    A[pos] = c;
                else
                    sh[1] = 1u;
            }
        }
    }
    __syncthreads();
    int na = (int)sh[0];
    const bool slow = sh[1] != 0;
    __syncthreads();
    if (slow) {
        build_gtab<QT>(L, (const QT *)qtables + q * L->T, gtab);
        exact_select<KIND, QT>(L, gtab, codes, n, R, A, hist, sh);
        __syncthreads();
        na = (int)sh[2];
    }
    rank_and_write(A, na, R, prm, qmax, o);
}

// ------------------------------------------------------------------ host ---
template <int KIND, typename QT>
static int launch_scan(const pq_index *idx, const void *qtables, const pq_qparams_t *qparams, int nq,
                       const uint8_t *codes, int64_t n, int R, int32_t *out_ids, uint16_t *out_keys,
                       float *out_dist, char *ws, const ScanPlan &p, hipStream_t s) {
    const size_t gtab_bytes = (size_t)idx->h.gtab_len * sizeof(QT);
    hipLaunchKernelGGL((k_pilot<KIND, QT>), dim3(nq), dim3(1024), gtab_bytes, s, idx->dev, qtables,
                       qparams, codes, p.pilot_codes, R, ws, p.per_query);
    QADC_LAUNCH_CHECK("k_pilot");
    qadc_prof_begin(s);
    hipLaunchKernelGGL((k_scan<KIND, QT>), dim3(p.G, nq), dim3(256), gtab_bytes, s, idx->dev,
                       qtables, codes, n, R, ws, p.per_query, p.counts_off, p.slots_off, p.cap_b);
    qadc_prof_end(s);
    QADC_LAUNCH_CHECK("k_scan");
    hipLaunchKernelGGL((k_final<KIND, QT>), dim3(nq), dim3(1024), FINAL_CAP * 8 + gtab_bytes, s,
                       idx->dev, qtables, qparams, codes, n, R, ws, p.per_query, p.counts_off,
                       p.slots_off, p.cap_b, p.G, out_ids, out_keys, out_dist);
    QADC_LAUNCH_CHECK("k_final");
    return PQ_OK;
}

extern "C" int pq_adc_scan_topk(const pq_index_t *idx, const void *qtables,
                                const pq_qparams_t *qparams, int nq, const uint8_t *codes,
                                int64_t n, int R, int32_t *out_ids, uint16_t *out_keys,
                                float *out_dist, void *workspace, size_t workspace_bytes,
                                void *stream) {
    if (!idx || nq < 0 || n < 0 || n >= ((int64_t)1 << 31)) {
        qadc_set_error("pq_adc_scan_topk: bad handle, nq or n (need 0 <= n < 2^31)");
        return PQ_EINVAL;
    }
    if (R < 1 || R > PQ_MAX_R) {
        qadc_set_error("pq_adc_scan_topk: need 1<=R<=%d (got %d)", PQ_MAX_R, R);
        return PQ_EINVAL;
    }
    if (nq == 0) return PQ_OK;
    if (nq > 65535) {
        qadc_set_error("pq_adc_scan_topk: at most 65535 queries per call (got %d)", nq);
        return PQ_EINVAL;
    }
    if (!qtables || !qparams || !out_ids || !out_keys || !out_dist || !workspace || (n > 0 && !codes)) {
        qadc_set_error("pq_adc_scan_topk: null pointer");
        return PQ_EINVAL;
    }
    if (((uintptr_t)codes & 15u) != 0 || ((uintptr_t)workspace & 255u) != 0) {
        qadc_set_error("pq_adc_scan_topk: codes must be 16-byte and workspace 256-byte aligned");
        return PQ_EINVAL;
    }
    const ScanPlan p = qadc_scan_plan(idx, nq, n, R);
    if (workspace_bytes < p.total) {
        qadc_set_error("pq_adc_scan_topk: workspace of %zu bytes, need %zu", workspace_bytes, p.total);
        return PQ_ENOMEM;
    }
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const bool u8 = idx->h.acc_bits == 8;
#define QADC_GO(KIND, QT) \
    return launch_scan<KIND, QT>(idx, qtables, qparams, nq, codes, n, R, out_ids, out_keys, out_dist, ws, p, s)
    switch (idx->h.kind) {
        case SCAN_NIB8:
            if (u8) QADC_GO(SCAN_NIB8, uint8_t); else QADC_GO(SCAN_NIB8, uint16_t);
        case SCAN_NIB16:
            if (u8) QADC_GO(SCAN_NIB16, uint8_t); else QADC_GO(SCAN_NIB16, uint16_t);
        default:
            if (u8) QADC_GO(SCAN_GENERIC, uint8_t); else QADC_GO(SCAN_GENERIC, uint16_t);
    }
#undef QADC_GO
}
