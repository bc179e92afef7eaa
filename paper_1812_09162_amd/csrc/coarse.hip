// ivf_coarse_search: the nprobe cells nearest to each query (Section 2.1.1: a query is routed
// to the cells of the inverted index whose centroids are closest).
//
// Cells are ranked by score(c) = ||c||^2 - 2 z.c (the squared distance minus ||z||^2, equal for
// all cells of a query), in fp32:
//   z.c      a chain of fused multiply-adds over the dimensions in ascending order
//   ||c||^2  the same chain over c*c
//   score    fma(-2, z.c, ||c||^2)
// The dot products are a dense [nq x d] x [d x K] contraction and run on the matrix cores:
// v_mfma_f32_32x32x2f32 accumulates its two products per call in ascending k with one rounding
// each, i.e. exactly the chain above (verified bit for bit on gfx950), so the scores, and with
// them the ranking, are reproducible by a scalar fmaf loop.
//
//   k_cnorm    ||c||^2 per centroid
//   k_scores   128 x 128 score tiles per block of four waves, each wave a 64 x 64 quarter as
//              2 x 2 MFMA tiles; operands staged through LDS in chunks of 32 dimensions, the
//              next chunk prefetched into registers while the current one is multiplied
//   k_select   one block per query: the cells in the low tail of the score range are gathered
//              and ranked by (score, id); exact radix selection when that tail is crowded
#include <math.h>
#include <string.h>

#include "qadc_device.h"

typedef float f32x16 __attribute__((ext_vector_type(16)));

#define CS_TILE 128   // queries and centroids per block tile
#define CS_KC 32      // dimensions per LDS chunk
#define CS_MAX_NPROBE 1024

// --------------------------------------------------------------------- k_cnorm ---
__global__ void __launch_bounds__(256)
k_cnorm(const float *__restrict__ centroids, int K, int d, float *__restrict__ cnorm) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= K) return;
    const float *p = centroids + (size_t)c * d;
    float acc = 0.0f;
    for (int l = 0; l < d; ++l) acc = __fmaf_rn(p[l], p[l], acc);
    cnorm[c] = acc;
}

// -------------------------------------------------------------------- k_scores ---
// scores[q][c] for q in [q0, q0 + nqc), c in [0, K); row stride ld (floats).
// LDS: As[k][row], Bs[k][col], k-major so that the 32 lanes of an MFMA operand read 32
// consecutive floats.
__device__ __forceinline__ void cs_load_chunk(const float *__restrict__ base, int rows_valid, int d,
                                              int k0, bool vec, float4 (&r)[4]) {
    // wave w, lane l: row = w*32 + l%32, float4 columns (l/32)*4 + i, i < 4
    const int w = threadIdx.x / QADC_WAVE, l = threadIdx.x % QADC_WAVE;
    const int row = w * 32 + (l & 31);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int k = k0 + ((l >> 5) * 4 + i) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < rows_valid) {
            const float *p = base + (size_t)row * d + k;
            if (vec && k + 3 < d) {
                v = *(const float4 *)p;
            } else {
                if (k + 0 < d) v.x = p[0];
                if (k + 1 < d) v.y = p[1];
                if (k + 2 < d) v.z = p[2];
                if (k + 3 < d) v.w = p[3];
            }
        }
        r[i] = v;
    }
}

__device__ __forceinline__ void cs_store_chunk(float *S, const float4 (&r)[4]) {
    const int w = threadIdx.x / QADC_WAVE, l = threadIdx.x % QADC_WAVE;
    const int row = w * 32 + (l & 31);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int k = ((l >> 5) * 4 + i) * 4;
        S[(k + 0) * CS_TILE + row] = r[i].x;
        S[(k + 1) * CS_TILE + row] = r[i].y;
        S[(k + 2) * CS_TILE + row] = r[i].z;
        S[(k + 3) * CS_TILE + row] = r[i].w;
    }
}

__global__ void __launch_bounds__(256)
k_scores(const float *__restrict__ queries, int nqc, const float *__restrict__ centroids, int K,
         int d, const float *__restrict__ cnorm, float *__restrict__ scores, size_t ld, int vec) {
    __shared__ float As[CS_KC * CS_TILE];
    __shared__ float Bs[CS_KC * CS_TILE];
    const int c0 = blockIdx.x * CS_TILE, q0 = blockIdx.y * CS_TILE;
    const int w = threadIdx.x / QADC_WAVE, l = threadIdx.x % QADC_WAVE;
    const int wr = w >> 1, wc = w & 1;  // this wave's 64 x 64 quarter
    const float *qa = queries + (size_t)q0 * d;
    const float *cb = centroids + (size_t)c0 * d;
    const int qv = nqc - q0 < CS_TILE ? nqc - q0 : CS_TILE;
    const int cv = K - c0 < CS_TILE ? K - c0 : CS_TILE;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    float4 ra[4], rb[4];
    cs_load_chunk(qa, qv, d, 0, vec != 0, ra);
    cs_load_chunk(cb, cv, d, 0, vec != 0, rb);
    for (int k0 = 0; k0 < d; k0 += CS_KC) {
        __syncthreads();  // the previous chunk has been consumed
        cs_store_chunk(As, ra);
        cs_store_chunk(Bs, rb);
        __syncthreads();
        if (k0 + CS_KC < d) {  // next chunk in flight during the multiplications
            cs_load_chunk(qa, qv, d, k0 + CS_KC, vec != 0, ra);
            cs_load_chunk(cb, cv, d, k0 + CS_KC, vec != 0, rb);
        }
#pragma unroll
        for (int kk = 0; kk < CS_KC; kk += 2) {
            const int kr = (kk + (l >> 5)) * CS_TILE + (l & 31);
            const float a0 = As[kr + wr * 64], a1 = As[kr + wr * 64 + 32];
            const float b0 = Bs[kr + wc * 64], b1 = Bs[kr + wc * 64 + 32];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
    }
    // element r of a 32 x 32 result: row (r/4)*8 + (lane/32)*4 + r%4, column lane%32
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int col = c0 + wc * 64 + j * 32 + (l & 31);
        if (col >= K) continue;
        const float cn = cnorm[col];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = q0 + wr * 64 + i * 32 + (r >> 2) * 8 + (l >> 5) * 4 + (r & 3);
                if (row < nqc) scores[(size_t)row * ld + col] = __fmaf_rn(-2.0f, acc[i][j][r], cn);
            }
    }
}

// -------------------------------------------------------------------- k_select ---
// One block of 1024 threads per query; keys = order-preserving integers of the scores; the
// result is the k = min(nprobe, K) smallest (key, id), ascending.
//
// Fast path: the keys are binned by (key - min) >> shift into 256 bins spanning [min, max]; the
// nearest cells sit in the sparse low tail, so the bin that holds the k-th key and the bins
// below it hold only a few cells more than k.  They are gathered into LDS and ranked by
// counting.  Three passes over the query's scores (range, histogram, gather), which stay in L2.
// Exact path (taken when those bins hold more than CS_CAND cells, e.g. many equal scores): four
// radix passes give the k-th key and how many keys lie below it; the keys below it and the
// lowest ids among its equals are collected and ranked.
#define CS_CAND 2048

// histogram increment: one LDS atomic per wave when all its active lanes hit the same bin
// (crowded keys), else one per lane
__device__ __forceinline__ void cs_hist_add(uint32_t *hist, uint32_t bin, bool active) {
    const uint64_t act = __ballot(active);
    if (act == 0) return;
    const int leader = __ffsll((unsigned long long)act) - 1;
    const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
    if (__ballot(active && bin != b) == 0) {
        if (__lane_id() == leader) atomicAdd(&hist[b], (uint32_t)__popcll(act));
    } else if (active) {
        atomicAdd(&hist[bin], 1u);
    }
}

__device__ inline void cs_rank_and_write(const uint64_t *A, int na, int k, int nprobe, int32_t *oid,
                                         float *osc) {
    for (int i = threadIdx.x; i < na; i += blockDim.x) {
        const uint64_t mine = A[i];
        int r = 0;
        for (int j = 0; j < na; ++j) r += A[j] < mine ? 1 : 0;
        if (r < k) {
            oid[r] = (int32_t)(uint32_t)mine;
            if (osc) osc[r] = qadc_ord2f((uint32_t)(mine >> 32));
        }
    }
    for (int r = k + threadIdx.x; r < nprobe; r += blockDim.x) {
        oid[r] = -1;
        if (osc) osc[r] = INFINITY;
    }
}

__global__ void __launch_bounds__(1024)
k_select(const float *__restrict__ scores, size_t ld, int K, int nprobe,
         int32_t *__restrict__ probe_ids, float *__restrict__ probe_scores) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sel[2];
    __shared__ uint64_t A[CS_CAND];
    __shared__ uint32_t wcnt[16];
    __shared__ uint32_t s_lo[16], s_hi[16];
    __shared__ uint32_t s_taken, s_ties;
    const size_t q = blockIdx.x;
    const float *s = scores + q * ld;
    int32_t *oid = probe_ids + q * nprobe;
    float *osc = probe_scores ? probe_scores + q * nprobe : nullptr;
    const int k = nprobe < K ? nprobe : K;
    const int wave = threadIdx.x / QADC_WAVE, lane = threadIdx.x % QADC_WAVE;
    // 16-byte loads: thread t takes scores 4*(j*1024 + t) .. +3, UB loads in flight together.
    // Row starts are 128-byte aligned and padded to a multiple of 32 scores; what lies past K is
    // masked by index.
    constexpr int UB = 8;
    const int nj = (K + 4095) / 4096;
    auto load_keys = [&](int j0, uint32_t (&v)[UB][4]) {
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int i = ((j0 + u) * 1024 + (int)threadIdx.x) * 4;
            float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < K) f = *(const float4 *)(s + i);
            v[u][0] = i + 0 < K ? qadc_f2ord(f.x) : 0xffffffffu;
            v[u][1] = i + 1 < K ? qadc_f2ord(f.y) : 0xffffffffu;
            v[u][2] = i + 2 < K ? qadc_f2ord(f.z) : 0xffffffffu;
            v[u][3] = i + 3 < K ? qadc_f2ord(f.w) : 0xffffffffu;
        }
    };

    // range of the keys
    uint32_t lo = 0xffffffffu, hi = 0u;
    for (int j0 = 0; j0 < nj; j0 += UB) {
        uint32_t v[UB][4];
        load_keys(j0, v);
#pragma unroll
        for (int u = 0; u < UB; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (((j0 + u) * 1024 + (int)threadIdx.x) * 4 + c < K) {
                    lo = v[u][c] < lo ? v[u][c] : lo;
                    hi = v[u][c] > hi ? v[u][c] : hi;
                }
            }
    }
    lo = qadc_wave_min(lo);
    hi = ~qadc_wave_min(~hi);
    if (lane == 0) {
        s_lo[wave] = lo;
        s_hi[wave] = hi;
    }
    for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
    if (threadIdx.x == 0) {
        s_taken = 0;
        s_ties = 0;
    }
    __syncthreads();
#pragma unroll
    for (int w2 = 0; w2 < 16; ++w2) {
        lo = s_lo[w2] < lo ? s_lo[w2] : lo;
        hi = s_hi[w2] > hi ? s_hi[w2] : hi;
    }
    const uint32_t span = hi - lo;
    const int shift = span < 256u ? 0 : 24 - __clz(span);  // (span >> shift) < 256
    for (int j0 = 0; j0 < nj; j0 += UB) {
        uint32_t v[UB][4];
        load_keys(j0, v);
#pragma unroll
        for (int u = 0; u < UB; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool in = ((j0 + u) * 1024 + (int)threadIdx.x) * 4 + c < K;
                cs_hist_add(hist, in ? (v[u][c] - lo) >> shift : 0u, in);
            }
    }
    __syncthreads();
    if (threadIdx.x < QADC_WAVE) qadc_wave_select_bin(hist, (uint32_t)k, 0u, sel);
    __syncthreads();
    const uint32_t kbin = sel[0];
    const uint32_t cand = sel[1] + hist[kbin];  // cells in the bins up to kbin
    if (cand <= CS_CAND) {
        for (int j0 = 0; j0 < nj; j0 += UB) {
            uint32_t v[UB][4];
            load_keys(j0, v);
#pragma unroll
            for (int u = 0; u < UB; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int i = ((j0 + u) * 1024 + (int)threadIdx.x) * 4 + c;
                    const bool take = i < K && ((v[u][c] - lo) >> shift) <= kbin;
                    const uint64_t m = __ballot(take);
                    if (m != 0) {
                        uint32_t base = 0;
                        if (lane == 0) base = atomicAdd(&s_taken, (uint32_t)__popcll(m));
                        base = __builtin_amdgcn_readfirstlane(base);
                        if (take)
                            A[base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull))] =
                                ((uint64_t)v[u][c] << 32) | (uint32_t)i;
                    }
                }
        }
        __syncthreads();
        cs_rank_and_write(A, (int)cand, k, nprobe, oid, osc);
        return;
    }

    // exact path: the keys are re-read from memory in every pass
#define CS_KEYM(j) ((j) * 1024 + (int)threadIdx.x < K ? qadc_f2ord(s[(j) * 1024 + threadIdx.x]) : 0xffffffffu)
    const int njm = (K + 1023) / 1024;
    __syncthreads();
    uint32_t prefix = 0, mask = 0, kk = (uint32_t)k;
    for (int pass = 3; pass >= 0; --pass) {
        const int sh = pass * 8;
        for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
        __syncthreads();
        for (int j = 0; j < njm; ++j) {
            const uint32_t v = CS_KEYM(j);
            const bool in = j * 1024 + (int)threadIdx.x < K && (v & mask) == prefix;
            cs_hist_add(hist, (v >> sh) & 255u, in);
        }
        __syncthreads();
        if (threadIdx.x < QADC_WAVE) qadc_wave_select_bin(hist, kk, 0u, sel);
        __syncthreads();
        prefix |= sel[0] << sh;
        mask |= 255u << sh;
        kk -= sel[1];
        __syncthreads();
    }
    // prefix = the k-th smallest key; kk = how many cells with that key belong to the result
    const uint32_t kth = prefix, need = kk, below = (uint32_t)k - need;
    for (int j = 0; j < njm; ++j) {  // cells below the k-th key, in any order
        const uint32_t v = CS_KEYM(j);
        const int i = j * 1024 + (int)threadIdx.x;
        const bool lt = i < K && v < kth;
        const uint64_t m = __ballot(lt);
        if (m != 0) {
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(&s_taken, (uint32_t)__popcll(m));
            base = __builtin_amdgcn_readfirstlane(base);
            if (lt) A[base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull))] = ((uint64_t)v << 32) | (uint32_t)i;
        }
    }
    __syncthreads();
    // cells equal to the k-th key: the `need` lowest ids.  Rounds of 1024 consecutive ids in
    // ascending order; within a round positions come from the wave counts.
    for (int j = 0; j < njm; ++j) {
        const int i = j * 1024 + (int)threadIdx.x;
        const bool eq = i < K && CS_KEYM(j) == kth;
        const uint64_t m = __ballot(eq);
        if (lane == 0) wcnt[wave] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t before = s_ties, total = 0;
        for (int w2 = 0; w2 < 16; ++w2) {
            before += w2 < wave ? wcnt[w2] : 0u;
            total += wcnt[w2];
        }
        if (eq) {
            const uint32_t pos = before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            if (pos < need) A[below + pos] = ((uint64_t)kth << 32) | (uint32_t)i;
        }
        __syncthreads();
        if (threadIdx.x == 0) s_ties += total;
        __syncthreads();
        if (s_ties >= need) break;
    }
    __syncthreads();
    cs_rank_and_write(A, k, k, nprobe, oid, osc);
#undef CS_KEYM
}

// ------------------------------------------------------------------------ host ---
static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

// queries per pass: the score matrix of a pass stays within 256 MB
static int coarse_chunk(int nq, int K) {
    const size_t ld = ((size_t)K + 31) & ~(size_t)31;
    size_t qc = ((size_t)256 << 20) / (ld * sizeof(float));
    qc = qc / CS_TILE * CS_TILE;
    if (qc < CS_TILE) qc = CS_TILE;
    const size_t nqr = ((size_t)(nq > 0 ? nq : 1) + CS_TILE - 1) / CS_TILE * CS_TILE;
    return (int)(qc < nqr ? qc : nqr);
}

extern "C" size_t ivf_coarse_workspace_bytes(int nq, int K) {
    if (nq < 0 || K < 1) return 0;
    const size_t ld = ((size_t)K + 31) & ~(size_t)31;
    return up256((size_t)K * sizeof(float)) + up256((size_t)coarse_chunk(nq, K) * ld * sizeof(float));
}

extern "C" int ivf_coarse_search(const float *queries, int nq, const float *centroids, int K, int d,
                                 int nprobe, int32_t *probe_ids, float *probe_scores,
                                 void *workspace, size_t workspace_bytes, void *stream) {
    if (nq < 0 || K < 1 || d < 1 || d > PQ_MAX_DIM || nprobe < 1 || nprobe > CS_MAX_NPROBE) {
        qadc_set_error("ivf_coarse_search: need nq>=0, K>=1, 1<=d<=%d, 1<=nprobe<=%d (got nq=%d K=%d d=%d nprobe=%d)",
                       PQ_MAX_DIM, CS_MAX_NPROBE, nq, K, d, nprobe);
        return PQ_EINVAL;
    }
    if (nq == 0) return PQ_OK;
    if (!queries || !centroids || !probe_ids || !workspace) {
        qadc_set_error("ivf_coarse_search: null pointer");
        return PQ_EINVAL;
    }
    if (((uintptr_t)workspace & 255u) != 0) {
        qadc_set_error("ivf_coarse_search: workspace must be 256-byte aligned");
        return PQ_EINVAL;
    }
    const size_t need = ivf_coarse_workspace_bytes(nq, K);
    if (workspace_bytes < need) {
        qadc_set_error("ivf_coarse_search: workspace of %zu bytes, need %zu", workspace_bytes, need);
        return PQ_ENOMEM;
    }
    hipStream_t s = (hipStream_t)stream;
    float *cnorm = (float *)workspace;
    float *scores = (float *)((char *)workspace + up256((size_t)K * sizeof(float)));
    const size_t ld = ((size_t)K + 31) & ~(size_t)31;
    const int qc = coarse_chunk(nq, K);
    // 16-byte loads need rows that start on 16-byte boundaries
    const int vec = (d % 4 == 0) && (((uintptr_t)queries | (uintptr_t)centroids) & 15u) == 0;
    hipLaunchKernelGGL(k_cnorm, dim3((K + 255) / 256), dim3(256), 0, s, centroids, K, d, cnorm);
    QADC_LAUNCH_CHECK("k_cnorm");
    for (int q0 = 0; q0 < nq; q0 += qc) {
        const int nqc = nq - q0 < qc ? nq - q0 : qc;
        hipLaunchKernelGGL(k_scores, dim3((K + CS_TILE - 1) / CS_TILE, (nqc + CS_TILE - 1) / CS_TILE),
                           dim3(256), 0, s, queries + (size_t)q0 * d, nqc, centroids, K, d, cnorm,
                           scores, ld, vec);
        QADC_LAUNCH_CHECK("k_scores");
        int32_t *pid = probe_ids + (size_t)q0 * nprobe;
        float *psc = probe_scores ? probe_scores + (size_t)q0 * nprobe : nullptr;
        hipLaunchKernelGGL(k_select, dim3(nqc), dim3(1024), 0, s, scores, ld, K, nprobe, pid, psc);
        QADC_LAUNCH_CHECK("k_select");
    }
    return PQ_OK;
}
