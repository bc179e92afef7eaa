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
//   k_scores   128 x 256 (queries x cells) score tiles per block of four waves, each wave a
//              64 x 128 part as 2 x 4 MFMA tiles; operands staged through LDS in chunks of 32
//              dimensions, the next chunk prefetched into registers while the current one is
//              multiplied
//   k_select   one block per query: the cells in the low tail of the score range are gathered
//              and ranked by (score, id); exact radix selection when that tail is crowded
// For large K the score matrix is never written.  A pilot (the first P cells, through the two
// kernels above) gives every query a bound: the nprobe-th smallest pilot score, which no result
// can exceed.  k_scores then runs over all cells in its filtering form: a score within the bound
// goes, as (ordered score << 32 | cell), to a short private list per (query, block of 256
// cells); k_select_cand gathers a query's lists and ranks them.  If a list overflows (far more
// near cells in one block than the pilot predicts), a flag sends the whole pass of queries
// through the matrix form again, which is exact for any input.
#include <math.h>
#include <string.h>

#include "scan_device.h"

typedef float f32x16 __attribute__((ext_vector_type(16)));

#define CS_TQ 128     // queries per block tile
#define CS_TC 256     // cells per block tile
#define CS_KC 32      // dimensions per LDS chunk
#ifndef CS_NT
#define CS_NT 512     // threads per k_scores block: 8 waves as 2 x 4, 64 x 64 results each
#endif
#ifndef CS_KK_UNROLL
#define CS_KK_UNROLL 5  // steps of two dimensions unrolled together (all 16: operand reads hoisted until registers spill)
#endif
#define CS_NW (CS_NT / 64)
#define CS_WC (CS_NW / 2)            // waves side by side over the tile's cells
#define CS_NJ (CS_TC / CS_WC / 32)   // 32 x 32 MFMA tiles side by side per wave
#define CS_MAX_NPROBE 1024
#define CS_SLOT 32    // candidate slots per (query, block of CS_TC cells) in the filtering form

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
// consecutive floats; rows of an odd number of floats ( so that the transposing stores spread over
// the banks).  Global loads: eight adjacent lanes fetch the 128 contiguous bytes that one row
// contributes to a chunk, so every cache line is requested once.
template <int NI>  // rows rowb + (CS_NT / 8) i, i < NI: a tile of (CS_NT / 8) NI rows
__device__ __forceinline__ void cs_load_chunk(const float *__restrict__ base, int rows_valid, int d,
                                              int k0, bool vec, float4 (&r)[NI]) {
    const int piece = threadIdx.x & 7, rowb = threadIdx.x >> 3;
    const int k = k0 + piece * 4;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int row = rowb + (CS_NT / 8) * i;
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

// The same for a tile whose rows all exist and a chunk that lies inside the rows, 16-byte
// loads allowed: no tests, one address per row.
template <int NI>
__device__ __forceinline__ void cs_load_chunk_full(const float *__restrict__ base, int d, int k0,
                                                   float4 (&r)[NI]) {
    const int piece = threadIdx.x & 7, rowb = threadIdx.x >> 3;
    const float *p = base + (size_t)rowb * d + k0 + piece * 4;
#pragma unroll
    for (int i = 0; i < NI; ++i) r[i] = *(const float4 *)(p + (size_t)((CS_NT / 8) * i) * d);
}

template <int NI>
__device__ __forceinline__ void cs_store_chunk(float *S, const float4 (&r)[NI]) {
    constexpr int LD = (CS_NT / 8) * NI + 1;
    const int piece = threadIdx.x & 7, rowb = threadIdx.x >> 3;
    const int k = piece * 4;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int row = rowb + (CS_NT / 8) * i;
        S[(k + 0) * LD + row] = r[i].x;
        S[(k + 1) * LD + row] = r[i].y;
        S[(k + 2) * LD + row] = r[i].z;
        S[(k + 3) * LD + row] = r[i].w;
    }
}

// FILTER: scores are not stored; those <= bound[query] (bound = pilot[q * pstride + koff]) are
// appended to slots[(q * ncb + block) * CS_SLOT ...] and counted in counts[q * ncb + block].
// guard: if non-null and *guard == 0 the kernel does nothing (the matrix form as a fallback).
template <bool FILTER>
__global__ void __launch_bounds__(CS_NT) __attribute__((amdgpu_waves_per_eu(CS_NT / 128, CS_NT / 128)))
k_scores(const float *__restrict__ queries, int nqc, const float *__restrict__ centroids, int K,
         int d, const float *__restrict__ cnorm, float *__restrict__ scores, size_t ld, int vec,
         const float *__restrict__ pilot, int pstride, int koff, uint64_t *__restrict__ slots,
         uint32_t *__restrict__ counts, const int *__restrict__ guard, int gx, int gy) {
    if (guard && *guard == 0) return;
    constexpr int LDA = CS_TQ + 1, LDB = CS_TC + 1;
    __shared__ float As[CS_KC * LDA];
    __shared__ __align__(16) float Bs[CS_KC * LDB];
    __shared__ __align__(16) float s_bound[FILTER ? CS_TQ : 4];
    __shared__ uint32_t s_cnt[FILTER ? CS_TQ : 1];
    const int w = threadIdx.x / QADC_WAVE, l = threadIdx.x % QADC_WAVE;
    const int wr = w / CS_WC, wc = w % CS_WC;  // this wave's 64 x (32 CS_NJ) part: 2 x CS_NJ MFMA tiles
    const int ncb = gx;
    const int nch = (d + CS_KC - 1) / CS_KC;
    constexpr int RPP = CS_NT / 8;  // rows per pass of the loads
    float4 ra[CS_TQ / RPP], rb[CS_TC / RPP];
    {
        const int tile = blockIdx.x;  // cell block tile % gx, query block tile / gx
        const int c0 = (tile % gx) * CS_TC, q0 = (tile / gx) * CS_TQ, cbx = tile % gx;
        const bool full_a = vec != 0 && nqc - q0 >= CS_TQ, full_b = vec != 0 && K - c0 >= CS_TC;  // (block-uniform)
        auto load = [&](int kc) {
            const bool inside = (kc + 1) * CS_KC <= d;
            if (full_a && inside)
                cs_load_chunk_full<CS_TQ / RPP>(queries + (size_t)q0 * d, d, kc * CS_KC, ra);
            else
                cs_load_chunk<CS_TQ / RPP>(queries + (size_t)q0 * d, nqc - q0 < CS_TQ ? nqc - q0 : CS_TQ, d,
                                           kc * CS_KC, vec != 0, ra);
            if (full_b && inside)
                cs_load_chunk_full<CS_TC / RPP>(centroids + (size_t)c0 * d, d, kc * CS_KC, rb);
            else
                cs_load_chunk<CS_TC / RPP>(centroids + (size_t)c0 * d, K - c0 < CS_TC ? K - c0 : CS_TC, d,
                                           kc * CS_KC, vec != 0, rb);
        };
        load(0);
        float cnv[CS_NJ];  // the norms of this lane's columns, in flight during the multiplications
#pragma unroll
        for (int j = 0; j < CS_NJ; ++j) {
            const int col = c0 + wc * (32 * CS_NJ) + j * 32 + (l & 31);
            cnv[j] = col < K ? cnorm[col] : 0.0f;
        }
        f32x16 acc[2][CS_NJ];  // set by the first multiplications (zero as their addend)
        if (FILTER && threadIdx.x < CS_TQ) {  // visible after the barriers of the first chunk
            const int row = q0 + (int)threadIdx.x;
            s_bound[threadIdx.x] = row < nqc ? pilot[(size_t)row * pstride + koff] : -INFINITY;
            s_cnt[threadIdx.x] = 0;
        }
        auto chunk = [&](int kc, bool first) {
            __syncthreads();  // the previous chunk has been consumed
            cs_store_chunk<CS_TQ / RPP>(As, ra);
            cs_store_chunk<CS_TC / RPP>(Bs, rb);
            __syncthreads();
            if (kc + 1 < nch) load(kc + 1);  // in flight during the multiplications
            auto step = [&](int kk, bool zero_addend) {
                const int ka = (kk + (l >> 5)) * LDA + (l & 31) + wr * 64;
                const int kb = (kk + (l >> 5)) * LDB + (l & 31) + wc * (32 * CS_NJ);
                const float a0 = As[ka], a1 = As[ka + 32];
                float bv[CS_NJ];
#pragma unroll
                for (int j = 0; j < CS_NJ; ++j) bv[j] = Bs[kb + 32 * j];
#pragma unroll
                for (int j = 0; j < CS_NJ; ++j) {
                    if (zero_addend) {
                        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                        acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, bv[j], zero, 0, 0, 0);
                        acc[1][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, bv[j], zero, 0, 0, 0);
                    } else {
                        acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, bv[j], acc[0][j], 0, 0, 0);
                        acc[1][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, bv[j], acc[1][j], 0, 0, 0);
                    }
                }
            };
            step(0, first);
#pragma unroll CS_KK_UNROLL
            for (int kk = 2; kk < CS_KC; kk += 2) step(kk, false);
        };
        chunk(0, true);
        for (int kc = 1; kc < nch; ++kc) chunk(kc, false);
        // element r of a 32 x 32 result: row (r/4)*8 + (lane/32)*4 + r%4, column lane%32
        //
        // FILTER: 1.6 % of the results survive, about one lane in two of the wave's 128 compares.
        // A survivor is only pushed, as (score bits, local row << 16 | local column), onto a queue
        // of its wave in the operand buffers (position: a wave-uniform count plus the lane's rank
        // among the survivors, no atomic); the queue is emptied densely afterwards, one entry per
        // lane: position in the (query, cell block) list by an LDS atomic, then the 8-byte store.
        constexpr uint32_t QCAP = CS_KC * LDB / 2 / CS_NW;  // entries per wave: its share of Bs
        constexpr int RG = QCAP >= 16 * QADC_WAVE ? 4 : 2;  // groups of four rows between two looks at the room
        uint2 *queue = (uint2 *)Bs + w * QCAP;
        uint32_t nqueued = 0;  // wave-uniform
        auto flush = [&]() {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            for (uint32_t e = (uint32_t)l; e < nqueued; e += QADC_WAVE) {
                const uint2 v = queue[e];
                const int rl = (int)(v.y >> 16), cl = (int)(v.y & 0xffffu);
                const uint32_t pos = atomicAdd(&s_cnt[rl], 1u);
                if (pos < CS_SLOT)
                    slots[((size_t)(q0 + rl) * ncb + cbx) * CS_SLOT + pos] =
                        ((uint64_t)qadc_f2ord(__uint_as_float(v.x)) << 32) | (uint32_t)(c0 + cl);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            nqueued = 0;
        };
        if (FILTER) __syncthreads();  // every wave has read its last operands: Bs is free
#pragma unroll
        for (int j = 0; j < CS_NJ; ++j) {
            const int cl = wc * (32 * CS_NJ) + j * 32 + (l & 31), col = c0 + cl;
            const bool colok = col < K;
            const uint64_t colmask = __ballot(colok);
            const uint32_t pl = ((uint32_t)(wr * 64 + (l >> 5) * 4) << 16) | (uint32_t)cl;  // first row | column
            if (!FILTER && !colok) continue;
            const float cn = cnv[j];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                // room for the next 4 RG results per lane (looked at here, not at every result:
                // the flush code exists a few times instead of 128)
                static_assert(4 * RG * QADC_WAVE <= QCAP, "the survivors between two looks fit the queue");
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    if (FILTER && r4 % RG == 0 && nqueued + 4 * RG * QADC_WAVE > QCAP) flush();
                    const int rl0 = wr * 64 + i * 32 + r4 * 8 + (l >> 5) * 4;
                    float bnd[4] = {0.f, 0.f, 0.f, 0.f};
                    if (FILTER) {  // four consecutive rows: their bounds come as one 16-byte LDS read
                        const float4 b4 = *(const float4 *)&s_bound[rl0];
                        bnd[0] = b4.x; bnd[1] = b4.y; bnd[2] = b4.z; bnd[3] = b4.w;
                    }
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const int rl = rl0 + rr, row = q0 + rl;
                        const float sc = __fmaf_rn(-2.0f, acc[i][j][4 * r4 + rr], cn);
                        if (!FILTER) {
                            if (row < nqc) scores[(size_t)row * ld + col] = sc;
                        } else {
                            // (the compare's lane mask taken as it is: a ballot of the combined
                            // condition costs two more vector instructions per result)
                            const uint64_t m = __builtin_amdgcn_fcmpf(sc, bnd[rr], 5 /* ordered <= */) & colmask;
                            if (m != 0) {
                                const bool pass = colok && sc <= bnd[rr];  // rows past the end: bound -inf
                                if (pass) {
                                    const uint32_t at = nqueued + __builtin_amdgcn_mbcnt_hi(
                                        (uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                                    queue[at] = make_uint2(__float_as_uint(sc), pl + ((uint32_t)(i * 32 + r4 * 8 + rr) << 16));
                                }
                                nqueued = __builtin_amdgcn_readfirstlane(nqueued + (uint32_t)__popcll(m));
                            }
                        }
                    }
                }
            }
        }
        if (FILTER) flush();
        if (FILTER) {
            __syncthreads();
            if (threadIdx.x < CS_TQ && q0 + (int)threadIdx.x < nqc)
                counts[(size_t)(q0 + threadIdx.x) * ncb + cbx] = s_cnt[threadIdx.x];  // uncapped
        }
    }
}

// -------------------------------------------------------------------- k_select ---
// One block of 1024 threads per query; keys = order-preserving integers of the scores; the
// result is the k = min(nprobe, K) smallest (key, id), ascending.
//
// Fast path: the scores are binned into 256 equal steps between the smallest and the largest; the
// nearest cells sit in the sparse low tail, so the bin that holds the k-th key and the bins
// below it hold only a few cells more than k.  They are gathered into LDS and ranked by
// counting.  Three passes over the query's scores (range, histogram, gather), which stay in L2.
// Exact path (taken when those bins hold more than CS_CAND cells, e.g. many equal scores): four
// radix passes give the k-th key and how many keys lie below it; the keys below it and the
// lowest ids among its equals are collected and ranked.
#define CS_CAND 2048
#define CS_SMALL_CAP 1024  // candidates a 256-thread k_select_cand block ranks

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

// guard: if non-null and *guard == 0 the kernel does nothing.  clear: if non-null, set to 0.
template <int BD>  // threads per block: 256 (a few thousand scores) or 1024
__global__ void __launch_bounds__(BD)
k_select(const float *__restrict__ scores, size_t ld, int K, int nprobe,
         int32_t *__restrict__ probe_ids, float *__restrict__ probe_scores,
         const int *__restrict__ guard, int *__restrict__ clear) {
    if (guard && *guard == 0) return;
    if (clear && blockIdx.x == 0 && threadIdx.x == 0) *clear = 0;
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
    // 16-byte loads: thread t takes scores 4*(j*BD + t) .. +3, UB loads in flight together.
    // Row starts are 128-byte aligned and padded to a multiple of 32 scores; what lies past K is
    // masked by index.
    constexpr int UB = 8;
    const int nj = (K + 4 * BD - 1) / (4 * BD);
    auto load_keys = [&](int j0, uint32_t (&v)[UB][4]) {
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int i = ((j0 + u) * BD + (int)threadIdx.x) * 4;
            float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < K) f = *(const float4 *)(s + i);
            v[u][0] = i + 0 < K ? qadc_f2ord(f.x) : 0xffffffffu;
            v[u][1] = i + 1 < K ? qadc_f2ord(f.y) : 0xffffffffu;
            v[u][2] = i + 2 < K ? qadc_f2ord(f.z) : 0xffffffffu;
            v[u][3] = i + 3 < K ? qadc_f2ord(f.w) : 0xffffffffu;
        }
    };

    // Up to RC rounds of keys (the pilot's few thousand scores) stay in registers after the first
    // pass: the three passes are bound by the memory system, not by their arithmetic.
    constexpr int RC = 4;
    const bool cached = nj <= RC;  // (block-uniform)
    uint32_t kc[RC][4];
    auto keys = [&](int j0, uint32_t (&v)[UB][4]) {
        if (cached) {
#pragma unroll
            for (int u = 0; u < UB; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c) v[u][c] = u < RC ? kc[u < RC ? u : 0][c] : 0xffffffffu;
        } else {
            load_keys(j0, v);
        }
    };
    // range of the keys
    uint32_t lo = 0xffffffffu, hi = 0u;
    for (int j0 = 0; j0 < nj; j0 += UB) {
        uint32_t v[UB][4];
        load_keys(j0, v);
        if (cached) {
#pragma unroll
            for (int u = 0; u < RC; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c) kc[u][c] = v[u][c];
        }
#pragma unroll
        for (int u = 0; u < UB; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (((j0 + u) * BD + (int)threadIdx.x) * 4 + c < K) {
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
    for (int w2 = 0; w2 < BD / QADC_WAVE; ++w2) {
        lo = s_lo[w2] < lo ? s_lo[w2] : lo;
        hi = s_hi[w2] > hi ? s_hi[w2] : hi;
    }
    // 256 equal steps of the score itself between the smallest and the largest (equal steps of the
    // ordered integer would put nearly every score into the top bins whenever the smallest score
    // is negative and the others are not: the integers of floats near zero are far apart)
    const float flo = qadc_ord2f(lo), fspan = qadc_ord2f(hi) - qadc_ord2f(lo);
    const float fscale = (fspan > 0.0f && isfinite(fspan)) ? 255.0f / fspan : 0.0f;
    auto bin_of = [flo, fscale](uint32_t key) -> uint32_t {
        const float x = (qadc_ord2f(key) - flo) * fscale;  // >= 0, monotone in the key
        return x >= 255.0f ? 255u : (uint32_t)x;
    };
    for (int j0 = 0; j0 < nj; j0 += UB) {
        uint32_t v[UB][4];
        keys(j0, v);
#pragma unroll
        for (int u = 0; u < UB; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool in = ((j0 + u) * BD + (int)threadIdx.x) * 4 + c < K;
                cs_hist_add(hist, in ? bin_of(v[u][c]) : 0u, in);
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
            keys(j0, v);
#pragma unroll
            for (int u = 0; u < UB; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int i = ((j0 + u) * BD + (int)threadIdx.x) * 4 + c;
                    const bool take = i < K && bin_of(v[u][c]) <= kbin;
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
#define CS_KEYM(j) ((j) * BD + (int)threadIdx.x < K ? qadc_f2ord(s[(j) * BD + threadIdx.x]) : 0xffffffffu)
    const int njm = (K + BD - 1) / BD;
    __syncthreads();
    uint32_t prefix = 0, mask = 0, kk = (uint32_t)k;
    for (int pass = 3; pass >= 0; --pass) {
        const int sh = pass * 8;
        for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
        __syncthreads();
        for (int j = 0; j < njm; ++j) {
            const uint32_t v = CS_KEYM(j);
            const bool in = j * BD + (int)threadIdx.x < K && (v & mask) == prefix;
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
        const int i = j * BD + (int)threadIdx.x;
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
    // cells equal to the k-th key: the `need` lowest ids.  Rounds of BD consecutive ids in
    // ascending order; within a round positions come from the wave counts.
    for (int j = 0; j < njm; ++j) {
        const int i = j * BD + (int)threadIdx.x;
        const bool eq = i < K && CS_KEYM(j) == kth;
        const uint64_t m = __ballot(eq);
        if (lane == 0) wcnt[wave] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t before = s_ties, total = 0;
        for (int w2 = 0; w2 < BD / QADC_WAVE; ++w2) {
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

// ---------------------------------------------------------------- k_select_cand ---
// One block of NT threads per query: gather the query's candidate lists (one per block of 256
// cells), keep those up to the bin of the k-th (at most ACAP), rank by (score, id).  256 threads
// take the lists of up to 65,536 cells in one batch and leave room for eight blocks per CU.  An
// overflowing list, or more candidates than fit, raises *flag.
template <int NT, int ACAP>
__global__ void __launch_bounds__(NT)
k_select_cand(const uint32_t *__restrict__ counts, const uint64_t *__restrict__ slots, int ncb,
              const float *__restrict__ pilot, int pstride, int koff, int K, int nprobe, int logw,
              int32_t *__restrict__ probe_ids, float *__restrict__ probe_scores, int *__restrict__ flag) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint64_t *A = (uint64_t *)smem;  // ACAP entries
    __shared__ uint32_t hist[256];
    __shared__ uint32_t whist[NT / QADC_WAVE][256];
    __shared__ uint32_t sh[32];
    __shared__ uint32_t wsum[16];
    const size_t q = blockIdx.x;
    const int k = nprobe < K ? nprobe : K;
    // 256 equal steps of the score itself between the pilot's best score and the bound (not of
    // the ordered integer: see k_select); better scores than the pilot's best go to bin 0
    const float flo = pilot[q * pstride], fspan = pilot[q * pstride + koff] - flo;
    const float fscale = (fspan > 0.0f && isfinite(fspan)) ? 255.0f / fspan : 0.0f;
    FinalShared S;
    S.hist = hist;
    S.whist = whist;
    S.sh = sh;
    S.wsum = wsum;
    S.off = nullptr;
    auto binf = [flo, fscale](uint64_t c) -> uint32_t {
        const float x = (qadc_ord2f((uint32_t)(c >> 32)) - flo) * fscale;  // monotone in the key
        return x >= 255.0f ? 255u : (x > 0.0f ? (uint32_t)x : 0u);
    };
    int na = 0;
    const int per_batch = (ncb + (NT >> logw) - 1) / (NT >> logw);
    bool slow;
    const uint32_t *cq = counts + q * ncb;
    const uint64_t *sq = slots + q * ncb * CS_SLOT;
    if (per_batch <= 8)
        slow = gather_select_rows<8, NT, ACAP>(cq, sq, ncb, CS_SLOT, k, logw, binf, A, S, na);
    else if (per_batch <= 16)
        slow = gather_select_rows<16, NT, ACAP>(cq, sq, ncb, CS_SLOT, k, logw, binf, A, S, na);
    else
        slow = gather_select_rows<32, NT, ACAP>(cq, sq, ncb, CS_SLOT, k, logw, binf, A, S, na);
    if (slow) {
        if (threadIdx.x == 0) atomicOr(flag, 1);
        return;
    }
    cs_rank_and_write(A, na, k, nprobe, probe_ids + q * nprobe,
                      probe_scores ? probe_scores + q * nprobe : nullptr);
}

// ------------------------------------------------------------------------ host ---
static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

// Queries per pass: as many as a 1 GiB score matrix (the fallback's) holds.  Larger passes give the
// pilot, the selections and the guarded fallback launches more blocks each (10,000 queries over
// 65,536 cells: 2.70 ms per call with 256 MiB, 2.42 with 512 MiB, 2.29 with 1 GiB).
#define QADC_COARSE_MATRIX_BYTES ((size_t)1 << 30)
static int coarse_chunk(int nq, int K) {
    const size_t ld = ((size_t)K + 31) & ~(size_t)31;
    size_t qc = ((size_t)QADC_COARSE_MATRIX_BYTES) / (ld * sizeof(float));
    qc = qc / CS_TQ * CS_TQ;
    if (qc < CS_TQ) qc = CS_TQ;
    const size_t nqr = ((size_t)(nq > 0 ? nq : 1) + CS_TQ - 1) / CS_TQ * CS_TQ;
    return (int)(qc < nqr ? qc : nqr);
}

// one k_scores block per tile, cell blocks fastest
static unsigned cs_grid(unsigned gx, unsigned gy) { return gx * gy; }

// The filtering form: pilot size (0 = use the matrix form) and what it needs per pass of qc queries.
static int coarse_pilot(int K, int nprobe) {
    const bool off = qadc_option(PQ_OPT_COARSE_FILTER) == 0;
    int64_t P = 64 * (int64_t)nprobe;
    if (P < 4096) P = 4096;
    P = (P + CS_TC - 1) / CS_TC * CS_TC;
    const int64_t ncb = ((int64_t)K + CS_TC - 1) / CS_TC;
    if (off || P > K / 4 || ncb > MAX_G) return 0;
    return (int)P;
}
static size_t coarse_filter_bytes(int qc, int K, int nprobe) {
    const size_t ncb = ((size_t)K + CS_TC - 1) / CS_TC;
    return up256((size_t)qc * ncb * CS_SLOT * sizeof(uint64_t)) + up256((size_t)qc * ncb * sizeof(uint32_t)) +
           up256((size_t)qc * nprobe * sizeof(int32_t)) + up256((size_t)qc * nprobe * sizeof(float)) + 256;
}

extern "C" size_t ivf_coarse_workspace_bytes(int nq, int K) {
    if (nq < 0 || K < 1) return 0;
    const size_t ld = ((size_t)K + 31) & ~(size_t)31;
    const int qc = coarse_chunk(nq, K);
    return up256((size_t)K * sizeof(float)) + up256((size_t)qc * ld * sizeof(float)) +
           coarse_filter_bytes(qc, K, CS_MAX_NPROBE);
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
    const int P = coarse_pilot(K, nprobe);
    const int ncb = (K + CS_TC - 1) / CS_TC;
    char *fb = (char *)scores + up256((size_t)qc * ld * sizeof(float));
    uint64_t *slots = (uint64_t *)fb;
    uint32_t *counts = (uint32_t *)(fb + up256((size_t)qc * ncb * CS_SLOT * sizeof(uint64_t)));
    int32_t *pilot_ids = (int32_t *)((char *)counts + up256((size_t)qc * ncb * sizeof(uint32_t)));
    float *pilot_sc = (float *)((char *)pilot_ids + up256((size_t)qc * nprobe * sizeof(int32_t)));
    int *flag = (int *)((char *)pilot_sc + up256((size_t)qc * nprobe * sizeof(float)));
    // expected candidates per list: CS_TC nprobe / P <= 4
    const int logw = 3;
    for (int q0 = 0; q0 < nq; q0 += qc) {
        const int nqc = nq - q0 < qc ? nq - q0 : qc;
        const float *qp = queries + (size_t)q0 * d;
        int32_t *pid = probe_ids + (size_t)q0 * nprobe;
        float *psc = probe_scores ? probe_scores + (size_t)q0 * nprobe : nullptr;
        const dim3 gq((K + CS_TC - 1) / CS_TC, (nqc + CS_TQ - 1) / CS_TQ);
        const int *guard = nullptr;
        if (P > 0) {
            // pilot: matrix form over the first P cells -> bound and best score per query
            hipLaunchKernelGGL(k_scores<false>, dim3(cs_grid(P / CS_TC, gq.y)), dim3(CS_NT), 0, s, qp, nqc,
                               centroids, P, d, cnorm, scores, (size_t)P, vec, (const float *)nullptr, 0, 0,
                               (uint64_t *)nullptr, (uint32_t *)nullptr, (const int *)nullptr, P / CS_TC,
                               (int)gq.y);
            QADC_LAUNCH_CHECK("k_scores (pilot)");
            hipLaunchKernelGGL(k_select<256>, dim3(nqc), dim3(256), 0, s, scores, (size_t)P, P, nprobe, pilot_ids,
                               pilot_sc, (const int *)nullptr, flag);
            QADC_LAUNCH_CHECK("k_select (pilot)");
            hipLaunchKernelGGL(k_scores<true>, dim3(cs_grid(gq.x, gq.y)), dim3(CS_NT), 0, s, qp, nqc, centroids, K,
                               d, cnorm, (float *)nullptr, ld, vec, (const float *)pilot_sc, nprobe, nprobe - 1,
                               slots, counts, (const int *)nullptr, (int)gq.x, (int)gq.y);
            QADC_LAUNCH_CHECK("k_scores (filter)");
            if (ncb <= (256 >> logw) * 8 && nprobe <= CS_SMALL_CAP / 8)
                hipLaunchKernelGGL((k_select_cand<256, CS_SMALL_CAP>), dim3(nqc), dim3(256),
                                   CS_SMALL_CAP * sizeof(uint64_t), s, (const uint32_t *)counts,
                                   (const uint64_t *)slots, ncb, (const float *)pilot_sc, nprobe, nprobe - 1, K,
                                   nprobe, logw, pid, psc, flag);
            else
                hipLaunchKernelGGL((k_select_cand<1024, FINAL_CAP>), dim3(nqc), dim3(1024),
                                   FINAL_CAP * sizeof(uint64_t), s, (const uint32_t *)counts,
                                   (const uint64_t *)slots, ncb, (const float *)pilot_sc, nprobe, nprobe - 1, K,
                                   nprobe, logw, pid, psc, flag);
            QADC_LAUNCH_CHECK("k_select_cand");
            guard = flag;  // the matrix form below only runs if a list overflowed
        }
        hipLaunchKernelGGL(k_scores<false>, dim3(cs_grid(gq.x, gq.y)), dim3(CS_NT), 0, s, qp, nqc, centroids, K, d,
                           cnorm, scores, ld, vec, (const float *)nullptr, 0, 0, (uint64_t *)nullptr,
                           (uint32_t *)nullptr, guard, (int)gq.x, (int)gq.y);
        QADC_LAUNCH_CHECK("k_scores");
        hipLaunchKernelGGL(k_select<1024>, dim3(nqc), dim3(1024), 0, s, scores, ld, K, nprobe, pid, psc, guard,
                           (int *)nullptr);
        QADC_LAUNCH_CHECK("k_select");
    }
    return PQ_OK;
}
