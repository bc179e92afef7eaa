// pq_adc_scan_topk: scan of packed codes with quantized tables (eq. (2),
// Section 3.4 saturating sums, Section 3.5) and exact top-R by (key, id).
//
//   k_scan   G blocks per query stream the codes once.  A code is kept when its key is <=
//            the query's bound (an upper bound on the R-th best key, so nothing that can be
//            a result is dropped) and appended to the query's candidate list in the
//            workspace (one atomic add per wave that holds candidates).
//   k_final  one block per query reads the list, finds the R-th key by histogram, ranks the
//            few candidates up to it by (key, id) and writes the R best.  If the list
//            overflowed (huge tie classes, or a caller that supplied no bound) it runs an
//            exact two-pass selection over all codes instead.
// The result is defined as a sort by (key, id), so it does not depend on the order in which
// blocks run or candidates arrive.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "scan_device.h"

#ifndef SCAN_THREADS
#define SCAN_THREADS 256
#endif
#ifndef QADC_U8
#define QADC_U8 2
#endif
#ifndef QADC_U5
#define QADC_U5 1
#endif
constexpr int U8 = QADC_U8;  // 16-byte chunks per thread and tile, 8-byte codes
constexpr int U5 = QADC_U5;  // 20-byte chunks per thread and tile, 5-byte codes

// ------------------------------------------------------------- k_prepare ---
// One block per query: the query's group tables, written where k_scan blocks pick them up.
template <int KIND, typename QT>
__global__ void __launch_bounds__(256)
k_prepare(const DevLayout *__restrict__ L, const void *__restrict__ qtables, char *__restrict__ ws,
          size_t per_query, size_t gtab_off) {
    extern __shared__ __align__(16) unsigned char smem[];
    QT *gtab = (QT *)smem;
    uint16_t *qs = (uint16_t *)(smem + (((size_t)L->gtab_len * sizeof(QT) + 15) & ~(size_t)15));
    const size_t q = blockIdx.x;
    stage_qtable<QT>((const QT *)qtables + q * L->T, L->T, qs);
    build_gtab<KIND, QT>(L, qs, gtab);
    QT *dst = (QT *)(ws + q * per_query + gtab_off);
    for (int e = threadIdx.x; e < L->gtab_len; e += blockDim.x) dst[e] = gtab[e];
    scan_hdr_clear((ScanHdr *)(ws + q * per_query));  // empty candidate lists for the scan that follows
}

// Copy prepared group tables (a multiple of 16 bytes is allocated for them) into LDS.
template <typename QT>
__device__ __forceinline__ void load_gtab(const char *__restrict__ src, int gtab_len, QT *gtab) {
    const int n16 = (gtab_len * (int)sizeof(QT) + 15) >> 4;
    for (int i = threadIdx.x; i < n16; i += blockDim.x) ((uint4 *)gtab)[i] = ((const uint4 *)src)[i];
    __syncthreads();
}

// -------------------------------------------------------------- selection ---
struct FinalOut {
    int32_t *ids;
    uint16_t *keys;
    float *dist;
};

// Rank the na candidates of S.A by (key, id) and write the first R, padding the rest.  The
// candidates are first grouped by key bin (key >> shift, at most 256 bins) with a counting
// sort of their indices; a candidate's rank is the number of candidates in lower bins plus
// the number of smaller ones within its bin.  Block of NT threads.
template <int NT, int ACAP>
__device__ inline void rank_and_write(SelectLds<NT, ACAP> &S, int na, int R, const pq_qparams_t &prm,
                                      uint32_t qmax, const FinalOut &o, int shift) {
    const float fdelta = (float)prm.delta, fdmin = (float)prm.d_min;
    const uint64_t *A = S.A;
    if (na <= 2 * NT) {
        // few candidates (the usual case): every candidate counts the smaller ones; all lanes
        // read the same entry at a time
        for (int i = threadIdx.x; i < na; i += NT) {
            const uint64_t mine = A[i];
            int r = 0;
            for (int j = 0; j < na; ++j) r += (A[j] < mine) ? 1 : 0;
            if (r < R) {
                const uint32_t key = (uint32_t)(mine >> 32);
                o.ids[r] = (int32_t)(uint32_t)mine;
                o.keys[r] = (uint16_t)key;
                o.dist[r] = fmaf((float)key, fdelta, fdmin);
            }
        }
    } else {
        uint32_t *cnt = &S.whist[0][0], *start = cnt + 256, *fill = cnt + 512;  // (NT >= 256: 1024 words there)
        for (int i = threadIdx.x; i < 768; i += NT) cnt[i] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < na; i += NT) atomicAdd(&cnt[((uint32_t)(A[i] >> 32) >> shift) & 255u], 1u);
        __syncthreads();
        if (threadIdx.x < QADC_WAVE) {  // exclusive prefix of the 256 counts, four bins per lane
            const int lane = threadIdx.x;
            uint32_t c[4], sum = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                c[k] = cnt[4 * lane + k];
                sum += c[k];
            }
            uint32_t run = qadc_wave_incl_scan(sum) - sum;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                start[4 * lane + k] = run;
                run += c[k];
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < na; i += NT) {
            const uint32_t b = ((uint32_t)(A[i] >> 32) >> shift) & 255u;
            S.order[start[b] + atomicAdd(&fill[b], 1u)] = (uint16_t)i;
        }
        __syncthreads();
        for (int p = threadIdx.x; p < na; p += NT) {
            const uint64_t mine = A[S.order[p]];
            const uint32_t b = ((uint32_t)(mine >> 32) >> shift) & 255u;
            const int gs = (int)start[b], ge = gs + (int)cnt[b];
            int r = gs;
            if (gs < R) {  // (a whole bin at or beyond rank R cannot hold a result)
                for (int j = gs; j < ge; ++j) r += (A[S.order[j]] < mine) ? 1 : 0;
                if (r < R) {
                    const uint32_t key = (uint32_t)(mine >> 32);
                    o.ids[r] = (int32_t)(uint32_t)mine;
                    o.keys[r] = (uint16_t)key;
                    o.dist[r] = fmaf((float)key, fdelta, fdmin);
                }
            }
        }
    }
    for (int r = (na < R ? na : R) + threadIdx.x; r < R; r += NT) {
        o.ids[r] = -1;
        o.keys[r] = (uint16_t)qmax;
        o.dist[r] = INFINITY;
    }
}

// Exact selection over all n codes by one block: histogram of key bins (two
// levels for 16-bit keys) gives the R-th key k*; a second pass in id order keeps
// every code below k* and the first (R - count_below) codes equal to k*.  A receives
// min(R, n) entries; their number is left in sh[2].
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
        if (threadIdx.x < QADC_WAVE) qadc_wave_select_bin(hist, (uint32_t)Rn, below, sh);
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

// The selection of one query by a block of NT threads: from the candidate list, or from the
// codes when the list overflowed.  gtab: the query's group tables in LDS if the caller has
// them there already, else null (they are then staged from gsrc on the slow path only, into
// gtab_room).  COHERENT: see select_from_list.
template <int KIND, typename QT, int NT, int ACAP, bool COHERENT>
__device__ inline void select_query(const DevLayout *L, const char *__restrict__ wq, size_t cand_off,
                                    size_t gtab_off, uint32_t cap, const uint8_t *__restrict__ codes,
                                    int64_t n, int R, const pq_qparams_t &prm, const FinalOut &o,
                                    SelectLds<NT, ACAP> &S, const QT *gtab, QT *gtab_room) {
    const int shift = L->acc_bits == 8 ? 0 : 8;
    const uint32_t qmax = (uint32_t)L->qmax;
    // (inside the scan kernel, whose register budget is small, half as many entries per round:
    // sixteen made the compiler reserve per-lane scratch memory for every scan block)
    int na = select_from_lists<NT, ACAP, COHERENT, COHERENT ? 8 : 16>((const ScanHdr *)wq,
                                                                      (const uint64_t *)(wq + cand_off), cap, R, shift, S);
    if (na < 0) {
        if (!gtab) {
            const int n16 = (L->gtab_len * (int)sizeof(QT) + 15) >> 4;
            for (int i = threadIdx.x; i < n16; i += NT) ((uint4 *)gtab_room)[i] = ((const uint4 *)(wq + gtab_off))[i];
            __syncthreads();
            gtab = gtab_room;
        }
        exact_select<KIND, QT>(L, gtab, codes, n, R, S.A, S.hist, S.sh);
        __syncthreads();
        na = (int)S.sh[2];
        __syncthreads();
    }
    rank_and_write<NT, ACAP>(S, na, R, prm, qmax, o, shift);
}

// ---------------------------------------------------------------- k_scan ---
// NG > 0: the layout has NG groups (per 64-bit half for 16-byte irregular codes), none
// crossing a dword boundary of the code; NG == 0: group descriptors are read from the layout.
// MODE says where the groups lie: 0 = decided per group at run time, 1 = the first NG/2 in the
// low dword, 2 = all but the last in the low dword.
// (Eight waves per SIMD, i.e. at most 64 vector registers: the streaming loop needs a fraction
// of that, and the selection at the end, which runs in one block per query, must not cost the
// loop its occupancy.)
template <int KIND, typename QT, int NG, int MODE>
__global__ void __launch_bounds__(SCAN_THREADS) __attribute__((amdgpu_waves_per_eu(8, 8)))
k_scan(const DevLayout *__restrict__ L, const void *__restrict__ qtables,
       const pq_qparams_t *__restrict__ qparams, const uint8_t *__restrict__ codes, int64_t n,
       char *__restrict__ ws, size_t per_query, size_t cand_off, size_t gtab_off, uint32_t cap,
       int gtab_len, uint32_t qmax, GroupDesc gd, int fuse, int R, int32_t *__restrict__ out_ids,
       uint16_t *__restrict__ out_keys, float *__restrict__ out_dist,
       const uint16_t *__restrict__ bound_rec, int recP, uint32_t reck) {
    extern __shared__ __align__(16) unsigned char smem[];
    QT *gtab = (QT *)smem;
    __shared__ uint32_t s_last, s_bin[SCAN_THREADS / QADC_WAVE];
    const size_t q = blockIdx.y;
    const int b = blockIdx.x, G = gridDim.x;
    char *wq = ws + q * per_query;
    const int sl = b % QADC_NSUB;  // this block's candidate list
    uint32_t *count = &((ScanHdr *)wq)->count[sl][0];
    uint64_t *cand = (uint64_t *)(wq + cand_off) + (size_t)sl * cap;
    const char *gsrc = wq + gtab_off;
    // this wave's staging buffer for candidates, behind the tables (the selection at the end
    // reuses the room: every wave has emptied its buffer by then)
    uint64_t *wbuf = (uint64_t *)(smem + (((size_t)gtab_len * sizeof(QT) + 15) & ~(size_t)15)) +
                     (threadIdx.x / QADC_WAVE) * QADC_WSTAGE;
    uint32_t nbuf = 0;
    // Sums are compared unsaturated.  A sum above q_max is the key q_max (Section 3.4), an
    // ordinary largest key: with a bound below q_max such a code never passes, and with the
    // bound at q_max every code does (the keys are saturated where they are stored).
    // The bound: from the query's parameters, or (bound_rec) added up from the records the
    // quantizer's pilot blocks left; the waves' parts meet in LDS behind the barrier that ends
    // the staging of the tables.
    const pq_qparams_t prm = qparams[q];  // (delta and d_min are used by the selection at the very end)
    uint32_t thr = prm.key_bound;
    if (bound_rec) scan_bound_bins_256(bound_rec + q * (QADC_REC_BINS * QADC_REC_SLOTS), recP, reck, s_bin);
    constexpr bool g32 = NG > 0;
    constexpr int NLO = MODE == 1 ? NG / 2 : (MODE == 2 ? NG - 1 : -1);

    if (KIND == SCAN_NIB8 || KIND == SCAN_W64) {
        // 16-byte chunks of two codes, U8 chunks per thread and tile (U8*16 bytes per lane in
        // flight); an odd last code is handled after the loop
        // (chunk indices fit 32 bits: ids are int32, so n < 2^31)
        constexpr int U = U8;
        const int nfull = (int)(n >> 1);
        const int ntiles = (nfull + U * SCAN_THREADS - 1) / (U * SCAN_THREADS);
        const uint4 *__restrict__ p = (const uint4 *)codes;
        uint4 cur[U];
        int tile = b;
        auto load_tile = [&](int t) {  // t < ntiles, hence nfull >= 1; past the end: the last chunk again
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = t * (U * SCAN_THREADS) + u * SCAN_THREADS + (int)threadIdx.x;
                cur[u] = p[c < nfull ? c : nfull - 1];
            }
        };
        if (tile < ntiles) load_tile(tile);  // in flight while the tables are staged
        load_gtab<QT>(gsrc, gtab_len, gtab);
        if (bound_rec) thr = scan_bound_of_bin(min(min(s_bin[0], s_bin[1]), min(s_bin[2], s_bin[3])), sizeof(QT) == 1 ? 0 : 8, qmax);
        thr = thr >= qmax ? 0xffffffffu : thr;
        while (tile < ntiles) {
            uint32_t s[2 * U];
            bool pass[2 * U], any = false;
            // 64-bit irregular codes: the next tile is requested before this one is looked up (their
            // look-ups take longer than the m x 4 kind's, for which the later request measured faster)
            constexpr bool EARLY = KIND != SCAN_NIB8;
            uint4 w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) w[u] = cur[u];
            if (EARLY && tile + G < ntiles) load_tile(tile + G);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = tile * (U * SCAN_THREADS) + u * SCAN_THREADS + (int)threadIdx.x;
                if (KIND == SCAN_NIB8) {
                    s[2 * u] = sum8(gtab, w[u].x, w[u].y);
                    s[2 * u + 1] = sum8(gtab, w[u].z, w[u].w);
                } else if (g32) {
                    s[2 * u] = sum_groups_desc<NG, NLO>(gd, gtab, w[u].x, w[u].y);
                    s[2 * u + 1] = sum_groups_desc<NG, NLO>(gd, gtab, w[u].z, w[u].w);
                } else {
                    s[2 * u] = sum_groups64(L, gtab, ((uint64_t)w[u].y << 32) | w[u].x);
                    s[2 * u + 1] = sum_groups64(L, gtab, ((uint64_t)w[u].w << 32) | w[u].z);
                }
                pass[2 * u] = (c < nfull) && s[2 * u] <= thr;
                pass[2 * u + 1] = (c < nfull) && s[2 * u + 1] <= thr;
                any = any || pass[2 * u] || pass[2 * u + 1];
            }
            if (__ballot(any) != 0) {
                uint32_t id[2 * U];
#pragma unroll
                for (int u = 0; u < 2 * U; ++u) {
                    const int c = tile * (U * SCAN_THREADS) + (u >> 1) * SCAN_THREADS + (int)threadIdx.x;
                    id[u] = (uint32_t)(2 * c + (u & 1));
                    s[u] = s[u] > qmax ? qmax : s[u];
                }
                stage_append_multi<2 * U>(pass, s, id, wbuf, nbuf, cand, cap, count);
            }
            tile += G;
            if (!EARLY && tile < ntiles) load_tile(tile);
        }
        if ((n & 1) && b == 0) {  // the odd last code, by one wave of block 0
            if (threadIdx.x < QADC_WAVE) {
                const bool me = threadIdx.x == 0;
                uint32_t key = 0;
                if (me) {
                    uint2 w = *(const uint2 *)(codes + (n - 1) * 8);
                    key = KIND == SCAN_NIB8 ? sum8(gtab, w.x, w.y)
                                            : sum_groups64(L, gtab, ((uint64_t)w.y << 32) | w.x);
                }
                stage_append(me && key <= thr, key > qmax ? qmax : key, (uint32_t)(n - 1), wbuf, nbuf, cand, cap, count);
            }
        }
    } else if (KIND == SCAN_C5) {
        // 20-byte chunks of four 5-byte codes: five dwords per lane, U5 chunks per thread and
        // tile; the last n % 4 codes are handled after the loop
        constexpr int U = U5;
        // (chunk and dword indices fit 32 bits: ids are int32, so n < 2^31 and 5 * (n / 4) < 2^32)
        const uint32_t nfull = (uint32_t)(n >> 2);
        const uint32_t ntiles = (nfull + U * SCAN_THREADS - 1) / (U * SCAN_THREADS);
        const uint32_t *__restrict__ p = (const uint32_t *)codes;
        uint32_t cur[U][5];
        uint32_t tile = b;
        auto load_tile = [&](uint32_t t) {  // t < ntiles, hence nfull >= 1; past the end: the last chunk again
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t c = t * (U * SCAN_THREADS) + u * SCAN_THREADS + threadIdx.x;
                const uint32_t *__restrict__ pc = p + (c < nfull ? c : nfull - 1) * 5u;
#pragma unroll
                for (int i = 0; i < 5; ++i) cur[u][i] = pc[i];
            }
        };
        if (tile < ntiles) load_tile(tile);  // the first tile is in flight while the tables are staged
        load_gtab<QT>(gsrc, gtab_len, gtab);
        if (bound_rec) thr = scan_bound_of_bin(min(min(s_bin[0], s_bin[1]), min(s_bin[2], s_bin[3])), sizeof(QT) == 1 ? 0 : 8, qmax);
        thr = thr >= qmax ? 0xffffffffu : thr;
        while (tile < ntiles) {
            uint32_t s[4 * U];
            bool pass[4 * U], any = false;
            // the next tile is requested before this one is looked up
            uint32_t w[U][5];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < 5; ++i) w[u][i] = cur[u][i];
            if (tile + G < ntiles) load_tile(tile + G);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t c = tile * (U * SCAN_THREADS) + u * SCAN_THREADS + threadIdx.x;
                // code v = bits [40v, 40v+40) of the 160-bit chunk, as (low dword, high byte)
                uint32_t lo[4], hi[4];
                lo[0] = w[u][0];
                hi[0] = w[u][1] & 0xffu;
                lo[1] = __builtin_amdgcn_alignbit(w[u][2], w[u][1], 8);
                hi[1] = (w[u][2] >> 8) & 0xffu;
                lo[2] = __builtin_amdgcn_alignbit(w[u][3], w[u][2], 16);
                hi[2] = (w[u][3] >> 16) & 0xffu;
                lo[3] = __builtin_amdgcn_alignbit(w[u][4], w[u][3], 24);
                hi[3] = w[u][4] >> 24;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    s[4 * u + v] = g32 ? sum_groups_desc<NG, NLO>(gd, gtab, lo[v], hi[v])
                                       : sum_groups64(L, gtab, ((uint64_t)hi[v] << 32) | lo[v]);
                    pass[4 * u + v] = (c < nfull) && s[4 * u + v] <= thr;
                    any = any || pass[4 * u + v];
                }
            }
            if (__ballot(any) != 0) {
                uint32_t id[4 * U];
#pragma unroll
                for (int u = 0; u < 4 * U; ++u) {
                    const uint32_t c = tile * (U * SCAN_THREADS) + (u >> 2) * SCAN_THREADS + threadIdx.x;
                    id[u] = 4u * c + (u & 3);
                    s[u] = s[u] > qmax ? qmax : s[u];
                }
                stage_append_multi<4 * U>(pass, s, id, wbuf, nbuf, cand, cap, count);
            }
            tile += G;
        }
        if ((n & 3) && b == 0 && threadIdx.x < QADC_WAVE) {  // the last n % 4 codes
            const int64_t id = (nfull << 2) + threadIdx.x;
            const bool me = id < n;
            uint32_t key = me ? key_at<KIND, QT>(L, gtab, codes, id) : 0u;
            stage_append(me && key <= thr, key, (uint32_t)id, wbuf, nbuf, cand, cap, count);
        }
    } else {
        // one 16-byte code (or one code of the byte-wise kind) per thread and chunk, four chunks
        // per tile; positions fit 32 bits unsigned (n < 2^31); loads past the end repeat the
        // last code
        const uint32_t un = (uint32_t)n;
        const uint32_t ntiles = (un + 4 * SCAN_THREADS - 1) / (4 * SCAN_THREADS);
        const uint4 *__restrict__ p = (const uint4 *)codes;
        uint4 cur[4];
        uint32_t tile = b;
        auto load_tile = [&](uint32_t t) {  // t < ntiles, hence n >= 1
            if (KIND != SCAN_NIB16 && KIND != SCAN_W128) return;  // others read byte by byte
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t c = t * (4 * SCAN_THREADS) + u * SCAN_THREADS + threadIdx.x;
                cur[u] = p[c < un ? c : un - 1];
            }
        };
        if (tile < ntiles) load_tile(tile);  // the first tile is in flight while the tables are staged
        load_gtab<QT>(gsrc, gtab_len, gtab);
        if (bound_rec) thr = scan_bound_of_bin(min(min(s_bin[0], s_bin[1]), min(s_bin[2], s_bin[3])), sizeof(QT) == 1 ? 0 : 8, qmax);
        thr = thr >= qmax ? 0xffffffffu : thr;
        while (tile < ntiles) {
            uint32_t s[4];
            bool pass[4], any = false;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t c = tile * (4 * SCAN_THREADS) + u * SCAN_THREADS + threadIdx.x;
                if (KIND == SCAN_NIB16)
                    s[u] = sum8(gtab, cur[u].x, cur[u].y) + sum8(gtab + 2048, cur[u].z, cur[u].w);
                else if (KIND == SCAN_W128)
                    s[u] = sum_groups_desc<NG, NLO>(gd, gtab, cur[u].x, cur[u].y) +
                           sum_groups_desc<NG, NLO>(gd, gtab, cur[u].z, cur[u].w, true);
                else
                    s[u] = c < un ? key_generic(L, gtab, codes + (size_t)c * L->cs) : 0u;
                pass[u] = (c < un) && s[u] <= thr;
                any = any || pass[u];
            }
            if (__ballot(any) != 0) {
                uint32_t id[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    id[u] = tile * (4 * SCAN_THREADS) + u * SCAN_THREADS + threadIdx.x;
                    s[u] = s[u] > qmax ? qmax : s[u];
                }
                stage_append_multi<4>(pass, s, id, wbuf, nbuf, cand, cap, count);
            }
            tile += G;
            if (tile < ntiles) load_tile(tile);
        }
    }
    stage_flush(wbuf, nbuf, cand, cap, count);
    if (!fuse) return;
    // Selection by the block that finishes last.  Candidates were stored and counted with
    // device-scope operations; every thread waits until its own have completed, then the block
    // counts itself in, and the block that completes the count reads all lists with
    // device-scope loads and turns them into the result.  (No cache write-back or invalidation
    // is involved: a release fence in each of the 2048 blocks made the kernel fifteen times
    // slower.)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        // two levels, because atomic adds to one address are served one by one (about 10 ns
        // each): first among the blocks of this block's list, then among the lists
        ScanHdr *hd = (ScanHdr *)wq;
        const uint32_t in_list = (uint32_t)(G - sl + QADC_NSUB - 1) / QADC_NSUB;
        const uint32_t lists = (uint32_t)(G < QADC_NSUB ? G : QADC_NSUB);
        uint32_t last = 0;
        if (__hip_atomic_fetch_add(&hd->count[sl][1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u == in_list)
            last = __hip_atomic_fetch_add(&hd->arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u == lists;
        s_last = last;
    }
    __syncthreads();
    if (s_last == 0) return;
    typedef SelectLds<SCAN_THREADS, FUSED_CAP> Lds;
    Lds &S = *(Lds *)(smem + (((size_t)gtab_len * sizeof(QT) + 15) & ~(size_t)15));
    FinalOut o;
    o.ids = out_ids + q * R;
    o.keys = out_keys + q * R;
    o.dist = out_dist + q * R;
    select_query<KIND, QT, SCAN_THREADS, FUSED_CAP, true>(L, wq, cand_off, gtab_off, cap, codes, n, R, prm, o, S,
                                                          (const QT *)gtab, (QT *)nullptr);
}

// -------------------------------------------------------------- k_scan_mq ---
// Four queries per pass over the codes (m x 4 layouts with 8-bit tables).  The four
// queries' byte-indexed group tables are interleaved in LDS as one 8-byte entry
// {u16 q0, u16 q1, u16 q2, u16 q3}, so one ds_read_b64 serves four queries and two plain
// 32-bit adds accumulate them (eight or sixteen addends of at most 255 cannot carry out
// of a 16-bit field).  Code bytes are loaded and split into indices once for all four.
// NG = groups per code (8: 64-bit codes, 16: 128-bit codes).
#define MQ 4
#define MQ_STAGE_BYTES ((SCAN_THREADS / QADC_WAVE) * MQ * QADC_WSTAGE * 8)
template <int NG>
__global__ void __launch_bounds__(SCAN_THREADS)
k_scan_mq(const pq_qparams_t *__restrict__ qparams, int nq, const uint8_t *__restrict__ codes,
          int64_t n, char *__restrict__ ws, size_t per_query, size_t cand_off, size_t gtab_off,
          uint32_t cap, uint32_t qmax, const uint16_t *__restrict__ bound_rec, int recP, uint32_t reck) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint2 *tab = (uint2 *)smem;  // [NG][256], at LDS offset 0: entry offsets go into the reads as they are
    uint32_t *s_thr = (uint32_t *)(smem + NG * 256 * 8);  // [MQ] bounds added up from the pilot's records
    // this wave's staging buffers for candidates, one per query
    uint64_t *wbuf = (uint64_t *)(smem + NG * 256 * 8 + 16) + (threadIdx.x / QADC_WAVE) * (MQ * QADC_WSTAGE);
    uint32_t nbuf[MQ] = {0u, 0u, 0u, 0u};
    if (bound_rec) {  // wave j adds up the records of query q0 + j (SCAN_THREADS / 64 == MQ)
        const int j = threadIdx.x / QADC_WAVE;
        const size_t q = (blockIdx.y * MQ + j < nq) ? blockIdx.y * MQ + j : blockIdx.y * MQ;
        const uint32_t t = scan_bound_from_records(bound_rec + q * (QADC_REC_BINS * QADC_REC_SLOTS), recP, reck, 0, qmax);
        if (threadIdx.x % QADC_WAVE == 0) s_thr[j] = t;
    }
    const int q0 = blockIdx.y * MQ;
    const int b = blockIdx.x, G = gridDim.x;
    uint32_t thr[MQ];
    uint64_t *cand[MQ];
    uint32_t *count[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) {
        const bool have = q0 + j < nq;
        const size_t q = have ? q0 + j : q0;
        uint32_t t = qparams[q].key_bound;
        thr[j] = t >= qmax ? 0xffffffffu : t;  // sums are compared unsaturated (see k_scan)
        cand[j] = (uint64_t *)(ws + q * per_query + cand_off) + (size_t)(b % QADC_NSUB) * cap;
        count[j] = &((ScanHdr *)(ws + q * per_query))->count[b % QADC_NSUB][0];
    }
    // interleave the four prepared tables: thread handles 4 consecutive entries at a time
    for (int w = threadIdx.x; w < NG * 64; w += SCAN_THREADS) {
        uint32_t v[MQ];
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            const size_t q = (q0 + j < nq) ? q0 + j : q0;
            v[j] = ((const uint32_t *)(ws + q * per_query + gtab_off))[w];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint2 e;
            e.x = ((v[0] >> (8 * i)) & 255u) | (((v[1] >> (8 * i)) & 255u) << 16);
            e.y = ((v[2] >> (8 * i)) & 255u) | (((v[3] >> (8 * i)) & 255u) << 16);
            tab[4 * w + i] = e;
        }
    }
    __syncthreads();
    if (bound_rec) {
#pragma unroll
        for (int j = 0; j < MQ; ++j) thr[j] = s_thr[j] >= qmax ? 0xffffffffu : s_thr[j];
    }

    constexpr int CPC = NG == 8 ? 2 : 1;  // codes per 16-byte chunk
    constexpr int U = 2;                  // chunks per thread and tile
    const int64_t nfull = NG == 8 ? (n >> 1) : n;
    const int64_t ntiles = (nfull + U * SCAN_THREADS - 1) / (U * SCAN_THREADS);
    const uint4 *__restrict__ p = (const uint4 *)codes;
    const uint32_t three = 3;  // shift count of mq_byte_x8, held in a register
    for (int64_t tile = b; tile < ntiles; tile += G) {
        uint4 cur[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t c = tile * (U * SCAN_THREADS) + u * SCAN_THREADS + threadIdx.x;
            cur[u] = c < nfull ? p[c] : make_uint4(0, 0, 0, 0);
        }
        uint32_t sum[MQ][U * CPC], id[U * CPC];
        bool ok[U * CPC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t c = tile * (U * SCAN_THREADS) + u * SCAN_THREADS + threadIdx.x;
            const uint32_t w[4] = {cur[u].x, cur[u].y, cur[u].z, cur[u].w};
#pragma unroll
            for (int k = 0; k < CPC; ++k) {
                uint32_t lo = 0, hi = 0;
#pragma unroll
                for (int g = 0; g < NG; g += 4) {
                    const uint32_t word = w[(NG == 8 ? 2 * k : 0) + (g >> 2)];
                    const uint2 e0 = mq_entry<0>(g, word, three), e1 = mq_entry<1>(g + 1, word, three);
                    const uint2 e2 = mq_entry<2>(g + 2, word, three), e3 = mq_entry<3>(g + 3, word, three);
                    lo += e0.x + e1.x + e2.x + e3.x;
                    hi += e0.y + e1.y + e2.y + e3.y;
                }
                const int sidx = u * CPC + k;
                sum[0][sidx] = lo & 0xffffu;
                sum[1][sidx] = lo >> 16;
                sum[2][sidx] = hi & 0xffffu;
                sum[3][sidx] = hi >> 16;
                id[sidx] = (uint32_t)(CPC * c + k);
                ok[sidx] = c < nfull;
            }
        }
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            bool pass[U * CPC], any = false;
#pragma unroll
            for (int i = 0; i < U * CPC; ++i) {
                pass[i] = ok[i] && sum[j][i] <= thr[j] && (q0 + j < nq);
                any = any || pass[i];
            }
            if (__ballot(any) != 0) {
#pragma unroll
                for (int i = 0; i < U * CPC; ++i) sum[j][i] = sum[j][i] > qmax ? qmax : sum[j][i];
                stage_append_multi<U * CPC>(pass, sum[j], id, wbuf + j * QADC_WSTAGE, nbuf[j], cand[j], cap, count[j]);
            }
        }
    }
    if (NG == 8 && (n & 1) && b == 0 && threadIdx.x < QADC_WAVE) {  // the odd last 64-bit code
        const bool me = threadIdx.x == 0;
        uint32_t lo = 0, hi = 0;
        if (me) {
            const uint2 w = *(const uint2 *)(codes + (n - 1) * 8);
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                const uint32_t byte = ((g < 4 ? w.x : w.y) >> (8 * (g & 3))) & 255u;
                const uint2 e = tab[g * 256 + byte];
                lo += e.x;
                hi += e.y;
            }
        }
        const uint32_t sj[MQ] = {lo & 0xffffu, lo >> 16, hi & 0xffffu, hi >> 16};
#pragma unroll
        for (int j = 0; j < MQ; ++j)
            stage_append(me && (q0 + j < nq) && sj[j] <= thr[j], sj[j] > qmax ? qmax : sj[j],
                         (uint32_t)(n - 1), wbuf + j * QADC_WSTAGE, nbuf[j], cand[j], cap, count[j]);
    }
#pragma unroll
    for (int j = 0; j < MQ; ++j) stage_flush(wbuf + j * QADC_WSTAGE, nbuf[j], cand[j], cap, count[j]);
}

// ------------------------------------------------------------- k_scan_mqg ---
// The same for the irregular layouts (5-, 8- and 16-byte codes with group descriptors, 8- or
// 16-bit tables): entry e of the interleaved table holds the four queries' values of group
// table entry e as {u16 q0, u16 q1, u16 q2, u16 q3}; a code's four sums live in two packed words.
typedef unsigned short mq_u16x2 __attribute__((ext_vector_type(2)));
// a += b on both 16-bit halves, saturating at 65535 (one packed instruction)
__device__ __forceinline__ uint32_t mq_add_sat16(uint32_t a, uint32_t b) {
    const mq_u16x2 r = __builtin_elementwise_add_sat(__builtin_bit_cast(mq_u16x2, a), __builtin_bit_cast(mq_u16x2, b));
    return __builtin_bit_cast(uint32_t, r);
}

// Sums of four queries as two packed words: a = q0 | q1 << 16, b = q2 | q3 << 16.  8-bit tables:
// plain adds (at most 16 groups of at most 255 cannot carry).  16-bit tables: saturating packed
// adds, which is the saturating accumulation of Section 3.4 itself (q_max = 65535).
template <typename QT>
struct MqAcc {
    uint32_t a, b;
    __device__ __forceinline__ void zero() { a = b = 0; }
    __device__ __forceinline__ void add(const uint2 e) {
        if (sizeof(QT) == 1) {
            a += e.x;
            b += e.y;
        } else {
            a = mq_add_sat16(a, e.x);
            b = mq_add_sat16(b, e.y);
        }
    }
    __device__ __forceinline__ uint32_t sum(int j) const {
        return j == 0 ? (a & 0xffffu) : j == 1 ? (a >> 16) : j == 2 ? (b & 0xffffu) : (b >> 16);
    }
};

template <int NG, int NLO, typename QT>
__device__ __forceinline__ void mq_add_groups(const GroupDesc &d, const uint2 *tab, uint32_t lo,
                                              uint32_t hi, bool upper, MqAcc<QT> &acc) {
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const uint32_t x = NLO >= 0 ? (g < NLO ? lo : hi) : (d.off[g] >= 32 ? hi : lo);
        const int base = upper ? d.base2[g] : d.base[g];
        acc.add(tab[base + __builtin_amdgcn_ubfe(x, (uint32_t)(d.off[g] & 31), (uint32_t)d.w[g])]);
    }
}

template <int KIND, typename QT, int NG, int MODE>
__global__ void __launch_bounds__(SCAN_THREADS)
k_scan_mqg(const pq_qparams_t *__restrict__ qparams, int nq, const uint8_t *__restrict__ codes,
           int64_t n, char *__restrict__ ws, size_t per_query, size_t cand_off, size_t gtab_off,
           uint32_t cap, int gtab_len, uint32_t qmax, GroupDesc gd, const uint16_t *__restrict__ bound_rec,
           int recP, uint32_t reck) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint2 *tab = (uint2 *)smem;  // [gtab_len]
    __shared__ uint32_t s_thr[MQ];
    __shared__ uint64_t s_stage[SCAN_THREADS / QADC_WAVE][MQ][QADC_WSTAGE];  // per wave and query
    uint64_t *wbuf = &s_stage[threadIdx.x / QADC_WAVE][0][0];
    uint32_t nbuf[MQ] = {0u, 0u, 0u, 0u};
    if (bound_rec) {  // wave j adds up the records of query q0 + j (SCAN_THREADS / 64 == MQ)
        const int j = threadIdx.x / QADC_WAVE;
        const size_t q = (blockIdx.y * MQ + j < nq) ? blockIdx.y * MQ + j : blockIdx.y * MQ;
        const uint32_t t = scan_bound_from_records(bound_rec + q * (QADC_REC_BINS * QADC_REC_SLOTS), recP, reck,
                                                   sizeof(QT) == 1 ? 0 : 8, qmax);
        if (threadIdx.x % QADC_WAVE == 0) s_thr[j] = t;
    }
    constexpr int NLO = MODE == 1 ? NG / 2 : (MODE == 2 ? NG - 1 : -1);
    constexpr int NC = KIND == SCAN_W128 ? 2 : 4;  // codes per thread and tile
    const int q0 = blockIdx.y * MQ;
    const int b = blockIdx.x, G = gridDim.x;
    uint32_t thr[MQ];
    uint64_t *cand[MQ];
    uint32_t *count[MQ];
    const QT *src[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) {
        const size_t q = (q0 + j < nq) ? q0 + j : q0;
        uint32_t t = qparams[q].key_bound;
        thr[j] = t > qmax ? qmax : t;
        cand[j] = (uint64_t *)(ws + q * per_query + cand_off) + (size_t)(b % QADC_NSUB) * cap;
        count[j] = &((ScanHdr *)(ws + q * per_query))->count[b % QADC_NSUB][0];
        src[j] = (const QT *)(ws + q * per_query + gtab_off);
    }
    for (int e = threadIdx.x; e < gtab_len; e += SCAN_THREADS) {
        uint2 v;
        v.x = (uint32_t)src[0][e] | ((uint32_t)src[1][e] << 16);
        v.y = (uint32_t)src[2][e] | ((uint32_t)src[3][e] << 16);
        tab[e] = v;
    }
    __syncthreads();
    if (bound_rec) {
#pragma unroll
        for (int j = 0; j < MQ; ++j) thr[j] = s_thr[j];
    }

    // tiles of NC * SCAN_THREADS codes; thread t takes the codes NC*t .. NC*t+NC-1 of a tile
    const int ntiles = (int)((n + NC * SCAN_THREADS - 1) / (NC * SCAN_THREADS));
    for (int tile = b; tile < ntiles; tile += G) {
        const int64_t first = ((int64_t)tile * SCAN_THREADS + threadIdx.x) * NC;  // first code of this thread
        MqAcc<QT> acc[NC];
#pragma unroll
        for (int i = 0; i < NC; ++i) acc[i].zero();
        if (KIND == SCAN_W64) {
            // four 8-byte codes: two 16-byte loads (first is a multiple of 4 and the array is
            // 16-byte aligned); code by code in the ragged last tile
            uint2 cw[4];
            if (first + 3 < n) {
                const uint4 x0 = *(const uint4 *)(codes + first * 8);
                const uint4 x1 = *(const uint4 *)(codes + first * 8 + 16);
                cw[0] = make_uint2(x0.x, x0.y);
                cw[1] = make_uint2(x0.z, x0.w);
                cw[2] = make_uint2(x1.x, x1.y);
                cw[3] = make_uint2(x1.z, x1.w);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    cw[i] = first + i < n ? *(const uint2 *)(codes + (first + i) * 8) : make_uint2(0, 0);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) mq_add_groups<NG, NLO, QT>(gd, tab, cw[i].x, cw[i].y, false, acc[i]);
        } else if (KIND == SCAN_C5) {
            // five dwords: four 5-byte codes (first is a multiple of 4, so the chunk is 4-byte aligned)
            uint32_t w[5] = {0, 0, 0, 0, 0};
            if (first + 3 < n) {
                const uint32_t *p = (const uint32_t *)(codes + first * 5);
#pragma unroll
                for (int i = 0; i < 5; ++i) w[i] = p[i];
            } else {
                for (int i = 0; i < 20; ++i)
                    if (first * 5 + i < n * 5) w[i >> 2] |= (uint32_t)codes[first * 5 + i] << (8 * (i & 3));
            }
            uint32_t lo[4], hi[4];
            lo[0] = w[0];
            hi[0] = w[1] & 0xffu;
            lo[1] = __builtin_amdgcn_alignbit(w[2], w[1], 8);
            hi[1] = (w[2] >> 8) & 0xffu;
            lo[2] = __builtin_amdgcn_alignbit(w[3], w[2], 16);
            hi[2] = (w[3] >> 16) & 0xffu;
            lo[3] = __builtin_amdgcn_alignbit(w[4], w[3], 24);
            hi[3] = w[4] >> 24;
#pragma unroll
            for (int i = 0; i < 4; ++i) mq_add_groups<NG, NLO, QT>(gd, tab, lo[i], hi[i], false, acc[i]);
        } else {
            // two 16-byte codes
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int64_t c = first + i < n ? first + i : (n > 0 ? n - 1 : 0);
                const uint4 w = *(const uint4 *)(codes + c * 16);
                mq_add_groups<NG, NLO, QT>(gd, tab, w.x, w.y, false, acc[i]);
                mq_add_groups<NG, NLO, QT>(gd, tab, w.z, w.w, true, acc[i]);
            }
        }
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            bool pass[NC], any = false;
            uint32_t key[NC], id[NC];
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                const uint32_t sm = acc[i].sum(j);
                key[i] = sm > qmax ? qmax : sm;
                id[i] = (uint32_t)(first + i);
                pass[i] = first + i < n && key[i] <= thr[j] && (q0 + j < nq);
                any = any || pass[i];
            }
            if (__ballot(any) != 0)
                stage_append_multi<NC>(pass, key, id, wbuf + j * QADC_WSTAGE, nbuf[j], cand[j], cap, count[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < MQ; ++j) stage_flush(wbuf + j * QADC_WSTAGE, nbuf[j], cand[j], cap, count[j]);
}

// --------------------------------------------------------------- k_final ---
// NT threads per query; ACAP = candidates it can rank in LDS.
template <int KIND, typename QT, int NT, int ACAP>
__global__ void __launch_bounds__(NT)
k_final(const DevLayout *__restrict__ L, const pq_qparams_t *__restrict__ qparams,
        const uint8_t *__restrict__ codes, int64_t n, int R, char *__restrict__ ws, size_t per_query,
        size_t cand_off, size_t gtab_off, uint32_t cap, int32_t *__restrict__ out_ids,
        uint16_t *__restrict__ out_keys, float *__restrict__ out_dist) {
    extern __shared__ __align__(16) unsigned char smem[];
    typedef SelectLds<NT, ACAP> Lds;
    Lds &S = *(Lds *)smem;
    QT *gtab_room = (QT *)(smem + sizeof(Lds));  // only filled on the slow path
    const size_t q = blockIdx.x;
    char *wq = ws + q * per_query;
    FinalOut o;
    o.ids = out_ids + q * R;
    o.keys = out_keys + q * R;
    o.dist = out_dist + q * R;
    const pq_qparams_t prm = qparams[q];
    select_query<KIND, QT, NT, ACAP, false>(L, wq, cand_off, gtab_off, cap, codes, n, R, prm, o, S,
                                            (const QT *)nullptr, gtab_room);
}

// ------------------------------------------------------------------ host ---
// what: 4 = prepare the group tables, 1 = scan kernel, 2 = selection kernel
template <int KIND, typename QT>
static int launch_scan(const pq_index *idx, const void *qtables, const pq_qparams_t *qparams, int nq,
                       const uint8_t *codes, int64_t n, int R, int32_t *out_ids, uint16_t *out_keys,
                       float *out_dist, char *ws, const ScanPlan &p, hipStream_t s, int what,
                       const uint16_t *bound_rec, int recP, uint32_t reck) {
    const DevLayout &h = idx->h;
    const size_t gtab_bytes = ((size_t)h.gtab_len * sizeof(QT) + 15) & ~(size_t)15;
    if (what & 4) {
        hipLaunchKernelGGL((k_prepare<KIND, QT>), dim3(nq), dim3(256), gtab_bytes + (size_t)h.T * 2, s,
                           idx->dev, qtables, ws, p.per_query, p.gtab_off);
        QADC_LAUNCH_CHECK("k_prepare");
    }
    const bool no_mq = qadc_option(PQ_OPT_SHARED_PASSES) == 0;
    bool fused = false;  // the scan kernel's last block does the selection
    if ((what & 1) && sizeof(QT) == 1 && nq >= 2 && (KIND == SCAN_NIB8 || KIND == SCAN_NIB16) && !no_mq) {
        // several queries: four of them share every pass over the codes
        const int groups = (nq + MQ - 1) / MQ;
        // k_scan_mq addresses its tables from LDS address 0: it must have no static LDS
        static const int mq_static_lds = [] {
            hipFuncAttributes a8, a16;
            if (hipFuncGetAttributes(&a8, (const void *)k_scan_mq<8>) != hipSuccess ||
                hipFuncGetAttributes(&a16, (const void *)k_scan_mq<16>) != hipSuccess)
                return -1;
            return (int)(a8.sharedSizeBytes + a16.sharedSizeBytes);
        }();
        if (mq_static_lds != 0) {
            qadc_set_error("k_scan_mq: static LDS of %d bytes (its tables must start at LDS address 0)", mq_static_lds);
            return PQ_EHIP;
        }
        if (KIND == SCAN_NIB8)
            hipLaunchKernelGGL((k_scan_mq<8>), dim3(p.G, groups), dim3(SCAN_THREADS), 8 * 256 * 8 + 16 + MQ_STAGE_BYTES, s,
                               qparams, nq, codes, n, ws, p.per_query, p.cand_off, p.gtab_off,
                               p.cap, (uint32_t)h.qmax, bound_rec, recP, reck);
        else
            hipLaunchKernelGGL((k_scan_mq<16>), dim3(p.G, groups), dim3(SCAN_THREADS), 16 * 256 * 8 + 16 + MQ_STAGE_BYTES, s,
                               qparams, nq, codes, n, ws, p.per_query, p.cand_off, p.gtab_off,
                               p.cap, (uint32_t)h.qmax, bound_rec, recP, reck);
        QADC_LAUNCH_CHECK("k_scan_mq");
    } else if (what & 1) {
        GroupDesc gd;
        memset(&gd, 0, sizeof(gd));
        gd.ng = h.ng;
        for (int g = 0; g < QADC_MAXG_FAST && g < h.ng; ++g) {
            gd.off[g] = h.goff[g];
            gd.w[g] = h.gw[g];
            gd.base[g] = h.gbase[g];
        }
        if (KIND == SCAN_W128)  // NG = groups per 64-bit half
            for (int g = 0; g < h.ng / 2; ++g) gd.base2[g] = h.gbase[g + h.ng / 2];
        constexpr bool desc_kind = KIND == SCAN_W64 || KIND == SCAN_C5 || KIND == SCAN_W128;
        const bool fast = (KIND == SCAN_W64 || KIND == SCAN_C5) && h.g32ok != 0 && h.ng >= 1 &&
                          h.ng <= QADC_MAXG_FAST;
        const int ngt = KIND == SCAN_W128 ? h.ng / 2 : (fast ? h.ng : 0);
        // where the groups lie (see k_scan's MODE)
        int nlo = 0;
        const int gper = KIND == SCAN_W128 ? h.ng / 2 : h.ng;
        for (int g = 0; g < gper; ++g) nlo += h.goff[g] < 32 ? 1 : 0;
        const int mode = (ngt > 0 && ngt % 2 == 0 && nlo == ngt / 2) ? 1 : ((ngt > 1 && nlo == ngt - 1) ? 2 : 0);
        // several queries over an irregular layout: four of them share every pass over the codes
        const size_t mq_lds = (size_t)h.gtab_len * sizeof(uint2);
        const bool mqg = desc_kind && nq >= 2 && ngt > 0 && mq_lds <= 96 * 1024 && !no_mq;
        // one query (or a few) per pass, a short result list, scan and selection asked for
        // together: the block of the scan kernel that finishes last does the selection, which
        // saves a dependent launch; the selection's LDS is then part of every scan block's
        const size_t lds_fused = gtab_bytes + sizeof(SelectLds<SCAN_THREADS, FUSED_CAP>);
        fused = !mqg && (what & 2) && R <= FUSED_R && lds_fused <= 20 * 1024;
        const size_t lds_scan = fused ? lds_fused : gtab_bytes + (SCAN_THREADS / QADC_WAVE) * QADC_WSTAGE * sizeof(uint64_t);
        const int fuse = fused ? 1 : 0;
#define QADC_SCAN_GO(NGV, MODEV)                                                                     \
    hipLaunchKernelGGL((k_scan<KIND, QT, NGV, MODEV>), dim3(p.G, nq), dim3(SCAN_THREADS), lds_scan, \
                       s, idx->dev, qtables, qparams, codes, n, ws, p.per_query, p.cand_off,        \
                       p.gtab_off, p.cap, h.gtab_len, (uint32_t)h.qmax, gd, fuse, R, out_ids,       \
                       out_keys, out_dist, bound_rec, recP, reck)
#define QADC_MQG_GO(NGV, MODEV)                                                                      \
    do {                                                                                             \
        if (mq_lds > 48 * 1024)                                                                      \
            QADC_HIP_TRY(hipFuncSetAttribute((const void *)k_scan_mqg<KIND, QT, NGV, MODEV>,         \
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)mq_lds)); \
        hipLaunchKernelGGL((k_scan_mqg<KIND, QT, NGV, MODEV>), dim3(p.G, (nq + MQ - 1) / MQ),        \
                           dim3(SCAN_THREADS), mq_lds, s, qparams, nq, codes, n, ws, p.per_query,    \
                           p.cand_off, p.gtab_off, p.cap, h.gtab_len, (uint32_t)h.qmax, gd,         \
                           bound_rec, recP, reck);                                                   \
    } while (0)
#define QADC_SCAN_ANY(NGV, MODEV)                                       \
    do {                                                                \
        if (mqg) QADC_MQG_GO(NGV, MODEV); else QADC_SCAN_GO(NGV, MODEV); \
    } while (0)
#define QADC_SCAN_NG(NGV)                                              \
    do {                                                               \
        if (KIND == SCAN_C5) {                                         \
            if (mode == 2) QADC_SCAN_ANY(NGV, 2); else QADC_SCAN_ANY(NGV, 0); \
        } else {                                                       \
            if (mode == 1) QADC_SCAN_ANY(NGV, 1); else QADC_SCAN_ANY(NGV, 0); \
        }                                                              \
    } while (0)
        if constexpr (desc_kind) {
            switch (ngt) {
                case 1: QADC_SCAN_NG(1); break;
                case 2: QADC_SCAN_NG(2); break;
                case 3: QADC_SCAN_NG(3); break;
                case 4: QADC_SCAN_NG(4); break;
                case 5: QADC_SCAN_NG(5); break;
                case 6: QADC_SCAN_NG(6); break;
                case 7: QADC_SCAN_NG(7); break;
                case 8: QADC_SCAN_NG(8); break;
                default: QADC_SCAN_GO(0, 0); break;
            }
        } else {
            QADC_SCAN_GO(0, 0);
        }
#undef QADC_MQG_GO
#undef QADC_SCAN_ANY
#undef QADC_SCAN_GO
#undef QADC_SCAN_NG
        QADC_LAUNCH_CHECK("k_scan");
    }
    if (!(what & 2) || fused) return PQ_OK;
    // short result lists: a small block (cheap barriers, little LDS); long ones: 1024 threads
    if (R <= FINAL_SMALL_R) {
        const size_t lds_final = sizeof(SelectLds<256, FINAL_SMALL_CAP>) + gtab_bytes;
        if (lds_final > 48 * 1024)
            QADC_HIP_TRY(hipFuncSetAttribute((const void *)k_final<KIND, QT, 256, FINAL_SMALL_CAP>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_final));
        hipLaunchKernelGGL((k_final<KIND, QT, 256, FINAL_SMALL_CAP>), dim3(nq), dim3(256), lds_final, s,
                           idx->dev, qparams, codes, n, R, ws, p.per_query, p.cand_off, p.gtab_off, p.cap,
                           out_ids, out_keys, out_dist);
    } else {
        const size_t lds_final = sizeof(SelectLds<1024, FINAL_CAP>) + gtab_bytes;
        QADC_HIP_TRY(hipFuncSetAttribute((const void *)k_final<KIND, QT, 1024, FINAL_CAP>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_final));
        hipLaunchKernelGGL((k_final<KIND, QT, 1024, FINAL_CAP>), dim3(nq), dim3(1024), lds_final, s,
                           idx->dev, qparams, codes, n, R, ws, p.per_query, p.cand_off, p.gtab_off, p.cap,
                           out_ids, out_keys, out_dist);
    }
    QADC_LAUNCH_CHECK("k_final");
    return PQ_OK;
}

static int scan_dispatch(const pq_index *idx, const void *qtables, const pq_qparams_t *qparams,
                         int nq, const uint8_t *codes, int64_t n, int R, int32_t *out_ids,
                         uint16_t *out_keys, float *out_dist, char *ws, const ScanPlan &p,
                         hipStream_t s, int what, const uint16_t *bound_rec = nullptr, int recP = 0,
                         uint32_t reck = 0) {
    const bool u8 = idx->h.acc_bits == 8;
#define QADC_GO(KIND, QT) \
    return launch_scan<KIND, QT>(idx, qtables, qparams, nq, codes, n, R, out_ids, out_keys, out_dist, ws, p, s, what, \
                                 bound_rec, recP, reck)
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

static int check_scan_args(const char *who, const pq_index_t *idx, int nq, int64_t n, int R) {
    if (!idx || nq < 0 || n < 0 || n >= ((int64_t)1 << 31)) {
        qadc_set_error("%s: bad handle, nq or n (need 0 <= n < 2^31)", who);
        return PQ_EINVAL;
    }
    if (R < 1 || R > PQ_MAX_R) {
        qadc_set_error("%s: need 1<=R<=%d (got %d)", who, PQ_MAX_R, R);
        return PQ_EINVAL;
    }
    if (nq > 65535) {
        qadc_set_error("%s: at most 65535 queries per call (got %d)", who, nq);
        return PQ_EINVAL;
    }
    return PQ_OK;
}

static int scan_entry(const char *who, int what, const pq_index_t *idx, const void *qtables,
                      const pq_qparams_t *qparams, int nq, const uint8_t *codes, int64_t n, int R,
                      int32_t *out_ids, uint16_t *out_keys, float *out_dist, void *workspace,
                      size_t workspace_bytes, void *stream) {
    int rc = check_scan_args(who, idx, nq, n, R);
    if (rc != PQ_OK) return rc;
    if (nq == 0) return PQ_OK;
    if (!qtables || !qparams || !workspace || (n > 0 && !codes) ||
        ((what & 2) && (!out_ids || !out_keys || !out_dist))) {
        qadc_set_error("%s: null pointer", who);
        return PQ_EINVAL;
    }
    if (((uintptr_t)codes & 15u) != 0 || ((uintptr_t)workspace & 255u) != 0) {
        qadc_set_error("%s: codes must be 16-byte and workspace 256-byte aligned", who);
        return PQ_EINVAL;
    }
    const ScanPlan p = qadc_scan_plan(idx, nq, n, R);
    if (workspace_bytes < p.total) {
        qadc_set_error("%s: workspace of %zu bytes, need %zu", who, workspace_bytes, p.total);
        return PQ_ENOMEM;
    }
    return scan_dispatch(idx, qtables, qparams, nq, codes, n, R, out_ids, out_keys, out_dist,
                         (char *)workspace, p, (hipStream_t)stream, what);
}

extern "C" int pq_adc_scan_topk(const pq_index_t *idx, const void *qtables,
                                const pq_qparams_t *qparams, int nq, const uint8_t *codes,
                                int64_t n, int R, int32_t *out_ids, uint16_t *out_keys,
                                float *out_dist, void *workspace, size_t workspace_bytes,
                                void *stream) {
    return scan_entry("pq_adc_scan_topk", 7, idx, qtables, qparams, nq, codes, n, R, out_ids,
                      out_keys, out_dist, workspace, workspace_bytes, stream);
}

extern "C" int pq_adc_scan_candidates(const pq_index_t *idx, const void *qtables,
                                      const pq_qparams_t *qparams, int nq, const uint8_t *codes,
                                      int64_t n, int R, void *workspace, size_t workspace_bytes,
                                      void *stream) {
    return scan_entry("pq_adc_scan_candidates", 5, idx, qtables, qparams, nq, codes, n, R, nullptr,
                      nullptr, nullptr, workspace, workspace_bytes, stream);
}

extern "C" int pq_adc_rescan_candidates(const pq_index_t *idx, const void *qtables,
                                        const pq_qparams_t *qparams, int nq, const uint8_t *codes,
                                        int64_t n, int R, void *workspace, size_t workspace_bytes,
                                        void *stream) {
    return scan_entry("pq_adc_rescan_candidates", 1, idx, qtables, qparams, nq, codes, n, R, nullptr,
                      nullptr, nullptr, workspace, workspace_bytes, stream);
}

extern "C" int pq_select_topk(const pq_index_t *idx, const void *qtables,
                              const pq_qparams_t *qparams, int nq, const uint8_t *codes, int64_t n,
                              int R, int32_t *out_ids, uint16_t *out_keys, float *out_dist,
                              void *workspace, size_t workspace_bytes, void *stream) {
    return scan_entry("pq_select_topk", 2, idx, qtables, qparams, nq, codes, n, R, out_ids, out_keys,
                      out_dist, workspace, workspace_bytes, stream);
}

// ------------------------------------------- entry point that allocates nothing ---
// pq_adc_scan_topk with the workspace in a device array of this library instead of caller
// memory.  Every GPU holds its own copy of the array at its own address: the address is asked
// for once per device (with that device current) and kept; host code only ever uses that
// address, never the array's name.
static __device__ __align__(256) unsigned char scratch[PQ_STATIC_SCRATCH_BYTES];

#define QADC_MAX_DEVICES 64
static void *g_scratch_ptr[QADC_MAX_DEVICES];  // per device; null until first use there
static std::mutex g_scratch_mutex;

static int static_scratch(void **out) {
    int dev = -1;
    QADC_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= QADC_MAX_DEVICES) {
        qadc_set_error("pq_adc_scan_topk_static: device %d out of range (0..%d)", dev, QADC_MAX_DEVICES - 1);
        return PQ_EINVAL;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        QADC_HIP_TRY(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) {
            qadc_set_error("pq_adc_scan_topk_static: no address for the scratch array on device %d", dev);
            return PQ_EHIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PQ_OK;
}

extern "C" int pq_adc_scan_topk_static(const pq_index_t *idx, const void *qtables,
                                       const pq_qparams_t *qparams, int nq, const uint8_t *codes,
                                       int64_t n, int R, int32_t *out_ids, uint16_t *out_keys,
                                       float *out_dist, void *stream) {
    int rc = check_scan_args("pq_adc_scan_topk_static", idx, nq, n, R);
    if (rc != PQ_OK) return rc;
    if (nq == 0) return PQ_OK;
    const size_t need = qadc_scan_plan(idx, nq, n, R).total;
    if (need > (size_t)PQ_STATIC_SCRATCH_BYTES) {
        qadc_set_error("pq_adc_scan_topk_static: nq=%d n=%lld R=%d need %zu bytes of scratch, the "
                       "library's array holds %zu; use pq_adc_scan_topk with a workspace",
                       nq, (long long)n, R, need, (size_t)PQ_STATIC_SCRATCH_BYTES);
        return PQ_ENOMEM;
    }
    void *ptr = nullptr;
    if ((rc = static_scratch(&ptr)) != PQ_OK) return rc;
    // (the scan's workspace needs no initial contents: every word read was written by this call)
    return scan_entry("pq_adc_scan_topk_static", 7, idx, qtables, qparams, nq, codes, n, R, out_ids,
                      out_keys, out_dist, ptr, (size_t)PQ_STATIC_SCRATCH_BYTES, stream);
}

// ------------------------------------------------------- fused search call ---
static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

extern "C" size_t pq_search_workspace_bytes(const pq_index_t *idx, int nq, int64_t n, int R) {
    if (!idx || nq < 0 || n < 0 || R < 1) return 0;
    const size_t esz = idx->h.acc_bits == 8 ? 1 : 2;
    return up256((size_t)nq * sizeof(pq_qparams_t)) + up256((size_t)nq * idx->h.T * esz) +
           up256(pq_workspace_bytes(idx, nq, n, R)) + qadc_pilot_scratch_bytes(nq);
}

extern "C" int pq_search_topk(const pq_index_t *idx, const float *queries, int nq,
                              const uint8_t *codes, int64_t n, int t, int R, int32_t *out_ids,
                              uint16_t *out_keys, float *out_dist, void *workspace,
                              size_t workspace_bytes, void *stream) {
    int rc = check_scan_args("pq_search_topk", idx, nq, n, R);
    if (rc != PQ_OK) return rc;
    const int64_t want = t > 4 * (int64_t)R ? t : 4 * (int64_t)R;
    if (t < 1 || want > PQ_MAX_T_EFF) {
        qadc_set_error("pq_search_topk: need t>=1 and max(t,4R)<=%d (got t=%d R=%d)", PQ_MAX_T_EFF, t, R);
        return PQ_EINVAL;
    }
    if (nq == 0) return PQ_OK;
    if (!queries || !out_ids || !out_keys || !out_dist || !workspace || (n > 0 && !codes)) {
        qadc_set_error("pq_search_topk: null pointer");
        return PQ_EINVAL;
    }
    if (((uintptr_t)codes & 15u) != 0 || ((uintptr_t)workspace & 255u) != 0) {
        qadc_set_error("pq_search_topk: codes must be 16-byte and workspace 256-byte aligned");
        return PQ_EINVAL;
    }
    const size_t need = pq_search_workspace_bytes(idx, nq, n, R);
    if (workspace_bytes < need) {
        qadc_set_error("pq_search_topk: workspace of %zu bytes, need %zu", workspace_bytes, need);
        return PQ_ENOMEM;
    }
    const size_t esz = idx->h.acc_bits == 8 ? 1 : 2;
    char *w = (char *)workspace;
    pq_qparams_t *qparams = (pq_qparams_t *)w;
    void *qtables = w + up256((size_t)nq * sizeof(pq_qparams_t));
    char *ws = (char *)qtables + up256((size_t)nq * idx->h.T * esz);
    hipStream_t s = (hipStream_t)stream;
    const ScanPlan p = qadc_scan_plan(idx, nq, n, R);
    char *scratch = ws + up256(p.total);
    PilotPlan pp;
    rc = qadc_quantize_launch(idx, queries, nullptr, nullptr, nq, codes, n, t, R, qtables, qparams,
                              ws + p.gtab_off, p.per_query, ws, scratch, &pp, s);
    if (rc != PQ_OK) return rc;
    // several pilot blocks per query: the scan adds their records up; one: the bound is in qparams
    const uint16_t *rec = pp.P > 1 ? (const uint16_t *)scratch : nullptr;
    const uint32_t reck = (uint32_t)(R < pp.pilot ? R : pp.pilot);
    return scan_dispatch(idx, qtables, qparams, nq, codes, n, R, out_ids, out_keys, out_dist, ws, p, s, 3, rec,
                         pp.P, reck);
}
