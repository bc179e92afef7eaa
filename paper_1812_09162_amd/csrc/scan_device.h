// Device code shared by the exhaustive and the inverted-list scan kernels.
#pragma once
#include <math.h>

#include "qadc_device.h"

#define FINAL_CAP 5120  // candidates a final kernel can rank in LDS

// ------------------------------------------------------------ group tables --
// gtab[gbase[g] + e] = min(q_max, sum of the quantized entries of the
// sub-quantizers of group g selected by the bits of e).  `qs` is the quantized
// table of one query as 16-bit words in LDS.  Ends with a block barrier.
template <int KIND, typename QT>
__device__ inline void build_gtab(const DevLayout *L, const uint16_t *qs, QT *gtab) {
    const uint32_t qmax = (uint32_t)L->qmax;
    if (KIND == SCAN_NIB8 || KIND == SCAN_NIB16) {
        // group g = code byte g = sub-quantizers 2g (low nibble) and 2g+1 (high nibble);
        // four consecutive entries share the high nibble
        const int nquads = (KIND == SCAN_NIB8 ? 8 : 16) * 64;
        for (int w = threadIdx.x; w < nquads; w += blockDim.x) {
            const int g = w >> 6, e0 = (w & 63) << 2;
            const uint16_t *lo = qs + 32 * g + (e0 & 15);
            const uint32_t hv = qs[32 * g + 16 + (e0 >> 4)];
            uint32_t v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t x = (uint32_t)lo[i] + hv;
                v[i] = x > qmax ? qmax : x;
            }
            if (sizeof(QT) == 1) {
                ((uint32_t *)gtab)[w] = v[0] | (v[1] << 8) | (v[2] << 16) | (v[3] << 24);
            } else {
                ((uint32_t *)gtab)[2 * w] = v[0] | (v[1] << 16);
                ((uint32_t *)gtab)[2 * w + 1] = v[2] | (v[3] << 16);
            }
        }
    } else {
        const int ng = L->ng;
        for (int g = 0; g < ng; ++g) {
            const int entries = 1 << L->gw[g];
            const int first = L->gfirst[g], cnt = L->gcount[g];
            const int base = L->gbase[g];
            if (cnt <= 3) {
                // descriptors of the (at most three) sub-quantizers of the group in registers
                const int b0 = L->nbits[first], t0 = L->toff[first];
                const int b1 = cnt > 1 ? L->nbits[first + 1] : 0, t1 = cnt > 1 ? L->toff[first + 1] : 0;
                const int b2 = cnt > 2 ? L->nbits[first + 2] : 0, t2 = cnt > 2 ? L->toff[first + 2] : 0;
                for (int e = threadIdx.x; e < entries; e += blockDim.x) {
                    uint32_t s = qs[t0 + (e & ((1 << b0) - 1))];
                    if (cnt > 1) s += qs[t1 + ((e >> b0) & ((1 << b1) - 1))];
                    if (cnt > 2) s += qs[t2 + ((e >> (b0 + b1)) & ((1 << b2) - 1))];
                    gtab[base + e] = (QT)(s > qmax ? qmax : s);
                }
            } else {
                for (int e = threadIdx.x; e < entries; e += blockDim.x) {
                    uint32_t rem = (uint32_t)e, s = 0;
                    for (int c = 0; c < cnt; ++c) {
                        const int j = first + c, bb = L->nbits[j];
                        s += qs[L->toff[j] + (rem & ((1u << bb) - 1u))];
                        rem >>= bb;
                    }
                    gtab[base + e] = (QT)(s > qmax ? qmax : s);
                }
            }
        }
    }
    __syncthreads();
}

// Copy one query's quantized table from global memory into LDS as 16-bit words.
// Ends with a block barrier.
template <typename QT>
__device__ inline void stage_qtable(const QT *__restrict__ qtab, int T, uint16_t *qs) {
    for (int e = threadIdx.x; e < T; e += blockDim.x) qs[e] = (uint16_t)qtab[e];
    __syncthreads();
}

// eight byte-indexed lookups for the two words of a 64-bit m x 4 code slice
template <typename QT>
__device__ __forceinline__ uint32_t sum8(const QT *t, uint32_t lo, uint32_t hi) {
    return (uint32_t)t[lo & 255u] + (uint32_t)t[256 + ((lo >> 8) & 255u)] +
           (uint32_t)t[512 + ((lo >> 16) & 255u)] + (uint32_t)t[768 + (lo >> 24)] +
           (uint32_t)t[1024 + (hi & 255u)] + (uint32_t)t[1280 + ((hi >> 8) & 255u)] +
           (uint32_t)t[1536 + ((hi >> 16) & 255u)] + (uint32_t)t[1792 + (hi >> 24)];
}

template <typename QT>
__device__ __forceinline__ uint32_t key_generic(const DevLayout *L, const QT *gtab,
                                                const uint8_t *code) {
    const int ng = L->ng, cs = L->cs;
    uint32_t s = 0;
    for (int g = 0; g < ng; ++g)
        s += gtab[L->gbase[g] + qadc_extract_group(code, cs, L->goff[g], L->gw[g])];
    const uint32_t qmax = (uint32_t)L->qmax;
    return s > qmax ? qmax : s;
}

// sum of the group entries selected by the fields of a code held in one 64-bit word
template <typename QT>
__device__ __forceinline__ uint32_t sum_groups64(const DevLayout *L, const QT *gtab, uint64_t v) {
    const int ng = L->ng;
    uint32_t s = 0;
    for (int g = 0; g < ng; ++g)
        s += gtab[L->gbase[g] + ((uint32_t)(v >> L->goff[g]) & ((1u << L->gw[g]) - 1u))];
    return s;
}

// the same for a code of at most 64 bits given as two dwords, when no group field crosses
// the dword boundary (DevLayout::g32ok): one select and one bit-field extract per group
template <typename QT>
__device__ __forceinline__ uint32_t sum_groups32(const DevLayout *L, const QT *gtab, uint32_t lo,
                                                 uint32_t hi) {
    const int ng = L->ng;
    uint32_t s = 0;
    for (int g = 0; g < ng; ++g) {
        const int off = L->goff[g];
        const uint32_t x = off >= 32 ? hi : lo;
        s += gtab[L->gbase[g] + __builtin_amdgcn_ubfe(x, (uint32_t)(off & 31), (uint32_t)L->gw[g])];
    }
    return s;
}

// Group descriptors of a layout with at most eight groups, read once into (scalar)
// registers so that the scan loop does no descriptor loads.
#define QADC_MAXG_FAST 8
struct GroupDesc {
    int ng;
    int off[QADC_MAXG_FAST], w[QADC_MAXG_FAST], base[QADC_MAXG_FAST];
};
__device__ __forceinline__ GroupDesc load_group_desc(const DevLayout *L) {
    GroupDesc d;
    d.ng = L->ng;
#pragma unroll
    for (int g = 0; g < QADC_MAXG_FAST; ++g) {
        d.off[g] = L->goff[g];
        d.w[g] = L->gw[g];
        d.base[g] = L->gbase[g];
    }
    return d;
}
// code of at most 64 bits as two dwords, no group crossing the dword boundary
template <typename QT>
__device__ __forceinline__ uint32_t sum_groups_desc(const GroupDesc &d, const QT *gtab, uint32_t lo,
                                                    uint32_t hi) {
    uint32_t s = 0;
#pragma unroll
    for (int g = 0; g < QADC_MAXG_FAST; ++g) {
        if (g < d.ng) {
            const uint32_t x = d.off[g] >= 32 ? hi : lo;
            s += gtab[d.base[g] + __builtin_amdgcn_ubfe(x, (uint32_t)(d.off[g] & 31), (uint32_t)d.w[g])];
        }
    }
    return s;
}

// key of the code at position id (simple per-code loads; used off the hot loop)
template <int KIND, typename QT>
__device__ __forceinline__ uint32_t key_at(const DevLayout *L, const QT *gtab,
                                           const uint8_t *__restrict__ codes, int64_t id) {
    const uint32_t qmax = (uint32_t)L->qmax;
    if (KIND == SCAN_NIB8) {
        uint2 w = *(const uint2 *)(codes + id * 8);
        uint32_t s = sum8(gtab, w.x, w.y);
        return s > qmax ? qmax : s;
    } else if (KIND == SCAN_NIB16) {
        uint4 w = *(const uint4 *)(codes + id * 16);
        uint32_t s = sum8(gtab, w.x, w.y) + sum8(gtab + 2048, w.z, w.w);
        return s > qmax ? qmax : s;
    } else if (KIND == SCAN_W64) {
        uint2 w = *(const uint2 *)(codes + id * 8);
        uint32_t s = sum_groups64(L, gtab, ((uint64_t)w.y << 32) | w.x);
        return s > qmax ? qmax : s;
    } else if (KIND == SCAN_C5) {
        const uint8_t *c = codes + id * 5;
        const uint64_t v = (uint64_t)c[0] | ((uint64_t)c[1] << 8) | ((uint64_t)c[2] << 16) |
                           ((uint64_t)c[3] << 24) | ((uint64_t)c[4] << 32);
        uint32_t s = sum_groups64(L, gtab, v);
        return s > qmax ? qmax : s;
    } else {
        return key_generic(L, gtab, codes + id * L->cs);
    }
}

// Keys of U codes at positions base + u*stride (u < U) with all loads issued
// before any lookup; positions >= n are clamped for the load and yield
// 0xffffffff.  n must be >= 1.
template <int KIND, typename QT, int U>
__device__ __forceinline__ void keys_batch(const DevLayout *L, const QT *gtab,
                                           const uint8_t *__restrict__ codes, int64_t base,
                                           int64_t stride, int64_t n, uint32_t *key) {
    const uint32_t qmax = (uint32_t)L->qmax;
    if (KIND == SCAN_NIB8) {
        uint2 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t id = base + u * stride;
            id = id < n ? id : n - 1;
            w[u] = *(const uint2 *)(codes + id * 8);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t s = sum8(gtab, w[u].x, w[u].y);
            key[u] = (base + u * stride < n) ? (s > qmax ? qmax : s) : 0xffffffffu;
        }
    } else if (KIND == SCAN_NIB16) {
        uint4 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t id = base + u * stride;
            id = id < n ? id : n - 1;
            w[u] = *(const uint4 *)(codes + id * 16);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t s = sum8(gtab, w[u].x, w[u].y) + sum8(gtab + 2048, w[u].z, w[u].w);
            key[u] = (base + u * stride < n) ? (s > qmax ? qmax : s) : 0xffffffffu;
        }
    } else if (KIND == SCAN_W64) {
        uint2 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t id = base + u * stride;
            id = id < n ? id : n - 1;
            w[u] = *(const uint2 *)(codes + id * 8);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t s = sum_groups64(L, gtab, ((uint64_t)w[u].y << 32) | w[u].x);
            key[u] = (base + u * stride < n) ? (s > qmax ? qmax : s) : 0xffffffffu;
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t id = base + u * stride;
            key[u] = id < n ? key_at<KIND, QT>(L, gtab, codes, id) : 0xffffffffu;
        }
    }
}

// -------------------------------------------------------------- threshold --
// Smallest bin x with hist[0..x] summing to >= R, or 0xffffffff.  One wave.
__device__ inline uint32_t wave_bound_from_hist(const uint32_t *hist, uint32_t R) {
    const int lane = __lane_id();
    uint32_t h[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        h[i] = __hip_atomic_load(&hist[4 * lane + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t s = h[0] + h[1] + h[2] + h[3];
    uint32_t run = qadc_wave_incl_scan(s) - s;
    uint32_t mine = 0xffffffffu;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        run += h[i];
        if (run >= R && mine == 0xffffffffu) mine = (uint32_t)(4 * lane + i);
    }
    return qadc_wave_min(mine);
}

struct SlotRef {
    uint64_t *slot;
    uint32_t cap;
    uint32_t *lds_count;
    ScanState *st;
};

// Append the lanes with `pass` set.  Wave-uniform call.
__device__ __forceinline__ void wave_append(bool pass, uint32_t key, uint32_t id, uint32_t bin,
                                            const SlotRef &r) {
    const uint64_t mask = __ballot(pass);
    if (mask == 0) return;
    const int lane = __lane_id();
    const int leader = __ffsll((unsigned long long)mask) - 1;
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(r.lds_count, (uint32_t)__popcll(mask));
    base = __shfl(base, leader, QADC_WAVE);
    if (pass) {
        uint32_t pos = base + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
        if (pos < r.cap) {
            r.slot[pos] = ((uint64_t)key << 32) | (uint64_t)id;
            atomicAdd(&r.st->hist[bin], 1u);
        } else {
            r.st->overflow = 1u;
        }
    }
}

