// Device code shared by the exhaustive and the inverted-list scan kernels.
#pragma once
#include <math.h>

#include "qadc_device.h"

#define FINAL_CAP 5120        // candidates a selection block of 1024 threads can rank in LDS
#define FINAL_SMALL_CAP 2048  // ... a block of 256 threads, used for result lists up to FINAL_SMALL_R
#define FINAL_SMALL_R 256
#define FUSED_CAP 1024        // ... the last block of the scan kernel itself, for result lists up to FUSED_R
#define FUSED_R 128

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
    int base2[QADC_MAXG_FAST];  // 128-bit codes: table bases of the same groups in the upper half
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
// the same with the number of groups (at most QADC_MAXG_FAST) known only at run time
template <typename QT>
__device__ __forceinline__ uint32_t sum_groups_rt(const GroupDesc &d, const QT *gtab, uint32_t lo,
                                                  uint32_t hi) {
    uint32_t s = 0;
#pragma unroll
    for (int g = 0; g < QADC_MAXG_FAST; ++g)
        if (g < d.ng) {
            const uint32_t x = d.off[g] >= 32 ? hi : lo;
            s += gtab[d.base[g] + __builtin_amdgcn_ubfe(x, (uint32_t)(d.off[g] & 31), (uint32_t)d.w[g])];
        }
    return s;
}
// code of at most 64 bits as two dwords, no group crossing the dword boundary; NG = number
// of groups, fixed at compile time so that all lookups of a code are issued together
// NLO >= 0: the first NLO groups lie in the low dword and the rest in the high one, known at
// compile time; NLO < 0: decided per group from its offset.
template <int NG, int NLO, typename QT>
__device__ __forceinline__ uint32_t sum_groups_desc(const GroupDesc &d, const QT *gtab, uint32_t lo,
                                                    uint32_t hi, bool upper = false) {
    uint32_t s = 0;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const uint32_t x = NLO >= 0 ? (g < NLO ? lo : hi) : (d.off[g] >= 32 ? hi : lo);
        const int base = upper ? d.base2[g] : d.base[g];
        s += gtab[base + __builtin_amdgcn_ubfe(x, (uint32_t)(d.off[g] & 31), (uint32_t)d.w[g])];
    }
    return s;
}

// 128-bit code as two 64-bit words, no group crossing the word boundary (descriptors from the layout)
template <typename QT>
__device__ __forceinline__ uint32_t sum_groups128(const DevLayout *L, const QT *gtab, uint64_t lo,
                                                  uint64_t hi) {
    const int ng = L->ng;
    uint32_t s = 0;
    for (int g = 0; g < ng; ++g) {
        const int off = L->goff[g];
        const uint64_t v = off >= 64 ? hi : lo;
        s += gtab[L->gbase[g] + ((uint32_t)(v >> (off & 63)) & ((1u << L->gw[g]) - 1u))];
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
    } else if (KIND == SCAN_W128) {
        uint4 w = *(const uint4 *)(codes + id * 16);
        uint32_t s = sum_groups128(L, gtab, ((uint64_t)w.y << 32) | w.x, ((uint64_t)w.w << 32) | w.z);
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
    } else if (KIND == SCAN_W128) {
        uint4 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t id = base + u * stride;
            id = id < n ? id : n - 1;
            w[u] = *(const uint4 *)(codes + id * 16);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t s = sum_groups128(L, gtab, ((uint64_t)w[u].y << 32) | w[u].x,
                                             ((uint64_t)w[u].w << 32) | w[u].z);
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

// ------------------------------------- interleaved tables of four queries ---
// Byte N of w, times 8 (the byte offset of an 8-byte table entry), as one instruction: a shift
// whose operand is selected by sub-dword addressing.
template <int N>
__device__ __forceinline__ uint32_t mq_byte_x8(uint32_t w, uint32_t three) {
    uint32_t r;
    if (N == 0)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "v"(three), "v"(w));
    else if (N == 1)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(three), "v"(w));
    else if (N == 2)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "v"(three), "v"(w));
    else
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "v"(three), "v"(w));
    return r;
}
// Entry `byte N of w` of group g of the interleaved tables, which start at LDS address 0 (the
// kernel has no other LDS but what follows them): the read takes the shifted byte as its
// address and g * 2048 as its immediate offset.
typedef const unsigned long long __attribute__((address_space(3))) mq_lds_entry;
template <int N>
__device__ __forceinline__ uint2 mq_entry(int g, uint32_t w, uint32_t three) {
    const unsigned long long e = *(mq_lds_entry *)(g * 2048u + mq_byte_x8<N>(w, three));
    return make_uint2((uint32_t)e, (uint32_t)(e >> 32));
}

// ------------------------------------------------------------ slot lists ---
#define MAX_G 4096                 // slot lists per query a final kernel can gather
#define FINAL_LPT (MAX_G / 1024)   // slot lists per thread of a 1024-thread final kernel
#define FINAL_REG 16               // candidates per thread kept in registers

// Append the lanes with `pass` set to the block's slot list.  Wave-uniform call.
__device__ __forceinline__ void slot_append(bool pass, uint32_t key, uint32_t id, uint64_t *slot,
                                            uint32_t cap, uint32_t *lds_count) {
    const uint64_t mask = __ballot(pass);
    if (mask == 0) return;
    const int lane = __lane_id();
    const int leader = __ffsll((unsigned long long)mask) - 1;
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(lds_count, (uint32_t)__popcll(mask));
    base = __shfl(base, leader, QADC_WAVE);
    if (pass) {
        const uint32_t pos = base + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
        if (pos < cap) slot[pos] = ((uint64_t)key << 32) | (uint64_t)id;
    }
}

// Append the (lane, slot) pairs with pass[u] set, NS slots per lane, to the block's list:
// one LDS atomic per call, positions from ballots and lane-mask popcounts.  Wave-uniform
// call.  The order within the list does not matter.
template <int NS>
__device__ __forceinline__ void slot_append_multi(const bool *pass, const uint32_t *key,
                                                  const uint32_t *id, uint64_t *slot, uint32_t cap,
                                                  uint32_t *lds_count) {
    uint64_t m[NS];
    uint32_t total = 0;
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        m[u] = __ballot(pass[u]);
        total += (uint32_t)__popcll(m[u]);
    }
    if (total == 0) return;
    const int lane = __lane_id();
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(lds_count, total);
    base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        const uint32_t pos = base + (uint32_t)__popcll(m[u] & ((1ull << lane) - 1ull));
        if (pass[u] && pos < cap) slot[pos] = ((uint64_t)key[u] << 32) | (uint64_t)id[u];
        base += (uint32_t)__popcll(m[u]);
    }
}


// ------------------------------------------------------- candidate lists ---
// The exhaustive scan keeps QADC_NSUB candidate lists per query in the workspace, each with its
// own counter on a cache line of its own: entries `key << 32 | id`, appended by whichever wave
// finds candidates (a block appends to list blockIdx.x % QADC_NSUB), in no particular order
// (the result is defined as a sort).  A wave reserves room with one atomic add for all the
// candidates its lanes hold.  (One list per query would be simpler, but atomic adds to one
// address are served one by one, about 10 ns each: 3000 of them per query took longer than
// the scan itself.)  Entries beyond a list's capacity are not stored, and a count above the
// capacity tells the selection that it must work from the codes themselves.
#define QADC_NSUB 64
struct ScanHdr {                      // first bytes of a query's workspace
    uint32_t arrive;                  // lists whose blocks have all finished (fused selection only)
    uint32_t pad[31];
    uint32_t count[QADC_NSUB][32];    // count[l][0] = candidates appended to list l (may exceed the capacity)
                                      // count[l][1] = blocks of list l that have finished (fused selection only)
};

// Zero a query's header: an empty set of candidate lists.  Block-wide, any block size.
__device__ __forceinline__ void scan_hdr_clear(ScanHdr *h) {
    for (int l = threadIdx.x; l < QADC_NSUB; l += blockDim.x) {
        h->count[l][0] = 0;
        h->count[l][1] = 0;
    }
    if (threadIdx.x == 0) h->arrive = 0;
}

// Append the (lane, slot) pairs with pass[u] set, NS slots per lane.  Wave-uniform call.
template <int NS>
__device__ __forceinline__ void cand_append_multi(const bool *pass, const uint32_t *key,
                                                  const uint32_t *id, uint64_t *cand, uint32_t cap,
                                                  uint32_t *count) {
    uint64_t m[NS];
    uint32_t total = 0;
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        m[u] = __ballot(pass[u]);
        total += (uint32_t)__popcll(m[u]);
    }
    if (total == 0) return;
    const int lane = __lane_id();
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(count, total);
    base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        const uint32_t pos = base + (uint32_t)__popcll(m[u] & ((1ull << lane) - 1ull));
        // (a device-scope store: written through to where every compute unit of the chip reads
        // it, so that the block which finishes last can pick it up within this same kernel)
        if (pass[u] && pos < cap)
            __hip_atomic_store((unsigned long long *)cand + pos, ((unsigned long long)key[u] << 32) | id[u],
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        base += (uint32_t)__popcll(m[u]);
    }
}
__device__ __forceinline__ void cand_append(bool pass, uint32_t key, uint32_t id, uint64_t *cand,
                                            uint32_t cap, uint32_t *count) {
    cand_append_multi<1>(&pass, &key, &id, cand, cap, count);
}

// Candidates on their way to the lists are staged per wave in LDS (QADC_WSTAGE entries), so that
// the streaming loop issues no global atomic: a wave adds what it holds to its list when its
// buffer would overflow and when it is done.  `nbuf` (entries staged) is wave-uniform.
#define QADC_WSTAGE 32
__device__ __forceinline__ void stage_flush(uint64_t *wbuf, uint32_t &nbuf, uint64_t *cand, uint32_t cap,
                                            uint32_t *count) {
    if (nbuf == 0) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // the lanes' LDS writes before other lanes' reads
    const uint32_t lane = __lane_id();
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(count, nbuf);
    base = __builtin_amdgcn_readfirstlane(base);
    if (lane < nbuf && base + lane < cap)
        __hip_atomic_store((unsigned long long *)cand + base + lane, (unsigned long long)wbuf[lane],
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // ... and the reads before the buffer is reused
    nbuf = 0;
}
template <int NS>
__device__ __forceinline__ void stage_append_multi(const bool *pass, const uint32_t *key, const uint32_t *id,
                                                   uint64_t *wbuf, uint32_t &nbuf, uint64_t *cand,
                                                   uint32_t cap, uint32_t *count) {
    uint64_t m[NS];
    uint32_t total = 0;
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        m[u] = __ballot(pass[u]);
        total += (uint32_t)__popcll(m[u]);
    }
    if (total == 0) return;
    if (nbuf + total > QADC_WSTAGE) stage_flush(wbuf, nbuf, cand, cap, count);
    if (total > QADC_WSTAGE) {  // more than the buffer holds (a crowd of ties): straight to the list
        cand_append_multi<NS>(pass, key, id, cand, cap, count);
        return;
    }
    const int lane = __lane_id();
    uint32_t base = nbuf;
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        if (pass[u])
            wbuf[base + (uint32_t)__popcll(m[u] & ((1ull << lane) - 1ull))] = ((uint64_t)key[u] << 32) | (uint64_t)id[u];
        base += (uint32_t)__popcll(m[u]);
    }
    nbuf = base;
}
__device__ __forceinline__ void stage_append(bool pass, uint32_t key, uint32_t id, uint64_t *wbuf, uint32_t &nbuf,
                                             uint64_t *cand, uint32_t cap, uint32_t *count) {
    stage_append_multi<1>(&pass, &key, &id, wbuf, nbuf, cand, cap, count);
}

// ------------------------------------------------- pruning bound from records ---
// The quantizer's pilot may be counted by several blocks that never meet: block p of query q
// leaves, for each of QADC_REC_BINS coarse key bins t (a coarse bin = four bins of the 256-bin
// key histogram, i.e. keys >> shift >> 2), how many of its pilot codes have a key in bin t or
// below: rec[q][t][p], 16-bit, saturating.  The sum over p is the number of pilot codes up to
// bin t; the first bin where it reaches k (the k-th smallest pilot key lies in it) gives an
// upper bound on the k-th smallest key of the whole list: the bin's largest key.
#define QADC_REC_BINS 64
#define QADC_REC_SLOTS 128
// Sum of the first P 16-bit slots of a record row, chunks [c0, c1) of 8 slots (16 bytes) each.
__device__ __forceinline__ uint32_t scan_rec_row_sum(const uint16_t *__restrict__ row, int P, int c0, int c1) {
    uint32_t s = 0;
    for (int c = c0; c < c1; c += 4) {  // four 16-byte loads in flight at a time
        uint4 v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            v[i] = (c + i < c1 && (c + i) * 8 < P) ? ((const uint4 *)row)[c + i] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                if ((c + i) * 8 + 2 * h < P) s += w[h] & 0xffffu;
                if ((c + i) * 8 + 2 * h + 1 < P) s += w[h] >> 16;
            }
        }
    }
    return s;
}
__device__ __forceinline__ uint32_t scan_bound_of_bin(uint32_t bin, int shift, uint32_t qmax) {
    if (bin >= QADC_REC_BINS) return qmax;  // (fewer than k pilot codes in all: no bound)
    const uint32_t bound = (((bin << 2) | 3u) << shift) | ((1u << shift) - 1u);
    return bound > qmax ? qmax : bound;
}
// Called by one full wave (lane t adds up bin t); returns the bound to every lane.
__device__ __forceinline__ uint32_t scan_bound_from_records(const uint16_t *__restrict__ rec, int P,
                                                            uint32_t k, int shift, uint32_t qmax) {
    const uint32_t s = scan_rec_row_sum(rec + (size_t)__lane_id() * QADC_REC_SLOTS, P, 0, QADC_REC_SLOTS / 8);
    const uint64_t reached = __ballot(s >= k);
    return scan_bound_of_bin(reached ? (uint32_t)(__ffsll((unsigned long long)reached) - 1) : 0xffffffffu, shift, qmax);
}
// The same by a block of 256 threads with few registers each: four adjacent lanes share a bin
// (two chunks each), so every wave covers 16 bins; the wave's first bin that reaches k (or
// 0xffffffff) goes to first_bin[wave], and after the block's next barrier the bound is
// scan_bound_of_bin(min of the four).  All 256 threads call it.
__device__ __forceinline__ void scan_bound_bins_256(const uint16_t *__restrict__ rec, int P, uint32_t k,
                                                    uint32_t *first_bin) {
    const int wave = threadIdx.x / QADC_WAVE, lane = threadIdx.x % QADC_WAVE;
    const int bin = wave * 16 + lane / 4, part = lane % 4;
    constexpr int CPL = QADC_REC_SLOTS / 8 / 4;  // 16-byte chunks per lane
    uint32_t s = scan_rec_row_sum(rec + (size_t)bin * QADC_REC_SLOTS, P, CPL * part, CPL * part + CPL);
    s += QADC_DPP_STEP(0u, s, 0xB1, 0xf);  // quad_perm [1,0,3,2]
    s += QADC_DPP_STEP(0u, s, 0x4E, 0xf);  // quad_perm [2,3,0,1]
    const uint64_t reached = __ballot(s >= k);
    if (lane == 0) first_bin[wave] = reached ? (uint32_t)(wave * 16 + (__ffsll((unsigned long long)reached) - 1) / 4) : 0xffffffffu;
}

// LDS of a selection block of NT threads that can rank ACAP candidates.
template <int NT, int ACAP>
struct SelectLds {
    uint64_t A[ACAP];                 // candidates up to the bin of the R-th
    uint32_t whist[NT / 64][256];     // one key-bin histogram per wave; later: counts / starts / cursors
    uint32_t hist[256];
    uint32_t sh[32];
    uint16_t order[ACAP];
};

// Block-wide (NT threads): from the QADC_NSUB candidate lists of a query (list l: min(count_l,
// cap) entries at cand + l * cap), find the key bin (key >> shift) of the kk-th smallest
// candidate, kk = min(R, all of them), and leave every candidate up to that bin in S.A.
// NT / QADC_NSUB adjacent threads share a list, REG entries each per round (held in
// registers), all loads of a round in flight together.  COHERENT: the lists were written by other blocks of this same
// kernel (they are read with device-scope loads).  Returns the number kept, or -1 when a list
// overflowed or the kept ones exceed ACAP.
template <int NT, int ACAP, bool COHERENT, int REG>
__device__ inline int select_from_lists(const ScanHdr *__restrict__ h, const uint64_t *__restrict__ cand,
                                        uint32_t cap, int R, int shift, SelectLds<NT, ACAP> &S) {
    constexpr int W = NT / QADC_NSUB;  // threads per list
    const int wave = threadIdx.x / QADC_WAVE, lane = threadIdx.x % QADC_WAVE;
    const int l = threadIdx.x / W, sub = threadIdx.x % W;
    const uint64_t *mine = cand + (size_t)l * cap;
    auto load = [&](uint32_t e) -> uint64_t {
        if (COHERENT)
            return __hip_atomic_load((const unsigned long long *)mine + e, __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
        return mine[e];
    };
    // the list's length and its first W * REG entries are requested together (entries beyond
    // the length are read and ignored; none beyond the capacity), before anything else
    uint32_t cnt = COHERENT ? __hip_atomic_load(&h->count[l][0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                            : h->count[l][0];
    uint64_t c[REG];
#pragma unroll
    for (int u = 0; u < REG; ++u) {
        const uint32_t e = u * W + sub;
        c[u] = e < cap ? load(e) : ~0ull;
    }
    for (int i = threadIdx.x; i < (NT / 64) * 256; i += NT) (&S.whist[0][0])[i] = 0;
    if (threadIdx.x < 8) S.sh[threadIdx.x] = 0;  // 0: kept, 1: overflow flag, 2: all candidates, 3: longest list
    __syncthreads();
    if (sub == 0) {
        if (cnt > cap) S.sh[1] = 1u;
        atomicAdd(&S.sh[2], cnt);
        atomicMax(&S.sh[3], cnt);
    }
    // first round of the histogram from the registers
#pragma unroll
    for (int u = 0; u < REG; ++u)
        if ((uint32_t)(u * W + sub) < cnt && (uint32_t)(u * W + sub) < cap)
            atomicAdd(&S.whist[wave][((uint32_t)(c[u] >> 32) >> shift) & 255u], 1u);
    __syncthreads();
    if (S.sh[1] != 0) {
        __syncthreads();
        return -1;
    }
    const uint32_t E = S.sh[2], longest = S.sh[3];
    const bool single = longest <= (uint32_t)(W * REG);  // the second pass reuses the registers
    uint32_t kbin = 255;
    for (int pass = 0; pass < 2; ++pass) {
        for (uint32_t base = (pass == 0 ? W * REG : 0); base < longest; base += W * REG) {
            if (pass == 0 || !single) {
#pragma unroll
                for (int u = 0; u < REG; ++u) {
                    const uint32_t e = base + u * W + sub;
                    c[u] = e < cnt ? load(e) : ~0ull;
                }
            }
            if (pass == 0) {
#pragma unroll
                for (int u = 0; u < REG; ++u)
                    if (base + u * W + sub < cnt)
                        atomicAdd(&S.whist[wave][((uint32_t)(c[u] >> 32) >> shift) & 255u], 1u);
            } else {
                // (few candidates reach this point -- about R of some thousands -- so each takes
                // its place with an LDS atomic of its own)
#pragma unroll
                for (int u = 0; u < REG; ++u) {
                    if (base + u * W + sub < cnt && (((uint32_t)(c[u] >> 32) >> shift) & 255u) <= kbin) {
                        const uint32_t pos = atomicAdd(&S.sh[0], 1u);
                        if (pos < (uint32_t)ACAP) S.A[pos] = c[u]; else S.sh[1] = 1u;
                    }
                }
            }
        }
        __syncthreads();
        if (pass == 0) {
            // the bin of the kk-th smallest: wave 0 adds up the waves' histograms, four bins per lane
            if (threadIdx.x < QADC_WAVE) {
                uint32_t hb[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int w = 0; w < NT / 64; ++w) {
                    const uint4 x = *(const uint4 *)&S.whist[w][4 * lane];
                    hb[0] += x.x; hb[1] += x.y; hb[2] += x.z; hb[3] += x.w;
                }
                const uint32_t kk = E < (uint32_t)R ? E : (uint32_t)R;
                const uint32_t s4 = hb[0] + hb[1] + hb[2] + hb[3];
                uint32_t run = qadc_wave_incl_scan(s4) - s4;
                uint32_t my = 0xffffffffu;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (my == 0xffffffffu && (run + hb[i] >= kk || 4 * lane + i == 255)) my = (uint32_t)(4 * lane + i);
                    run += hb[i];
                }
                const uint32_t best = qadc_wave_min(my);
                if (lane == 0) S.sh[4] = best;
            }
            __syncthreads();
            kbin = S.sh[4];
        }
    }
    const int na = S.sh[1] != 0 ? -1 : (int)S.sh[0];
    __syncthreads();
    return na;
}

struct FinalShared {
    uint32_t *hist;            // [256]
    uint32_t (*whist)[256];    // [16][256] per-wave histograms
    uint32_t *sh;              // [32] scalars
    uint32_t *wsum;            // [16]
    uint32_t *off;             // [MAX_G + 1] exclusive prefix of the list lengths
};

// Block-wide (256 to 1024 threads): gather the candidates of G slot lists (counts[],
// slots[][cap_b]), find the bin of the R-th smallest by histogram (binf maps a candidate to a
// bin 0..255 that is monotone in its sort key) and leave the candidates up to that bin in A (at
// most cap_a).  Returns true if a list overflowed or A would overflow: the caller must then
// select exactly by other means.  na = entries in A.
template <class BinF>
__device__ inline bool gather_select(const uint32_t *__restrict__ counts,
                                     const uint64_t *__restrict__ slots, int G, int cap_b, int R,
                                     BinF binf, uint64_t *A, int cap_a, const FinalShared &S, int &na) {
    const uint32_t bd = blockDim.x;  // any multiple of 64 up to 1024 with FINAL_LPT * bd >= G
    const int nwaves = (int)(bd / QADC_WAVE);
    const int wave = threadIdx.x / QADC_WAVE, lane = threadIdx.x % QADC_WAVE;
    // exclusive prefix sum of the G per-block counts: FINAL_LPT consecutive lists per thread
    uint32_t cnt[FINAL_LPT], mine = 0;
    bool over = false;
#pragma unroll
    for (int l = 0; l < FINAL_LPT; ++l) {
        const int list = FINAL_LPT * (int)threadIdx.x + l;
        cnt[l] = list < G ? counts[list] : 0u;
        over = over || cnt[l] > (uint32_t)cap_b;
        mine += cnt[l];
    }
    for (int i = threadIdx.x; i < nwaves * 256; i += blockDim.x) (&S.whist[0][0])[i] = 0;
    const uint32_t incl = qadc_wave_incl_scan(mine);
    if (lane == QADC_WAVE - 1) S.wsum[wave] = incl;
    if (threadIdx.x == 0) {
        S.sh[0] = 0;  // entries gathered into A
        S.sh[1] = 0;  // slow-path flag
    }
    __syncthreads();
    uint32_t wbase = 0, E = 0;
    for (int w = 0; w < (int)(blockDim.x / QADC_WAVE); ++w) {
        wbase += (w < wave) ? S.wsum[w] : 0u;
        E += S.wsum[w];
    }
    {
        uint32_t run = wbase + incl - mine;
#pragma unroll
        for (int l = 0; l < FINAL_LPT; ++l) {
            const int list = FINAL_LPT * (int)threadIdx.x + l;
            if (list < G) S.off[list] = run;
            run += cnt[l];
        }
    }
    if (threadIdx.x == 0) S.off[G] = E;
    if (over) S.sh[1] = 1u;
    __syncthreads();
    const bool slow0 = S.sh[1] != 0;

    na = 0;
    bool slow = slow0;
    if (!slow0) {
        // Candidates are dealt out evenly: thread t takes entries t, t+1024, ... of the
        // concatenated slot lists, FINAL_REG at a time with all loads in flight together.
        // pass 0: histogram of candidate key bins -> bin of the R-th key;
        // pass 1: keep the candidates up to that bin.  When everything fits one batch
        // the second pass reuses the registers of the first.
        uint64_t c[FINAL_REG];
        const bool single = E <= (uint32_t)FINAL_REG * bd;
        uint32_t kbin = 255;
        for (int pass = 0; pass < 2; ++pass) {
            for (uint32_t base = 0; base < E; base += FINAL_REG * bd) {
                if (pass == 0 || !single) {
                    // list of each entry: largest index with S.off[list] <= e, by a branch-free
                    // binary search whose FINAL_REG chains run interleaved
                    uint32_t pos[FINAL_REG];
#pragma unroll
                    for (int u = 0; u < FINAL_REG; ++u) pos[u] = 0;
                    // first step: half the smallest power of two that is >= G
                    for (uint32_t s = G > 1 ? 1u << (31 - __clz(G - 1)) : 1u; s >= 1; s >>= 1) {
#pragma unroll
                        for (int u = 0; u < FINAL_REG; ++u) {
                            const uint32_t e = base + u * bd + threadIdx.x;
                            const uint32_t idx = pos[u] + s;
                            const uint32_t v = idx < (uint32_t)G ? S.off[idx] : 0xffffffffu;
                            pos[u] = v <= e ? idx : pos[u];
                        }
                    }
#pragma unroll
                    for (int u = 0; u < FINAL_REG; ++u) {
                        const uint32_t e = base + u * bd + threadIdx.x;
                        c[u] = e < E ? slots[(size_t)pos[u] * cap_b + (e - S.off[pos[u]])] : ~0ull;
                    }
                }
#pragma unroll
                for (int u = 0; u < FINAL_REG; ++u) {
                    const uint32_t e = base + u * bd + threadIdx.x;
                    if (e >= E) continue;
                    const uint32_t bin = binf(c[u]);
                    if (pass == 0) {
                        atomicAdd(&S.whist[wave][bin], 1u);
                    } else if (bin <= kbin) {
                        const uint32_t pos = atomicAdd(&S.sh[0], 1u);
                        if (pos < (uint32_t)cap_a) A[pos] = c[u]; else S.sh[1] = 1u;
                    }
                }
            }
            __syncthreads();
            if (pass == 0) {
                if (threadIdx.x < 256) {
                    uint32_t t = 0;
#pragma unroll
                    for (int w = 0; w < 16; ++w)
                        if (w < nwaves) t += S.whist[w][threadIdx.x];
                    S.hist[threadIdx.x] = t;
                }
                __syncthreads();
                const uint32_t kk = E < (uint32_t)R ? E : (uint32_t)R;
                if (threadIdx.x < QADC_WAVE) qadc_wave_select_bin(S.hist, kk, 0u, S.sh + 4);
                __syncthreads();
                kbin = S.sh[4];
            }
        }
        na = (int)S.sh[0];
        slow = S.sh[1] != 0;
        __syncthreads();
    }
    return slow;
}// Block-wide (1024 threads), for many short slot lists (the exhaustive scan leaves one list
// per scan block, a few entries each): same contract as gather_select.  W = 2^logw adjacent
// threads (4 <= W <= 32) read the first W entries of a list, each thread serving NU lists
// per batch, so that all loads of the common case, the list lengths included, are
// independent and in flight together; longer lists take extra rounds.  Entries beyond a
// list's length are loaded and ignored, which needs cap_b >= W.  NU is 8, 16 or 32.
template <int NU, int NT, int ACAP, class BinF>  // NT threads per block, A holds ACAP entries
__device__ inline bool gather_select_rows(const uint32_t *__restrict__ counts,
                                          const uint64_t *__restrict__ slots, int G, int cap_b,
                                          int R, int logw, BinF binf, uint64_t *A,
                                          const FinalShared &S, int &na) {
    const int W = 1 << logw;
    const int LP = NT >> logw;  // lists per batch row
    const int wave = threadIdx.x / QADC_WAVE, lane = threadIdx.x % QADC_WAVE;
    const int sub = threadIdx.x & (W - 1), row = threadIdx.x >> logw;
    for (int i = threadIdx.x; i < NT / QADC_WAVE * 256; i += NT) (&S.whist[0][0])[i] = 0;
    if (threadIdx.x < 8) S.sh[threadIdx.x] = 0;  // 0: entries in A, 1: slow flag, 2: candidates
    __syncthreads();
    const bool single = G <= LP * NU;  // one batch: pass 1 reuses the registers of pass 0
    uint32_t kbin = 255;
    uint64_t c[NU];
    uint32_t valid = 0;   // bit u: c[u] is an entry of its list
    uint32_t longer = 0;  // bit u: list u of this thread has more than W entries
    for (int pass = 0; pass < 2; ++pass) {
        uint32_t mine = 0;
        bool over = false;
        for (int kb = 0; kb < G; kb += LP * NU) {
            if (pass == 0 || !single) {
                uint32_t cnt[NU];
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    const int list = kb + row + LP * u;
                    const bool have = list < G;
                    cnt[u] = have ? counts[list] : 0u;
                    c[u] = have ? slots[(size_t)list * cap_b + sub] : ~0ull;
                }
                valid = 0;
                longer = 0;
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    valid |= ((uint32_t)sub < cnt[u] ? 1u : 0u) << u;
                    longer |= (cnt[u] > (uint32_t)W ? 1u : 0u) << u;
                    if (pass == 0 && sub == 0) {
                        mine += cnt[u];
                        over = over || cnt[u] > (uint32_t)cap_b;
                    }
                }
            }
            if (pass == 0) {
#pragma unroll
                for (int u = 0; u < NU; ++u)
                    if ((valid >> u) & 1u) atomicAdd(&S.whist[wave][binf(c[u])], 1u);
            } else {
                // keep the candidates up to the bin of the R-th: one LDS atomic per wave
                uint32_t keep = 0, total = 0;
#pragma unroll
                for (int u = 0; u < NU; ++u)
                    keep |= ((((valid >> u) & 1u) != 0 && binf(c[u]) <= kbin) ? 1u : 0u) << u;
#pragma unroll
                for (int u = 0; u < NU; ++u) total += (uint32_t)__popcll(__ballot((keep >> u) & 1u));
                if (total != 0) {
                    uint32_t base = 0;
                    if (lane == 0) base = atomicAdd(&S.sh[0], total);
                    base = __builtin_amdgcn_readfirstlane(base);
                    if (base + total > ACAP && lane == 0) S.sh[1] = 1u;
#pragma unroll
                    for (int u = 0; u < NU; ++u) {
                        const uint64_t m = __ballot((keep >> u) & 1u);
                        const uint32_t pos = base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
                        if (((keep >> u) & 1u) && pos < ACAP) A[pos] = c[u];
                        base += (uint32_t)__popcll(m);
                    }
                }
            }
            // lists longer than one round (rare): entry by entry
            for (uint32_t rest = longer; rest != 0; rest &= rest - 1) {
                const int u = __ffs(rest) - 1;
                const int list = kb + row + LP * u;
                uint32_t lim = counts[list];
                lim = lim > (uint32_t)cap_b ? (uint32_t)cap_b : lim;
                for (uint32_t r = W + sub; r < lim; r += W) {
                    const uint64_t e = slots[(size_t)list * cap_b + r];
                    const uint32_t bin = binf(e);
                    if (pass == 0) {
                        atomicAdd(&S.whist[wave][bin], 1u);
                    } else if (bin <= kbin) {
                        const uint32_t pos = atomicAdd(&S.sh[0], 1u);
                        if (pos < ACAP) A[pos] = e; else S.sh[1] = 1u;
                    }
                }
            }
        }
        if (pass == 0) {
            if (over) S.sh[1] = 1u;
            if (mine) atomicAdd(&S.sh[2], mine);
        }
        __syncthreads();
        if (S.sh[1] != 0) break;
        if (pass == 0) {
            if (threadIdx.x < 256) {
                uint32_t t = 0;
#pragma unroll
                for (int w = 0; w < NT / QADC_WAVE; ++w) t += S.whist[w][threadIdx.x];
                S.hist[threadIdx.x] = t;
            }
            __syncthreads();
            const uint32_t E = S.sh[2];
            const uint32_t kk = E < (uint32_t)R ? E : (uint32_t)R;
            if (threadIdx.x < QADC_WAVE) qadc_wave_select_bin(S.hist, kk, 0u, S.sh + 4);
            __syncthreads();
            kbin = S.sh[4];
        }
    }
    const bool slow = S.sh[1] != 0;
    na = slow ? 0 : (int)S.sh[0];
    __syncthreads();
    return slow;
}
