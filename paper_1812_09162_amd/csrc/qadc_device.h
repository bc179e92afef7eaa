// Device-side helpers shared by the kernels of libqadc (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qadc_internal.h"

#define QADC_WAVE 64

// Sub-code extraction from a little-endian bit stream (Section 3.3): `b` bits
// starting at bit `off`; b <= 8, so at most two bytes are touched and the
// second one is only read when the field really reaches into it.
__device__ __forceinline__ uint32_t qadc_extract_sub(const uint8_t *code, int off, int b) {
    int byte = off >> 3, sh = off & 7;
    uint32_t v = (uint32_t)code[byte] >> sh;
    if (sh + b > 8) v |= (uint32_t)code[byte + 1] << (8 - sh);
    return v & ((1u << b) - 1u);
}

// A code of at most 16 bytes as four little-endian dwords (missing bytes read as zero): one
// 8- or 16-byte load when the size allows, byte loads otherwise.
__device__ __forceinline__ void qadc_load_code16(const uint8_t *code, int cs, uint32_t w[4]) {
    if (cs == 8) {
        const uint2 v = *(const uint2 *)code;
        w[0] = v.x; w[1] = v.y; w[2] = 0; w[3] = 0;
    } else if (cs == 16) {
        const uint4 v = *(const uint4 *)code;
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    } else {
        w[0] = w[1] = w[2] = w[3] = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (i < cs) w[i >> 2] |= (uint32_t)code[i] << (8 * (i & 3));
    }
}

// Sub-code of `b` <= 8 bits at bit `off` (uniform across the wave) of a code held as dwords.
__device__ __forceinline__ uint32_t qadc_extract_sub16(const uint32_t w[4], int off, int b) {
    const int i = off >> 5, sh = off & 31;
    const uint32_t lo = i == 0 ? w[0] : (i == 1 ? w[1] : (i == 2 ? w[2] : w[3]));
    const uint32_t hi = i == 0 ? w[1] : (i == 1 ? w[2] : (i == 2 ? w[3] : 0u));
    const uint32_t v = sh == 0 ? lo : ((lo >> sh) | (hi << (32 - sh)));
    return v & ((1u << b) - 1u);
}

// Group field extraction: `w` <= 12 bits starting at bit `off` of a code of
// `cs` bytes; touches at most three bytes, never past the end of the code.
__device__ __forceinline__ uint32_t qadc_extract_group(const uint8_t *code, int cs, int off, int w) {
    int byte = off >> 3, sh = off & 7;
    uint32_t v = code[byte];
    if (byte + 1 < cs) v |= (uint32_t)code[byte + 1] << 8;
    if (byte + 2 < cs) v |= (uint32_t)code[byte + 2] << 16;
    return (v >> sh) & ((1u << w) - 1u);
}

// esub[e] = sub-quantizer that table entry e belongs to.  Block-wide; ends with a barrier.
__device__ inline void qadc_build_entry_map(const DevLayout *L, uint8_t *esub) {
    const int m = L->m;
    for (int j = 0; j < m; ++j) {
        const int kj = 1 << L->nbits[j], t0 = L->toff[j];
        for (int i = threadIdx.x; i < kj; i += blockDim.x) esub[t0 + i] = (uint8_t)j;
    }
    __syncthreads();
}

// Order-preserving map float -> uint32 (and back) for radix selection.
__device__ __forceinline__ uint32_t qadc_f2ord(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float qadc_ord2f(uint32_t o) {
    uint32_t u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
    return __uint_as_float(u);
}

// Wave-wide operations (wave64) through data-parallel-primitive moves: shifts within rows of 16
// lanes by 1, 2, 4, 8, then lane 15 of rows 0 and 2 broadcast to the next row, then lane 31 to
// rows 2 and 3.  Lanes without a source take the neutral element.  (Six register moves; the
// same through cross-lane shuffles takes six trips through the LDS crossbar.)
#define QADC_DPP_STEP(OLD, V, CTRL, ROWS) (uint32_t)__builtin_amdgcn_update_dpp((int)(OLD), (int)(V), CTRL, ROWS, 0xf, false)

// inclusive prefix sum
__device__ __forceinline__ uint32_t qadc_wave_incl_scan(uint32_t v) {
    v += QADC_DPP_STEP(0u, v, 0x111, 0xf);
    v += QADC_DPP_STEP(0u, v, 0x112, 0xf);
    v += QADC_DPP_STEP(0u, v, 0x114, 0xf);
    v += QADC_DPP_STEP(0u, v, 0x118, 0xf);
    v += QADC_DPP_STEP(0u, v, 0x142, 0xa);
    v += QADC_DPP_STEP(0u, v, 0x143, 0xc);
    return v;
}

// minimum / maximum over the wave, returned to every lane
__device__ __forceinline__ uint32_t qadc_wave_min(uint32_t v) {
    uint32_t t;
    t = QADC_DPP_STEP(0xffffffffu, v, 0x111, 0xf); v = t < v ? t : v;
    t = QADC_DPP_STEP(0xffffffffu, v, 0x112, 0xf); v = t < v ? t : v;
    t = QADC_DPP_STEP(0xffffffffu, v, 0x114, 0xf); v = t < v ? t : v;
    t = QADC_DPP_STEP(0xffffffffu, v, 0x118, 0xf); v = t < v ? t : v;
    t = QADC_DPP_STEP(0xffffffffu, v, 0x142, 0xa); v = t < v ? t : v;
    t = QADC_DPP_STEP(0xffffffffu, v, 0x143, 0xc); v = t < v ? t : v;
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ uint32_t qadc_wave_max(uint32_t v) { return ~qadc_wave_min(~v); }

// Over 256 bins: the smallest bin b with base + hist[0..b] >= kk (bin 255 if
// none), and base + hist[0..b-1].  Called by one full wave; the result goes to
// out[0], out[1] (LDS or registers of the caller via the return value).
__device__ inline void qadc_wave_select_bin(const uint32_t *hist, uint32_t kk, uint32_t base,
                                            uint32_t *out) {
    const int lane = __lane_id();
    uint32_t h[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) h[i] = hist[4 * lane + i];
    const uint32_t s = h[0] + h[1] + h[2] + h[3];
    uint32_t run = base + qadc_wave_incl_scan(s) - s;
    uint32_t mine = 0xffffffffu, below = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t bin = (uint32_t)(4 * lane + i);
        if (mine == 0xffffffffu && (run + h[i] >= kk || bin == 255u)) {
            mine = bin;
            below = run;
        }
        run += h[i];
    }
    const uint32_t best = qadc_wave_min(mine);
    if (mine == best) {
        out[0] = best;
        out[1] = below;
    }
}

// k-th smallest (k >= 1, k <= cnt) of cnt > 0 uint32 values in LDS, by radix selection over
// the bits in which the values differ at all: the bits above the highest differing one are
// common to all values (ordered floats of similar size share their upper bytes, and counting
// those would send every value to one histogram bin), the rest is taken eight bits at a time
// from the top.  All threads of the block call it; `hist` is 256 words of LDS, `sel` two
// words.  Returns the value to every thread.  (`nbytes` is kept for callers: the values'
// width in bytes.)
__device__ inline uint32_t qadc_block_kth_u32(const uint32_t *vals, int cnt, int k, int nbytes,
                                              uint32_t *hist, uint32_t *sel) {
    (void)nbytes;
    uint32_t mn = 0xffffffffu, mxn = 0xffffffffu;  // minimum, and minimum of the complements
    for (int i = threadIdx.x; i < cnt; i += blockDim.x) {
        const uint32_t v = vals[i];
        mn = v < mn ? v : mn;
        mxn = ~v < mxn ? ~v : mxn;
    }
    mn = qadc_wave_min(mn);
    mxn = qadc_wave_min(mxn);
    if (threadIdx.x == 0) {
        sel[0] = 0xffffffffu;
        sel[1] = 0xffffffffu;
    }
    __syncthreads();
    if (threadIdx.x % QADC_WAVE == 0) {
        atomicMin(&sel[0], mn);
        atomicMin(&sel[1], mxn);
    }
    __syncthreads();
    mn = sel[0];
    const uint32_t mx = ~sel[1];
    __syncthreads();
    if (mn == mx) return mn;
    int rb = 32 - __clz((int)(mn ^ mx));  // the bits [0, rb) are undecided
    uint32_t prefix = rb >= 32 ? 0u : (mn >> rb) << rb;
    int kk = k;
    // Equal values are common (a saturated key gives one distance per list), and LDS atomics of
    // one wave to one word are served one lane at a time: every bin is kept as eight adjacent
    // words (eight banks), lane l counting in word l % 8, and summed before the selection.
    __shared__ __align__(16) uint32_t hist8[256 * 8];
    while (rb > 0) {
        const int w = rb < 8 ? rb : 8, shift = rb - w;
        for (int i = threadIdx.x; i < 256 * 8; i += blockDim.x) hist8[i] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < cnt; i += blockDim.x) {
            const uint32_t v = vals[i];
            const bool in = rb >= 32 || (v >> rb) == (prefix >> rb);
            if (in) atomicAdd(&hist8[(((v >> shift) & ((1u << w) - 1u)) << 3) + (threadIdx.x & 7u)], 1u);
        }
        __syncthreads();
        for (int i = threadIdx.x; i < 256; i += blockDim.x) {
            const uint4 a = *(const uint4 *)&hist8[8 * i], b = *(const uint4 *)&hist8[8 * i + 4];
            hist[i] = a.x + a.y + a.z + a.w + b.x + b.y + b.z + b.w;
        }
        __syncthreads();
        if (threadIdx.x < QADC_WAVE) qadc_wave_select_bin(hist, (uint32_t)kk, 0u, sel);
        __syncthreads();
        prefix |= sel[0] << shift;
        kk -= (int)sel[1];
        rb = shift;
        __syncthreads();
    }
    return prefix;
}


// k-th smallest (1 <= k <= cnt) of cnt > 0 finite floats held in LDS as ordered words
// (qadc_f2ord), for the common case of values that are spread out: 256 equal bins over
// [min, max] (subtraction, multiplication by a positive factor and truncation are all monotone
// under rounding, so a lower bin never holds a larger value), the bin that holds the k-th, and
// an exact pick among that bin's few members by counting.  Five short steps with a barrier
// each instead of the radix selection's four passes; a crowded bin (many equal values) or a
// degenerate range falls back to qadc_block_kth_u32.  All threads of the block call it; `hist`
// is 256 words of LDS, `sel` eight, `mem` QADC_KTH_MEM.  Returns the value to every thread.
#define QADC_KTH_MEM 256
__device__ inline uint32_t qadc_block_kth_f32(const uint32_t *vals, int cnt, int k, uint32_t *hist,
                                              uint32_t *sel, uint32_t *mem) {
    uint32_t mn = 0xffffffffu, mx = 0u;
    for (int i = threadIdx.x; i < cnt; i += blockDim.x) {
        const uint32_t v = vals[i];
        mn = v < mn ? v : mn;
        mx = v > mx ? v : mx;
    }
    mn = qadc_wave_min(mn);
    mx = qadc_wave_max(mx);
    if (threadIdx.x == 0) {
        sel[0] = 0xffffffffu;
        sel[1] = 0u;
        sel[2] = 0u;  // members gathered
    }
    for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
    __syncthreads();
    if (threadIdx.x % QADC_WAVE == 0) {
        atomicMin(&sel[0], mn);
        atomicMax(&sel[1], mx);
    }
    __syncthreads();
    mn = sel[0];
    mx = sel[1];
    if (mn == mx) {
        __syncthreads();
        return mn;
    }
    const float fmn = qadc_ord2f(mn);
    const float scale = 256.0f / (qadc_ord2f(mx) - fmn);
    const bool usable = scale > 0.0f && scale <= 3.0e38f;  // (block-uniform)
    auto bin_of = [fmn, scale](uint32_t v) {
        const float x = (qadc_ord2f(v) - fmn) * scale;  // >= 0
        return x >= 255.0f ? 255u : (uint32_t)x;
    };
    if (usable) {
        for (int i = threadIdx.x; i < cnt; i += blockDim.x) atomicAdd(&hist[bin_of(vals[i])], 1u);
        __syncthreads();
        if (threadIdx.x < QADC_WAVE) qadc_wave_select_bin(hist, (uint32_t)k, 0u, sel + 4);
        __syncthreads();
    }
    const uint32_t b = usable ? sel[4] : 0u, below = usable ? sel[5] : 0u;
    const uint32_t nm = usable ? hist[b] : 0xffffffffu;
    if (nm > QADC_KTH_MEM) {
        __syncthreads();
        return qadc_block_kth_u32(vals, cnt, k, 4, hist, sel);
    }
    for (int i = threadIdx.x; i < cnt; i += blockDim.x) {
        const uint32_t v = vals[i];
        if (bin_of(v) == b) mem[atomicAdd(&sel[2], 1u)] = v;
    }
    __syncthreads();
    const uint32_t r = (uint32_t)k - below;  // 1-based rank among the nm members
    for (uint32_t i = threadIdx.x; i < nm; i += blockDim.x) {
        const uint32_t mine = mem[i];
        uint32_t lt = 0, le = 0;
        for (uint32_t j = 0; j < nm; ++j) {
            const uint32_t o = mem[j];
            lt += o < mine ? 1u : 0u;
            le += o <= mine ? 1u : 0u;
        }
        if (lt < r && r <= le) sel[3] = mine;  // (equal values may all write: the same word)
    }
    __syncthreads();
    const uint32_t res = sel[3];
    __syncthreads();
    return res;
}
