// Index handle, layout planning and error reporting.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "scan_device.h"

static thread_local char g_err[512] = "";

void qadc_set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char *pq_last_error(void) { return g_err; }

// ----------------------------------------------------------- tuning options ---
// Process-wide, set through pq_set_option; none changes a result.
#include <atomic>
static std::atomic<int64_t> g_opt[PQ_OPT_COUNT] = {
    {2048},    // PQ_OPT_SCAN_BLOCKS
    {524288},  // PQ_OPT_PILOT_CODES
    {65536},   // PQ_OPT_PILOT_CODES_SINGLE
    {128},     // PQ_OPT_PILOT_BLOCKS
    {128},     // PQ_OPT_IVF_THREADS
    {1},       // PQ_OPT_SHARED_PASSES
    {1},       // PQ_OPT_COARSE_FILTER
    {1},       // PQ_OPT_IVF_SHARED_LISTS
};

int64_t qadc_option(int option) { return g_opt[option].load(std::memory_order_relaxed); }

extern "C" int pq_set_option(int option, int64_t value) {
    bool ok = option >= 0 && option < PQ_OPT_COUNT;
    if (ok) switch (option) {
        case PQ_OPT_SCAN_BLOCKS: ok = value >= 1 && value <= 4096; break;
        case PQ_OPT_PILOT_CODES: ok = value >= 0 && value <= ((int64_t)1 << 24); break;
        case PQ_OPT_PILOT_CODES_SINGLE: ok = value >= 0 && value <= ((int64_t)1 << 24); break;
        case PQ_OPT_PILOT_BLOCKS: ok = value >= 1 && value <= 128; break;
        case PQ_OPT_IVF_THREADS: ok = value == 64 || value == 128 || value == 256; break;
        case PQ_OPT_IVF_SHARED_LISTS: ok = value >= 0 && value <= 2; break;
        default: ok = value == 0 || value == 1; break;
    }
    if (!ok) {
        qadc_set_error("pq_set_option: option %d does not take the value %lld", option, (long long)value);
        return PQ_EINVAL;
    }
    g_opt[option].store(value, std::memory_order_relaxed);
    return PQ_OK;
}

extern "C" int64_t pq_get_option(int option) {
    return option >= 0 && option < PQ_OPT_COUNT ? qadc_option(option) : -1;
}

// Partition the sub-quantizers into consecutive groups of at most gmax bits.
static void plan_groups(DevLayout &L, int gmax) {
    L.ng = 0;
    L.gtab_len = 0;
    L.g32ok = 1;
    int j = 0;
    while (j < L.m) {
        int g = L.ng++;
        L.gfirst[g] = (int32_t)j;
        L.goff[g] = L.bitoff[j];
        int w = L.nbits[j];
        int cnt = 1;
        // a group never crosses a 32-bit boundary of the code unless a single sub-quantizer does
        while (j + cnt < L.m && w + L.nbits[j + cnt] <= gmax &&
               (L.bitoff[j] % 32) + w + L.nbits[j + cnt] <= 32) {
            w += L.nbits[j + cnt];
            ++cnt;
        }
        L.gw[g] = (int32_t)w;
        L.gcount[g] = (int32_t)cnt;
        L.gbase[g] = (int32_t)L.gtab_len;
        L.gtab_len += 1 << w;
        if ((L.bitoff[j] % 32) + w > 32) L.g32ok = 0;
        j += cnt;
    }
}

extern "C" int pq_index_create(pq_index_t **out, int d, int m, const int32_t *nbits,
                               const int32_t *dsub, const float *codebooks, int acc_bits) {
    if (!out || !nbits || !dsub || !codebooks) {
        qadc_set_error("pq_index_create: null argument");
        return PQ_EINVAL;
    }
    *out = nullptr;
    if (d < 1 || d > PQ_MAX_DIM || m < 1 || m > PQ_MAX_M || (acc_bits != 8 && acc_bits != 16)) {
        qadc_set_error("pq_index_create: need 1<=d<=%d, 1<=m<=%d, acc_bits in {8,16} (got d=%d m=%d acc_bits=%d)",
                       PQ_MAX_DIM, PQ_MAX_M, d, m, acc_bits);
        return PQ_EINVAL;
    }
    DevLayout L;
    memset(&L, 0, sizeof(L));
    L.d = d;
    L.m = m;
    L.acc_bits = acc_bits;
    L.qmax = (1 << acc_bits) - 1;
    int bit = 0, t = 0, dim = 0;
    size_t cb = 0;
    for (int j = 0; j < m; ++j) {
        if (nbits[j] < 1 || nbits[j] > 8 || dsub[j] < 1) {
            qadc_set_error("pq_index_create: nbits[%d]=%d (1..8) dsub[%d]=%d (>=1)", j, nbits[j], j, dsub[j]);
            return PQ_EINVAL;
        }
        L.nbits[j] = (int32_t)nbits[j];
        L.bitoff[j] = (int32_t)bit;
        L.toff[j] = (int32_t)t;
        L.dimoff[j] = (int32_t)dim;
        L.dsub[j] = (int32_t)dsub[j];
        L.cboff[j] = (int32_t)cb;
        bit += nbits[j];
        t += 1 << nbits[j];
        dim += dsub[j];
        cb += ((size_t)1 << nbits[j]) * (size_t)dsub[j];
        if (dim > d) break;
    }
    if (dim != d) {
        qadc_set_error("pq_index_create: sum(dsub)=%d differs from d=%d", dim, d);
        return PQ_EINVAL;
    }
    if (t > PQ_MAX_TABLE_LEN) {
        qadc_set_error("pq_index_create: table length %d exceeds %d", t, PQ_MAX_TABLE_LEN);
        return PQ_EINVAL;
    }
    L.T = t;
    L.code_bits = bit;
    L.cs = (bit + 7) / 8;

    // group plan: widest groups whose tables stay within 18 KB of LDS (eight scan blocks per CU)
    const int esz = acc_bits == 8 ? 1 : 2;
    bool all4 = true;
    for (int j = 0; j < m; ++j) all4 = all4 && nbits[j] == 4;
    if (all4 && m % 2 == 0) {
        plan_groups(L, 8);
    } else {
        // (groups of at most 10 bits: for {6,5,5,6,5,5,4,4} the tables 6 | 5,5 | 6 | 5,5 | 4,4 hold
        // 2,432 entries and scan 5 % faster than 6,5 | 5,6 | 5,5 | 4,4 with 5,376: the two 64- and
        // the 256-entry tables are read without bank conflicts)
        int gmax = 10;
        for (; gmax >= 8; --gmax) {
            plan_groups(L, gmax);
            if ((size_t)L.gtab_len * esz <= 18432) break;
        }
        if (gmax < 8) plan_groups(L, 1);  // every sub-quantizer alone: T entries
    }
    L.ds_uniform = dsub[0] <= 8 ? dsub[0] : 0;
    for (int j = 1; j < m; ++j)
        if (dsub[j] != dsub[0]) L.ds_uniform = 0;
    L.kind = SCAN_GENERIC;
    if (all4 && m == 16) L.kind = SCAN_NIB8;
    if (all4 && m == 32) L.kind = SCAN_NIB16;
    if (L.kind == SCAN_GENERIC && L.cs == 8) L.kind = SCAN_W64;
    if (L.kind == SCAN_GENERIC && L.cs == 5) L.kind = SCAN_C5;
    if (L.kind == SCAN_GENERIC && L.cs == 16 && L.code_bits == 128 && L.g32ok && L.ng % 2 == 0 &&
        L.ng <= 16) {
        // two 64-bit halves with the same group pattern
        bool same = true;
        for (int g = 0; g < L.ng / 2; ++g)
            same = same && L.goff[g + L.ng / 2] == L.goff[g] + 64 && L.gw[g + L.ng / 2] == L.gw[g];
        if (same) L.kind = SCAN_W128;
    }

    pq_index *idx = new pq_index;
    idx->h = L;
    idx->codebooks = codebooks;
    idx->dev = nullptr;
    std::vector<EntryDesc> ed((size_t)L.T);
    for (int j = 0; j < m; ++j)
        for (int i = 0; i < (1 << L.nbits[j]); ++i) {
            EntryDesc &x = ed[(size_t)L.toff[j] + i];
            x.j = j;
            x.cb_off = L.cboff[j] + i * L.dsub[j];
            x.dim_off = L.dimoff[j];
            x.ds = L.dsub[j];
        }
    const size_t lay_bytes = (sizeof(DevLayout) + 15) & ~(size_t)15;
    hipError_t e = hipGetDevice(&idx->device);
    if (e == hipSuccess) e = hipMalloc((void **)&idx->dev, lay_bytes + ed.size() * sizeof(EntryDesc));
    if (e == hipSuccess) e = hipMemcpy(idx->dev, &L, sizeof(DevLayout), hipMemcpyHostToDevice);
    if (e == hipSuccess) {
        idx->edesc = (const EntryDesc *)((char *)idx->dev + lay_bytes);
        e = hipMemcpy((void *)idx->edesc, ed.data(), ed.size() * sizeof(EntryDesc), hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        qadc_set_error("pq_index_create: %s", hipGetErrorString(e));
        if (idx->dev) (void)hipFree(idx->dev);
        delete idx;
        return PQ_EHIP;
    }
    *out = idx;
    return PQ_OK;
}

extern "C" void pq_index_destroy(pq_index_t *idx) {
    if (!idx) return;
    if (idx->dev) (void)hipFree(idx->dev);
    delete idx;
}

extern "C" size_t pq_code_size(const pq_index_t *idx) { return idx ? (size_t)idx->h.cs : 0; }
extern "C" size_t pq_table_len(const pq_index_t *idx) { return idx ? (size_t)idx->h.T : 0; }

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

ScanPlan qadc_scan_plan(const pq_index *idx, int nq, int64_t n, int R) {
    ScanPlan p;
    const int64_t tile_codes = 1024;
    int64_t tiles = (n + tile_codes - 1) / tile_codes;
    // A single query gets several times more blocks than fit on the chip at once: blocks
    // start cheaply (their tables are prepared beforehand) and the hardware hands the
    // next block to whichever compute unit finishes first, which evens out the tail.
    const int64_t g1 = qadc_option(PQ_OPT_SCAN_BLOCKS);
    int64_t gmax = 32768 / (nq > 0 ? nq : 1);
    if (gmax < 64) gmax = 64;
    if (gmax > g1) gmax = g1;
    int64_t G = tiles < 1 ? 1 : (tiles > gmax ? gmax : tiles);
    p.G = (int)G;
    // candidate lists (QADC_NSUB per query): together four times the candidates expected when
    // the bound comes from a 65536-code pilot (the quantizer's smallest), plus slack for ties and
    // for an uneven spread; never more entries than codes (a list that overflows only makes the
    // selection take its slow exact path)
    int64_t cap = (4 * (n / 65536 + 1) * (int64_t)R) / QADC_NSUB + 64;
    if (cap > n + 8) cap = n + 8;
    if (cap > ((int64_t)1 << 20)) cap = (int64_t)1 << 20;
    cap = (cap + 7) & ~(int64_t)7;
    p.cap = (uint32_t)cap;
    p.gtab_off = align_up(sizeof(ScanHdr), 256);
    p.cand_off = p.gtab_off + align_up((size_t)idx->h.gtab_len * (idx->h.acc_bits == 8 ? 1 : 2), 256);
    p.per_query = align_up(p.cand_off + (size_t)QADC_NSUB * p.cap * sizeof(uint64_t), 256);
    p.total = p.per_query * (size_t)(nq > 0 ? nq : 0);
    return p;
}

IvfPlan qadc_ivf_plan(const pq_index *idx, int nq, int nprobe, int R) {
    (void)idx;
    IvfPlan p;
    p.cap_b = R <= 128 ? 1024 : 4096;
    p.counts_off = align_up(sizeof(IvfState), 256);
    p.slots_off = p.counts_off + align_up((size_t)nprobe * sizeof(uint32_t), 256);
    p.per_query = align_up(p.slots_off + (size_t)nprobe * (size_t)p.cap_b * sizeof(uint64_t), 256);
    p.total = p.per_query * (size_t)(nq > 0 ? nq : 0);
    return p;
}

extern "C" size_t ivf_workspace_bytes(const pq_index_t *idx, int nq, int nprobe, int R) {
    if (!idx || nq < 0 || nprobe < 1 || R < 1) return 0;
    size_t t = qadc_ivf_plan(idx, nq, nprobe, R).total;
    return t ? t : 256;
}

extern "C" size_t pq_workspace_bytes(const pq_index_t *idx, int nq, int64_t n, int R) {
    if (!idx || nq < 0 || n < 0 || R < 1) return 0;
    size_t t = qadc_scan_plan(idx, nq, n, R).total;
    return t ? t : 256;
}

// ------------------------------------------------------------ plain copy ---
// A copy kernel of exactly known traffic (nbytes read, nbytes written), used to
// scale hardware-counter readings taken around the scan kernel.
__global__ void __launch_bounds__(256) k_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                              size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256)
        dst[i] = src[i];
}

extern "C" int pq_copy_bytes(void *dst, const void *src, size_t nbytes, void *stream) {
    if (!dst || !src || (nbytes & 15u) || ((uintptr_t)dst & 15u) || ((uintptr_t)src & 15u)) {
        qadc_set_error("pq_copy_bytes: need non-null 16-byte aligned pointers and a multiple of 16 bytes");
        return PQ_EINVAL;
    }
    if (nbytes == 0) return PQ_OK;
    hipLaunchKernelGGL(k_copy, dim3(2048), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src,
                       (uint4 *)dst, nbytes / 16);
    QADC_LAUNCH_CHECK("k_copy");
    return PQ_OK;
}

// 8-byte LDS reads at the rate the hardware sustains for a given address pattern: every lane
// reads 8 * iters entries of eight 2 KB tables (256 entries of 8 bytes each, the shape of the
// batched scan's interleaved group tables).  The addresses change from read to read by an
// exclusive-or with a wave-uniform value, which keeps each pattern's bank behaviour.
template <int PATTERN>
__global__ void __launch_bounds__(256) k_lds_read_probe(int iters, uint32_t *__restrict__ sink) {
    __shared__ unsigned long long t[8 * 256];
    for (int i = threadIdx.x; i < 8 * 256; i += 256) t[i] = (unsigned long long)i * 0x9e3779b97f4a7c15ull;
    __syncthreads();
    uint32_t r[8];
    uint32_t x = threadIdx.x * 2654435761u + blockIdx.x;
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        x = x * 1664525u + 1013904223u;
        r[g] = PATTERN == PQ_LDS_UNIFORM ? 0u
               : (PATTERN == PQ_LDS_LINEAR ? (threadIdx.x & 63u) * 8u
                                           : ((x >> 20) & (PATTERN == PQ_LDS_RANDOM_2K ? 0x7f8u : 0x78u)));
    }
    const uint32_t mask = PATTERN == PQ_LDS_LINEAR ? 0x1f8u : (PATTERN == PQ_LDS_RANDOM_128 ? 0x78u : 0x7f8u);
    uint32_t acc = 0;
    const char *tb = (const char *)t;
    for (int it = 0; it < iters; ++it) {
        const uint32_t s = (uint32_t)it * 0x9e3779b8u;  // wave-uniform multiple of 8
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            const unsigned long long v = *(const unsigned long long *)(tb + g * 2048 + ((r[g] ^ s) & mask));
            acc ^= (uint32_t)v ^ (uint32_t)(v >> 32);
        }
    }
    if (acc == 0x1234567u) sink[0] = acc;  // (keeps the reads alive; practically never taken)
}

extern "C" int pq_lds_read_probe(int pattern, int iters, void *sink, void *stream) {
    if (pattern < 0 || pattern > PQ_LDS_RANDOM_128 || iters < 1 || !sink) {
        qadc_set_error("pq_lds_read_probe: pattern 0..%d, iters >= 1 and a device word to write to", PQ_LDS_RANDOM_128);
        return PQ_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    const dim3 grid(PQ_LDS_PROBE_BLOCKS), block(256);
    switch (pattern) {
        case PQ_LDS_UNIFORM: hipLaunchKernelGGL(k_lds_read_probe<PQ_LDS_UNIFORM>, grid, block, 0, s, iters, (uint32_t *)sink); break;
        case PQ_LDS_LINEAR: hipLaunchKernelGGL(k_lds_read_probe<PQ_LDS_LINEAR>, grid, block, 0, s, iters, (uint32_t *)sink); break;
        case PQ_LDS_RANDOM_2K: hipLaunchKernelGGL(k_lds_read_probe<PQ_LDS_RANDOM_2K>, grid, block, 0, s, iters, (uint32_t *)sink); break;
        default: hipLaunchKernelGGL(k_lds_read_probe<PQ_LDS_RANDOM_128>, grid, block, 0, s, iters, (uint32_t *)sink); break;
    }
    QADC_LAUNCH_CHECK("k_lds_read_probe");
    return PQ_OK;
}
