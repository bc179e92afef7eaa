// Internal declarations shared by the translation units of libqadc.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qadc.h"
#include "qadc_bench.h"

// Layout of a product quantizer as the kernels see it.  A copy lives in device
// memory; kernels read it through uniform (scalar) loads.
//
// Sub-quantizers are additionally partitioned into consecutive *groups* of at
// most 12 code bits.  The scan looks up one pre-summed, pre-saturated entry per
// group instead of one entry per sub-quantizer: because every addend is
// non-negative, min(q_max, a+b+c+...) equals the saturating chain of Section
// 3.4 no matter how the addends are bracketed.  For m x 4 layouts a group is
// one code byte (two nibbles, 256 entries).
struct DevLayout {
    int32_t d, m, T, cs, acc_bits, qmax, code_bits;
    int32_t ng;        // number of groups
    int32_t gtab_len;  // total group-table entries
    int32_t kind;      // SCAN_* below
    int32_t g32ok;     // 1 if no group field crosses a 32-bit boundary of the code
    int32_t ds_uniform;  // the sub-space width if all sub-quantizers share one (at most 8), else 0
    // all 32-bit so that uniform reads compile to scalar loads (gfx9 has no
    // sub-dword scalar loads)
    int32_t nbits[PQ_MAX_M];
    int32_t bitoff[PQ_MAX_M];  // first code bit of sub-quantizer j
    int32_t toff[PQ_MAX_M];    // first table entry of sub-quantizer j
    int32_t dimoff[PQ_MAX_M];  // first vector dimension of sub-quantizer j
    int32_t dsub[PQ_MAX_M];
    int32_t cboff[PQ_MAX_M];   // first codebook float of sub-quantizer j
    int32_t gw[PQ_MAX_M];      // bits of group g
    int32_t goff[PQ_MAX_M];    // first code bit of group g
    int32_t gfirst[PQ_MAX_M];  // first sub-quantizer of group g
    int32_t gcount[PQ_MAX_M];  // sub-quantizers in group g
    int32_t gbase[PQ_MAX_M];   // first group-table entry of group g
};

// Scan specialisations by code shape:
//   NIB8 / NIB16  16 or 32 four-bit sub-quantizers (64- / 128-bit codes): one group per byte
//   W64           any other 8-byte code: group fields cut out of one 64-bit word
//   C5            5-byte codes (33..40 bits): four codes per lane from five dwords
//   GENERIC       everything else, byte by byte
enum { SCAN_GENERIC = 0, SCAN_NIB8 = 1, SCAN_NIB16 = 2, SCAN_C5 = 3, SCAN_W64 = 4, SCAN_W128 = 5 };

// One table entry: its sub-quantizer, where its centroid starts in the codebook array (in
// floats), the first dimension of its sub-space and that sub-space's width.
struct EntryDesc {
    int32_t j, cb_off, dim_off, ds;
};

struct pq_index {
    DevLayout h;          // host copy
    DevLayout *dev;       // device copy; T EntryDesc records follow it in the same allocation
    const EntryDesc *edesc;  // device
    const float *codebooks;
    int device;
};

// Per-query state of the inverted-list search.
struct IvfState {
    float dmax;        // calibration bound (Section 3.4) shared by the probed lists
    float thr0;        // bound on a result's distance: R-th smallest among the pilot codes
    float lo, scale;   // bin(dist) = min(255, (dist - lo) * scale), 0 below lo
};

struct IvfPlan {
    int cap_b;         // candidate slots per (query, probe)
    size_t per_query;  // bytes per query
    size_t counts_off, slots_off;
    size_t total;
};
IvfPlan qadc_ivf_plan(const pq_index *idx, int nq, int nprobe, int R);

struct ScanPlan {
    int G;             // blocks per query in the scan kernel
    uint32_t cap;      // entries of each of a query's candidate lists
    size_t per_query;  // bytes per query: header | prepared group tables | candidate lists
    size_t gtab_off;   // prepared group tables of the query (gtab_len entries)
    size_t cand_off;   // candidate lists (QADC_NSUB x cap 64-bit entries)
    size_t total;
};

void qadc_set_error(const char *fmt, ...);
// Current value of a tuning option (PQ_OPT_*), set through pq_set_option.
int64_t qadc_option(int option);
ScanPlan qadc_scan_plan(const pq_index *idx, int nq, int64_t n, int R);

// Pilot of the distance quantizer: `pilot` codes, counted by P blocks per query, `slice` each.
struct PilotPlan {
    int pilot, P, slice;
};
int qadc_pilot_blocks_max(int nq);
size_t qadc_pilot_scratch_bytes(int nq);
PilotPlan qadc_pilot_plan(int nq, int64_t n, int t_eff, int R, bool have_scratch, bool cheap_lookups);

// gtab_out: if non-null, query q's group tables are also written to gtab_out + q*gtab_stride bytes.
// hdr_out: if non-null, the scan header at hdr_out + q*gtab_stride is cleared (an empty candidate list).
// scratch: null, or qadc_pilot_scratch_bytes(nq) bytes (256-byte aligned, any contents) that let
// several blocks share a query's pilot (they leave their records there).  plan_used: if non-null, receives the pilot plan.
int qadc_quantize_launch(const pq_index *idx, const float *queries, const float *tables_in,
                         float *tables_out, int nq, const uint8_t *codes, int64_t n, int t, int R,
                         void *qtables, pq_qparams_t *qparams, char *gtab_out, size_t gtab_stride,
                         char *hdr_out, char *scratch, PilotPlan *plan_used, hipStream_t s);


#define QADC_HIP_TRY(expr)                                                        \
    do {                                                                          \
        hipError_t e__ = (expr);                                                  \
        if (e__ != hipSuccess) {                                                  \
            qadc_set_error("%s failed: %s", #expr, hipGetErrorString(e__));       \
            return PQ_EHIP;                                                       \
        }                                                                         \
    } while (0)

#define QADC_LAUNCH_CHECK(what)                                                   \
    do {                                                                          \
        hipError_t e__ = hipGetLastError();                                       \
        if (e__ != hipSuccess) {                                                  \
            qadc_set_error("launch of %s failed: %s", what, hipGetErrorString(e__)); \
            return PQ_EHIP;                                                       \
        }                                                                         \
    } while (0)
