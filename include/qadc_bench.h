/*
 * qadc_bench.h -- entry points of libqadc that exist for measurement only.  They are not
 * part of the search interface (qadc.h) and a caller of the library never needs them.
 */
#ifndef QADC_BENCH_H
#define QADC_BENCH_H

#include "qadc.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The scan kernel of pq_adc_scan_topk alone (eq. (2), Section 3.4 saturating sums), with the
 * tables that a previous pq_adc_scan_candidates call on the same workspace and the same
 * qtables prepared.  Same arguments as pq_adc_scan_candidates.  Benchmarks launch it back to
 * back to time that kernel by itself; the candidate lists in the workspace keep growing from
 * launch to launch (entries beyond their capacity are dropped), so no result may be read
 * from the workspace afterwards.
 */
int pq_adc_rescan_candidates(const pq_index_t *idx, const void *qtables,
                             const pq_qparams_t *qparams, int nq, const uint8_t *codes, int64_t n,
                             int R, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Plain device-to-device copy by a library kernel (k_copy) whose traffic is known exactly:
 * nbytes read and nbytes written.  For scaling hardware-counter readings (rocprofv3
 * FETCH_SIZE / WRITE_SIZE) taken in the same run as the scan kernel.
 * dst, src [dev], 16-byte aligned, non-overlapping; nbytes a multiple of 16.
 */
int pq_copy_bytes(void *dst, const void *src, size_t nbytes, void *stream);

/*
 * The rate at which this GPU serves 8-byte LDS reads (ds_read_b64) for an address pattern:
 * launches PQ_LDS_PROBE_BLOCKS blocks of 256 threads in which every lane reads 8 * iters entries
 * of eight 2 KB tables (the shape of the interleaved group tables of the batched scan, Section
 * 3.4 tables for four queries side by side).  The caller times the launch; the number of lane
 * reads is PQ_LDS_PROBE_BLOCKS * 256 * 8 * iters.  PQ_LDS_RANDOM_2K is the batched scan's own
 * pattern (every lane an independent entry of a 256-entry table), PQ_LDS_LINEAR is free of bank
 * conflicts.  sink: [dev] one 32-bit word the kernel may write.
 */
enum { PQ_LDS_UNIFORM = 0, PQ_LDS_LINEAR = 1, PQ_LDS_RANDOM_2K = 2, PQ_LDS_RANDOM_128 = 3 };
#define PQ_LDS_PROBE_BLOCKS 2048
int pq_lds_read_probe(int pattern, int iters, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QADC_BENCH_H */
