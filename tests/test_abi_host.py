"""CPU-side checks of the C-ABI library: it loads, exports every function that
include/qadc.h declares, and rejects bad arguments with an error code and a message
(no compute call is made here: there is no GPU in this tier)."""
import ctypes
import os
import re

import pytest

from paper_1812_09162_amd import binding as qb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("qadc.h", "qadc_bench.h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:pq|ivf)_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = qb.load()
    names = declared_functions()
    assert len(names) >= 13
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(qb.EXPORTS)


def test_qparams_record_is_24_bytes():
    import numpy as np
    rec = np.dtype([("d_min", "<f8"), ("delta", "<f8"), ("d_max", "<f4"), ("key_bound", "<u4")])
    assert rec.itemsize == qb.QPARAMS_BYTES


def test_index_create_rejects_bad_shapes_before_touching_the_gpu():
    lib = qb.load()
    h = ctypes.c_void_p()

    def create(d, nbits, dsub, acc, cb=0x1000):
        nb = (ctypes.c_int32 * len(nbits))(*nbits)
        ds = (ctypes.c_int32 * len(dsub))(*dsub)
        return lib.pq_index_create(ctypes.byref(h), d, len(nbits), ctypes.cast(nb, ctypes.c_void_p),
                                   ctypes.cast(ds, ctypes.c_void_p), cb, acc)

    assert create(8, [4, 4], [4, 4], 12) == qb.PQ_EINVAL          # acc_bits
    assert b"acc_bits" in lib.pq_last_error()
    assert create(8, [4, 9], [4, 4], 8) == qb.PQ_EINVAL           # nbits out of range
    assert create(8, [4, 4], [4, 3], 8) == qb.PQ_EINVAL           # sum(dsub) != d
    assert b"sum(dsub)" in lib.pq_last_error()
    assert create(8, [4, 4], [8, 0], 8) == qb.PQ_EINVAL           # empty sub-vector
    assert create(8, [4, 4], [4, 4], 8, cb=None) == qb.PQ_EINVAL  # null codebooks
    assert create(0, [4], [0], 8) == qb.PQ_EINVAL
    assert create(17 * 8, [8] * 17, [8] * 17, 8) == qb.PQ_EINVAL  # table longer than the limit
    assert h.value is None


def test_options_are_validated_and_kept():
    lib = qb.load()
    assert lib.pq_get_option(qb.PQ_OPT_SCAN_BLOCKS) == 2048
    assert lib.pq_set_option(qb.PQ_OPT_SCAN_BLOCKS, 0) == qb.PQ_EINVAL       # out of range: unchanged
    assert lib.pq_set_option(qb.PQ_OPT_IVF_THREADS, 100) == qb.PQ_EINVAL
    assert lib.pq_set_option(qb.PQ_OPT_IVF_SHARED_LISTS, 3) == qb.PQ_EINVAL
    assert lib.pq_get_option(qb.PQ_OPT_IVF_SHARED_LISTS) == 1
    assert lib.pq_set_option(99, 1) == qb.PQ_EINVAL and b"option 99" in lib.pq_last_error()
    assert lib.pq_get_option(99) == -1
    assert lib.pq_set_option(qb.PQ_OPT_SCAN_BLOCKS, 1024) == qb.PQ_OK
    assert lib.pq_get_option(qb.PQ_OPT_SCAN_BLOCKS) == 1024
    assert lib.pq_set_option(qb.PQ_OPT_SCAN_BLOCKS, 2048) == qb.PQ_OK


def test_calls_reject_null_handle():
    lib = qb.load()
    assert lib.pq_compute_tables(None, None, 1, None, None) == qb.PQ_EINVAL
    assert lib.pq_quantize_tables(None, None, 1, None, 0, 400, 10, None, None, None) == qb.PQ_EINVAL
    assert lib.pq_adc_scan_topk(None, None, None, 1, None, 0, 10, None, None, None, None, 0,
                                None) == qb.PQ_EINVAL
    assert lib.ivf_adc_scan_topk(None, None, 1, None, None, None, None, 1, None, 1, 400, 10, None,
                                 None, None, 0, None) == qb.PQ_EINVAL
    assert lib.ivf_adc_scan_topk_tightening(None, None, 1, None, None, None, None, 1, None, 1, 400, 10,
                                            None, None, None, 0, None) == qb.PQ_EINVAL
    assert b"ivf_adc_scan_topk_tightening" in lib.pq_last_error()
    assert lib.pq_code_size(None) == 0 and lib.pq_table_len(None) == 0
    assert lib.pq_workspace_bytes(None, 1, 10, 10) == 0
    lib.pq_index_destroy(None)
