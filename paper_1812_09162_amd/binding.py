"""Thin ctypes binding of libqadc.so: argument marshalling only.

Every function here has the name of the C entry point it forwards to (see
``include/qadc.h``).  PyTorch supplies device memory (``tensor.data_ptr()``) and
the stream; no step of the search path runs in Python or in PyTorch ops.  There
is no CPU fallback: if the library is missing or a call fails, an exception is
raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqadc.so")
_lib = None

PQ_OK, PQ_EINVAL, PQ_ENOMEM, PQ_EHIP = 0, -1, -2, -3
QPARAMS_BYTES = 24

EXPORTS = [
    "pq_index_create", "pq_index_destroy", "pq_code_size", "pq_table_len", "pq_workspace_bytes",
    "ivf_workspace_bytes", "ivf_sorted_workspace_bytes", "pq_compute_tables", "pq_quantize_tables", "pq_adc_scan_topk",
    "ivf_adc_scan_topk", "pq_search_workspace_bytes", "pq_search_topk",
    "pq_adc_scan_candidates", "pq_adc_rescan_candidates", "pq_select_topk", "pq_copy_bytes", "pq_last_error",
    "ivf_coarse_workspace_bytes", "ivf_coarse_search", "pq_encode", "pq_adc_scan_topk_static",
    "pq_set_option", "pq_get_option", "ivf_adc_scan_topk_tightening", "pq_lds_read_probe",
]
PQ_KEY_BOUND_UNKNOWN = 0xFFFFFFFF
(PQ_OPT_SCAN_BLOCKS, PQ_OPT_PILOT_CODES, PQ_OPT_PILOT_CODES_SINGLE, PQ_OPT_PILOT_BLOCKS, PQ_OPT_IVF_THREADS,
 PQ_OPT_SHARED_PASSES, PQ_OPT_COARSE_FILTER, PQ_OPT_IVF_SHARED_LISTS) = range(8)


class QadcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libqadc error {code}: {msg}")
        self.code = code


def load() -> ctypes.CDLL:
    """Load libqadc.so, building it first only if it was never built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
    lib.pq_index_create.argtypes = [ctypes.POINTER(vp), i32, i32, vp, vp, vp, i32]
    lib.pq_index_create.restype = i32
    lib.pq_index_destroy.argtypes = [vp]
    lib.pq_index_destroy.restype = None
    lib.pq_code_size.argtypes = [vp]
    lib.pq_code_size.restype = sz
    lib.pq_table_len.argtypes = [vp]
    lib.pq_table_len.restype = sz
    lib.pq_workspace_bytes.argtypes = [vp, i32, i64, i32]
    lib.pq_workspace_bytes.restype = sz
    lib.ivf_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.ivf_workspace_bytes.restype = sz
    lib.ivf_sorted_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    lib.ivf_sorted_workspace_bytes.restype = sz
    lib.pq_compute_tables.argtypes = [vp, vp, i32, vp, vp]
    lib.pq_compute_tables.restype = i32
    lib.pq_quantize_tables.argtypes = [vp, vp, i32, vp, i64, i32, i32, vp, vp, vp]
    lib.pq_quantize_tables.restype = i32
    lib.pq_adc_scan_topk.argtypes = [vp, vp, vp, i32, vp, i64, i32, vp, vp, vp, vp, sz, vp]
    lib.pq_adc_scan_topk.restype = i32
    lib.pq_adc_scan_topk_static.argtypes = [vp, vp, vp, i32, vp, i64, i32, vp, vp, vp, vp]
    lib.pq_adc_scan_topk_static.restype = i32
    lib.ivf_adc_scan_topk.argtypes = [vp, vp, i32, vp, vp, vp, vp, i32, vp, i32, i32, i32, vp, vp,
                                      vp, sz, vp]
    lib.ivf_adc_scan_topk.restype = i32
    lib.ivf_adc_scan_topk_tightening.argtypes = lib.ivf_adc_scan_topk.argtypes
    lib.ivf_adc_scan_topk_tightening.restype = i32
    lib.pq_lds_read_probe.argtypes = [i32, i32, vp, vp]
    lib.pq_lds_read_probe.restype = i32
    lib.pq_search_workspace_bytes.argtypes = [vp, i32, i64, i32]
    lib.pq_search_workspace_bytes.restype = sz
    lib.pq_search_topk.argtypes = [vp, vp, i32, vp, i64, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.pq_search_topk.restype = i32
    lib.pq_adc_scan_candidates.argtypes = [vp, vp, vp, i32, vp, i64, i32, vp, sz, vp]
    lib.pq_adc_scan_candidates.restype = i32
    lib.pq_adc_rescan_candidates.argtypes = [vp, vp, vp, i32, vp, i64, i32, vp, sz, vp]
    lib.pq_adc_rescan_candidates.restype = i32
    lib.pq_select_topk.argtypes = [vp, vp, vp, i32, vp, i64, i32, vp, vp, vp, vp, sz, vp]
    lib.pq_select_topk.restype = i32
    lib.pq_copy_bytes.argtypes = [vp, vp, sz, vp]
    lib.pq_copy_bytes.restype = i32
    lib.pq_set_option.argtypes = [i32, i64]
    lib.pq_set_option.restype = i32
    lib.pq_get_option.argtypes = [i32]
    lib.pq_get_option.restype = i64
    lib.pq_last_error.argtypes = []
    lib.pq_last_error.restype = ctypes.c_char_p
    lib.pq_encode.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    lib.pq_encode.restype = i32
    lib.ivf_coarse_workspace_bytes.argtypes = [i32, i32]
    lib.ivf_coarse_workspace_bytes.restype = sz
    lib.ivf_coarse_search.argtypes = [vp, i32, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.ivf_coarse_search.restype = i32
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != PQ_OK:
        raise QadcError(rc, load().pq_last_error().decode("utf-8", "replace"))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "libqadc needs contiguous tensors"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _dev(t: torch.Tensor, dtype) -> None:
    assert t.is_cuda and t.dtype == dtype, (t.device, t.dtype, dtype)


class PqIndex:
    """Owner of a ``pq_index_t*`` (pq_index_create / pq_index_destroy)."""

    def __init__(self, d: int, nbits: Sequence[int], dsub: Sequence[int], codebooks: torch.Tensor,
                 acc_bits: int):
        lib = load()
        _dev(codebooks, torch.float32)
        self.codebooks = codebooks.contiguous()  # the handle keeps this pointer
        nb = (ctypes.c_int32 * len(nbits))(*nbits)
        ds = (ctypes.c_int32 * len(dsub))(*dsub)
        h = ctypes.c_void_p()
        with torch.cuda.device(codebooks.device):
            _check(lib.pq_index_create(ctypes.byref(h), d, len(nbits), ctypes.cast(nb, ctypes.c_void_p),
                                       ctypes.cast(ds, ctypes.c_void_p), self.codebooks.data_ptr(),
                                       acc_bits))
        self.handle = h
        self.d, self.m, self.acc_bits = d, len(nbits), acc_bits
        self.nbits, self.dsub = list(nbits), list(dsub)
        self.code_size = int(lib.pq_code_size(h))
        self.table_len = int(lib.pq_table_len(h))
        self.q_max = (1 << acc_bits) - 1
        self.qdtype = torch.uint8 if acc_bits == 8 else torch.uint16
        self.device = codebooks.device

    def close(self) -> None:
        if getattr(self, "handle", None):
            load().pq_index_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pq_workspace_bytes(idx: PqIndex, nq: int, n: int, R: int) -> int:
    return int(load().pq_workspace_bytes(idx.handle, nq, n, R))


def ivf_workspace_bytes(idx: PqIndex, nq: int, nprobe: int, R: int) -> int:
    return int(load().ivf_workspace_bytes(idx.handle, nq, nprobe, R))


def ivf_sorted_workspace_bytes(idx: PqIndex, nq: int, nprobe: int, R: int, K: int) -> int:
    return int(load().ivf_sorted_workspace_bytes(idx.handle, nq, nprobe, R, K))


def pq_compute_tables(idx: PqIndex, queries: torch.Tensor, tables: Optional[torch.Tensor] = None,
                      stream=None) -> torch.Tensor:
    _dev(queries, torch.float32)
    nq = queries.shape[0]
    if tables is None:
        tables = torch.empty((nq, idx.table_len), dtype=torch.float32, device=queries.device)
    _check(load().pq_compute_tables(idx.handle, _ptr(queries), nq, _ptr(tables), _stream(stream)))
    return tables


def pq_quantize_tables(idx: PqIndex, tables: torch.Tensor, codes: torch.Tensor, t: int, R: int,
                       qtables: Optional[torch.Tensor] = None,
                       qparams: Optional[torch.Tensor] = None, stream=None
                       ) -> Tuple[torch.Tensor, torch.Tensor]:
    """qparams is a [nq, 24] uint8 tensor holding pq_qparams_t records."""
    _dev(tables, torch.float32)
    _dev(codes, torch.uint8)
    nq = tables.shape[0]
    if qtables is None:
        qtables = torch.empty((nq, idx.table_len), dtype=idx.qdtype, device=tables.device)
    if qparams is None:
        qparams = torch.empty((nq, QPARAMS_BYTES), dtype=torch.uint8, device=tables.device)
    _check(load().pq_quantize_tables(idx.handle, _ptr(tables), nq, _ptr(codes), codes.shape[0], t, R,
                                     _ptr(qtables), _ptr(qparams), _stream(stream)))
    return qtables, qparams


def pq_adc_scan_topk(idx: PqIndex, qtables: torch.Tensor, qparams: torch.Tensor,
                     codes: torch.Tensor, R: int, workspace: Optional[torch.Tensor] = None,
                     out=None, stream=None):
    _dev(codes, torch.uint8)
    nq, n = qtables.shape[0], codes.shape[0]
    dev = codes.device
    if workspace is None:
        workspace = torch.empty(pq_workspace_bytes(idx, nq, n, R), dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty((nq, R), dtype=torch.int32, device=dev),
               torch.empty((nq, R), dtype=torch.uint16, device=dev),
               torch.empty((nq, R), dtype=torch.float32, device=dev))
    ids, keys, dist = out
    _check(load().pq_adc_scan_topk(idx.handle, _ptr(qtables), _ptr(qparams), nq, _ptr(codes), n, R,
                                   _ptr(ids), _ptr(keys), _ptr(dist), _ptr(workspace),
                                   workspace.numel(), _stream(stream)))
    return ids, keys, dist


def pq_adc_scan_topk_static(idx: PqIndex, qtables: torch.Tensor, qparams: torch.Tensor,
                            codes: torch.Tensor, R: int, out, stream=None):
    """The caller passes inputs and outputs; the library's own scratch array is the workspace."""
    _dev(codes, torch.uint8)
    ids, keys, dist = out
    _check(load().pq_adc_scan_topk_static(idx.handle, _ptr(qtables), _ptr(qparams), qtables.shape[0],
                                          _ptr(codes), codes.shape[0], R, _ptr(ids), _ptr(keys),
                                          _ptr(dist), _stream(stream)))
    return ids, keys, dist


def pq_search_workspace_bytes(idx: PqIndex, nq: int, n: int, R: int) -> int:
    return int(load().pq_search_workspace_bytes(idx.handle, nq, n, R))


def pq_search_topk(idx: PqIndex, queries: torch.Tensor, codes: torch.Tensor, t: int, R: int,
                   workspace: Optional[torch.Tensor] = None, out=None, stream=None):
    _dev(queries, torch.float32)
    _dev(codes, torch.uint8)
    nq, n = queries.shape[0], codes.shape[0]
    dev = codes.device
    if workspace is None:
        workspace = torch.empty(pq_search_workspace_bytes(idx, nq, n, R), dtype=torch.uint8,
                                device=dev)
    if out is None:
        out = (torch.empty((nq, R), dtype=torch.int32, device=dev),
               torch.empty((nq, R), dtype=torch.uint16, device=dev),
               torch.empty((nq, R), dtype=torch.float32, device=dev))
    ids, keys, dist = out
    _check(load().pq_search_topk(idx.handle, _ptr(queries), nq, _ptr(codes), n, t, R, _ptr(ids),
                                 _ptr(keys), _ptr(dist), _ptr(workspace), workspace.numel(),
                                 _stream(stream)))
    return ids, keys, dist


def ivf_adc_scan_topk(idx: PqIndex, coarse: torch.Tensor, list_offsets: torch.Tensor,
                      list_codes: torch.Tensor, list_ids: torch.Tensor, queries: torch.Tensor,
                      probe_ids: torch.Tensor, t: int, R: int,
                      workspace: Optional[torch.Tensor] = None, out=None, stream=None):
    _dev(coarse, torch.float32)
    _dev(list_offsets, torch.int64)
    _dev(list_codes, torch.uint8)
    _dev(list_ids, torch.int32)
    _dev(queries, torch.float32)
    _dev(probe_ids, torch.int32)
    nq, nprobe = probe_ids.shape
    dev = queries.device
    if workspace is None:
        workspace = torch.empty(ivf_sorted_workspace_bytes(idx, nq, nprobe, R, coarse.shape[0]),
                                dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty((nq, R), dtype=torch.int32, device=dev),
               torch.empty((nq, R), dtype=torch.float32, device=dev))
    ids, dist = out
    _check(load().ivf_adc_scan_topk(idx.handle, _ptr(coarse), coarse.shape[0], _ptr(list_offsets),
                                    _ptr(list_codes), _ptr(list_ids), _ptr(queries), nq,
                                    _ptr(probe_ids), nprobe, t, R, _ptr(ids), _ptr(dist),
                                    _ptr(workspace), workspace.numel(), _stream(stream)))
    return ids, dist


def ivf_adc_scan_topk_tightening(idx: PqIndex, coarse: torch.Tensor, list_offsets: torch.Tensor,
                                 list_codes: torch.Tensor, list_ids: torch.Tensor, queries: torch.Tensor,
                                 probe_ids: torch.Tensor, t: int, R: int,
                                 workspace: Optional[torch.Tensor] = None, out=None, stream=None):
    _dev(coarse, torch.float32)
    _dev(list_offsets, torch.int64)
    _dev(list_codes, torch.uint8)
    _dev(list_ids, torch.int32)
    _dev(queries, torch.float32)
    _dev(probe_ids, torch.int32)
    nq, nprobe = probe_ids.shape
    dev = queries.device
    if workspace is None:
        workspace = torch.empty(ivf_workspace_bytes(idx, nq, nprobe, R), dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty((nq, R), dtype=torch.int32, device=dev),
               torch.empty((nq, R), dtype=torch.float32, device=dev))
    ids, dist = out
    _check(load().ivf_adc_scan_topk_tightening(idx.handle, _ptr(coarse), coarse.shape[0], _ptr(list_offsets),
                                               _ptr(list_codes), _ptr(list_ids), _ptr(queries), nq,
                                               _ptr(probe_ids), nprobe, t, R, _ptr(ids), _ptr(dist),
                                               _ptr(workspace), workspace.numel(), _stream(stream)))
    return ids, dist


def pq_adc_scan_candidates(idx: PqIndex, qtables: torch.Tensor, qparams: torch.Tensor,
                           codes: torch.Tensor, R: int, workspace: torch.Tensor, stream=None) -> None:
    _dev(codes, torch.uint8)
    _check(load().pq_adc_scan_candidates(idx.handle, _ptr(qtables), _ptr(qparams), qtables.shape[0],
                                         _ptr(codes), codes.shape[0], R, _ptr(workspace),
                                         workspace.numel(), _stream(stream)))


def pq_adc_rescan_candidates(idx: PqIndex, qtables: torch.Tensor, qparams: torch.Tensor,
                             codes: torch.Tensor, R: int, workspace: torch.Tensor, stream=None) -> None:
    _dev(codes, torch.uint8)
    _check(load().pq_adc_rescan_candidates(idx.handle, _ptr(qtables), _ptr(qparams),
                                           qtables.shape[0], _ptr(codes), codes.shape[0], R,
                                           _ptr(workspace), workspace.numel(), _stream(stream)))


def pq_select_topk(idx: PqIndex, qtables: torch.Tensor, qparams: torch.Tensor, codes: torch.Tensor,
                   R: int, workspace: torch.Tensor, out=None, stream=None):
    _dev(codes, torch.uint8)
    nq, dev = qtables.shape[0], codes.device
    if out is None:
        out = (torch.empty((nq, R), dtype=torch.int32, device=dev),
               torch.empty((nq, R), dtype=torch.uint16, device=dev),
               torch.empty((nq, R), dtype=torch.float32, device=dev))
    ids, keys, dist = out
    _check(load().pq_select_topk(idx.handle, _ptr(qtables), _ptr(qparams), nq, _ptr(codes),
                                 codes.shape[0], R, _ptr(ids), _ptr(keys), _ptr(dist),
                                 _ptr(workspace), workspace.numel(), _stream(stream)))
    return ids, keys, dist


def pq_copy_bytes(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(load().pq_copy_bytes(_ptr(dst), _ptr(src), nbytes, _stream(stream)))


PQ_LDS_UNIFORM, PQ_LDS_LINEAR, PQ_LDS_RANDOM_2K, PQ_LDS_RANDOM_128 = range(4)
PQ_LDS_PROBE_BLOCKS = 2048


def pq_lds_read_probe(pattern: int, iters: int, sink: torch.Tensor, stream=None) -> int:
    """Launches the probe; returns the number of 8-byte lane reads it performs."""
    _dev(sink, torch.int32)
    _check(load().pq_lds_read_probe(pattern, iters, _ptr(sink), _stream(stream)))
    return PQ_LDS_PROBE_BLOCKS * 256 * 8 * iters


def pq_set_option(option: int, value: int) -> None:
    _check(load().pq_set_option(option, value))


def pq_get_option(option: int) -> int:
    return int(load().pq_get_option(option))


def unpack_qparams(qparams: torch.Tensor):
    """[nq,24] uint8 -> dict of numpy arrays (d_min, delta, d_max, key_bound)."""
    import numpy as np
    raw = qparams.detach().cpu().numpy()
    rec = np.dtype([("d_min", "<f8"), ("delta", "<f8"), ("d_max", "<f4"), ("key_bound", "<u4")])
    return raw.view(rec).reshape(-1)


def ivf_coarse_workspace_bytes(nq: int, K: int) -> int:
    return int(load().ivf_coarse_workspace_bytes(nq, K))


def ivf_coarse_search(queries: torch.Tensor, centroids: torch.Tensor, nprobe: int,
                      workspace: Optional[torch.Tensor] = None, out=None, want_scores: bool = True,
                      stream=None):
    """Returns (probe_ids [nq, nprobe] int32, probe_scores [nq, nprobe] float32 or None)."""
    _dev(queries, torch.float32)
    _dev(centroids, torch.float32)
    nq, d = queries.shape
    K = centroids.shape[0]
    assert centroids.shape[1] == d
    dev = queries.device
    if workspace is None:
        workspace = torch.empty(ivf_coarse_workspace_bytes(nq, K), dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty((nq, nprobe), dtype=torch.int32, device=dev),
               torch.empty((nq, nprobe), dtype=torch.float32, device=dev) if want_scores else None)
    ids, sc = out
    _check(load().ivf_coarse_search(_ptr(queries), nq, _ptr(centroids), K, d, nprobe, _ptr(ids),
                                    _ptr(sc) if sc is not None else None, _ptr(workspace),
                                    workspace.numel(), _stream(stream)))
    return ids, sc


def pq_encode(idx: PqIndex, vectors: torch.Tensor, shift_rows: Optional[torch.Tensor] = None,
              shift_ids: Optional[torch.Tensor] = None, codes: Optional[torch.Tensor] = None,
              stream=None) -> torch.Tensor:
    """Packed codes [n, code_size] uint8 of vectors [n, d] (minus shift_rows[shift_ids], if given)."""
    _dev(vectors, torch.float32)
    if shift_rows is not None:
        _dev(shift_rows, torch.float32)
        _dev(shift_ids, torch.int32)
    n = vectors.shape[0]
    if codes is None:
        codes = torch.empty((n, idx.code_size), dtype=torch.uint8, device=vectors.device)
    _check(load().pq_encode(idx.handle, _ptr(vectors), n, _ptr(shift_rows), _ptr(shift_ids),
                            _ptr(codes), _stream(stream)))
    return codes
