"""ctypes front end of the CPU oracle (``adc_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The product package never imports this.
Everything here is argument marshalling around the C functions; the arithmetic
lives in ``adc_oracle.c``, which cites the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adc_oracle.c")
_LIB = os.path.join(_HERE, "libadc_oracle.so")
_lib = None

CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-Wall"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_t_eff.restype = ctypes.c_int64
        _lib.oracle_t_eff.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _f32(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.float32))


def _u8(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.uint8))


def code_size(nbits: Sequence[int]) -> int:
    nb = _i32(nbits)
    return int(_load().oracle_code_size(len(nb), _p(nb)))


def table_len(nbits: Sequence[int]) -> int:
    nb = _i32(nbits)
    return int(_load().oracle_table_len(len(nb), _p(nb)))


def t_eff(n: int, t: int, R: int) -> int:
    return int(_load().oracle_t_eff(int(n), int(t), int(R)))


def unpack(nbits, codes) -> np.ndarray:
    nb, codes = _i32(nbits), _u8(codes)
    n = codes.shape[0]
    sub = np.empty((n, len(nb)), dtype=np.uint8)
    _load().oracle_unpack(len(nb), _p(nb), _p(codes), ctypes.c_int64(n), _p(sub))
    return sub


def tables(d, nbits, dsub, codebooks, z, shift=None) -> np.ndarray:
    """O1 for one query vector z (optionally minus ``shift``): [T] float32."""
    nb, ds, cb, z = _i32(nbits), _i32(dsub), _f32(codebooks), _f32(z)
    sh = None if shift is None else _f32(shift)
    out = np.empty(table_len(nb), dtype=np.float32)
    _load().oracle_tables(int(d), len(nb), _p(nb), _p(ds), _p(cb), _p(z), _p(sh), _p(out))
    return out


def adc_float(nbits, table, codes) -> np.ndarray:
    """eq. (2) with the float table, fp32, for every code: [n] float32."""
    nb, table, codes = _i32(nbits), _f32(table), _u8(codes)
    n = codes.shape[0]
    out = np.empty(n, dtype=np.float32)
    _load().oracle_adc_float(len(nb), _p(nb), _p(table), _p(codes), ctypes.c_int64(n), _p(out))
    return out


def quantize(nbits, acc_bits, table, codes, t, R) -> Tuple[np.ndarray, float, float, float]:
    """O2+O3: (qtable[T] uint16, d_min, delta, d_max)."""
    nb, table, codes = _i32(nbits), _f32(table), _u8(codes)
    n = codes.shape[0]
    qt = np.empty(table.shape[0], dtype=np.uint16)
    prm = np.empty(3, dtype=np.float64)
    _load().oracle_quantize(len(nb), _p(nb), int(acc_bits), _p(table), _p(codes),
                            ctypes.c_int64(n), int(t), int(R), _p(qt), _p(prm))
    return qt, float(prm[0]), float(prm[1]), float(prm[2])


def scan_keys(nbits, acc_bits, qtable, codes) -> np.ndarray:
    """O4: [n] uint16 keys."""
    nb, codes = _i32(nbits), _u8(codes)
    qt = np.ascontiguousarray(np.asarray(qtable, dtype=np.uint16))
    n = codes.shape[0]
    keys = np.empty(n, dtype=np.uint16)
    _load().oracle_scan_keys(len(nb), _p(nb), int(acc_bits), _p(qt), _p(codes),
                             ctypes.c_int64(n), _p(keys))
    return keys


def topk(acc_bits, keys, R, d_min, delta):
    """O5: (ids[R] int32, keys[R] uint16, dist[R] float32)."""
    keys = np.ascontiguousarray(np.asarray(keys, dtype=np.uint16))
    ids = np.empty(R, dtype=np.int32)
    ok = np.empty(R, dtype=np.uint16)
    od = np.empty(R, dtype=np.float32)
    _load().oracle_topk(int(acc_bits), _p(keys), ctypes.c_int64(keys.shape[0]), int(R),
                        ctypes.c_double(d_min), ctypes.c_double(delta), _p(ids), _p(ok), _p(od))
    return ids, ok, od


def search(d, nbits, dsub, acc_bits, codebooks, z, codes, t, R):
    """O1..O5 for one query: (ids, keys, dist)."""
    nb, ds, cb, z, codes = _i32(nbits), _i32(dsub), _f32(codebooks), _f32(z), _u8(codes)
    n = codes.shape[0]
    ids = np.empty(R, dtype=np.int32)
    ok = np.empty(R, dtype=np.uint16)
    od = np.empty(R, dtype=np.float32)
    _load().oracle_search(int(d), len(nb), _p(nb), _p(ds), int(acc_bits), _p(cb), _p(z),
                          _p(codes), ctypes.c_int64(n), int(t), int(R), _p(ids), _p(ok), _p(od))
    return ids, ok, od


def search_ivf(d, nbits, dsub, acc_bits, codebooks, coarse, list_offsets, list_codes, list_ids,
               z, probe, t, R):
    """O6 for one query: (ids[R], dist[R], d_max)."""
    nb, ds, cb, z = _i32(nbits), _i32(dsub), _f32(codebooks), _f32(z)
    coarse = _f32(coarse)
    lo = np.ascontiguousarray(np.asarray(list_offsets, dtype=np.int64))
    lc, li, pr = _u8(list_codes), _i32(list_ids), _i32(probe)
    ids = np.empty(R, dtype=np.int32)
    od = np.empty(R, dtype=np.float32)
    dmax = np.empty(1, dtype=np.float32)
    _load().oracle_search_ivf(int(d), len(nb), _p(nb), _p(ds), int(acc_bits), _p(cb), _p(coarse),
                              _p(lo), _p(lc), _p(li), _p(z), _p(pr), int(pr.shape[0]), int(t),
                              int(R), _p(ids), _p(od), _p(dmax))
    return ids, od, float(dmax[0])


def search_ivf_tightening(d, nbits, dsub, acc_bits, codebooks, coarse, list_offsets, list_codes, list_ids,
                          z, probe, t, R):
    """O6b for one query: (ids[R], dist[R], d_max, bounds[nprobe])."""
    nb, ds, cb, z = _i32(nbits), _i32(dsub), _f32(codebooks), _f32(z)
    coarse = _f32(coarse)
    lo = np.ascontiguousarray(np.asarray(list_offsets, dtype=np.int64))
    lc, li, pr = _u8(list_codes), _i32(list_ids), _i32(probe)
    ids = np.empty(R, dtype=np.int32)
    od = np.empty(R, dtype=np.float32)
    dmax = np.empty(1, dtype=np.float32)
    bounds = np.empty(pr.shape[0], dtype=np.float32)
    _load().oracle_search_ivf_tightening(int(d), len(nb), _p(nb), _p(ds), int(acc_bits), _p(cb), _p(coarse),
                                         _p(lo), _p(lc), _p(li), _p(z), _p(pr), int(pr.shape[0]), int(t),
                                         int(R), _p(ids), _p(od), _p(dmax), _p(bounds))
    return ids, od, float(dmax[0]), bounds


def coarse_search(centroids, z, nprobe):
    """O7 for one query: (ids[nprobe], scores[nprobe]) of the nearest cells."""
    cen, z = _f32(centroids), _f32(z)
    K, d = cen.shape
    ids = np.empty(nprobe, dtype=np.int32)
    sc = np.empty(nprobe, dtype=np.float32)
    _load().oracle_coarse_search(int(d), ctypes.c_int64(K), _p(cen), _p(z), int(nprobe), _p(ids), _p(sc))
    return ids, sc


def encode(d, nbits, dsub, codebooks, x, shift=None) -> np.ndarray:
    """O8: packed codes [n, code_size] of the vectors x [n, d] (minus shift [n, d], if given)."""
    nb, ds, cb, x = _i32(nbits), _i32(dsub), _f32(codebooks), _f32(x)
    sh = _f32(shift) if shift is not None else None
    n = x.shape[0]
    codes = np.empty((n, code_size(nbits)), dtype=np.uint8)
    _load().oracle_encode(int(d), len(nb), _p(nb), _p(ds), _p(cb), _p(x), _p(sh), ctypes.c_int64(n),
                          _p(codes))
    return codes
