"""Seeded synthetic inputs for the ADC-scan path: vectors, codebooks, codes, lists.

This module only *fabricates inputs* (vectors, k-means codebooks, encoded and
bit-packed short codes, inverted lists).  None of the search path's arithmetic
lives here: no distance tables, no distance quantizer, no scan, no top-R.  Both
the CPU oracle's tests and the HIP path's tests draw their inputs from here, so
the two are always fed identical bytes.

The public datasets the paper evaluates on (Section 4: SIFT1M, Deep1M,
SIFT1000M, Deep1B) are not available; the generators below only mirror their
shapes and value ranges:

* ``gamma_ints``  : non-negative byte-range integers stored as float32, heavy
  tailed with about 40 % zeros (stand-in for 128-d SIFT-like descriptors).
* ``aniso_gauss`` : Gaussian with per-dimension variance 1/(1+i/8), then
  L2-normalised (stand-in for 96-d deep descriptors).

Training and encoding follow Section 2.1.2 (nearest-centroid vector quantizers
per sub-space, code = concatenation of sub-codes); packing follows Section 3.3
(sub-code 0 in the low bits, little-endian bit stream).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np
import torch

GAMMA_THETA = 7.27  # P(value == 0) = erf(sqrt(1/theta)) ~= 0.40
CHUNK_ROWS = 1 << 20  # generation granularity: chunk c uses seed stream (seed, c)


# --------------------------------------------------------------------------
# raw vectors
# --------------------------------------------------------------------------
def _gen(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(stream) * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    return g


def gamma_ints(n: int, d: int, seed: int, device="cpu") -> torch.Tensor:
    """[n,d] float32 holding integers min(255, floor(Gamma(shape 0.5, scale theta))).

    Gamma(0.5, theta) is theta/2 times the square of a standard normal, which
    keeps the generator a pure function of torch's seeded normal stream.
    """
    out = torch.empty((n, d), dtype=torch.float32, device=device)
    for c, lo in enumerate(range(0, n, CHUNK_ROWS)):
        hi = min(n, lo + CHUNK_ROWS)
        z = torch.randn((hi - lo, d), generator=_gen(seed, c, device), device=device,
                        dtype=torch.float32)
        out[lo:hi] = torch.clamp(torch.floor(z * z * (GAMMA_THETA / 2.0)), max=255.0)
    return out


def aniso_gauss(n: int, d: int, seed: int, device="cpu") -> torch.Tensor:
    """[n,d] float32: N(0, 1/(1+i/8)) per dimension i, rows L2-normalised."""
    scale = torch.rsqrt(1.0 + torch.arange(d, dtype=torch.float32, device=device) / 8.0)
    out = torch.empty((n, d), dtype=torch.float32, device=device)
    for c, lo in enumerate(range(0, n, CHUNK_ROWS)):
        hi = min(n, lo + CHUNK_ROWS)
        z = torch.randn((hi - lo, d), generator=_gen(seed, c, device), device=device,
                        dtype=torch.float32) * scale
        out[lo:hi] = z / z.norm(dim=1, keepdim=True).clamp_min(1e-20)
    return out


GENERATORS = {"gamma_ints": gamma_ints, "aniso_gauss": aniso_gauss}


# --------------------------------------------------------------------------
# layout helpers (Section 3.1: dimensions are allotted in proportion to bits)
# --------------------------------------------------------------------------
def dim_split(d: int, nbits: Sequence[int]) -> List[int]:
    """floor(d*b_j/B) dims for sub-quantizer j, leftovers handed out one by one
    to sub-quantizers 0,1,... (Section 3.1, last paragraph before the results)."""
    B = sum(nbits)
    ds = [(d * b) // B for b in nbits]
    j = 0
    while sum(ds) < d:
        ds[j % len(ds)] += 1
        j += 1
    assert sum(ds) == d and min(ds) >= 1, (d, nbits, ds)
    return ds


@dataclass
class Layout:
    """Runtime description of a (possibly irregular) product quantizer."""
    d: int
    nbits: List[int]
    dsub: List[int]
    acc_bits: int = 8  # width of quantized table entries and of the accumulator

    @property
    def m(self) -> int:
        return len(self.nbits)

    @property
    def ksub(self) -> List[int]:
        return [1 << b for b in self.nbits]

    @property
    def table_len(self) -> int:
        return sum(self.ksub)

    @property
    def code_bits(self) -> int:
        return sum(self.nbits)

    @property
    def code_size(self) -> int:
        return (self.code_bits + 7) // 8

    @property
    def codebook_len(self) -> int:
        return sum(k * s for k, s in zip(self.ksub, self.dsub))

    @property
    def q_max(self) -> int:
        return (1 << self.acc_bits) - 1


def make_layout(d: int, nbits: Sequence[int], acc_bits: int = 8) -> Layout:
    return Layout(d=d, nbits=list(nbits), dsub=dim_split(d, nbits), acc_bits=acc_bits)


# --------------------------------------------------------------------------
# k-means (Lloyd), encoder, packer  -- harness only
# --------------------------------------------------------------------------
def _assign(x: torch.Tensor, c: torch.Tensor, chunk: int = 1 << 16) -> torch.Tensor:
    """index of the nearest row of c for every row of x (ties -> lowest index)."""
    chunk = max(1, min(chunk, (1 << 28) // max(1, c.shape[0])))  # distance block <= 1 GiB
    out = torch.empty(x.shape[0], dtype=torch.int64, device=x.device)
    cn = (c * c).sum(1)
    for lo in range(0, x.shape[0], chunk):
        xb = x[lo:lo + chunk]
        dist = cn[None, :] - 2.0 * (xb @ c.t())
        out[lo:lo + chunk] = torch.argmin(dist, dim=1)
    return out


def kmeans(x: torch.Tensor, k: int, iters: int, seed: int) -> torch.Tensor:
    """Lloyd's algorithm; init = first k rows of a seeded permutation; an empty
    cluster keeps its previous centroid."""
    n = x.shape[0]
    assert n >= k, "k-means sample smaller than k"
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    perm = torch.randperm(n, generator=g)[:k].to(x.device)
    c = x[perm].clone()
    for _ in range(iters):
        a = _assign(x, c)
        sums = torch.zeros_like(c).index_add_(0, a, x)
        cnt = torch.zeros(k, dtype=x.dtype, device=x.device).index_add_(
            0, a, torch.ones(n, dtype=x.dtype, device=x.device))
        nz = cnt > 0
        c[nz] = sums[nz] / cnt[nz, None]
    return c


def train_codebooks(sample: torch.Tensor, lay: Layout, iters: int, seed: int) -> torch.Tensor:
    """Concatenated codebooks: for j ascending, [2^nbits[j], dsub[j]] row-major, float32."""
    parts = []
    o = 0
    for j, (k, s) in enumerate(zip(lay.ksub, lay.dsub)):
        c = kmeans(sample[:, o:o + s].contiguous(), k, iters, seed * 131 + j)
        parts.append(c.reshape(-1))
        o += s
    return torch.cat(parts).to(torch.float32).contiguous()


def encode(x: torch.Tensor, lay: Layout, codebooks: torch.Tensor) -> torch.Tensor:
    """[n,m] uint8 sub-codes: nearest centroid in every sub-space."""
    n = x.shape[0]
    sub = torch.empty((n, lay.m), dtype=torch.uint8, device=x.device)
    o = 0
    cb = 0
    for j, (k, s) in enumerate(zip(lay.ksub, lay.dsub)):
        c = codebooks[cb:cb + k * s].reshape(k, s).to(x.device)
        sub[:, j] = _assign(x[:, o:o + s].contiguous(), c).to(torch.uint8)
        o += s
        cb += k * s
    return sub


def pack_codes(sub: torch.Tensor, lay: Layout) -> torch.Tensor:
    """[n,m] sub-codes -> [n,code_size] uint8: little-endian bit stream, sub-code
    j in bits [off_j, off_j+nbits[j]), bit 0 = least significant bit of byte 0."""
    n = sub.shape[0]
    cs = lay.code_size
    if all(b == 4 for b in lay.nbits) and lay.m % 2 == 0:
        return (sub[:, 0::2] | (sub[:, 1::2] << 4)).contiguous()
    out = torch.empty((n, cs), dtype=torch.uint8, device=sub.device)
    step = 1 << 18
    for lo in range(0, n, step):
        blk = sub[lo:lo + step].to(torch.int32)
        acc = torch.zeros((blk.shape[0], cs), dtype=torch.int32, device=sub.device)
        off = 0
        for j, b in enumerate(lay.nbits):
            for kbit in range(b):
                pos = off + kbit
                acc[:, pos >> 3] |= ((blk[:, j] >> kbit) & 1) << (pos & 7)
            off += b
        out[lo:lo + step] = acc.to(torch.uint8)
    return out


# --------------------------------------------------------------------------
# whole synthetic problems
# --------------------------------------------------------------------------
@dataclass
class Problem:
    """An exhaustive-search problem: one list of packed codes."""
    layout: Layout
    codebooks: torch.Tensor   # float32 [codebook_len]
    codes: torch.Tensor       # uint8 [n, code_size]
    queries: torch.Tensor     # float32 [nq, d]
    meta: dict = field(default_factory=dict)


def make_problem(n: int, nq: int, d: int, nbits: Sequence[int], acc_bits: int, dist: str,
                 seed: int, train_n: Optional[int] = None, kmeans_iters: int = 10,
                 device="cpu", encode_chunk: int = 1 << 21) -> Problem:
    lay = make_layout(d, nbits, acc_bits)
    gen = GENERATORS[dist]
    train_n = min(n, train_n or max(20000, 256 * max(lay.ksub)))
    train_n = max(train_n, max(lay.ksub))
    sample = gen(train_n, d, seed * 10 + 1, device)
    codebooks = train_codebooks(sample, lay, kmeans_iters, seed * 10 + 2)
    del sample
    codes = torch.empty((n, lay.code_size), dtype=torch.uint8, device=device)
    # base vectors are generated chunk by chunk so that 1e7..1e8 rows never sit in memory at once
    for c, lo in enumerate(range(0, n, encode_chunk)):
        hi = min(n, lo + encode_chunk)
        xb = gen(hi - lo, d, (seed * 10 + 3) * 4099 + c, device)
        codes[lo:hi] = pack_codes(encode(xb, lay, codebooks), lay)
    queries = gen(nq, d, seed * 10 + 4, device)
    meta = dict(n=n, nq=nq, d=d, nbits=list(nbits), acc_bits=acc_bits, dist=dist, seed=seed,
                train_n=train_n, kmeans_iters=kmeans_iters, torch=torch.__version__)
    return Problem(lay, codebooks, codes, queries, meta)


@dataclass
class IvfProblem:
    """IVF + residual PQ: codes grouped by coarse cell, ids stored beside them."""
    layout: Layout
    codebooks: torch.Tensor      # residual codebooks
    coarse: torch.Tensor         # float32 [K, d]
    list_offsets: torch.Tensor   # int64 [K+1]
    list_codes: torch.Tensor     # uint8 [n, code_size], list by list
    list_ids: torch.Tensor       # int32 [n]
    queries: torch.Tensor        # float32 [nq, d]
    probe_ids: torch.Tensor      # int32 [nq, nprobe], nearest cells first
    meta: dict = field(default_factory=dict)


def nearest_cells(q: torch.Tensor, coarse: torch.Tensor, nprobe: int) -> torch.Tensor:
    """Harness stand-in for the index search: the nprobe nearest coarse centroids
    by exact L2, nearest first (ties -> lowest cell id)."""
    cn = (coarse * coarse).sum(1)
    out = torch.empty((q.shape[0], nprobe), dtype=torch.int32, device=q.device)
    for lo in range(0, q.shape[0], 1024):
        qb = q[lo:lo + 1024]
        dist = cn[None, :] - 2.0 * (qb @ coarse.t())
        key = dist.double()
        _, idx = torch.sort(key, dim=1, stable=True)
        out[lo:lo + 1024] = idx[:, :nprobe].to(torch.int32)
    return out


def make_ivf_problem(n: int, nq: int, d: int, nbits: Sequence[int], acc_bits: int, dist: str,
                     K: int, nprobe: int, seed: int, train_n: Optional[int] = None,
                     kmeans_iters: int = 10, device="cpu",
                     encode_chunk: int = 1 << 21) -> IvfProblem:
    lay = make_layout(d, nbits, acc_bits)
    gen = GENERATORS[dist]
    train_n = min(n, train_n or max(20000, 16 * K))
    train_n = max(train_n, K, max(lay.ksub))
    sample = gen(train_n, d, seed * 10 + 1, device)
    coarse = kmeans(sample, K, kmeans_iters, seed * 10 + 5).to(torch.float32).contiguous()
    res = sample - coarse[_assign(sample, coarse)]
    codebooks = train_codebooks(res, lay, kmeans_iters, seed * 10 + 2)
    del sample, res
    assign = torch.empty(n, dtype=torch.int64, device=device)
    codes = torch.empty((n, lay.code_size), dtype=torch.uint8, device=device)
    for c, lo in enumerate(range(0, n, encode_chunk)):
        hi = min(n, lo + encode_chunk)
        xb = gen(hi - lo, d, (seed * 10 + 3) * 4099 + c, device)
        a = _assign(xb, coarse)
        assign[lo:hi] = a
        codes[lo:hi] = pack_codes(encode(xb - coarse[a], lay, codebooks), lay)
    order = torch.sort(assign, stable=True)[1]
    list_codes = codes[order].contiguous()
    list_ids = order.to(torch.int32).contiguous()
    counts = torch.bincount(assign, minlength=K)
    list_offsets = torch.zeros(K + 1, dtype=torch.int64, device=device)
    list_offsets[1:] = torch.cumsum(counts, 0)
    queries = gen(nq, d, seed * 10 + 4, device)
    probe_ids = nearest_cells(queries, coarse, nprobe)
    meta = dict(n=n, nq=nq, d=d, nbits=list(nbits), acc_bits=acc_bits, dist=dist, K=K,
                nprobe=nprobe, seed=seed, train_n=train_n, kmeans_iters=kmeans_iters,
                torch=torch.__version__)
    return IvfProblem(lay, codebooks, coarse, list_offsets, list_codes, list_ids, queries,
                      probe_ids, meta)


# --------------------------------------------------------------------------
# the five benchmark configurations and their small twins
# --------------------------------------------------------------------------
BASE_SEED = 18120916

C3_BITS = [6, 5, 5, 6, 5, 5, 4, 4]

CONFIGS = {
    # name: kwargs for make_problem / make_ivf_problem, plus R values
    "C0": dict(kind="flat", n=100_000, nq=100, d=128, nbits=[4] * 16, acc_bits=8,
               dist="gamma_ints", seed=BASE_SEED + 0, train_n=20_000, R=[100]),
    "C1": dict(kind="flat", n=10_000_000, nq=10_000, d=96, nbits=[4] * 16, acc_bits=8,
               dist="aniso_gauss", seed=BASE_SEED + 1, train_n=100_000, R=[100]),
    "C2": dict(kind="flat", n=20_000_000, nq=1_000, d=128, nbits=[4] * 32, acc_bits=8,
               dist="gamma_ints", seed=BASE_SEED + 2, train_n=100_000, R=[10, 1000]),
    "C3": dict(kind="flat", n=10_000_000, nq=1_000, d=128, nbits=C3_BITS, acc_bits=16,
               dist="gamma_ints", seed=BASE_SEED + 3, train_n=100_000, R=[100]),
    "C4": dict(kind="ivf", n=100_000_000, nq=10_000, d=96, nbits=[4] * 16, acc_bits=8,
               dist="aniso_gauss", seed=BASE_SEED + 4, K=65_536, nprobe=64,
               train_n=1_000_000, R=[100]),
    # further layouts of the paper (Sections 3.1-3.3): 64-bit and 128-bit codes, 16-bit tables
    "L8x8": dict(kind="flat", n=10_000_000, nq=1_000, d=128, nbits=[8] * 8, acc_bits=16,
                 dist="gamma_ints", seed=BASE_SEED + 5, train_n=100_000, R=[100]),
    "L664": dict(kind="flat", n=10_000_000, nq=1_000, d=128, nbits=[6, 6, 4] * 4, acc_bits=16,
                 dist="gamma_ints", seed=BASE_SEED + 6, train_n=100_000, R=[100]),
    "L655": dict(kind="flat", n=10_000_000, nq=1_000, d=128, nbits=[6, 5, 5] * 4, acc_bits=16,
                 dist="gamma_ints", seed=BASE_SEED + 7, train_n=100_000, R=[100]),
    "L16x8": dict(kind="flat", n=10_000_000, nq=1_000, d=128, nbits=[8] * 16, acc_bits=16,
                  dist="gamma_ints", seed=BASE_SEED + 8, train_n=100_000, R=[100]),
    "L664x2": dict(kind="flat", n=10_000_000, nq=1_000, d=128, nbits=[6, 6, 4] * 8, acc_bits=16,
                   dist="gamma_ints", seed=BASE_SEED + 9, train_n=100_000, R=[100]),
}


def scaled(name: str, n: int, nq: int, **over) -> dict:
    """A smaller twin of a named configuration (same layout, distribution, seed)."""
    cfg = dict(CONFIGS[name])
    cfg.update(n=n, nq=nq)
    cfg["train_n"] = min(cfg["train_n"], max(n // 2, 4096))
    cfg.update(over)
    return cfg


def build(cfg: dict, device="cpu"):
    cfg = dict(cfg)
    kind = cfg.pop("kind")
    cfg.pop("R", None)
    if kind == "flat":
        return make_problem(device=device, **cfg)
    return make_ivf_problem(device=device, **cfg)
