"""GPU parity of pq_encode (through the C ABI) against the CPU oracle: packed codes byte for byte,
on all layouts, ragged counts, with and without the residual shift, and at a size that spans many
blocks; plus the chain encode -> search on the GPU against the oracle's own chain."""
import numpy as np
import pytest
import torch

import oracle
from harness import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    from paper_1812_09162_amd import binding
    binding.load()
    return binding


def dev():
    return torch.device("cuda:0")


def layout_and_codebooks(d, nbits, seed, integer=False):
    lay = synth.make_layout(d, nbits, 16)
    rng = np.random.default_rng(seed)
    ncb = sum((1 << b) * s for b, s in zip(lay.nbits, lay.dsub))
    cb = (rng.integers(-6, 7, ncb) if integer else rng.normal(size=ncb)).astype(np.float32)
    return lay, cb


@pytest.mark.parametrize("d,nbits", [
    (128, [4] * 16), (96, [4] * 16), (128, [4] * 32), (128, synth.C3_BITS), (128, [8] * 8),
    (128, [6, 6, 4] * 8), (13, [3, 7, 1, 2]), (64, [8] * 16), (256, [4] * 16), (15, [5, 5, 5]),
])
@pytest.mark.parametrize("n", [1, 63, 64, 65, 127, 129, 1000])
def test_encode_bit_exact(qb, d, nbits, n):
    lay, cb = layout_and_codebooks(d, nbits, seed=len(nbits) + d)
    rng = np.random.default_rng(n)
    x = rng.normal(size=(n, d)).astype(np.float32)
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, torch.from_numpy(cb).to(dev()), 16)
    got = qb.pq_encode(idx, torch.from_numpy(x).to(dev())).cpu().numpy()
    assert np.array_equal(got, oracle.encode(d, lay.nbits, lay.dsub, cb, x))
    idx.close()


def test_encode_ties_go_to_the_lowest_index(qb):
    lay, cb = layout_and_codebooks(24, [4, 5, 3, 6], seed=3, integer=True)   # duplicate centroids abound
    rng = np.random.default_rng(4)
    x = rng.integers(-6, 7, (777, 24)).astype(np.float32)
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, torch.from_numpy(cb).to(dev()), 16)
    got = qb.pq_encode(idx, torch.from_numpy(x).to(dev())).cpu().numpy()
    assert np.array_equal(got, oracle.encode(24, lay.nbits, lay.dsub, cb, x))
    idx.close()


def test_encode_residuals(qb):
    lay, cb = layout_and_codebooks(96, [4] * 16, seed=8)
    rng = np.random.default_rng(9)
    n, K = 5000, 37
    x = rng.normal(size=(n, 96)).astype(np.float32)
    coarse = rng.normal(size=(K, 96)).astype(np.float32)
    ids = rng.integers(0, K, n).astype(np.int32)
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, torch.from_numpy(cb).to(dev()), 8)
    got = qb.pq_encode(idx, torch.from_numpy(x).to(dev()), torch.from_numpy(coarse).to(dev()),
                       torch.from_numpy(ids).to(dev())).cpu().numpy()
    assert np.array_equal(got, oracle.encode(96, lay.nbits, lay.dsub, cb, x, coarse[ids]))
    idx.close()


def test_encode_then_search_matches_the_oracle_chain(qb):
    pr = synth.build(synth.scaled("C3", n=20_000, nq=3))
    lay = pr.layout
    rng = np.random.default_rng(12)
    x = np.minimum(255, np.floor(rng.gamma(0.5, 7.27, (20_000, lay.d)))).astype(np.float32)
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, pr.codebooks.to(dev()), lay.acc_bits)
    codes = qb.pq_encode(idx, torch.from_numpy(x).to(dev()))
    ocodes = oracle.encode(lay.d, lay.nbits, lay.dsub, pr.codebooks.numpy(), x)
    assert np.array_equal(codes.cpu().numpy(), ocodes)
    ids, keys, dist = qb.pq_search_topk(idx, pr.queries.to(dev()), codes, 400, 50)
    torch.cuda.synchronize()
    for q in range(pr.queries.shape[0]):
        oi, ok, od = oracle.search(lay.d, lay.nbits, lay.dsub, lay.acc_bits, pr.codebooks.numpy(),
                                   pr.queries[q].numpy(), ocodes, 400, 50)
        assert np.array_equal(ids[q].cpu().numpy(), oi)
        assert np.array_equal(dist[q].cpu().numpy(), od)
    idx.close()


def test_encode_large_sampled(qb):
    """2,000,003 vectors of the C1 shape: every code must decode to a nearest centroid; a sample is
    compared with the oracle."""
    cfg = synth.scaled("C1", n=1000, nq=1)
    pr = synth.build(cfg)
    lay = pr.layout
    g = torch.Generator(device=dev()).manual_seed(77)
    n = 2_000_003
    x = torch.randn((n, lay.d), generator=g, device=dev(), dtype=torch.float32)
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, pr.codebooks.to(dev()), lay.acc_bits)
    codes = qb.pq_encode(idx, x)
    torch.cuda.synchronize()
    sel = np.r_[0:300, n // 2:n // 2 + 300, n - 300:n]
    want = oracle.encode(lay.d, lay.nbits, lay.dsub, pr.codebooks.numpy(), x[sel].cpu().numpy())
    assert np.array_equal(codes[sel].cpu().numpy(), want)
    idx.close()


def test_encode_errors(qb):
    lay, cb = layout_and_codebooks(16, [4] * 4, seed=1)
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, torch.from_numpy(cb).to(dev()), 8)
    x = torch.zeros((4, 16), dtype=torch.float32, device=dev())
    rc = qb.load().pq_encode(idx.handle, x.data_ptr(), 4, x.data_ptr(), None, x.data_ptr(), None)
    assert rc == qb.PQ_EINVAL
    assert qb.pq_encode(idx, x[:0]).shape == (0, 2)
    idx.close()
