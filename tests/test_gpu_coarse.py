"""GPU parity of ivf_coarse_search (through the C ABI) against the CPU oracle: probe ids and
scores bit for bit, on float and on integer-valued data, ragged shapes, ties and padding; and
the chain coarse search -> inverted-list search against the oracle's own chain."""
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


def check(qb, cen, qs, nprobe, nq_oracle=None):
    ids, sc = qb.ivf_coarse_search(torch.from_numpy(qs).to(dev()), torch.from_numpy(cen).to(dev()), nprobe)
    torch.cuda.synchronize()
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    sel = range(qs.shape[0]) if nq_oracle is None else np.linspace(0, qs.shape[0] - 1, nq_oracle).astype(int)
    for q in sel:
        oi, os_ = oracle.coarse_search(cen, qs[q], nprobe)
        assert np.array_equal(ids[q], oi), (q, ids[q][:8], oi[:8])
        assert np.array_equal(sc[q], os_), (q, sc[q][:4], os_[:4])
    return ids


@pytest.mark.parametrize("K,d,nq,nprobe,seed", [
    (1000, 96, 37, 64, 0), (4099, 128, 130, 16, 1), (257, 13, 5, 8, 2), (128, 32, 128, 128, 3),
    (33, 7, 3, 40, 4), (1, 4, 2, 1, 5), (5000, 96, 300, 1, 6), (700, 100, 260, 1024, 7),
])
def test_coarse_search_float_data_bit_exact(qb, K, d, nq, nprobe, seed):
    rng = np.random.default_rng(seed)
    cen = rng.normal(size=(K, d)).astype(np.float32)
    qs = rng.normal(size=(nq, d)).astype(np.float32)
    check(qb, cen, qs, nprobe)


def test_coarse_search_integer_data_with_duplicates(qb):
    rng = np.random.default_rng(11)
    K, d, nq = 3000, 24, 50
    cen = rng.integers(-3, 4, (K, d)).astype(np.float32)   # few distinct values: many exact ties
    cen[1000:1100] = cen[0]                                # a hundred copies of one centroid
    qs = rng.integers(-3, 4, (nq, d)).astype(np.float32)
    qs[0] = cen[0]
    ids = check(qb, cen, qs, 64)
    # exact arithmetic: the oracle's answer is the exact squared-L2 ranking with ties by id
    dist = ((cen.astype(np.int64)[None] - qs.astype(np.int64)[:, None]) ** 2).sum(2)
    for q in range(nq):
        assert ids[q].tolist() == np.lexsort((np.arange(K), dist[q]))[:64].tolist()


def test_coarse_search_all_equal_scores(qb):
    cen = np.ones((2500, 8), np.float32)
    qs = np.zeros((3, 8), np.float32)
    ids = check(qb, cen, qs, 100)
    assert ids[0].tolist() == list(range(100))


def test_coarse_search_c4_shape_and_chain_into_ivf(qb):
    """The C4 shape at a fortieth of its size: cells found on the GPU feed the inverted-list
    search; both stages match the oracle fed with its own cells."""
    cfg = synth.scaled("C4", n=200_000, nq=12, K=1638, train_n=20_000, kmeans_iters=3)
    ip = synth.build(cfg, device=dev())
    lay = ip.layout
    nprobe = ip.probe_ids.shape[1]
    pid, _ = qb.ivf_coarse_search(ip.queries, ip.coarse, nprobe)
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, ip.codebooks, lay.acc_bits)
    gi, gd = qb.ivf_adc_scan_topk(idx, ip.coarse, ip.list_offsets, ip.list_codes, ip.list_ids,
                                  ip.queries, pid, 400, 100)
    torch.cuda.synchronize()
    coarse, qs = ip.coarse.cpu().numpy(), ip.queries.cpu().numpy()
    for q in range(qs.shape[0]):
        oi, _ = oracle.coarse_search(coarse, qs[q], nprobe)
        assert np.array_equal(pid[q].cpu().numpy(), oi)
        ri, rd, _ = oracle.search_ivf(lay.d, lay.nbits, lay.dsub, lay.acc_bits, ip.codebooks.cpu().numpy(),
                                      coarse, ip.list_offsets.cpu().numpy(), ip.list_codes.cpu().numpy(),
                                      ip.list_ids.cpu().numpy(), qs[q], oi, 400, 100)
        assert np.array_equal(gi[q].cpu().numpy(), ri)
        assert np.array_equal(gd[q].cpu().numpy(), rd)
    idx.close()


def test_coarse_search_full_k_sampled(qb):
    """K = 65,536 cells, d = 96, 2,100 queries (three passes of the score matrix would need more;
    here two tiles of queries are ragged): a sample of queries against the oracle."""
    rng = np.random.default_rng(21)
    K, d, nq = 65_536, 96, 2100
    cen = rng.normal(size=(K, d)).astype(np.float32)
    cen /= np.linalg.norm(cen, axis=1, keepdims=True)
    qs = rng.normal(size=(nq, d)).astype(np.float32)
    check(qb, cen, qs, 64, nq_oracle=12)


@pytest.mark.parametrize("K,d,nq,nprobe,seed", [
    (20_000, 96, 70, 64, 31), (16_511, 40, 130, 1, 32), (30_001, 128, 9, 20, 33), (17_000, 17, 257, 64, 34),
    (70_001, 24, 33, 64, 35), (60_000, 16, 20, 200, 36),   # the 1024-thread candidate selection
])
def test_coarse_search_filtering_form_bit_exact(qb, K, d, nq, nprobe, seed):
    """K large enough for the form that never writes the score matrix (pilot bound, candidate
    lists per block of 256 cells)."""
    rng = np.random.default_rng(seed)
    cen = rng.normal(size=(K, d)).astype(np.float32)
    qs = rng.normal(size=(nq, d)).astype(np.float32)
    check(qb, cen, qs, nprobe, nq_oracle=min(nq, 24))


def test_coarse_search_filtering_form_overflow_falls_back(qb):
    """Forty copies of one cell inside a single block of 256 overflow that block's candidate list
    for the queries near it; the pass is then redone in the matrix form.  Also: all cells equal."""
    rng = np.random.default_rng(41)
    K, d = 20_000, 32
    cen = rng.normal(size=(K, d)).astype(np.float32)
    cen[12_800:12_840] = cen[12_800]
    qs = rng.normal(size=(40, d)).astype(np.float32)
    qs[:5] = cen[12_800] + 0.01 * rng.normal(size=(5, d)).astype(np.float32)
    ids = check(qb, cen, qs, 64)
    assert set(range(12_800, 12_840)) <= set(ids[0].tolist())
    same = np.ones((18_000, 8), np.float32)
    ids = check(qb, same, np.zeros((3, 8), np.float32), 100)
    assert ids[2].tolist() == list(range(100))


@pytest.mark.parametrize("K,d,nq,nprobe,seed,unit", [
    (3000, 96, 40, 64, 51, False),      # matrix form
    (20_000, 128, 70, 32, 52, False),   # filtering form
    (65_536, 96, 48, 64, 53, True),     # the C4 shape: unit-norm centroids and queries
    (513, 9, 130, 513, 54, False),      # every cell returned
])
def test_coarse_search_against_the_plain_definition_in_fp64(qb, K, d, nq, nprobe, seed, unit):
    """Section 2.1.1 says only that a query goes to the cells whose centroids are nearest.  This
    check does not use the oracle or its arithmetic: squared distances ||z - c||^2 by brute force
    in fp64, and the GPU's answer must be a valid nearest-cell set up to the rounding of an fp32
    evaluation of ||c||^2 - 2 z.c (d products and sums, each rounded once: |error| <=
    (d + 2) 2^-23 (||c||^2 + 2 ||z|| ||c||))."""
    rng = np.random.default_rng(seed)
    cen = rng.normal(size=(K, d)).astype(np.float32)
    qs = rng.normal(size=(nq, d)).astype(np.float32)
    if unit:
        cen /= np.linalg.norm(cen, axis=1, keepdims=True)
        qs /= np.linalg.norm(qs, axis=1, keepdims=True)
    ids, sc = qb.ivf_coarse_search(torch.from_numpy(qs).to(dev()), torch.from_numpy(cen).to(dev()), nprobe)
    torch.cuda.synchronize()
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy().astype(np.float64)
    c64, q64 = cen.astype(np.float64), qs.astype(np.float64)
    cn = (c64 ** 2).sum(1)
    cmax = np.sqrt(cn.max())
    k = min(nprobe, K)
    for q in range(nq):
        true = ((c64 - q64[q][None, :]) ** 2).sum(1)              # ||z - c||^2 for every cell
        zn = np.sqrt((q64[q] ** 2).sum())
        tol = (d + 2) * 2.0 ** -23 * (cmax ** 2 + 2 * zn * cmax)
        got = ids[q, :k]
        assert np.all(ids[q, k:] == -1)
        assert got.min() >= 0 and got.max() < K and len(set(got.tolist())) == k      # distinct cells
        kth = np.partition(true, k - 1)[k - 1]
        assert np.all(true[got] <= kth + 2 * tol)                  # nothing returned is farther
        rest = np.ones(K, bool)
        rest[got] = False
        assert not rest.any() or true[rest].min() >= kth - 2 * tol  # nothing left out is nearer
        assert np.all(np.diff(true[got]) >= -2 * tol)              # nearest first
        assert np.all(np.abs(sc[q, :k] + (q64[q] ** 2).sum() - true[got]) <= tol)   # the scores themselves


def _random_coarse_cases(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        big = rng.random() < 0.7   # large enough for the form that writes no score matrix
        out.append((int(rng.integers(16_500, 90_000)) if big else int(rng.integers(1, 16_500)),
                    int(rng.choice([4, 7, 16, 33, 64, 96, 128])), int(rng.integers(1, 300)),
                    int(rng.choice([1, 3, 16, 64, 100, 128, 129, 200, 256])), int(rng.integers(0, 4)),
                    int(rng.integers(1, 1 << 30))))
    return out


@pytest.mark.parametrize("K,d,nq,nprobe,mode,seed", _random_coarse_cases(16, seed=20240612))
def test_coarse_search_random_cases(qb, K, d, nq, nprobe, mode, seed):
    """Drawn shapes over both forms and both candidate-selection kernels; mode 0: small integers
    (many exact ties), 1: unit-norm centroids, 2: scores of both signs with fifty equal cells,
    3: plain normal data."""
    r = np.random.default_rng(seed)
    if mode == 0:
        cen = r.integers(0, 6, (K, d)).astype(np.float32)
        qs = r.integers(0, 6, (nq, d)).astype(np.float32)
    elif mode == 1:
        cen = r.normal(size=(K, d)).astype(np.float32)
        cen /= np.linalg.norm(cen, axis=1, keepdims=True)
        qs = r.normal(size=(nq, d)).astype(np.float32)
    elif mode == 2:
        cen = (r.normal(size=(K, d)) * 0.3).astype(np.float32)
        cen[K // 2: K // 2 + min(50, K - K // 2)] = cen[K // 2]
        qs = (r.normal(size=(nq, d)) * 3).astype(np.float32)
    else:
        cen = r.normal(size=(K, d)).astype(np.float32)
        qs = r.normal(size=(nq, d)).astype(np.float32)
    check(qb, cen, qs, nprobe, nq_oracle=min(nq, 10))


def test_coarse_search_errors(qb):
    cen = torch.zeros((10, 4), dtype=torch.float32, device=dev())
    qs = torch.zeros((2, 4), dtype=torch.float32, device=dev())
    with pytest.raises(qb.QadcError):
        qb.ivf_coarse_search(qs, cen, 0)
    with pytest.raises(qb.QadcError):
        qb.ivf_coarse_search(qs, cen, 2000)
    with pytest.raises(qb.QadcError):
        qb.ivf_coarse_search(qs, cen, 4, workspace=torch.empty(256, dtype=torch.uint8, device=dev()))
    ids, _ = qb.ivf_coarse_search(qs[:0], cen, 4)
    assert ids.shape == (0, 4)
