"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(fused pq_search_topk, one query per call, and a 32-query batch): a sample of queries is
compared bit for bit with the CPU oracle, and all batch sizes must agree with each other.

Data sets are fabricated on the GPU (seconds); the oracle runs one query per host thread.
The 10^8-vector IVF configuration is fabricated with 3 Lloyd iterations for its 65,536-cell
coarse quantizer (instead of 10) to keep the test under a minute; a tenth-size twin with the
same cell occupancy runs as well.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
from paper_1812_09162_amd import synth

pytestmark = pytest.mark.gpu
T_CAL = 400


@pytest.fixture(scope="module")
def qb():
    from paper_1812_09162_amd import binding
    binding.load()
    return binding


def dev():
    return torch.device("cuda:0")


def oracle_many(pr, qsel, R, codes_np):
    lay = pr.layout
    cb = pr.codebooks.cpu().numpy()
    qs = pr.queries[qsel].cpu().numpy()

    def one(i):
        return oracle.search(lay.d, lay.nbits, lay.dsub, lay.acc_bits, cb, qs[i], codes_np, T_CAL, R)

    with ThreadPoolExecutor(max_workers=min(len(qsel), 8)) as ex:
        return list(ex.map(one, range(len(qsel))))


def run_flat(qb, name, Rs, nq_oracle, nq_gpu=64):
    cfg = dict(synth.CONFIGS[name])
    cfg["nq"] = nq_gpu
    pr = synth.build(cfg, device=dev())
    lay = pr.layout
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, pr.codebooks, lay.acc_bits)
    codes_np = pr.codes.cpu().numpy()
    qsel = list(range(nq_oracle))
    for R in Rs:
        # the configuration bench.py times: one query per fused call
        singles = [qb.pq_search_topk(idx, pr.queries[q:q + 1].contiguous(), pr.codes, T_CAL, R)
                   for q in qsel]
        batch = qb.pq_search_topk(idx, pr.queries[:32].contiguous(), pr.codes, T_CAL, R)
        torch.cuda.synchronize()
        ref = oracle_many(pr, qsel, R, codes_np)
        for q in qsel:
            oi, ok, od = ref[q]
            gi, gk, gd = (x[0].cpu().numpy() for x in singles[q])
            assert np.array_equal(gi, oi), (name, R, q, gi[:8], oi[:8])
            assert np.array_equal(gk.astype(np.uint16), ok)
            assert np.array_equal(gd, od)
            for a, b in zip(singles[q], batch):
                assert torch.equal(a[0], b[q])
        # property that holds at any size: keys ascending, ids ascending within equal keys, all valid
        k = batch[1].cpu().numpy().astype(np.int64)
        i = batch[0].cpu().numpy().astype(np.int64)
        assert np.all(np.diff(k, axis=1) >= 0)
        assert np.all((np.diff(k, axis=1) > 0) | (np.diff(i, axis=1) > 0))
        assert i.min() >= 0 and i.max() < pr.codes.shape[0]
    idx.close()


def test_c1_full_size(qb):
    run_flat(qb, "C1", [100], nq_oracle=6)


def test_c2_full_size(qb):
    run_flat(qb, "C2", [10, 1000], nq_oracle=3)


def test_c3_full_size(qb):
    run_flat(qb, "C3", [100], nq_oracle=4)


@pytest.mark.parametrize("name", ["L8x8", "L664", "L16x8", "L664x2"])
def test_further_layouts_full_size(qb, name):
    """The 64- and 128-bit layouts bench.py offers as workloads, at their 10^7 codes."""
    run_flat(qb, name, [100], nq_oracle=2, nq_gpu=32)


def run_ivf(qb, cfg, nq_oracle, R=100):
    ip = synth.build(cfg, device=dev())
    lay = ip.layout
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, ip.codebooks, lay.acc_bits)
    gi, gd = qb.ivf_adc_scan_topk(idx, ip.coarse, ip.list_offsets, ip.list_codes, ip.list_ids,
                                  ip.queries, ip.probe_ids, T_CAL, R)
    torch.cuda.synchronize()
    host = dict(cb=ip.codebooks.cpu().numpy(), coarse=ip.coarse.cpu().numpy(),
                off=ip.list_offsets.cpu().numpy(), codes=ip.list_codes.cpu().numpy(),
                ids=ip.list_ids.cpu().numpy(), q=ip.queries.cpu().numpy(),
                probe=ip.probe_ids.cpu().numpy())

    def one(q):
        return oracle.search_ivf(lay.d, lay.nbits, lay.dsub, lay.acc_bits, host["cb"], host["coarse"],
                                 host["off"], host["codes"], host["ids"], host["q"][q],
                                 host["probe"][q], T_CAL, R)

    with ThreadPoolExecutor(max_workers=8) as ex:
        ref = list(ex.map(one, range(nq_oracle)))
    gi_np, gd_np = gi.cpu().numpy(), gd.cpu().numpy()
    for q in range(nq_oracle):
        assert np.array_equal(gi_np[q], ref[q][0]), (q, gi_np[q][:8], ref[q][0][:8])
        assert np.array_equal(gd_np[q], ref[q][1])
    # any-size properties on all queries: sorted by (dist, id), ids come from probed lists
    assert np.all(np.diff(gd_np, axis=1) >= 0)
    sizes = np.diff(host["off"])
    cell_of = np.repeat(np.arange(len(sizes)), sizes)
    pos_of_id = np.empty(len(cell_of), np.int64)
    pos_of_id[host["ids"]] = np.arange(len(cell_of))
    for q in range(0, gi_np.shape[0], max(1, gi_np.shape[0] // 64)):
        got = gi_np[q][gi_np[q] >= 0]
        assert np.all(np.isin(cell_of[pos_of_id[got]], host["probe"][q]))
    idx.close()


def test_c4_tenth_size(qb):
    cfg = synth.scaled("C4", n=10_000_000, nq=256, K=6_554, train_n=200_000, kmeans_iters=4)
    run_ivf(qb, cfg, nq_oracle=48)


def test_c4_full_size(qb):
    cfg = dict(synth.CONFIGS["C4"])
    cfg.update(nq=1024, kmeans_iters=3)
    run_ivf(qb, cfg, nq_oracle=64)
