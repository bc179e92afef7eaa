"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(fused pq_search_topk, one query per call): every configured query is run in batches of 1, 32
and 256, which must agree byte for byte, and a sample of queries is compared bit for bit with
the CPU oracle.

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
from harness import synth

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


def run_flat(qb, name, Rs, nq_oracle, nq_gpu=None):
    """nq_gpu = None: every query the configuration has (10,000 for C1, 1,000 for C2 and C3)."""
    cfg = dict(synth.CONFIGS[name])
    if nq_gpu is not None:
        cfg["nq"] = nq_gpu
    pr = synth.build(cfg, device=dev())
    lay = pr.layout
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, pr.codebooks, lay.acc_bits)
    codes_np = pr.codes.cpu().numpy()
    nq, n = pr.queries.shape[0], pr.codes.shape[0]
    qsel = list(range(nq_oracle))
    for R in Rs:
        def outputs():
            return (torch.full((nq, R), -7, dtype=torch.int32, device=dev()),
                    torch.full((nq, R), 9, dtype=torch.uint16, device=dev()),
                    torch.full((nq, R), -1.0, dtype=torch.float32, device=dev()))

        # every query in batches of 1 (the configuration bench.py times), 32 and 256: the result
        # is defined as a sort, so the three must agree byte for byte
        by_batch = {}
        for bs in (1, 32, 256):
            out = outputs()
            ws = torch.empty(qb.pq_search_workspace_bytes(idx, bs, n, R), dtype=torch.uint8, device=dev())
            for lo in range(0, nq, bs):
                hi = min(nq, lo + bs)
                qb.pq_search_topk(idx, pr.queries[lo:hi], pr.codes, T_CAL, R, workspace=ws,
                                  out=tuple(o[lo:hi] for o in out))
            torch.cuda.synchronize()
            by_batch[bs] = out
        for bs in (32, 256):
            for a, b in zip(by_batch[1], by_batch[bs]):
                assert torch.equal(a, b), (name, R, bs, int((a != b).any(dim=1).nonzero()[0]))
        # a sample of them against the oracle
        ref = oracle_many(pr, qsel, R, codes_np)
        for q in qsel:
            oi, ok, od = ref[q]
            gi, gk, gd = (x[q].cpu().numpy() for x in by_batch[1])
            assert np.array_equal(gi, oi), (name, R, q, gi[:8], oi[:8])
            assert np.array_equal(gk.astype(np.uint16), ok)
            assert np.array_equal(gd, od)
        # property that holds at any size: keys ascending, ids ascending within equal keys, all valid
        k = by_batch[1][1].cpu().numpy().astype(np.int64)
        i = by_batch[1][0].cpu().numpy().astype(np.int64)
        assert np.all(np.diff(k, axis=1) >= 0)
        assert np.all((np.diff(k, axis=1) > 0) | (np.diff(i, axis=1) > 0))
        assert i.min() >= 0 and i.max() < n
    idx.close()


def test_c1_full_size(qb):
    run_flat(qb, "C1", [100], nq_oracle=6)


def test_c2_full_size(qb):
    run_flat(qb, "C2", [10, 1000], nq_oracle=3)


def test_c3_full_size(qb):
    run_flat(qb, "C3", [100], nq_oracle=4)


@pytest.mark.parametrize("name", ["L8x8", "L664", "L655", "L16x8", "L664x2"])
def test_further_layouts_full_size(qb, name):
    """The 64- and 128-bit layouts bench.py offers as workloads, at their 10^7 codes."""
    run_flat(qb, name, [100], nq_oracle=2, nq_gpu=300)


def run_ivf(qb, cfg, nq_oracle, R=100):
    ip = synth.build(cfg, device=dev())
    lay = ip.layout
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, ip.codebooks, lay.acc_bits)
    # the default workspace (blocks in the order of the probed cells) and the minimal one (grid order)
    gi, gd = qb.ivf_adc_scan_topk(idx, ip.coarse, ip.list_offsets, ip.list_codes, ip.list_ids,
                                  ip.queries, ip.probe_ids, T_CAL, R)
    small = torch.empty(qb.ivf_workspace_bytes(idx, ip.probe_ids.shape[0], ip.probe_ids.shape[1], R),
                        dtype=torch.uint8, device=dev())
    gi2, gd2 = qb.ivf_adc_scan_topk(idx, ip.coarse, ip.list_offsets, ip.list_codes, ip.list_ids,
                                    ip.queries, ip.probe_ids, T_CAL, R, workspace=small)
    ti, td = qb.ivf_adc_scan_topk_tightening(idx, ip.coarse, ip.list_offsets, ip.list_codes, ip.list_ids,
                                             ip.queries, ip.probe_ids, T_CAL, R, workspace=small)
    torch.cuda.synchronize()
    assert torch.equal(gi, gi2) and torch.equal(gd, gd2)
    del small, gi2, gd2
    # one pass per list for up to four of the queries that probe it, whatever the number of pairs per cell
    qb.pq_set_option(qb.PQ_OPT_IVF_SHARED_LISTS, 2)
    try:
        gi3, gd3 = qb.ivf_adc_scan_topk(idx, ip.coarse, ip.list_offsets, ip.list_codes, ip.list_ids,
                                        ip.queries, ip.probe_ids, T_CAL, R)
        torch.cuda.synchronize()
    finally:
        qb.pq_set_option(qb.PQ_OPT_IVF_SHARED_LISTS, 1)
    assert torch.equal(gi, gi3) and torch.equal(gd, gd3)
    del gi3, gd3
    host = dict(cb=ip.codebooks.cpu().numpy(), coarse=ip.coarse.cpu().numpy(),
                off=ip.list_offsets.cpu().numpy(), codes=ip.list_codes.cpu().numpy(),
                ids=ip.list_ids.cpu().numpy(), q=ip.queries.cpu().numpy(),
                probe=ip.probe_ids.cpu().numpy())

    def one(q):
        return oracle.search_ivf(lay.d, lay.nbits, lay.dsub, lay.acc_bits, host["cb"], host["coarse"],
                                 host["off"], host["codes"], host["ids"], host["q"][q],
                                 host["probe"][q], T_CAL, R)

    def one_tightening(q):
        return oracle.search_ivf_tightening(lay.d, lay.nbits, lay.dsub, lay.acc_bits, host["cb"],
                                            host["coarse"], host["off"], host["codes"], host["ids"],
                                            host["q"][q], host["probe"][q], T_CAL, R)

    with ThreadPoolExecutor(max_workers=8) as ex:
        ref = list(ex.map(one, range(nq_oracle)))
        ref_t = list(ex.map(one_tightening, range(nq_oracle)))
    gi_np, gd_np = gi.cpu().numpy(), gd.cpu().numpy()
    ti_np, td_np = ti.cpu().numpy(), td.cpu().numpy()
    for q in range(nq_oracle):
        assert np.array_equal(gi_np[q], ref[q][0]), (q, gi_np[q][:8], ref[q][0][:8])
        assert np.array_equal(gd_np[q], ref[q][1])
        assert np.array_equal(ti_np[q], ref_t[q][0]), ("tightening", q, ti_np[q][:8], ref_t[q][0][:8])
        assert np.array_equal(td_np[q], ref_t[q][1])
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


def test_largest_n(qb):
    """n = 2^31 - 1, the largest list the scan accepts (ids are int32): 17 GB of 8-byte codes.

    Codebooks and queries are those of a small C1-shaped data set; the code bytes are uniform
    random (so the best codes lie anywhere in the list), and for each query its best possible code
    (every sub-quantizer at its table minimum) is planted at positions spread up to n - 1.  Quantized tables come from the oracle (it needs the first t codes only); the
    expected top-R by (key, id) over all n codes is computed chunk by chunk with plain torch
    indexing and top-k, and the float distances of those keys by the oracle.
    """
    n = 2 ** 31 - 1
    R = 100
    if torch.cuda.mem_get_info()[1] < 48e9:
        pytest.skip("needs 17 GB for the code list plus temporaries")
    pr = synth.build(synth.scaled("C1", n=100_000, nq=3), device=dev())
    lay = pr.layout
    assert lay.m == 16 and set(lay.nbits) == {4}
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, pr.codebooks, lay.acc_bits)
    g = torch.Generator(device=dev())
    g.manual_seed(20_231)
    codes = torch.empty((n, 8), dtype=torch.uint8, device=dev())
    CH = 1 << 26
    for a in range(0, n, CH):
        b = min(n, a + CH)
        codes[a:b] = torch.randint(0, 256, (b - a, 8), generator=g, device=dev(), dtype=torch.uint8)
    cb = pr.codebooks.cpu().numpy()
    qs = pr.queries.cpu().numpy()
    nq = qs.shape[0]
    ftab = [oracle.tables(lay.d, lay.nbits, lay.dsub, cb, qs[q]) for q in range(nq)]
    planted = [n - 1, n - 2, n - 3 - 2, 2 ** 30 - 1, 2 ** 30, 2 ** 30 + 1, 2 ** 31 - 1024, 3 * 2 ** 29 + 7]
    for q in range(nq):
        arg = ftab[q].reshape(16, 16).argmin(axis=1)
        best = np.array([arg[2 * i] | (arg[2 * i + 1] << 4) for i in range(8)], dtype=np.uint8)
        for p in planted:
            codes[p - 16 * q] = torch.from_numpy(best).to(dev())
    head = codes[:4 * R + T_CAL].cpu().numpy()
    quant = [oracle.quantize(lay.nbits, lay.acc_bits, ftab[q], head, T_CAL, R) for q in range(nq)]

    def reference(q):
        qt = torch.from_numpy(quant[q][0].astype(np.int32)).to(dev()).view(16, 16)
        best = None
        for a in range(0, n, CH):
            c = codes[a:min(n, a + CH)]
            key = torch.zeros(c.shape[0], dtype=torch.int32, device=dev())
            for b in range(8):
                byte = c[:, b].long()
                key += qt[2 * b][byte & 15] + qt[2 * b + 1][byte >> 4]
            key.clamp_(max=255)
            comp = (key.long() << 32) | torch.arange(a, a + c.shape[0], device=dev(), dtype=torch.int64)
            top = torch.topk(comp, R, largest=False).values
            best = top if best is None else torch.topk(torch.cat([best, top]), R, largest=False).values
            del key, comp, byte
        best = torch.sort(best).values.cpu().numpy()
        keys = (best >> 32).astype(np.uint16)
        ids = (best & 0xffffffff).astype(np.int32)
        _, _, dist = oracle.topk(lay.acc_bits, keys, R, quant[q][1], quant[q][2])
        return ids, keys, dist

    one = [qb.pq_search_topk(idx, pr.queries[q:q + 1].contiguous(), codes, T_CAL, R) for q in range(nq)]
    many = qb.pq_search_topk(idx, pr.queries.contiguous(), codes, T_CAL, R)
    torch.cuda.synchronize()
    for q in range(nq):
        ids, keys, dist = reference(q)
        assert set(p - 16 * q for p in planted) <= set(ids.tolist()), "planted codes must be found"
        for got in ([x[0] for x in one[q]], [x[q] for x in many]):
            assert np.array_equal(got[0].cpu().numpy(), ids), (q, got[0][:12], ids[:12])
            assert np.array_equal(got[1].cpu().numpy().astype(np.uint16), keys)
            assert np.array_equal(got[2].cpu().numpy(), dist)
    idx.close()
