"""The tuning values of pq_set_option never change a result: the exhaustive search (batch and
single query), both inverted-list modes and the coarse search give the same bytes under drawn
settings as under the defaults (which the other tests compare with the oracle)."""
import numpy as np
import pytest
import torch

from harness import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    from paper_1812_09162_amd import binding
    binding.load()
    return binding


def dev():
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def workloads(qb):
    flat = []
    for nbits, d, acc, n, R, nq in [([4] * 16, 96, 8, 700_000, 100, 5), (list(synth.C3_BITS), 128, 16, 300_000, 10, 3),
                                    ([4] * 32, 128, 8, 250_000, 1000, 2), ([8] * 8, 64, 16, 150_000, 100, 9)]:
        flat.append((synth.make_problem(n=n, nq=nq, d=d, nbits=nbits, acc_bits=acc, dist="gamma_ints", seed=5 + n,
                                        train_n=20000, kmeans_iters=2, device=dev()), R))
    ivf = [(synth.make_ivf_problem(n=80_000, nq=40, d=96, nbits=[4] * 16, acc_bits=8, dist="aniso_gauss", K=60,
                                   nprobe=24, seed=3, train_n=6000, kmeans_iters=2), 100),
           (synth.make_ivf_problem(n=40_000, nq=6, d=128, nbits=list(synth.C3_BITS), acc_bits=16, dist="gamma_ints",
                                   K=90, nprobe=30, seed=4, train_n=6000, kmeans_iters=2), 50)]
    g = torch.Generator(device="cpu").manual_seed(9)
    cen = torch.randn((30_000, 64), generator=g).to(dev())
    cq = torch.randn((70, 64), generator=g).to(dev())
    return flat, ivf, cen, cq


def run_all(qb, workloads):
    flat, ivf, cen, cq = workloads
    out = []
    for pr, R in flat:
        lay = pr.layout
        idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, pr.codebooks.to(dev()), lay.acc_bits)
        out += list(qb.pq_search_topk(idx, pr.queries.to(dev()), pr.codes.to(dev()), 400, R))
        out += list(qb.pq_search_topk(idx, pr.queries[:1].to(dev()).contiguous(), pr.codes.to(dev()), 400, R))
        torch.cuda.synchronize()
        idx.close()
    for ip, R in ivf:
        lay = ip.layout
        idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, ip.codebooks.to(dev()), lay.acc_bits)
        args = (idx, ip.coarse.to(dev()), ip.list_offsets.to(dev()), ip.list_codes.to(dev()), ip.list_ids.to(dev()),
                ip.queries.to(dev()), ip.probe_ids.to(dev()), 400, R)
        out += list(qb.ivf_adc_scan_topk(*args))
        out += list(qb.ivf_adc_scan_topk_tightening(*args))
        torch.cuda.synchronize()
        idx.close()
    out += list(qb.ivf_coarse_search(cq, cen, 32))
    torch.cuda.synchronize()
    return [o.clone() for o in out]


def test_drawn_option_values_leave_every_result_unchanged(qb, workloads):
    defaults = {o: qb.pq_get_option(o) for o in range(8)}
    ref = run_all(qb, workloads)
    rng = np.random.default_rng(20240614)
    for trial in range(12):
        opts = {qb.PQ_OPT_SCAN_BLOCKS: int(rng.choice([1, 7, 64, 100, 512, 1024, 2048, 4096])),
                qb.PQ_OPT_PILOT_CODES: int(rng.choice([0, 1000, 65536, 262144, 524288, 1 << 20])),
                qb.PQ_OPT_PILOT_CODES_SINGLE: int(rng.choice([0, 4096, 65536, 200000])),
                qb.PQ_OPT_PILOT_BLOCKS: int(rng.choice([1, 3, 16, 64, 128])),
                qb.PQ_OPT_IVF_THREADS: int(rng.choice([64, 128, 256])),
                qb.PQ_OPT_SHARED_PASSES: int(rng.choice([0, 1])),
                qb.PQ_OPT_COARSE_FILTER: int(rng.choice([0, 1])),
                qb.PQ_OPT_IVF_SHARED_LISTS: int(rng.choice([0, 1, 2]))}
        try:
            for k, v in opts.items():
                qb.pq_set_option(k, v)
            got = run_all(qb, workloads)
        finally:
            for k, v in defaults.items():
                qb.pq_set_option(k, v)
        for i, (a, b) in enumerate(zip(ref, got)):
            assert torch.equal(a, b), (trial, i, opts)
