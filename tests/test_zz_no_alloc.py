"""pq_adc_scan_topk_static (the entry point that allocates nothing; its scratch memory is an
array inside the library) against pq_adc_scan_topk with a caller workspace, through the C ABI:
identical bytes on two calls in a row, the second with a smaller input, and a clear error beyond
the array's size."""
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


def empty_out(nq, R, fill):
    return (torch.full((nq, R), fill, dtype=torch.int32, device=dev()),
            torch.full((nq, R), 7, dtype=torch.uint16, device=dev()),
            torch.full((nq, R), -1.0, dtype=torch.float32, device=dev()))


@pytest.mark.parametrize("name", ["C1", "C3"])
def test_static_scratch_entry_equals_workspace_entry_twice(qb, name):
    R = 100
    big = synth.build(synth.scaled(name, n=300_001, nq=5))
    lay = big.layout
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, big.codebooks.to(dev()), lay.acc_bits)
    codes = big.codes.to(dev())
    qs = big.queries.to(dev())
    # first call: 5 queries over 300,001 codes; second: 2 queries over the first 40,003 codes
    for nq, n in ((5, 300_001), (2, 40_003)):
        c = codes[:n].contiguous()
        tables = qb.pq_compute_tables(idx, qs[:nq].contiguous())
        qt, qp = qb.pq_quantize_tables(idx, tables, c, 400, R)
        want = qb.pq_adc_scan_topk(idx, qt, qp, c, R)
        assert qb.pq_workspace_bytes(idx, nq, n, R) <= 16 << 20
        got = qb.pq_adc_scan_topk_static(idx, qt, qp, c, R, empty_out(nq, R, -5))
        torch.cuda.synchronize()
        for a, b in zip(want, got):
            assert torch.equal(a, b), (name, nq, n)
    # beyond the array: a clear error, nothing launched
    nq_big, r_big = 64, 2048
    tables = qb.pq_compute_tables(idx, qs[:1].repeat(nq_big, 1).contiguous())
    qt, qp = qb.pq_quantize_tables(idx, tables, codes, 400, r_big)
    assert qb.pq_workspace_bytes(idx, nq_big, codes.shape[0], r_big) > 16 << 20
    with pytest.raises(qb.QadcError) as e:
        qb.pq_adc_scan_topk_static(idx, qt, qp, codes, r_big, empty_out(nq_big, r_big, -5))
    assert e.value.code == qb.PQ_ENOMEM and "scratch" in str(e.value)
    torch.cuda.synchronize()
    idx.close()
