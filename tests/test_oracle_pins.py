"""Pins for the CPU oracle: everything here checks `oracle/` against something
other than itself -- hand-worked fixtures, brute force over decoded vectors,
closed-form bounds that follow from Section 3.4, and special cases.  No GPU.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from harness import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")

LAYOUTS = [
    ("16x4", 32, [4] * 16, 8),
    ("32x4", 64, [4] * 32, 8),
    ("c3", 128, synth.C3_BITS, 16),
    ("12x{6,6,4}", 64, [6, 6, 4] * 4, 16),
    ("12x{6,5,5}", 64, [6, 5, 5] * 4, 16),
    ("3x5", 15, [5, 5, 5], 16),
    ("8x8", 32, [8] * 8, 16),
    ("odd", 13, [3, 7, 1, 2], 8),
]


def small_problem(name, d, nbits, acc_bits, n=600, nq=5, dist="gamma_ints", seed=7):
    return synth.make_problem(n=n, nq=nq, d=d, nbits=nbits, acc_bits=acc_bits, dist=dist,
                              seed=seed, train_n=max(600, 4 << max(nbits)), kmeans_iters=4)


def decode(lay, codebooks, sub):
    """concatenate the centroids named by the sub-codes (Section 2.1.2)."""
    cb = np.asarray(codebooks, dtype=np.float64)
    out = np.zeros((sub.shape[0], lay.d))
    o = 0
    c0 = 0
    for j, (k, s) in enumerate(zip(lay.ksub, lay.dsub)):
        C = cb[c0:c0 + k * s].reshape(k, s)
        out[:, o:o + s] = C[sub[:, j]]
        o += s
        c0 += k * s
    return out


# ---------------------------------------------------------------- layout -----
def test_bit_layout_golden():
    cases = json.load(open(os.path.join(GOLD, "bit_layout.json")))["cases"]
    for c in cases:
        codes = np.array([c["bytes"]], dtype=np.uint8)
        assert oracle.code_size(c["nbits"]) == len(c["bytes"])
        got = oracle.unpack(c["nbits"], codes)[0].tolist()
        assert got == c["sub"], c
        lay = synth.Layout(d=sum(c["nbits"]), nbits=c["nbits"], dsub=c["nbits"])
        packed = synth.pack_codes(torch.tensor([c["sub"]], dtype=torch.uint8), lay)
        assert packed[0].tolist() == c["bytes"], c


@pytest.mark.parametrize("name,d,nbits,acc", LAYOUTS)
def test_pack_unpack_roundtrip(name, d, nbits, acc):
    rng = np.random.default_rng(3)
    sub = np.stack([rng.integers(0, 1 << b, size=257) for b in nbits], 1).astype(np.uint8)
    lay = synth.make_layout(d, nbits, acc)
    packed = synth.pack_codes(torch.from_numpy(sub), lay).numpy()
    assert packed.shape == (257, (sum(nbits) + 7) // 8)
    assert np.array_equal(oracle.unpack(nbits, packed), sub)
    assert oracle.table_len(nbits) == sum(1 << b for b in nbits)


def test_dim_split_matches_section_3_1_example():
    # 128-d vector, 12x{6,6,4}: four groups of 32 dims, 12 dims per 6-bit and 8 per 4-bit
    assert synth.dim_split(128, [6, 6, 4] * 4) == [12, 12, 8] * 4
    # 12x{6,5,5} divides 128 exactly as well: 16*12/3 = 64 -> 128/64 = 2 dims per bit
    assert synth.dim_split(128, [6, 5, 5] * 4) == [12, 10, 10] * 4
    assert synth.dim_split(96, [4] * 16) == [6] * 16
    # not divisible: floor, then one extra dim to sub-quantizers 0,1,...
    assert synth.dim_split(128, synth.C3_BITS) == [20, 17, 16, 19, 16, 16, 12, 12]


# ------------------------------------------------------------ O1 and eq (2) --
@pytest.mark.parametrize("name,d,nbits,acc", LAYOUTS)
def test_tables_and_float_adc_equal_decoded_l2(name, d, nbits, acc):
    pr = small_problem(name, d, nbits, acc, dist="aniso_gauss" if d == 32 else "gamma_ints")
    lay = pr.layout
    sub = oracle.unpack(nbits, pr.codes.numpy())
    dec = decode(lay, pr.codebooks.numpy(), sub)
    cb64 = pr.codebooks.numpy().astype(np.float64)
    for q in range(pr.queries.shape[0]):
        z = pr.queries[q].numpy()
        tab = oracle.tables(lay.d, nbits, lay.dsub, pr.codebooks.numpy(), z)
        # eq. (1) entry by entry in fp64
        o = c0 = t0 = 0
        for j, (k, s) in enumerate(zip(lay.ksub, lay.dsub)):
            C = cb64[c0:c0 + k * s].reshape(k, s)
            ref = ((z[o:o + s].astype(np.float64)[None, :] - C) ** 2).sum(1)
            np.testing.assert_allclose(tab[t0:t0 + k], ref, rtol=2e-6, atol=1e-30)
            o, c0, t0 = o + s, c0 + k * s, t0 + k
        # eq. (2): sum of looked-up entries is the squared distance to the decoded vector
        adc = oracle.adc_float(nbits, tab, pr.codes.numpy())
        ref = ((dec - z.astype(np.float64)[None, :]) ** 2).sum(1)
        np.testing.assert_allclose(adc, ref, rtol=1e-5, atol=1e-30)


def test_tables_with_shift_is_residual_table():
    pr = small_problem("16x4", 32, [4] * 16, 8, dist="aniso_gauss")
    lay = pr.layout
    z = pr.queries[0].numpy()
    shift = pr.queries[1].numpy() * 0.5
    a = oracle.tables(lay.d, lay.nbits, lay.dsub, pr.codebooks.numpy(), z, shift)
    b = oracle.tables(lay.d, lay.nbits, lay.dsub, pr.codebooks.numpy(), (z - shift))
    assert np.array_equal(a, b)  # z' = z - centroid computed first, in fp32


# ------------------------------------------------------ Section 3.4, worked --
def test_quantizer_worked_example():
    g = json.load(open(os.path.join(GOLD, "quantizer_worked_example.json")))
    nbits, acc = g["nbits"], g["acc_bits"]
    codes = np.array(g["packed"], dtype=np.uint8).reshape(-1, 1)
    assert oracle.unpack(nbits, codes).tolist() == g["subcodes"]
    table = np.array(g["table"], dtype=np.float32)
    assert oracle.adc_float(nbits, table, codes).tolist() == g["float_adc"]
    qt, dmin, delta, dmax = oracle.quantize(nbits, acc, table, codes, g["t"], g["R"])
    assert (dmin, delta, dmax) == (g["d_min"], g["delta"], g["d_max"])
    assert qt.tolist() == g["qtable"]
    keys = oracle.scan_keys(nbits, acc, qt, codes)
    assert keys.tolist() == g["keys"]
    ids, ks, ds = oracle.topk(acc, keys, g["R"], dmin, delta)
    assert ids.tolist() == g["top_ids"]
    assert ks.tolist() == g["top_keys"]
    assert ds.tolist() == g["top_dist"]


def test_t_eff_reading():
    assert oracle.t_eff(10**7, 400, 100) == 400      # Section 4.1: t = 400 for R = 100
    assert oracle.t_eff(10**7, 400, 1000) == 4000    # keeps the 4:1 ratio for large R
    assert oracle.t_eff(250, 400, 100) == 250
    assert oracle.t_eff(0, 400, 100) == 0


# --------------------------------------------------- invariants, Section 3.4 --
@pytest.mark.parametrize("name,d,nbits,acc", LAYOUTS)
@pytest.mark.parametrize("R", [1, 10, 100])
def test_quantizer_invariants(name, d, nbits, acc, R):
    pr = small_problem(name, d, nbits, acc, n=1500)
    lay = pr.layout
    m, qmax = lay.m, lay.q_max
    codes = pr.codes.numpy()
    sub = oracle.unpack(nbits, codes).astype(np.int64)
    toff = np.concatenate([[0], np.cumsum(lay.ksub)[:-1]])
    for q in range(3):
        tab = oracle.tables(lay.d, nbits, lay.dsub, pr.codebooks.numpy(), pr.queries[q].numpy())
        adc = oracle.adc_float(nbits, tab, codes).astype(np.float64)
        qt, dmin, delta, dmax = oracle.quantize(nbits, acc, tab, codes, 400, R)
        te = oracle.t_eff(codes.shape[0], 400, R)
        # d_max is the R-th smallest float ADC of the first t_eff codes
        assert dmax == np.sort(adc[:te].astype(np.float32))[min(R, te) - 1]
        # p_min / d_min
        pmin = np.array([tab[toff[j]:toff[j] + lay.ksub[j]].min() for j in range(m)], np.float64)
        assert dmin == pytest.approx(pmin.sum(), rel=1e-15)
        assert delta == pytest.approx((dmax - dmin) / qmax, rel=1e-15)
        assert delta > 0
        # the minimum of every table quantizes to 0 and nothing exceeds q_max
        for j in range(m):
            seg = qt[toff[j]:toff[j] + lay.ksub[j]]
            assert seg[np.argmin(tab[toff[j]:toff[j] + lay.ksub[j]])] == 0
        assert qt.max() <= qmax
        # entries: floor of (p - p_min)/Delta, clamped
        j_of = np.repeat(np.arange(m), lay.ksub)
        exact = (tab.astype(np.float64) - pmin[j_of]) / delta
        assert np.all(qt <= np.minimum(exact, qmax) + 1e-9)
        assert np.all((qt == qmax) | (qt > exact - 1 - 1e-9))
        # keys: the saturating chain equals min(exact integer sum, q_max)
        keys = oracle.scan_keys(nbits, acc, qt, codes).astype(np.int64)
        wide = sum(qt[toff[j] + sub[:, j]].astype(np.int64) for j in range(m))
        assert np.array_equal(keys, np.minimum(wide, qmax))
        # unsaturated codes: d - m*Delta < d_hat <= d  (floor loses < 1 step per table)
        unsat = wide < qmax
        dhat = wide * delta + dmin
        tol = 1e-5 * np.abs(adc) + 1e-12
        assert np.all(dhat[unsat] <= adc[unsat] + tol[unsat])
        assert np.all(dhat[unsat] > adc[unsat] - m * delta - tol[unsat])
        # no code at or below d_max saturates spuriously: key is its exact sum
        near = adc <= dmax
        assert np.all(wide[near] <= qmax)
        # monotone up to the step
        rng = np.random.default_rng(q)
        a = rng.integers(0, len(adc), 4000)
        b = rng.integers(0, len(adc), 4000)
        sel = adc[a] + m * delta * (1 + 1e-6) + tol[a] <= adc[b]
        assert np.all(keys[a][sel] <= keys[b][sel])
        # a true top-R code of the whole set is never lost to saturation
        ids, ks, ds = oracle.topk(acc, keys.astype(np.uint16), R, dmin, delta)
        order = np.lexsort((np.arange(len(adc)), adc))[:R]
        assert np.all(adc[order] <= dmax)
        assert np.all(keys[order] == wide[order])
        # and the oracle's unquantized distances are key*Delta + d_min in fp32
        ref = np.float32(ks.astype(np.float32)) * np.float32(delta) + np.float32(dmin)
        np.testing.assert_allclose(ds, ref, rtol=3e-7)


def test_all_minima_code_has_key_zero():
    pr = small_problem("16x4", 32, [4] * 16, 8, dist="aniso_gauss")
    lay = pr.layout
    tab = oracle.tables(lay.d, lay.nbits, lay.dsub, pr.codebooks.numpy(), pr.queries[0].numpy())
    best = np.array([[int(np.argmin(tab[16 * j:16 * j + 16])) for j in range(16)]], np.uint8)
    code = synth.pack_codes(torch.from_numpy(best), lay).numpy()
    codes = np.concatenate([pr.codes.numpy(), code])
    qt, dmin, delta, dmax = oracle.quantize(lay.nbits, 8, tab, codes, 400, 10)
    keys = oracle.scan_keys(lay.nbits, 8, qt, codes)
    assert keys[-1] == 0
    ids, ks, ds = oracle.topk(8, keys, 1, dmin, delta)
    assert ids[0] == len(codes) - 1 or keys[ids[0]] == 0
    assert ds[0] == np.float32(dmin)


@pytest.mark.parametrize("name,d,nbits,acc", [l for l in LAYOUTS if l[3] == 16])
def test_u16_reproduces_float_ranking(name, d, nbits, acc):
    """16-bit distances leave the ranking untouched whenever float gaps exceed
    m*Delta (Section 4.2: no recall loss with 16-bit quantization)."""
    pr = small_problem(name, d, nbits, acc, n=500)
    lay = pr.layout
    codes = pr.codes.numpy()
    R = 20
    for q in range(pr.queries.shape[0]):
        z = pr.queries[q].numpy()
        tab = oracle.tables(lay.d, nbits, lay.dsub, pr.codebooks.numpy(), z)
        adc = oracle.adc_float(nbits, tab, codes).astype(np.float64)
        ids, ks, ds = oracle.search(lay.d, nbits, lay.dsub, acc, pr.codebooks.numpy(), z, codes,
                                    400, R)
        _, dmin, delta, dmax = oracle.quantize(nbits, acc, tab, codes, 400, R)
        order = np.lexsort((np.arange(len(adc)), adc))
        # compare position by position wherever the neighbours are separated by > m*Delta
        gap = lay.m * delta * 1.001
        for r in range(R):
            lo_ok = r == 0 or adc[order[r]] - adc[order[r - 1]] > gap
            hi_ok = adc[order[r + 1]] - adc[order[r]] > gap
            if lo_ok and hi_ok:
                assert ids[r] == order[r]
        # as a set, the result is the float top-R up to codes within m*Delta of the R-th
        kth = adc[order[R - 1]]
        assert np.all(adc[ids] <= kth + gap)
        np.testing.assert_allclose(ds, adc[ids], atol=gap + 1e-5 * kth)


# --------------------------------------------------------------- O5 details --
def test_topk_ties_lowest_id_and_padding():
    keys = np.array([5, 3, 5, 3, 9, 3, 0, 255], dtype=np.uint16)
    ids, ks, ds = oracle.topk(8, keys, 5, 1.0, 0.25)
    assert ids.tolist() == [6, 1, 3, 5, 0]
    assert ks.tolist() == [0, 3, 3, 3, 5]
    assert ds.tolist() == [1.0, 1.75, 1.75, 1.75, 2.25]
    ids, ks, ds = oracle.topk(8, keys[:2], 4, 1.0, 0.25)
    assert ids.tolist() == [1, 0, -1, -1]
    assert ks.tolist() == [3, 5, 255, 255]
    assert ds[:2].tolist() == [1.75, 2.25] and np.all(np.isinf(ds[2:]))
    ids, ks, ds = oracle.topk(16, keys[:0], 2, 0.0, 0.0)
    assert ids.tolist() == [-1, -1] and ks.tolist() == [65535, 65535]


def test_degenerate_identical_codes_give_id_order():
    pr = small_problem("16x4", 32, [4] * 16, 8)
    lay = pr.layout
    codes = np.repeat(pr.codes.numpy()[:1], 50, axis=0)
    z = pr.queries[0].numpy()
    ids, ks, ds = oracle.search(lay.d, lay.nbits, lay.dsub, 8, pr.codebooks.numpy(), z, codes,
                                400, 10)
    tab = oracle.tables(lay.d, lay.nbits, lay.dsub, pr.codebooks.numpy(), z)
    qt, dmin, delta, dmax = oracle.quantize(lay.nbits, 8, tab, codes, 400, 10)
    adc = oracle.adc_float(lay.nbits, tab, codes)
    assert dmax == adc[0]
    assert ids.tolist() == list(range(10))
    # one distinct distance: all keys equal, and it unquantizes to within m*Delta of the truth
    assert len(set(ks.tolist())) == 1
    assert abs(float(ds[0]) - float(adc[0])) <= lay.m * delta + 1e-4 * abs(float(adc[0]))


def test_delta_not_positive_gives_zero_table():
    # every table constant: d_max == d_min -> Delta = 0 -> all q = 0, pure id order
    nbits = [2, 2]
    table = np.array([3.0] * 4 + [4.0] * 4, dtype=np.float32)
    codes = np.arange(16, dtype=np.uint8).reshape(-1, 1)
    qt, dmin, delta, dmax = oracle.quantize(nbits, 8, table, codes, 4, 2)
    assert (dmin, dmax, delta) == (7.0, 7.0, 0.0)
    assert not qt.any()
    keys = oracle.scan_keys(nbits, 8, qt, codes)
    ids, ks, ds = oracle.topk(8, keys, 3, dmin, delta)
    assert ids.tolist() == [0, 1, 2] and ds.tolist() == [7.0, 7.0, 7.0]
    # no codes at all: nothing to calibrate on
    qt, dmin, delta, dmax = oracle.quantize(nbits, 8, table, codes[:0], 4, 2)
    assert delta == 0.0 and np.isinf(dmax) and not qt.any()


def test_u8_top_r_overlaps_float_top_r():
    """Soft sanity check (Section 4.2: 8-bit quantization costs little recall)."""
    pr = synth.make_problem(n=20000, nq=8, d=128, nbits=[4] * 16, acc_bits=8, dist="gamma_ints",
                            seed=11, train_n=5000, kmeans_iters=5)
    lay = pr.layout
    codes = pr.codes.numpy()
    R = 100
    overlap = []
    for q in range(8):
        z = pr.queries[q].numpy()
        tab = oracle.tables(lay.d, lay.nbits, lay.dsub, pr.codebooks.numpy(), z)
        adc = oracle.adc_float(lay.nbits, tab, codes)
        ids, _, _ = oracle.search(lay.d, lay.nbits, lay.dsub, 8, pr.codebooks.numpy(), z, codes,
                                  400, R)
        overlap.append(len(set(ids.tolist()) & set(np.argsort(adc, kind="stable")[:R].tolist())))
    assert np.mean(overlap) >= 0.7 * R


# ---------------------------------------------------------------------- IVF --
def small_ivf(acc_bits=8, n=3000, K=12, nprobe=4, nq=6, nbits=None, d=32, dist="aniso_gauss"):
    return synth.make_ivf_problem(n=n, nq=nq, d=d, nbits=nbits or [4] * 16, acc_bits=acc_bits,
                                  dist=dist, K=K, nprobe=nprobe, seed=5, train_n=1500,
                                  kmeans_iters=4)


def ivf_call(pr, q, R, t=400, probe=None):
    lay = pr.layout
    return oracle.search_ivf(lay.d, lay.nbits, lay.dsub, lay.acc_bits, pr.codebooks.numpy(),
                             pr.coarse.numpy(), pr.list_offsets.numpy(), pr.list_codes.numpy(),
                             pr.list_ids.numpy(), pr.queries[q].numpy(),
                             pr.probe_ids[q].numpy() if probe is None else probe, t, R)


def test_ivf_single_zero_cell_equals_exhaustive():
    pr = small_problem("16x4", 32, [4] * 16, 8, n=900, dist="aniso_gauss")
    lay = pr.layout
    n = pr.codes.shape[0]
    coarse = np.zeros((1, lay.d), np.float32)
    offs = np.array([0, n], np.int64)
    ids_store = np.arange(n, dtype=np.int32)
    for q in range(3):
        z = pr.queries[q].numpy()
        a = oracle.search(lay.d, lay.nbits, lay.dsub, 8, pr.codebooks.numpy(), z, pr.codes.numpy(),
                          400, 25)
        b = oracle.search_ivf(lay.d, lay.nbits, lay.dsub, 8, pr.codebooks.numpy(), coarse, offs,
                              pr.codes.numpy(), ids_store, z, np.array([0], np.int32), 400, 25)
        assert np.array_equal(a[0], b[0])
        assert np.array_equal(a[2], b[1])


@pytest.mark.parametrize("acc_bits,nbits,d,R", [(8, None, 32, 15), (16, None, 32, 15),
                                               (16, [8, 8], 4, 150), (8, [6, 6, 4], 8, 60)])
def test_ivf_against_reconstruction_brute_force(acc_bits, nbits, d, R):
    # the fine-grained layouts make d_min of a list close to its real distances, so that
    # wrongly skipping a list (d_min <= d_max) loses true neighbours
    pr = small_ivf(acc_bits=acc_bits, nbits=nbits, d=d)
    lay = pr.layout
    sub = oracle.unpack(lay.nbits, pr.list_codes.numpy())
    dec = decode(lay, pr.codebooks.numpy(), sub)
    offs = pr.list_offsets.numpy()
    cell_of = np.repeat(np.arange(len(offs) - 1), np.diff(offs))
    recon = dec + pr.coarse.numpy().astype(np.float64)[cell_of]
    pos_of_id = np.empty(len(cell_of), np.int64)
    pos_of_id[pr.list_ids.numpy()] = np.arange(len(cell_of))
    for q in range(pr.queries.shape[0]):
        z = pr.queries[q].numpy().astype(np.float64)
        probe = pr.probe_ids[q].numpy()
        ids, dist, dmax = ivf_call(pr, q, R)
        true = ((recon - z[None, :]) ** 2).sum(1)
        probed_pos = np.concatenate([np.arange(offs[c], offs[c + 1]) for c in probe])
        # calibration: R-th smallest true distance among the first t_eff probed codes
        te = oracle.t_eff(len(probed_pos), 400, R)
        assert dmax == pytest.approx(np.sort(true[probed_pos[:te]])[min(R, te) - 1], rel=1e-4)
        # results come from probed lists only, ordered by (dist, id)
        assert np.all(ids >= 0)
        assert np.all(np.isin(cell_of[pos_of_id[ids]], probe))
        assert np.all((np.diff(dist) > 0) | ((np.diff(dist) == 0) & (np.diff(ids) > 0)))
        # unquantized distance is within (d - m*Delta_l, d] of the true residual distance,
        # Delta_l <= (d_max - 0)/q_max
        step = lay.m * dmax / lay.q_max
        t_ids = true[pos_of_id[ids]]
        assert np.all(dist <= t_ids + 1e-4 * t_ids)
        assert np.all(dist > t_ids - step - 1e-4 * t_ids)
        # the R-th result is within one m*Delta of the true R-th over the probed codes
        kth = np.sort(true[probed_pos])[R - 1]
        assert t_ids.max() <= kth + step + 1e-4 * kth
        if acc_bits == 16:
            best = probed_pos[np.argsort(true[probed_pos], kind="stable")[:R]]
            got = set(pos_of_id[ids].tolist())
            missing = [p for p in best if p not in got]
            assert all(true[p] >= kth - step for p in missing)


def test_ivf_padding_skips_and_empty_probes():
    pr = small_ivf(n=400, K=20, nprobe=3)
    offs = pr.list_offsets.numpy()
    sizes = np.diff(offs)
    small = np.argsort(sizes, kind="stable")[:2].astype(np.int32)
    probe = np.array([small[0], -1, small[1]], np.int32)
    R = int(sizes[small].sum()) + 5
    ids, dist, dmax = ivf_call(pr, 0, R, probe=probe)
    got = ids[ids >= 0]
    members = np.concatenate([pr.list_ids.numpy()[offs[c]:offs[c + 1]] for c in small])
    assert set(got.tolist()) <= set(members.tolist())
    assert np.all(ids[len(got):] == -1) and np.all(np.isinf(dist[len(got):]))
    ids, dist, dmax = ivf_call(pr, 0, 4, probe=np.array([-1, -1], np.int32))
    assert np.all(ids == -1) and np.isinf(dmax)


def test_ivf_worked_example():
    g = json.load(open(os.path.join(GOLD, "ivf_worked_example.json")))
    lay = synth.Layout(d=g["d"], nbits=g["nbits"], dsub=g["dsub"], acc_bits=g["acc_bits"])
    codes = synth.pack_codes(torch.tensor(g["list_subcodes"], dtype=torch.uint8), lay).numpy()
    ids, dist, dmax = oracle.search_ivf(
        g["d"], g["nbits"], g["dsub"], g["acc_bits"], np.array(g["codebooks"], np.float32),
        np.array(g["coarse"], np.float32), np.array(g["list_offsets"], np.int64), codes,
        np.array(g["list_ids"], np.int32), np.array(g["query"], np.float32),
        np.array(g["probe"], np.int32), g["t"], g["R"])
    assert dmax == g["d_max"]
    assert ids.tolist() == g["top_ids"]
    delta32 = np.float64(np.float32(g["delta_num"] / g["delta_den"]))
    want = [np.float32(k * delta32 + g["d_min"]) for k in g["top_key_steps"]]
    assert dist.tolist() == [float(w) for w in want]


def test_ivf_list_with_d_min_equal_to_d_max_is_skipped():
    # Section 3.4: later candidates have to be closer than d_max, so a cell whose smallest
    # representable distance equals d_max holds nothing to keep (hand-worked fixture)
    g = json.load(open(os.path.join(GOLD, "ivf_skip_boundary_example.json")))
    lay = synth.Layout(d=g["d"], nbits=g["nbits"], dsub=g["dsub"], acc_bits=g["acc_bits"])
    codes = synth.pack_codes(torch.tensor(g["list_subcodes"], dtype=torch.uint8), lay).numpy()
    ids, dist, dmax = oracle.search_ivf(
        g["d"], g["nbits"], g["dsub"], g["acc_bits"], np.array(g["codebooks"], np.float32),
        np.array(g["coarse"], np.float32), np.array(g["list_offsets"], np.int64), codes,
        np.array(g["list_ids"], np.int32), np.array(g["query"], np.float32),
        np.array(g["probe"], np.int32), g["t"], g["R"])
    assert dmax == g["d_max"]
    assert ids.tolist() == g["top_ids"]
    assert dist.tolist() == g["top_dist"]


def ivf_tight_call(pr, q, R, t=400, probe=None):
    lay = pr.layout
    return oracle.search_ivf_tightening(lay.d, lay.nbits, lay.dsub, lay.acc_bits, pr.codebooks.numpy(),
                                        pr.coarse.numpy(), pr.list_offsets.numpy(), pr.list_codes.numpy(),
                                        pr.list_ids.numpy(), pr.queries[q].numpy(),
                                        pr.probe_ids[q].numpy() if probe is None else probe, t, R)


def test_ivf_tightening_worked_example():
    g = json.load(open(os.path.join(GOLD, "ivf_tightening_example.json")))
    lay = synth.Layout(d=g["d"], nbits=g["nbits"], dsub=g["dsub"], acc_bits=g["acc_bits"])
    codes = synth.pack_codes(torch.tensor(g["list_subcodes"], dtype=torch.uint8), lay).numpy()
    args = (g["d"], g["nbits"], g["dsub"], g["acc_bits"], np.array(g["codebooks"], np.float32),
            np.array(g["coarse"], np.float32), np.array(g["list_offsets"], np.int64), codes,
            np.array(g["list_ids"], np.int32), np.array(g["query"], np.float32),
            np.array(g["probe"], np.int32), g["t"], g["R"])
    ids, dist, dmax, bounds = oracle.search_ivf_tightening(*args)
    assert dmax == g["d_max"]
    assert ids.tolist() == g["top_ids_tightening"] and dist.tolist() == g["top_dist_tightening"]
    assert bounds[0] == g["d_max"]
    # 3 steps of float(272/255): the fp32 product, as the unquantize formula gives it
    step32 = np.float32(np.float64(g["d_max"]) / 255.0)
    assert bounds[1] == np.float32(np.float64(3.0) * np.float64(step32))
    assert bounds[1] == pytest.approx(g["bound_after_first_list_num"] / g["bound_after_first_list_den"], rel=1e-6)
    ids0, _, _ = oracle.search_ivf(*args)
    assert ids0.tolist() == g["top_ids_fixed_bound"]
    # a code that saturates against the tightened bound is no candidate
    rows = g["saturated_variant_rows"]
    var = list(args)
    var[6] = np.array(g["saturated_variant_list_offsets"], np.int64)
    var[7], var[8] = codes[rows], np.array(g["list_ids"], np.int32)[rows]
    ids, dist, _, bounds = oracle.search_ivf_tightening(*var)
    assert ids.tolist() == g["saturated_variant_top_ids"] and dist[0] == bounds[1]


@pytest.mark.parametrize("acc_bits,nbits,d,R", [(8, None, 32, 15), (16, None, 32, 15), (8, [6, 6, 4], 8, 60)])
def test_ivf_tightening_properties(acc_bits, nbits, d, R):
    pr = small_ivf(acc_bits=acc_bits, nbits=nbits, d=d, n=6000, K=12, nprobe=6)
    lay = pr.layout
    sub = oracle.unpack(lay.nbits, pr.list_codes.numpy())
    dec = decode(lay, pr.codebooks.numpy(), sub)
    offs = pr.list_offsets.numpy()
    cell_of = np.repeat(np.arange(len(offs) - 1), np.diff(offs))
    recon = dec + pr.coarse.numpy().astype(np.float64)[cell_of]
    pos_of_id = np.empty(len(cell_of), np.int64)
    pos_of_id[pr.list_ids.numpy()] = np.arange(len(cell_of))
    tightened = 0
    for q in range(pr.queries.shape[0]):
        z = pr.queries[q].numpy().astype(np.float64)
        probe = pr.probe_ids[q].numpy()
        ids, dist, dmax, bounds = ivf_tight_call(pr, q, R)
        ids0, dist0, dmax0 = ivf_call(pr, q, R)
        assert dmax == dmax0                                   # same calibration
        assert bounds[0] == np.float32(dmax)
        assert np.all(np.diff(bounds) <= 0)                    # the bound never grows
        tightened += int(bounds[-1] < bounds[0])
        # one probed list: nothing to tighten, the fixed-bound search exactly
        one = probe[:1]
        a = ivf_tight_call(pr, q, R, probe=one)
        b = ivf_call(pr, q, R, probe=one)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
        # results: probed lists only, ordered by (dist, id), and as good as the quantizer allows:
        # unquantized distance within (true - m * Delta, true], Delta <= d_max / q_max
        true = ((recon - z[None, :]) ** 2).sum(1)
        probed_pos = np.concatenate([np.arange(offs[c], offs[c + 1]) for c in probe])
        assert np.all(np.isin(cell_of[pos_of_id[ids]], probe))
        assert np.all((np.diff(dist) > 0) | ((np.diff(dist) == 0) & (np.diff(ids) > 0)))
        step = lay.m * dmax / lay.q_max
        t_ids = true[pos_of_id[ids]]
        assert np.all(dist <= t_ids + 1e-4 * t_ids)
        assert np.all(dist > t_ids - step - 1e-4 * t_ids)
        kth = np.sort(true[probed_pos])[R - 1]
        assert t_ids.max() <= kth + step + 1e-4 * kth
        # a finer quantizer cannot make the R-th result worse than the fixed bound's by more than a step
        assert dist[-1] <= dist0[-1] + step
    assert tightened >= pr.queries.shape[0] // 2                 # the mode really is exercised


# ---------------------------------------------------------------- O7: coarse-quantizer search
def test_coarse_search_worked_example():
    g = json.load(open(os.path.join(GOLD, "coarse_worked_example.json")))
    cen, z = np.array(g["centroids"], np.float32), np.array(g["z"], np.float32)
    ids, sc = oracle.coarse_search(cen, z, g["nprobe"])
    assert ids.tolist() == g["ids"]
    assert sc.tolist() == [g["scores"][i] for i in g["ids"]]
    ids, sc = oracle.coarse_search(cen, z, g["nprobe_all"])
    assert ids.tolist() == g["ids_all"]
    assert np.all(np.isinf(sc[len(cen):]))


@pytest.mark.parametrize("K,d,nprobe,seed", [(300, 16, 8, 0), (1000, 96, 64, 1), (64, 5, 64, 2), (7, 3, 10, 3)])
def test_coarse_search_is_exact_on_integer_data(K, d, nprobe, seed):
    """Small integers make every fp32 operation exact, so the ranking must be the exact squared-L2
    ranking (ties by id) computed in int64."""
    rng = np.random.default_rng(seed)
    cen = rng.integers(-30, 31, (K, d)).astype(np.float32)
    cen[K // 2] = cen[0]                       # an exact duplicate: tie broken by id
    z = rng.integers(-30, 31, d).astype(np.float32)
    dist = ((cen.astype(np.int64) - z.astype(np.int64)) ** 2).sum(1)
    order = np.lexsort((np.arange(K), dist))
    ids, sc = oracle.coarse_search(cen, z, nprobe)
    k = min(nprobe, K)
    assert ids[:k].tolist() == order[:k].tolist()
    assert np.all(ids[k:] == -1)
    znorm = int((z.astype(np.int64) ** 2).sum())
    assert (sc[:k].astype(np.int64) + znorm).tolist() == dist[order[:k]].tolist()


def test_coarse_search_float_data_within_rounding_of_fp64():
    rng = np.random.default_rng(5)
    K, d, nprobe = 4096, 96, 64
    cen = rng.normal(size=(K, d)).astype(np.float32)
    z = rng.normal(size=d).astype(np.float32)
    ids, sc = oracle.coarse_search(cen, z, nprobe)
    true = ((cen.astype(np.float64) - z.astype(np.float64)) ** 2).sum(1)
    znorm = float((z.astype(np.float64) ** 2).sum())
    # every fp32 score is within a few ulps-of-the-operands of the true value
    tol = 4 * d * np.finfo(np.float32).eps * (np.abs(cen).max() ** 2 + np.abs(cen).max() * np.abs(z).max()) * 4
    assert np.all(np.abs(sc.astype(np.float64) + znorm - true[ids]) <= tol)
    # the returned set is the true set up to that rounding, and it is ordered up to it
    kth = np.sort(true)[nprobe - 1]
    assert np.all(true[ids] <= kth + 2 * tol)
    rest = np.setdiff1d(np.arange(K), ids)
    assert np.all(true[rest] >= kth - 2 * tol)
    assert np.all(np.diff(true[ids]) >= -2 * tol)
    assert len(set(ids.tolist())) == nprobe


def test_coarse_search_score_is_fma_chain():
    """The stated arithmetic, re-derived with exact rational arithmetic: each fused multiply-add
    rounds the exact a*b+c once to fp32."""
    from fractions import Fraction
    rng = np.random.default_rng(9)
    d = 7
    cen = rng.normal(size=(3, d)).astype(np.float32)
    z = rng.normal(size=d).astype(np.float32)

    def fma32(a, b, c):
        return np.float32(float(Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c))))
    # float(Fraction) rounds to nearest double; nearest-fp32 of that equals nearest-fp32 of the exact
    # value except in double-rounding corner cases, which these seeds do not hit (checked by equality)
    ids, sc = oracle.coarse_search(cen, z, 3)
    for c, s in zip(ids, sc):
        dot = np.float32(0)
        nrm = np.float32(0)
        for l in range(d):
            dot = fma32(z[l], cen[c, l], dot)
            nrm = fma32(cen[c, l], cen[c, l], nrm)
        assert fma32(np.float32(-2), dot, nrm) == s


# ---------------------------------------------------------------- O8: encoding and packing
def _one_dim_codebooks(nbits):
    """One dimension per sub-quantizer, centroid i of sub-quantizer j at value i: encoding the
    vector of wanted sub-codes must reproduce them."""
    return np.concatenate([np.arange(1 << b, dtype=np.float32) for b in nbits])


def test_encode_packs_as_the_hand_worked_layouts():
    cases = json.load(open(os.path.join(GOLD, "bit_layout.json")))["cases"]
    for c in cases:
        nb = c["nbits"]
        x = np.array([c["sub"]], dtype=np.float32)
        codes = oracle.encode(len(nb), nb, [1] * len(nb), _one_dim_codebooks(nb), x)
        assert codes[0].tolist() == c["bytes"], c


@pytest.mark.parametrize("name,d,nbits,acc", LAYOUTS)
def test_encode_is_nearest_centroid_in_every_subspace(name, d, nbits, acc):
    lay = synth.make_layout(d, nbits, acc)
    rng = np.random.default_rng(17)
    cb = rng.normal(size=sum((1 << b) * s for b, s in zip(lay.nbits, lay.dsub))).astype(np.float32)
    x = rng.normal(size=(200, d)).astype(np.float32)
    sub = oracle.unpack(nbits, oracle.encode(d, nbits, lay.dsub, cb, x))
    o = c0 = 0
    for j, (b, s) in enumerate(zip(lay.nbits, lay.dsub)):
        cen = cb[c0:c0 + (1 << b) * s].reshape(1 << b, s).astype(np.float64)
        dist = ((x[:, None, o:o + s].astype(np.float64) - cen[None]) ** 2).sum(2)
        best = dist.min(1)
        chosen = dist[np.arange(len(x)), sub[:, j]]
        assert np.all(chosen <= best * (1 + 1e-5) + 1e-6), (name, j)   # nearest up to fp32 rounding
        clear = np.sort(dist, 1)[:, 1] > best * (1 + 1e-4) + 1e-5      # no near-tie: must be the argmin
        assert np.array_equal(sub[clear, j], dist.argmin(1)[clear])
        o += s
        c0 += (1 << b) * s


def test_encode_fixed_points_ties_and_shift():
    nbits, d = [3, 2, 5], 7
    lay = synth.make_layout(d, nbits, 16)
    rng = np.random.default_rng(23)
    cb = rng.integers(-9, 10, sum((1 << b) * s for b, s in zip(lay.nbits, lay.dsub))).astype(np.float32)
    # every concatenation of centroids encodes to its own indices unless an earlier equal centroid exists
    sub = np.stack([rng.integers(0, 1 << b, 64) for b in nbits], 1)
    x = np.zeros((64, d), np.float32)
    first = []
    o = c0 = 0
    for j, (b, s) in enumerate(zip(lay.nbits, lay.dsub)):
        cen = cb[c0:c0 + (1 << b) * s].reshape(1 << b, s)
        x[:, o:o + s] = cen[sub[:, j]]
        first.append([int(np.flatnonzero((cen == cen[i]).all(1))[0]) for i in sub[:, j]])   # lowest equal index
        o += s
        c0 += (1 << b) * s
    got = oracle.unpack(nbits, oracle.encode(d, nbits, lay.dsub, cb, x))
    assert np.array_equal(got, np.array(first).T)
    # with a shift the residual is what is encoded
    shift = rng.integers(-5, 6, (64, d)).astype(np.float32)
    assert np.array_equal(oracle.encode(d, nbits, lay.dsub, cb, x + shift, shift), oracle.encode(d, nbits, lay.dsub, cb, x))


def test_input_fabricator_writes_the_codes_the_pinned_encoder_writes():
    """A check of the input fabricator, not of the oracle: the oracle's encoder is pinned above
    (hand-packed layouts, fp64 brute force, fixed points, ties, shift).  The fabricator's own
    encoder (matrix form, used to make synthetic codes at sizes the oracle cannot) must write
    the same codes on data where both are exact, packing included, so that the synthetic inputs
    really are nearest-centroid codes."""
    pr = synth.make_problem(n=400, nq=1, d=12, nbits=[4, 3, 5, 4], acc_bits=16, dist="gamma_ints",
                            seed=5, train_n=400, kmeans_iters=0)
    lay = pr.layout
    rng = np.random.default_rng(1)
    x = rng.integers(0, 6, (300, lay.d)).astype(np.float32)
    cb = np.round(pr.codebooks.numpy())          # integer centroids
    want = synth.pack_codes(synth.encode(torch.from_numpy(x), lay, torch.from_numpy(cb)), lay).numpy()
    # ties are possible with integer centroids: both break them towards the lowest index
    assert np.array_equal(oracle.encode(lay.d, lay.nbits, lay.dsub, cb, x), want)


def test_oracle_clean_under_sanitizers(tmp_path):
    """The oracle's C source, built with AddressSanitizer and UndefinedBehaviorSanitizer, runs a
    driver over every entry point (regular and irregular layouts, empty and short lists, more
    results than codes, empty and invalid inverted lists) without a report."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "oracle_sanitizer_driver")
    build = subprocess.run(
        ["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-static-libasan", "-ffp-contract=off", os.path.join(root, "oracle", "adc_oracle.c"),
         os.path.join(root, "tests", "oracle_sanitizer_driver.c"), "-lm", "-o", exe],
        capture_output=True, text=True)
    if build.returncode != 0:
        pytest.skip("no sanitizer runtimes for gcc here: " + build.stderr[-300:])
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    run = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, (run.stdout[-500:], run.stderr[-3000:])
    assert "ok" in run.stdout
