"""Pins for oracle/compress.py (appendix on quantised communication, Table 9: b-bit compression of
the communicated parameters, b = 8 ... 4; reassembly from the compressed copies, Sec. 2.3)."""
import numpy as np
import pytest

from oracle import aggregate as OA
from oracle import compress as OC
from oracle import partition as OP
from resist_inputs import get_config, make_params

BITS = [8, 7, 6, 5, 4]      # the compression levels of Table 9


@pytest.mark.parametrize("bits", BITS + [2])
def test_arithmetic_progression_has_its_index_as_code(bits):
    """w_k = -1 + k / 8 for k = 0..L is exact in fp32 and so is its step: code(w_k) = k, and the
    decoded value is w_k bit for bit (closed form)."""
    L = (1 << bits) - 1
    k = np.arange(L + 1)
    w = (-1.0 + k / 8.0).astype(np.float32)
    perm = np.random.default_rng(bits).permutation(L + 1)
    codes, lo, delta = OC.quantize_tensor(w[perm], bits)
    assert lo == np.float32(-1.0) and delta == np.float32(0.125)
    np.testing.assert_array_equal(codes, k[perm])
    np.testing.assert_array_equal(OC.dequantize_tensor(codes, lo, delta), w[perm].astype(np.float64))


@pytest.mark.parametrize("bits", BITS)
def test_code_is_the_nearest_level_by_brute_force(bits):
    """Brute force in float64: the code is the index of the closest of the L+1 levels, except where
    the value sits within fp32 rounding of the midpoint between two levels."""
    rng = np.random.default_rng(10 + bits)
    w = (0.05 * rng.standard_normal(2000)).astype(np.float32)
    codes, lo, delta = OC.quantize_tensor(w, bits)
    L = (1 << bits) - 1
    lev = np.float64(lo) + np.arange(L + 1) * np.float64(delta)
    dist = np.abs(w.astype(np.float64)[:, None] - lev[None, :])
    nearest = dist.argmin(axis=1)
    two = np.sort(dist, axis=1)[:, :2]
    clear = (two[:, 1] - two[:, 0]) > 1e-5 * float(delta)
    assert clear.mean() > 0.99
    np.testing.assert_array_equal(codes[clear], nearest[clear])
    assert np.all(np.abs(codes.astype(int) - nearest) <= 1)


@pytest.mark.parametrize("bits", BITS)
def test_half_step_error_bound_end_points_and_monotonic(bits):
    rng = np.random.default_rng(20 + bits)
    w = rng.uniform(-3, 5, 4096).astype(np.float32)
    codes, lo, delta = OC.quantize_tensor(w, bits)
    L = (1 << bits) - 1
    assert lo == w.min()
    assert abs(float(delta) - (float(w.max()) - float(w.min())) / L) <= 1e-6 * float(delta)
    back = OC.dequantize_tensor(codes, lo, delta)
    assert np.max(np.abs(back - w)) <= 0.5 * float(delta) * (1 + 1e-5)
    assert np.max(np.abs(back - w)) >= 0.4 * float(delta)          # the bound is attained, not vacuous
    assert codes[w.argmin()] == 0 and codes[w.argmax()] == L
    assert back[w.argmin()] == float(w.min())
    order = np.argsort(w, kind="stable")
    assert np.all(np.diff(codes[order].astype(int)) >= 0)
    assert len(np.unique(codes)) == L + 1                        # every level is used on dense data


def test_fewer_bits_give_coarser_steps():
    w = np.random.default_rng(3).standard_normal(1000).astype(np.float32)
    errs = [np.abs(OC.dequantize_tensor(*OC.quantize_tensor(w, b)) - w).mean() for b in BITS]
    assert all(a < b for a, b in zip(errs, errs[1:]))
    # halving the number of levels doubles the step
    d8, d4 = OC.quantize_tensor(w, 8)[2], OC.quantize_tensor(w, 4)[2]
    assert abs(float(d4) / float(d8) - 255.0 / 15.0) < 1e-5


def test_constant_tensor_and_ties():
    codes, lo, delta = OC.quantize_tensor(np.full(7, 1.0, np.float32), 8)     # BN gamma at initialisation
    assert delta == 0 and lo == 1 and not codes.any()
    np.testing.assert_array_equal(OC.dequantize_tensor(codes, lo, delta), np.ones(7))
    # lo = 0, delta = 1 with b = 2: 0.5 and 2.5 are ties, resolved to the even code
    codes, lo, delta = OC.quantize_tensor(np.array([0, 0.5, 1.5, 2.5, 3], np.float32), 2)
    assert (lo, delta) == (0, 1)
    np.testing.assert_array_equal(codes, [0, 0, 2, 2, 3])
    with pytest.raises(ValueError):
        OC.quantize_tensor(np.zeros(3, np.float32), 9)


def _setup(S=3, seed=0):
    model = dict(get_config("cfg1")["model"], widths=[4, 8], blocks=[3, 3], in_h=8, in_w=8)
    g = make_params(model, seed, perturb_bn=True)
    subs, owner = OP.partition(model["blocks"], S, 0, 5, 0)
    B = sum(model["blocks"])
    rng = np.random.default_rng(seed + 1)
    sp = []
    for s in range(S):
        d = {}
        for key in [-1, B] + subs[s]:
            d[key] = {k: (v + 0.1 * rng.standard_normal(v.shape).astype(np.float32)) for k, v in g[key].items()}
        sp.append(d)
    return g, subs, owner, sp, B


@pytest.mark.parametrize("bits", [8, 4])
def test_reassembly_from_compressed_copies(bits):
    g, subs, owner, sp, B = _setup()
    sq = [{key: OC.quantize_block(t, bits) for key, t in d.items()} for d in sp]
    out = OC.aggregate_quantized(g, subs, sq)
    exact = OA.aggregate(g, subs, sp)
    for key in g:
        holders = [s for s in range(3) if key in (-1, B) or key in subs[s]]
        for name in g[key]:
            if not holders:
                np.testing.assert_array_equal(out[key][name], g[key][name])
                continue
            # the mean of the decoded copies is within the mean half-step of the uncompressed mean
            bound = np.mean([0.5 * float(sq[s][key][name][2]) for s in holders])
            err = np.abs(out[key][name] - np.asarray(exact[key][name], np.float64)).max()
            assert err <= bound * (1 + 1e-5) + 1e-12
            if len(holders) == 1:
                np.testing.assert_array_equal(out[key][name], OC.dequantize_tensor(*sq[holders[0]][key][name]))


def test_reassembly_of_identical_copies_decodes_one_of_them():
    g, subs, owner, sp, B = _setup()
    same = [{key: {k: v.copy() for k, v in g[key].items()} for key in d} for d in sp]
    sq = [{key: OC.quantize_block(t, 6) for key, t in d.items()} for d in same]
    out = OC.aggregate_quantized(g, subs, sq)
    for key in g:
        if key not in (-1, B) and not any(key in s for s in subs):
            continue
        for name in g[key]:
            one = OC.dequantize_tensor(*OC.quantize_tensor(g[key][name], 6))
            np.testing.assert_allclose(out[key][name], one, rtol=1e-15, atol=0)
