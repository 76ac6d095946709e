"""Pins for oracle/aggregate.py (Sec. 2.3; Appendix B, W = sum_v W_v M_v / sum_v M_v)."""
import numpy as np

from oracle import aggregate as OA
from oracle import partition as OP
from resist_inputs import get_config, make_params


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
            d[key] = {k: (v + rng.standard_normal(v.shape).astype(np.float32)) for k, v in g[key].items()}
        sp.append(d)
    return model, g, subs, owner, sp, B


def test_closed_form_hand_values():
    g = {-1: {"w": np.zeros(2, np.float32)}, 0: {"w": np.zeros(2, np.float32)},
         1: {"w": np.array([7., 7.], np.float32)}, 2: {"w": np.zeros(2, np.float32)}}
    subs = [[0], [0]]                             # B = 2 is the head; block 1 held by nobody
    sp = [{-1: {"w": np.array([1., 2.], np.float32)}, 0: {"w": np.array([1., 1.], np.float32)},
           2: {"w": np.array([0., 4.], np.float32)}},
          {-1: {"w": np.array([3., 6.], np.float32)}, 0: {"w": np.array([2., 5.], np.float32)},
           2: {"w": np.array([2., 0.], np.float32)}}]
    out = OA.aggregate(g, subs, sp)
    np.testing.assert_array_equal(out[-1]["w"], [2., 4.])
    np.testing.assert_array_equal(out[0]["w"], [1.5, 3.])
    np.testing.assert_array_equal(out[2]["w"], [1., 2.])
    np.testing.assert_array_equal(out[1]["w"], [7., 7.])   # unheld: previous value kept


def test_mean_over_holders_and_single_owner_copy():
    model, g, subs, owner, sp, B = _setup()
    out = OA.aggregate(g, subs, sp)
    assert any(o == 1 for o in owner) and any(1 < o < 3 for o in owner)
    for b in range(B):
        holders = [s for s in range(3) if b in subs[s]]
        assert len(holders) == owner[b]
        for k in g[b]:
            if len(holders) == 1:
                assert out[b][k].dtype == np.float32
                assert out[b][k].tobytes() == sp[holders[0]][b][k].tobytes()
            else:
                want = sum(sp[s][b][k].astype(np.float64) for s in holders) / len(holders)
                np.testing.assert_allclose(out[b][k], want, rtol=1e-15)
    for key in (-1, B):                                      # shared by all S (a = sum a_v / S)
        for k in g[key]:
            want = sum(sp[s][key][k].astype(np.float64) for s in range(3)) / 3
            np.testing.assert_allclose(out[key][k], want, rtol=1e-15)


def test_identical_copies_identity_and_linearity():
    model, g, subs, owner, sp, B = _setup()
    same = [{key: {k: g[key][k].copy() for k in g[key]} for key in d} for d in sp]
    out = OA.aggregate(g, subs, same)
    for key in g:
        for k in g[key]:
            np.testing.assert_allclose(out[key][k], g[key][k], rtol=1e-15)
    shifted = [{key: {k: v + 0.5 for k, v in t.items()} for key, t in d.items()} for d in sp]
    a, b = OA.aggregate(g, subs, sp), OA.aggregate(g, subs, shifted)
    for key in g:
        for k in g[key]:
            np.testing.assert_allclose(b[key][k], a[key][k].astype(np.float64) + 0.5, rtol=1e-6, atol=1e-6)


def test_s1_is_copy():
    model, g, subs, owner, sp, B = _setup(S=1)
    out = OA.aggregate(g, subs, sp)
    for key in g:
        for k in g[key]:
            assert out[key][k].tobytes() == sp[0][key][k].tobytes()
