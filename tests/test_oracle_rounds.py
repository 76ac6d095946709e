"""Pins for oracle/rounds.py: the composition partition -> local steps -> aggregation (Algorithm 1)."""
import numpy as np

from oracle import partition as OP
from oracle import resnet as OR
from oracle import rounds as ORD
from resist_inputs import get_config, make_batch, make_params, zeros_like_params


def _model():
    return dict(get_config("cfg1")["model"], widths=[8, 16], blocks=[2, 4], in_h=8, in_w=8, num_classes=5)


def _batch_fn(model, batch):
    return lambda t, s, it: make_batch(model, batch, 10000 * t + 100 * s + it)


def test_single_subresnet_is_plain_sgd_with_momentum_restart():
    model = _model()
    params = make_params(model, 0, perturb_bn=True)
    B = sum(model["blocks"])
    fn = _batch_fn(model, 3)
    got, log = ORD.run_rounds(model, params, 1, 0, 5, 2, 2, fn, 0.05, 0.9, 1e-3)
    p = params
    for t in range(2):
        v = zeros_like_params(params)
        for it in range(2):
            x, y = fn(t, 0, it)
            _, _, p, v = OR.local_step(model, list(range(B)), p, v, x, y, 0.05, 0.9, 1e-3)
    for k in p:
        for n in p[k]:
            np.testing.assert_allclose(got[k][n], p[k][n], rtol=1e-13, atol=1e-15)
    assert log[0]["subs"] == [list(range(B))]


def test_rounds_use_fresh_partitions_and_leave_untrained_tensors_alone():
    model = _model()
    params = make_params(model, 1)
    B = sum(model["blocks"])
    mask = [0, 0, 0, 1, 1, 1]                        # only three blocks of the second stage are dealt
    got, log = ORD.run_rounds(model, params, 3, 0, 11, 3, 1, _batch_fn(model, 2), 0.1, 0.9, 0.0, partitionable=mask)
    for t, entry in enumerate(log):
        assert (entry["subs"], entry["owner"]) == OP.partition(model["blocks"], 3, 0, 11, t, mask)
        assert all(len(s) == 4 for s in entry["subs"])       # 3 fixed blocks + 1 dealt each
    assert len({tuple(map(tuple, e["subs"])) for e in log}) > 1          # the split changes between rounds
    for k in got:                                    # everything was trained by somebody: all tensors moved
        assert any(not np.array_equal(got[k][n], params[k][n]) for n in got[k])
    # with zero learning rate nothing but the BN running statistics changes, whatever the partition
    same, _ = ORD.run_rounds(model, params, 3, 0, 11, 2, 1, _batch_fn(model, 2), 0.0, 0.9, 0.0, partitionable=mask)
    for k in same:
        for n in same[k]:
            if OR.is_trainable(n):
                np.testing.assert_allclose(same[k][n], params[k][n], rtol=0, atol=1e-7)


def test_round_with_compressed_communication_stays_within_half_a_step():
    """Appendix on quantised communication: with b-bit codes on the way back, every reassembled value
    is within the mean half-step of the uncompressed round's value; 8 bits is closer than 4."""
    from oracle import compress as OC
    model = dict(get_config("cfg1")["model"], widths=[8, 16], blocks=[2, 3], in_h=8, in_w=8, num_classes=5)
    params = make_params(model, 1, perturb_bn=True)

    def batch_fn(t, s, it):
        return make_batch(model, 4, 100 * t + 10 * s + it)

    exact, log = ORD.run_rounds(model, params, 2, 0, 3, 1, 2, batch_fn, 0.05, 0.9, 0.0)
    errs = {}
    for bits in (8, 4):
        got, log_q = ORD.run_rounds(model, params, 2, 0, 3, 1, 2, batch_fn, 0.05, 0.9, 0.0, compress_bits=bits)
        assert log_q[0]["subs"] == log[0]["subs"] and log_q[0]["losses"] == log[0]["losses"]
        worst = 0.0
        for k in exact:
            held = k in (-1, max(exact)) or any(k in s for s in log[0]["subs"])
            for n in exact[k]:
                e = np.asarray(exact[k][n], np.float64)
                d = np.abs(np.asarray(got[k][n], np.float64) - e)
                if not held:
                    assert d.max() == 0
                    continue
                # a worker's copy differs from the mean by less than the tensor's spread: bound with twice it
                bound = 0.5 * 2.0 * (e.max() - e.min() + 1e-3) / ((1 << bits) - 1)
                assert d.max() <= bound, (bits, k, n, d.max(), bound)
                worst = max(worst, d.max())
        errs[bits] = worst
    assert 0 < errs[8] < errs[4]
