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


def _on_grid(params, bits):
    """Every tensor replaced by its own b-bit decode: values the quantiser reproduces exactly."""
    from oracle import compress as OC
    return {k: {n: OC.dequantize_tensor(*OC.quantize_tensor(np.asarray(a, np.float32), bits)).astype(np.float32)
                for n, a in t.items()} for k, t in params.items()}


def test_compressing_the_way_down_changes_the_start_of_the_local_steps():
    """Server-to-worker compression (appendix on quantised communication, both directions): a worker
    starts its local steps from the decoded b-bit copy of the global model.  (1) When every global
    tensor already lies on its own b-bit grid, decoding its codes gives the tensor back to fp32
    rounding, so the first local losses are those of the round without compression on the way down;
    for generic tensors they differ at the scale of the quantiser's step.  (2) With one worker, one
    step and zero learning rate the trainable tensors come back as their b-bit decode, and the BN
    running statistics are those of a forward pass through the DECODED weights (not through the
    original ones), then compressed on the way back."""
    from oracle import compress as OC
    model = dict(get_config("cfg1")["model"], widths=[8, 16], blocks=[2, 3], in_h=8, in_w=8, num_classes=5)
    B = sum(model["blocks"])
    fn = _batch_fn(model, 4)
    bits = 5
    # (1)
    generic = make_params(model, 1, perturb_bn=True)
    grid = _on_grid(generic, bits)
    for k in grid:
        for n, a in grid[k].items():
            again = OC.dequantize_tensor(*OC.quantize_tensor(a, bits))
            assert np.max(np.abs(again - a)) <= 2.4e-7 * float(np.max(np.abs(a))) + 1e-12, (k, n)     # two fp32 roundings
    first = {}
    for name, start in (("grid", grid), ("generic", generic)):
        _, log_up = ORD.run_rounds(model, start, 2, 0, 3, 1, 1, fn, 0.05, 0.9, 0.0, compress_bits=bits)
        _, log_both = ORD.run_rounds(model, start, 2, 0, 3, 1, 1, fn, 0.05, 0.9, 0.0, compress_bits=bits, compress_down=True)
        first[name] = max(abs(a[0] - b[0]) / abs(a[0]) for a, b in zip(log_up[0]["losses"], log_both[0]["losses"]))
    assert first["grid"] <= 1e-5 and first["generic"] >= 1e-4, first
    # (2)
    params = make_params(model, 2, perturb_bn=True)
    got, _ = ORD.run_rounds(model, params, 1, 0, 3, 1, 1, fn, 0.0, 0.9, 0.0, compress_bits=bits, compress_down=True)
    decoded = _on_grid(params, bits)
    x, y = fn(0, 0, 0)
    _, _, after, _ = OR.local_step(model, list(range(B)), decoded, zeros_like_params(params), x, y, 0.0, 0.9, 0.0)
    _, _, after_plain, _ = OR.local_step(model, list(range(B)), params, zeros_like_params(params), x, y, 0.0, 0.9, 0.0)
    moved = 0
    for k in got:
        for n in got[k]:
            want = OC.dequantize_tensor(*OC.quantize_tensor(np.asarray(after[k][n], np.float32), bits))
            np.testing.assert_array_equal(got[k][n], want, err_msg=f"{k} {n}")
            if n.endswith(("_rm", "_rv")):
                plain = OC.dequantize_tensor(*OC.quantize_tensor(np.asarray(after_plain[k][n], np.float32), bits))
                moved += int(not np.array_equal(plain, want))
    assert moved > 0        # the statistics tell the decoded start from the original one
