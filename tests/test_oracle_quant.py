"""Pins for oracle/quant.py (bfloat16 storage rounding) and for the places where the oracle's
training step applies it."""
import numpy as np
import torch

from oracle import quant as Q
from oracle import resnet as OR
from resist_inputs import get_config, make_batch, make_params


def test_hand_computed_values():
    # bfloat16 keeps 7 fraction bits: neighbours of 1 are 1 - 2^-8 and 1 + 2^-7
    cases = [(1.0, 1.0),
             (1.0 + 2.0 ** -7, 1.0 + 2.0 ** -7),          # representable
             (1.0 + 2.0 ** -8, 1.0),                      # tie -> even (fraction 0)
             (1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -6),      # tie -> even (fraction 2)
             (1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 2.0 ** -7),   # just above the tie
             (1.0 + 2.0 ** -8 - 2.0 ** -20, 1.0),               # just below the tie
             (-3.0 - 2.0 ** -6 - 2.0 ** -9, -3.0 - 2.0 ** -6),  # sign is symmetric (ulp at 3 is 2^-6)
             (0.0, 0.0), (np.inf, np.inf), (-np.inf, -np.inf),
             (2.0 ** -126, 2.0 ** -126),                  # fp32's smallest normal is a bfloat16
             (3.3895313892515355e38, 3.3895313892515355e38)]   # largest finite bfloat16
    for x, want in cases:
        assert Q.round_bf16(np.array([x]))[0] == want, (x, want)
    assert np.isnan(Q.round_bf16(np.array([np.nan]))[0])


def test_properties_and_library_opinion():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, 20000),
                        rng.standard_normal(2000)])
    r = Q.round_bf16(x)
    assert np.array_equal(Q.round_bf16(r), r)                       # idempotent
    assert np.all(np.abs(r - x) <= 2.0 ** -8 * np.abs(x) * (1 + 1e-6))    # half an ulp <= 2^-9 * 2|x|
    assert np.all(np.abs(r - x) <= 2.0 ** -9 * 2.0 ** np.ceil(np.log2(np.abs(x))) * (1 + 1e-6))
    o = np.argsort(x)
    assert np.all(np.diff(r[o]) >= 0)                               # monotone
    assert np.array_equal((r.astype(np.float32).view(np.uint32) & 0xFFFF), np.zeros(x.size, np.uint32))
    lib = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(lib, r)
    assert Q.round_bf16(np.ones((2, 3, 4))).shape == (2, 3, 4)


def test_emulated_step_is_a_small_perturbation_and_rounds_where_stated():
    """With bf16 storage the forward pass stays within a fraction of a percent of the unrounded one
    (each rounding is 2^-9 relative).  Gradients move by much more than 2^-9: a pre-activation
    within rounding distance of zero flips its ReLU decision, a fraction f of flipped decisions
    moves a gradient tensor by about sqrt(f) of its norm, and the effect adds up over the layers
    below.  The step is a function of the rounded operands only."""
    basic = get_config("cfg1")["model"]
    model = dict(basic, block_kind=1, stem_kind=1, widths=[8, 16], blocks=[2, 2], in_h=24, in_w=24, num_classes=6)
    blocks = [0, 2, 3]
    params = make_params(model, 1, perturb_bn=True)
    x, y = make_batch(model, 6, 2)
    l0, g0, t0, _ = OR.forward_backward(model, blocks, params, x, y)
    l1, g1, t1, dx1 = OR.forward_backward(model, blocks, params, x, y, emulate_bf16=True, need_input_grad=True)
    assert l0 != l1 and abs(l0 - l1) <= 5e-3 * abs(l0)
    B = sum(model["blocks"])
    for b in g0:
        for k in g0[b]:
            rel = np.linalg.norm(g1[b][k] - g0[b][k]) / np.linalg.norm(g0[b][k])
            assert 0 < rel <= (3e-2 if b == B else 0.6), (b, k, rel)   # the head sees no ReLU decision
    # batch statistics are those of bfloat16-stored convolution outputs: they differ from the
    # unrounded ones by about 2^-9 of a standard deviation
    for key in t0.stats:
        m0, v0, _ = t0.stats[key]
        m1, v1, _ = t1.stats[key]
        assert np.all(np.abs(m0 - m1) <= 2e-2 * np.sqrt(v0) + 1e-12)
    # rounding identical inputs first changes nothing more: the step is a function of rounded operands
    xr = Q.round_bf16(x)
    l2, g2, _, _ = OR.forward_backward(model, blocks, params, xr, y, emulate_bf16=True)
    assert l2 == l1
    pr = {b: {k: (Q.round_bf16(v).astype(np.float32) if k.endswith("_w") and not k.startswith("fc") else v)
              for k, v in p.items()} for b, p in params.items()}
    l3, g3, _, _ = OR.forward_backward(model, blocks, pr, x, y, emulate_bf16=True)
    assert l3 == l1
    for b in g1:
        for k in g1[b]:
            assert np.array_equal(g1[b][k], g3[b][k])
