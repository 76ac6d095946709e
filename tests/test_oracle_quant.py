"""Pins for oracle/quant.py (bfloat16 storage rounding) and for the places where the oracle's
training step applies it."""
import numpy as np
import pytest
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


# ---- where the emulation rounds: an autograd library's evaluation with explicit storage roundings ----
# The bf16 storage points of a training step (the ImageNet-shaped configuration: "bf16 activations/weights
# with fp32 accumulation and fp32 master weights"), written down once more, from the statement alone, as
# rounding nodes in a float64 autograd graph:
#   forward   image         the input image as a convolution operand
#             filter        the copy of a filter a convolution multiplies with (the master stays unrounded)
#             conv_out      every convolution output (BN statistics are those of the stored values)
#             act           every BN+ReLU output inside a block and in the stem
#             block_out     a block's output: branch + shortcut (+ ReLU), rounded once
#   backward  g_conv_out    the gradient a BN hands to its convolution (read by data and weight gradient)
#             g_act         a convolution's data gradient w.r.t. an activation inside a block
#             g_shortcut    the shortcut convolution's data gradient, stored before the branch's is added
#             g_block       the gradient w.r.t. a block's input / the residual stream: all contributions
#                           summed in full precision, rounded once (after the mean pool for the last block)
#             g_maxpool     the gradient w.r.t. the stem output behind the max pool
# A rounding node either rounds the value going forward (gradient passes unchanged) or the gradient coming
# back (value passes unchanged).  The oracle's emulate_bf16 option must agree with this graph to float64
# rounding, and leaving out any single kind of node must break the agreement.
def _lib_round(t):
    return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)


class _RoundValue(torch.autograd.Function):
    @staticmethod
    def forward(ctx, t):
        return _lib_round(t)

    @staticmethod
    def backward(ctx, g):
        return g


class _RoundGrad(torch.autograd.Function):
    @staticmethod
    def forward(ctx, t):
        return t.view_as(t)

    @staticmethod
    def backward(ctx, g):
        return _lib_round(g)


def _rounded_graph_loss(model, blocks, params, x, labels, skip=None):
    from torch.nn import functional as F
    tab = OR.block_table(model)
    B = len(tab)
    tp = {b: {k: torch.tensor(np.asarray(v, np.float64), requires_grad=OR.is_trainable(k)) for k, v in p.items()}
          for b, p in params.items()}
    eps = model["bn_eps"]

    def rv(t, tag):
        return t if tag == skip else _RoundValue.apply(t)

    def rg(t, tag):
        return t if tag == skip else _RoundGrad.apply(t)

    def conv(a, w, stride, pad):
        return rg(rv(F.conv2d(a, rv(w, "filter"), stride=stride, padding=pad), "conv_out"), "g_conv_out")

    def bn(y, p, name):
        return F.batch_norm(y, None, None, p[name + "_g"], p[name + "_b"], True, 0.1, eps)

    img = rv(torch.tensor(np.asarray(x, np.float64)), "image")
    if model["block_kind"] < 2:
        st = tp[-1]
        if model["stem_kind"] == 0:
            a = rv(F.relu(bn(conv(img, st["conv_w"], 1, 1), st, "bn")), "act")
        else:
            a = rg(rv(F.relu(bn(conv(img, st["conv_w"], 2, 3), st, "bn")), "act"), "g_maxpool")
            a = F.max_pool2d(a, 3, 2, 1)
        for b in blocks:
            t, p = tab[b], tp[b]
            inp = rg(a, "g_block")
            if model["block_kind"] == 0:
                h = rg(rv(F.relu(bn(conv(inp, p["conv1_w"], t["stride"], 1), p, "bn1")), "act"), "g_act")
                h = bn(conv(h, p["conv2_w"], 1, 1), p, "bn2")
            else:
                h = rg(rv(F.relu(bn(conv(inp, p["conv1_w"], 1, 0), p, "bn1")), "act"), "g_act")
                h = rg(rv(F.relu(bn(conv(h, p["conv2_w"], t["stride"], 1), p, "bn2")), "act"), "g_act")
                h = bn(conv(h, p["conv3_w"], 1, 0), p, "bn3")
            sc = bn(conv(rg(inp, "g_shortcut"), p["ds_w"], t["stride"], 0), p, "dsbn") if t["has_ds"] else inp
            a = rv(F.relu(h + sc), "block_out")
        feat = rg(a, "g_block")
    else:
        u = rv(F.conv2d(img, rv(tp[-1]["conv_w"], "filter"), stride=1, padding=1), "conv_out")
        for b in blocks:
            t, p = tab[b], tp[b]
            xin = rg(u, "g_block")
            layers = OR._preact_layers(model, t)
            h, a1 = xin, None
            for j, (bname, cname, k, stride, pad) in enumerate(layers):
                a = rg(rv(F.relu(bn(h, p, bname)), "act"), "g_act")
                a1 = a if a1 is None else a1
                h = F.conv2d(a, rv(p[cname + "_w"], "filter"), stride=stride, padding=pad)
                if j + 1 < len(layers):
                    h = rg(rv(h, "conv_out"), "g_conv_out")
            if t["has_ds"]:
                sc = rv(F.conv2d(rg(a1, "g_shortcut"), rv(p["ds_w"], "filter"), stride=t["stride"]), "conv_out")
            else:
                sc = xin
            u = rv(h + sc, "block_out")
        f = rv(F.relu(bn(rg(u, "g_block"), tp[B], "bn")), "act")
        feat = rg(f, "g_act")
    z = F.linear(feat.mean(dim=(2, 3)), tp[B]["fc_w"], tp[B]["fc_b"])
    return F.cross_entropy(z, torch.tensor(np.asarray(labels), dtype=torch.long)), tp


def _storage_models():
    basic = get_config("cfg1")["model"]
    return {
        "basic": (dict(basic, widths=[8, 16], blocks=[2, 2], in_h=8, in_w=8, num_classes=5), [0, 1, 2, 3],
                  ["image", "filter", "conv_out", "act", "block_out", "g_conv_out", "g_act", "g_shortcut", "g_block"]),
        "bottleneck": (dict(basic, block_kind=1, stem_kind=1, widths=[4, 8], blocks=[2, 2], in_h=20, in_w=20, num_classes=7),
                       [0, 2, 3], ["image", "filter", "conv_out", "act", "block_out", "g_conv_out", "g_act", "g_shortcut",
                                   "g_block", "g_maxpool"]),
        "preact": (dict(basic, block_kind=2, widths=[8, 16], blocks=[2, 2], in_h=8, in_w=8, num_classes=5), [0, 1, 2, 3],
                   ["image", "filter", "conv_out", "act", "block_out", "g_conv_out", "g_act", "g_shortcut", "g_block"]),
        "preact_bottleneck": (dict(basic, block_kind=3, widths=[4, 8], blocks=[2, 2], in_h=8, in_w=8, num_classes=6),
                              [0, 2, 3], ["image", "filter", "conv_out", "act", "block_out", "g_conv_out", "g_act", "g_shortcut", "g_block"]),
    }


def _max_rel_gap(grads, tp):
    worst = 0.0
    for b in grads:
        for k, g in grads[b].items():
            t = tp[b][k].grad.numpy()
            worst = max(worst, float(np.linalg.norm(g - t) / max(np.linalg.norm(t), 1e-300)))
    return worst



@pytest.mark.parametrize("name", ["basic", "bottleneck", "preact", "preact_bottleneck"])
def test_emulation_rounds_exactly_at_the_stated_storage_points(name):
    model, blocks, tags = _storage_models()[name]
    params = make_params(model, 3, perturb_bn=True)
    x, y = make_batch(model, 4, 5)
    loss, grads, _, _ = OR.forward_backward(model, blocks, params, x, y, emulate_bf16=True)
    tl, tp = _rounded_graph_loss(model, blocks, params, x, y)
    tl.backward()
    assert abs(loss - float(tl.detach())) <= 1e-12 * abs(loss)
    assert _max_rel_gap(grads, tp) <= 1e-9
    # every kind of storage point is live: without it the graph no longer reproduces the oracle
    for tag in tags:
        tl2, tp2 = _rounded_graph_loss(model, blocks, params, x, y, skip=tag)
        tl2.backward()
        gap = max(_max_rel_gap(grads, tp2), abs(loss - float(tl2.detach())) / abs(loss))
        assert gap >= 1e-6, f"{name}: leaving out the '{tag}' roundings changes nothing ({gap:.1e})"
