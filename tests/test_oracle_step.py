"""Pins for oracle/resnet.py: finite differences of the loss, an independent float64 autograd
network as third opinion, SGD closed form, sub-ResNet semantics (Appendix B: mask = 1 is the
full network, mask = 0 passes the residual stream through)."""
import copy
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import resnet as OR
from resist_inputs import get_config, make_batch, make_params, zeros_like_params


def _tiny_models():
    basic = get_config("cfg1")["model"]
    strided = dict(basic, widths=[8, 16], blocks=[2, 2], in_h=8, in_w=8, num_classes=5)
    bottle = dict(basic, block_kind=1, stem_kind=1, widths=[4, 8], blocks=[2, 2], in_h=20, in_w=20,
                  num_classes=7)
    return {"basic": basic, "strided": strided, "bottleneck": bottle}


def _torch_loss(model, blocks, params, x, labels):
    """The same network written with a float64 autograd library (library special case)."""
    tab = OR.block_table(model)
    B = len(tab)
    tp = {b: {k: torch.tensor(np.asarray(v, np.float64), requires_grad=OR.is_trainable(k))
              for k, v in p.items()} for b, p in params.items()}
    eps = model["bn_eps"]

    def cbn(a, p, conv, bn, stride, pad, relu):
        y = F.conv2d(a, p[conv + "_w"], stride=stride, padding=pad)
        y = F.batch_norm(y, None, None, p[bn + "_g"], p[bn + "_b"], True, 0.1, eps)
        return F.relu(y) if relu else y

    a = torch.tensor(np.asarray(x, np.float64))
    if model["stem_kind"] == 0:
        a = cbn(a, tp[-1], "conv", "bn", 1, 1, True)
    else:
        a = F.max_pool2d(cbn(a, tp[-1], "conv", "bn", 2, 3, True), 3, 2, 1)
    for b in blocks:
        t, p = tab[b], tp[b]
        if model["block_kind"] == 0:
            h = cbn(a, p, "conv1", "bn1", t["stride"], 1, True)
            h = cbn(h, p, "conv2", "bn2", 1, 1, False)
        else:
            h = cbn(a, p, "conv1", "bn1", 1, 0, True)
            h = cbn(h, p, "conv2", "bn2", t["stride"], 1, True)
            h = cbn(h, p, "conv3", "bn3", 1, 0, False)
        sc = cbn(a, p, "ds", "dsbn", t["stride"], 0, False) if t["has_ds"] else a
        a = F.relu(h + sc)
    z = F.linear(a.mean(dim=(2, 3)), tp[B]["fc_w"], tp[B]["fc_b"])
    loss = F.cross_entropy(z, torch.tensor(np.asarray(labels), dtype=torch.long))
    return loss, tp


@pytest.mark.parametrize("name", ["basic", "strided", "bottleneck"])
@pytest.mark.parametrize("drop", [False, True])
def test_gradients_match_autograd_library(name, drop):
    model = _tiny_models()[name]
    B = sum(model["blocks"])
    blocks = list(range(B))
    if drop:                                   # a sub-ResNet: drop one non-first block
        blocks.remove(1)
    params = make_params(model, 3, perturb_bn=True)
    x, y = make_batch(model, 4, 5)
    loss, grads, _, _ = OR.forward_backward(model, blocks, params, x, y)
    tl, tp = _torch_loss(model, blocks, params, x, y)
    tl.backward()
    assert math.isclose(loss, float(tl.detach()), rel_tol=1e-12)
    for b in [-1] + blocks + [B]:
        for k, g in grads[b].items():
            np.testing.assert_allclose(g, tp[b][k].grad.numpy(), rtol=1e-8, atol=1e-11,
                                       err_msg=f"block {b} {k}")
    assert set(grads.keys()) == set([-1, B] + blocks)


def test_finite_differences_every_parameter_cfg1():
    """Central differences of the float64 loss w.r.t. all 9 978 parameters of the tiny config."""
    cfg = get_config("cfg1")
    model = cfg["model"]
    params = {b: {k: v.astype(np.float64) for k, v in p.items()}
              for b, p in make_params(model, 0, perturb_bn=True).items()}
    x, y = make_batch(model, cfg["batch"], 0)
    blocks = [0, 1]
    loss, grads, _, _ = OR.forward_backward(model, blocks, params, x, y)
    assert sum(g.size for gb in grads.values() for g in gb.values()) == 9978
    h = 1e-5
    worst = 0.0
    for b, gb in grads.items():
        for k, g in gb.items():
            w = params[b][k]
            flat = w.reshape(-1)
            fd = np.empty(flat.size)
            for i in range(flat.size):
                old = flat[i]
                flat[i] = old + h
                lp = OR.forward_backward(model, blocks, params, x, y, backward=False)[0]
                flat[i] = old - h
                lm = OR.forward_backward(model, blocks, params, x, y, backward=False)[0]
                flat[i] = old
                fd[i] = (lp - lm) / (2 * h)
            tol = 1e-7 + 1e-5 * np.abs(g.reshape(-1))
            # a ReLU kink inside [w-h, w+h] breaks the difference quotient, not the gradient:
            # such elements are re-measured with a 100x smaller step
            for i in np.nonzero(np.abs(fd - g.reshape(-1)) > tol)[0]:
                old = flat[i]
                flat[i] = old + h / 100
                lp = OR.forward_backward(model, blocks, params, x, y, backward=False)[0]
                flat[i] = old - h / 100
                lm = OR.forward_backward(model, blocks, params, x, y, backward=False)[0]
                flat[i] = old
                fd[i] = (lp - lm) / (2 * h / 100)
            err = np.abs(fd - g.reshape(-1))
            worst = max(worst, float((err / tol).max()))
            assert (err <= tol).all(), f"block {b} {k}: max err {err.max():.3e}"
    assert worst < 1.0


@pytest.mark.parametrize("name", ["strided", "bottleneck"])
def test_finite_differences_sampled(name):
    model = _tiny_models()[name]
    B = sum(model["blocks"])
    blocks = [0, 2, 3]                        # block 1 dropped: a genuine sub-ResNet
    params = {b: {k: v.astype(np.float64) for k, v in p.items()}
              for b, p in make_params(model, 11, perturb_bn=True).items()}
    x, y = make_batch(model, 3, 12)
    loss, grads, _, dx = OR.forward_backward(model, blocks, params, x, y, need_input_grad=True)
    rng = np.random.default_rng(0)
    h = 1e-5
    for b, gb in grads.items():
        for k, g in gb.items():
            flat = params[b][k].reshape(-1)
            for i in rng.choice(flat.size, size=min(6, flat.size), replace=False):
                old = flat[i]
                flat[i] = old + h
                lp = OR.forward_backward(model, blocks, params, x, y, backward=False)[0]
                flat[i] = old - h
                lm = OR.forward_backward(model, blocks, params, x, y, backward=False)[0]
                flat[i] = old
                fd = (lp - lm) / (2 * h)
                assert abs(fd - g.reshape(-1)[i]) <= 1e-7 + 1e-5 * abs(fd), f"block {b} {k}[{i}]"
    # input gradient (exercises the stem's data gradient and the max-pool routing)
    xd = x.astype(np.float64)
    for idx in [(0, 0, 3, 3), (2, 2, 7, 1), (1, 1, 0, 0)]:
        e = np.zeros_like(xd)
        e[idx] = h
        fd = (OR.forward_backward(model, blocks, params, xd + e, y, backward=False)[0]
              - OR.forward_backward(model, blocks, params, xd - e, y, backward=False)[0]) / (2 * h)
        assert abs(fd - dx[idx]) <= 1e-7 + 1e-5 * abs(fd)


def test_absent_block_is_identity_and_untouched():
    """A block outside the list neither affects the loss nor receives a gradient/update."""
    model = _tiny_models()["strided"]
    params = make_params(model, 1)
    x, y = make_batch(model, 4, 2)
    mom = zeros_like_params(params)
    loss_a, grads, new_p, _ = OR.local_step(model, [0, 2, 3], params, mom, x, y, 0.1, 0.9, 0.0)
    params2 = copy.deepcopy(params)
    params2[1]["conv1_w"] += 1.0
    loss_b = OR.local_step(model, [0, 2, 3], params2, mom, x, y, 0.1, 0.9, 0.0)[0]
    assert loss_a == loss_b
    assert 1 not in grads and 1 not in new_p


def test_sgd_closed_form_two_steps():
    cfg = get_config("cfg1")
    model = cfg["model"]
    p0 = make_params(model, 0)
    x, y = make_batch(model, 4, 0)
    lr, mu, wd = 0.1, 0.9, 5e-4
    v0 = zeros_like_params(p0)
    _, g1, p1, v1 = OR.local_step(model, [0, 1], p0, v0, x, y, lr, mu, wd)
    for b, gb in g1.items():
        for k, g in gb.items():
            w0 = p0[b][k].astype(np.float64)
            np.testing.assert_allclose(p1[b][k], w0 - lr * (g + wd * w0), rtol=1e-14, atol=1e-16)
            np.testing.assert_allclose(v1[b][k], g + wd * w0, rtol=1e-14, atol=1e-16)
    _, g2, p2, v2 = OR.local_step(model, [0, 1], p1, v1, x, y, lr, mu, wd)
    for b, gb in g2.items():
        for k, g in gb.items():
            v = mu * v1[b][k] + g + wd * p1[b][k]
            np.testing.assert_allclose(v2[b][k], v, rtol=1e-14, atol=1e-16)
            np.testing.assert_allclose(p2[b][k], p1[b][k] - lr * v, rtol=1e-14, atol=1e-16)
    # running statistics move toward the batch statistics and are not touched by SGD
    assert not np.allclose(p1[-1]["bn_rm"], p0[-1]["bn_rm"])
    assert "bn_rm" not in g1[-1]


def test_param_count_matches_tensors():
    for name in ["cfg1", "cfg2", "cfg4"]:
        model = get_config(name)["model"]
        params = make_params(model, 0)
        for b, p in params.items():
            n_train = sum(v.size for k, v in p.items() if OR.is_trainable(k))
            n_all = sum(v.size for v in p.values())
            assert OR.param_count(model, b) == n_train
            assert OR.param_count(model, b, trainable_only=False) == n_all


# ---- test-time forward (Sec. 2.6 "Scaling Activations") ---------------------------------------------

@pytest.mark.parametrize("name", ["basic", "strided", "bottleneck"])
def test_forward_eval_pins(name):
    model = _tiny_models()[name]
    B = sum(model["blocks"])
    blocks = list(range(B))
    params = make_params(model, 6, perturb_bn=True)
    x, y = make_batch(model, 5, 7)
    z, loss = OR.forward_eval(model, blocks, params, x, branch_scale=None, labels=y)

    # (1) an autograd library's evaluation-mode batch norm as third opinion
    tab = OR.block_table(model)
    tp = {b: {k: torch.tensor(np.asarray(v, np.float64)) for k, v in p.items()} for b, p in params.items()}
    eps = model["bn_eps"]

    def cbn(a, p, conv, bn, stride, pad, relu):
        h = F.conv2d(a, p[conv + "_w"], stride=stride, padding=pad)
        h = F.batch_norm(h, p[bn + "_rm"], p[bn + "_rv"], p[bn + "_g"], p[bn + "_b"], False, 0.1, eps)
        return F.relu(h) if relu else h

    a = torch.tensor(np.asarray(x, np.float64))
    if model["stem_kind"] == 0:
        a = cbn(a, tp[-1], "conv", "bn", 1, 1, True)
    else:
        a = F.max_pool2d(cbn(a, tp[-1], "conv", "bn", 2, 3, True), 3, 2, 1)
    for b in blocks:
        t, p = tab[b], tp[b]
        if model["block_kind"] == 0:
            h = cbn(cbn(a, p, "conv1", "bn1", t["stride"], 1, True), p, "conv2", "bn2", 1, 1, False)
        else:
            h = cbn(a, p, "conv1", "bn1", 1, 0, True)
            h = cbn(cbn(h, p, "conv2", "bn2", t["stride"], 1, True), p, "conv3", "bn3", 1, 0, False)
        sc = cbn(a, p, "ds", "dsbn", t["stride"], 0, False) if t["has_ds"] else a
        a = F.relu(h + sc)
    zt = F.linear(a.mean(dim=(2, 3)), tp[B]["fc_w"], tp[B]["fc_b"])
    np.testing.assert_allclose(z, zt.numpy(), rtol=1e-10, atol=1e-12)
    assert math.isclose(loss, float(F.cross_entropy(zt, torch.tensor(y, dtype=torch.long))), rel_tol=1e-12)

    # (2) with the running statistics set to this batch's own statistics, the evaluation-mode pass is
    #     the training-mode pass (whose loss the finite-difference tests pin)
    tr_loss, _, tape, _ = OR.forward_backward(model, blocks, params, x, y, backward=False)
    p2 = copy.deepcopy(params)
    for (b, bn), (mean, var, m) in tape.stats.items():
        p2[b][bn + "_rm"], p2[b][bn + "_rv"] = mean, var
    _, loss2 = OR.forward_eval(model, blocks, p2, x, labels=y)
    assert math.isclose(loss2, tr_loss, rel_tol=1e-12)

    # (3) a branch scaled by zero is an absent block (identity shortcuts; Appendix B, mask 0), and the
    #     scale is linear in the branch: scaling gamma and beta of the last BN by s is the same thing
    drop = 1                                              # a non-first block in every tiny model
    scale = [1.0] * B
    scale[drop] = 0.0
    z0 = OR.forward_eval(model, blocks, params, x, branch_scale=scale)
    z1 = OR.forward_eval(model, [b for b in blocks if b != drop], params, x)
    np.testing.assert_allclose(z0, z1, rtol=1e-12, atol=1e-13)
    scale[drop] = 0.25
    p3 = copy.deepcopy(params)
    last = "bn3" if model["block_kind"] == 1 else "bn2"
    p3[drop][last + "_g"] = params[drop][last + "_g"] * 0.25
    p3[drop][last + "_b"] = params[drop][last + "_b"] * 0.25
    np.testing.assert_allclose(OR.forward_eval(model, blocks, params, x, branch_scale=scale),
                               OR.forward_eval(model, blocks, p3, x), rtol=1e-12, atol=1e-13)


# ---- pre-activation blocks (Sec. 2.1, Fig. 2: BN -> ReLU -> conv) ---------------------------------------

def _preact_models():
    basic = get_config("cfg1")["model"]
    return {"preact_basic": dict(basic, block_kind=2, widths=[8, 16], blocks=[2, 2], in_h=8, in_w=8, num_classes=5),
            "preact_bottleneck": dict(basic, block_kind=3, widths=[4, 8], blocks=[2, 2], in_h=8, in_w=8, num_classes=6)}


def _torch_loss_preact(model, blocks, params, x, labels):
    """The pre-activation network written with a float64 autograd library (library special case)."""
    tab = OR.block_table(model)
    B = len(tab)
    tp = {b: {k: torch.tensor(np.asarray(v, np.float64), requires_grad=OR.is_trainable(k))
              for k, v in p.items()} for b, p in params.items()}
    eps = model["bn_eps"]

    def bnrelu(u, p, bn):
        return F.relu(F.batch_norm(u, None, None, p[bn + "_g"], p[bn + "_b"], True, 0.1, eps))

    u = F.conv2d(torch.tensor(np.asarray(x, np.float64)), tp[-1]["conv_w"], stride=1, padding=1)
    for b in blocks:
        t, p = tab[b], tp[b]
        a1 = bnrelu(u, p, "bn1")
        if model["block_kind"] == 2:
            h = F.conv2d(a1, p["conv1_w"], stride=t["stride"], padding=1)
            h = F.conv2d(bnrelu(h, p, "bn2"), p["conv2_w"], stride=1, padding=1)
        else:
            h = F.conv2d(a1, p["conv1_w"])
            h = F.conv2d(bnrelu(h, p, "bn2"), p["conv2_w"], stride=t["stride"], padding=1)
            h = F.conv2d(bnrelu(h, p, "bn3"), p["conv3_w"])
        sc = F.conv2d(a1, p["ds_w"], stride=t["stride"]) if t["has_ds"] else u
        u = h + sc
    f = bnrelu(u, tp[B], "bn")
    z = F.linear(f.mean(dim=(2, 3)), tp[B]["fc_w"], tp[B]["fc_b"])
    return F.cross_entropy(z, torch.tensor(np.asarray(labels), dtype=torch.long)), tp


@pytest.mark.parametrize("name", ["preact_basic", "preact_bottleneck"])
@pytest.mark.parametrize("drop", [False, True])
def test_preact_gradients_match_autograd_library(name, drop):
    model = _preact_models()[name]
    B = sum(model["blocks"])
    blocks = [b for b in range(B) if not (drop and b == 1)]
    params = make_params(model, 3, perturb_bn=True)
    x, y = make_batch(model, 4, 5)
    loss, grads, _, _ = OR.forward_backward(model, blocks, params, x, y)
    tl, tp = _torch_loss_preact(model, blocks, params, x, y)
    tl.backward()
    assert math.isclose(loss, float(tl.detach()), rel_tol=1e-12)
    assert set(grads.keys()) == set([-1, B] + blocks)
    for b in grads:
        assert set(grads[b]) == {k for k in params[b] if OR.is_trainable(k)}
        for k, g in grads[b].items():
            np.testing.assert_allclose(g, tp[b][k].grad.numpy(), rtol=1e-8, atol=1e-11, err_msg=f"block {b} {k}")


@pytest.mark.parametrize("name", ["preact_basic", "preact_bottleneck"])
def test_preact_finite_differences_sampled(name):
    model = _preact_models()[name]
    blocks = [0, 2, 3]
    params = {b: {k: v.astype(np.float64) for k, v in p.items()}
              for b, p in make_params(model, 11, perturb_bn=True).items()}
    x, y = make_batch(model, 3, 12)
    loss, grads, _, dx = OR.forward_backward(model, blocks, params, x, y, need_input_grad=True)
    rng = np.random.default_rng(0)
    h = 1e-5
    for b, gb in grads.items():
        for k, g in gb.items():
            flat = params[b][k].reshape(-1)
            for i in rng.choice(flat.size, size=min(6, flat.size), replace=False):
                old = flat[i]
                flat[i] = old + h
                lp = OR.forward_backward(model, blocks, params, x, y, backward=False)[0]
                flat[i] = old - h
                lm = OR.forward_backward(model, blocks, params, x, y, backward=False)[0]
                flat[i] = old
                fd = (lp - lm) / (2 * h)
                assert abs(fd - g.reshape(-1)[i]) <= 1e-7 + 1e-5 * abs(fd), f"block {b} {k}[{i}]"
    xd = x.astype(np.float64)
    for idx in [(0, 0, 3, 3), (2, 2, 7, 1)]:
        e = np.zeros_like(xd)
        e[idx] = h
        fd = (OR.forward_backward(model, blocks, params, xd + e, y, backward=False)[0]
              - OR.forward_backward(model, blocks, params, xd - e, y, backward=False)[0]) / (2 * h)
        assert abs(fd - dx[idx]) <= 1e-7 + 1e-5 * abs(fd)


def test_preact_step_updates_every_tensor_and_running_statistics():
    model = _preact_models()["preact_basic"]
    params = make_params(model, 2)
    x, y = make_batch(model, 4, 3)
    _, grads, new_p, _ = OR.local_step(model, [0, 2], params, zeros_like_params(params), x, y, 0.1, 0.9, 1e-3)
    assert OR.param_count(model, -1) == params[-1]["conv_w"].size
    for b in (-1, 0, 2, 4):
        assert sum(g.size for g in grads[b].values()) == OR.param_count(model, b)
        for k in params[b]:
            assert not np.array_equal(new_p[b][k], params[b][k]), (b, k)      # running stats included
    assert 1 not in new_p and 3 not in new_p


@pytest.mark.parametrize("name", ["preact_basic", "preact_bottleneck"])
def test_preact_forward_eval_pins(name):
    """Evaluation-mode forward of the pre-activation network: equals the training-mode forward when the
    running statistics are this batch's own; a branch scaled by zero is an absent block; the scale is
    linear in the last convolution's filter."""
    model = _preact_models()[name]
    B = sum(model["blocks"])
    blocks = list(range(B))
    params = make_params(model, 6, perturb_bn=True)
    x, y = make_batch(model, 5, 7)
    tr_loss, _, tape, _ = OR.forward_backward(model, blocks, params, x, y, backward=False)
    p2 = copy.deepcopy(params)
    for (b, bn), (mean, var, m) in tape.stats.items():
        p2[b][bn + "_rm"], p2[b][bn + "_rv"] = mean, var
    _, loss2 = OR.forward_eval(model, blocks, p2, x, labels=y)
    assert math.isclose(loss2, tr_loss, rel_tol=1e-12)
    drop = 1
    scale = [1.0] * B
    scale[drop] = 0.0
    np.testing.assert_allclose(OR.forward_eval(model, blocks, params, x, branch_scale=scale),
                               OR.forward_eval(model, [b for b in blocks if b != drop], params, x), rtol=1e-12, atol=1e-13)
    scale[drop] = 0.25
    p3 = copy.deepcopy(params)
    last = OR.units_last_name(model)
    p3[drop][last + "_w"] = params[drop][last + "_w"] * 0.25
    np.testing.assert_allclose(OR.forward_eval(model, blocks, params, x, branch_scale=scale),
                               OR.forward_eval(model, blocks, p3, x), rtol=1e-12, atol=1e-13)
