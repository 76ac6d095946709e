"""Seeded random tensors in logical layout (numpy only; no arithmetic of the method)."""
import numpy as np

from .configs import model_blocks


def make_batch(model, batch, seed):
    """Images [N,C,H,W] ~ N(0,1) float32 and labels uniform in [0, classes) int32."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, model["in_c"], model["in_h"], model["in_w"]), dtype=np.float32)
    y = rng.integers(0, model["num_classes"], size=batch).astype(np.int32)
    return x, y


def _conv_w(rng, k, c, r, s):
    # Kaiming-normal, fan-out mode: std = sqrt(2 / (K*R*S))
    std = float(np.sqrt(2.0 / (k * r * s)))
    return (rng.standard_normal((k, c, r, s), dtype=np.float32) * np.float32(std)).astype(np.float32)


def _bn(rng, prefix, c, perturb):
    g = np.ones(c, np.float32)
    b = np.zeros(c, np.float32)
    rm = np.zeros(c, np.float32)
    rv = np.ones(c, np.float32)
    if perturb:
        # optional: non-trivial affine/running values so tests see every term
        g = (1.0 + 0.1 * rng.standard_normal(c)).astype(np.float32)
        b = (0.1 * rng.standard_normal(c)).astype(np.float32)
        rm = (0.1 * rng.standard_normal(c)).astype(np.float32)
        rv = (1.0 + 0.1 * rng.random(c)).astype(np.float32)
    return {prefix + "_g": g, prefix + "_b": b, prefix + "_rm": rm, prefix + "_rv": rv}


def make_params(model, seed, perturb_bn=False):
    """Initial weights of the GLOBAL network, keyed -1 (stem), 0..B-1 (blocks), B (head).

    Conv weights [K,C,R,S] Kaiming-normal; BN gamma=1, beta=0, running mean 0 / var 1;
    FC weight/bias uniform in +-1/sqrt(fan_in).  All float32.
    """
    if model["block_kind"] >= 2:
        return _make_params_preact(model, seed, perturb_bn)
    rng = np.random.default_rng(seed)
    blocks = model_blocks(model)
    params = {}
    w0 = model["widths"][0]
    rs = 3 if model["stem_kind"] == 0 else 7
    stem = {"conv_w": _conv_w(rng, w0, model["in_c"], rs, rs)}
    stem.update(_bn(rng, "bn", w0, perturb_bn))
    params[-1] = stem
    for b, blk in enumerate(blocks):
        p = {}
        if model["block_kind"] == 0:
            p["conv1_w"] = _conv_w(rng, blk["width"], blk["c_in"], 3, 3)
            p.update(_bn(rng, "bn1", blk["width"], perturb_bn))
            p["conv2_w"] = _conv_w(rng, blk["c_out"], blk["width"], 3, 3)
            p.update(_bn(rng, "bn2", blk["c_out"], perturb_bn))
        else:
            p["conv1_w"] = _conv_w(rng, blk["width"], blk["c_in"], 1, 1)
            p.update(_bn(rng, "bn1", blk["width"], perturb_bn))
            p["conv2_w"] = _conv_w(rng, blk["width"], blk["width"], 3, 3)
            p.update(_bn(rng, "bn2", blk["width"], perturb_bn))
            p["conv3_w"] = _conv_w(rng, blk["c_out"], blk["width"], 1, 1)
            p.update(_bn(rng, "bn3", blk["c_out"], perturb_bn))
        if blk["has_ds"]:
            p["ds_w"] = _conv_w(rng, blk["c_out"], blk["c_in"], 1, 1)
            p.update(_bn(rng, "dsbn", blk["c_out"], perturb_bn))
        params[b] = p
    c_last = blocks[-1]["c_out"]
    bound = 1.0 / float(np.sqrt(c_last))
    nc = model["num_classes"]
    params[len(blocks)] = {
        "fc_w": rng.uniform(-bound, bound, size=(nc, c_last)).astype(np.float32),
        "fc_b": rng.uniform(-bound, bound, size=(nc,)).astype(np.float32),
    }
    return params


def _make_params_preact(model, seed, perturb_bn):
    """Pre-activation networks: the stem is a bare 3x3 convolution, every BN sits before its
    convolution (so it has that convolution's input channels), the shortcut convolution has no BN,
    and the head starts with a BN."""
    rng = np.random.default_rng(seed)
    blocks = model_blocks(model)
    w0 = model["widths"][0]
    params = {-1: {"conv_w": _conv_w(rng, w0, model["in_c"], 3, 3)}}
    for b, blk in enumerate(blocks):
        p = {}
        if model["block_kind"] == 2:
            units = [("bn1", "conv1", blk["c_in"], blk["width"], 3), ("bn2", "conv2", blk["width"], blk["c_out"], 3)]
        else:
            units = [("bn1", "conv1", blk["c_in"], blk["width"], 1), ("bn2", "conv2", blk["width"], blk["width"], 3),
                     ("bn3", "conv3", blk["width"], blk["c_out"], 1)]
        for bn, conv, c, k, r in units:
            p.update(_bn(rng, bn, c, perturb_bn))
            p[conv + "_w"] = _conv_w(rng, k, c, r, r)
        if blk["has_ds"]:
            p["ds_w"] = _conv_w(rng, blk["c_out"], blk["c_in"], 1, 1)
        params[b] = p
    c_last = blocks[-1]["c_out"]
    bound = 1.0 / float(np.sqrt(c_last))
    nc = model["num_classes"]
    head = _bn(rng, "bn", c_last, perturb_bn)
    head["fc_w"] = rng.uniform(-bound, bound, size=(nc, c_last)).astype(np.float32)
    head["fc_b"] = rng.uniform(-bound, bound, size=(nc,)).astype(np.float32)
    params[len(blocks)] = head
    return params


def zeros_like_params(params):
    return {b: {k: np.zeros_like(v) for k, v in p.items()} for b, p in params.items()}
