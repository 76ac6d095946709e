"""Oracle: one local SGD iteration of one sub-ResNet, float64 -- TEST INFRASTRUCTURE ONLY.

Algorithm 1's inner loop (W_s <- W_s - eta * dL/dW_s) on the network a worker keeps:
the stem, the residual blocks in its block list (ascending global index), and the head.
A block that is absent contributes nothing: the residual stream passes through unchanged
(Appendix B, forward recursion with mask M = 0; with M = 1 everywhere the sub-ResNet is the
global ResNet).

block_kind 0 / 1: post-activation basic / bottleneck blocks (the benchmark configurations' layer list);
block_kind 2 / 3: pre-activation basic / bottleneck blocks (the architecture the paper prefers, Sec. 2.1 and
Fig. 2: BN -> ReLU -> conv, twice, identity added without a ReLU after it), see the second list.

Network (post-activation blocks):
  stem   conv (3x3 s1 p1 | 7x7 s2 p3) -> BN -> ReLU [-> maxpool 3x3 s2 p1]
  basic  conv3x3(stride) -> BN -> ReLU -> conv3x3 -> BN ; + shortcut ; ReLU
  bottle conv1x1 -> BN -> ReLU -> conv3x3(stride) -> BN -> ReLU -> conv1x1(x4) -> BN ; + shortcut ; ReLU
  shortcut: identity, or conv1x1(stride) -> BN in the first block of a stage when shape changes
  head   global mean pool -> FC + bias -> softmax cross-entropy, mean over the batch
Network (pre-activation blocks; what the paper leaves open is read as in the pre-activation ResNet it cites):
  stem   conv 3x3 s1 p1 only
  basic  BN -> ReLU -> conv3x3(stride) -> BN -> ReLU -> conv3x3 ; + shortcut        (no ReLU after the add)
  bottle BN -> ReLU -> conv1x1 -> BN -> ReLU -> conv3x3(stride) -> BN -> ReLU -> conv1x1(x4) ; + shortcut
  shortcut: identity, or conv1x1(stride) applied to the block's first ReLU output (no BN) where shape changes
  head   BN -> ReLU -> global mean pool -> FC + bias -> softmax cross-entropy
Update (momentum per the paper's experimental section; form is the usual one):
  g <- g + wd*w ; v <- mu*v + g ; w <- w - lr*v   (every trainable parameter alike)
Parameters are dicts keyed -1 (stem), b (block), B (head) of logical-layout arrays.
Optional bfloat16 storage (the ImageNet-shaped configuration: "bf16 activations/weights with fp32
accumulation and fp32 master weights"): with emulate_bf16=True every tensor that configuration keeps
in bfloat16 is rounded where it is stored -- the input image and the filters as convolution operands,
every convolution output, every BN(+ReLU, +shortcut) output, every activation gradient (after the
mean-pool, max-pool, BN and convolution data-gradient steps; the shortcut's gradient is stored before
it is added to the branch's).  Statistics, weight gradients, the head, the loss and the update are
not rounded.  With emulate_bf16=False (default) nothing is rounded.
Pins: tests/test_oracle_step.py (finite differences of the loss w.r.t. every parameter,
a float64 autograd library as third opinion, SGD closed form, all-blocks == full model).
"""
import numpy as np

from . import layers as L
from . import quant as Q


def is_preact(model):
    return model["block_kind"] >= 2


def block_table(model):
    exp = 4 if model["block_kind"] in (1, 3) else 1
    tab, c_in = [], model["widths"][0]
    for si, (w, nb) in enumerate(zip(model["widths"], model["blocks"])):
        for bi in range(nb):
            stride = 2 if (bi == 0 and si > 0) else 1
            c_out = w * exp
            tab.append(dict(c_in=c_in, width=w, c_out=c_out, stride=stride,
                            has_ds=(bi == 0 and (stride != 1 or c_in != c_out))))
            c_in = c_out
    return tab


TRAINABLE_SUFFIXES = ("_w", "_g", "_b")


def is_trainable(name):
    return name.endswith(TRAINABLE_SUFFIXES)


def param_count(model, block, trainable_only=True):
    """Number of parameters of the stem (-1), a block, or the head (B) -- closed form from the
    layer shapes (no conv bias; BN gamma+beta; FC weight+bias)."""
    tab = block_table(model)
    B = len(tab)
    bn = (lambda c: 2 * c) if trainable_only else (lambda c: 4 * c)
    if is_preact(model):
        if block == -1:
            return model["widths"][0] * model["in_c"] * 9
        if block == B:
            return model["num_classes"] * tab[-1]["c_out"] + model["num_classes"] + bn(tab[-1]["c_out"])
        t = tab[block]
        if model["block_kind"] == 2:
            n = bn(t["c_in"]) + t["width"] * t["c_in"] * 9 + bn(t["width"]) + t["c_out"] * t["width"] * 9
        else:
            n = (bn(t["c_in"]) + t["width"] * t["c_in"] + bn(t["width"]) + t["width"] * t["width"] * 9
                 + bn(t["width"]) + t["c_out"] * t["width"])
        return n + (t["c_out"] * t["c_in"] if t["has_ds"] else 0)
    if block == -1:
        rs = 3 if model["stem_kind"] == 0 else 7
        w0 = model["widths"][0]
        return w0 * model["in_c"] * rs * rs + bn(w0)
    if block == B:
        return model["num_classes"] * tab[-1]["c_out"] + model["num_classes"]
    t = tab[block]
    if model["block_kind"] == 0:
        n = t["width"] * t["c_in"] * 9 + bn(t["width"]) + t["c_out"] * t["width"] * 9 + bn(t["c_out"])
    else:
        n = (t["width"] * t["c_in"] + bn(t["width"]) + t["width"] * t["width"] * 9 + bn(t["width"])
             + t["c_out"] * t["width"] + bn(t["c_out"]))
    if t["has_ds"]:
        n += t["c_out"] * t["c_in"] + bn(t["c_out"])
    return n


class _Tape:
    """Forward caches, so the backward is the exact adjoint of the forward just computed."""

    def __init__(self):
        self.stats = {}      # (block, bn name) -> (mean, biased var, m)
        self.relu_margin = np.inf   # smallest |input| any ReLU saw (how close a decision was to a tie)

    def saw_relu_input(self, z):
        self.relu_margin = min(self.relu_margin, float(np.abs(z).min()))


def _conv_bn(x, p, conv, bn, stride, pad, eps, relu, tape, key, q):
    """q: storage rounding of activations and convolution operands (identity unless bf16 is emulated).
    The BN output is returned unrounded when it ends a block (relu=False): the caller adds the
    shortcut first and rounds the sum."""
    wq = q(p[conv + "_w"])
    y = q(L.conv2d_fwd(x, wq, stride, pad))
    z, cache = L.bn_fwd(y, p[bn + "_g"].astype(np.float64), p[bn + "_b"].astype(np.float64), eps)
    m = y.shape[0] * y.shape[2] * y.shape[3]
    tape.stats[(key, bn)] = (cache[2], cache[3], m)
    if relu:
        tape.saw_relu_input(z)
    a = q(np.maximum(z, 0.0)) if relu else z
    return a, dict(x=x, cache=cache, z=z, conv=conv, bn=bn, stride=stride, pad=pad, relu=relu, wq=wq)


def _conv_bn_bwd(da, ctx, p, grads, q):
    """da: gradient w.r.t. the (post-ReLU if relu) output.  ReLU'(0) = 0."""
    dz = da * (ctx["z"] > 0) if ctx["relu"] else da
    dy, dg, db = L.bn_bwd(dz, ctx["cache"], p[ctx["bn"] + "_g"].astype(np.float64))
    dy = q(dy)
    grads[ctx["bn"] + "_g"] = dg
    grads[ctx["bn"] + "_b"] = db
    w = ctx["wq"]
    grads[ctx["conv"] + "_w"] = L.conv2d_wgrad(dy, ctx["x"], w.shape, ctx["stride"], ctx["pad"])
    return dy, w


def forward_backward(model, blocks, params, x, labels, need_input_grad=False, backward=True,
                     emulate_bf16=False):
    """Loss and gradients of the sub-ResNet made of `blocks` (ascending global indices).

    Returns loss, grads (same keys as params, trainable tensors only), tape (batch statistics),
    and the input gradient if asked.  backward=False stops after the loss (grads = None).
    """
    if is_preact(model):
        return _forward_backward_preact(model, blocks, params, x, labels, need_input_grad, backward, emulate_bf16)
    tab = block_table(model)
    B = len(tab)
    eps = model["bn_eps"]
    tape = _Tape()
    q = Q.round_bf16 if emulate_bf16 else Q.identity
    x = q(np.asarray(x, np.float64))
    # ---- forward
    st = params[-1]
    if model["stem_kind"] == 0:
        a, stem_ctx = _conv_bn(x, st, "conv", "bn", 1, 1, eps, True, tape, -1, q)
        pool_cache = None
    else:
        a, stem_ctx = _conv_bn(x, st, "conv", "bn", 2, 3, eps, True, tape, -1, q)
        a, pool_cache = L.maxpool_fwd(a, 3, 2, 1)
    ctxs = []
    for b in blocks:
        t, p = tab[b], params[b]
        inp = a
        if model["block_kind"] == 0:
            h, c1 = _conv_bn(inp, p, "conv1", "bn1", t["stride"], 1, eps, True, tape, b, q)
            h, c2 = _conv_bn(h, p, "conv2", "bn2", 1, 1, eps, False, tape, b, q)
            chain = [c1, c2]
        else:
            h, c1 = _conv_bn(inp, p, "conv1", "bn1", 1, 0, eps, True, tape, b, q)
            h, c2 = _conv_bn(h, p, "conv2", "bn2", t["stride"], 1, eps, True, tape, b, q)
            h, c3 = _conv_bn(h, p, "conv3", "bn3", 1, 0, eps, False, tape, b, q)
            chain = [c1, c2, c3]
        if t["has_ds"]:
            sc, cd = _conv_bn(inp, p, "ds", "dsbn", t["stride"], 0, eps, False, tape, b, q)
        else:
            sc, cd = inp, None
        pre = h + sc
        tape.saw_relu_input(pre)
        a = q(np.maximum(pre, 0.0))
        ctxs.append((b, chain, cd, pre))
    feat_shape = a.shape
    pooled = L.avgpool_fwd(a)
    hd = params[B]
    z = L.fc_fwd(pooled, hd["fc_w"].astype(np.float64), hd["fc_b"].astype(np.float64))
    loss, dz = L.softmax_ce(z, np.asarray(labels))
    if not backward:
        return loss, None, tape, None
    # ---- backward
    grads = {}
    dpooled, dw, db = L.fc_bwd(dz, pooled, hd["fc_w"].astype(np.float64))
    grads[B] = {"fc_w": dw, "fc_b": db}
    g = q(L.avgpool_bwd(dpooled, feat_shape))
    for b, chain, cd, pre in reversed(ctxs):
        t, p = tab[b], params[b]
        gb = {}
        gpre = g * (pre > 0)
        d = gpre
        for ctx in reversed(chain):
            dy, w = _conv_bn_bwd(d, ctx, p, gb, q)
            d = L.conv2d_dgrad(dy, w, ctx["x"].shape, ctx["stride"], ctx["pad"])
            if ctx is not chain[0]:
                d = q(d)
        if cd is not None:
            dy, w = _conv_bn_bwd(gpre, cd, p, gb, q)
            d = d + q(L.conv2d_dgrad(dy, w, cd["x"].shape, cd["stride"], cd["pad"]))
        else:
            d = d + gpre
        g = q(d)
        grads[b] = gb
    gs = {}
    if pool_cache is not None:
        g = q(L.maxpool_bwd(g, pool_cache))
    dy, w = _conv_bn_bwd(g, stem_ctx, st, gs, q)
    grads[-1] = gs
    dx = None
    if need_input_grad:
        dx = L.conv2d_dgrad(dy, w, stem_ctx["x"].shape, stem_ctx["stride"], stem_ctx["pad"])
    return loss, grads, tape, dx


def _preact_layers(model, t):
    """(bn name, conv name, kernel, stride, pad) of the BN-ReLU-conv units of a pre-activation block."""
    if model["block_kind"] == 2:
        return [("bn1", "conv1", 3, t["stride"], 1), ("bn2", "conv2", 3, 1, 1)]
    return [("bn1", "conv1", 1, 1, 0), ("bn2", "conv2", 3, t["stride"], 1), ("bn3", "conv3", 1, 1, 0)]


def _forward_backward_preact(model, blocks, params, x, labels, need_input_grad, backward, emulate_bf16):
    """forward_backward for pre-activation blocks (block_kind 2, 3).  In a block with units
    j = 1..n:  a_j = ReLU(BN_j(u_j)), h_j = conv_j(a_j), u_1 = x, u_j = h_{j-1};  out = h_n + shortcut.
    With bf16 emulation everything stored is rounded: a_j, h_j (j < n), the shortcut convolution's
    output, out (the sum, rounded once), and the matching gradients on the way back."""
    tab = block_table(model)
    B = len(tab)
    eps = model["bn_eps"]
    tape = _Tape()
    q = Q.round_bf16 if emulate_bf16 else Q.identity
    if model["stem_kind"] != 0:
        raise ValueError("pre-activation networks use the 3x3 stem")

    def bn_relu(u, p, bn, key):
        z, cache = L.bn_fwd(u, p[bn + "_g"].astype(np.float64), p[bn + "_b"].astype(np.float64), eps)
        tape.stats[(key, bn)] = (cache[2], cache[3], u.shape[0] * u.shape[2] * u.shape[3])
        tape.saw_relu_input(z)
        return q(np.maximum(z, 0.0)), (z, cache)

    # ---- forward
    ximg = q(np.asarray(x, np.float64))
    wstem = q(params[-1]["conv_w"])
    u = q(L.conv2d_fwd(ximg, wstem, 1, 1))
    ctxs = []
    for b in blocks:
        t, p = tab[b], params[b]
        xin, units = u, []
        for bn, conv, k, stride, pad in _preact_layers(model, t):
            a, (z, cache) = bn_relu(u, p, bn, b)
            wq = q(p[conv + "_w"])
            h = L.conv2d_fwd(a, wq, stride, pad)
            units.append(dict(bn=bn, conv=conv, stride=stride, pad=pad, a=a, z=z, cache=cache, wq=wq, u_shape=u.shape))
            u = q(h) if conv != units_last_name(model) else h
        ds = None
        if t["has_ds"]:
            wd_ = q(p["ds_w"])
            sc = q(L.conv2d_fwd(units[0]["a"], wd_, t["stride"], 0))
            ds = dict(wq=wd_)
        else:
            sc = xin
        u = q(u + sc)
        ctxs.append((b, units, ds))
    hd = params[B]
    f, (zf, cachef) = bn_relu(u, hd, "bn", B)
    feat_shape = f.shape
    pooled = L.avgpool_fwd(f)
    z = L.fc_fwd(pooled, hd["fc_w"].astype(np.float64), hd["fc_b"].astype(np.float64))
    loss, dz = L.softmax_ce(z, np.asarray(labels))
    if not backward:
        return loss, None, tape, None
    # ---- backward
    grads = {}
    dpooled, dw, db = L.fc_bwd(dz, pooled, hd["fc_w"].astype(np.float64))
    gf = q(L.avgpool_bwd(dpooled, feat_shape))
    du, dg, dbt = L.bn_bwd(gf * (zf > 0), cachef, hd["bn_g"].astype(np.float64))
    grads[B] = {"fc_w": dw, "fc_b": db, "bn_g": dg, "bn_b": dbt}
    g = q(du)
    for b, units, ds in reversed(ctxs):
        t, p = tab[b], params[b]
        gb = {}
        gcur = g
        for j in range(len(units) - 1, -1, -1):
            un = units[j]
            gb[un["conv"] + "_w"] = L.conv2d_wgrad(gcur, un["a"], un["wq"].shape, un["stride"], un["pad"])
            da = L.conv2d_dgrad(gcur, un["wq"], un["a"].shape, un["stride"], un["pad"])
            if j == 0 and ds is not None:
                gb["ds_w"] = L.conv2d_wgrad(g, un["a"], ds["wq"].shape, t["stride"], 0)
                da = da + q(L.conv2d_dgrad(g, ds["wq"], un["a"].shape, t["stride"], 0))
            da = q(da)
            du, dgam, dbet = L.bn_bwd(da * (un["z"] > 0), un["cache"], p[un["bn"] + "_g"].astype(np.float64))
            gb[un["bn"] + "_g"], gb[un["bn"] + "_b"] = dgam, dbet
            if j > 0:
                gcur = q(du)
            else:
                g = q(du + g) if ds is None else q(du)
        grads[b] = gb
    grads[-1] = {"conv_w": L.conv2d_wgrad(g, ximg, wstem.shape, 1, 1)}
    dx = L.conv2d_dgrad(g, wstem, ximg.shape, 1, 1) if need_input_grad else None
    return loss, grads, tape, dx


def units_last_name(model):
    return "conv2" if model["block_kind"] == 2 else "conv3"


def sgd_update(params, momentum_buf, grads, lr, mu, wd):
    """g <- g + wd*w ; v <- mu*v + g ; w <- w - lr*v on every trainable tensor (float64)."""
    new_p, new_v = {}, {}
    for b, gb in grads.items():
        new_p[b] = {k: np.asarray(v, np.float64).copy() for k, v in params[b].items()}
        new_v[b] = {k: np.asarray(v, np.float64).copy() for k, v in momentum_buf[b].items()}
        for name, g in gb.items():
            w = np.asarray(params[b][name], np.float64)
            gg = g + wd * w
            v = mu * np.asarray(momentum_buf[b][name], np.float64) + gg
            new_v[b][name] = v
            new_p[b][name] = w - lr * v
    return new_p, new_v


def local_step(model, blocks, params, momentum_buf, x, labels, lr, mu, wd, emulate_bf16=False):
    """One local SGD iteration of the sub-ResNet holding `blocks`.

    params / momentum_buf need entries for -1, every b in blocks, and B.
    Returns loss, grads, new_params (incl. updated BN running statistics), new_momentum.
    """
    loss, grads, tape, _ = forward_backward(model, blocks, params, x, labels, emulate_bf16=emulate_bf16)
    new_p, new_v = sgd_update(params, momentum_buf, grads, lr, mu, wd)
    mom = model["bn_momentum"]
    for (b, bn), (mean, var, m) in tape.stats.items():
        rm, rv = L.bn_running_update(np.asarray(params[b][bn + "_rm"], np.float64),
                                     np.asarray(params[b][bn + "_rv"], np.float64),
                                     mean, var, m, mom)
        new_p[b][bn + "_rm"], new_p[b][bn + "_rv"] = rm, rv
    return loss, grads, new_p, new_v


def forward_eval(model, blocks, params, x, branch_scale=None, labels=None):
    """Test-time forward pass (Sec. 2.6, "Scaling Activations"): BN normalises with the running
    statistics stored with each block, and the residual branch of block blocks[i] is multiplied by
    branch_scale[i] before the shortcut is added -- the paper scales the output of the partitioned
    blocks by 1/S when all of them are used together; blocks that every sub-ResNet trained get 1.
        out = ReLU(shortcut + branch_scale * BN(last conv of the branch))
    Returns the logits [N, classes] (and the mean cross-entropy if labels are given).  float64, no
    rounding anywhere."""
    tab = block_table(model)
    B = len(tab)
    eps = model["bn_eps"]
    if branch_scale is None:
        branch_scale = [1.0] * len(blocks)
    if is_preact(model):
        return _forward_eval_preact(model, blocks, params, x, branch_scale, labels)

    def cbn(a, p, conv, bn, stride, pad, relu, scale=1.0):
        y = L.conv2d_fwd(a, p[conv + "_w"], stride, pad)
        g, b = p[bn + "_g"].astype(np.float64), p[bn + "_b"].astype(np.float64)
        rm, rv = p[bn + "_rm"].astype(np.float64), p[bn + "_rv"].astype(np.float64)
        z = (y - rm[None, :, None, None]) / np.sqrt(rv + eps)[None, :, None, None] * g[None, :, None, None] \
            + b[None, :, None, None]
        z = scale * z
        return np.maximum(z, 0.0) if relu else z

    a = np.asarray(x, np.float64)
    if model["stem_kind"] == 0:
        a = cbn(a, params[-1], "conv", "bn", 1, 1, True)
    else:
        a, _ = L.maxpool_fwd(cbn(a, params[-1], "conv", "bn", 2, 3, True), 3, 2, 1)
    for b, sc in zip(blocks, branch_scale):
        t, p = tab[b], params[b]
        if model["block_kind"] == 0:
            h = cbn(a, p, "conv1", "bn1", t["stride"], 1, True)
            h = cbn(h, p, "conv2", "bn2", 1, 1, False, sc)
        else:
            h = cbn(a, p, "conv1", "bn1", 1, 0, True)
            h = cbn(h, p, "conv2", "bn2", t["stride"], 1, True)
            h = cbn(h, p, "conv3", "bn3", 1, 0, False, sc)
        short = cbn(a, p, "ds", "dsbn", t["stride"], 0, False) if t["has_ds"] else a
        a = np.maximum(h + short, 0.0)
    z = L.fc_fwd(L.avgpool_fwd(a), params[B]["fc_w"].astype(np.float64), params[B]["fc_b"].astype(np.float64))
    if labels is None:
        return z
    loss, _ = L.softmax_ce(z, np.asarray(labels))
    return z, loss


def _forward_eval_preact(model, blocks, params, x, branch_scale, labels):
    """forward_eval for pre-activation blocks:  out = shortcut + branch_scale * (last convolution of the branch)."""
    tab = block_table(model)
    B = len(tab)
    eps = model["bn_eps"]

    def bn_relu(u, p, bn):
        g, b = p[bn + "_g"].astype(np.float64), p[bn + "_b"].astype(np.float64)
        rm, rv = p[bn + "_rm"].astype(np.float64), p[bn + "_rv"].astype(np.float64)
        z = (u - rm[None, :, None, None]) / np.sqrt(rv + eps)[None, :, None, None] * g[None, :, None, None] \
            + b[None, :, None, None]
        return np.maximum(z, 0.0)

    u = L.conv2d_fwd(np.asarray(x, np.float64), params[-1]["conv_w"], 1, 1)
    for b, sc in zip(blocks, branch_scale):
        t, p = tab[b], params[b]
        xin, a1, h = u, None, u
        for bn, conv, k, stride, pad in _preact_layers(model, t):
            a = bn_relu(h, p, bn)
            a1 = a if a1 is None else a1
            h = L.conv2d_fwd(a, p[conv + "_w"], stride, pad)
        short = L.conv2d_fwd(a1, p["ds_w"], t["stride"], 0) if t["has_ds"] else xin
        u = short + sc * h
    f = bn_relu(u, params[B], "bn")
    z = L.fc_fwd(L.avgpool_fwd(f), params[B]["fc_w"].astype(np.float64), params[B]["fc_b"].astype(np.float64))
    if labels is None:
        return z
    loss, _ = L.softmax_ce(z, np.asarray(labels))
    return z, loss
