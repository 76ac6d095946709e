"""GPU parity: resist_local_step and resist_aggregate, through the C ABI, against the oracle on
the same seeded inputs.  fp32 bound: |gpu - oracle| <= 1e-5 + 1e-4*|oracle| element-wise on the
loss, every weight gradient and every updated parameter."""
import numpy as np
import pytest
import torch

import paper_2107_00961_amd as R
from oracle import aggregate as OA
from oracle import partition as OP
from oracle import resnet as OR
from paper_2107_00961_amd.harness import DeviceModel, SubResNet, to_device_batch
from resist_inputs import get_config, make_batch, make_params, zeros_like_params
from tests.bf16_cases import bf16_cases
from tests.gpu_util import assert_close, bf16_step_check, compare_trees, full_size_check

pytestmark = pytest.mark.gpu


def _small_models():
    basic = get_config("cfg1")["model"]
    return {
        "cfg1": (basic, [0, 1], 4),
        "strided_sub": (dict(basic, widths=[16, 32, 64], blocks=[2, 3, 2], in_h=16, in_w=16, num_classes=10),
                        [0, 2, 3, 5], 6),                      # blocks 1, 4, 6 dropped
        "bottleneck_sub": (dict(basic, block_kind=1, stem_kind=1, widths=[16, 32], blocks=[2, 3], in_h=40, in_w=40,
                                num_classes=12), [0, 2, 4], 5),  # 7x7 stem + max-pool, bottlenecks
        "ragged": (dict(basic, widths=[16, 32], blocks=[2, 2], in_h=12, in_w=12, num_classes=3), [0, 1, 2, 3], 3),
        # pre-activation blocks (the paper's preferred architecture, Sec. 2.1)
        "preact_sub": (dict(basic, block_kind=2, widths=[16, 32, 64], blocks=[2, 3, 2], in_h=16, in_w=16, num_classes=10),
                       [0, 2, 3, 5], 6),
        "preact_bottleneck_sub": (dict(basic, block_kind=3, widths=[16, 32], blocks=[2, 3], in_h=12, in_w=12, num_classes=7),
                                  [0, 2, 4], 5),
        "preact_full": (dict(basic, block_kind=2, widths=[16, 32], blocks=[2, 2], in_h=12, in_w=12, num_classes=3),
                        [0, 1, 2, 3], 3),
        # one image per batch (BN statistics over the spatial positions alone), and a classifier whose
        # class count and batch leave ragged tails in every tile of its three kernels
        "one_image": (dict(basic, widths=[16, 32], blocks=[2, 2], in_h=8, in_w=8, num_classes=5), [0, 2, 3], 1),
        "ragged_head": (dict(basic, widths=[16, 32], blocks=[2, 2], in_h=8, in_w=8, num_classes=37), [0, 1, 2], 17),
        # channel counts that leave ragged tiles in every kernel: 48, 80 (and 192, 320) in bottleneck blocks
        "odd_widths": (dict(basic, block_kind=1, widths=[48, 80], blocks=[2, 2], in_h=12, in_w=12, num_classes=6),
                       [0, 1, 2, 3], 5),
        # images that are not square, through a strided stage and, in the second case, the 7x7 stem and the max-pool
        "rectangular": (dict(basic, widths=[16, 32], blocks=[2, 2], in_h=12, in_w=20, num_classes=5), [0, 1, 2, 3], 3),
        "rectangular_bottleneck": (dict(basic, block_kind=1, stem_kind=1, widths=[16, 32], blocks=[1, 2], in_h=24, in_w=40,
                                        num_classes=5), [0, 1, 2], 3),
        # four stages on 8x8 images: the last stage works on one pixel per image, its BNs on 6 values per channel.
        # (Batch 3 is too badly conditioned for an fp32 bound: in the float64 oracle itself an input perturbed by
        # 6e-8 moves that stage's filter gradients by 9e-6 in norm, thirty times what it does at batch 6.)
        "one_pixel": (dict(basic, widths=[16, 32, 64, 128], blocks=[1, 1, 1, 1], in_h=8, in_w=8, num_classes=4), [0, 1, 2, 3], 6),
    }


def _run_steps(model, blocks, batch, steps, lr, mu, wd, seed=0, perturb_bn=True):
    params = make_params(model, seed, perturb_bn=perturb_bn)
    sub = SubResNet(model, blocks, params, batch)
    o_params, o_mom = params, zeros_like_params(params)
    for it in range(steps):
        x, y = make_batch(model, batch, 100 * seed + it)
        print(f"step {it} blocks {blocks} batch {batch}", flush=True)
        xd, yd = to_device_batch(x, y)
        sub.step(xd, yd, lr, mu, wd)
        torch.cuda.synchronize()
        loss, grads, o_params, o_mom = OR.local_step(model, blocks, o_params, o_mom, x, y, lr, mu, wd)
        assert_close(sub.loss.cpu().numpy()[0], loss, f"loss step {it}")
        compare_trees(sub.download_grads(), grads, f"grad step {it}")
        got = sub.download()
        compare_trees(got, {k: o_params[k] for k in sub.keys}, f"params step {it}")
        compare_trees(sub.download_momentum(), {k: {n: v for n, v in o_mom[k].items() if OR.is_trainable(n)}
                                                for k in sub.keys}, f"momentum step {it}")
    return sub


@pytest.mark.parametrize("name", ["cfg1", "strided_sub", "bottleneck_sub", "ragged", "preact_sub", "preact_bottleneck_sub",
                                  "preact_full", "one_image", "ragged_head", "odd_widths", "rectangular",
                                  "rectangular_bottleneck", "one_pixel"])
def test_local_step_small(name):
    model, blocks, batch = _small_models()[name]
    # data seeds for which the oracle's closest ReLU decision is > 1e-5 from a tie (seed 0 of
    # "preact_full" has one at 1.6e-8: no fp32 evaluation can be expected to decide it the same way)
    seed = {"preact_full": 1}.get(name, 0)
    _run_steps(model, blocks, batch, steps=2, lr=0.1, mu=0.9, wd=5e-4, seed=seed)


@pytest.mark.parametrize("name", ["cfg1", "strided_sub", "bottleneck_sub", "ragged"])
def test_local_step_small_bn_first_pass_from_the_data_gradient(name):
    """In bf16 steps the stride-1 data gradients leave the first pass of the next BN backward (per-row-tile
    sums) from their epilogue.  Switched on for fp32 here, the same code meets the element-wise fp32 bound
    against the oracle: gradients, updated parameters and momentum over two steps (strided layers and the
    shortcut BNs keep the separate pass; "ragged" has a short last row tile)."""
    model, blocks, batch = _small_models()[name]
    try:
        R.set_bn_fusion(2)
        _run_steps(model, blocks, batch, steps=2, lr=0.1, mu=0.9, wd=5e-4, seed=0)
    finally:
        R.set_bn_fusion(1)


@pytest.mark.parametrize("beta", [6.0, 50.0])
def test_bn_input_with_mean_far_from_zero(beta):
    """Every BN offset set to `beta`: every activation is beta + O(1), so the convolution outputs the
    next BN normalises have a mean of beta * (sum of the filter) against a deviation of about the
    filter's root sum of squares: |mean|/std reaches ~50 for beta = 6 and ~400 for beta = 50.  The
    batch variance must not be formed as a difference of large sums.  No ReLU is near a tie here.
    beta = 6: the element-wise bound on everything.  beta = 50: fp32 storage of the convolution output
    itself (2^-24 * |mean|/std = 2.5e-5 of a standard deviation per element, more after fp32
    accumulation) is what limits the step, so the element-wise bound is kept for the loss and the
    batch statistics, and each gradient tensor gets max|gpu - oracle| <= 1e-5 + 5e-3*max|oracle| (measured:
    1e-3 of the norm on the worst tensor that does not cancel to nothing)."""
    model, blocks, batch = _small_models()["strided_sub"]
    params = make_params(model, 2, perturb_bn=True)
    for k in params:
        for name in params[k]:
            if name.endswith("_b") and not name.startswith("fc"):
                params[k][name] = np.full_like(params[k][name], beta)
    x, y = make_batch(model, batch, 7)
    sub = SubResNet(model, blocks, params, batch)
    xd, yd = to_device_batch(x, y)
    sub.step(xd, yd, 0.01, 0.9, 5e-4)
    torch.cuda.synchronize()
    loss, grads, new_p, _ = OR.local_step(model, blocks, params, zeros_like_params(params), x, y, 0.01, 0.9, 5e-4)
    _, _, tape, _ = OR.forward_backward(model, blocks, params, x, y, backward=False)
    far = max(float(np.max(np.abs(m) / np.sqrt(v + 1e-30))) for (m, v, _) in tape.stats.values())
    print(f"largest |mean|/std of a BN input: {far:.0f}", flush=True)
    assert far >= 5 * beta
    assert_close(sub.loss.cpu().numpy()[0], loss, "loss")
    got, got_g = sub.download(), sub.download_grads()
    worst_rv = worst_g = 0.0
    for k in sub.keys:                      # batch statistics, seen through the running statistics
        for name in new_p[k]:
            if name.endswith(("_rv", "_rm")):
                assert_close(got[k][name], new_p[k][name], f"running statistic block {k} {name}")
            if name.endswith("_rv"):
                worst_rv = max(worst_rv, float(np.max(np.abs(got[k][name] - new_p[k][name]) / np.abs(new_p[k][name]))))
        for name, g in grads[k].items():
            r = float(np.linalg.norm(got_g[k][name] - g) / np.linalg.norm(g))
            worst_g = max(worst_g, r)
    print(f"beta {beta}: worst relative error of a running variance {worst_rv:.2e}, worst gradient tensor (rel L2) {worst_g:.2e}", flush=True)
    if beta <= 6.0:
        compare_trees(got_g, grads, "grad")
        compare_trees(got, {k: new_p[k] for k in sub.keys}, "params")
    else:
        # every weight gradient is a sum of (gradient x activation) with activations of 50-100 whose
        # offset part cancels exactly in exact arithmetic (a BN's output gradients sum to zero), and some
        # (a BN offset followed by another BN) cancel to 1e-5 of their terms: errors are measured against
        # the largest entry of the tensor
        for k in sub.keys:
            for name, g in grads[k].items():
                err = float(np.max(np.abs(got_g[k][name] - g)))
                assert err <= 1e-5 + 5e-3 * float(np.max(np.abs(g))), f"grad block {k} {name}: max error {err:.2e}"


def test_cfg1_exact_config():
    cfg = get_config("cfg1")
    _run_steps(cfg["model"], [0, 1], cfg["batch"], 1, cfg["lr"], cfg["momentum"], cfg["weight_decay"],
               seed=cfg["data_seed"], perturb_bn=False)


def test_absent_blocks_untouched_and_deterministic():
    model, blocks, batch = _small_models()["strided_sub"]
    params = make_params(model, 3)
    x, y = make_batch(model, batch, 4)
    xd, yd = to_device_batch(x, y)
    outs = []
    for rep in range(2):
        sub = SubResNet(model, blocks, params, batch)
        sub.step(xd, yd, 0.1, 0.9, 1e-4)
        torch.cuda.synchronize()
        outs.append([p.cpu().numpy().copy() for p in sub.params] + [sub.loss.cpu().numpy().copy()])
    for a, b in zip(*outs):
        assert a.tobytes() == b.tobytes()           # bit-identical from run to run


def test_step_rejects_small_workspace():
    model, blocks, batch = _small_models()["cfg1"]
    sub = SubResNet(model, blocks, make_params(model, 0), batch)
    x, y = to_device_batch(*make_batch(model, batch, 0))
    sub.workspace = sub.workspace[:1024]
    with pytest.raises(R.ResistError, match="workspace"):
        sub.step(x, y, 0.1, 0.9, 0.0)


@pytest.mark.parametrize("S", [3, 7, 13])      # 4, 8 and 16 sources per kernel instance
def test_aggregate_matches_oracle_and_invariants(S):
    model = dict(get_config("cfg1")["model"], widths=[16, 32], blocks=[4, 5], in_h=8, in_w=8)
    g = make_params(model, 0, perturb_bn=True)
    subs, owner = R.partition(model, S, 0, 9, 0)
    assert (subs, owner) == OP.partition(model["blocks"], S, 0, 9, 0)
    assert S != 3 or (1 in owner and 2 in owner)
    nb = R.num_blocks(model)
    rng = np.random.default_rng(1)
    sub_logical = []
    for s in range(S):
        d = {k: {n: (v + rng.standard_normal(v.shape).astype(np.float32)) for n, v in g[k].items()}
             for k in [-1] + subs[s] + [nb]}
        sub_logical.append(d)
    devs = [DeviceModel(model, subs[s], sub_logical[s]) for s in range(S)]
    glob = DeviceModel(model, list(range(nb)), g)
    R.aggregate(model, subs, [d.params for d in devs], glob.params)
    torch.cuda.synchronize()
    want = OA.aggregate(g, subs, sub_logical)
    got = glob.download()
    for k in want:
        for n in want[k]:
            if owner[k] == 1 if 0 <= k < nb else False:
                holder = [s for s in range(S) if k in subs[s]][0]
                assert got[k][n].tobytes() == sub_logical[holder][k][n].tobytes()   # bitwise copy
            else:
                assert_close(got[k][n], want[k][n], f"aggregate {k} {n}", rtol=max(2e-7, 6e-8 * S), atol=1e-7)
    # identical copies -> identity (exact for 1, 2, 4 holders; S = 3 within one rounding)
    same = [DeviceModel(model, subs[s], g) for s in range(S)]
    glob2 = DeviceModel(model, list(range(nb)), zeros_like_params(g))
    R.aggregate(model, subs, [d.params for d in same], glob2.params)
    torch.cuda.synchronize()
    got2 = glob2.download()
    for k in g:
        for n in g[k]:
            np.testing.assert_allclose(got2[k][n], g[k][n], rtol=max(2e-7, 6e-8 * S), atol=0)   # up to S fp32 roundings
    # a block held by nobody keeps its value: drop sub-ResNet 0 and aggregate the rest
    lonely = [b for b in range(nb) if owner[b] == 1 and b in subs[0]]
    assert lonely or S != 3
    glob3 = DeviceModel(model, list(range(nb)), g)
    R.aggregate(model, subs[1:], [d.params for d in devs[1:]], glob3.params)
    torch.cuda.synchronize()
    got3 = glob3.download()
    for b in lonely:
        for n in g[b]:
            assert got3[b][n].tobytes() == g[b][n].tobytes()


# ---- bf16 storage (compute_dtype = 1): cases in tests/bf16_cases.py, checks in gpu_util.bf16_step_check
@pytest.mark.parametrize("name", ["cfg1", "strided_sub", "bottleneck_sub", "ragged", "preact_sub", "preact_bottleneck_sub",
                                  "odd_widths"])
def test_local_step_small_bf16(name):
    bf16_step_check(f"bf16 {name}")


@pytest.mark.parametrize("name", ["basic", "strided", "bottleneck", "preact"])
def test_local_step_shallow_bf16_matches_emulation(name):
    bf16_step_check(f"bf16 shallow {name}")


def test_cfg4_shape_reduced_bf16():
    """The ImageNet-shaped configuration's layer types (7x7 stride-2 stem, max-pool, bottleneck
    blocks with downsample shortcuts, bf16 storage) at its real channel widths, reduced depth,
    batch and image size."""
    bf16_step_check("cfg4 reduced")


def test_cfg4_full_depth_small_batch_bf16():
    """The ImageNet-shaped configuration itself -- 224x224 images, 1000 classes, its own partition
    (seed 2, S=2, sub-ResNet 0: ten bottleneck blocks), bf16 storage -- at batch 4 instead of 64."""
    cfg = get_config("cfg4")
    subs, _ = R.partition(cfg["model"], cfg["S"], cfg["min_depth"], cfg["part_seed"], 0)
    assert subs[0] == bf16_cases()["cfg4 batch 4"]["blocks"]
    bf16_step_check("cfg4 batch 4")


def test_cfg2_full_size_step():
    """The benchmark configuration itself: CIFAR-shaped sub-ResNet 0 of S=4, batch 128."""
    full_size_check("cfg2", "cfg2")


def test_cfg3_full_size_step_of_another_subresnet():
    """cfg3 (100 classes): the first local step of sub-ResNet 2 of the round, on its own batch."""
    full_size_check("cfg3", "cfg3 sub 2", which=2)


def test_cfg2_widths_reduced_depth_strict():
    """Same channel widths and tile shapes as the benchmark network, strict element-wise bound.

    The bound can only hold where no ReLU decision is within fp32 rounding distance of a tie, and
    with z ~ N(0,1) pre-activations a network with D decisions has about 0.8*D*m of them within m of
    zero.  The case is therefore kept small (batch 2, 16x16 images, ~0.5 M decisions) and the data
    seed is the first one for which the oracle's closest decision is at least 1e-5 away from a tie
    (fp32 accumulation over up to 4608 terms moves a normalised value by ~1e-6)."""
    model = dict(get_config("cfg2")["model"], blocks=[2, 2, 3, 2], in_h=16, in_w=16)
    blocks, batch = [0, 1, 2, 4, 6, 7, 8], 2
    params = make_params(model, 0, perturb_bn=False)
    for seed in range(40):
        x, y = make_batch(model, batch, 100 * seed)
        _, _, tape, _ = OR.forward_backward(model, blocks, params, x, y, backward=False)
        print(f"seed {seed}: closest ReLU decision {tape.relu_margin:.2e}", flush=True)
        if tape.relu_margin >= 1e-5:
            break
    else:
        pytest.fail("no seed with a clear ReLU margin")
    _run_steps(model, blocks, batch, steps=1, lr=0.1, mu=0.9, wd=5e-4, seed=seed, perturb_bn=False)


@pytest.mark.parametrize("name", ["strided_sub", "bottleneck_sub", "preact_full", "preact_bottleneck_sub"])
@pytest.mark.parametrize("bf16", [False, True])
def test_second_stream_changes_no_bit(name, bf16):
    """The weight gradients run on the library's second stream by default.  Three consecutive steps
    with it give the same bits -- parameters, momentum, gradients, loss -- as with every kernel on the
    caller's stream: the events order every buffer reuse."""
    model, blocks, batch = _small_models()[name]
    if bf16:
        model = dict(model, compute_dtype=1)
    params = make_params(model, 5, perturb_bn=True)
    outs = []
    try:
        for overlap in (0, 2, 2):            # 2: also for steps this small
            R.set_overlap(overlap)
            sub = SubResNet(model, blocks, params, batch)
            for it in range(3):
                xd, yd = to_device_batch(*make_batch(model, batch, 40 + it))
                sub.step(xd, yd, 0.05, 0.9, 1e-4)
            torch.cuda.synchronize()
            outs.append([t.cpu().numpy().copy() for t in sub.params + sub.momentum + sub.grads] + [sub.loss.cpu().numpy().copy()])
    finally:
        R.set_overlap(True)
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert a.tobytes() == b.tobytes()


@pytest.mark.parametrize("bf16", [False, True])
def test_second_stream_changes_no_bit_when_a_step_takes_more_events_than_the_ring_holds(bf16):
    """The events that order the two streams come from a ring of 256 per device.  A step of a 90-block
    network records about 370 of them, so the ring wraps inside a step; every event that is still to be
    waited for must have been waited for by then.  Same check as above: bit-identical to one stream."""
    basic = get_config("cfg1")["model"]
    model = dict(basic, widths=[16, 32], blocks=[45, 45], in_h=8, in_w=8, num_classes=10, compute_dtype=1 if bf16 else 0)
    blocks, batch = list(range(90)), 8
    params = make_params(model, 9, perturb_bn=True)
    outs = []
    try:
        for overlap in (0, 2):
            R.set_overlap(overlap)
            sub = SubResNet(model, blocks, params, batch)
            for it in range(3):
                xd, yd = to_device_batch(*make_batch(model, batch, 70 + it))
                sub.step(xd, yd, 0.01, 0.9, 1e-4)
            torch.cuda.synchronize()
            outs.append([t.cpu().numpy().copy() for t in sub.params + sub.momentum + sub.grads] + [sub.loss.cpu().numpy().copy()])
    finally:
        R.set_overlap(True)
    assert np.isfinite(outs[0][-1]).all()
    for a, b in zip(*outs):
        assert a.tobytes() == b.tobytes()


@pytest.mark.parametrize("workload", ["cfg2", "cfg2_preact", "cfg4"])
def test_second_stream_changes_no_bit_full_size(workload):
    """The same at the sizes the benchmark times, where kernels on the two streams really run
    side by side for most of the backward pass."""
    cfg = get_config(workload)
    model, batch = cfg["model"], cfg["batch"]
    if workload == "cfg4":
        batch = 16
    subs, _ = R.partition(model, cfg["S"], cfg.get("min_depth", 0), cfg["part_seed"], 0)
    params = make_params(model, 0)
    xd, yd = to_device_batch(*make_batch(model, batch, cfg["data_seed"]))
    outs = []
    try:
        for overlap in (False, True):
            R.set_overlap(overlap)
            sub = SubResNet(model, subs[0], params, batch)
            for it in range(3):
                sub.step(xd, yd, cfg["lr"] * 0.01, cfg["momentum"], cfg["weight_decay"])
            torch.cuda.synchronize()
            outs.append([t.cpu().numpy().copy() for t in sub.params + sub.momentum + sub.grads] + [sub.loss.cpu().numpy().copy()])
            del sub
    finally:
        R.set_overlap(True)
    for a, b in zip(*outs):
        assert a.tobytes() == b.tobytes()


@pytest.mark.parametrize("workload", ["cfg2", "cfg4", "cfg5_bf16"])
def test_bn_first_pass_from_the_data_gradient_full_size(workload):
    """The first pass of the BN backward taken by the data gradients' epilogue (bf16 default) against the
    separate pass, at the benchmark's sizes and tile configurations (128-row tiles whose epilogue runs
    in groups of passes, eight-wave tiles): one step each way from the same state.  The two differ only
    in how the per-channel sums are accumulated (fp32 per row tile, then float64, against float64
    throughout).  In fp32 every gradient tensor then agrees to 1e-5 of its norm.  In bf16 a change in
    the last bit of a sum moves a few stored gradients by one bf16 ulp, and the backward pass of a deep
    BN network amplifies that on the way down (2e-4 in the last block, 2e-2 at the stem of the 33-block
    model, 6e-2 at the ImageNet-shaped stem): the bound there is 0.15 -- an indexing error in the fused
    sums would put the BN parameter gradients of its layer off by O(1) at any depth -- and 5e-3 on the
    last block, where nothing has been amplified yet."""
    cfg = get_config(workload)
    model, batch = cfg["model"], cfg["batch"]
    subs, _ = R.partition(model, cfg["S"], cfg.get("min_depth", 0), cfg["part_seed"], 0)
    params = make_params(model, 0)
    xd, yd = to_device_batch(*make_batch(model, batch, cfg["data_seed"]))
    outs = []
    try:
        for mode in (0, 2):
            R.set_bn_fusion(mode)
            sub = SubResNet(model, subs[0], params, batch)
            sub.step(xd, yd, cfg["lr"], cfg["momentum"], cfg["weight_decay"])
            torch.cuda.synchronize()
            outs.append((sub.download_grads(), float(sub.loss.cpu()[0])))
            keys = sub.keys
            del sub
    finally:
        R.set_bn_fusion(1)
    assert outs[0][1] == outs[1][1]                      # the forward pass is the same code
    bf16 = model.get("compute_dtype", 0) == 1
    last = max(k for k in keys if k < R.num_blocks(model))
    worst, worst_last = 0.0, 0.0
    for k in keys:
        for name, a in outs[0][0][k].items():
            a = a.astype(np.float64)
            rel = float(np.linalg.norm(a - outs[1][0][k][name]) / max(np.linalg.norm(a), 1e-30))
            worst = max(worst, rel)
            if k == last:
                worst_last = max(worst_last, rel)
    print(f"{workload}: gradients with and without the fused first pass differ by at most {worst:.2e} "
          f"(relative L2 per tensor), {worst_last:.2e} in the last block", flush=True)
    assert 0.0 < worst <= (0.15 if bf16 else 1e-5), worst        # > 0: the fused path really ran
    assert worst_last <= (5e-3 if bf16 else 1e-5), worst_last


def test_aggregate_full_size_cfg3():
    """Reassembly of the CIFAR-shaped global model (cfg3: 41 M parameters, S = 4) at the size the round
    benchmark times: sampled blocks against the oracle, single-owner blocks bit for bit."""
    cfg = get_config("cfg3")
    model, S = cfg["model"], cfg["S"]
    nb = R.num_blocks(model)
    subs, owner = R.partition(model, S, 0, cfg["part_seed"], 0)
    assert (subs, owner) == OP.partition(model["blocks"], S, 0, cfg["part_seed"], 0)
    g = make_params(model, 0, perturb_bn=True)
    rng = np.random.default_rng(0)
    logical = [{k: {n: (v + np.float32(0.01 * (s + 1)) * rng.standard_normal(v.shape).astype(np.float32)) for n, v in g[k].items()}
                for k in [-1] + subs[s] + [nb]} for s in range(S)]
    devs = [DeviceModel(model, subs[s], logical[s]) for s in range(S)]
    glob = DeviceModel(model, list(range(nb)), g)
    R.aggregate(model, subs, [d.params for d in devs], glob.params)
    torch.cuda.synchronize()
    got = glob.download()
    sample = [-1, 0, 3, 4, 7, 20, 30, 32, nb]
    checked = 0
    for k in sample:
        holders = [s for s in range(S) if k in (-1, nb) or k in subs[s]]
        for n in g[k]:
            if len(holders) == 1:
                assert got[k][n].tobytes() == logical[holders[0]][k][n].tobytes(), (k, n)
            else:
                acc = np.zeros(g[k][n].shape, np.float64)
                for s in holders:
                    acc += logical[s][k][n]
                assert_close(got[k][n], acc / len(holders), f"cfg3 reassembly {k} {n}", rtol=3e-7, atol=1e-7)
            checked += 1
    assert checked > 50 and any(owner[b] == 1 for b in sample if 0 <= b < nb)
