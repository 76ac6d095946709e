"""The bf16 step-parity cases as plain data: what each GPU test steps, and what
tests/golden/make_bf16_storage_reach.py evaluates with the oracle alone."""
from oracle import partition as OP
from resist_inputs import get_config


def _small_models():
    basic = get_config("cfg1")["model"]
    return {
        "cfg1": (basic, [0, 1], 4),
        "strided_sub": (dict(basic, widths=[16, 32, 64], blocks=[2, 3, 2], in_h=16, in_w=16, num_classes=10), [0, 2, 3, 5], 6),
        "bottleneck_sub": (dict(basic, block_kind=1, stem_kind=1, widths=[16, 32], blocks=[2, 3], in_h=40, in_w=40,
                                num_classes=12), [0, 2, 4], 5),
        "ragged": (dict(basic, widths=[16, 32], blocks=[2, 2], in_h=12, in_w=12, num_classes=3), [0, 1, 2, 3], 3),
        "preact_sub": (dict(basic, block_kind=2, widths=[16, 32, 64], blocks=[2, 3, 2], in_h=16, in_w=16, num_classes=10),
                       [0, 2, 3, 5], 6),
        "preact_bottleneck_sub": (dict(basic, block_kind=3, widths=[16, 32], blocks=[2, 3], in_h=12, in_w=12, num_classes=7),
                                  [0, 2, 4], 5),
        # channel counts that leave ragged tiles in every kernel: 48, 80 (and 192, 320) in bottleneck blocks
        "odd_widths": (dict(basic, block_kind=1, widths=[48, 80], blocks=[2, 2], in_h=12, in_w=12, num_classes=6),
                       [0, 1, 2, 3], 5),
    }


def _shallow_models():
    basic = get_config("cfg1")["model"]
    return {
        "basic": (dict(basic, widths=[64], blocks=[1], in_h=16, in_w=16), [0], 16, 5e-3),
        "strided": (dict(basic, widths=[32, 64], blocks=[1, 1], in_h=16, in_w=16), [0, 1], 16, 5e-3),
        # behind a max-pool the step is sensitive to the last bit of the BN statistics: the same kernels with
        # 64-row instead of 128-row statistic tiles (identical convolution outputs) move these gradients by 1-3e-2
        "bottleneck": (dict(basic, block_kind=1, stem_kind=1, widths=[32], blocks=[1], in_h=32, in_w=32), [0], 16, 6e-2),
        "preact": (dict(basic, block_kind=2, widths=[32, 64], blocks=[1, 1], in_h=16, in_w=16), [0, 1], 16, 5e-3),
    }


def bf16_cases():
    """name -> dict(model, blocks, batch, lr, mu, wd, seed, perturb_bn, data_seed, emu_bar)."""
    out = {}
    for name, (model, blocks, batch) in _small_models().items():
        out[f"bf16 {name}"] = dict(model=model, blocks=blocks, batch=batch, lr=0.1, mu=0.9, wd=5e-4, seed=1,
                                   perturb_bn=True, data_seed=100, emu_bar=None)
    for name, (model, blocks, batch, bar) in _shallow_models().items():
        out[f"bf16 shallow {name}"] = dict(model=model, blocks=blocks, batch=batch, lr=0.1, mu=0.9, wd=5e-4, seed=3,
                                           perturb_bn=True, data_seed=300, emu_bar=bar)
    c4 = get_config("cfg4")
    subs4, _ = OP.partition(c4["model"]["blocks"], c4["S"], c4["min_depth"], c4["part_seed"], 0)
    common4 = dict(lr=c4["lr"], mu=c4["momentum"], wd=c4["weight_decay"], perturb_bn=False, emu_bar=None)
    # the ImageNet-shaped configuration's layer types at its real channel widths, reduced depth, batch and image size
    out["cfg4 reduced"] = dict(model=dict(c4["model"], blocks=[2, 2, 2, 2], in_h=96, in_w=96, num_classes=100),
                               blocks=[0, 1, 2, 4, 5, 6], batch=16, seed=2, data_seed=200, **common4)
    # the configuration itself at batch 4 instead of 64
    out["cfg4 batch 4"] = dict(model=c4["model"], blocks=subs4[0], batch=4, seed=0, data_seed=0, **common4)
    for which in (0, 1):
        out[f"cfg4 sub {which} batch 64"] = dict(model=c4["model"], blocks=subs4[which], batch=c4["batch"], seed=0,
                                                 data_seed=c4["data_seed"] + 1000 * which, **common4)
    c5 = get_config("cfg5_bf16")
    out["cfg5 bf16"] = dict(model=c5["model"], blocks=list(range(sum(c5["model"]["blocks"]))), batch=c5["batch"],
                            lr=c5["lr"], mu=c5["momentum"], wd=c5["weight_decay"], seed=0, perturb_bn=False,
                            data_seed=c5["data_seed"], emu_bar=None)
    return out
