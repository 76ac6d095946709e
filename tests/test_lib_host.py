"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every declared symbol,
and its host-only calls (partition, sizes, layout, argument validation) agree with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2107_00961_amd as R
from oracle import partition as OP
from oracle import resnet as OR
from resist_inputs import get_config, make_params

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_every_declared_symbol():
    lib = R.lib()
    declared = set()
    for hdr in ("resist.h", "resist_ops.h"):
        src = open(os.path.join(ROOT, "include", hdr)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        declared |= set(re.findall(r"\b(resist_[a-z0-9_]+)\s*\(", src))
    assert {"resist_partition", "resist_local_step", "resist_aggregate"} <= declared
    for name in declared:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("cfg,S,min_depth", [("cfg1", 1, 0), ("cfg2", 4, 0), ("cfg4", 2, 0), ("cfg2", 8, 5),
                                             ("cfg2", 3, 12), ("cfg2", 16, 0), ("cfg4", 5, 10)])
def test_partition_bit_exact(cfg, S, min_depth):
    model = get_config(cfg)["model"]
    for seed in (0, 1, 2, 12345678901234567890):
        for rnd in (0, 1, 7):
            assert R.partition(model, S, min_depth, seed, rnd) == OP.partition(model["blocks"], S, min_depth, seed, rnd)


def test_partition_paper_mask_and_errors():
    model = get_config("cfg3")["model"]
    nb = R.num_blocks(model)
    mask = [1 if 7 < b < 30 else 0 for b in range(nb)]
    for S, md in ((2, 0), (4, 0), (8, 4)):
        assert R.partition(model, S, md, 3, 2, mask) == OP.partition(model["blocks"], S, md, 3, 2, mask)
    with pytest.raises(R.ResistError):
        R.partition(model, 0, 0, 0, 0)
    with pytest.raises(R.ResistError):
        R.partition(model, 2, -1, 0, 0)
    # capacity error: nothing is written past cap
    d = R.model_desc(model)
    offs = (ctypes.c_int32 * 5)()
    blocks = (ctypes.c_int32 * 8)(*([-7] * 8))
    owner = (ctypes.c_int32 * nb)()
    rc = R.lib().resist_partition(ctypes.byref(d), None, 4, 0, 1, 0, offs, blocks, 8, owner)
    assert rc == -3 and list(blocks) == [-7] * 8
    assert b"cap" in R.lib().resist_last_error()


@pytest.mark.parametrize("cfg", ["cfg1", "cfg2", "cfg3", "cfg4"])
def test_param_counts_and_layout(cfg):
    model = get_config(cfg)["model"]
    nb = R.num_blocks(model)
    assert nb == sum(model["blocks"])
    params = make_params(model, 0, perturb_bn=True)
    for b in range(-1, nb + 1):
        tot, tr = R.block_param_count(model, b)
        lay = R.block_layout(model, b)
        assert sum(t["count"] for t in lay if t["kind"] not in (3, 4)) == OR.param_count(model, b)
        assert sum(t["count"] for t in lay) == OR.param_count(model, b, trainable_only=False)
        assert all(t["offset"] % 4 == 0 for t in lay)
        assert tr <= tot and tr % 4 == 0 and tot % 4 == 0
        ends = [t["offset"] + t["count"] for t in lay]
        assert all(lay[i + 1]["offset"] >= ends[i] for i in range(len(lay) - 1)) and ends[-1] <= tot
        # pack -> unpack is the identity on logical tensors
        flat = R.pack_block(model, b, params[b])
        back = R.unpack_block(model, b, flat)
        assert set(back) == set(params[b])
        for k in back:
            np.testing.assert_array_equal(back[k], params[b][k])


def test_conv_weight_layout_is_krsc():
    model = get_config("cfg1")["model"]
    w = np.arange(16 * 16 * 9, dtype=np.float32).reshape(16, 16, 3, 3)
    flat = R.pack_block(model, 0, {"conv1_w": w})
    k, c, r, s = 5, 7, 2, 1
    assert flat[((k * 3 + r) * 3 + s) * 16 + c] == w[k, c, r, s]


def test_workspace_and_step_argument_errors():
    model = get_config("cfg2")["model"]
    with pytest.raises(R.ResistError, match="first block"):
        R.workspace_bytes(model, [0, 1, 2], 8)
    with pytest.raises(R.ResistError, match="ascending"):
        R.workspace_bytes(model, [0, 3, 3, 7, 30], 8)
    with pytest.raises(R.ResistError):
        R.workspace_bytes(model, [0, 3, 7, 30, 99], 8)
    with pytest.raises(R.ResistError):
        R.workspace_bytes(model, [0, 3, 7, 30], 0)
    assert R.workspace_bytes(model, [0, 3, 7, 30], 8) > 0
    bad = dict(model, widths=[60, 128, 256, 512])
    with pytest.raises(R.ResistError, match="multiple of 16"):
        R.num_blocks(bad)
    # NULL buffers are refused before anything is launched (no GPU needed to see the error)
    d = R.model_desc(model)
    blocks = (ctypes.c_int32 * 4)(0, 3, 7, 30)
    rc = R.lib().resist_local_step(ctypes.byref(d), blocks, 4, None, None, None, None, None, 8, 0.1, 0.9, 0.0,
                                   None, 0, None, None)
    assert rc == -1
