"""Pins for oracle/partition.py (Sec. 2.2, Fig. 1, Table 1, Sec. 2.6 'Subnetwork Depth')."""
import os

import pytest

from oracle import partition as OP
from oracle import resnet as OR
from resist_inputs import get_config


def _read(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_splitmix64_vector(golden_dir):
    want = [int(r[0], 16) for r in _read(golden_dir, "splitmix64_vector.txt")]
    rng = OP.SplitMix64(0)
    assert [rng.next(), rng.next()] == want


def test_fig1_shape(golden_dir):
    P, S, per_sub, shared = map(int, _read(golden_dir, "fig1_example.txt")[0])
    for seed in range(20):
        subs, owner = OP.partition([P + 1], S, 0, seed, 0)   # block 0 is the stage's fixed first block
        dealt = [[b for b in s if b != 0] for s in subs]
        assert all(len(d) == per_sub for d in dealt)
        assert sum(1 for b in range(1, P + 1) if owner[b] == 2) == shared
        assert all(owner[b] >= 1 for b in range(P + 1))
        assert set(dealt[0]) | set(dealt[1]) == set(range(1, P + 1))


def test_table1_bytes(golden_dir):
    """Bytes per round = 2 * machines * 4 B * (parameters of one worker's network)."""
    cfg = get_config("cfg3")                     # ResNet101-shaped, 100 classes
    model = cfg["model"]
    nblk = sum(model["blocks"])
    full = sum(OR.param_count(model, b) for b in range(-1, nblk + 1))
    assert full == 41_399_716
    first3 = model["blocks"][0] + model["blocks"][1]
    # the paper partitions only the non-strided blocks of the third section
    mask = [1 if first3 < b < first3 + model["blocks"][2] else 0 for b in range(nblk)]
    for m, lsgd_gb, resist_gb in _read(golden_dir, "table1_bytes.txt"):
        M = int(m)
        assert abs(2 * M * 4 * full / 1e9 - float(lsgd_gb)) < 1e-3
        min_depth = 4 if M == 8 else 0        # Table 1's 8-machine entry implies 4 dealt blocks
        subs, owner = OP.partition(model["blocks"], M, min_depth, 7, 0, mask)
        sizes = [sum(OR.param_count(model, b) for b in [-1] + s + [nblk]) for s in subs]
        assert len(set(sizes)) == 1
        assert abs(2 * M * 4 * sizes[0] / 1e9 - float(resist_gb)) < 1e-3


@pytest.mark.parametrize("blocks,S,min_depth", [([3, 4, 23, 3], 4, 0), ([3, 4, 6, 3], 2, 0),
                                                 ([3, 4, 23, 3], 8, 5), ([2], 1, 0), ([1, 1], 3, 2),
                                                 ([3, 4, 23, 3], 40, 5)])
def test_invariants(blocks, S, min_depth):
    first, B = OP.stage_first_blocks(blocks)
    P = B - len(first)
    for seed in range(5):
        for rnd in range(3):
            subs, owner = OP.partition(blocks, S, min_depth, seed, rnd)
            assert len(subs) == S and len(owner) == B
            sizes = {len(s) for s in subs}
            assert len(sizes) == 1                               # equal number of blocks
            D = max(-(-P // S), min(min_depth, P)) if P else 0
            assert sizes == {len(first) + D}
            for s in subs:
                assert s == sorted(set(s)) and set(first) <= set(s)
            assert all(o >= 1 for o in owner)                    # no block left out of a round
            assert owner == [sum(b in s for s in subs) for b in range(B)]
            assert all(owner[b] == S for b in first)
            if P:
                assert sorted(OP.permutation(P, seed, rnd)) == list(range(P))


def test_rounds_differ_and_seed_reproducible():
    a = OP.partition([3, 4, 23, 3], 4, 0, 1, 0)
    assert a == OP.partition([3, 4, 23, 3], 4, 0, 1, 0)
    assert a != OP.partition([3, 4, 23, 3], 4, 0, 1, 1)
    assert a != OP.partition([3, 4, 23, 3], 4, 0, 2, 0)


def test_written_rule_examples():
    """Worked values of the written rule (permute, deal s, s+S, ... mod P, skip held blocks)."""
    subs, owner = OP.partition([3, 4, 23, 3], 4, 0, 1, 0)
    assert OP.permutation(29, 1, 0) == [28, 13, 23, 6, 21, 9, 27, 17, 14, 26, 18, 5, 2, 24, 1, 19,
                                        22, 16, 20, 10, 15, 25, 4, 8, 11, 3, 12, 7, 0]
    assert subs[0] == [0, 1, 3, 4, 7, 14, 17, 18, 24, 25, 30, 32]
    assert subs[1] == [0, 3, 5, 7, 12, 16, 19, 27, 28, 29, 30, 32]
    assert subs[2] == [0, 2, 3, 6, 7, 15, 16, 21, 23, 26, 30, 31]
    assert subs[3] == [0, 3, 7, 8, 9, 10, 11, 13, 20, 22, 26, 30]
    assert sorted(b for b in range(33) if owner[b] == 2) == [16, 26, 32]
    subs, _ = OP.partition([3, 4, 6, 3], 2, 0, 2, 0)
    assert subs[0] == [0, 1, 3, 4, 5, 6, 7, 8, 13, 15]
    assert subs[1] == [0, 2, 3, 7, 9, 10, 11, 12, 13, 14]
