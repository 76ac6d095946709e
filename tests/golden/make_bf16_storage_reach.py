#!/usr/bin/env python3
"""Writes tests/golden/bf16_storage_reach.json: for every bf16 step-parity case, the weight tensors
that bf16 storage by itself moves by more than 1e-2 (relative L2 norm) in one SGD step.

For each case (tests/bf16_cases.py) the float64 oracle takes the step twice, once unrounded and once
rounding at the bf16 storage points (the ImageNet-shaped configuration: "bf16 activations/weights
with fp32 accumulation and fp32 master weights"), and the relative L2 distance between the two updated
tensors is recorded when it exceeds 1e-2.  For those tensors the stated bar for bf16 variants -- updated
weights within relative 2e-2 of the unrounded result -- cannot be asked of any bf16 implementation; the
GPU tests hold them to 1.5 x the recorded distance instead and every other tensor to the stated 2e-2.
Calls the oracle only (no GPU, no HIP library).  Usage: python tests/golden/make_bf16_storage_reach.py [case ...]
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import resnet as OR                                          # noqa: E402
from resist_inputs import make_batch, make_params, zeros_like_params     # noqa: E402
from tests.bf16_cases import bf16_cases                                  # noqa: E402

OUT = os.path.join(ROOT, "tests", "golden", "bf16_storage_reach.json")
THRESHOLD = 1e-2


def reach(case):
    model = dict(case["model"], compute_dtype=1)
    params = make_params(model, case["seed"], perturb_bn=case["perturb_bn"])
    x, y = make_batch(model, case["batch"], case["data_seed"])
    zero = zeros_like_params(params)
    args = (model, case["blocks"], params, zero, x, y, case["lr"], case["mu"], case["wd"])
    _, _, p_e, _ = OR.local_step(*args, emulate_bf16=True)
    _, _, p_f, _ = OR.local_step(*args)
    out = {}
    for k in p_f:
        for name, w in p_f[k].items():
            if name.endswith(("_rm", "_rv")) or np.linalg.norm(params[k][name]) == 0:
                continue
            r = float(np.linalg.norm(p_e[k][name] - w) / np.linalg.norm(w))
            if r > THRESHOLD:
                out[f"{k}/{name}"] = float(f"{r:.4e}")
    return out


def main():
    cases = bf16_cases()
    table = {}
    if os.path.exists(OUT):
        with open(OUT) as f:
            table = json.load(f)
    for name in (sys.argv[1:] or cases):
        print(name, flush=True)
        table[name] = reach(cases[name])
        with open(OUT, "w") as f:
            json.dump({k: table[k] for k in cases if k in table}, f, indent=1)
            f.write("\n")


if __name__ == "__main__":
    main()
