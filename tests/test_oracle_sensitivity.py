"""How well-conditioned is the quantity the full-size GPU check compares?

The float64 oracle's own weight gradients move when the input images are perturbed by half an
fp32 unit in the last place: ReLU decisions of pre-activations that sit within rounding distance
of zero flip, and the gradient of a deep BN-ReLU network responds far above the perturbation.
This measurement is what the full-size GPU parity check's relative-L2 bound (2e-2) is derived
from: no fp32 implementation can be element-wise closer to the oracle than the oracle is to itself
under such a perturbation."""
import numpy as np

from oracle import partition as OP
from oracle import resnet as OR
from resist_inputs import get_config, make_batch, make_params


def test_gradient_response_to_half_ulp_input_perturbation():
    cfg = get_config("cfg2")
    model = cfg["model"]
    subs, _ = OP.partition(model["blocks"], cfg["S"], 0, cfg["part_seed"], 0)
    params = make_params(model, 0)
    x, y = make_batch(model, 24, 0)
    l0, g0, _, _ = OR.forward_backward(model, subs[0], params, x, y)
    rng = np.random.default_rng(5)
    x2 = x.astype(np.float64) * (1 + 6e-8 * rng.standard_normal(x.shape))
    l1, g1, _, _ = OR.forward_backward(model, subs[0], params, x2, y)
    assert abs(l0 - l1) <= 1e-6 * abs(l0)                    # the loss itself is well conditioned
    worst = 0.0
    for b in g0:
        for k in g0[b]:
            rel = np.linalg.norm(g0[b][k] - g1[b][k]) / np.linalg.norm(g0[b][k])
            worst = max(worst, rel)
    # response is orders of magnitude above the 6e-8 perturbation and above the 1e-4 element bound,
    # yet well inside the 2e-2 bound of the full-size check
    assert 1e-4 < worst < 1e-2, worst
