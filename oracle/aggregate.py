"""Oracle: reassembly of the global model from S sub-ResNets -- TEST INFRASTRUCTURE ONLY.

Sec. 2.3: every global parameter becomes its average over the sub-ResNets it was given to;
a parameter given to one sub-ResNet is copied.  Appendix B writes the same thing as
W^(h) = sum_v W_v^(h) M_v^(h) / sum_v M_v^(h), and a = sum_v a_v / S for the shared last layer.
A block nobody holds cannot occur in the method (Sec. 4); here it keeps its previous value.
The running BN statistics stored with a block are averaged like its parameters.
Pins: tests/test_oracle_aggregate.py (closed form on hand-made values, identity on identical
copies, single-owner bitwise copy, linearity).
"""
import numpy as np


def aggregate(global_params, sub_blocks, sub_params):
    """global_params: dict key -> {name: array}; sub_blocks[s]: block list of sub s;
    sub_params[s]: dict for keys -1, blocks of s, B.  Returns the new global dict (float64,
    except single-owner tensors which are returned bit-for-bit as stored)."""
    B = max(global_params.keys())
    out = {}
    for key, tensors in global_params.items():
        holders = [s for s in range(len(sub_blocks))
                   if key in (-1, B) or key in sub_blocks[s]]
        out[key] = {}
        for name, old in tensors.items():
            if not holders:
                out[key][name] = old.copy()
            elif len(holders) == 1:
                out[key][name] = sub_params[holders[0]][key][name].copy()
            else:
                acc = np.zeros(old.shape, np.float64)
                for s in holders:                      # ascending s
                    acc = acc + np.asarray(sub_params[s][key][name], np.float64)
                out[key][name] = acc / float(len(holders))
    return out
