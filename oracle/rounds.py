"""Oracle: the outer loop of the method -- TEST INFRASTRUCTURE ONLY.

Algorithm 1: for every synchronisation round t, the global ResNet is split into S sub-ResNets
(a fresh random partition per round), each sub-ResNet runs its local SGD iterations from the
current global parameters, and the global model is reassembled by averaging what was shared
(Sec. 2.3).  Momentum restarts at every synchronisation (the paper's experimental set-up), so the
momentum buffers start at zero in every round.  Sub-ResNets are independent within a round.
Pins: this module only composes oracle/partition.py, oracle/resnet.py and oracle/aggregate.py,
each pinned on its own; tests/test_oracle_rounds.py pins the composition (S=1 equals plain SGD
over the same batches; blocks nobody trained in a round keep their values; a fresh partition
per round; with compression on the way down the local steps start from the decoded weights).
"""
import numpy as np

from . import aggregate as OA
from . import compress as OC
from . import partition as OP
from . import resnet as OR


def run_rounds(model, global_params, S, min_depth, seed, rounds, local_iters, batch_fn, lr, mu, wd,
               partitionable=None, first_round=0, compress_bits=0, compress_down=False):
    """batch_fn(round, s, it) -> (x, labels).  Returns (new global params, log) where log[t] holds
    the partition of round t and the losses of every local step."""
    g = {k: {n: np.asarray(v) for n, v in p.items()} for k, p in global_params.items()}
    B = max(g.keys())
    log = []
    for t in range(first_round, first_round + rounds):
        subs, owner = OP.partition(model["blocks"], S, min_depth, seed, t, partitionable)
        sub_params, losses = [], []
        for s in range(S):
            keys = [-1] + subs[s] + [B]
            p = {k: g[k] for k in keys}
            if compress_bits and compress_down:
                # the worker receives b-bit codes of the global model and starts from the decoded fp32 values
                p = {k: {n: OC.dequantize_tensor(*OC.quantize_tensor(np.asarray(a, np.float32), compress_bits)).astype(np.float32)
                         for n, a in t.items()} for k, t in p.items()}
            v = {k: {n: np.zeros_like(a, dtype=np.float64) for n, a in g[k].items()} for k in keys}   # momentum restart
            ls = []
            for it in range(local_iters):
                x, y = batch_fn(t, s, it)
                loss, _, p, v = OR.local_step(model, subs[s], p, v, x, y, lr, mu, wd)
                ls.append(loss)
            sub_params.append(p)
            losses.append(ls)
        if compress_bits:
            # appendix on quantised communication: the workers' parameters travel as b-bit codes
            sq = [{k: OC.quantize_block({n: np.asarray(a, np.float32) for n, a in t.items()}, compress_bits)
                   for k, t in p.items()} for p in sub_params]
            g = OC.aggregate_quantized(g, subs, sq)
        else:
            g = OA.aggregate(g, subs, sub_params)
        log.append(dict(subs=subs, owner=owner, losses=losses))
    return g, log
