"""Device-side containers for a sub-ResNet and the global model (allocation + marshalling only).

PyTorch provides device memory and streams; all arithmetic happens inside libresist.so.
"""
import numpy as np
import torch

from . import binding as B


class DeviceModel:
    """Block buffers of a set of blocks on the GPU: [stem, blocks..., head] as float32 tensors."""

    def __init__(self, model, blocks, logical_params, device="cuda"):
        self.model = model
        self.blocks = list(blocks)
        self.nb = B.num_blocks(model)
        self.keys = [-1] + self.blocks + [self.nb]
        self.device = device
        self.params = [torch.from_numpy(B.pack_block(model, k, logical_params[k])).to(device)
                       for k in self.keys]

    @classmethod
    def from_device(cls, model, blocks, source, **kw):
        """The blocks `blocks` of another DeviceModel (device-to-device copies of its buffers)."""
        self = cls.__new__(cls)
        self._init_from_tensors(model, blocks, {k: p.clone() for k, p in zip(source.keys, source.params)}, **kw)
        return self

    def _init_from_tensors(self, model, blocks, by_key):
        self.model = model
        self.blocks = list(blocks)
        self.nb = B.num_blocks(model)
        self.keys = [-1] + self.blocks + [self.nb]
        self.params = [by_key[k] for k in self.keys]
        self.device = self.params[0].device

    def predict(self, x, branch_scale=None, labels=None, stream=None):
        """Test-time forward pass of these blocks (BN running statistics; the residual branch of block i
        times branch_scale[i]).  x: device float32 [N,C,H,W].  -> logits [N, classes] (and the loss)."""
        n = x.shape[0]
        ws = torch.empty(B.forward_workspace_bytes(self.model, self.blocks, n), dtype=torch.uint8, device=x.device)
        logits = torch.empty((n, self.model["num_classes"]), dtype=torch.float32, device=x.device)
        loss = torch.zeros(1, dtype=torch.float32, device=x.device) if labels is not None else None
        B.forward(self.model, self.blocks, self.params, x, logits, ws, branch_scale, labels, loss, stream)
        return (logits, loss) if labels is not None else logits

    def compress(self, bits, stream=None):
        """b-bit compressed copies of all block buffers -> (codes, ranges): per buffer a uint8 tensor of
        codes and an int32 tensor [n_tensors, 4] holding the header records (lo and delta are the float32
        bit patterns of columns 0 and 1)."""
        sizes = [B.compressed_block_size(self.model, k, bits) for k in self.keys]
        codes = [torch.empty(nb, dtype=torch.uint8, device=self.device) for nb, _ in sizes]
        ranges = [torch.empty((nt, 4), dtype=torch.int32, device=self.device) for _, nt in sizes]
        B.compress_blocks(self.model, self.keys, bits, self.params, codes, ranges, stream)
        return codes, ranges

    def download(self):
        """-> {key: {name: logical array}} of the current parameter buffers."""
        return {k: B.unpack_block(self.model, k, p.cpu().numpy()) for k, p in zip(self.keys, self.params)}


class SubResNet(DeviceModel):
    """One worker's sub-ResNet: parameters, momentum, gradient buffers and workspace."""

    def __init__(self, model, blocks, logical_params, batch, device="cuda", keep_grads=True):
        super().__init__(model, blocks, logical_params, device)
        self._alloc(batch, keep_grads)

    def _init_from_tensors(self, model, blocks, by_key, batch=None, keep_grads=False):
        super()._init_from_tensors(model, blocks, by_key)
        self._alloc(batch, keep_grads)

    def _alloc(self, batch, keep_grads):
        model, device = self.model, self.device
        self.batch = batch
        sizes = [B.block_param_count(model, k)[1] for k in self.keys]
        self.momentum = [torch.zeros(n, dtype=torch.float32, device=device) for n in sizes]
        self.grads = ([torch.zeros(n, dtype=torch.float32, device=device) for n in sizes]
                      if keep_grads else None)
        self.workspace = torch.empty(B.workspace_bytes(model, self.blocks, batch), dtype=torch.uint8,
                                     device=device)
        self.loss = torch.zeros(1, dtype=torch.float32, device=device)

    def step(self, x, labels, lr, mu, wd, stream=None):
        """x: device float32 [N,C,H,W]; labels: device int32 [N].  Asynchronous."""
        assert x.shape[0] == self.batch and x.dtype == torch.float32 and labels.dtype == torch.int32
        B.local_step(self.model, self.blocks, self.params, self.momentum, self.grads, x, labels,
                     lr, mu, wd, self.workspace, self.loss, stream)

    def download_grads(self):
        return {k: B.unpack_block(self.model, k, g.cpu().numpy()) for k, g in zip(self.keys, self.grads)}

    def download_momentum(self):
        return {k: B.unpack_block(self.model, k, v.cpu().numpy()) for k, v in zip(self.keys, self.momentum)}

    def reset_momentum(self):
        for v in self.momentum:
            v.zero_()


def to_device_batch(x, labels, device="cuda"):
    return (torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(device),
            torch.from_numpy(np.ascontiguousarray(labels, np.int32)).to(device))


def run_round(model, glob, S, min_depth, seed, rnd, local_iters, batch_fn, batch, lr, mu, wd,
              partitionable=None, stream=None, compress_bits=0, compress_down=False):
    """One synchronisation round of Algorithm 1 on one GPU: split the global model (a DeviceModel
    holding every block) into S sub-ResNets for round `rnd`, run `local_iters` local steps of each, one
    sub-ResNet after the other, from the current global parameters and with fresh (zero) momentum,
    then reassemble the global model in place.  batch_fn(rnd, s, it) -> device (x, labels).
    With compress_bits = b in 2..8 every worker sends its blocks back compressed to b bits and the
    global model is reassembled from the compressed copies; with compress_down as well, the workers
    also receive their blocks as b-bit codes of the global model and start from the decoded values.
    Returns the partition and the workers (their loss buffers hold the last local loss)."""
    subs, owner = B.partition(model, S, min_depth, seed, rnd, partitionable)
    workers = []
    down = glob.compress(compress_bits, stream) if (compress_bits and compress_down) else None
    for s in range(S):
        w = SubResNet.from_device(model, subs[s], _Select(glob, subs[s]), batch=batch, keep_grads=False)
        if down is not None:
            idx = {k: i for i, k in enumerate(glob.keys)}
            B.decompress_blocks(model, w.keys, compress_bits, [down[0][idx[k]] for k in w.keys],
                                [down[1][idx[k]] for k in w.keys], w.params, stream)
        for it in range(local_iters):
            x, y = batch_fn(rnd, s, it)
            w.step(x, y, lr, mu, wd, stream)
        workers.append(w)
    if compress_bits:
        comp = [w.compress(compress_bits, stream) for w in workers]
        B.aggregate_compressed(model, subs, compress_bits, [c for c, _ in comp], [r for _, r in comp], glob.params, stream)
    else:
        B.aggregate(model, subs, [w.params for w in workers], glob.params, stream)
    return subs, owner, workers


class _Select:
    """View of a DeviceModel restricted to stem, the given blocks and head."""

    def __init__(self, glob, blocks):
        idx = {k: i for i, k in enumerate(glob.keys)}
        self.keys = [-1] + list(blocks) + [glob.nb]
        self.params = [glob.params[idx[k]] for k in self.keys]
