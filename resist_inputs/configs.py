"""The benchmark workloads as plain data (no arithmetic of the method).

A model description is a dict with the keys
  block_kind   0 = basic block (3x3, 3x3), 1 = bottleneck (1x1, 3x3, 1x1, expansion 4);
               2, 3 = the same two in pre-activation form (BN-ReLU before every convolution)
  stem_kind    0 = conv3x3 stride 1 pad 1;  1 = conv7x7 stride 2 pad 3 + maxpool 3x3 stride 2 pad 1
  in_c,in_h,in_w, widths (per stage), blocks (per stage), num_classes,
  compute_dtype 0 = fp32, 1 = bf16 operands with fp32 accumulation
  bn_eps, bn_momentum
The global network follows Sec. 2.1 ("four sections of blocks of equal channel
dimension"); sizes are those of the benchmark configurations.
"""

def _model(block_kind, stem_kind, in_hw, widths, blocks, num_classes, compute_dtype=0):
    return dict(block_kind=block_kind, stem_kind=stem_kind, in_c=3, in_h=in_hw, in_w=in_hw,
                widths=list(widths), blocks=list(blocks), num_classes=num_classes,
                compute_dtype=compute_dtype, bn_eps=1e-5, bn_momentum=0.1)


CONFIGS = {
    # tiny: two basic blocks at 16 channels, S = 1
    "cfg1": dict(model=_model(0, 0, 16, [16], [2], 10), batch=4, S=1, part_seed=0, data_seed=0,
                 lr=0.1, momentum=0.9, weight_decay=0.0, min_depth=0),
    # CIFAR-shaped sub-ResNet (the configuration the metric is quoted on)
    "cfg2": dict(model=_model(0, 0, 32, [64, 128, 256, 512], [3, 4, 23, 3], 10), batch=128, S=4,
                 part_seed=1, data_seed=0, lr=0.1, momentum=0.9, weight_decay=5e-4, min_depth=0),
    # the same sub-ResNet with pre-activation blocks (the architecture the paper prefers)
    "cfg2_preact": dict(model=_model(2, 0, 32, [64, 128, 256, 512], [3, 4, 23, 3], 10), batch=128, S=4,
                        part_seed=1, data_seed=0, lr=0.1, momentum=0.9, weight_decay=5e-4, min_depth=0),
    # CIFAR-shaped full round: S=4 x 50 local iterations, 100 classes, then aggregation
    "cfg3": dict(model=_model(0, 0, 32, [64, 128, 256, 512], [3, 4, 23, 3], 100), batch=128, S=4,
                 part_seed=1, data_seed=0, lr=0.1, momentum=0.9, weight_decay=5e-4, min_depth=0,
                 local_iters=50),
    # ImageNet-shaped bottleneck sub-ResNet, bf16 operands
    "cfg4": dict(model=_model(1, 1, 224, [64, 128, 256, 512], [3, 4, 6, 3], 1000, compute_dtype=1),
                 batch=64, S=2, part_seed=2, data_seed=0, lr=0.1, momentum=0.9, weight_decay=0.0,
                 min_depth=0),
    # full model (S = 1) at CIFAR shape, fp32 and bf16
    "cfg5": dict(model=_model(0, 0, 32, [64, 128, 256, 512], [3, 4, 23, 3], 10), batch=128, S=1,
                 part_seed=1, data_seed=0, lr=0.1, momentum=0.9, weight_decay=5e-4, min_depth=0),
    "cfg5_bf16": dict(model=_model(0, 0, 32, [64, 128, 256, 512], [3, 4, 23, 3], 10, compute_dtype=1),
                      batch=128, S=1, part_seed=1, data_seed=0, lr=0.1, momentum=0.9,
                      weight_decay=5e-4, min_depth=0),
}


def get_config(name):
    import copy
    return copy.deepcopy(CONFIGS[name])


def model_blocks(model):
    """Static shape table of the global network: one dict per residual block, in network order.

    Pure bookkeeping (channel counts, strides), used only to size random tensors.
    """
    exp = 4 if model["block_kind"] in (1, 3) else 1
    out = []
    c_in = model["widths"][0]
    for si, (w, nb) in enumerate(zip(model["widths"], model["blocks"])):
        for bi in range(nb):
            stride = 2 if (bi == 0 and si > 0) else 1
            c_out = w * exp
            has_ds = bi == 0 and (stride != 1 or c_in != c_out)
            out.append(dict(stage=si, index=bi, c_in=c_in, width=w, c_out=c_out, stride=stride,
                            has_ds=has_ds, first=(bi == 0)))
            c_in = c_out
    return out
