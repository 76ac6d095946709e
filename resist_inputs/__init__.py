"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module holds NO arithmetic of the method: it only describes the five
benchmark workloads as plain data (model descriptions, hyper-parameters) and
draws seeded random tensors (images, labels, initial weights) in the *logical*
layout of the paper's networks: images [N,C,H,W], conv weights [K,C,R,S],
FC weights [classes,C].  Both sides receive these tensors as data.

The paper trains on CIFAR10/100 and ImageNet (Sec. 5, "Small-Scale Image
Classification" / "ImageNet Classification"); those datasets are not available
here, so N(0,1) images and uniform labels of the same shapes stand in for them.
"""
from .configs import CONFIGS, get_config, model_blocks
from .gen import make_batch, make_params, zeros_like_params

__all__ = ["CONFIGS", "get_config", "model_blocks", "make_batch", "make_params",
           "zeros_like_params"]
