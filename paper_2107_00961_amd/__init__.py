"""MI355X (gfx950) library for the data-parallel hot path of ResIST: thin Python binding.

Every step of the path runs in the HIP kernels behind the C ABI declared in include/resist.h;
this package only marshals arguments (ctypes) and packs logical tensors into the library's
buffer layout.  There is no CPU fallback: importing works without a GPU (host-only calls such
as `partition` run anywhere), device calls need the built library and a gfx950 device.
"""
from . import binding
from .binding import (ResistError, aggregate, aggregate_compressed, block_layout, block_param_count, compress_blocks,
                      compressed_block_size, decompress_blocks, conv2d_dgrad, conv2d_forward, conv2d_wgrad, conv2d_wgrad_static, conv2d_wgrad_static_limit, forward, forward_workspace_bytes, lib, local_step, model_desc, num_blocks,
                      pack_block, partition, profile_enable, profile_read, set_bn_fusion, set_overlap, stem_conv2d_forward, stem_conv2d_wgrad,
                      unpack_block, workspace_bytes)

__all__ = ["ResistError", "aggregate", "aggregate_compressed", "block_layout", "block_param_count",
           "compress_blocks", "compressed_block_size", "conv2d_dgrad", "decompress_blocks",
           "conv2d_forward", "conv2d_wgrad", "conv2d_wgrad_static", "conv2d_wgrad_static_limit", "forward", "forward_workspace_bytes", "lib", "local_step", "model_desc", "num_blocks",
           "pack_block", "partition", "profile_enable", "profile_read", "set_bn_fusion", "set_overlap", "stem_conv2d_forward",
           "stem_conv2d_wgrad", "unpack_block", "workspace_bytes"]
