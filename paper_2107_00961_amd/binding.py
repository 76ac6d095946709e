"""ctypes binding of libresist.so -- argument marshalling only (same names as include/resist.h)."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libresist.so")
_lib = None


class ResistError(RuntimeError):
    pass


class _ModelDesc(C.Structure):
    _fields_ = [("block_kind", C.c_int32), ("stem_kind", C.c_int32), ("in_c", C.c_int32),
                ("in_h", C.c_int32), ("in_w", C.c_int32), ("num_stages", C.c_int32),
                ("width", C.c_int32 * 4), ("blocks", C.c_int32 * 4), ("num_classes", C.c_int32),
                ("compute_dtype", C.c_int32), ("bn_eps", C.c_float), ("bn_momentum", C.c_float)]


class _TensorInfo(C.Structure):
    _fields_ = [("kind", C.c_int32), ("layer", C.c_int32), ("offset", C.c_int64),
                ("count", C.c_int64), ("dims", C.c_int32 * 4)]


class _KernelStat(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("launches", C.c_int64), ("ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double)]


class _ConvShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "H", "W", "C", "K", "R", "S", "stride", "pad", "dtype")]


def lib():
    """The loaded library; raises loudly if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ResistError(f"{_LIB_PATH} is missing: run `python -m paper_2107_00961_amd.build` "
                              "(there is no CPU fallback)")
        # PyTorch-ROCm ships its own HIP runtime; loaded after this library it would be a second runtime in
        # the process (the first one then reports no device).  Import it first where it is installed.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(_LIB_PATH)
        L.resist_last_error.restype = C.c_char_p
        for name in ("resist_num_blocks", "resist_partition", "resist_block_param_count",
                     "resist_block_layout", "resist_workspace_bytes", "resist_local_step",
                     "resist_aggregate", "resist_forward", "resist_forward_workspace_bytes",
                     "resist_conv2d_workspace_bytes", "resist_conv2d_forward",
                     "resist_conv2d_dgrad", "resist_conv2d_wgrad", "resist_profile_enable",
                     "resist_profile_read", "resist_compressed_block_size",
                     "resist_compress_blocks", "resist_decompress_blocks", "resist_aggregate_compressed",
                     "resist_set_overlap", "resist_set_bn_fusion", "resist_conv2d_wgrad_static", "resist_conv2d_wgrad_static_limit",
                     "resist_stem_conv2d_workspace_bytes", "resist_stem_conv2d_forward", "resist_stem_conv2d_wgrad"):
            getattr(L, name).restype = C.c_int
        L.resist_local_step.argtypes = [
            C.POINTER(_ModelDesc), C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_void_p),
            C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p, C.c_int32,
            C.c_float, C.c_float, C.c_float, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        L.resist_aggregate.argtypes = [
            C.POINTER(_ModelDesc), C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
            C.POINTER(C.POINTER(C.c_void_p)), C.POINTER(C.c_void_p), C.c_void_p]
        L.resist_compressed_block_size.argtypes = [
            C.POINTER(_ModelDesc), C.c_int32, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        L.resist_compress_blocks.argtypes = [
            C.POINTER(_ModelDesc), C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_void_p),
            C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p]
        L.resist_decompress_blocks.argtypes = L.resist_compress_blocks.argtypes
        L.resist_aggregate_compressed.argtypes = [
            C.POINTER(_ModelDesc), C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32,
            C.POINTER(C.POINTER(C.c_void_p)), C.POINTER(C.POINTER(C.c_void_p)), C.POINTER(C.c_void_p),
            C.c_void_p]
        L.resist_forward.argtypes = [
            C.POINTER(_ModelDesc), C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_void_p),
            C.POINTER(C.c_float), C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
            C.c_void_p, C.c_void_p]
        L.resist_partition.argtypes = [
            C.POINTER(_ModelDesc), C.POINTER(C.c_uint8), C.c_int32, C.c_int32, C.c_uint64,
            C.c_uint64, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32)]
        for name in ("resist_conv2d_forward", "resist_conv2d_dgrad", "resist_conv2d_wgrad", "resist_stem_conv2d_forward",
                     "resist_stem_conv2d_wgrad"):
            getattr(L, name).argtypes = [C.POINTER(_ConvShape), C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_int64, C.c_void_p]
        L.resist_conv2d_wgrad_static.argtypes = [C.POINTER(_ConvShape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise ResistError(f"resist status {rc}: {lib().resist_last_error().decode()}")


def model_desc(model):
    """dict (see resist_inputs.configs) -> C struct."""
    d = _ModelDesc()
    d.block_kind, d.stem_kind = model["block_kind"], model["stem_kind"]
    d.in_c, d.in_h, d.in_w = model["in_c"], model["in_h"], model["in_w"]
    d.num_stages = len(model["widths"])
    for i, (w, b) in enumerate(zip(model["widths"], model["blocks"])):
        d.width[i], d.blocks[i] = w, b
    d.num_classes = model["num_classes"]
    d.compute_dtype = model.get("compute_dtype", 0)
    d.bn_eps, d.bn_momentum = model["bn_eps"], model["bn_momentum"]
    return d


def num_blocks(model):
    n = C.c_int32()
    _check(lib().resist_num_blocks(C.byref(model_desc(model)), C.byref(n)))
    return n.value


def partition(model, S, min_depth, seed, rnd, partitionable=None):
    """Returns (list of S block lists, owner_count list)."""
    d = model_desc(model)
    B = num_blocks(model)
    cap = S * B if S > 0 else 1
    offs = (C.c_int32 * (max(S, 0) + 1))()
    blocks = (C.c_int32 * max(cap, 1))()
    owner = (C.c_int32 * B)()
    mask = None
    if partitionable is not None:
        mask = (C.c_uint8 * B)(*[int(bool(v)) for v in partitionable])
    _check(lib().resist_partition(C.byref(d), mask, S, min_depth, C.c_uint64(seed), C.c_uint64(rnd),
                                  offs, blocks, cap, owner))
    subs = [list(blocks[offs[s]:offs[s + 1]]) for s in range(S)]
    return subs, list(owner)


def block_param_count(model, block):
    tot, tr = C.c_int64(), C.c_int64()
    _check(lib().resist_block_param_count(C.byref(model_desc(model)), block, C.byref(tot), C.byref(tr)))
    return tot.value, tr.value


def block_layout(model, block):
    n = C.c_int32()
    d = model_desc(model)
    _check(lib().resist_block_layout(C.byref(d), block, None, 0, C.byref(n)))
    arr = (_TensorInfo * n.value)()
    _check(lib().resist_block_layout(C.byref(d), block, arr, n.value, C.byref(n)))
    return [dict(kind=t.kind, layer=t.layer, offset=t.offset, count=t.count, dims=list(t.dims)) for t in arr]


# logical tensor names <-> (kind, layer) of the library's layout
_KIND_SUFFIX = {0: "_w", 1: "_g", 2: "_b", 3: "_rm", 4: "_rv"}


def _tensor_name(block, B, t):
    if t["kind"] == 5:
        return "fc_w"
    if t["kind"] == 6:
        return "fc_b"
    if block == -1 or block == B:
        return ("conv" if t["kind"] == 0 else "bn") + _KIND_SUFFIX[t["kind"]]
    conv = ["conv1", "conv2", "conv3", "ds"][t["layer"]]
    bn = ["bn1", "bn2", "bn3", "dsbn"][t["layer"]]
    return (conv if t["kind"] == 0 else bn) + _KIND_SUFFIX[t["kind"]]


def pack_block(model, block, tensors, trainable_only=False):
    """Logical tensors {name: array} -> flat float32 array in the library's buffer layout
    (conv weights [K,C,R,S] are permuted to [K,R,S,C]).  Missing tensors stay zero."""
    B = num_blocks(model)
    tot, tr = block_param_count(model, block)
    out = np.zeros(tr if trainable_only else tot, np.float32)
    for t in block_layout(model, block):
        if trainable_only and t["kind"] in (3, 4):
            continue
        name = _tensor_name(block, B, t)
        if name not in tensors:
            continue
        a = np.asarray(tensors[name], np.float32)
        if t["kind"] == 0:
            a = a.transpose(0, 2, 3, 1)
        out[t["offset"]:t["offset"] + t["count"]] = np.ascontiguousarray(a).reshape(-1)
    return out


def unpack_block(model, block, flat):
    """Inverse of pack_block: flat buffer -> {name: array in logical layout}."""
    B = num_blocks(model)
    flat = np.asarray(flat)
    out = {}
    for t in block_layout(model, block):
        if t["offset"] + t["count"] > flat.size:
            continue
        a = flat[t["offset"]:t["offset"] + t["count"]]
        if t["kind"] == 0:
            K, R, S, Cc = t["dims"]
            a = a.reshape(K, R, S, Cc).transpose(0, 3, 1, 2)
        elif t["kind"] == 5:
            a = a.reshape(t["dims"][0], t["dims"][1])
        out[_tensor_name(block, B, t)] = np.ascontiguousarray(a)
    return out


def workspace_bytes(model, blocks, batch):
    n = C.c_int64()
    arr = (C.c_int32 * len(blocks))(*blocks)
    _check(lib().resist_workspace_bytes(C.byref(model_desc(model)), arr, len(blocks), batch, C.byref(n)))
    return n.value


def _ptr_array(tensors):
    return (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def local_step(model, blocks, params, momentum, grads, x, labels, lr, mu, wd, workspace, loss_out,
               stream=None):
    """params/momentum/grads: lists of device float32 tensors [stem, blocks..., head]
    (grads may be None); x [N,C,H,W] float32, labels int32, workspace uint8, loss_out 1 float."""
    arr = (C.c_int32 * len(blocks))(*blocks)
    _check(lib().resist_local_step(
        C.byref(model_desc(model)), arr, len(blocks), _ptr_array(params), _ptr_array(momentum),
        _ptr_array(grads) if grads is not None else None, x.data_ptr(), labels.data_ptr(),
        x.shape[0], lr, mu, wd, workspace.data_ptr(), workspace.numel() * workspace.element_size(),
        loss_out.data_ptr(), _stream_ptr(stream)))


def forward_workspace_bytes(model, blocks, batch):
    n = C.c_int64()
    arr = (C.c_int32 * len(blocks))(*blocks)
    _check(lib().resist_forward_workspace_bytes(C.byref(model_desc(model)), arr, len(blocks), batch, C.byref(n)))
    return n.value


def forward(model, blocks, params, x, logits_out, workspace, branch_scale=None, labels=None, loss_out=None,
            stream=None):
    """Test-time forward pass: params = device float32 tensors [stem, blocks..., head]; x [N,C,H,W]
    float32; logits_out [N, classes] float32 (written); branch_scale: one float per block or None."""
    arr = (C.c_int32 * len(blocks))(*blocks)
    sc = (C.c_float * len(blocks))(*branch_scale) if branch_scale is not None else None
    _check(lib().resist_forward(
        C.byref(model_desc(model)), arr, len(blocks), _ptr_array(params), sc, x.data_ptr(), x.shape[0],
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), logits_out.data_ptr(),
        labels.data_ptr() if labels is not None else None,
        loss_out.data_ptr() if loss_out is not None else None, _stream_ptr(stream)))


def aggregate(model, subs, sub_params, global_params, stream=None):
    """subs: list of S block lists; sub_params[s]: device tensors [stem, blocks of s..., head];
    global_params: device tensors [stem, blocks 0..B-1, head] (written)."""
    S = len(subs)
    offs = [0]
    flat = []
    for s in subs:
        flat += list(s)
        offs.append(len(flat))
    offs_a = (C.c_int32 * (S + 1))(*offs)
    flat_a = (C.c_int32 * max(len(flat), 1))(*flat)
    keep = [_ptr_array(p) for p in sub_params]
    outer = (C.POINTER(C.c_void_p) * S)(*[C.cast(k, C.POINTER(C.c_void_p)) for k in keep])
    _check(lib().resist_aggregate(C.byref(model_desc(model)), S, offs_a, flat_a, outer,
                                  _ptr_array(global_params), _stream_ptr(stream)))


def compressed_block_size(model, block, bits):
    """-> (bytes of the code array, number of header records) of `block` (-1 stem, 0..B-1, B head)."""
    nb, nt = C.c_int64(), C.c_int32()
    _check(lib().resist_compressed_block_size(C.byref(model_desc(model)), block, bits, C.byref(nb), C.byref(nt)))
    return nb.value, nt.value


def compress_blocks(model, keys, bits, params, codes, ranges, stream=None):
    """keys: block keys; params: device fp32 block buffers; codes: device uint8 tensors of
    compressed_block_size()[0] bytes; ranges: device tensors of 16 bytes per header record."""
    n = len(keys)
    keys_a = (C.c_int32 * max(n, 1))(*keys)
    _check(lib().resist_compress_blocks(C.byref(model_desc(model)), n, keys_a, bits, _ptr_array(params),
                                        _ptr_array(codes), _ptr_array(ranges), _stream_ptr(stream)))


def decompress_blocks(model, keys, bits, codes, ranges, params, stream=None):
    """The inverse direction: decodes compressed blocks (as written by compress_blocks) into the device
    fp32 block buffers `params`."""
    n = len(keys)
    keys_a = (C.c_int32 * max(n, 1))(*keys)
    _check(lib().resist_decompress_blocks(C.byref(model_desc(model)), n, keys_a, bits, _ptr_array(codes),
                                          _ptr_array(ranges), _ptr_array(params), _stream_ptr(stream)))


def aggregate_compressed(model, subs, bits, sub_codes, sub_ranges, global_params, stream=None):
    """aggregate() with every source a compressed block: sub_codes[s] / sub_ranges[s] are device
    tensors [stem, blocks of s..., head] as written by compress_blocks."""
    S = len(subs)
    offs = [0]
    flat = []
    for s in subs:
        flat += list(s)
        offs.append(len(flat))
    offs_a = (C.c_int32 * (S + 1))(*offs)
    flat_a = (C.c_int32 * max(len(flat), 1))(*flat)
    keep_c = [_ptr_array(p) for p in sub_codes]
    keep_r = [_ptr_array(p) for p in sub_ranges]
    outer_c = (C.POINTER(C.c_void_p) * S)(*[C.cast(k, C.POINTER(C.c_void_p)) for k in keep_c])
    outer_r = (C.POINTER(C.c_void_p) * S)(*[C.cast(k, C.POINTER(C.c_void_p)) for k in keep_r])
    _check(lib().resist_aggregate_compressed(C.byref(model_desc(model)), S, offs_a, flat_a, bits, outer_c,
                                             outer_r, _ptr_array(global_params), _stream_ptr(stream)))


def set_overlap(mode):
    """Second stream for the weight gradients of local_step: 0/False never, 1/True for steps with
    enough work (default), 2 always."""
    _check(lib().resist_set_overlap(int(mode)))


def set_bn_fusion(mode):
    """First pass of a BN backward from the epilogue of the data gradient above it: 0 never, 1 in bf16
    steps (default), 2 always."""
    _check(lib().resist_set_bn_fusion(int(mode)))


def profile_enable(on):
    """Switch per-kernel event timing on/off (clears the statistics)."""
    _check(lib().resist_profile_enable(1 if on else 0))


def profile_read():
    """-> list of dicts(name, launches, ms, flops, bytes), one per kernel launched since enable."""
    n = C.c_int32()
    _check(lib().resist_profile_read(None, 0, C.byref(n)))
    arr = (_KernelStat * max(n.value, 1))()
    _check(lib().resist_profile_read(arr, n.value, C.byref(n)))
    return [dict(name=a.name.decode(), launches=a.launches, ms=a.ms, flops=a.flops, bytes=a.bytes)
            for a in arr[:n.value]]


def _conv_shape(N, H, W, Cc, K, R, stride, pad, dtype=0):
    return _ConvShape(N, H, W, Cc, K, R, R, stride, pad, dtype)


def _dtype_code(t):
    """torch dtype of an activation tensor -> the library's dtype code (0 fp32, 1 bf16)."""
    import torch
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.bfloat16:
        return 1
    raise ResistError(f"unsupported tensor dtype {t.dtype}")


def _conv_ws(shape):
    import torch
    n = C.c_int64()
    _check(lib().resist_conv2d_workspace_bytes(C.byref(shape), C.byref(n)))
    return torch.empty(n.value, dtype=torch.uint8, device="cuda")


def conv2d_forward(x, w, stride, pad, stream=None):
    """x [N,H,W,C], w [K,R,S,C] device tensors (both float32 or both bfloat16) -> y [N,P,Q,K]."""
    import torch
    N, H, W, Cc = x.shape
    K, R = w.shape[0], w.shape[1]
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    y = torch.empty((N, P, Q, K), dtype=x.dtype, device=x.device)
    sh = _conv_shape(N, H, W, Cc, K, R, stride, pad, _dtype_code(x))
    ws = _conv_ws(sh)
    _check(lib().resist_conv2d_forward(C.byref(sh), x.data_ptr(), w.data_ptr(), y.data_ptr(),
                                       ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return y


def conv2d_dgrad(dy, w, x_shape, stride, pad, stream=None):
    import torch
    N, H, W, Cc = x_shape
    K, R = w.shape[0], w.shape[1]
    dx = torch.empty((N, H, W, Cc), dtype=dy.dtype, device=dy.device)
    sh = _conv_shape(N, H, W, Cc, K, R, stride, pad, _dtype_code(dy))
    ws = _conv_ws(sh)
    _check(lib().resist_conv2d_dgrad(C.byref(sh), dy.data_ptr(), w.data_ptr(), dx.data_ptr(),
                                     ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return dx


def conv2d_wgrad(dy, x, w_shape, stride, pad, stream=None):
    import torch
    N, H, W, Cc = x.shape
    K, R = w_shape[0], w_shape[1]
    dw = torch.empty((K, R, R, Cc), dtype=torch.float32, device=x.device)
    sh = _conv_shape(N, H, W, Cc, K, R, stride, pad, _dtype_code(x))
    ws = _conv_ws(sh)
    _check(lib().resist_conv2d_wgrad(C.byref(sh), dy.data_ptr(), x.data_ptr(), dw.data_ptr(),
                                     ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return dw


def conv2d_wgrad_static_limit():
    """Bytes of the library's static scratch that conv2d_wgrad_static keeps its split partial sums in."""
    n = C.c_int64()
    _check(lib().resist_conv2d_wgrad_static_limit(C.byref(n)))
    return n.value


def conv2d_wgrad_static(dy, x, dw, stride, pad, stream=None):
    """resist_conv2d_wgrad_static: like conv2d_wgrad but no workspace and no allocation anywhere; the
    caller passes the output dw [K,R,S,C] float32."""
    N, H, W, Cc = x.shape
    K, R = dw.shape[0], dw.shape[1]
    sh = _conv_shape(N, H, W, Cc, K, R, stride, pad, _dtype_code(x))
    _check(lib().resist_conv2d_wgrad_static(C.byref(sh), dy.data_ptr(), x.data_ptr(), dw.data_ptr(),
                                            _stream_ptr(stream)))


def _stem_ws(shape):
    import torch
    n = C.c_int64()
    _check(lib().resist_stem_conv2d_workspace_bytes(C.byref(shape), C.byref(n)))
    return torch.empty(n.value, dtype=torch.uint8, device="cuda")


def stem_conv2d_forward(x, w, stride, pad, bf16=False, stream=None):
    """The stem convolution on its own: x [N,C,H,W] float32 (as passed to local_step), w [K,R,S,C]
    float32 -> y [N,P,Q,K] float32 or bfloat16."""
    import torch
    N, Cc, H, W = x.shape
    K, R = w.shape[0], w.shape[1]
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    y = torch.empty((N, P, Q, K), dtype=torch.bfloat16 if bf16 else torch.float32, device=x.device)
    sh = _conv_shape(N, H, W, Cc, K, R, stride, pad, 1 if bf16 else 0)
    ws = _stem_ws(sh)
    _check(lib().resist_stem_conv2d_forward(C.byref(sh), x.data_ptr(), w.data_ptr(), y.data_ptr(), ws.data_ptr(), ws.numel(),
                                            _stream_ptr(stream)))
    return y


def stem_conv2d_wgrad(dy, x, w_shape, stride, pad, stream=None):
    """dy [N,P,Q,K] float32 or bfloat16, x [N,C,H,W] float32 -> dw [K,R,S,C] float32."""
    import torch
    N, Cc, H, W = x.shape
    K, R = w_shape[0], w_shape[1]
    dw = torch.empty((K, R, R, Cc), dtype=torch.float32, device=x.device)
    sh = _conv_shape(N, H, W, Cc, K, R, stride, pad, _dtype_code(dy))
    ws = _stem_ws(sh)
    _check(lib().resist_stem_conv2d_wgrad(C.byref(sh), dy.data_ptr(), x.data_ptr(), dw.data_ptr(), ws.data_ptr(), ws.numel(),
                                          _stream_ptr(stream)))
    return dw
