"""Thin ctypes binding of the C ABI in include/conv2d.h (same names).

Argument marshalling only: every step of the convolution runs in the HIP
library.  torch is used for device memory and streams.  There is no CPU
fallback: if the shared library is missing, loading raises.
"""
import ctypes
import os

PAD_VALID = 0
PAD_SAME = 1
F32 = 0
BF16 = 1

STATUS_OK = 0
STATUS_INVALID_ARGUMENT = -1
STATUS_UNSUPPORTED = -2
STATUS_WORKSPACE_TOO_SMALL = -3
STATUS_LAUNCH_FAILED = -4
STATUS_TOO_LARGE = -5

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libconv2d_mi355x.so")

EXPORTS = (
    "conv2d_get_geometry", "conv2d_workspace_size", "conv2d_workspace_size_variant",
    "conv2d_forward", "conv2d_forward_static_scratch", "conv2d_forward_variant",
    "conv2d_forward_bias_act",
    "conv2d_forward_bias_act_pool", "conv2d_pool_workspace_size",
    "conv2d_pool_workspace_size_variant", "conv2d_packed_filter_size", "conv2d_pack_filter",
    "conv2d_forward_packed", "conv2d_last_launch_error", "conv2d_debug_force_variant",
    "conv2d_debug_split_reduce_separate",
    "conv2d_num_variants",
    "conv2d_variant_name",
    "conv2d_variant_supports", "conv2d_selected_variant", "conv2d_select_variant",
    "conv2d_status_string", "conv2d_version",
)


class Params(ctypes.Structure):
    """conv2d_params: the parameter tuple of the paper's Figure 1 caption plus
    batch, padding mode and element types."""
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "in_rows", "in_cols", "channels", "features", "window_rows", "window_cols",
        "stride_rows", "stride_cols", "padding", "in_dtype", "out_dtype")]


class Geometry(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "out_rows", "out_cols", "pad_top", "pad_bottom", "pad_left", "pad_right")]


class Conv2dError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        detail = ""
        if status == STATUS_LAUNCH_FAILED:
            detail = ": " + lib().conv2d_last_launch_error().decode()
        super().__init__("%s: %s%s (status %d)" % (where, status_string(status), detail, status))


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_1904_04174_amd.build` "
                "(there is no CPU fallback)" % LIB_PATH)
        # torch ships a HIP runtime of its own and loads it by path.  Loaded after this
        # library (which would then have pulled in the system's runtime), it is a second
        # runtime in the process, and this library's launches fail on device pointers of the
        # other one ("no ROCm-capable device is detected").  Loaded first, it is the one this
        # library binds to (same soname).
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        l = ctypes.CDLL(LIB_PATH)
        pp, gp = ctypes.POINTER(Params), ctypes.POINTER(Geometry)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        l.conv2d_get_geometry.argtypes = [pp, gp]
        l.conv2d_workspace_size.argtypes = [pp, ctypes.POINTER(sz)]
        l.conv2d_workspace_size_variant.argtypes = [pp, ctypes.c_int, ctypes.POINTER(sz)]
        l.conv2d_forward.argtypes = [pp, vp, vp, vp, vp, sz, vp]
        l.conv2d_forward_variant.argtypes = [pp, vp, vp, vp, vp, sz, vp, ctypes.c_int]
        l.conv2d_forward_static_scratch.argtypes = [pp, vp, vp, vp, vp]
        l.conv2d_debug_force_variant.argtypes = [ctypes.c_int]
        l.conv2d_debug_split_reduce_separate.argtypes = [ctypes.c_int]
        l.conv2d_num_variants.argtypes = []
        l.conv2d_variant_name.argtypes = [ctypes.c_int]
        l.conv2d_variant_name.restype = ctypes.c_char_p
        l.conv2d_variant_supports.argtypes = [pp, ctypes.c_int]
        l.conv2d_selected_variant.argtypes = [pp, ctypes.POINTER(ctypes.c_int)]
        l.conv2d_forward_bias_act.argtypes = [pp, vp, vp, vp, ctypes.c_int, vp, vp, ctypes.c_size_t,
                                              vp]
        l.conv2d_forward_bias_act_pool.argtypes = [pp, vp, vp, vp, ctypes.c_int, vp, vp,
                                                   ctypes.c_size_t, vp]
        l.conv2d_pool_workspace_size.argtypes = [pp, ctypes.POINTER(sz)]
        l.conv2d_pool_workspace_size_variant.argtypes = [pp, ctypes.c_int, ctypes.POINTER(sz)]
        l.conv2d_packed_filter_size.argtypes = [pp, ctypes.c_int, ctypes.POINTER(sz)]
        l.conv2d_pack_filter.argtypes = [pp, ctypes.c_int, vp, vp, sz, vp]
        l.conv2d_forward_packed.argtypes = [pp, ctypes.c_int, vp, vp, vp, ctypes.c_int, vp, vp, sz,
                                            vp]
        l.conv2d_last_launch_error.argtypes = []
        l.conv2d_last_launch_error.restype = ctypes.c_char_p
        l.conv2d_select_variant.argtypes = [pp, ctypes.c_uint32, ctypes.POINTER(ctypes.c_int)]
        l.conv2d_status_string.argtypes = [ctypes.c_int]
        l.conv2d_status_string.restype = ctypes.c_char_p
        l.conv2d_version.argtypes = []
        _lib = l
    return _lib


def make_params(batch, in_rows, in_cols, channels, features, window_rows, window_cols,
                stride_rows=1, stride_cols=1, padding=PAD_SAME, in_dtype=F32, out_dtype=F32):
    return Params(batch, in_rows, in_cols, channels, features, window_rows, window_cols,
                  stride_rows, stride_cols, padding, in_dtype, out_dtype)


def params_of_layer(layer, in_dtype=F32, out_dtype=F32, batch=None):
    """conv2d_params for a workloads.Layer."""
    return make_params(layer.batch if batch is None else batch, layer.in_rows, layer.in_cols,
                       layer.channels, layer.features, layer.window_rows, layer.window_cols,
                       layer.stride_rows, layer.stride_cols, layer.padding, in_dtype, out_dtype)


def status_string(status):
    return lib().conv2d_status_string(int(status)).decode()


def conv2d_version():
    return int(lib().conv2d_version())


def conv2d_get_geometry(params):
    g = Geometry()
    rc = lib().conv2d_get_geometry(ctypes.byref(params), ctypes.byref(g))
    if rc:
        raise Conv2dError(rc, "conv2d_get_geometry")
    return g


def conv2d_workspace_size(params, variant_id=None):
    n = ctypes.c_size_t(0)
    if variant_id is None:
        rc = lib().conv2d_workspace_size(ctypes.byref(params), ctypes.byref(n))
    else:
        rc = lib().conv2d_workspace_size_variant(ctypes.byref(params), int(variant_id),
                                                 ctypes.byref(n))
    if rc:
        raise Conv2dError(rc, "conv2d_workspace_size")
    return int(n.value)


def conv2d_num_variants():
    return int(lib().conv2d_num_variants())


def conv2d_variant_name(variant_id):
    s = lib().conv2d_variant_name(int(variant_id))
    return None if s is None else s.decode()


def conv2d_variant_supports(params, variant_id):
    rc = lib().conv2d_variant_supports(ctypes.byref(params), int(variant_id))
    if rc < 0:
        raise Conv2dError(rc, "conv2d_variant_supports")
    return bool(rc)


def conv2d_selected_variant(params):
    v = ctypes.c_int(-1)
    rc = lib().conv2d_selected_variant(ctypes.byref(params), ctypes.byref(v))
    if rc:
        raise Conv2dError(rc, "conv2d_selected_variant")
    return int(v.value)


SELECT_DIRECT_SUM_ONLY = 1


def conv2d_select_variant(params, flags=0):
    v = ctypes.c_int(-1)
    rc = lib().conv2d_select_variant(ctypes.byref(params), flags, ctypes.byref(v))
    if rc:
        raise Conv2dError(rc, "conv2d_select_variant")
    return int(v.value)


def variant_id_by_name(name):
    for i in range(conv2d_num_variants()):
        if conv2d_variant_name(i) == name:
            return i
    raise KeyError(name)


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def conv2d_forward_raw(params, in_ptr, filt_ptr, out_ptr, workspace_ptr=0, workspace_bytes=0,
                       stream_handle=0, variant_id=None):
    """Direct pointer-level call; returns the status code without raising."""
    l = lib()
    if variant_id is None:
        return l.conv2d_forward(ctypes.byref(params), in_ptr, filt_ptr, out_ptr, workspace_ptr,
                                workspace_bytes, stream_handle)
    return l.conv2d_forward_variant(ctypes.byref(params), in_ptr, filt_ptr, out_ptr,
                                    workspace_ptr, workspace_bytes, stream_handle,
                                    int(variant_id))


def conv2d_debug_force_variant(variant_id):
    """Forces `variant_id` (None or -1: off) for the calling thread's selecting entry points."""
    rc = lib().conv2d_debug_force_variant(-1 if variant_id is None else int(variant_id))
    if rc:
        raise Conv2dError(rc, "conv2d_debug_force_variant")


def conv2d_debug_split_reduce_separate(on):
    """True: the split-reduction variants add their partial sums in a second launch, always."""
    rc = lib().conv2d_debug_split_reduce_separate(1 if on else 0)
    if rc:
        raise Conv2dError(rc, "conv2d_debug_split_reduce_separate")


STATIC_SCRATCH_BYTES = 32 << 20   # CONV2D_STATIC_SCRATCH_BYTES
STATUS_SCRATCH_EXCEEDED = -6


def conv2d_forward_static_scratch_raw(params, in_ptr, filt_ptr, out_ptr, stream_handle=0):
    """conv2d_forward_static_scratch on raw device pointers: no workspace argument, nothing is
    allocated (the caller owns `out`); returns the status code without raising."""
    return lib().conv2d_forward_static_scratch(ctypes.byref(params), in_ptr, filt_ptr, out_ptr,
                                               stream_handle)


ACT_NONE = 0
ACT_RELU = 1


def conv2d_forward_bias_act(params, x, filt, bias, activation, out=None, workspace=None,
                            stream=None):
    """out = act(conv(x, filt) + bias): `bias` a float32 device tensor of `features` values or
    None, `activation` ACT_NONE or ACT_RELU.  Otherwise as conv2d_forward."""
    return conv2d_forward(params, x, filt, out, workspace, stream, None, bias, activation, True)


def conv2d_packed_filter_size(params, variant_id):
    n = ctypes.c_size_t(0)
    rc = lib().conv2d_packed_filter_size(ctypes.byref(params), int(variant_id), ctypes.byref(n))
    if rc:
        raise Conv2dError(rc, "conv2d_packed_filter_size")
    return int(n.value)


def conv2d_pack_filter(params, variant_id, filt, stream=None):
    """The filter (a contiguous HWCF device tensor) packed for `variant_id`: a uint8 device
    tensor to hand to conv2d_forward_packed."""
    import torch
    need = conv2d_packed_filter_size(params, variant_id)
    packed = torch.empty(max(need, 16), dtype=torch.uint8, device=filt.device)
    rc = lib().conv2d_pack_filter(ctypes.byref(params), int(variant_id), filt.data_ptr(),
                                  packed.data_ptr(), need, _stream_handle(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_pack_filter")
    return packed


def conv2d_forward_packed_raw(params, variant_id, in_ptr, packed_ptr, bias_ptr, activation, out_ptr,
                              ws_ptr, ws_bytes, stream_handle):
    """The C call itself on raw device pointers; returns the status."""
    return lib().conv2d_forward_packed(ctypes.byref(params), int(variant_id), in_ptr, packed_ptr,
                                       bias_ptr, int(activation), out_ptr, ws_ptr, ws_bytes,
                                       stream_handle)


def conv2d_forward_packed(params, variant_id, x, packed, bias=None, activation=ACT_NONE, out=None,
                          workspace=None, stream=None):
    """out = act(conv(x, filter) + bias) with `variant_id` on a filter packed by
    conv2d_pack_filter for the same variant and parameters."""
    import torch
    g = conv2d_get_geometry(params)
    want_out = torch.float32 if params.out_dtype == F32 else torch.bfloat16
    if tuple(x.shape) != (params.batch, params.in_rows, params.in_cols, params.channels) or \
            not (x.is_cuda and x.is_contiguous()):
        raise ValueError("input does not match params")
    oshape = (params.batch, g.out_rows, g.out_cols, params.features)
    if out is None:
        out = torch.empty(oshape, dtype=want_out, device=x.device)
    elif tuple(out.shape) != oshape or out.dtype != want_out or not out.is_contiguous():
        raise ValueError("output tensor does not match params")
    need = conv2d_workspace_size(params, variant_id)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    rc = conv2d_forward_packed_raw(
        params, variant_id, x.data_ptr(), packed.data_ptr(),
        bias.data_ptr() if bias is not None else 0, activation, out.data_ptr(),
        workspace.data_ptr() if workspace is not None else 0,
        workspace.numel() * workspace.element_size() if workspace is not None else 0,
        _stream_handle(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_forward_packed")
    return out


def conv2d_pool_workspace_size(params, variant_id=None):
    n = ctypes.c_size_t(0)
    if variant_id is None:
        rc = lib().conv2d_pool_workspace_size(ctypes.byref(params), ctypes.byref(n))
    else:
        rc = lib().conv2d_pool_workspace_size_variant(ctypes.byref(params), int(variant_id),
                                                      ctypes.byref(n))
    if rc:
        raise Conv2dError(rc, "conv2d_pool_workspace_size")
    return int(n.value)


def conv2d_forward_bias_act_pool(params, x, filt, bias, activation, out=None, workspace=None,
                                 stream=None):
    """out = max_pool_2x2(act(conv(x, filt) + bias)); `out` is [batch, out_rows // 2,
    out_cols // 2, features].  Otherwise as conv2d_forward_bias_act."""
    import torch
    g = conv2d_get_geometry(params)
    want_in = torch.float32 if params.in_dtype == F32 else torch.bfloat16
    want_out = torch.float32 if params.out_dtype == F32 else torch.bfloat16
    if x.dtype != want_in or filt.dtype != want_in:
        raise TypeError("input/filter dtype does not match params.in_dtype")
    if not (x.is_cuda and filt.is_cuda and x.is_contiguous() and filt.is_contiguous()):
        raise ValueError("input and filter must be contiguous device tensors")
    if tuple(x.shape) != (params.batch, params.in_rows, params.in_cols, params.channels):
        raise ValueError("input shape does not match params")
    if tuple(filt.shape) != (params.window_rows, params.window_cols, params.channels,
                             params.features):
        raise ValueError("filter shape does not match params")
    if bias is not None and not (bias.is_cuda and bias.dtype == torch.float32 and
                                 bias.is_contiguous() and bias.numel() == params.features):
        raise ValueError("bias must be a contiguous float32 device tensor of `features` values")
    oshape = (params.batch, g.out_rows // 2, g.out_cols // 2, params.features)
    if out is None:
        out = torch.empty(oshape, dtype=want_out, device=x.device)
    elif tuple(out.shape) != oshape or out.dtype != want_out or not out.is_contiguous():
        raise ValueError("output tensor does not match params")
    need = conv2d_pool_workspace_size(params)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib().conv2d_forward_bias_act_pool(
        ctypes.byref(params), x.data_ptr(), filt.data_ptr(),
        bias.data_ptr() if bias is not None else 0, int(activation), out.data_ptr(), ws_ptr,
        ws_bytes, _stream_handle(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_forward_bias_act_pool")
    return out


def conv2d_forward(params, x, filt, out=None, workspace=None, stream=None, variant_id=None,
                   bias=None, activation=ACT_NONE, fused=False):
    """Enqueue the forward convolution of torch device tensors.

    x: NHWC, filt: HWCF, contiguous, float32 or bfloat16 matching params.in_dtype.
    Returns `out` (allocated here if not given).  Does not synchronise.
    """
    import torch
    g = conv2d_get_geometry(params)
    want_in = torch.float32 if params.in_dtype == F32 else torch.bfloat16
    want_out = torch.float32 if params.out_dtype == F32 else torch.bfloat16
    if x.dtype != want_in or filt.dtype != want_in:
        raise TypeError("input/filter dtype does not match params.in_dtype")
    if not (x.is_cuda and filt.is_cuda and x.is_contiguous() and filt.is_contiguous()):
        raise ValueError("input and filter must be contiguous device tensors")
    if tuple(x.shape) != (params.batch, params.in_rows, params.in_cols, params.channels):
        raise ValueError("input shape does not match params")
    if tuple(filt.shape) != (params.window_rows, params.window_cols, params.channels,
                             params.features):
        raise ValueError("filter shape does not match params")
    oshape = (params.batch, g.out_rows, g.out_cols, params.features)
    if out is None:
        out = torch.empty(oshape, dtype=want_out, device=x.device)
    elif tuple(out.shape) != oshape or out.dtype != want_out or not out.is_contiguous():
        raise ValueError("output tensor does not match params")
    need = conv2d_workspace_size(params, variant_id)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    if fused:
        if variant_id is not None:
            raise ValueError("the fused entry point selects the variant itself")
        if bias is not None and not (bias.is_cuda and bias.dtype == torch.float32 and
                                     bias.is_contiguous() and bias.numel() == params.features):
            raise ValueError("bias must be a contiguous float32 device tensor of `features` values")
        rc = lib().conv2d_forward_bias_act(
            ctypes.byref(params), x.data_ptr(), filt.data_ptr(),
            bias.data_ptr() if bias is not None else 0, int(activation), out.data_ptr(), ws_ptr,
            ws_bytes, _stream_handle(stream))
        if rc:
            raise Conv2dError(rc, "conv2d_forward_bias_act")
        return out
    rc = conv2d_forward_raw(params, x.data_ptr(), filt.data_ptr(), out.data_ptr(), ws_ptr,
                            ws_bytes, _stream_handle(stream), variant_id)
    if rc:
        raise Conv2dError(rc, "conv2d_forward")
    return out
