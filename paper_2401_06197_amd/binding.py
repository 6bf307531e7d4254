"""ctypes binding of include/dcnv4.h: same names, argument marshalling only.

The tensor arguments are torch tensors on the GPU (torch is used for device memory and
streams, nothing else); every step of the operator runs inside libdcnv4.so.  If the
library has not been built the import of it fails loudly -- there is no fallback path.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdcnv4.so")

DCNV4_F32, DCNV4_F16 = 0, 1
DCNV4_OK = 0

# every symbol include/dcnv4.h declares
EXPORTS = (
    "dcnv4_output_hw", "dcnv4_forward", "dcnv4_backward", "dcnv4_forward_merged", "dcnv4_backward_merged",
    "dcnv4_forward_softmax", "dcnv4_backward_softmax",
    "dcnv4_linear", "dcnv4_depthwise3x3", "dcnv4_module_forward", "dcnv4_module_workspace_bytes",
    "dcnv4_module_forward_static", "dcnv4_module_static_workspace_limit",
    "dcnv4_forward_algorithmic_bytes", "dcnv4_backward_algorithmic_bytes",
    "dcnv4_forward_merged_algorithmic_bytes", "dcnv4_backward_merged_algorithmic_bytes",
    "dcnv4_set_option", "dcnv4_last_kernel_name", "dcnv4_status_string",
)

_lib = None


class Dcnv4Error(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: status {status} ({dcnv4_status_string(status)})")


def load_library():
    """Load libdcnv4.so (built in-tree by paper_2401_06197_amd.build); raise if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2401_06197_amd.build` "
            "(the DCNv4 operator has no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    ip = ctypes.POINTER(ctypes.c_int)
    lib.dcnv4_output_hw.argtypes = [ci] * 10 + [ip, ip]
    lib.dcnv4_output_hw.restype = ci
    geo = [ci] * 13 + [cf, ci, vp]
    lib.dcnv4_forward.argtypes = [vp] * 4 + geo
    lib.dcnv4_forward.restype = ci
    lib.dcnv4_backward.argtypes = [vp] * 7 + geo
    lib.dcnv4_backward.restype = ci
    lib.dcnv4_forward_softmax.argtypes = [vp] * 4 + geo
    lib.dcnv4_forward_softmax.restype = ci
    lib.dcnv4_backward_softmax.argtypes = [vp] * 7 + geo
    lib.dcnv4_backward_softmax.restype = ci
    lib.dcnv4_forward_merged.argtypes = [vp] * 3 + geo
    lib.dcnv4_forward_merged.restype = ci
    lib.dcnv4_backward_merged.argtypes = [vp] * 5 + geo
    lib.dcnv4_backward_merged.restype = ci
    for f in (lib.dcnv4_forward_algorithmic_bytes, lib.dcnv4_backward_algorithmic_bytes,
              lib.dcnv4_forward_merged_algorithmic_bytes, lib.dcnv4_backward_merged_algorithmic_bytes):
        f.argtypes = [ci] * 8
        f.restype = ctypes.c_longlong
    lib.dcnv4_linear.argtypes = [vp] * 4 + [ctypes.c_longlong, ci, ci, ci, vp]
    lib.dcnv4_linear.restype = ci
    lib.dcnv4_depthwise3x3.argtypes = [vp] * 4 + [ci] * 5 + [vp]
    lib.dcnv4_depthwise3x3.restype = ci
    lib.dcnv4_module_forward.argtypes = [vp] * 10 + [ctypes.c_longlong, vp] + geo
    lib.dcnv4_module_forward.restype = ci
    lib.dcnv4_module_forward_static.argtypes = [vp] * 10 + geo
    lib.dcnv4_module_forward_static.restype = ci
    lib.dcnv4_module_static_workspace_limit.argtypes = []
    lib.dcnv4_module_static_workspace_limit.restype = ctypes.c_longlong
    lib.dcnv4_module_workspace_bytes.argtypes = [ci] * 8
    lib.dcnv4_module_workspace_bytes.restype = ctypes.c_longlong
    lib.dcnv4_set_option.argtypes = [ctypes.c_char_p, ci]
    lib.dcnv4_set_option.restype = ci
    lib.dcnv4_last_kernel_name.argtypes = [ci]
    lib.dcnv4_last_kernel_name.restype = ctypes.c_char_p
    lib.dcnv4_status_string.argtypes = [ci]
    lib.dcnv4_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _pair(v):
    return (int(v), int(v)) if isinstance(v, int) else (int(v[0]), int(v[1]))


def dcnv4_status_string(status):
    return load_library().dcnv4_status_string(int(status)).decode()


def dcnv4_output_hw(H, W, kernel=3, stride=1, pad=1, dilation=1):
    (kh, kw), (sh, sw), (ph, pw), (dh, dw) = map(_pair, (kernel, stride, pad, dilation))
    ho, wo = ctypes.c_int(0), ctypes.c_int(0)
    rc = load_library().dcnv4_output_hw(H, W, kh, kw, sh, sw, ph, pw, dh, dw, ctypes.byref(ho), ctypes.byref(wo))
    if rc:
        raise Dcnv4Error(rc, "dcnv4_output_hw")
    return ho.value, wo.value


def dcnv4_set_option(key, value):
    rc = load_library().dcnv4_set_option(key.encode(), int(value))
    if rc:
        raise Dcnv4Error(rc, f"dcnv4_set_option({key!r}, {value})")


def dcnv4_last_kernel_name(backward):
    s = load_library().dcnv4_last_kernel_name(int(backward))
    return s.decode() if s else None


def dcnv4_forward_algorithmic_bytes(N, H, W, G, Cg, Ho, Wo, dtype):
    return int(load_library().dcnv4_forward_algorithmic_bytes(N, H, W, G, Cg, Ho, Wo, dtype))


def dcnv4_backward_algorithmic_bytes(N, H, W, G, Cg, Ho, Wo, dtype):
    return int(load_library().dcnv4_backward_algorithmic_bytes(N, H, W, G, Cg, Ho, Wo, dtype))


def dcnv4_forward_merged_algorithmic_bytes(N, H, W, G, Cg, Ho, Wo, dtype):
    return int(load_library().dcnv4_forward_merged_algorithmic_bytes(N, H, W, G, Cg, Ho, Wo, dtype))


def dcnv4_backward_merged_algorithmic_bytes(N, H, W, G, Cg, Ho, Wo, dtype):
    return int(load_library().dcnv4_backward_merged_algorithmic_bytes(N, H, W, G, Cg, Ho, Wo, dtype))


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return DCNV4_F32
    if t.dtype == torch.float16:
        return DCNV4_F16
    raise TypeError(f"dcnv4: unsupported tensor dtype {t.dtype}")


def _check(name, t, ref):
    if not t.is_cuda:
        raise ValueError(f"dcnv4: {name} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"dcnv4: {name} must be contiguous")
    if t.dtype != ref.dtype or t.device != ref.device:
        raise ValueError(f"dcnv4: {name} must share dtype and device with x")


def _stream_ptr(stream, device):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(device)
    return ctypes.c_void_p(stream.cuda_stream)


def _shape_args(x, offset, mask, kernel, stride, pad, dilation):
    (kh, kw), (sh, sw), (ph, pw), (dh, dw) = map(_pair, (kernel, stride, pad, dilation))
    if x.dim() != 4 or offset.dim() != 6 or mask.dim() != 5:
        raise ValueError("dcnv4: expected x [N,H,W,C], offset [N,Ho,Wo,G,K,2], mask [N,Ho,Wo,G,K]")
    N, H, W, C = x.shape
    G = mask.shape[3]
    if G < 1 or C % G:
        raise ValueError("dcnv4: C must be a multiple of G")
    Ho, Wo = dcnv4_output_hw(H, W, (kh, kw), (sh, sw), (ph, pw), (dh, dw))
    K = kh * kw
    if tuple(mask.shape) != (N, Ho, Wo, G, K) or tuple(offset.shape) != (N, Ho, Wo, G, K, 2):
        raise ValueError(f"dcnv4: offset/mask shapes {tuple(offset.shape)}/{tuple(mask.shape)} do not match "
                         f"N={N} Ho={Ho} Wo={Wo} G={G} K={K}")
    return (N, H, W, G, C // G, kh, kw, sh, sw, ph, pw, dh, dw), (N, Ho, Wo, C)


def dcnv4_forward(x, offset, mask, kernel=3, stride=1, pad=1, dilation=1, offset_scale=1.0, out=None, stream=None,
                  prepare_only=False, _entry="dcnv4_forward"):
    """y [N,Ho,Wo,C] = DCNv4 aggregation of x [N,H,W,C] (Eq. 1-2 of the paper, no softmax).

    With prepare_only the checked argument tuple for load_library().dcnv4_forward is returned
    instead of launching (for launch loops that must not pay the checks every time)."""
    import torch
    geo, yshape = _shape_args(x, offset, mask, kernel, stride, pad, dilation)
    for name, t in (("x", x), ("offset", offset), ("mask", mask)):
        _check(name, t, x)
    if out is None:
        out = torch.empty(yshape, dtype=x.dtype, device=x.device)
    else:
        _check("out", out, x)
        if tuple(out.shape) != yshape:
            raise ValueError("dcnv4: out has the wrong shape")
    args = (x.data_ptr(), offset.data_ptr(), mask.data_ptr(), out.data_ptr(), *geo,
            float(offset_scale), _dtype_code(x), _stream_ptr(stream, x.device))
    if prepare_only:
        return args
    with torch.cuda.device(x.device):
        rc = getattr(load_library(), _entry)(*args)
    if rc:
        raise Dcnv4Error(rc, _entry)
    return out


def dcnv4_forward_softmax(x, offset, mask_logits, **kw):
    """dcnv4_forward with m = softmax of mask_logits over the 9 taps (the DCNv3 form)."""
    return dcnv4_forward(x, offset, mask_logits, _entry="dcnv4_forward_softmax", **kw)


def dcnv4_backward_softmax(x, offset, mask_logits, grad_y, **kw):
    """(grad_x, grad_offset, grad_mask_logits) of dcnv4_forward_softmax."""
    return dcnv4_backward(x, offset, mask_logits, grad_y, _entry="dcnv4_backward_softmax", **kw)


def dcnv4_backward(x, offset, mask, grad_y, kernel=3, stride=1, pad=1, dilation=1, offset_scale=1.0,
                   out=None, stream=None, prepare_only=False, _entry="dcnv4_backward"):
    """(grad_x, grad_offset, grad_mask) of dcnv4_forward for upstream gradient grad_y."""
    import torch
    geo, yshape = _shape_args(x, offset, mask, kernel, stride, pad, dilation)
    for name, t in (("x", x), ("offset", offset), ("mask", mask), ("grad_y", grad_y)):
        _check(name, t, x)
    if tuple(grad_y.shape) != yshape:
        raise ValueError("dcnv4: grad_y has the wrong shape")
    if out is None:
        out = (torch.empty_like(x), torch.empty_like(offset), torch.empty_like(mask))
    gx, go, gm = out
    for name, t, ref in (("grad_x", gx, x), ("grad_offset", go, offset), ("grad_mask", gm, mask)):
        _check(name, t, x)
        if t.shape != ref.shape:
            raise ValueError(f"dcnv4: {name} has the wrong shape")
    args = (x.data_ptr(), offset.data_ptr(), mask.data_ptr(), grad_y.data_ptr(),
            gx.data_ptr(), go.data_ptr(), gm.data_ptr(), *geo,
            float(offset_scale), _dtype_code(x), _stream_ptr(stream, x.device))
    if prepare_only:
        return args
    with torch.cuda.device(x.device):
        rc = getattr(load_library(), _entry)(*args)
    if rc:
        raise Dcnv4Error(rc, _entry)
    return gx, go, gm


def _merged_shape_args(x, om, kernel, stride, pad, dilation):
    (kh, kw), (sh, sw), (ph, pw), (dh, dw) = map(_pair, (kernel, stride, pad, dilation))
    if x.dim() != 4 or om.dim() != 5 or om.shape[4] != 32:
        raise ValueError("dcnv4: expected x [N,H,W,C] and offset_mask [N,Ho,Wo,G,32]")
    N, H, W, C = x.shape
    G = om.shape[3]
    if G < 1 or C % G:
        raise ValueError("dcnv4: C must be a multiple of G")
    Ho, Wo = dcnv4_output_hw(H, W, (kh, kw), (sh, sw), (ph, pw), (dh, dw))
    if tuple(om.shape) != (N, Ho, Wo, G, 32):
        raise ValueError(f"dcnv4: offset_mask shape {tuple(om.shape)} does not match N={N} Ho={Ho} Wo={Wo} G={G}")
    return (N, H, W, G, C // G, kh, kw, sh, sw, ph, pw, dh, dw), (N, Ho, Wo, C)


def dcnv4_forward_merged(x, offset_mask, kernel=3, stride=1, pad=1, dilation=1, offset_scale=1.0, out=None, stream=None,
                         prepare_only=False):
    """dcnv4_forward with the offsets and mask values in one tensor [N,Ho,Wo,G,32]: 18 offsets, 9 mask
    values, 5 unused entries per (pixel, group)."""
    import torch
    geo, yshape = _merged_shape_args(x, offset_mask, kernel, stride, pad, dilation)
    for name, t in (("x", x), ("offset_mask", offset_mask)):
        _check(name, t, x)
    if out is None:
        out = torch.empty(yshape, dtype=x.dtype, device=x.device)
    else:
        _check("out", out, x)
        if tuple(out.shape) != yshape:
            raise ValueError("dcnv4: out has the wrong shape")
    args = (x.data_ptr(), offset_mask.data_ptr(), out.data_ptr(), *geo,
            float(offset_scale), _dtype_code(x), _stream_ptr(stream, x.device))
    if prepare_only:
        return args
    with torch.cuda.device(x.device):
        rc = load_library().dcnv4_forward_merged(*args)
    if rc:
        raise Dcnv4Error(rc, "dcnv4_forward_merged")
    return out


def dcnv4_backward_merged(x, offset_mask, grad_y, kernel=3, stride=1, pad=1, dilation=1, offset_scale=1.0,
                          out=None, stream=None, prepare_only=False):
    """(grad_x, grad_offset_mask) of dcnv4_forward_merged; grad_offset_mask is laid out like offset_mask."""
    import torch
    geo, yshape = _merged_shape_args(x, offset_mask, kernel, stride, pad, dilation)
    for name, t in (("x", x), ("offset_mask", offset_mask), ("grad_y", grad_y)):
        _check(name, t, x)
    if tuple(grad_y.shape) != yshape:
        raise ValueError("dcnv4: grad_y has the wrong shape")
    if out is None:
        out = (torch.empty_like(x), torch.empty_like(offset_mask))
    gx, gom = out
    for name, t, ref in (("grad_x", gx, x), ("grad_offset_mask", gom, offset_mask)):
        _check(name, t, x)
        if t.shape != ref.shape:
            raise ValueError(f"dcnv4: {name} has the wrong shape")
    args = (x.data_ptr(), offset_mask.data_ptr(), grad_y.data_ptr(), gx.data_ptr(), gom.data_ptr(), *geo,
            float(offset_scale), _dtype_code(x), _stream_ptr(stream, x.device))
    if prepare_only:
        return args
    with torch.cuda.device(x.device):
        rc = load_library().dcnv4_backward_merged(*args)
    if rc:
        raise Dcnv4Error(rc, "dcnv4_backward_merged")
    return gx, gom


def dcnv4_linear(x, w, b=None, out=None, stream=None, prepare_only=False):
    """y[..., o] = sum_k x[..., k] * w[o, k] + b[o]: a linear layer over the last axis of x (a 1x1
    point-wise convolution of an NHWC map), on the matrix cores."""
    import torch
    if x.dim() < 2 or w.dim() != 2 or w.shape[1] != x.shape[-1] or (b is not None and tuple(b.shape) != (w.shape[0],)):
        raise ValueError("dcnv4: expected x [..., K], w [Nout, K], b [Nout]")
    for name, t in (("x", x), ("w", w)) + ((("b", b),) if b is not None else ()):
        _check(name, t, x)
    yshape = tuple(x.shape[:-1]) + (w.shape[0],)
    if out is None:
        out = torch.empty(yshape, dtype=x.dtype, device=x.device)
    else:
        _check("out", out, x)
        if tuple(out.shape) != yshape:
            raise ValueError("dcnv4: out has the wrong shape")
    P = x.numel() // x.shape[-1]
    args = (x.data_ptr(), w.data_ptr(), b.data_ptr() if b is not None else None, out.data_ptr(), P, x.shape[-1],
            w.shape[0], _dtype_code(x), _stream_ptr(stream, x.device))
    if prepare_only:
        return args
    with torch.cuda.device(x.device):
        rc = load_library().dcnv4_linear(*args)
    if rc:
        raise Dcnv4Error(rc, "dcnv4_linear")
    return out


def dcnv4_depthwise3x3(x, w, b=None, out=None, stream=None):
    """y[n,h,w,c] = b[c] + sum_ij w[i,j,c] * x[n,h+i-1,w+j-1,c] (zero padding): x [N,H,W,C], w [3,3,C]."""
    import torch
    if x.dim() != 4 or tuple(w.shape) != (3, 3, x.shape[3]) or (b is not None and tuple(b.shape) != (x.shape[3],)):
        raise ValueError("dcnv4: expected x [N,H,W,C], w [3,3,C], b [C]")
    for name, t in (("x", x), ("w", w)) + ((("b", b),) if b is not None else ()):
        _check(name, t, x)
    if out is None:
        out = torch.empty_like(x)
    else:
        _check("out", out, x)
        if out.shape != x.shape:
            raise ValueError("dcnv4: out has the wrong shape")
    N, H, W, C = x.shape
    with torch.cuda.device(x.device):
        rc = load_library().dcnv4_depthwise3x3(x.data_ptr(), w.data_ptr(), b.data_ptr() if b is not None else None,
                                               out.data_ptr(), N, H, W, C, _dtype_code(x), _stream_ptr(stream, x.device))
    if rc:
        raise Dcnv4Error(rc, "dcnv4_depthwise3x3")
    return out


def dcnv4_module_workspace_bytes(N, H, W, G, Cg, dtype, lightweight, depthwise=False):
    return int(load_library().dcnv4_module_workspace_bytes(N, H, W, G, Cg, dtype, int(bool(lightweight)), int(bool(depthwise))))


def dcnv4_module_forward(x, w_om, b_om, G, w_in=None, b_in=None, w_out=None, b_out=None, w_dw=None, b_dw=None, kernel=3,
                         stride=1, pad=1, dilation=1, offset_scale=1.0, workspace=None, out=None, stream=None,
                         prepare_only=False):
    """Forward of the DCNv4 module: (value projection,) ONE linear layer for offsets and modulation
    scalars, the operator, (output projection).  w_om [G*32, C] / b_om [G*32] in the merged layout
    (row g*32 + e: entry e of group g; 0..17 offsets, 18..26 scalars, 27..31 ignored); w_in, w_out
    [C, C] or both None (the lightweight variant); w_dw [3, 3, C] / b_dw [C]: the optional depthwise
    convolution in front of the offset/scalar layer."""
    import torch
    if x.dim() != 4 or x.shape[3] % G:
        raise ValueError("dcnv4: expected x [N,H,W,C] with C a multiple of G")
    N, H, W, C = x.shape
    (kh, kw), (sh, sw), (ph, pw), (dh, dw) = map(_pair, (kernel, stride, pad, dilation))
    if (w_in is None) != (w_out is None):
        raise ValueError("dcnv4: the input and output projections come together")
    shapes = [("w_om", w_om, (G * 32, C)), ("b_om", b_om, (G * 32,)), ("w_in", w_in, (C, C)), ("b_in", b_in, (C,)),
              ("w_out", w_out, (C, C)), ("b_out", b_out, (C,)), ("w_dw", w_dw, (3, 3, C)), ("b_dw", b_dw, (C,))]
    for name, t, shape in shapes:
        if t is not None:
            _check(name, t, x)
            if tuple(t.shape) != shape:
                raise ValueError(f"dcnv4: {name} must have shape {shape}")
    _check("x", x, x)
    light = w_in is None
    need = dcnv4_module_workspace_bytes(N, H, W, G, C // G, _dtype_code(x), light, w_dw is not None)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    elif not workspace.is_cuda or workspace.device != x.device or not workspace.is_contiguous():
        raise ValueError("dcnv4: workspace must be a contiguous tensor on x's device")
    if out is None:
        out = torch.empty_like(x)
    else:
        _check("out", out, x)
        if out.shape != x.shape:
            raise ValueError("dcnv4: out has the wrong shape")
    ptr = lambda t: t.data_ptr() if t is not None else None
    args = (x.data_ptr(), ptr(w_in), ptr(b_in), ptr(w_dw), ptr(b_dw), w_om.data_ptr(), ptr(b_om), ptr(w_out), ptr(b_out), workspace.data_ptr(),
            workspace.numel() * workspace.element_size(), out.data_ptr(), N, H, W, G, C // G, kh, kw, sh, sw, ph, pw,
            dh, dw, float(offset_scale), _dtype_code(x), _stream_ptr(stream, x.device))
    if prepare_only:
        return args
    with torch.cuda.device(x.device):
        rc = load_library().dcnv4_module_forward(*args)
    if rc:
        raise Dcnv4Error(rc, "dcnv4_module_forward")
    return out


def dcnv4_module_static_workspace_limit():
    return int(load_library().dcnv4_module_static_workspace_limit())


def dcnv4_module_forward_static(x, w_om, b_om, G, out, w_in=None, b_in=None, w_out=None, b_out=None, w_dw=None, b_dw=None,
                                kernel=3, stride=1, pad=1, dilation=1, offset_scale=1.0, stream=None):
    """dcnv4_module_forward with the workspace in the library's built-in buffer: nothing is allocated, here
    or in the library (the caller passes `out`).  Raises Dcnv4Error (status 6) if the call needs more than
    dcnv4_module_static_workspace_limit() bytes."""
    args = dcnv4_module_forward(x, w_om, b_om, G, w_in=w_in, b_in=b_in, w_out=w_out, b_out=b_out, w_dw=w_dw, b_dw=b_dw,
                                kernel=kernel, stride=stride, pad=pad, dilation=dilation, offset_scale=offset_scale,
                                workspace=x, out=out, stream=stream, prepare_only=True)
    args = args[:9] + args[11:]                      # the same arguments without (workspace, workspace_bytes)
    import torch
    with torch.cuda.device(x.device):
        rc = load_library().dcnv4_module_forward_static(*args)
    if rc:
        raise Dcnv4Error(rc, "dcnv4_module_forward_static")
    return out
