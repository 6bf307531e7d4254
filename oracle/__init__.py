"""CPU oracle for the DCNv4 spatial-aggregation operator.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around oracle/dcnv4_oracle.c (plain double-precision loops that
write out Eq. 1-2 of the paper and their chain-rule gradients).  Only the tests, the
smoke check and the benchmark's CPU-baseline leg may import this package; the
product package never does, and this package imports nothing from the product.

Arrays are numpy, any float dtype on input (widened exactly to float64), float64 out:
  x [N,H,W,C]   offset [N,Ho,Wo,G,K,2] ([...,0] along width, [...,1] along height)
  mask [N,Ho,Wo,G,K]   y / grad_y [N,Ho,Wo,C]
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        # (the mutation check of the pins points this at a deliberately broken copy, built elsewhere)
        path = os.environ.get("DCNV4_ORACLE_LIB") or _build.build(force=False)
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ints = [ctypes.c_int] * 13
        lib.dcnv4_oracle_forward.argtypes = [dp, dp, dp, dp] + ints + [ctypes.c_double]
        lib.dcnv4_oracle_forward.restype = ctypes.c_int
        lib.dcnv4_oracle_backward.argtypes = [dp] * 7 + ints + [ctypes.c_double]
        lib.dcnv4_oracle_backward.restype = ctypes.c_int
        lib.dcnv4_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    """Number of host threads the oracle's loops run on."""
    return int(_load().dcnv4_oracle_threads())


def _pair(v):
    return (int(v), int(v)) if np.isscalar(v) else (int(v[0]), int(v[1]))


def output_hw(H, W, kernel=3, stride=1, pad=1, dilation=1):
    (kh, kw), (sh, sw), (ph, pw), (dh, dw) = map(_pair, (kernel, stride, pad, dilation))
    Ho = (H + 2 * ph - dh * (kh - 1) - 1) // sh + 1
    Wo = (W + 2 * pw - dw * (kw - 1) - 1) // sw + 1
    return Ho, Wo


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _geometry(x, offset, mask, kernel, stride, pad, dilation):
    (kh, kw), (sh, sw), (ph, pw), (dh, dw) = map(_pair, (kernel, stride, pad, dilation))
    N, H, W, C = x.shape
    Ho, Wo = output_hw(H, W, kernel, stride, pad, dilation)
    K = kh * kw
    if mask.ndim != 5 or mask.shape[:3] != (N, Ho, Wo) or mask.shape[4] != K:
        raise ValueError(f"mask shape {mask.shape} does not match [N={N},Ho={Ho},Wo={Wo},G,K={K}]")
    G = mask.shape[3]
    if offset.shape != (N, Ho, Wo, G, K, 2):
        raise ValueError(f"offset shape {offset.shape} != {(N, Ho, Wo, G, K, 2)}")
    if C % G:
        raise ValueError("C must be a multiple of G")
    return (N, H, W, G, C // G, kh, kw, sh, sw, ph, pw, dh, dw), (Ho, Wo)


def forward(x, offset, mask, kernel=3, stride=1, pad=1, dilation=1, offset_scale=1.0):
    """y = sum_k m_k * bilinear(x_g, p0 + p_k + offset_scale * dp_k)   (Eq. 1-2, no softmax)."""
    x, offset, mask = _f64(x), _f64(offset), _f64(mask)
    geo, (Ho, Wo) = _geometry(x, offset, mask, kernel, stride, pad, dilation)
    y = np.empty((x.shape[0], Ho, Wo, x.shape[3]), dtype=np.float64)
    rc = _load().dcnv4_oracle_forward(_ptr(x), _ptr(offset), _ptr(mask), _ptr(y), *geo,
                                      float(offset_scale))
    if rc:
        raise ValueError("dcnv4_oracle_forward: bad geometry")
    return y


def backward(x, offset, mask, grad_y, kernel=3, stride=1, pad=1, dilation=1, offset_scale=1.0):
    """Chain-rule gradients of forward(): returns (grad_x, grad_offset, grad_mask)."""
    x, offset, mask, grad_y = _f64(x), _f64(offset), _f64(mask), _f64(grad_y)
    geo, (Ho, Wo) = _geometry(x, offset, mask, kernel, stride, pad, dilation)
    if grad_y.shape != (x.shape[0], Ho, Wo, x.shape[3]):
        raise ValueError("grad_y shape mismatch")
    gx = np.empty_like(x)
    go = np.empty_like(offset)
    gm = np.empty_like(mask)
    rc = _load().dcnv4_oracle_backward(_ptr(x), _ptr(offset), _ptr(mask), _ptr(grad_y),
                                       _ptr(gx), _ptr(go), _ptr(gm), *geo, float(offset_scale))
    if rc:
        raise ValueError("dcnv4_oracle_backward: bad geometry")
    return gx, go, gm


def split_merged(om, kernel=3):
    """[N,Ho,Wo,G,32] buffer of Sec. 3.2 "Micro design" (the single linear layer's output per group:
    2K offsets, K mask values, padding up to 32) -> (offset [N,Ho,Wo,G,K,2], mask [N,Ho,Wo,G,K])."""
    kh, kw = _pair(kernel)
    K = kh * kw
    om = np.asarray(om)
    if om.ndim != 5 or om.shape[4] < 3 * K:
        raise ValueError(f"merged offset/mask buffer of shape {om.shape}: last dimension must hold {3 * K} values")
    offset = om[..., :2 * K].reshape(om.shape[:4] + (K, 2))
    mask = om[..., 2 * K:3 * K]
    return offset, mask


def forward_merged(x, om, **kw):
    offset, mask = split_merged(om, kw.get("kernel", 3))
    return forward(x, offset, mask, **kw)


def backward_merged(x, om, grad_y, **kw):
    """Returns (grad_x, grad_om) with grad_om laid out like om; its padding entries are zero."""
    offset, mask = split_merged(om, kw.get("kernel", 3))
    gx, go, gm = backward(x, offset, mask, grad_y, **kw)
    K = mask.shape[4]
    gom = np.zeros(np.asarray(om).shape, dtype=np.float64)
    gom[..., :2 * K] = go.reshape(go.shape[:4] + (2 * K,))
    gom[..., 2 * K:3 * K] = gm
    return gx, gom


def softmax_taps(logits):
    """Softmax over the last axis (the K sampling points), in double precision."""
    z = _f64(logits)
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def forward_softmax(x, offset, mask_logits, **kw):
    """The DCNv3 form of Eq. 1 (Sec. 3.1): the modulation scalars are softmax-normalised over the K points
    before the aggregation.  Written out as that definition: normalise, then forward()."""
    return forward(x, offset, softmax_taps(mask_logits), **kw)


def backward_softmax(x, offset, mask_logits, grad_y, **kw):
    """Gradients of forward_softmax(): grad_x and grad_offset as in backward() with the normalised m; the
    gradient w.r.t. logit k is m_k * (g_k - sum_j m_j g_j), g being the gradient w.r.t. m."""
    m = softmax_taps(mask_logits)
    gx, go, gm = backward(x, offset, m, grad_y, **kw)
    gl = m * (gm - (m * gm).sum(axis=-1, keepdims=True))
    return gx, go, gl


def linear(x, w, b=None):
    """A linear layer over the channel axis (a 1x1 point-wise convolution, Sec. 3.1):
    y[..., o] = sum_c x[..., c] * w[o, c] + b[o], in double precision."""
    y = _f64(x) @ _f64(w).T
    if b is not None:
        y = y + _f64(b)
    return y


def _stored(a, storage):
    """What a layer hands to the next one: the double-precision value, or that value rounded once to
    the type the tensors are stored in (the half-precision module keeps every tensor in fp16, Sec. 3.2)."""
    return a if storage is None else a.astype(storage).astype(np.float64)


def module_forward(x, w_om, b_om, G, w_in=None, b_in=None, w_out=None, b_out=None, w_dw=None, b_dw=None,
                   storage=None, **kw):
    """The DCNv4 module (Sec. 3.1 last paragraph of the DCNv3 review, Sec. 3.2 "Micro design", and the
    two variants of the module-level benchmark in the appendix), no depthwise convolution:
        value = x W_in^T + b_in                      (left out in the lightweight variant: value = x)
        om    = x' W_om^T + b_om                     ONE linear layer: per group 2K offsets (tap-major,
                                                     width then height), then the K modulation scalars;
                                                     x' = depthwise3x3(x) if w_dw is given (the separable
                                                     structure of Sec. 3.2), else x
        y_op  = Eq. 1-2 on (value, offsets, scalars) no softmax
        y     = y_op W_out^T + b_out                 (left out in the lightweight variant)
    x [N,H,W,C]; w_om [G*3K, C]; w_in, w_out [C, C] (both given, or both None).  The window must keep
    the map's size (stride 1, pad = dilation*(kernel-1)/2): the layer predicts one set of offsets per
    input pixel.  `storage` (None, np.float16 or np.float32): the type the tensors between the layers are
    rounded to."""
    if (w_in is None) != (w_out is None):
        raise ValueError("input and output projections come together")
    x = _f64(x)
    kh, kw_ = _pair(kw.get("kernel", 3))
    K = kh * kw_
    N, H, W, C = x.shape
    if _f64(w_om).shape != (G * 3 * K, C):
        raise ValueError(f"w_om of shape {np.shape(w_om)}, expected {(G * 3 * K, C)}")
    value = x if w_in is None else _stored(linear(x, w_in, b_in), storage)
    x_om = x if w_dw is None else _stored(depthwise3x3(x, w_dw, b_dw), storage)
    om = _stored(linear(x_om, w_om, b_om), storage).reshape(N, H, W, G, 3 * K)
    offset, mask = split_merged(om, kw.get("kernel", 3))
    y = forward(value, offset, mask, **kw)
    if y.shape[1:3] != (H, W):
        raise ValueError("the module needs a window that keeps the map's size")
    if w_out is None:
        return y
    return linear(_stored(y, storage), w_out, b_out)


def depthwise3x3(x, w, b=None):
    """The 3x3 depthwise convolution of the separable structure the module uses to compute offsets and
    scalars (Sec. 3.2 "Micro design"), zero padding, stride 1:
        y[n,h,w,c] = b[c] + sum_{i,j in 0..2} w[i,j,c] * x[n, h+i-1, w+j-1, c]     (x = 0 outside the map)
    x [N,H,W,C]; w [3,3,C] (i: height tap, j: width tap); b [C] or None."""
    x, w = _f64(x), _f64(w)
    N, H, W, C = x.shape
    if w.shape != (3, 3, C):
        raise ValueError(f"depthwise weights of shape {w.shape}, expected {(3, 3, C)}")
    xp = np.zeros((N, H + 2, W + 2, C))
    xp[:, 1:-1, 1:-1] = x
    y = np.zeros_like(x)
    for i in range(3):
        for j in range(3):
            y += w[i, j] * xp[:, i:i + H, j:j + W]
    if b is not None:
        y = y + _f64(b)
    return y
