"""Seeded synthetic inputs for the DCNv4 operator (shapes of the benchmark configs).

This module holds no arithmetic of the operator itself: it only draws random tensors
of the right shapes on the CPU, so that the HIP path and the CPU checker can be fed
identical values.  Recipe (one torch CPU generator per call, draw order fixed):
  x ~ N(0,1) [N,H,W,C];  offset = sigma * N(0,1) [N,Ho,Wo,G,K,2];  mask ~ N(0,1)
  [N,Ho,Wo,G,K] (unnormalised);  grad_y ~ N(0,1) [N,Ho,Wo,C];  then a Bernoulli(1/8)
  draw per (n,h,w,g,k) selects offset pairs that are rounded to whole numbers, so some
  samples land exactly on pixel centres.  For an fp16 run every tensor is rounded to
  fp16 once, here, so both consumers see the same already-rounded values.
These stand in for InternImage / FlashInternImage stage feature maps at 224x224 input
(4x..32x downsampling) and for a detection-sized feature map; no dataset is involved.
"""
from dataclasses import dataclass, asdict

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    name: str
    N: int
    H: int
    W: int
    C: int
    G: int
    sigma: float = 2.0          # std of the raw offsets, in pixels
    kernel: int = 3
    stride: int = 1
    pad: int = 1
    dilation: int = 1
    offset_scale: float = 1.0

    @property
    def Cg(self):
        return self.C // self.G

    @property
    def out_hw(self):
        k, s, p, d = self.kernel, self.stride, self.pad, self.dilation
        return ((self.H + 2 * p - d * (k - 1) - 1) // s + 1,
                (self.W + 2 * p - d * (k - 1) - 1) // s + 1)

    def with_(self, **kw):
        d = asdict(self)
        d.update(kw)
        return Config(**d)


CONFIGS = {
    # tiny forward+backward case
    "c1": Config("c1", N=1, H=14, W=14, C=64, G=4),
    # InternImage stage-1 shape (forward fp32/fp16; with grad_y it is the training-step case)
    "c2": Config("c2", N=64, H=56, W=56, C=128, G=8),
    # stage sweep
    "c3_28": Config("c3_28", N=64, H=28, W=28, C=256, G=16),
    "c3_14": Config("c3_14", N=64, H=14, W=14, C=512, G=32),
    "c3_7": Config("c3_7", N=64, H=7, W=7, C=1024, G=64),
    # dense-prediction high-resolution shape, wider offsets
    "c4": Config("c4", N=2, H=200, W=336, C=256, G=16, sigma=4.0),
}
CONFIGS["c5"] = CONFIGS["c2"].with_(name="c5")

# The paper's own op-level benchmark shapes (Sec. 4.1, Tab. 2 and 3): 32 channels per group,
# batch 64 for the standard shapes and batch 1 for the high-resolution ones.  Not benchmark
# configs of this repository; kept so that a like-for-like line can be measured beside the
# paper's A100 numbers.
for _n, _h, _w, _c in ((64, 56, 56, 128), (64, 28, 28, 256), (64, 14, 14, 512), (64, 7, 7, 1024), (64, 14, 14, 768),
                       (1, 200, 320, 128), (1, 100, 160, 256), (1, 50, 80, 512), (1, 25, 40, 1024), (1, 64, 64, 768)):
    CONFIGS[f"paper_{_h}x{_w}x{_c}"] = Config(f"paper_{_h}x{_w}x{_c}", N=_n, H=_h, W=_w, C=_c, G=_c // 32)


def make_inputs(cfg: Config, dtype: str = "f32", seed: int = 0, integer_fraction: float = 0.125):
    """Return dict(x, offset, mask, grad_y) of numpy arrays in `dtype` ('f32' or 'f16')."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    K = cfg.kernel * cfg.kernel
    Ho, Wo = cfg.out_hw
    x = torch.randn((cfg.N, cfg.H, cfg.W, cfg.C), generator=gen, dtype=torch.float32)
    off = torch.randn((cfg.N, Ho, Wo, cfg.G, K, 2), generator=gen, dtype=torch.float32) * cfg.sigma
    m = torch.randn((cfg.N, Ho, Wo, cfg.G, K), generator=gen, dtype=torch.float32)
    gy = torch.randn((cfg.N, Ho, Wo, cfg.C), generator=gen, dtype=torch.float32)
    if integer_fraction > 0:
        pick = torch.rand((cfg.N, Ho, Wo, cfg.G, K), generator=gen) < integer_fraction
        off = torch.where(pick[..., None], torch.round(off), off)
    out = {"x": x, "offset": off, "mask": m, "grad_y": gy}
    np_dtype = {"f32": np.float32, "f16": np.float16}[dtype]
    return {k: v.numpy().astype(np_dtype) for k, v in out.items()}


def merge_offset_mask(offset, mask, pad_value=0.0):
    """Pack offset [N,Ho,Wo,G,9,2] and mask [N,Ho,Wo,G,9] into one [N,Ho,Wo,G,32] array: 18 offsets,
    9 mask values, 5 entries of pad_value (what one linear layer with 32 outputs per group would
    hand over; the operator must ignore the last five)."""
    N, Ho, Wo, G, K = mask.shape
    om = np.full((N, Ho, Wo, G, 32), pad_value, dtype=mask.dtype)
    om[..., :2 * K] = offset.reshape(N, Ho, Wo, G, 2 * K)
    om[..., 2 * K:3 * K] = mask
    return om


def make_module_params(cfg: Config, dtype: str = "f32", seed: int = 0, lightweight: bool = False, pad_value: float = 0.0,
                       depthwise: bool = False):
    """Seeded random weights of the module's linear layers (numpy, `dtype`), sized so that with x ~ N(0,1)
    the predicted offsets have a standard deviation of about cfg.sigma pixels and the modulation scalars
    and projected values of about 1 -- the distributions of the operator-level inputs above:
      w_om [G*27, C] / b_om [G*27]: per group 18 offset rows, then 9 scalar rows (what the single layer
      of the module has); w_om_padded [G*32, C] / b_om_padded [G*32]: the same rows in the 32-entry
      layout, the five padding rows filled with pad_value (their outputs must be ignored);
      w_in, b_in, w_out, b_out [C, C] / [C] unless lightweight; with depthwise also w_dw [3,3,C] ~ N(0, 1/9)
      (so the convolved map keeps unit variance) and b_dw [C]."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed + 7919)
    C, G = cfg.C, cfg.G
    K = cfg.kernel * cfg.kernel
    scale = torch.cat([torch.full((2 * K,), cfg.sigma), torch.ones(K)]).repeat(G)[:, None] / float(np.sqrt(C))
    w_om = torch.randn((G * 3 * K, C), generator=gen) * scale
    b_om = 0.1 * torch.randn((G * 3 * K,), generator=gen)
    out = {"w_om": w_om, "b_om": b_om}
    if not lightweight:
        for name in ("in", "out"):
            out["w_" + name] = torch.randn((C, C), generator=gen) / float(np.sqrt(C))
            out["b_" + name] = 0.1 * torch.randn((C,), generator=gen)
    if depthwise:
        out["w_dw"] = torch.randn((3, 3, C), generator=gen) / 3.0
        out["b_dw"] = 0.1 * torch.randn((C,), generator=gen)
    np_dtype = {"f32": np.float32, "f16": np.float16}[dtype]
    out = {k: v.numpy().astype(np_dtype) for k, v in out.items()}
    wp = np.full((G, 32, C), pad_value, dtype=np_dtype)
    bp = np.full((G, 32), pad_value, dtype=np_dtype)
    wp[:, :3 * K] = out["w_om"].reshape(G, 3 * K, C)
    bp[:, :3 * K] = out["b_om"].reshape(G, 3 * K)
    out["w_om_padded"], out["b_om_padded"] = wp.reshape(G * 32, C), bp.reshape(G * 32)
    return out
