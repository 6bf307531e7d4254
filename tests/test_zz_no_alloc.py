"""The module forward for callers that cannot allocate (dcnv4_module_forward_static: workspace in a buffer
built into the library) against dcnv4_module_forward with a caller-owned workspace, through the C ABI:
the same kernels on the same inputs, so the outputs must be identical bit for bit.  Two calls in a row on
the shared buffer, the second with a smaller input, then a call that is too large for the buffer."""
import numpy as np
import pytest
import torch

from paper_2401_06197_amd import binding as dcn
from paper_2401_06197_amd.synth import Config, make_inputs, make_module_params

pytestmark = pytest.mark.gpu

TORCH_DT = {"f32": torch.float32, "f16": torch.float16}


def both_ways(cfg, dtype, lightweight, depthwise, seed):
    x = torch.from_numpy(make_inputs(cfg, dtype, seed=seed)["x"]).cuda()
    prm = {k: torch.from_numpy(np.ascontiguousarray(v)).cuda()
           for k, v in make_module_params(cfg, dtype, seed=seed, lightweight=lightweight, depthwise=depthwise).items()}
    kw = dict(w_in=prm.get("w_in"), b_in=prm.get("b_in"), w_out=prm.get("w_out"), b_out=prm.get("b_out"),
              w_dw=prm.get("w_dw"), b_dw=prm.get("b_dw"), kernel=cfg.kernel, stride=cfg.stride, pad=cfg.pad,
              dilation=cfg.dilation, offset_scale=cfg.offset_scale)
    ref = dcn.dcnv4_module_forward(x, prm["w_om_padded"], prm["b_om_padded"], cfg.G, **kw)
    out = torch.full_like(x, 7.0)
    got = dcn.dcnv4_module_forward_static(x, prm["w_om_padded"], prm["b_om_padded"], cfg.G, out, **kw)
    torch.cuda.synchronize()
    assert got.data_ptr() == out.data_ptr()
    assert torch.isfinite(got.float()).all()
    assert torch.equal(got, ref), f"{cfg.name}: {(got.float() - ref.float()).abs().max().item()}"
    return got


def test_static_workspace_module_forward_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    big = Config("na_big", N=2, H=24, W=30, C=64, G=4)
    small = Config("na_small", N=1, H=9, W=11, C=32, G=2, pad=2, dilation=2)
    first = both_ways(big, "f16", lightweight=False, depthwise=True, seed=3).clone()
    both_ways(small, "f32", lightweight=True, depthwise=False, seed=4)          # smaller, on the buffer the first call left
    again = both_ways(big, "f16", lightweight=False, depthwise=True, seed=3)    # and the first once more
    assert torch.equal(first, again)


def test_static_workspace_module_forward_refuses_what_does_not_fit():
    cfg = Config("na_huge", N=64, H=56, W=56, C=128, G=8)
    assert dcn.dcnv4_module_workspace_bytes(cfg.N, cfg.H, cfg.W, cfg.G, cfg.Cg, dcn.DCNV4_F16, False) > \
        dcn.dcnv4_module_static_workspace_limit() == 32 << 20
    x = torch.zeros((cfg.N, cfg.H, cfg.W, cfg.C), dtype=torch.float16, device="cuda")
    prm = {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in make_module_params(cfg, "f16").items()}
    out = torch.full_like(x, 7.0)
    with pytest.raises(dcn.Dcnv4Error) as e:
        dcn.dcnv4_module_forward_static(x, prm["w_om_padded"], prm["b_om_padded"], cfg.G, out, w_in=prm["w_in"],
                                        b_in=prm["b_in"], w_out=prm["w_out"], b_out=prm["b_out"])
    assert e.value.status == 6 and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


def test_static_workspace_module_forward_replays_from_a_hip_graph():
    """What the entry point is for: under capture nothing may allocate.  (The first call on a device, which
    looks the buffer's address up, is made before the capture.)  Every replay, with new input values in the
    same buffers and eager work in between, must equal the eager call with a caller-owned workspace."""
    cfg = Config("na_graph", N=1, H=20, W=24, C=64, G=4)
    prm = {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in make_module_params(cfg, "f16", seed=5).items()}
    kw = dict(w_in=prm["w_in"], b_in=prm["b_in"], w_out=prm["w_out"], b_out=prm["b_out"])
    x = torch.from_numpy(make_inputs(cfg, "f16", seed=5)["x"]).cuda()
    out = torch.empty_like(x)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        dcn.dcnv4_module_forward_static(x, prm["w_om_padded"], prm["b_om_padded"], cfg.G, out, stream=s, **kw)
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        dcn.dcnv4_module_forward_static(x, prm["w_om_padded"], prm["b_om_padded"], cfg.G, out, stream=s, **kw)
    for rep in range(3):
        x.copy_(torch.from_numpy(make_inputs(cfg, "f16", seed=50 + rep)["x"]))
        out.fill_(3.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ref = dcn.dcnv4_module_forward(x, prm["w_om_padded"], prm["b_om_padded"], cfg.G, **kw)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), rep
