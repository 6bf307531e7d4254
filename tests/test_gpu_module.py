"""Parity of the module's linear layers (matrix-core kernel) and of the whole DCNv4 module forward with
the CPU oracle, through the C ABI.  The linear layer alone keeps the operator's tolerances (1e-5 fp32,
2e-2 fp16).  The module chains three layers: the offsets it predicts carry the rounding of their own
accumulation (about 1e-6 in fp32; in fp16 a value near a rounding boundary may land on the neighbouring
fp16 number, 0.004 pixels away at |offset| in [4, 8)), and a sample moves by that much times the local slope
of the image (values of order 1 per pixel, times |m|): the module's bars are 1e-4 (fp32) and 4e-2 (fp16),
with at least 99.9 % of the elements inside the operator's own tolerance."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_06197_amd import binding as dcn
from paper_2401_06197_amd.synth import CONFIGS, Config, make_inputs, make_module_params

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "f16": 2e-2}
MODULE_TOL = {"f32": 1e-4, "f16": 4e-2}
TORCH_DT = {"f32": torch.float32, "f16": torch.float16}
NP_DT = {"f32": np.float32, "f16": np.float16}


def close(name, got, ref, tol, bulk_tol=None):
    got = got.astype(np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    err = np.abs(got - ref)
    lim = tol + tol * np.abs(ref)
    bad = err > lim
    if bad.any():
        idx = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError(f"{name}: {int(bad.sum())} of {bad.size} outside tol {tol}; worst at {idx}: "
                             f"got {got[idx]!r} ref {ref[idx]!r}")
    if bulk_tol is not None:
        inside = np.mean(err <= bulk_tol + bulk_tol * np.abs(ref))
        assert inside >= 0.999, f"{name}: only {inside:.5f} of the elements inside {bulk_tol}"
    return float(err.max())


def gpu(a, dtype):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to("cuda", TORCH_DT[dtype])


LINEAR_CASES = [  # P, K, Nout
    (1, 16, 32), (37, 32, 32), (256, 64, 96), (300, 128, 128), (1000, 128, 384), (777, 256, 160), (513, 1024, 256),
    (3136, 768, 768), (64, 144, 32),
]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("P,K,Nout", LINEAR_CASES)
def test_linear_layer_matches_oracle(P, K, Nout, dtype):
    rng = np.random.default_rng(P * 7 + K + Nout)
    x = rng.standard_normal((P, K)).astype(NP_DT[dtype])
    w = (rng.standard_normal((Nout, K)) / np.sqrt(K)).astype(NP_DT[dtype])
    b = rng.standard_normal(Nout).astype(NP_DT[dtype])
    out = torch.full((P, Nout), 7.0, device="cuda", dtype=TORCH_DT[dtype])
    y = dcn.dcnv4_linear(gpu(x, dtype), gpu(w, dtype), gpu(b, dtype), out=out)
    torch.cuda.synchronize()
    close(f"linear {P}x{K}->{Nout} {dtype}", y.cpu().numpy(), oracle.linear(x, w, b), TOL[dtype])
    y0 = dcn.dcnv4_linear(gpu(x, dtype), gpu(w, dtype))                      # no bias
    torch.cuda.synchronize()
    close(f"linear {P}x{K}->{Nout} {dtype} (no bias)", y0.cpu().numpy(), oracle.linear(x, w), TOL[dtype])


def test_linear_layer_on_an_nhwc_map_and_its_refusals():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 5, 7, 64)).astype(np.float32)
    w = rng.standard_normal((32, 64)).astype(np.float32)
    y = dcn.dcnv4_linear(gpu(x, "f32"), gpu(w, "f32"))
    torch.cuda.synchronize()
    close("linear on a map", y.cpu().numpy(), oracle.linear(x, w), 1e-5)
    out = torch.full((4, 40), 7.0, device="cuda")
    for K, Nout in ((12, 32), (64, 40)):                                     # K*4 not a multiple of 32; Nout not of 32
        with pytest.raises(dcn.Dcnv4Error) as e:
            dcn.dcnv4_linear(torch.zeros((4, K), device="cuda"), torch.zeros((Nout, K), device="cuda"),
                             out=torch.full((4, Nout), 7.0, device="cuda") if Nout != 40 else out)
        assert e.value.status == 3
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


MODULE_CASES = [Config("m_small", N=2, H=9, W=11, C=64, G=4), Config("m_cg32", N=1, H=12, W=10, C=128, G=4),
                Config("m_ring", N=2, H=24, W=30, C=32, G=2), Config("m_dil", N=1, H=14, W=13, C=96, G=6, pad=2, dilation=2),
                Config("m_wide", N=1, H=7, W=7, C=1024, G=64, sigma=1.0), Config("m_cg8", N=3, H=6, W=7, C=32, G=4),
                Config("m_cg64", N=3, H=10, W=9, C=128, G=2)]


def run_module(cfg, dtype, lightweight, seed=0, depthwise=False):
    x = make_inputs(cfg, dtype, seed=seed)["x"]
    prm = make_module_params(cfg, dtype, seed=seed, lightweight=lightweight, pad_value=3.0, depthwise=depthwise)
    g = {k: gpu(v, dtype) for k, v in prm.items()}
    out = torch.full(x.shape, 7.0, device="cuda", dtype=TORCH_DT[dtype])
    kw = dict(kernel=cfg.kernel, stride=cfg.stride, pad=cfg.pad, dilation=cfg.dilation, offset_scale=cfg.offset_scale)
    y = dcn.dcnv4_module_forward(gpu(x, dtype), g["w_om_padded"], g["b_om_padded"], cfg.G, w_in=g.get("w_in"),
                                 b_in=g.get("b_in"), w_out=g.get("w_out"), b_out=g.get("b_out"), w_dw=g.get("w_dw"),
                                 b_dw=g.get("b_dw"), out=out, **kw)
    torch.cuda.synchronize()
    ref = oracle.module_forward(x, prm["w_om"], prm["b_om"], cfg.G, w_in=prm.get("w_in"), b_in=prm.get("b_in"),
                                w_out=prm.get("w_out"), b_out=prm.get("b_out"), w_dw=prm.get("w_dw"), b_dw=prm.get("b_dw"),
                                storage=NP_DT[dtype], **kw)
    return close(f"module {cfg.name} {dtype} light={lightweight} dw={depthwise}", y.cpu().numpy(), ref, MODULE_TOL[dtype], bulk_tol=TOL[dtype])


@pytest.mark.parametrize("lightweight", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("cfg", MODULE_CASES, ids=[c.name for c in MODULE_CASES])
def test_module_forward_matches_oracle(cfg, dtype, lightweight):
    run_module(cfg, dtype, lightweight)


@pytest.mark.parametrize("lightweight", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("cfg", MODULE_CASES[:4], ids=[c.name for c in MODULE_CASES[:4]])
def test_module_forward_with_the_depthwise_convolution(cfg, dtype, lightweight):
    run_module(cfg, dtype, lightweight, depthwise=True)


DW_CASES = [(1, 1, 1, 8), (2, 5, 7, 64), (1, 14, 14, 48), (3, 9, 4, 128), (1, 56, 56, 128), (2, 3, 33, 1024)]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("N,H,W,C", DW_CASES)
def test_depthwise_convolution_matches_oracle(N, H, W, C, dtype):
    rng = np.random.default_rng(N + H * 3 + W * 5 + C)
    x = rng.standard_normal((N, H, W, C)).astype(NP_DT[dtype])
    w = (rng.standard_normal((3, 3, C)) / 3.0).astype(NP_DT[dtype])
    b = rng.standard_normal(C).astype(NP_DT[dtype])
    out = torch.full((N, H, W, C), 7.0, device="cuda", dtype=TORCH_DT[dtype])
    y = dcn.dcnv4_depthwise3x3(gpu(x, dtype), gpu(w, dtype), gpu(b, dtype), out=out)
    torch.cuda.synchronize()
    close(f"depthwise {N}x{H}x{W}x{C} {dtype}", y.cpu().numpy(), oracle.depthwise3x3(x, w, b), TOL[dtype])
    y0 = dcn.dcnv4_depthwise3x3(gpu(x, dtype), gpu(w, dtype))
    torch.cuda.synchronize()
    close(f"depthwise {N}x{H}x{W}x{C} {dtype} (no bias)", y0.cpu().numpy(), oracle.depthwise3x3(x, w), TOL[dtype])


@pytest.mark.parametrize("depthwise", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("cfg", MODULE_CASES, ids=[c.name for c in MODULE_CASES])
def test_module_forward_with_channel_last_tensors_between_the_layers(cfg, dtype, depthwise):
    """By default the full module keeps its intermediate tensors plane-major (one (image, group) after the
    other); the switch "module_rows" keeps them channel-last.  Both must match the oracle."""
    if depthwise and cfg.name == "m_wide":
        pytest.skip("covered without the depthwise convolution")
    dcn.dcnv4_set_option("module_rows", 1)
    run_module(cfg, dtype, lightweight=False, depthwise=depthwise)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_module_forward_at_the_stage1_shape(dtype):
    """Full size of the headline workload (N64, 56x56, C128, G8), both projections."""
    run_module(CONFIGS["c2"], dtype, lightweight=False)


@pytest.mark.parametrize("name", ["paper_28x28x256", "paper_14x14x512", "paper_7x7x1024"])
@pytest.mark.parametrize("lightweight", [False, True])
def test_module_forward_at_the_papers_module_benchmark_shapes_fp16(name, lightweight):
    """Full size (batch 64, 32 channels per group), the shapes of the paper's module-level table."""
    run_module(CONFIGS[name], "f16", lightweight)


def test_linear_layer_on_random_shapes():
    """Seeded random (P, K, Nout) within the kernel's rules: K * element size a multiple of 32 bytes, Nout of 32."""
    rng = np.random.default_rng(77)
    for case in range(24):
        dtype = "f16" if case % 2 else "f32"
        kstep = 16 if dtype == "f16" else 8
        P = int(rng.integers(1, 700))
        K = int(rng.integers(1, 40)) * kstep
        Nout = int(rng.integers(1, 14)) * 32
        x = rng.standard_normal((P, K)).astype(NP_DT[dtype])
        w = (rng.standard_normal((Nout, K)) / np.sqrt(K)).astype(NP_DT[dtype])
        b = rng.standard_normal(Nout).astype(NP_DT[dtype]) if case % 3 else None
        y = dcn.dcnv4_linear(gpu(x, dtype), gpu(w, dtype), gpu(b, dtype))
        torch.cuda.synchronize()
        close(f"linear case {case}: {P}x{K}->{Nout} {dtype}", y.cpu().numpy(), oracle.linear(x, w, b), TOL[dtype])


def test_module_refusals_leave_y_untouched():
    cfg = Config("m_bad", N=1, H=8, W=8, C=64, G=4)
    x = gpu(make_inputs(cfg, "f32")["x"], "f32")
    prm = {k: gpu(v, "f32") for k, v in make_module_params(cfg, "f32", lightweight=True).items()}
    out = torch.full_like(x, 7.0)
    for kw, status in ((dict(pad=0), 3), (dict(stride=2), 3), (dict(kernel=5, pad=2), 3)):
        with pytest.raises(dcn.Dcnv4Error) as e:
            dcn.dcnv4_module_forward(x, prm["w_om_padded"], prm["b_om_padded"], cfg.G, out=out, **kw)
        assert e.value.status == status, kw
    with pytest.raises(dcn.Dcnv4Error) as e:                                   # workspace too small
        dcn.dcnv4_module_forward(x, prm["w_om_padded"], prm["b_om_padded"], cfg.G, out=out,
                                 workspace=torch.empty(1024, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 2
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
