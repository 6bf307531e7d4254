"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

import oracle
from paper_2401_06197_amd import binding as dcn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = 4096  # a nonzero, 16-byte aligned fake address; validation never dereferences it


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dcnv4.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dcnv4_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = dcn.load_library()
    names = declared_functions()
    assert "dcnv4_forward" in names and "dcnv4_backward" in names and len(names) >= 8
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(dcn.EXPORTS) == names


def fwd(lib, x=A, off=A, m=A, y=A, N=1, H=14, W=14, G=4, Cg=16, k=(3, 3), s=(1, 1), p=(1, 1), d=(1, 1),
        scale=1.0, dtype=0):
    return lib.dcnv4_forward(x, off, m, y, N, H, W, G, Cg, k[0], k[1], s[0], s[1], p[0], p[1], d[0], d[1],
                             scale, dtype, None)


def bwd(lib, ptrs=(A,) * 7, N=1, H=14, W=14, G=4, Cg=16, k=(3, 3), dtype=0):
    return lib.dcnv4_backward(*ptrs, N, H, W, G, Cg, k[0], k[1], 1, 1, 1, 1, 1, 1, 1.0, dtype, None)


def test_forward_argument_validation_happens_on_the_host():
    lib = dcn.load_library()
    assert fwd(lib, x=None) == 1 and fwd(lib, off=None) == 1 and fwd(lib, m=None) == 1 and fwd(lib, y=None) == 1
    assert fwd(lib, N=0) == 2 and fwd(lib, H=0) == 2 and fwd(lib, G=0) == 2 and fwd(lib, s=(0, 1)) == 2
    assert fwd(lib, p=(-1, 0)) == 2 and fwd(lib, d=(1, 0)) == 2
    assert fwd(lib, H=2, W=2, p=(0, 0)) == 2                     # 3x3 window does not fit
    assert fwd(lib, k=(7, 7), p=(3, 3)) == 3 and fwd(lib, k=(3, 5), p=(1, 2)) == 3 and fwd(lib, k=(2, 2)) == 3
    assert fwd(lib, k=(5, 5), p=(2, 2), Cg=8) == 3                # a 5x5 window needs groups of 16 channels or more
    assert fwd(lib, Cg=12) == 3 and fwd(lib, Cg=128) == 3 and fwd(lib, dtype=2) == 3
    assert fwd(lib, scale=float("nan")) == 3 and fwd(lib, scale=float("inf")) == 3
    assert fwd(lib, x=A + 8) == 4 and fwd(lib, y=A + 2) == 4 and fwd(lib, m=A + 4) == 4
    # one image too large for 32-bit byte offsets
    assert fwd(lib, H=8192, W=8192, G=16, Cg=16) == 3
    assert fwd(lib, H=1 << 22, W=1, G=1, Cg=16, p=(1, 1)) == 3


def test_backward_argument_validation_happens_on_the_host():
    lib = dcn.load_library()
    for i in range(7):
        ptrs = [A] * 7
        ptrs[i] = None
        assert bwd(lib, tuple(ptrs)) == 1
    ptrs = [A] * 7
    ptrs[4] = A + 4
    assert bwd(lib, tuple(ptrs)) == 4
    assert bwd(lib, k=(3, 5)) == 3
    assert bwd(lib, dtype=1, Cg=64) == 3                          # fp16 backward exists for Cg 8, 16 and 32 only
    assert bwd(lib, N=-1) == 2


def fwd_m(lib, x=A, om=A, y=A, N=1, H=14, W=14, G=4, Cg=16, k=(3, 3), dtype=0):
    return lib.dcnv4_forward_merged(x, om, y, N, H, W, G, Cg, k[0], k[1], 1, 1, 1, 1, 1, 1, 1.0, dtype, None)


def bwd_m(lib, ptrs=(A,) * 5, N=1, H=14, W=14, G=4, Cg=16, k=(3, 3), dtype=0):
    return lib.dcnv4_backward_merged(*ptrs, N, H, W, G, Cg, k[0], k[1], 1, 1, 1, 1, 1, 1, 1.0, dtype, None)


def test_merged_entry_points_validate_on_the_host_too():
    lib = dcn.load_library()
    assert fwd_m(lib, x=None) == 1 and fwd_m(lib, om=None) == 1 and fwd_m(lib, y=None) == 1
    assert fwd_m(lib, om=A + 8) == 4 and fwd_m(lib, N=0) == 2 and fwd_m(lib, k=(5, 5)) in (2, 3) and fwd_m(lib, Cg=12) == 3
    for i in range(5):
        ptrs = [A] * 5
        ptrs[i] = None
        assert bwd_m(lib, tuple(ptrs)) == 1
    ptrs = [A] * 5
    ptrs[4] = A + 4
    assert bwd_m(lib, tuple(ptrs)) == 4
    assert bwd_m(lib, dtype=1, Cg=64) == 3 and bwd_m(lib, H=0) == 2
    c2 = (64, 56, 56, 8, 16, 56, 56)
    assert dcn.dcnv4_forward_merged_algorithmic_bytes(*c2, dcn.DCNV4_F16) == 2 * 64 * 56 * 56 * (2 * 128 + 32 * 8)
    assert dcn.dcnv4_backward_merged_algorithmic_bytes(*c2, dcn.DCNV4_F32) == 4 * 64 * 56 * 56 * (3 * 128 + 64 * 8)


def test_linear_and_module_entry_points_validate_on_the_host():
    lib = dcn.load_library()
    lin = lambda x=A, w=A, b=None, y=A, P=100, K=64, Nout=32, dtype=0: lib.dcnv4_linear(x, w, b, y, P, K, Nout, dtype, None)
    assert lin(x=None) == 1 and lin(w=None) == 1 and lin(y=None) == 1
    assert lin(P=0) == 2 and lin(K=0) == 2 and lin(Nout=0) == 2
    assert lin(K=12) == 3 and lin(K=8, dtype=1) == 3 and lin(Nout=40) == 3 and lin(dtype=2) == 3
    assert lin(P=1 << 24, K=64) == 3                                 # x of 4 GiB: beyond 32-bit byte offsets
    assert lin(x=A + 8) == 4 and lin(w=A + 4) == 4 and lin(y=A + 2) == 4 and lin(b=A + 2) == 4

    def mod(x=A, w_in=A, w_om=A, w_out=A, w_dw=None, ws=A, ws_bytes=1 << 40, y=A, N=1, H=14, W=14, G=4, Cg=16, k=3, s=1, p=1, d=1, dtype=0):
        return lib.dcnv4_module_forward(x, w_in, None, w_dw, None, w_om, None, w_out, None, ws, ws_bytes, y, N, H, W, G, Cg, k, k,
                                        s, s, p, p, d, d, 1.0, dtype, None)
    assert mod(x=None) == 1 and mod(w_om=None) == 1 and mod(ws=None) == 1 and mod(y=None) == 1
    assert mod(w_in=None) == 1 and mod(w_out=None) == 1              # the projections come together
    assert mod(N=0) == 2 and mod(ws_bytes=1000) == 2
    assert mod(p=0) == 3 and mod(s=2) == 3 and mod(k=5, p=2) == 3 and mod(k=1, p=0) == 3 and mod(Cg=12) == 3
    assert mod(G=3, Cg=16) == 3                                      # C = 48: not a multiple of 32 output channels
    assert mod(ws=A + 8) == 4 and mod(w_dw=A + 4) == 4

    def mod_static(x=A, w_in=A, w_om=A, w_out=A, y=A, N=1, H=14, W=14, G=4, Cg=16, dtype=0):
        return lib.dcnv4_module_forward_static(x, w_in, None, None, None, w_om, None, w_out, None, y, N, H, W, G, Cg, 3, 3,
                                               1, 1, 1, 1, 1, 1, 1.0, dtype, None)
    assert mod_static(x=None) == 1 and mod_static(w_om=None) == 1 and mod_static(y=None) == 1 and mod_static(w_in=None) == 1
    assert mod_static(N=0) == 2 and mod_static(dtype=2) == 3
    assert mod_static(N=64, H=56, W=56, G=8) == 6                    # more workspace than the built-in buffer holds
    assert dcn.dcnv4_module_static_workspace_limit() == 32 << 20 and "scratch" in dcn.dcnv4_status_string(6)
    dwc = lambda x=A, w=A, b=None, y=A, N=1, H=8, W=8, C=64, dtype=0: lib.dcnv4_depthwise3x3(x, w, b, y, N, H, W, C, dtype, None)
    assert dwc(x=None) == 1 and dwc(w=None) == 1 and dwc(y=None) == 1 and dwc(H=0) == 2 and dwc(C=6) == 3 and dwc(dtype=3) == 3
    assert dwc(C=4, dtype=1) == 3 and dwc(N=1 << 12, H=256, W=256, C=64) == 3 and dwc(w=A + 8) == 4 and dwc(b=A + 4) == 4
    P, C, G = 64 * 56 * 56, 128, 8
    assert dcn.dcnv4_module_workspace_bytes(64, 56, 56, G, 16, dcn.DCNV4_F16, True) == 2 * P * G * 32
    assert dcn.dcnv4_module_workspace_bytes(64, 56, 56, G, 16, dcn.DCNV4_F16, False) == 2 * P * (G * 32 + 2 * C)
    assert dcn.dcnv4_module_workspace_bytes(64, 56, 56, G, 16, dcn.DCNV4_F16, True, True) == 2 * P * (G * 32 + C)
    assert dcn.dcnv4_module_workspace_bytes(0, 56, 56, G, 16, dcn.DCNV4_F16, False) == -1


def test_options():
    assert dcn.dcnv4_last_kernel_name(0) is None or dcn.dcnv4_last_kernel_name(0).startswith("dcnv4_fwd")
    for key, bad in (("fwd_cpt", 5), ("nonsense", 1), ("fwd_path", 4), ("bwd_path", 3), ("fwd_single", 3), ("wg_per_cu", 33), ("halo", 65), ("lds_kb", 4), ("fwd_threads", 100)):
        with pytest.raises(dcn.Dcnv4Error):
            dcn.dcnv4_set_option(key, bad)
    for key, ok in (("fwd_cpt", 8), ("fwd_path", 2), ("bwd_path", 2), ("halo", 10), ("lds_kb", 64), ("fwd_threads", 512), ("fwd_threads", 128), ("bwd_cpt", 4)):
        dcn.dcnv4_set_option(key, ok)
        dcn.dcnv4_set_option(key, 0)
    assert "aligned" in dcn.dcnv4_status_string(4) and dcn.dcnv4_status_string(0) == "ok"


@pytest.mark.parametrize("H,W,k,s,p,d", [(56, 56, 3, 1, 1, 1), (15, 14, 3, 2, 1, 1), (16, 13, 3, 1, 2, 2),
                                          (17, 19, 3, 3, 2, 2), (9, 9, 3, 1, 0, 1), (200, 336, 3, 1, 1, 1)])
def test_output_hw_matches_sliding_window_rule(H, W, k, s, p, d):
    assert dcn.dcnv4_output_hw(H, W, k, s, p, d) == oracle.output_hw(H, W, k, s, p, d)
    ho, wo = dcn.dcnv4_output_hw(H, W, k, s, p, d)
    # last window starts inside the padded image and the next one would not fit
    assert (ho - 1) * s + d * (k - 1) + 1 <= H + 2 * p < ho * s + d * (k - 1) + 1


def test_algorithmic_bytes_follow_the_ideal_memory_access_model():
    # Sec. 3.2: 2*H*W*C + 27*H*W*G values, each touched once
    assert dcn.dcnv4_forward_algorithmic_bytes(64, 56, 56, 8, 16, 56, 56, dcn.DCNV4_F16) == 189_464_576
    assert dcn.dcnv4_forward_algorithmic_bytes(64, 56, 56, 8, 16, 56, 56, dcn.DCNV4_F32) == 378_929_152
    assert dcn.dcnv4_forward_algorithmic_bytes(2, 200, 336, 16, 16, 200, 336, dcn.DCNV4_F16) == 253_747_200
    assert dcn.dcnv4_backward_algorithmic_bytes(64, 56, 56, 8, 16, 56, 56, dcn.DCNV4_F32) == 655_097_856
    N, H, W, G, Cg = 3, 10, 12, 2, 32
    assert dcn.dcnv4_forward_algorithmic_bytes(N, H, W, G, Cg, H, W, 0) == 4 * N * H * W * (2 * G * Cg + 27 * G)


def test_missing_library_is_an_error_not_a_fallback(monkeypatch):
    monkeypatch.setattr(dcn, "_lib", None)
    monkeypatch.setattr(dcn, "LIB_PATH", "/nonexistent/libdcnv4.so")
    with pytest.raises(ImportError):
        dcn.load_library()
