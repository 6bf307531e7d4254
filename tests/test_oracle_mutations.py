"""Mutation check of the oracle's pins (CPU only): every planted mistake in a temporary copy of
oracle/dcnv4_oracle.c -- a swapped operand, a dropped term, a wrong sign or index -- must make
tests/test_oracle_pins.py fail.  The tracked oracle is never touched: the copy is patched and
compiled in a temporary directory, and the pins run against it in a child process."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "dcnv4_oracle.c")

# (what is planted, text to find, replacement, occurrences to replace: 0 = all)
MUTATIONS = [
    ("forward reads the height offset where the width offset belongs",
     "const double dX = offset[(pg * K + k) * 2 + 0];", "const double dX = offset[(pg * K + k) * 2 + 1];", 1),
    ("tap order transposed everywhere", "const int k = j * kh + i;", "const int k = i * kw + j;", 0),
    ("tap order transposed in the forward only", "const int k = j * kh + i;", "const int k = i * kw + j;", 1),
    ("forward drops the lh*lw corner", "lh * lw * pixel(x, H, W, C, n, h0 + 1.0, w0 + 1.0, ch);", "0.0;", 1),
    ("padding added instead of subtracted", "(double)(oh * sh - ph + i * dh)", "(double)(oh * sh + ph + i * dh)", 0),
    ("dilation ignored along the width", "(double)(ow * sw - pw + j * dw)", "(double)(ow * sw - pw + j)", 0),
    ("offset_scale ignored along the width", "+ offset_scale * dX", "+ dX", 0),
    ("grad_offset stores the height derivative in the width slot",
     "grad_offset[(pg * K + k) * 2 + 0] = offset_scale * m * gdx;", "grad_offset[(pg * K + k) * 2 + 0] = offset_scale * m * gdy;", 1),
    ("height derivative interpolates with the wrong fraction",
     "(1.0 - lw) * (X10 - X00) + lw * (X11 - X01)", "(1.0 - lh) * (X10 - X00) + lh * (X11 - X01)", 1),
    ("grad_x row weights swapped", "(a ? lh : 1.0 - lh) * (b ? lw : 1.0 - lw)", "(a ? 1.0 - lh : lh) * (b ? lw : 1.0 - lw)", 1),
    ("grad_offset misses offset_scale", "= offset_scale * m * gdy;", "= m * gdy;", 1),
    ("grad_mask drops a corner", "lh * (1.0 - lw) * X10 + lh * lw * X11;", "lh * (1.0 - lw) * X10;", 1),
    ("backward ignores the stride",
     "\n                            const double hy = (double)(oh * sh - ph + i * dh)",
     "\n                            const double hy = (double)(oh - ph + i * dh)", 1),
    ("out-of-image samples clamp to the border instead of reading zero", "return 0.0;\n    return x[",
     "{ r = r < 0 ? 0 : (r > H-1 ? H-1 : r); q = q < 0 ? 0 : (q > W-1 ? W-1 : q);}\n    return x[", 1),
    ("output channels interleaved across groups instead of concatenated",
     "y[(pg / G) * C + ch] = acc;", "y[(pg / G) * C + (c * G + g)] = acc;", 1),
]


def _pins_fail_with(tmp, idx, old, new, count):
    text = open(SRC).read()
    if old not in text:
        return "pattern not found in the oracle source (update the mutation list)"
    text = text.replace(old, new, count) if count > 0 else text.replace(old, new)
    c_file = os.path.join(tmp, f"mutant_{idx}.c")
    so_file = os.path.join(tmp, f"libmutant_{idx}.so")
    with open(c_file, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-w", "-o", so_file,
                           c_file, "-lm"])
    env = dict(os.environ, DCNV4_ORACLE_LIB=so_file, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    if r.returncode == 0:
        return "the pins still pass"
    if " failed" not in r.stdout:
        return "the pins did not run to a failing assertion:\n" + r.stdout[-800:] + r.stderr[-800:]
    return None


def test_the_unmodified_copy_passes(tmp_path):
    """The harness itself: an unpatched copy, built the same way, passes every pin."""
    so_file = str(tmp_path / "libcopy.so")
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-w", "-o", so_file,
                           SRC, "-lm"])
    env = dict(os.environ, DCNV4_ORACLE_LIB=so_file, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-1500:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    with ThreadPoolExecutor(max_workers=4) as pool:
        futures = [pool.submit(_pins_fail_with, str(tmp_path), i, old, new, count)
                   for i, (_, old, new, count) in enumerate(MUTATIONS)]
        survivors = [f"{MUTATIONS[i][0]}: {f.result()}" for i, f in enumerate(futures) if f.result() is not None]
    assert not survivors, "\n".join(survivors)
    assert len(MUTATIONS) == 15
