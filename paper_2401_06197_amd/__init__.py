"""MI355X-native DCNv4 spatial-aggregation operator (forward + backward) behind a C ABI.

`dcnv4_forward` / `dcnv4_backward` marshal arguments into libdcnv4.so (hand-written
HIP kernels for gfx950); every step of the operator runs in those kernels.  The
shared library is loaded on first use and a missing library is an error, never a
fallback.  `synth` draws the seeded benchmark inputs and touches neither the
library nor any arithmetic of the operator.
"""

__all__ = ["dcnv4_forward", "dcnv4_backward", "dcnv4_output_hw", "dcnv4_status_string", "load_library"]


def __getattr__(name):
    if name in __all__:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
