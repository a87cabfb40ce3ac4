"""MI355X-native diagonal linear-recurrence scan (selective fwd/bwd, LTI complex-diagonal).

The product is the C-ABI library built from ``csrc/`` (``liblrnnx.so``); ``api``
is a thin ctypes binding with the same entry-point names.  Nothing here falls
back to a CPU path: calling an entry point without the built library raises.
"""
__all__ = ["api", "workloads"]
