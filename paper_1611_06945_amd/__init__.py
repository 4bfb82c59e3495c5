"""MI355X-native forward 2D convolution (fused bias + ReLU) behind a C ABI.

`workloads` holds shapes and seeded inputs; `binding` is the thin ctypes layer
over `libconvfwd.so` (built from `csrc/` by `build.py`).  The binding is loaded
lazily so that shape/input helpers import on machines without the library.
"""
__all__ = ["workloads", "binding", "build"]
