"""MI355X-native sampled-SGD step for FastTucker-style sparse Tucker decomposition.

`binding` wraps the C ABI of libftk.so (include/ftk.h); `synth` draws the synthetic
workloads; `build` compiles the HIP library in-tree.  Nothing here computes on the CPU.
"""
from . import synth  # noqa: F401
from .binding import FastTucker, FtkError, load  # noqa: F401
