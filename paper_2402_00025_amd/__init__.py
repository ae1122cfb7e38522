"""MI355X-native fused W4A16 skinny GEMM (SplitK and data-parallel kernels).

`binding` wraps the C ABI of libw4a16.so (include/w4a16.h); `inputs` draws the seeded
synthetic workloads; `build` compiles the HIP sources for gfx950.
"""
from . import inputs  # noqa: F401

__all__ = ["inputs", "binding", "build"]
