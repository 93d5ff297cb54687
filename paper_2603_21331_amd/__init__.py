"""MI355X-native row-wise RMSNorm forward (hand-written HIP for gfx950).

`binding` holds the Python face of the C ABI declared in include/rmsnorm.h,
`softmax` and `layernorm` those of include/softmax.h and include/layernorm.h (the next
reduce-then-scale kernels),
`inputs` the seeded synthetic workloads, `build` the hipcc build step.  The
HIP library is loaded on first use, so importing the package (or `inputs`
alone) needs neither a GPU nor the built library.
"""
from . import inputs  # noqa: F401

__all__ = ["inputs", "binding", "softmax", "layernorm", "build"]
