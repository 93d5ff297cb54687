"""MI355X-native row-wise RMSNorm forward (hand-written HIP for gfx950).

`binding` holds the Python face of the C ABI declared in include/rmsnorm.h,
`softmax`, `layernorm`, `crossentropy` and `rowsum` those of include/softmax.h,
include/layernorm.h, include/crossentropy.h and include/rowsum.h (the next row kernels),
`inputs` the seeded synthetic workloads, `build` the hipcc build step.  The
HIP library is loaded on first use, so importing the package (or `inputs`
alone) needs neither a GPU nor the built library.
"""
from . import inputs  # noqa: F401

__all__ = ["inputs", "binding", "softmax", "layernorm", "crossentropy", "rowsum", "build"]
