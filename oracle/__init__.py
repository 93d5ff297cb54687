"""CPU oracles (RMSNorm forward, row softmax, LayerNorm forward, row cross-entropy, row sum): test infrastructure, not part of the product.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It wraps oracle/rmsnorm_oracle.cpp, oracle/softmax_oracle.cpp and
oracle/layernorm_oracle.cpp and oracle/crossentropy_oracle.cpp
(plain C++17, fp64; each file stands alone) through ctypes on host numpy arrays
and imports nothing from the HIP package.
"""
from .binding import (FP32, FP16, BF16, build, decode, encode, hardware_threads,
                      rmsnorm_oracle, rmsnorm_oracle_rstd, softmax_oracle, layernorm_oracle, crossentropy_oracle, rowsum_oracle)

__all__ = ["FP32", "FP16", "BF16", "build", "decode", "encode", "hardware_threads",
           "rmsnorm_oracle", "rmsnorm_oracle_rstd", "softmax_oracle", "layernorm_oracle", "crossentropy_oracle", "rowsum_oracle"]
