"""Seeded synthetic inputs for the RMSNorm forward workloads.

This module only *draws numbers*: a counter-based generator, a Box-Muller
transform, and a rounding of the drawn values to the storage dtype.  It holds
none of the normalisation arithmetic, so both the CPU oracle's tests and the
HIP path's tests/benchmark can take their inputs from here without sharing any
of the method's code.

Generator: value k of stream s under seed z is a pure function of (z, s, k):

    key  = mix64(z + GOLDEN * (s + 1))
    u64  = mix64(key + GOLDEN * (k + 1))

with mix64 the splitmix64 output finaliser (Steele, Lea & Flood 2014) and
GOLDEN = 0x9E3779B97F4A7C15.  Normals use Box-Muller on the pair of draws
(2k, 2k+1) in fp64.  Because each element depends only on its own index, any
sub-range of a tensor can be generated on its own (the full 16384 x 8192
workload is produced in row blocks) and the result does not depend on how the
range was cut.

The workloads follow the paper's evaluation protocol, which benchmarks random
tensors at fixed shapes (Section 7 "Experimental Evaluation" and the kernel
performance table); no dataset is involved.
"""
from __future__ import annotations

import numpy as np

# dtype codes used at the C ABI (same integers as include/rmsnorm.h)
FP32 = 0
FP16 = 1
BF16 = 2

DTYPE_NAMES = {FP32: "fp32", FP16: "fp16", BF16: "bf16"}
DTYPE_BYTES = {FP32: 4, FP16: 2, BF16: 2}

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 20


def _mix64(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def _key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        z = np.array([(int(seed) + int(_GOLDEN) * (int(stream) + 1)) & 0xFFFFFFFFFFFFFFFF],
                     dtype=np.uint64)
        return _mix64(z)[0]


def raw_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """Draws `count` 64-bit words with counters start .. start+count-1."""
    key = _key(seed, stream)
    with np.errstate(over="ignore"):
        k = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        return _mix64(key + _GOLDEN * k)


def uniform(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """Uniform draws in (0, 1], fp64, 53 random bits each."""
    r = raw_u64(seed, stream, start, count)
    return ((r >> np.uint64(11)).astype(np.float64) + 1.0) * (2.0 ** -53)


def normal(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """Standard normal draws (fp64); element k uses counters 2k and 2k+1."""
    out = np.empty(count, dtype=np.float64)
    for lo in range(0, count, _CHUNK):
        n = min(_CHUNK, count - lo)
        u = uniform(seed, stream, 2 * (start + lo), 2 * n)
        u1 = u[0::2]
        u2 = u[1::2]
        out[lo:lo + n] = np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * np.pi) * u2)
    return out


def to_storage(values: np.ndarray, dtype: int) -> np.ndarray:
    """Rounds fp64 values to the storage dtype.

    Returns a float32 array for FP32 and an array of uint16 bit patterns for
    FP16 / BF16.  The bit patterns that come out of here ARE the inputs; both
    the oracle and the GPU read these same bits.
    """
    v = np.asarray(values, dtype=np.float64)
    if dtype == FP32:
        return v.astype(np.float32)
    if dtype == FP16:
        v = np.clip(v, -65504.0, 65504.0)
        return v.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        b = v.astype(np.float32).view(np.uint32)
        b = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
        return b.astype(np.uint16)
    raise ValueError(f"unknown dtype code {dtype}")


def storage_to_f64(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Widens stored values to fp64 (exact); a convenience for building inputs."""
    if dtype == FP32:
        return np.asarray(bits, dtype=np.float32).astype(np.float64)
    if dtype == FP16:
        return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)) \
            .view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype code {dtype}")


def normal_matrix(seed: int, stream: int, M: int, N: int, dtype: int,
                  mean: float = 0.0, std: float = 1.0, row_start: int = 0) -> np.ndarray:
    """M x N draws of N(mean, std) rounded to `dtype`; rows row_start.. of the stream."""
    sample = to_storage(np.zeros(1), dtype)
    out = np.empty((M, N), dtype=sample.dtype)
    rows_per_block = max(1, _CHUNK // max(N, 1))
    for r0 in range(0, M, rows_per_block):
        r1 = min(M, r0 + rows_per_block)
        z = normal(seed, stream, (row_start + r0) * N, (r1 - r0) * N)
        out[r0:r1] = to_storage(mean + std * z, dtype).reshape(r1 - r0, N)
    return out


def uniform_vector(seed: int, stream: int, N: int, dtype: int, lo: float, hi: float) -> np.ndarray:
    return to_storage(lo + (hi - lo) * uniform(seed, stream, 0, N), dtype)


# ----------------------------------------------------------------------------
# The five workload recipes (stream ids: 16*cfg + {0: x, 1: w, 2..: structure})
# ----------------------------------------------------------------------------

def config1(seed: int = 0):
    """fp32, 64 x 1024, eps 1e-6, x ~ N(0,1), w ~ N(1,0.1)."""
    M, N = 64, 1024
    return dict(name="cfg1_fp32_64x1024", dtype=FP32, M=M, N=N, eps=1e-6,
                x=normal_matrix(seed, 16, M, N, FP32),
                w=normal_matrix(seed, 17, 1, N, FP32, 1.0, 0.1)[0])


def config2(seed: int = 0, M: int = 4096):
    """bf16, 4096 (batch 8 x seq 512) x 4096, eps 1e-6."""
    N = 4096
    return dict(name=f"cfg2_bf16_{M}x{N}", dtype=BF16, M=M, N=N, eps=1e-6,
                x=normal_matrix(seed, 32, M, N, BF16),
                w=normal_matrix(seed, 33, 1, N, BF16, 1.0, 0.1)[0])


def config3(seed: int = 0, M: int = 16384, row_start: int = 0):
    """bf16, 16384 x 8192, eps 1e-5: the bandwidth-roofline headline shape."""
    N = 8192
    return dict(name=f"cfg3_bf16_{M}x{N}", dtype=BF16, M=M, N=N, eps=1e-5,
                x=normal_matrix(seed, 48, M, N, BF16, row_start=row_start),
                w=normal_matrix(seed, 49, 1, N, BF16, 1.0, 0.1)[0])


CONFIG4_N = (768, 5120, 13824)


def config4(N: int, seed: int = 0, M: int = 8191):
    """fp16 shape sweep, M = 8191, N in {768, 5120, 13824}, eps 1e-6, w ~ U(0.5,1.5)."""
    sub = CONFIG4_N.index(N) if N in CONFIG4_N else 3
    return dict(name=f"cfg4_fp16_{M}x{N}", dtype=FP16, M=M, N=N, eps=1e-6,
                x=normal_matrix(seed, 64 + 4 * sub, M, N, FP16),
                w=uniform_vector(seed, 65 + 4 * sub, N, FP16, 0.5, 1.5))


def config5(seed: int = 0, M: int = 4096, N: int = 4096):
    """fp16 adversarial magnitudes, 4096 x 4096, eps 1e-6.

    Row i is N(0,1) scaled by 10**u_i with u_i ~ U(-4, 4), clamped to the fp16
    range.  The rows are ranked by a separate uniform draw: the lowest 1 % are
    set to all-zero, the next 1 % get one element (uniform column, uniform
    sign) overwritten with +/-60000, which fp16 represents exactly.
    """
    z = normal(seed, 80, 0, M * N).reshape(M, N)
    u = -4.0 + 8.0 * uniform(seed, 82, 0, M)
    x = to_storage(z * (10.0 ** u)[:, None], FP16)
    order = np.argsort(uniform(seed, 83, 0, M), kind="stable")
    k = int(round(0.01 * M))
    zero_rows = np.sort(order[:k])
    spike_rows = np.sort(order[k:2 * k])
    x[zero_rows, :] = 0
    cols = np.minimum((uniform(seed, 84, 0, M) * N).astype(np.int64), N - 1)
    neg = uniform(seed, 85, 0, M) <= 0.5
    spike = to_storage(np.where(neg, -60000.0, 60000.0), FP16)
    x[spike_rows, cols[spike_rows]] = spike[spike_rows]
    return dict(name=f"cfg5_fp16adv_{M}x{N}", dtype=FP16, M=M, N=N, eps=1e-6,
                x=x, w=normal_matrix(seed, 81, 1, N, FP16, 1.0, 0.1)[0],
                zero_rows=zero_rows, spike_rows=spike_rows, spike_cols=cols[spike_rows],
                log10_scale=u)


def random_case(seed: int, stream: int, M: int, N: int, dtype: int, eps: float = 1e-6):
    """Generic N(0,1) x with N(1,0.1) w at any shape (shape sweeps and edge cases)."""
    return dict(name=f"rand_{DTYPE_NAMES[dtype]}_{M}x{N}", dtype=dtype, M=M, N=N, eps=eps,
                x=normal_matrix(seed, stream, M, N, dtype),
                w=normal_matrix(seed, stream + 1, 1, N, dtype, 1.0, 0.1)[0])


RMSNORM_PAPER_SHAPES = ((4096, 4096), (8192, 4096), (8192, 8192))


def rmsnorm_paper_shape(which: int, seed: int = 0):
    """FP16 4096 x 4096, 8192 x 4096 or 8192 x 8192 (which = 0, 1, 2): the three RMSNorm rows
    of the paper's table "Kernel performance on H100"; x ~ N(0,1), w ~ N(1,0.1), eps 1e-6."""
    M, N = RMSNORM_PAPER_SHAPES[which]
    case = random_case(seed, 160 + 4 * which, M, N, FP16)
    case["name"] = f"paper_fp16_{M}x{N}"
    return case


def algorithmic_bytes(M: int, N: int, dtype: int) -> int:
    """HBM bytes one launch must move: read x once, write y once, read w once.

    Same bytes model as the throughput column of the paper's kernel performance
    table (2*M*N*sizeof(dtype) divided by the time reproduces its GB/s figures).
    """
    s = DTYPE_BYTES[dtype]
    return 2 * M * N * s + N * s


# ----------------------------------------------------------------------------
# Row softmax workloads (the paper's table lists 4096 x 4096 and 8192 x 8192, FP16)
# ----------------------------------------------------------------------------

def softmax_case(seed: int, stream: int, M: int, N: int, dtype: int, std: float = 1.0):
    """Logits x ~ N(0, std) at any shape."""
    return dict(name=f"softmax_{DTYPE_NAMES[dtype]}_{M}x{N}_std{std:g}", dtype=dtype, M=M, N=N,
                x=normal_matrix(seed, stream, M, N, dtype, 0.0, std))


def softmax_paper_shape(n: int, seed: int = 0):
    """FP16 n x n logits, N(0, 1): the two softmax rows of the paper's performance table."""
    return softmax_case(seed, 96 + (0 if n == 4096 else 2), n, n, FP16)


def softmax_bytes(M: int, N: int, dtype: int) -> int:
    """Read x once, write y once (the model behind the paper's GB/s column for softmax)."""
    return 2 * M * N * DTYPE_BYTES[dtype]


# ----------------------------------------------------------------------------
# LayerNorm workloads (the paper's table lists 4096 x 5120 and 8192 x 4096, FP16)
# ----------------------------------------------------------------------------

def layernorm_case(seed: int, stream: int, M: int, N: int, dtype: int, eps: float = 1e-5,
                   mean: float = 0.0, std: float = 1.0, bias: bool = True):
    """x ~ N(mean, std), w ~ N(1, 0.1), b ~ N(0, 0.1) (or no bias) at any shape."""
    return dict(name=f"layernorm_{DTYPE_NAMES[dtype]}_{M}x{N}", dtype=dtype, M=M, N=N, eps=eps,
                x=normal_matrix(seed, stream, M, N, dtype, mean, std),
                w=normal_matrix(seed, stream + 1, 1, N, dtype, 1.0, 0.1)[0],
                b=normal_matrix(seed, stream + 2, 1, N, dtype, 0.0, 0.1)[0] if bias else None)


def layernorm_paper_shape(which: int, seed: int = 0):
    """FP16 4096 x 5120 (which = 0) or 8192 x 4096 (which = 1): the paper's two LayerNorm rows."""
    M, N = ((4096, 5120), (8192, 4096))[which]
    return layernorm_case(seed, 112 + 4 * which, M, N, FP16)


def layernorm_bytes(M: int, N: int, dtype: int) -> int:
    """Read x once, write y once, read w and b once."""
    return (2 * M * N + 2 * N) * DTYPE_BYTES[dtype]


# ----------------------------------------------------------------------------
# Cross-entropy workloads (the paper's table lists 4096 x 32k and 8192 x 32k, FP16; its
# throughput column fixes "32k" as 32000 classes and the bytes as one read of the logits)
# ----------------------------------------------------------------------------

IGNORED_TARGET = -100


def crossentropy_case(seed: int, stream: int, M: int, N: int, dtype: int, std: float = 1.0,
                      ignore_every: int = 0):
    """Logits x ~ N(0, std), targets uniform over the N classes (stream + 1); with
    ignore_every = k, rows 0, k, 2k, ... carry the out-of-range target that marks an ignored row."""
    target = (raw_u64(seed, stream + 1, 0, M) % np.uint64(N)).astype(np.int64)
    if ignore_every:
        target[::ignore_every] = IGNORED_TARGET
    return dict(name=f"crossentropy_{DTYPE_NAMES[dtype]}_{M}x{N}_std{std:g}", dtype=dtype, M=M, N=N,
                x=normal_matrix(seed, stream, M, N, dtype, 0.0, std), target=target)


def crossentropy_paper_shape(which: int, seed: int = 0):
    """FP16 4096 x 32000 (which = 0) or 8192 x 32000 (which = 1): the paper's two cross_ent rows."""
    M = (4096, 8192)[which]
    return crossentropy_case(seed, 128 + 4 * which, M, 32000, FP16)


def crossentropy_bytes(M: int, N: int, dtype: int) -> int:
    """Read the logits once (the model behind the paper's GB/s column for cross_ent; the M
    targets and M losses, 12 bytes per row, are left out as the paper leaves them out)."""
    return M * N * DTYPE_BYTES[dtype]


# ----------------------------------------------------------------------------
# Row-sum workloads (the paper's table lists 8192 x 8192 and 16384 x 4096, FP16, for "reduce")
# ----------------------------------------------------------------------------

def rowsum_case(seed: int, stream: int, M: int, N: int, dtype: int, mean: float = 0.0,
                std: float = 1.0):
    """x ~ N(mean, std) at any shape."""
    return dict(name=f"rowsum_{DTYPE_NAMES[dtype]}_{M}x{N}", dtype=dtype, M=M, N=N,
                x=normal_matrix(seed, stream, M, N, dtype, mean, std))


def rowsum_paper_shape(which: int, seed: int = 0):
    """FP16 8192 x 8192 (which = 0) or 16384 x 4096 (which = 1): the paper's two reduce rows."""
    M, N = ((8192, 8192), (16384, 4096))[which]
    return rowsum_case(seed, 144 + 4 * which, M, N, FP16)


def rowsum_bytes(M: int, N: int, dtype: int) -> int:
    """Read x once (the model behind the paper's GB/s column for reduce; the M results, 4
    bytes per row, are left out: they change the figure by less than 0.1 %)."""
    return M * N * DTYPE_BYTES[dtype]
