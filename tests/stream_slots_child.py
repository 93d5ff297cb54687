"""Child process of tests/test_stream_slots_gpu.py: a fresh process, so that the libraries' tables
of stream slots start empty.  Creates 34 HIP streams of its own, runs RMSNorm and LayerNorm on
each at shapes where the automatic path takes the work-queue kernels, and checks what the headers
promise: the first 32 streams of a device get a block of counters (the forced variant runs),
later ones get none (the forced variant reports that it cannot run, the automatic path takes
another kernel), and every result has the bits of the kernels that need no counters.  Prints one
line per step and "ok" at the end; any failure raises."""
import ctypes
import sys

import torch

from paper_2603_21331_amd import binding, layernorm

EPS = 1e-5
STREAMS = 34
SLOTS = 32


def say(text):
    print(text, flush=True)


def loaded_hip_runtime():
    """Path of the HIP runtime this process already runs on (the streams must come from that one)."""
    paths = set()
    with open("/proc/self/maps") as f:
        for line in f:
            path = line.split()[-1]
            if "libamdhip64" in path:
                paths.add(path)
    assert len(paths) == 1, f"expected one HIP runtime in the process, found {sorted(paths)}"
    return paths.pop()


def main():
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    torch.zeros(1, device=dev)
    binding.load()
    layernorm.load()
    hip = ctypes.CDLL(loaded_hip_runtime())
    hip.hipStreamCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipStreamCreate.restype = ctypes.c_int
    hip.hipStreamDestroy.argtypes = [ctypes.c_void_p]
    hip.hipStreamDestroy.restype = ctypes.c_int

    gen = torch.Generator(device=dev).manual_seed(61)
    M, N = 6144, 8192                      # bf16, 96 MiB: RMSNorm's automatic path takes the queue
    x = torch.randn((M, N), generator=gen, device=dev).to(torch.bfloat16)
    w = (1.0 + 0.1 * torch.randn(N, generator=gen, device=dev)).to(torch.bfloat16)
    b = (0.1 * torch.randn(N, generator=gen, device=dev)).to(torch.bfloat16)
    LM, LN = 4096, 12288                   # bf16, 96 MiB of 24 KiB rows: LayerNorm's does too
    lx = torch.randn((LM, LN), generator=gen, device=dev).to(torch.bfloat16)
    lw = (1.0 + 0.1 * torch.randn(LN, generator=gen, device=dev)).to(torch.bfloat16)
    lb = (0.1 * torch.randn(LN, generator=gen, device=dev)).to(torch.bfloat16)
    assert binding.rmsnorm_queue_plan(M, N, binding.RMSNORM_DTYPE_BF16)[0]
    assert layernorm.layernorm_queue_plan(LM, LN, layernorm.LAYERNORM_DTYPE_BF16)[0]
    want_r = binding.rmsnorm_fwd_tuned(x, w, EPS, 512)
    want_l = layernorm.layernorm_fwd_tuned(lx, lw, lb, EPS, 512)
    torch.cuda.synchronize()

    handles = []
    for k in range(STREAMS):
        h = ctypes.c_void_p()
        rc = hip.hipStreamCreate(ctypes.byref(h))
        assert rc == 0 and h.value, f"hipStreamCreate: {rc}"
        handles.append(h)
    assert len({h.value for h in handles}) == STREAMS
    y = torch.empty_like(x)
    ly = torch.empty_like(lx)
    for k, h in enumerate(handles):
        s = torch.cuda.ExternalStream(h.value, device=dev)
        say(f"stream {k}")
        with torch.cuda.stream(s):
            for name, forced, auto, out, want, err, unsupported in (
                    ("rmsnorm", lambda: binding.rmsnorm_fwd_variant(x, w, EPS, binding.RMSNORM_VARIANT_QUEUE, y),
                     lambda: binding.rmsnorm_fwd(x, w, EPS, y), y, want_r, binding.RmsnormError,
                     binding.RMSNORM_ERR_UNSUPPORTED),
                    ("layernorm", lambda: layernorm.layernorm_fwd_variant(lx, lw, lb, EPS, layernorm.LAYERNORM_VARIANT_QUEUE, ly),
                     lambda: layernorm.layernorm_fwd(lx, lw, lb, EPS, ly), ly, want_l, layernorm.LayerNormError,
                     layernorm.LAYERNORM_ERR_UNSUPPORTED)):
                out.fill_(5.0)
                try:
                    forced()
                    ran = True
                except err as e:
                    assert e.status == unsupported, (name, k, e.status)
                    ran = False
                assert ran == (k < SLOTS), f"{name}: forced variant on stream {k}: ran={ran}"
                s.synchronize()
                if ran:
                    assert torch.equal(out.view(torch.int16), want.view(torch.int16)), f"{name} forced, stream {k}"
                out.fill_(5.0)
                auto()
                s.synchronize()
                assert torch.equal(out.view(torch.int16), want.view(torch.int16)), f"{name} auto, stream {k}"
    torch.cuda.synchronize()
    for h in handles:
        assert hip.hipStreamDestroy(h) == 0
    say("ok")
    return 0


if __name__ == "__main__":
    sys.exit(main())
