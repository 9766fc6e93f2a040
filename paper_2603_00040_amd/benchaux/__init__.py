"""Bench-only helpers (not part of the attention library): the 16-bit MFMA rate the GPU sustains on its own, and a copy
kernel of known size for calibrating the profiler's traffic counters."""
import ctypes
import os

import torch

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libattnqat_benchaux.so")
_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.benchaux_mfma_burn.restype = ctypes.c_int
        _lib.benchaux_mfma_burn.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        _lib.benchaux_copy.restype = ctypes.c_int
        _lib.benchaux_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    return _lib


def copy_calibration(gib: float = 1.0, launches: int = 3):
    """Runs the plain copy kernel on `gib` GiB `launches` times (reads and writes exactly that many bytes per launch) and
    returns (bytes per launch, ms of the last launch)."""
    lib = _load()
    n = int(gib * (1 << 30)) // 16 * 16
    src = torch.zeros(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(launches):
        e0.record()
        if lib.benchaux_copy(src.data_ptr(), dst.data_ptr(), n, st):
            raise RuntimeError("benchaux_copy failed")
        e1.record()
        torch.cuda.synchronize()
    return n, e0.elapsed_time(e1)


def mfma_sustained(rounds: int = 4, iters: int = 40000):
    """Returns (TFLOP/s, GHz): the rate of a loop of v_mfma_f32_32x32x16_f16 on register operands, two waves per SIMD on
    every CU, and the clock held meanwhile.  rounds: how many times the launch fills the chip."""
    lib = _load()
    ncu = torch.cuda.get_device_properties(0).multi_processor_count
    blocks = 2 * ncu * rounds
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    clk = torch.zeros(2 * blocks, dtype=torch.int64, device="cuda")
    st = torch.cuda.current_stream().cuda_stream

    def go(n):
        rc = lib.benchaux_mfma_burn(blocks, n, out.data_ptr(), clk.data_ptr(), st)
        if rc:
            raise RuntimeError(f"benchaux_mfma_burn failed ({rc})")
    go(max(1, iters // 8))                                # warm-up
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    go(iters)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    c = clk.cpu().numpy().reshape(blocks, 2).astype("float64")
    flops = blocks * 4.0 * iters * 16.0 * 32768.0
    return flops / (ms * 1e-3) / 1e12, float(c[:, 0].sum() / c[:, 1].sum()) * 0.1
