"""Bench-only helper (not part of the attention library): the 16-bit MFMA rate the GPU sustains on its own."""
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
    return _lib


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
