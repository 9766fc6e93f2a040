"""Seeded synthetic workloads shaped like the paper's diffusion and LLM attention calls.

This module only draws inputs (it contains none of the method's arithmetic) and
is the one piece of code that both the CPU oracle's tests and the HIP path's
tests/bench use.  Tensors come back as numpy ``uint16`` arrays holding bf16 bit
patterns in ``[B, H, L, d]`` layout; ``bf16_bits_to_f32`` widens them exactly.

Shapes follow the models the paper trains and serves (Sec. 3 "Experiments" and
the appendix "Detailed Training Setup"): Wan 2.1 1.3B at 480p (12 heads, d=128,
21x30x52 latent tokens), Wan 2.1 14B at 720p (40 heads, 21x45x80 tokens), and
GQA LLMs of the Qwen3-14B / Llama-3.1-70B class.  The paper's latents, prompts
and weights are not available; these seeded draws stand in for them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libsynthgen.so")

TENSOR_Q, TENSOR_K, TENSOR_V, TENSOR_DO = 1, 2, 3, 4


def build(force: bool = False) -> str:
    """Compile the generator with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.synth_fill_bf16.restype = ctypes.c_int
        _lib.synth_fill_bf16.argtypes = [
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_long, ctypes.c_int,
            ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int, ctypes.c_double,
            ctypes.c_int, ctypes.c_double, ctypes.c_int, ctypes.c_double]
    return _lib


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    L: int
    d: int
    causal: bool
    seed: int
    dist: str            # "normal" | "t3"
    scale: float
    k_outlier_channels: int = 0      # K only: channels multiplied by 20
    outlier_token_mod: int = 0       # Q,K,V: token l is x10 iff hash(seed,l) % mod == 0
    passes: str = "fwd+bwd"          # or "fwd_infer"

    @property
    def fwd_flops(self) -> float:
        f = 4.0 * self.B * self.Hq * float(self.L) ** 2 * self.d
        return f * (0.5 if self.causal else 1.0)

    @property
    def bwd_flops(self) -> float:
        return 2.5 * self.fwd_flops


# The five benchmark shapes (index 0 is the small case, index 3 the headline).
CONFIGS = [
    Workload("tiny_ref", 1, 2, 2, 256, 64, False, 0, "normal", 1.0),
    Workload("dit480p_infer", 2, 12, 12, 32760, 128, False, 1, "t3", 0.5, passes="fwd_infer"),
    Workload("llm4k_gqa", 4, 32, 8, 4096, 128, True, 2, "normal", 1.0, k_outlier_channels=4),
    Workload("dit720p_train", 1, 40, 40, 75600, 128, False, 3, "t3", 0.5, outlier_token_mod=100),
    Workload("llm32k_gqa", 1, 64, 8, 32768, 128, True, 4, "normal", 1.0, k_outlier_channels=8),
]


# Not a benchmark configuration: the shape on which Sec. 3.4 quotes its peak forward throughput on B200
# (b=1, s=32768, h=32, d=128), for a like-for-like context line of the inference forward.
CONTEXT = [
    Workload("paper_peak_fwd_shape", 1, 32, 32, 32768, 128, False, 5, "normal", 1.0, passes="fwd_infer"),
]


def by_name(name: str) -> Workload:
    for w in CONFIGS + CONTEXT:
        if w.name == name:
            return w
    raise KeyError(name)


def fill(B, H, L, d, seed, tensor_id, dist="normal", scale=1.0,
         n_chan=0, chan_mult=1.0, tok_mod=0, tok_mult=1.0) -> np.ndarray:
    """One seeded tensor, bf16 bits as uint16 ``[B,H,L,d]``."""
    out = np.empty((B, H, L, d), dtype=np.uint16)
    rc = _load().synth_fill_bf16(
        out.ctypes.data, B, H, L, d, seed, tensor_id, {"normal": 0, "t3": 1}[dist],
        float(scale), n_chan, float(chan_mult), tok_mod, float(tok_mult))
    if rc != 0:
        raise ValueError("synth_fill_bf16 rejected its arguments")
    return out


def make_inputs(w: Workload, with_do: bool = True) -> dict:
    """Q, K, V (and dO) for a workload, as bf16-bit uint16 arrays."""
    tm = w.outlier_token_mod
    q = fill(w.B, w.Hq, w.L, w.d, w.seed, TENSOR_Q, w.dist, w.scale, tok_mod=tm, tok_mult=10.0)
    k = fill(w.B, w.Hkv, w.L, w.d, w.seed, TENSOR_K, w.dist, w.scale,
             n_chan=w.k_outlier_channels, chan_mult=20.0, tok_mod=tm, tok_mult=10.0)
    v = fill(w.B, w.Hkv, w.L, w.d, w.seed, TENSOR_V, w.dist, w.scale, tok_mod=tm, tok_mult=10.0)
    out = {"q": q, "k": k, "v": v}
    if with_do:
        out["do"] = fill(w.B, w.Hq, w.L, w.d, w.seed, TENSOR_DO, w.dist, w.scale)
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even narrowing of float32 to bf16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)
