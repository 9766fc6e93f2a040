"""Helpers shared by the GPU parity tests (marshalling and error metrics only)."""
import numpy as np
import torch

import workloads as W


def to_dev(bits: np.ndarray) -> torch.Tensor:
    """bf16 bit patterns (uint16 numpy) -> bf16 CUDA tensor, bit exact."""
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def f32(bits: np.ndarray) -> np.ndarray:
    return W.bf16_bits_to_f32(bits)


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_l2(x, ref, zero_rms=0.0):
    """||x - ref|| / max(||ref||, zero_rms * sqrt(numel)).

    zero_rms is an absolute floor for references that are analytically zero (L = 1: P = 1
    and dP = D, so dQ = dK = 0 and only fp32 cancellation noise remains); inputs are O(1)."""
    x = np.asarray(x, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    den = max(np.linalg.norm(ref), zero_rms * np.sqrt(ref.size), 1e-300)
    return float(np.linalg.norm(x - ref) / den)


def max_abs(x, ref):
    return float(np.max(np.abs(np.asarray(x, dtype=np.float64) - np.asarray(ref, dtype=np.float64))))


def random_inputs(B, Hq, Hkv, L, d, seed, dist="normal", scale=1.0, k_chan=0, tok_mod=0):
    q = W.fill(B, Hq, L, d, seed, W.TENSOR_Q, dist, scale, tok_mod=tok_mod, tok_mult=10.0)
    k = W.fill(B, Hkv, L, d, seed, W.TENSOR_K, dist, scale, n_chan=k_chan, chan_mult=20.0,
               tok_mod=tok_mod, tok_mult=10.0)
    v = W.fill(B, Hkv, L, d, seed, W.TENSOR_V, dist, scale, tok_mod=tok_mod, tok_mult=10.0)
    do = W.fill(B, Hq, L, d, seed, W.TENSOR_DO, dist, scale)
    return {"q": q, "k": k, "v": v, "do": do}
