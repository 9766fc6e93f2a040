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


def bf16_rne(x):
    """x (float64) rounded to the nearest bf16 value (ties to even), returned as float64."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    return W.bf16_bits_to_f32(W.f32_to_bf16_bits(x32)).astype(np.float64)


def bf16_spacing(x):
    """Distance between neighbouring bf16 values at the magnitude of x (float64 array; 8 significant bits)."""
    a = np.maximum(np.abs(np.asarray(x, dtype=np.float64)), 2.0 ** -126)
    return np.exp2(np.floor(np.log2(a)) - 7)


# Bars on what is left of the error once the rounding of the output to bf16 is taken out (see bf16_output_error).
# O and dV come from exactly representable operands (only P-tilde in fp16 and the softmax arithmetic are rounded); dQ and dK
# contain dS rounded to fp16 (11 bits), summed with cancellation over all keys / queries.
# Measured: O <= 2.6e-5, dV 0, dQ and dK <= 1.3e-4 (small cases and sampled rows / all keys of the full-size shapes).
EXCESS_BAR = {"O": 1.0e-4, "dV": 1.0e-4, "dQ": 4.0e-4, "dK": 4.0e-4}
MAX_ULP_BAR = 1.0          # largest error, in bf16 spacings at the largest magnitude of the tensor (0.5 = output rounding alone)


def bf16_output_error(got, ref):
    """Error of a bf16 output tensor against fp64 reference values, with the output rounding taken out.

    Rounding a result to bf16 alone costs about 1.65e-3 relative L2, which hides kernel errors of up to about 1e-3
    under the 2e-3 bar.  These figures do not have that floor:
      excess       || max(0, |got - ref| - half a bf16 spacing at ref) || / ||ref||: zero for a kernel that is exact up to
                   its output rounding; a kernel whose fp32 result is off by a relative e lands on the wrong neighbour
                   for about e * 2^7.5 of the elements and exceeds the half spacing there by up to e |ref|, so this
                   grows like e^1.5 (about 4e-5 at e = 3e-4, 1.2e-4 at 6e-4, 1e-3 at 2.5e-3).
      off_nearest  the fraction of such elements (either neighbour counts on a tie); counts small elements like
                   large ones, so it depends on the spread of magnitudes inside the tensor.  Printed.
      max_ulp      largest |got - ref| in units of the bf16 spacing at the tensor's largest magnitude (0.5 from the
                   output rounding alone)."""
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    den = max(np.linalg.norm(ref), 1e-300)
    top = float(np.abs(ref).max())
    err = np.abs(got - ref)
    # half a spacing, taken at the magnitude of the larger of the two so that a reference just below a power of two may
    # round up to it; the 2^-10 slack accepts both neighbours of a tie
    half = 0.5 * np.maximum(bf16_spacing(ref), bf16_spacing(got)) * (1.0 + 2.0 ** -10)
    over = np.maximum(err - half, 0.0)
    return {"rel": float(np.linalg.norm(got - ref) / den), "excess": float(np.linalg.norm(over) / den),
            "off_nearest": float((over > 0).mean()), "max_abs": float(err.max()),
            "max_ulp": float(err.max() / bf16_spacing(top)) if top > 0 else 0.0}


def fmt_err(e):
    return (f"rel-L2 {e['rel']:.2e}, beyond output rounding {e['excess']:.2e} (off-nearest {e['off_nearest']:.4f}), "
            f"max-abs {e['max_abs']:.2e} = {e['max_ulp']:.2f} bf16 spacings of the largest")


def check_bf16_output(name, got, ref, tol=2e-3, kind=None, zero_rms=0.0, label=""):
    """The parity bar for a bf16 output: rel-L2 <= tol against the fp64 reference, and, unless the reference is
    (analytically) zero, the bar that sees the kernel's own error and the bound on the largest element error."""
    kind = kind or name
    e = bf16_output_error(got, ref)
    rel = rel_l2(got, ref, zero_rms)
    print(f"    {label}{name}: {fmt_err(e)}", flush=True)
    assert rel <= tol, (name, rel)
    if np.linalg.norm(ref) > zero_rms * np.sqrt(np.asarray(ref).size):
        assert e["excess"] <= EXCESS_BAR[kind], (name, e)
        assert e["max_ulp"] <= MAX_ULP_BAR, (name, e)
    return e


def random_inputs(B, Hq, Hkv, L, d, seed, dist="normal", scale=1.0, k_chan=0, tok_mod=0):
    q = W.fill(B, Hq, L, d, seed, W.TENSOR_Q, dist, scale, tok_mod=tok_mod, tok_mult=10.0)
    k = W.fill(B, Hkv, L, d, seed, W.TENSOR_K, dist, scale, n_chan=k_chan, chan_mult=20.0,
               tok_mod=tok_mod, tok_mult=10.0)
    v = W.fill(B, Hkv, L, d, seed, W.TENSOR_V, dist, scale, tok_mod=tok_mod, tok_mult=10.0)
    do = W.fill(B, Hq, L, d, seed, W.TENSOR_DO, dist, scale)
    return {"q": q, "k": k, "v": v, "do": do}
