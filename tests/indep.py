"""Independent re-derivations used only to pin the oracle (never imported by it).

Two implementations of phi (Eq. 1, Eq. 2 with an E4M3 block scale):
  * ``phi_block_exact``: pure Python on ``fractions.Fraction`` -- every rounding
    decision is taken on exact rationals by nearest-value search with
    ties-to-even, no thresholds;
  * ``fake_quant_np``: vectorised numpy; the E4M3 grid comes from torch's own
    float8_e4m3fn decoder (a library table), decisions by ``searchsorted``.
and a row-at-a-time numpy transcription of the training forward (Alg. 2).

For the MX variant (E2M1, blocks of 32, power-of-two scale): ``phi_mx_block_exact`` on
rationals and ``fake_quant_mx_np``, whose scale exponent comes from ``numpy.frexp``.
"""
from fractions import Fraction

import numpy as np
import torch

E2M1 = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2),
        Fraction(2), Fraction(3), Fraction(4), Fraction(6)]


def e4m3_grid_torch():
    """All finite non-negative E4M3 values (bytes 0x00..0x7E) decoded by torch."""
    b = torch.arange(0, 0x7F, dtype=torch.uint8)
    return b.view(torch.float8_e4m3fn).to(torch.float64).numpy()


_E4M3_FR = None


def e4m3_grid_exact():
    global _E4M3_FR
    if _E4M3_FR is None:
        vals = []
        for byte in range(0x7F):
            e, m = byte >> 3, byte & 7
            if e == 0:
                vals.append(Fraction(m, 8) * Fraction(1, 64))
            else:
                vals.append((1 + Fraction(m, 8)) * (Fraction(2) ** (e - 7)))
        _E4M3_FR = vals
    return _E4M3_FR


def nearest_even_index(x: Fraction, grid) -> int:
    """Index of the grid value nearest to x; ties to the even index; saturating."""
    best, bi = None, 0
    for i, g in enumerate(grid):
        dist = abs(x - g)
        if best is None or dist < best or (dist == best and i % 2 == 0 and bi % 2 == 1):
            best, bi = dist, i
    return bi


def phi_block_exact(xs):
    """xs: list of python floats (<=16). Returns (codes, scale_byte, dequantized Fractions)."""
    fx = [Fraction(float(x)) for x in xs]
    amax = max(abs(f) for f in fx) if fx else Fraction(0)
    sb = nearest_even_index(amax / 6, e4m3_grid_exact())
    s = e4m3_grid_exact()[sb]
    codes, deq = [], []
    for x, f in zip(xs, fx):
        sign = 8 if np.signbit(np.float64(x)) else 0
        mag = nearest_even_index(abs(f) / s, E2M1) if s > 0 else 0
        codes.append(sign | mag)
        deq.append((-1 if sign else 1) * s * E2M1[mag])
    return codes, sb, deq


def fake_quant_np(x, axis=-1):
    """phi^-1(phi(x)) in float64 along ``axis`` in aligned blocks of 16 (zero padded)."""
    x = np.moveaxis(np.asarray(x, dtype=np.float64), axis, -1)
    n = x.shape[-1]
    pad = (-n) % 16
    xp = np.concatenate([x, np.zeros(x.shape[:-1] + (pad,))], axis=-1) if pad else x
    blk = xp.reshape(xp.shape[:-1] + (-1, 16))
    amax = np.abs(blk).max(axis=-1)
    grid = e4m3_grid_torch()
    mid6 = 6.0 * 0.5 * (grid[:-1] + grid[1:])             # exact in fp64
    lo = np.searchsorted(mid6, amax, side="left")          # # of midpoints < amax
    on_tie = (lo < mid6.size) & (mid6[np.minimum(lo, mid6.size - 1)] == amax)
    idx = np.where(on_tie & (lo % 2 == 1), lo + 1, lo)     # at a tie pick the even byte
    s = grid[idx][..., None]
    vals = np.array([0, .5, 1, 1.5, 2, 3, 4, 6.0])
    mids = 0.5 * (vals[:-1] + vals[1:])
    a = np.abs(blk)
    thr = mids[None, :] * s[..., None]                     # [..., 1, 7] exact products
    gt = (a[..., None] > thr).sum(-1)
    eq = (a[..., None] == thr)
    tie_idx = np.argmax(eq, axis=-1)
    has_tie = eq.any(-1)
    mag = np.where(has_tie, np.where(tie_idx % 2 == 1, tie_idx + 1, tie_idx), gt)
    mag = np.where(s > 0, mag, 0)
    out = np.sign(blk) * s * vals[mag]
    out = out.reshape(xp.shape)[..., :n]
    return np.moveaxis(out, -1, axis)


def phi_mx_block_exact(xs):
    """xs: list of python floats (<=32).  Returns (codes, scale exponent, dequantized Fractions).
    The scale is the smallest power of two s >= 2^-126 with 6 s >= max|x|, found on rationals
    from the bit lengths of numerator and denominator."""
    fx = [Fraction(float(x)) for x in xs]
    amax = max(abs(f) for f in fx) if fx else Fraction(0)
    if amax == 0:
        e = -126
    else:
        t = amax / 6                                   # want the smallest e with 2^e >= t
        e = t.numerator.bit_length() - t.denominator.bit_length()      # 2^(e-1) < t < 2^(e+1)
        if Fraction(2) ** (e - 1) >= t:
            e -= 1
        elif Fraction(2) ** e < t:
            e += 1
        e = max(e, -126)
    s = Fraction(2) ** e
    codes, deq = [], []
    for x, f in zip(xs, fx):
        sign = 8 if np.signbit(np.float64(x)) else 0
        mag = nearest_even_index(abs(f) / s, E2M1)
        codes.append(sign | mag)
        deq.append((-1 if sign else 1) * s * E2M1[mag])
    return codes, e, deq


def fake_quant_mx_np(x, axis=-1):
    """MX phi^-1(phi(x)) in float64 along ``axis`` in aligned blocks of 32 (zero padded).
    With amax = m 2^x, m in [0.5, 1) (frexp): 6 * 2^e >= amax first holds at e = x - 3 for
    m <= 0.75 and at e = x - 2 above."""
    x = np.moveaxis(np.asarray(x, dtype=np.float64), axis, -1)
    n = x.shape[-1]
    pad = (-n) % 32
    xp = np.concatenate([x, np.zeros(x.shape[:-1] + (pad,))], axis=-1) if pad else x
    blk = xp.reshape(xp.shape[:-1] + (-1, 32))
    amax = np.abs(blk).max(axis=-1)
    m, ex = np.frexp(amax)
    e = np.where(amax > 0, ex - 3 + (m > 0.75), -126)
    e = np.maximum(e, -126)
    s = np.ldexp(1.0, e)[..., None]
    vals = np.array([0, .5, 1, 1.5, 2, 3, 4, 6.0])
    r = np.abs(blk) / s                                    # exact: division by a power of two
    lo = np.floor(r * 2) / 2                               # E2M1 grid is a subset of the half-integers
    idx = np.searchsorted(vals, np.minimum(r, 6.0), side="right") - 1      # largest grid value <= r
    up = np.minimum(idx + 1, 7)
    dlo, dup = r - vals[idx], vals[up] - r
    pick_up = (dup < dlo) | ((dup == dlo) & (up % 2 == 0) & (up != idx))
    mag = np.where(pick_up, up, idx)
    del lo
    out = np.sign(blk) * s * vals[mag]
    out = out.reshape(xp.shape)[..., :n]
    return np.moveaxis(out, -1, axis)


def fake_quant_mx8_np(x, axis=-1):
    """MXFP8 phi^-1(phi(x)) in float64 along ``axis`` (E4M3 elements, aligned blocks of 32, zero padded).
    Scale: with amax = m 2^x, m in [0.5, 1) (frexp) and 448 = 0.875 * 2^9, 448 * 2^e >= amax first holds at
    e = x - 9 for m <= 0.875 and at e = x - 8 above.  Elements: torch's own float32 -> float8_e4m3fn cast
    (round to nearest even) of the exactly scaled values, which never exceed 448."""
    x = np.moveaxis(np.asarray(x, dtype=np.float64), axis, -1)
    n = x.shape[-1]
    pad = (-n) % 32
    xp = np.concatenate([x, np.zeros(x.shape[:-1] + (pad,))], axis=-1) if pad else x
    blk = xp.reshape(xp.shape[:-1] + (-1, 32))
    amax = np.abs(blk).max(axis=-1)
    m, ex = np.frexp(amax)
    e = np.where(amax > 0, ex - 9 + (m > 0.875), -126)
    e = np.maximum(e, -126)
    s = np.ldexp(1.0, e)[..., None]
    r = (blk / s).astype(np.float32)                       # exact: power-of-two scaling of fp32 inputs, |r| <= 448
    q = torch.from_numpy(np.ascontiguousarray(r)).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    out = (q * s).reshape(xp.shape)[..., :n]
    return np.moveaxis(out, -1, axis)


def fake_quant_two_level_np(p, axis=-1, span=64):
    """Two-level quantization of P along ``axis`` (values >= 0): aligned groups of ``span`` are divided by a power-of-two
    row factor s1 = smallest 2^k with 2688 * 2^k >= max(group max, 2^-24), NVFP4-quantized in blocks of 16, and
    multiplied back.  With base = m 2^x, m in [0.5, 1) (frexp) and 2688 = 0.65625 * 2^12: k = x - 12 for
    m <= 0.65625, else x - 11."""
    x = np.moveaxis(np.asarray(p, dtype=np.float64), axis, -1)
    n = x.shape[-1]
    pad = (-n) % span
    xp = np.concatenate([x, np.zeros(x.shape[:-1] + (pad,))], axis=-1) if pad else x
    grp = xp.reshape(xp.shape[:-1] + (-1, span))
    base = np.maximum(grp.max(axis=-1), 2.0 ** -24)
    m, ex = np.frexp(base)
    s1 = np.ldexp(1.0, ex - 12 + (m > 0.65625))[..., None]
    out = (fake_quant_np(grp / s1, axis=-1) * s1).reshape(xp.shape)[..., :n]
    return np.moveaxis(out, -1, axis)


def attn_fwd_rowwise_np(qf, kf, vf, causal, Bk, quant_p=True, fq=None):
    """Alg. 2, one query row at a time, numpy float64; inputs already fake-quantized.
    qf [L,d], kf/vf [L,d] (one head).  fq: the fake-quantizer of P-tilde (default: NVFP4).
    Returns O, O', Lse."""
    fq = fq or fake_quant_np
    L, d = qf.shape
    O = np.zeros((L, d)); Op = np.zeros((L, d)); Lse = np.zeros(L)
    for i in range(L):
        m, l = -np.inf, 0.0
        o = np.zeros(d); op = np.zeros(d)
        kend = i + 1 if causal else L
        for k0 in range(0, kend, Bk):
            k1 = min(k0 + Bk, kend)
            s = (kf[k0:k1] @ qf[i]) / np.sqrt(d)
            mnew = max(m, s.max())
            alpha = 0.0 if m == -np.inf else np.exp(m - mnew)
            pt = np.exp(s - mnew).astype(np.float32).astype(np.float64)
            pf = fq(pt) if quant_p else pt                 # blocks start at k0 (a multiple of the block)
            l = alpha * l + pt.sum()
            o = alpha * o + pf @ vf[k0:k1]
            op = alpha * op + pt @ vf[k0:k1]
            m = mnew
        O[i], Op[i], Lse[i] = o / l, op / l, m + np.log(l)
    return O, Op, Lse
