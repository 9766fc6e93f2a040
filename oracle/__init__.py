"""ctypes front end of the CPU oracle (``attnqat_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  It shares no code with the
HIP library and never imports it.

All tensors are numpy arrays; inputs are float32 (holding bf16-representable
values), outputs float64.  Citations are to the paper's sections, equations
and algorithms; see the C file's header for the readings taken.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attnqat_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

E2M1_VALUES = (0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0)


_LIB_SAN = os.path.join(_HERE, "liboracle_san.so")
# ATTNQAT_ORACLE_SANITIZED=1 (set by tests/test_oracle_sanitized.py for a child process that preloads the sanitizer
# runtime) makes this module load the build with AddressSanitizer and UndefinedBehaviorSanitizer instead.
_SANITIZED = os.environ.get("ATTNQAT_ORACLE_SANITIZED") == "1"


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Plain -O2: no fast-math, no reassociation."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def build_sanitized(force: bool = False) -> str:
    """The same source with -fsanitize=address,undefined (any finding aborts the process).  Host code only."""
    if force or not os.path.exists(_LIB_SAN) or os.path.getmtime(_LIB_SAN) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=all", "-shared", "-fPIC", "-o", _LIB_SAN, _SRC, "-lm"])
    return _LIB_SAN


_lib = None
_vp, _i, _l, _d = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_double


def _load():
    global _lib
    if _lib is not None:
        return _lib
    L = ctypes.CDLL(build_sanitized() if _SANITIZED else build())
    L.oracle_e2m1_value.restype = _d
    L.oracle_e2m1_value.argtypes = [_i]
    L.oracle_e4m3_value.restype = _d
    L.oracle_e4m3_value.argtypes = [_i]
    L.oracle_e4m3_from_amax.restype = _i
    L.oracle_e4m3_from_amax.argtypes = [_d]
    L.oracle_e2m1_round.restype = _i
    L.oracle_e2m1_round.argtypes = [_d, _d]
    L.oracle_phi.restype = _i
    L.oracle_phi.argtypes = [_vp, _l, _i, _i, _vp, _vp, _vp]
    L.oracle_fwd_rows.restype = _i
    L.oracle_fwd_rows.argtypes = [_vp, _vp, _vp, _i, _i, _i, _l, _i, _i, _i, _i, _i,
                                  _l, _vp, _vp, _vp, _vp, _vp]
    L.oracle_e8m0_from_amax.restype = _i
    L.oracle_e8m0_from_amax.argtypes = [_d]
    L.oracle_phi_mx.restype = _i
    L.oracle_phi_mx.argtypes = [_vp, _l, _l, _vp, _vp, _vp]
    L.oracle_e8m0_from_amax_fp8.restype = _i
    L.oracle_e8m0_from_amax_fp8.argtypes = [_d]
    L.oracle_e4m3_round.restype = _i
    L.oracle_e4m3_round.argtypes = [_d, _d]
    L.oracle_phi_mx8.restype = _i
    L.oracle_phi_mx8.argtypes = [_vp, _l, _l, _vp, _vp, _vp]
    L.oracle_two_level_s1.restype = _d
    L.oracle_two_level_s1.argtypes = [_d]
    L.oracle_fwd_rows_masked.restype = _i
    L.oracle_fwd_rows_masked.argtypes = [_vp, _vp, _vp, _i, _i, _i, _l, _i, _i, _i, _i, _i,
                                         _l, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i]
    L.oracle_bwd.restype = _i
    L.oracle_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _l, _i, _i, _i, _i,
                             _vp, _vp, _vp]
    L.oracle_bwd_dq_rows.restype = _i
    L.oracle_bwd_dq_rows.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _l, _i, _i, _i, _i,
                                     _l, _vp, _vp, _vp, _vp]
    L.oracle_bwd_dkdv_keys.restype = _i
    L.oracle_bwd_dkdv_keys.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _l, _i, _i, _i, _i,
                                       _i, _i, _l, _vp, _vp, _vp, _vp, _vp, _vp]
    L.oracle_bwd_rows_dkdv.restype = _i
    L.oracle_bwd_rows_dkdv.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _l, _i, _i, _i, _i,
                                       _l, _vp, _vp, _vp, _vp, _vp]
    L.oracle_num_threads.restype = _i
    _lib = L
    return L


def _p(a):
    return None if a is None else a.ctypes.data


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    return _load().oracle_num_threads()


# ---------------------------------------------------------------- formats

def e2m1_value(code: int) -> float:
    return _load().oracle_e2m1_value(code)


def e4m3_value(byte: int) -> float:
    return _load().oracle_e4m3_value(byte)


def e4m3_from_amax(amax: float) -> int:
    """Byte of RNE_E4M3(amax/6), saturating at 448 (Eq. 1 with an E4M3 scale)."""
    return _load().oracle_e4m3_from_amax(float(amax))


def e2m1_round(ax: float, s: float) -> int:
    """Magnitude index of RNE_E2M1(ax/s), saturating at 6 (Eq. 1)."""
    return _load().oracle_e2m1_round(float(ax), float(s))


def phi(x, scale_mode: int = 0):
    """phi and phi^-1 along the last axis in blocks of 16 (Eq. 1, Eq. 2).

    Returns (packed codes uint8 [..., d/2], E4M3 scale bytes uint8 [..., d/16],
    dequantized float32 [..., d])."""
    x = _f32(x)
    d = x.shape[-1]
    n = x.size // d
    packed = np.empty(x.shape[:-1] + (d // 2,), np.uint8)
    scales = np.empty(x.shape[:-1] + (d // 16,), np.uint8)
    xf = np.empty_like(x)
    rc = _load().oracle_phi(_p(x), n, d, scale_mode, _p(packed), _p(scales), _p(xf))
    if rc:
        raise ValueError(f"oracle_phi failed ({rc})")
    return packed, scales, xf


def fake_quant(x, scale_mode: int = 0):
    """phi^-1(phi(x)) along the last axis."""
    return phi(x, scale_mode)[2]


# ---------------------------------------------------------------- MX format

def e8m0_from_amax(amax: float) -> int:
    """E8M0 byte of the smallest power of two s >= 2^-126 with 6 s >= amax."""
    return _load().oracle_e8m0_from_amax(float(amax))


def phi_mx(x):
    """MX phi and phi^-1 along the last axis in blocks of 32 (a short last block is zero padded).

    Returns (packed codes uint8 [..., nb*16], E8M0 scale bytes uint8 [..., nb],
    dequantized float32 [..., n]) with nb = ceil(n/32)."""
    x = _f32(x)
    n = x.shape[-1]
    nb = (n + 31) // 32
    rows = x.size // n
    packed = np.empty(x.shape[:-1] + (nb * 16,), np.uint8)
    scales = np.empty(x.shape[:-1] + (nb,), np.uint8)
    xf = np.empty_like(x)
    rc = _load().oracle_phi_mx(_p(x), rows, n, _p(packed), _p(scales), _p(xf))
    if rc:
        raise ValueError(f"oracle_phi_mx failed ({rc})")
    return packed, scales, xf


def fake_quant_mx(x, axis: int = -1):
    """MX phi^-1(phi(x)) with the blocks of 32 running along `axis`."""
    xt = np.ascontiguousarray(np.moveaxis(_f32(x), axis, -1))
    return np.ascontiguousarray(np.moveaxis(phi_mx(xt)[2], -1, axis))


def e8m0_from_amax_fp8(amax: float) -> int:
    """E8M0 byte of the smallest power of two s >= 2^-126 with 448 s >= amax."""
    return _load().oracle_e8m0_from_amax_fp8(float(amax))


def e4m3_round(ax: float, s: float) -> int:
    """E4M3 byte of RNE_E4M3(ax/s), ax >= 0, saturating at 448."""
    return _load().oracle_e4m3_round(float(ax), float(s))


def phi_mx8(x):
    """MXFP8 phi and phi^-1 (E4M3 elements, blocks of 32 along the last axis, E8M0 scale).
    Returns (E4M3 bytes uint8 [..., nb*32], E8M0 scale bytes uint8 [..., nb], dequantized float32 [..., n])."""
    x = _f32(x)
    n = x.shape[-1]
    nb = (n + 31) // 32
    rows = x.size // n
    codes = np.empty(x.shape[:-1] + (nb * 32,), np.uint8)
    scales = np.empty(x.shape[:-1] + (nb,), np.uint8)
    xf = np.empty_like(x)
    rc = _load().oracle_phi_mx8(_p(x), rows, n, _p(codes), _p(scales), _p(xf))
    if rc:
        raise ValueError(f"oracle_phi_mx8 failed ({rc})")
    return codes, scales, xf


def fake_quant_mx8(x, axis: int = -1):
    """MXFP8 phi^-1(phi(x)) with the blocks of 32 running along `axis`."""
    xt = np.ascontiguousarray(np.moveaxis(_f32(x), axis, -1))
    return np.ascontiguousarray(np.moveaxis(phi_mx8(xt)[2], -1, axis))


def fwd_mx(q, k, v, causal: bool, Bk: int, quant_p: bool = True, rows=None, dump_p: bool = False):
    """Alg. 1 / Alg. 2 in the MX format: Q^F, K^F blocked along d, V^F and P-tilde^F along the keys.
    Same outputs as fwd()."""
    return fwd(q, k, v, causal, Bk, quant_p=quant_p, scale_mode=MX, rows=rows, dump_p=dump_p)


# ---------------------------------------------------------------- K smoothing

def two_level_s1(rowmax: float) -> float:
    """Row factor of the two-level quantization of P: the smallest power of two s1 with 2688 s1 >= max(rowmax, 2^-24)."""
    return _load().oracle_two_level_s1(float(rowmax))


def smooth_k(k):
    """K minus its mean over the tokens, per (batch, kv head, channel): the K smoothing of SageAttention that
    Sec. 2.1 describes and Sec. 3.2 switches on inside QAT.  S changes by a per-query constant, which softmax
    ignores, and the centred K quantizes better.  Mean = fp64 sum / L rounded to fp32; the subtraction is an fp32
    subtraction.  Callers pass the result to fwd()/bwd() in place of K.  Gradient: dK = dK' - mean_j(dK'_j), and
    sum_j dK'_j = sum_i rowsum(dS_i) Q^F_i = 0 because D comes from O' (Sec. 2.3), so dK = dK'."""
    k = _f32(k)
    mean = (k.astype(np.float64).sum(axis=-2, keepdims=True) / k.shape[-2]).astype(np.float32)
    return k - mean


# ---------------------------------------------------------------- attention

MX = 2      # scale_mode of the MX format: E2M1 blocks of 32 with E8M0 scales, V and P blocked along the keys
TWO_LEVEL_P = 4  # NVFP4 with SageAttention3's two-level quantization of P (row factor, then blocks of 16); Bk = 64
MX_FP8PV = 3    # mixed recipe: Q, K as in MX (FP4), V and P in MXFP8 (E4M3 elements, same blocks and scale format)
BF16_PV = 5     # mixed recipe of Sec. 2.5: Q, K in NVFP4, P-tilde rounded to bf16, V left in bf16 (inference only)


def _prep_qkv(q, k, v, quant_qkv, scale_mode):
    q, k, v = _f32(q), _f32(k), _f32(v)
    if quant_qkv and scale_mode == MX:
        q, k, v = fake_quant_mx(q), fake_quant_mx(k), fake_quant_mx(v, axis=-2)
    elif quant_qkv and scale_mode == MX_FP8PV:
        q, k, v = fake_quant_mx(q), fake_quant_mx(k), fake_quant_mx8(v, axis=-2)
    elif quant_qkv and scale_mode == BF16_PV:
        q, k = fake_quant(q), fake_quant(k)
    elif quant_qkv:    # Alg. 2 first line: Q^F, K^F, V^F (the two-level option only concerns P)
        sm = 0 if scale_mode == TWO_LEVEL_P else scale_mode
        q, k, v = fake_quant(q, sm), fake_quant(k, sm), fake_quant(v, sm)
    return q, k, v


def flat_rows(B, Hq, L, rows):
    """rows: iterable of (b, h, i) -> flat ids."""
    return np.asarray([(b * Hq + h) * L + i for (b, h, i) in rows], dtype=np.int64)


def fwd(q, k, v, causal: bool, Bk: int, quant_qkv: bool = True, quant_p: bool = True,
        scale_mode: int = 0, rows=None, dump_p: bool = False, block_mask=None, mask_block=(128, 128)):
    """Alg. 2 (training forward; Alg. 1's O and L are the same numbers).

    q [B,Hq,L,d], k/v [B,Hkv,L,d].  rows: None (all rows; outputs shaped
    [B,Hq,L,...]) or an int64 array of flat ids (outputs shaped [n,...]).
    Returns dict(O, Op, L[, P]) in float64 (P float32 [n, L])."""
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    qf, kf, vf = _prep_qkv(q, k, v, quant_qkv, scale_mode)
    if rows is None:
        n, shp, rp = B * Hq * L, (B, Hq, L), None
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        n, shp, rp = rows.size, (rows.size,), rows
    O = np.empty(shp + (d,)); Op = np.empty(shp + (d,)); Lse = np.empty(shp)
    P = np.empty((n, L), np.float32) if dump_p else None
    if block_mask is None:
        rc = _load().oracle_fwd_rows(_p(qf), _p(kf), _p(vf), B, Hq, Hkv, L, d, int(causal), Bk,
                                     int(quant_p), scale_mode, n, _p(rp),
                                     _p(O), _p(Op), _p(Lse), _p(P))
    else:
        # block-sparse attention: block_mask uint8 [B,Hq,ceil(L/bq),ceil(L/bk)], zero = the block is left out
        bq, bk = mask_block
        bm = np.ascontiguousarray(block_mask, dtype=np.uint8)
        assert bm.shape == (B, Hq, (L + bq - 1) // bq, (L + bk - 1) // bk), bm.shape
        rc = _load().oracle_fwd_rows_masked(_p(qf), _p(kf), _p(vf), B, Hq, Hkv, L, d, int(causal), Bk,
                                            int(quant_p), scale_mode, n, _p(rp),
                                            _p(O), _p(Op), _p(Lse), _p(P), _p(bm), bq, bk)
    if rc:
        raise ValueError(f"oracle_fwd_rows failed ({rc})")
    out = {"O": O, "Op": Op, "L": Lse}
    if dump_p:
        out["P"] = P
    return out


def bwd(q, k, v, do, Lse, Op, causal: bool, quant_qkv: bool = True, quant_p: bool = True,
        scale_mode: int = 0):
    """Alg. 3 on the whole problem.  Lse, Op: the forward's L and O'.
    Returns dict(dQ, dK, dV) float64."""
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    qf, kf, vf = _prep_qkv(q, k, v, quant_qkv, scale_mode)
    do, Lse, Op = _f32(do), _f64(Lse), _f64(Op)
    dQ = np.empty((B, Hq, L, d)); dK = np.empty((B, Hkv, L, d)); dV = np.empty((B, Hkv, L, d))
    rc = _load().oracle_bwd(_p(qf), _p(kf), _p(vf), _p(do), _p(Lse), _p(Op),
                            B, Hq, Hkv, L, d, int(causal), int(quant_p), scale_mode,
                            _p(dQ), _p(dK), _p(dV))
    if rc:
        raise ValueError(f"oracle_bwd failed ({rc})")
    return {"dQ": dQ, "dK": dK, "dV": dV}


def bwd_dq_rows(q, k, v, do, rows, Lse_rows, Op_rows, causal: bool,
                quant_qkv: bool = True, quant_p: bool = True, scale_mode: int = 0):
    """dQ of Alg. 3 for listed query rows (flat ids); Lse_rows/Op_rows from fwd(rows=...)."""
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    qf, kf, vf = _prep_qkv(q, k, v, quant_qkv, scale_mode)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    do, Lse_rows, Op_rows = _f32(do), _f64(Lse_rows), _f64(Op_rows)
    dQ = np.empty((rows.size, d))
    rc = _load().oracle_bwd_dq_rows(_p(qf), _p(kf), _p(vf), _p(do), B, Hq, Hkv, L, d,
                                    int(causal), int(quant_p), scale_mode,
                                    rows.size, _p(rows), _p(Lse_rows), _p(Op_rows), _p(dQ))
    if rc:
        raise ValueError(f"oracle_bwd_dq_rows failed ({rc})")
    return dQ


def bwd_dkdv_keys(q, k, v, do, b, hk, keys, Lse_grp, Op_grp, causal: bool,
                  quant_qkv: bool = True, quant_p: bool = True, scale_mode: int = 0,
                  dump_p: bool = False):
    """dK, dV of Alg. 3 for listed key rows of kv head (b, hk).
    Lse_grp [G,L], Op_grp [G,L,d]: forward outputs of the G query heads of the group."""
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    qf, kf, vf = _prep_qkv(q, k, v, quant_qkv, scale_mode)
    keys = np.ascontiguousarray(keys, dtype=np.int64)
    do, Lse_grp, Op_grp = _f32(do), _f64(Lse_grp), _f64(Op_grp)
    assert Lse_grp.shape == (G, L) and Op_grp.shape == (G, L, d)
    dK = np.empty((keys.size, d)); dV = np.empty((keys.size, d))
    P = np.empty((keys.size, G, L), np.float32) if dump_p else None
    rc = _load().oracle_bwd_dkdv_keys(_p(qf), _p(kf), _p(vf), _p(do), B, Hq, Hkv, L, d,
                                      int(causal), int(quant_p), scale_mode, b, hk,
                                      keys.size, _p(keys), _p(Lse_grp), _p(Op_grp),
                                      _p(dK), _p(dV), _p(P))
    if rc:
        raise ValueError(f"oracle_bwd_dkdv_keys failed ({rc})")
    return (dK, dV, P) if dump_p else (dK, dV)


def bwd_rows_dkdv(q, k, v, do, rows, Lse_rows, Op_rows, causal: bool,
                  quant_qkv: bool = True, quant_p: bool = True, scale_mode: int = 0):
    """dK, dV of Alg. 3 with the sums over query rows restricted to ``rows`` (flat ids), for
    all keys.  Equals the full backward when dO is zero outside the listed rows (dS and
    dV are linear in dO).  Returns (dK, dV) float64 [B,Hkv,L,d]."""
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    qf, kf, vf = _prep_qkv(q, k, v, quant_qkv, scale_mode)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    do, Lse_rows, Op_rows = _f32(do), _f64(Lse_rows), _f64(Op_rows)
    dK = np.empty((B, Hkv, L, d)); dV = np.empty((B, Hkv, L, d))
    rc = _load().oracle_bwd_rows_dkdv(_p(qf), _p(kf), _p(vf), _p(do), B, Hq, Hkv, L, d,
                                      int(causal), int(quant_p), scale_mode,
                                      rows.size, _p(rows), _p(Lse_rows), _p(Op_rows), _p(dK), _p(dV))
    if rc:
        raise ValueError(f"oracle_bwd_rows_dkdv failed ({rc})")
    return dK, dV
