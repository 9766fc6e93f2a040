"""Pins of the oracle's MX variant (E2M1 elements, blocks of 32, power-of-two E8M0 scale).

The format is the OCP microscaling FP4 named in Sec. 2.1 beside NVFP4; the scale rule is
the power-of-two counterpart of Eq. 1: the smallest 2^e with 6 * 2^e >= max|X|.  Pinned by
closed forms, an exact-rational twin, a numpy twin whose exponent comes from frexp, exact
invariants of a power-of-two scale, and for the forward the same pins as the NVFP4 path
(textbook attention with phi(P) off, an independent row-wise transcription with it on).
"""
import math

import numpy as np
import pytest

import oracle
from tests import indep


def _bf16(x):
    u = np.asarray(x, np.float32).view(np.uint32)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.view(np.float32)


def _rand(B, Hq, Hkv, L, d, seed, outlier=False):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, Hq, L, d)); k = rng.standard_normal((B, Hkv, L, d)); v = rng.standard_normal((B, Hkv, L, d))
    if outlier:
        k[..., 3] *= 6.0; q[..., 3] *= 2.0
    return _bf16(q), _bf16(k), _bf16(v)


def test_e8m0_hand_cases():
    # 6 * 2^e >= amax first holds at: amax = 6 -> e = 0; just above 6 -> 1; 3 -> -1; just above 3 -> 0;
    # 1 -> -2 (6/4 = 1.5 >= 1 > 0.75); 0.75 -> -3; 0 -> the floor -126
    cases = [(6.0, 0), (np.nextafter(6.0, 7.0), 1), (3.0, -1), (np.nextafter(3.0, 4.0), 0), (1.0, -2), (0.75, -3),
             (0.0, -126), (448.0, 7), (2.0 ** -140, -126), (6 * 2.0 ** 100, 100), (3.3e38, 126)]
    for amax, e in cases:
        assert oracle.e8m0_from_amax(amax) == e + 127, (amax, e)


def test_e8m0_matches_log2_closed_form_on_every_bf16_amax():
    # every positive finite bf16 value as a block maximum; ceil(log2(amax/6)) evaluated without rounding
    # issues through frexp: amax = m 2^x, m in [0.5, 1): e = x - 3 if m <= 0.75 else x - 2
    u = (np.arange(0x0080, 0x7F80, dtype=np.uint32) << 16).view(np.float32).astype(np.float64)
    m, x = np.frexp(u)
    want = np.maximum(x - 3 + (m > 0.75), -126) + 127
    got = np.array([oracle.e8m0_from_amax(a) for a in u])
    assert np.array_equal(got, want)
    s = np.ldexp(1.0, got - 127)
    big = got > 1
    assert (6 * s >= u).all() and (6 * (s[big] / 2) < u[big]).all()       # smallest such power of two


def test_phi_mx_matches_exact_rational_twin():
    rng = np.random.default_rng(5)
    for t in range(300):
        scale = 2.0 ** rng.integers(-20, 20)
        blk = _bf16(rng.standard_normal(32) * scale * (10.0 if t % 7 == 0 else 1.0))
        if t % 5 == 0:
            blk[rng.integers(0, 32, 8)] = 0.0
        packed, sb, xf = oracle.phi_mx(blk[None, :])
        codes, e, deq = indep.phi_mx_block_exact([float(v) for v in blk])
        got = [(int(packed[0, i // 2]) >> (4 * (i % 2))) & 15 for i in range(32)]
        assert sb[0, 0] == e + 127
        # -0.0 and +0.0 of a zero magnitude are the same number
        assert all(g == c or ((g & 7) == 0 and (c & 7) == 0) for g, c in zip(got, codes))
        assert np.array_equal(xf[0].astype(np.float64), np.array([float(v) for v in deq]))


def test_phi_mx_numpy_twin_on_gaussian_rows_and_both_axes():
    rng = np.random.default_rng(6)
    x = _bf16(rng.standard_normal((3, 70, 96)) * np.exp(rng.standard_normal((3, 70, 1))))
    assert np.array_equal(oracle.fake_quant_mx(x).astype(np.float64), indep.fake_quant_mx_np(x))
    # blocks along the second-to-last axis (how V is blocked), with a short last block (70 = 2*32 + 6)
    assert np.array_equal(oracle.fake_quant_mx(x, axis=-2).astype(np.float64), indep.fake_quant_mx_np(x, axis=-2))
    # and the two axes differ
    assert not np.array_equal(oracle.fake_quant_mx(x), oracle.fake_quant_mx(x, axis=-2))


def test_phi_mx_invariants():
    rng = np.random.default_rng(7)
    x = _bf16(rng.standard_normal((64, 128)))
    packed, sb, xf = oracle.phi_mx(x)
    s = np.ldexp(1.0, sb.astype(np.int64) - 127)
    blk = x.reshape(64, 4, 32).astype(np.float64); q = xf.reshape(64, 4, 32).astype(np.float64)
    # no element saturates, so the error is at most half the largest grid gap (2 s) ...
    assert (np.abs(blk - q) <= s[..., None]).all()
    # ... the maximum lands on 4 or 6 times the scale (amax / s in (3, 6]: at least 3, and 3 < amax/s rounds to >= 3)
    top = np.abs(q).max(-1) / s
    assert np.isin(top, [3.0, 4.0, 6.0]).all() and (top >= 3).all()
    # exact homogeneity under powers of two: same codes, shifted scale byte
    for kexp in (-9, 5):
        p2, sb2, xf2 = oracle.phi_mx(x * 2.0 ** kexp)
        assert np.array_equal(p2, packed) and np.array_equal(sb2.astype(int), sb.astype(int) + kexp)
        assert np.array_equal(xf2, xf * np.float32(2.0 ** kexp))
    # idempotent: quantized values are representable with the same or a finer scale
    assert np.array_equal(oracle.phi_mx(xf)[2], xf)
    # sign symmetry
    assert np.array_equal(oracle.phi_mx(-x)[2], -xf)


def test_phi_mx_round_trip_of_every_code_and_packing():
    vals = np.array([0, .5, 1, 1.5, 2, 3, 4, 6.0])
    codes = np.arange(32) % 16
    blk = np.where(codes & 8, -1.0, 1.0) * vals[codes & 7]
    for e in (-30, 0, 17):
        packed, sb, xf = oracle.phi_mx((blk * 2.0 ** e)[None, :].astype(np.float32))
        assert sb[0, 0] == 127 + e
        got = np.array([(int(packed[0, i // 2]) >> (4 * (i % 2))) & 15 for i in range(32)])
        assert np.array_equal(got & 7, codes & 7)
        nz = (codes & 7) != 0
        assert np.array_equal(got[nz], codes[nz])
        assert np.array_equal(xf[0], (blk * 2.0 ** e).astype(np.float32))
    # a block of zeros: the floor scale, all codes zero
    packed, sb, xf = oracle.phi_mx(np.zeros((1, 32), np.float32))
    assert sb[0, 0] == 1 and not packed.any() and not xf.any()


def test_e2m1_ties_go_to_even_under_a_power_of_two_scale():
    # midpoints of the grid times the scale; a 6 in the block pins the scale at 2^e
    mids = [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]
    even = [0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0]
    for e in (-3, 0, 4):
        blk = np.zeros(32, np.float32); blk[0] = 6.0 * 2.0 ** e
        blk[1:8] = np.array(mids) * 2.0 ** e
        xf = oracle.phi_mx(blk[None, :])[2][0]
        assert np.array_equal(xf[1:8], np.array(even, np.float32) * np.float32(2.0 ** e))


def _textbook(q, k, v, causal):
    d = q.shape[-1]
    s = q @ np.swapaxes(k, -1, -2) / math.sqrt(d)
    if causal:
        L = s.shape[-1]
        s = np.where(np.tril(np.ones((L, L), bool)), s, -np.inf)
    m = s.max(-1, keepdims=True)
    p = np.exp(s - m)
    return p @ v / p.sum(-1, keepdims=True), (m + np.log(p.sum(-1, keepdims=True)))[..., 0]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Bk", [32, 64])
def test_mx_forward_with_phi_p_off_is_textbook_attention_of_the_mx_inputs(causal, Bk):
    q, k, v = _rand(1, 2, 2, 150, 64, seed=21)
    r = oracle.fwd_mx(q, k, v, causal, Bk, quant_p=False)
    qf = indep.fake_quant_mx_np(q); kf = indep.fake_quant_mx_np(k); vf = indep.fake_quant_mx_np(v, axis=-2)
    O, L = _textbook(qf, kf, vf, causal)
    assert np.allclose(r["O"], O, rtol=0, atol=1e-6)          # fp32 rounding of P-tilde
    assert np.allclose(r["L"], L, rtol=0, atol=1e-6)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Bk", [32, 64])
def test_mx_forward_matches_independent_rowwise_transcription(causal, Bk):
    q, k, v = _rand(1, 2, 1, 200, 32, seed=22, outlier=True)
    r = oracle.fwd_mx(q, k, v, causal, Bk)
    qf = indep.fake_quant_mx_np(q); kf = indep.fake_quant_mx_np(k); vf = indep.fake_quant_mx_np(v, axis=-2)
    for h in range(2):
        O, Op, L = indep.attn_fwd_rowwise_np(qf[0, h], kf[0, 0], vf[0, 0], causal, Bk, fq=indep.fake_quant_mx_np)
        assert np.allclose(r["O"][0, h], O, rtol=0, atol=1e-12)
        assert np.allclose(r["Op"][0, h], Op, rtol=0, atol=1e-12)
        assert np.allclose(r["L"][0, h], L, rtol=0, atol=1e-12)


def test_mx_single_tile_closed_form_and_row_subset():
    q, k, v = _rand(1, 2, 2, 48, 32, seed=23)
    r = oracle.fwd_mx(q, k, v, False, 64)
    qf = indep.fake_quant_mx_np(q); kf = indep.fake_quant_mx_np(k); vf = indep.fake_quant_mx_np(v, axis=-2)
    for h in range(2):
        s = qf[0, h] @ kf[0, h].T / np.sqrt(32)
        pt = np.exp(s - s.max(-1, keepdims=True)).astype(np.float32).astype(np.float64)
        o = indep.fake_quant_mx_np(pt) @ vf[0, h] / pt.sum(-1, keepdims=True)
        assert np.allclose(r["O"][0, h], o, rtol=0, atol=1e-12)
    rows = oracle.flat_rows(1, 2, 48, [(0, 1, 47), (0, 0, 3)])
    sub = oracle.fwd_mx(q, k, v, False, 64, rows=rows, dump_p=True)
    assert np.array_equal(sub["O"][0], r["O"][0, 1, 47]) and np.array_equal(sub["O"][1], r["O"][0, 0, 3])
    # every dumped P-tilde^F value is (an E2M1 value) * 2^e with one e per block of 32 keys
    p = sub["P"][0].astype(np.float64)
    vals = np.array([0, .5, 1, 1.5, 2, 3, 4, 6.0])
    for b0 in (0, 32):
        blk = p[b0:b0 + 32]
        ok = False
        for e in range(-40, 4):
            if np.isin(blk / 2.0 ** e, vals).all():
                ok = True
        assert ok


def test_mx_and_nvfp4_forward_differ_at_quantization_noise_level():
    q, k, v = _rand(1, 1, 1, 256, 64, seed=24)
    a = oracle.fwd(q, k, v, False, 64)["O"]; b = oracle.fwd_mx(q, k, v, False, 64)["O"]
    ref, _ = _textbook(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), False)
    ea = np.linalg.norm(a - ref) / np.linalg.norm(ref); eb = np.linalg.norm(b - ref) / np.linalg.norm(ref)
    assert 1e-2 < ea < 0.5 and 1e-2 < eb < 0.5
    assert eb > 0.8 * ea        # coarser blocks and power-of-two scales do not beat NVFP4 by a margin


# ---------------------------------------------------------------- backward (Alg. 3) in the MX format

def _autograd_mx(q, k, v, do, causal):
    """torch autograd (fp64) through the unrolled MX fake-quant graph, straight-through at every
    phi^-1 phi: Q, K blocked along d, V and P blocked along the keys."""
    import torch

    def ste(x, axis):
        fq = torch.from_numpy(indep.fake_quant_mx_np(x.detach().numpy(), axis=axis))
        return x + (fq - x).detach()

    q, k, v, do = (torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True) for a in (q, k, v, do))
    G = q.shape[1] // k.shape[1]
    qf, kf, vf = ste(q, -1), ste(k, -1), ste(v, -2)
    kf = kf.repeat_interleave(G, dim=1); vf = vf.repeat_interleave(G, dim=1)
    s = qf @ kf.transpose(-1, -2) / np.sqrt(q.shape[-1])
    if causal:
        L = q.shape[2]
        s = s.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
    p = torch.softmax(s, -1)
    p32 = p.detach().to(torch.float32).to(torch.float64)
    pq = torch.from_numpy(indep.fake_quant_mx_np(p32.numpy(), axis=-1))
    p = p + (pq - p).detach()
    o = p @ vf
    (o * do.detach()).sum().backward()
    return q.grad.numpy(), k.grad.numpy(), v.grad.numpy()


@pytest.mark.parametrize("causal", [False, True])
def test_mx_backward_matches_autograd_of_unrolled_ste_graph(causal):
    q, k, v = _rand(1, 4, 2, 80, 32, seed=31, outlier=True)        # 80 = 2 * 32 + 16: a short last block
    do = _bf16(np.random.default_rng(131).standard_normal(q.shape))
    f = oracle.fwd(q, k, v, causal, 32, scale_mode=oracle.MX)
    g = oracle.bwd(q, k, v, do, f["L"], f["Op"], causal, scale_mode=oracle.MX)
    dq, dk, dv = _autograd_mx(q, k, v, do, causal)
    for name, a, b in (("dQ", g["dQ"], dq), ("dK", g["dK"], dk), ("dV", g["dV"], dv)):
        assert np.allclose(a, b, rtol=0, atol=5e-6 * np.abs(b).max()), name
    # and it is not the NVFP4 backward
    g16 = oracle.bwd(q, k, v, do, f["L"], f["Op"], causal)
    assert np.linalg.norm(g16["dV"] - g["dV"]) > 1e-3 * np.linalg.norm(g["dV"])


def test_mx_dV_is_PF_transpose_dO_with_blocks_of_32_keys():
    q, k, v = _rand(1, 2, 1, 96, 32, seed=32)
    do = _bf16(np.random.default_rng(132).standard_normal(q.shape))
    f = oracle.fwd(q, k, v, True, 64, scale_mode=oracle.MX)
    g = oracle.bwd(q, k, v, do, f["L"], f["Op"], True, scale_mode=oracle.MX)
    qf, kf = indep.fake_quant_mx_np(q), indep.fake_quant_mx_np(k)
    dv = np.zeros((96, 32))
    for h in range(2):
        s = qf[0, h] @ kf[0, 0].T / np.sqrt(32)
        s[np.triu(np.ones((96, 96), bool), 1)] = -np.inf
        p = np.exp(s - f["L"][0, h][:, None]).astype(np.float32).astype(np.float64)
        dv += indep.fake_quant_mx_np(p, axis=-1).T @ do[0, h]
    assert np.allclose(g["dV"][0, 0], dv, rtol=0, atol=1e-10)


@pytest.mark.parametrize("causal", [False, True])
def test_mx_sampled_backward_entry_points_match_full(causal):
    q, k, v = _rand(2, 4, 2, 70, 32, seed=33)
    do = _bf16(np.random.default_rng(133).standard_normal(q.shape))
    f = oracle.fwd(q, k, v, causal, 64, scale_mode=oracle.MX)
    g = oracle.bwd(q, k, v, do, f["L"], f["Op"], causal, scale_mode=oracle.MX)
    rows = oracle.flat_rows(2, 4, 70, [(0, 0, 0), (1, 3, 69), (0, 2, 33), (1, 1, 31), (1, 1, 32)])
    fr = oracle.fwd(q, k, v, causal, 64, scale_mode=oracle.MX, rows=rows)
    dq = oracle.bwd_dq_rows(q, k, v, do, rows, fr["L"], fr["Op"], causal, scale_mode=oracle.MX)
    assert np.allclose(dq, g["dQ"].reshape(-1, 32)[rows], rtol=0, atol=1e-12)
    keys = np.array([0, 31, 32, 47, 64, 69])
    b, hk = 1, 1
    dk, dv = oracle.bwd_dkdv_keys(q, k, v, do, b, hk, keys, f["L"][b, 2:4], f["Op"][b, 2:4], causal,
                                  scale_mode=oracle.MX)
    assert np.allclose(dk, g["dK"][b, hk, keys], rtol=0, atol=1e-12)
    assert np.allclose(dv, g["dV"][b, hk, keys], rtol=0, atol=1e-12)
    sparse = np.zeros_like(do).reshape(-1, 32); sparse[rows] = do.reshape(-1, 32)[rows]
    gs = oracle.bwd(q, k, v, sparse.reshape(do.shape), f["L"], f["Op"], causal, scale_mode=oracle.MX)
    dk2, dv2 = oracle.bwd_rows_dkdv(q, k, v, do, rows, fr["L"], fr["Op"], causal, scale_mode=oracle.MX)
    assert np.allclose(dk2, gs["dK"], rtol=0, atol=1e-12) and np.allclose(dv2, gs["dV"], rtol=0, atol=1e-12)


# ---------------------------------------------------------------- mixed recipe: FP4 Q K^T, MXFP8 (E4M3) P and V

def test_fp8_scale_rule_hand_cases():
    # 448 * 2^e >= amax first holds at: 448 -> 0; just above -> 1; 1 -> -8 (1.75 >= 1 > 0.875); 0.875 -> -9; 0 -> floor
    for amax, e in [(448.0, 0), (np.nextafter(448.0, 500.0), 1), (1.0, -8), (0.875, -9), (np.nextafter(0.875, 1.0), -8),
                    (0.0, -126), (3e38, 120)]:
        assert oracle.e8m0_from_amax_fp8(amax) == e + 127, (amax, e)


def test_e4m3_rounding_matches_torch_cast_including_ties():
    import torch
    rng = np.random.default_rng(40)
    grid = np.array([oracle.e4m3_value(b) for b in range(0x7F)])
    mids = 0.5 * (grid[:-1] + grid[1:])
    near = np.concatenate([np.nextafter(mids.astype(np.float32), np.float32(0)), mids.astype(np.float32),
                           np.nextafter(mids.astype(np.float32), np.float32(500))])
    vals = np.concatenate([grid, near, rng.uniform(0, 448, 4000), rng.uniform(0, 0.05, 2000)]).astype(np.float32)
    want = torch.from_numpy(vals).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    for sexp in (0, -7, 5):
        s = 2.0 ** sexp
        got = np.array([oracle.e4m3_round(float(v) * s, s) for v in vals])
        assert np.array_equal(got, want)
    assert oracle.e4m3_round(1000.0, 1.0) == 0x7E           # saturates at 448


def test_phi_mx8_numpy_twin_invariants_and_bytes():
    rng = np.random.default_rng(41)
    x = _bf16(rng.standard_normal((3, 70, 96)) * np.exp(rng.standard_normal((3, 70, 1))))
    assert np.array_equal(oracle.fake_quant_mx8(x).astype(np.float64), indep.fake_quant_mx8_np(x))
    assert np.array_equal(oracle.fake_quant_mx8(x, axis=-2).astype(np.float64), indep.fake_quant_mx8_np(x, axis=-2))
    codes, sb, xf = oracle.phi_mx8(x)
    s = np.ldexp(1.0, sb.astype(np.int64) - 127)
    blk = x.reshape(3, 70, 3, 32).astype(np.float64); q = xf.reshape(3, 70, 3, 32).astype(np.float64)
    # no saturation: the block maximum is in (224, 448] scale units and lands on 224 .. 448; normal elements are within 2^-4 relative
    top = np.abs(q).max(-1) / s
    assert (top >= 224).all() and (top <= 448).all()
    normal = np.abs(blk) >= s[..., None] * 2.0 ** -6
    assert (np.abs(blk - q)[normal] <= np.abs(blk)[normal] * 2.0 ** -4).all()
    # the bytes decode to the dequantized values
    dec = np.array([oracle.e4m3_value(b) for b in range(0x7F)])
    cb = codes.reshape(3, 70, 3, 32)
    val = np.where(cb & 0x80, -1.0, 1.0) * dec[cb & 0x7F] * s[..., None]
    assert np.array_equal(val, q)
    # exact homogeneity under powers of two, idempotence
    c2, sb2, xf2 = oracle.phi_mx8(x * 2.0 ** -5)
    assert np.array_equal(c2, codes) and np.array_equal(sb2.astype(int), sb.astype(int) - 5)
    assert np.array_equal(oracle.phi_mx8(xf)[2], xf)


@pytest.mark.parametrize("causal", [False, True])
def test_fp8pv_forward_matches_textbook_and_rowwise_transcription(causal):
    q, k, v = _rand(1, 2, 1, 200, 32, seed=42, outlier=True)
    qf = indep.fake_quant_mx_np(q); kf = indep.fake_quant_mx_np(k); vf = indep.fake_quant_mx8_np(v, axis=-2)
    r0 = oracle.fwd(q, k, v, causal, 64, quant_p=False, scale_mode=oracle.MX_FP8PV)
    O, L = _textbook(qf, np.repeat(kf, 2, 1), np.repeat(vf, 2, 1), causal)
    assert np.allclose(r0["O"], O, rtol=0, atol=1e-6) and np.allclose(r0["L"], L, rtol=0, atol=1e-6)
    r = oracle.fwd(q, k, v, causal, 64, scale_mode=oracle.MX_FP8PV)
    for h in range(2):
        O, Op, L = indep.attn_fwd_rowwise_np(qf[0, h], kf[0, 0], vf[0, 0], causal, 64, fq=indep.fake_quant_mx8_np)
        assert np.allclose(r["O"][0, h], O, rtol=0, atol=1e-12)
        assert np.allclose(r["Op"][0, h], Op, rtol=0, atol=1e-12)
        assert np.allclose(r["L"][0, h], L, rtol=0, atol=1e-12)
    # FP8 for P and V is closer to the un-quantized-P output than FP4 is
    r4 = oracle.fwd(q, k, v, causal, 64, scale_mode=oracle.MX)
    e8 = np.linalg.norm(r["O"] - r0["O"]) / np.linalg.norm(r0["O"])
    r40 = oracle.fwd(q, k, v, causal, 64, quant_p=False, scale_mode=oracle.MX)
    e4 = np.linalg.norm(r4["O"] - r40["O"]) / np.linalg.norm(r40["O"])
    assert e8 < 0.5 * e4
