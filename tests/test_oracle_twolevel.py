"""Pins of the oracle's two-level quantization of P (Sec. 2.1: each row of P is rescaled to [0, 448 * 6] before the
NVFP4 blocks; an option inside QAT in Sec. 3.2).  Readings pinned here: rows are the 64 keys of a key tile, in the
forward and (the same aligned groups of the recomputed P) in the backward; the row factor is the smallest power of two
that keeps the row maximum below 448 * 6, with a floor of 2^-24 on that maximum."""
import numpy as np
import pytest
import torch

import oracle
from tests import indep
from tests.test_oracle_fwd import _rand

TL = oracle.TWO_LEVEL_P


def _bf(a):
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def test_row_factor_hand_cases_and_closed_form():
    # 2688 = 1.3125 * 2^11: rowmax 1 -> 2^-11; 1.3125 -> 2^-11; just above -> 2^-10; 0.65625 -> 2^-12; the floor 2^-24 -> 2^-35
    for rmax, k in [(1.0, -11), (1.3125, -11), (np.nextafter(1.3125, 2.0), -10), (0.65625, -12), (0.0, -35), (2.0 ** -30, -35),
                    (2.0 ** -24, -35), (1e-3, -21)]:
        assert oracle.two_level_s1(rmax) == 2.0 ** k, (rmax, k)
    rng = np.random.default_rng(70)
    r = np.exp(rng.uniform(np.log(1e-7), 0.0, 2000)).astype(np.float32).astype(np.float64)
    s1 = np.array([oracle.two_level_s1(v) for v in r])
    assert (2688 * s1 >= r).all() and (2688 * s1 / 2 < r).all()           # the smallest such power of two
    m, ex = np.frexp(r)
    assert np.array_equal(s1, np.ldexp(1.0, ex - 12 + (m > 0.65625)))


@pytest.mark.parametrize("causal", [False, True])
def test_forward_matches_independent_rowwise_transcription(causal):
    q, k, v = _rand(1, 2, 1, 200, 32, seed=71, outlier=True)
    r = oracle.fwd(q, k, v, causal, 64, scale_mode=TL)
    qf, kf, vf = (indep.fake_quant_np(a) for a in (q, k, v))
    for h in range(2):
        O, Op, L = indep.attn_fwd_rowwise_np(qf[0, h], kf[0, 0], vf[0, 0], causal, 64, fq=indep.fake_quant_two_level_np)
        assert np.allclose(r["O"][0, h], O, rtol=0, atol=1e-12)
        assert np.allclose(r["Op"][0, h], Op, rtol=0, atol=1e-12)
        assert np.allclose(r["L"][0, h], L, rtol=0, atol=1e-12)
    # O' and L do not see the quantizer of P; Q, K, V are quantized as in the plain method
    plain = oracle.fwd(q, k, v, causal, 64)
    assert np.array_equal(plain["Op"], r["Op"]) and np.array_equal(plain["L"], r["L"])
    assert not np.array_equal(plain["O"], r["O"])
    with pytest.raises(ValueError):
        oracle.fwd(q, k, v, causal, 32, scale_mode=TL)                   # rows are 64-key tiles


def test_two_levels_keep_the_probabilities_that_plain_nvfp4_flushes():
    """A block whose largest P-tilde is below 6 * 2^-10 gets the scale 0 in plain NVFP4 and vanishes; with the row
    factor it is quantized with the usual relative error.  One dominant key per row, all others 2-3 e-3 of it."""
    rng = np.random.default_rng(72)
    L, d = 512, 32
    q = np.zeros((1, 1, L, d), np.float32); k = np.zeros((1, 1, L, d), np.float32)
    q[..., 0] = 8.0
    k[..., 0] = rng.uniform(0.0, 0.3, L)                                  # scores within a narrow band ...
    k[0, 0, 5, 0] = 4.5                                                   # ... except one key far above
    v = _bf(rng.standard_normal((1, 1, L, d)))
    q, k = _bf(q), _bf(k)
    ref = oracle.fwd(q, k, v, False, 64, quant_p=False)["O"]
    plain = oracle.fwd(q, k, v, False, 64)["O"]
    two = oracle.fwd(q, k, v, False, 64, scale_mode=TL)["O"]
    e_plain = np.linalg.norm(plain - ref) / np.linalg.norm(ref); e_two = np.linalg.norm(two - ref) / np.linalg.norm(ref)
    assert e_two < 0.8 * e_plain
    p = oracle.fwd(q, k, v, False, 64, rows=np.array([100]), dump_p=True)["P"][0]
    p2 = oracle.fwd(q, k, v, False, 64, scale_mode=TL, rows=np.array([100]), dump_p=True)["P"][0]
    assert (p[64:] == 0).all() and (p2[64:] > 0).mean() > 0.9            # tiles without the dominant key


@pytest.mark.parametrize("causal", [False, True])
def test_backward_matches_autograd_of_unrolled_ste_graph(causal):
    q, k, v = _rand(1, 4, 2, 150, 32, seed=73, outlier=True)             # 150 = 2 * 64 + 22: a short last group
    do = _bf(np.random.default_rng(74).standard_normal(q.shape))
    f = oracle.fwd(q, k, v, causal, 64, scale_mode=TL)
    g = oracle.bwd(q, k, v, do, f["L"], f["Op"], causal, scale_mode=TL)

    def ste(x):
        fq = torch.from_numpy(indep.fake_quant_np(x.detach().numpy(), axis=-1))
        return x + (fq - x).detach()
    tq, tk, tv = (torch.tensor(np.asarray(a, np.float64), requires_grad=True) for a in (q, k, v))
    qf, kf, vf = ste(tq), ste(tk), ste(tv)
    kf = kf.repeat_interleave(2, dim=1); vf = vf.repeat_interleave(2, dim=1)
    s = qf @ kf.transpose(-1, -2) / np.sqrt(32)
    if causal:
        s = s.masked_fill(torch.triu(torch.ones(150, 150, dtype=torch.bool), 1), float("-inf"))
    p = torch.softmax(s, -1)
    # the same operator as the forward: the row factor is taken per aligned group of 64 keys
    pq = torch.from_numpy(indep.fake_quant_two_level_np(p.detach().to(torch.float32).to(torch.float64).numpy(), axis=-1))
    p = p + (pq - p).detach()
    ((p @ vf) * torch.from_numpy(do.astype(np.float64))).sum().backward()
    for name, a, b in (("dQ", g["dQ"], tq.grad.numpy()), ("dK", g["dK"], tk.grad.numpy()), ("dV", g["dV"], tv.grad.numpy())):
        assert np.allclose(a, b, rtol=0, atol=5e-6 * np.abs(b).max()), name
    # only dV sees the quantizer of P (dS uses the fp32 P, Sec. 2.3)
    g0 = oracle.bwd(q, k, v, do, f["L"], f["Op"], causal)
    assert np.array_equal(g0["dQ"], g["dQ"]) and np.array_equal(g0["dK"], g["dK"]) and not np.array_equal(g0["dV"], g["dV"])


@pytest.mark.parametrize("causal", [False, True])
def test_sampled_backward_entry_points_match_full(causal):
    q, k, v = _rand(2, 4, 2, 140, 32, seed=75)
    do = _bf(np.random.default_rng(76).standard_normal(q.shape))
    f = oracle.fwd(q, k, v, causal, 64, scale_mode=TL)
    g = oracle.bwd(q, k, v, do, f["L"], f["Op"], causal, scale_mode=TL)
    rows = oracle.flat_rows(2, 4, 140, [(0, 0, 0), (1, 3, 139), (0, 2, 63), (1, 1, 64), (1, 1, 100)])
    fr = oracle.fwd(q, k, v, causal, 64, scale_mode=TL, rows=rows)
    keys = np.array([0, 15, 16, 63, 64, 127, 128, 139])
    b, hk = 1, 1
    dk, dv = oracle.bwd_dkdv_keys(q, k, v, do, b, hk, keys, f["L"][b, 2:4], f["Op"][b, 2:4], causal, scale_mode=TL)
    assert np.allclose(dk, g["dK"][b, hk, keys], rtol=0, atol=1e-12)
    assert np.allclose(dv, g["dV"][b, hk, keys], rtol=0, atol=1e-12)
    sparse = np.zeros_like(do).reshape(-1, 32); sparse[rows] = do.reshape(-1, 32)[rows]
    gs = oracle.bwd(q, k, v, sparse.reshape(do.shape), f["L"], f["Op"], causal, scale_mode=TL)
    dk2, dv2 = oracle.bwd_rows_dkdv(q, k, v, do, rows, fr["L"], fr["Op"], causal, scale_mode=TL)
    assert np.allclose(dk2, gs["dK"], rtol=0, atol=1e-12) and np.allclose(dv2, gs["dV"], rtol=0, atol=1e-12)
