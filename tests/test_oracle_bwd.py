"""Pins for the oracle's backward (Alg. 3, Eq. 5-7)."""
import numpy as np
import pytest
import torch

import oracle
from tests import indep
from tests.test_oracle_fwd import _rand


def _bf(a):
    return torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()


def _autograd(q, k, v, do, causal, quant_qkv, quant_p):
    """torch autograd (fp64) through the explicitly unrolled fake-quant graph with a
    straight-through estimator at every phi^-1 phi (Eq. 4, Eq. 5): identity gradient."""
    def ste(x, axis=-1):
        fq = torch.from_numpy(indep.fake_quant_np(x.detach().numpy(), axis=axis))
        return x + (fq - x).detach()

    q, k, v, do = (torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
                   for a in (q, k, v, do))
    G = q.shape[1] // k.shape[1]
    qf, kf, vf = (ste(q), ste(k), ste(v)) if quant_qkv else (q, k, v)
    kf = kf.repeat_interleave(G, dim=1); vf = vf.repeat_interleave(G, dim=1)
    s = qf @ kf.transpose(-1, -2) / np.sqrt(q.shape[-1])
    if causal:
        L = q.shape[2]
        s = s.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
    p = torch.softmax(s, -1)
    if quant_p:
        p32 = p.detach().to(torch.float32).to(torch.float64)        # phi sees the fp32 softmax
        pq = torch.from_numpy(indep.fake_quant_np(p32.numpy(), axis=-1))
        p = p + (pq - p).detach()
    o = p @ vf
    (o * do.detach()).sum().backward()
    return q.grad.numpy(), k.grad.numpy(), v.grad.numpy()


def _oracle_fwd_bwd(q, k, v, do, causal, Bk=64, **kw):
    f = oracle.fwd(q, k, v, causal, Bk, **kw)
    return f, oracle.bwd(q, k, v, do, f["L"], f["Op"], causal, **kw)


@pytest.mark.parametrize("causal", [False, True])
def test_phi_off_is_analytic_attention_gradient(causal):
    q, k, v = _rand(2, 4, 2, 70, 32, seed=20)
    do = _bf(np.random.default_rng(21).standard_normal(q.shape).astype(np.float32))
    _, g = _oracle_fwd_bwd(q, k, v, do, causal, quant_qkv=False, quant_p=False)
    dq, dk, dv = _autograd(q, k, v, do, causal, False, False)
    for a, b in ((g["dQ"], dq), (g["dK"], dk), (g["dV"], dv)):
        assert np.allclose(a, b, rtol=0, atol=2e-6 * np.abs(b).max())


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("seed", [22, 23])
def test_phi_on_matches_autograd_of_unrolled_ste_graph(causal, seed):
    """Alg. 3 (P re-quantized, D from O', dS from the fp32 P) equals brute-force STE autograd."""
    q, k, v = _rand(1, 4, 2, 80, 32, seed=seed, outlier=True)
    do = _bf(np.random.default_rng(seed + 100).standard_normal(q.shape).astype(np.float32))
    _, g = _oracle_fwd_bwd(q, k, v, do, causal, Bk=32)
    dq, dk, dv = _autograd(q, k, v, do, causal, True, True)
    for name, a, b in (("dQ", g["dQ"], dq), ("dK", g["dK"], dk), ("dV", g["dV"], dv)):
        assert np.allclose(a, b, rtol=0, atol=5e-6 * np.abs(b).max()), name


def test_D_from_low_precision_O_breaks_the_identity():
    """Eq. 7: rowsum(P o dP) = rowsum(dO o O') holds with O', not with O (Sec. 2.3)."""
    q, k, v = _rand(1, 2, 2, 64, 32, seed=24)
    do = _bf(np.random.default_rng(25).standard_normal(q.shape).astype(np.float32))
    f = oracle.fwd(q, k, v, False, 64)
    qf, kf, vf = (indep.fake_quant_np(a) for a in (q, k, v))
    s = qf @ np.swapaxes(kf, -1, -2) / np.sqrt(32)
    p = np.exp(s - f["L"][..., None])
    dP = do.astype(np.float64) @ np.swapaxes(vf, -1, -2)
    lhs = (p * dP).sum(-1)
    assert np.allclose(lhs, (do * f["Op"]).sum(-1), rtol=0, atol=1e-6)
    assert not np.allclose(lhs, (do * f["O"]).sum(-1), rtol=0, atol=1e-3)


def test_constant_keys_give_zero_dQ():
    """rowsum(dS) = 0 when D comes from O' (softmax Jacobian, Eq. 6): with all key rows
    equal, dQ_i = (sum_k dS_ik) * k vanishes."""
    q, k, v = _rand(1, 2, 2, 64, 32, seed=26)
    k[:] = k[:, :, :1, :]
    do = _bf(np.random.default_rng(27).standard_normal(q.shape).astype(np.float32))
    _, g = _oracle_fwd_bwd(q, k, v, do, False)
    assert np.abs(g["dQ"]).max() < 1e-6 * np.abs(g["dK"]).max() + 1e-9


def test_dV_is_PF_transpose_dO():
    q, k, v = _rand(1, 2, 1, 64, 32, seed=28)
    do = _bf(np.random.default_rng(29).standard_normal(q.shape).astype(np.float32))
    f, g = _oracle_fwd_bwd(q, k, v, do, True)
    qf, kf = indep.fake_quant_np(q), indep.fake_quant_np(k)
    dv = np.zeros((64, 32))
    for h in range(2):
        s = qf[0, h] @ kf[0, 0].T / np.sqrt(32)
        s[np.triu(np.ones((64, 64), bool), 1)] = -np.inf
        p = np.exp(s - f["L"][0, h][:, None]).astype(np.float32).astype(np.float64)
        dv += indep.fake_quant_np(p, axis=-1).T @ do[0, h]
    assert np.allclose(g["dV"][0, 0], dv, rtol=0, atol=1e-10)


@pytest.mark.parametrize("causal", [False, True])
def test_sampled_entry_points_match_full(causal):
    q, k, v = _rand(2, 4, 2, 50, 32, seed=30)
    do = _bf(np.random.default_rng(31).standard_normal(q.shape).astype(np.float32))
    f, g = _oracle_fwd_bwd(q, k, v, do, causal, Bk=16)
    rows = oracle.flat_rows(2, 4, 50, [(0, 0, 0), (1, 3, 49), (0, 2, 33), (1, 1, 7)])
    fr = oracle.fwd(q, k, v, causal, 16, rows=rows)
    dq = oracle.bwd_dq_rows(q, k, v, do, rows, fr["L"], fr["Op"], causal)
    assert np.allclose(dq, g["dQ"].reshape(-1, 32)[rows], rtol=0, atol=1e-12)
    keys = np.array([0, 15, 16, 37, 49])
    b, hk = 1, 1
    dk, dv, P = oracle.bwd_dkdv_keys(q, k, v, do, b, hk, keys, f["L"][b, 2:4], f["Op"][b, 2:4],
                                     causal, dump_p=True)
    assert np.allclose(dk, g["dK"][b, hk, keys], rtol=0, atol=1e-12)
    assert np.allclose(dv, g["dV"][b, hk, keys], rtol=0, atol=1e-12)
    # P = 1 quantizes to 6 * RNE_E4M3(1/6) = 6 * 0.171875 = 1.03125
    assert P.shape == (5, 2, 50) and P.max() <= 1.03125


@pytest.mark.parametrize("causal", [False, True])
def test_rows_restricted_dkdv_equals_full_backward_with_sparse_dO(causal):
    q, k, v = _rand(1, 4, 2, 70, 32, seed=40)
    do = _bf(np.random.default_rng(41).standard_normal(q.shape).astype(np.float32))
    rows = oracle.flat_rows(1, 4, 70, [(0, 0, 0), (0, 1, 69), (0, 3, 35), (0, 2, 16), (0, 2, 17)])
    sparse = np.zeros_like(do).reshape(-1, 32)
    sparse[rows] = do.reshape(-1, 32)[rows]
    sparse = sparse.reshape(do.shape)
    f, g = _oracle_fwd_bwd(q, k, v, sparse, causal)
    fr = oracle.fwd(q, k, v, causal, 64, rows=rows)
    dk, dv = oracle.bwd_rows_dkdv(q, k, v, do, rows, fr["L"], fr["Op"], causal)
    assert np.allclose(dk, g["dK"], rtol=0, atol=1e-12) and np.allclose(dv, g["dV"], rtol=0, atol=1e-12)
    assert np.abs(g["dK"]).max() > 1e-3
