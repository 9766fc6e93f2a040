"""Pins of the oracle's K smoothing (Sec. 2.1: K minus its token mean; an option inside QAT in Sec. 3.2)."""
import numpy as np
import pytest
import torch

import oracle
from tests import indep
from tests.test_oracle_fwd import _rand


def _bf(a):
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def test_smoothing_is_the_centred_k():
    q, k, v = _rand(2, 4, 2, 70, 32, seed=60)
    k = _bf(k + 3.0)
    ks = oracle.smooth_k(k)
    assert ks.dtype == np.float32 and ks.shape == k.shape
    want = k.astype(np.float64) - k.astype(np.float64).mean(axis=-2, keepdims=True)
    assert np.allclose(ks, want, rtol=0, atol=4e-7 * np.abs(k).max())           # two fp32 roundings
    assert np.abs(ks.astype(np.float64).mean(axis=-2)).max() < 1e-6


@pytest.mark.parametrize("causal", [False, True])
def test_softmax_ignores_the_shift_when_nothing_is_quantized(causal):
    q, k, v = _rand(1, 4, 2, 90, 32, seed=61)
    k = _bf(k + 2.5)
    a = oracle.fwd(q, k, v, causal, 64, quant_qkv=False, quant_p=False)
    b = oracle.fwd(q, oracle.smooth_k(k), v, causal, 64, quant_qkv=False, quant_p=False)
    assert np.allclose(a["O"], b["O"], rtol=0, atol=2e-5)
    # L moves by the per-query constant q . mean(k) / sqrt(d)
    G = 2
    mean = k.astype(np.float64).mean(axis=-2)                                    # [B, Hkv, d]
    shift = np.einsum("bhld,bhd->bhl", q.astype(np.float64), np.repeat(mean, G, axis=1)) / np.sqrt(32)
    assert np.allclose(a["L"] - b["L"], shift, rtol=0, atol=2e-5)


def test_smoothing_reduces_the_quantization_error_of_offset_keys():
    q, k, v = _rand(1, 2, 2, 256, 64, seed=62)
    k = _bf(k * 0.5 + 4.0)                                                       # a common offset dominates every block
    ref = oracle.fwd(q, k, v, False, 64, quant_qkv=False, quant_p=False)["O"]
    plain = oracle.fwd(q, k, v, False, 64)["O"]
    smooth = oracle.fwd(q, oracle.smooth_k(k), v, False, 64)["O"]
    e0 = np.linalg.norm(plain - ref) / np.linalg.norm(ref); e1 = np.linalg.norm(smooth - ref) / np.linalg.norm(ref)
    assert e1 < 0.7 * e0


@pytest.mark.parametrize("causal", [False, True])
def test_backward_through_the_smoothing_is_the_backward_of_the_centred_keys(causal):
    """Autograd through K' = K - mean(K) (Jacobian I - 11^T / L) and the unrolled straight-through graph gives the
    oracle's dK of the centred keys: the correction mean_j(dK'_j) vanishes because rowsum(dS) = 0 with D from O'."""
    q, k, v = _rand(1, 4, 2, 80, 32, seed=63, outlier=True)
    k = _bf(k + 1.5)
    do = _bf(np.random.default_rng(64).standard_normal(q.shape))
    ks = oracle.smooth_k(k)
    f = oracle.fwd(q, ks, v, causal, 32)
    g = oracle.bwd(q, ks, v, do, f["L"], f["Op"], causal)

    def ste(x, axis=-1):
        fq = torch.from_numpy(indep.fake_quant_np(x.detach().numpy(), axis=axis))
        return x + (fq - x).detach()
    tq, tk, tv = (torch.tensor(np.asarray(a, np.float64), requires_grad=True) for a in (q, k, v))
    tks = tk - tk.mean(dim=-2, keepdim=True)
    tks = tks + (torch.from_numpy(ks.astype(np.float64)) - tks).detach()          # the oracle's fp32 values, autograd's Jacobian
    qf, kf, vf = ste(tq), ste(tks), ste(tv)
    kf = kf.repeat_interleave(2, dim=1); vf = vf.repeat_interleave(2, dim=1)
    s = qf @ kf.transpose(-1, -2) / np.sqrt(32)
    if causal:
        s = s.masked_fill(torch.triu(torch.ones(80, 80, dtype=torch.bool), 1), float("-inf"))
    p = torch.softmax(s, -1)
    pq = torch.from_numpy(indep.fake_quant_np(p.detach().to(torch.float32).to(torch.float64).numpy(), axis=-1))
    p = p + (pq - p).detach()
    ((p @ vf) * torch.from_numpy(do.astype(np.float64))).sum().backward()
    for name, a, b in (("dQ", g["dQ"], tq.grad.numpy()), ("dK", g["dK"], tk.grad.numpy()), ("dV", g["dV"], tv.grad.numpy())):
        assert np.allclose(a, b, rtol=0, atol=5e-6 * np.abs(b).max()), name
