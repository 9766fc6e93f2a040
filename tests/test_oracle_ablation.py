"""The backward ablations of Sec. 3.2 (Exp. 7: D from the low-precision O; Exp. 8: no fake quantization
of P in the backward) as the oracle computes them, pinned by what Sec. 2.3 says must and must not hold."""
import numpy as np

import oracle
import workloads as W
from tests.indep import fake_quant_np


def _inputs(B=1, Hq=2, Hkv=1, L=96, d=64, seed=21):
    f = lambda t, h: W.bf16_bits_to_f32(W.fill(B, h, L, d, seed, t, "normal", 1.0))
    return f(W.TENSOR_Q, Hq), f(W.TENSOR_K, Hkv), f(W.TENSOR_V, Hkv), f(W.TENSOR_DO, Hq)


def test_row_sums_of_dS_vanish_only_with_the_high_precision_output():
    """Eq. 6-7: with D = rowsum(dO o O'), rowsum(dS) = 0, hence sum_j dK_j = sum_i (sum_j dS_ij) Q^F_i = 0
    (a common shift of all keys moves every logit of a row alike and cannot change the loss).  With D taken
    from the low-precision O = P-tilde^F V^F / l that sum is far from zero."""
    q, k, v, do = _inputs()
    for causal in (False, True):
        r = oracle.fwd(q, k, v, causal, 64)
        good = oracle.bwd(q, k, v, do, r["L"], r["Op"], causal)
        bad = oracle.bwd(q, k, v, do, r["L"], r["O"], causal)
        scale = np.abs(good["dK"]).sum(axis=2)
        # (the oracle rounds P to fp32 before phi(P) and uses that P throughout: 6e-8 relative)
        assert np.abs(good["dK"].sum(axis=2)).max() <= 1e-6 * scale.max()
        assert np.abs(bad["dK"].sum(axis=2)).max() >= 1e-3 * scale.max()
        # dV does not depend on D at all
        assert np.array_equal(good["dV"], bad["dV"])


def test_unquantized_P_changes_dV_only_and_equals_the_plain_product():
    q, k, v, do = _inputs(L=80)
    causal = True
    r = oracle.fwd(q, k, v, causal, 64)
    a = oracle.bwd(q, k, v, do, r["L"], r["Op"], causal)
    b = oracle.bwd(q, k, v, do, r["L"], r["Op"], causal, quant_p=False)
    assert np.array_equal(a["dQ"], b["dQ"]) and np.array_equal(a["dK"], b["dK"])     # dS uses the fp32 P in both
    assert not np.array_equal(a["dV"], b["dV"])
    # dV = P^T dO with P = exp(S - L), summed over the query heads of the group
    qf, kf = fake_quant_np(q).astype(np.float64), fake_quant_np(k).astype(np.float64)
    L_, d = q.shape[2], q.shape[3]
    want = np.zeros_like(b["dV"])
    for h in range(q.shape[1]):
        s = qf[0, h] @ kf[0, 0].T / np.sqrt(d)
        p = np.exp(s - r["L"][0, h][:, None]) * np.tril(np.ones((L_, L_)))
        want[0, 0] += p.T @ do[0, h].astype(np.float64)
    assert np.abs(b["dV"] - want).max() <= 1e-5 * np.abs(want).max()     # P is rounded to fp32 inside the oracle
