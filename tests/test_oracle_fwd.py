"""Pins for the oracle's forward (Alg. 1 / Alg. 2)."""
import numpy as np
import pytest
import torch

import oracle
from tests import indep


def _rand(B, Hq, Hkv, L, d, seed, outlier=False):
    rng = np.random.default_rng(seed)
    bf = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    q = bf(rng.standard_normal((B, Hq, L, d)).astype(np.float32))
    k = bf(rng.standard_normal((B, Hkv, L, d)).astype(np.float32))
    v = bf(rng.standard_normal((B, Hkv, L, d)).astype(np.float32))
    if outlier:
        k[..., 3] *= 20
    return q, k, v


def _textbook(q, k, v, causal):
    """softmax(QK^T/sqrt d)V and logsumexp with torch's library routines, fp64."""
    q, k, v = (torch.from_numpy(np.asarray(a, dtype=np.float64)) for a in (q, k, v))
    G = q.shape[1] // k.shape[1]
    k = k.repeat_interleave(G, dim=1); v = v.repeat_interleave(G, dim=1)
    s = q @ k.transpose(-1, -2) / np.sqrt(q.shape[-1])
    if causal:
        L = q.shape[2]
        s = s.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
    return (torch.softmax(s, -1) @ v).numpy(), torch.logsumexp(s, -1).numpy()


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Bk", [16, 64, 128])
def test_phi_off_is_textbook_attention_for_any_tile(causal, Bk):
    q, k, v = _rand(2, 4, 2, 100, 32, seed=10)            # GQA, ragged L
    r = oracle.fwd(q, k, v, causal, Bk, quant_qkv=False, quant_p=False)
    O, L = _textbook(q, k, v, causal)
    assert np.allclose(r["O"], O, rtol=0, atol=1e-6)      # P-tilde is rounded to fp32
    assert np.allclose(r["Op"], O, rtol=0, atol=1e-6)
    assert np.allclose(r["L"], L, rtol=0, atol=1e-6)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Bk", [16, 64])
def test_L_and_Oprime_ignore_P_quantization(causal, Bk):
    """With phi on: L = logsumexp(Q^F K^F^T/sqrt d), O' = softmax(.) V^F (Alg. 2, Sec. 2.3)."""
    q, k, v = _rand(1, 4, 2, 150, 64, seed=11, outlier=True)
    r = oracle.fwd(q, k, v, causal, Bk)
    qf, kf, vf = (indep.fake_quant_np(a) for a in (q, k, v))
    O, L = _textbook(qf, kf, vf, causal)
    assert np.allclose(r["Op"], O, rtol=0, atol=2e-6)
    assert np.allclose(r["L"], L, rtol=0, atol=1e-6)
    # and O differs from O' by quantization noise, not by a bug-sized amount
    rel = np.linalg.norm(r["O"] - r["Op"]) / np.linalg.norm(r["Op"])
    assert 1e-3 < rel < 0.2


def test_single_tile_closed_form():
    """L <= Bk: one tile, no running max: O = phi^-1 phi(exp(S - rowmax)) V^F / rowsum(exp(S - rowmax))."""
    q, k, v = _rand(1, 2, 2, 48, 32, seed=12)
    r = oracle.fwd(q, k, v, False, 64)
    qf, kf, vf = (indep.fake_quant_np(a) for a in (q, k, v))
    for h in range(2):
        s = qf[0, h] @ kf[0, h].T / np.sqrt(32)
        pt = np.exp(s - s.max(-1, keepdims=True)).astype(np.float32).astype(np.float64)
        o = indep.fake_quant_np(pt, axis=-1) @ vf[0, h] / pt.sum(-1, keepdims=True)
        assert np.allclose(r["O"][0, h], o, rtol=0, atol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Bk", [16, 32, 64])
def test_multi_tile_matches_independent_rowwise_transcription(causal, Bk):
    q, k, v = _rand(1, 2, 1, 200, 32, seed=13, outlier=True)
    r = oracle.fwd(q, k, v, causal, Bk)
    qf, kf, vf = (indep.fake_quant_np(a) for a in (q, k, v))
    for h in range(2):
        O, Op, L = indep.attn_fwd_rowwise_np(qf[0, h], kf[0, 0], vf[0, 0], causal, Bk)
        assert np.allclose(r["O"][0, h], O, rtol=0, atol=1e-12)
        assert np.allclose(r["Op"][0, h], Op, rtol=0, atol=1e-12)
        assert np.allclose(r["L"][0, h], L, rtol=0, atol=1e-12)


def test_tile_size_is_semantic_only_with_phi_on():
    q, k, v = _rand(1, 1, 1, 256, 32, seed=14)
    a = oracle.fwd(q, k, v, False, 16)["O"]; b = oracle.fwd(q, k, v, False, 128)["O"]
    assert np.linalg.norm(a - b) / np.linalg.norm(a) > 1e-3        # quantization-noise sized
    a = oracle.fwd(q, k, v, False, 16, quant_p=False)["O"]
    b = oracle.fwd(q, k, v, False, 128, quant_p=False)["O"]
    assert np.allclose(a, b, rtol=0, atol=1e-6)


def test_row_subset_and_P_dump():
    q, k, v = _rand(2, 2, 1, 96, 32, seed=15)
    full = oracle.fwd(q, k, v, True, 32)
    rows = oracle.flat_rows(2, 2, 96, [(0, 0, 0), (1, 1, 95), (0, 1, 40), (1, 0, 17)])
    sub = oracle.fwd(q, k, v, True, 32, rows=rows, dump_p=True)
    for n, rid in enumerate(rows):
        b, h, i = rid // (2 * 96), (rid // 96) % 2, rid % 96
        assert np.array_equal(sub["O"][n], full["O"][b, h, i])
        assert np.array_equal(sub["L"][n], full["L"][b, h, i])
        assert not sub["P"][n, i + 1:].any()                          # causal mask
    # the dumped P-tilde^F reproduces O when only one tile precedes (row 17 sees tile 0 only)
    n = 3; vf = indep.fake_quant_np(v)[1, 0]
    qf = indep.fake_quant_np(q)[1, 0, 17]; kf = indep.fake_quant_np(k)[1, 0]
    s = kf[:18] @ qf / np.sqrt(32)
    l = np.exp(s - s.max()).astype(np.float32).astype(np.float64).sum()
    assert np.allclose(sub["P"][n, :96].astype(np.float64) @ vf / l, sub["O"][n], atol=1e-12)


def test_fp4_attention_error_band():
    """Sanity band only (Appendix, per-call error table): cosine similarity to the
    unquantized output is about 0.99 for FP4 attention."""
    q, k, v = _rand(1, 4, 4, 256, 64, seed=16)
    r = oracle.fwd(q, k, v, False, 64)
    O, _ = _textbook(q, k, v, False)
    cos = (r["O"] * O).sum() / np.linalg.norm(r["O"]) / np.linalg.norm(O)
    assert 0.97 < cos < 0.9999
