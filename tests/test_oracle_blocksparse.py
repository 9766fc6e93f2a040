"""Pins of the oracle's block-sparse forward (the datacenter inference kernel of Sec. 2.5 supports block-sparse attention, Sec. 5):
a zero byte of the block mask removes a block of queries x keys."""
import numpy as np
import pytest

import oracle
from tests import indep
from tests.test_oracle_fwd import _rand


def _mask(B, Hq, L, bq, bk, seed, keep=0.5):
    rng = np.random.default_rng(seed)
    m = (rng.random((B, Hq, (L + bq - 1) // bq, (L + bk - 1) // bk)) < keep).astype(np.uint8)
    m[..., 0] = 1                      # every row keeps its first key block (so no row is empty, also under the causal mask)
    return m


def _dense(m, L, bq, bk):
    return np.repeat(np.repeat(m, bq, axis=-2), bk, axis=-1)[..., :L, :L].astype(bool)


@pytest.mark.parametrize("causal", [False, True])
def test_block_mask_with_phi_off_is_masked_textbook_attention(causal):
    B, Hq, Hkv, L, d = 1, 4, 2, 300, 32
    q, k, v = _rand(B, Hq, Hkv, L, d, seed=80)
    bm = _mask(B, Hq, L, 128, 128, 81)
    r = oracle.fwd(q, k, v, causal, 64, quant_qkv=False, quant_p=False, block_mask=bm)
    keep = _dense(bm, L, 128, 128)
    if causal:
        keep &= np.tril(np.ones((L, L), bool))
    kk = np.repeat(k.astype(np.float64), 2, 1); vv = np.repeat(v.astype(np.float64), 2, 1)
    s = np.where(keep, q.astype(np.float64) @ np.swapaxes(kk, -1, -2) / np.sqrt(d), -np.inf)
    mx = s.max(-1, keepdims=True); p = np.exp(s - mx)
    assert np.allclose(r["O"], p @ vv / p.sum(-1, keepdims=True), rtol=0, atol=1e-6)
    assert np.allclose(r["L"], (mx + np.log(p.sum(-1, keepdims=True)))[..., 0], rtol=0, atol=1e-6)


def test_full_mask_is_no_mask_and_other_block_sizes():
    q, k, v = _rand(1, 2, 1, 200, 32, seed=82)
    a = oracle.fwd(q, k, v, True, 64)
    b = oracle.fwd(q, k, v, True, 64, block_mask=np.ones((1, 2, 2, 2), np.uint8))
    assert np.array_equal(a["O"], b["O"]) and np.array_equal(a["L"], b["L"])
    bm = _mask(1, 2, 200, 64, 64, 83)
    c = oracle.fwd(q, k, v, False, 64, block_mask=bm, mask_block=(64, 64))
    assert not np.array_equal(a["O"], c["O"])
    with pytest.raises(ValueError):
        oracle.fwd(q, k, v, False, 64, block_mask=np.ones((1, 2, 7, 7), np.uint8), mask_block=(32, 32))   # key blocks are whole tiles


@pytest.mark.parametrize("sm", [0, oracle.MX])
def test_masked_forward_equals_the_rowwise_transcription_on_the_kept_tiles(sm):
    """With phi on: a row visits exactly the key tiles of its kept blocks, in increasing order."""
    L, d = 320, 32
    q, k, v = _rand(1, 1, 1, L, d, seed=84, outlier=True)
    bm = _mask(1, 1, L, 128, 128, 85, keep=0.6)
    r = oracle.fwd(q, k, v, False, 64, scale_mode=sm, block_mask=bm, dump_p=True)
    if sm == oracle.MX:
        qf, kf, vf = indep.fake_quant_mx_np(q), indep.fake_quant_mx_np(k), indep.fake_quant_mx_np(v, axis=-2)
        fq = indep.fake_quant_mx_np
    else:
        qf, kf, vf = (indep.fake_quant_np(a) for a in (q, k, v))
        fq = indep.fake_quant_np
    for i in (0, 127, 128, 300):
        m, l, o = -np.inf, 0.0, np.zeros(d)
        for k0 in range(0, L, 64):
            if not bm[0, 0, i // 128, k0 // 128]:
                assert not r["P"].reshape(L, L)[i, k0:k0 + 64].any()
                continue
            s = kf[0, 0, k0:k0 + 64] @ qf[0, 0, i] / np.sqrt(d)
            mn = max(m, s.max()); al = 0.0 if m == -np.inf else np.exp(m - mn)
            pt = np.exp(s - mn).astype(np.float32).astype(np.float64)
            l = al * l + pt.sum(); o = al * o + fq(pt) @ vf[0, 0, k0:k0 + 64]; m = mn
        assert np.allclose(r["O"][0, 0, i], o / l, rtol=0, atol=1e-12)
        assert np.isclose(r["L"][0, 0, i], m + np.log(l), rtol=0, atol=1e-12)


def test_rows_without_any_key_give_zero_output():
    q, k, v = _rand(1, 1, 1, 256, 32, seed=86)
    bm = np.ones((1, 1, 2, 2), np.uint8); bm[0, 0, 1, :] = 0
    r = oracle.fwd(q, k, v, False, 64, block_mask=bm)
    assert not r["O"][0, 0, 128:].any() and np.isneginf(r["L"][0, 0, 128:]).all()
    assert np.isfinite(r["L"][0, 0, :128]).all()
