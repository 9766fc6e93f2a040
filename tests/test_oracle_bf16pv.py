"""Pins of the oracle's mixed recipe "NVFP4 Q K^T, BF16 P V" (Sec. 2.5, "Bypassing the softmax bottleneck": the
quantization of P is what makes the all-FP4 kernel slow, so P and V stay in 16 bits).  Reading: Q and K are NVFP4
fake-quantized as everywhere, V is the bf16 input itself, P-tilde is rounded to bf16 (nearest even) where the all-FP4
recipe block-quantizes it; l, L and the running maximum are untouched."""
import numpy as np
import pytest
import torch

import oracle
from tests import indep
from tests.test_oracle_fwd import _rand, _textbook

BP = oracle.BF16_PV


def _bf16(a):      # the library's own rounding
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


@pytest.mark.parametrize("causal", [False, True])
def test_matches_independent_rowwise_transcription(causal):
    q, k, v = _rand(1, 4, 2, 150, 32, seed=90, outlier=True)
    r = oracle.fwd(q, k, v, causal, 64, scale_mode=BP)
    qf, kf = indep.fake_quant_np(q), indep.fake_quant_np(k)
    for h in range(4):
        O, Op, L = indep.attn_fwd_rowwise_np(qf[0, h], kf[0, h // 2], v[0, h // 2].astype(np.float64), causal, 64, fq=_bf16)
        assert np.allclose(r["O"][0, h], O, rtol=0, atol=1e-12)
        assert np.allclose(r["L"][0, h], L, rtol=0, atol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
def test_L_is_logsumexp_and_O_is_textbook_up_to_the_rounding_of_P(causal):
    q, k, v = _rand(2, 4, 2, 200, 64, seed=91)
    r = oracle.fwd(q, k, v, causal, 64, scale_mode=BP)
    O, L = _textbook(indep.fake_quant_np(q), indep.fake_quant_np(k), v, causal)
    assert np.allclose(r["L"], L, rtol=0, atol=1e-6)
    # every P is off by at most 2^-9 relative, so every output element by at most 2^-9 of sum |P V| / l <= max |V|
    assert np.abs(r["O"] - O).max() <= 2.0 ** -9 * np.abs(v).max()
    assert 1e-5 < np.linalg.norm(r["O"] - O) / np.linalg.norm(O) < 3e-3       # and it is not simply the textbook result


def test_dumped_P_is_bf16_and_closer_to_the_unquantized_P_than_fp4():
    q, k, v = _rand(1, 2, 1, 192, 32, seed=92, outlier=True)
    rows = np.arange(192, dtype=np.int64)
    bp = oracle.fwd(q, k, v, False, 64, scale_mode=BP, rows=rows, dump_p=True)
    assert np.array_equal(bp["P"], _bf16(bp["P"]).astype(np.float32))
    # V is not quantized in this recipe: compare with the all-NVFP4 recipe on an already representable V
    vf = oracle.fake_quant(v)
    ref = oracle.fwd(q, k, vf, False, 64, quant_p=False)["O"]
    e_bf = np.linalg.norm(oracle.fwd(q, k, vf, False, 64, scale_mode=BP)["O"] - ref)
    e_f4 = np.linalg.norm(oracle.fwd(q, k, vf, False, 64)["O"] - ref)
    assert e_bf < 0.05 * e_f4


def test_backward_refuses_the_inference_recipe():
    q, k, v = _rand(1, 2, 1, 64, 32, seed=93)
    f = oracle.fwd(q, k, v, False, 64)
    with pytest.raises(ValueError):
        oracle.bwd(q, k, v, q, f["L"], f["Op"], False, scale_mode=BP)
