"""K smoothing option (attnqat_fwd_opt / attnqat_bwd_opt with OPT_SMOOTH_K) against the oracle run on the centred K."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from tests.gpu_util import f32, host, max_abs, random_inputs, rel_l2, to_dev

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _inputs(B, Hq, Hkv, L, d, seed, offset, **kw):
    x = random_inputs(B, Hq, Hkv, L, d, seed, **kw)
    k = f32(x["k"]) + np.float32(offset)                      # a common offset: what the smoothing removes
    x["k"] = W.f32_to_bf16_bits(k).reshape(k.shape)
    return x


def _run(B, Hq, Hkv, L, d, causal, seed, offset=1.5, **kw):
    import paper_2603_00040_amd as aq
    x = _inputs(B, Hq, Hkv, L, d, seed, offset, **kw)
    q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
    o, lse, ohp = aq.attnqat_fwd_opt(q, k, v, causal, aq.OPT_SMOOTH_K)
    oi, lsei, _ = aq.attnqat_fwd_opt(q, k, v, causal, aq.OPT_SMOOTH_K, train=False)
    dq, dk, dv = aq.attnqat_bwd_opt(q, k, v, do, lse, ohp, causal, aq.OPT_SMOOTH_K)
    torch.cuda.synchronize()
    fq, fk, fv, fdo = (f32(x[n]) for n in ("q", "k", "v", "do"))
    ks = oracle.smooth_k(fk)
    rf = oracle.fwd(fq, ks, fv, causal, aq.block_k())
    rb = oracle.bwd(fq, ks, fv, fdo, rf["L"], rf["Op"], causal)
    r = {"O": rel_l2(host(o), rf["O"]), "Op": rel_l2(host(ohp), rf["Op"]), "L": max_abs(host(lse), rf["L"])}
    r.update({n: rel_l2(host(t), rb[n], zero_rms=1e-2) for n, t in (("dQ", dq), ("dK", dk), ("dV", dv))})
    print(f"smooth-k B{B} Hq{Hq} Hkv{Hkv} L{L} d{d} causal{int(causal)}: " + " ".join(f"{n} {a:.2e}" for n, a in r.items()), flush=True)
    assert r["O"] <= TOL and r["Op"] <= 2e-4 and r["L"] <= 2e-5 * max(1.0, np.abs(rf["L"]).max())
    for n in ("dQ", "dK", "dV"):
        assert r[n] <= TOL, (n, r[n])
    assert torch.equal(o, oi) and torch.equal(lse, lsei)
    return x, rf


def test_smoothk_tiny_ref_config():
    _run(1, 2, 2, 256, 64, False, seed=0)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("L", [1, 65, 300])
def test_smoothk_ragged_lengths_d128_gqa(L, causal):
    _run(2, 4, 2, L, 128, causal, seed=500 + L, k_chan=4)


def test_smoothk_changes_and_improves_the_output():
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = 1, 2, 2, 512, 128
    x = _inputs(B, Hq, Hkv, L, d, 7, 4.0)
    q, k, v = (to_dev(x[n]) for n in "qkv")
    o_plain, _, _ = aq.attnqat_fwd(q, k, v, False)
    o_s, _, _ = aq.attnqat_fwd_opt(q, k, v, False, aq.OPT_SMOOTH_K)
    o_0, _, _ = aq.attnqat_fwd_opt(q, k, v, False, 0)
    torch.cuda.synchronize()
    assert torch.equal(o_plain, o_0)                          # no option bits: the plain forward
    ref = oracle.fwd(f32(x["q"]), f32(x["k"]), f32(x["v"]), False, 64, quant_qkv=False, quant_p=False)["O"]
    e_plain, e_s = rel_l2(host(o_plain), ref), rel_l2(host(o_s), ref)
    print(f"error against un-quantized attention: plain {e_plain:.3e}, with K smoothing {e_s:.3e}", flush=True)
    assert e_s < 0.7 * e_plain


def test_smoothk_option_errors():
    import paper_2603_00040_amd as aq
    L_ = aq.lib()
    q = torch.zeros((1, 2, 64, 128), dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(q); lse = torch.empty((1, 2, 64), device="cuda")
    need = aq.workspace_bytes(aq.WS_FWD, 1, 2, 2, 64, 128)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    call = lambda opt: L_.attnqat_fwd_opt(q.data_ptr(), q.data_ptr(), q.data_ptr(), 1, 2, 2, 64, 128, 0, 0, opt,
                                         o.data_ptr(), lse.data_ptr(), None, ws.data_ptr(), need, None)
    assert call(0) == aq.OK and call(1) == aq.OK and call(2) == aq.OK and call(4) == aq.OK          # 4: the bf16 P V recipe
    assert call(8) == aq.EINVAL and call(6) == aq.EINVAL and call(-1) == aq.EINVAL                  # unknown bit; 2 | 4 exclude each other
    torch.cuda.synchronize()
