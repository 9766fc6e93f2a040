"""attnqat_fwd / attnqat_fwd_infer against the oracle (Alg. 1, Alg. 2), small and ragged cases."""
import numpy as np
import pytest
import torch

import oracle
from tests.gpu_util import check_bf16_output, f32, host, max_abs, random_inputs, rel_l2, to_dev

pytestmark = pytest.mark.gpu

TOL = 2e-3            # rel-L2 bar for O (bf16 output rounding alone is about 1.7e-3; check_bf16_output adds the bars
                      # that do not contain that rounding, and a bound on the largest element error)
FLIP_BAR = 1e-4       # fraction of P-tilde^F elements that may differ from the oracle's


def _run(B, Hq, Hkv, L, d, causal, seed, **kw):
    import paper_2603_00040_amd as aq
    x = random_inputs(B, Hq, Hkv, L, d, seed, **kw)
    q, k, v = (to_dev(x[n]) for n in "qkv")
    o, lse, ohp = aq.attnqat_fwd(q, k, v, causal)
    oi, lsei = aq.attnqat_fwd_infer(q, k, v, causal)
    torch.cuda.synchronize()
    ref = oracle.fwd(f32(x["q"]), f32(x["k"]), f32(x["v"]), causal, aq.block_k())
    r = {"O": rel_l2(host(o), ref["O"]), "Op": rel_l2(host(ohp), ref["Op"]),
         "L": max_abs(host(lse), ref["L"]), "Omax": max_abs(host(o), ref["O"])}
    print(f"fwd B{B} Hq{Hq} Hkv{Hkv} L{L} d{d} causal{int(causal)}: {r}", flush=True)
    check_bf16_output("O", host(o), ref["O"], TOL)
    assert r["Op"] <= 2e-4 and r["L"] <= 2e-5 * max(1.0, np.abs(ref["L"]).max())
    # Eq. 3 == Eq. 4: the inference entry point returns the same O and L
    assert torch.equal(o, oi) and torch.equal(lse, lsei)
    return x, ref


def test_tiny_ref_config():
    _run(1, 2, 2, 256, 64, False, seed=0)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("L", [1, 63, 64, 65, 300, 520])
def test_ragged_lengths_d128_gqa(L, causal):
    _run(2, 4, 2, L, 128, causal, seed=100 + L, k_chan=4)


@pytest.mark.parametrize("causal", [False, True])
def test_d64_heavy_tails(causal):
    _run(1, 3, 1, 333, 64, causal, seed=7, dist="t3", scale=0.5, tok_mod=50)


@pytest.mark.parametrize("causal", [False, True])
def test_P_code_flips(causal):
    """The dequantized P-tilde^F entering the O update, element by element."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = 1, 2, 1, 640, 128
    x = random_inputs(B, Hq, Hkv, L, d, seed=11, k_chan=4)
    q, k, v = (to_dev(x[n]) for n in "qkv")
    bad = tot = 0
    for row0 in (0, 512):
        _, _, p = aq.attnqat_debug_fwd_p(q, k, v, causal, row0)
        torch.cuda.synchronize()
        nrow = min(128, L - row0)
        rows = oracle.flat_rows(B, Hq, L, [(0, h, row0 + i) for h in range(Hq) for i in range(nrow)])
        ref = oracle.fwd(f32(x["q"]), f32(x["k"]), f32(x["v"]), causal, aq.block_k(), rows=rows, dump_p=True)
        got = p.cpu().numpy()[0, :, :nrow].reshape(-1, L)
        bad += int((got != ref["P"]).sum()); tot += got.size
    print(f"P flips causal{int(causal)}: {bad} of {tot} ({bad / tot:.2e})", flush=True)
    assert bad / tot < FLIP_BAR


def test_argument_errors():
    import paper_2603_00040_amd as aq
    L = aq.lib()
    q = torch.zeros((1, 2, 64, 128), dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(q); lse = torch.empty((1, 2, 64), device="cuda")
    ws = torch.empty(aq.workspace_bytes(aq.WS_FWD_INFER, 1, 2, 2, 64, 128), dtype=torch.uint8, device="cuda")
    f = lambda *a: L.attnqat_fwd_infer(*a)
    args = lambda d=128, hkv=2, dt=0, wsb=ws.numel(), qp=q.data_ptr(): (
        qp, q.data_ptr(), q.data_ptr(), 1, 2, hkv, 64, d, 0, dt, o.data_ptr(), lse.data_ptr(),
        ws.data_ptr(), wsb, None)
    assert f(*args()) == aq.OK
    assert f(*args(d=96)) == aq.ESHAPE
    assert f(*args(hkv=3)) == aq.ESHAPE
    assert f(*args(dt=1)) == aq.EDTYPE
    assert f(*args(wsb=16)) == aq.EWORKSPACE
    assert f(*args(qp=None)) == aq.EINVAL
    assert aq.workspace_bytes(aq.WS_FWD, 1, 2, 2, 64, 96) == 0
    torch.cuda.synchronize()
