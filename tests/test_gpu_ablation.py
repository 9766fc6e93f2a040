"""attnqat_bwd_ablation (Sec. 3.2, Exp. 7 and Exp. 8) against the oracle's switches."""
import numpy as np
import pytest
import torch

import oracle
from tests.gpu_util import f32, host, random_inputs, rel_l2, to_dev

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _setup(causal, seed=41, B=1, Hq=4, Hkv=2, L=300, d=128):
    import paper_2603_00040_amd as aq
    x = random_inputs(B, Hq, Hkv, L, d, seed, k_chan=4)
    t = {n: to_dev(x[n]) for n in ("q", "k", "v", "do")}
    o, lse, ohp = aq.attnqat_fwd(t["q"], t["k"], t["v"], causal)
    torch.cuda.synchronize()
    return aq, x, t, o, lse, ohp


@pytest.mark.parametrize("causal", [False, True])
def test_no_ablation_is_the_backward(causal):
    aq, x, t, o, lse, ohp = _setup(causal)
    ref = aq.attnqat_bwd(t["q"], t["k"], t["v"], t["do"], lse, ohp, causal)
    got = aq.attnqat_bwd_ablation(t["q"], t["k"], t["v"], t["do"], lse, ohp, None, causal, 0)
    torch.cuda.synchronize()
    for a, b in zip(ref, got):
        assert torch.equal(a, b)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("ablation", [1, 2, 3])
def test_ablations_match_the_oracle(ablation, causal):
    aq, x, t, o, lse, ohp = _setup(causal)
    dq, dk, dv = aq.attnqat_bwd_ablation(t["q"], t["k"], t["v"], t["do"], lse, ohp, o, causal, ablation)
    torch.cuda.synchronize()
    fq, fk, fv, fdo = (f32(x[n]) for n in ("q", "k", "v", "do"))
    # both sides get the same L and the same O / O' (the GPU forward's), so only the backward is compared
    acc = host(o) if ablation & aq.ABL_D_FROM_O else host(ohp)
    rb = oracle.bwd(fq, fk, fv, fdo, host(lse), acc, causal, quant_p=not (ablation & aq.ABL_P_UNQUANTIZED))
    for n, g in (("dQ", dq), ("dK", dk), ("dV", dv)):
        e = rel_l2(host(g), rb[n])
        print(f"ablation {ablation} causal {int(causal)}: {n} rel-L2 {e:.2e}", flush=True)
        assert e <= TOL, (n, e)


def test_D_from_the_low_precision_output_breaks_the_row_sums():
    """sum_j dK_j = sum_i (rowsum dS_i) Q^F_i: rounding noise with D from O', large with D from O."""
    aq, x, t, o, lse, ohp = _setup(False)
    _, dk_good, _ = aq.attnqat_bwd(t["q"], t["k"], t["v"], t["do"], lse, ohp, False)
    dq_bad, dk_bad, _ = aq.attnqat_bwd_ablation(t["q"], t["k"], t["v"], t["do"], lse, ohp, o, False, aq.ABL_D_FROM_O)
    torch.cuda.synchronize()
    good = float(dk_good.float().sum(2).abs().max())
    bad = float(dk_bad.float().sum(2).abs().max())
    print(f"max |sum_j dK_j|: D from O' {good:.3e}, D from O {bad:.3e}", flush=True)
    assert bad > 5.0 * good
