"""Seeded random problem shapes (batch, head grouping, length, head size, mask, value distribution) through the NVFP4
forward and backward (Alg. 1-3) against the oracle, with both workgroup shapes of the backward passes: shapes nobody
picked by hand, sized so that the oracle takes a second or two each."""
import numpy as np
import pytest
import torch

import oracle
from tests.gpu_util import check_bf16_output, f32, host, max_abs, random_inputs, rel_l2, to_dev

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        d = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2, 3]))
        g = int(rng.choice([1, 2, 4]))
        b = int(rng.choice([1, 2]))
        # lengths around the edges of the 32-, 64-, 128- and 256-row tiles as often as anywhere else
        L = int(rng.choice([rng.integers(1, 40), rng.integers(120, 140), rng.integers(250, 262), rng.integers(300, 600)]))
        causal = bool(rng.integers(0, 2))
        dist = str(rng.choice(["normal", "t3"]))
        out.append(pytest.param(b, hkv * g, hkv, L, d, causal, dist, 1000 + 17 * i + seed,
                                id=f"B{b}-Hq{hkv * g}-Hkv{hkv}-L{L}-d{d}-{'causal' if causal else 'full'}-{dist}"))
    return out


@pytest.mark.parametrize("B,Hq,Hkv,L,d,causal,dist,seed", _shapes(14, 5))
def test_random_shape_forward_backward(B, Hq, Hkv, L, d, causal, dist, seed):
    import paper_2603_00040_amd as aq
    x = random_inputs(B, Hq, Hkv, L, d, seed, dist=dist, scale=0.5 if dist == "t3" else 1.0, k_chan=2)
    q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
    o, lse, ohp = aq.attnqat_fwd(q, k, v, causal)
    torch.cuda.synchronize()
    fq, fk, fv, fdo = (f32(x[n]) for n in ("q", "k", "v", "do"))
    rf = oracle.fwd(fq, fk, fv, causal, aq.block_k())
    check_bf16_output("O", host(o), rf["O"], TOL)
    assert rel_l2(host(ohp), rf["Op"]) <= 2e-4
    assert max_abs(host(lse), rf["L"]) <= 2e-5 * max(1.0, np.abs(rf["L"]).max())
    rb = oracle.bwd(fq, fk, fv, fdo, rf["L"], rf["Op"], causal)
    grads = {}
    try:
        for waves in (4, 8):
            aq.debug_bwd_waves(waves)
            grads[waves] = aq.attnqat_bwd(q, k, v, do, lse, ohp, causal)
            torch.cuda.synchronize()
    finally:
        aq.debug_bwd_waves(0)
    for n, t in zip(("dQ", "dK", "dV"), grads[4]):
        check_bf16_output(n, host(t), rb[n], TOL, zero_rms=1e-2)
    for a, b in zip(grads[4], grads[8]):
        assert torch.equal(a, b)
