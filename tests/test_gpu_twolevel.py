"""Two-level quantization of P (attnqat_fwd_opt / attnqat_bwd_opt with OPT_TWO_LEVEL_P) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from tests.gpu_util import f32, host, max_abs, random_inputs, rel_l2, to_dev

pytestmark = pytest.mark.gpu

TOL, FLIP_BAR = 2e-3, 1e-4
TL = oracle.TWO_LEVEL_P


def _run(B, Hq, Hkv, L, d, causal, seed, options=None, **kw):
    import paper_2603_00040_amd as aq
    options = aq.OPT_TWO_LEVEL_P if options is None else options
    x = random_inputs(B, Hq, Hkv, L, d, seed, **kw)
    q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
    o, lse, ohp = aq.attnqat_fwd_opt(q, k, v, causal, options)
    oi, lsei, _ = aq.attnqat_fwd_opt(q, k, v, causal, options, train=False)
    dq, dk, dv = aq.attnqat_bwd_opt(q, k, v, do, lse, ohp, causal, options)
    torch.cuda.synchronize()
    fq, fk, fv, fdo = (f32(x[n]) for n in ("q", "k", "v", "do"))
    if options & aq.OPT_SMOOTH_K:
        fk = oracle.smooth_k(fk)
    rf = oracle.fwd(fq, fk, fv, causal, aq.block_k(), scale_mode=TL)
    rb = oracle.bwd(fq, fk, fv, fdo, rf["L"], rf["Op"], causal, scale_mode=TL)
    r = {"O": rel_l2(host(o), rf["O"]), "Op": rel_l2(host(ohp), rf["Op"]), "L": max_abs(host(lse), rf["L"])}
    r.update({n: rel_l2(host(t), rb[n], zero_rms=1e-2) for n, t in (("dQ", dq), ("dK", dk), ("dV", dv))})
    print(f"two-level B{B} Hq{Hq} Hkv{Hkv} L{L} d{d} causal{int(causal)} opt{options}: " + " ".join(f"{n} {a:.2e}" for n, a in r.items()), flush=True)
    assert r["O"] <= TOL and r["Op"] <= 2e-4 and r["L"] <= 2e-5 * max(1.0, np.abs(rf["L"]).max())
    for n in ("dQ", "dK", "dV"):
        assert r[n] <= TOL, (n, r[n])
    assert torch.equal(o, oi) and torch.equal(lse, lsei)


def test_twolevel_tiny_ref_config():
    _run(1, 2, 2, 256, 64, False, seed=0)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("L", [1, 65, 300])
def test_twolevel_ragged_lengths_d128_gqa(L, causal):
    _run(2, 4, 2, L, 128, causal, seed=600 + L, k_chan=4)


@pytest.mark.parametrize("causal", [False, True])
def test_twolevel_d64_heavy_tails(causal):
    # heavy tails: most 64-key tiles of a row sit far below the row maximum, where the plain method flushes P to 0
    _run(1, 3, 1, 333, 64, causal, seed=9, dist="t3", scale=0.5, tok_mod=50)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(2, 4, 2, 129, 128), (1, 3, 1, 333, 64), (1, 2, 1, 700, 128)])
def test_twolevel_eight_wave_backward(shape, causal):
    """The 256-row / 256-key workgroups of the backward passes (large problems pick them by themselves): against
    the oracle, and the same bits as the 128-row shape.  The pairs of waves that exchange row maxima stay pairs."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = shape
    try:
        aq.debug_bwd_waves(8)
        _run(B, Hq, Hkv, L, d, causal, seed=640 + L, k_chan=2)
        x = random_inputs(B, Hq, Hkv, L, d, 641 + L)
        q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
        o, lse, ohp = aq.attnqat_fwd_opt(q, k, v, causal, aq.OPT_TWO_LEVEL_P)
        g8 = aq.attnqat_bwd_opt(q, k, v, do, lse, ohp, causal, aq.OPT_TWO_LEVEL_P)
        aq.debug_bwd_waves(4)
        g4 = aq.attnqat_bwd_opt(q, k, v, do, lse, ohp, causal, aq.OPT_TWO_LEVEL_P)
        torch.cuda.synchronize()
    finally:
        aq.debug_bwd_waves(0)
    for a, b in zip(g4, g8):
        assert torch.equal(a, b)


def test_twolevel_with_k_smoothing():
    import paper_2603_00040_amd as aq
    _run(1, 4, 2, 200, 128, True, seed=21, options=aq.OPT_TWO_LEVEL_P | aq.OPT_SMOOTH_K, k_chan=4)


@pytest.mark.parametrize("causal", [False, True])
def test_twolevel_P_code_flips(causal):
    """The dequantized P-tilde^F (row factor included) entering the O update, element by element."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = 1, 2, 1, 640, 128
    x = random_inputs(B, Hq, Hkv, L, d, seed=11, dist="t3", scale=0.5)
    q, k, v = (to_dev(x[n]) for n in "qkv")
    bad = tot = nonzero = plain_nonzero = 0
    for row0 in (0, 512):
        _, _, p = aq.attnqat_debug_fwd_p_opt(q, k, v, causal, row0, aq.OPT_TWO_LEVEL_P)
        _, _, p0 = aq.attnqat_debug_fwd_p(q, k, v, causal, row0)
        torch.cuda.synchronize()
        nrow = min(128, L - row0)
        rows = oracle.flat_rows(B, Hq, L, [(0, h, row0 + i) for h in range(Hq) for i in range(nrow)])
        ref = oracle.fwd(f32(x["q"]), f32(x["k"]), f32(x["v"]), causal, aq.block_k(), scale_mode=TL, rows=rows, dump_p=True)
        got = p.cpu().numpy()[0, :, :nrow].reshape(-1, L)
        bad += int((got != ref["P"]).sum()); tot += got.size
        nonzero += int((got != 0).sum()); plain_nonzero += int((p0.cpu().numpy()[0, :, :nrow] != 0).sum())
    print(f"two-level P flips causal{int(causal)}: {bad} of {tot} ({bad / tot:.2e}); non-zero P-tilde^F: {nonzero} with the row factor, "
          f"{plain_nonzero} without", flush=True)
    assert bad / tot < FLIP_BAR
    assert nonzero > plain_nonzero                       # what the option is for: fewer values flushed to zero
