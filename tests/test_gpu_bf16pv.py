"""attnqat_fwd_infer_bf16pv (Sec. 2.5: NVFP4 Q K^T with BF16 P V) against the oracle's mode of the same recipe."""
import numpy as np
import pytest
import torch

import oracle
from tests.gpu_util import bf16_spacing, check_bf16_output, f32, host, max_abs, random_inputs, to_dev

pytestmark = pytest.mark.gpu

TOL = 2e-3
# A P-tilde that the two sides compute one fp32 rounding apart (exp2 by the hardware's instruction against the oracle's
# correctly rounded one, and the rounding of s c - m c with |s c| up to 2^5: relative 2^-18) rounds to different bf16
# neighbours when a rounding boundary (spaced 2^-8 relative) lies between them: up to 2^-18 / 2^-8 = 1e-3 of the elements,
# each then off by exactly one bf16 spacing.  With FP4 blocks the boundaries are 2^6 times further apart.
FLIP_BAR = 2e-3


def _run(B, Hq, Hkv, L, d, causal, seed, **kw):
    import paper_2603_00040_amd as aq
    x = random_inputs(B, Hq, Hkv, L, d, seed, **kw)
    q, k, v = (to_dev(x[n]) for n in "qkv")
    o, lse = aq.attnqat_fwd_infer_bf16pv(q, k, v, causal)
    o2, lse2, none = aq.attnqat_fwd_opt(q, k, v, causal, aq.OPT_BF16_PV, train=False)
    _, lse_fp4 = aq.attnqat_fwd_infer(q, k, v, causal)
    torch.cuda.synchronize()
    ref = oracle.fwd(f32(x["q"]), f32(x["k"]), f32(x["v"]), causal, aq.block_k(), scale_mode=oracle.BF16_PV)
    print(f"bf16pv B{B} Hq{Hq} Hkv{Hkv} L{L} d{d} causal{int(causal)}: L {max_abs(host(lse), ref['L']):.2e}", flush=True)
    check_bf16_output("O", host(o), ref["O"], TOL)
    assert max_abs(host(lse), ref["L"]) <= 2e-5 * max(1.0, np.abs(ref["L"]).max())
    assert none is None and torch.equal(o, o2) and torch.equal(lse, lse2)
    assert torch.equal(lse, lse_fp4)          # the recipe leaves S, m and l alone
    return x, ref, host(o)


def test_tiny_ref_config():
    _run(1, 2, 2, 256, 64, False, seed=0)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("L", [1, 63, 65, 300, 520])
def test_ragged_lengths_d128_gqa(L, causal):
    _run(2, 4, 2, L, 128, causal, seed=300 + L, k_chan=4)


@pytest.mark.parametrize("causal", [False, True])
def test_d64_heavy_tails_and_v_is_not_quantized(causal):
    import paper_2603_00040_amd as aq
    x, ref, o = _run(1, 3, 1, 333, 64, causal, seed=17, dist="t3", scale=0.5, tok_mod=50)
    # with a quantized V the result is measurably different: the kernel did use V itself
    q, k = to_dev(x["q"]), to_dev(x["k"])
    _, _, vf = aq.attnqat_quantize(to_dev(x["v"]))
    o_vf, _ = aq.attnqat_fwd_infer_bf16pv(q, k, vf, causal)
    torch.cuda.synchronize()
    assert np.linalg.norm(host(o_vf) - ref["O"]) > 10 * np.linalg.norm(o - ref["O"])


@pytest.mark.parametrize("causal", [False, True])
def test_P_entering_the_product(causal):
    """The bf16 P-tilde entering the O update, element by element: equal to the oracle's or its bf16 neighbour."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = 1, 2, 1, 640, 128
    x = random_inputs(B, Hq, Hkv, L, d, seed=21, k_chan=4)
    q, k, v = (to_dev(x[n]) for n in "qkv")
    bad = tot = 0
    for row0 in (0, 512):
        _, _, p = aq.attnqat_debug_fwd_p_opt(q, k, v, causal, row0, aq.OPT_BF16_PV)
        torch.cuda.synchronize()
        nrow = min(128, L - row0)
        rows = oracle.flat_rows(B, Hq, L, [(0, h, row0 + i) for h in range(Hq) for i in range(nrow)])
        ref = oracle.fwd(f32(x["q"]), f32(x["k"]), f32(x["v"]), causal, aq.block_k(), rows=rows, dump_p=True,
                         scale_mode=oracle.BF16_PV)
        got = p.cpu().numpy()[0, :, :nrow].reshape(-1, L)
        diff = got != ref["P"]
        assert np.all(np.abs(got - ref["P"])[diff] <= bf16_spacing(np.maximum(got, ref["P"]))[diff])
        bad += int(diff.sum()); tot += got.size
    print(f"bf16 P neighbours causal{int(causal)}: {bad} of {tot} ({bad / tot:.2e})", flush=True)
    assert bad / tot < FLIP_BAR


def test_argument_errors():
    import paper_2603_00040_amd as aq
    q = torch.zeros((1, 2, 64, 128), dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(q); lse = torch.empty((1, 2, 64), device="cuda"); ohp = torch.empty((1, 2, 64, 128), device="cuda")
    ws = torch.empty(aq.workspace_bytes(aq.WS_BWD, 1, 2, 2, 64, 128), dtype=torch.uint8, device="cuda")
    p = q.data_ptr()
    fwd = lambda opt, hp: aq.lib().attnqat_fwd_opt(p, p, p, 1, 2, 2, 64, 128, 0, 0, opt, o.data_ptr(), lse.data_ptr(), hp,
                                                   ws.data_ptr(), ws.numel(), None)
    assert fwd(aq.OPT_BF16_PV, None) == aq.OK
    assert fwd(aq.OPT_BF16_PV | aq.OPT_SMOOTH_K, None) == aq.OK
    assert fwd(aq.OPT_BF16_PV, ohp.data_ptr()) == aq.EINVAL                       # no training forward
    assert fwd(aq.OPT_BF16_PV | aq.OPT_TWO_LEVEL_P, None) == aq.EINVAL
    assert aq.lib().attnqat_bwd_opt(p, p, p, p, lse.data_ptr(), ohp.data_ptr(), 1, 2, 2, 64, 128, 0, 0, aq.OPT_BF16_PV,
                                    o.data_ptr(), o.data_ptr(), o.data_ptr(), ws.data_ptr(), ws.numel(), None) == aq.EINVAL
    assert aq.lib().attnqat_fwd_infer_bf16pv(p, p, p, 1, 2, 2, 64, 128, 0, 0, o.data_ptr(), lse.data_ptr(), ws.data_ptr(), 16, None) \
        == aq.EWORKSPACE
    torch.cuda.synchronize()
