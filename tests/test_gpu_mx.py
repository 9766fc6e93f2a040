"""MX variant on the GPU: attnqat_quantize_mx bit exact against the oracle's MX phi, and
attnqat_fwd_infer_mx (Alg. 1 on the scaled FP4 matrix instruction) against the oracle's MX forward."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from tests.gpu_util import f32, host, max_abs, random_inputs, rel_l2, to_dev

pytestmark = pytest.mark.gpu

TOL = 2e-3            # rel-L2 bar for O (bf16 output rounding alone is about 1.7e-3)


def _canon(c):
    """-0 and +0 are the same value: clear the sign of zero codes."""
    lo, hi = c & 15, c >> 4
    lo = np.where((lo & 7) == 0, 0, lo); hi = np.where((hi & 7) == 0, 0, hi)
    return lo | (hi << 4)


def _compare(bits, axis):
    import paper_2603_00040_amd as aq
    codes, scales, xf = aq.attnqat_quantize_mx(to_dev(bits), axis=axis)
    torch.cuda.synchronize()
    x = W.bf16_bits_to_f32(bits)
    if axis == 0:
        pc, ps, pxf = oracle.phi_mx(x)
    else:
        pc, ps, pxf = oracle.phi_mx(np.ascontiguousarray(np.swapaxes(x, -1, -2)))
        pxf = np.ascontiguousarray(np.swapaxes(pxf, -1, -2))
    gc = codes.cpu().numpy(); gs = scales.cpu().numpy()
    assert gc.shape == pc.shape and gs.shape == ps.shape
    assert np.array_equal(gs, ps), f"{(gs != ps).sum()} scale bytes differ"
    assert np.array_equal(_canon(gc), _canon(pc)), f"{(_canon(gc) != _canon(pc)).sum()} code bytes differ"
    assert np.array_equal(xf.to(torch.float32).cpu().numpy(), pxf), "dequantized copy differs"


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("d", [64, 128])
def test_quantize_all_bf16_magnitudes_and_ties(d, axis):
    """Every finite bf16 bit pattern appears; blocks mix magnitudes so ties and the scale boundary occur."""
    rng = np.random.default_rng(0)
    allb = np.arange(1 << 16, dtype=np.uint16)
    allb = allb[(allb & 0x7F80) != 0x7F80]
    L = 300                                   # 300 = 9 * 32 + 12: a short last block along the sequence
    n = 2 * L * d
    bits = rng.choice(allb, size=n).astype(np.uint16)
    base = rng.integers(90, 160, size=n // 32).repeat(32).astype(np.uint16)
    jitter = rng.integers(0, 4, size=n).astype(np.uint16)
    bits = (bits & 0x807F) | ((base + jitter) << 7)
    x = bits.reshape(1, 2, L, d)
    # exact ties: a 6 pins the scale at 1, the other elements sit on the E2M1 midpoints; and block maxima
    # just below / at / above 1.5 * 2^x, where the scale steps
    tie = np.zeros(32, np.float32)
    tie[:15] = [6.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, -0.25, -0.75, -1.25, -1.75, -2.5, -3.5, -5.0]
    edge = np.zeros((3, 32), np.float32)
    edge[0, 0] = 1.4921875; edge[1, 0] = 1.5; edge[2, 0] = 1.5078125        # bf16 neighbours of 1.5
    edge[:, 1:8] = [0.1, 0.2, 0.3, 0.4, 0.6, 0.9, 1.2]
    if axis == 0:
        x[0, 0, 0, :32] = W.f32_to_bf16_bits(tie)
        for i in range(3):
            x[0, 0, 1 + i, :32] = W.f32_to_bf16_bits(edge[i])
    else:
        x[0, 0, :32, 0] = W.f32_to_bf16_bits(tie)
        for i in range(3):
            x[0, 0, :32, 1 + i] = W.f32_to_bf16_bits(edge[i])
    _compare(np.ascontiguousarray(x), axis)


@pytest.mark.parametrize("axis", [0, 1])
def test_quantize_tiny_huge_zero_blocks(axis):
    x = np.zeros((1, 1, 77, 64), np.float32)
    r = np.random.default_rng(1)
    x[0, 0, 0, :32] = 1e-38                                   # below 6 * 2^-126: the floor scale
    x[0, 0, 1, :32] = 3e38
    x[0, 0, 2, :32] = -0.0
    x[0, 0, 3, :] = r.standard_normal(64) * 1e-3
    x[0, 0, 40:, :] = r.standard_normal((37, 64)) * 50
    _compare(W.f32_to_bf16_bits(x).reshape(x.shape), axis)


def _run(B, Hq, Hkv, L, d, causal, seed, **kw):
    import paper_2603_00040_amd as aq
    x = random_inputs(B, Hq, Hkv, L, d, seed, **kw)
    q, k, v = (to_dev(x[n]) for n in "qkv")
    o, lse = aq.attnqat_fwd_infer_mx(q, k, v, causal)
    torch.cuda.synchronize()
    ref = oracle.fwd_mx(f32(x["q"]), f32(x["k"]), f32(x["v"]), causal, aq.block_k())
    r = {"O": rel_l2(host(o), ref["O"]), "L": max_abs(host(lse), ref["L"]), "Omax": max_abs(host(o), ref["O"])}
    print(f"fwd_mx B{B} Hq{Hq} Hkv{Hkv} L{L} d{d} causal{int(causal)}: {r}", flush=True)
    assert r["O"] <= TOL and r["L"] <= 2e-5 * max(1.0, np.abs(ref["L"]).max())


def test_fwd_mx_tiny_ref_config():
    _run(1, 2, 2, 256, 64, False, seed=0)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("L", [1, 31, 64, 65, 300, 520])
def test_fwd_mx_ragged_lengths_d128_gqa(L, causal):
    _run(2, 4, 2, L, 128, causal, seed=100 + L, k_chan=4)


@pytest.mark.parametrize("causal", [False, True])
def test_fwd_mx_d64_heavy_tails(causal):
    _run(1, 3, 1, 333, 64, causal, seed=7, dist="t3", scale=0.5, tok_mod=50)


def test_fwd_mx_argument_errors():
    import paper_2603_00040_amd as aq
    L = aq.lib()
    q = torch.zeros((1, 2, 64, 128), dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(q); lse = torch.empty((1, 2, 64), device="cuda")
    need = aq.workspace_bytes(aq.WS_FWD_INFER_MX, 1, 2, 2, 64, 128)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    args = lambda d=128, hkv=2, dt=0, wsb=need, qp=q.data_ptr(): (
        qp, q.data_ptr(), q.data_ptr(), 1, 2, hkv, 64, d, 0, dt, o.data_ptr(), lse.data_ptr(),
        ws.data_ptr(), wsb, None)
    assert L.attnqat_fwd_infer_mx(*args()) == aq.OK
    assert L.attnqat_fwd_infer_mx(*args(d=96)) == aq.ESHAPE
    assert L.attnqat_fwd_infer_mx(*args(hkv=3)) == aq.ESHAPE
    assert L.attnqat_fwd_infer_mx(*args(dt=1)) == aq.EDTYPE
    assert L.attnqat_fwd_infer_mx(*args(wsb=need - 1)) == aq.EWORKSPACE
    assert L.attnqat_fwd_infer_mx(*args(qp=None)) == aq.EINVAL
    assert L.attnqat_quantize_mx(q.data_ptr(), 1, 2, 64, 128, 0, 2, o.data_ptr(), None, None, None) == aq.EINVAL
    torch.cuda.synchronize()


# ---------------------------------------------------------------- training forward and backward in the MX format

FLIP_BAR = 1e-4       # fraction of P-tilde^F elements that may differ from the oracle's
F16_FLUSH = 2.0 ** -25   # the 16-bit path holds P-tilde^F in fp16: below 2^-24 a value is rounded to a multiple of 2^-24


def _run_train(B, Hq, Hkv, L, d, causal, seed, **kw):
    import paper_2603_00040_amd as aq
    x = random_inputs(B, Hq, Hkv, L, d, seed, **kw)
    q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
    o, lse, ohp = aq.attnqat_fwd_mx(q, k, v, causal)
    oi, lsei = aq.attnqat_fwd_infer_mx(q, k, v, causal)
    dq, dk, dv = aq.attnqat_bwd_mx(q, k, v, do, lse, ohp, causal)
    torch.cuda.synchronize()
    fq, fk, fv, fdo = (f32(x[n]) for n in ("q", "k", "v", "do"))
    rf = oracle.fwd(fq, fk, fv, causal, aq.block_k(), scale_mode=oracle.MX)
    rb = oracle.bwd(fq, fk, fv, fdo, rf["L"], rf["Op"], causal, scale_mode=oracle.MX)
    r = {"O": rel_l2(host(o), rf["O"]), "Op": rel_l2(host(ohp), rf["Op"]), "L": max_abs(host(lse), rf["L"])}
    r.update({n: rel_l2(host(t), rb[n], zero_rms=1e-2) for n, t in (("dQ", dq), ("dK", dk), ("dV", dv))})
    # Eq. 3 == Eq. 4: the FP4-instruction forward and the 16-bit forward compute the same O and L
    r["O_vs_fp4_path"] = max_abs(host(o), host(oi)); r["L_vs_fp4_path"] = max_abs(host(lse), host(lsei))
    print(f"mx train B{B} Hq{Hq} Hkv{Hkv} L{L} d{d} causal{int(causal)}: " + " ".join(f"{n} {a:.2e}" for n, a in r.items()), flush=True)
    assert r["O"] <= TOL and r["Op"] <= 2e-4 and r["L"] <= 2e-5 * max(1.0, np.abs(rf["L"]).max())
    for n in ("dQ", "dK", "dV"):
        assert r[n] <= TOL, (n, r[n])
    scale = max(1.0, float(np.abs(rf["O"]).max()))
    assert r["O_vs_fp4_path"] <= 2.0 ** -7 * scale and r["L_vs_fp4_path"] <= 1e-4       # one bf16 rounding step of O apart at most


def test_mx_train_tiny_ref_config():
    _run_train(1, 2, 2, 256, 64, False, seed=0)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("L", [1, 31, 64, 129, 300])
def test_mx_train_ragged_lengths_d128_gqa(L, causal):
    _run_train(2, 4, 2, L, 128, causal, seed=300 + L, k_chan=4)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(2, 4, 2, 129, 128), (1, 3, 1, 333, 64), (1, 2, 1, 700, 128)])
def test_mx_train_eight_wave_backward(shape, causal):
    """The 256-row / 256-key workgroups of the backward passes (large problems pick them by themselves): against
    the oracle, and the same bits as the 128-row shape."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = shape
    try:
        aq.debug_bwd_waves(8)
        _run_train(B, Hq, Hkv, L, d, causal, seed=340 + L, k_chan=2)
        x = random_inputs(B, Hq, Hkv, L, d, 341 + L)
        q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
        o, lse, ohp = aq.attnqat_fwd_mx(q, k, v, causal)
        g8 = aq.attnqat_bwd_mx(q, k, v, do, lse, ohp, causal)
        aq.debug_bwd_waves(4)
        g4 = aq.attnqat_bwd_mx(q, k, v, do, lse, ohp, causal)
        torch.cuda.synchronize()
    finally:
        aq.debug_bwd_waves(0)
    for a, b in zip(g4, g8):
        assert torch.equal(a, b)


@pytest.mark.parametrize("causal", [False, True])
def test_mx_train_d64_heavy_tails(causal):
    _run_train(1, 3, 1, 333, 64, causal, seed=9, dist="t3", scale=0.5, tok_mod=50)


@pytest.mark.parametrize("causal", [False, True])
def test_mx_P_code_flips(causal):
    """The dequantized P-tilde^F entering the O update of attnqat_fwd_mx, element by element."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = 1, 2, 1, 640, 128
    x = random_inputs(B, Hq, Hkv, L, d, seed=11, k_chan=4)
    q, k, v = (to_dev(x[n]) for n in "qkv")
    bad = tot = 0
    for row0 in (0, 512):
        _, _, p = aq.attnqat_debug_fwd_p_mx(q, k, v, causal, row0)
        torch.cuda.synchronize()
        nrow = min(128, L - row0)
        rows = oracle.flat_rows(B, Hq, L, [(0, h, row0 + i) for h in range(Hq) for i in range(nrow)])
        ref = oracle.fwd(f32(x["q"]), f32(x["k"]), f32(x["v"]), causal, aq.block_k(), scale_mode=oracle.MX,
                         rows=rows, dump_p=True)
        got = p.cpu().numpy()[0, :, :nrow].reshape(-1, L)
        bad += int((np.abs(got.astype(np.float64) - ref["P"]) > F16_FLUSH).sum()); tot += got.size
    print(f"MX P flips causal{int(causal)}: {bad} of {tot} ({bad / tot:.2e})", flush=True)
    assert bad / tot < FLIP_BAR


# ---------------------------------------------------------------- mixed recipe: FP4 Q K^T, MXFP8 P V

@pytest.mark.parametrize("d", [64, 128])
def test_quantize_mxfp8_bit_exact(d):
    import paper_2603_00040_amd as aq
    rng = np.random.default_rng(50)
    allb = np.arange(1 << 16, dtype=np.uint16)
    allb = allb[(allb & 0x7F80) != 0x7F80]
    L = 300
    n = 2 * L * d
    bits = rng.choice(allb, size=n).astype(np.uint16)
    base = rng.integers(90, 160, size=n // 32).repeat(32).astype(np.uint16)
    bits = (bits & 0x807F) | ((base + rng.integers(0, 6, size=n).astype(np.uint16)) << 7)
    x = bits.reshape(1, 2, L, d)
    # a 448 pins the scale at 1: E4M3 midpoints (ties) and their bf16 neighbours below it; maxima around 1.75 * 2^x
    tie = np.zeros(32, np.float32)
    tie[:12] = [448.0, 0.0009765625, 0.0029296875, 17.0, 19.0, 208.0, 240.0, 416.0, -17.0, -19.0, -208.0, -416.0]
    x[0, 0, :32, 0] = W.f32_to_bf16_bits(tie)
    for i, top in enumerate((1.7421875, 1.75, 1.7578125)):
        col = np.zeros(32, np.float32); col[0] = top; col[1:6] = [0.1, 0.3, 0.7, 1.1, 1.6]
        x[0, 0, :32, 1 + i] = W.f32_to_bf16_bits(col)
    x = np.ascontiguousarray(x)
    codes, scales, xf = aq.attnqat_quantize_mxfp8(to_dev(x))
    torch.cuda.synchronize()
    xs = np.ascontiguousarray(np.swapaxes(W.bf16_bits_to_f32(x), -1, -2))
    pc, ps, pxf = oracle.phi_mx8(xs)
    gc, gs = codes.cpu().numpy(), scales.cpu().numpy()
    assert gc.shape == pc.shape and gs.shape == ps.shape
    assert np.array_equal(gs, ps), f"{(gs != ps).sum()} scale bytes differ"
    canon = lambda c: np.where((c & 0x7F) == 0, 0, c)                  # -0 and +0 are the same value
    assert np.array_equal(canon(gc), canon(pc)), f"{(canon(gc) != canon(pc)).sum()} code bytes differ"
    # the bf16 copy rounds 4-bit-significand values times a power of two: exact
    want = np.ascontiguousarray(np.swapaxes(pxf, -1, -2))
    assert np.array_equal(xf.to(torch.float32).cpu().numpy(), want)


def _run_fp8pv(B, Hq, Hkv, L, d, causal, seed, **kw):
    import paper_2603_00040_amd as aq
    x = random_inputs(B, Hq, Hkv, L, d, seed, **kw)
    q, k, v = (to_dev(x[n]) for n in "qkv")
    o, lse = aq.attnqat_fwd_infer_mx_fp8pv(q, k, v, causal)
    torch.cuda.synchronize()
    ref = oracle.fwd(f32(x["q"]), f32(x["k"]), f32(x["v"]), causal, aq.block_k(), scale_mode=oracle.MX_FP8PV)
    r = {"O": rel_l2(host(o), ref["O"]), "L": max_abs(host(lse), ref["L"]), "Omax": max_abs(host(o), ref["O"])}
    print(f"fwd_mx_fp8pv B{B} Hq{Hq} Hkv{Hkv} L{L} d{d} causal{int(causal)}: {r}", flush=True)
    assert r["O"] <= TOL and r["L"] <= 2e-5 * max(1.0, np.abs(ref["L"]).max())


def test_fp8pv_tiny_ref_config():
    _run_fp8pv(1, 2, 2, 256, 64, False, seed=0)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("L", [1, 31, 65, 300, 520])
def test_fp8pv_ragged_lengths_d128_gqa(L, causal):
    _run_fp8pv(2, 4, 2, L, 128, causal, seed=400 + L, k_chan=4)


@pytest.mark.parametrize("causal", [False, True])
def test_fp8pv_d64_heavy_tails(causal):
    _run_fp8pv(1, 3, 1, 333, 64, causal, seed=7, dist="t3", scale=0.5, tok_mod=50)
