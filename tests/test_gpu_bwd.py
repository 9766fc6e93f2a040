"""attnqat_bwd against the oracle (Alg. 3): GPU forward -> GPU backward vs oracle forward -> oracle backward."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from tests.gpu_util import check_bf16_output, f32, host, max_abs, random_inputs, rel_l2, to_dev

pytestmark = pytest.mark.gpu

TOL = 2e-3     # rel-L2 per tensor; the bf16 rounding of the outputs alone is about 1.7e-3 (check_bf16_output adds the
               # bars that do not contain that rounding, and a bound on the largest element error)


def _run(B, Hq, Hkv, L, d, causal, seed, **kw):
    import paper_2603_00040_amd as aq
    x = random_inputs(B, Hq, Hkv, L, d, seed, **kw)
    q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
    o, lse, ohp = aq.attnqat_fwd(q, k, v, causal)
    dq, dk, dv = aq.attnqat_bwd(q, k, v, do, lse, ohp, causal)
    torch.cuda.synchronize()
    fq, fk, fv, fdo = (f32(x[n]) for n in ("q", "k", "v", "do"))
    rf = oracle.fwd(fq, fk, fv, causal, aq.block_k())
    rb = oracle.bwd(fq, fk, fv, fdo, rf["L"], rf["Op"], causal)
    print(f"bwd B{B} Hq{Hq} Hkv{Hkv} L{L} d{d} causal{int(causal)}:", flush=True)
    for n, t in (("dQ", dq), ("dK", dk), ("dV", dv)):
        check_bf16_output(n, host(t), rb[n], TOL, zero_rms=1e-2)
    # determinism: no atomics anywhere, a second call returns the same bits
    dq2, dk2, dv2 = aq.attnqat_bwd(q, k, v, do, lse, ohp, causal)
    torch.cuda.synchronize()
    assert torch.equal(dq, dq2) and torch.equal(dk, dk2) and torch.equal(dv, dv2)


def test_tiny_ref_config():
    _run(1, 2, 2, 256, 64, False, seed=0)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("L", [1, 31, 64, 129, 300])
def test_ragged_lengths_d128_gqa(L, causal):
    _run(2, 4, 2, L, 128, causal, seed=200 + L, k_chan=4)


@pytest.mark.parametrize("causal", [False, True])
def test_d64_heavy_tails(causal):
    _run(1, 3, 1, 333, 64, causal, seed=9, dist="t3", scale=0.5, tok_mod=50)


@pytest.fixture
def eight_waves():
    import paper_2603_00040_amd as aq
    aq.debug_bwd_waves(8)
    yield
    aq.debug_bwd_waves(0)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 2, 2, 256, 64), (2, 4, 2, 129, 128), (1, 3, 1, 333, 64), (1, 2, 1, 700, 128)])
def test_eight_wave_backward_shape(shape, causal, eight_waves):
    """The 256-row / 256-key workgroups of the dQ and dK/dV passes, which small problems never pick by themselves: against the
    oracle, with lengths that leave the last workgroup a single wave (129), a ragged second half (333, 700) or exactly
    full (256)."""
    B, Hq, Hkv, L, d = shape
    _run(B, Hq, Hkv, L, d, causal, seed=77 + L, k_chan=2)


@pytest.mark.parametrize("causal", [False, True])
def test_eight_wave_backward_equals_four_wave(causal):
    """Both shapes add the same 32 x 32 tile products in the same order: the same bits."""
    import paper_2603_00040_amd as aq
    x = random_inputs(1, 4, 2, 900, 128, seed=5)
    q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
    o, lse, ohp = aq.attnqat_fwd(q, k, v, causal)
    out = {}
    try:
        for w in (4, 8):
            aq.debug_bwd_waves(w)
            out[w] = aq.attnqat_bwd(q, k, v, do, lse, ohp, causal)
            torch.cuda.synchronize()
    finally:
        aq.debug_bwd_waves(0)
    for a, b in zip(out[4], out[8]):
        assert torch.equal(a, b)
    with pytest.raises(aq.AttnQatError):
        aq.debug_bwd_waves(6)


def test_backward_with_oracle_forward_state():
    """Feeding the oracle's L and O' (instead of the GPU forward's) isolates the backward."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d, causal = 1, 4, 2, 200, 128, True
    x = random_inputs(B, Hq, Hkv, L, d, seed=31)
    q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
    fq, fk, fv, fdo = (f32(x[n]) for n in ("q", "k", "v", "do"))
    rf = oracle.fwd(fq, fk, fv, causal, aq.block_k())
    rb = oracle.bwd(fq, fk, fv, fdo, rf["L"], rf["Op"], causal)
    lse = torch.from_numpy(rf["L"].astype(np.float32)).cuda()
    ohp = torch.from_numpy(rf["Op"].astype(np.float32)).cuda()
    dq, dk, dv = aq.attnqat_bwd(q, k, v, do, lse, ohp, causal)
    torch.cuda.synchronize()
    for n, t in (("dQ", dq), ("dK", dk), ("dV", dv)):
        check_bf16_output(n, host(t), rb[n], TOL)


@pytest.mark.parametrize("log2_scale", [-40, 0, 30])
def test_do_dynamic_range(log2_scale):
    """dS is rounded to fp16 after a power-of-two scaling taken from a bound of |dS| (per query row
    for dQ, per kv head for dK): rows of dO that differ by 2^30 in magnitude, all-zero rows, an
    all-zero head and a very small or very large overall scale must not cost accuracy."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d, causal = 1, 4, 2, 300, 128, False
    x = random_inputs(B, Hq, Hkv, L, d, seed=77, k_chan=4)
    fdo = f32(x["do"])
    row_exp = ((np.arange(L) * 7) % 31) - 20                       # 2^-20 .. 2^10, exact in bf16
    fdo = fdo * np.exp2(row_exp + log2_scale)[None, None, :, None]
    fdo[:, :, ::17] = 0.0                                          # zero rows
    fdo[:, 3] = 0.0                                                # a zero head
    do_bits = W.f32_to_bf16_bits(fdo.astype(np.float32))
    assert np.array_equal(f32(do_bits), fdo.astype(np.float32))    # the scaling stayed exact
    q, k, v, do = to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"]), to_dev(do_bits)
    o, lse, ohp = aq.attnqat_fwd(q, k, v, causal)
    dq, dk, dv = aq.attnqat_bwd(q, k, v, do, lse, ohp, causal)
    torch.cuda.synchronize()
    fq, fk, fv = f32(x["q"]), f32(x["k"]), f32(x["v"])
    rf = oracle.fwd(fq, fk, fv, causal, aq.block_k())
    rb = oracle.bwd(fq, fk, fv, fdo.astype(np.float32), rf["L"], rf["Op"], causal)
    for n, t in (("dK", dk), ("dV", dv)):
        e = rel_l2(host(t), rb[n])
        print(f"scale 2^{log2_scale}: {n} rel-L2 {e:.2e}", flush=True)
        assert e <= TOL, (n, e)
    # dQ row by row: every row carries its own scale, so every row must be accurate on its own
    gq, rq = host(dq), rb["dQ"]
    num = np.linalg.norm(gq - rq, axis=-1); den = np.linalg.norm(rq, axis=-1)
    zero = den == 0
    assert np.all(gq[zero] == 0)
    worst = float((num[~zero] / den[~zero]).max())
    print(f"scale 2^{log2_scale}: dQ worst row rel-L2 {worst:.2e} over {int((~zero).sum())} rows", flush=True)
    assert worst <= 4e-3


def test_dkdv_tile_count_hook():
    """The measurement variant of the dK/dV pass counts the tiles it visits and those with a non-zero
    P^F, and returns the same bits as the production variant."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = 1, 2, 2, 256, 64
    x = random_inputs(B, Hq, Hkv, L, d, seed=5)
    q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
    o, lse, ohp = aq.attnqat_fwd(q, k, v, False)
    ref = aq.attnqat_bwd(q, k, v, do, lse, ohp, False)
    counts = torch.zeros(2, dtype=torch.int64, device="cuda")
    aq.debug_dkdv_tile_counts(counts)
    try:
        got = aq.attnqat_bwd(q, k, v, do, lse, ohp, False)
        torch.cuda.synchronize()
    finally:
        aq.debug_dkdv_tile_counts(None)
    visited, nonzero = (int(c) for c in counts.cpu())
    assert visited == B * Hq * (L // 32) ** 2
    # P^F of a 32x32 tile is non-zero iff some P of it exceeds 6 * 2^-10 ... checked against the oracle's P
    rf = oracle.fwd(f32(x["q"]), f32(x["k"]), f32(x["v"]), False, aq.block_k())
    qf, kf = oracle.fake_quant(f32(x["q"])), oracle.fake_quant(f32(x["k"]))
    s = np.einsum("bhid,bhjd->bhij", qf.astype(np.float64), kf.astype(np.float64)) / np.sqrt(d)
    p = np.exp(s - rf["L"][..., None])
    blk = p.reshape(B, Hq, L // 32, 32, L // 16, 16).max(-1)          # per query row and 16-key block
    # scale of a block = RNE_E4M3(max/6) > 0 iff max/6 > 2^-10 (half the smallest subnormal 2^-9, ties to even -> 0)
    tile_nz = (blk > 6.0 * 2.0 ** -10).reshape(B, Hq, L // 32, 32, L // 32, 2).any(axis=(3, 5))
    assert nonzero == int(tile_nz.sum())
    for a, b in zip(ref, got):
        assert torch.equal(a, b)


@pytest.mark.parametrize("causal", [False, True])
def test_PF_code_flips_in_the_backward(causal):
    """P^F = phi^-1(phi(P)) of the recomputed P (Alg. 3), the operand of dV, element by element against the oracle's: short
    rows, so that the block scales do not round to zero and every tile is quantized.  Both sides are fed the oracle's L."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = 1, 4, 2, 200, 128
    x = random_inputs(B, Hq, Hkv, L, d, seed=41, k_chan=4)
    q, k, v, do = (to_dev(x[n]) for n in ("q", "k", "v", "do"))
    fq, fk, fv, fdo = (f32(x[n]) for n in ("q", "k", "v", "do"))
    rf = oracle.fwd(fq, fk, fv, causal, aq.block_k())
    lse = torch.from_numpy(rf["L"].astype(np.float32)).cuda()
    ohp = torch.from_numpy(rf["Op"].astype(np.float32)).cuda()
    G = Hq // Hkv
    keys = np.arange(L, dtype=np.int64)
    bad = tot = nonzero = 0
    for row0 in (0, 128):
        _, _, _, p = aq.attnqat_debug_bwd_p(q, k, v, do, lse, ohp, causal, row0)
        torch.cuda.synchronize()
        nrow = min(128, L - row0)
        got = p.cpu().numpy()[0, :, :nrow]                                    # [Hq, rows, keys]
        for hk in range(Hkv):
            _, _, P = oracle.bwd_dkdv_keys(fq, fk, fv, fdo, 0, hk, keys, rf["L"][0, hk * G:(hk + 1) * G], rf["Op"][0, hk * G:(hk + 1) * G],
                                           causal, dump_p=True)             # [keys, G, queries]
            ref = np.transpose(P, (1, 2, 0))[:, row0:row0 + nrow]             # [G, rows, keys]
            g = got[hk * G:(hk + 1) * G]
            bad += int((g != ref).sum()); tot += ref.size; nonzero += int((ref != 0).sum())
    print(f"backward P^F flips causal{int(causal)}: {bad} of {tot} ({bad / tot:.2e}); {nonzero} non-zero", flush=True)
    assert nonzero > 0.05 * tot * (0.5 if causal else 1.0)          # enough quantized elements for the count to mean something
    assert bad / tot < 1e-4
