"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle cannot run these problems whole, so each check is one it can do exactly:
  * O, L, O' and dQ on seeded sampled query rows (rows are independent given all K, V);
  * dK and dV on ALL keys of the selected kv heads, by running the GPU backward with a dO
    that is zero outside the sampled rows: dP, D, dS and dV = P^F^T dO are linear in dO, so
    the oracle only has to visit the sampled rows, while the kernel still walks every
    (query tile, key tile) pair of the full problem; heads without sampled rows must come
    back exactly zero;
  * the dequantized P-tilde^F of one 128-row query tile, element by element (flip count);
  * codes and scales of complete Q/K/V tensors, bit exact.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from tests.gpu_util import check_bf16_output, f32, host, max_abs, rel_l2, to_dev

pytestmark = pytest.mark.gpu

TOL, FLIP_BAR = 2e-3, 1e-4


def _selection(w):
    """kv heads to check (first and last), their query heads, and sampled rows per query head."""
    G = w.Hq // w.Hkv
    kv = sorted({0, w.Hkv - 1})
    b = w.B - 1
    qheads = [hk * G + g for hk in kv for g in range(G)]
    rng = np.random.default_rng(1000 + w.seed)
    nrand = 6 if len(qheads) <= 4 else 2
    rows = []
    for h in qheads:
        fixed = [0, 1, w.L - 1, w.L - 2, (w.L // 128) * 128 - 1, (w.L // 128) * 128]
        extra = rng.integers(0, w.L, nrand).tolist()
        rows.append(sorted({r for r in fixed + extra if 0 <= r < w.L}))
    return b, kv, qheads, rows


def _sub(x, b, kv, qheads):
    """The sub-problem (B=1) made of the selected heads, as float32 for the oracle."""
    s = {"q": f32(x["q"][b:b + 1, qheads]), "k": f32(x["k"][b:b + 1, kv]), "v": f32(x["v"][b:b + 1, kv])}
    if "do" in x:
        s["do"] = f32(x["do"][b:b + 1, qheads])
    return s


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_full_size(cfg):
    import paper_2603_00040_amd as aq
    w = W.CONFIGS[cfg]
    train = w.passes == "fwd+bwd"
    print(f"\n[{w.name}] generating inputs", flush=True)
    x = W.make_inputs(w, with_do=train)
    q, k, v = to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"])
    b, kv, qheads, rows = _selection(w)
    L, d, Bk = w.L, w.d, aq.block_k()
    sub = _sub(x, b, kv, qheads)
    flat = np.asarray([hi * L + r for hi, rs in enumerate(rows) for r in rs], dtype=np.int64)
    gi = [(b, h, r) for h, rs in zip(qheads, rows) for r in rs]                # (b, h, row) on the GPU side
    pick = lambda t: torch.stack([t[bb, hh, rr] for bb, hh, rr in gi])

    # ---- forward
    print(f"[{w.name}] GPU forward", flush=True)
    if train:
        o, lse, ohp = aq.attnqat_fwd(q, k, v, w.causal)
    else:
        o, lse = aq.attnqat_fwd_infer(q, k, v, w.causal)
    torch.cuda.synchronize()
    print(f"[{w.name}] oracle forward on {flat.size} rows", flush=True)
    rf = oracle.fwd(sub["q"], sub["k"], sub["v"], w.causal, Bk, rows=flat)
    eL = max_abs(host(pick(lse)), rf["L"])
    print(f"[{w.name}] L max-abs {eL:.2e}", flush=True)
    check_bf16_output("O", host(pick(o)), rf["O"], TOL, label=f"[{w.name}] ")
    assert eL <= 2e-5 * max(1.0, np.abs(rf["L"]).max())
    if train:
        eOp = rel_l2(host(pick(ohp)), rf["Op"])
        print(f"[{w.name}] O' rel-L2 {eOp:.2e}", flush=True)
        assert eOp <= 2e-4

    # ---- P-tilde^F of one query tile of the selected heads
    row0 = ((L // 2) // 128) * 128
    _, _, p = aq.attnqat_debug_fwd_p(q, k, v, w.causal, row0)
    torch.cuda.synchronize()
    nrow = min(128, L - row0)
    hsel = list(range(len(qheads)))[:2]
    prow = np.asarray([hi * L + row0 + i for hi in hsel for i in range(nrow)], dtype=np.int64)
    rp = oracle.fwd(sub["q"], sub["k"], sub["v"], w.causal, Bk, rows=prow, dump_p=True)
    got = torch.stack([p[b, qheads[hi], :nrow] for hi in hsel]).cpu().numpy().reshape(-1, L)
    flips = int((got != rp["P"]).sum())
    print(f"[{w.name}] P-tilde^F flips {flips} of {got.size} ({flips / got.size:.2e})", flush=True)
    assert flips / got.size < FLIP_BAR
    del p

    # ---- codes and scales of whole tensors
    for name in (("k", "v") if cfg == 3 else ("q", "k", "v")):
        t = {"q": q, "k": k, "v": v}[name]
        codes, scales, _ = aq.attnqat_quantize(t, want_xf=False)
        torch.cuda.synchronize()
        pc, ps, _ = oracle.phi(f32(x[name]))
        gc, gs = codes.cpu().numpy(), scales.cpu().numpy()
        canon = lambda c: np.where((c & 7) == 0, c & 0xF0, c) & np.where((c & 0x70) == 0, 0x0F, 0xFF)
        nbad_s = int((gs != ps).sum()); nbad_c = int((canon(gc) != canon(pc)).sum())
        print(f"[{w.name}] phi({name}): {gs.size} scales, {nbad_s} differ; {gc.size} code bytes, {nbad_c} differ", flush=True)
        assert nbad_s == 0 and nbad_c == 0
        del codes, scales, pc, ps, gc, gs
    if not train:
        return

    # ---- backward: dQ on the sampled rows (full dO)
    do = to_dev(x["do"])
    print(f"[{w.name}] GPU backward (dense dO)", flush=True)
    dq, dk, dv = aq.attnqat_bwd(q, k, v, do, lse, ohp, w.causal)
    torch.cuda.synchronize()
    rdq = oracle.bwd_dq_rows(sub["q"], sub["k"], sub["v"], sub["do"], flat, rf["L"], rf["Op"], w.causal)
    check_bf16_output("dQ", host(pick(dq)), rdq, TOL, label=f"[{w.name}] ")
    # Eq. 5: sum_i dQ_i . Q^F_i = sum_k dK_k . K^F_k (both equal sum_ik dS_ik S_ik sqrt(d)) ties the
    # dense dK of EVERY head to dQ at any size
    _, _, qf = aq.attnqat_quantize(q, want_codes=False)
    _, _, kf = aq.attnqat_quantize(k, want_codes=False)
    G = w.Hq // w.Hkv
    lhs = (dq.float() * qf.float()).sum((2, 3)).double().view(w.B, w.Hkv, G).sum(-1)
    rhs = (dk.float() * kf.float()).sum((2, 3)).double()
    scale = (dq.float().abs() * qf.float().abs()).sum((2, 3)).double().view(w.B, w.Hkv, G).sum(-1)
    ident = float(((lhs - rhs).abs() / scale).max())
    print(f"[{w.name}] max |sum dQ.Q - sum dK.K| / sum |dQ||Q| over heads = {ident:.2e}", flush=True)
    assert ident < 2e-3
    del dq, dk, dv, qf, kf

    # ---- backward with dO zero outside the sampled rows: dK, dV on all keys
    dos = torch.zeros_like(do)
    for bb, hh, rr in gi:
        dos[bb, hh, rr] = do[bb, hh, rr]
    print(f"[{w.name}] GPU backward (sparse dO)", flush=True)
    _, dk, dv = aq.attnqat_bwd(q, k, v, dos, lse, ohp, w.causal)
    torch.cuda.synchronize()
    rdk, rdv = oracle.bwd_rows_dkdv(sub["q"], sub["k"], sub["v"], sub["do"], flat, rf["L"], rf["Op"], w.causal)
    gk = host(dk[b, kv]); gv = host(dv[b, kv])
    print(f"[{w.name}] oracle dV non-zero fraction {float((rdv[0] != 0).mean()):.3f}", flush=True)
    check_bf16_output("dK", gk, rdk[0], TOL, label=f"[{w.name}] ")
    check_bf16_output("dV", gv, rdv[0], TOL, zero_rms=1e-6, label=f"[{w.name}] ")
    other = [hk for hk in range(w.Hkv) if hk not in kv]
    if other:
        assert not dk[:, other].any() and not dv[:, other].any()
    if w.B > 1:
        assert not dk[:b].any() and not dv[:b].any()


@pytest.mark.parametrize("fp8pv", [False, True])
@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_full_size_mx_forward(cfg, fp8pv):
    """The MX forward (scaled FP4 MFMA; fp8pv: the mixed recipe with MXFP8 P and V) on the full shapes: O and L on
    sampled rows, and the MX codes and scales of whole K (blocks along d) and V (blocks along the keys) tensors, bit exact."""
    import paper_2603_00040_amd as aq
    w = W.CONFIGS[cfg]
    print(f"\n[{w.name}] generating inputs", flush=True)
    x = W.make_inputs(w, with_do=False)
    q, k, v = to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"])
    b, kv, qheads, rows = _selection(w)
    L, Bk = w.L, aq.block_k()
    sub = _sub(x, b, kv, qheads)
    flat = np.asarray([hi * L + r for hi, rs in enumerate(rows) for r in rs], dtype=np.int64)
    gi = [(b, h, r) for h, rs in zip(qheads, rows) for r in rs]
    pick = lambda t: torch.stack([t[bb, hh, rr] for bb, hh, rr in gi])
    print(f"[{w.name}] GPU MX forward", flush=True)
    o, lse = (aq.attnqat_fwd_infer_mx_fp8pv if fp8pv else aq.attnqat_fwd_infer_mx)(q, k, v, w.causal)
    torch.cuda.synchronize()
    print(f"[{w.name}] oracle MX forward on {flat.size} rows", flush=True)
    rf = oracle.fwd(sub["q"], sub["k"], sub["v"], w.causal, Bk, scale_mode=oracle.MX_FP8PV if fp8pv else oracle.MX, rows=flat)
    eO = rel_l2(host(pick(o)), rf["O"]); eL = max_abs(host(pick(lse)), rf["L"])
    print(f"[{w.name}] MX O rel-L2 {eO:.2e} max-abs {max_abs(host(pick(o)), rf['O']):.2e}  L max-abs {eL:.2e}", flush=True)
    assert eO <= TOL and eL <= 2e-5 * max(1.0, np.abs(rf["L"]).max())
    canon = lambda c: np.where((c & 7) == 0, c & 0xF0, c) & np.where((c & 0x70) == 0, 0x0F, 0xFF)
    if fp8pv:
        canon = lambda c: np.where((c & 0x7F) == 0, 0, c)
    for name, axis in ((("v", 1),) if fp8pv else (("k", 0), ("v", 1))):
        t = {"k": k, "v": v}[name][b:b + 1, kv].contiguous()
        codes, scales, _ = aq.attnqat_quantize_mxfp8(t, want_xf=False) if fp8pv else aq.attnqat_quantize_mx(t, axis=axis, want_xf=False)
        torch.cuda.synchronize()
        xs = sub[name] if axis == 0 else np.ascontiguousarray(np.swapaxes(sub[name], -1, -2))
        pc, ps, _ = oracle.phi_mx8(xs) if fp8pv else oracle.phi_mx(xs)
        gc, gs = codes.cpu().numpy(), scales.cpu().numpy()
        nbad_s = int((gs != ps).sum()); nbad_c = int((canon(gc) != canon(pc)).sum())
        print(f"[{w.name}] MX phi({name}, axis {axis}): {gs.size} scales, {nbad_s} differ; {gc.size} code bytes, {nbad_c} differ", flush=True)
        assert nbad_s == 0 and nbad_c == 0


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_full_size_mx_training(cfg):
    """attnqat_fwd_mx + attnqat_bwd_mx on the full training shapes: O, O', L and dQ on sampled rows; dK and dV
    on all keys of the selected kv heads through a dO that is zero outside the sampled rows (as above)."""
    import paper_2603_00040_amd as aq
    w = W.CONFIGS[cfg]
    print(f"\n[{w.name}] generating inputs", flush=True)
    x = W.make_inputs(w, with_do=True)
    q, k, v, do = to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"]), to_dev(x["do"])
    b, kv, qheads, rows = _selection(w)
    L, Bk, MX = w.L, aq.block_k(), oracle.MX
    sub = _sub(x, b, kv, qheads)
    flat = np.asarray([hi * L + r for hi, rs in enumerate(rows) for r in rs], dtype=np.int64)
    gi = [(b, h, r) for h, rs in zip(qheads, rows) for r in rs]
    pick = lambda t: torch.stack([t[bb, hh, rr] for bb, hh, rr in gi])
    print(f"[{w.name}] GPU MX training forward", flush=True)
    o, lse, ohp = aq.attnqat_fwd_mx(q, k, v, w.causal)
    torch.cuda.synchronize()
    rf = oracle.fwd(sub["q"], sub["k"], sub["v"], w.causal, Bk, scale_mode=MX, rows=flat)
    eO = rel_l2(host(pick(o)), rf["O"]); eOp = rel_l2(host(pick(ohp)), rf["Op"]); eL = max_abs(host(pick(lse)), rf["L"])
    print(f"[{w.name}] MX train O rel-L2 {eO:.2e}  O' rel-L2 {eOp:.2e}  L max-abs {eL:.2e}", flush=True)
    assert eO <= TOL and eOp <= 2e-4 and eL <= 2e-5 * max(1.0, np.abs(rf["L"]).max())
    print(f"[{w.name}] GPU MX backward (dense dO)", flush=True)
    dq, dk, dv = aq.attnqat_bwd_mx(q, k, v, do, lse, ohp, w.causal)
    torch.cuda.synchronize()
    rdq = oracle.bwd_dq_rows(sub["q"], sub["k"], sub["v"], sub["do"], flat, rf["L"], rf["Op"], w.causal, scale_mode=MX)
    eQ = rel_l2(host(pick(dq)), rdq)
    print(f"[{w.name}] MX dQ rel-L2 {eQ:.2e}", flush=True)
    assert eQ <= TOL
    del dq, dk, dv
    dos = torch.zeros_like(do)
    for bb, hh, rr in gi:
        dos[bb, hh, rr] = do[bb, hh, rr]
    print(f"[{w.name}] GPU MX backward (sparse dO)", flush=True)
    _, dk, dv = aq.attnqat_bwd_mx(q, k, v, dos, lse, ohp, w.causal)
    torch.cuda.synchronize()
    rdk, rdv = oracle.bwd_rows_dkdv(sub["q"], sub["k"], sub["v"], sub["do"], flat, rf["L"], rf["Op"], w.causal, scale_mode=MX)
    gk = host(dk[b, kv]); gv = host(dv[b, kv])
    eK, eV = rel_l2(gk, rdk[0]), rel_l2(gv, rdv[0], zero_rms=1e-6)
    print(f"[{w.name}] MX dK rel-L2 {eK:.2e}  dV rel-L2 {eV:.2e} (oracle dV non-zero fraction {float((rdv[0] != 0).mean()):.3f})", flush=True)
    assert eK <= TOL and eV <= TOL
    other = [hk for hk in range(w.Hkv) if hk not in kv]
    if other:
        assert not dk[:, other].any() and not dv[:, other].any()


@pytest.mark.parametrize("cfg,opts", [(2, 1), (4, 1), (3, 2), (2, 3)])
def test_full_size_options(cfg, opts):
    """The option bits of attnqat_fwd_opt / attnqat_bwd_opt (1: K smoothing, 2: two-level quantization of P) on full
    shapes: O, O', L and dQ on sampled rows against the oracle with the same options; dK, dV through a dO that is zero
    outside the sampled rows."""
    import paper_2603_00040_amd as aq
    w = W.CONFIGS[cfg]
    print(f"\n[{w.name}] options {opts}: generating inputs", flush=True)
    x = W.make_inputs(w, with_do=True)
    q, k, v, do = to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"]), to_dev(x["do"])
    b, kv, qheads, rows = _selection(w)
    L, Bk = w.L, aq.block_k()
    sm = oracle.TWO_LEVEL_P if opts & aq.OPT_TWO_LEVEL_P else 0
    sub = _sub(x, b, kv, qheads)
    if opts & aq.OPT_SMOOTH_K:
        sub["k"] = oracle.smooth_k(sub["k"])
    flat = np.asarray([hi * L + r for hi, rs in enumerate(rows) for r in rs], dtype=np.int64)
    gi = [(b, h, r) for h, rs in zip(qheads, rows) for r in rs]
    pick = lambda t: torch.stack([t[bb, hh, rr] for bb, hh, rr in gi])
    o, lse, ohp = aq.attnqat_fwd_opt(q, k, v, w.causal, opts)
    torch.cuda.synchronize()
    rf = oracle.fwd(sub["q"], sub["k"], sub["v"], w.causal, Bk, scale_mode=sm, rows=flat)
    eO = rel_l2(host(pick(o)), rf["O"]); eOp = rel_l2(host(pick(ohp)), rf["Op"]); eL = max_abs(host(pick(lse)), rf["L"])
    print(f"[{w.name}] options {opts}: O rel-L2 {eO:.2e}  O' rel-L2 {eOp:.2e}  L max-abs {eL:.2e}", flush=True)
    assert eO <= TOL and eOp <= 2e-4 and eL <= 2e-5 * max(1.0, np.abs(rf["L"]).max())
    dq, _, _ = aq.attnqat_bwd_opt(q, k, v, do, lse, ohp, w.causal, opts)
    torch.cuda.synchronize()
    rdq = oracle.bwd_dq_rows(sub["q"], sub["k"], sub["v"], sub["do"], flat, rf["L"], rf["Op"], w.causal, scale_mode=sm)
    eQ = rel_l2(host(pick(dq)), rdq)
    print(f"[{w.name}] options {opts}: dQ rel-L2 {eQ:.2e}", flush=True)
    assert eQ <= TOL
    del dq
    dos = torch.zeros_like(do)
    for bb, hh, rr in gi:
        dos[bb, hh, rr] = do[bb, hh, rr]
    _, dk, dv = aq.attnqat_bwd_opt(q, k, v, dos, lse, ohp, w.causal, opts)
    torch.cuda.synchronize()
    rdk, rdv = oracle.bwd_rows_dkdv(sub["q"], sub["k"], sub["v"], sub["do"], flat, rf["L"], rf["Op"], w.causal, scale_mode=sm)
    eK, eV = rel_l2(host(dk[b, kv]), rdk[0]), rel_l2(host(dv[b, kv]), rdv[0], zero_rms=1e-6)
    print(f"[{w.name}] options {opts}: dK rel-L2 {eK:.2e}  dV rel-L2 {eV:.2e} (oracle dV non-zero fraction {float((rdv[0] != 0).mean()):.3f})", flush=True)
    assert eK <= TOL and eV <= TOL


@pytest.mark.parametrize("cfg", [1, 4])
def test_full_size_block_sparse_forward(cfg):
    """attnqat_fwd_infer_mx_sparse on the full inference shapes under a seeded random mask that keeps a quarter of the
    128 x 128 blocks plus the diagonal (under the causal mask also blocks above the diagonal, which then hold no visible
    key): O and L on sampled rows against the oracle's forward under the same mask."""
    import paper_2603_00040_amd as aq
    w = W.CONFIGS[cfg]
    print(f"\n[{w.name}] generating inputs", flush=True)
    x = W.make_inputs(w, with_do=False)
    q, k, v = to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"])
    b, kv, qheads, rows = _selection(w)
    L, Bk = w.L, aq.block_k()
    nb = (L + 127) // 128
    bm = (np.random.default_rng(77 + w.seed).random((w.B, w.Hq, nb, nb)) < 0.25).astype(np.uint8)
    bm[:, :, np.arange(nb), np.arange(nb)] = 1
    sub = _sub(x, b, kv, qheads)
    flat = np.asarray([hi * L + r for hi, rs in enumerate(rows) for r in rs], dtype=np.int64)
    gi = [(b, h, r) for h, rs in zip(qheads, rows) for r in rs]
    pick = lambda t: torch.stack([t[bb, hh, rr] for bb, hh, rr in gi])
    print(f"[{w.name}] GPU block-sparse MX forward, {bm.mean():.3f} of the blocks kept", flush=True)
    o, lse = aq.attnqat_fwd_infer_mx_sparse(q, k, v, w.causal, torch.from_numpy(bm).cuda())
    torch.cuda.synchronize()
    print(f"[{w.name}] oracle on {flat.size} rows", flush=True)
    rf = oracle.fwd(sub["q"], sub["k"], sub["v"], w.causal, Bk, scale_mode=oracle.MX, rows=flat,
                    block_mask=np.ascontiguousarray(bm[b:b + 1, qheads]))
    eO = rel_l2(host(pick(o)), rf["O"]); eL = max_abs(host(pick(lse)), rf["L"])
    print(f"[{w.name}] sparse MX O rel-L2 {eO:.2e}  L max-abs {eL:.2e}", flush=True)
    assert np.isfinite(rf["L"]).all()
    assert eO <= TOL and eL <= 2e-5 * max(1.0, np.abs(rf["L"]).max())


@pytest.mark.parametrize("fmt", ["mx", "nvfp4"])
@pytest.mark.parametrize("Lq", [1, 512])
def test_full_size_paged_serving(Lq, fmt):
    """attnqat_fwd_infer_mx_paged / attnqat_fwd_infer_paged on the serving shape bench.py --paged-lq times (32 sequences of
    4096..16384 keys, 32 query and 8 kv heads, d = 128, causal, pages scattered over the cache): a decode step (NVFP4: the
    kernel that cuts sequences into chunks, up to 16 per sequence here) and a 512-query chunk; O and L of sampled (sequence,
    head, position) against the oracle's forward of that sequence in the same format."""
    import paper_2603_00040_amd as aq
    nv = fmt == "nvfp4"
    page_bytes, write, fwd = ((aq.kv_cache_page_bytes_nvfp4, aq.attnqat_kv_cache_write, aq.attnqat_fwd_infer_paged) if nv else
                              (aq.kv_cache_page_bytes, aq.attnqat_kv_cache_write_mx, aq.attnqat_fwd_infer_mx_paged))
    B, Hq, Hkv, d = 32, 32, 8, 128
    rng = np.random.default_rng(7)
    kv_lens = np.maximum(rng.integers(4096, 16385, B), Lq).astype(np.int32)
    pages_of = [(int(n) + 127) // 128 for n in kv_lens]
    max_pages, num_pages = max(pages_of), sum(pages_of)
    perm = rng.permutation(num_pages).astype(np.int32)
    table = np.zeros((B, max_pages), np.int32)
    cache = torch.empty(num_pages * page_bytes(Hkv, d), dtype=torch.uint8, device="cuda")
    cache.random_(0, 256)
    check = sorted({0, B - 1, int(np.argmin(kv_lens)), int(np.argmax(kv_lens))})
    kept, qb, nxt = {}, [], 0
    print(f"\n[paged Lq={Lq}] writing {num_pages} pages", flush=True)
    for bb in range(B):
        n = int(kv_lens[bb])
        table[bb, :pages_of[bb]] = perm[nxt:nxt + pages_of[bb]]; nxt += pages_of[bb]
        kb = W.fill(1, Hkv, n, d, 500 + bb, W.TENSOR_K, "normal", 1.0, n_chan=4, chan_mult=20.0)
        vb = W.fill(1, Hkv, n, d, 500 + bb, W.TENSOR_V, "normal", 1.0)
        qf = W.fill(1, Hq, Lq, d, 500 + bb, W.TENSOR_Q, "normal", 1.0)
        write(to_dev(kb), to_dev(vb), cache, torch.from_numpy(table[bb, :pages_of[bb]].copy()).cuda())
        qb.append(qf[0])
        if bb in check:
            kept[bb] = (kb, vb)
    qall = np.ascontiguousarray(np.stack(qb))
    o, lse = fwd(to_dev(qall), cache, num_pages, torch.from_numpy(table).cuda(), torch.from_numpy(kv_lens).cuda(), Hkv, True)
    torch.cuda.synchronize()
    assert not torch.isnan(o.float()).any() and not torch.isnan(lse).any()
    pos = sorted({0, Lq - 1, Lq // 2, *np.random.default_rng(8).integers(0, Lq, 3).tolist()})
    for bb in check:
        n = int(kv_lens[bb])
        kb, vb = kept[bb]
        qf = np.zeros((1, Hq, n, d), np.float32)
        qf[0, :, n - Lq:] = f32(qall[bb])
        rows = oracle.flat_rows(1, Hq, n, [(0, h, n - Lq + i) for h in range(Hq) for i in pos])
        ref = oracle.fwd(qf, f32(kb), f32(vb), True, aq.block_k(), scale_mode=0 if nv else oracle.MX, rows=rows)
        got_o = host(o[bb][:, pos]).reshape(-1, d); got_l = host(lse[bb][:, pos]).reshape(-1)
        eO = rel_l2(got_o, ref["O"]); eL = max_abs(got_l, ref["L"])
        print(f"[paged {fmt} Lq={Lq}] sequence {bb} ({n} keys): O rel-L2 {eO:.2e}  L max-abs {eL:.2e} on {rows.size} rows", flush=True)
        assert eO <= TOL and eL <= 2e-5 * max(1.0, np.abs(ref["L"]).max())
