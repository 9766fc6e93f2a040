"""FP4 KV cache in pages and the MX forward over it (attnqat_kv_cache_write_mx, attnqat_fwd_infer_mx_paged) against the
oracle's MX forward of every sequence on its own: variable lengths, scattered pages, chunked prefill and decode."""
import numpy as np
import pytest
import torch

import oracle
from tests.gpu_util import f32, host, max_abs, random_inputs, rel_l2, to_dev

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _run(Hq, Hkv, d, kv_lens, Lq, causal, seed, **kw):
    import paper_2603_00040_amd as aq
    B = len(kv_lens)
    Lmax = max(kv_lens)
    x = random_inputs(B, Hq, Hkv, Lmax, d, seed, **kw)              # sequence b uses its first kv_lens[b] positions
    max_pages = (Lmax + 127) // 128
    num_pages = B * max_pages + 3
    rng = np.random.default_rng(seed)
    perm = rng.permutation(num_pages).astype(np.int32)              # pages scattered over the cache
    table = np.full((B, max_pages), -1, np.int32)
    cache = torch.empty(num_pages * aq.kv_cache_page_bytes(Hkv, d), dtype=torch.uint8, device="cuda")
    cache.random_(0, 256)                                           # stale content everywhere: nothing may depend on it
    k_all, v_all = to_dev(x["k"]), to_dev(x["v"])
    nxt = 0
    for b, n in enumerate(kv_lens):
        npg = (n + 127) // 128
        table[b, :npg] = perm[nxt:nxt + npg]; nxt += npg
        ids = torch.from_numpy(table[b, :npg].copy()).cuda()
        aq.attnqat_kv_cache_write_mx(k_all[b:b + 1, :, :n].contiguous(), v_all[b:b + 1, :, :n].contiguous(), cache, ids)
    table[table < 0] = 0
    # queries: the last Lq positions of every sequence
    qb = np.stack([x["q"][b, :, n - Lq:n] for b, n in enumerate(kv_lens)])
    q = to_dev(np.ascontiguousarray(qb))
    o, lse = aq.attnqat_fwd_infer_mx_paged(q, cache, num_pages, torch.from_numpy(table).cuda(),
                                           torch.tensor(kv_lens, dtype=torch.int32, device="cuda"), Hkv, causal)
    torch.cuda.synchronize()
    worst = {"O": 0.0, "L": 0.0}
    for b, n in enumerate(kv_lens):
        qf = np.zeros((1, Hq, n, d), np.float32)
        qf[0, :, n - Lq:] = f32(qb[b])
        rows = oracle.flat_rows(1, Hq, n, [(0, h, i) for h in range(Hq) for i in range(n - Lq, n)])
        ref = oracle.fwd(qf, f32(x["k"][b:b + 1, :, :n]), f32(x["v"][b:b + 1, :, :n]), causal, aq.block_k(),
                         scale_mode=oracle.MX, rows=rows)
        eO = rel_l2(host(o[b]).reshape(-1, d), ref["O"]); eL = max_abs(host(lse[b]).reshape(-1), ref["L"])
        worst["O"] = max(worst["O"], eO); worst["L"] = max(worst["L"], eL)
        assert eO <= TOL and eL <= 2e-5 * max(1.0, np.abs(ref["L"]).max()), (b, n, eO, eL)
    print(f"paged Hq{Hq} Hkv{Hkv} d{d} kv_lens{kv_lens} Lq{Lq} causal{int(causal)}: worst O rel-L2 {worst['O']:.2e}, L {worst['L']:.2e}", flush=True)
    return q, cache, table, o, lse


@pytest.mark.parametrize("causal", [False, True])
def test_paged_chunked_prefill_variable_lengths(causal):
    _run(4, 2, 128, [300, 128, 77, 513], 64, causal, seed=1, k_chan=4)


@pytest.mark.parametrize("causal", [False, True])
def test_paged_decode_step(causal):
    # one new query per sequence: under the causal mask it sees every key, so both settings agree with the full prefill's last row
    _run(4, 4, 128, [1, 33, 129, 640], 1, causal, seed=2)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
def test_paged_decode_kernel_shapes(d, causal):
    # at most 32 rows per (sequence, kv head): the kernel whose waves share the keys of a page.  Lengths around the tile
    # and page edges, one long enough for the copy ring to wrap several times; 7 positions without grouping (each row
    # has its own causal limit), and 8 heads x 4 positions = exactly 32 packed rows
    _run(2, 2, d, [64, 65, 128, 129, 2500], 7, causal, seed=40 + d, k_chan=4)
    _run(16, 2, d, [4, 257, 1111], 4, causal, seed=41 + d)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Lq", [1, 5, 16, 100])
def test_paged_grouped_query_heads_share_a_tile(Lq, causal):
    # G = 8 query heads per kv head: G * Lq <= 128 packs them into one tile (Lq = 1, 5, 16), Lq = 100 does not
    _run(16, 2, 128, [131, 64 + Lq, 700], Lq, causal, seed=10 + Lq, k_chan=4)


def test_paged_whole_sequences_d64_gqa():
    _run(6, 2, 64, [200, 200, 200], 200, True, seed=3, dist="t3", scale=0.5)


def test_paged_long_queries_spanning_several_tiles():
    _run(2, 1, 128, [700, 389], 300, True, seed=4)


def test_paged_matches_the_contiguous_forward_bit_for_bit():
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = 1, 4, 2, 384, 128
    q, cache, table, o, lse = _run(Hq, Hkv, d, [L], L, True, seed=5)
    x = random_inputs(B, Hq, Hkv, L, d, 5)
    oc, lc = aq.attnqat_fwd_infer_mx(to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"]), True)
    torch.cuda.synchronize()
    assert torch.equal(o, oc) and torch.equal(lse, lc)


def test_paged_argument_errors_and_bad_page_ids():
    import paper_2603_00040_amd as aq
    L_ = aq.lib()
    Hq = Hkv = 2; d = 128
    q = torch.zeros((1, Hq, 64, d), dtype=torch.bfloat16, device="cuda")
    cache = torch.zeros(2 * aq.kv_cache_page_bytes(Hkv, d), dtype=torch.uint8, device="cuda")
    table = torch.tensor([[7]], dtype=torch.int32, device="cuda")      # outside the cache: clamped, no fault
    lens = torch.tensor([64], dtype=torch.int32, device="cuda")
    o, lse = aq.attnqat_fwd_infer_mx_paged(q, cache, 2, table, lens, Hkv, True)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all()
    need = aq.workspace_bytes(aq.WS_FWD_INFER_MX_PAGED, 1, Hq, Hkv, 64, d)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    call = lambda **kw: L_.attnqat_fwd_infer_mx_paged(
        kw.get("q", q.data_ptr()), 1, Hq, kw.get("hkv", Hkv), 64, kw.get("d", d), 1, 0, cache.data_ptr(), kw.get("np", 2),
        table.data_ptr(), kw.get("mp", 1), lens.data_ptr(), o.data_ptr(), lse.data_ptr(), ws.data_ptr(), kw.get("wsb", need), None)
    assert call() == aq.OK
    assert call(q=None) == aq.EINVAL and call(np=0) == aq.EINVAL and call(mp=0) == aq.EINVAL
    assert call(d=96) == aq.ESHAPE and call(hkv=3) == aq.ESHAPE and call(wsb=need - 1) == aq.EWORKSPACE
    assert aq.kv_cache_page_bytes(2, 128) == 2 * 2 * 8704 and aq.kv_cache_page_bytes(2, 96) == 0
    torch.cuda.synchronize()
    # the writer: a page id outside the cache is left out (nothing outside the cache, and no other page, is touched)
    x = random_inputs(1, Hkv, Hkv, 256, d, 9)
    k, v = to_dev(x["k"]), to_dev(x["v"])
    page = aq.kv_cache_page_bytes(Hkv, d)
    guard = torch.full((4 * page,), 0xAB, dtype=torch.uint8, device="cuda")
    cache2 = guard[page:3 * page]                       # two pages with a guard page on either side
    aq.attnqat_kv_cache_write_mx(k, v, cache2, torch.tensor([1, 5], dtype=torch.int32, device="cuda"), num_pages=2)
    aq.attnqat_kv_cache_write_mx(k, v, cache2, torch.tensor([-1, 2], dtype=torch.int32, device="cuda"), num_pages=2)
    torch.cuda.synchronize()
    g = guard.cpu()
    assert bool((g[:2 * page] == 0xAB).all()) and bool((g[3 * page:] == 0xAB).all())      # guards and page 0 untouched
    assert not bool((g[2 * page:3 * page] == 0xAB).all())                                   # page 1 was written
