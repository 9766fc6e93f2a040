"""NVFP4 KV cache in pages and Alg. 1 over it (attnqat_kv_cache_write, attnqat_fwd_infer_paged) against the oracle's forward
of every sequence on its own: variable lengths, scattered pages, chunked prefill, decode steps, sequences that grow."""
import numpy as np
import pytest
import torch

import oracle
from tests.gpu_util import check_bf16_output, f32, host, max_abs, random_inputs, to_dev

pytestmark = pytest.mark.gpu


def host_bits(t):
    """bf16 CUDA tensor -> its bit patterns (uint16 numpy)."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)

TOL = 2e-3


def _fill_cache(aq, x, Hkv, d, kv_lens, seed, pieces=1):
    """Pages scattered over a cache full of stale bytes; every sequence written in `pieces` successive appends."""
    B = len(kv_lens)
    max_pages = (max(kv_lens) + 127) // 128
    num_pages = B * max_pages + 3
    rng = np.random.default_rng(seed)
    perm = rng.permutation(num_pages).astype(np.int32)
    table = np.full((B, max_pages), -1, np.int32)
    cache = torch.empty(num_pages * aq.kv_cache_page_bytes_nvfp4(Hkv, d), dtype=torch.uint8, device="cuda")
    cache.random_(0, 256)
    k_all, v_all = to_dev(x["k"]), to_dev(x["v"])
    nxt = 0
    for b, n in enumerate(kv_lens):
        npg = (n + 127) // 128
        table[b, :npg] = perm[nxt:nxt + npg]; nxt += npg
        ids = torch.from_numpy(table[b, :npg].copy()).cuda()
        cuts = sorted(set([0, n] + [int(c) for c in rng.integers(1, max(n, 2), size=pieces - 1)])) if pieces > 1 else [0, n]
        for p0, p1 in zip(cuts[:-1], cuts[1:]):
            if p1 > p0:
                aq.attnqat_kv_cache_write(k_all[b:b + 1, :, p0:p1].contiguous(), v_all[b:b + 1, :, p0:p1].contiguous(), cache, ids, pos0=p0)
    table[table < 0] = num_pages + 5            # unused entries point outside the cache: they must never matter
    return cache, num_pages, table


def _run(Hq, Hkv, d, kv_lens, Lq, causal, seed, pieces=1, tol=TOL, **kw):
    import paper_2603_00040_amd as aq
    B = len(kv_lens)
    x = random_inputs(B, Hq, Hkv, max(kv_lens), d, seed, **kw)      # sequence b uses its first kv_lens[b] positions
    cache, num_pages, table = _fill_cache(aq, x, Hkv, d, kv_lens, seed, pieces)
    qb = np.stack([x["q"][b, :, n - Lq:n] for b, n in enumerate(kv_lens)])      # the last Lq positions of every sequence
    q = to_dev(np.ascontiguousarray(qb))
    o, lse = aq.attnqat_fwd_infer_paged(q, cache, num_pages, torch.from_numpy(table).cuda(),
                                        torch.tensor(kv_lens, dtype=torch.int32, device="cuda"), Hkv, causal)
    torch.cuda.synchronize()
    worst = 0.0
    for b, n in enumerate(kv_lens):
        qf = np.zeros((1, Hq, n, d), np.float32)
        qf[0, :, n - Lq:] = f32(qb[b])
        rows = oracle.flat_rows(1, Hq, n, [(0, h, i) for h in range(Hq) for i in range(n - Lq, n)])
        ref = oracle.fwd(qf, f32(x["k"][b:b + 1, :, :n]), f32(x["v"][b:b + 1, :, :n]), causal, aq.block_k(), rows=rows)
        check_bf16_output("O", host(o[b]).reshape(-1, d), ref["O"], tol, label=f"sequence {b} ({n} keys)")
        eL = max_abs(host(lse[b]).reshape(-1), ref["L"])
        worst = max(worst, eL)
        assert eL <= 2e-5 * max(1.0, np.abs(ref["L"]).max()), (b, n, eL)
    print(f"paged nvfp4 Hq{Hq} Hkv{Hkv} d{d} kv_lens{kv_lens} Lq{Lq} causal{int(causal)} pieces{pieces}: worst L {worst:.2e}", flush=True)
    return x, q, cache, num_pages, table, o, lse


@pytest.mark.parametrize("causal", [False, True])
def test_chunked_prefill_variable_lengths(causal):
    _run(4, 2, 128, [300, 128, 77, 513], 64, causal, seed=1, k_chan=4)


@pytest.mark.parametrize("causal", [False, True])
def test_decode_step(causal):
    _run(4, 4, 128, [1, 33, 129, 640], 1, causal, seed=2)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
def test_few_positions_grouped_heads(d, causal):
    _run(2, 2, d, [64, 65, 128, 129, 2500], 7, causal, seed=40 + d, k_chan=4)
    _run(16, 2, d, [4, 257, 1111], 4, causal, seed=41 + d)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
def test_decode_sequences_cut_into_chunks(d, causal):
    # 4 rows per (sequence, kv head): chunks of 1024 keys, up to 5 of them; 12 rows: chunks of 256 keys, up to 12; 16 rows (the
    # most the decode kernel takes); lengths at chunk and tile edges; more (sequence, head, chunk) units than workgroups wait for
    _run(8, 2, d, [5000, 1030, 1024, 3, 2049], 1, causal, seed=50 + d, k_chan=4)
    _run(8, 2, d, [3000, 700, 257], 3, causal, seed=51 + d)
    _run(16, 1, d, [1500, 256], 1, causal, seed=52 + d, dist="t3", scale=0.5)
    # more than 16 chunks in front of a chunk (19 chunks of 256 keys): the maxima a lane did not ask for early
    _run(16, 1, d, [4700, 300], 1, causal, seed=53 + d, k_chan=2)


def test_decode_many_short_sequences():
    """More sequences than the chunk list's builder stages next to its lanes (2048): the list is built from the lengths in
    memory, and every sequence is a single chunk."""
    rng = np.random.default_rng(9)
    lens = [int(n) for n in rng.integers(1, 41, size=2100)]
    # (128 output values per sequence: the rounding of the bf16 output alone scatters to 2.2e-3 in rel-L2 on so few; the
    #  bars that leave that rounding out are the usual ones)
    _run(2, 1, 64, lens, 1, True, seed=60, tol=3e-3)


def test_decode_wait_limit_is_honoured_and_leaves_no_state():
    """The bounded wait of a chunk for the maxima of the chunks before it: with no polls allowed the kernel still finishes
    (waits that found nothing are reported), and the next ordinary call is unaffected."""
    import paper_2603_00040_amd as aq
    Hq, Hkv, d, lens = 8, 2, 128, [6000, 4100, 5000, 2100]
    x = random_inputs(len(lens), Hq, Hkv, max(lens), d, 77)
    cache, num_pages, table = _fill_cache(aq, x, Hkv, d, lens, 77)
    q = to_dev(np.ascontiguousarray(np.stack([x["q"][b, :, n - 1:n] for b, n in enumerate(lens)])))
    tab, kl = torch.from_numpy(table).cuda(), torch.tensor(lens, dtype=torch.int32, device="cuda")
    o0, l0, expired0 = aq.attnqat_fwd_infer_paged(q, cache, num_pages, tab, kl, Hkv, True, spin_limit=0)
    o1, l1, expired1 = aq.attnqat_fwd_infer_paged(q, cache, num_pages, tab, kl, Hkv, True, spin_limit=1 << 22)
    o2, l2 = aq.attnqat_fwd_infer_paged(q, cache, num_pages, tab, kl, Hkv, True)
    torch.cuda.synchronize()
    print(f"decode wait limit 0: expired={expired0}; limit 2^22: expired={expired1}", flush=True)
    assert expired1 is False
    assert torch.equal(l1, l2)          # lse depends on the scores and the row sums of P-tilde only: the same in any order of arrival
    for b, n in enumerate(lens):
        qf = np.zeros((1, Hq, n, d), np.float32)
        qf[0, :, n - 1:] = f32(host_bits(q[b]))
        rows = oracle.flat_rows(1, Hq, n, [(0, h, n - 1) for h in range(Hq)])
        ref = oracle.fwd(qf, f32(x["k"][b:b + 1, :, :n]), f32(x["v"][b:b + 1, :, :n]), True, aq.block_k(), rows=rows)
        check_bf16_output("O", host(o2[b]).reshape(-1, d), ref["O"], TOL, label=f"sequence {b}")


def test_whole_sequences_d64_gqa():
    _run(6, 2, 64, [200, 200, 200], 200, True, seed=3, dist="t3", scale=0.5)


def test_long_queries_spanning_several_tiles():
    # 300 and 600 queries: two and three 256-row tiles, paired long/short under the causal mask, diagonals shifted by 400 / 89 / 100 keys
    _run(2, 1, 128, [700, 389], 300, True, seed=4)
    _run(2, 2, 128, [700, 1000], 600, True, seed=6)


def test_sequences_written_in_pieces_give_the_same_pages():
    """A sequence that grows: appends at arbitrary positions leave the same bytes as one write of the whole sequence."""
    import paper_2603_00040_amd as aq
    Hkv, d, lens = 2, 128, [300, 129, 640]
    x = random_inputs(len(lens), Hkv, Hkv, max(lens), d, 7)
    c1, n1, t1 = _fill_cache(aq, x, Hkv, d, lens, seed=7, pieces=1)
    c5, n5, t5 = _fill_cache(aq, x, Hkv, d, lens, seed=7, pieces=5)
    torch.cuda.synchronize()
    page = aq.kv_cache_page_bytes_nvfp4(Hkv, d)
    assert np.array_equal(t1, t5)
    a, b = c1.cpu().numpy().reshape(n1, page), c5.cpu().numpy().reshape(n5, page)
    used = sorted(set(int(p) for p in t1.ravel() if p < n1))
    assert len(used) == sum((n + 127) // 128 for n in lens)
    assert np.array_equal(a[used], b[used])
    _run(4, 2, d, lens, 1, True, seed=7, pieces=4)


def test_matches_the_contiguous_forward_bit_for_bit():
    import paper_2603_00040_amd as aq
    Hq, Hkv, L, d = 4, 2, 384, 128
    x, q, cache, num_pages, table, o, lse = _run(Hq, Hkv, d, [L], L, True, seed=5)
    oc, lc = aq.attnqat_fwd_infer(to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"]), True)
    torch.cuda.synchronize()
    assert torch.equal(o, oc) and torch.equal(lse, lc)
    # and the pages hold exactly what the public quantizer gives
    kc, ks, _ = aq.attnqat_quantize(to_dev(x["k"]), want_xf=False)
    page = aq.kv_cache_page_bytes_nvfp4(Hkv, d)
    pg = cache.cpu().numpy().reshape(num_pages, Hkv, 2, 128 * (d // 2 + d // 16))
    for i in range(L // 128):
        got = pg[table[0, i], :, 0]
        assert np.array_equal(got[:, :128 * d // 2].reshape(Hkv, 128, d // 2), kc[0, :, 128 * i:128 * i + 128].cpu().numpy())
        assert np.array_equal(got[:, 128 * d // 2:].reshape(Hkv, 128, d // 16), ks[0, :, 128 * i:128 * i + 128].cpu().numpy())


def test_argument_errors_and_bad_page_ids():
    import paper_2603_00040_amd as aq
    L_ = aq.lib()
    Hq = Hkv = 2; d = 128
    q = torch.zeros((1, Hq, 64, d), dtype=torch.bfloat16, device="cuda")
    page = aq.kv_cache_page_bytes_nvfp4(Hkv, d)
    assert page == Hkv * 2 * 128 * 72 and aq.kv_cache_page_bytes_nvfp4(2, 96) == 0
    cache = torch.full((2 * page,), 0xFF, dtype=torch.uint8, device="cuda")          # NaN scales everywhere
    table = torch.tensor([[7]], dtype=torch.int32, device="cuda")                    # outside the cache: reads as zeros
    lens = torch.tensor([64], dtype=torch.int32, device="cuda")
    o, lse = aq.attnqat_fwd_infer_paged(q, cache, 2, table, lens, Hkv, True)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all()
    need = L_.attnqat_paged_workspace_bytes(1, Hq, Hkv, 64, 1, d)
    assert need > 0 and L_.attnqat_paged_workspace_bytes(1, Hq, 3, 64, 1, d) == 0 and L_.attnqat_paged_workspace_bytes(1, Hq, Hkv, 64, 0, d) == 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    call = lambda **kw: L_.attnqat_fwd_infer_paged(
        kw.get("q", q.data_ptr()), 1, Hq, kw.get("hkv", Hkv), 64, kw.get("d", d), 1, 0, cache.data_ptr(), kw.get("np", 2),
        table.data_ptr(), kw.get("mp", 1), lens.data_ptr(), o.data_ptr(), lse.data_ptr(), ws.data_ptr(), kw.get("wsb", need), None)
    assert call() == aq.OK
    assert call(q=None) == aq.EINVAL and call(np=0) == aq.EINVAL and call(mp=0) == aq.EINVAL
    assert call(d=96) == aq.ESHAPE and call(hkv=3) == aq.ESHAPE and call(wsb=need - 1) == aq.EWORKSPACE
    torch.cuda.synchronize()
    # the writer: a page id outside the cache is left out (nothing outside the cache, and no other page, is touched)
    x = random_inputs(1, Hkv, Hkv, 256, d, 9)
    k, v = to_dev(x["k"]), to_dev(x["v"])
    guard = torch.full((4 * page,), 0xAB, dtype=torch.uint8, device="cuda")
    cache2 = guard[page:3 * page]                       # two pages with a guard page on either side
    aq.attnqat_kv_cache_write(k, v, cache2, torch.tensor([1, 5], dtype=torch.int32, device="cuda"), num_pages=2)
    aq.attnqat_kv_cache_write(k, v, cache2, torch.tensor([-1, 2], dtype=torch.int32, device="cuda"), num_pages=2)
    torch.cuda.synchronize()
    g = guard.cpu()
    assert bool((g[:2 * page] == 0xAB).all()) and bool((g[3 * page:] == 0xAB).all())      # guards and page 0 untouched
    assert float((g[2 * page:3 * page] == 0xAB).float().mean()) < 0.02                      # page 1 was written all over
    wr = lambda **kw: L_.attnqat_kv_cache_write(k.data_ptr(), v.data_ptr(), Hkv, 256, kw.get("d", d), 0, kw.get("pos0", 0),
                                                cache2.data_ptr(), kw.get("np", 2), table.data_ptr(), None)
    assert wr(pos0=-1) == aq.EINVAL and wr(np=0) == aq.EINVAL and wr(d=96) == aq.ESHAPE
