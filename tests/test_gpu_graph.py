"""The training step and the MX inference forward recorded into a HIP graph (torch.cuda.CUDAGraph) and replayed: the
entry points only enqueue kernels on the given stream (no allocation, no synchronisation, no memset), so a capture
takes them as they are.  Every replay is checked bit for bit against the eager result, with eager work and
synchronisations of the program's own between the replays and with new input values written into the captured buffers."""
import numpy as np
import pytest
import torch

from tests.gpu_util import random_inputs, to_dev

pytestmark = pytest.mark.gpu


def _bufs(aq, B, Hq, Hkv, L, d):
    q = torch.empty((B, Hq, L, d), dtype=torch.bfloat16, device="cuda")
    k = torch.empty((B, Hkv, L, d), dtype=torch.bfloat16, device="cuda")
    v, do = torch.empty_like(k), torch.empty_like(q)
    o, lse = torch.empty_like(q), torch.empty((B, Hq, L), dtype=torch.float32, device="cuda")
    ohp = torch.empty((B, Hq, L, d), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    nbytes = max(aq.workspace_bytes(w, B, Hq, Hkv, L, d) for w in (aq.WS_FWD, aq.WS_BWD, aq.WS_FWD_INFER_MX))
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    return q, k, v, do, o, lse, ohp, dq, dk, dv, ws


@pytest.mark.parametrize("causal", [False, True])
def test_graph_replay_of_training_step_and_mx_forward(causal):
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = 2, 4, 2, 333, 128
    q, k, v, do, o, lse, ohp, dq, dk, dv, ws = _bufs(aq, B, Hq, Hkv, L, d)
    o_mx, lse_mx = torch.empty_like(o), torch.empty_like(lse)

    def step():
        aq.attnqat_fwd(q, k, v, causal, workspace=ws, out=(o, lse, ohp))
        aq.attnqat_bwd(q, k, v, do, lse, ohp, causal, workspace=ws, out=(dq, dk, dv))
        aq.attnqat_fwd_infer_mx(q, k, v, causal, workspace=ws, out=(o_mx, lse_mx))

    def load(seed):
        x = random_inputs(B, Hq, Hkv, L, d, seed, k_chan=4)
        for t, n in ((q, "q"), (k, "k"), (v, "v"), (do, "do")):
            t.copy_(to_dev(x[n]))

    outs = (o, lse, ohp, dq, dk, dv, o_mx, lse_mx)
    load(1)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()                                        # warm-up off the default stream, as captures want
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep, seed in enumerate((1, 2, 3, 2)):
        load(seed)
        step()                                        # eager, on the current stream
        torch.cuda.synchronize()
        want = [t.clone() for t in outs]
        for t in outs:
            t.fill_(float("nan")) if t.dtype != torch.bfloat16 else t.zero_()
        _ = (want[0].float().sum() + q.float().sum()).item()       # eager work and a synchronisation between replays
        g.replay()
        torch.cuda.synchronize()
        for t, w in zip(outs, want):
            assert torch.equal(t, w), (rep, seed)
        assert not torch.isnan(lse).any()
    print(f"graph replays bit-identical to eager, causal={int(causal)}", flush=True)


def test_two_streams_with_their_own_workspaces_do_not_interfere():
    """The entry points keep no state between calls besides the caller's workspace: a training step on each of two
    streams at once, different inputs, each with its own workspace, gives what each gives alone."""
    import paper_2603_00040_amd as aq
    B, Hq, Hkv, L, d = 1, 8, 4, 700, 128
    sets = []
    for seed in (11, 12):
        x = random_inputs(B, Hq, Hkv, L, d, seed, k_chan=4)
        t = {n: to_dev(x[n]) for n in ("q", "k", "v", "do")}
        bufs = _bufs(aq, B, Hq, Hkv, L, d)
        sets.append((t, bufs))

    def step(t, bufs):
        _, _, _, _, o, lse, ohp, dq, dk, dv, ws = bufs
        aq.attnqat_fwd(t["q"], t["k"], t["v"], True, workspace=ws, out=(o, lse, ohp))
        aq.attnqat_bwd(t["q"], t["k"], t["v"], t["do"], lse, ohp, True, workspace=ws, out=(dq, dk, dv))
        return o, lse, ohp, dq, dk, dv

    alone = []
    for t, bufs in sets:
        alone.append([r.clone() for r in step(t, bufs)])
        torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for _ in range(3):
        outs = []
        for (t, bufs), st in zip(sets, streams):
            with torch.cuda.stream(st):
                outs.append(step(t, bufs))
        torch.cuda.synchronize()
        for got, want in zip(outs, alone):
            for g_, w_ in zip(got, want):
                assert torch.equal(g_, w_)


def test_mfma_sustained_probe_reports_a_plausible_rate_and_clock():
    from paper_2603_00040_amd import benchaux            # bench-only helper library, not part of the attention ABI
    tf, ghz = benchaux.mfma_sustained(rounds=1, iters=4000)
    print(f"sustained MFMA probe: {tf:.0f} TFLOP/s at {ghz:.2f} GHz", flush=True)
    assert 1.0 < ghz < 2.6          # the part's clock range
    assert 800.0 < tf < 2600.0      # below the published 2.5 PFLOP/s, well above what a stalled launch would give


def test_graph_replay_of_the_paged_nvfp4_forward():
    """The NVFP4 paged forward under capture: the decode path (counter reset, chunk queue, merge: three kernels, tickets and row
    maxima in the workspace) and the chunked-prefill path, replayed after the cache, the lengths and the queries changed."""
    import paper_2603_00040_amd as aq
    Hq, Hkv, d, max_pages = 8, 2, 128, 24
    B = 3
    num_pages = B * max_pages
    cache = torch.empty(num_pages * aq.kv_cache_page_bytes_nvfp4(Hkv, d), dtype=torch.uint8, device="cuda")
    table = torch.arange(num_pages, dtype=torch.int32, device="cuda").reshape(B, max_pages).flip(1).contiguous()
    lens = torch.zeros(B, dtype=torch.int32, device="cuda")
    q1 = torch.empty((B, Hq, 1, d), dtype=torch.bfloat16, device="cuda")
    q64 = torch.empty((B, Hq, 64, d), dtype=torch.bfloat16, device="cuda")
    o1, l1 = torch.empty_like(q1), torch.empty((B, Hq, 1), dtype=torch.float32, device="cuda")
    o64, l64 = torch.empty_like(q64), torch.empty((B, Hq, 64), dtype=torch.float32, device="cuda")
    nb = max(aq.lib().attnqat_paged_workspace_bytes(B, Hq, Hkv, 1, max_pages, d), aq.lib().attnqat_paged_workspace_bytes(B, Hq, Hkv, 64, max_pages, d))
    ws1 = torch.empty(nb, dtype=torch.uint8, device="cuda"); ws64 = torch.empty(nb, dtype=torch.uint8, device="cuda")

    def step():
        aq.attnqat_fwd_infer_paged(q1, cache, num_pages, table, lens, Hkv, True, workspace=ws1, out=(o1, l1))
        aq.attnqat_fwd_infer_paged(q64, cache, num_pages, table, lens, Hkv, True, workspace=ws64, out=(o64, l64))

    def load(seed, kv_lens):
        cache.random_(0, 256)
        x = random_inputs(B, Hq, Hkv, max(kv_lens), d, seed, k_chan=4)
        for b, n in enumerate(kv_lens):
            aq.attnqat_kv_cache_write(to_dev(x["k"][b:b + 1, :, :n]).contiguous(), to_dev(x["v"][b:b + 1, :, :n]).contiguous(), cache, table[b].contiguous())
        lens.copy_(torch.tensor(kv_lens, dtype=torch.int32))
        q1.copy_(to_dev(np.ascontiguousarray(np.stack([x["q"][b, :, n - 1:n] for b, n in enumerate(kv_lens)]))))
        q64.copy_(to_dev(np.ascontiguousarray(np.stack([x["q"][b, :, n - 64:n] for b, n in enumerate(kv_lens)]))))

    outs = (o1, l1, o64, l64)
    load(1, [3000, 1025, 70])                         # decode: three chunks, two chunks, one
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep, (seed, kv_lens) in enumerate(((1, [3000, 1025, 70]), (2, [64, 2049, 3072]), (3, [1500, 1500, 100]), (2, [64, 2049, 3072]))):
        load(seed, kv_lens)
        step()
        torch.cuda.synchronize()
        want = [t.clone() for t in outs]
        for t in outs:
            t.fill_(float("nan")) if t.dtype != torch.bfloat16 else t.zero_()
        _ = (want[0].float().sum() + q64.float().sum()).item()
        g.replay()
        torch.cuda.synchronize()
        for t, w in zip(outs, want):
            assert torch.equal(t, w), (rep, seed)
        assert not torch.isnan(l1).any() and not torch.isnan(l64).any()
    print("paged NVFP4 forward: graph replays bit-identical to eager", flush=True)
