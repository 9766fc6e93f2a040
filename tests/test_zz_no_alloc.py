"""attnqat_fwd_infer_static (the entry point that allocates nothing: its scratch is a fixed array inside the library's
device image) against attnqat_fwd_infer, through the C ABI.  Same kernels on the same inputs, so the bar is bit equality
for O (bf16) and for the logsumexp (fp32).  Two calls in a row share the one array, the second with a smaller input."""
import pytest
import torch

from tests.gpu_util import random_inputs, to_dev

pytestmark = pytest.mark.gpu


def _both(aq, B, Hq, Hkv, L, d, causal, seed):
    L_ = aq.lib()
    x = random_inputs(B, Hq, Hkv, L, d, seed, k_chan=4)
    q, k, v = (to_dev(x[n]) for n in "qkv")
    st = torch.cuda.current_stream().cuda_stream
    # reference: the existing entry point with a caller-owned workspace
    o_ref = torch.empty_like(q); lse_ref = torch.empty((B, Hq, L), dtype=torch.float32, device="cuda")
    nbytes = aq.workspace_bytes(aq.WS_FWD_INFER, B, Hq, Hkv, L, d)
    assert 0 < nbytes <= aq.STATIC_SCRATCH_BYTES
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    rc = L_.attnqat_fwd_infer(q.data_ptr(), k.data_ptr(), v.data_ptr(), B, Hq, Hkv, L, d, int(causal), aq.BF16,
                              o_ref.data_ptr(), lse_ref.data_ptr(), ws.data_ptr(), nbytes, st)
    assert rc == aq.OK
    # the entry point under test: outputs pre-filled so that stale values cannot pass for results
    o = torch.full_like(q, 7.0); lse = torch.full((B, Hq, L), -3.0, dtype=torch.float32, device="cuda")
    print(f"attnqat_fwd_infer_static B{B} Hq{Hq} Hkv{Hkv} L{L} d{d} causal{int(causal)} seed{seed}", flush=True)
    rc = L_.attnqat_fwd_infer_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), B, Hq, Hkv, L, d, int(causal), aq.BF16,
                                     o.data_ptr(), lse.data_ptr(), st)
    assert rc == aq.OK, L_.attnqat_strerror(rc)
    torch.cuda.synchronize()
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)


def test_static_scratch_forward_matches_workspace_forward_twice():
    import paper_2603_00040_amd as aq
    _both(aq, 2, 4, 2, 1000, 128, True, seed=41)      # several query tiles, ragged tail, grouped-query heads
    _both(aq, 1, 2, 2, 300, 64, False, seed=42)       # smaller, right after it, on the same array
    _both(aq, 2, 4, 2, 1000, 128, False, seed=43)     # and larger again


def test_static_scratch_rejects_what_does_not_fit():
    import paper_2603_00040_amd as aq
    L_ = aq.lib()
    B, Hq, Hkv, L, d = 1, 16, 16, 8192, 128           # 96 MiB of copies: more than the array holds
    assert aq.workspace_bytes(aq.WS_FWD_INFER, B, Hq, Hkv, L, d) > aq.STATIC_SCRATCH_BYTES
    q = torch.zeros((1, 1, 64, 128), dtype=torch.bfloat16, device="cuda")       # never read: the call is refused first
    o = torch.full_like(q, 7.0); lse = torch.zeros((1, 1, 64), device="cuda")
    rc = L_.attnqat_fwd_infer_static(q.data_ptr(), q.data_ptr(), q.data_ptr(), B, Hq, Hkv, L, d, 0, aq.BF16,
                                     o.data_ptr(), lse.data_ptr(), None)
    assert rc == aq.ESTATIC
    assert b"ATTNQAT_STATIC_SCRATCH_BYTES" in L_.attnqat_strerror(rc)
    torch.cuda.synchronize()
    assert bool((o == 7.0).all())                     # nothing was enqueued
    assert L_.attnqat_fwd_infer_static(None, None, None, 1, 1, 1, 64, 128, 0, aq.BF16, None, None, None) == aq.EINVAL
