"""Block-sparse MX forward (attnqat_fwd_infer_mx_sparse) against the oracle's forward under the same block mask: random
masks, causal and not, grouped-query heads, a ragged tail, rows whose first kept blocks lie in their causal future, and
rows left without any key."""
import numpy as np
import pytest
import torch

import oracle
from tests.gpu_util import f32, host, max_abs, random_inputs, rel_l2, to_dev

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _mask(B, Hq, L, keep, seed, diag=True):
    nb = (L + 127) // 128
    rng = np.random.default_rng(seed)
    m = (rng.random((B, Hq, nb, nb)) < keep).astype(np.uint8)
    if diag:
        m[:, :, np.arange(nb), np.arange(nb)] = 1          # every query keeps its own block: no empty rows under the causal mask
    return m


def _run(B, Hq, Hkv, L, d, causal, bm, seed, **kw):
    import paper_2603_00040_amd as aq
    x = random_inputs(B, Hq, Hkv, L, d, seed, **kw)
    o, lse = aq.attnqat_fwd_infer_mx_sparse(to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"]), causal, torch.from_numpy(bm).cuda())
    torch.cuda.synchronize()
    ref = oracle.fwd(f32(x["q"]), f32(x["k"]), f32(x["v"]), causal, aq.block_k(), scale_mode=oracle.MX, block_mask=bm)
    o, lse = host(o), host(lse)
    empty = np.isneginf(ref["L"])
    assert np.array_equal(np.isneginf(lse), empty)
    assert not np.isnan(o).any() and not np.isnan(lse).any()
    assert np.all(o[empty] == 0)
    eO = rel_l2(o, ref["O"])
    eL = max_abs(lse[~empty], ref["L"][~empty]) if (~empty).any() else 0.0
    print(f"sparse B{B} Hq{Hq} Hkv{Hkv} L{L} d{d} causal{int(causal)} kept {bm.mean():.2f} empty rows {int(empty.sum())}: "
          f"O rel-L2 {eO:.2e}, L {eL:.2e}", flush=True)
    assert eO <= TOL and eL <= 2e-5 * max(1.0, np.abs(ref["L"][~empty]).max() if (~empty).any() else 1.0)
    return o, lse


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
def test_sparse_random_mask(d, causal):
    L = 700                                                # 6 blocks, the last one ragged
    _run(1, 4, 2, L, d, causal, _mask(1, 4, L, 0.4, seed=3), seed=20 + d, k_chan=4)


def test_sparse_full_mask_equals_dense():
    import paper_2603_00040_amd as aq
    L = 515
    bm = np.ones((2, 2, 5, 5), np.uint8)
    x = random_inputs(2, 2, 2, L, 128, 31)
    q, k, v = to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"])
    for causal in (False, True):
        o, lse = aq.attnqat_fwd_infer_mx_sparse(q, k, v, causal, torch.from_numpy(bm).cuda())
        o2, lse2 = aq.attnqat_fwd_infer_mx(q, k, v, causal)
        assert torch.equal(o, o2) and torch.equal(lse, lse2)


def test_sparse_future_blocks_first_and_empty_rows():
    # causal, and the mask keeps blocks above the diagonal too: such a block comes first in some rows' lists although
    # the causal mask hides all of it; query block 2 keeps nothing at all, query block 3 only a block in its future
    L = 640
    bm = np.zeros((1, 2, 5, 5), np.uint8)
    bm[0, :, 0, [0, 3]] = 1
    bm[0, :, 1, [1, 4]] = 1
    bm[0, :, 3, 4] = 1
    bm[0, :, 4, [0, 2, 4]] = 1
    _run(1, 2, 1, L, 128, True, bm, seed=33)
    bm2 = bm.copy()
    bm2[0, 1] = 0                                          # a whole head without keys
    _run(1, 2, 1, L, 128, False, bm2, seed=34)


def test_sparse_per_head_masks_with_grouped_queries():
    L = 1024
    _run(2, 8, 2, L, 128, False, _mask(2, 8, L, 0.3, seed=5, diag=False), seed=35, k_chan=4)


def test_sparse_argument_errors():
    import paper_2603_00040_amd as aq
    x = random_inputs(1, 2, 2, 256, 128, 1)
    q, k, v = to_dev(x["q"]), to_dev(x["k"]), to_dev(x["v"])
    with pytest.raises(aq.AttnQatError):
        aq.attnqat_fwd_infer_mx_sparse(q, k, v, False, torch.ones((1, 2, 2, 3), dtype=torch.uint8, device="cuda"))
    with pytest.raises(aq.AttnQatError):
        aq.attnqat_fwd_infer_mx_sparse(q, k, v, False, torch.ones((1, 2, 2, 2), dtype=torch.int32, device="cuda"))
