"""The C-ABI library loads on a machine without a GPU and exports every declared symbol."""
import ctypes
import os
import re

import paper_2603_00040_amd as aq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "attnqat.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(attnqat_\w+)\s*\(", text))


def test_library_exports_every_declared_symbol():
    L = ctypes.CDLL(aq.LIB_PATH)
    names = _declared()
    assert {"attnqat_quantize", "attnqat_fwd", "attnqat_bwd", "attnqat_fwd_infer"} <= names
    for n in names:
        assert hasattr(L, n), n
    assert set(aq.EXPORTS) == names          # the binding covers the same names


def test_host_side_queries_need_no_gpu():
    assert aq.block_k() == 64
    assert aq.lib().attnqat_strerror(aq.ESHAPE).decode().startswith("unsupported shape")
    # workspace: three fp16 copies padded to 128 rows (forward); Q, K, V, dO copies, the per-row {L, D}
    # pairs and 3 x 64 partial maxima per query head that bound |dS| (backward); both end with the scratch of
    # the K smoothing option: 32 fp64 partial column sums and the fp32 column mean per kv head
    B, Hq, Hkv, L, d = 1, 4, 2, 300, 128
    Lp = 384
    ksm = Hkv * 32 * d * 8 + Hkv * d * 4
    assert aq.workspace_bytes(aq.WS_FWD, B, Hq, Hkv, L, d) == (Hq + 2 * Hkv) * Lp * d * 2 + ksm
    assert aq.workspace_bytes(aq.WS_BWD, B, Hq, Hkv, L, d) == (2 * Hq + 2 * Hkv) * Lp * d * 2 + Hq * Lp * 8 + 3 * Hq * 64 * 4 + ksm
    # the MX training path adds the dequantized bf16 tensor that the MX fake-quantizer hands to the layout copy (V), and one
    # dword of scale bytes per lane and group of 32 query rows for the Q operands of the FP4 instruction
    assert aq.workspace_bytes(aq.WS_FWD_MX, B, Hq, Hkv, L, d) == (aq.workspace_bytes(aq.WS_FWD, B, Hq, Hkv, L, d) + Hq * L * d * 2
                                                                  + Hq * (Lp // 32) * 64 * 4)
    assert aq.workspace_bytes(aq.WS_FWD, B, Hq, 3, L, d) == 0
    assert aq.workspace_bytes(99, B, Hq, Hkv, L, d) == 0


def test_argument_validation_happens_before_any_gpu_call():
    f = aq.lib().attnqat_fwd_infer
    assert f(None, None, None, 1, 2, 2, 64, 128, 0, 0, None, None, None, 0, None) == aq.EINVAL
    assert aq.lib().attnqat_quantize(None, 1, 1, 16, 64, 0, None, None, None, None) == aq.EINVAL
    # every entry point that takes tensors rejects null pointers and bad sizes with a status, without touching a GPU
    L = aq.lib()
    assert L.attnqat_fwd_infer_mx(None, None, None, 1, 2, 2, 64, 128, 0, 0, None, None, None, 0, None) == aq.EINVAL
    assert L.attnqat_fwd_infer_mx_sparse(None, None, None, 1, 2, 2, 64, 128, 0, 0, None, None, None, None, 0, None) == aq.EINVAL
    assert L.attnqat_kv_cache_write_mx(None, None, 1, 1, 128, 0, None, 1, None, None) == aq.EINVAL
    # the measurement hooks keep their state per stream: switching something off that was never on is accepted
    assert L.attnqat_profile_enable(None, 0) == aq.OK and L.attnqat_debug_dkdv_tile_counts(None, None) == aq.OK
    assert L.attnqat_profile_read(None, 0, None, None) == aq.EINVAL

