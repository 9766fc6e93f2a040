"""Thin Python binding of the gfx950 Attn-QAT C ABI (``include/attnqat.h``).

Argument marshalling only: every step of the path runs in the HIP kernels of
``libattnqat.so``.  PyTorch supplies device memory and the current stream.
There is no CPU or PyTorch fallback: if the shared library is missing, loading
fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattnqat.so")

OK, EINVAL, ESHAPE, EDTYPE, EWORKSPACE, ELAUNCH, ESTATIC = 0, -1, -2, -3, -4, -5, -6
STATIC_SCRATCH_BYTES = 32 << 20
BF16 = 0
(WS_FWD, WS_FWD_INFER, WS_BWD, WS_FWD_INFER_MX, WS_FWD_MX, WS_BWD_MX, WS_FWD_INFER_MX_FP8PV,
 WS_FWD_INFER_MX_PAGED, WS_FWD_INFER_MX_SPARSE) = 0, 1, 2, 3, 4, 5, 6, 7, 8

_vp, _i, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
_SIGNATURES = {
    "attnqat_quantize": (_i, [_vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "attnqat_fwd": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_fwd_infer": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_fwd_infer_bf16pv": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_fwd_infer_static": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp]),
    "attnqat_fwd_infer_packed": (_i, [_vp] * 6 + [_i] * 7 + [_vp, _vp, _vp, _sz, _vp]),
    "attnqat_bwd_packed": (_i, [_vp] * 9 + [_i] * 7 + [_vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_bwd": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i,
                         _vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_bwd_ablation": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _i,
                                  _vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_quantize_mx": (_i, [_vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "attnqat_fwd_infer_mx": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_quantize_mxfp8": (_i, [_vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "attnqat_fwd_infer_mx_fp8pv": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_fwd_opt": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_bwd_opt": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _i,
                             _vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_debug_fwd_p_opt": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _i, _vp,
                                     _vp, _sz, _vp]),
    "attnqat_kv_cache_page_bytes": (_sz, [_i, _i]),
    "attnqat_kv_cache_write_mx": (_i, [_vp, _vp, _i, _i, _i, _i, _vp, _i, _vp, _vp]),
    "attnqat_fwd_infer_mx_paged": (_i, [_vp, _i, _i, _i, _i, _i, _i, _i, _vp, _i, _vp, _i, _vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_kv_cache_page_bytes_nvfp4": (_sz, [_i, _i]),
    "attnqat_kv_cache_write": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _vp, _i, _vp, _vp]),
    "attnqat_paged_workspace_bytes": (_sz, [_i, _i, _i, _i, _i, _i]),
    "attnqat_fwd_infer_paged": (_i, [_vp, _i, _i, _i, _i, _i, _i, _i, _vp, _i, _vp, _i, _vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_debug_fwd_infer_paged": (_i, [_vp, _i, _i, _i, _i, _i, _i, _i, _vp, _i, _vp, _i, _vp, _vp, _vp, _vp, _sz, _vp, _i, _vp]),
    "attnqat_fwd_infer_mx_sparse": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_fwd_mx": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_bwd_mx": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i,
                            _vp, _vp, _vp, _vp, _sz, _vp]),
    "attnqat_debug_fwd_p_mx": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _i, _vp,
                                    _vp, _sz, _vp]),
    "attnqat_workspace_bytes": (_sz, [_i, _i, _i, _i, _i, _i]),
    "attnqat_block_k": (_i, []),
    "attnqat_strerror": (ctypes.c_char_p, [_i]),
    "attnqat_debug_fwd_p": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _i, _vp,
                                 _vp, _sz, _vp]),
    "attnqat_debug_bwd_p": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _i, _vp, _vp, _sz, _vp]),
    "attnqat_debug_dkdv_tile_counts": (_i, [_vp, _vp]),
    "attnqat_debug_bwd_waves": (_i, [_i]),
    "attnqat_profile_enable": (_i, [_vp, _i]),
    "attnqat_profile_read": (_i, [_vp, _i, _vp, _vp]),
}
EXPORTS = tuple(_SIGNATURES)

_lib = None


class AttnQatError(RuntimeError):
    pass


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise AttnQatError(
                f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "(hipcc --offload-arch=gfx950). There is no fallback path.")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(rc: int):
    if rc != OK:
        raise AttnQatError(f"attnqat error {rc}: {lib().attnqat_strerror(rc).decode()}")


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _dev_bf16(t, name):
    if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.dim() == 4):
        raise AttnQatError(f"{name} must be a contiguous 4-d bf16 CUDA tensor [B,H,L,d]")


def block_k() -> int:
    return lib().attnqat_block_k()


def workspace_bytes(which: int, B: int, Hq: int, Hkv: int, L: int, d: int) -> int:
    return lib().attnqat_workspace_bytes(which, B, Hq, Hkv, L, d)


def _workspace(which, B, Hq, Hkv, L, d, workspace):
    need = workspace_bytes(which, B, Hq, Hkv, L, d)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
    return workspace, workspace.numel()


def attnqat_quantize(x, want_codes=True, want_xf=True):
    """phi of Eq. 1 along d.  Returns (codes u8 [B,H,L,d/2], scales u8 [B,H,L,d/16], xf bf16)."""
    _dev_bf16(x, "x")
    B, H, L, d = x.shape
    codes = torch.empty((B, H, L, d // 2), dtype=torch.uint8, device=x.device) if want_codes else None
    scales = torch.empty((B, H, L, d // 16), dtype=torch.uint8, device=x.device) if want_codes else None
    xf = torch.empty_like(x) if want_xf else None
    _check(lib().attnqat_quantize(_ptr(x), B, H, L, d, BF16, _ptr(codes), _ptr(scales), _ptr(xf), _stream()))
    return codes, scales, xf


OPT_SMOOTH_K, OPT_TWO_LEVEL_P, OPT_BF16_PV = 1, 2, 4


def attnqat_fwd_infer_mx_sparse(q, k, v, causal: bool, block_mask, workspace=None, out=None):
    """Alg. 1 (MX, FP4 matrix instruction) with a block mask: uint8 CUDA tensor [B,Hq,nb,nb], nb = ceil(L/128), zero =
    the 128 x 128 block is left out.  Returns (o bf16, lse fp32)."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _dev_bf16(t, n)
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    nb = (L + 127) // 128
    if not (block_mask.is_cuda and block_mask.dtype == torch.uint8 and block_mask.is_contiguous()
            and tuple(block_mask.shape) == (B, Hq, nb, nb)):
        raise AttnQatError("block_mask must be a contiguous uint8 CUDA tensor [B,Hq,ceil(L/128),ceil(L/128)]")
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq, L), dtype=torch.float32, device=q.device)
    else:
        o, lse = out
    ws, nbytes = _workspace(WS_FWD_INFER_MX_SPARSE, B, Hq, Hkv, L, d, workspace)
    _check(lib().attnqat_fwd_infer_mx_sparse(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, L, d, int(causal), BF16, _ptr(block_mask),
                                             _ptr(o), _ptr(lse), _ptr(ws), nbytes, _stream()))
    return o, lse


def kv_cache_page_bytes(Hkv: int, d: int) -> int:
    return lib().attnqat_kv_cache_page_bytes(Hkv, d)


def attnqat_kv_cache_write_mx(k, v, cache, page_ids, num_pages=None):
    """Quantize one sequence's k, v [1,Hkv,L,d] bf16 into the pages ``page_ids`` (int32 CUDA tensor) of the FP4 KV
    ``cache`` (uint8 CUDA tensor of num_pages * kv_cache_page_bytes(Hkv, d) bytes)."""
    _dev_bf16(k, "k"); _dev_bf16(v, "v")
    _, Hkv, L, d = k.shape
    if k.shape[0] != 1 or v.shape != k.shape:
        raise AttnQatError("k and v must be [1,Hkv,L,d] of one sequence")
    if not (page_ids.is_cuda and page_ids.dtype == torch.int32 and page_ids.is_contiguous() and page_ids.numel() >= (L + 127) // 128):
        raise AttnQatError("page_ids must be a contiguous int32 CUDA tensor with ceil(L/128) entries")
    if num_pages is None:
        num_pages = cache.numel() // kv_cache_page_bytes(Hkv, d)
    _check(lib().attnqat_kv_cache_write_mx(_ptr(k), _ptr(v), Hkv, L, d, BF16, _ptr(cache), int(num_pages), _ptr(page_ids), _stream()))


def attnqat_fwd_infer_mx_paged(q, cache, num_pages, page_table, kv_lens, Hkv, causal: bool, workspace=None, out=None):
    """Alg. 1 (MX, FP4 matrix instruction) over a paged FP4 KV cache.  q [B,Hq,Lq,d]: the last Lq positions of every
    sequence; page_table int32 [B,max_pages]; kv_lens int32 [B].  Returns (o bf16, lse fp32)."""
    _dev_bf16(q, "q")
    B, Hq, Lq, d = q.shape
    for t, n in ((page_table, "page_table"), (kv_lens, "kv_lens")):
        if not (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
            raise AttnQatError(f"{n} must be a contiguous int32 CUDA tensor")
    if page_table.dim() != 2 or page_table.shape[0] != B or kv_lens.numel() != B:
        raise AttnQatError("page_table must be [B,max_pages] and kv_lens [B]")
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device=q.device)
    else:
        o, lse = out
    ws, nb = _workspace(WS_FWD_INFER_MX_PAGED, B, Hq, Hkv, Lq, d, workspace)
    _check(lib().attnqat_fwd_infer_mx_paged(_ptr(q), B, Hq, Hkv, Lq, d, int(causal), BF16, _ptr(cache), int(num_pages),
                                            _ptr(page_table), page_table.shape[1], _ptr(kv_lens),
                                            _ptr(o), _ptr(lse), _ptr(ws), nb, _stream()))
    return o, lse


def kv_cache_page_bytes_nvfp4(Hkv: int, d: int) -> int:
    return lib().attnqat_kv_cache_page_bytes_nvfp4(Hkv, d)


def attnqat_kv_cache_write(k, v, cache, page_ids, pos0: int = 0, num_pages=None):
    """Quantize positions pos0 .. pos0+n-1 of one sequence, k, v [1,Hkv,n,d] bf16, into the pages ``page_ids`` (int32 CUDA
    tensor, the sequence's page list from its first page on) of the NVFP4 KV ``cache`` (uint8 CUDA tensor)."""
    _dev_bf16(k, "k"); _dev_bf16(v, "v")
    _, Hkv, n, d = k.shape
    if k.shape[0] != 1 or v.shape != k.shape:
        raise AttnQatError("k and v must be [1,Hkv,n,d] of one sequence")
    if not (page_ids.is_cuda and page_ids.dtype == torch.int32 and page_ids.is_contiguous() and page_ids.numel() >= (pos0 + n + 127) // 128):
        raise AttnQatError("page_ids must be a contiguous int32 CUDA tensor with ceil((pos0+n)/128) entries")
    if num_pages is None:
        num_pages = cache.numel() // kv_cache_page_bytes_nvfp4(Hkv, d)
    _check(lib().attnqat_kv_cache_write(_ptr(k), _ptr(v), Hkv, n, d, BF16, int(pos0), _ptr(cache), int(num_pages), _ptr(page_ids), _stream()))


def attnqat_fwd_infer_paged(q, cache, num_pages, page_table, kv_lens, Hkv, causal: bool, workspace=None, out=None, spin_limit=None):
    """Alg. 1 over a paged NVFP4 KV cache.  q [B,Hq,Lq,d]: the last Lq positions of every sequence; page_table int32
    [B,max_pages]; kv_lens int32 [B].  Returns (o bf16, lse fp32); with spin_limit (test hook) also whether a wait of the
    decode path expired."""
    _dev_bf16(q, "q")
    B, Hq, Lq, d = q.shape
    for t, n in ((page_table, "page_table"), (kv_lens, "kv_lens")):
        if not (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
            raise AttnQatError(f"{n} must be a contiguous int32 CUDA tensor")
    if page_table.dim() != 2 or page_table.shape[0] != B or kv_lens.numel() != B:
        raise AttnQatError("page_table must be [B,max_pages] and kv_lens [B]")
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device=q.device)
    else:
        o, lse = out
    max_pages = page_table.shape[1]
    need = lib().attnqat_paged_workspace_bytes(B, Hq, Hkv, Lq, max_pages, d)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
    if spin_limit is not None:
        expired = ctypes.c_int(0)
        _check(lib().attnqat_debug_fwd_infer_paged(_ptr(q), B, Hq, Hkv, Lq, d, int(causal), BF16, _ptr(cache), int(num_pages),
                                                   _ptr(page_table), max_pages, _ptr(kv_lens), _ptr(o), _ptr(lse), _ptr(workspace),
                                                   workspace.numel(), _stream(), int(spin_limit), ctypes.addressof(expired)))
        return o, lse, bool(expired.value)
    _check(lib().attnqat_fwd_infer_paged(_ptr(q), B, Hq, Hkv, Lq, d, int(causal), BF16, _ptr(cache), int(num_pages),
                                         _ptr(page_table), max_pages, _ptr(kv_lens),
                                         _ptr(o), _ptr(lse), _ptr(workspace), workspace.numel(), _stream()))
    return o, lse


def attnqat_debug_fwd_p_opt(q, k, v, causal: bool, row0: int, options: int):
    """attnqat_debug_fwd_p with the option bits of attnqat_fwd_opt."""
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, L), dtype=torch.float32, device=q.device)
    p = torch.zeros((B, Hq, 128, L), dtype=torch.float32, device=q.device)
    ws, nb = _workspace(WS_FWD, B, Hq, Hkv, L, d, None)
    _check(lib().attnqat_debug_fwd_p_opt(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, L, d, int(causal), BF16, int(options),
                                         _ptr(o), _ptr(lse), row0, _ptr(p), _ptr(ws), nb, _stream()))
    return o, lse, p


def attnqat_debug_bwd_p(q, k, v, d_o, lse, o_hp, causal: bool, row0: int):
    """attnqat_bwd that also returns P^F (the re-quantized recomputed P of Alg. 3) of query rows [row0, row0+128):
    (dq, dk, dv, p [B,Hq,128,L] fp32)."""
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    p = torch.zeros((B, Hq, 128, L), dtype=torch.float32, device=q.device)
    ws, nb = _workspace(WS_BWD, B, Hq, Hkv, L, d, None)
    _check(lib().attnqat_debug_bwd_p(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(lse), _ptr(o_hp), B, Hq, Hkv, L, d, int(causal), BF16,
                                     _ptr(dq), _ptr(dk), _ptr(dv), int(row0), _ptr(p), _ptr(ws), nb, _stream()))
    return dq, dk, dv, p


def attnqat_fwd_opt(q, k, v, causal: bool, options: int, train: bool = True, workspace=None, out=None):
    """Alg. 2 (train) or Alg. 1 with the option bits of Sec. 3.2 (OPT_SMOOTH_K).  Returns (o, lse, o_hp or None)."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _dev_bf16(t, n)
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq, L), dtype=torch.float32, device=q.device)
        o_hp = torch.empty((B, Hq, L, d), dtype=torch.float32, device=q.device) if train else None
    else:
        o, lse, o_hp = out
    ws, nb = _workspace(WS_FWD, B, Hq, Hkv, L, d, workspace)
    _check(lib().attnqat_fwd_opt(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, L, d, int(causal), BF16, int(options),
                                 _ptr(o), _ptr(lse), _ptr(o_hp), _ptr(ws), nb, _stream()))
    return o, lse, o_hp


def attnqat_bwd_opt(q, k, v, d_o, lse, o_hp, causal: bool, options: int, workspace=None, out=None):
    """Alg. 3 with the same option bits as the forward.  Returns (dq, dk, dv) bf16."""
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (d_o, "d_o")):
        _dev_bf16(t, n)
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    if out is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    else:
        dq, dk, dv = out
    ws, nb = _workspace(WS_BWD, B, Hq, Hkv, L, d, workspace)
    _check(lib().attnqat_bwd_opt(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(lse), _ptr(o_hp),
                                 B, Hq, Hkv, L, d, int(causal), BF16, int(options),
                                 _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), nb, _stream()))
    return dq, dk, dv


def attnqat_fwd_mx(q, k, v, causal: bool, workspace=None, out=None):
    """Alg. 2 in the MX format (16-bit matrix path).  Returns (o bf16, lse fp32 [B,Hq,L], o_hp fp32)."""
    return attnqat_fwd(q, k, v, causal, workspace, out, _mx=True)


def attnqat_bwd_mx(q, k, v, d_o, lse, o_hp, causal: bool, workspace=None, out=None):
    """Alg. 3 in the MX format.  Returns (dq, dk, dv) bf16."""
    return attnqat_bwd(q, k, v, d_o, lse, o_hp, causal, workspace, out, _mx=True)


def attnqat_fwd(q, k, v, causal: bool, workspace=None, out=None, _mx=False):
    """Alg. 2.  Returns (o bf16, lse fp32 [B,Hq,L], o_hp fp32)."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _dev_bf16(t, n)
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq, L), dtype=torch.float32, device=q.device)
        o_hp = torch.empty((B, Hq, L, d), dtype=torch.float32, device=q.device)
    else:
        o, lse, o_hp = out
    ws, nb = _workspace(WS_FWD_MX if _mx else WS_FWD, B, Hq, Hkv, L, d, workspace)
    _check((lib().attnqat_fwd_mx if _mx else lib().attnqat_fwd)(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, L, d, int(causal), BF16,
                             _ptr(o), _ptr(lse), _ptr(o_hp), _ptr(ws), nb, _stream()))
    return o, lse, o_hp


def attnqat_fwd_infer(q, k, v, causal: bool, workspace=None, out=None):
    """Alg. 1.  Returns (o bf16, lse fp32)."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _dev_bf16(t, n)
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq, L), dtype=torch.float32, device=q.device)
    else:
        o, lse = out
    ws, nb = _workspace(WS_FWD_INFER, B, Hq, Hkv, L, d, workspace)
    _check(lib().attnqat_fwd_infer(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, L, d, int(causal), BF16,
                                   _ptr(o), _ptr(lse), _ptr(ws), nb, _stream()))
    return o, lse


def attnqat_fwd_infer_bf16pv(q, k, v, causal: bool, workspace=None, out=None):
    """Alg. 1 in the mixed recipe of Sec. 2.5: NVFP4 Q K^T, P-tilde and V in bf16.  Returns (o bf16, lse fp32)."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _dev_bf16(t, n)
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq, L), dtype=torch.float32, device=q.device)
    else:
        o, lse = out
    ws, nb = _workspace(WS_FWD_INFER, B, Hq, Hkv, L, d, workspace)
    _check(lib().attnqat_fwd_infer_bf16pv(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, L, d, int(causal), BF16,
                                          _ptr(o), _ptr(lse), _ptr(ws), nb, _stream()))
    return o, lse


def attnqat_fwd_infer_static(q, k, v, causal: bool, out):
    """attnqat_fwd_infer on the library's static scratch array: allocates nothing, so the outputs (o bf16, lse fp32)
    must be passed in.  Raises for problems that need more than STATIC_SCRATCH_BYTES of scratch."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _dev_bf16(t, n)
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    o, lse = out
    _check(lib().attnqat_fwd_infer_static(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, L, d, int(causal), BF16,
                                          _ptr(o), _ptr(lse), _stream()))
    return o, lse


def attnqat_fwd_infer_packed(qp, kp, vp, causal: bool, d: int, workspace=None, out=None):
    """Alg. 1 on already quantized tensors: qp, kp, vp are (codes, scales) pairs from attnqat_quantize.
    Returns (o bf16, lse fp32), bit-identical to attnqat_fwd_infer on the tensors the codes came from."""
    (qc, qs), (kc, ks), (vc, vs) = qp, kp, vp
    B, Hq, L, _ = qc.shape
    Hkv = kc.shape[1]
    if out is None:
        o = torch.empty((B, Hq, L, d), dtype=torch.bfloat16, device=qc.device)
        lse = torch.empty((B, Hq, L), dtype=torch.float32, device=qc.device)
    else:
        o, lse = out
    ws, nb = _workspace(WS_FWD_INFER, B, Hq, Hkv, L, d, workspace)
    _check(lib().attnqat_fwd_infer_packed(_ptr(qc), _ptr(qs), _ptr(kc), _ptr(ks), _ptr(vc), _ptr(vs), B, Hq, Hkv, L, d,
                                          int(causal), BF16, _ptr(o), _ptr(lse), _ptr(ws), nb, _stream()))
    return o, lse


def attnqat_bwd_packed(qp, kp, vp, d_o, lse, o_hp, causal: bool, workspace=None, out=None):
    """Alg. 3 from the saved quantized Q, K, V of the forward ((codes, scales) pairs).  Returns (dq, dk, dv) bf16."""
    (qc, qs), (kc, ks), (vc, vs) = qp, kp, vp
    _dev_bf16(d_o, "d_o")
    B, Hq, L, d = d_o.shape
    Hkv = kc.shape[1]
    if out is None:
        dq = torch.empty_like(d_o)
        dk = torch.empty((B, Hkv, L, d), dtype=torch.bfloat16, device=d_o.device)
        dv = torch.empty_like(dk)
    else:
        dq, dk, dv = out
    ws, nb = _workspace(WS_BWD, B, Hq, Hkv, L, d, workspace)
    _check(lib().attnqat_bwd_packed(_ptr(qc), _ptr(qs), _ptr(kc), _ptr(ks), _ptr(vc), _ptr(vs), _ptr(d_o), _ptr(lse), _ptr(o_hp),
                                    B, Hq, Hkv, L, d, int(causal), BF16, _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), nb, _stream()))
    return dq, dk, dv


def attnqat_quantize_mx(x, axis: int = 0, want_codes=True, want_xf=True):
    """MX phi (E2M1, blocks of 32, E8M0 scale) along d (axis 0) or along the sequence (axis 1).
    Returns (codes u8, scales u8, xf bf16): axis 0 [B,H,L,d/2], [B,H,L,d/32]; axis 1 [B,H,d,Lc/2],
    [B,H,d,Lc/32] with Lc = L rounded up to 32."""
    _dev_bf16(x, "x")
    B, H, L, d = x.shape
    if axis == 0:
        cshape, sshape = (B, H, L, d // 2), (B, H, L, d // 32)
    else:
        Lc = (L + 31) // 32 * 32
        cshape, sshape = (B, H, d, Lc // 2), (B, H, d, Lc // 32)
    codes = torch.empty(cshape, dtype=torch.uint8, device=x.device) if want_codes else None
    scales = torch.empty(sshape, dtype=torch.uint8, device=x.device) if want_codes else None
    xf = torch.empty_like(x) if want_xf else None
    _check(lib().attnqat_quantize_mx(_ptr(x), B, H, L, d, BF16, int(axis), _ptr(codes), _ptr(scales), _ptr(xf), _stream()))
    return codes, scales, xf


def attnqat_quantize_mxfp8(x, want_codes=True, want_xf=True):
    """MXFP8 phi (E4M3 elements, blocks of 32 along the sequence, E8M0 scale): how V is held in the mixed recipe.
    Returns (codes u8 [B,H,d,Lc], scales u8 [B,H,d,Lc/32], xf bf16) with Lc = L rounded up to 32."""
    _dev_bf16(x, "x")
    B, H, L, d = x.shape
    Lc = (L + 31) // 32 * 32
    codes = torch.empty((B, H, d, Lc), dtype=torch.uint8, device=x.device) if want_codes else None
    scales = torch.empty((B, H, d, Lc // 32), dtype=torch.uint8, device=x.device) if want_codes else None
    xf = torch.empty_like(x) if want_xf else None
    _check(lib().attnqat_quantize_mxfp8(_ptr(x), B, H, L, d, BF16, 1, _ptr(codes), _ptr(scales), _ptr(xf), _stream()))
    return codes, scales, xf


def attnqat_fwd_infer_mx_fp8pv(q, k, v, causal: bool, workspace=None, out=None):
    """Alg. 1, mixed recipe: FP4 (MX) Q K^T, MXFP8 P V.  Returns (o bf16, lse fp32)."""
    return attnqat_fwd_infer_mx(q, k, v, causal, workspace, out, _fp8pv=True)


def attnqat_fwd_infer_mx(q, k, v, causal: bool, workspace=None, out=None, _fp8pv=False):
    """Alg. 1 in the MX format on the scaled FP4 MFMA.  Returns (o bf16, lse fp32)."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _dev_bf16(t, n)
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq, L), dtype=torch.float32, device=q.device)
    else:
        o, lse = out
    ws, nb = _workspace(WS_FWD_INFER_MX_FP8PV if _fp8pv else WS_FWD_INFER_MX, B, Hq, Hkv, L, d, workspace)
    _check((lib().attnqat_fwd_infer_mx_fp8pv if _fp8pv else lib().attnqat_fwd_infer_mx)(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, L, d, int(causal), BF16,
                                      _ptr(o), _ptr(lse), _ptr(ws), nb, _stream()))
    return o, lse


def attnqat_bwd(q, k, v, d_o, lse, o_hp, causal: bool, workspace=None, out=None, _mx=False):
    """Alg. 3.  Returns (dq, dk, dv) bf16."""
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (d_o, "d_o")):
        _dev_bf16(t, n)
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    if not (lse.dtype == torch.float32 and lse.is_contiguous() and o_hp.dtype == torch.float32
            and o_hp.is_contiguous()):
        raise AttnQatError("lse and o_hp must be contiguous fp32 tensors")
    if out is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    else:
        dq, dk, dv = out
    ws, nb = _workspace(WS_BWD_MX if _mx else WS_BWD, B, Hq, Hkv, L, d, workspace)
    _check((lib().attnqat_bwd_mx if _mx else lib().attnqat_bwd)(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(lse), _ptr(o_hp),
                             B, Hq, Hkv, L, d, int(causal), BF16,
                             _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), nb, _stream()))
    return dq, dk, dv


ABL_D_FROM_O, ABL_P_UNQUANTIZED = 1, 2


def attnqat_bwd_ablation(q, k, v, d_o, lse, o_hp, o, causal: bool, ablation: int, workspace=None, out=None):
    """Alg. 3 with the ablations of Sec. 3.2 switched on by the bit set ``ablation``
    (ABL_D_FROM_O: D from the bf16 output ``o``; ABL_P_UNQUANTIZED: dV from the fp32 P).
    Returns (dq, dk, dv) bf16."""
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (d_o, "d_o")):
        _dev_bf16(t, n)
    if ablation & ABL_D_FROM_O:
        _dev_bf16(o, "o")
    elif not (o_hp.dtype == torch.float32 and o_hp.is_contiguous()):
        raise AttnQatError("o_hp must be a contiguous fp32 tensor")
    if not (lse.dtype == torch.float32 and lse.is_contiguous()):
        raise AttnQatError("lse must be a contiguous fp32 tensor")
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    if out is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    else:
        dq, dk, dv = out
    ws, nb = _workspace(WS_BWD, B, Hq, Hkv, L, d, workspace)
    _check(lib().attnqat_bwd_ablation(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(lse),
                                      _ptr(o_hp) if o_hp is not None else None, _ptr(o) if o is not None else None,
                                      B, Hq, Hkv, L, d, int(causal), BF16, int(ablation),
                                      _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), nb, _stream()))
    return dq, dk, dv


def attnqat_debug_fwd_p_mx(q, k, v, causal: bool, row0: int):
    """attnqat_debug_fwd_p for the MX forward of attnqat_fwd_mx."""
    return attnqat_debug_fwd_p(q, k, v, causal, row0, _mx=True)


def attnqat_debug_fwd_p(q, k, v, causal: bool, row0: int, _mx=False):
    """Test hook: (o, lse, P-tilde^F fp32 [B,Hq,128,L]) for query rows [row0, row0+128)."""
    B, Hq, L, d = q.shape
    Hkv = k.shape[1]
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, L), dtype=torch.float32, device=q.device)
    p = torch.zeros((B, Hq, 128, L), dtype=torch.float32, device=q.device)    # skipped (masked) tiles are not written
    ws, nb = _workspace(WS_FWD_MX if _mx else WS_FWD_INFER, B, Hq, Hkv, L, d, None)
    _check((lib().attnqat_debug_fwd_p_mx if _mx else lib().attnqat_debug_fwd_p)(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, L, d, int(causal), BF16,
                                     _ptr(o), _ptr(lse), row0, _ptr(p), _ptr(ws), nb, _stream()))
    return o, lse, p


def debug_dkdv_tile_counts(counts):
    """counts: zeroed int64 CUDA tensor of 2 elements (tiles visited, tiles with non-zero P^F) or None; applies to
    attnqat_bwd calls on the current stream."""
    _check(lib().attnqat_debug_dkdv_tile_counts(_stream(), _ptr(counts) if counts is not None else None))


def debug_bwd_waves(waves: int):
    """Force the workgroup shape of the dQ and dK/dV passes (4 or 8 waves; 0 = automatic).  Process-wide."""
    _check(lib().attnqat_debug_bwd_waves(int(waves)))


def profile_enable(on: bool):
    """Per-kernel timing of the calls made on the current stream."""
    _check(lib().attnqat_profile_enable(_stream(), int(on)))


def profile_read():
    """[(kernel label, milliseconds)] of the most recent call on the current stream; synchronise the stream first."""
    ms = (ctypes.c_float * 16)()
    names = (ctypes.c_char_p * 16)()
    n = lib().attnqat_profile_read(_stream(), 16, ctypes.cast(ms, ctypes.c_void_p), ctypes.cast(names, ctypes.c_void_p))
    if n < 0:
        _check(n)
    return [(names[i].decode(), float(ms[i])) for i in range(n)]
