"""MI355X-native hot path of one DualDiffusion draft-then-verify step.

Thin ctypes binding over the C ABI in ``include/dd.h`` (``libdd.so``, hand-written
gfx950 HIP kernels).  The functions here have the C entry points' names and only
marshal arguments: torch tensors supply device memory and the current stream, every
step of the computation runs in the library's kernels.  There is no CPU fallback:
if the library cannot be loaded, importing the binding's functions raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

F32, BF16, FP8_E4M3 = 0, 1, 2
TRUST, KL_THRESH, CONF_THRESH, KL_PROB, CONF_PROB, KL_TOPK, CONF_TOPK = 0, 1, 2, 3, 4, 5, 6
UNMASK_THRESH, UNMASK_TOPK = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdd.so")
_lib = None


class DDError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().dd_strerror(status).decode()} (status {status})")


def lib():
    """The loaded C-ABI library (built on first use only when no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from .build import build_library
        build_library(force=True)
    # torch ships its own copy of the HIP runtime (same soname).  It has to be mapped first so
    # that this library binds to that copy: streams and device pointers handed over by torch
    # are only valid inside the runtime instance that created them.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i, sz = C.c_void_p, C.c_int, C.c_size_t
    L.dd_strerror.restype = C.c_char_p
    L.dd_strerror.argtypes = [i]
    L.dd_version.restype = i
    L.dd_bidir_attention.restype = i
    L.dd_bidir_attention.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, vp, vp, vp, sz, vp]
    L.dd_bidir_attention_workspace_bytes.restype = sz
    L.dd_bidir_attention_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    L.dd_block_attention_cached.restype = i
    L.dd_block_attention_cached.argtypes = [vp, vp, vp, vp, i, i, vp, vp, i, i, i, i, i, i, i, vp, vp, vp, sz, vp]
    L.dd_block_attention_cached_workspace_bytes.restype = sz
    L.dd_block_attention_cached_workspace_bytes.argtypes = [i, i, i, i, i, i, i, i]
    L.dd_bidir_attention_fp8v.restype = i
    L.dd_bidir_attention_fp8v.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp, vp, vp, vp]
    L.dd_bidir_attention_mx.restype = i
    L.dd_bidir_attention_mx.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, vp]
    L.dd_block_attention_cached_fp8v.restype = i
    L.dd_block_attention_cached_fp8v.argtypes = [vp, vp, vp, vp, i, i, vp, vp, i, i, i, i, i, vp, vp, vp, vp, sz, vp]
    L.dd_block_attention_cached_fp8v_workspace_bytes.restype = sz
    L.dd_block_attention_cached_fp8v_workspace_bytes.argtypes = [i, i, i, i, i, i]
    L.dd_verify_remask.restype = i
    L.dd_verify_remask.argtypes = [vp, vp, vp, i, C.c_float, C.c_uint64, vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.dd_verify_remask_workspace_bytes.restype = sz
    L.dd_verify_remask_workspace_bytes.argtypes = [i, i, i, i]
    L.dd_verify_remask_static.restype = i
    L.dd_verify_remask_static.argtypes = [vp, vp, vp, i, C.c_float, C.c_uint64, vp, vp, vp, i, i, i, i, vp]
    L.dd_unmask.restype = i
    L.dd_unmask.argtypes = [vp, vp, i, C.c_float, vp, vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.dd_unmask_workspace_bytes.restype = sz
    L.dd_unmask_workspace_bytes.argtypes = [i, i, i, i]
    L.dd_block_attention_refresh.restype = i
    L.dd_block_attention_refresh.argtypes = [vp, vp, vp, vp, i, i, vp, vp, i, i, i, i, i, i, i, vp, vp, vp, sz, vp]
    L.dd_block_attention_refresh_workspace_bytes.restype = sz
    L.dd_block_attention_refresh_workspace_bytes.argtypes = [i, i, i, i, i, i, i, i]
    L.dd_block_attention_window.restype = i
    L.dd_block_attention_window.argtypes = [vp, vp, vp, vp, i, i, i, i, vp, vp, i, i, i, i, i, i, i, vp, vp, vp, sz, vp]
    L.dd_block_attention_window_workspace_bytes.restype = sz
    L.dd_block_attention_window_workspace_bytes.argtypes = [i, i, i, i, i, i, i, i, i]
    L.dd_block_attention_batched.restype = i
    L.dd_block_attention_batched.argtypes = [vp, vp, vp, vp, vp, i, vp, vp, i, i, i, i, i, i, i, vp, vp, vp, sz, vp]
    L.dd_block_attention_batched_workspace_bytes.restype = sz
    L.dd_block_attention_batched_workspace_bytes.argtypes = [i, i, i, i, i, i, i, i]
    L.dd_cache_insert_rows.restype = i
    L.dd_cache_insert_rows.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
    L.dd_verify_scores.restype = i
    L.dd_verify_scores.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, vp, sz, vp]
    L.dd_verify_scores_workspace_bytes.restype = sz
    L.dd_verify_scores_workspace_bytes.argtypes = [i, i, i]
    _lib = L
    return L


EXPORTS = ("dd_strerror", "dd_version", "dd_bidir_attention", "dd_bidir_attention_workspace_bytes",
           "dd_block_attention_cached", "dd_block_attention_cached_workspace_bytes",
           "dd_verify_remask", "dd_verify_remask_workspace_bytes", "dd_verify_remask_static", "dd_unmask", "dd_unmask_workspace_bytes",
           "dd_verify_scores", "dd_verify_scores_workspace_bytes",
           "dd_block_attention_refresh", "dd_block_attention_refresh_workspace_bytes",
           "dd_block_attention_window", "dd_block_attention_window_workspace_bytes", "dd_cache_insert_rows",
           "dd_block_attention_batched", "dd_block_attention_batched_workspace_bytes",
           "dd_bidir_attention_fp8v", "dd_block_attention_cached_fp8v", "dd_block_attention_cached_fp8v_workspace_bytes",
           "dd_bidir_attention_mx")


# ---------------------------------------------------------------- marshalling helpers
def _torch():
    import torch
    return torch


def _dtype_tag(t, what: str) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return F32
    if t.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        return BF16
    if t.dtype in (torch.uint8, torch.float8_e4m3fn):
        return FP8_E4M3
    raise TypeError(f"{what}: unsupported tensor dtype {t.dtype}")


def _dev(t, what: str):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{what}: must live in GPU memory")
    if not t.is_contiguous():
        raise ValueError(f"{what}: must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    """torch's current HIP stream on the current device, as a raw handle."""
    torch = _torch()
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)       # a few times cheaper than the Stream object
    if raw is not None:
        return raw(torch.cuda.current_device())
    return torch.cuda.current_stream().cuda_stream


_ws_cache = {}


def _workspace(nbytes: int, device):
    """A scratch tensor per (device, stream) - device memory only; the library never allocates.  Calls on one
    stream run in order and may share it; calls on different streams may overlap and must not."""
    if nbytes == 0:
        return None, 0
    global _ws_peak
    torch = _torch()
    _ws_peak = max(_ws_peak, nbytes)
    if _ws_fixed is not None:
        if _ws_fixed.numel() < nbytes or _ws_fixed.device != device:
            raise RuntimeError(f"the fixed workspace holds {_ws_fixed.numel()} bytes on {_ws_fixed.device}; "
                               f"this call needs {nbytes} on {device}")
        return _ws_fixed, _ws_fixed.numel()
    if torch.cuda.is_current_stream_capturing():
        # memory allocated under capture would come from that graph's private pool and a cached tensor of it
        # could be handed to a later, unrelated call: the scratch memory of captured calls is allocated beforehand
        raise RuntimeError("a call that needs scratch memory is being captured without a fixed workspace: "
                           "capture through paper_2604_05250_amd.step.capture_step, or inside fixed_workspace()")
    key = (device, _stream())
    cur = _ws_cache.get(key)
    if cur is None or cur.numel() < nbytes:
        cur = torch.empty(max(nbytes, 1 << 20), dtype=torch.uint8, device=device)
        _ws_cache[key] = cur
    return cur, cur.numel()


_ws_fixed = None      # set by fixed_workspace(): every call inside uses this tensor
_ws_peak = 0          # largest scratch size any call has asked for since reset_workspace_peak()


def reset_workspace_peak() -> None:
    global _ws_peak
    _ws_peak = 0


def workspace_peak() -> int:
    return _ws_peak


class fixed_workspace:
    """Context manager: calls of the binding inside it use `tensor` (uint8, on the GPU) as their scratch memory
    instead of the per-stream cached one; they must all be ordered on one stream.  For graph capture: the
    tensor is allocated before the capture and kept alive by whoever keeps the graph."""

    def __init__(self, tensor):
        self.tensor = tensor

    def __enter__(self):
        global _ws_fixed
        self.prev, _ws_fixed = _ws_fixed, self.tensor
        return self.tensor

    def __exit__(self, *exc):
        global _ws_fixed
        _ws_fixed = self.prev
        return False


def _check_vec(t, n, dtype, what):
    """A per-position vector handed to the library: n elements of the given torch dtype (or None)."""
    if t is None:
        return
    if t.dtype != dtype or t.numel() != n:
        raise ValueError(f"{what}: must have {n} elements of {dtype}, has {t.numel()} of {t.dtype}")


# ---------------------------------------------------------------- entry points
def dd_bidir_attention_workspace_bytes(B, H, Hkv, N, d, qk_dtype, v_dtype) -> int:
    return lib().dd_bidir_attention_workspace_bytes(B, H, Hkv, N, d, qk_dtype, v_dtype)


def dd_bidir_attention(Q, K, V, O=None, q_scale=None, k_scale=None, qk_dtype: Optional[int] = None,
                       v_dtype: Optional[int] = None):
    """Verifier attention over all positions.  Q [B,H,N,d], K,V [B,Hkv,N,d] -> O [B,H,N,d] (V's type)."""
    torch = _torch()
    B, H, N, d = Q.shape
    Hkv = K.shape[1]
    if tuple(K.shape) != (B, Hkv, N, d) or tuple(V.shape) != (B, Hkv, N, d):
        raise ValueError("K/V shape must be [B,Hkv,N,d] matching Q")
    qk = _dtype_tag(Q, "Q") if qk_dtype is None else qk_dtype
    vd = _dtype_tag(V, "V") if v_dtype is None else v_dtype
    if O is None:
        O = torch.empty((B, H, N, d), dtype=V.dtype, device=V.device)
    ws, wsn = _workspace(dd_bidir_attention_workspace_bytes(B, H, Hkv, N, d, qk, vd), Q.device)
    rc = lib().dd_bidir_attention(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(O, "O"), B, H, Hkv, N, d, qk, vd,
                                  _dev(q_scale, "q_scale"), _dev(k_scale, "k_scale"), _dev(ws, "workspace"), wsn,
                                  _stream())
    if rc != 0:
        raise DDError(rc, "dd_bidir_attention")
    return O


def dd_block_attention_cached_workspace_bytes(block_len, B, H, Hkv, N, d, qk_dtype, v_dtype) -> int:
    return lib().dd_block_attention_cached_workspace_bytes(block_len, B, H, Hkv, N, d, qk_dtype, v_dtype)


def dd_block_attention_cached(Qblk, Kc, Vc, block_start: int, O=None, Kblk=None, Vblk=None, q_scale=None,
                              k_scale=None, qk_dtype: Optional[int] = None, v_dtype: Optional[int] = None,
                              _refresh: bool = False):
    """Drafter attention: the active block's queries over cached K/V.
    Qblk [B,H,bl,d], Kc,Vc [B,Hkv,N,d], optional Kblk,Vblk [B,Hkv,bl,d] -> O [B,H,bl,d]."""
    torch = _torch()
    fn = lib().dd_block_attention_refresh if _refresh else lib().dd_block_attention_cached
    name = "dd_block_attention_refresh" if _refresh else "dd_block_attention_cached"
    B, H, bl, d = Qblk.shape
    _, Hkv, N, _ = Kc.shape
    if tuple(Kc.shape) != (B, Hkv, N, d) or tuple(Vc.shape) != (B, Hkv, N, d):
        raise ValueError("Kc/Vc shape must be [B,Hkv,N,d]")
    if Kblk is not None and (tuple(Kblk.shape) != (B, Hkv, bl, d) or tuple(Vblk.shape) != (B, Hkv, bl, d)):
        raise ValueError("Kblk/Vblk shape must be [B,Hkv,block_len,d]")
    qk = _dtype_tag(Qblk, "Qblk") if qk_dtype is None else qk_dtype
    vd = _dtype_tag(Vc, "Vc") if v_dtype is None else v_dtype
    if O is None:
        O = torch.empty((B, H, bl, d), dtype=Vc.dtype, device=Vc.device)
    ws, wsn = _workspace(dd_block_attention_cached_workspace_bytes(bl, B, H, Hkv, N, d, qk, vd), Qblk.device)
    rc = fn(_dev(Qblk, "Qblk"), _dev(Kc, "Kc"), _dev(Vc, "Vc"), _dev(O, "O"),
            int(block_start), bl, _dev(Kblk, "Kblk"), _dev(Vblk, "Vblk"),
            B, H, Hkv, N, d, qk, vd, _dev(q_scale, "q_scale"), _dev(k_scale, "k_scale"),
            _dev(ws, "workspace"), wsn, _stream())
    if rc != 0:
        raise DDError(rc, name)
    return O


def dd_bidir_attention_fp8v(Q, K, V, q_scale, k_scale, v_scale, O=None):
    """Verifier attention with Q, K and V all stored as e4m3 codes (uint8) and per-head fp32 scales -> O bf16
    (as int16 bit patterns unless O is given)."""
    torch = _torch()
    B, H, N, d = Q.shape
    Hkv = K.shape[1]
    if tuple(K.shape) != (B, Hkv, N, d) or tuple(V.shape) != (B, Hkv, N, d):
        raise ValueError("K/V shape must be [B,Hkv,N,d] matching Q")
    for t, what in ((Q, "Q"), (K, "K"), (V, "V")):
        if t.element_size() != 1:
            raise TypeError(f"{what}: one byte per element (e4m3 codes) expected")
    if O is None:
        O = torch.empty((B, H, N, d), dtype=torch.int16, device=V.device)
    rc = lib().dd_bidir_attention_fp8v(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(O, "O"), B, H, Hkv, N, d,
                                       _dev(q_scale, "q_scale"), _dev(k_scale, "k_scale"), _dev(v_scale, "v_scale"),
                                       _stream())
    if rc != 0:
        raise DDError(rc, "dd_bidir_attention_fp8v")
    return O


def dd_bidir_attention_mx(Q, Qs, K, Ks, V, Vs, O=None):
    """Verifier attention on block-scaled inputs: Q [B,H,N,d], K [B,Hkv,N,d] e4m3 codes, V [B,Hkv,N,d/2] packed e2m1
    codes, each with E8M0 scales [..., d/32] (all uint8) -> O bf16 (as int16 bit patterns unless O is given)."""
    torch = _torch()
    B, H, N, d = Q.shape
    Hkv = K.shape[1]
    if tuple(K.shape) != (B, Hkv, N, d) or tuple(V.shape) != (B, Hkv, N, d // 2):
        raise ValueError("K must be [B,Hkv,N,d] and V [B,Hkv,N,d/2] matching Q")
    if tuple(Qs.shape) != (B, H, N, d // 32) or tuple(Ks.shape) != (B, Hkv, N, d // 32) or tuple(Vs.shape) != (B, Hkv, N, d // 32):
        raise ValueError("scales must be [..., d/32] matching their tensors")
    for t, what in ((Q, "Q"), (K, "K"), (V, "V"), (Qs, "Qs"), (Ks, "Ks"), (Vs, "Vs")):
        if t.element_size() != 1:
            raise TypeError(f"{what}: one byte per entry expected")
    if O is None:
        O = torch.empty((B, H, N, d), dtype=torch.int16, device=V.device)
    rc = lib().dd_bidir_attention_mx(_dev(Q, "Q"), _dev(Qs, "Qs"), _dev(K, "K"), _dev(Ks, "Ks"), _dev(V, "V"),
                                     _dev(Vs, "Vs"), _dev(O, "O"), B, H, Hkv, N, d, _stream())
    if rc != 0:
        raise DDError(rc, "dd_bidir_attention_mx")
    return O


def dd_block_attention_cached_fp8v(Qblk, Kc, Vc, block_start: int, q_scale, k_scale, v_scale, O=None, Kblk=None, Vblk=None):
    """Drafter attention with every operand stored as e4m3 codes; shapes as for dd_block_attention_cached -> O bf16."""
    torch = _torch()
    B, H, bl, d = Qblk.shape
    _, Hkv, N, _ = Kc.shape
    if tuple(Kc.shape) != (B, Hkv, N, d) or tuple(Vc.shape) != (B, Hkv, N, d):
        raise ValueError("Kc/Vc shape must be [B,Hkv,N,d]")
    if Kblk is not None and (tuple(Kblk.shape) != (B, Hkv, bl, d) or tuple(Vblk.shape) != (B, Hkv, bl, d)):
        raise ValueError("Kblk/Vblk shape must be [B,Hkv,block_len,d]")
    for t, what in ((Qblk, "Qblk"), (Kc, "Kc"), (Vc, "Vc")):
        if t.element_size() != 1:
            raise TypeError(f"{what}: one byte per element (e4m3 codes) expected")
    if O is None:
        O = torch.empty((B, H, bl, d), dtype=torch.int16, device=Vc.device)
    ws, wsn = _workspace(lib().dd_block_attention_cached_fp8v_workspace_bytes(bl, B, H, Hkv, N, d), Qblk.device)
    rc = lib().dd_block_attention_cached_fp8v(_dev(Qblk, "Qblk"), _dev(Kc, "Kc"), _dev(Vc, "Vc"), _dev(O, "O"),
                                              int(block_start), bl, _dev(Kblk, "Kblk"), _dev(Vblk, "Vblk"),
                                              B, H, Hkv, N, d, _dev(q_scale, "q_scale"), _dev(k_scale, "k_scale"),
                                              _dev(v_scale, "v_scale"), _dev(ws, "workspace"), wsn, _stream())
    if rc != 0:
        raise DDError(rc, "dd_block_attention_cached_fp8v")
    return O


def dd_block_attention_refresh_workspace_bytes(block_len, B, H, Hkv, N, d, qk_dtype, v_dtype) -> int:
    return lib().dd_block_attention_refresh_workspace_bytes(block_len, B, H, Hkv, N, d, qk_dtype, v_dtype)


def dd_block_attention_refresh(Qblk, Kc, Vc, block_start: int, Kblk, Vblk, O=None, q_scale=None, k_scale=None,
                               qk_dtype: Optional[int] = None, v_dtype: Optional[int] = None):
    """Drafter attention of a completed block: as dd_block_attention_cached with Kblk/Vblk, and rows
    [block_start, block_start + bl) of Kc / Vc are overwritten with Kblk / Vblk in the same call."""
    return dd_block_attention_cached(Qblk, Kc, Vc, block_start, O=O, Kblk=Kblk, Vblk=Vblk, q_scale=q_scale,
                                     k_scale=k_scale, qk_dtype=qk_dtype, v_dtype=v_dtype, _refresh=True)


def dd_block_attention_window_workspace_bytes(block_len, win_len, B, H, Hkv, N, d, qk_dtype, v_dtype) -> int:
    return lib().dd_block_attention_window_workspace_bytes(block_len, win_len, B, H, Hkv, N, d, qk_dtype, v_dtype)


def dd_block_attention_window(Qblk, Kc, Vc, block_start: int, win_start: int, win_len: int, O=None, Kblk=None,
                              Vblk=None, q_scale=None, k_scale=None, qk_dtype: Optional[int] = None,
                              v_dtype: Optional[int] = None):
    """Drafter attention over the key rows [win_start, win_start + win_len) of the cache only.
    Shapes as for dd_block_attention_cached (Kc, Vc are the whole cache)."""
    torch = _torch()
    B, H, bl, d = Qblk.shape
    _, Hkv, N, _ = Kc.shape
    if tuple(Kc.shape) != (B, Hkv, N, d) or tuple(Vc.shape) != (B, Hkv, N, d):
        raise ValueError("Kc/Vc shape must be [B,Hkv,N,d]")
    if Kblk is not None and (tuple(Kblk.shape) != (B, Hkv, bl, d) or tuple(Vblk.shape) != (B, Hkv, bl, d)):
        raise ValueError("Kblk/Vblk shape must be [B,Hkv,block_len,d]")
    qk = _dtype_tag(Qblk, "Qblk") if qk_dtype is None else qk_dtype
    vd = _dtype_tag(Vc, "Vc") if v_dtype is None else v_dtype
    if O is None:
        O = torch.empty((B, H, bl, d), dtype=Vc.dtype, device=Vc.device)
    ws, wsn = _workspace(dd_block_attention_window_workspace_bytes(bl, int(win_len), B, H, Hkv, N, d, qk, vd), Qblk.device)
    rc = lib().dd_block_attention_window(_dev(Qblk, "Qblk"), _dev(Kc, "Kc"), _dev(Vc, "Vc"), _dev(O, "O"),
                                         int(block_start), bl, int(win_start), int(win_len),
                                         _dev(Kblk, "Kblk"), _dev(Vblk, "Vblk"), B, H, Hkv, N, d, qk, vd,
                                         _dev(q_scale, "q_scale"), _dev(k_scale, "k_scale"),
                                         _dev(ws, "workspace"), wsn, _stream())
    if rc != 0:
        raise DDError(rc, "dd_block_attention_window")
    return O


def dd_block_attention_batched(Qblk, Kc, Vc, block_starts, Kblk, Vblk, O=None, q_scale=None, k_scale=None,
                               qk_dtype: Optional[int] = None, v_dtype: Optional[int] = None):
    """Drafter attention with one block position per batch entry: block_starts [B] i32 on the device."""
    torch = _torch()
    B, H, bl, d = Qblk.shape
    _, Hkv, N, _ = Kc.shape
    if tuple(Kc.shape) != (B, Hkv, N, d) or tuple(Vc.shape) != (B, Hkv, N, d):
        raise ValueError("Kc/Vc shape must be [B,Hkv,N,d]")
    if tuple(Kblk.shape) != (B, Hkv, bl, d) or tuple(Vblk.shape) != (B, Hkv, bl, d):
        raise ValueError("Kblk/Vblk shape must be [B,Hkv,block_len,d]")
    if block_starts.dtype != torch.int32 or block_starts.numel() != B:
        raise ValueError("block_starts must be int32 with B entries")
    qk = _dtype_tag(Qblk, "Qblk") if qk_dtype is None else qk_dtype
    vd = _dtype_tag(Vc, "Vc") if v_dtype is None else v_dtype
    if O is None:
        O = torch.empty((B, H, bl, d), dtype=Vc.dtype, device=Vc.device)
    ws, wsn = _workspace(lib().dd_block_attention_batched_workspace_bytes(bl, B, H, Hkv, N, d, qk, vd), Qblk.device)
    rc = lib().dd_block_attention_batched(_dev(Qblk, "Qblk"), _dev(Kc, "Kc"), _dev(Vc, "Vc"), _dev(O, "O"),
                                          _dev(block_starts, "block_starts"), bl, _dev(Kblk, "Kblk"), _dev(Vblk, "Vblk"),
                                          B, H, Hkv, N, d, qk, vd, _dev(q_scale, "q_scale"), _dev(k_scale, "k_scale"),
                                          _dev(ws, "workspace"), wsn, _stream())
    if rc != 0:
        raise DDError(rc, "dd_block_attention_batched")
    return O


def dd_cache_insert_rows(Kc, Vc, Krows, Vrows, positions, qk_dtype: Optional[int] = None, v_dtype: Optional[int] = None):
    """Kc/Vc [B,Hkv,N,d] <- rows of Krows/Vrows [B,Hkv,n,d] at positions [B,n] (i32, on the device; entries outside
    [0, N) skip their row).  In place; returns None."""
    torch = _torch()
    B, Hkv, N, d = Kc.shape
    n = Krows.shape[2]
    if tuple(Vc.shape) != (B, Hkv, N, d) or tuple(Krows.shape) != (B, Hkv, n, d) or tuple(Vrows.shape) != (B, Hkv, n, d):
        raise ValueError("shapes must be Kc,Vc [B,Hkv,N,d] and Krows,Vrows [B,Hkv,n,d]")
    if positions.dtype != torch.int32 or positions.numel() != B * n:
        raise ValueError("positions must be int32 with B*n entries")
    qk = _dtype_tag(Kc, "Kc") if qk_dtype is None else qk_dtype
    vd = _dtype_tag(Vc, "Vc") if v_dtype is None else v_dtype
    rc = lib().dd_cache_insert_rows(_dev(Kc, "Kc"), _dev(Vc, "Vc"), _dev(Krows, "Krows"), _dev(Vrows, "Vrows"),
                                    _dev(positions, "positions"), n, B, Hkv, N, d, qk, vd, _stream())
    if rc != 0:
        raise DDError(rc, "dd_cache_insert_rows")


def dd_verify_remask_workspace_bytes(B, G, V, logit_dtype) -> int:
    return lib().dd_verify_remask_workspace_bytes(B, G, V, logit_dtype)


def dd_verify_remask(logits_d, logits_v, mask, mode: int, threshold: float, seed: int, B: int, G: int,
                     out_mask=None, out_tokens=None, out_scores=None, logit_dtype: Optional[int] = None):
    """Verification rule over the vocabulary.  logits [B*G, V]; mask [B*G] u8 (1 = still masked).
    Returns (out_mask u8, out_tokens i32, out_scores f32)."""
    torch = _torch()
    P, V = logits_v.shape
    if P != B * G:
        raise ValueError("logits_v must have B*G rows")
    if logits_d is not None and tuple(logits_d.shape) != (P, V):
        raise ValueError("logits_d shape must match logits_v")
    dt = _dtype_tag(logits_v, "logits_v") if logit_dtype is None else logit_dtype
    dev = logits_v.device
    _check_vec(mask, P, torch.uint8, "mask")
    _check_vec(out_mask, P, torch.uint8, "out_mask")
    _check_vec(out_tokens, P, torch.int32, "out_tokens")
    _check_vec(out_scores, P, torch.float32, "out_scores")
    if out_mask is None:
        out_mask = torch.empty(P, dtype=torch.uint8, device=dev)
    if out_tokens is None:
        out_tokens = torch.empty(P, dtype=torch.int32, device=dev)
    if out_scores is None:
        out_scores = torch.empty(P, dtype=torch.float32, device=dev)
    ws, wsn = _workspace(dd_verify_remask_workspace_bytes(B, G, V, dt), dev)
    rc = lib().dd_verify_remask(_dev(logits_d, "logits_d"), _dev(logits_v, "logits_v"), _dev(mask, "mask"),
                                int(mode), float(threshold), int(seed) & (2 ** 64 - 1),
                                _dev(out_mask, "out_mask"), _dev(out_tokens, "out_tokens"),
                                _dev(out_scores, "out_scores"), B, G, V, dt, _dev(ws, "workspace"), wsn, _stream())
    if rc != 0:
        raise DDError(rc, "dd_verify_remask")
    return out_mask, out_tokens, out_scores


def dd_verify_remask_static(logits_d, logits_v, mask, mode: int, threshold: float, seed: int, B: int, G: int,
                            out_mask, out_tokens, out_scores, logit_dtype: Optional[int] = None):
    """dd_verify_remask without a workspace: the library's static device array holds the partial states.  The
    three output tensors are the caller's (nothing is allocated here either).  Returns them."""
    torch = _torch()
    P, V = logits_v.shape
    if P != B * G:
        raise ValueError("logits_v must have B*G rows")
    if logits_d is not None and tuple(logits_d.shape) != (P, V):
        raise ValueError("logits_d shape must match logits_v")
    dt = _dtype_tag(logits_v, "logits_v") if logit_dtype is None else logit_dtype
    _check_vec(mask, P, torch.uint8, "mask")
    _check_vec(out_mask, P, torch.uint8, "out_mask")
    _check_vec(out_tokens, P, torch.int32, "out_tokens")
    _check_vec(out_scores, P, torch.float32, "out_scores")
    rc = lib().dd_verify_remask_static(_dev(logits_d, "logits_d"), _dev(logits_v, "logits_v"), _dev(mask, "mask"),
                                       int(mode), float(threshold), int(seed) & (2 ** 64 - 1),
                                       _dev(out_mask, "out_mask"), _dev(out_tokens, "out_tokens"),
                                       _dev(out_scores, "out_scores"), B, G, V, dt, _stream())
    if rc != 0:
        raise DDError(rc, "dd_verify_remask_static")
    return out_mask, out_tokens, out_scores


def dd_unmask_workspace_bytes(B, G, V, logit_dtype) -> int:
    return lib().dd_unmask_workspace_bytes(B, G, V, logit_dtype)


def dd_unmask(logits_d, mask, mode: int, threshold: float, B: int, G: int, x_tokens=None, out_mask=None,
              out_tokens=None, out_conf=None, logit_dtype: Optional[int] = None):
    """One drafter unmasking step.  logits_d [B*G, V]; mask [B*G] u8 (1 = still masked); x_tokens [B*G] i32
    (optional, updated in place where a position is revealed).  Returns (out_mask u8, out_tokens i32, out_conf f32)."""
    torch = _torch()
    P, V = logits_d.shape
    if P != B * G:
        raise ValueError("logits_d must have B*G rows")
    dt = _dtype_tag(logits_d, "logits_d") if logit_dtype is None else logit_dtype
    dev = logits_d.device
    _check_vec(mask, P, torch.uint8, "mask")
    _check_vec(x_tokens, P, torch.int32, "x_tokens")
    _check_vec(out_mask, P, torch.uint8, "out_mask")
    _check_vec(out_tokens, P, torch.int32, "out_tokens")
    _check_vec(out_conf, P, torch.float32, "out_conf")
    if out_mask is None:
        out_mask = torch.empty(P, dtype=torch.uint8, device=dev)
    if out_tokens is None:
        out_tokens = torch.empty(P, dtype=torch.int32, device=dev)
    if out_conf is None:
        out_conf = torch.empty(P, dtype=torch.float32, device=dev)
    ws, wsn = _workspace(dd_unmask_workspace_bytes(B, G, V, dt), dev)
    rc = lib().dd_unmask(_dev(logits_d, "logits_d"), _dev(mask, "mask"), int(mode), float(threshold),
                         _dev(x_tokens, "x_tokens"), _dev(out_mask, "out_mask"), _dev(out_tokens, "out_tokens"),
                         _dev(out_conf, "out_conf"), B, G, V, dt, _dev(ws, "workspace"), wsn, _stream())
    if rc != 0:
        raise DDError(rc, "dd_unmask")
    return out_mask, out_tokens, out_conf


def dd_verify_scores_workspace_bytes(P, V, logit_dtype) -> int:
    return lib().dd_verify_scores_workspace_bytes(P, V, logit_dtype)


def dd_verify_scores(logits_d, logits_v, drafter: bool = True, logit_dtype: Optional[int] = None):
    """Divergence, both confidences and both argmax tokens of every row in one pass.  logits_d, logits_v [P, V].
    Returns (kl f32, conf_v f32, tok_v i32, conf_d f32 | None, tok_d i32 | None)."""
    torch = _torch()
    P, V = logits_v.shape
    if tuple(logits_d.shape) != (P, V):
        raise ValueError("logits_d and logits_v must have the same shape")
    dt = _dtype_tag(logits_v, "logits_v") if logit_dtype is None else logit_dtype
    if logit_dtype is None and _dtype_tag(logits_d, "logits_d") != dt:
        raise ValueError("logits_d and logits_v must have the same dtype")
    dev = logits_v.device
    kl = torch.empty(P, dtype=torch.float32, device=dev)
    conf_v = torch.empty(P, dtype=torch.float32, device=dev)
    tok_v = torch.empty(P, dtype=torch.int32, device=dev)
    conf_d = torch.empty(P, dtype=torch.float32, device=dev) if drafter else None
    tok_d = torch.empty(P, dtype=torch.int32, device=dev) if drafter else None
    ws, wsn = _workspace(dd_verify_scores_workspace_bytes(P, V, dt), dev)
    rc = lib().dd_verify_scores(_dev(logits_d, "logits_d"), _dev(logits_v, "logits_v"), _dev(kl, "out_kl"),
                                _dev(conf_v, "out_conf_v"), _dev(tok_v, "out_tok_v"), _dev(conf_d, "out_conf_d"),
                                _dev(tok_d, "out_tok_d"), P, V, dt, _dev(ws, "workspace"), wsn, _stream())
    if rc != 0:
        raise DDError(rc, "dd_verify_scores")
    return kl, conf_v, tok_v, conf_d, tok_d
