"""TEST INFRASTRUCTURE: ctypes front end of the CPU oracle (oracle/dd_oracle.c).

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It marshals numpy arrays into the C functions and returns
fp64 results; all arithmetic lives in the C file.  It neither imports nor is imported
by the HIP library's package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dd_oracle.c")
_LIB = os.path.join(_HERE, "libdd_oracle.so")

F32, BF16, FP8_E4M3, F64 = 0, 1, 2, 3
MX_E4M3, MX_E2M1 = 0, 1      # element kinds of block-scaled tensors
TRUST, KL_THRESH, CONF_THRESH, KL_PROB, CONF_PROB, KL_TOPK, CONF_TOPK = 0, 1, 2, 3, 4, 5, 6
UNMASK_THRESH, UNMASK_TOPK = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over rows; no fast-math, no reassociation)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        vp, ip, dp, fp = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_float)
        _lib.ora_decode_e4m3.restype = C.c_double
        _lib.ora_decode_e4m3.argtypes = [C.c_uint8]
        _lib.ora_decode_bf16.restype = C.c_double
        _lib.ora_decode_bf16.argtypes = [C.c_uint16]
        _lib.ora_decode_e8m0.restype = C.c_double
        _lib.ora_decode_e8m0.argtypes = [C.c_uint8]
        _lib.ora_decode_e2m1.restype = C.c_double
        _lib.ora_decode_e2m1.argtypes = [C.c_uint8]
        _lib.ora_decode_mx.restype = C.c_int
        _lib.ora_decode_mx.argtypes = [vp, vp, dp, C.c_size_t, C.c_int, C.c_int]
        _lib.ora_bidir_attention.restype = C.c_int
        _lib.ora_bidir_attention.argtypes = [vp, vp, vp, dp] + [C.c_int] * 7 + [vp, vp, vp, C.c_int]
        _lib.ora_block_attention_cached.restype = C.c_int
        _lib.ora_block_attention_cached.argtypes = [vp, vp, vp, dp, C.c_int, C.c_int, vp, vp] + [C.c_int] * 7 + \
            [vp, vp, vp, C.c_int]
        _lib.ora_attention_vs.restype = C.c_int
        _lib.ora_attention_vs.argtypes = [vp, vp, vp, dp] + [C.c_int] * 8 + [vp, vp, vp, vp, vp, C.c_int, C.c_int, vp, C.c_int]
        _lib.ora_verify_scores.restype = C.c_int
        _lib.ora_verify_scores.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, vp, C.c_int, dp, dp, ip]
        _lib.ora_philox4x32_10.restype = None
        _lib.ora_philox4x32_10.argtypes = [C.POINTER(C.c_uint32)] * 3
        _lib.ora_row_uniform.restype = C.c_double
        _lib.ora_row_uniform.argtypes = [C.c_uint64, C.c_uint64]
        _lib.ora_remask_decide.restype = C.c_int
        _lib.ora_remask_decide.argtypes = [fp, C.POINTER(C.c_uint8), C.c_int, C.c_float, C.c_uint64,
                                           C.c_int, C.c_int, C.POINTER(C.c_uint8), dp]
        _lib.ora_unmask_decide.restype = C.c_int
        _lib.ora_unmask_decide.argtypes = [fp, C.POINTER(C.c_uint8), C.c_int, C.c_float, C.c_int, C.c_int,
                                           C.POINTER(C.c_uint8)]
    return _lib


def num_threads() -> int:
    """Threads the oracle's OpenMP loops use (OMP_NUM_THREADS or the visible cores)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return max(1, int(v.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


_NP_OF = {F32: np.float32, BF16: np.uint16, FP8_E4M3: np.uint8, F64: np.float64}


def _chk(a: np.ndarray, dtype: int, name: str) -> np.ndarray:
    if a.dtype != _NP_OF[dtype]:
        raise TypeError(f"{name}: expected {_NP_OF[dtype]} storage for dtype tag {dtype}, got {a.dtype}")
    return np.ascontiguousarray(a)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _rows3(rows) -> Optional[np.ndarray]:
    if rows is None:
        return None
    r = np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1, 3))
    return r


def decode_e4m3(code: int) -> float:
    return lib().ora_decode_e4m3(int(code))


def decode_bf16(bits: int) -> float:
    return lib().ora_decode_bf16(int(bits))


def decode_e8m0(code: int) -> float:
    return lib().ora_decode_e8m0(int(code))


def decode_e2m1(code: int) -> float:
    return lib().ora_decode_e2m1(int(code))


def decode_mx(elems: np.ndarray, scales: np.ndarray, kind: int) -> np.ndarray:
    """Block-scaled tensor [..., d] -> fp64.  elems: uint8 [..., d] (MX_E4M3) or [..., d/2] (MX_E2M1, two elements
    per byte, the even one in the low four bits); scales: uint8 [..., d/32] E8M0 codes, one per 32 elements."""
    elems = np.ascontiguousarray(elems, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    d = scales.shape[-1] * 32
    assert elems.shape[:-1] == scales.shape[:-1] and elems.shape[-1] == (d if kind == MX_E4M3 else d // 2)
    rows = int(np.prod(scales.shape[:-1], dtype=np.int64))
    out = np.empty(scales.shape[:-1] + (d,), dtype=np.float64)
    rc = lib().ora_decode_mx(_ptr(elems), _ptr(scales), out.ctypes.data_as(C.POINTER(C.c_double)), rows, d, kind)
    if rc != 0:
        raise ValueError("ora_decode_mx: bad argument")
    return out


def bidir_attention_mx(Q, Qs, K, Ks, V, Vs, rows=None) -> np.ndarray:
    """Full bidirectional attention on block-scaled inputs: Q, K with e4m3 elements, V with e2m1 elements, each with
    E8M0 scales per 32 elements of the head dimension: the tensors are decoded (decode_mx) and attended as fp64."""
    return bidir_attention(decode_mx(Q, Qs, MX_E4M3), decode_mx(K, Ks, MX_E4M3), decode_mx(V, Vs, MX_E2M1),
                           F64, F64, rows=rows)


def bidir_attention(Q, K, V, qk_dtype: int, v_dtype: int, q_scale=None, k_scale=None, rows=None, v_scale=None) -> np.ndarray:
    """Full bidirectional attention.  Q [B,H,N,d], K,V [B,Hkv,N,d] in storage form.
    rows=None -> O [B,H,N,d] fp64;  rows=[(b,h,i),...] -> O [len(rows), d].
    v_scale [B*Hkv] (optional): multiplier of the decoded values of V (fp8 V is stored like fp8 K)."""
    Q = _chk(Q, qk_dtype, "Q"); K = _chk(K, qk_dtype, "K"); V = _chk(V, v_dtype, "V")
    B, H, N, d = Q.shape
    Hkv = K.shape[1]
    assert K.shape == (B, Hkv, N, d) and V.shape == (B, Hkv, N, d)
    qs = None if q_scale is None else np.ascontiguousarray(q_scale, dtype=np.float32).reshape(B * H)
    ks = None if k_scale is None else np.ascontiguousarray(k_scale, dtype=np.float32).reshape(B * Hkv)
    r = _rows3(rows)
    O = np.empty((B, H, N, d) if r is None else (len(r), d), dtype=np.float64)
    if v_scale is not None:
        vs = np.ascontiguousarray(v_scale, dtype=np.float32).reshape(B * Hkv)
        rc = lib().ora_attention_vs(_ptr(Q), _ptr(K), _ptr(V), O.ctypes.data_as(C.POINTER(C.c_double)),
                                    B, H, Hkv, N, N, d, qk_dtype, v_dtype, _ptr(qs), _ptr(ks), _ptr(vs),
                                    None, None, 0, 0, _ptr(r), 0 if r is None else len(r))
        if rc != 0:
            raise ValueError("oracle bidir_attention: bad argument")
        return O
    rc = lib().ora_bidir_attention(_ptr(Q), _ptr(K), _ptr(V), O.ctypes.data_as(C.POINTER(C.c_double)),
                                   B, H, Hkv, N, d, qk_dtype, v_dtype, _ptr(qs), _ptr(ks),
                                   _ptr(r), 0 if r is None else len(r))
    if rc != 0:
        raise ValueError("oracle bidir_attention: bad argument")
    return O


def block_attention_cached(Qblk, Kc, Vc, block_start: int, qk_dtype: int, v_dtype: int, Kblk=None, Vblk=None,
                           q_scale=None, k_scale=None, rows=None, v_scale=None) -> np.ndarray:
    """Active-block queries over cached K/V.  Qblk [B,H,bl,d]; Kc,Vc [B,Hkv,N,d];
    optional Kblk,Vblk [B,Hkv,bl,d] replace cache rows [block_start, block_start+bl)."""
    Qblk = _chk(Qblk, qk_dtype, "Qblk"); Kc = _chk(Kc, qk_dtype, "Kc"); Vc = _chk(Vc, v_dtype, "Vc")
    B, H, bl, d = Qblk.shape
    _, Hkv, N, _ = Kc.shape
    assert Kc.shape == (B, Hkv, N, d) and Vc.shape == (B, Hkv, N, d)
    if Kblk is not None:
        Kblk = _chk(Kblk, qk_dtype, "Kblk"); Vblk = _chk(Vblk, v_dtype, "Vblk")
        assert Kblk.shape == (B, Hkv, bl, d) and Vblk.shape == (B, Hkv, bl, d)
    qs = None if q_scale is None else np.ascontiguousarray(q_scale, dtype=np.float32).reshape(B * H)
    ks = None if k_scale is None else np.ascontiguousarray(k_scale, dtype=np.float32).reshape(B * Hkv)
    r = _rows3(rows)
    O = np.empty((B, H, bl, d) if r is None else (len(r), d), dtype=np.float64)
    if v_scale is not None:
        if not (0 <= block_start and block_start + bl <= N):
            raise ValueError("oracle block_attention_cached: bad argument")
        vs = np.ascontiguousarray(v_scale, dtype=np.float32).reshape(B * Hkv)
        rc = lib().ora_attention_vs(_ptr(Qblk), _ptr(Kc), _ptr(Vc), O.ctypes.data_as(C.POINTER(C.c_double)),
                                    B, H, Hkv, bl, N, d, qk_dtype, v_dtype, _ptr(qs), _ptr(ks), _ptr(vs),
                                    _ptr(Kblk), _ptr(Vblk), block_start, bl, _ptr(r), 0 if r is None else len(r))
        if rc != 0:
            raise ValueError("oracle block_attention_cached: bad argument")
        return O
    rc = lib().ora_block_attention_cached(_ptr(Qblk), _ptr(Kc), _ptr(Vc), O.ctypes.data_as(C.POINTER(C.c_double)),
                                          block_start, bl, _ptr(Kblk), _ptr(Vblk), B, H, Hkv, N, d,
                                          qk_dtype, v_dtype, _ptr(qs), _ptr(ks), _ptr(r), 0 if r is None else len(r))
    if rc != 0:
        raise ValueError("oracle block_attention_cached: bad argument")
    return O


def block_attention_refresh(Qblk, Kc, Vc, block_start: int, qk_dtype: int, v_dtype: int, Kblk, Vblk,
                            q_scale=None, k_scale=None, rows=None):
    """Block completion (Sec. 2.3): the block's rows replace rows [block_start, block_start+bl) of the cache, and the
    block's queries attend over the refreshed cache.  Written as that definition: new cache arrays first, then the
    plain cached call on them.  Returns (O, Kc_new, Vc_new); the inputs are not modified."""
    Kc = _chk(Kc, qk_dtype, "Kc"); Vc = _chk(Vc, v_dtype, "Vc")
    Kblk = _chk(Kblk, qk_dtype, "Kblk"); Vblk = _chk(Vblk, v_dtype, "Vblk")
    bl = Kblk.shape[2]
    Kn, Vn = Kc.copy(), Vc.copy()
    Kn[:, :, block_start:block_start + bl, :] = Kblk
    Vn[:, :, block_start:block_start + bl, :] = Vblk
    O = block_attention_cached(Qblk, Kn, Vn, block_start, qk_dtype, v_dtype, None, None, q_scale, k_scale, rows)
    return O, Kn, Vn


def block_attention_window(Qblk, Kc, Vc, block_start: int, win_start: int, win_len: int, qk_dtype: int, v_dtype: int,
                           Kblk=None, Vblk=None, q_scale=None, k_scale=None, rows=None) -> np.ndarray:
    """Drafter attention restricted to key rows [win_start, win_start + win_len) (local-window drafters, Sec. 2.3):
    by definition the cached call on the sequence that consists of those rows only."""
    Kc = _chk(Kc, qk_dtype, "Kc"); Vc = _chk(Vc, v_dtype, "Vc")
    N = Kc.shape[2]
    bl = Qblk.shape[2]
    if not (0 <= win_start <= block_start and block_start + bl <= win_start + win_len <= N):
        raise ValueError("oracle block_attention_window: the window must lie in the cache and contain the block")
    Kw = np.ascontiguousarray(Kc[:, :, win_start:win_start + win_len, :])
    Vw = np.ascontiguousarray(Vc[:, :, win_start:win_start + win_len, :])
    return block_attention_cached(Qblk, Kw, Vw, block_start - win_start, qk_dtype, v_dtype, Kblk, Vblk, q_scale, k_scale, rows)


def block_attention_batched(Qblk, Kc, Vc, block_starts, qk_dtype: int, v_dtype: int, Kblk, Vblk,
                            q_scale=None, k_scale=None) -> np.ndarray:
    """Drafter attention with one block position per batch entry: by definition the cached call on each batch
    entry alone, at its own position.  Rows of a block that fall outside [0, N) replace nothing."""
    B, H, bl, d = Qblk.shape
    N = Kc.shape[2]
    Hkv = Kc.shape[1]
    out = np.empty((B, H, bl, d), dtype=np.float64)
    qs = None if q_scale is None else np.asarray(q_scale, dtype=np.float32).reshape(B, H)
    ks = None if k_scale is None else np.asarray(k_scale, dtype=np.float32).reshape(B, Hkv)
    for b in range(B):
        s0 = int(block_starts[b])
        Kn, Vn = np.array(Kc[b:b + 1], copy=True), np.array(Vc[b:b + 1], copy=True)
        for r in range(bl):                                   # splice the block's rows that lie inside the sequence
            if 0 <= s0 + r < N:
                Kn[0, :, s0 + r, :] = Kblk[b, :, r, :]
                Vn[0, :, s0 + r, :] = Vblk[b, :, r, :]
        out[b] = block_attention_cached(Qblk[b:b + 1], Kn, Vn, 0, qk_dtype, v_dtype, None, None,
                                        None if qs is None else qs[b:b + 1], None if ks is None else ks[b:b + 1])[0]
    return out


def cache_insert_rows(Kc, Vc, Krows, Vrows, positions):
    """Token-granular cache update (Sec. 2.3, delayed insertion): row r of Krows/Vrows [B,Hkv,n,d] replaces cache
    row positions[b][r] of every kv head of batch b; entries outside [0, N) are skipped.  Plain loops; returns new
    arrays."""
    Kn, Vn = np.array(Kc, copy=True), np.array(Vc, copy=True)
    B, Hkv, N, _ = Kn.shape
    pos = np.asarray(positions).reshape(B, -1)
    for b in range(B):
        for r in range(pos.shape[1]):
            p = int(pos[b, r])
            if 0 <= p < N:
                for g in range(Hkv):
                    Kn[b, g, p, :] = Krows[b, g, r, :]
                    Vn[b, g, p, :] = Vrows[b, g, r, :]
    return Kn, Vn


def verify_scores(logits_d, logits_v, dtype: int, rows: Optional[Sequence[int]] = None):
    """(kl, conf, token) per row; logits [P,V] in storage form; logits_d may be None (kl = NaN)."""
    lv = _chk(logits_v, dtype, "logits_v")
    ld = None if logits_d is None else _chk(logits_d, dtype, "logits_d")
    P, V = lv.shape
    r = None if rows is None else np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1))
    n = P if r is None else len(r)
    kl = np.empty(n, dtype=np.float64); conf = np.empty(n, dtype=np.float64); tok = np.empty(n, dtype=np.int32)
    rc = lib().ora_verify_scores(_ptr(ld), _ptr(lv), P, V, dtype, _ptr(r), n,
                                 kl.ctypes.data_as(C.POINTER(C.c_double)), conf.ctypes.data_as(C.POINTER(C.c_double)),
                                 tok.ctypes.data_as(C.POINTER(C.c_int32)))
    if rc != 0:
        raise ValueError("oracle verify_scores: bad argument")
    return kl, conf, tok


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (C.c_uint32 * 4)()
    lib().ora_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def row_uniform(seed: int, row: int) -> float:
    return lib().ora_row_uniform(int(seed) & (2**64 - 1), int(row))


def remask_decide(score32, mask, mode: int, threshold: float, seed: int, B: int, G: int):
    """(out_mask, prob) from fp32 per-row scores; see ora_remask_decide in the C file."""
    s = np.ascontiguousarray(score32, dtype=np.float32).reshape(B * G)
    m = np.ascontiguousarray(mask, dtype=np.uint8).reshape(B * G)
    out = np.empty(B * G, dtype=np.uint8)
    prob = np.empty(B * G, dtype=np.float64)
    rc = lib().ora_remask_decide(s.ctypes.data_as(C.POINTER(C.c_float)), m.ctypes.data_as(C.POINTER(C.c_uint8)),
                                 mode, float(np.float32(threshold)), int(seed) & (2**64 - 1), B, G,
                                 out.ctypes.data_as(C.POINTER(C.c_uint8)), prob.ctypes.data_as(C.POINTER(C.c_double)))
    if rc != 0:
        raise ValueError("oracle remask_decide: bad argument")
    return out, prob


def verify_remask(logits_d, logits_v, mask, mode: int, threshold: float, seed: int, B: int, G: int, dtype: int):
    """Whole verification pass: scores for every row, then the remask rule.
    Returns dict(out_mask, out_tokens, out_scores (fp32-rounded), kl, conf, prob)."""
    need_d = mode in (KL_THRESH, KL_PROB, KL_TOPK)
    if need_d and logits_d is None:
        raise ValueError("KL modes need drafter logits")
    kl, conf, tok = verify_scores(logits_d if need_d else None, logits_v, dtype)
    score = kl if need_d else conf
    score32 = score.astype(np.float32)
    out_mask, prob = remask_decide(score32, mask, mode, threshold, seed, B, G)
    return {"out_mask": out_mask, "out_tokens": tok, "out_scores": score32, "kl": kl, "conf": conf,
            "prob": prob, "score64": score}


def unmask_decide(conf32, mask, mode: int, threshold: float, B: int, G: int) -> np.ndarray:
    """out_mask of one drafter unmasking step from fp32 confidences; see ora_unmask_decide in the C file."""
    c = np.ascontiguousarray(conf32, dtype=np.float32).reshape(B * G)
    m = np.ascontiguousarray(mask, dtype=np.uint8).reshape(B * G)
    out = np.empty(B * G, dtype=np.uint8)
    rc = lib().ora_unmask_decide(c.ctypes.data_as(C.POINTER(C.c_float)), m.ctypes.data_as(C.POINTER(C.c_uint8)),
                                 mode, float(np.float32(threshold)), B, G, out.ctypes.data_as(C.POINTER(C.c_uint8)))
    if rc != 0:
        raise ValueError("oracle unmask_decide: bad argument")
    return out


def unmask(logits_d, mask, mode: int, threshold: float, B: int, G: int, dtype: int, x_tokens=None):
    """Whole drafter unmasking step: confidence and most likely token of every row, then the selection.
    Returns dict(out_mask, out_tokens, out_conf (fp32-rounded), conf64, x_tokens (updated copy or None))."""
    _, conf, tok = verify_scores(None, logits_d, dtype)
    conf32 = conf.astype(np.float32)
    out_mask = unmask_decide(conf32, mask, mode, threshold, B, G)
    m = np.asarray(mask).reshape(-1)
    x = None
    if x_tokens is not None:
        x = np.array(x_tokens, dtype=np.int32).reshape(-1)
        sel = (m != 0) & (out_mask == 0)
        x[sel] = tok[sel]
    return {"out_mask": out_mask, "out_tokens": tok, "out_conf": conf32, "conf64": conf, "x_tokens": x}
