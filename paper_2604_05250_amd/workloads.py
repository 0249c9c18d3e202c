"""Seeded synthetic inputs for one DualDiffusion draft-then-verify step.

This module only *draws and stores* tensors: normal variates from numpy's
Philox bit generator, rounded to the storage type (fp32, bf16 or OCP fp8
e4m3).  It holds none of the method's arithmetic (no softmax, no attention,
no KL, no remask rule), so that the HIP library and the CPU oracle can both be
fed from it without sharing any of the computation under test.

Shapes follow the five benchmark configurations (LLaDA-8B-like head geometry
and vocabulary); the paper's own workloads (Section 4.1: benchmark prompts run
through trained drafter / verifier weights) are not available, so seeded
Gaussian tensors of the same shape stand in for them.

Storage conventions (all arrays are C-contiguous numpy arrays on the host):
  fp32  -> np.float32
  bf16  -> np.uint16  holding the upper 16 bits of the fp32 pattern (RNE)
  fp8   -> np.uint8   holding OCP e4m3 codes (RNE, saturating at +-448),
           real value = per-(batch, head) fp32 scale * decoded code
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

# dtype tags: numerically equal to dd_dtype in include/dd.h
F32, BF16, FP8_E4M3 = 0, 1, 2
# remask modes: numerically equal to dd_mode in include/dd.h
TRUST, KL_THRESH, CONF_THRESH, KL_PROB, CONF_PROB, KL_TOPK, CONF_TOPK = 0, 1, 2, 3, 4, 5, 6
UNMASK_THRESH, UNMASK_TOPK = 0, 1
MODE_NAMES = {TRUST: "trust", KL_THRESH: "kl_thresh", CONF_THRESH: "conf_thresh",
              KL_PROB: "kl_prob", CONF_PROB: "conf_prob", KL_TOPK: "kl_topk", CONF_TOPK: "conf_topk"}

_ELEM_BYTES = {F32: 4, BF16: 2, FP8_E4M3: 1}


def elem_bytes(dtype: int) -> int:
    return _ELEM_BYTES[dtype]


# --------------------------------------------------------------------------
# storage-type rounding (encoding only; no method arithmetic)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to OCP fp8 e4m3 (bias 7, no infinities, max finite 448),
    nearest-even, saturating; returns the 8-bit codes.  Input must be finite."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    sign = (x.view(np.uint32) >> np.uint32(24)).astype(np.uint8) & np.uint8(0x80)
    a = np.minimum(np.abs(x), np.float32(448.0))
    # subnormal range: multiples of 2^-9 below 2^-6
    sub = a < np.float32(2.0 ** -6)
    q_sub = np.rint(a * np.float32(512.0)).astype(np.int32)          # 0..8 (8 = first normal)
    _, e1 = np.frexp(a)                                              # a = m * 2^e1, m in [0.5, 1)
    e = e1.astype(np.int32) - 1
    e = np.where(sub, -6, e)
    q = np.rint(np.ldexp(a, 3 - e)).astype(np.int32)                 # 8..16
    carry = q == 16
    e = np.where(carry, e + 1, e)
    q = np.where(carry, 8, q)
    code_norm = ((e + 7) << 3) | (q - 8)
    code = np.where(sub, q_sub, code_norm).astype(np.uint8)
    return code | sign


def f32_to_e2m1_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to the 4-bit float e2m1 (values +-{0, 0.5, 1, 1.5, 2, 3, 4, 6}), nearest with ties to the even
    code, saturating at +-6; returns the 4-bit codes (sign in bit 3), one per byte.  Input must be finite."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    sign = ((x.view(np.uint32) >> np.uint32(28)) & np.uint32(8)).astype(np.uint8)
    a = np.minimum(np.abs(x), np.float32(6.0))
    grid = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float32)
    hi = np.clip(np.searchsorted(grid, a, side="left"), 1, 7)          # grid[hi-1] <= a <= grid[hi] (or a == 0)
    lo = hi - 1
    dl, dh = a - grid[lo], grid[hi] - a
    code = np.where(dl < dh, lo, np.where(dh < dl, hi, np.where(lo % 2 == 0, lo, hi)))
    return code.astype(np.uint8) | sign


def mx_quantize(x: np.ndarray, kind: str):
    """Block-scaled (OCP Microscaling v1.0) storage of a tensor [..., d], d % 32 == 0: every 32 consecutive elements
    share a power-of-two scale 2^(floor(log2(amax)) - emax) with emax = 8 (e4m3 elements) or 2 (e2m1), stored as the
    E8M0 code exponent + 127 (clamped to 0..254; an all-zero block takes 127); elements = value / scale rounded to
    the element type, saturating.  Returns (elements, scales): elements uint8 [..., d] for "e4m3", [..., d/2] for
    "e2m1" (two per byte, the even element in the low four bits); scales uint8 [..., d/32]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    d = x.shape[-1]
    assert d % 32 == 0 and kind in ("e4m3", "e2m1")
    xb = x.reshape(x.shape[:-1] + (d // 32, 32))
    amax = np.max(np.abs(xb), axis=-1)
    _, e1 = np.frexp(amax)                                            # amax = m * 2^e1, m in [0.5, 1)
    shared = np.where(amax > 0, e1.astype(np.int32) - 1 - (8 if kind == "e4m3" else 2), 0)
    shared = np.clip(shared, -127, 127)
    scaled = np.ldexp(xb, -shared[..., None]).astype(np.float32)      # exact: a power of two
    if kind == "e4m3":
        elems = f32_to_e4m3_bits(scaled).reshape(x.shape)
    else:
        c = f32_to_e2m1_bits(scaled).reshape(x.shape[:-1] + (d // 2, 2))
        elems = (c[..., 0] | (c[..., 1] << np.uint8(4))).astype(np.uint8)
    return elems, (shared + 127).astype(np.uint8)


# --------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class StepConfig:
    name: str
    B: int            # batch (sequences)
    H: int            # query heads
    Hkv: int          # key/value heads
    N: int            # sequence length (prompt + gen)
    prompt: int       # prompt positions
    G: int            # gen positions per sequence (verified rows per sequence)
    d: int            # head dim
    qk_dtype: int
    v_dtype: int
    bl: int           # drafter block length
    K: int            # drafter steps per cycle
    V: int            # vocabulary
    logit_dtype: int
    sigma_d: float    # std of drafter logits
    sigma_n: float    # std of the verifier-minus-drafter perturbation
    spike: float      # added to one uniformly chosen token per drafter row (0 = none)
    decoded_frac: Optional[float]   # None: every gen position decoded (mask all 0)
    modes: Tuple[Tuple[int, float], ...]   # (mode, threshold) pairs run in this config
    qk_prescale: float = 1.0        # multiplier on Q, K, V draws

    @property
    def P(self) -> int:
        return self.B * self.G


CONFIGS: Dict[int, StepConfig] = {
    1: StepConfig("cfg1_tiny_fp32", 1, 4, 4, 128, 64, 64, 64, F32, F32, 16, 4, 1024, F32,
                  2.0, 0.5, 0.0, None, ((TRUST, 0.0), (KL_THRESH, 0.5), (CONF_THRESH, 0.9))),
    2: StepConfig("cfg2_llada_n512", 1, 32, 32, 512, 256, 256, 128, BF16, BF16, 32, 8, 126464, BF16,
                  3.0, 1.0, 0.0, None, ((KL_THRESH, 0.3),)),
    3: StepConfig("cfg3_batched_n1024", 8, 32, 32, 1024, 512, 512, 128, BF16, BF16, 64, 8, 126464, BF16,
                  3.0, 1.0, 0.0, 0.3, ((TRUST, 0.0), (CONF_THRESH, 0.9))),
    4: StepConfig("cfg4_long_n4096", 1, 32, 32, 4096, 3584, 512, 128, BF16, BF16, 64, 8, 126464, BF16,
                  3.0, 1.0, 0.0, None, ((KL_THRESH, 0.3),)),
    5: StepConfig("cfg5_gqa_fp8_n2048", 16, 32, 8, 2048, 1536, 512, 128, FP8_E4M3, BF16, 64, 8, 152064, BF16,
                  2.0, 1.0, 8.0, None, ((CONF_THRESH, 0.9),)),
}

# tensor stream ids (second Philox key word = id << 32 | chunk)
_T_Q, _T_K, _T_V, _T_KC, _T_VC, _T_QBLK, _T_KBLK, _T_VBLK, _T_LD, _T_NOISE, _T_MASK, _T_SPIKE = range(1, 13)


def _gen(seed: int, tensor_id: int, chunk: int = 0) -> np.random.Generator:
    key = np.array([np.uint64(seed), np.uint64((tensor_id << 32) | chunk)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def _threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _store(x32: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == F32:
        return x32
    if dtype == BF16:
        return f32_to_bf16_bits(x32)
    raise ValueError("fp8 tensors are stored with a per-head scale; use _head_tensor")


def _head_tensor(seed: int, tensor_id: int, B: int, Hn: int, rows: int, d: int, dtype: int,
                 prescale: float, salt: int = 0):
    """[B, Hn, rows, d] tensor of N(0, prescale^2) draws, one Philox stream per (b, head).
    fp8: per-(b, head) scale = amax / 448, codes = e4m3(x / scale).  Returns (array, scales|None)."""
    np_dt = {F32: np.float32, BF16: np.uint16, FP8_E4M3: np.uint8}[dtype]
    out = np.empty((B, Hn, rows, d), dtype=np_dt)
    scales = np.empty((B, Hn), dtype=np.float32) if dtype == FP8_E4M3 else None

    def work(idx):
        b, h = divmod(idx, Hn)
        g = _gen(seed, tensor_id, (salt << 20) | idx)
        x = g.standard_normal((rows, d), dtype=np.float32)
        if prescale != 1.0:
            x *= np.float32(prescale)
        if dtype == FP8_E4M3:
            amax = np.float32(np.max(np.abs(x)))
            s = np.float32(amax / np.float32(448.0)) if amax > 0 else np.float32(1.0)
            scales[b, h] = s
            out[b, h] = f32_to_e4m3_bits(x / s)
        else:
            out[b, h] = _store(x, dtype)

    with ThreadPoolExecutor(_threads()) as ex:
        list(ex.map(work, range(B * Hn)))
    return out, scales


def attention_inputs(cfg: StepConfig, seed: int = 0) -> dict:
    """Q [B,H,N,d], K,V [B,Hkv,N,d] for the verifier's full attention."""
    Q, qs = _head_tensor(seed, _T_Q, cfg.B, cfg.H, cfg.N, cfg.d, cfg.qk_dtype, cfg.qk_prescale)
    K, ks = _head_tensor(seed, _T_K, cfg.B, cfg.Hkv, cfg.N, cfg.d, cfg.qk_dtype, cfg.qk_prescale)
    V, vs = _head_tensor(seed, _T_V, cfg.B, cfg.Hkv, cfg.N, cfg.d, cfg.v_dtype, cfg.qk_prescale)
    return {"Q": Q, "K": K, "V": V, "q_scale": qs, "k_scale": ks, "v_scale": vs}


def mx_attention_inputs(cfg: StepConfig, seed: int = 0) -> dict:
    """The verifier's attention inputs of `cfg` in block-scaled storage (the same fp32 draws as attention_inputs
    would make): Q [B,H,N,d] and K [B,Hkv,N,d] with e4m3 elements, V [B,Hkv,N,d/2] with e2m1 elements, each with
    E8M0 scales [..., d/32]."""
    out = {}
    for name, tid, Hn, kind in (("Q", _T_Q, cfg.H, "e4m3"), ("K", _T_K, cfg.Hkv, "e4m3"), ("V", _T_V, cfg.Hkv, "e2m1")):
        x, _ = _head_tensor(seed, tid, cfg.B, Hn, cfg.N, cfg.d, F32, cfg.qk_prescale)
        x = x.reshape(cfg.B * Hn, cfg.N, cfg.d)
        with ThreadPoolExecutor(_threads()) as ex:
            parts = list(ex.map(lambda i: mx_quantize(x[i], kind), range(cfg.B * Hn)))
        out[name] = np.stack([p[0] for p in parts]).reshape(cfg.B, Hn, cfg.N, -1)
        out[name + "s"] = np.stack([p[1] for p in parts]).reshape(cfg.B, Hn, cfg.N, cfg.d // 32)
    return out


def cache_inputs(cfg: StepConfig, seed: int = 0) -> dict:
    """Stale drafter cache Kc, Vc [B,Hkv,N,d] (independent of the current K, V)."""
    Kc, ks = _head_tensor(seed, _T_KC, cfg.B, cfg.Hkv, cfg.N, cfg.d, cfg.qk_dtype, cfg.qk_prescale)
    Vc, vs = _head_tensor(seed, _T_VC, cfg.B, cfg.Hkv, cfg.N, cfg.d, cfg.v_dtype, cfg.qk_prescale)
    return {"Kc": Kc, "Vc": Vc, "k_scale": ks, "v_scale": vs}


def block_start(cfg: StepConfig, step: int) -> int:
    """Draft step k works on gen block k (first block right after the prompt)."""
    return cfg.prompt + (step % (cfg.G // cfg.bl)) * cfg.bl


def block_inputs(cfg: StepConfig, seed: int = 0, step: int = 0, k_scale: Optional[np.ndarray] = None,
                 v_scale: Optional[np.ndarray] = None) -> dict:
    """Fresh active-block tensors for draft step `step`: Qblk [B,H,bl,d], Kblk,Vblk [B,Hkv,bl,d].
    With fp8 K (V) the block rows are quantised with the *cache's* per-head scale (`k_scale`, `v_scale`),
    since one scale per (b, kv head) covers cached and fresh rows alike."""
    Qb, qs = _head_tensor(seed, _T_QBLK, cfg.B, cfg.H, cfg.bl, cfg.d, cfg.qk_dtype, cfg.qk_prescale, salt=step + 1)
    if cfg.qk_dtype == FP8_E4M3:
        if k_scale is None:
            raise ValueError("fp8 block K needs the cache's k_scale")
        Kf, _ = _head_tensor(seed, _T_KBLK, cfg.B, cfg.Hkv, cfg.bl, cfg.d, F32, cfg.qk_prescale, salt=step + 1)
        Kb = f32_to_e4m3_bits(Kf / k_scale[:, :, None, None].astype(np.float32))
    else:
        Kb, _ = _head_tensor(seed, _T_KBLK, cfg.B, cfg.Hkv, cfg.bl, cfg.d, cfg.qk_dtype, cfg.qk_prescale, salt=step + 1)
    if cfg.v_dtype == FP8_E4M3:
        if v_scale is None:
            raise ValueError("fp8 block V needs the cache's v_scale")
        Vf, _ = _head_tensor(seed, _T_VBLK, cfg.B, cfg.Hkv, cfg.bl, cfg.d, F32, cfg.qk_prescale, salt=step + 1)
        Vb = f32_to_e4m3_bits(Vf / v_scale[:, :, None, None].astype(np.float32))
    else:
        Vb, _ = _head_tensor(seed, _T_VBLK, cfg.B, cfg.Hkv, cfg.bl, cfg.d, cfg.v_dtype, cfg.qk_prescale, salt=step + 1)
    return {"Qblk": Qb, "Kblk": Kb, "Vblk": Vb, "q_scale": qs, "block_start": block_start(cfg, step)}


_ROWS_PER_CHUNK = 32


def verify_inputs(cfg: StepConfig, seed: int = 0, rows: Optional[int] = None) -> dict:
    """logits_d, logits_v [P, V] and mask [P] (1 = still [MASK], 0 = decoded => eligible).

    drafter row  = sigma_d * z1 (+ spike on one uniformly chosen token)
    verifier row = drafter row (before storage rounding) + sigma_n * z2
    both rounded to the logit storage type.  `rows` limits generation to the first rows
    (rows are generated in independent chunks, so a prefix equals the full tensor's prefix)."""
    P = cfg.P if rows is None else min(rows, cfg.P)
    V = cfg.V
    np_dt = np.float32 if cfg.logit_dtype == F32 else np.uint16
    ld = np.empty((P, V), dtype=np_dt)
    lv = np.empty((P, V), dtype=np_dt)
    nchunks = (P + _ROWS_PER_CHUNK - 1) // _ROWS_PER_CHUNK

    def work(c):
        r0 = c * _ROWS_PER_CHUNK
        r1 = min(P, r0 + _ROWS_PER_CHUNK)
        n = r1 - r0
        x = _gen(seed, _T_LD, c).standard_normal((n, V), dtype=np.float32)
        x *= np.float32(cfg.sigma_d)
        if cfg.spike != 0.0:
            col = _gen(seed, _T_SPIKE, c).integers(0, V, size=n)
            x[np.arange(n), col] += np.float32(cfg.spike)
        ld[r0:r1] = _store(x, cfg.logit_dtype)
        z = _gen(seed, _T_NOISE, c).standard_normal((n, V), dtype=np.float32)
        z *= np.float32(cfg.sigma_n)
        z += x
        lv[r0:r1] = _store(z, cfg.logit_dtype)

    with ThreadPoolExecutor(_threads()) as ex:
        list(ex.map(work, range(nchunks)))

    if cfg.decoded_frac is None:
        mask = np.zeros(P, dtype=np.uint8)
    else:
        u = _gen(seed, _T_MASK).random(cfg.P)
        mask = (u >= cfg.decoded_frac).astype(np.uint8)[:P]
    return {"logits_d": ld, "logits_v": lv, "mask": mask}


def custom_config(**kw) -> StepConfig:
    """A StepConfig for parity / edge-case tests (ragged sizes, odd head counts ...)."""
    base = dict(name="custom", B=1, H=2, Hkv=2, N=96, prompt=32, G=64, d=64, qk_dtype=BF16, v_dtype=BF16,
                bl=16, K=2, V=1000, logit_dtype=BF16, sigma_d=2.0, sigma_n=0.5, spike=0.0,
                decoded_frac=None, modes=((KL_THRESH, 0.3),))
    base.update(kw)
    return StepConfig(**base)
