"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, and rejects bad arguments on the host before any GPU call (no compute here)."""
import ctypes as C
import os
import re

import pytest

import paper_2604_05250_amd as dd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "dd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dd_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert set(names) == set(dd.EXPORTS)
    L = dd.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert L.dd_version() >= 100
    assert L.dd_strerror(0) == b"ok"
    for code in range(-7, 0):
        assert L.dd_strerror(code) not in (b"ok", b"unknown status")
    assert L.dd_strerror(-99) == b"unknown status"


FAKE = 0x1000   # a non-NULL, 16-byte aligned address that is never dereferenced: every call below fails validation first


def test_attention_argument_validation():
    L = dd.lib()
    ok_args = dict(B=1, H=4, Hkv=2, N=64, d=128, qk=dd.BF16, v=dd.BF16)

    def call(Q=FAKE, K=FAKE, V=FAKE, O=FAKE, qs=None, ks=None, **kw):
        a = dict(ok_args); a.update(kw)
        return L.dd_bidir_attention(Q, K, V, O, a["B"], a["H"], a["Hkv"], a["N"], a["d"], a["qk"], a["v"], qs, ks,
                                    None, 0, None)
    assert call(Q=None) == -1 and call(O=None) == -1
    assert call(B=0) == -2 and call(N=0) == -2 and call(H=3) == -2 and call(d=96) == -2
    assert call(qk=dd.BF16, v=dd.F32) == -3 and call(qk=dd.FP8_E4M3, v=dd.FP8_E4M3) == -3 and call(qk=7) == -3
    assert call(qk=dd.FP8_E4M3, v=dd.BF16) == -1          # fp8 needs both scales
    assert call(Q=FAKE + 4) == -6

    def blk(bs=0, bl=16, Kblk=None, Vblk=None, ws=None, wsn=0, **kw):
        a = dict(ok_args); a.update(kw)
        return L.dd_block_attention_cached(FAKE, FAKE, FAKE, FAKE, bs, bl, Kblk, Vblk, a["B"], a["H"], a["Hkv"],
                                           a["N"], a["d"], a["qk"], a["v"], None, None, ws, wsn, None)
    assert blk(bs=-1) == -2 and blk(bs=60, bl=16) == -2 and blk(bl=0) == -2
    assert blk(Kblk=FAKE) == -1                            # Kblk and Vblk come together
    # workspace: needed once the key range is split
    need = L.dd_block_attention_cached_workspace_bytes(64, 1, 32, 32, 4096, 128, dd.BF16, dd.BF16)
    assert need > 0
    big = dict(B=1, H=32, Hkv=32, N=4096)
    assert blk(bs=0, bl=64, **big) == -5
    assert blk(bs=0, bl=64, ws=FAKE, wsn=need - 1, **big) == -5
    assert blk(bs=0, bl=64, ws=FAKE + 16, wsn=need, **big) == -5      # 256-byte alignment

    def refresh(Kblk=FAKE, Vblk=FAKE, bs=0, bl=16, **kw):
        a = dict(ok_args); a.update(kw)
        return L.dd_block_attention_refresh(FAKE, FAKE, FAKE, FAKE, bs, bl, Kblk, Vblk, a["B"], a["H"], a["Hkv"],
                                            a["N"], a["d"], a["qk"], a["v"], None, None, None, 0, None)
    assert refresh(Kblk=None, Vblk=None) == -1             # a refresh needs the block's rows
    assert refresh(Vblk=None) == -1 and refresh(bs=60) == -2 and refresh(Kblk=FAKE + 8) == -6
    assert refresh(bs=0, bl=64, **big) == -5               # same workspace rule as the plain call
    assert L.dd_block_attention_refresh_workspace_bytes(64, 1, 32, 32, 4096, 128, dd.BF16, dd.BF16) == need

    def batched(starts=FAKE, Kblk=FAKE, Vblk=FAKE, bl=16, **kw):
        a = dict(ok_args); a.update(kw)
        return L.dd_block_attention_batched(FAKE, FAKE, FAKE, FAKE, starts, bl, Kblk, Vblk, a["B"], a["H"], a["Hkv"],
                                            a["N"], a["d"], a["qk"], a["v"], None, None, None, 0, None)
    assert batched(starts=None) == -1 and batched(Kblk=None, Vblk=None) == -1 and batched(starts=FAKE + 2) == -6
    assert batched(bl=0) == -2 and batched(bl=65) == -2
    assert batched(bl=64, **big) == -5
    assert L.dd_block_attention_batched_workspace_bytes(64, 1, 32, 32, 4096, 128, dd.BF16, dd.BF16) == need

    def window(bs=16, bl=16, w0=0, wl=64, **kw):
        a = dict(ok_args); a.update(kw)
        return L.dd_block_attention_window(FAKE, FAKE, FAKE, FAKE, bs, bl, w0, wl, None, None, a["B"], a["H"], a["Hkv"],
                                           a["N"], a["d"], a["qk"], a["v"], None, None, None, 0, None)
    assert window(wl=0) == -2 and window(w0=-1) == -2 and window(w0=8, wl=60) == -2         # window leaves the cache
    assert window(w0=17, wl=40) == -2 and window(w0=0, wl=31) == -2                         # block not inside the window
    assert window(bs=0, bl=64, w0=0, wl=4096, **big) == -5                                  # wide window: split keys
    assert L.dd_block_attention_window_workspace_bytes(64, 4096, 1, 32, 32, 8192, 128, dd.BF16, dd.BF16) == need
    assert L.dd_block_attention_window_workspace_bytes(64, 0, 1, 32, 32, 8192, 128, dd.BF16, dd.BF16) == 0


def test_block_scaled_attention_argument_validation():
    L = dd.lib()

    def call(Q=FAKE, Qs=FAKE, K=FAKE, Ks=FAKE, V=FAKE, Vs=FAKE, O=FAKE, B=1, H=4, Hkv=2, N=64, d=128):
        return L.dd_bidir_attention_mx(Q, Qs, K, Ks, V, Vs, O, B, H, Hkv, N, d, None)
    for name in ("Q", "Qs", "K", "Ks", "V", "Vs", "O"):
        assert call(**{name: None}) == -1
    assert call(B=0) == -2 and call(N=0) == -2 and call(H=3) == -2 and call(d=96) == -2 and call(d=32) == -2
    assert call(Q=FAKE + 4) == -6 and call(V=FAKE + 8) == -6 and call(O=FAKE + 2) == -6
    assert call(Qs=FAKE + 1) == -6 and call(Ks=FAKE + 2) == -6 and call(Vs=FAKE + 3) == -6   # a row's scales are read as a word


def test_cache_insert_argument_validation():
    L = dd.lib()

    def call(Kc=FAKE, Vc=FAKE, Kr=FAKE, Vr=FAKE, pos=FAKE, n=4, B=2, Hkv=2, N=64, d=128, qk=dd.BF16, v=dd.BF16):
        return L.dd_cache_insert_rows(Kc, Vc, Kr, Vr, pos, n, B, Hkv, N, d, qk, v, None)
    assert call(n=-1) == -2 and call(B=0) == -2 and call(d=96) == -2 and call(qk=dd.BF16, v=dd.F32) == -3
    assert call(Kc=None) == -1 and call(Vr=None) == -1 and call(pos=None) == -1
    assert call(Kr=FAKE + 8) == -6 and call(pos=FAKE + 2) == -6
    assert call(n=0, Kc=None, pos=None) == 0               # nothing to insert


def test_verify_argument_validation():
    L = dd.lib()

    def call(ld=FAKE, lv=FAKE, mask=FAKE, mode=dd.KL_THRESH, om=FAKE + 4096, ot=FAKE, osc=FAKE, B=2, G=8, V=1024,
             dt=dd.BF16, ws=None, wsn=0, tau=0.3):
        return L.dd_verify_remask(ld, lv, mask, mode, C.c_float(tau), 0, om, ot, osc, B, G, V, dt, ws, wsn, None)
    assert call(mode=7) == -4 and call(mode=-1) == -4
    # the budget of the budgeted modes is a non-negative finite number; drafter logits only for the KL form
    assert call(mode=dd.KL_TOPK, tau=-1.0) == -2 and call(mode=dd.CONF_TOPK, tau=float("inf")) == -2
    assert call(mode=dd.CONF_TOPK, tau=float("nan")) == -2
    assert call(mode=dd.KL_TOPK, ld=None, tau=3.0) == -1 and call(mode=dd.CONF_TOPK, ld=None, tau=3.0) == -5
    assert call(dt=dd.FP8_E4M3) == -3
    assert call(B=-1) == -2 and call(V=0) == -2
    assert call(V=1001) == -6                              # row pitch not a multiple of 16 bytes
    assert call(lv=None) == -1 and call(ld=None) == -1 and call(om=None) == -1
    assert call(ld=None, mode=dd.TRUST) == -5              # drafter logits optional outside the KL modes; workspace is not
    assert call(B=0) == 0 and call(G=0) == 0               # empty input is a no-op
    need = L.dd_verify_remask_workspace_bytes(2, 8, 1024, dd.BF16)
    assert need >= 16 * 32
    assert call(ws=FAKE, wsn=need - 1) == -5
    # updating the mask in place: fine for the per-row rules (validation goes on to the missing workspace),
    # refused for the rules that read a whole sequence's mask; ranges that merely overlap are always refused
    for mode in (dd.TRUST, dd.KL_THRESH, dd.CONF_THRESH, dd.CONF_PROB):
        assert call(mode=mode, om=FAKE) == -5
        assert call(mode=mode, om=FAKE + 15) == -2 and call(mode=mode, mask=FAKE + 8, om=FAKE) == -2
        assert call(mode=mode, om=FAKE + 16) == -5         # P = 16 bytes: adjacent, not overlapping
    for mode in (dd.KL_PROB, dd.KL_TOPK, dd.CONF_TOPK):
        assert call(mode=mode, om=FAKE, tau=2.0) == -2 and call(mode=mode, om=FAKE + 3, tau=2.0) == -2
        assert call(mode=mode, om=FAKE + 16, tau=2.0) == -5


def test_unmask_argument_validation():
    L = dd.lib()

    def call(ld=FAKE, mask=FAKE, mode=dd.UNMASK_THRESH, tau=0.5, x=None, om=FAKE + 4096, ot=FAKE, oc=FAKE, B=2, G=8,
             V=1024, dt=dd.BF16, ws=None, wsn=0):
        return L.dd_unmask(ld, mask, mode, C.c_float(tau), x, om, ot, oc, B, G, V, dt, ws, wsn, None)
    assert call(mode=2) == -4 and call(mode=-1) == -4
    assert call(mode=dd.UNMASK_TOPK, tau=-1.0) == -2 and call(mode=dd.UNMASK_TOPK, tau=float("nan")) == -2
    assert call(dt=dd.FP8_E4M3) == -3 and call(B=-1) == -2 and call(V=0) == -2 and call(V=1001) == -6
    assert call(ld=None) == -1 and call(mask=None) == -1 and call(om=None) == -1 and call(oc=None) == -1
    assert call(om=FAKE) == -2 and call(om=FAKE + 15) == -2 and call(mask=FAKE + 15, om=FAKE) == -2   # no overlap with mask
    assert call(om=FAKE + 16) == -5
    assert call() == -5                                    # everything valid except the missing workspace
    assert call(B=0) == 0 and call(G=0) == 0
    assert L.dd_unmask_workspace_bytes(2, 8, 1024, dd.BF16) == L.dd_verify_remask_workspace_bytes(2, 8, 1024, dd.BF16)


def test_verify_scores_argument_validation():
    L = dd.lib()

    def call(ld=FAKE, lv=FAKE, okl=FAKE, ocv=FAKE, otv=FAKE, ocd=None, otd=None, P=16, V=1024, dt=dd.BF16, ws=None,
             wsn=0):
        return L.dd_verify_scores(ld, lv, okl, ocv, otv, ocd, otd, P, V, dt, ws, wsn, None)
    assert call(dt=dd.FP8_E4M3) == -3 and call(P=-1) == -2 and call(V=0) == -2 and call(V=1001) == -6
    assert call(ld=None) == -1 and call(lv=None) == -1 and call(okl=None) == -1 and call(ocv=None) == -1
    assert call(otv=None) == -1 and call(lv=FAKE + 4) == -6
    assert call() == -5                                    # the drafter's outputs are optional; the workspace is not
    assert call(P=0) == 0
    assert L.dd_verify_scores_workspace_bytes(16, 1024, dd.BF16) == L.dd_verify_remask_workspace_bytes(2, 8, 1024, dd.BF16)


def test_binding_refuses_cpu_tensors():
    import torch
    q = torch.zeros(1, 1, 4, 64)
    with pytest.raises(ValueError):
        dd.dd_bidir_attention(q, q, q, O=q)
