"""No entry point writes outside its outputs: every output, the workspace and (for the calls that update it) the
cache are carved out of poison-filled allocations, and the bands around them - and every input - are compared
byte for byte after the call.  Ragged shapes, every kernel family."""
import numpy as np
import pytest

import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from _util import to_dev

pytestmark = pytest.mark.gpu

BAND = 8192          # bytes of poison on either side (a multiple of 256: the views stay aligned)
POISON = 0xA5


class Guarded:
    """Device tensors inside poison-filled bands."""

    def __init__(self):
        self.items = []

    def empty(self, shape, dtype):
        import torch
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        pad = (-n) % 256
        base = torch.full((BAND + n + pad + BAND,), POISON, dtype=torch.uint8, device="cuda:0")
        view = base[BAND:BAND + n].view(dtype).view(shape)
        self.items.append((base, n))
        return view

    def like(self, host):
        """a guarded copy of a host array (an input, or an in-place operand)"""
        t = to_dev(host)
        g = self.empty(tuple(t.shape), t.dtype)
        g.copy_(t)
        return g

    def check(self, what):
        import torch
        torch.cuda.synchronize()
        for k, (base, n) in enumerate(self.items):
            lo, hi = base[:BAND], base[BAND + n:]
            assert bool((lo == POISON).all()) and bool((hi == POISON).all()), f"{what}: tensor {k} ({n} bytes): a band was written"


def guarded_workspace(g, nbytes):
    import torch
    return g.empty((max(nbytes, 256),), torch.uint8)


def unchanged(dev, host, what):
    import torch
    got = dev.contiguous().view(torch.uint8).cpu().numpy().reshape(-1)
    assert np.array_equal(got, np.ascontiguousarray(host).view(np.uint8).reshape(-1)), f"{what}: an input was modified"


ATTN = [
    # (B, H, Hkv, N, d, qk, env)
    (1, 3, 1, 77, 64, wl.BF16, {}), (2, 4, 2, 200, 128, wl.BF16, {"DD_TUNE_ATTN_WIDE": "1"}),
    (1, 4, 1, 257, 64, wl.BF16, {"DD_TUNE_ATTN_WIDE": "1", "DD_TUNE_ATTN_WIDE_GRID": "2"}),
    (1, 2, 1, 2111, 128, wl.BF16, {"DD_TUNE_ATTN_WIDE": "1"}),           # folded-scale form, ragged last tile
    (2, 8, 2, 130, 128, wl.FP8_E4M3, {"DD_TUNE_ATTN_WIDE": "1"}), (1, 4, 4, 96, 64, wl.FP8_E4M3, {}),
    (1, 2, 2, 333, 128, wl.BF16, {"DD_TUNE_ATTN_WIDE": "0", "DD_TUNE_BIDIR_STREAM": "1"}),
    (1, 2, 2, 333, 128, wl.BF16, {"DD_TUNE_ATTN_WIDE": "0", "DD_TUNE_BIDIR_STREAM": "0"}),
    (1, 2, 1, 257, 128, wl.F32, {}),
]


@pytest.mark.parametrize("B,H,Hkv,N,d,qk,env", ATTN)
def test_bidir_attention_stays_inside_its_output(monkeypatch, B, H, Hkv, N, d, qk, env):
    import torch
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    vd = wl.F32 if qk == wl.F32 else wl.BF16
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=vd, prompt=0, G=N, bl=min(16, N))
    inp = wl.attention_inputs(cfg, seed=N)
    g = Guarded()
    Q, K, V = g.like(inp["Q"]), g.like(inp["K"]), g.like(inp["V"])
    O = g.empty((B, H, N, d), V.dtype)
    dd.dd_bidir_attention(Q, K, V, O=O, q_scale=to_dev(inp["q_scale"]), k_scale=to_dev(inp["k_scale"]), qk_dtype=qk, v_dtype=vd)
    g.check(f"bidir {B}x{H}/{Hkv}x{N}x{d} {env}")
    for t, h in ((Q, inp["Q"]), (K, inp["K"]), (V, inp["V"])):
        unchanged(t, h, "bidir")
    assert not bool((O.view(torch.uint8) == POISON).all())


BLOCK = [
    # (B, H, Hkv, N, d, bl, bs, qk, env): streaming / MFMA / wide / fp32 kernels, with and without key splits
    (2, 4, 2, 333, 128, 32, 101, wl.BF16, {}), (1, 2, 2, 4096, 128, 64, 2000, wl.BF16, {}),
    (1, 4, 2, 700, 128, 32, 668, wl.BF16, {"DD_TUNE_BLOCK_STREAM": "0"}),
    (1, 2, 2, 4096, 128, 64, 37, wl.BF16, {"DD_TUNE_BLOCK_STREAM": "0"}),
    (1, 4, 1, 1000, 128, 80, 700, wl.BF16, {}), (1, 4, 1, 4097, 128, 128, 2000, wl.BF16, {}),
    (2, 8, 2, 641, 128, 64, 256, wl.FP8_E4M3, {}), (2, 2, 1, 600, 128, 48, 200, wl.F32, {}),
    (1, 2, 1, 150, 64, 1, 77, wl.BF16, {}),
    # the wide kernel's 128-row tiles: a partly filled tile (2 x 40 rows), fp8 with key splits
    (3, 4, 2, 333, 128, 40, 101, wl.BF16, {}), (1, 4, 2, 4097, 128, 64, 2000, wl.FP8_E4M3, {}),
    # ... with 128-byte rows a wave's 32 output rows are four stores: the last wave of the call ends at the buffer's end
    (1, 2, 1, 300, 64, 64, 100, wl.BF16, {}), (2, 5, 1, 221, 64, 64, 61, wl.BF16, {"DD_TUNE_BLOCK_WIDE_ROWS": "128"}),
]


@pytest.mark.parametrize("call", ["cached", "refresh", "window", "batched"])
@pytest.mark.parametrize("B,H,Hkv,N,d,bl,bs,qk,env", BLOCK)
def test_block_attention_calls_stay_inside_their_outputs(monkeypatch, call, B, H, Hkv, N, d, bl, bs, qk, env):
    import torch
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    vd = wl.F32 if qk == wl.F32 else wl.BF16
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=vd, bl=bl, prompt=0, G=N)
    cache = wl.cache_inputs(cfg, seed=bs + N)
    blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
    g = Guarded()
    Q, Kc, Vc = g.like(blk["Qblk"]), g.like(cache["Kc"]), g.like(cache["Vc"])
    Kb, Vb = g.like(blk["Kblk"]), g.like(blk["Vblk"])
    O = g.empty((B, H, bl, d), Vc.dtype)
    qs, ks = to_dev(blk["q_scale"]), to_dev(cache["k_scale"])
    need = {"cached": dd.dd_block_attention_cached_workspace_bytes(bl, B, H, Hkv, N, d, qk, vd),
            "refresh": dd.dd_block_attention_refresh_workspace_bytes(bl, B, H, Hkv, N, d, qk, vd),
            "batched": dd.lib().dd_block_attention_batched_workspace_bytes(bl, B, H, Hkv, N, d, qk, vd)}
    w0 = max(0, bs - 70)
    wlen = min(N - w0, bl + 70 + 133)
    need["window"] = dd.dd_block_attention_window_workspace_bytes(bl, wlen, B, H, Hkv, N, d, qk, vd)
    ws = guarded_workspace(g, need[call])
    kw = dict(O=O, q_scale=qs, k_scale=ks, qk_dtype=qk, v_dtype=vd)
    with dd.fixed_workspace(ws):
        if call == "cached":
            dd.dd_block_attention_cached(Q, Kc, Vc, bs, Kblk=Kb, Vblk=Vb, **kw)
        elif call == "refresh":
            dd.dd_block_attention_refresh(Q, Kc, Vc, bs, Kb, Vb, **kw)
        elif call == "window":
            dd.dd_block_attention_window(Q, Kc, Vc, bs, w0, wlen, Kblk=Kb, Vblk=Vb, **kw)
        else:
            starts = to_dev(np.array([(bs + 17 * b) % (N - bl + 1) for b in range(B)], np.int32))
            dd.dd_block_attention_batched(Q, Kc, Vc, starts, Kb, Vb, **kw)
    what = f"{call} {B}x{H}/{Hkv} N{N} d{d} bl{bl}@{bs} dtype {qk} {env}"
    g.check(what)
    unchanged(Q, blk["Qblk"], what); unchanged(Kb, blk["Kblk"], what); unchanged(Vb, blk["Vblk"], what)
    if call == "refresh":                                   # exactly the block's rows changed, nothing else
        Kn, Vn = cache["Kc"].copy(), cache["Vc"].copy()
        Kn[:, :, bs:bs + bl] = blk["Kblk"]; Vn[:, :, bs:bs + bl] = blk["Vblk"]
        unchanged(Kc, Kn, what); unchanged(Vc, Vn, what)
    else:
        unchanged(Kc, cache["Kc"], what); unchanged(Vc, cache["Vc"], what)


def test_cache_insert_rows_stays_inside_the_cache():
    cfg = wl.custom_config(B=3, H=4, Hkv=2, N=301, d=128, bl=16, prompt=0, G=301)
    cache = wl.cache_inputs(cfg, seed=4)
    rows = wl.block_inputs(cfg, 4, 0, k_scale=cache["k_scale"])          # 16 fresh rows per (batch, kv head)
    pos = np.array([[0, 300, 5, -1, 301, 17, 299, 2**31 - 1, 44, 45, 46, 100, 200, 250, 7, 8]] * 3, np.int32)
    pos[1] = (pos[1] + 3) % 305 - 2
    pos[2, :] = -7
    g = Guarded()
    Kc, Vc = g.like(cache["Kc"]), g.like(cache["Vc"])
    Kr, Vr = g.like(rows["Kblk"]), g.like(rows["Vblk"])
    dd.dd_cache_insert_rows(Kc, Vc, Kr, Vr, to_dev(pos))
    g.check("cache insert")
    import oracle
    Kn, Vn = oracle.cache_insert_rows(cache["Kc"], cache["Vc"], rows["Kblk"], rows["Vblk"], pos)
    unchanged(Kc, Kn, "cache insert"); unchanged(Vc, Vn, "cache insert")
    unchanged(Kr, rows["Kblk"], "cache insert")


VERIFY = [
    # (B, G, V, dtype): split path (few rows), fused path (512 and 256 lanes per row), ragged vocabularies
    (2, 5, 40008, wl.BF16), (3, 50, 126464, wl.BF16), (4, 75, 1000, wl.BF16), (2, 1100, 520, wl.F32), (1, 191, 8200, wl.BF16),
]


@pytest.mark.parametrize("B,G,V,dtype", VERIFY)
def test_verification_calls_stay_inside_their_outputs(B, G, V, dtype):
    import torch
    cfg = wl.custom_config(B=B, G=G, V=V, logit_dtype=dtype, sigma_d=3.0, sigma_n=1.0, decoded_frac=0.5)
    inp = wl.verify_inputs(cfg, seed=G)
    P = B * G
    need = dd.dd_verify_remask_workspace_bytes(B, G, V, dtype)
    for mode, tau in ((wl.KL_THRESH, 0.4), (wl.CONF_THRESH, 0.02), (wl.KL_PROB, 0.0), (wl.KL_TOPK, 3.0), (wl.CONF_TOPK, 2.0),
                      (wl.TRUST, 0.0), (wl.CONF_PROB, 0.0)):
        g = Guarded()
        ld, lv, mk = g.like(inp["logits_d"]), g.like(inp["logits_v"]), g.like(inp["mask"])
        om, ot, osc = g.empty((P,), torch.uint8), g.empty((P,), torch.int32), g.empty((P,), torch.float32)
        ws = guarded_workspace(g, need)
        with dd.fixed_workspace(ws):
            dd.dd_verify_remask(ld, lv, mk, mode, tau, 3, B, G, out_mask=om, out_tokens=ot, out_scores=osc, logit_dtype=dtype)
        g.check(f"verify mode {mode} {B}x{G}x{V}")
        unchanged(ld, inp["logits_d"], "verify"); unchanged(lv, inp["logits_v"], "verify"); unchanged(mk, inp["mask"], "verify")
        g2 = Guarded()
        om2, ot2, osc2 = g2.empty((P,), torch.uint8), g2.empty((P,), torch.int32), g2.empty((P,), torch.float32)
        dd.dd_verify_remask_static(ld, lv, mk, mode, tau, 3, B, G, om2, ot2, osc2, logit_dtype=dtype)
        g2.check(f"verify (static scratch) mode {mode}")
        assert torch.equal(om, om2) and torch.equal(ot, ot2) and torch.equal(osc, osc2)
    # the unmasking step and the all-scores pass
    g = Guarded()
    ld, lv, mk = g.like(inp["logits_d"]), g.like(inp["logits_v"]), g.like(inp["mask"])
    om, ot, oc = g.empty((P,), torch.uint8), g.empty((P,), torch.int32), g.empty((P,), torch.float32)
    x = g.empty((P,), torch.int32)
    x.fill_(-3)
    ws = guarded_workspace(g, need)
    with dd.fixed_workspace(ws):
        for umode, thr in ((dd.UNMASK_THRESH, 0.05), (dd.UNMASK_TOPK, 4.0)):
            dd.dd_unmask(ld, mk, umode, thr, B, G, x_tokens=x, out_mask=om, out_tokens=ot, out_conf=oc, logit_dtype=dtype)
    g.check("unmask")
    unchanged(ld, inp["logits_d"], "unmask"); unchanged(mk, inp["mask"], "unmask")
