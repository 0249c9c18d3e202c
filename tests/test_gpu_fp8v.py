"""GPU parity of the fp8-V precision workload (dd_bidir_attention_fp8v, dd_block_attention_cached_fp8v: Q, K and V
all e4m3 with per-head scales) against the CPU oracle, at the tolerance of the fp8 path."""
import numpy as np
import pytest

import oracle
import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from _util import assert_attention_close, out_to_f64, to_dev

pytestmark = pytest.mark.gpu
FP8 = wl.FP8_E4M3


def gpu_bidir(inp):
    import torch
    O = dd.dd_bidir_attention_fp8v(to_dev(inp["Q"]), to_dev(inp["K"]), to_dev(inp["V"]), to_dev(inp["q_scale"]),
                                   to_dev(inp["k_scale"]), to_dev(inp["v_scale"]))
    torch.cuda.synchronize()
    return out_to_f64(O, wl.BF16)


SHAPES = [(1, 2, 2, 1, 64), (1, 2, 2, 33, 128), (2, 4, 2, 200, 128), (1, 3, 1, 77, 64), (2, 8, 2, 130, 128), (1, 16, 2, 320, 128),
          (1, 4, 1, 1000, 128)]


@pytest.mark.parametrize("B,H,Hkv,N,d", SHAPES)
def test_bidir_fp8v_small_shapes(B, H, Hkv, N, d):
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=FP8, v_dtype=FP8, prompt=0, G=N, bl=min(16, N))
    inp = wl.attention_inputs(cfg, seed=N)
    got = gpu_bidir(inp)
    ref = oracle.bidir_attention(inp["Q"], inp["K"], inp["V"], FP8, FP8, inp["q_scale"], inp["k_scale"], v_scale=inp["v_scale"])
    assert_attention_close(got, ref, FP8, f"fp8-V bidir {B}x{H}/{Hkv}x{N}x{d}")


def test_bidir_fp8v_scale_and_closed_form():
    # identical keys -> v_scale x mean(decoded V); doubling v_scale doubles the bf16 output exactly
    import torch
    cfg = wl.custom_config(B=1, H=2, Hkv=2, N=192, d=128, qk_dtype=FP8, v_dtype=FP8, prompt=0, G=192)
    inp = wl.attention_inputs(cfg, 1)
    K1 = np.broadcast_to(inp["K"][:, :, :1], inp["K"].shape).copy()
    got = gpu_bidir(dict(inp, K=K1))
    table = np.array([oracle.decode_e4m3(c) for c in range(256)])
    mean = (table[inp["V"]] * inp["v_scale"][:, :, None, None].astype(np.float64)).mean(axis=2, keepdims=True)
    assert np.abs(got - mean).max() < 6e-3
    a = gpu_bidir(inp)
    b = gpu_bidir(dict(inp, v_scale=inp["v_scale"] * np.float32(2)))
    assert np.array_equal(b, 2 * a)


def test_bidir_fp8v_cfg5_shape():
    # the all-fp8 form of the throughput workload (B16, 32 query / 8 kv heads, N 2048): a stratified sample of rows
    # (one per 32-row block of every (batch, kv head)) against the oracle
    base = wl.CONFIGS[5]
    cfg = wl.custom_config(B=base.B, H=base.H, Hkv=base.Hkv, N=base.N, d=base.d, qk_dtype=FP8, v_dtype=FP8, prompt=base.prompt,
                           G=base.G, bl=base.bl)
    inp = wl.attention_inputs(cfg, 0)
    got = gpu_bidir(inp)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(5)
    group, per = cfg.H // cfg.Hkv, (cfg.H // cfg.Hkv) * cfg.N
    rows = []
    for b in range(cfg.B):
        for g in range(cfg.Hkv):
            starts = np.arange(0, per, 128)
            v = np.minimum(starts + rng.integers(0, 128, len(starts)), per - 1)
            rows += [(b, g * group + int(x) // cfg.N, int(x) % cfg.N) for x in v]
    ref = oracle.bidir_attention(inp["Q"], inp["K"], inp["V"], FP8, FP8, inp["q_scale"], inp["k_scale"], rows=rows,
                                 v_scale=inp["v_scale"])
    idx = np.asarray(rows)
    assert_attention_close(got[idx[:, 0], idx[:, 1], idx[:, 2]], ref, FP8, f"fp8-V cfg5 shape ({len(rows)} rows)")


BLOCKS = [(1, 2, 2, 100, 64, 16, 84), (2, 4, 2, 333, 128, 32, 101), (1, 8, 2, 1000, 128, 64, 936), (1, 2, 2, 4096, 128, 64, 2000),
          (1, 2, 1, 150, 64, 1, 77), (1, 16, 4, 2048, 128, 64, 1536)]


@pytest.mark.parametrize("B,H,Hkv,N,d,bl,bs", BLOCKS)
def test_block_fp8v(B, H, Hkv, N, d, bl, bs):
    import torch
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=FP8, v_dtype=FP8, bl=bl, prompt=0, G=N)
    cache = wl.cache_inputs(cfg, seed=bs + N)
    blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"], v_scale=cache["v_scale"])
    for fresh in (True, False):
        Kb, Vb = (blk["Kblk"], blk["Vblk"]) if fresh else (None, None)
        O = dd.dd_block_attention_cached_fp8v(to_dev(blk["Qblk"]), to_dev(cache["Kc"]), to_dev(cache["Vc"]), bs,
                                              to_dev(blk["q_scale"]), to_dev(cache["k_scale"]), to_dev(cache["v_scale"]),
                                              Kblk=to_dev(Kb), Vblk=to_dev(Vb))
        torch.cuda.synchronize()
        ref = oracle.block_attention_cached(blk["Qblk"], cache["Kc"], cache["Vc"], bs, FP8, FP8, Kb, Vb, blk["q_scale"],
                                            cache["k_scale"], v_scale=cache["v_scale"])
        assert_attention_close(out_to_f64(O, wl.BF16), ref, FP8, f"fp8-V block {B}x{H}/{Hkv} N{N} d{d} bl{bl}@{bs} fresh={fresh}")


def test_fp8v_needs_its_scale():
    import torch
    q = torch.zeros((1, 2, 16, 64), dtype=torch.uint8, device="cuda:0")
    s = torch.ones(2, dtype=torch.float32, device="cuda:0")
    with pytest.raises(dd.DDError):
        dd.dd_bidir_attention_fp8v(q, q, q, s, s, None)
