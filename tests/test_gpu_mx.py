"""GPU parity of the block-scaled precision workload (dd_bidir_attention_mx: e4m3 Q/K and e2m1 V with E8M0 scales per
32 elements of the head dimension) against the CPU oracle, at the tolerance of the fp8 path."""
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
    O = dd.dd_bidir_attention_mx(*(to_dev(inp[k]) for k in ("Q", "Qs", "K", "Ks", "V", "Vs")))
    torch.cuda.synchronize()
    return out_to_f64(O, wl.BF16)


def ora_bidir(inp, rows=None):
    return oracle.bidir_attention_mx(inp["Q"], inp["Qs"], inp["K"], inp["Ks"], inp["V"], inp["Vs"], rows=rows)


SHAPES = [(1, 2, 2, 1, 64), (1, 2, 2, 33, 128), (2, 4, 2, 200, 128), (1, 3, 1, 77, 64), (2, 8, 2, 130, 128), (1, 16, 2, 320, 128),
          (1, 4, 1, 1000, 128)]


@pytest.mark.parametrize("B,H,Hkv,N,d", SHAPES)
def test_bidir_mx_small_shapes(B, H, Hkv, N, d):
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, prompt=0, G=N, bl=min(16, N))
    inp = wl.mx_attention_inputs(cfg, seed=N)
    assert_attention_close(gpu_bidir(inp), ora_bidir(inp), FP8, f"MX bidir {B}x{H}/{Hkv}x{N}x{d}")


def test_bidir_mx_scales_block_by_block():
    # scales that differ wildly from block to block and row to row (a misplaced scale is then a gross error), and the
    # exact laws: V's scales up by 3 -> the bf16 output times 8; Q up by 2 with K down by 2 -> bit-identical output
    cfg = wl.custom_config(B=1, H=4, Hkv=2, N=192, d=128, prompt=0, G=192)
    inp = wl.mx_attention_inputs(cfg, 3)
    rng = np.random.default_rng(9)
    inp["Vs"] = rng.integers(110, 140, size=inp["Vs"].shape, dtype=np.uint8)
    inp["Qs"] = (inp["Qs"].astype(np.int32) + rng.integers(-2, 3, size=inp["Qs"].shape)).astype(np.uint8)
    inp["Ks"] = (inp["Ks"].astype(np.int32) + rng.integers(-2, 3, size=inp["Ks"].shape)).astype(np.uint8)
    got = gpu_bidir(inp)
    ref = ora_bidir(inp)
    scale = np.abs(ref).max()
    assert np.abs(got - ref).max() <= 6e-2 * max(1.0, scale) and np.linalg.norm(got - ref) <= 5e-3 * np.linalg.norm(ref)
    up = gpu_bidir(dict(inp, Vs=inp["Vs"] + np.uint8(3)))
    assert np.array_equal(up, 8.0 * got)
    same = gpu_bidir(dict(inp, Qs=inp["Qs"] + np.uint8(2), Ks=inp["Ks"] - np.uint8(2)))
    assert np.array_equal(same, got)
    # identical keys -> the mean of the decoded V rows
    K1 = np.broadcast_to(inp["K"][:, :, :1], inp["K"].shape).copy()
    Ks1 = np.broadcast_to(inp["Ks"][:, :, :1], inp["Ks"].shape).copy()
    flat = gpu_bidir(dict(inp, K=K1, Ks=Ks1))
    mean = oracle.decode_mx(inp["V"], inp["Vs"], oracle.MX_E2M1).mean(axis=2, keepdims=True)
    assert np.abs(flat - np.repeat(mean, 2, axis=1)).max() <= 2 ** -7 * np.abs(mean).max()


def test_bidir_mx_extreme_v_scales():
    # V blocks whose scale codes are so small that the scaled values are no normal bf16 numbers (codes 0 and 1: the
    # kernel's table decode hands those to its plain path) among ordinary ones, and, in other blocks, a very large one
    # (230, i.e. 2^103: the unnormalised fp32 accumulation of some hundred such values times weights of up to 2^8
    # still fits)
    cfg = wl.custom_config(B=1, H=4, Hkv=2, N=160, d=128, prompt=0, G=160)
    inp = wl.mx_attention_inputs(cfg, 11)
    rng = np.random.default_rng(4)
    Vs = inp["Vs"].copy()
    tiny = rng.random(Vs.shape) < 0.2
    Vs[tiny] = rng.integers(0, 2, size=int(tiny.sum()), dtype=np.uint8)
    got = gpu_bidir(dict(inp, Vs=Vs))
    ref = ora_bidir(dict(inp, Vs=Vs))
    assert_attention_close(got, ref, FP8, "MX bidir, V scale codes 0 and 1")
    Vs = np.where(rng.random(Vs.shape) < 0.1, np.uint8(230), inp["Vs"]).astype(np.uint8)
    got = gpu_bidir(dict(inp, Vs=Vs))
    ref = ora_bidir(dict(inp, Vs=Vs))
    assert np.isfinite(got).all()
    assert np.linalg.norm(got - ref) <= 5e-3 * np.linalg.norm(ref)


def test_bidir_mx_cfg5_shape():
    # the block-scaled form of the throughput workload (B16, 32 query / 8 kv heads, N 2048): a stratified sample of
    # rows (one per 128-row block of every (batch, kv head)) against the oracle
    base = wl.CONFIGS[5]
    cfg = wl.custom_config(B=base.B, H=base.H, Hkv=base.Hkv, N=base.N, d=base.d, prompt=base.prompt, G=base.G, bl=base.bl)
    inp = wl.mx_attention_inputs(cfg, 0)
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
    ref = ora_bidir(inp, rows=rows)
    idx = np.asarray(rows)
    assert_attention_close(got[idx[:, 0], idx[:, 1], idx[:, 2]], ref, FP8, f"MX cfg5 shape ({len(rows)} rows)")
