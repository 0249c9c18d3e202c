"""GPU parity of dd_block_attention_refresh (block completion: attend, and write the block's K/V rows into the
cache in the same call) against the CPU oracle, on every kernel that serves the drafter's call."""
import numpy as np
import pytest

import oracle
import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from _util import assert_attention_close, out_to_f64, to_dev

pytestmark = pytest.mark.gpu


def raw(t):
    """device tensor -> the stored bytes as a numpy array shaped like the tensor"""
    import torch
    return t.contiguous().view(torch.uint8).cpu().numpy()


def raw_np(a):
    return np.ascontiguousarray(a).view(np.uint8)


def check_refresh(cfg, cache, blk, bs, what):
    import torch
    Kc, Vc = to_dev(cache["Kc"]), to_dev(cache["Vc"])
    Kb, Vb = to_dev(blk["Kblk"]), to_dev(blk["Vblk"])
    Q = to_dev(blk["Qblk"])
    qs, ks = to_dev(blk["q_scale"]), to_dev(cache["k_scale"])
    O = dd.dd_block_attention_refresh(Q, Kc, Vc, bs, Kb, Vb, q_scale=qs, k_scale=ks,
                                      qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
    torch.cuda.synchronize()
    ref, Kn, Vn = oracle.block_attention_refresh(blk["Qblk"], cache["Kc"], cache["Vc"], bs, cfg.qk_dtype, cfg.v_dtype,
                                                 blk["Kblk"], blk["Vblk"], blk["q_scale"], cache["k_scale"])
    assert_attention_close(out_to_f64(O, cfg.v_dtype), ref, cfg.qk_dtype, what)
    # the cache afterwards, byte for byte: block rows replaced, every other row untouched
    assert np.array_equal(raw(Kc), raw_np(Kn)), f"{what}: K cache differs"
    assert np.array_equal(raw(Vc), raw_np(Vn)), f"{what}: V cache differs"
    assert np.array_equal(raw(Kb), raw_np(blk["Kblk"])) and np.array_equal(raw(Vb), raw_np(blk["Vblk"]))
    # a plain cached call on the refreshed cache now sees the block's rows
    O2 = dd.dd_block_attention_cached(Q, Kc, Vc, bs, q_scale=qs, k_scale=ks, qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
    torch.cuda.synchronize()
    assert_attention_close(out_to_f64(O2, cfg.v_dtype), ref, cfg.qk_dtype, what + " (cached call afterwards)")
    # same output as the splicing call that leaves the cache alone (same kernels, same order of operations)
    O3 = dd.dd_block_attention_cached(Q, to_dev(cache["Kc"]), to_dev(cache["Vc"]), bs, Kblk=Kb, Vblk=Vb, q_scale=qs,
                                      k_scale=ks, qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
    assert torch.equal(O3, O), f"{what}: output differs from dd_block_attention_cached with Kblk/Vblk"


SHAPES = [
    # (B, H, Hkv, N, d, bl, block_start, qk, env): every kernel of the drafter's call, with and without key splits,
    # block at the start / end / inside, ragged sizes, GQA, one query row, all storage types
    (1, 2, 2, 64, 128, 64, 0, wl.BF16, {}),                                   # streaming kernel, one tile, no split
    (2, 4, 2, 333, 128, 32, 101, wl.BF16, {}),                                # streaming kernel
    (1, 2, 2, 4096, 128, 64, 2000, wl.BF16, {}),                              # streaming kernel, key splits
    (1, 2, 1, 150, 64, 1, 77, wl.BF16, {}),                                   # one query row
    (1, 4, 2, 700, 128, 32, 668, wl.BF16, {"DD_TUNE_BLOCK_STREAM": "0"}),     # MFMA kernel, block at the end
    (1, 2, 2, 4096, 128, 64, 0, wl.BF16, {"DD_TUNE_BLOCK_STREAM": "0"}),      # MFMA kernel, key splits
    (1, 8, 2, 1000, 128, 64, 936, wl.FP8_E4M3, {}),                           # fp8 keys: a byte copy under one scale
    (2, 8, 2, 640, 128, 64, 256, wl.FP8_E4M3, {}),                            # wide kernel, fp8
    (2, 8, 2, 640, 128, 64, 200, wl.BF16, {}),                                # wide kernel
    (1, 4, 1, 4096, 128, 128, 2000, wl.BF16, {}),                             # wide kernel, key splits
    (1, 4, 1, 512, 128, 64, 448, wl.BF16, {"DD_TUNE_BLOCK_WIDE": "0"}),
    (1, 8, 2, 400, 64, 64, 64, wl.BF16, {}),
    (2, 4, 2, 640, 128, 64, 256, wl.FP8_E4M3, {}),                            # wide kernel, 128-row tiles
    (1, 4, 2, 4096, 128, 64, 2000, wl.BF16, {}),                              # ... key splits
    (1, 4, 4, 128, 64, 16, 64, wl.F32, {}),                                   # fp32 kernel
    (2, 2, 1, 600, 128, 48, 200, wl.F32, {}),
    (1, 1, 1, 64, 128, 64, 0, wl.BF16, {}),                                   # the block is the whole sequence
]


@pytest.mark.parametrize("B,H,Hkv,N,d,bl,bs,qk,env", SHAPES)
def test_refresh_every_kernel(monkeypatch, B, H, Hkv, N, d, bl, bs, qk, env):
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    vd = wl.F32 if qk == wl.F32 else wl.BF16
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=vd, bl=bl, prompt=0, G=N)
    cache = wl.cache_inputs(cfg, seed=bs + N)
    blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
    check_refresh(cfg, cache, blk, bs, f"refresh {B}x{H}/{Hkv} N{N} d{d} bl{bl}@{bs} dtype {qk} {env}")


@pytest.mark.parametrize("cfg_id", [1, 2, 3, 4, 5])
def test_refresh_configs(cfg_id):
    # every benchmark configuration at full size (cfg3: no key split, the copy is a launch of its own; cfg4: eight
    # splits; cfg5: the wide kernel's drafter form): every output row against the oracle, the cache byte for byte
    cfg = wl.CONFIGS[cfg_id]
    cache = wl.cache_inputs(cfg, 0)
    blk = wl.block_inputs(cfg, 0, cfg.K - 1, k_scale=cache["k_scale"])
    check_refresh(cfg, cache, blk, blk["block_start"], f"{cfg.name} refresh")


def test_refreshing_every_block_makes_the_drafter_exact():
    # after each block of the generation region has been completed with the current K/V, the cache equals K/V
    # there, and the drafter's output on any block equals the rows of the verifier's full attention (Sec. 2.3)
    import torch
    cfg = wl.custom_config(B=1, H=4, Hkv=2, N=512, d=128, bl=64, prompt=0, G=512)
    cur = wl.attention_inputs(cfg, 8)
    cache = wl.cache_inputs(cfg, 8)
    Kc, Vc = to_dev(cache["Kc"]), to_dev(cache["Vc"])
    for bs in range(0, cfg.N, cfg.bl):
        sl = slice(bs, bs + cfg.bl)
        dd.dd_block_attention_refresh(to_dev(np.ascontiguousarray(cur["Q"][:, :, sl])), Kc, Vc, bs,
                                      to_dev(np.ascontiguousarray(cur["K"][:, :, sl])),
                                      to_dev(np.ascontiguousarray(cur["V"][:, :, sl])))
    torch.cuda.synchronize()
    assert np.array_equal(raw(Kc), raw_np(cur["K"])) and np.array_equal(raw(Vc), raw_np(cur["V"]))
    bs = 192
    got = dd.dd_block_attention_cached(to_dev(np.ascontiguousarray(cur["Q"][:, :, bs:bs + cfg.bl])), Kc, Vc, bs)
    ref = oracle.bidir_attention(cur["Q"], cur["K"], cur["V"], wl.BF16, wl.BF16)[:, :, bs:bs + cfg.bl]
    assert_attention_close(out_to_f64(got, wl.BF16), ref, wl.BF16, "drafter on a fully refreshed cache")


def test_refresh_requires_block_tensors():
    import torch
    q = torch.zeros(1, 2, 16, 64, dtype=torch.bfloat16, device="cuda:0")
    kc = torch.zeros(1, 2, 64, 64, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(dd.DDError):
        dd.dd_block_attention_refresh(q, kc, kc.clone(), 0, None, None)
