"""GPU parity of dd_block_attention_window (drafter attention over a local window of the cache) against the oracle."""
import numpy as np
import pytest

import oracle
import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from _util import assert_attention_close, out_to_f64, to_dev

pytestmark = pytest.mark.gpu


def gpu_window(cfg, blk, cache, bs, w0, wlen, fresh):
    import torch
    Kb, Vb = (to_dev(blk["Kblk"]), to_dev(blk["Vblk"])) if fresh else (None, None)
    O = dd.dd_block_attention_window(to_dev(blk["Qblk"]), to_dev(cache["Kc"]), to_dev(cache["Vc"]), bs, w0, wlen,
                                     Kblk=Kb, Vblk=Vb, q_scale=to_dev(blk["q_scale"]), k_scale=to_dev(cache["k_scale"]),
                                     qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
    torch.cuda.synchronize()
    return O


SHAPES = [
    # (B, H, Hkv, N, d, bl, block_start, win_start, win_len, qk, env): every kernel of the drafter's call; windows at
    # the start / end / inside the cache, equal to the block, ragged lengths, with and without key splits
    (2, 4, 2, 333, 128, 32, 101, 64, 200, wl.BF16, {}),                              # streaming kernel
    (1, 2, 2, 4096, 128, 64, 2000, 1000, 2048, wl.BF16, {}),                         # streaming kernel, key splits
    (1, 2, 2, 4096, 128, 64, 4032, 3000, 1096, wl.BF16, {}),                         # window and block end at N
    (1, 2, 1, 150, 64, 1, 77, 77, 1, wl.BF16, {}),                                   # one query, one key
    (1, 3, 3, 500, 128, 33, 100, 100, 33, wl.BF16, {}),                              # window = block
    (1, 4, 2, 700, 128, 32, 60, 0, 129, wl.BF16, {"DD_TUNE_BLOCK_STREAM": "0"}),     # MFMA kernel
    (1, 2, 2, 4096, 128, 64, 1000, 7, 3001, wl.BF16, {"DD_TUNE_BLOCK_STREAM": "0"}),
    (1, 8, 2, 1000, 128, 64, 936, 500, 500, wl.FP8_E4M3, {}),
    (2, 8, 2, 640, 128, 64, 256, 128, 384, wl.FP8_E4M3, {}),                         # wide kernel, fp8
    (2, 8, 2, 640, 128, 64, 200, 136, 300, wl.BF16, {}),                             # wide kernel, ragged parts
    (1, 4, 1, 4096, 128, 128, 2000, 1024, 2048, wl.BF16, {}),                        # wide kernel, key splits
    (1, 4, 1, 4096, 128, 128, 2000, 1990, 150, wl.BF16, {}),                         # parts shorter than a tile
    (1, 8, 2, 400, 64, 64, 64, 0, 256, wl.BF16, {}),
    (2, 4, 2, 640, 128, 64, 256, 128, 384, wl.FP8_E4M3, {}),                         # wide kernel, 128-row tiles
    (1, 4, 2, 4096, 128, 64, 2000, 1990, 150, wl.BF16, {}),                          # ... parts shorter than a tile
    (1, 4, 4, 128, 64, 16, 64, 32, 64, wl.F32, {}),                                  # fp32 kernel
    (2, 2, 1, 600, 128, 48, 200, 150, 301, wl.F32, {}),
]


@pytest.mark.parametrize("B,H,Hkv,N,d,bl,bs,w0,wlen,qk,env", SHAPES)
def test_window_every_kernel(monkeypatch, B, H, Hkv, N, d, bl, bs, w0, wlen, qk, env):
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    vd = wl.F32 if qk == wl.F32 else wl.BF16
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=vd, bl=bl, prompt=0, G=N)
    cache = wl.cache_inputs(cfg, seed=bs + N + w0)
    blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
    for fresh in (True, False):
        got = out_to_f64(gpu_window(cfg, blk, cache, bs, w0, wlen, fresh), vd)
        Kb, Vb = (blk["Kblk"], blk["Vblk"]) if fresh else (None, None)
        ref = oracle.block_attention_window(blk["Qblk"], cache["Kc"], cache["Vc"], bs, w0, wlen, qk, vd, Kb, Vb,
                                            blk["q_scale"], cache["k_scale"])
        assert_attention_close(got, ref, qk, f"window {B}x{H}/{Hkv} N{N} d{d} bl{bl}@{bs} win [{w0},+{wlen}) dtype {qk} fresh={fresh} {env}")


def test_window_ignores_rows_outside_and_full_window_is_the_cached_call():
    import torch
    cfg = wl.custom_config(B=2, H=4, Hkv=2, N=1024, d=128, bl=64, prompt=0, G=1024)
    cache = wl.cache_inputs(cfg, seed=3)
    bs, w0, wlen = 512, 256, 512
    blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
    O = gpu_window(cfg, blk, cache, bs, w0, wlen, True)
    # rows outside the window overwritten with huge values (NaN patterns included): bit-identical output
    poisoned = {k: v.copy() if isinstance(v, np.ndarray) else v for k, v in cache.items()}
    for name in ("Kc", "Vc"):
        poisoned[name][:, :, :w0] = 0x7FC0          # bf16 NaN
        poisoned[name][:, :, w0 + wlen:] = 0x7F80   # bf16 +inf
    O2 = gpu_window(cfg, blk, poisoned, bs, w0, wlen, True)
    assert torch.equal(O, O2) and torch.isfinite(O2.view(torch.bfloat16).float()).all()
    # the whole cache as the window: the plain cached call, bit for bit
    O3 = gpu_window(cfg, blk, cache, bs, 0, cfg.N, True)
    O4 = dd.dd_block_attention_cached(to_dev(blk["Qblk"]), to_dev(cache["Kc"]), to_dev(cache["Vc"]), bs,
                                      Kblk=to_dev(blk["Kblk"]), Vblk=to_dev(blk["Vblk"]))
    assert torch.equal(O3, O4)


@pytest.mark.parametrize("cfg_id", [2, 4, 5])
def test_window_configs(cfg_id):
    # the workload's last draft step over a window of half the sequence around the block
    cfg = wl.CONFIGS[cfg_id]
    cache = wl.cache_inputs(cfg, 0)
    blk = wl.block_inputs(cfg, 0, cfg.K - 1, k_scale=cache["k_scale"])
    bs = blk["block_start"]
    wlen = cfg.N // 2
    w0 = min(max(0, bs + cfg.bl // 2 - wlen // 2), cfg.N - wlen)
    got = out_to_f64(gpu_window(cfg, blk, cache, bs, w0, wlen, True), cfg.v_dtype)
    rng = np.random.default_rng(5)
    rows = sorted(set(zip(rng.integers(0, cfg.B, 96).tolist(), rng.integers(0, cfg.H, 96).tolist(),
                          rng.integers(0, cfg.bl, 96).tolist())))
    ref = oracle.block_attention_window(blk["Qblk"], cache["Kc"], cache["Vc"], bs, w0, wlen, cfg.qk_dtype, cfg.v_dtype,
                                        blk["Kblk"], blk["Vblk"], blk["q_scale"], cache["k_scale"], rows=rows)
    assert_attention_close(np.stack([got[b, h, i] for b, h, i in rows]), ref, cfg.qk_dtype, f"{cfg.name} window")
