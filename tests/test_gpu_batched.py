"""GPU parity of dd_block_attention_batched (one block position per batch entry) against the oracle."""
import numpy as np
import pytest

import oracle
import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from _util import assert_attention_close, out_to_f64, to_dev

pytestmark = pytest.mark.gpu


def run(cfg, cache, blk, starts):
    import torch
    O = dd.dd_block_attention_batched(to_dev(blk["Qblk"]), to_dev(cache["Kc"]), to_dev(cache["Vc"]),
                                      torch.from_numpy(np.asarray(starts, np.int32)).to("cuda:0"),
                                      to_dev(blk["Kblk"]), to_dev(blk["Vblk"]), q_scale=to_dev(blk["q_scale"]),
                                      k_scale=to_dev(cache["k_scale"]), qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
    torch.cuda.synchronize()
    return O


SHAPES = [
    # (B, H, Hkv, N, d, bl, qk, env): the three kernels that serve per-sequence positions, with and without key
    # splits, GQA, ragged lengths; 256 rows per kv head (a shape the wide kernel would take for one position)
    (4, 4, 2, 333, 128, 32, wl.BF16, {}),                                  # streaming kernel
    (3, 2, 2, 4096, 128, 64, wl.BF16, {}),                                 # streaming kernel, key splits
    (5, 2, 1, 150, 64, 1, wl.BF16, {}),                                    # one query row
    (4, 4, 2, 700, 128, 32, wl.BF16, {"DD_TUNE_BLOCK_STREAM": "0"}),       # MFMA kernel
    (2, 2, 2, 4096, 128, 64, wl.BF16, {"DD_TUNE_BLOCK_STREAM": "0"}),      # MFMA kernel, key splits
    (3, 8, 2, 1000, 128, 64, wl.FP8_E4M3, {}),                             # wide kernel: fp8 keys, 256 rows per kv head
    (2, 16, 4, 2048, 128, 64, wl.BF16, {}),                                # wide kernel (folded-scale form), key splits
    (5, 12, 4, 700, 128, 64, wl.BF16, {}),                                 # wide kernel: 192 rows per kv head, ragged length
    (3, 8, 2, 1000, 128, 64, wl.FP8_E4M3, {"DD_TUNE_BLOCK_WIDE": "0"}),    # the same shapes on the MFMA kernel
    (2, 16, 4, 2048, 128, 64, wl.BF16, {"DD_TUNE_BLOCK_WIDE": "0"}),
    (4, 4, 4, 128, 64, 16, wl.F32, {}),                                    # fp32 kernel
    (3, 2, 1, 600, 128, 48, wl.F32, {}),
    (3, 4, 2, 1000, 128, 64, wl.FP8_E4M3, {}),                             # wide kernel, 128-row tiles (128 rows per kv head)
    (5, 6, 2, 700, 128, 40, wl.BF16, {}),                                  # ... 120 rows per kv head, blocks shorter than a key tile
    (2, 16, 4, 2048, 128, 64, wl.BF16, {"DD_TUNE_BLOCK_WIDE_ROWS": "128"}),   # ... forced on 256 rows per kv head
]


@pytest.mark.parametrize("B,H,Hkv,N,d,bl,qk,env", SHAPES)
def test_batched_positions(monkeypatch, B, H, Hkv, N, d, bl, qk, env):
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    vd = wl.F32 if qk == wl.F32 else wl.BF16
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=vd, bl=bl, prompt=0, G=N)
    cache = wl.cache_inputs(cfg, seed=N + bl)
    blk = wl.block_inputs(cfg, 0, 0, k_scale=cache["k_scale"])
    rng = np.random.default_rng(N + B)
    starts = rng.integers(0, N - bl + 1, B).astype(np.int32)
    starts[0] = 0
    starts[-1] = N - bl                                                    # first and last legal positions
    if B >= 3:
        starts[1] = min(7, N - bl)                                         # seven cache rows before the block: a part shorter than a tile
    got = out_to_f64(run(cfg, cache, blk, starts), vd)
    ref = oracle.block_attention_batched(blk["Qblk"], cache["Kc"], cache["Vc"], starts, qk, vd, blk["Kblk"],
                                         blk["Vblk"], blk["q_scale"], cache["k_scale"])
    assert_attention_close(got, ref, qk, f"batched {B}x{H}/{Hkv} N{N} d{d} bl{bl} dtype {qk} {env} starts {starts}")


@pytest.mark.parametrize("qk", [wl.BF16, wl.FP8_E4M3])
def test_wide_kernel_short_parts_and_positions_outside(qk):
    # 256 query rows per kv head: the wide kernel.  Parts of the key stream shorter than a 64-row tile on either
    # side of the block, blocks that hang over an end of the sequence (their tile list is shorter: with key
    # splits, an empty last split) or lie outside it altogether
    import torch
    for N, B in ((1000, 8), (4096, 8), (191, 8)):
        cfg = wl.custom_config(B=B, H=8, Hkv=2, N=N, d=128, bl=64, qk_dtype=qk, v_dtype=wl.BF16, prompt=0, G=N)
        cache = wl.cache_inputs(cfg, seed=N)
        blk = wl.block_inputs(cfg, N, 0, k_scale=cache["k_scale"])
        starts = np.array([1, N - 64 - 1, -10, N - 30, -64, N, 63, -(2**31)], np.int32)
        got = out_to_f64(run(cfg, cache, blk, starts), wl.BF16)
        ref = oracle.block_attention_batched(blk["Qblk"], cache["Kc"], cache["Vc"], starts, qk, wl.BF16, blk["Kblk"],
                                             blk["Vblk"], blk["q_scale"], cache["k_scale"])
        assert_attention_close(got, ref, qk, f"wide kernel, positions {starts.tolist()} N{N} dtype {qk}")


def test_equal_positions_are_the_plain_call_and_outside_positions_are_safe(monkeypatch):
    import torch
    monkeypatch.setenv("DD_TUNE_BLOCK_WIDE", "0")        # the plain call on the same kernels as the batched one
    cfg = wl.custom_config(B=3, H=4, Hkv=2, N=512, d=128, bl=64, prompt=0, G=512)
    cache = wl.cache_inputs(cfg, seed=1)
    blk = wl.block_inputs(cfg, 0, 0, k_scale=cache["k_scale"])
    O = run(cfg, cache, blk, [192, 192, 192])
    P = dd.dd_block_attention_cached(to_dev(blk["Qblk"]), to_dev(cache["Kc"]), to_dev(cache["Vc"]), 192,
                                     Kblk=to_dev(blk["Kblk"]), Vblk=to_dev(blk["Vblk"]))
    assert torch.equal(O, P)
    # blocks that hang over the ends of the sequence or lie far outside: no fault, the oracle's result
    starts = np.array([-10, 500, 2**31 - 1], np.int32)
    got = out_to_f64(run(cfg, cache, blk, starts), wl.BF16)
    ref = oracle.block_attention_batched(blk["Qblk"], cache["Kc"], cache["Vc"], starts, wl.BF16, wl.BF16, blk["Kblk"],
                                         blk["Vblk"])
    assert_attention_close(got, ref, wl.BF16, "positions outside the sequence")
    starts = np.array([-(2**31), -64, 512], np.int32)
    got = out_to_f64(run(cfg, cache, blk, starts), wl.BF16)
    ref = oracle.block_attention_batched(blk["Qblk"], cache["Kc"], cache["Vc"], starts, wl.BF16, wl.BF16, blk["Kblk"],
                                         blk["Vblk"])
    assert_attention_close(got, ref, wl.BF16, "positions far outside the sequence")
