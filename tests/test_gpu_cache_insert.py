"""GPU parity of dd_cache_insert_rows (token-granular cache update) against the oracle: byte-exact."""
import numpy as np
import pytest

import oracle
import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from _util import out_to_f64, to_dev, assert_attention_close

pytestmark = pytest.mark.gpu


def raw(t):
    import torch
    return t.contiguous().view(torch.uint8).cpu().numpy()


@pytest.mark.parametrize("B,Hkv,N,d,n,qk", [(2, 2, 333, 128, 7, wl.BF16), (1, 8, 2048, 128, 64, wl.FP8_E4M3),
                                             (3, 1, 100, 64, 100, wl.BF16), (2, 4, 128, 64, 16, wl.F32),
                                             (4, 2, 1000, 128, 1, wl.FP8_E4M3), (16, 8, 2048, 128, 33, wl.BF16)])
def test_insert_rows_matches_oracle(B, Hkv, N, d, n, qk):
    import torch
    vd = wl.F32 if qk == wl.F32 else wl.BF16
    cfg = wl.custom_config(B=B, H=Hkv, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=vd, bl=n, prompt=0, G=N)
    cache = wl.cache_inputs(cfg, seed=N + n)
    blk = wl.block_inputs(cfg, 0, 0, k_scale=cache["k_scale"])          # n fresh rows per (batch, kv head)
    rng = np.random.default_rng(N * 7 + n)
    pos = np.stack([rng.permutation(N)[:n] for _ in range(B)]).astype(np.int32)      # distinct per batch entry
    if n >= 4:                                                          # entries that must be skipped
        pos[0, 1] = -1
        pos[B - 1, 2] = N
        pos[0, 3] = 2**31 - 1
    Kc, Vc = to_dev(cache["Kc"]), to_dev(cache["Vc"])
    dd.dd_cache_insert_rows(Kc, Vc, to_dev(blk["Kblk"]), to_dev(blk["Vblk"]), torch.from_numpy(pos).to("cuda:0"),
                            qk_dtype=qk, v_dtype=vd)
    torch.cuda.synchronize()
    Kn, Vn = oracle.cache_insert_rows(cache["Kc"], cache["Vc"], blk["Kblk"], blk["Vblk"], pos)
    assert np.array_equal(raw(Kc), np.ascontiguousarray(Kn).view(np.uint8))
    assert np.array_equal(raw(Vc), np.ascontiguousarray(Vn).view(np.uint8))


def test_delayed_insertion_then_window_attention():
    # the dKV-Cache pair: last step's rows enter the cache one step late, then the block attends over a local window
    import torch
    cfg = wl.custom_config(B=2, H=8, Hkv=2, N=1024, d=128, bl=32, prompt=0, G=1024)
    cache = wl.cache_inputs(cfg, seed=2)
    prev = wl.block_inputs(cfg, 5, 0, k_scale=cache["k_scale"])         # rows "decoded at the previous step"
    cur = wl.block_inputs(cfg, 6, 1, k_scale=cache["k_scale"])
    bs, w0, wlen = 512, 384, 320
    pos = np.stack([np.arange(400, 400 + 2 * cfg.bl, 2), np.arange(bs - cfg.bl, bs)]).astype(np.int32)
    Kc, Vc = to_dev(cache["Kc"]), to_dev(cache["Vc"])
    dd.dd_cache_insert_rows(Kc, Vc, to_dev(prev["Kblk"]), to_dev(prev["Vblk"]), torch.from_numpy(pos).to("cuda:0"))
    O = dd.dd_block_attention_window(to_dev(cur["Qblk"]), Kc, Vc, bs, w0, wlen, Kblk=to_dev(cur["Kblk"]),
                                     Vblk=to_dev(cur["Vblk"]))
    torch.cuda.synchronize()
    Kn, Vn = oracle.cache_insert_rows(cache["Kc"], cache["Vc"], prev["Kblk"], prev["Vblk"], pos)
    ref = oracle.block_attention_window(cur["Qblk"], Kn, Vn, bs, w0, wlen, wl.BF16, wl.BF16, cur["Kblk"], cur["Vblk"])
    assert_attention_close(out_to_f64(O, wl.BF16), ref, wl.BF16, "insert + window")
