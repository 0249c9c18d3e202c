"""GPU parity of dd_bidir_attention and dd_block_attention_cached against the CPU oracle."""
import numpy as np
import pytest

import oracle
import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from _util import ATTN_TOL, assert_attention_close, attn_errors, out_to_f64, to_dev

pytestmark = pytest.mark.gpu


def gpu_bidir(inp, cfg):
    import torch
    O = dd.dd_bidir_attention(to_dev(inp["Q"]), to_dev(inp["K"]), to_dev(inp["V"]),
                              q_scale=to_dev(inp["q_scale"]), k_scale=to_dev(inp["k_scale"]),
                              qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
    torch.cuda.synchronize()
    return out_to_f64(O, cfg.v_dtype)


def gpu_block(cfg, Qblk, Kc, Vc, bs, Kblk=None, Vblk=None, q_scale=None, k_scale=None):
    import torch
    O = dd.dd_block_attention_cached(to_dev(Qblk), to_dev(Kc), to_dev(Vc), bs, Kblk=to_dev(Kblk), Vblk=to_dev(Vblk),
                                     q_scale=to_dev(q_scale), k_scale=to_dev(k_scale),
                                     qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
    torch.cuda.synchronize()
    return out_to_f64(O, cfg.v_dtype)


def sample_rows(rng, B, H, Nq, n):
    """(b, h, i) rows: corners, tile boundaries and random positions."""
    fixed = [(0, 0, 0), (B - 1, H - 1, Nq - 1), (0, H - 1, min(127, Nq - 1)), (B - 1, 0, min(128, Nq - 1)),
             (0, 0, Nq // 2), (B // 2, H // 2, min(31, Nq - 1)), (B // 2, H // 2, min(32, Nq - 1))]
    rnd = list(zip(rng.integers(0, B, n).tolist(), rng.integers(0, H, n).tolist(), rng.integers(0, Nq, n).tolist()))
    return sorted(set(fixed + rnd))


# ------------------------------------------------------------------ full attention
def test_cfg1_fp32_full():
    cfg = wl.CONFIGS[1]
    inp = wl.attention_inputs(cfg, 0)
    got = gpu_bidir(inp, cfg)
    ref = oracle.bidir_attention(inp["Q"], inp["K"], inp["V"], cfg.qk_dtype, cfg.v_dtype)
    assert_attention_close(got, ref, cfg.qk_dtype, "cfg1 bidir")


SMALL = [
    # (B, H, Hkv, N, d, qk_dtype): ragged N, one wave / partial tiles, GQA, both head dims
    (1, 2, 2, 1, 64, wl.BF16), (1, 2, 2, 33, 128, wl.BF16), (2, 4, 2, 200, 128, wl.BF16), (1, 3, 1, 77, 64, wl.BF16),
    (1, 2, 2, 320, 64, wl.BF16), (2, 8, 2, 130, 128, wl.FP8_E4M3), (1, 4, 4, 96, 64, wl.FP8_E4M3),
    (1, 2, 1, 257, 128, wl.F32), (2, 4, 4, 50, 64, wl.F32), (1, 1, 1, 640, 128, wl.BF16),
]


# A bf16 call that is too small for the wide kernel goes to the streaming kernel (64-row workgroups) when it
# would leave compute units idle, else to the MFMA kernel with 128-row workgroups; DD_TUNE_BIDIR_STREAM forces it.
@pytest.mark.parametrize("stream", ["0", "1"])
@pytest.mark.parametrize("B,H,Hkv,N,d,qk", SMALL)
def test_bidir_small_shapes(monkeypatch, B, H, Hkv, N, d, qk, stream):
    if qk != wl.BF16 and stream == "1":
        pytest.skip("only bf16 calls have the choice")
    monkeypatch.setenv("DD_TUNE_ATTN_WIDE", "0")
    monkeypatch.setenv("DD_TUNE_BIDIR_STREAM", stream)
    vd = wl.F32 if qk == wl.F32 else wl.BF16
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=vd, prompt=0, G=N, bl=min(16, N))
    inp = wl.attention_inputs(cfg, seed=N)
    got = gpu_bidir(inp, cfg)
    ref = oracle.bidir_attention(inp["Q"], inp["K"], inp["V"], qk, vd, inp["q_scale"], inp["k_scale"])
    assert_attention_close(got, ref, qk, f"bidir {B}x{H}/{Hkv}x{N}x{d} dtype {qk}")


def test_bidir_closed_forms_on_gpu():
    # identical keys -> mean(V); a dominant key -> that V row; both readings of the cfg2 input scale
    cfg = wl.custom_config(B=1, H=2, Hkv=2, N=192, d=128, prompt=0, G=192)
    inp = wl.attention_inputs(cfg, 1)
    K1 = np.broadcast_to(inp["K"][:, :, :1], inp["K"].shape).copy()
    got = gpu_bidir(dict(inp, K=K1), cfg)
    meanV = wl.bf16_bits_to_f32(inp["V"]).astype(np.float64).mean(axis=2, keepdims=True)
    assert np.abs(got - meanV).max() < 2e-3
    small = wl.custom_config(B=1, H=2, Hkv=2, N=192, d=128, prompt=0, G=192, qk_prescale=1.0 / np.sqrt(128.0))
    inp2 = wl.attention_inputs(small, 1)
    got2 = gpu_bidir(inp2, small)
    ref2 = oracle.bidir_attention(inp2["Q"], inp2["K"], inp2["V"], wl.BF16, wl.BF16)
    assert_attention_close(got2, ref2, wl.BF16, "prescaled inputs")
    assert np.abs(got2 - wl.bf16_bits_to_f32(inp2["V"]).astype(np.float64).mean(axis=2, keepdims=True)).max() < 0.05


def test_bidir_is_deterministic():
    cfg = wl.custom_config(B=2, H=4, Hkv=4, N=300, d=128, prompt=0, G=300)
    inp = wl.attention_inputs(cfg, 4)
    assert np.array_equal(gpu_bidir(inp, cfg), gpu_bidir(inp, cfg))


import functools


@functools.lru_cache(maxsize=None)
def _cfg_inputs(cfg_id):
    return wl.attention_inputs(wl.CONFIGS[cfg_id], 0)


def stratified_rows(cfg, seed):
    """One query row out of every 32-row block of every (batch, kv head): the rows of a kv head's query heads form
    one run of group * N rows that the kernels cut into 256-row tiles, 64-row waves and 32-row blocks, so every
    (batch, kv head, row tile, wave, block) of the launch is compared; the row inside its block is drawn."""
    rng = np.random.default_rng(seed)
    group, per = cfg.H // cfg.Hkv, (cfg.H // cfg.Hkv) * cfg.N
    rows = []
    for b in range(cfg.B):
        for g in range(cfg.Hkv):
            starts = np.arange(0, per, 32)
            v = np.minimum(starts + rng.integers(0, 32, len(starts)), per - 1)
            rows += [(b, g * group + int(x) // cfg.N, int(x) % cfg.N) for x in v]
    return rows


@functools.lru_cache(maxsize=None)
def _bidir_reference(cfg_id):
    """The oracle's result for a benchmark configuration, computed once per test session: every row for
    cfg1-cfg4; for cfg5 (a million rows) the stratified sample."""
    cfg, inp = wl.CONFIGS[cfg_id], _cfg_inputs(cfg_id)
    rows = stratified_rows(cfg, cfg_id) if cfg_id == 5 else None
    ref = oracle.bidir_attention(inp["Q"], inp["K"], inp["V"], cfg.qk_dtype, cfg.v_dtype, inp["q_scale"], inp["k_scale"],
                                 rows=rows)
    return rows, ref


def _bidir_full_size(cfg_id):
    cfg, inp = wl.CONFIGS[cfg_id], _cfg_inputs(cfg_id)
    got = gpu_bidir(inp, cfg)
    assert np.isfinite(got).all()
    rows, ref = _bidir_reference(cfg_id)
    if rows is None:
        assert_attention_close(got, ref, cfg.qk_dtype, f"cfg{cfg_id} bidir (all rows)")
        # the tolerances also hold head by head, not only over the whole tensor
        d = got - ref
        rl = np.sqrt((d ** 2).sum(axis=(2, 3)) / (ref ** 2).sum(axis=(2, 3)))
        assert rl.max() <= ATTN_TOL[cfg.qk_dtype][1], f"cfg{cfg_id}: worst head rel-L2 {rl.max():.3e}"
    else:
        idx = np.asarray(rows)
        sel = got[idx[:, 0], idx[:, 1], idx[:, 2]]
        assert_attention_close(sel, ref, cfg.qk_dtype, f"cfg{cfg_id} bidir ({len(rows)} stratified rows)")


def test_cfg2_bidir_full_size():
    _bidir_full_size(2)


def test_cfg3_bidir_full_size():
    _bidir_full_size(3)


def test_cfg4_bidir_full_size():
    _bidir_full_size(4)


def test_cfg5_bidir_full_size():
    _bidir_full_size(5)


# The bf16 verifier call has two kernels (128-row workgroups with two waves per SIMD; 256-row workgroups with
# one 64-row wave per SIMD); the library picks by problem size and DD_TUNE_ATTN_WIDE forces the choice.
WIDE = [
    # (B, H, Hkv, N, d): the smallest N the wide kernel takes (one 64-key tile; shorter calls stay on the
    # other kernel, which the first two shapes check), last tiles that overlap the one before by 1 .. 63 keys,
    # odd tile counts, GQA groups that straddle 256-row tiles, idle waves
    (1, 1, 1, 1, 128), (1, 2, 2, 33, 64), (1, 2, 1, 64, 128), (1, 2, 1, 65, 128), (1, 4, 2, 100, 64),
    (1, 2, 1, 127, 64), (1, 2, 1, 191, 128), (1, 2, 1, 193, 128), (2, 4, 2, 200, 128), (1, 4, 1, 257, 64),
    (1, 2, 2, 1000, 128), (1, 3, 1, 130, 64), (1, 8, 2, 200, 128), (2, 6, 6, 300, 128), (1, 12, 4, 70, 64),
]


# The wide kernel's workgroups are persistent: each walks through a contiguous range of 256-row tiles.
# DD_TUNE_ATTN_WIDE_GRID caps the number of workgroups, so that small shapes also exercise the hand-over
# from one row tile to the next (and ranges of unequal length).
@pytest.mark.parametrize("grid", [None, "1", "3"])
@pytest.mark.parametrize("B,H,Hkv,N,d", WIDE)
def test_bidir_wide_kernel_small_shapes(monkeypatch, B, H, Hkv, N, d, grid):
    monkeypatch.setenv("DD_TUNE_ATTN_WIDE", "1")
    if grid is not None:
        if B * Hkv * -(-(H // Hkv) * N // 256) <= int(grid):
            pytest.skip("no more row tiles than workgroups: same launch as the uncapped case")
        monkeypatch.setenv("DD_TUNE_ATTN_WIDE_GRID", grid)
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, prompt=0, G=N, bl=min(16, N))
    inp = wl.attention_inputs(cfg, seed=N + d)
    got = gpu_bidir(inp, cfg)
    ref = oracle.bidir_attention(inp["Q"], inp["K"], inp["V"], wl.BF16, wl.BF16, inp["q_scale"], inp["k_scale"])
    assert_attention_close(got, ref, wl.BF16, f"wide kernel {B}x{H}/{Hkv}x{N}x{d}")


WIDE_FP8 = [
    # (B, H, Hkv, N): fp8 Q/K with per-head scales, d = 128; GQA, overlapping last tiles, several row tiles
    (1, 2, 1, 64), (1, 4, 2, 100), (2, 8, 2, 130), (1, 4, 1, 257), (1, 2, 2, 1000), (1, 16, 2, 320),
]


@pytest.mark.parametrize("grid", [None, "2"])
@pytest.mark.parametrize("B,H,Hkv,N", WIDE_FP8)
def test_bidir_wide_kernel_fp8(monkeypatch, B, H, Hkv, N, grid):
    monkeypatch.setenv("DD_TUNE_ATTN_WIDE", "1")
    if grid is not None:
        if B * Hkv * -(-(H // Hkv) * N // 256) <= int(grid):
            pytest.skip("no more row tiles than workgroups: same launch as the uncapped case")
        monkeypatch.setenv("DD_TUNE_ATTN_WIDE_GRID", grid)
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=128, qk_dtype=wl.FP8_E4M3, v_dtype=wl.BF16, prompt=0, G=N,
                           bl=min(16, N))
    inp = wl.attention_inputs(cfg, seed=N)
    got = gpu_bidir(inp, cfg)
    ref = oracle.bidir_attention(inp["Q"], inp["K"], inp["V"], wl.FP8_E4M3, wl.BF16, inp["q_scale"], inp["k_scale"])
    assert_attention_close(got, ref, wl.FP8_E4M3, f"wide kernel fp8 {B}x{H}/{Hkv}x{N}")


def test_bidir_wide_kernel_scales_change_between_row_tiles(monkeypatch):
    # one workgroup walks through the row tiles of four heads, each with its own score scale
    monkeypatch.setenv("DD_TUNE_ATTN_WIDE", "1")
    monkeypatch.setenv("DD_TUNE_ATTN_WIDE_GRID", "1")
    cfg = wl.custom_config(B=1, H=4, Hkv=2, N=256, d=128, prompt=0, G=256)
    inp = wl.attention_inputs(cfg, seed=11)
    rng = np.random.default_rng(5)
    inp["q_scale"] = rng.uniform(0.4, 2.5, size=cfg.B * cfg.H).astype(np.float32)
    inp["k_scale"] = rng.uniform(0.4, 2.5, size=cfg.B * cfg.Hkv).astype(np.float32)
    got = gpu_bidir(inp, cfg)
    ref = oracle.bidir_attention(inp["Q"], inp["K"], inp["V"], wl.BF16, wl.BF16, inp["q_scale"], inp["k_scale"])
    assert_attention_close(got, ref, wl.BF16, "wide kernel, per-head scales")


@pytest.mark.parametrize("wide", ["0", "1"])
def test_cfg5_bidir_each_kernel(monkeypatch, wide):
    monkeypatch.setenv("DD_TUNE_ATTN_WIDE", wide)
    _bidir_full_size(5)


@pytest.mark.parametrize("wide,stream", [("1", "0"), ("0", "0"), ("0", "1")])
def test_cfg3_bidir_each_kernel(monkeypatch, wide, stream):
    monkeypatch.setenv("DD_TUNE_ATTN_WIDE", wide)
    monkeypatch.setenv("DD_TUNE_BIDIR_STREAM", stream)
    _bidir_full_size(3)


@pytest.mark.parametrize("wide,stream", [("1", "0"), ("0", "0"), ("0", "1")])
def test_cfg2_bidir_each_kernel(monkeypatch, wide, stream):
    monkeypatch.setenv("DD_TUNE_ATTN_WIDE", wide)
    monkeypatch.setenv("DD_TUNE_BIDIR_STREAM", stream)
    _bidir_full_size(2)


@pytest.mark.parametrize("wide", ["0", "1"])
def test_bidir_long_sequence(monkeypatch, wide):
    # 16384 positions: byte offsets inside one head pass 4 MB, 256 key tiles per pass; sampled rows against the oracle
    monkeypatch.setenv("DD_TUNE_ATTN_WIDE", wide)
    monkeypatch.setenv("DD_TUNE_BIDIR_STREAM", "0")
    cfg = wl.custom_config(B=1, H=4, Hkv=2, N=16384, d=128, prompt=0, G=16384)
    inp = wl.attention_inputs(cfg, seed=21)
    got = gpu_bidir(inp, cfg)
    assert np.isfinite(got).all()
    rows = sample_rows(np.random.default_rng(21), cfg.B, cfg.H, cfg.N, 40)
    ref = oracle.bidir_attention(inp["Q"], inp["K"], inp["V"], wl.BF16, wl.BF16, rows=rows)
    sel = np.stack([got[b, h, i] for b, h, i in rows])
    assert_attention_close(sel, ref, wl.BF16, f"N=16384 bidir wide={wide}")


def test_block_long_cache():
    # 65536 cached positions, the block near the end: the key range is split 16 ways
    cfg = wl.custom_config(B=1, H=4, Hkv=4, N=65536, d=128, bl=64, prompt=0, G=65536)
    cache = wl.cache_inputs(cfg, seed=9)
    bs = 65536 - 64 - 37
    blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
    got = gpu_block(cfg, blk["Qblk"], cache["Kc"], cache["Vc"], bs, blk["Kblk"], blk["Vblk"])
    rows = sample_rows(np.random.default_rng(5), cfg.B, cfg.H, cfg.bl, 24)
    ref = oracle.block_attention_cached(blk["Qblk"], cache["Kc"], cache["Vc"], bs, wl.BF16, wl.BF16, blk["Kblk"], blk["Vblk"],
                                        rows=rows)
    sel = np.stack([got[b, h, i] for b, h, i in rows])
    assert_attention_close(sel, ref, wl.BF16, "N=65536 block")


# ------------------------------------------------------------------ block attention over the cache
def _block_case(cfg, seed, step, full_rows=True, n_rows=256):
    cache = wl.cache_inputs(cfg, seed)
    blk = wl.block_inputs(cfg, seed, step, k_scale=cache["k_scale"])
    bs = blk["block_start"]
    got = gpu_block(cfg, blk["Qblk"], cache["Kc"], cache["Vc"], bs, blk["Kblk"], blk["Vblk"], blk["q_scale"], cache["k_scale"])
    if full_rows:
        ref = oracle.block_attention_cached(blk["Qblk"], cache["Kc"], cache["Vc"], bs, cfg.qk_dtype, cfg.v_dtype,
                                            blk["Kblk"], blk["Vblk"], blk["q_scale"], cache["k_scale"])
        assert_attention_close(got, ref, cfg.qk_dtype, f"{cfg.name} block step {step}")
    else:
        rows = sample_rows(np.random.default_rng(seed + step), cfg.B, cfg.H, cfg.bl, n_rows)
        ref = oracle.block_attention_cached(blk["Qblk"], cache["Kc"], cache["Vc"], bs, cfg.qk_dtype, cfg.v_dtype,
                                            blk["Kblk"], blk["Vblk"], blk["q_scale"], cache["k_scale"], rows=rows)
        sel = np.stack([got[b, h, i] for b, h, i in rows])
        assert_attention_close(sel, ref, cfg.qk_dtype, f"{cfg.name} block step {step} (sampled)")


def test_cfg1_block_all_steps():
    cfg = wl.CONFIGS[1]
    for step in range(cfg.K):
        _block_case(cfg, 0, step)


def test_cfg2_block_all_steps():
    cfg = wl.CONFIGS[2]
    for step in range(cfg.K):
        _block_case(cfg, 0, step)


@pytest.mark.parametrize("cfg_id", [3, 4, 5])
def test_large_block_first_and_last_step(cfg_id):
    cfg = wl.CONFIGS[cfg_id]
    for step in (0, cfg.K - 1):
        _block_case(cfg, 0, step)                             # every row of the call


BLOCK_SMALL = [
    # (B, H, Hkv, N, d, bl, block_start, qk): first / last / unaligned blocks, ragged N, GQA, one query
    (1, 2, 2, 100, 64, 16, 0, wl.BF16), (1, 2, 2, 100, 64, 16, 84, wl.BF16), (2, 4, 2, 333, 128, 32, 101, wl.BF16),
    (1, 8, 2, 1000, 128, 64, 936, wl.FP8_E4M3), (1, 2, 1, 150, 64, 1, 77, wl.BF16), (1, 4, 4, 128, 64, 16, 64, wl.F32),
    (2, 2, 1, 600, 128, 48, 200, wl.F32), (1, 16, 2, 2048, 128, 64, 1024, wl.BF16), (1, 1, 1, 64, 128, 64, 0, wl.BF16),
    # 65 .. 191 query rows per kv head at a benchmark-like size
    (2, 8, 4, 2048, 128, 64, 1024, wl.BF16), (1, 32, 32, 2048, 128, 96, 1000, wl.BF16), (1, 4, 2, 2048, 128, 80, 1900, wl.BF16),
    (1, 8, 4, 2048, 128, 64, 1984, wl.FP8_E4M3),
]


# The bf16 drafter call has two kernels as well: the streaming kernel (up to 64 query rows per kv head) and the
# MFMA kernel with 128-row workgroups; DD_TUNE_BLOCK_STREAM=0 keeps every call on the latter.
STREAM_SHAPES = [
    # (B, H, Hkv, N, d, bl, block_start): one tile, ragged last tile, block at both ends and across tiles,
    # one query, 33 rows (second row block nearly empty), GQA 2 x 32 rows, key splits with a short last split
    (1, 2, 2, 64, 128, 64, 0), (1, 2, 2, 100, 64, 16, 84), (2, 4, 2, 333, 128, 32, 101), (1, 2, 1, 150, 64, 1, 77),
    (1, 3, 3, 500, 128, 33, 467), (1, 4, 2, 700, 128, 32, 60), (1, 2, 2, 4096, 128, 64, 2000), (1, 1, 1, 1090, 64, 64, 1026),
]


@pytest.mark.parametrize("stream", ["1", "0"])
@pytest.mark.parametrize("B,H,Hkv,N,d,bl,bs", STREAM_SHAPES)
def test_block_each_kernel(monkeypatch, stream, B, H, Hkv, N, d, bl, bs):
    monkeypatch.setenv("DD_TUNE_BLOCK_STREAM", stream)
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, bl=bl, prompt=0, G=N)
    cache = wl.cache_inputs(cfg, seed=bs + d)
    blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
    for fresh in (True, False):
        Kb, Vb = (blk["Kblk"], blk["Vblk"]) if fresh else (None, None)
        got = gpu_block(cfg, blk["Qblk"], cache["Kc"], cache["Vc"], bs, Kb, Vb, blk["q_scale"], cache["k_scale"])
        ref = oracle.block_attention_cached(blk["Qblk"], cache["Kc"], cache["Vc"], bs, wl.BF16, wl.BF16, Kb, Vb,
                                            blk["q_scale"], cache["k_scale"])
        assert_attention_close(got, ref, wl.BF16, f"block kernel stream={stream} {B}x{H}/{Hkv} N{N} d{d} bl{bl}@{bs} fresh={fresh}")


# A drafter call with more than 64 query rows per kv head (GQA group x block length) runs on the wide kernel when
# every part of its key stream (cache before the block, block tensors, cache after it) is empty or at least 64
# rows long; DD_TUNE_BLOCK_WIDE=0 keeps it on the other kernels.
WIDE_BLOCK = [
    # (B, H, Hkv, N, d, bl, block_start, qk): block at the start / end / inside, ragged parts (overlapping last
    # tiles), key splits that begin at an overlapping tile (N=321, bs=193), 192 and 320 rows per kv head, fp8, d=64
    (1, 4, 1, 512, 128, 64, 0, wl.BF16), (1, 4, 1, 512, 128, 64, 448, wl.BF16), (2, 8, 2, 640, 128, 64, 200, wl.BF16),
    (1, 3, 1, 300, 128, 64, 100, wl.BF16), (1, 4, 1, 321, 128, 64, 193, wl.BF16), (1, 4, 1, 385, 128, 64, 129, wl.BF16),
    (1, 4, 1, 1000, 128, 80, 700, wl.BF16), (2, 8, 2, 640, 128, 64, 256, wl.FP8_E4M3), (1, 16, 4, 2048, 128, 64, 1536, wl.FP8_E4M3),
    (1, 8, 2, 400, 64, 64, 64, wl.BF16), (1, 4, 1, 4096, 128, 128, 2000, wl.BF16),
    # parts shorter than a tile on either side of the block (1, 63 and 5 rows), block directly at an end
    (1, 4, 1, 512, 128, 64, 1, wl.BF16), (1, 4, 1, 512, 128, 64, 63, wl.BF16), (1, 4, 1, 512, 128, 64, 512 - 64 - 5, wl.BF16),
    (2, 8, 2, 2500, 128, 64, 2500 - 64 - 1, wl.BF16), (1, 16, 4, 700, 128, 64, 33, wl.FP8_E4M3), (1, 4, 1, 129, 128, 64, 64, wl.BF16),
]


@pytest.mark.parametrize("wide", ["1", "0"])
@pytest.mark.parametrize("B,H,Hkv,N,d,bl,bs,qk", WIDE_BLOCK)
def test_block_many_rows_each_kernel(monkeypatch, wide, B, H, Hkv, N, d, bl, bs, qk):
    monkeypatch.setenv("DD_TUNE_BLOCK_WIDE", wide)
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=wl.BF16, bl=bl, prompt=0, G=N)
    cache = wl.cache_inputs(cfg, seed=bs + N)
    blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
    for fresh in (True, False):
        Kb, Vb = (blk["Kblk"], blk["Vblk"]) if fresh else (None, None)
        got = gpu_block(cfg, blk["Qblk"], cache["Kc"], cache["Vc"], bs, Kb, Vb, blk["q_scale"], cache["k_scale"])
        ref = oracle.block_attention_cached(blk["Qblk"], cache["Kc"], cache["Vc"], bs, qk, wl.BF16, Kb, Vb,
                                            blk["q_scale"], cache["k_scale"])
        assert_attention_close(got, ref, qk, f"block wide={wide} {B}x{H}/{Hkv} N{N} d{d} bl{bl}@{bs} dtype {qk} fresh={fresh}")


# The wide kernel's drafter form has a second row tile, 128 rows per workgroup (one 32-row block per wave), taken
# where a kv head has no more rows than that or where it spares the call its key splits (cfg5: 256 workgroups
# instead of 128 x 2 splits).  DD_TUNE_BLOCK_WIDE_ROWS forces the tile on every shape: 66, 96, 128 and 160 rows per
# kv head at N = 2048 among them.
NARROW_BLOCK = WIDE_BLOCK + [
    (2, 8, 4, 2048, 128, 64, 1024, wl.BF16), (1, 32, 32, 2048, 128, 96, 1000, wl.BF16), (1, 4, 2, 2048, 128, 80, 1900, wl.BF16),
    (1, 8, 4, 2048, 128, 64, 1984, wl.FP8_E4M3), (1, 4, 2, 300, 64, 64, 130, wl.BF16), (3, 2, 1, 777, 128, 33, 700, wl.BF16),
    (16, 8, 2, 1024, 128, 64, 512, wl.FP8_E4M3),            # 32 kv heads x 256 rows: the tile is chosen, not forced
    # d = 64: a wave's 32 output rows are four stores, not eight (320 rows per kv head: two whole tiles and half a one)
    (3, 10, 2, 221, 64, 64, 61, wl.BF16), (3, 4, 1, 115, 64, 80, 2, wl.BF16), (1, 5, 1, 512, 64, 64, 64, wl.BF16),
]


@pytest.mark.parametrize("B,H,Hkv,N,d,bl,bs,qk", NARROW_BLOCK)
def test_block_128_row_tiles(monkeypatch, B, H, Hkv, N, d, bl, bs, qk):
    monkeypatch.setenv("DD_TUNE_BLOCK_WIDE", "1")
    if B < 16:
        monkeypatch.setenv("DD_TUNE_BLOCK_WIDE_ROWS", "128")
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=wl.BF16, bl=bl, prompt=0, G=N)
    cache = wl.cache_inputs(cfg, seed=bs + N + 1)
    blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
    for fresh in (True, False):
        Kb, Vb = (blk["Kblk"], blk["Vblk"]) if fresh else (None, None)
        got = gpu_block(cfg, blk["Qblk"], cache["Kc"], cache["Vc"], bs, Kb, Vb, blk["q_scale"], cache["k_scale"])
        ref = oracle.block_attention_cached(blk["Qblk"], cache["Kc"], cache["Vc"], bs, qk, wl.BF16, Kb, Vb,
                                            blk["q_scale"], cache["k_scale"])
        assert_attention_close(got, ref, qk, f"block 128-row tiles {B}x{H}/{Hkv} N{N} d{d} bl{bl}@{bs} dtype {qk} fresh={fresh}")


# DD_TUNE_BLOCK_SPLITS sets the number of key splits of the streaming / MFMA kernels against the library's own rule
# (it keeps at least 128 keys per split): odd counts, short last splits, a split that is nothing but block rows.
@pytest.mark.parametrize("stream", ["1", "0"])
@pytest.mark.parametrize("splits", ["2", "3", "5", "7", "16"])
def test_block_forced_key_splits(monkeypatch, stream, splits):
    monkeypatch.setenv("DD_TUNE_BLOCK_STREAM", stream)
    monkeypatch.setenv("DD_TUNE_BLOCK_WIDE", "0")
    monkeypatch.setenv("DD_TUNE_BLOCK_SPLITS", splits)
    for (B, H, Hkv, N, d, bl, bs, qk) in ((1, 2, 2, 1000, 128, 64, 500, wl.BF16), (2, 4, 2, 777, 64, 32, 745, wl.BF16),
                                          (1, 4, 2, 2049, 128, 48, 128, wl.FP8_E4M3), (1, 2, 1, 900, 128, 16, 0, wl.F32)):
        vd = wl.F32 if qk == wl.F32 else wl.BF16
        cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=vd, bl=bl, prompt=0, G=N)
        cache = wl.cache_inputs(cfg, seed=N)
        blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
        got = gpu_block(cfg, blk["Qblk"], cache["Kc"], cache["Vc"], bs, blk["Kblk"], blk["Vblk"], blk["q_scale"], cache["k_scale"])
        ref = oracle.block_attention_cached(blk["Qblk"], cache["Kc"], cache["Vc"], bs, qk, vd, blk["Kblk"], blk["Vblk"],
                                            blk["q_scale"], cache["k_scale"])
        assert_attention_close(got, ref, qk, f"block, {splits} key splits, stream={stream} {B}x{H}/{Hkv} N{N} d{d} bl{bl}@{bs} dtype {qk}")


@pytest.mark.parametrize("B,H,Hkv,N,d,bl,bs,qk", BLOCK_SMALL)
def test_block_small_shapes(B, H, Hkv, N, d, bl, bs, qk):
    vd = wl.F32 if qk == wl.F32 else wl.BF16
    cfg = wl.custom_config(B=B, H=H, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=vd, bl=bl, prompt=0, G=N)
    cache = wl.cache_inputs(cfg, seed=bs)
    blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
    for fresh in (True, False):
        Kb, Vb = (blk["Kblk"], blk["Vblk"]) if fresh else (None, None)
        got = gpu_block(cfg, blk["Qblk"], cache["Kc"], cache["Vc"], bs, Kb, Vb, blk["q_scale"], cache["k_scale"])
        ref = oracle.block_attention_cached(blk["Qblk"], cache["Kc"], cache["Vc"], bs, qk, vd, Kb, Vb,
                                            blk["q_scale"], cache["k_scale"])
        assert_attention_close(got, ref, qk, f"block {B}x{H}/{Hkv} N{N} d{d} bl{bl}@{bs} fresh={fresh}")


def test_block_equals_rows_of_full_attention_when_cache_is_current():
    cfg = wl.custom_config(B=2, H=4, Hkv=2, N=512, d=128, bl=64, prompt=256, G=256)
    inp = wl.attention_inputs(cfg, 6)
    full = gpu_bidir(inp, cfg)
    for bs in (0, 256, 448):
        Qblk = np.ascontiguousarray(inp["Q"][:, :, bs:bs + cfg.bl])
        got = gpu_block(cfg, Qblk, inp["K"], inp["V"], bs)
        mx, rl = attn_errors(got, full[:, :, bs:bs + cfg.bl])
        assert mx <= 2e-2 and rl <= 5e-3, (bs, mx, rl)       # two tilings of the same sum: equal up to bf16 rounding
        ref = oracle.block_attention_cached(Qblk, inp["K"], inp["V"], bs, wl.BF16, wl.BF16)
        assert_attention_close(got, ref, wl.BF16, f"block@{bs} vs oracle")


def test_errors_raise_through_the_binding():
    import torch
    q = torch.zeros((1, 2, 16, 64), dtype=torch.bfloat16, device="cuda:0")
    kv = torch.zeros((1, 2, 64, 64), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(dd.DDError):
        dd.dd_block_attention_cached(q, kv, kv, 60)           # block runs past N
    q96 = torch.zeros((1, 2, 16, 96), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(dd.DDError):
        dd.dd_bidir_attention(q96, q96, q96)
