"""Seeded random shapes of the attention entry points against the CPU oracle, on every kernel that can serve them.
The fixed shape lists of the other files aim at known boundaries; these cases cover combinations nobody thought of
(a sweep of this kind found the four-stores-per-wave case of the wide kernel's 128-row tiles at d = 64)."""
import numpy as np
import pytest

import oracle
import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from _util import out_to_f64, to_dev

pytestmark = pytest.mark.gpu
HOOKS = ("DD_TUNE_ATTN_WIDE", "DD_TUNE_ATTN_WIDE_GRID", "DD_TUNE_BIDIR_STREAM", "DD_TUNE_BLOCK_WIDE", "DD_TUNE_BLOCK_STREAM",
         "DD_TUNE_BLOCK_WIDE_ROWS")
TOL = {wl.BF16: (2e-2, 5e-3), wl.FP8_E4M3: (6e-2, 5e-3), wl.F32: (1e-4, 1e-5)}


def close(got, ref, qk, what):
    mx = np.abs(got - ref).max()
    rl = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    assert np.isfinite(got).all() and mx <= TOL[qk][0] and rl <= TOL[qk][1], f"{what}: max-abs {mx:.3e} rel-L2 {rl:.3e}"


def set_hooks(monkeypatch, env):
    for k in HOOKS:
        monkeypatch.delenv(k, raising=False)
    for k, v in env.items():
        monkeypatch.setenv(k, v)


@pytest.mark.parametrize("seed", range(6))
def test_random_verifier_calls(monkeypatch, seed):
    import torch
    rng = np.random.default_rng(1000 + seed)
    for it in range(10):
        d = int(rng.choice([64, 128]))
        qk = wl.FP8_E4M3 if rng.random() < 0.35 else wl.BF16
        Hkv, G = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        N = int(rng.choice([rng.integers(1, 70), rng.integers(64, 400), rng.integers(400, 1300)]))
        B = int(rng.integers(1, 3))
        kern = str(rng.choice(["auto", "wide", "stream", "mfma"]))
        env = {"wide": {"DD_TUNE_ATTN_WIDE": "1"}, "stream": {"DD_TUNE_ATTN_WIDE": "0", "DD_TUNE_BIDIR_STREAM": "1"},
               "mfma": {"DD_TUNE_ATTN_WIDE": "0", "DD_TUNE_BIDIR_STREAM": "0"}, "auto": {}}[kern]
        if kern == "wide" and rng.random() < 0.5:
            env = dict(env, DD_TUNE_ATTN_WIDE_GRID=str(int(rng.integers(1, 4))))
        set_hooks(monkeypatch, env)
        cfg = wl.custom_config(B=B, H=Hkv * G, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=wl.BF16, prompt=0, G=N, bl=min(16, N))
        inp = wl.attention_inputs(cfg, 100 * seed + it)
        O = dd.dd_bidir_attention(to_dev(inp["Q"]), to_dev(inp["K"]), to_dev(inp["V"]), q_scale=to_dev(inp["q_scale"]),
                                  k_scale=to_dev(inp["k_scale"]), qk_dtype=qk, v_dtype=wl.BF16)
        torch.cuda.synchronize()
        ref = oracle.bidir_attention(inp["Q"], inp["K"], inp["V"], qk, wl.BF16, inp["q_scale"], inp["k_scale"])
        close(out_to_f64(O, wl.BF16), ref, qk, f"bidir B{B} H{Hkv * G}/{Hkv} N{N} d{d} dtype {qk} {env}")


@pytest.mark.parametrize("seed", range(8))
def test_random_drafter_calls(monkeypatch, seed):
    import torch
    rng = np.random.default_rng(2000 + seed)
    for it in range(10):
        d = int(rng.choice([64, 128]))
        r = rng.random()
        qk = wl.FP8_E4M3 if r < 0.3 else wl.F32 if r < 0.38 else wl.BF16
        vd = wl.F32 if qk == wl.F32 else wl.BF16
        Hkv, G = int(rng.integers(1, 4)), int(rng.integers(1, 6))
        bl = int(rng.choice([1, 16, 32, 33, 40, 48, 64, 64, 80, 96, 128]))
        N = int(rng.choice([rng.integers(bl, bl + 70), rng.integers(bl + 64, 500), rng.integers(500, 1400)]))
        if qk == wl.F32:
            N = min(N, 300)
        B = int(rng.integers(1, 4))
        bs = int(rng.integers(0, N - bl + 1))
        c = rng.random()
        env = ({"DD_TUNE_BLOCK_WIDE": "0"} if c < 0.15 else {"DD_TUNE_BLOCK_STREAM": "0"} if c < 0.3 else
               {"DD_TUNE_BLOCK_WIDE_ROWS": str(rng.choice(["128", "256"]))} if c < 0.6 else {})
        set_hooks(monkeypatch, env)
        cfg = wl.custom_config(B=B, H=Hkv * G, Hkv=Hkv, N=N, d=d, qk_dtype=qk, v_dtype=vd, bl=bl, prompt=0, G=N)
        cache = wl.cache_inputs(cfg, seed=100 * seed + it)
        blk = wl.block_inputs(cfg, bs, 0, k_scale=cache["k_scale"])
        Q, Kc, Vc = to_dev(blk["Qblk"]), to_dev(cache["Kc"]), to_dev(cache["Vc"])
        qs, ks = to_dev(blk["q_scale"]), to_dev(cache["k_scale"])
        entry = str(rng.choice(["cached", "cached", "window", "batched"]))
        what = f"{entry} B{B} H{Hkv * G}/{Hkv} N{N} d{d} bl{bl}@{bs} dtype {qk} {env}"
        if entry == "cached":
            fresh = bool(rng.random() < 0.6)
            Kb, Vb = (blk["Kblk"], blk["Vblk"]) if fresh else (None, None)
            O = dd.dd_block_attention_cached(Q, Kc, Vc, bs, Kblk=to_dev(Kb), Vblk=to_dev(Vb), q_scale=qs, k_scale=ks,
                                             qk_dtype=qk, v_dtype=vd)
            ref = oracle.block_attention_cached(blk["Qblk"], cache["Kc"], cache["Vc"], bs, qk, vd, Kb, Vb, blk["q_scale"],
                                                cache["k_scale"])
        elif entry == "window":
            w0, wend = int(rng.integers(0, bs + 1)), int(rng.integers(bs + bl, N + 1))
            O = dd.dd_block_attention_window(Q, Kc, Vc, bs, w0, wend - w0, Kblk=to_dev(blk["Kblk"]), Vblk=to_dev(blk["Vblk"]),
                                             q_scale=qs, k_scale=ks, qk_dtype=qk, v_dtype=vd)
            ref = oracle.block_attention_window(blk["Qblk"], cache["Kc"], cache["Vc"], bs, w0, wend - w0, qk, vd, blk["Kblk"],
                                                blk["Vblk"], blk["q_scale"], cache["k_scale"])
            what += f" window [{w0}, {wend})"
        else:
            starts = rng.integers(-bl, N + 1, B).astype(np.int32)         # positions outside the sequence included
            O = dd.dd_block_attention_batched(Q, Kc, Vc, torch.from_numpy(starts).to("cuda:0"), to_dev(blk["Kblk"]),
                                              to_dev(blk["Vblk"]), q_scale=qs, k_scale=ks, qk_dtype=qk, v_dtype=vd)
            ref = oracle.block_attention_batched(blk["Qblk"], cache["Kc"], cache["Vc"], starts, qk, vd, blk["Kblk"],
                                                 blk["Vblk"], blk["q_scale"], cache["k_scale"])
            what += f" starts {starts.tolist()}"
        torch.cuda.synchronize()
        close(out_to_f64(O, vd), ref, qk, what)
