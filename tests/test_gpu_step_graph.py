"""One draft-then-verify cycle recorded as a HIP graph gives, on every replay, what the eager calls give."""
import numpy as np
import pytest

import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from paper_2604_05250_amd.step import capture_step
from _util import to_dev

pytestmark = pytest.mark.gpu


def test_step_graph_replays_match_eager_calls():
    import torch
    cfg = wl.custom_config(B=2, H=4, Hkv=2, N=320, d=128, prompt=192, G=128, bl=32, K=4, V=4096, logit_dtype=wl.BF16,
                           sigma_d=3.0, sigma_n=1.0, decoded_frac=0.5)
    att, cache, ver = wl.attention_inputs(cfg, 3), wl.cache_inputs(cfg, 3), wl.verify_inputs(cfg, 3)
    blocks = [wl.block_inputs(cfg, 3, k, k_scale=cache["k_scale"]) for k in range(cfg.K)]
    Q, K, V = (to_dev(att[n]) for n in "QKV")
    Kc, Vc = to_dev(cache["Kc"]), to_dev(cache["Vc"])
    ld, lv, mask = to_dev(ver["logits_d"]), to_dev(ver["logits_v"]), to_dev(ver["mask"])
    blk = [{n: to_dev(b[n]) for n in ("Qblk", "Kblk", "Vblk")} | {"bs": b["block_start"]} for b in blocks]
    O = torch.zeros((cfg.B, cfg.H, cfg.N, cfg.d), dtype=torch.int16, device="cuda")
    Ob = [torch.zeros((cfg.B, cfg.H, cfg.bl, cfg.d), dtype=torch.int16, device="cuda") for _ in blk]
    om = torch.zeros(cfg.P, dtype=torch.uint8, device="cuda")
    ot = torch.zeros(cfg.P, dtype=torch.int32, device="cuda")
    osc = torch.zeros(cfg.P, dtype=torch.float32, device="cuda")
    outs = [O, om, ot, osc] + Ob

    def step():
        for b, o in zip(blk, Ob):
            dd.dd_block_attention_cached(b["Qblk"], Kc, Vc, b["bs"], O=o, Kblk=b["Kblk"], Vblk=b["Vblk"],
                                         qk_dtype=wl.BF16, v_dtype=wl.BF16)
        dd.dd_bidir_attention(Q, K, V, O=O, qk_dtype=wl.BF16, v_dtype=wl.BF16)
        dd.dd_verify_remask(ld, lv, mask, wl.KL_PROB, 0.0, 5, cfg.B, cfg.G, out_mask=om, out_tokens=ot, out_scores=osc,
                            logit_dtype=wl.BF16)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in outs]
    assert any(bool(t.any()) for t in want)
    graph = capture_step(step)
    for rep in range(4):
        for t in outs:
            t.zero_()                                       # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for w, t in zip(want, outs):
            assert torch.equal(w, t), f"replay {rep} differs from the eager calls"
        step()                                              # eager calls in between leave the graph intact
        torch.cuda.synchronize()
