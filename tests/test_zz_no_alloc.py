"""dd_verify_remask_static (no workspace argument, static device scratch) gives what dd_verify_remask gives."""
import numpy as np
import pytest

import oracle
import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from _util import assert_scores_close, to_dev

pytestmark = pytest.mark.gpu


def _both(cfg, inp, mode, tau, seed):
    import torch
    ld, lv, mk = to_dev(inp["logits_d"]), to_dev(inp["logits_v"]), to_dev(inp["mask"])
    P = cfg.B * cfg.G
    # the outputs of the static call start from a pattern no result can equal, so a call that wrote nothing shows
    om = torch.full((P,), 7, dtype=torch.uint8, device="cuda:0")
    ot = torch.full((P,), -5, dtype=torch.int32, device="cuda:0")
    osc = torch.full((P,), float("nan"), dtype=torch.float32, device="cuda:0")
    dd.dd_verify_remask_static(ld, lv, mk, mode, tau, seed, cfg.B, cfg.G, om, ot, osc, logit_dtype=cfg.logit_dtype)
    want = dd.dd_verify_remask(ld, lv, mk, mode, tau, seed, cfg.B, cfg.G, logit_dtype=cfg.logit_dtype)
    torch.cuda.synchronize()
    got = (om.cpu().numpy(), ot.cpu().numpy(), osc.cpu().numpy())
    want = tuple(t.cpu().numpy() for t in want)
    return got, want


def test_static_scratch_entry_point_matches_the_workspace_one():
    # two calls in a row on the split path (fewer than 192 rows: partial states go through the scratch array),
    # the second smaller in rows, splits and vocabulary, then one on the path that needs no scratch at all
    shapes = [dict(B=3, G=50, V=126464), dict(B=2, G=20, V=4096), dict(B=4, G=75, V=1000)]
    for k, sh in enumerate(shapes):
        cfg = wl.custom_config(logit_dtype=wl.BF16, sigma_d=3.0, sigma_n=1.0, decoded_frac=0.6, **sh)
        assert (dd.dd_verify_remask_workspace_bytes(cfg.B, cfg.G, cfg.V, wl.BF16) > 0) == (k < 2)
        inp = wl.verify_inputs(cfg, seed=40 + k)
        for mode, tau in ((wl.KL_THRESH, 0.45), (wl.CONF_THRESH, 0.02), (wl.KL_PROB, 0.0), (wl.KL_TOPK, 7.0)):
            got, want = _both(cfg, inp, mode, tau, 11)
            for g, w in zip(got, want):
                assert np.array_equal(g, w), f"shape {sh} mode {mode}: differs from dd_verify_remask"
            # and against the oracle, at the bar of the other verification tests
            kl_mode = mode in (wl.KL_THRESH, wl.KL_PROB, wl.KL_TOPK)
            kl, conf, tok = oracle.verify_scores(inp["logits_d"] if kl_mode else None, inp["logits_v"], wl.BF16)
            assert np.array_equal(got[1], tok)
            assert_scores_close(got[2], kl if kl_mode else conf, f"static entry point, shape {sh} mode {mode}")
            own, _ = oracle.remask_decide(got[2], inp["mask"], mode, tau, 11, cfg.B, cfg.G)
            assert np.array_equal(got[0], own)


def test_static_entry_point_validates_like_the_other():
    import torch
    lv = torch.zeros((4, 1024), dtype=torch.float32, device="cuda:0")
    m = torch.zeros(4, dtype=torch.uint8, device="cuda:0")
    om, ot, osc = torch.zeros_like(m), torch.zeros(4, dtype=torch.int32, device="cuda:0"), torch.zeros(4, device="cuda:0")
    with pytest.raises(dd.DDError):
        dd.dd_verify_remask_static(None, lv, m, wl.KL_THRESH, 0.3, 0, 1, 4, om, ot, osc)      # KL needs the drafter
    with pytest.raises(dd.DDError):
        dd.dd_verify_remask_static(lv, lv, m, 9, 0.3, 0, 1, 4, om, ot, osc)                   # unknown mode
