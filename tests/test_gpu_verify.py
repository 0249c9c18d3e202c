"""GPU parity of dd_verify_remask against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest

import oracle
import paper_2604_05250_amd as dd
from paper_2604_05250_amd import workloads as wl
from _util import assert_scores_close, remask_exempt, to_dev

pytestmark = pytest.mark.gpu

ALL_MODES = ((wl.TRUST, 0.0), (wl.KL_THRESH, 0.5), (wl.CONF_THRESH, 0.9), (wl.KL_PROB, 0.0), (wl.CONF_PROB, 0.0))


def run_gpu(inp, mode, tau, seed, B, G, dtype, with_drafter=True):
    ld = to_dev(inp["logits_d"]) if with_drafter else None
    om, ot, osc = dd.dd_verify_remask(ld, to_dev(inp["logits_v"]), to_dev(inp["mask"]), mode, tau, seed, B, G,
                                      logit_dtype=dtype)
    import torch
    torch.cuda.synchronize()
    return om.cpu().numpy(), ot.cpu().numpy(), osc.cpu().numpy()


def check_against_oracle(inp, mode, tau, seed, B, G, dtype, what):
    kl_mode = mode in (wl.KL_THRESH, wl.KL_PROB)
    om, ot, osc = run_gpu(inp, mode, tau, seed, B, G, dtype, with_drafter=kl_mode)
    ora = oracle.verify_remask(inp["logits_d"] if kl_mode else None, inp["logits_v"], inp["mask"], mode, tau, seed,
                               B, G, dtype)
    assert np.array_equal(ot, ora["out_tokens"]), f"{what}: argmax tokens differ"
    assert_scores_close(osc, ora["score64"], what)
    exempt = remask_exempt(ora, mode, tau, seed)
    if mode == wl.KL_PROB:
        # the GPU's probability uses its own fp32 scores; rows where the draw is within their
        # propagated error of the probability are exempt as well
        exempt |= np.abs(np.array([oracle.row_uniform(seed, i) for i in range(B * G)]) - ora["prob"]) <= 2e-3 * ora["prob"] + 1e-5
    diff = (om != ora["out_mask"]) & ~exempt
    assert not diff.any(), f"{what}: remask decisions differ at rows {np.nonzero(diff)[0][:8]}"
    assert np.array_equal(om[inp["mask"] != 0], np.ones(int((inp["mask"] != 0).sum()), np.uint8))
    # no exemption at all for the rule itself: the oracle's decision function applied to the library's own fp32
    # scores reproduces the library's decisions (thresholds, Eq. 6 with its per-sequence sum, the draws)
    own, _ = oracle.remask_decide(osc, inp["mask"], mode, tau, seed, B, G)
    assert np.array_equal(om, own), f"{what}: the rule applied to the library's own scores gives other decisions"
    return om, ot, osc, ora


@pytest.mark.parametrize("mode,tau", ALL_MODES)
def test_cfg1_all_modes(mode, tau):
    cfg = wl.CONFIGS[1]
    inp = wl.verify_inputs(cfg, seed=0)
    om, ot, osc, ora = check_against_oracle(inp, mode, tau, 0, cfg.B, cfg.G, cfg.logit_dtype, f"cfg1 mode {mode}")
    if mode == wl.TRUST:
        assert np.array_equal(om, inp["mask"])
        assert np.array_equal(ot, inp["logits_v"].argmax(axis=1))


@pytest.mark.parametrize("mode", [wl.KL_THRESH, wl.CONF_THRESH, wl.KL_PROB, wl.CONF_PROB])
def test_median_threshold_exercises_both_branches(mode):
    cfg = wl.custom_config(B=3, G=50, V=4096, logit_dtype=wl.BF16, sigma_d=3.0, sigma_n=1.0, decoded_frac=0.6)
    inp = wl.verify_inputs(cfg, seed=3)
    kl, conf, _ = oracle.verify_scores(inp["logits_d"], inp["logits_v"], wl.BF16)
    tau = float(np.median(kl if mode in (wl.KL_THRESH, wl.KL_PROB) else conf))
    om, _, _, ora = check_against_oracle(inp, mode, tau, 12345, cfg.B, cfg.G, wl.BF16, f"median mode {mode}")
    elig = inp["mask"] == 0
    if mode in (wl.KL_THRESH, wl.CONF_THRESH):
        frac = om[elig].mean()
        assert 0.3 < frac < 0.7


@pytest.mark.parametrize("V,dtype", [(8, wl.BF16), (1000, wl.BF16), (4, wl.F32), (1028, wl.F32), (8200, wl.BF16),
                                     (40000, wl.BF16), (126464, wl.BF16)])
def test_ragged_vocab_and_row_splits(V, dtype):
    # small P with a large V makes the library split every row over several workgroups
    cfg = wl.custom_config(B=2, G=5, V=V, logit_dtype=dtype, sigma_d=3.0, sigma_n=1.0)
    inp = wl.verify_inputs(cfg, seed=5)
    for mode, tau in ((wl.KL_THRESH, 0.4), (wl.CONF_THRESH, 0.01)):
        check_against_oracle(inp, mode, tau, 0, cfg.B, cfg.G, dtype, f"V={V} dtype={dtype} mode={mode}")


@pytest.mark.parametrize("P,V,dtype", [(200, 1000, wl.BF16), (300, 33000, wl.BF16), (1100, 520, wl.F32),
                                        (2100, 4104, wl.BF16), (192, 8, wl.BF16)])
def test_one_workgroup_per_row_path(P, V, dtype):
    # enough rows for the fused kernel (workgroup sizes 512 and 256), ragged vocabularies
    cfg = wl.custom_config(B=4, G=P // 4, V=V, logit_dtype=dtype, sigma_d=3.0, sigma_n=1.0, decoded_frac=0.5)
    assert dd.dd_verify_remask_workspace_bytes(cfg.B, cfg.G, V, dtype) == 0
    inp = wl.verify_inputs(cfg, seed=P)
    for mode, tau in ((wl.KL_THRESH, 0.45), (wl.CONF_THRESH, 0.02), (wl.KL_PROB, 0.0), (wl.TRUST, 0.0)):
        check_against_oracle(inp, mode, tau, 9, cfg.B, cfg.G, dtype, f"fused P={P} V={V} mode={mode}")


def test_degenerate_rows():
    V = 2048
    rng = np.random.default_rng(0)
    rows = []
    base = (rng.standard_normal(V) * 3).astype(np.float32)
    r_tie = base.copy(); r_tie[[1500, 7, 900]] = 20.0                  # exact ties: lowest index wins
    r_flat = np.zeros(V, np.float32)                                   # uniform: c = 1/V, token 0
    r_hot = base.copy(); r_hot[1234] = 60.0                            # near one-hot: c -> 1
    r_big = base + np.float32(1000.0)                                  # large magnitude: no overflow
    r_neg = base - np.float32(80.0)
    r_last = base.copy(); r_last[V - 1] = 30.0                         # maximum in the last vector
    lv = np.stack([r_tie, r_flat, r_hot, r_big, r_neg, r_last, base, base])
    ld = np.stack([base, r_flat, base, base + np.float32(1000.0), r_neg, base, base, r_hot])
    for dtype in (wl.F32, wl.BF16):
        inp = {"logits_d": ld if dtype == wl.F32 else wl.f32_to_bf16_bits(ld),
               "logits_v": lv if dtype == wl.F32 else wl.f32_to_bf16_bits(lv),
               "mask": np.zeros(8, np.uint8)}
        om, ot, osc, ora = check_against_oracle(inp, wl.KL_THRESH, 0.3, 0, 1, 8, dtype, f"degenerate dtype {dtype}")
        assert ot[0] == 7 and ot[1] == 0 and ot[2] == 1234 and ot[5] == V - 1
        assert osc[6] == 0.0 and osc[1] == 0.0                         # KL(p || p) = 0 exactly
        _, _, conf, _ = check_against_oracle(inp, wl.CONF_THRESH, 0.5, 0, 1, 8, dtype, "degenerate conf")
        assert abs(conf[1] - 1.0 / V) < 1e-9 and conf[2] > 0.999


def test_mask_extremes_and_threshold_equality():
    cfg = wl.custom_config(B=2, G=16, V=512, logit_dtype=wl.F32)
    inp = wl.verify_inputs(cfg, seed=9)
    P = cfg.P
    for m in (np.ones(P, np.uint8), np.zeros(P, np.uint8)):
        inp2 = dict(inp, mask=m)
        for mode, tau in ALL_MODES:
            om, _, _, _ = check_against_oracle(inp2, mode, tau, 4, cfg.B, cfg.G, wl.F32, "mask extremes")
            if m[0] == 1:
                assert om.all()
    # a score exactly equal to the threshold keeps the token (strict inequalities)
    _, _, osc = run_gpu(inp, wl.KL_THRESH, 0.0, 0, cfg.B, cfg.G, wl.F32)
    tau = float(osc[3])
    om, _, osc2 = run_gpu(inp, wl.KL_THRESH, tau, 0, cfg.B, cfg.G, wl.F32)
    assert osc2[3] == osc[3] and om[3] == 0
    assert np.array_equal(om, (osc2 > np.float32(tau)).astype(np.uint8))
    _, _, conf = run_gpu(inp, wl.CONF_THRESH, 0.0, 0, cfg.B, cfg.G, wl.F32, with_drafter=False)
    om, _, conf2 = run_gpu(inp, wl.CONF_THRESH, float(conf[5]), 0, cfg.B, cfg.G, wl.F32, with_drafter=False)
    assert om[5] == 0 and np.array_equal(om, (conf2 < conf[5]).astype(np.uint8))
    # +-inf thresholds
    om, _, _ = run_gpu(inp, wl.KL_THRESH, float("inf"), 0, cfg.B, cfg.G, wl.F32)
    assert not om.any()
    om, _, _ = run_gpu(inp, wl.KL_THRESH, float("-inf"), 0, cfg.B, cfg.G, wl.F32)
    assert om.all()


def test_empty_input_and_determinism():
    import torch
    e8 = torch.empty(0, dtype=torch.uint8, device="cuda:0")
    lv = torch.empty((0, 1024), dtype=torch.float32, device="cuda:0")
    om, ot, osc = dd.dd_verify_remask(lv, lv, e8, wl.KL_THRESH, 0.3, 0, 0, 16)
    assert om.numel() == 0
    cfg = wl.custom_config(B=2, G=20, V=32768, logit_dtype=wl.BF16)
    inp = wl.verify_inputs(cfg, seed=2)
    a = run_gpu(inp, wl.KL_PROB, 0.0, 77, cfg.B, cfg.G, wl.BF16)
    b = run_gpu(inp, wl.KL_PROB, 0.0, 77, cfg.B, cfg.G, wl.BF16)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    c = run_gpu(inp, wl.KL_PROB, 0.0, 78, cfg.B, cfg.G, wl.BF16)
    assert np.array_equal(a[2], c[2])          # the seed changes draws, not scores


def test_probabilistic_rate_matches_probability():
    # many rows with a known confidence: remask frequency ~ 1 - c
    V, P = 16, 4096
    lv = np.zeros((P, V), np.float32)
    lv[:, 0] = np.log(3.0 * (V - 1))           # c = 0.75
    inp = {"logits_d": lv, "logits_v": lv, "mask": np.zeros(P, np.uint8)}
    om, _, osc = run_gpu(inp, wl.CONF_PROB, 0.0, 5, 1, P, wl.F32, with_drafter=False)
    assert abs(float(osc[0]) - 0.75) < 1e-6
    assert abs(om.mean() - 0.25) < 5 * np.sqrt(0.25 * 0.75 / P)
    u = np.array([oracle.row_uniform(5, i) for i in range(P)])
    want = (u < 1.0 - osc.astype(np.float64)).astype(np.uint8)
    assert np.array_equal(om, want)


# ------------------------------------------------------------------ benchmark configurations, full size
def _full_size(cfg_id, seed=0):
    """Every row of the configuration's verification call against the oracle: tokens exact, scores within the
    score tolerance, decisions exact outside the threshold exemption, and the rule exact on the library's scores."""
    cfg = wl.CONFIGS[cfg_id]
    inp = wl.verify_inputs(cfg, seed=seed)
    import torch
    ld = to_dev(inp["logits_d"]); lv = to_dev(inp["logits_v"]); mk = to_dev(inp["mask"])
    need_kl = any(mode in (wl.KL_THRESH, wl.KL_PROB) for mode, _ in cfg.modes)
    kl, conf, tok = oracle.verify_scores(inp["logits_d"] if need_kl else None, inp["logits_v"], cfg.logit_dtype)
    for mode, tau in cfg.modes:
        kl_mode = mode in (wl.KL_THRESH, wl.KL_PROB)
        om, ot, osc = dd.dd_verify_remask(ld if kl_mode else None, lv, mk, mode, tau, seed, cfg.B, cfg.G,
                                          logit_dtype=cfg.logit_dtype)
        torch.cuda.synchronize()
        om, ot, osc = om.cpu().numpy(), ot.cpu().numpy(), osc.cpu().numpy()
        score = kl if kl_mode else conf
        assert np.array_equal(ot, tok), f"cfg{cfg_id} mode {mode}: tokens"
        assert_scores_close(osc, score, f"cfg{cfg_id} mode {mode}")
        ora_mask, _ = oracle.remask_decide(score.astype(np.float32), inp["mask"], mode, tau, seed, cfg.B, cfg.G)
        exempt = np.abs(score - tau) <= 1e-5 * max(1.0, abs(tau))
        assert np.array_equal(om[~exempt], ora_mask[~exempt]), f"cfg{cfg_id} mode {mode}: decisions"
        own, _ = oracle.remask_decide(osc, inp["mask"], mode, tau, seed, cfg.B, cfg.G)
        assert np.array_equal(om, own), f"cfg{cfg_id} mode {mode}: the rule on the library's own scores"
        if mode == wl.TRUST:
            assert np.array_equal(om, inp["mask"])


def test_cfg2_full_size():
    _full_size(2)


def test_cfg3_full_size():
    _full_size(3)


def test_cfg4_full_size():
    _full_size(4)


def test_cfg5_full_size():
    _full_size(5)


# ------------------------------------------------------------------ budgeted remasking (k worst positions per sequence)
def check_budgeted(inp, mode, k, B, G, dtype, what):
    kl_mode = mode == wl.KL_TOPK
    om, ot, osc = run_gpu(inp, mode, float(k), 0, B, G, dtype, with_drafter=kl_mode)
    ora = oracle.verify_remask(inp["logits_d"] if kl_mode else None, inp["logits_v"], inp["mask"], mode, float(k), 0,
                               B, G, dtype)
    assert np.array_equal(ot, ora["out_tokens"]), f"{what}: argmax tokens differ"
    assert_scores_close(osc, ora["score64"], what)
    mask = inp["mask"].reshape(B, G)
    s = ora["score64"].reshape(B, G)
    exempt = np.zeros((B, G), bool)
    for b in range(B):
        elig = np.flatnonzero(mask[b] == 0)
        n = min(int(k), len(elig))
        # exactly min(k, eligible) positions per sequence, whatever happens at the boundary
        assert int(om.reshape(B, G)[b].sum()) - int((mask[b] != 0).sum()) == n, f"{what}: sequence {b} remask count"
        if 0 < n < len(elig):
            srt = np.sort(s[b][elig])
            edge = srt[::-1][n - 1] if kl_mode else srt[n - 1]           # score of the last position inside the budget
            # the two sides rank their own fp32 scores, which agree to 1e-3 relative: positions that close
            # to the boundary score may swap
            exempt[b] = np.abs(s[b] - edge) <= 2e-3 * abs(edge) + 2e-6
    diff = (om != ora["out_mask"]) & ~exempt.reshape(-1)
    assert not diff.any(), f"{what}: remask decisions differ at rows {np.nonzero(diff)[0][:8]}"
    assert (om[inp["mask"] != 0] == 1).all()
    return om, osc


@pytest.mark.parametrize("mode", [wl.KL_TOPK, wl.CONF_TOPK])
def test_budgeted_modes_small_and_fused_paths(mode):
    for (B, G, V, dtype, frac) in ((3, 50, 4096, wl.BF16, 0.6), (4, 300, 1000, wl.BF16, 0.5), (1, 64, 1024, wl.F32, None),
                                   (2, 2500, 520, wl.F32, 0.7)):
        cfg = wl.custom_config(B=B, G=G, V=V, logit_dtype=dtype, sigma_d=3.0, sigma_n=1.0, decoded_frac=frac)
        inp = wl.verify_inputs(cfg, seed=G)
        for k in (0, 1, 7, G // 3, G, 10 * G):
            check_budgeted(inp, mode, k, B, G, dtype, f"budget {k} mode {mode} B{B} G{G} V{V}")


@pytest.mark.parametrize("mode", [wl.KL_TOPK, wl.CONF_TOPK])
def test_budgeted_modes_break_ties_by_position(mode):
    # identical rows give bit-identical scores: the budget boundary falls inside groups of equal scores
    cfg = wl.custom_config(B=2, G=96, V=2048, logit_dtype=wl.BF16, sigma_d=3.0, sigma_n=1.0)
    inp = wl.verify_inputs(cfg, seed=2)
    for name in ("logits_d", "logits_v"):
        a = inp[name].reshape(cfg.B, cfg.G, -1)
        a[:, 8:, :] = a[:, np.arange(8, cfg.G) % 8, :]               # every sequence: 12 copies of 8 distinct rows
    mask = np.zeros(cfg.P, np.uint8); mask[5::11] = 1
    inp["mask"] = mask
    for k in (1, 5, 13, 30, 50):
        om, osc = check_budgeted(inp, mode, k, cfg.B, cfg.G, wl.BF16, f"ties budget {k} mode {mode}")
        s = osc.reshape(cfg.B, cfg.G)
        assert (s[:, 8:] == s[:, np.arange(8, cfg.G) % 8]).all()
        ora_mask = oracle.remask_decide(osc, mask, mode, float(k), 0, cfg.B, cfg.G)[0]
        assert np.array_equal(om, ora_mask)                           # the rule itself, on the GPU's own scores: exact


def test_cfg3_budgeted_kl():
    cfg = wl.CONFIGS[3]
    inp = wl.verify_inputs(cfg, seed=0)
    om, ot, osc = run_gpu(inp, wl.KL_TOPK, 32.0, 0, cfg.B, cfg.G, cfg.logit_dtype)
    assert np.array_equal(om, oracle.remask_decide(osc, inp["mask"], wl.KL_TOPK, 32.0, 0, cfg.B, cfg.G)[0])
    rows = np.random.default_rng(3).integers(0, cfg.P, 64)
    kl, _, tok = oracle.verify_scores(inp["logits_d"], inp["logits_v"], cfg.logit_dtype, rows=rows)
    assert np.array_equal(ot[rows], tok)
    assert_scores_close(osc[rows], kl, "cfg3 budgeted KL (sampled rows)")


# ------------------------------------------------------------------ drafter unmasking step (dd_unmask)
def check_unmask(inp, mask, mode, thr, B, G, dtype, what, x0=None):
    import torch
    x_dev = None if x0 is None else to_dev(x0.copy())
    om, ot, oc = dd.dd_unmask(to_dev(inp["logits_d"]), to_dev(mask), mode, thr, B, G, x_tokens=x_dev, logit_dtype=dtype)
    torch.cuda.synchronize()
    om, ot, oc = om.cpu().numpy(), ot.cpu().numpy(), oc.cpu().numpy()
    ora = oracle.unmask(inp["logits_d"], mask, mode, thr, B, G, dtype, x_tokens=x0)
    assert np.array_equal(ot, ora["out_tokens"]), f"{what}: argmax tokens differ"
    assert_scores_close(oc, ora["conf64"], what)
    # the selection itself, applied to the GPU's own fp32 confidences: exact
    assert np.array_equal(om, oracle.unmask_decide(oc, mask, mode, thr, B, G)), f"{what}: selection rule"
    # against the oracle's confidences: exact except where a confidence is within the score tolerance of what decides
    c = ora["conf64"].reshape(B, G)
    m2 = mask.reshape(B, G)
    exempt = np.zeros((B, G), bool)
    for b in range(B):
        cand = np.flatnonzero(m2[b])
        if len(cand) == 0:
            continue
        srt = np.sort(c[b][cand])[::-1]
        edges = [srt[0]]
        if mode == wl.UNMASK_THRESH:
            edges.append(thr)
        else:
            k = int(thr)
            if 0 < k < len(cand):
                edges.append(srt[k - 1])
        for e in edges:
            exempt[b] |= np.abs(c[b] - e) <= 2e-3 * abs(e) + 2e-6
    diff = (om != ora["out_mask"]) & ~exempt.reshape(-1)
    assert not diff.any(), f"{what}: selections differ at rows {np.nonzero(diff)[0][:8]}"
    assert (om[mask == 0] == 0).all() and (om <= mask).all()          # decoded stays decoded; nothing gets masked
    if x0 is not None:
        x = x_dev.cpu().numpy()
        sel = (mask != 0) & (om == 0)
        assert np.array_equal(x[sel], ot[sel]) and np.array_equal(x[~sel], x0[~sel])
    return om


@pytest.mark.parametrize("mode", [wl.UNMASK_THRESH, wl.UNMASK_TOPK])
def test_unmask_small_and_fused_paths(mode):
    for (B, G, V, dtype, frac) in ((3, 50, 4096, wl.BF16, 0.4), (4, 300, 1000, wl.BF16, 0.5), (1, 64, 1024, wl.F32, 0.2),
                                   (2, 2500, 520, wl.F32, 0.7), (2, 16, 126464, wl.BF16, 0.0)):
        cfg = wl.custom_config(B=B, G=G, V=V, logit_dtype=dtype, sigma_d=3.0, sigma_n=1.0, decoded_frac=frac)
        inp = wl.verify_inputs(cfg, seed=G + 1)
        mask = inp["mask"]
        x0 = np.full(cfg.P, 126336, np.int32)
        conf = oracle.verify_scores(None, inp["logits_d"], dtype)[1]
        thrs = (0.0, float(np.median(conf)), 2.0) if mode == wl.UNMASK_THRESH else (0.0, 1.0, 7.0, float(G // 3), float(10 * G))
        for thr in thrs:
            om = check_unmask(inp, mask, mode, thr, B, G, dtype, f"unmask mode {mode} thr {thr} B{B} G{G} V{V}", x0=x0)
            if mode == wl.UNMASK_THRESH and thr == 2.0:               # nothing exceeds: exactly one per unfinished sequence
                assert ((mask.reshape(B, G) != 0).sum(1) - om.reshape(B, G).sum(1) == (mask.reshape(B, G).any(1))).all()


def test_unmask_ties_and_finished_sequences():
    cfg = wl.custom_config(B=3, G=96, V=2048, logit_dtype=wl.BF16, sigma_d=3.0, sigma_n=1.0)
    inp = wl.verify_inputs(cfg, seed=8)
    a = inp["logits_d"].reshape(cfg.B, cfg.G, -1)
    a[:, 8:, :] = a[:, np.arange(8, cfg.G) % 8, :]                    # 12 copies of 8 distinct rows: exact ties
    mask = np.ones(cfg.P, np.uint8); mask[3::7] = 0
    mask.reshape(cfg.B, cfg.G)[1] = 0                                  # sequence 1 is finished
    for k in (1, 5, 13, 40):
        om = check_unmask(inp, mask, wl.UNMASK_TOPK, float(k), cfg.B, cfg.G, wl.BF16, f"unmask ties k={k}")
        assert not om.reshape(cfg.B, cfg.G)[1].any()
    check_unmask(inp, mask, wl.UNMASK_THRESH, 0.05, cfg.B, cfg.G, wl.BF16, "unmask ties threshold")


def test_unmask_block_of_cfg3():
    # one draft step of cfg3: the drafter's logits of the active block (64 positions per sequence)
    cfg = wl.CONFIGS[3]
    blk = wl.custom_config(B=cfg.B, G=cfg.bl, V=cfg.V, logit_dtype=cfg.logit_dtype, sigma_d=cfg.sigma_d, sigma_n=cfg.sigma_n,
                           decoded_frac=0.25)
    inp = wl.verify_inputs(blk, seed=0)
    check_unmask(inp, inp["mask"], wl.UNMASK_THRESH, 0.02, blk.B, blk.G, blk.logit_dtype, "cfg3 block unmask")


# ---- dd_verify_scores: every per-position quantity of Sec. 3.2 from one pass -----------------------------------------
def check_all_scores(ld, lv, dtype, what, drafter=True):
    import torch
    kl, cv, tv, cd, td = dd.dd_verify_scores(to_dev(ld), to_dev(lv), drafter=drafter, logit_dtype=dtype)
    torch.cuda.synchronize()
    o_kl, o_cv, o_tv = oracle.verify_scores(ld, lv, dtype)
    assert np.array_equal(tv.cpu().numpy(), o_tv), f"{what}: verifier tokens differ"
    assert_scores_close(kl.cpu().numpy(), o_kl, what + " kl")
    assert_scores_close(cv.cpu().numpy(), o_cv, what + " conf_v")
    if drafter:
        _, o_cd, o_td = oracle.verify_scores(None, ld, dtype)         # the drafter's own confidence and argmax
        assert np.array_equal(td.cpu().numpy(), o_td), f"{what}: drafter tokens differ"
        assert_scores_close(cd.cpu().numpy(), o_cd, what + " conf_d")
    else:
        assert cd is None and td is None
    return kl.cpu().numpy(), cv.cpu().numpy(), tv.cpu().numpy()


@pytest.mark.parametrize("P,V,dtype", [(10, 8200, wl.BF16), (10, 1028, wl.F32), (7, 126464, wl.BF16), (1, 8, wl.BF16),
                                        (200, 1000, wl.BF16), (300, 33000, wl.BF16), (1100, 520, wl.F32),
                                        (2100, 4104, wl.BF16)])
def test_all_scores_one_pass(P, V, dtype):
    # few rows: every row split over workgroups and merged by the finishing kernel; many rows: one workgroup per row
    cfg = wl.custom_config(B=1, G=P, V=V, logit_dtype=dtype, sigma_d=3.0, sigma_n=1.0)
    inp = wl.verify_inputs(cfg, seed=21)
    kl, cv, tv = check_all_scores(inp["logits_d"], inp["logits_v"], dtype, f"scores P={P} V={V} dtype={dtype}")
    # the same numbers as the rule-applying entry point reports (same kernels)
    _, ot, osc = run_gpu(dict(inp, mask=np.zeros(P, np.uint8)), wl.KL_THRESH, 0.5, 0, 1, P, dtype)
    assert np.array_equal(ot, tv) and np.array_equal(osc, kl)
    _, _, osc = run_gpu(dict(inp, mask=np.zeros(P, np.uint8)), wl.CONF_THRESH, 0.5, 0, 1, P, dtype, with_drafter=False)
    assert np.array_equal(osc, cv)
    check_all_scores(inp["logits_d"], inp["logits_v"], dtype, "scores without the drafter's pair", drafter=False)


@pytest.mark.parametrize("P", [8, 256])
def test_all_scores_drafter_ties_and_extremes(P):
    # the drafter's most likely token under exact ties (lowest index), maxima in the first and last vector of a
    # row and on both sides of every split boundary, flat rows, large offsets
    V = 40960
    rng = np.random.default_rng(2)
    base = (rng.standard_normal(V) * 3).astype(np.float32)
    rows_d = []
    for i in range(P):
        r = base.copy()
        k = i % 8
        if k == 0: r[[V - 1, 31000, 12]] = 25.0
        elif k == 1: r[:] = 0.0
        elif k == 2: r[V - 1] = 40.0
        elif k == 3: r[0] = 40.0
        elif k == 4: r[[20479, 20480]] = 30.0
        elif k == 5: r += np.float32(900.0)
        elif k == 6: r[[2559, 2560, 5119, 5120, 38400]] = 22.0
        rows_d.append(r)
    ld = np.stack(rows_d)
    lv = np.stack([np.roll(base, i + 1) for i in range(P)]).astype(np.float32)
    for dtype in (wl.F32, wl.BF16):
        a = ld if dtype == wl.F32 else wl.f32_to_bf16_bits(ld)
        b = lv if dtype == wl.F32 else wl.f32_to_bf16_bits(lv)
        import torch
        _, _, _, cd, td = dd.dd_verify_scores(to_dev(a), to_dev(b), logit_dtype=dtype)
        td = td.cpu().numpy()
        assert td[0] == 12 and td[1] == 0 and td[2] == V - 1 and td[3] == 0 and td[4] == 20479 and td[6] == 2559
        assert abs(float(cd[1]) - 1.0 / V) < 1e-9
        check_all_scores(a, b, dtype, f"scores ties P={P} dtype={dtype}")


def test_all_scores_identical_models_and_empty():
    import torch
    cfg = wl.custom_config(B=1, G=12, V=2048, logit_dtype=wl.BF16)
    inp = wl.verify_inputs(cfg, seed=4)
    kl, cv, tv, cd, td = dd.dd_verify_scores(to_dev(inp["logits_v"]), to_dev(inp["logits_v"]), logit_dtype=wl.BF16)
    assert (kl == 0).all() and torch.equal(cv, cd) and torch.equal(tv, td)        # KL(p || p) = 0 exactly
    empty = torch.empty(0, 2048, dtype=torch.bfloat16, device="cuda:0")
    out = dd.dd_verify_scores(empty, empty)
    assert all(o.numel() == 0 for o in out)
