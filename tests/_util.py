"""Helpers shared by the tests: host <-> device transfer and the parity criteria."""
import numpy as np

from paper_2604_05250_amd import workloads as wl


def to_dev(a):
    """numpy storage array -> torch tensor on cuda:0 (uint16 travels as int16: same bits)."""
    import torch
    if a is None:
        return None
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def out_to_f64(t, dtype_tag):
    """device output tensor -> float64 numpy, decoding bf16 bit patterns."""
    a = t.cpu().numpy()
    if dtype_tag == wl.BF16:
        return wl.bf16_bits_to_f32(a.view(np.uint16)).astype(np.float64)
    return a.astype(np.float64)


ATTN_TOL = {wl.F32: (1e-4, 1e-5), wl.BF16: (2e-2, 5e-3), wl.FP8_E4M3: (6e-2, 5e-3)}   # (max-abs, rel-L2) by qk dtype


def attn_errors(got, ref):
    diff = got - ref
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))


def assert_attention_close(got, ref, qk_dtype, what=""):
    mx, rl = attn_errors(got, ref)
    tol_mx, tol_rl = ATTN_TOL[qk_dtype]
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert mx <= tol_mx and rl <= tol_rl, f"{what}: max-abs {mx:.3e} (tol {tol_mx}), rel-L2 {rl:.3e} (tol {tol_rl})"
    return mx, rl


def assert_scores_close(got, ref, what=""):
    """KL / confidence: |got - ref| <= 1e-3 |ref| + 1e-6."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    err = np.abs(got - ref)
    tol = 1e-3 * np.abs(ref) + 1e-6
    bad = np.nonzero(~(err <= tol))[0]
    assert bad.size == 0, f"{what}: {bad.size} scores off, worst row {bad[:5]}, got {got[bad[:5]]}, ref {ref[bad[:5]]}"


def remask_exempt(ora, mode, threshold, seed, rows=None):
    """Rows whose decision may legitimately differ: score within 1e-5 (x max(1,|tau|)) of the
    threshold, or the uniform draw within 1e-5 of the remask probability."""
    import oracle
    s = ora["score64"]
    n = len(s)
    if mode in (wl.KL_THRESH, wl.CONF_THRESH):
        return np.abs(s - threshold) <= 1e-5 * max(1.0, abs(threshold))
    if mode in (wl.KL_PROB, wl.CONF_PROB):
        idx = np.arange(n) if rows is None else np.asarray(rows)
        u = np.array([oracle.row_uniform(seed, int(i)) for i in idx])
        return np.abs(u - ora["prob"]) <= 1e-5
    return np.zeros(n, bool)
