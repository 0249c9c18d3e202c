#!/usr/bin/env python3
"""Benchmark of one DualDiffusion draft-then-verify step on one MI355X.

A step = K drafter block-attention calls over the cached K/V, one verifier full
bidirectional attention, one verification pass over the vocabulary (Alg. 1, one cycle),
on seeded synthetic inputs already resident in HBM.  Prints ONE JSON line:
  value        = verifier attention TFLOP/s (4*B*H*N^2*d FLOP per call / its measured time)
  ms_per_step  = wall time of the whole step (events around all kernels of the step)
  roofline     = the attention kernel against the dense MFMA peak of its operand types
  roofline_verify = the verification kernels against the HBM peak
  roofline_block  = the drafter's call against the HBM peak (every call on another copy of the cache: cold)
  cpu_baseline = the fp64 CPU oracle timed on a bounded sample of the same workload
  per_config   = the same rates for the other benchmark configurations, timed in a light form (default run only)
Rates come from events around each call inside the timed steps; back_to_back_* repeat each part alone as a stream of
launches; `traffic` is the HBM bytes per call recorded in profiles/ for the kernel sources in the tree (else null).
--fp8v / --mx time the reduced-precision workloads, --no-streams / --no-per-config / --no-graph shorten profiler runs.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "verifier attn TFLOP/s (% MFMA peak); verify GB/s (% HBM); draft+verify step ms"
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP8_TFLOPS = 5000.0      # MI355X dense fp8 MFMA
PEAK_FP32_VALU_TFLOPS = 157.3 # MI355X fp32 vector
PEAK_HBM_GBPS = 8000.0        # MI355X HBM3E
LLC_ROTATE_BYTES = 600e6      # rotate input sets until their total exceeds 2x the 256 MB last-level cache
KERNEL_SOURCES = ("attention_wide.hip", "attention_mfma.hip", "attention_stream.hip", "attention_common.h", "verify.hip")


def kernel_source_digest():
    """Short hash of the kernel sources, comments and blank space left out (a comment edit is no other kernel): a
    profile records the one it was taken with."""
    import hashlib
    import re
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2604_05250_amd", "csrc", name), "r", encoding="utf-8") as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)           # block comments
        text = re.sub(r"//[^\n]*", "", text)                          # line comments (no string in these files holds "//")
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:12]


def profiled_traffic(config_id, part):
    """HBM bytes per launch of the dominant kernel of `part`, as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE (scaled by what the same counters read for a copy of known size) and recorded in
    profiles/step_kernels_cfg<N>_*.md on a line `traffic_bytes: attention=... verify=... kernels=<digest>`.
    None when there is no such record or when it was taken with other kernel sources than the ones in the tree."""
    import glob
    import re
    for path in glob.glob(os.path.join(ROOT, "profiles", f"step_kernels_cfg{config_id}_*.md")):
        for line in open(path):
            m = re.match(r"\s*traffic_bytes:\s*(.*)", line)
            if not m:
                continue
            kv = dict(t.split("=", 1) for t in m.group(1).split() if "=" in t)
            if kv.get("kernels") != kernel_source_digest() or part not in kv:
                return None
            return float(kv[part])
    return None


def wl_mode_names():
    from paper_2604_05250_amd import workloads as wl
    return list(wl.MODE_NAMES.values())


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--parts", default="block,attention,verify",
                    help="comma list of the step's parts to run (profiling a single kernel); default: the whole step; "
                         "'unmask' adds the drafter's unmasking step after the K block calls, 'scores' one "
                         "dd_verify_scores call (KL, both confidences, both argmax tokens) after the verification")
    ap.add_argument("--refresh-last", action="store_true",
                    help="the last of the K drafter calls completes its block: dd_block_attention_refresh")
    ap.add_argument("--window", type=int, default=0,
                    help="the drafter attends over a window of this many key rows around the block "
                         "(dd_block_attention_window) instead of the whole cache")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="after the timed steps, run one device-to-device copy of this many MiB (a kernel of known "
                         "traffic, used to scale the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    ap.add_argument("--verify-mode", default=None, choices=sorted(wl_mode_names()),
                    help="verification rule to run instead of the workload's own (kl_topk / conf_topk: threshold = budget k)")
    ap.add_argument("--verify-threshold", type=float, default=0.0)
    ap.add_argument("--unmask-threshold", type=float, default=0.9,
                    help="confidence threshold of the optional 'unmask' part (add it to --parts)")
    ap.add_argument("--layers", type=int, default=0,
                    help="additionally time the cycle of an L-layer model (attention only): every draft step runs the "
                         "drafter's block attention on L caches, the last one with the block-completion refresh, then "
                         "the unmasking step; the verifier runs L full attentions, then the verification rule. "
                         "Reported as the extra object 'multi_layer' (32 = LLaDA-8B's depth)")
    ap.add_argument("--no-graph", action="store_true", help="skip the additional HIP-graph replay of the step")
    ap.add_argument("--prewarm-ms", type=float, default=300.0,
                    help="before the W warm-up steps, run untimed steps for this many milliseconds: an idle MI355X "
                         "needs some 30 ms of load to reach its sustained clocks (the first calls after idling run "
                         "15 %% slower), and a fresh process starts on an idle chip")
    ap.add_argument("--no-warm", action="store_true",
                    help="skip the additional warm-cache repetition of the steps (profiling: every launch in the "
                         "trace then belongs to the rotated, cold-cache steps)")
    ap.add_argument("--fp8v", action="store_true",
                    help="second precision workload: the configuration with Q, K and V all stored as e4m3 codes with "
                         "per-head scales (dd_bidir_attention_fp8v / dd_block_attention_cached_fp8v); meant for --config 5")
    ap.add_argument("--mx", action="store_true",
                    help="third precision workload: the verifier's attention on block-scaled inputs (e4m3 Q/K, e2m1 V, E8M0 "
                         "scales per 32 elements: dd_bidir_attention_mx) drawn from the same fp32 values; the drafter's "
                         "calls and the verification run as in the chosen config; meant for --config 5")
    ap.add_argument("--no-streams", action="store_true",
                    help="skip the back-to-back streams of single parts after the timed steps (profiler runs: the timed "
                         "steps are then the last launches of the trace)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="time only the configuration named by --config (the default run also times the other benchmark "
                         "configurations, reported under 'per_config')")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="CPU oracle time budget per sampled part")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding or collectives are part of it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    out = run_config(args, args.config)
    if not args.no_per_config:
        # the other benchmark configurations, same protocol (rotated inputs, events around each part), fewer steps,
        # no graph replay and no CPU baseline: every rate of every configuration comes from this one run
        import copy
        light = copy.copy(args)
        light.steps, light.warmup, light.prewarm_ms = max(5, args.steps // 4), 3, min(args.prewarm_ms, 150.0)
        light.no_graph = light.no_warm = light.no_cpu_baseline = True
        light.no_streams = False
        light.layers, light.calib_copy_mb, light.verify_mode = 0, 0, None
        light.parts, light.window, light.refresh_last, light.fp8v = "block,attention,verify", 0, False, False
        light.mx = False
        out["per_config"] = {}
        for cid in (2, 4, 5, 3):
            if cid == args.config:
                continue
            r = run_config(light, cid)
            out["per_config"][f"cfg{cid}"] = {
                "workload": r["config"]["workload"], "steps": r["steps"], "ms_per_step": r["ms_per_step"],
                "components_ms": r["components_ms"], "dtype": r["dtype"],
                "roofline": r["roofline"], "roofline_verify": r["roofline_verify"],
                "roofline_block": r["roofline_block"]}
    print(json.dumps(out), flush=True)


def run_config(args, config_id):
    import gc

    import numpy as np
    import torch

    import paper_2604_05250_amd as dd
    from paper_2604_05250_amd import workloads as wl

    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[config_id]
    fp8v = bool(getattr(args, "fp8v", False))
    if fp8v:
        import dataclasses
        cfg = dataclasses.replace(cfg, name=cfg.name + "_fp8v", qk_dtype=wl.FP8_E4M3, v_dtype=wl.FP8_E4M3)
    mx = bool(getattr(args, "mx", False))
    if mx and fp8v:
        print("bench.py: --mx and --fp8v are different workloads", file=sys.stderr)
        sys.exit(2)
    mode, tau = cfg.modes[-1]
    if args.verify_mode is not None:                     # another rule of the same call on the same inputs
        mode = {v: k for k, v in wl.MODE_NAMES.items()}[args.verify_mode]
        tau = args.verify_threshold
    kl_mode = mode in (wl.KL_THRESH, wl.KL_PROB, wl.KL_TOPK)

    def up(a):
        if a is None:
            return None
        if a.dtype == np.uint16:
            a = a.view(np.int16)
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # ---- seeded inputs, generated on the host (the oracle reads the same arrays), resident in HBM before timing
    att = wl.attention_inputs(cfg, args.seed)
    att_mx = wl.mx_attention_inputs(cfg, args.seed) if mx else None
    cache = wl.cache_inputs(cfg, args.seed)
    ver = wl.verify_inputs(cfg, args.seed)
    blocks = [wl.block_inputs(cfg, args.seed, k, k_scale=cache["k_scale"], v_scale=cache["v_scale"]) for k in range(cfg.K)]

    eb_qk, eb_v, eb_l = wl.elem_bytes(cfg.qk_dtype), wl.elem_bytes(cfg.v_dtype), wl.elem_bytes(cfg.logit_dtype)
    q_elems = cfg.B * cfg.H * cfg.N * cfg.d
    kv_elems = cfg.B * cfg.Hkv * cfg.N * cfg.d
    attn_bytes = q_elems * eb_qk + kv_elems * eb_qk + kv_elems * eb_v + q_elems * eb_v          # Q + K + V + O once
    if mx:                                               # e4m3 Q, K; packed e2m1 V; one scale byte per 32 elements; bf16 O
        attn_bytes = q_elems + kv_elems + kv_elems // 2 + (q_elems + 2 * kv_elems) // 32 + q_elems * 2
    verify_bytes = (2 if kl_mode else 1) * cfg.P * cfg.V * eb_l                               # logits read once
    blk_rows = cfg.B * cfg.H * cfg.bl * cfg.d
    block_bytes = kv_elems * (eb_qk + eb_v) + blk_rows * (eb_qk + eb_v)                       # cache + Qblk + O
    cache_bytes = kv_elems * (eb_qk + eb_v)
    set_bytes = attn_bytes + verify_bytes
    n_sets = max(1, min(8, math.ceil(LLC_ROTATE_BYTES / set_bytes)))
    # the K drafter calls of a step follow each other directly: each reads ANOTHER copy of the cache, enough
    # copies that a call never finds its operands in the 256 MB last-level cache because an earlier call read them
    n_caches = max(2, min(96, math.ceil(LLC_ROTATE_BYTES / cache_bytes)))

    sets = []
    for _ in range(n_sets):
        src = att_mx if mx else att
        sets.append({
            "Q": up(src["Q"]), "K": up(src["K"]), "V": up(src["V"]),
            "mx": tuple(up(att_mx[k]) for k in ("Qs", "Ks", "Vs")) if mx else None,
            "ld": up(ver["logits_d"]) if (kl_mode or "scores" in args.parts.split(",")) else None, "lv": up(ver["logits_v"]),
        })
    caches = [{"Kc": up(cache["Kc"]), "Vc": up(cache["Vc"])} for _ in range(n_caches)]
    qs, ks = up(att["q_scale"]), up(att["k_scale"])
    kcs = up(cache["k_scale"])
    vs, vcs = up(att["v_scale"]), up(cache["v_scale"])
    mask = up(ver["mask"])
    blk_dev = [{"Q": up(b["Qblk"]), "K": up(b["Kblk"]), "V": up(b["Vblk"]), "qs": up(b["q_scale"]),
                "bs": b["block_start"]} for b in blocks]
    o_dtype = torch.int16 if fp8v else caches[0]["Vc"].dtype
    O = torch.empty((cfg.B, cfg.H, cfg.N, cfg.d), dtype=torch.int16 if mx else o_dtype, device=dev)
    Oblk = torch.empty((cfg.B, cfg.H, cfg.bl, cfg.d), dtype=o_dtype, device=dev)
    out_mask = torch.empty(cfg.P, dtype=torch.uint8, device=dev)
    out_tok = torch.empty(cfg.P, dtype=torch.int32, device=dev)
    out_sc = torch.empty(cfg.P, dtype=torch.float32, device=dev)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    parts = set(args.parts.split(","))

    # optional part: the drafter's unmasking step after each of the K block calls (Alg. 1, drafting phase), on the
    # drafter's logits of the active block: [B*bl, V] per step, cut from the workload's drafter logits
    unmask_dev = []
    unmask_bytes = cfg.B * cfg.bl * cfg.V * eb_l
    if "unmask" in parts:
        ld_full = up(ver["logits_d"]).view(cfg.B, cfg.G, cfg.V)
        rng_m = np.random.default_rng(args.seed + 77)
        for k in range(cfg.K):
            g0 = (k * cfg.bl) % max(1, cfg.G - cfg.bl + 1)
            unmask_dev.append({"ld": ld_full[:, g0:g0 + cfg.bl, :].contiguous().view(cfg.B * cfg.bl, cfg.V),
                               "mask": up((rng_m.random(cfg.B * cfg.bl) < 0.5).astype(np.uint8))})
        del ld_full
        um_mask = torch.empty(cfg.B * cfg.bl, dtype=torch.uint8, device=dev)
        um_tok = torch.empty(cfg.B * cfg.bl, dtype=torch.int32, device=dev)
        um_conf = torch.empty(cfg.B * cfg.bl, dtype=torch.float32, device=dev)
        um_x = torch.zeros(cfg.B * cfg.bl, dtype=torch.int32, device=dev)

    win = min(args.window, cfg.N) if args.window > 0 else 0
    if win and win < cfg.bl:
        print("bench.py: --window must cover the block", file=sys.stderr)
        sys.exit(2)
    if win:                                              # K/V bytes of a call follow the window
        block_bytes = cfg.B * cfg.Hkv * win * cfg.d * (eb_qk + eb_v) + blk_rows * (eb_qk + eb_v)

    def step(i, rec=None, one_cache=False):
        s = sets[i % n_sets]
        marks = [ev() for _ in range(6)] if rec is not None else None
        if marks: marks[0].record()
        for k, b in enumerate(blk_dev if "block" in parts else ()):
            kc = caches[0 if one_cache else (i * cfg.K + k) % n_caches]
            kw = dict(O=Oblk, Kblk=b["K"], Vblk=b["V"], q_scale=b["qs"], k_scale=kcs, qk_dtype=cfg.qk_dtype,
                      v_dtype=cfg.v_dtype)
            if fp8v:
                dd.dd_block_attention_cached_fp8v(b["Q"], kc["Kc"], kc["Vc"], b["bs"], b["qs"], kcs, vcs, O=Oblk,
                                                  Kblk=b["K"], Vblk=b["V"])
            elif win:
                w0 = min(max(0, b["bs"] + cfg.bl // 2 - win // 2), cfg.N - win)
                dd.dd_block_attention_window(b["Q"], kc["Kc"], kc["Vc"], b["bs"], w0, win, **kw)
            elif args.refresh_last and k == cfg.K - 1:
                kw.pop("Kblk"); kw.pop("Vblk")
                dd.dd_block_attention_refresh(b["Q"], kc["Kc"], kc["Vc"], b["bs"], b["K"], b["V"], **kw)
            else:
                dd.dd_block_attention_cached(b["Q"], kc["Kc"], kc["Vc"], b["bs"], **kw)
        if marks: marks[1].record()
        for u in unmask_dev:
            dd.dd_unmask(u["ld"], u["mask"], dd.UNMASK_THRESH, args.unmask_threshold, cfg.B, cfg.bl, x_tokens=um_x,
                         out_mask=um_mask, out_tokens=um_tok, out_conf=um_conf, logit_dtype=cfg.logit_dtype)
        if marks: marks[4].record()
        if "attention" in parts and mx:
            dd.dd_bidir_attention_mx(s["Q"], s["mx"][0], s["K"], s["mx"][1], s["V"], s["mx"][2], O=O)
        elif "attention" in parts and fp8v:
            dd.dd_bidir_attention_fp8v(s["Q"], s["K"], s["V"], qs, ks, vs, O=O)
        elif "attention" in parts:
            dd.dd_bidir_attention(s["Q"], s["K"], s["V"], O=O, q_scale=qs, k_scale=ks,
                                  qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
        if marks: marks[2].record()
        if "verify" in parts:
            dd.dd_verify_remask(s["ld"] if kl_mode else None, s["lv"], mask, mode, tau, args.seed, cfg.B, cfg.G,
                                out_mask=out_mask, out_tokens=out_tok, out_scores=out_sc, logit_dtype=cfg.logit_dtype)
        if marks: marks[3].record()
        if "scores" in parts:
            dd.dd_verify_scores(s["ld"], s["lv"], logit_dtype=cfg.logit_dtype)
        if marks:
            marks[5].record()
            rec.append(marks)

    # bring the chip to its sustained clocks (untimed; the count is reported), then the W warm-up steps
    prewarm_steps = 0
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.prewarm_ms:
        for _ in range(8):
            step(prewarm_steps)
            prewarm_steps += 1
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    rec = []
    t_begin, t_end = ev(), ev()
    wall0 = time.perf_counter()
    t_begin.record()
    for i in range(args.steps):
        step(args.warmup + i, rec)
    t_end.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    total_ms = t_begin.elapsed_time(t_end)
    ms_per_step = total_ms / args.steps
    t_block = sum(m[0].elapsed_time(m[1]) for m in rec) / len(rec)         # K calls
    t_unmask = sum(m[1].elapsed_time(m[4]) for m in rec) / len(rec)
    t_attn = sum(m[4].elapsed_time(m[2]) for m in rec) / len(rec)
    t_ver = sum(m[2].elapsed_time(m[3]) for m in rec) / len(rec)
    if "verify" in parts:
        assert torch.isfinite(out_sc).all().item(), "non-finite verification scores"
    t_block, t_attn, t_ver = (max(t, 1e-9) for t in (t_block, t_attn, t_ver))
    per_step = {"block_attention_xK": [m[0].elapsed_time(m[1]) for m in rec],
                "bidir_attention": [m[4].elapsed_time(m[2]) for m in rec],
                "verify_remask": [m[2].elapsed_time(m[3]) for m in rec]}

    # Each part alone, as a stream of back-to-back launches on rotated (cold) inputs: the average launch duration of its
    # kernels, which is what rocprofv3 reports per kernel.  Inside a step every part follows a kernel of another
    # kind, and the events around it also see the hand-over between the two (2-5 us, which matters for parts of 30 us).
    # (A change of load pattern is followed by some tens of milliseconds of lower clocks - the attention kernel's first
    # launches of such a stream take a fifth longer than its later ones - so each stream first runs untimed for 80 ms.)
    def stream_us(call, n=30):
        j0 = 0
        t_s = time.perf_counter()
        while (time.perf_counter() - t_s) * 1e3 < 80.0:
            for _ in range(5):
                call(j0)
                j0 += 1
            torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for j in range(n):
            call(j0 + j)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n * 1e3

    saved_parts = set(parts)
    stream = {}
    for name in ("attention", "verify", "block"):
        if name not in saved_parts or getattr(args, "no_streams", False):
            continue
        parts.clear()
        parts.add(name)
        stream[name] = stream_us(lambda j: step(j)) / (cfg.K if name == "block" else 1)
    parts.clear()
    parts.update(saved_parts)

    # the same parts with every step on ONE input set: whatever fits stays in the 256 MB last-level cache.
    # Reported beside the figures above, which rotate input sets and are the ones every rate is computed from.
    warm_rec = []
    if not args.no_warm:
        for i in range(args.warmup):
            step(0, one_cache=True)
        for i in range(args.steps):
            step(0, warm_rec, one_cache=True)
        torch.cuda.synchronize()

    # the same steps replayed as HIP graphs (one per input set): what the cycle costs without the host in the loop
    graph_ms = None
    if not args.no_graph:
        from paper_2604_05250_amd.step import capture_step
        graphs = [capture_step(lambda i=i: step(i)) for i in range(n_sets)]
        t_pre = time.perf_counter()              # capturing left the chip idle: back to sustained clocks first
        while (time.perf_counter() - t_pre) * 1e3 < min(args.prewarm_ms, 100.0):
            for i in range(8):
                graphs[i % n_sets].replay()
            torch.cuda.synchronize()
        for i in range(args.warmup):
            graphs[i % n_sets].replay()
        torch.cuda.synchronize()
        g_begin, g_end = ev(), ev()
        g_begin.record()
        for i in range(args.steps):
            graphs[(args.warmup + i) % n_sets].replay()
        g_end.record()
        torch.cuda.synchronize()
        graph_ms = g_begin.elapsed_time(g_end) / args.steps
        if "verify" in parts:
            assert torch.isfinite(out_sc).all().item(), "non-finite verification scores after graph replay"

    if args.calib_copy_mb > 0:
        src = torch.empty(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        src.fill_(1)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()

    attn_flops = 4.0 * cfg.B * cfg.H * cfg.N * cfg.N * cfg.d
    attn_tflops = attn_flops / (t_attn * 1e-3) / 1e12
    ver_gbps = verify_bytes / (t_ver * 1e-3) / 1e9
    blk_gbps = block_bytes / (t_block / cfg.K * 1e-3) / 1e9
    attn_stream_tflops = attn_flops / (stream["attention"] * 1e-6) / 1e12 if "attention" in stream else attn_tflops
    ver_stream_gbps = verify_bytes / (stream["verify"] * 1e-6) / 1e9 if "verify" in stream else ver_gbps
    blk_stream_gbps = block_bytes / (stream["block"] * 1e-6) / 1e9 if "block" in stream else blk_gbps

    def attn_kernel_name(c):
        """The kernel the library's size rule picks for this call (the rule itself lives in the library)."""
        group = c.H // c.Hkv
        wide_tiles = c.B * c.Hkv * -(-group * c.N // 256)
        fp8 = c.qk_dtype == wl.FP8_E4M3
        if wide_tiles >= 192 and c.N >= 512 and (not fp8 or c.d == 128):
            fold = not fp8 and c.N >= 1024          # bf16 without per-head scales: the folded-scale form
            return f"attn_wide_kernel<{c.d}, {'true' if fp8 else 'false'}, false, {'true' if fold else 'false'}, 2>"
        if not fp8 and c.B * c.Hkv * -(-group * c.N // 128) < 256:
            return f"attn_stream_kernel<{c.d}>"
        return f"attn_mfma_kernel<{c.d}, {'true' if fp8 else 'false'}, false, false, false>"

    # the peak the attention call is priced against: each contraction at the peak of its own operand type
    if mx:
        attn_kernel, attn_bound = f"attn_mfma_kernel<{cfg.d}, true, false, false, true>", "mfma"
        attn_peak = 2.0 / (1.0 / PEAK_FP8_TFLOPS + 1.0 / PEAK_BF16_TFLOPS)
        attn_peak_note = ("half of the FLOPs (S = Q K^T) run on the block-scaled fp8 matrix instruction (5.0 PFLOP/s), half "
                          "(O = P V, V decoded to bf16 on its way into LDS) as bf16 MFMA (2.5 PFLOP/s): time-weighted peak "
                          "3.33 PFLOP/s")
    elif fp8v:
        attn_kernel, attn_bound = f"attn_mfma_kernel<{cfg.d}, true, false, true, false>", "mfma"
        attn_peak = 2.0 / (1.0 / PEAK_FP8_TFLOPS + 1.0 / PEAK_BF16_TFLOPS)
        attn_peak_note = ("half of the FLOPs (S = Q K^T) run as fp8 MFMA on the e4m3 operands as stored (5.0 PFLOP/s), half "
                          "(O = P V, V decoded to bf16 on its way into LDS) as bf16 MFMA (2.5 PFLOP/s): time-weighted peak "
                          "3.33 PFLOP/s")
    elif cfg.qk_dtype == wl.F32:
        attn_kernel, attn_bound, attn_peak = "attn_f32_kernel", "alu", PEAK_FP32_VALU_TFLOPS
        attn_peak_note = "fp32 inputs: vector ALUs (no fp32 MFMA path is used), 157.3 TFLOP/s"
    elif cfg.qk_dtype == wl.FP8_E4M3:
        attn_kernel, attn_bound = attn_kernel_name(cfg), "mfma"
        attn_peak = 2.0 / (1.0 / PEAK_FP8_TFLOPS + 1.0 / PEAK_BF16_TFLOPS)
        attn_peak_note = ("half of the FLOPs (S = Q K^T) run as fp8 MFMA (5.0 PFLOP/s), half (O = P V) as bf16 MFMA "
                          "(2.5 PFLOP/s): time-weighted peak 3.33 PFLOP/s")
    else:
        attn_kernel, attn_bound, attn_peak = attn_kernel_name(cfg), "mfma", PEAK_BF16_TFLOPS
        attn_peak_note = "dense bf16 MFMA, 2.5 PFLOP/s"

    out = {
        "metric": METRIC, "value": round(attn_tflops, 3), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "mxfp8_e4m3(QK)+mxfp4_e2m1(V)" if mx else "fp8_e4m3(QKV)" if fp8v else {wl.F32: "f32", wl.BF16: "bf16", wl.FP8_E4M3: "fp8_e4m3(QK)+bf16(V)"}[cfg.qk_dtype],
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}{'_mx' if mx else ''}: B={cfg.B} H={cfg.H} Hkv={cfg.Hkv} N={cfg.N} d={cfg.d}, "
                               f"drafter block_len={cfg.bl} x K={cfg.K} steps, verify P={cfg.P} x V={cfg.V} "
                               f"mode={wl.MODE_NAMES[mode]} tau={tau}",
                   "baseline_config_index": config_id - 1, "input_sets_rotated": n_sets, "cache_copies_rotated": n_caches,
                   "seed": args.seed,
                   "prewarm_steps": prewarm_steps,
                   "parts": sorted(parts)},
        "verify_GBps": round(ver_gbps, 1),
        "components_ms": {"block_attention_xK": round(t_block, 4), "bidir_attention": round(t_attn, 4),
                          "verify_remask": round(t_ver, 4), "host_wall_per_step": round(wall * 1e3 / args.steps, 4)},
        "components_median_ms": {k: round(float(np.median(v)), 4) for k, v in per_step.items()},
        "components_min_ms": {k: round(float(np.min(v)), 4) for k, v in per_step.items()},
        "warm_cache_components_ms": None if not warm_rec else {
            "block_attention_xK": round(sum(m[0].elapsed_time(m[1]) for m in warm_rec) / len(warm_rec), 4),
            "bidir_attention": round(sum(m[4].elapsed_time(m[2]) for m in warm_rec) / len(warm_rec), 4),
            "verify_remask": round(sum(m[2].elapsed_time(m[3]) for m in warm_rec) / len(warm_rec), 4),
            "note": "every step on the same input set (operands that fit stay in the last-level cache); not used for any rate"},
        "block_attention_GBps": round(blk_gbps, 1),
        "block_attention_warm_GBps": None if not warm_rec else round(
            block_bytes / (sum(m[0].elapsed_time(m[1]) for m in warm_rec) / len(warm_rec) / cfg.K * 1e-3) / 1e9, 1),
        "graph_replay": None if graph_ms is None else {
            "ms_per_step": round(graph_ms, 4),
            "note": "the same steps captured once per input set and replayed as HIP graphs; ms_per_step above is the eager "
                    "sequence of calls through the Python binding"},
        "roofline": {"kernel": attn_kernel, "bound": attn_bound,
                     "achieved": round(attn_tflops, 3), "peak": round(attn_peak, 1), "unit": "TFLOP/s",
                     "frac": round(attn_tflops / attn_peak, 4), "peak_note": attn_peak_note,
                     "frac_of_bf16_peak": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                     "launch_us": round(t_attn * 1e3, 2),
                     "timing": "HIP events around the call inside every timed step (mean); back_to_back_*: the same call "
                               "as a stream of launches on rotated inputs, nothing else on the chip",
                     "back_to_back_us": None if "attention" not in stream else round(stream["attention"], 2),
                     "back_to_back_achieved": round(attn_stream_tflops, 3),
                     "traffic": profiled_traffic(config_id, "attention"),
                     "algorithmic_flops": attn_flops, "algorithmic_bytes": attn_bytes},
        "roofline_verify": {"kernel": ("verify_row_kernel" if cfg.P >= 192 else "verify_partial_kernel + verify_finalize_kernel")
                                      + {wl.KL_PROB: " + verify_klprob_kernel", wl.KL_TOPK: " + verify_topk_kernel",
                                         wl.CONF_TOPK: " + verify_topk_kernel"}.get(mode, "") + " (dd_verify_remask)",
                            "bound": "hbm", "achieved": round(ver_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                            "frac": round(ver_gbps / PEAK_HBM_GBPS, 4),
                            "launch_us": round(t_ver * 1e3, 2),
                            "back_to_back_us": None if "verify" not in stream else round(stream["verify"], 2),
                            "back_to_back_achieved": round(ver_stream_gbps, 1),
                            "traffic": profiled_traffic(config_id, "verify"),
                            "algorithmic_bytes": verify_bytes},
    }

    out["roofline_block"] = {"kernel": "dd_block_attention_cached (attn_stream_kernel / attn_wide_kernel<.., BLOCK> / "
                                       "attn_mfma_kernel + attn_combine_kernel, by shape)",
                             "bound": "hbm", "achieved": round(blk_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                             "frac": round(blk_gbps / PEAK_HBM_GBPS, 4), "traffic": profiled_traffic(config_id, "block"),
                             "launch_us": round(t_block / cfg.K * 1e3, 2),
                             "back_to_back_us": None if "block" not in stream else round(stream["block"], 2),
                             "back_to_back_achieved": round(blk_stream_gbps, 1),
                             "algorithmic_bytes": block_bytes, "cache_copies_rotated": n_caches,
                             "note": f"per call, K={cfg.K} calls per step, each on another copy of the cache (cold); "
                                     "block_attention_warm_GBps: every call on one copy"}
    if "scores" in parts:
        t_sc = max(sum(m[3].elapsed_time(m[5]) for m in rec) / len(rec), 1e-9)
        sc_bytes = 2 * cfg.P * cfg.V * eb_l
        out["components_ms"]["verify_scores"] = round(t_sc, 4)
        out["roofline_scores"] = {"kernel": "verify_row_kernel<.., KL, .., TRACKD> / verify_partial_kernel + verify_finalize_kernel (dd_verify_scores)",
                                  "bound": "hbm", "achieved": round(sc_bytes / (t_sc * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBPS,
                                  "unit": "GB/s", "frac": round(sc_bytes / (t_sc * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                                  "traffic": None, "algorithmic_bytes": sc_bytes,
                                  "note": "both logit matrices read once; outputs allocated by the binding inside the timed call"}
    if win or args.refresh_last:
        out["config"]["drafter_call"] = (f"dd_block_attention_window, {win} key rows" if win else
                                         "dd_block_attention_cached x (K-1) + dd_block_attention_refresh")
    if "unmask" in parts:
        um_gbps = unmask_bytes / (max(t_unmask, 1e-9) / cfg.K * 1e-3) / 1e9
        out["components_ms"]["unmask_xK"] = round(t_unmask, 4)
        out["roofline_unmask"] = {"kernel": "verify_row_kernel / verify_partial_kernel + unmask_select_kernel (dd_unmask)",
                                  "bound": "hbm", "achieved": round(um_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                  "frac": round(um_gbps / PEAK_HBM_GBPS, 4), "traffic": None,
                                  "algorithmic_bytes": unmask_bytes,
                                  "note": f"K={cfg.K} calls per step on the active block's drafter logits [{cfg.B * cfg.bl}, {cfg.V}]"}

    if args.layers > 0:
        out["multi_layer"] = multi_layer_cycle(args, cfg, dd, wl, torch, dict(sets[0], **caches[0]), blk_dev, qs, ks, kcs, mask, mode, tau,
                                               up(ver["logits_d"]), O, Oblk, out_mask, out_tok, out_sc)

    if not args.no_cpu_baseline:
        import oracle
        att_host = att
        rng = np.random.default_rng(args.seed)

        def rows(n):
            return np.stack([rng.integers(0, cfg.B, n), rng.integers(0, cfg.H, n), rng.integers(0, cfg.N, n)], axis=1)

        def run_attn(n):
            t0 = time.perf_counter()
            if mx:                                   # (decodes the whole tensors first: part of what this oracle costs)
                oracle.bidir_attention_mx(att_mx["Q"], att_mx["Qs"], att_mx["K"], att_mx["Ks"], att_mx["V"], att_mx["Vs"],
                                          rows=rows(n))
                return time.perf_counter() - t0
            oracle.bidir_attention(att_host["Q"], att_host["K"], att_host["V"], cfg.qk_dtype, cfg.v_dtype,
                                   att_host["q_scale"], att_host["k_scale"], rows=rows(n), v_scale=att_host["v_scale"])
            return time.perf_counter() - t0
        n0 = 64
        t0 = run_attn(n0)
        n = int(min(max(n0, args.cpu_seconds / max(t0 / n0, 1e-9)), cfg.B * cfg.H * cfg.N))
        t = run_attn(n)
        cpu_tflops = n * 4.0 * cfg.N * cfg.d / t / 1e12
        out["cpu_baseline"] = {"value": float(f"{cpu_tflops:.3e}"), "unit": "TFLOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"fp64 oracle attention on {n} random (b,h,i) query rows of this workload "
                                         f"({t:.1f} s); rate = rows*4*N*d FLOP / time"}
        # the same oracle on one thread (a shorter sample), through the OpenMP runtime the oracle is linked to
        gomp = None
        try:
            import ctypes
            gomp = ctypes.CDLL("libgomp.so.1")
            gomp.omp_set_num_threads(1)
            n1 = max(16, n // (4 * oracle.num_threads()))
            t1 = run_attn(n1)
            out["cpu_baseline"]["value_1_thread"] = float(f"{n1 * 4.0 * cfg.N * cfg.d / t1 / 1e12:.3e}")
            out["cpu_baseline"]["sample_1_thread"] = f"{n1} rows ({t1:.1f} s)"
        except OSError:
            gomp = None
        finally:
            if gomp is not None:
                gomp.omp_set_num_threads(oracle.num_threads())

        def run_ver(n):
            r = rng.integers(0, cfg.P, n)
            t0 = time.perf_counter()
            oracle.verify_scores(ver["logits_d"] if kl_mode else None, ver["logits_v"], cfg.logit_dtype, rows=r)
            return time.perf_counter() - t0
        n0 = 32
        t0 = run_ver(n0)
        n = int(min(max(n0, args.cpu_seconds / max(t0 / n0, 1e-9)), 4 * cfg.P))
        t = run_ver(n)
        out["cpu_baseline_verify"] = {"value": round(n * (2 if kl_mode else 1) * cfg.V * eb_l / t / 1e9, 4),
                                      "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
                                      "sample": f"fp64 oracle verify scores on {n} logit rows ({t:.1f} s)"}
        if gomp is not None:
            gomp.omp_set_num_threads(1)
            n1 = max(8, n // (4 * oracle.num_threads()))
            t1 = run_ver(n1)
            gomp.omp_set_num_threads(oracle.num_threads())
            out["cpu_baseline_verify"]["value_1_thread"] = round(n1 * (2 if kl_mode else 1) * cfg.V * eb_l / t1 / 1e9, 4)
            out["cpu_baseline_verify"]["sample_1_thread"] = f"{n1} logit rows ({t1:.1f} s)"
    del sets, blk_dev, caches
    gc.collect()
    torch.cuda.empty_cache()
    return out


def multi_layer_cycle(args, cfg, dd, wl, torch, s0, blk_dev, qs, ks, kcs, mask, mode, tau, ld_full, O, Oblk,
                      out_mask, out_tok, out_sc):
    """One draft-then-verify cycle (Alg. 1) of an L-layer model, attention and vocabulary passes only (the
    projections and MLPs between them are outside this library).  Every layer has its own Q/K/V and cache in HBM
    (rolled copies of the workload's tensors: same distribution, distinct memory, so that no layer finds its
    operands in a cache because the previous one used them).  Timed eagerly and as one HIP graph."""
    from paper_2604_05250_amd.step import capture_step
    L, K = args.layers, cfg.K
    kl_mode = mode in (wl.KL_THRESH, wl.KL_PROB, wl.KL_TOPK)
    layers = [{k: torch.roll(s0[k], shifts=l, dims=2) if l else s0[k] for k in ("Q", "K", "V", "Kc", "Vc")}
              for l in range(L)]
    dev = O.device
    nb = cfg.B * cfg.bl
    ld3 = ld_full.view(cfg.B, cfg.G, cfg.V)
    um = []
    rng = __import__("numpy").random.default_rng(args.seed + 78)
    for k in range(K):
        g0 = (k * cfg.bl) % max(1, cfg.G - cfg.bl + 1)
        um.append({"ld": ld3[:, g0:g0 + cfg.bl, :].contiguous().view(nb, cfg.V),
                   "mask": torch.from_numpy((rng.random(nb) < 0.5).astype("uint8")).to(dev)})
    um_mask = torch.empty(nb, dtype=torch.uint8, device=dev)
    um_tok = torch.empty(nb, dtype=torch.int32, device=dev)
    um_conf = torch.empty(nb, dtype=torch.float32, device=dev)
    um_x = torch.zeros(nb, dtype=torch.int32, device=dev)
    ld = ld_full if kl_mode else None

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def cycle(marks=None):
        if marks: marks[0].record()
        for k, b in enumerate(blk_dev):
            for lay in layers:
                if k == K - 1:      # the block is complete after its last draft step: its rows enter the cache
                    dd.dd_block_attention_refresh(b["Q"], lay["Kc"], lay["Vc"], b["bs"], b["K"], b["V"], O=Oblk,
                                                  q_scale=b["qs"], k_scale=kcs, qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
                else:
                    dd.dd_block_attention_cached(b["Q"], lay["Kc"], lay["Vc"], b["bs"], O=Oblk, Kblk=b["K"], Vblk=b["V"],
                                                 q_scale=b["qs"], k_scale=kcs, qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
            u = um[k]
            dd.dd_unmask(u["ld"], u["mask"], dd.UNMASK_THRESH, args.unmask_threshold, cfg.B, cfg.bl, x_tokens=um_x,
                         out_mask=um_mask, out_tokens=um_tok, out_conf=um_conf, logit_dtype=cfg.logit_dtype)
        if marks: marks[1].record()
        for lay in layers:
            dd.dd_bidir_attention(lay["Q"], lay["K"], lay["V"], O=O, q_scale=qs, k_scale=ks,
                                  qk_dtype=cfg.qk_dtype, v_dtype=cfg.v_dtype)
        if marks: marks[2].record()
        dd.dd_verify_remask(ld, s0["lv"], mask, mode, tau, args.seed, cfg.B, cfg.G,
                            out_mask=out_mask, out_tokens=out_tok, out_scores=out_sc, logit_dtype=cfg.logit_dtype)
        if marks: marks[3].record()

    n = max(2, min(args.steps, 5))
    for _ in range(2):
        cycle()
    torch.cuda.synchronize()
    rec = []
    for _ in range(n):
        m = [ev() for _ in range(4)]
        cycle(m)
        rec.append(m)
    torch.cuda.synchronize()
    t = [sum(m[i].elapsed_time(m[i + 1]) for m in rec) / n for i in range(3)]
    res = {"layers": L, "cycles_timed": n,
           "launch_calls_per_cycle": K * L + K + L + 1,
           "ms_per_cycle": round(sum(t), 4),
           "components_ms": {"draft_phase (K x (L block attentions + unmask))": round(t[0], 4),
                             "verifier_attention_xL": round(t[1], 4), "verify_remask": round(t[2], 4)},
           "verifier_attention_TFLOPs": round(4.0 * cfg.B * cfg.H * cfg.N * cfg.N * cfg.d * L / (t[1] * 1e-3) / 1e12, 1),
           "note": "attention and vocabulary passes only; per-layer tensors are distinct HBM buffers"}
    if not args.no_graph:
        g = capture_step(lambda: cycle())
        for _ in range(2):
            g.replay()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(n):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        res["graph_ms_per_cycle"] = round(e0.elapsed_time(e1) / n, 4)
    return res


if __name__ == "__main__":
    main()
