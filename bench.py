#!/usr/bin/env python3
"""Benchmark of the RNN-T greedy-decoding hot path on one MI355X.

A step is one whole decode call (encoder-side joint projection + persistent
decode kernel) over the Parakeet-RNN-T-1.1B-shaped synthetic batch (B = 32,
T ~ U[200, 500], F = 1024), inputs and packed weights resident in HBM.  Prints
one JSON line: frames/s with the roofline of the decode kernel and the CPU
oracle timed on the host cores beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--variant frame|label|tdt]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# Phase timers of a profile build (rnnt_engine_phase_timers), in the order of their slots.
# "general" = prediction step of teams with more than four utterances (barriers, inputs filled
# from the exchange buffers); the fast step of smaller teams leaves those slots at zero.
PHASES = ["pred: stage-0 input filled (general)", "pred: recurrent stage of all layers",
          "pred: layer-0 cell and store", "pred: barrier (general)",
          "pred: hidden vectors of the layer below received", "pred: input stage of a layer",
          "pred: cell of a layer and store", "pred: barrier (general)",
          "pred: top hidden vectors received", "pred: prediction-side projection stage",
          "pred: q stored", "pred: barrier (general)", "pred: q received",
          "joint: z rows complete (work-group barrier)", "joint: output stage", "joint: candidates scanned, partial published",
          "control: results walked, labels emitted", "joint: argmax exchange", "control: before a step",
          "control: row states exchanged between joint groups", "joint: candidates from partial sums",
          "unused", "joint: frame loads and first weight loads issued", "joint: z formed"]


def algorithmic_bytes(dims, B, variant, enc_len, tok_frames, S, wbytes=4):
    """Bytes the method must touch per launch: every weight once per batched
    step of the schedule (Algorithm 1 / label looping run on the whole batch),
    recurrent state read and written, embedding and projected-frame rows."""
    H, L, J, E, nout = dims.H, dims.L, dims.J, dims.E, dims.n_out
    # matrices in their stored width (layer 0's input weights are never stored compactly),
    # biases, state and gathered rows in fp32
    lstm_w = sum(4 * H * (4 * E if l == 0 else wbytes * H) + 4 * H * wbytes * H + 4 * 8 * H
                 for l in range(L))
    pred_bytes = lstm_w + wbytes * J * H + 4 * J + 4 * (2 * L * 2 * B * H) + 4 * B * E
    joint_bytes = wbytes * nout * J + 4 * nout + 4 * B * J
    counts = [np.bincount(f, minlength=int(n))[:int(n)] if int(n) else np.zeros(0, int)
              for f, n in zip(tok_frames, enc_len)]
    tok = np.array([len(f) for f in tok_frames])
    if variant == "frame":
        steps = 0
        for t in range(int(enc_len.max())):
            per_row = [min(S, int(c[t]) + 1) for c, n in zip(counts, enc_len) if t < n]
            steps += max(per_row)
        pred_steps, joint_steps = steps, steps      # prediction() runs at every inner step
    else:
        pred_steps = int(tok.max()) + 1
        if variant == "tdt":
            joint_steps = int(tok.max()) + 1        # lower bound: one evaluation per label
        else:
            forced = np.array([int((c == S).sum()) for c in counts])
            joint_steps = int((enc_len + tok - forced).max())
    pred_flops = 2 * B * (sum(4 * H * ((E if l == 0 else H) + H) for l in range(L)) + J * H)
    joint_flops = 2 * B * J * nout
    return (pred_steps * pred_bytes + joint_steps * joint_bytes, pred_steps, joint_steps,
            pred_steps * pred_flops + joint_steps * joint_flops)


def issued_weight_bytes(dims, stats, bytes_per_weight=4):
    """Bytes of the steps the device ran, from its own step counters: every prediction
    step of a team streams the recurrent and upper-layer LSTM weights and W_pred (layer 0's
    input weights are folded into a table and never stream), every joint step of a joint
    group streams W_out.  The joint counter covers the first group of each team; the other
    groups are taken to be alike.  Part of it is served by the L2 of an XCD that several
    teams share, so the profiled HBM traffic is lower."""
    H, L, J = dims.H, dims.L, dims.J
    pred = bytes_per_weight * (sum(4 * H * (H + (H if l else 0)) for l in range(L)) + J * H)
    joint = bytes_per_weight * dims.n_out * J
    return stats["pred_steps"] * pred + stats["joint_steps"] * stats["joint_groups"] * joint


def mfma_fraction(dims, stats, B, dec_ms):
    """Multiply-adds of the counted steps (rows a team really has, samples the joint really
    evaluated; the folded layer-0 input product is a gather and not counted)."""
    H, L, J = dims.H, dims.L, dims.J
    w_pred_step = sum(4 * H * (H + (H if l else 0)) for l in range(L)) + J * H
    rows_per_team = B / min(B, stats["n_teams"])
    flops = 2.0 * (stats["pred_steps"] * rows_per_team * w_pred_step +
                   stats["joint_samples"] * stats["joint_groups"] * dims.n_out * J)
    ach = flops / (dec_ms * 1e-3) / 1e12
    return {"useful_flops": flops, "peak": 157.3, "unit": "TFLOP/s", "achieved": ach,
            "frac": ach / 157.3}


def profiled(variant, key):
    """A `key: value` figure from the committed rocprofv3 summary of the decode kernel for this
    variant (profiles/decode_kernel_parakeet_b32_*.md), or None when there is none."""
    tag = {"frame": "frame_looping", "label": "label_looping", "tdt": "tdt_label_looping"}[variant]
    path = os.path.join(ROOT, "profiles", f"decode_kernel_parakeet_b32_{tag}.md")
    try:
        for ln in open(path):
            if ln.startswith(key + ":"):
                return float(ln.split(":")[1])
    except OSError:
        pass
    return None


def measured_ceiling(key):
    """A figure from the committed output of `bench.py --probes` (profiles/probes.md), or None."""
    try:
        for ln in open(os.path.join(ROOT, "profiles", "probes.md")):
            if ln.startswith(key + ":"):
                return float(ln.split(":")[1])
    except OSError:
        pass
    return None


def minimum_schedule_bytes(dims, B, variant, enc_len, tok_frames, S, wbytes=4):
    """The method's own minimum: the fewest batched steps any exact schedule needs on this
    batch (label looping: one prediction step per label of the utterance with the most labels,
    plus the first; one joint step per frame and per label of the utterance that needs the
    most), each touching every weight once."""
    return algorithmic_bytes(dims, B, "tdt" if variant == "tdt" else "label", enc_len, tok_frames, S, wbytes)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--variant", default="frame", choices=["frame", "label", "tdt"])
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--storage", default="fp32", choices=["fp32", "bf16", "fp8", "fp4"],
                    help="storage of the streamed weights for the timed decoder; bf16 / fp8 decode "
                         "another model (the one with weights rounded to that format), so their "
                         "figures stand beside the fp32 headline, never for it")
    ap.add_argument("--arithmetic", default="f32", choices=["f32", "bf16"],
                    help="bf16: the engine's RNNT_FLAG_BF16_ARITHMETIC mode (weights and every input "
                         "of a dense product rounded to bfloat16, float accumulation); a reduced-"
                         "precision mode, so its figures stand beside the f32 headline, never for it")
    ap.add_argument("--plain-launch", action="store_true",
                    help="create the engines with RNNT_FLAG_PLAIN_LAUNCH (ordinary instead of "
                         "cooperative launch): for runs under rocprofv3, see the header")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-variants", action="store_true",
                    help="time the chosen decoder only (profiler runs: one decode kernel per trace)")
    ap.add_argument("--phases", action="store_true",
                    help="with a library built with RNNT_PROFILE=1: add the phase timers of the "
                         "slowest team's first work-group to the line (microseconds per launch)")
    ap.add_argument("--probes", action="store_true",
                    help="run the library's microbenchmarks instead of the decode (stream out of "
                         "L2 and out of HBM, team exchanges, fp32 MFMA rate) and print them as JSON: "
                         "the measured ceilings the roofline figures are read against")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy instead of the decode: under rocprofv3 "
                         "--pmc it gives the FETCH_SIZE / WRITE_SIZE reading for a known traffic")
    ap.add_argument("--sweep", action="store_true",
                    help="also time Algorithm 1 and label looping over batch sizes 1..128 on the "
                         "typical workload and on the adversarial batches; listed under 'sweep'")
    ap.add_argument("--team-sweep", action="store_true",
                    help="instead of the benchmark line: time the decoders under other team layouts "
                         "(rnnt_engine_configure) than the default ones, one utterance and B = 32, and "
                         "print them as JSON (the figures behind the default layouts)")
    ap.add_argument("--all-variants", action="store_true",
                    help="also time label looping with log-probabilities, the single-layer second "
                         "workload and the three decoders with bf16-stored and 8-bit (e4m3) stored "
                         "weights, listed under 'variants'")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (utterances are independent, so a batch "
              "shards over GPUs with no exchange; each GPU would run this same path on its "
              "share); run with --gpus 1", file=sys.stderr)
        return 2

    import torch

    import paper_2406_03791_amd as pkg
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    pkg.load_library()

    if args.probes:
        torch.zeros(1, device="cuda")              # the device is initialised through torch first
        l2, l2_cu = pkg.rnnt_probe_stream(True)
        hbm, hbm_cu = pkg.rnnt_probe_stream(False)
        exch = []
        for ts in (8, 16, 32, 64, 256):
            for tagged in (False, True):
                exch.append({"team_size": ts, "floats": 640, "tagged_words": tagged,
                             "us_per_exchange": pkg.rnnt_probe_exchange(ts, 640, tagged)})
        for rows, ts in ((2, 16), (4, 32), (16, 16)):
            for tagged in (False, True):
                exch.append({"team_size": ts, "floats": 640 * rows, "tagged_words": tagged,
                             "us_per_exchange": pkg.rnnt_probe_exchange(ts, 640 * rows, tagged)})
        print(json.dumps({"probes": {
            "stream_from_l2": {"GBs": l2, "GBs_per_cu": l2_cu,
                               "pattern": "16 slices of 1.5 MiB, slice i%16 for work-group i, 64 passes"},
            "stream_from_hbm": {"GBs": hbm, "GBs_per_cu": hbm_cu, "pattern": "8 MiB per work-group, one pass"},
            "exchange": exch,
            "mfma_f32_tflops": {"4x4x1_16_blocks": pkg.rnnt_probe_mfma(0), "32x32x2": pkg.rnnt_probe_mfma(1),
                                "published_peak": 157.3}}}))
        return 0

    if args.team_sweep:
        rows = []
        for variant, B, layouts in (("label", 1, ((8, 1), (4, 1), (2, 1), (1, 1))),
                                    ("label", 32, ((16, 2), (16, 1), (8, 4), (8, 2), (32, 1))),
                                    ("frame", 32, ((32, 1), (16, 1), (8, 1))),
                                    ("tdt", 32, ((16, 2), (8, 4), (32, 1)))):
            w = synth.make_workload({"frame": 2, "label": 3, "tdt": 4}[variant], B=B)
            eng = pkg.Engine(w.model, w.B, w.T)
            enc = torch.from_numpy(w.enc_out).cuda().contiguous()
            ln = torch.from_numpy(w.enc_len).cuda()
            out = eng.alloc_outputs(w.B, w.T * w.max_symbols)
            ref = None
            for n_teams, groups in layouts:
                try:
                    eng.configure(n_teams=n_teams, joint_groups=groups if variant != "frame" else 0)
                except Exception as exc:                 # a layout the LDS cannot hold
                    rows.append({"variant": variant, "B": B, "n_teams": n_teams, "joint_groups": groups,
                                 "refused": str(exc)})
                    continue
                ms = []
                for i in range(8):
                    eng.decode(variant, enc, ln, w.max_symbols, out=out)
                    st = eng.stats()
                    if i >= 2:
                        ms.append(st["decode_ms"])
                tok = out["tokens"].cpu().numpy()
                ref = tok if ref is None else ref
                rows.append({"variant": variant, "B": B, "n_teams": st["n_teams"], "team_size": st["team_size"],
                             "joint_groups": st["joint_groups"], "decode_ms": float(np.median(ms)),
                             "decode_ms_min": float(np.min(ms)), "status": eng.status(),
                             "tokens_equal_first_layout": bool(np.array_equal(tok, ref))})
            eng.close()
        print(json.dumps({"team_sweep": rows}))
        return 0

    if args.copy_calibration:
        n = 1 << 28                                    # 2^28 floats = 1 GiB read + 1 GiB written
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 4 * n, "bytes_written": 4 * n,
                                               "launches": 4}}))
        return 0

    def run_variant(variant, steps, warmup, storage="fp32", logp=False, cfg=None, arithmetic="f32"):
        cfg = {"frame": 2, "label": 3, "tdt": 4}[variant] if cfg is None else cfg
        w = synth.make_workload(cfg, B=args.batch)
        w_orig = w
        flags = 0
        if storage == "fp8" and arithmetic == "bf16":
            # weight-only 8-bit quantisation: every streamed matrix row by row to e4m3 codes with a
            # power-of-two scale (the library's host-side quantiser), kept in that form by the engine
            import dataclasses
            flags = pkg.RNNT_FLAG_FP8_WEIGHTS
            w = dataclasses.replace(w, model=synth.with_streamed_weights(
                w.model, lambda a: pkg.rnnt_quantize_rows_e4m3(a)[0]))
        elif storage == "fp4":
            # weight-only 4-bit quantisation: e2m1 codes with a power-of-two scale per 128 weights
            import dataclasses
            flags = pkg.RNNT_FLAG_FP4_WEIGHTS
            w = dataclasses.replace(w, model=synth.with_streamed_weights(
                w.model, lambda a: pkg.rnnt_quantize_blocks_e2m1(a)[0]))
        elif storage != "fp32":
            # the model a bf16 / 8-bit e4m3 checkpoint would give for the streamed matrices, kept
            # in that format by the engine (lossless); fp32 arithmetic, checked against the
            # oracle on that model
            import dataclasses
            transform, flags = {
                "bf16": (synth.with_bf16_streamed_weights, pkg.RNNT_FLAG_BF16_WEIGHTS),
                "fp8": (synth.with_fp8_streamed_weights, pkg.RNNT_FLAG_FP8_WEIGHTS)}[storage]
            w = dataclasses.replace(w, model=transform(w.model))
        if arithmetic == "bf16":
            flags |= pkg.RNNT_FLAG_BF16_ARITHMETIC
        if args.plain_launch:
            flags |= pkg.RNNT_FLAG_PLAIN_LAUNCH
        eng = pkg.Engine(w.model, w.B, w.T, flags=flags)
        enc = torch.from_numpy(w.enc_out).cuda().contiguous()
        ln = torch.from_numpy(w.enc_len).cuda()
        out = eng.alloc_outputs(w.B, w.T * w.max_symbols)
        for _ in range(warmup):
            eng.decode(variant, enc, ln, w.max_symbols, out=out, logp=logp)
        torch.cuda.synchronize()
        dec_ms, proj_ms = [], []
        t0 = time.perf_counter()
        for _ in range(steps):
            eng.decode(variant, enc, ln, w.max_symbols, out=out, logp=logp)
            # the stats call waits for the device: each step is timed on its own events
            st = eng.stats()
            dec_ms.append(st["decode_ms"])
            proj_ms.append(st["projection_ms"])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        status = eng.status()
        tok_len = out["tok_len"].cpu().numpy()
        frames = [out["frames"][b, :tok_len[b]].cpu().numpy() for b in range(w.B)]
        tokens = [out["tokens"][b, :tok_len[b]].cpu().numpy() for b in range(w.B)]
        phases = None
        if args.phases:
            per_team = [eng.phase_timers(t) for t in range(st["n_teams"])]
            slow = max(range(len(per_team)), key=lambda t: sum(per_team[t]))
            phases = {"team": slow, "us": dict(zip(PHASES, per_team[slow]))}
        res = dict(w=w, w_orig=w_orig, wall=wall, steps=steps, phases=phases, dec_ms=float(np.median(dec_ms)),
                   proj_ms=float(np.median(proj_ms)), dec_ms_min=float(np.min(dec_ms)), stats=st,
                   status=status, frames=frames, tokens=tokens, tok_len=tok_len)
        eng.close()
        return res

    if args.storage == "fp4" and args.arithmetic != "bf16":
        print("bench.py: --storage fp4 exists for --arithmetic bf16 only", file=sys.stderr)
        return 2
    if args.arithmetic == "bf16" and args.storage == "bf16":
        print("bench.py: --arithmetic bf16 stores its weights as bf16 already; leave --storage "
              "at fp32, or give fp8 for the weight-only 8-bit form of the mode", file=sys.stderr)
        return 2
    r = run_variant(args.variant, args.steps, args.warmup, storage=args.storage,
                    arithmetic=args.arithmetic)
    w = r["w"]
    n_frames = w.frames
    ms_per_step = 1e3 * r["wall"] / r["steps"]
    value = n_frames * r["steps"] / r["wall"]
    wb = {"fp32": 4, "bf16": 2, "fp8": 1, "fp4": 0.5}[args.storage]
    if args.arithmetic == "bf16" and args.storage == "fp32":
        wb = 2
    lit_bytes, lit_pred, lit_joint, _ = algorithmic_bytes(
        w.model.dims, w.B, args.variant, w.enc_len, r["frames"], w.max_symbols, wb)
    min_bytes, min_pred, min_joint, _ = minimum_schedule_bytes(
        w.model.dims, w.B, args.variant, w.enc_len, r["frames"], w.max_symbols, wb)
    # bytes of the steps the device counted (every team step reads its streamed weights once,
    # out of the L2 of its XCD)
    step_bytes = issued_weight_bytes(w.model.dims, r["stats"], wb)
    t_dec = r["dec_ms"] * 1e-3
    achieved = min_bytes / t_dec / 1e9
    std = args.batch == 32 and args.storage == "fp32" and args.arithmetic == "f32"
    traffic = profiled(args.variant, "decode_kernel_traffic_bytes_per_launch") if std else None
    l2_peak = measured_ceiling("stream_from_l2_GBs")
    line = {
        "metric": "encoder frames decoded/sec, Parakeet-1.1B decoder shape, B=32",
        "value": value, "unit": "frames/s", "n_gpus": 1, "steps": r["steps"],
        "warmup": args.warmup, "ms_per_step": ms_per_step, "us_per_frame": 1e6 / value,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.arithmetic,
        "data": "synthetic",
        "timing_note": "value and ms_per_step are host wall time over the timed calls, each followed "
                       "by rnnt_engine_stats (a device synchronisation and a small copy), so they "
                       "are conservative; kernel_ms are HIP-event times around each launch, median "
                       "and minimum over the timed calls",
        "config": {"workload": f"config {dict(frame=2, label=3, tdt=4)[args.variant]}: "
                               f"{w.name}, B={w.B}, T<={w.T}, frames={n_frames}, "
                               f"max_symbols={w.max_symbols}, variant={args.variant}" +
                               ("" if args.storage == "fp32" else
                                f", streamed weights rounded to and stored as {args.storage} "
                                f"(another model than the headline's" +
                                ("; fp32 arithmetic)" if args.arithmetic == "f32" else ")")) +
                               ("" if args.arithmetic == "f32" else
                                ", bfloat16 products with float accumulation (reduced precision: "
                                "not the headline)"),
                   "tokens": int(r["tok_len"].sum()), "device_status": r["status"],
                   "kernel_ms": {"decode": r["dec_ms"], "decode_min": r["dec_ms_min"],
                                 "encoder_projection": r["proj_ms"]},
                   "engine": r["stats"]},
        # The numerator is the method's minimum: the bytes of the fewest batched steps an exact
        # schedule needs on this batch, every weight once per step.  The kernel is not bound by
        # HBM: its weight streams are served by the XCD L2s and its time is the latency of the
        # longest utterance's chain of dependent steps; the fraction says how far that leaves it
        # from streaming the minimum schedule at HBM speed.
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "decode_kernel", "algorithmic_bytes": min_bytes,
                     "bytes_from": "minimum batched schedule: prediction steps = most labels of an "
                                   "utterance + 1, joint steps = most (frames + labels) of an "
                                   "utterance, each step touching every weight once",
                     "limited_by": "latency of the dependent step chain of the longest utterance "
                                   "(weight streams come out of the XCD L2s, not HBM)",
                     "minimum_schedule": {"prediction_steps": min_pred, "joint_steps": min_joint},
                     "hbm_measured": None if traffic is None else {
                         "bytes": traffic, "GBs": traffic / t_dec / 1e9,
                         "frac": traffic / t_dec / 1e9 / HBM_PEAK_GBS},
                     "l2_stream": {"served_bytes": step_bytes, "achieved": step_bytes / t_dec / 1e9,
                                   "peak_measured": l2_peak, "unit": "GB/s",
                                   "frac": None if not l2_peak else step_bytes / t_dec / 1e9 / l2_peak,
                                   "note": "bytes of the team steps the device counted x weights "
                                           "streamed per step; peak from bench.py --probes"},
                     "literal_schedule": {"prediction_steps": lit_pred, "joint_steps": lit_joint,
                                          "bytes": lit_bytes, "achieved": lit_bytes / t_dec / 1e9,
                                          "note": "the timed decoder's own schedule run on the whole "
                                                  "batch in lock-step; above the peak means the "
                                                  "kernel does less than that schedule (unchanged "
                                                  "prediction steps skipped, utterances independent)"},
                     # useful flops of the counted steps against the fp32 matrix peak: small, the
                     # path is not a dense contraction at these batch sizes (the counter-based
                     # figure of the MFMA work executed, row padding included, is in profiles/)
                     "mfma": mfma_fraction(w.model.dims, r["stats"], w.B, r["dec_ms"]),
                     "gpu_busy_frac": (r["dec_ms"] + r["proj_ms"]) / ms_per_step,
                     "us_per_lockstep_frame": 1e3 * ms_per_step / int(w.enc_len.max())},
    }
    if r["phases"]:
        line["phases"] = r["phases"]
    # the other decoders on their configurations (label looping decodes config 2's inputs and
    # emits the same tokens; TDT is config 4's model): always listed beside the headline
    line["variants"] = {}
    for v in ("frame", "label", "tdt"):
        if v == args.variant or args.no_variants:
            continue
        rv = run_variant(v, max(3, args.steps // 2), 2)
        line["variants"][v] = {"frames_per_s": rv["w"].frames * rv["steps"] / rv["wall"],
                               "decode_ms": rv["dec_ms"], "status": rv["status"]}
    # the engine's bfloat16 mode (bf16 MFMA, float accumulation): reduced precision, so it is
    # listed beside the f32 figures and never stands for them
    for v in ("frame", "label", "tdt"):
        if args.no_variants or args.arithmetic == "bf16":
            break
        rv = run_variant(v, max(3, args.steps // 2), 2, arithmetic="bf16")
        line["variants"][v + "_bf16_arithmetic"] = {
            "frames_per_s": rv["w"].frames * rv["steps"] / rv["wall"], "decode_ms": rv["dec_ms"],
            "tokens": int(rv["tok_len"].sum()), "status": rv["status"]}
        # the same mode with the streamed weights quantised to e4m3 codes with row scales
        rv = run_variant(v, max(3, args.steps // 2), 2, arithmetic="bf16", storage="fp8")
        line["variants"][v + "_bf16_arithmetic_e4m3_weights"] = {
            "frames_per_s": rv["w"].frames * rv["steps"] / rv["wall"], "decode_ms": rv["dec_ms"],
            "tokens": int(rv["tok_len"].sum()), "status": rv["status"]}
        # and quantised to e2m1 codes with a scale per 128 weights
        rv = run_variant(v, max(3, args.steps // 2), 2, arithmetic="bf16", storage="fp4")
        line["variants"][v + "_bf16_arithmetic_e2m1_weights"] = {
            "frames_per_s": rv["w"].frames * rv["steps"] / rv["wall"], "decode_ms": rv["dec_ms"],
            "tokens": int(rv["tok_len"].sum()), "status": rv["status"]}
    if args.all_variants:
        # label looping that also returns the log-probability of every label (fused log-sum-exp)
        rv = run_variant("label", max(3, args.steps // 2), 2, logp=True)
        line["variants"]["label_with_logp"] = {
            "frames_per_s": rv["w"].frames * rv["steps"] / rv["wall"], "decode_ms": rv["dec_ms"],
            "status": rv["status"]}
        # second workload: the single-layer model that stands in for the paper's smaller one
        for v in ("frame", "label"):
            rv = run_variant(v, max(3, args.steps // 2), 2, cfg=5)
            line["variants"][v + "_small_model"] = {
                "frames_per_s": rv["w"].frames * rv["steps"] / rv["wall"], "decode_ms": rv["dec_ms"],
                "frames": rv["w"].frames, "tokens": int(rv["tok_len"].sum()), "status": rv["status"]}
        # the bfloat16 mode (bf16 and e4m3 storage) with its divergence counts: rows whose tokens are
        # those of the oracle's emulation of the same arithmetic, and rows whose tokens differ
        # from the fp32 oracle's on the same model
        import oracle as _orc
        for v in ("frame", "label", "tdt"):
            for storage in ("fp32", "fp8", "fp4"):
                rv = run_variant(v, max(3, args.steps // 2), 2, arithmetic="bf16", storage=storage)
                wv = rv["w"]
                nthr = min(16, os.cpu_count() or 1)
                emul = _orc.decode(_orc.LstmNet(wv.model, bf16=True), wv.enc_out, wv.enc_len,
                                   wv.max_symbols, "seq", n_threads=nthr)
                f32 = _orc.decode(_orc.LstmNet(wv.model), wv.enc_out, wv.enc_len, wv.max_symbols,
                                  "seq", n_threads=nthr)
                same = sum(int(np.array_equal(emul.tokens[b], rv["tokens"][b])) for b in range(wv.B))
                moved = sum(int(not np.array_equal(f32.tokens[b], rv["tokens"][b])) for b in range(wv.B))
                name = v + "_bf16_arithmetic" + {"fp32": "", "fp8": "_e4m3_weights", "fp4": "_e2m1_weights"}[storage]
                extra = {}
                if storage != "fp32":
                    # against the fp32 decode of the model before it was quantised
                    wo = rv["w_orig"]
                    f32o = _orc.decode(_orc.LstmNet(wo.model), wo.enc_out, wo.enc_len, wo.max_symbols,
                                       "seq", n_threads=nthr)
                    extra = {"rows_differing_from_fp32_oracle_on_unquantised_model":
                             sum(int(not np.array_equal(f32o.tokens[b], rv["tokens"][b])) for b in range(wv.B)),
                             "tokens_fp32_oracle_unquantised_model": int(f32o.tok_len.sum())}
                line["variants"][name + "_divergence"] = {
                    "decode_ms": rv["dec_ms"], "tokens": int(rv["tok_len"].sum()),
                    "tokens_fp32_oracle_same_model": int(f32.tok_len.sum()),
                    "rows": wv.B, "rows_token_identical_to_emulating_oracle": same,
                    "rows_differing_from_fp32_oracle": moved,
                    "max_pred_steps": rv["stats"]["max_pred_steps"],
                    "max_joint_steps": rv["stats"]["max_joint_steps"], "status": rv["status"], **extra}
        # the multi-blank transducer of configuration 6 (two big blanks that skip 2 and 4 frames)
        rv = run_variant("label", max(3, args.steps // 2), 2, cfg=6)
        line["variants"]["label_multi_blank_model"] = {
            "frames_per_s": rv["w"].frames * rv["steps"] / rv["wall"], "decode_ms": rv["dec_ms"],
            "frames": rv["w"].frames, "tokens": int(rv["tok_len"].sum()),
            "max_pred_steps": rv["stats"]["max_pred_steps"],
            "max_joint_steps": rv["stats"]["max_joint_steps"], "status": rv["status"]}
        # the same decoders on the models with bf16-valued / e4m3-valued streamed weights, stored
        # in that format: other models (their tokens differ from the fp32 model's), reported
        # beside, never as value
        import oracle as _oracle
        for v, storage in [(v, s) for s in ("bf16", "fp8") for v in ("frame", "label", "tdt")]:
            rv = run_variant(v, max(3, args.steps // 2), 2, storage=storage)
            wv = rv["w"]
            ref = _oracle.decode(_oracle.LstmNet(wv.model), wv.enc_out, wv.enc_len, wv.max_symbols,
                                 "seq", n_threads=min(16, os.cpu_count() or 1))
            same = sum(int(np.array_equal(ref.tokens[b], rv["tokens"][b])) for b in range(wv.B))
            line["variants"][f"{v}_{storage}_weights"] = {
                "frames_per_s": wv.frames * rv["steps"] / rv["wall"], "decode_ms": rv["dec_ms"],
                "max_pred_steps": rv["stats"]["max_pred_steps"],
                "max_joint_steps": rv["stats"]["max_joint_steps"], "tokens": int(rv["tok_len"].sum()),
                "status": rv["status"], "rows_token_identical_to_oracle_on_same_model": same}
    if args.sweep:
        # batch-size and input-pattern sweep: how the two schedules take a slow row, the
        # alternating batch and an input that emits max_symbols labels on every frame
        line["sweep"] = []
        for kind in ("typical",) + tuple(synth.PATTERNS[1:]):
            for B in (1, 8, 32, 128) + ((256,) if kind == "typical" else ()):   # 256: two launches of 128
                if kind == "typical":
                    ws = synth.make_workload(2, B=B)
                else:
                    ws = synth.make_adversarial(kind, cfg=2, B=B, T=200)
                eng = pkg.Engine(ws.model, ws.B, ws.T)
                enc = torch.from_numpy(ws.enc_out).cuda().contiguous()
                ln = torch.from_numpy(ws.enc_len).cuda()
                out = eng.alloc_outputs(ws.B, ws.T * ws.max_symbols)
                for v in ("frame", "label"):
                    ms = []
                    for i in range(4):
                        eng.decode(v, enc, ln, ws.max_symbols, out=out)
                        st = eng.stats()
                        if i:
                            ms.append(st["decode_ms"] + st["projection_ms"])
                    line["sweep"].append({
                        "workload": kind, "B": B, "T": ws.T, "variant": v, "frames": ws.frames,
                        "tokens": int(out["tok_len"].sum().item()), "call_ms": float(np.median(ms)),
                        "frames_per_s": ws.frames / (float(np.median(ms)) * 1e-3),
                        "max_pred_steps": st["max_pred_steps"], "max_joint_steps": st["max_joint_steps"],
                        "status": eng.status()})
                eng.close()
    if not args.no_cpu_baseline:
        import oracle
        cores = min(16, os.cpu_count() or 1)
        # in the bfloat16 mode the reference is the oracle's emulation of that arithmetic (token
        # identity is then not expected on every row: near-ties resolve by rounding order)
        net = oracle.LstmNet(w.model, bf16=args.arithmetic == "bf16")
        sched = "seq"
        # repeat the batch until about 12 CPU-seconds have been spent (at most 8 passes)
        passes, dt = 0, 0.0
        while passes < 8 and dt * cores < 12.0:
            t0 = time.perf_counter()
            ref = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, sched, n_threads=cores)
            dt += time.perf_counter() - t0
            passes += 1
        same = sum(int(np.array_equal(ref.tokens[b], r["tokens"][b])) for b in range(w.B))
        line["cpu_baseline"] = {"value": passes * n_frames / dt, "unit": "frames/s",
                                "cores": cores, "kind": "oracle",
                                "sample": f"the whole batch ({w.B} utterances, {n_frames} frames) "
                                          f"{passes} times, per-utterance decode, one utterance "
                                          f"per thread, {dt:.2f} s wall in total",
                                "rows_token_identical_to_gpu": same}
        # one thread: the literal schedule of the timed decoder and the per-utterance
        # schedule, on the two shortest utterances of the batch
        nb = min(2, w.B)
        pick = np.argsort(w.enc_len, kind="stable")[:nb]
        xs, ls = np.ascontiguousarray(w.enc_out[pick]), np.ascontiguousarray(w.enc_len[pick])
        literal = {"frame": "frame", "label": "label", "tdt": "tdt"}[args.variant]
        one = {}
        for name, s in (("literal_schedule", literal), ("per_utterance", "seq")):
            t0 = time.perf_counter()
            oracle.decode(net, xs, ls, w.max_symbols, s, n_threads=1)
            one[name] = int(ls.sum()) / (time.perf_counter() - t0)
        line["cpu_baseline"]["one_thread"] = dict(
            one, unit="frames/s", sample=f"the {nb} shortest utterances ({int(ls.sum())} frames)")
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
