"""Find the blank-logit bias that gives a target blank rate per joint
evaluation on a synthetic configuration, by bisection on the oracle's
per-utterance decode.  The values it prints are the ones stored in
synth/workloads.py (CONFIGS[*]['model_kw']['blank_bias']).

    python -m oracle.tune_blank_bias 2 4        # configurations to tune
"""
from __future__ import annotations

import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import oracle  # noqa: E402
import synth  # noqa: E402


def blank_stats(cfg: int, blank_bias: float, n_threads: int):
    w = synth.make_workload(cfg, model_overrides=dict(blank_bias=blank_bias))
    net = oracle.LstmNet(w.model)
    r = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "seq", record=True,
                      n_threads=n_threads)
    blank = w.model.dims.blank
    evals = sum(len(k) for k in r.records.k)
    blanks = sum(int((k == blank).sum()) for k in r.records.k)
    hist = np.zeros(w.max_symbols + 1, dtype=np.int64)
    for b in range(w.B):
        n = int(w.enc_len[b])
        per_frame = np.bincount(r.frames[b], minlength=n)[:n]
        hist += np.bincount(per_frame, minlength=w.max_symbols + 1)[:w.max_symbols + 1]
    dur_hist = None
    if w.model.dims.D:
        dur_hist = np.bincount(np.concatenate(r.records.d), minlength=5)
    return blanks / max(1, evals), r.tok_len, hist, dur_hist


def tune(cfg: int, target: float = 0.85, lo: float = 0.0, hi: float = 16.0,
         iters: int = 10, n_threads: int = 8):
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        rate, _, _, _ = blank_stats(cfg, mid, n_threads)
        print(f"  cfg {cfg}: bias {mid:.4f} -> blank rate {rate:.4f}", flush=True)
        if rate < target:
            lo = mid
        else:
            hi = mid
    # round to 2 decimals so the stored constant is short
    best = round(0.5 * (lo + hi), 2)
    rate, tok_len, hist, dur_hist = blank_stats(cfg, best, n_threads)
    print(f"cfg {cfg}: blank_bias = {best}  blank rate {rate:.4f}  tokens/utt "
          f"mean {tok_len.mean():.1f} max {tok_len.max()}  symbols-per-frame hist {hist.tolist()}"
          + (f"  duration hist {dur_hist.tolist()}" if dur_hist is not None else ""))
    return best


if __name__ == "__main__":
    for c in [int(a) for a in sys.argv[1:]] or [2, 4]:
        tune(c)
