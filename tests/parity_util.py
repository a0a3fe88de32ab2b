"""Comparison of a GPU decode with the oracle's, row by row.

Bar: token sequences bit-exact; emitted logits within 1e-4 relative.  A row
whose tokens differ is only accepted if the oracle, walked along the GPU's
hypothesis, departs from its own argmax solely at evaluations where the chosen
logit lies less than 1e-5 (absolute, fp32) below the maximum; every such row is
reported.

The bfloat16 mode has its own two numbers (BF16_MARGIN, BF16_LOGIT_RTOL).  There
the engine and the oracle round every operand of a product to bfloat16, and
rounding is discontinuous: where the two sides' fp32 values of one operand (equal
up to summation order, ~1e-7 relative) straddle a rounding boundary, the operand
differs by a whole bfloat16 step, 2^-8 relative.  One such step in a unit of the
joint's hidden vector (magnitude up to ~6 on these workloads, output weights up
to 0.1) moves a logit by up to 0.1 * 6 * 2^-8 = 2.3e-3, one in a hidden unit of
the prediction network by about half that; a few can coincide.  Hence logits
within 1e-2 * max(1, |v|) and divergences accepted below a margin of 2e-2, every
one reported and counted.
"""
from __future__ import annotations

import numpy as np

import oracle

MARGIN = 1e-5
LOGIT_RTOL = 1e-4
BF16_MARGIN = 2e-2
BF16_LOGIT_RTOL = 1e-2


def to_lists(out, B):
    """Device tensors of one decode -> numpy rows cut at tok_len."""
    tok_len = out["tok_len"].cpu().numpy()
    cap = out["tokens"].shape[1]
    n = np.minimum(tok_len, cap)
    cut = lambda key: [out[key][b, :n[b]].cpu().numpy() for b in range(B)]
    res = dict(tok_len=tok_len, tokens=cut("tokens"), frames=cut("frames"), logits=cut("logits"),
               raw_tokens=out["tokens"].cpu().numpy())
    res["durs"] = cut("durs") if "durs" in out else [np.zeros(n[b], np.int32) for b in range(B)]
    if "logps" in out:
        res["logps"] = cut("logps")
    return res


def compare(w, net, ref, got, S, check_fill=True, margin=MARGIN, logit_rtol=LOGIT_RTOL):
    """ref: oracle.Decoded; got: to_lists(...) of the GPU run.  Returns the list
    of accepted near-tie rows; raises AssertionError on a real mismatch."""
    near_ties = []
    B = w.B
    for b in range(B):
        same = (got["tok_len"][b] == ref.tok_len[b]
                and np.array_equal(got["tokens"][b], ref.tokens[b])
                and np.array_equal(got["frames"][b], ref.frames[b])
                and np.array_equal(got["durs"][b], ref.durs[b]))
        if same:
            rv, gv = ref.scores[b].astype(np.float64), got["logits"][b].astype(np.float64)
            tol = logit_rtol * np.maximum(1.0, np.abs(rv))
            assert np.all(np.abs(rv - gv) <= tol), (
                f"row {b}: logits differ by {np.max(np.abs(rv - gv)):.3e}")
            if "logps" in got:
                rl, gl = ref.logps[b].astype(np.float64), got["logps"][b].astype(np.float64)
                # a log-probability is the difference of the top logit and the log-sum-exp of all
                # logits, each within the logit tolerance
                tol = 2 * logit_rtol * np.maximum(1.0, np.abs(rl))
                assert np.all(np.abs(rl - gl) <= tol), (
                    f"row {b}: log-probabilities differ by {np.max(np.abs(rl - gl)):.3e}")
        else:
            f = oracle.follow(net, w.enc_out[b], int(w.enc_len[b]), S, got["tokens"][b],
                              got["frames"][b], got["durs"][b] if w.model.dims.D else None, tol=margin)
            assert f.departures > 0, (
                f"row {b}: GPU hypothesis differs from the oracle's and is "
                f"{'impossible' if f.departures < 0 else 'identical under follow?'}; "
                f"oracle {ref.tokens[b][:12]} gpu {got['tokens'][b][:12]}")
            assert f.worst_gap < margin, (
                f"row {b}: GPU departs from the oracle argmax by {f.worst_gap:.3e} "
                f"(allowed < {margin}) at {f.where[:3]}")
            near_ties.append(dict(row=b, departures=f.departures, worst_gap=f.worst_gap,
                                  where=f.where[:4]))
        if check_fill:
            n = int(min(got["tok_len"][b], got["raw_tokens"].shape[1]))
            assert np.all(got["raw_tokens"][b, n:] == -1), f"row {b}: fill beyond tok_len"
    return near_ties
