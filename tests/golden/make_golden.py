"""Writes tests/golden/oracle_tokens.json from the CPU oracle alone (float
build, per-utterance decode).  The file guards the oracle and the synthetic
generator against silent changes; the paper prints no decode to compare with.

    python tests/golden/make_golden.py
"""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
import synth  # noqa: E402

CASES = {
    "cfg0": dict(cfg=0),
    "cfg1": dict(cfg=1),
    "cfg2_cut": dict(cfg=2, B=4, T=60, len_lo=30, len_hi=60),
    "cfg4_cut": dict(cfg=4, B=4, T=60, len_lo=30, len_hi=60),
    "cfg6_cut": dict(cfg=6, B=4, T=60, len_lo=30, len_hi=60),      # multi-blank
}


def run(spec):
    spec = dict(spec)
    w = synth.make_workload(spec.pop("cfg"), **spec)
    r = oracle.decode(oracle.LstmNet(w.model), w.enc_out, w.enc_len, w.max_symbols, "seq")
    return dict(enc_len=w.enc_len.tolist(), tokens=[t.tolist() for t in r.tokens],
                frames=[f.tolist() for f in r.frames], durs=[d.tolist() for d in r.durs])


if __name__ == "__main__":
    out = {name: run(spec) for name, spec in CASES.items()}
    with open(os.path.join(HERE, "oracle_tokens.json"), "w") as fh:
        json.dump(out, fh)
    print({k: [len(t) for t in v["tokens"]] for k, v in out.items()})
