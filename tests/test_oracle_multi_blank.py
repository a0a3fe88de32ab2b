"""Pins for the oracle's multi-blank rule (big-blank symbols that skip encoder frames; the
paper's related work names these models beside TDT): hand traces, an independent recursion
on random tables, reductions to the plain transducer, the score.  No GPU."""
import dataclasses
import json
import os

import numpy as np
import pytest
import torch

import oracle
import synth

HERE = os.path.dirname(os.path.abspath(__file__))
BIG = 10.0

with open(os.path.join(HERE, "golden", "multi_blank_traces.json")) as fh:
    GOLD = json.load(fh)


def table_from_cells(B, T, U, V1, NB, cells):
    """[B, T, U, V1 (last), V1 + NB]: blank everywhere except the listed cells
    [b, t, u, last (-1 = any), column]."""
    tab = np.zeros((B, T, U, V1, V1 + NB), dtype=np.float32)
    tab[..., V1 - 1] = BIG
    for b, t, u, last, col in cells:
        for la in (range(V1) if last < 0 else [last]):
            tab[b, t, u, la, :] = 0.0
            tab[b, t, u, la, col] = BIG
    return tab


@pytest.mark.parametrize("case", GOLD["cases"], ids=[c["name"] for c in GOLD["cases"]])
def test_hand_traced_multi_blank(case):
    V1, spans, S, T = GOLD["V1"], GOLD["spans"], case["S"], case["T"]
    B = len(case["len"])
    tab = table_from_cells(B, T, S * T + 2, V1, len(spans), case["cells"])
    net = oracle.TableNet(tab, V1, big_blanks=spans)
    for sched in ("label", "seq"):
        r = oracle.decode(net, net.frames(), np.array(case["len"]), S, sched, record=True)
        for b in range(B):
            assert r.tokens[b].tolist() == case["tokens"][b], (sched, b)
            assert r.frames[b].tolist() == case["frames"][b], (sched, b)
            assert len(r.records.k[b]) == case["joint_evals"][b], (sched, b)
        assert r.status == 0
    # Algorithm 1 keeps one frame index for the whole batch: the oracle refuses these models there
    with pytest.raises(ValueError):
        oracle.decode(net, net.frames(), np.array(case["len"]), S, "frame")


def walk(choice, spans, V1, length, S):
    """The decode of one utterance as a recursion on (frame, labels emitted, labels on this
    frame), written without looking at the oracle: returns [(label, frame), ...]."""
    def step(t, u, n):
        if t >= length:
            return []
        k = choice(t, u)
        if k == V1 - 1:
            return step(t + 1, u, 0)
        if k >= V1:
            return step(t + spans[k - V1], u, 0)
        if n + 1 == S:
            return [(k, t)] + step(t + 1, u + 1, 0)
        return [(k, t)] + step(t, u + 1, n + 1)
    return step(0, 0, 0)


def test_random_tables_against_the_recursion():
    rng = np.random.default_rng(7)
    V1, spans = 3, (2, 3)
    for trial in range(300):
        T, S, B = int(rng.integers(1, 7)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
        U = S * T + 2
        lens = rng.integers(0, T + 1, size=B)
        # a column per cell: labels 30 %, blank 40 %, big blanks 30 %
        cols = rng.choice(V1 + len(spans), size=(B, T, U), p=[0.15, 0.15, 0.4, 0.15, 0.15])
        tab = np.zeros((B, T, U, V1 + len(spans)), dtype=np.float32)
        np.put_along_axis(tab, cols[..., None], BIG, axis=-1)
        net = oracle.TableNet(tab, V1, big_blanks=spans)
        for sched in ("label", "seq"):
            r = oracle.decode(net, net.frames(), lens, S, sched)
            for b in range(B):
                want = walk(lambda t, u: int(cols[b, t, min(u, U - 1)]), spans, V1, int(lens[b]), S)
                assert r.tokens[b].tolist() == [k for k, _ in want], (trial, sched, b)
                assert r.frames[b].tolist() == [t for _, t in want], (trial, sched, b)


def test_big_blank_of_span_one_is_a_blank():
    """Replacing every blank choice by a big blank of span 1 changes nothing."""
    rng = np.random.default_rng(11)
    V1 = 4
    for trial in range(50):
        T, S = int(rng.integers(1, 6)), int(rng.integers(1, 4))
        U = S * T + 2
        cols = rng.choice(V1, size=(1, T, U), p=[0.15, 0.15, 0.15, 0.55])
        plain = np.zeros((1, T, U, V1), dtype=np.float32)
        np.put_along_axis(plain, cols[..., None], BIG, axis=-1)
        swapped_cols = np.where(cols == V1 - 1, V1, cols)           # blank -> the big blank
        multi = np.zeros((1, T, U, V1 + 1), dtype=np.float32)
        np.put_along_axis(multi, swapped_cols[..., None], BIG, axis=-1)
        a = oracle.decode(oracle.TableNet(plain, V1), np.arange(T, dtype=np.float32).reshape(1, T, 1),
                          np.array([T]), S, "seq")
        b = oracle.decode(oracle.TableNet(multi, V1, big_blanks=(1,)),
                          np.arange(T, dtype=np.float32).reshape(1, T, 1), np.array([T]), S, "label")
        assert a.tokens[0].tolist() == b.tokens[0].tolist() and a.frames[0].tolist() == b.frames[0].tolist()


def test_silent_big_blanks_give_the_plain_transducer():
    """LSTM nets: with the big-blank logits pushed far down, the multi-blank model decodes as
    the transducer made of its first V1 output columns does (tokens, frames and logits)."""
    w = synth.make_workload(6, B=3, T=60, len_lo=30, len_hi=60,
                            model_overrides=dict(big_blank_bias=(-1e4, -1e4)))
    d = w.model.dims
    plain = dataclasses.replace(w.model, dims=dataclasses.replace(d, big_blanks=()),
                                w_out=w.model.w_out[:d.V1].copy(), b_out=w.model.b_out[:d.V1].copy())
    a = oracle.decode(oracle.LstmNet(w.model), w.enc_out, w.enc_len, w.max_symbols, "label")
    b = oracle.decode(oracle.LstmNet(plain), w.enc_out, w.enc_len, w.max_symbols, "label")
    assert sum(map(len, a.tokens)) > 20
    for x, y in zip(a.tokens + a.frames, b.tokens + b.frames):
        assert np.array_equal(x, y)
    for x, y in zip(a.scores, b.scores):
        assert np.array_equal(x, y)


def test_schedules_agree_and_big_blanks_are_taken():
    w = synth.make_workload(6, B=4, T=120, len_lo=60, len_hi=120)
    net = oracle.LstmNet(w.model)
    seq = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "seq", record=True)
    lab = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "label", record=True)
    V1 = w.model.dims.V1
    ks = np.concatenate(seq.records.k)
    assert (ks >= V1).sum() > 20 and (ks == V1 - 1).sum() > 20 and (ks < V1 - 1).sum() > 20
    for b in range(w.B):
        assert np.array_equal(seq.tokens[b], lab.tokens[b]) and np.array_equal(seq.frames[b], lab.frames[b])
        assert np.array_equal(seq.records.k[b], lab.records.k[b])
        # the recorded walk is consistent with the rule: frames advance by 1 on a blank, by the
        # span on a big blank, and never on a label unless max_symbols labels sit on the frame
        t = seq.records.t[b]; k = seq.records.k[b]
        spans = w.model.dims.big_blanks
        for i in range(len(k) - 1):
            if k[i] == V1 - 1:
                assert t[i + 1] == t[i] + 1
            elif k[i] >= V1:
                assert t[i + 1] == t[i] + spans[k[i] - V1]
            else:
                assert t[i + 1] in (t[i], t[i] + 1)


def test_score_is_the_log_softmax_over_all_outputs():
    """The log-probability of an emitted label is taken over the labels, the blank and the big
    blanks together (they form one distribution)."""
    rng = np.random.default_rng(5)
    V1, spans, T = 4, (2, 3), 3
    tab = rng.standard_normal((1, T, 3, V1 + 2)).astype(np.float32)
    tab[0, :, :, V1 - 1] -= 4.0          # labels win mostly
    tab[0, :, :, V1:] -= 4.0
    net = oracle.TableNet(tab, V1, big_blanks=spans)
    r = oracle.decode(net, net.frames(), np.array([T]), 1, "seq")
    assert len(r.tokens[0]) >= 2
    for k, t, u, lp in zip(r.tokens[0], r.frames[0], range(len(r.tokens[0])), r.logps[0]):
        want = torch.log_softmax(torch.from_numpy(tab[0, t, min(u, 2)].astype(np.float64)), dim=0)[k]
        assert abs(float(lp) - float(want)) < 1e-5


def test_follow_on_a_multi_blank_model():
    """The follow mode on these models: the oracle's own hypothesis has no departure; an altered
    token is reported where it sits; and between labels the walk finds the chain of blanks and
    big blanks by itself."""
    w = synth.make_workload(6, B=3, T=80, len_lo=50, len_hi=80)
    net = oracle.LstmNet(w.model)
    ref = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "seq", record=True)
    V1 = w.model.dims.V1
    assert (np.concatenate(ref.records.k) >= V1).sum() > 5          # big blanks are on the way
    for b in range(w.B):
        f = oracle.follow(net, w.enc_out[b], int(w.enc_len[b]), w.max_symbols, ref.tokens[b], ref.frames[b])
        assert f.departures == 0 and f.worst_gap == 0.0, (b, f)
    b = int(np.argmax(ref.tok_len))
    tok = ref.tokens[b].copy()
    u = len(tok) // 2
    tok[u] = (tok[u] + 1) % (V1 - 1)
    f = oracle.follow(net, w.enc_out[b], int(w.enc_len[b]), w.max_symbols, tok, ref.frames[b])
    assert f.departures >= 1
    first = f.where[0]
    assert first["u"] == u and first["t"] == ref.frames[b][u]
    assert first["want"] == ref.tokens[b][u] and first["got"] == tok[u] and first["gap"] > 0


def test_follow_takes_a_big_blank_that_is_nearly_the_maximum():
    """Hand-made table (labels 0 and 1, blank 2, one big blank of span 2): on frame 0 the blank
    wins by 0.005 over the big blank; frame 1 would emit label 1; the hypothesis has label 0 on
    frame 2.  Only the big blank on frame 0 leads there.  With a tolerance above that gap the
    walk reports that one choice and its gap; with none it falls back to plain blanks and
    reports the label it had to pass over on frame 1."""
    V1, T = 3, 3
    tab = np.zeros((1, T, 3, V1 + 1), dtype=np.float32)
    tab[..., V1 - 1] = 10.0                       # blank wherever nothing else is said
    tab[0, 0, 0] = [0, 0, 10.0, 9.995]
    tab[0, 1, 0] = [0, 10.0, 0, 0]
    tab[0, 2, 0] = [10.0, 0, 0, 0]
    net = oracle.TableNet(tab, V1, big_blanks=(2,))
    x = net.frames()[0]
    own = oracle.decode(net, net.frames(), np.array([T]), 2, "seq")
    assert own.tokens[0].tolist() == [1] and own.frames[0].tolist() == [1]   # the model's own walk
    near = oracle.follow(net, x, T, 2, [0], [2], tol=0.01)
    assert near.departures == 1
    assert near.where[0]["t"] == 0 and near.where[0]["want"] == 2 and near.where[0]["got"] == 3
    assert abs(near.where[0]["gap"] - 0.005) < 1e-5 and abs(near.worst_gap - 0.005) < 1e-5
    strict = oracle.follow(net, x, T, 2, [0], [2])
    assert strict.departures == 1 and strict.where[0]["t"] == 1
    assert strict.where[0]["want"] == 1 and strict.where[0]["got"] == 2 and strict.worst_gap == 10.0
