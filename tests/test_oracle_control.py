"""Pins for the oracle's loop control (Algorithm 1, label looping, TDT, the
per-utterance definition), using table-driven networks so that only the control
flow is under test.  No GPU."""
import itertools
import json
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
BIG = 10.0


def table_from_choices(B, T, U, V1, D, cells):
    """Logit table [B,T,U,V1(last),V1+D]: every cell chooses blank / duration
    index 0 unless listed in `cells` as [b,t,u,last(-1 = any),choice,dur_idx]."""
    tab = np.zeros((B, T, U, V1, V1 + D), dtype=np.float32)
    tab[..., V1 - 1] = BIG
    if D:
        tab[..., V1] = BIG
    for b, t, u, last, choice, di in cells:
        lasts = range(V1) if last < 0 else [last]
        for la in lasts:
            row = tab[b, t, u, la]
            row[:] = 0.0
            row[choice] = BIG
            if D:
                row[V1 + di] = BIG
    return tab


def schedules_for(D):
    return ["label", "seq"] if D else ["frame", "label", "seq"]


with open(os.path.join(HERE, "golden", "hand_traces.json")) as fh:
    HAND = json.load(fh)["cases"]


@pytest.mark.parametrize("case", HAND, ids=[c["name"] for c in HAND])
def test_hand_traced_cases(case):
    V1, dur, S, T = case["V1"], case["durations"], case["S"], case["T"]
    B = len(case["len"])
    U = S * T + 2
    tab = table_from_choices(B, T, U, V1, len(dur), case["cells"])
    net = oracle.TableNet(tab, V1, dur)
    for sched in schedules_for(len(dur)):
        r = oracle.decode(net, net.frames(), np.array(case["len"]), S, sched, record=True)
        for b in range(B):
            assert r.tokens[b].tolist() == case["tokens"][b], (sched, b)
            assert r.frames[b].tolist() == case["frames"][b], (sched, b)
            if dur:
                assert r.durs[b].tolist() == case["durs"][b], (sched, b)
            assert len(r.records.k[b]) == case["joint_evals"][b], (sched, b)
        assert r.status == 0
    if not dur:
        # Algorithm 1 as written (every row evaluated at every inner step) and the form that
        # passes over masked rows give the same outputs and the same records
        lit = oracle.decode(net, net.frames(), np.array(case["len"]), S, "frame", record=True)
        skp = oracle.decode(net, net.frames(), np.array(case["len"]), S, "frame", record=True,
                            skip_masked=True)
        assert np.array_equal(lit.raw_tokens, skp.raw_tokens)
        for b in range(B):
            assert np.array_equal(lit.frames[b], skp.frames[b])
            assert np.array_equal(lit.records.k[b], skp.records.k[b])
        assert lit.stats["pred_rows"] == lit.stats["inner"] * B >= skp.stats["pred_rows"]


def lattice_walk(choice, dur_choice, durations, length, S, blank):
    """Independent statement of the per-utterance decode as a recursion on the
    (frame, labels emitted, labels at this frame) lattice node."""
    def step(t, u, n):
        if t >= length:
            return []
        k = choice(t, u)
        d = durations[dur_choice(t, u)] if durations else None
        if k == blank:
            return step(t + (max(d, 1) if durations else 1), u, 0)
        if durations and d > 0:
            return [(k, t, d)] + step(t + d, u + 1, 0)
        if n + 1 == S:
            return [(k, t, d)] + step(t + 1, u + 1, 0)
        return [(k, t, d)] + step(t, u + 1, n + 1)
    return step(0, 0, 0)


@pytest.mark.parametrize("S", [1, 2, 3])
def test_brute_force_all_tables_T2_one_label(S):
    """Every argmax table on T=2 frames with one label plus blank, every
    length 0..2: all schedules equal the lattice recursion."""
    T, V1 = 2, 2
    U = S * T + 1
    cells = [(t, u) for t in range(T) for u in range(U)]
    combos = list(itertools.product(range(V1), repeat=len(cells)))
    B = len(combos)
    tab = np.zeros((B, T, U, V1), dtype=np.float32)
    for b, combo in enumerate(combos):
        for (t, u), c in zip(cells, combo):
            tab[b, t, u, c] = BIG
    net = oracle.TableNet(tab, V1)
    for length in range(T + 1):
        lens = np.full(B, length, dtype=np.int32)
        want = []
        for combo in combos:
            ch = dict(zip(cells, combo))
            want.append(lattice_walk(lambda t, u: ch[(t, min(u, U - 1))], None, None,
                                     length, S, V1 - 1))
        for sched in ["frame", "label", "seq"]:
            r = oracle.decode(net, net.frames(), lens, S, sched)
            for b in range(B):
                assert list(zip(r.tokens[b].tolist(), r.frames[b].tolist())) == \
                    [(k, t) for k, t, _ in want[b]], (sched, length, combos[b])


def test_brute_force_two_labels_S2():
    """3^10 = 59049 tables (two labels plus blank, T=2, S=2)."""
    T, V1, S = 2, 3, 2
    U = S * T + 1
    cells = [(t, u) for t in range(T) for u in range(U)]
    combos = np.array(list(itertools.product(range(V1), repeat=len(cells))), dtype=np.int64)
    B = combos.shape[0]
    tab = np.zeros((B, T, U, V1), dtype=np.float32)
    flat = tab.reshape(B, T * U, V1)
    flat[np.arange(B)[:, None], np.arange(T * U)[None, :], combos] = BIG
    net = oracle.TableNet(tab, V1)
    lens = np.full(B, T, dtype=np.int32)
    ref = oracle.decode(net, net.frames(), lens, S, "seq")
    for sched in ["frame", "label"]:
        r = oracle.decode(net, net.frames(), lens, S, sched)
        assert np.array_equal(r.raw_tokens, ref.raw_tokens), sched
        assert np.array_equal(r.tok_len, ref.tok_len), sched
    rng = np.random.default_rng(0)
    for b in rng.choice(B, size=400, replace=False):
        ch = {c: int(v) for c, v in zip(cells, combos[b])}
        want = lattice_walk(lambda t, u: ch[(t, min(u, U - 1))], None, None, T, S, V1 - 1)
        assert list(zip(ref.tokens[b].tolist(), ref.frames[b].tolist())) == \
            [(k, t) for k, t, _ in want]


def test_random_tables_T4_V4_with_and_without_durations():
    """Random tables at T<=4, vocabulary 4 (three labels plus blank), tables
    that depend on the last label, ragged lengths, RNN-T and TDT."""
    rng = np.random.default_rng(1)
    T, V1 = 4, 4
    for durations in [(), (0, 1, 2, 3, 4)]:
        D = len(durations)
        for S in [1, 2, 3]:
            B, U = 300, S * T + 1
            tab = rng.standard_normal((B, T, U, V1, V1 + D)).astype(np.float32)
            tab[..., V1 - 1] += 1.0        # more blanks, longer walks
            lens = rng.integers(0, T + 1, size=B).astype(np.int32)
            net = oracle.TableNet(tab, V1, durations)
            ref = oracle.decode(net, net.frames(), lens, S, "seq", record=True)
            for sched in schedules_for(D):
                r = oracle.decode(net, net.frames(), lens, S, sched, record=True)
                assert np.array_equal(r.raw_tokens, ref.raw_tokens), (sched, S, D)
                for b in range(B):
                    assert np.array_equal(r.frames[b], ref.frames[b])
                    assert np.array_equal(r.durs[b], ref.durs[b])
                    assert np.array_equal(r.scores[b], ref.scores[b])
                    assert np.array_equal(r.records.t[b], ref.records.t[b])
                    assert np.array_equal(r.records.k[b], ref.records.k[b])
            # an independent walk in Python that carries the label history
            for b in range(0, B, 7):
                hist, got = [], []
                t = u = n = 0
                while t < lens[b]:
                    last = hist[-1] if hist else V1 - 1
                    row = tab[b, t, min(u, U - 1), last]
                    k = int(np.argmax(row[:V1]))
                    d = durations[int(np.argmax(row[V1:]))] if D else None
                    if k == V1 - 1:
                        t += max(d, 1) if D else 1
                        n = 0
                        continue
                    got.append((k, t, d))
                    hist.append(k)
                    u += 1
                    if D and d > 0:
                        t += d
                        n = 0
                    else:
                        n += 1
                        if n == S:
                            t += 1
                            n = 0
                assert [g[0] for g in got] == ref.tokens[b].tolist()
                assert [g[1] for g in got] == ref.frames[b].tolist()
                if D:
                    assert [g[2] for g in got] == ref.durs[b].tolist()


def test_argmax_tie_takes_lowest_index():
    tab = np.zeros((1, 2, 3, 3), dtype=np.float32)   # all logits equal: label 0 wins
    net = oracle.TableNet(tab, 3)
    for sched in ["frame", "label", "seq"]:
        r = oracle.decode(net, net.frames(), np.array([2]), 1, sched, record=True)
        assert r.tokens[0].tolist() == [0, 0]
        assert np.all(r.records.margin[0] == 0.0)


def test_paper_alternating_batch_step_counts():
    """Related Work scenario: B=2, max_symbols=5; element 0 emits 5 labels on
    even frames and a blank on odd ones, element 1 the opposite.  Algorithm 1
    needs 5 inner steps on every frame; label looping lets both rows progress,
    about 3 batched joint steps per frame."""
    T, S, V1 = 20, 5, 3
    U = S * T + 1
    cells = []
    for b in range(2):
        for t in range(T):
            if t % 2 == b:
                for u in range(U):
                    cells.append([b, t, u, -1, u % 2, 0])
    tab = table_from_choices(2, T, U, V1, 0, cells)
    net = oracle.TableNet(tab, V1)
    lens = np.array([T, T], dtype=np.int32)
    fr = oracle.decode(net, net.frames(), lens, S, "frame")
    la = oracle.decode(net, net.frames(), lens, S, "label")
    sq = oracle.decode(net, net.frames(), lens, S, "seq")
    assert fr.tok_len.tolist() == [S * T // 2, S * T // 2]
    assert np.array_equal(fr.raw_tokens, la.raw_tokens)
    assert np.array_equal(fr.raw_tokens, sq.raw_tokens)
    assert fr.stats["inner"] == S * T
    assert la.stats["outer"] <= S * T // 2 + 2
    assert la.stats["inner"] <= 3 * T + 2
    assert la.stats["inner"] < fr.stats["inner"]


def test_status_bits_and_capacity():
    T, S, V1 = 3, 2, 2
    tab = np.zeros((1, T, S * T + 1, V1), dtype=np.float32)
    tab[..., 0] = BIG      # never blank
    net = oracle.TableNet(tab, V1)
    for sched in ["frame", "label", "seq"]:
        r = oracle.decode(net, net.frames(), np.array([T + 5]), S, sched)
        assert r.status & 1                        # length clamped to T
        assert r.tok_len[0] == S * T
        r = oracle.decode(net, net.frames(), np.array([T]), S, sched, cap=4)
        assert r.status & 2                        # capacity overflow flagged
        assert r.tok_len[0] == S * T and len(r.tokens[0]) == 4
        r = oracle.decode(net, net.frames(), np.array([-3]), S, sched)
        assert r.status & 1 and r.tok_len[0] == 0


def test_follow_finds_the_blank_durations_a_tdt_hypothesis_does_not_record():
    """A TDT hypothesis lists labels with frames and durations, not the durations taken on
    blanks.  Two tables that differ in one blank cell only: there the duration logits of 1 and 2
    frames are 1e-3 apart, with either sign.  Each table's decode is a hypothesis that the
    other table's walk can only reach through the runner-up duration of that blank.  With a
    tolerance above the gap, follow mode finds that chain and reports exactly that departure
    (duration column, gap 1e-3); with tolerance 0 it walks the argmax durations and ends
    somewhere else."""
    V1, durations, S, T = 3, (0, 1, 2), 2, 6
    D, U = len(durations), 8
    cells = [[0, 1, 0, -1, 0, 2],     # frame 1, before any label: label 0, then jump two frames
             [0, 3, 1, -1, 1, 1],     # frame 3, one label out: label 1, then one frame on
             [0, 2, 0, -1, 1, 1],     # frame 2 (reached only through the 2-frame blank at 0): label 1
             [0, 4, 2, -1, 0, 1]]
    tabs = []
    for eps in (+1e-3, -1e-3):
        tab = table_from_choices(1, T, U, V1, D, cells)
        # blank at frame 0, nothing emitted yet: durations "1 frame" and "2 frames" nearly tied
        tab[0, 0, 0, :, V1:] = 0.0
        tab[0, 0, 0, :, V1 + 1] = BIG
        tab[0, 0, 0, :, V1 + 2] = BIG + eps
        tabs.append(tab)
    nets = [oracle.TableNet(t, V1, durations) for t in tabs]
    lens = np.array([T], dtype=np.int32)
    hyps = [oracle.decode(n, n.frames(), lens, S, "seq") for n in nets]
    assert hyps[0].frames[0].tolist() != hyps[1].frames[0].tolist()     # the blank's duration matters
    for a, b in ((0, 1), (1, 0)):
        net, h = nets[a], hyps[b]
        args = (net, net.frames()[0], T, S, h.tokens[0], h.frames[0], h.durs[0])
        own = oracle.follow(nets[b], nets[b].frames()[0], T, S, h.tokens[0], h.frames[0], h.durs[0], tol=1e-2)
        assert own.departures == 0
        found = oracle.follow(*args, tol=1e-2)
        assert found.departures == 1, found
        rep = found.where[0]
        assert rep["t"] == 0 and rep["want"] >= V1 and rep["got"] >= V1 and rep["want"] != rep["got"]
        assert abs(rep["gap"] - 1e-3) < 1e-4 and abs(found.worst_gap - 1e-3) < 1e-4
        assert oracle.follow(*args, tol=1e-4).departures != 1      # the gap is above this tolerance
        strict = oracle.follow(*args)                               # argmax durations only
        assert strict.departures == -1 or strict.worst_gap > 1.0
