"""Pins for the oracle's two sub-networks and for whole decodes with the LSTM
network: torch CPU library routines, closed forms, special cases, invariants.
No GPU."""
import numpy as np
import pytest
import torch

import oracle
import synth
from synth import ModelDims, make_model, param_count


def small_model(durations=(), seed=7, **kw):
    # all widths different so a transposed operand cannot go unnoticed
    dims = ModelDims(F=5, E=7, H=6, L=2, J=4, V1=9, durations=tuple(durations))
    return make_model(dims, seed, weight_range=0.8, **kw)


def torch_pred(model, last, state, dtype):
    d = model.dims
    lstm = torch.nn.LSTM(d.E, d.H, num_layers=d.L).to(dtype)
    with torch.no_grad():
        for l in range(d.L):
            getattr(lstm, f"weight_ih_l{l}").copy_(torch.from_numpy(model.w_ih[l]).to(dtype))
            getattr(lstm, f"weight_hh_l{l}").copy_(torch.from_numpy(model.w_hh[l]).to(dtype))
            getattr(lstm, f"bias_ih_l{l}").copy_(torch.from_numpy(model.b_ih[l]).to(dtype))
            getattr(lstm, f"bias_hh_l{l}").copy_(torch.from_numpy(model.b_hh[l]).to(dtype))
        st = torch.from_numpy(np.asarray(state)).to(dtype).reshape(d.L, 2, d.H)
        h0 = st[:, 0, :].reshape(d.L, 1, d.H).contiguous()
        c0 = st[:, 1, :].reshape(d.L, 1, d.H).contiguous()
        x = torch.from_numpy(model.emb[last]).to(dtype).reshape(1, 1, d.E)
        out, (h1, c1) = lstm(x, (h0, c0))
    new_state = torch.stack([h1[:, 0, :], c1[:, 0, :]], dim=1).reshape(-1)
    return out.reshape(-1).numpy(), new_state.numpy()


def torch_joint(model, x_row, g, dtype):
    F = torch.nn.functional
    t = lambda a: torch.from_numpy(np.asarray(a)).to(dtype)
    p = F.linear(t(x_row), t(model.w_enc), t(model.b_enc))
    q = F.linear(t(g), t(model.w_pred), t(model.b_pred))
    return F.linear(torch.relu(p + q), t(model.w_out), t(model.b_out)).numpy()


@pytest.mark.parametrize("real,dtype,tol", [("float", torch.float32, 2e-6),
                                            ("double", torch.float64, 1e-13)])
def test_prediction_network_matches_torch_lstm(real, dtype, tol):
    model = small_model()
    net = oracle.LstmNet(model, real)
    state = np.zeros(net.state_size)
    rng = np.random.default_rng(0)
    for step in range(6):
        last = int(rng.integers(0, model.dims.V1))
        g, s2 = net.pred(last, state)
        g_t, s_t = torch_pred(model, last, state, dtype)
        assert np.max(np.abs(g - g_t)) <= tol
        assert np.max(np.abs(s2 - s_t)) <= tol
        assert np.array_equal(g, s2[(model.dims.L - 1) * 2 * model.dims.H:][:model.dims.H])
        state = s2


@pytest.mark.parametrize("real,dtype,tol", [("float", torch.float32, 5e-6),
                                            ("double", torch.float64, 1e-13)])
def test_joint_matches_torch_linear(real, dtype, tol):
    model = small_model(durations=(0, 1, 2))
    net = oracle.LstmNet(model, real)
    rng = np.random.default_rng(1)
    for _ in range(5):
        x = rng.standard_normal(model.dims.F)
        g = rng.uniform(-1, 1, model.dims.H)
        got = net.joint(net.prep(x), g)
        want = torch_joint(model, x, g, dtype)
        assert got.shape == (model.dims.n_out,)
        assert np.max(np.abs(got - want)) <= tol * max(1.0, np.max(np.abs(want)))


def test_zero_weight_lstm_closed_form():
    """With all weight matrices zero the cell is driven by the biases alone:
    c_n = s(b_f) c_{n-1} + s(b_i) tanh(b_g),  h_n = s(b_o) tanh(c_n)."""
    model = small_model()
    d = model.dims
    for l in range(d.L):
        model.w_ih[l][:] = 0
        model.w_hh[l][:] = 0
    net = oracle.LstmNet(model, "double")
    sig = lambda v: 1.0 / (1.0 + np.exp(-v))
    state = np.zeros(net.state_size)
    c = [np.zeros(d.H) for _ in range(d.L)]
    for n in range(4):
        g, state = net.pred(3, state)
        for l in range(d.L):
            b = (model.b_ih[l] + model.b_hh[l]).astype(np.float64)
            bi, bf, bg, bo = b[:d.H], b[d.H:2 * d.H], b[2 * d.H:3 * d.H], b[3 * d.H:]
            c[l] = sig(bf) * c[l] + sig(bi) * np.tanh(bg)
            h = sig(bo) * np.tanh(c[l])
            assert np.allclose(state[l * 2 * d.H:l * 2 * d.H + d.H], h, atol=1e-14)
            assert np.allclose(state[l * 2 * d.H + d.H:(l + 1) * 2 * d.H], c[l], atol=1e-14)
        assert np.allclose(g, h, atol=1e-14)


def test_parakeet_shape_has_the_papers_parameter_count():
    # Introduction: prediction and joint networks together hold about 8.9 million parameters
    assert param_count(synth.CONFIGS[2]["dims"]) == 8_943_105
    assert param_count(synth.CONFIGS[4]["dims"]) == 8_946_310
    assert param_count(synth.CONFIGS[0]["dims"]) == 43_793
    assert param_count(synth.CONFIGS[1]["dims"]) == 1_171_457


def test_start_of_sequence_is_a_zero_embedding():
    for cfg in range(5):
        c = synth.CONFIGS[cfg]
        m = make_model(c["dims"], c["seed"], **c["model_kw"]) if cfg < 2 else None
        if m is not None:
            assert np.all(m.emb[m.dims.blank] == 0)


def decode_all(w, real="float", **kw):
    net = oracle.LstmNet(w.model, real)
    scheds = ["label", "seq"] if w.model.dims.D else ["frame", "label", "seq"]
    return {s: oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, s, record=True, **kw)
            for s in scheds}


def assert_same(a, b):
    assert np.array_equal(a.tok_len, b.tok_len)
    assert np.array_equal(a.raw_tokens, b.raw_tokens)
    for i in range(len(a.tokens)):
        assert np.array_equal(a.frames[i], b.frames[i])
        assert np.array_equal(a.scores[i], b.scores[i])      # bit-identical logits
        assert np.array_equal(a.durs[i], b.durs[i])
        assert np.array_equal(a.records.t[i], b.records.t[i])
        assert np.array_equal(a.records.margin[i], b.records.margin[i])


def check_invariants(w, r, S):
    blank = w.model.dims.blank
    for b in range(w.B):
        n = int(min(max(w.enc_len[b], 0), w.T))
        assert r.tok_len[b] <= S * n
        fr = r.frames[b]
        assert np.all(np.diff(fr) >= 0)
        if len(fr):
            assert fr.max() < n and np.bincount(fr).max() <= S
        assert np.all(r.tokens[b] != blank) and np.all(r.tokens[b] >= 0)
        if not w.model.dims.D:
            per_frame = np.bincount(fr, minlength=n) if n else np.zeros(0, int)
            forced = int((per_frame == S).sum())
            assert len(r.records.k[b]) == n + r.tok_len[b] - forced


@pytest.mark.parametrize("cfg,kw", [
    (0, {}),
    (1, {}),
    (2, dict(B=6, T=40, len_lo=15, len_hi=40)),
    (4, dict(B=6, T=60, len_lo=20, len_hi=60)),
    (5, dict(B=6, T=40, len_lo=15, len_hi=40)),
])
def test_schedules_agree_bit_for_bit(cfg, kw):
    """Frame looping, label looping and the per-utterance decode give identical
    tokens, frames and scores (the paper's exactness claim), with NaN padding."""
    w = synth.make_workload(cfg, pad="nan", **kw)
    rs = decode_all(w)
    for s, r in rs.items():
        assert r.status == 0
        assert_same(r, rs["seq"])
        check_invariants(w, r, w.max_symbols)
    assert rs["seq"].tok_len.sum() > 0


def test_schedules_agree_on_random_models():
    """The same claim on seeded random models: 1-3 layers, small widths, RNN-T, TDT and
    multi-blank, random lengths and max_symbols; float and double builds."""
    rng = np.random.default_rng(8)
    emitted = 0
    for case in range(40):
        kind = ["rnnt", "tdt", "multi-blank"][case % 3]
        durations = tuple(sorted(set([0] + [int(d) for d in rng.integers(1, 4, size=2)]))) if kind == "tdt" else ()
        spans = (2, int(rng.integers(3, 6))) if kind == "multi-blank" else ()
        dims = synth.ModelDims(F=16, E=int(rng.integers(3, 20)), H=4 * int(rng.integers(1, 9)),
                               L=int(rng.integers(1, 4)), J=4 * int(rng.integers(1, 9)),
                               V1=int(rng.integers(2, 30)), durations=durations, big_blanks=spans)
        model = synth.make_model(dims, seed=300 + case, weight_range=0.4, blank_bias=float(rng.uniform(0.3, 1.5)))
        B, T, S = int(rng.integers(1, 7)), int(rng.integers(3, 25)), int(rng.integers(1, 4))
        x, ln = synth.make_inputs(700 + case, B, T, dims.F, 1, T, pad="nan")
        w = synth.Workload(f"r{case}", "label", model, x, ln, S)
        for real in ("float", "double"):
            net = oracle.LstmNet(w.model, real)
            scheds = ["label", "seq"] if (durations or spans) else ["frame", "label", "seq"]
            rs = {sc: oracle.decode(net, w.enc_out, w.enc_len, S, sc, record=True) for sc in scheds}
            for sc, r in rs.items():
                assert r.status == 0
                assert_same(r, rs["seq"])
            emitted += int(rs["seq"].tok_len.sum())
    assert emitted > 200


def test_frame_looping_masked_rows_do_not_matter():
    """Algorithm 1 runs both networks for the whole batch at every inner step, rows that are
    already masked included (the oracle's default); their results are discarded, so passing
    over them (skip_masked, used where a large batch has to be timed) changes nothing: same
    tokens, frames, scores bit for bit and the same records, on the small model, on a cut of
    the two-layer Parakeet-shaped model and with padding frames that hold NaN."""
    for cfg, kw in [(1, dict(pad="normal", T=60, len_lo=20, len_hi=60)),
                    (2, dict(pad="nan", B=5, T=40, len_lo=12, len_hi=40)),
                    (1, dict(pad="nan", T=30, len_lo=0, len_hi=30))]:
        w = synth.make_workload(cfg, **kw)
        net = oracle.LstmNet(w.model)
        a = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "frame", record=True)
        b = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "frame", record=True,
                          skip_masked=True)
        assert_same(a, b)
        for i in range(w.B):
            assert np.array_equal(a.records.k[i], b.records.k[i])
            assert np.array_equal(a.records.t[i], b.records.t[i])
        # the literal form really evaluates every row at every inner step
        assert a.stats["pred_rows"] == a.stats["inner"] * w.B > b.stats["pred_rows"]
        assert a.stats["inner"] == b.stats["inner"]


def test_batch_row_equals_single_utterance_and_permutation():
    w = synth.make_workload(1, pad="nan", T=50, len_lo=10, len_hi=50)
    net = oracle.LstmNet(w.model)
    perm = np.random.default_rng(3).permutation(w.B)
    for sched in ["frame", "label", "seq"]:
        full = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, sched)
        shuf = oracle.decode(net, w.enc_out[perm], w.enc_len[perm], w.max_symbols, sched)
        for i, b in enumerate(perm):
            assert np.array_equal(shuf.tokens[i], full.tokens[b])
        for b in range(w.B):
            one = oracle.decode(net, w.enc_out[b:b + 1], w.enc_len[b:b + 1], w.max_symbols, sched)
            assert np.array_equal(one.tokens[0], full.tokens[b])
            assert np.array_equal(one.scores[0], full.scores[b])


def test_tdt_batch_row_equals_single_utterance():
    w = synth.make_workload(4, pad="nan", B=5, T=50, len_lo=10, len_hi=50)
    net = oracle.LstmNet(w.model)
    full = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "tdt")
    for b in range(w.B):
        one = oracle.decode(net, w.enc_out[b:b + 1], w.enc_len[b:b + 1], w.max_symbols, "tdt")
        assert np.array_equal(one.tokens[0], full.tokens[b])
        assert np.array_equal(one.durs[0], full.durs[b])


@pytest.mark.parametrize("sched", ["frame", "label", "seq"])
def test_all_blank_and_never_blank_closed_forms(sched):
    S = 3
    w = synth.make_workload(1, T=30, len_lo=5, len_hi=30, model_overrides=dict(blank_bias=1e4))
    net = oracle.LstmNet(w.model)
    r = oracle.decode(net, w.enc_out, w.enc_len, S, sched, record=True)
    assert np.all(r.tok_len == 0)
    assert [len(k) for k in r.records.k] == w.enc_len.tolist()   # one evaluation per frame
    w = synth.make_workload(1, T=30, len_lo=5, len_hi=30, model_overrides=dict(blank_bias=-1e4))
    net = oracle.LstmNet(w.model)
    r = oracle.decode(net, w.enc_out, w.enc_len, S, sched, record=True)
    assert r.tok_len.tolist() == (S * w.enc_len).tolist()
    for b in range(w.B):
        assert r.frames[b].tolist() == np.repeat(np.arange(w.enc_len[b]), S).tolist()


def test_max_symbols_one_gives_at_most_one_label_per_frame():
    w = synth.make_workload(1, T=60, len_lo=20, len_hi=60)
    net = oracle.LstmNet(w.model)
    for sched in ["frame", "label", "seq"]:
        r = oracle.decode(net, w.enc_out, w.enc_len, 1, sched, record=True)
        for b in range(w.B):
            assert len(set(r.frames[b].tolist())) == len(r.frames[b])
            assert len(r.records.k[b]) == w.enc_len[b]


def tdt_from(cfg_kw, dur_bias):
    return synth.make_workload(4, B=4, T=50, len_lo=20, len_hi=50,
                               model_overrides=dict(dur_bias=dur_bias), **cfg_kw)


def test_tdt_reduces_to_rnnt_when_duration_is_pinned():
    """Duration head forced to 0: TDT is RNN-T with the same token weights.
    Forced to 1: RNN-T with max_symbols = 1."""
    big = 1e4
    w0 = tdt_from({}, (big, 0, 0, 0, 0))
    w1 = tdt_from({}, (0, big, 0, 0, 0))
    m = w0.model
    V1 = m.dims.V1
    rn_dims = synth.ModelDims(F=m.dims.F, E=m.dims.E, H=m.dims.H, L=m.dims.L, J=m.dims.J, V1=V1)
    rn = synth.Model(rn_dims, m.emb, m.w_ih, m.w_hh, m.b_ih, m.b_hh, m.w_enc, m.b_enc,
                     m.w_pred, m.b_pred, m.w_out[:V1].copy(), m.b_out[:V1].copy(),
                     np.zeros(0, np.int32))
    rnet = oracle.LstmNet(rn)
    for sched in ["label", "seq"]:
        S = w0.max_symbols
        t0 = oracle.decode(oracle.LstmNet(w0.model), w0.enc_out, w0.enc_len, S, sched)
        r0 = oracle.decode(rnet, w0.enc_out, w0.enc_len, S, sched)
        assert np.array_equal(t0.raw_tokens, r0.raw_tokens) and t0.tok_len.sum() > 0
        assert all(np.all(d == 0) for d in t0.durs)
        t1 = oracle.decode(oracle.LstmNet(w1.model), w1.enc_out, w1.enc_len, S, sched)
        r1 = oracle.decode(rnet, w1.enc_out, w1.enc_len, 1, sched)
        assert np.array_equal(t1.tok_len, r1.tok_len)
        for b in range(w1.B):
            assert np.array_equal(t1.tokens[b], r1.tokens[b])
            assert np.array_equal(t1.frames[b], r1.frames[b])


def test_float_and_double_builds_agree_away_from_ties():
    w = synth.make_workload(1, T=80, len_lo=40, len_hi=80)
    f32 = oracle.decode(oracle.LstmNet(w.model, "float"), w.enc_out, w.enc_len,
                        w.max_symbols, "seq", record=True)
    f64 = oracle.decode(oracle.LstmNet(w.model, "double"), w.enc_out, w.enc_len,
                        w.max_symbols, "seq", record=True)
    for b in range(w.B):
        if f32.records.margin[b].min() > 1e-5:
            assert np.array_equal(f32.tokens[b], f64.tokens[b])
            assert np.allclose(f32.scores[b], f64.scores[b], rtol=1e-5, atol=1e-5)


def test_follow_reports_departures():
    w = synth.make_workload(1, T=40, len_lo=30, len_hi=40)
    net = oracle.LstmNet(w.model)
    r = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "seq")
    b = int(np.argmax(r.tok_len))
    ok = oracle.follow(net, w.enc_out[b], w.enc_len[b], w.max_symbols, r.tokens[b], r.frames[b])
    assert ok.departures == 0 and ok.worst_gap == 0.0
    toks = r.tokens[b].copy()
    toks[1] = (toks[1] + 1) % w.model.dims.blank
    bad = oracle.follow(net, w.enc_out[b], w.enc_len[b], w.max_symbols, toks, r.frames[b])
    assert bad.departures >= 1 and bad.worst_gap > 0
    assert bad.where[0]["u"] == 1 and bad.where[0]["want"] == int(r.tokens[b][1])
    # a hypothesis no walk can produce: a frame index beyond the utterance
    fr = r.frames[b].copy()
    fr[-1] = w.enc_len[b] + 3
    assert oracle.follow(net, w.enc_out[b], w.enc_len[b], w.max_symbols, r.tokens[b], fr).departures == -1


def test_follow_reports_tdt_departures():
    """Follow mode on a token-and-duration model: the oracle's own hypothesis has no departure;
    an altered token is reported with the oracle's label and the right gap; an altered duration
    is reported as column V1 + index with the gap between the two duration logits; a duration
    value the model does not have makes the hypothesis impossible."""
    w = synth.make_workload(4, pad="nan", B=4, T=60, len_lo=30, len_hi=60)
    net = oracle.LstmNet(w.model)
    V1, durations = w.model.dims.V1, list(w.model.dims.durations)
    r = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "seq", record=True)
    b = int(np.argmax(r.tok_len))
    n = int(r.tok_len[b])
    assert n >= 4
    args = (net, w.enc_out[b], int(w.enc_len[b]), w.max_symbols)
    ok = oracle.follow(*args, r.tokens[b], r.frames[b], r.durs[b])
    assert ok.departures == 0 and ok.worst_gap == 0.0

    def logits_at(u):
        """Logits of the evaluation that emitted label u, recomputed through the sub-network
        calls (prediction steps along the first u labels, joint at the label's frame)."""
        state = np.zeros(net.state_size, dtype=np.float32)
        g, cand = net.pred(net.blank, state)
        for i in range(u):
            g, cand = net.pred(int(r.tokens[b][i]), cand)
        return net.joint(net.prep(w.enc_out[b, int(r.frames[b][u])]), g)

    # 1. a token altered: first departure at that label, the oracle's label as `want`
    u = 1
    lg = logits_at(u)
    assert int(np.argmax(lg[:V1])) == int(r.tokens[b][u])
    toks = r.tokens[b].copy()
    toks[u] = (int(toks[u]) + 3) % (V1 - 1)
    bad = oracle.follow(*args, toks, r.frames[b], r.durs[b])
    assert bad.departures >= 1
    first = bad.where[0]
    assert (first["u"], first["t"]) == (u, int(r.frames[b][u]))
    assert first["want"] == int(r.tokens[b][u]) and first["got"] == int(toks[u])
    assert abs(first["gap"] - float(lg[:V1].max() - lg[toks[u]])) < 1e-6
    assert bad.worst_gap >= first["gap"] > 0

    # 2. a duration altered on the last label (no later label's frame index contradicts the
    # new landing frame; the blanks after it may still give further departures)
    u = n - 1
    lg = logits_at(u)
    di = int(np.argmax(lg[V1:]))
    assert durations[di] == int(r.durs[b][u])
    gi = (di + 1) % len(durations)
    durs = r.durs[b].copy()
    durs[u] = durations[gi]
    bad = oracle.follow(*args, r.tokens[b], r.frames[b], durs)
    assert bad.departures >= 1
    rep = bad.where[0]
    assert (rep["u"], rep["want"], rep["got"]) == (u, V1 + di, V1 + gi)
    assert abs(rep["gap"] - float(lg[V1 + di] - lg[V1 + gi])) < 1e-6
    assert bad.worst_gap >= rep["gap"] > 0

    # 3. a duration the model does not have: no walk produces it
    durs = r.durs[b].copy()
    durs[0] = 7
    assert oracle.follow(*args, r.tokens[b], r.frames[b], durs).departures == -1
    # 4. a duration altered in the middle moves the walk off the hypothesis' later frames
    # unless the frames follow: a skipped frame index makes the rest unreachable
    if n >= 3:
        durs = r.durs[b].copy()
        durs[0] = durations[-1] + 0 if int(durs[0]) != durations[-1] else durations[0]
        res = oracle.follow(*args, r.tokens[b], r.frames[b], durs)
        assert res.departures != 0


def test_stored_oracle_tokens_are_reproduced():
    """tests/golden/oracle_tokens.json was written by tests/golden/make_golden.py
    from the oracle alone; a change in the generator or the oracle shows here."""
    import importlib.util
    import json
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    with open(os.path.join(here, "golden", "oracle_tokens.json")) as fh:
        stored = json.load(fh)
    for name, case in mg.CASES.items():
        assert mg.run(case) == stored[name], name


def test_bf16_rounding_of_inputs_matches_torch():
    """synth.round_to_bf16 is round-to-nearest-even to bf16, as torch's conversion."""
    x = synth.normal(77, 1, (4096,)).astype(np.float32) * np.float32(0.1)
    x[:4] = [0.0, -0.0, 1.00390625, 3.0e38]
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(synth.round_to_bf16(x), want)
    m = synth.make_workload(0).model
    r = synth.with_bf16_streamed_weights(m)
    assert np.array_equal(r.emb, m.emb) and np.array_equal(r.w_ih[0], m.w_ih[0])
    assert not np.array_equal(r.w_out, m.w_out)
    assert np.all(r.w_out.view(np.uint32) & 0xFFFF == 0) and np.all(r.w_hh[0].view(np.uint32) & 0xFFFF == 0)


def test_e4m3_rounding_of_inputs_matches_torch():
    """synth.round_to_e4m3 rounds to the nearest 8-bit e4m3 value (ties to even, saturating at
    448), as torch's float8_e4m3fn conversion does inside that range; the 254 finite codes are
    fixed points."""
    x = np.concatenate([synth.normal(78, 1, (4096,)) * 0.1, synth.normal(78, 2, (4096,)) * 30.0,
                        synth.uniform(78, 3, (2048,), -0.01, 0.01)]).astype(np.float32)
    x[:10] = [0.0, -0.0, 448.0, -448.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10, 2.0 ** -6, 0.0625 + 2.0 ** -8, 440.0]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float32).numpy()
    got = synth.round_to_e4m3(x)
    assert np.array_equal(got, want) and np.array_equal(np.signbit(got), np.signbit(want))
    assert synth.round_to_e4m3(np.array([1000.0, -465.0], np.float32)).tolist() == [448.0, -448.0]
    codes = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    finite = codes[np.isfinite(codes)]
    assert finite.size == 254 and np.array_equal(synth.round_to_e4m3(finite), finite)
    m = synth.make_workload(0).model
    r = synth.with_fp8_streamed_weights(m)
    assert np.array_equal(r.emb, m.emb) and np.array_equal(r.w_ih[0], m.w_ih[0])
    assert np.array_equal(synth.round_to_e4m3(r.w_out), r.w_out) and not np.array_equal(r.w_out, m.w_out)


def test_log_probabilities_of_emitted_labels():
    """The value v that Algorithm 1 takes with the argmax k: log_softmax over the token columns at the
    chosen label.  Pinned against torch.log_softmax on table-driven logits (the duration
    columns of a TDT table do not enter), the closed form for equal logits, and the LSTM net's
    own joint output re-evaluated through the direct-access entry points."""
    rng = np.random.default_rng(11)
    B, T, U, V1 = 3, 5, 8, 6
    for durations in [(), (0, 1, 2)]:
        D = len(durations)
        tab = rng.normal(0.0, 2.0, size=(B, T, U, V1 + D)).astype(np.float32)
        net = oracle.TableNet(tab, V1, durations)
        lens = np.array([5, 3, 4], dtype=np.int32)
        for sched in (["label", "seq"] if D else ["frame", "label", "seq"]):
            r = oracle.decode(net, net.frames(), lens, 3, sched)
            for b in range(B):
                for i, (k, t) in enumerate(zip(r.tokens[b], r.frames[b])):
                    logits = torch.from_numpy(tab[b, t, min(i, U - 1), :V1].astype(np.float64))
                    want = torch.log_softmax(logits, dim=0)[int(k)].item()
                    assert abs(float(r.logps[b][i]) - want) < 1e-6, (sched, b, i)
                    assert abs(float(r.scores[b][i]) - float(logits.max())) == 0.0
    # equal logits: every label has probability 1 / V1
    net = oracle.TableNet(np.zeros((1, 2, 3, 4), dtype=np.float32), 4)
    r = oracle.decode(net, net.frames(), np.array([2]), 1, "seq")
    assert np.allclose(r.logps[0], -np.log(4.0), atol=1e-7)
    # LSTM net, float and double builds agree, and exp(logp) <= 1
    w = synth.make_workload(0)
    rf = oracle.decode(oracle.LstmNet(w.model), w.enc_out, w.enc_len, w.max_symbols, "frame")
    rd = oracle.decode(oracle.LstmNet(w.model, real="double"), w.enc_out.astype(np.float64),
                       w.enc_len, w.max_symbols, "frame")
    assert rf.tok_len[0] > 0 and np.array_equal(rf.tokens[0], rd.tokens[0])
    assert np.allclose(rf.logps[0], rd.logps[0], atol=1e-5)
    assert np.all(rf.logps[0] <= 0.0)


def test_bf16_rounding_matches_torch():
    """The oracle's bfloat16 rounding (ties to even on the float32 bit pattern) against torch's
    conversion: random values over the whole exponent range, exact ties, subnormals, signs."""
    lib = oracle._lib("float")
    rng = np.random.default_rng(7)
    vals = np.concatenate([
        (rng.standard_normal(4000) * np.exp(rng.uniform(-80, 80, 4000))).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.3895314e38, 1e-40, -1e-40,
                  65280.0, 65408.0, 0.1, -0.1, 2.0 ** -133], dtype=np.float32)])
    want = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([lib.orc_round_bf16(float(v)) for v in vals], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # the generator's rounding (used to build bf16-valued models) is the same function
    assert np.array_equal(synth.round_to_bf16(vals).view(np.uint32), want.view(np.uint32))


def test_bf16_emulation_matches_rounded_operands_in_float64():
    """bfloat16 emulation: each dense product of the three sub-networks equals the product of
    the bfloat16-rounded weights and the bfloat16-rounded input, accumulated exactly (torch,
    float64), plus the unrounded bias; everything else as in the float path.  A model whose
    widths all differ, non-zero state, two layers."""
    dims = synth.ModelDims(F=24, E=10, H=12, L=2, J=14, V1=9, durations=(0, 1, 2))
    m = synth.make_model(dims, seed=11, weight_range=0.7)
    bf = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float64)
    f64 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))
    rng = np.random.default_rng(3)
    x = rng.standard_normal(dims.F).astype(np.float32)
    state = (rng.standard_normal(2 * dims.L * dims.H) * 0.5).astype(np.float32)
    for real, tol in (("float", 3e-6), ("double", 1e-12)):
        net = oracle.LstmNet(m, real, bf16=True)
        plain = oracle.LstmNet(m, real)
        dt = np.float32 if real == "float" else np.float64
        # encoder-side projection
        want_p = bf(m.w_enc) @ bf(x) + f64(m.b_enc)
        got_p = net.prep(x.astype(dt))
        assert np.allclose(got_p, want_p.numpy(), rtol=tol, atol=tol)
        assert not np.allclose(got_p, plain.prep(x.astype(dt)), rtol=1e-4, atol=1e-4)   # the mode is on
        # one prediction step from a non-zero state with label 3
        H = dims.H
        inp = bf(m.emb[3])
        want_state = np.zeros_like(state, dtype=np.float64)
        for l in range(dims.L):
            h, cc = f64(state[2 * l * H:(2 * l + 1) * H]), f64(state[(2 * l + 1) * H:(2 * l + 2) * H])
            gates = (bf(m.w_ih[l]) @ inp + f64(m.b_ih[l])) + (bf(m.w_hh[l]) @ bf(h.numpy()) + f64(m.b_hh[l]))
            gi, gf, gg, go = (gates[j * H:(j + 1) * H] for j in range(4))
            cn = torch.sigmoid(gf) * cc + torch.sigmoid(gi) * torch.tanh(gg)
            hn = torch.sigmoid(go) * torch.tanh(cn)
            want_state[2 * l * H:(2 * l + 1) * H] = hn.numpy()
            want_state[(2 * l + 1) * H:(2 * l + 2) * H] = cn.numpy()
            inp = bf(hn.numpy())        # the next layer's product rounds its input again
        g, got_state = net.pred(3, state.astype(dt))
        assert np.allclose(got_state, want_state, rtol=10 * tol, atol=10 * tol)
        assert np.allclose(g, want_state[2 * (dims.L - 1) * H:(2 * dims.L - 1) * H], rtol=10 * tol, atol=10 * tol)
        # joint
        p_row = rng.standard_normal(dims.J).astype(dt)
        gv = (rng.standard_normal(dims.H) * 0.5).astype(dt)
        q = bf(m.w_pred) @ bf(gv) + f64(m.b_pred)
        z = torch.relu(f64(p_row) + q)
        want_l = bf(m.w_out) @ bf(z.numpy()) + f64(m.b_out)
        assert np.allclose(net.joint(p_row, gv), want_l.numpy(), rtol=10 * tol, atol=10 * tol)


def test_bf16_emulation_schedules_agree_and_differ_from_float():
    for cfg, kw in [(1, dict(T=50, len_lo=20, len_hi=50)), (4, dict(B=4, T=50, len_lo=20, len_hi=50))]:
        w = synth.make_workload(cfg, pad="nan", **kw)
        net = oracle.LstmNet(w.model, bf16=True)
        scheds = ["label", "seq"] if w.model.dims.D else ["frame", "label", "seq"]
        rs = [oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, s, record=True) for s in scheds]
        for r in rs[1:]:
            assert_same(rs[0], r)
        plain = oracle.decode(oracle.LstmNet(w.model), w.enc_out, w.enc_len, w.max_symbols, "seq")
        assert rs[0].tok_len.sum() > 0
        # same model, other arithmetic: the scores move by about a bfloat16 rounding step
        diff = max(float(np.max(np.abs(a[:min(len(a), len(b))] - b[:min(len(a), len(b))]))) if len(a) and len(b) else 0.0
                   for a, b in zip(rs[-1].scores, plain.scores))
        assert diff > 1e-4
