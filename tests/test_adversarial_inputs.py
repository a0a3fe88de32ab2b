"""The adversarial batches do to the oracle what the paper says such inputs do:
the two-utterance alternating batch makes lock-step frame looping run max_symbols
inner steps on every frame while label looping needs far fewer batched steps
(section on label looping), and an always-emitting input yields max_symbols
labels per frame (discussion of the experiments)."""
import numpy as np
import pytest

import oracle
import synth


@pytest.fixture(scope="module")
def net_and_inputs():
    out = {}
    for pat in synth.PATTERNS:
        w = synth.make_adversarial(pat, cfg=2, B=2, T=6)
        out[pat] = (w, oracle.LstmNet(w.model))
    return out


def test_emit_mask_patterns():
    m = synth.emit_mask("alternating", 2, 4)
    assert m.tolist() == [[True, False, True, False], [False, True, False, True]]
    assert synth.emit_mask("one_slow_row", 3, 2).tolist() == [[True, True], [False, False], [False, False]]
    assert not synth.emit_mask("all_blank", 2, 3).any() and synth.emit_mask("always_max", 2, 3).all()
    with pytest.raises(ValueError):
        synth.emit_mask("nope", 1, 1)


def test_steering_needs_wide_encoder():
    w = synth.make_workload(1, B=1, T=1, len_lo=1, len_hi=1)      # F = 256 < J = 320
    with pytest.raises(ValueError):
        synth.steer_frames(w.model)


def test_token_counts_follow_the_pattern(net_and_inputs):
    for pat in synth.PATTERNS:
        w, net = net_and_inputs[pat]
        S, T = w.max_symbols, w.T
        want = synth.emit_mask(pat, w.B, T).sum(axis=1) * S
        for sched in ("frame", "label", "seq"):
            got = oracle.decode(net, w.enc_out, w.enc_len, S, sched)
            assert got.tok_len.tolist() == want.tolist(), (pat, sched)
            for b in range(w.B):
                # every label sits on an emit frame, S of them per frame
                counts = np.bincount(got.frames[b], minlength=T)
                assert counts.tolist() == (synth.emit_mask(pat, w.B, T)[b] * S).tolist()


def test_alternating_batch_costs_frame_looping_max_symbols_steps_per_frame(net_and_inputs):
    w, net = net_and_inputs["alternating"]
    S, T = w.max_symbols, w.T
    frame = oracle.decode(net, w.enc_out, w.enc_len, S, "frame")
    label = oracle.decode(net, w.enc_out, w.enc_len, S, "label")
    assert frame.stats["inner"] == S * T            # every frame runs the full inner loop
    # label looping: one batched prediction step per label of the longer row (+1 to finish)
    assert label.stats["pred"] == S * T // 2 + 1
    assert label.stats["inner"] < frame.stats["inner"] * 0.7
    for b in range(w.B):
        assert np.array_equal(frame.tokens[b], label.tokens[b])
