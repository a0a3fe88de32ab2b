"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Token sequences, frame indices and durations must be
bit-exact; emitted logits within 1e-4 relative; a differing row is accepted only
at near-ties of the oracle (< 1e-5) and is reported (tests/parity_util.py)."""
import os
import sys

import numpy as np
import pytest

import oracle
import synth
from parity_util import BF16_LOGIT_RTOL, BF16_MARGIN, compare, to_lists

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
N_THREADS = min(16, os.cpu_count() or 1)


def log(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def pkg():
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    import paper_2406_03791_amd as m
    m.load_library()
    return m


_ENGINES = {}


def engine_for(pkg, key, model, max_B, max_T):
    k = (key, max_B, max_T)
    if k not in _ENGINES:
        _ENGINES[k] = pkg.Engine(model, max_B, max_T)
    return _ENGINES[k]


def run_gpu(eng, w, variant, S, cap=None, pad_nan=True, logp=False):
    x = w.enc_out.copy()
    if pad_nan:
        for b in range(w.B):
            x[b, max(0, min(int(w.enc_len[b]), w.T)):, :] = np.nan
    enc = torch.from_numpy(x).cuda().contiguous()
    ln = torch.from_numpy(w.enc_len.astype(np.int32)).cuda()
    done = torch.zeros(w.B, dtype=torch.int32, device="cuda")
    out = eng.decode(variant, enc, ln, S, cap=cap, logp=logp, done=done)
    torch.cuda.synchronize()
    assert bool((done == 1).all()), "every utterance is flagged complete when the call has ended"
    return to_lists(out, w.B), eng.status(), eng.stats()


def check(pkg, w, variant, key, S=None, max_B=None, engine=None, expect_status=0, logp=False,
          bf16=False):
    S = w.max_symbols if S is None else S
    eng = engine or engine_for(pkg, key, w.model, max_B or w.B, w.T)
    net = oracle.LstmNet(w.model, bf16=bf16)
    ref = oracle.decode(net, w.enc_out, w.enc_len, S, "seq", n_threads=N_THREADS)
    got, status, stats = run_gpu(eng, w, variant, S, logp=logp)
    log(f"[{key}/{variant}] B={w.B} T={w.T} S={S} tokens={int(ref.tok_len.sum())} "
        f"status={status} stats={stats}")
    assert status == expect_status
    assert stats["xcd_mismatch"] == 0
    if bf16:
        ties = compare(w, net, ref, got, S, margin=BF16_MARGIN, logit_rtol=BF16_LOGIT_RTOL)
    else:
        ties = compare(w, net, ref, got, S)
    for t in ties:
        log(f"  near-tie divergence accepted: {t}")
    if not bf16:
        assert len(ties) <= max(1, w.B // 8)
    stats["near_tie_rows"] = len(ties)
    return ref, got, stats


def test_encoder_projection_matches_oracle(pkg):
    for cfg, kw in [(1, {}), (2, dict(B=3, T=200, len_lo=130, len_hi=200))]:
        w = synth.make_workload(cfg, pad="nan", **kw)
        eng = engine_for(pkg, f"cfg{cfg}", w.model, w.B, w.T)
        enc = torch.from_numpy(w.enc_out).cuda().contiguous()
        ln = torch.from_numpy(w.enc_len).cuda()
        proj = eng.encoder_projection(enc, ln).cpu().numpy()
        net = oracle.LstmNet(w.model)
        worst = 0.0
        for b in range(w.B):
            n = int(w.enc_len[b])
            for t in range(n):          # every valid frame, element by element
                want = net.prep(w.enc_out[b, t])
                assert np.allclose(proj[b, t], want, rtol=1e-5, atol=2e-5), (cfg, b, t)
                worst = max(worst, float(np.max(np.abs(proj[b, t] - want))))
            assert np.all(proj[b, n:] == 0), "rows beyond enc_len must stay untouched"
        log(f"[projection cfg{cfg}] {int(w.enc_len.sum())} frames x {w.model.dims.J}, worst |diff| {worst:.2e}")


def test_cfg0_tiny_frame_and_label(pkg):
    w = synth.make_workload(0, pad="nan")
    check(pkg, w, "frame", "cfg0")
    check(pkg, w, "label", "cfg0")


def test_cfg1_small_frame_and_label(pkg):
    w = synth.make_workload(1, pad="nan")
    _, a, _ = check(pkg, w, "frame", "cfg1")
    _, b, _ = check(pkg, w, "label", "cfg1")
    assert np.array_equal(a["raw_tokens"], b["raw_tokens"])
    # with one team layout for both decoders the same kernels run on the same operands: same bits
    eng = pkg.Engine(w.model, w.B, w.T)
    eng.configure(n_teams=8)
    a, _, _ = run_gpu(eng, w, "frame", w.max_symbols)
    b, _, _ = run_gpu(eng, w, "label", w.max_symbols)
    eng.close()
    assert np.array_equal(a["raw_tokens"], b["raw_tokens"])
    for i in range(w.B):
        assert np.array_equal(a["logits"][i], b["logits"][i])


def test_cfg1_lookahead_settings_agree(pkg):
    w = synth.make_workload(1, pad="nan")
    eng = engine_for(pkg, "cfg1", w.model, w.B, w.T)
    for variant in ("label", "frame"):
        for la in (1, 3, 8, 16):
            eng.configure(lookahead=la)
            _, _, stats = check(pkg, w, variant, f"cfg1 la={la}", engine=eng)
            assert stats["lookahead"] == la
    eng.configure(lookahead=0)


def test_search_cut_off_settings_agree(pkg):
    """Label looping with the search cut off after 1, 2, 3 joint steps or never, with and
    without joint groups, RNN-T and TDT: the tokens do not change."""
    for cfg, variant, kw in [(3, "label", dict(B=12, T=120, len_lo=40, len_hi=120)),
                             (4, "tdt", dict(B=12, T=120, len_lo=40, len_hi=120))]:
        w = synth.make_workload(cfg, pad="nan", **kw)
        eng = pkg.Engine(w.model, w.B, w.T)
        for n_teams, groups in [(0, 0), (8, 1), (4, 2), (2, 4)]:
            for ss in (-1, 1, 2, 3):
                eng.configure(n_teams=n_teams, joint_groups=groups, search_steps=ss)
                _, _, stats = check(pkg, w, variant, f"cfg{cfg} teams={n_teams}/{groups} ss={ss}",
                                    engine=eng)
                assert stats["search_steps"] == (0 if ss < 0 else ss)
        eng.close()


def test_edge_cases(pkg):
    w = synth.make_workload(1, pad="nan", T=40, len_lo=5, len_hi=40)
    eng = engine_for(pkg, "cfg1", w.model, 8, 200)
    w.enc_len[:] = [0, 1, 40, 7, 0, 33, 2, 40]
    for variant in ("frame", "label"):
        check(pkg, w, variant, "cfg1-edge", engine=eng)
        check(pkg, w, variant, "cfg1-edge-S1", S=1, engine=eng)
    # lengths outside [0, T] are clamped and flagged
    w2 = synth.make_workload(1, pad="normal", T=30, len_lo=10, len_hi=30)
    w2.enc_len[0], w2.enc_len[1] = 99, -4
    for variant in ("frame", "label"):
        check(pkg, w2, variant, "cfg1-clamp", engine=eng, expect_status=1)
    # a ragged batch smaller than the engine's maximum
    w3 = synth.make_workload(1, pad="nan", B=3, T=25, len_lo=10, len_hi=25)
    for variant in ("frame", "label"):
        check(pkg, w3, variant, "cfg1-B3", engine=eng)


def test_all_blank_never_blank_and_capacity(pkg):
    S = 3
    for bias, name in [(1e4, "all-blank"), (-1e4, "never-blank")]:
        w = synth.make_workload(1, T=30, len_lo=5, len_hi=30, model_overrides=dict(blank_bias=bias))
        eng = pkg.Engine(w.model, w.B, w.T)
        for variant in ("frame", "label"):
            ref, got, stats = check(pkg, w, variant, name, S=S, engine=eng)
            if bias > 0:
                assert np.all(got["tok_len"] == 0)
            else:
                assert got["tok_len"].tolist() == (S * w.enc_len).tolist()
        if bias < 0:   # too small a capacity: excess dropped, count kept, bit set
            enc = torch.from_numpy(w.enc_out).cuda()
            ln = torch.from_numpy(w.enc_len).cuda()
            out = eng.decode("label", enc, ln, S, cap=7)
            torch.cuda.synchronize()
            assert eng.status() & 2
            assert out["tok_len"].cpu().numpy().tolist() == (S * w.enc_len).tolist()
        eng.close()


def test_host_side_errors(pkg):
    w = synth.make_workload(0)
    eng = engine_for(pkg, "cfg0", w.model, w.B, w.T)
    enc = torch.from_numpy(w.enc_out).cuda()
    ln = torch.from_numpy(w.enc_len).cuda()
    out = eng.alloc_outputs(1, 60)
    args = lambda **k: dict(dict(eng=eng.handle, enc_out=enc, enc_len=ln, B=1, T=w.T, max_symbols=3,
                                 tokens_out=out["tokens"], tok_len_out=out["tok_len"], cap=60), **k)
    for bad, code in [(dict(B=0), -2), (dict(B=2), -2), (dict(T=w.T + 1), -2),
                      (dict(max_symbols=0), -2), (dict(cap=0), -2), (dict(enc_out=None), -1)]:
        with pytest.raises(pkg.RnntError) as ei:
            pkg.rnnt_greedy_decode(**args(**bad))
        assert ei.value.code == code
    with pytest.raises(pkg.RnntError) as ei:
        pkg.tdt_label_looping_decode(**args())
    assert ei.value.code == -3
    # enc_out must be 16-byte aligned: a view that starts one float into a buffer is refused
    flat = torch.zeros(enc.numel() + 4, dtype=torch.float32, device="cuda")
    shifted = flat[1:1 + enc.numel()].view(enc.shape)
    assert shifted.data_ptr() % 16 != 0
    for fn in (pkg.rnnt_greedy_decode, pkg.rnnt_label_looping_decode, pkg.rnnt_label_looping_decode_noalloc):
        with pytest.raises(pkg.RnntError) as ei:
            fn(**args(enc_out=shifted))
        assert ei.value.code == -2
    with pytest.raises(pkg.RnntError) as ei:
        pkg.rnnt_encoder_projection(eng.handle, shifted, ln, 1, w.T, torch.zeros(1, w.T, 64, device="cuda"))
    assert ei.value.code == -2
    # more frames than 32-bit frame numbers can count are refused when the engine is created
    w2 = synth.make_workload(2, B=1, T=8, len_lo=8, len_hi=8)
    with pytest.raises(pkg.RnntError) as ei:
        pkg.Engine(w2.model, 1 << 20, 1 << 12)
    assert ei.value.code == -5


def test_calls_of_more_utterances_than_one_launch_takes(pkg):
    """A call with more than 128 utterances is decoded by consecutive launches of up to 128: 256
    (two full launches), 300 and 129 (a last launch of 44 and of one utterance) on one engine,
    all decoders, completion flags, log-probabilities, and the call's status and step counts;
    also small batches on an engine whose layouts were planned for 128 (four joint groups)."""
    w = synth.make_workload(2, pad="nan", B=300, T=40, len_lo=10, len_hi=40)
    eng = pkg.Engine(w.model, 300, w.T)
    import dataclasses
    for B in (300, 256, 129, 128, 17, 3, 1):
        wb = dataclasses.replace(w, enc_out=w.enc_out[:B].copy(), enc_len=w.enc_len[:B].copy())
        _, _, st_f = check(pkg, wb, "frame", f"parakeet300/{B}", engine=eng)
        _, _, st_l = check(pkg, wb, "label", f"parakeet300/{B}", engine=eng, logp=True)
        # every utterance takes at least one prediction step in either decoder
        assert st_f["pred_steps"] >= B and st_l["pred_steps"] >= 1
    # one configured layout for launches of every size
    eng.configure(n_teams=16, joint_groups=2)
    check(pkg, w, "label", "parakeet300/16 teams/2 groups", engine=eng)
    check(pkg, w, "frame", "parakeet300/16 teams", engine=eng)
    eng.close()
    w4 = synth.make_workload(4, pad="nan", B=200, T=40, len_lo=10, len_hi=40)
    check(pkg, w4, "tdt", "tdt200")
    # a length out of range in the second launch still sets the call's status bit
    wc = dataclasses.replace(w, enc_len=w.enc_len.copy())
    wc.enc_len[250] = w.T + 5
    eng = pkg.Engine(w.model, 300, w.T)
    x = torch.from_numpy(np.nan_to_num(wc.enc_out)).cuda().contiguous()
    eng.decode("label", x, torch.from_numpy(wc.enc_len.astype(np.int32)).cuda(), wc.max_symbols)
    torch.cuda.synchronize()
    assert eng.status() & 1
    eng.close()


def test_cfg2_cut_and_tdt_cut(pkg):
    w = synth.make_workload(2, pad="nan", B=6, T=40, len_lo=15, len_hi=40)
    check(pkg, w, "frame", "cfg2cut")
    check(pkg, w, "label", "cfg2cut")
    w4 = synth.make_workload(4, pad="nan", B=6, T=60, len_lo=20, len_hi=60)
    check(pkg, w4, "tdt", "cfg4cut")


def test_cfg2_parakeet_frame_looping_full(pkg):
    w = synth.make_workload(2, pad="nan")
    check(pkg, w, "frame", "parakeet")


def test_cfg3_parakeet_label_looping_full_and_batch_sizes(pkg):
    w = synth.make_workload(3, pad="nan")
    ref, got32, _ = check(pkg, w, "label", "parakeet")
    # B = 1: the first utterance, on an engine of its own (one team spanning the chip)
    w1 = synth.make_workload(3, pad="nan", B=1)
    _, got1, _ = check(pkg, w1, "label", "parakeet-b1")
    assert np.array_equal(got1["tokens"][0], got32["tokens"][0])
    # B = 128: four blocks of 32; the first 32 rows are the B = 32 workload
    w128 = synth.make_workload(3, pad="nan", B=128)
    _, got128, _ = check(pkg, w128, "label", "parakeet-b128")
    for b in range(32):
        assert np.array_equal(got128["tokens"][b], got32["tokens"][b])


def test_cfg4_tdt_full(pkg):
    w = synth.make_workload(4, pad="nan")
    check(pkg, w, "tdt", "tdt")


def test_cfg5_second_workload_single_layer_model(pkg):
    # the smaller model's shape (a guess: one LSTM layer at the Parakeet widths), full size
    w = synth.make_workload(5, pad="nan")
    check(pkg, w, "label", "small_model")
    check(pkg, w, "frame", "small_model")


def test_cfg6_multi_blank_transducer(pkg):
    """A multi-blank transducer at the Parakeet shape (two big blanks that skip 2 and 4 frames)
    against the oracle's rule: full size in the default layout, with the score (taken over all
    outputs), one utterance, 128 utterances, other team layouts and lookaheads on a cut, the
    bfloat16 mode, bf16 weight storage, and the decoders that do not run such a model."""
    w = synth.make_workload(6, pad="nan")
    eng = pkg.Engine(w.model, w.B, w.T)
    ref, got, stats = check(pkg, w, "label", "cfg6/full", engine=eng, logp=True)
    V1 = w.model.dims.V1
    assert stats["near_tie_rows"] == 0
    assert max(int(t.max()) for t in ref.tokens if len(t)) < V1 - 1      # big blanks are never emitted
    enc = torch.from_numpy(w.enc_out).cuda().contiguous()
    ln = torch.from_numpy(w.enc_len).cuda()
    for variant in ("frame", "tdt"):
        with pytest.raises(pkg.RnntError):
            eng.decode(variant, enc, ln, w.max_symbols)
    eng.close()
    for B in (1, 128):
        wb = synth.make_workload(6, pad="nan", B=B)
        check(pkg, wb, "label", f"cfg6/B{B}")
    wc = synth.make_workload(6, pad="nan", B=9, T=120, len_lo=40, len_hi=120)
    eng = pkg.Engine(wc.model, wc.B, wc.T)
    for n_teams, groups, la in [(8, 1, 1), (8, 2, 3), (2, 4, 8), (16, 1, 16), (4, 1, 5)]:
        eng.configure(n_teams=n_teams, joint_groups=groups, lookahead=la)
        check(pkg, wc, "label", f"cfg6/cut teams={n_teams}/{groups} la={la}", engine=eng)
    eng.close()
    # the bfloat16 mode, on the cut and at full size, against the emulating oracle
    for wm in (wc, w):
        eng = pkg.Engine(wm.model, wm.B, wm.T, flags=pkg.RNNT_FLAG_BF16_ARITHMETIC)
        _, _, st = check(pkg, wm, "label", f"cfg6/B{wm.B}/bf16 arithmetic", engine=eng, bf16=True, logp=True)
        assert st["near_tie_rows"] <= max(1, wm.B // 3)
        eng.close()
    # the model with bf16-valued streamed weights, stored as bf16 (fp32 arithmetic)
    import dataclasses
    wb = dataclasses.replace(wc, model=synth.with_bf16_streamed_weights(wc.model))
    eng = pkg.Engine(wb.model, wb.B, wb.T, flags=pkg.RNNT_FLAG_BF16_WEIGHTS)
    check(pkg, wb, "label", "cfg6/cut/bf16 weights", engine=eng)
    eng.close()


def test_widths_that_divide_unevenly(pkg):
    """Models whose widths are multiples of 4 and of nothing larger, three layers, a vocabulary
    of 23 and (TDT) three durations: hidden units, projection columns and output groups divide
    unevenly over the ranks, some ranks own none, and every K is padded.  All decoders, the
    default layouts for 3 and 20 utterances and two configured ones, fp32 and the bfloat16 mode."""
    for durations, variants in (((), ("frame", "label")), ((0, 1, 3), ("tdt",))):
        dims = synth.ModelDims(F=48, E=36, H=52, L=3, J=76, V1=23, durations=durations)
        model = synth.make_model(dims, seed=21, weight_range=0.3, blank_bias=1.5)
        for B, T in ((3, 40), (20, 30)):
            x, ln = synth.make_inputs(77 + B, B, T, dims.F, T // 3, T, pad="nan")
            w = synth.Workload("odd", variants[0], model, x, ln, 3)
            for flags, bf16 in ((0, False), (pkg.RNNT_FLAG_BF16_ARITHMETIC, True)):
                eng = pkg.Engine(model, B, T, flags=flags)
                for variant in variants:
                    check(pkg, w, variant, f"odd widths B={B}", engine=eng, bf16=bf16, logp=(variant != "frame"))
                    if B == 20:
                        for n_teams, groups in ((8, 2), (32, 1)):
                            eng.configure(n_teams=n_teams, joint_groups=groups if variant != "frame" else 0)
                            check(pkg, w, variant, f"odd widths teams={n_teams}/{groups}", engine=eng, bf16=bf16)
                        eng.configure()
                eng.close()


def test_wide_joint_and_wide_hidden_layers(pkg):
    """A joint layer wider than the 768 columns a wave holds in registers while it forms z (the
    rest of a row is loaded where it is used), and a hidden width above 1024, for which the
    teams of few utterances use the general prediction step (barriers) instead of the one with
    tagged words."""
    for dims, bias in ((synth.ModelDims(F=64, E=48, H=128, L=2, J=832, V1=33), 1.2),
                       (synth.ModelDims(F=64, E=48, H=1088, L=1, J=832, V1=33), 1.2),
                       (synth.ModelDims(F=64, E=48, H=1088, L=1, J=128, V1=33, durations=(0, 1, 2)), 0.4)):
        model = synth.make_model(dims, seed=31, weight_range=0.1, blank_bias=bias)
        x, ln = synth.make_inputs(91, 3, 24, dims.F, 10, 24, pad="nan")
        variants = ("tdt",) if dims.D else ("frame", "label")
        w = synth.Workload("wide", variants[0], model, x, ln, 3)
        eng = pkg.Engine(model, 3, 24)
        for variant in variants:
            ref, _, _ = check(pkg, w, variant, f"wide H={dims.H} J={dims.J}", engine=eng, logp=(variant == "label"))
            assert int(ref.tok_len.sum()) > 10
        eng.close()


def test_four_layers_and_large_vocabularies(pkg):
    """The largest layer count (4), and vocabularies of 4 097, 16 385 and 60 001 labels: the
    argmax candidates of the large ones fit the local memory only for engines of few utterances
    and, for the largest, only in a layout with more work-groups per team than the preferred
    one, which the engine falls back to; a vocabulary beyond the 16-bit column index of the
    argmax exchange is refused when the engine is created."""
    for dims, bias, sizes in ((synth.ModelDims(F=64, E=64, H=320, L=4, J=320, V1=129), 1.0, (3, 40)),
                              (synth.ModelDims(F=64, E=64, H=320, L=1, J=320, V1=4097), 1.5, (3, 40)),
                              (synth.ModelDims(F=64, E=64, H=320, L=1, J=320, V1=16385), 2.0, (3,)),
                              (synth.ModelDims(F=64, E=64, H=320, L=1, J=320, V1=60001), 1.1, (3,))):
        model = synth.make_model(dims, seed=41, weight_range=0.1, blank_bias=bias)
        for B in sizes:
            x, ln = synth.make_inputs(93, B, 24, dims.F, 10, 24, pad="nan")
            w = synth.Workload("vocab", "label", model, x, ln, 3)
            eng = pkg.Engine(model, B, 24)
            for variant in ("frame", "label"):
                check(pkg, w, variant, f"L={dims.L} V1={dims.V1} B={B}", engine=eng, logp=(variant == "label"))
            eng.close()
    big = synth.make_model(synth.ModelDims(F=64, E=64, H=320, L=1, J=320, V1=65536), seed=41)
    with pytest.raises(pkg.RnntError) as err:
        pkg.Engine(big, 3, 24)
    assert err.value.code == -5


def test_repeat_and_permutation_invariance(pkg):
    w = synth.make_workload(2, pad="nan", B=8, T=60, len_lo=20, len_hi=60)
    eng = engine_for(pkg, "parakeet8", w.model, 8, 60)
    a, _, _ = run_gpu(eng, w, "label", w.max_symbols)
    for _ in range(3):
        b, _, _ = run_gpu(eng, w, "label", w.max_symbols)
        assert np.array_equal(a["raw_tokens"], b["raw_tokens"])
    perm = np.random.default_rng(5).permutation(w.B)
    wp = synth.Workload(w.name, w.variant, w.model, w.enc_out[perm].copy(), w.enc_len[perm].copy(),
                        w.max_symbols)
    p, _, _ = run_gpu(eng, wp, "label", w.max_symbols)
    for i, b in enumerate(perm):
        assert np.array_equal(p["tokens"][i], a["tokens"][b])


def test_adversarial_batches(pkg):
    """Steered inputs: all blank, max_symbols labels on every frame, the alternating batch and
    one slow row among blank ones; Algorithm 1 and label looping against the oracle."""
    eng = None
    for pat in synth.PATTERNS:
        w = synth.make_adversarial(pat, cfg=2, B=5, T=24)
        eng = eng or engine_for(pkg, "cfg2-adv", w.model, 5, 24)
        want = synth.emit_mask(pat, w.B, w.T).sum(axis=1) * w.max_symbols
        for variant in ("frame", "label"):
            ref, got, stats = check(pkg, w, variant, f"adv/{pat}", engine=eng)
            assert ref.tok_len.tolist() == want.tolist()
            assert [len(t) for t in got["tokens"]] == want.tolist()


def test_finished_utterances_are_flagged_while_the_call_runs(pkg):
    # Row 0 emits max_symbols labels on every frame, the other rows only blanks: their
    # results must be readable from pinned host memory, and right, long before row 0 is done.
    import time
    w = synth.make_adversarial("one_slow_row", cfg=2, B=8, T=60)
    net = oracle.LstmNet(w.model)
    ref = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "seq", n_threads=N_THREADS)
    eng = engine_for(pkg, "parakeet_slow_row", w.model, w.B, w.T)
    enc = torch.from_numpy(w.enc_out).cuda()
    ln = torch.from_numpy(w.enc_len).cuda()
    cap = w.T * w.max_symbols
    for variant in ("label", "frame"):
        out = eng.alloc_outputs(w.B, cap, pinned=True)
        done = torch.zeros(w.B, dtype=torch.int32, pin_memory=True)
        flags, lens, toks = done.numpy(), out["tok_len"].numpy(), out["tokens"].numpy()
        stream, end = torch.cuda.Stream(), torch.cuda.Event()
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            eng.decode(variant, enc, ln, w.max_symbols, out=out, done=done)
            end.record()
        seen = {}
        deadline = time.monotonic() + 30.0
        while len(seen) < w.B and time.monotonic() < deadline:
            for b in range(w.B):
                if b not in seen and flags[b] == 1:
                    running = not end.query()      # asked after the flag was seen
                    n = int(lens[b])
                    seen[b] = (running, toks[b, :min(n, cap)].copy())
        stream.synchronize()
        assert eng.status() == 0
        assert sorted(seen) == list(range(w.B))
        early = [b for b in seen if seen[b][0]]
        log(f"[slow row/{variant}] flagged while the kernel ran: rows {early}; "
            f"tokens per row {[len(seen[b][1]) for b in range(w.B)]}")
        for b in range(w.B):
            assert np.array_equal(seen[b][1], ref.tokens[b]), (variant, b)
        assert any(b != 0 for b in early)
        assert len(ref.tokens[0]) == w.T * w.max_symbols


def test_compact_weight_storage(pkg):
    """Engines with the streamed weights kept as bf16 or as 8-bit e4m3 (lossless storage of a
    model whose streamed matrices hold such values) against the oracle on that same model; a
    model with other values is refused.  Also logs how many rows differ from the decode of the
    unrounded model."""
    import dataclasses
    kinds = [("bf16w", pkg.RNNT_FLAG_BF16_WEIGHTS, synth.with_bf16_streamed_weights),
             ("fp8w", pkg.RNNT_FLAG_FP8_WEIGHTS, synth.with_fp8_streamed_weights)]
    for cfg, variants, kw in [(3, ("frame", "label"), dict(B=6, T=120, len_lo=40, len_hi=120)),
                              (4, ("tdt",), dict(B=6, T=120, len_lo=40, len_hi=120)),
                              (1, ("frame", "label"), {})]:
        w32 = synth.make_workload(cfg, pad="nan", **kw)
        ref32 = oracle.decode(oracle.LstmNet(w32.model), w32.enc_out, w32.enc_len, w32.max_symbols,
                              "seq", n_threads=N_THREADS)
        for name, flag, transform in kinds:
            with pytest.raises(pkg.RnntError) as err:
                pkg.Engine(w32.model, w32.B, w32.T, flags=flag)
            assert err.value.code == -2
            w = dataclasses.replace(w32, model=transform(w32.model))
            eng = pkg.Engine(w.model, w.B, w.T, flags=flag)
            for variant in variants:
                ref, got, _ = check(pkg, w, variant, f"cfg{cfg}/{name}", engine=eng)
                moved = sum(int(not np.array_equal(ref.tokens[b], ref32.tokens[b])) for b in range(w.B))
                log(f"  rows whose tokens differ from the fp32 model's: {moved}/{w.B}")
            eng.close()
    # unknown flag bits and both storage flags at once are refused
    w8 = dataclasses.replace(w32, model=synth.with_fp8_streamed_weights(w32.model))
    for flags in (64, pkg.RNNT_FLAG_BF16_WEIGHTS | pkg.RNNT_FLAG_FP8_WEIGHTS):
        with pytest.raises(pkg.RnntError) as err:
            pkg.Engine(w8.model, w8.B, w8.T, flags=flags)
        assert err.value.code == -2


def test_log_probabilities(pkg):
    """The optional log-softmax output (fused log-sum-exp over the ranks) against the oracle's,
    for the three decoders, with and without joint groups; asking for it changes no token, and
    a later call without it leaves the buffer alone."""
    for cfg, variants, kw in [(1, ("frame", "label"), {}),
                              (3, ("frame", "label"), dict(B=9, T=100, len_lo=30, len_hi=100)),
                              (4, ("tdt",), dict(B=9, T=100, len_lo=30, len_hi=100))]:
        w = synth.make_workload(cfg, pad="nan", **kw)
        eng = pkg.Engine(w.model, w.B, w.T)
        for variant in variants:
            for n_teams, groups in [(0, 0), (8, 1), (2, 4)]:
                eng.configure(n_teams=n_teams, joint_groups=groups)
                _, got, _ = check(pkg, w, variant, f"cfg{cfg}/logp teams={n_teams}/{groups}",
                                  engine=eng, logp=True)
                assert all(np.all(x <= 1e-6) for x in got["logps"])
                _, plain, _ = check(pkg, w, variant, f"cfg{cfg}/no logp", engine=eng)
                assert np.array_equal(plain["raw_tokens"], got["raw_tokens"])
        eng.close()


def test_full_size_label_looping_with_scores_and_compact_storage(pkg):
    """Config 3 at its full size, in the launch configuration bench.py times: label looping with
    the log-probability output, and the same on the bf16-valued model stored as bf16 and the
    e4m3-valued model stored as e4m3."""
    import dataclasses
    w = synth.make_workload(3, pad="nan")
    check(pkg, w, "label", "cfg3/full/logp", logp=True)
    wb = dataclasses.replace(w, model=synth.with_bf16_streamed_weights(w.model))
    eng = pkg.Engine(wb.model, wb.B, wb.T, flags=pkg.RNNT_FLAG_BF16_WEIGHTS)
    check(pkg, wb, "label", "cfg3/full/bf16w", engine=eng, logp=True)
    check(pkg, wb, "frame", "cfg2/full/bf16w", engine=eng)
    eng.close()
    w8 = dataclasses.replace(w, model=synth.with_fp8_streamed_weights(w.model))
    eng = pkg.Engine(w8.model, w8.B, w8.T, flags=pkg.RNNT_FLAG_FP8_WEIGHTS)
    check(pkg, w8, "label", "cfg3/full/fp8w", engine=eng, logp=True)
    check(pkg, w8, "frame", "cfg2/full/fp8w", engine=eng)
    eng.close()


def test_row_group_counts_between_the_kernel_instances(pkg):
    """Teams of 9-12 utterances run the prediction kernels built for 16 rows: the LDS layout has
    to be sized for the instance, not for the rows.  96 utterances on 8 teams (12 rows per
    team), 4 teams with 40 utterances (10 rows), and 160 utterances in the default layouts (two
    launches)."""
    w = synth.make_workload(3, pad="nan", B=160, T=40, len_lo=10, len_hi=40)
    check(pkg, w, "label", "parakeet160")
    check(pkg, w, "frame", "parakeet160")
    w96 = synth.make_workload(3, pad="nan", B=96, T=40, len_lo=10, len_hi=40)
    eng = pkg.Engine(w96.model, w96.B, w96.T)
    eng.configure(n_teams=8, joint_groups=2)
    check(pkg, w96, "label", "parakeet96/8 teams/2 groups", engine=eng)
    check(pkg, w96, "frame", "parakeet96/8 teams", engine=eng)
    eng.close()
    w40 = synth.make_workload(3, pad="nan", B=40, T=40, len_lo=10, len_hi=40)
    eng = pkg.Engine(w40.model, w40.B, w40.T)
    eng.configure(n_teams=4)
    check(pkg, w40, "label", "parakeet40/4 teams", engine=eng)
    check(pkg, w40, "frame", "parakeet40/4 teams", engine=eng)
    eng.configure(n_teams=4, joint_groups=2)
    check(pkg, w40, "label", "parakeet40/4 teams/2 groups", engine=eng)
    eng.close()
    w4 = synth.make_workload(4, pad="nan", B=44, T=40, len_lo=10, len_hi=40)
    eng = pkg.Engine(w4.model, w4.B, w4.T)
    eng.configure(n_teams=4)
    check(pkg, w4, "tdt", "tdt44/4 teams", engine=eng)
    eng.close()


def test_joint_steps_between_the_kernel_instances(pkg):
    """Joint steps of 17-31 samples run the kernels built for 32: the z rows and the stride of
    the partial sums have to be those of that instance.  max_B = 96 and 80 in the default
    label-looping layout (3 rows per joint group x 8 frames = 24 samples), TDT at 72, and
    lookaheads that give 18, 20, 25 and 28 samples."""
    w = synth.make_workload(3, pad="nan", B=96, T=48, len_lo=10, len_hi=48)
    check(pkg, w, "label", "parakeet96")
    check(pkg, w, "frame", "parakeet96")
    eng = pkg.Engine(w.model, w.B, w.T)
    eng.configure(lookahead=6)                      # 3 rows x 6 frames
    check(pkg, w, "frame", "parakeet96/lookahead 6", engine=eng)
    check(pkg, w, "label", "parakeet96/lookahead 6", engine=eng)
    eng.close()
    w80 = synth.make_workload(3, pad="nan", B=80, T=48, len_lo=10, len_hi=48)
    check(pkg, w80, "label", "parakeet80")
    w40 = synth.make_workload(3, pad="nan", B=40, T=40, len_lo=10, len_hi=40)
    eng = pkg.Engine(w40.model, w40.B, w40.T)
    for la in (4, 5):                               # 5 rows per joint group x 4 or 5 frames
        eng.configure(n_teams=4, joint_groups=2, lookahead=la)
        check(pkg, w40, "label", f"parakeet40/4 teams/2 groups/lookahead {la}", engine=eng)
    eng.close()
    w56 = synth.make_workload(3, pad="nan", B=56, T=40, len_lo=10, len_hi=40)
    eng = pkg.Engine(w56.model, w56.B, w56.T)       # 7 rows per team x 4 frames
    eng.configure(n_teams=8, joint_groups=1, lookahead=4)
    check(pkg, w56, "label", "parakeet56/8 teams/lookahead 4", engine=eng)
    eng.close()
    w4 = synth.make_workload(4, pad="nan", B=72, T=48, len_lo=10, len_hi=48)
    check(pkg, w4, "tdt", "tdt72")


def test_every_default_layout_class_of_the_parakeet_shape(pkg):
    """Engines of many sizes, each decoding a full batch of short utterances in its default
    layout: every combination of rows per team, joint groups and lookahead the defaults
    produce between 1 and 256 utterances is run once against the oracle."""
    sizes = [1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 24, 31, 33, 40, 48, 56, 63, 65, 72, 88, 104, 112,
             120, 129, 144, 176, 192, 208, 224, 240, 255, 256]
    for B in sizes:
        w = synth.make_workload(3, pad="nan", B=B, T=16, len_lo=5, len_hi=16)
        eng = pkg.Engine(w.model, w.B, w.T)
        check(pkg, w, "label", f"parakeet{B}", engine=eng)
        check(pkg, w, "frame", f"parakeet{B}", engine=eng)
        eng.close()
    for B in [3, 9, 20, 36, 66, 90, 100, 136, 200, 250]:
        w = synth.make_workload(4, pad="nan", B=B, T=16, len_lo=5, len_hi=16)
        eng = pkg.Engine(w.model, w.B, w.T)
        check(pkg, w, "tdt", f"tdt{B}", engine=eng)
        eng.close()


def test_default_layout_classes_of_the_other_weight_forms(pkg):
    """The LDS layout depends on the K values a load carries: the same sweep, coarser, for bf16
    and e4m3 storage and for the bfloat16 arithmetic with bf16, e4m3 or e2m1 storage."""
    import dataclasses
    forms = [("bf16w", pkg.RNNT_FLAG_BF16_WEIGHTS, synth.with_bf16_streamed_weights, False),
             ("fp8w", pkg.RNNT_FLAG_FP8_WEIGHTS, synth.with_fp8_streamed_weights, False),
             ("bf16 arithmetic", pkg.RNNT_FLAG_BF16_ARITHMETIC, None, True),
             ("bf16 arithmetic/fp8w", pkg.RNNT_FLAG_BF16_ARITHMETIC | pkg.RNNT_FLAG_FP8_WEIGHTS,
              synth.with_fp8_streamed_weights, True),
             ("bf16 arithmetic/fp4w", pkg.RNNT_FLAG_BF16_ARITHMETIC | pkg.RNNT_FLAG_FP4_WEIGHTS,
              lambda m: synth.with_streamed_weights(m, lambda a: oracle.quantize_blocks_e2m1(a)[0]), True)]
    for B in [5, 24, 72, 104, 160, 256]:
        for cfg, variants in [(3, ("label", "frame")), (4, ("tdt",))]:
            w0 = synth.make_workload(cfg, pad="nan", B=B, T=16, len_lo=5, len_hi=16)
            for name, flag, transform, bf16 in forms:
                w = dataclasses.replace(w0, model=transform(w0.model)) if transform else w0
                eng = pkg.Engine(w.model, w.B, w.T, flags=flag)
                for variant in variants:
                    check(pkg, w, variant, f"cfg{cfg}/{name}/{B}", engine=eng, bf16=bf16)
                eng.close()


def test_optional_outputs_may_be_null(pkg):
    """frames_out, logit_out and durations_out are optional in the C ABI: with NULL for all of
    them every decoder still writes the same tokens and counts."""
    for cfg, variants, kw in [(1, ("frame", "label"), {}),
                              (4, ("tdt",), dict(B=6, T=60, len_lo=20, len_hi=60))]:
        w = synth.make_workload(cfg, pad="nan", **kw)
        eng = engine_for(pkg, f"cfg{cfg}-null", w.model, w.B, w.T)
        enc = torch.from_numpy(w.enc_out).cuda().contiguous()
        ln = torch.from_numpy(w.enc_len).cuda()
        cap = w.T * w.max_symbols
        for variant in variants:
            full, status, _ = run_gpu(eng, w, variant, w.max_symbols)
            assert status == 0
            tokens = torch.full((w.B, cap), 7, dtype=torch.int32, device="cuda")
            tok_len = torch.full((w.B,), -3, dtype=torch.int32, device="cuda")
            pkg.rnnt_engine_set_logp_output(eng.handle, None)
            pkg.rnnt_engine_set_done_flags(eng.handle, None)
            fn = {"frame": pkg.rnnt_greedy_decode, "label": pkg.rnnt_label_looping_decode,
                  "tdt": pkg.tdt_label_looping_decode}[variant]
            fn(eng.handle, enc, ln, w.B, w.T, w.max_symbols, tokens, tok_len, cap)   # the rest NULL
            torch.cuda.synchronize()
            assert eng.status() == 0
            assert np.array_equal(tok_len.cpu().numpy(), full["tok_len"])
            assert np.array_equal(tokens.cpu().numpy(), full["raw_tokens"])
            log(f"[null outputs cfg{cfg}/{variant}] {int(full['tok_len'].sum())} tokens equal")


def test_soak_repeated_calls_give_the_same_tokens(pkg):
    """The team barriers and tagged exchanges are built on relaxed device-scope atomics: a race
    would show as a run that differs.  200 calls per decoder on one engine at the full size of
    configurations 2 and 3 (B = 32), every output compared with the first call's, which is
    compared with the oracle; stops at the first difference or status bit."""
    w = synth.make_workload(3, pad="nan")
    eng = engine_for(pkg, "parakeet", w.model, w.B, w.T)
    enc = torch.from_numpy(w.enc_out).cuda().contiguous()
    ln = torch.from_numpy(w.enc_len).cuda()
    for variant in ("label", "frame"):
        _, first, _ = check(pkg, w, variant, "soak/first", engine=eng)
        ref_tok = torch.from_numpy(first["raw_tokens"]).cuda()
        ref_len = torch.from_numpy(first["tok_len"]).cuda()
        out = eng.alloc_outputs(w.B, w.T * w.max_symbols)
        for i in range(200):
            eng.decode(variant, enc, ln, w.max_symbols, out=out)
            same = bool(torch.equal(out["tokens"], ref_tok)) and bool(torch.equal(out["tok_len"], ref_len))
            status = eng.status()
            assert status == 0, f"{variant}: call {i} ended with status {status}"
            assert same, f"{variant}: call {i} differs from the first call"
        log(f"[soak/{variant}] 200 calls identical to the first")


def test_more_joint_steps_than_the_exchange_tag_counts(pkg):
    """The argmax partials carry a 16-bit step tag.  A never-blank decode of the tiny model over
    6 600 frames takes more than 65 536 joint steps in one call; the tokens must still be the
    oracle's (max_symbols labels on every frame)."""
    w = synth.make_workload(0, T=6600, len_lo=6600, len_hi=6600,
                            model_overrides=dict(blank_bias=-1e4))
    w.max_symbols = 10
    eng = pkg.Engine(w.model, w.B, w.T)
    for variant in ("frame", "label"):
        ref, got, stats = check(pkg, w, variant, "tag wrap", engine=eng)
        assert stats["joint_steps"] > 65536
        assert got["tok_len"].tolist() == [66000]
    eng.close()


def test_bf16_arithmetic_mode(pkg):
    """The bfloat16 mode (weights and every input of a dense product rounded to bfloat16, fp32
    sums) against the oracle's bfloat16 emulation, to the same bar as the fp32 path: tokens,
    frames and durations exact, logits within 1e-4, a differing row only at near-ties.  Also
    logs how many rows decode differently from the fp32 arithmetic on the same model, and checks
    the projection kernel of the mode element by element."""
    flag = pkg.RNNT_FLAG_BF16_ARITHMETIC
    for cfg, variants, kw in [(1, ("frame", "label"), {}),
                              (3, ("frame", "label"), dict(B=12, T=120, len_lo=40, len_hi=120)),
                              (4, ("tdt",), dict(B=12, T=120, len_lo=40, len_hi=120)),
                              (3, ("label", "frame"), {}), (4, ("tdt",), {})]:
        w = synth.make_workload(cfg, pad="nan", **kw)
        eng = pkg.Engine(w.model, w.B, w.T, flags=flag)
        ref32 = oracle.decode(oracle.LstmNet(w.model), w.enc_out, w.enc_len, w.max_symbols, "seq",
                              n_threads=N_THREADS)
        for variant in variants:
            ref, got, st = check(pkg, w, variant, f"cfg{cfg}/bf16 arithmetic", engine=eng, bf16=True,
                                 logp=(variant == "label"))
            same = sum(int(np.array_equal(ref.tokens[b], got["tokens"][b])) for b in range(w.B))
            log(f"  rows token-identical to the emulating oracle: {same}/{w.B}; rows accepted at a "
                f"bfloat16 near-tie: {st['near_tie_rows']}")
            assert st["near_tie_rows"] <= max(1, w.B // 3)
            moved = sum(int(not np.array_equal(ref.tokens[b], ref32.tokens[b])) for b in range(w.B))
            log(f"  rows whose tokens differ from the fp32 arithmetic's: {moved}/{w.B}")
        if w.B <= 12:
            enc = torch.from_numpy(w.enc_out).cuda().contiguous()
            ln = torch.from_numpy(w.enc_len).cuda()
            proj = eng.encoder_projection(enc, ln).cpu().numpy()
            net = oracle.LstmNet(w.model, bf16=True)
            for b in range(w.B):
                for t in range(0, int(w.enc_len[b]), 7):
                    assert np.allclose(proj[b, t], net.prep(w.enc_out[b, t]), rtol=1e-5, atol=2e-5), (cfg, b, t)
        eng.close()
    # the mode excludes bf16 storage of fp32-arithmetic engines
    with pytest.raises(pkg.RnntError) as err:
        pkg.Engine(w.model, w.B, w.T, flags=flag | pkg.RNNT_FLAG_BF16_WEIGHTS)
    assert err.value.code == -2


def test_e4m3_codes_widen_to_their_bf16_values(pkg):
    """The conversion instruction of the bfloat16 mode with e4m3-stored weights, on every code in
    every byte position, against the format's definition (1 sign, 4 exponent bits with bias 7, 3
    mantissa bits, subnormals m * 2^-9, the two all-ones codes NaN): every finite e4m3 value
    is a bf16 value, so the result must be that value exactly, times the power of two of the
    scale operand (a weight row's scale); the operand's mantissa is ignored."""
    for scale, factor in [(1.0, 1.0), (2.0 ** -12, 2.0 ** -12), (32.0, 32.0), (2.0 ** -30, 2.0 ** -30),
                          (1.5, 1.0), (0.75, 0.5)]:
        got = pkg.rnnt_probe_e4m3_widening(scale)
        for code in range(256):
            sign, expo, mant = code >> 7, (code >> 3) & 15, code & 7
            if expo == 15 and mant == 7:
                want = None                                   # NaN
            elif expo == 0:
                want = mant * 2.0 ** -9 * factor
            else:
                want = (1 + mant / 8.0) * 2.0 ** (expo - 7) * factor
            for pos in range(4):
                bits = np.array([int(got[pos, code]) << 16], dtype=np.uint32).view(np.float32)[0]
                if want is None:
                    assert np.isnan(bits), (scale, code, pos)
                else:
                    assert bits == np.float32(-want if sign else want), (scale, code, pos, bits)
                    assert np.signbit(bits) == bool(sign), (scale, code, pos)


def test_bf16_arithmetic_with_e4m3_weights(pkg):
    """Weight-only 8-bit form of the bfloat16 mode: the streamed weights are e4m3 values, stored
    as such and widened to bf16 for the bf16 matrix instructions.  Reference: the oracle's
    bfloat16 emulation on that model, to the bar of the bfloat16 mode.  A model with other
    weights is refused."""
    import dataclasses
    flags = pkg.RNNT_FLAG_BF16_ARITHMETIC | pkg.RNNT_FLAG_FP8_WEIGHTS
    for cfg, variants, kw in [(1, ("frame", "label"), {}),
                              (3, ("frame", "label"), dict(B=12, T=120, len_lo=40, len_hi=120)),
                              (4, ("tdt",), dict(B=12, T=120, len_lo=40, len_hi=120)),
                              (3, ("label", "frame"), {}), (4, ("tdt",), {}),
                              (3, ("label",), dict(B=128, T=100, len_lo=30, len_hi=100))]:
        w0 = synth.make_workload(cfg, pad="nan", **kw)
        w = dataclasses.replace(w0, model=synth.with_fp8_streamed_weights(w0.model))
        eng = pkg.Engine(w.model, w.B, w.T, flags=flags)
        for variant in variants:
            ref, got, st = check(pkg, w, variant, f"cfg{cfg}/bf16 arithmetic, e4m3 weights", engine=eng,
                                 bf16=True, logp=(variant == "label"))
            same = sum(int(np.array_equal(ref.tokens[b], got["tokens"][b])) for b in range(w.B))
            log(f"  rows token-identical to the emulating oracle: {same}/{w.B}; rows accepted at a "
                f"bfloat16 near-tie: {st['near_tie_rows']}")
            assert st["near_tie_rows"] <= max(1, w.B // 3)
        eng.close()
    with pytest.raises(pkg.RnntError) as err:      # weights that are not e4m3 values
        pkg.Engine(w0.model, w0.B, w0.T, flags=flags)
    assert err.value.code == -2


def test_weight_only_8_bit_quantised_models(pkg):
    """Any model, quantised row by row to e4m3 codes with a power-of-two scale (the library's
    host-side quantiser; the oracle's own gives the same matrices), decoded in the bfloat16 mode
    with those codes as the stored weights.  Reference: the oracle's bfloat16 emulation on the
    quantised model, to the bar of the bfloat16 mode.  Rows are also given very different
    magnitudes, so that the scales matter.  Logs how far the decode moves from the fp32 one."""
    import dataclasses
    flags = pkg.RNNT_FLAG_BF16_ARITHMETIC | pkg.RNNT_FLAG_FP8_WEIGHTS
    for cfg, variants, kw, spread in [(1, ("frame", "label"), {}, False),
                                      (3, ("frame", "label"), dict(B=12, T=120, len_lo=40, len_hi=120), True),
                                      (4, ("tdt",), dict(B=12, T=120, len_lo=40, len_hi=120), True),
                                      (3, ("label", "frame"), {}, False), (4, ("tdt",), {}, False),
                                      (6, ("label",), dict(B=12, T=120, len_lo=40, len_hi=120), False)]:
        w0 = synth.make_workload(cfg, pad="nan", **kw)
        model = w0.model
        if spread:
            # output rows of W_pred scaled by powers of two between 2^-10 and 2^6, undone in
            # the columns of W_out: the same function, rows of very different magnitudes
            rng = np.random.default_rng(5)
            f = np.ldexp(1.0, rng.integers(-10, 7, size=model.w_pred.shape[0])).astype(np.float32)
            model = dataclasses.replace(model, w_pred=model.w_pred * f[:, None], b_pred=model.b_pred * f,
                                        w_out=model.w_out / f[None, :])
            model = dataclasses.replace(model, w_enc=model.w_enc * f[:, None], b_enc=model.b_enc * f)
        m_lib = synth.with_streamed_weights(model, lambda a: pkg.rnnt_quantize_rows_e4m3(a)[0])
        m_orc = synth.with_streamed_weights(model, lambda a: oracle.quantize_rows_e4m3(a)[0])
        for a, b in [(m_lib.w_pred, m_orc.w_pred), (m_lib.w_out, m_orc.w_out)] + \
                list(zip(m_lib.w_hh, m_orc.w_hh)) + list(zip(m_lib.w_ih, m_orc.w_ih)):
            assert np.array_equal(a, b)
        w = dataclasses.replace(w0, model=m_orc)
        eng = pkg.Engine(m_lib, w.B, w.T, flags=flags)
        ref32 = oracle.decode(oracle.LstmNet(model), w.enc_out, w.enc_len, w.max_symbols, "seq",
                              n_threads=N_THREADS)
        for variant in variants:
            ref, got, st = check(pkg, w, variant, f"cfg{cfg}/quantised to e4m3 rows", engine=eng,
                                 bf16=True, logp=(variant == "label"))
            assert st["near_tie_rows"] <= max(1, w.B // 3)
            moved = sum(int(not np.array_equal(ref.tokens[b], ref32.tokens[b])) for b in range(w.B))
            log(f"  rows whose tokens differ from the fp32 decode of the unquantised model: {moved}/{w.B}")
        eng.close()
    # a row that no power of two brings onto the e4m3 grid is refused
    bad = dataclasses.replace(m_lib, w_pred=m_lib.w_pred.copy())
    bad.w_pred[3, 5] = np.float32(bad.w_pred[3, 5]) * np.float32(1.01)
    with pytest.raises(pkg.RnntError) as err:
        pkg.Engine(bad, w.B, w.T, flags=flags)
    assert err.value.code == -2


def test_e2m1_codes_widen_to_their_bf16_values(pkg):
    """The conversion instruction of the 4-bit form, on every byte value in every byte position,
    against the format's definition (1 sign, 2 exponent bits with bias 1, 1 mantissa bit; the low
    nibble is the first code), under several scale operands."""
    mags = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    for scale, factor in [(1.0, 1.0), (2.0 ** -12, 2.0 ** -12), (32.0, 32.0), (2.0 ** -30, 2.0 ** -30), (1.5, 1.0)]:
        got = pkg.rnnt_probe_e2m1_widening(scale)
        for byte in range(256):
            for half, code in enumerate((byte & 15, byte >> 4)):
                want = np.float32(mags[code & 7] * factor * (-1.0 if code & 8 else 1.0))
                for pos in range(4):
                    bits = np.array([int(got[pos, byte, half]) << 16], dtype=np.uint32).view(np.float32)[0]
                    assert bits == want and np.signbit(bits) == bool(code & 8), (scale, byte, half, pos, bits)


def test_weight_only_4_bit_quantised_models(pkg):
    """Any model, quantised to e2m1 codes with a power-of-two scale per block of 128 weights of a
    row (the library's host-side quantiser; the oracle's own gives the same matrices), decoded
    in the bfloat16 mode with those codes as the stored weights.  Reference: the oracle's
    bfloat16 emulation on the quantised model, to the bar of the bfloat16 mode."""
    import dataclasses
    flags = pkg.RNNT_FLAG_BF16_ARITHMETIC | pkg.RNNT_FLAG_FP4_WEIGHTS
    for cfg, variants, kw in [(1, ("frame", "label"), {}),
                              (3, ("frame", "label"), dict(B=12, T=120, len_lo=40, len_hi=120)),
                              (4, ("tdt",), dict(B=12, T=120, len_lo=40, len_hi=120)),
                              (3, ("label", "frame"), {}), (4, ("tdt",), {}),
                              (5, ("label", "frame"), dict(B=12, T=120, len_lo=40, len_hi=120)),
                              (6, ("label",), dict(B=12, T=120, len_lo=40, len_hi=120)),
                              (3, ("label",), dict(B=128, T=60, len_lo=20, len_hi=60))]:
        w0 = synth.make_workload(cfg, pad="nan", **kw)
        m_lib = synth.with_streamed_weights(w0.model, lambda a: pkg.rnnt_quantize_blocks_e2m1(a)[0])
        m_orc = synth.with_streamed_weights(w0.model, lambda a: oracle.quantize_blocks_e2m1(a)[0])
        for a, b in [(m_lib.w_pred, m_orc.w_pred), (m_lib.w_out, m_orc.w_out)] + \
                list(zip(m_lib.w_hh, m_orc.w_hh)) + list(zip(m_lib.w_ih, m_orc.w_ih)):
            assert np.array_equal(a, b)
        w = dataclasses.replace(w0, model=m_orc)
        eng = pkg.Engine(m_lib, w.B, w.T, flags=flags)
        ref32 = oracle.decode(oracle.LstmNet(w0.model), w.enc_out, w.enc_len, w.max_symbols, "seq",
                              n_threads=N_THREADS)
        for variant in variants:
            ref, got, st = check(pkg, w, variant, f"cfg{cfg}/quantised to e2m1 blocks", engine=eng,
                                 bf16=True, logp=(variant == "label"))
            assert st["near_tie_rows"] <= max(1, w.B // 3)
            moved = sum(int(not np.array_equal(ref.tokens[b], ref32.tokens[b])) for b in range(w.B))
            log(f"  rows whose tokens differ from the fp32 decode of the unquantised model: {moved}/{w.B}")
        eng.close()
    # refused: a weight off its block's grid; the flag without the bfloat16 mode; two formats
    bad = dataclasses.replace(m_lib, w_pred=m_lib.w_pred.copy())
    bad.w_pred[3, 5] = np.float32(bad.w_pred[3, 5] * 1.01 + 1e-6)
    for model, fl in [(bad, flags), (m_lib, pkg.RNNT_FLAG_FP4_WEIGHTS),
                      (m_lib, flags | pkg.RNNT_FLAG_FP8_WEIGHTS)]:
        with pytest.raises(pkg.RnntError) as err:
            pkg.Engine(model, w.B, w.T, flags=fl)
        assert err.value.code == -2


def test_a_wait_that_expires_ends_the_call_with_the_aborted_bit(pkg):
    """The failure path, forced from the host: with a wait limit of 0 polls the first wait on
    another work-group gives up, every other wait follows, and each launch ends in the ordinary
    way with RNNT_DEV_ABORTED.  The next call on the engine, with the default limit back,
    decodes as if nothing had happened."""
    w = synth.make_workload(1)
    eng = pkg.Engine(w.model, w.B, w.T)
    for bad in (-2, 1 << 32):
        with pytest.raises(pkg.RnntError) as ei:
            eng.set_wait_limit(bad)
        assert ei.value.code == -2
    enc = torch.from_numpy(w.enc_out).cuda().contiguous()
    ln = torch.from_numpy(w.enc_len).cuda()
    for variant in ("frame", "label"):
        check(pkg, w, variant, "abort/before", engine=eng)
        eng.set_wait_limit(0)
        eng.decode(variant, enc, ln, w.max_symbols)
        torch.cuda.synchronize()
        status = eng.status()
        log(f"[abort/{variant}] status with a wait limit of 0 polls: {status}")
        assert status & pkg.RNNT_DEV_ABORTED
        eng.set_wait_limit(-1)
        check(pkg, w, variant, "abort/after", engine=eng)
    eng.close()


def test_engines_side_by_side_and_engine_lifetime(pkg):
    """Calls of two engines (an RNN-T and a TDT model) queued back to back on one side stream
    with no host synchronisation between them, each engine twice with different inputs: the
    stream alone orders them and every result is the oracle's.  Then engines created, used and
    destroyed in a row: the device memory they held comes back."""
    wa1 = synth.make_workload(1, B=6, T=50, len_lo=10, len_hi=50)
    wt1 = synth.make_workload(4, B=5, T=40, len_lo=10, len_hi=40)
    rows = lambda w, r: synth.Workload(w.name, w.variant, w.model, w.enc_out[r].copy(), w.enc_len[r].copy(),
                                       w.max_symbols)
    wa2, wt2 = rows(wa1, [5, 2, 0]), rows(wt1, [4, 1])
    ea, et = pkg.Engine(wa1.model, 6, 50), pkg.Engine(wt1.model, 5, 40)
    side = torch.cuda.Stream()
    queued = []
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for eng, w, variant in ((ea, wa1, "label"), (et, wt1, "tdt"), (ea, wa2, "frame"), (et, wt2, "tdt")):
            enc = torch.from_numpy(w.enc_out).cuda().contiguous()
            ln = torch.from_numpy(w.enc_len.astype(np.int32)).cuda()
            queued.append((w, variant, eng.decode(variant, enc, ln, w.max_symbols), enc, ln))
    side.synchronize()
    assert ea.status() == 0 and et.status() == 0
    for w, variant, out, _, _ in queued:
        net = oracle.LstmNet(w.model)
        ref = oracle.decode(net, w.enc_out, w.enc_len, w.max_symbols, "seq", n_threads=N_THREADS)
        compare(w, net, ref, to_lists(out, w.B), w.max_symbols)
    ea.close(); et.close()
    enc = torch.from_numpy(wa1.enc_out).cuda().contiguous()
    ln = torch.from_numpy(wa1.enc_len.astype(np.int32)).cuda()
    first, free = None, []
    for i in range(16):
        eng = pkg.Engine(wa1.model, 64, 200)
        out = eng.decode("label", enc, ln, wa1.max_symbols)
        torch.cuda.synchronize()
        tok = out["tokens"].cpu().numpy()
        first = tok if first is None else first
        assert np.array_equal(tok, first) and eng.status() == 0
        eng.close()
        del out
        torch.cuda.synchronize()
        free.append(torch.cuda.mem_get_info()[0])
    # the first engines also pay for what the runtime and torch's allocator keep once
    free_before, free_after = free[3], free[-1]
    log(f"[lifetime] free memory after each engine, MiB below the first: {[(free[0] - x) >> 20 for x in free]}")
    assert free_before - free_after < (16 << 20), "engines give their device memory back"


def test_random_shapes_layouts_and_lookaheads(pkg):
    """Seeded random models (widths that are multiples of 4 and nothing else in particular, 1-4
    layers, vocabularies of 2-200; RNN-T, TDT and multi-blank models), batches, team layouts, joint
    groups, lookaheads and max_symbols, fp32 and the bfloat16 mode with bf16, e4m3 and e2m1
    storage: each case against the oracle.
    A layout the planner refuses (it does not divide the device, or does not fit) is skipped."""
    rng = np.random.default_rng(int(os.environ.get("RNNT_RANDOM_SEED", "2406")))
    ran = 0
    n_cases = int(os.environ.get("RNNT_RANDOM_CASES", "136"))      # more, or another seed, for a longer run
    for case in range(n_cases):
        big = case % 136 >= 120                # some cases: wide layers, large vocabularies, up to 96 utterances
        kind = str(rng.choice(["rnnt", "rnnt", "rnnt", "tdt", "tdt", "multi-blank"]))
        tdt = kind == "tdt"
        durations = tuple(sorted(set([0] + list(rng.integers(1, 5, size=rng.integers(1, 4)))))) if tdt else ()
        spans = tuple(int(x) for x in sorted(set(rng.integers(2, 6, size=rng.integers(1, 3))))) if kind == "multi-blank" else ()
        dims = synth.ModelDims(F=int(rng.choice([16, 48, 128])), E=int(rng.integers(4, 80)),
                               H=4 * int(rng.integers(100, 257) if big else rng.integers(1, 41)),
                               L=int(rng.integers(1, 5)),
                               J=4 * int(rng.integers(100, 257) if big else rng.integers(1, 61)),
                               V1=int(rng.integers(500, 5001) if big else rng.integers(2, 201)),
                               durations=tuple(int(d) for d in durations), big_blanks=spans)
        model = synth.make_model(dims, seed=1000 + case, weight_range=0.3 if not big else 0.1,
                                 blank_bias=float(rng.uniform(0.5, 2.0)))
        B, T, S = int(rng.integers(1, 97 if big else 49)), int(rng.integers(4, 21 if big else 31)), int(rng.integers(1, 5))
        # (every third case: lengths from zero on, so some utterances are empty)
        x, ln = synth.make_inputs(5000 + case, B, T, dims.F, 0 if case % 3 == 0 else max(1, T // 3), T, pad="nan")
        form = str(rng.choice(["f32", "f32", "bf16", "e4m3", "e2m1"]))
        bf16 = form != "f32"
        flags = pkg.RNNT_FLAG_BF16_ARITHMETIC if bf16 else 0
        if form == "e4m3":      # weights quantised by the oracle's quantisers, stored as codes with scales
            model = synth.with_streamed_weights(model, lambda a: oracle.quantize_rows_e4m3(a)[0])
            flags |= pkg.RNNT_FLAG_FP8_WEIGHTS
        elif form == "e2m1":
            model = synth.with_streamed_weights(model, lambda a: oracle.quantize_blocks_e2m1(a)[0])
            flags |= pkg.RNNT_FLAG_FP4_WEIGHTS
        variants = ("tdt",) if tdt else (("label",) if spans else ("frame", "label"))
        w = synth.Workload(f"random{case}", variants[0], model, x, ln, S)
        n_teams = int(rng.choice([0, 0, 4, 8, 16, 32]))
        groups = int(rng.choice([1, 2, 4])) if n_teams else 0
        la = int(rng.choice([0, 0, 1, 3, 8]))
        try:
            eng = pkg.Engine(model, B, T, flags=flags)
        except pkg.RnntError as err:        # the model's state for this many utterances does not fit a compute unit
            assert err.code == -5 and big, (err, dims, B)
            log(f"random {case}: refused (-5) {dims} B={B}")
            continue
        try:
            eng.configure(n_teams=n_teams, joint_groups=groups, lookahead=la)
        except pkg.RnntError as err:
            assert err.code in (-2, -5), err
            eng.close()
            continue
        for variant in variants:
            check(pkg, w, variant, f"random {case}: {dims} B={B} T={T} S={S} teams={n_teams}/{groups} la={la} {form}",
                  engine=eng, bf16=bf16, logp=(variant != "frame"))
        ran += 1
        eng.close()
    log(f"random cases run: {ran}")
    assert ran >= 90
