"""The entry point that allocates nothing (rnnt_label_looping_decode_noalloc, for callers that
cannot call hipMalloc) against rnnt_label_looping_decode on the same inputs: tokens, frame
indices and counts bit-exact, logits bit-identical (same kernels, same operands), on two calls
in a row, the second with a smaller input, so that what the first call left in the shared
static scratch array must not matter.  A call too large for the array is refused."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _decode(eng, w, variant):
    x = w.enc_out.copy()
    for b in range(w.B):
        x[b, int(w.enc_len[b]):, :] = np.nan
    enc = torch.from_numpy(x).cuda().contiguous()
    ln = torch.from_numpy(w.enc_len.astype(np.int32)).cuda()
    out = eng.decode(variant, enc, ln, w.max_symbols)
    torch.cuda.synchronize()
    assert eng.status() == 0
    return {k: v.cpu().numpy() for k, v in out.items()}, eng.stats()


def test_noalloc_entry_point_matches_the_allocating_one():
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    import paper_2406_03791_amd as pkg
    pkg.load_library()
    big = synth.make_workload(3, pad="nan", B=12, T=120, len_lo=40, len_hi=120)
    small = synth.make_workload(3, pad="nan", B=5, T=60, len_lo=20, len_hi=60)
    eng = pkg.Engine(big.model, big.B, big.T)
    try:
        for w in (big, small):
            want, st_w = _decode(eng, w, "label")
            got, st_g = _decode(eng, w, "label_noalloc")
            print(f"[noalloc] B={w.B} T={w.T} tokens={int(want['tok_len'].sum())} "
                  f"steps {st_g['pred_steps']}/{st_g['joint_steps']}", flush=True)
            assert int(want["tok_len"].sum()) > 0
            assert np.array_equal(got["tok_len"], want["tok_len"])
            assert np.array_equal(got["tokens"], want["tokens"])       # fill included
            assert np.array_equal(got["frames"], want["frames"])
            assert np.array_equal(got["logits"], want["logits"])
            assert (st_g["pred_steps"], st_g["joint_steps"]) == (st_w["pred_steps"], st_w["joint_steps"])
        # and once more the larger input after the smaller one
        want, _ = _decode(eng, big, "label")
        got, _ = _decode(eng, big, "label_noalloc")
        assert np.array_equal(got["tokens"], want["tokens"])
        assert np.array_equal(got["logits"], want["logits"])
    finally:
        eng.close()
    # a call whose projected frames alone exceed the static array is refused, nothing is queued
    full = synth.make_workload(3, B=32)
    eng = pkg.Engine(full.model, full.B, full.T)
    try:
        enc = torch.from_numpy(full.enc_out).cuda().contiguous()
        ln = torch.from_numpy(full.enc_len).cuda()
        with pytest.raises(pkg.RnntError) as err:
            eng.decode("label_noalloc", enc, ln, full.max_symbols)
        assert err.value.code == -6
        assert "scratch" in str(err.value)
    finally:
        eng.close()
