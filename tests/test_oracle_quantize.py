"""Pins of the oracle's weight-only quantisers (orc_quantize_rows_e4m3, orc_quantize_blocks_e2m1)
and of the library's host-side ones: the value sets are written out here from the formats'
definitions (e4m3: 1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits, subnormals
m * 2^-9, the all-ones code is NaN, largest value 448; e2m1: 1 sign bit, 2 exponent bits with
bias 1, 1 mantissa bit, subnormal 0.5, largest value 6), and every result is checked by brute
force against that set."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth


def e4m3_values():
    vals = []
    for code in range(127):
        expo, mant = code >> 3, code & 7
        vals.append(Fraction(mant, 512) if expo == 0 else Fraction(8 + mant, 8) * Fraction(2) ** (expo - 7))
    return vals            # ascending, vals[code]


VALS = e4m3_values()


def brute_force_row(row):
    """Row scale exponent and quantised row by exact rational arithmetic."""
    M = max(abs(Fraction(float(x))) for x in row)
    k = 0
    if M > 0:
        while M / Fraction(2) ** k > 448:
            k += 1
        while M / Fraction(2) ** (k - 1) <= 448 and k > -100:
            k -= 1
    out = []
    for x in row:
        v = abs(Fraction(float(x))) / Fraction(2) ** k
        dist = [abs(v - e) for e in VALS]
        d = min(dist)
        codes = [c for c in range(127) if dist[c] == d]
        code = codes[0] if len(codes) == 1 else [c for c in codes if c % 2 == 0][0]
        q = VALS[code] * Fraction(2) ** k
        out.append(float(-q if x < 0 else q))
    return k, np.array(out, dtype=np.float32)


def test_the_value_set_has_the_formats_landmarks():
    assert len(VALS) == 127 and VALS[0] == 0 and VALS[1] == Fraction(1, 512)
    assert VALS[8] == Fraction(1, 64) and VALS[0x38] == 1 and VALS[126] == 448
    assert all(a < b for a, b in zip(VALS, VALS[1:]))


@pytest.mark.parametrize("real", ["float", "double"])
def test_quantiser_matches_brute_force(real):
    rng = np.random.default_rng(11)
    rows = [rng.uniform(-0.1, 0.1, 40), rng.normal(0, 3.0, 40), rng.uniform(-1e-4, 1e-4, 40),
            rng.uniform(-5e4, 5e4, 40), np.zeros(40), np.full(40, 0.3),
            np.concatenate([[448.0 * 2.0 ** -7], rng.uniform(-1e-6, 1e-6, 39)]),      # deep subnormals
            np.concatenate([[449.0], rng.uniform(-449, 449, 39)])]                    # just above the top
    w = np.stack(rows).astype(np.float32)
    got, scales = oracle.quantize_rows_e4m3(w, real=real)
    for r in range(w.shape[0]):
        k, want = brute_force_row(w[r])
        assert float(scales[r]) == 2.0 ** k, r
        assert np.array_equal(got[r].astype(np.float32), want), r


def test_ties_go_to_the_even_code_and_the_scale_is_minimal():
    # row maximum 448 fixes k = 0; the other entries sit exactly between two neighbours
    mids = [float((VALS[c] + VALS[c + 1]) / 2) for c in range(0, 126)]
    w = np.array([[448.0] + mids + [-m for m in mids]], dtype=np.float32)
    got, scales = oracle.quantize_rows_e4m3(w)
    assert scales[0] == 1.0
    for i, c in enumerate(range(0, 126)):
        even = c if c % 2 == 0 else c + 1
        assert got[0, 1 + i] == np.float32(float(VALS[even])), c
        assert got[0, 1 + len(mids) + i] == -np.float32(float(VALS[even])), c
    # the scale: a maximum of 448 * 2^k gives k, anything above it up to twice that k + 1
    for m, k in [(448.0, 0), (448.0001, 1), (896.0, 1), (224.0, -1), (224.1, 0), (448.0 * 2 ** -20, -20)]:
        _, sc = oracle.quantize_rows_e4m3(np.array([[m, -m / 3]], dtype=np.float32))
        assert sc[0] == 2.0 ** k, (m, k)


def test_error_bound_idempotence_and_bf16_values():
    w = synth.make_workload(1).model.w_out
    q, sc = oracle.quantize_rows_e4m3(w)
    # normal range of the scaled grid: relative error at most 2^-4; below it: absolute 2^-10 * scale
    lim = np.maximum(np.abs(w) * 2.0 ** -4, (sc * 2.0 ** -10)[:, None])
    assert (np.abs(q - w) <= lim).all()
    assert np.abs(q).max(axis=1).min() > 0
    q2, sc2 = oracle.quantize_rows_e4m3(q)
    # the values are fixed points; a row whose maximum was rounded down may get a finer scale
    assert np.array_equal(q2, q) and (sc2 <= sc).all()
    assert np.array_equal(synth.round_to_bf16(q), q)          # every result is a bf16 value
    # sign symmetry and rows are independent
    qn, _ = oracle.quantize_rows_e4m3(-w)
    assert np.array_equal(qn, -q)
    q3, _ = oracle.quantize_rows_e4m3(w[5:9])
    assert np.array_equal(q3, q[5:9])


def test_library_quantiser_is_the_same_function():
    """The library's host-side quantiser (no device work) against the oracle's on random
    matrices with rows of very different magnitudes, and against brute force on a few rows."""
    import paper_2406_03791_amd as m
    rng = np.random.default_rng(3)
    w = (rng.normal(0, 1, (300, 96)) * np.ldexp(1.0, rng.integers(-40, 40, 300))[:, None]).astype(np.float32)
    w[7] = 0
    w[8, 1:] = 0
    a, sa = oracle.quantize_rows_e4m3(w)
    b, sb = m.rnnt_quantize_rows_e4m3(w)
    assert np.array_equal(a, b) and np.array_equal(sa, sb)
    for r in (0, 7, 8, 100):
        k, want = brute_force_row(w[r])
        assert sb[r] == 2.0 ** k and np.array_equal(b[r], want)
    with pytest.raises(m.RnntError):
        m.rnnt_quantize_rows_e4m3(np.array([[1.0, np.inf]], dtype=np.float32))


def e2m1_values():
    vals = []
    for code in range(8):
        expo, mant = code >> 1, code & 1
        vals.append(Fraction(mant, 2) if expo == 0 else Fraction(2 + mant, 2) * Fraction(2) ** (expo - 1))
    return vals


VALS4 = e2m1_values()


def brute_force_block(blk):
    M = max(abs(Fraction(float(x))) for x in blk)
    k = 0
    if M > 0:
        while M / Fraction(2) ** k > 6:
            k += 1
        while M / Fraction(2) ** (k - 1) <= 6 and k > -100:
            k -= 1
    out = []
    for x in blk:
        v = abs(Fraction(float(x))) / Fraction(2) ** k
        dist = [abs(v - e) for e in VALS4]
        d = min(dist)
        codes = [c for c in range(8) if dist[c] == d]
        code = codes[0] if len(codes) == 1 else [c for c in codes if c % 2 == 0][0]
        q = VALS4[code] * Fraction(2) ** k
        out.append(float(-q if x < 0 else q))
    return k, np.array(out, dtype=np.float32)


def test_e2m1_value_set():
    assert [float(v) for v in VALS4] == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


@pytest.mark.parametrize("real", ["float", "double"])
def test_block_quantiser_matches_brute_force(real):
    rng = np.random.default_rng(17)
    w = np.stack([rng.uniform(-0.1, 0.1, 300), rng.normal(0, 3.0, 300), rng.uniform(-1e-4, 1e-4, 300),
                  np.concatenate([np.zeros(128), rng.uniform(-5e4, 5e4, 172)]),
                  np.concatenate([[6.0 * 2.0 ** -9], rng.uniform(-1e-5, 1e-5, 299)]),
                  np.concatenate([[6.01], rng.uniform(-6, 6, 299)])]).astype(np.float32)
    for block in (128, 32):
        got, scales = oracle.quantize_blocks_e2m1(w, block=block, real=real)
        nb = (300 + block - 1) // block
        assert scales.shape == (w.shape[0], nb)
        for r in range(w.shape[0]):
            for b in range(nb):
                k, want = brute_force_block(w[r, b * block:(b + 1) * block])
                assert float(scales[r, b]) == 2.0 ** k, (r, b)
                assert np.array_equal(got[r, b * block:(b + 1) * block].astype(np.float32), want), (r, b)


def test_block_quantiser_ties_scales_and_idempotence():
    mids = [float((VALS4[c] + VALS4[c + 1]) / 2) for c in range(7)]          # 0.25 0.75 1.25 1.75 2.5 3.5 5
    w = np.array([[6.0] + mids + [-m for m in mids]], dtype=np.float32)
    got, scales = oracle.quantize_blocks_e2m1(w)
    assert scales[0, 0] == 1.0
    want = [0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0]                              # the even code of each pair
    assert list(got[0, 1:8]) == want and list(got[0, 8:]) == [-x for x in want]
    for m, k in [(6.0, 0), (6.0001, 1), (12.0, 1), (3.0, -1), (3.01, 0), (6.0 * 2 ** -20, -20)]:
        _, sc = oracle.quantize_blocks_e2m1(np.array([[m, -m / 3]], dtype=np.float32))
        assert sc[0, 0] == 2.0 ** k, (m, k)
    w = synth.make_workload(1).model.w_out
    q, sc = oracle.quantize_blocks_e2m1(w)
    q2, sc2 = oracle.quantize_blocks_e2m1(q)
    # the values are fixed points; a block whose maximum was rounded down gets a finer scale
    assert np.array_equal(q2, q) and (sc2 <= sc).all() and (sc2 < sc).any()
    assert np.array_equal(synth.round_to_bf16(q), q)
    # error: at most half the grid's largest relative gap (0.25 of the value) or a quarter of a scale unit
    lim = np.maximum(np.abs(w) * 0.25, np.repeat(sc, 128, axis=1)[:, :w.shape[1]] * 0.25)
    assert (np.abs(q - w) <= lim).all()
    # blocks are independent: a block quantised on its own gives the same values
    q3, _ = oracle.quantize_blocks_e2m1(w[:, 128:256])
    assert np.array_equal(q3, q[:, 128:256])


def test_library_block_quantiser_is_the_same_function():
    import paper_2406_03791_amd as m
    rng = np.random.default_rng(4)
    w = (rng.normal(0, 1, (200, 300)) * np.ldexp(1.0, rng.integers(-40, 40, 200))[:, None]).astype(np.float32)
    w[7] = 0
    w[8, 1:] = 0
    a, sa = oracle.quantize_blocks_e2m1(w)
    b, sb = m.rnnt_quantize_blocks_e2m1(w)
    assert np.array_equal(a, b) and np.array_equal(sa, sb)
    k, want = brute_force_block(w[3, 256:300])
    assert sb[3, 2] == 2.0 ** k and np.array_equal(b[3, 256:300], want)
    assert m.RNNT_FP4_BLOCK == 128
