"""Pins of the oracle's weight-only 8-bit quantiser (orc_quantize_rows_e4m3) and of the library's
host-side one: the e4m3 value set is written out here from the format's definition (1 sign bit,
4 exponent bits with bias 7, 3 mantissa bits, subnormals m * 2^-9, the all-ones code is NaN,
largest value 448), and every result is checked by brute force against that set."""
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
    assert np.array_equal(q2, q) and np.array_equal(sc2, sc)
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
