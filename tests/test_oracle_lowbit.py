"""Pins for the oracle's low-bit sketch states (Sec. 3.3, last paragraph; Sec. 4,
ablation with sketch states in low-bit types).

The paper names a third-party scalar quantiser and prints neither a format
nor values, so the format is this repository's reading: one binary16 scale per
sketch row of a group (its largest state magnitude), signed codes
q in [-qmax, qmax] with qmax = 127 / 7, state = q * scale / qmax rounded once
to binary16.  What can be pinned is the arithmetic: exact rational values,
end points, symmetry, the half-step error bound, hand-worked codes.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle

QMAX = {8: 127, 4: 7}


def h2f(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def f2h(vals):
    return np.asarray(vals, dtype=np.float16).view(np.uint16)


def deq_row(bits, codes, scale_bits):
    codes = np.asarray(codes, dtype=np.int8)
    return oracle.dequantize_states(1, 1, 1, 1, 1, [codes.size], bits, codes, [scale_bits])


def half_neighbours(bits):
    """the two binary16 values next to a finite pattern (as exact Fractions), None past the ends"""
    mag, sign = int(bits) & 0x7FFF, -1 if int(bits) >> 15 else 1
    out = []
    for m in (mag - 1, mag + 1):
        if 0 <= m < 0x7C00:
            out.append(sign * Fraction(float(h2f([m])[0])))
        elif m < 0:                      # below +-0: the smallest value of the other sign
            out.append(-sign * Fraction(float(h2f([1])[0])))
    return out


@pytest.mark.parametrize("bits", [8, 4])
def test_dequantised_state_is_the_correctly_rounded_quotient(bits):
    qmax = QMAX[bits]
    rng = np.random.default_rng(bits)
    scales = np.concatenate([rng.integers(0, 0x7C00, 400), [0, 1, 2, 3, 0x3FF, 0x400, 0x401, 0x3C00, 0x7BFF]])
    codes = np.arange(-qmax, qmax + 1)
    exact_hits = 0
    for s in scales:
        got = deq_row(bits, codes, int(s))
        sv = Fraction(float(h2f([s])[0]))
        for q, hb in zip(codes, got):
            exact = Fraction(int(q)) * sv / qmax
            hv = Fraction(float(h2f([hb])[0]))
            err = abs(hv - exact)
            for nb in half_neighbours(hb):
                e2 = abs(nb - exact)
                assert e2 >= err, (bits, int(s), int(q))
                # q * scale / qmax is never half-way between two binary16 values (qmax is odd: the
                # quotient is either exactly representable or no dyadic rational), so the rounding
                # mode's tie rule never comes into play
                assert not (e2 == err and e2 != 0), (bits, int(s), int(q))
            exact_hits += err == 0
            if q == 0:
                assert int(hb) == 0                    # code 0 is +0.0
            elif exact == 0:
                assert int(hb) == (0x8000 if q < 0 else 0)   # zero scale: a signed zero, as IEEE arithmetic gives
    assert exact_hits > len(scales)                    # end codes and code 0 at least


@pytest.mark.parametrize("bits", [8, 4])
def test_end_points_symmetry_and_order(bits):
    qmax = QMAX[bits]
    codes = np.arange(-qmax, qmax + 1)
    for s in [0x0001, 0x0400, 0x2E66, 0x3C00, 0x4700, 0x7BFF]:
        got = deq_row(bits, codes, s)
        assert got[-1] == s and got[0] == (s | 0x8000)           # +-qmax give +-scale exactly
        pos, neg = got[qmax + 1:], got[:qmax][::-1]
        assert np.array_equal(neg, pos | 0x8000)                  # odd symmetry, bit for bit
        v = h2f(got)
        assert np.all(np.diff(v) >= 0)                            # monotone in the code
    assert np.all((deq_row(bits, codes, 0) & 0x7FFF) == 0)        # an all-zero row


def test_hand_worked_codes_four_bit():
    # scale 7.0: one code step is exactly 1.0; 3.5, 2.5 and 0.5 are ties (to the even code)
    states = f2h([7.0, -7.0, 3.5, 2.5, -0.5, 0.49, 6.51, 0.0, -1.49, -1.51])
    sk = oracle.Sketch(1, 1, 1, 1, 1, np.array([1], np.uint32), np.array([0], np.uint32),
                       np.array([states.size], np.uint32), states)
    q = oracle.quantize(sk, 4)
    assert list(q.codes) == [7, -7, 4, 2, 0, 0, 7, 0, -1, -2]
    assert list(q.scales) == [int(f2h([7.0])[0])]
    assert list(h2f(q.states)) == [7.0, -7.0, 4.0, 2.0, 0.0, 0.0, 7.0, 0.0, -1.0, -2.0]
    assert q.states[4] == 0                                       # -0.5 -> code 0 -> +0.0


def test_hand_worked_codes_eight_bit():
    states = f2h([127.0, 63.5, 62.5, -1.5, -126.4, 0.25, -127.0])
    sk = oracle.Sketch(1, 1, 1, 1, 1, np.array([1], np.uint32), np.array([0], np.uint32),
                       np.array([states.size], np.uint32), states)
    q = oracle.quantize(sk, 8)
    assert list(q.codes) == [127, 64, 62, -2, -126, 0, -127]
    assert list(h2f(q.states)) == [127.0, 64.0, 62.0, -2.0, -126.0, 0.0, -127.0]


def test_hand_worked_non_integer_step():
    # scale 1.0, four bit: the states are q / 7 rounded to binary16.  Worked by hand from the binary
    # expansion 1/7 = 0.001001001...b: 1/7 -> 0x3092 (rounds down), 5/7 -> 0x39B7 (rounds up), ...
    got = deq_row(4, [1, 2, 3, -4, 5, 6], int(f2h([1.0])[0]))
    assert [int(v) for v in got] == [0x3092, 0x3492, 0x36DB, 0xB892, 0x39B7, 0x3ADB]
    want = [Fraction(1, 7), Fraction(2, 7), Fraction(3, 7), Fraction(-4, 7), Fraction(5, 7), Fraction(6, 7)]
    for hb, w in zip(got, want):
        assert abs(Fraction(float(h2f([hb])[0])) - w) <= Fraction(1, 2 ** 12) * abs(w)


def small_sketch(seed=3):
    rng = np.random.default_rng(seed)
    in_f, out_f, d = 24, 64, 3
    W = (rng.standard_normal((in_f, out_f)) * 0.02).astype(np.float16)
    W[5] *= 20
    width = rng.integers(3, 12, in_f).astype(np.uint32)
    A = rng.integers(1, 1 << 24, d) | 1
    C = rng.integers(0, 1 << 24, d)
    return oracle.update(W, 1, out_f, d, A, C, width)


@pytest.mark.parametrize("bits", [8, 4])
def test_scale_is_the_row_maximum_and_error_is_at_most_half_a_step(bits):
    qmax = QMAX[bits]
    sk = small_sketch()
    q = oracle.quantize(sk, bits)
    base = 0
    for g, K in enumerate(sk.group_width):
        for r in range(sk.d):
            row = sk.states[base + r * K: base + (r + 1) * K]
            top = int(np.max(row & 0x7FFF))
            assert q.scales[g * sk.d + r] == top
            sc = float(h2f([top])[0])
            err = np.abs(h2f(q.states[base + r * K: base + (r + 1) * K]) - h2f(row))
            ulp = float(np.spacing(np.float16(sc)))      # the one rounding to binary16, at most half a spacing at the row's top
            assert np.all(err <= sc / (2 * qmax) + ulp / 2 + 1e-12)
            codes = q.codes[base + r * K: base + (r + 1) * K].astype(int)
            assert np.all(np.abs(codes) <= qmax)
            assert np.all(np.sign(codes) * np.sign(h2f(row)) >= 0)       # no code flips a sign
            assert np.max(np.abs(codes)) == (qmax if top else 0)          # the largest state takes the end code
        base += sk.d * K
    assert base == sk.states.size


@pytest.mark.parametrize("bits", [8, 4])
def test_quantising_again_changes_nothing(bits):
    q1 = oracle.quantize(small_sketch(), bits)
    q2 = oracle.quantize(q1, bits)
    assert np.array_equal(q1.codes, q2.codes) and np.array_equal(q1.scales, q2.scales)
    assert np.array_equal(q1.states, q2.states)


@pytest.mark.parametrize("bits", [8, 4])
def test_query_returns_states_the_codes_stand_for(bits):
    sk = small_sketch(11)
    q = oracle.quantize(sk, bits)
    W_hat = oracle.query(q)
    base = 0
    for j, K in enumerate(q.group_width):
        rows = set(int(v) for v in q.states[base: base + q.d * K])
        assert set(int(v) for v in W_hat[j]) <= rows
        base += q.d * K
    # and it is the query of the same geometry over those states, nothing else
    plain = oracle.Sketch(q.in_features, q.out_features, q.tile_in, q.tile_out, q.d, q.hash_a, q.hash_c,
                          q.group_width, q.states)
    assert np.array_equal(W_hat, oracle.query(plain))


def test_bits_per_weight_counts_codes_and_scales():
    sk = small_sketch()
    q = oracle.quantize(sk, 4)
    n_w = sk.in_features * sk.out_features
    assert q.bits_per_weight == pytest.approx((4 * sk.states.size + 16 * sk.in_features * sk.d) / n_w)
    assert sk.bits_per_weight == pytest.approx(16 * sk.states.size / n_w)


def test_bad_codes_and_scales_are_refused():
    with pytest.raises(ValueError):
        deq_row(4, [8], 0x3C00)
    with pytest.raises(ValueError):
        deq_row(4, [-8], 0x3C00)
    with pytest.raises(ValueError):
        deq_row(8, [1], 0x7C00)          # infinite scale
    with pytest.raises(ValueError):
        deq_row(8, [1], 0xBC00)          # negative scale
    with pytest.raises(ValueError):
        deq_row(5, [1], 0x3C00)
