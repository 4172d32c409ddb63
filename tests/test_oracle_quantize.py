"""Pins for the oracle's quantizer: per-row symmetric absmax int8, round-half-to-even (the rounding primitive
of the paper's Listing 1; the per-row symmetric granularity is the benchmark configuration's)."""
import numpy as np
import pytest

from oracle import oracle as O


def test_closed_form_row_with_ties():
    # s = 127/127 = 1 exactly, so the two .5 values are true ties: both go to the even neighbour
    W = np.array([[-127.0, 0.0, 62.5, 63.5, 127.0]], np.float32)
    Q, s = O.quantize_rows(W)
    assert s.tolist() == [1.0]
    assert Q.tolist() == [[-127, 0, 62, 64, 127]]


def test_more_ties_and_signs():
    W = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, -126.5]], np.float32)
    Q, s = O.quantize_rows(W)
    assert Q.tolist() == [[127, 0, 2, 2, 0, -2, -2, 126, -126]]


def test_zero_row_and_mixed_rows():
    W = np.array([[0, 0, 0, 0], [0.5, -1.0, 0.25, 0.0]], np.float32)
    Q, s = O.quantize_rows(W)
    assert s[0] == 0 and Q[0].tolist() == [0, 0, 0, 0]
    assert s[1] == np.float32(1.0) / np.float32(127.0)
    assert Q[1, 1] == -127 and Q[1, 3] == 0


def test_power_of_two_scaling_invariance_and_bounds():
    rng = np.random.default_rng(0)
    W = (rng.standard_normal((64, 300)) * 0.02).astype(np.float32)
    Q, s = O.quantize_rows(W)
    for c in (0.25, 2.0, 1024.0):
        Q2, s2 = O.quantize_rows((W * np.float32(c)).astype(np.float32))
        assert np.array_equal(Q, Q2) and np.array_equal(s2, s * np.float32(c))
    assert Q.min() >= -127 and Q.max() <= 127
    # the absmax element of every row maps to +-127
    j = np.argmax(np.abs(W), axis=1)
    assert np.all(np.abs(Q[np.arange(64), j]) == 127)
    # reconstruction error at most half a step (plus fp32 rounding of the division)
    err = np.abs(W.astype(np.float64) - s[:, None].astype(np.float64) * Q)
    assert np.all(err <= 0.5 * s[:, None].astype(np.float64) * (1 + 1e-5))
    # odd symmetry
    Qn, sn = O.quantize_rows(-W)
    assert np.array_equal(Qn, -Q) and np.array_equal(sn, s)


def test_rows_are_independent():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((8, 50)).astype(np.float32)
    Q, s = O.quantize_rows(W)
    for r in range(8):
        q1, s1 = O.quantize_rows(W[r:r + 1])
        assert np.array_equal(q1[0], Q[r]) and s1[0] == s[r]


# ----- lower widths (paper section 3: the levels are set by the number of bits)

def test_four_bit_closed_form_with_ties():
    # amax = 7 -> s = 1 exactly; 2.5 -> 2 and 3.5 -> 4 (both ties to even), -6.5 -> -6
    W = np.array([[-7.0, 0.0, 2.5, 3.5, 7.0, -6.5, 0.49, 6.51]], np.float32)
    Q, s = O.quantize_rows(W, bits=4)
    assert s.tolist() == [1.0]
    assert Q.tolist() == [[-7, 0, 2, 4, 7, -6, 0, 7]]


def test_six_bit_closed_form():
    W = np.array([[31.0, -31.0, 15.5, 16.5, -0.5, 30.4999]], np.float32)
    Q, s = O.quantize_rows(W, bits=6)
    assert s.tolist() == [1.0]
    assert Q.tolist() == [[31, -31, 16, 16, 0, 30]]


def test_two_bits_is_ternary_with_threshold_at_half_the_maximum():
    # qmax = 1: s = amax, Q = rne(w / amax) -> 0 for |w| <= amax / 2 (the tie goes to the even 0), +-1 above
    W = np.array([[-4.0, 2.0, 1.9, -2.0, 4.0, 2.1, -2.5, 0.0]], np.float32)
    Q, s = O.quantize_rows(W, bits=2)
    assert s.tolist() == [4.0]
    assert Q.tolist() == [[-1, 0, 0, 0, 1, 1, -1, 0]]


def test_level_count_error_bound_and_eight_bits_is_the_default():
    rng = np.random.default_rng(4)
    W = (rng.standard_normal((24, 300)) * 0.02).astype(np.float32)
    for bits in range(2, 9):
        qmax = (1 << (bits - 1)) - 1
        Q, s = O.quantize_rows(W, bits=bits)
        assert Q.min() >= -qmax and Q.max() <= qmax
        assert np.all(np.max(np.abs(Q), axis=1) == qmax)          # the row maximum maps to the outermost level
        assert np.allclose(s * qmax, np.max(np.abs(W), axis=1), rtol=1e-6)
        err = np.abs(W.astype(np.float64) - s[:, None].astype(np.float64) * Q)
        assert np.all(err <= 0.5 * s[:, None] * (1 + 1e-5))       # nearest level: at most half a step away
    Q8, s8 = O.quantize_rows(W, bits=8)
    Qd, sd = O.quantize_rows(W)
    assert np.array_equal(Q8, Qd) and np.array_equal(s8, sd)
    with pytest.raises(ValueError):
        O.quantize_rows(W, bits=1)
    with pytest.raises(ValueError):
        O.quantize_rows(W, bits=9)
