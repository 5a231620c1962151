"""Pins of the oracle's rotary position embedding (the step a serving stack applies to the query
and the new Key ahead of the cache; not part of the paper's method).

Pinned against things other than the formula it is written from: complex multiplication, exact
quarter turns, the identity at angle zero, which channel is paired with which, and the property the
embedding exists for (a score depends on the distance of the two positions only)."""
import numpy as np
import pytest

from oracle import kvq_oracle as O


def _table(pos, hd=128, base=10000.0):
    """cos / sin (fp32) of position `pos` for the usual frequencies base^(-2i/hd)."""
    i = np.arange(hd // 2, dtype=np.float64)
    ang = pos * base ** (-2.0 * i / hd)
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def test_equals_complex_multiplication():
    """(x_i + j x_{i+hd/2}) e^{j angle}, in complex128 from the same fp32 table, to within the roundings
    the function is allowed (three fp32 ones and the final fp16 one)."""
    rng = np.random.default_rng(0)
    x = (rng.standard_normal((37, 128)) * 3).astype(np.float16)
    c, s = _table(1234)
    y = O.rope_rotate(x, c, s)
    z = (x[:, :64].astype(np.float64) + 1j * x[:, 64:].astype(np.float64)) * (c.astype(np.float64) + 1j * s.astype(np.float64))
    want = np.concatenate([z.real, z.imag], axis=-1)
    assert y.dtype == np.float16 and y.shape == x.shape
    tol = np.abs(want) * 2.0 ** -11 + 6 * 2.0 ** -24 * 3 * np.abs(x.astype(np.float64)).max()
    assert np.all(np.abs(y.astype(np.float64) - want) <= tol)
    # and not all of it equal to the unrotated input
    assert np.abs(y.astype(np.float64) - x.astype(np.float64)).max() > 1.0


def test_angle_zero_is_the_identity_bit_for_bit():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((5, 128)) * 50).astype(np.float16)
    c, s = _table(0)
    assert np.array_equal(O.rope_rotate(x, c, s).view(np.uint16), x.view(np.uint16))


def test_quarter_turn_pairs_channel_i_with_i_plus_half_and_turns_counter_clockwise():
    """cos = 0, sin = 1 at frequency 3 only: the first coordinate of pair 3 (channel 3) moves to its
    second (channel 67), the second moves to minus the first; every other pair stays."""
    x = np.zeros((1, 128), np.float16)
    x[0, 3] = 2.0
    x[0, 67] = 5.0
    x[0, 4] = 7.0
    x[0, 100] = -1.5
    c = np.ones(64, np.float32)
    s = np.zeros(64, np.float32)
    c[3], s[3] = 0.0, 1.0
    y = O.rope_rotate(x, c, s)
    want = np.zeros((1, 128), np.float16)
    want[0, 3] = -5.0
    want[0, 67] = 2.0
    want[0, 4] = 7.0
    want[0, 100] = -1.5
    assert np.array_equal(y, want)


def test_pair_norms_are_kept():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((64, 128)).astype(np.float16)
    c, s = _table(77)
    y = O.rope_rotate(x, c, s).astype(np.float64)
    n0 = np.hypot(x[:, :64].astype(np.float64), x[:, 64:].astype(np.float64))
    n1 = np.hypot(y[:, :64], y[:, 64:])
    assert np.all(np.abs(n1 - n0) <= 2.0 ** -10 * n0 + 1e-6)


@pytest.mark.parametrize("shift", [1, 17, 1000])
def test_scores_depend_on_the_distance_of_the_positions_only(shift):
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 128)).astype(np.float16)
    k = rng.standard_normal((1, 128)).astype(np.float16)
    def score(pq, pk):
        a = O.rope_rotate(q, *_table(pq)).astype(np.float64)
        b = O.rope_rotate(k, *_table(pk)).astype(np.float64)
        return float((a * b).sum())
    base = score(40, 25)
    moved = score(40 + shift, 25 + shift)
    other = score(40 + shift, 25)
    assert abs(moved - base) < 0.06            # fp16 rounding of 128 products of O(1) terms
    assert abs(other - base) > 0.5             # while the distance itself does matter


def test_each_operation_is_rounded_on_its_own():
    """A case where a fused multiply-add would give another fp16.  x_0 c_0 = 1025 (1 + 2^-23) needs 34 bits
    and rounds, in fp32, to 1025 + 2^-13, which is what x_64 s_0 is: separately rounded products cancel
    to 0, while a fused multiply-add would leave the 2^-23 the rounding dropped (twice the smallest fp16).
    (The table need not hold cosines and sines for this.)"""
    x = np.zeros((1, 128), np.float16)
    x[0, 0] = np.float16(1025.0)
    x[0, 64] = np.float16(1.0)
    c = np.ones(64, np.float32)
    s = np.zeros(64, np.float32)
    c[0] = np.float32(1.0 + 2.0 ** -23)
    s[0] = np.float32(1025.0 + 2.0 ** -13)
    assert float(s[0]) == 1025.0 + 2.0 ** -13 and float(c[0]) == 1.0 + 2.0 ** -23
    y = O.rope_rotate(x, c, s)
    assert float(y[0, 0]) == 0.0
    exact = 1025.0 * (1.0 + 2.0 ** -23) - (1025.0 + 2.0 ** -13)      # what a fused multiply-add would round
    assert float(np.float16(exact)) == 2.0 ** -23 != 0.0
