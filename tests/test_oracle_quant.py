"""Pins for the oracle's group quantiser (Eq. 2, Sec. 3.3; formula = asymmetric min-max RTN)."""
import numpy as np
import pytest

from oracle import rosaq_oracle as O


def _weights(seed, N, C):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((N, C)) * 0.02
    w[rng.random((N, C)) < 0.01] *= 10
    return w.astype(np.float16)


@pytest.mark.parametrize("bits", [3, 4])
@pytest.mark.parametrize("N,C,g", [(8, 8, 8), (4, 128, 128), (3, 256, 128)])
def test_code_is_nearest_bruteforce(bits, N, C, g):
    w16 = _weights(bits * 10 + N, N, C)
    q, s, z = O.quantize_groups(w16, bits, g)
    w = w16.astype(np.float64)
    qmax = 2 ** bits - 1
    assert q.max() <= qmax and z.astype(np.float64).max() <= qmax and z.astype(np.float64).min() >= 0
    for n in range(N):
        for c in range(C):
            sj = float(s[n, c // g]); zj = float(z[n, c // g])
            err = np.abs(w[n, c] - (np.arange(qmax + 1) - zj) * sj)
            best = err.min()
            mine = abs(w[n, c] - (float(q[n, c]) - zj) * sj)
            assert mine <= best * (1 + 1e-12) + 1e-300      # equal up to exact ties
    # scale is the fp16 rounding of range / qmax and zero is the rounded offset
    wg = w.reshape(N, C // g, g)
    rng_ = wg.max(2) - wg.min(2)
    assert np.array_equal(s, np.maximum(rng_ / qmax, 2.0 ** -14).astype(np.float16))
    assert np.array_equal(z.astype(np.float64),
                          np.clip(np.rint(-wg.min(2) / s.astype(np.float64)), 0, qmax))


@pytest.mark.parametrize("bits", [3, 4])
def test_round_trip_of_representable_weights(bits):
    rng = np.random.default_rng(7)
    qmax = 2 ** bits - 1
    N, G, g = 6, 3, 128
    codes = rng.integers(0, qmax + 1, size=(N, G, g))
    codes[:, :, 0] = 0
    codes[:, :, 1] = qmax                      # full range present in every group
    z = rng.integers(0, qmax + 1, size=(N, G, 1))
    s = (2.0 ** rng.integers(-9, -4, size=(N, G, 1))) * rng.choice([1.0, 1.5, 1.25], size=(N, G, 1))
    w = ((codes - z) * s).reshape(N, G * g)
    w16 = w.astype(np.float16)
    assert np.array_equal(w16.astype(np.float64), w)         # exactly representable
    q, s16, z16 = O.quantize_groups(w16, bits, g)
    assert np.array_equal(q.reshape(N, G, g), codes)
    assert np.array_equal(s16.astype(np.float64), s[:, :, 0])
    assert np.array_equal(z16.astype(np.float64), z[:, :, 0].astype(np.float64))
    assert np.array_equal(O.dequantize_groups(q, s16, z16, g), w)


def test_degenerate_groups():
    # constant group: scale floors at 2^-14, codes clamp
    w = np.full((2, 128), 0.25, np.float16)
    q, s, z = O.quantize_groups(w, 4, 128)
    assert np.all(s.astype(np.float64) == 2.0 ** -14)
    assert np.all(z == 0) and np.all(q == 15)
    w = np.zeros((1, 128), np.float16)
    q, s, z = O.quantize_groups(w, 3, 128)
    assert np.all(q == 0) and np.all(z == 0)
    assert np.all(O.dequantize_groups(q, s, z, 128) == 0)
    # all-negative group: zero point clamps at qmax
    w = np.linspace(-2.0, -1.0, 128).astype(np.float16)[None, :]
    q, s, z = O.quantize_groups(w, 4, 128)
    assert float(z[0, 0]) == 15.0 and q.max() <= 15


def test_half_way_cases_round_to_even():
    # s = 1/16 exactly; w/s = 0.5, 1.5, 2.5 -> 0, 2, 2
    w = np.zeros((1, 128), np.float16)
    w[0, 0] = 15 / 16.0                       # max -> range 15/16, qmax 15 -> s = 1/16
    w[0, 1] = 0.5 / 16
    w[0, 2] = 1.5 / 16
    w[0, 3] = 2.5 / 16
    q, s, z = O.quantize_groups(w, 4, 128)
    assert float(s[0, 0]) == 1 / 16 and float(z[0, 0]) == 0
    assert q[0, :4].tolist() == [15, 0, 2, 2]


def test_quantisation_error_bound():
    w16 = _weights(11, 16, 512)
    for bits in (3, 4):
        q, s, z = O.quantize_groups(w16, bits, 128)
        err = np.abs(O.dequantize_groups(q, s, z, 128) - w16.astype(np.float64))
        # inside the clamp range the error is at most half a step (+ fp16 rounding of s)
        bound = 0.5 * np.repeat(s.astype(np.float64), 128, axis=1) * (1 + 2 ** -9) + \
            (2 ** bits) * np.repeat(s.astype(np.float64), 128, axis=1) * 2 ** -10
        assert np.all(err <= bound)


def test_hand_worked_examples():
    """tests/golden/quantizer_worked_examples.txt: groups of eight weights quantised by hand from the
    definition (Sec. 3.3, Eq. 2; asymmetric min-max round-to-nearest)."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "quantizer_worked_examples.txt")
    cases = 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        bits, w, s, z, q = [f.strip() for f in line.split("|")]
        w = np.array([float(v) for v in w.split()], np.float64)
        w16 = w.astype(np.float16)[None, :]
        assert np.array_equal(w16[0].astype(np.float64), w)
        codes, scales, zeros = O.quantize_groups(w16, int(bits), 8)
        assert float(scales[0, 0]) == float(s), line
        assert float(zeros[0, 0]) == float(z), line
        assert codes[0].tolist() == [int(v) for v in q.split()], line
        cases += 1
    assert cases == 6
