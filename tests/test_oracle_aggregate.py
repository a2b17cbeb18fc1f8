"""Pins of the oracle's server-side aggregation (equal-weight federated average in fp32)."""
from fractions import Fraction

import numpy as np

from oracle import omc_oracle as orc


def test_one_client_is_the_identity_and_equal_clients_average_to_themselves():
    rng = np.random.default_rng(0)
    v = rng.standard_normal(1000).astype(np.float32)
    v[:4] = [0.0, -0.0, 1e-45, -3e38]
    assert np.array_equal(orc.aggregate_mean([v]).view(np.uint32), v.view(np.uint32))
    small = (v * np.float32(2.0 ** -8)).astype(np.float32)
    assert np.array_equal(orc.aggregate_mean([small, small]), small)      # x + x and the halving are exact
    ints = rng.integers(-1000, 1000, 1000).astype(np.float32)             # small integers: every sum is exact
    for R in (3, 4, 7, 16):
        assert np.array_equal(orc.aggregate_mean([ints] * R), ints)


def test_against_exact_rational_mean_within_the_rounding_bound():
    rng = np.random.default_rng(1)
    for R in (2, 3, 5, 7, 16):
        vs = [rng.standard_normal(200).astype(np.float32) * np.float32(10.0 ** rng.integers(-3, 3)) for _ in range(R)]
        got = orc.aggregate_mean(vs)
        for i in range(200):
            exact = sum(Fraction(float(v[i])) for v in vs) / R
            scale = sum(abs(Fraction(float(v[i]))) for v in vs) / R
            # R-1 additions and one division, each within half an ulp of a partial result <= sum |v|
            assert abs(Fraction(float(got[i])) - exact) <= scale * R * Fraction(1, 2 ** 23)


def test_order_is_client_index_order_left_to_right():
    # (1e8 + 1) - 1e8 in fp32 is 0 left to right, but 1 if the last two were added first
    a = np.array([1e8], np.float32)
    b = np.array([1.0], np.float32)
    c = np.array([-1e8], np.float32)
    assert orc.aggregate_mean([a, b, c])[0] == 0.0
    assert orc.aggregate_mean([a, c, b])[0] == np.float32(1.0) / np.float32(3.0)


def test_division_is_rounded_once_not_a_multiplication_by_the_reciprocal():
    x = np.arange(1, 2000, dtype=np.float32)
    got = orc.aggregate_mean([x, np.zeros_like(x), np.zeros_like(x)])
    want = np.array([np.float32(Fraction(int(k), 3)) for k in range(1, 2000)], np.float32)   # Fraction -> nearest float
    assert np.array_equal(got, want)
    recip = x * np.float32(1.0 / 3.0)
    assert np.any(recip != got)                   # the two differ somewhere: the test can tell them apart


def test_mixed_sources_match_decompress_then_average():
    """A variable that arrives as codes from some clients and in fp32 from others (Sec. 2.5)."""
    rng = np.random.default_rng(3)
    f = orc.Format(3, 7)
    V = [rng.standard_normal(500).astype(np.float32) * np.float32(0.05) for _ in range(4)]
    srcs = []
    for r, v in enumerate(V):
        if r % 2 == 0:
            p, sb = orc.compress(v, f)
            srcs.append(orc.decompress(p, v.size, f, sb))
        else:
            srcs.append(v)
    got = orc.aggregate_mean(srcs)
    ref = ((srcs[0] + srcs[1]).astype(np.float32) + srcs[2]).astype(np.float32)
    ref = ((ref + srcs[3]).astype(np.float32) / np.float32(4.0)).astype(np.float32)
    assert np.array_equal(got, ref)
    # and close to the fp32 clients' own mean: quantization noise averages down, never blows up
    assert np.max(np.abs(got - np.mean(V, axis=0))) < 1e-3
