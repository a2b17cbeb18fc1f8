"""Pins for the CPU oracle's codec (Sec. 2.2 formats) and bit packing.

The oracle is checked against things it does not define itself: library float
formats (numpy float16, torch bfloat16 / float8), brute force over exact
rationals on small formats, and order / symmetry / error-bound invariants.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import omc_oracle as orc
from oracle.omc_oracle import Format
from paper_2205_03494_amd import synth

PAPER_FORMATS = {                      # formats named in Sec. 3 of the paper
    "S1E4M14": Format(4, 14), "S1E3M7": Format(3, 7), "S1E2M3": Format(2, 3),
    "S1E5M10": Format(5, 10), "S1E3M9": Format(3, 9), "S1E4M8": Format(4, 8),
    "S1E5M7": Format(5, 7),
}
EXTRA_FORMATS = {
    "S1E4M3": Format(4, 3), "S1E5M2": Format(5, 2), "S1E8M7": Format(8, 7), "S1E1M2": Format(1, 2),
    "S1E2M1": Format(2, 1), "S1E3M0": Format(3, 0), "S1E4M3b4": Format(4, 3, bias=4),
    "S1E6M9": Format(6, 9), "S1E1M0": Format(1, 0),
}
ALL_FORMATS = {**PAPER_FORMATS, **EXTRA_FORMATS}


def valid_codes(fmt: Format) -> np.ndarray:
    """All codes whose value is a finite fp32 (everything unless E = 8)."""
    codes = np.arange(1 << fmt.bits, dtype=np.uint32)
    e = (codes >> fmt.man_bits) & ((1 << fmt.exp_bits) - 1)
    return codes[e.astype(np.int64) - fmt.resolved_bias <= 127]


def exact_value(code: int, fmt: Format) -> Fraction:
    """Sec. 2.2 value of a code as an exact rational, written independently of the oracle."""
    M, E, bias = fmt.man_bits, fmt.exp_bits, fmt.resolved_bias
    m = code & ((1 << M) - 1)
    e = (code >> M) & ((1 << E) - 1)
    sgn = -1 if (code >> (E + M)) & 1 else 1
    if e == 0:
        return sgn * Fraction(m, 1 << M) * Fraction(2) ** (1 - bias)
    return sgn * (1 + Fraction(m, 1 << M)) * Fraction(2) ** (e - bias)


# ------------------------------------------------------------------ P1: exhaustive round trip
@pytest.mark.parametrize("name", sorted(ALL_FORMATS))
def test_exhaustive_round_trip(name):
    fmt = ALL_FORMATS[name]
    codes = valid_codes(fmt)
    vals = orc.decode(codes, fmt)
    assert np.all(np.isfinite(vals))
    back = orc.encode(vals, fmt)
    assert np.array_equal(back, codes)           # includes +0 / -0 as distinct codes


def test_round_trip_fp32_identity_sampled():
    # FP32 is S1E8M23 (Sec. 3.1): compress / decompress is a bit copy on finite values
    fmt = Format(8, 23)
    rng = np.random.default_rng(3)
    bits = rng.integers(0, 1 << 32, size=200000, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    x = x[np.isfinite(x)]
    codes = orc.encode(x, fmt)
    assert np.array_equal(codes, x.view(np.uint32))
    assert np.array_equal(orc.decode(codes, fmt).view(np.uint32), x.view(np.uint32))


def test_decode_matches_exact_definition():
    for name in ("S1E2M3", "S1E4M3", "S1E3M7", "S1E1M2", "S1E3M0", "S1E4M3b4"):
        fmt = ALL_FORMATS[name]
        for c in valid_codes(fmt):
            v = exact_value(int(c), fmt)
            assert Fraction(orc.decode_value(int(c), fmt)) == v
            assert Fraction(float(orc.decode([c], fmt)[0])) == v


def test_format_constants_from_definition():
    # largest magnitude = 2^(2^E-1-bias) (2 - 2^-M); smallest step = 2^(1-bias-M)
    assert Format(4, 3).max == 480.0
    assert Format(3, 7).max == 31.875
    assert Format(5, 10).max == 131008.0
    assert Format(2, 3).max == 7.5
    assert Format(8, 7).max == float(torch.finfo(torch.bfloat16).max)
    assert orc.decode([1], Format(4, 3))[0] == 2.0 ** -9
    assert orc.decode([1], Format(3, 7))[0] == 2.0 ** -9
    assert orc.decode([1], Format(2, 3))[0] == 0.125
    assert orc.decode([1 << 3], Format(4, 3))[0] == 2.0 ** -6     # smallest normal


# ------------------------------------------------------------------ P2: brute-force nearest value
def brute_force_encode(x: float, fmt: Format, table) -> int:
    """Nearest representable value over exact rationals; ties go to the even mantissa field
    (for M = 0: to the candidate that is zero or the larger power of two, i.e. even integer
    significand); -x gives the mirrored code.  Non-negative candidates only."""
    neg = math.copysign(1.0, x) < 0
    a = abs(Fraction(x))
    best, best_d = None, None
    for code, v in table:
        d = abs(v - a)
        if best is None or d < best_d:
            best, best_d = [code], d
        elif d == best_d:
            best.append(code)
    if len(best) == 1:
        c = best[0]
    else:
        assert len(best) == 2
        if fmt.man_bits >= 1:
            c = best[0] if best[0] % 2 == 0 else best[1]
        else:
            lo, hi = sorted(best)
            c = lo if lo == 0 else hi
    return c | ((1 << (fmt.bits - 1)) if neg else 0)


@pytest.mark.parametrize("name", ["S1E2M3", "S1E4M3", "S1E1M2", "S1E2M1", "S1E3M0", "S1E4M3b4",
                                  "S1E5M2", "S1E1M0"])
def test_brute_force_nearest(name):
    fmt = ALL_FORMATS[name]
    half = 1 << (fmt.bits - 1)
    table = [(c, exact_value(c, fmt)) for c in range(half)]          # non-negative codes
    step = float(exact_value(1, fmt)) if fmt.man_bits else float(exact_value(1 << fmt.man_bits, fmt))
    xs = synth.adversarial_values(fmt.max, step, 1500, seed=11)
    # add every midpoint between neighbouring values and its fp32 neighbours
    vals = sorted(v for _, v in table)
    mids = []
    for lo, hi in zip(vals[:-1], vals[1:]):
        m = np.float32(float((lo + hi) / 2))
        mids += [m, np.nextafter(m, np.float32(np.inf)), np.nextafter(m, np.float32(-np.inf))]
    xs = np.concatenate([xs, np.asarray(mids, dtype=np.float32), -np.asarray(mids, dtype=np.float32)])
    got = orc.encode(xs, fmt)
    for x, g in zip(xs, got):
        assert int(g) == brute_force_encode(float(x), fmt, table), (name, float(x))


# ------------------------------------------------------------------ P3: invariants
@pytest.mark.parametrize("name", ["S1E4M3", "S1E3M7", "S1E5M10", "S1E4M14", "S1E2M3", "S1E8M7"])
def test_invariants(name):
    fmt = ALL_FORMATS[name]
    step = float(orc.decode([1], fmt)[0])
    x = synth.adversarial_values(fmt.max, step, 60000, seed=5)
    x = np.concatenate([x, synth.normal_f32(60000, 0.02, 6), synth.normal_f32(20000, min(fmt.max / 3, 1e30), 7)])
    codes = orc.encode(x, fmt)
    q = orc.decode(codes, fmt)
    # idempotence
    assert np.array_equal(orc.encode(q, fmt), codes)
    # sign symmetry: encode(-x) flips only the sign bit
    assert np.array_equal(orc.encode(-x, fmt), codes ^ np.uint32(1 << (fmt.bits - 1)))
    # monotone
    order = np.argsort(x, kind="stable")
    assert np.all(np.diff(q[order].astype(np.float64)) >= 0)
    # saturation
    big = np.abs(x.astype(np.float64)) > fmt.max
    assert np.all(np.abs(q[big]) == np.float32(fmt.max))
    # half-ulp error bound inside the range
    xin = x[~big].astype(np.float64)
    qin = q[~big].astype(np.float64)
    ex = np.floor(np.log2(np.maximum(np.abs(xin), 2.0 ** (1 - fmt.resolved_bias))))
    ulp = np.exp2(ex - fmt.man_bits)
    assert np.all(np.abs(xin - qin) <= 0.5 * ulp)
    # signed zero and tiny negatives
    assert orc.encode([0.0], fmt)[0] == 0
    assert orc.encode([-0.0], fmt)[0] == 1 << (fmt.bits - 1)
    assert orc.encode([-1e-45], fmt)[0] in (1 << (fmt.bits - 1),) or fmt.exp_bits == 8


def test_ties_go_to_even():
    fmt = Format(4, 3)                       # grid near 1.0 has step 1/8
    x = np.array([1.0 + 1 / 16, 1.0 + 3 / 16, 1.0 + 5 / 16, 2 ** -10, 3 * 2 ** -10, 464.0, 496.0],
                 dtype=np.float32)
    want = np.array([1.0, 1.25, 1.25, 0.0, 2 ** -8, 448.0, 480.0], dtype=np.float32)
    assert np.array_equal(orc.decode(orc.encode(x, fmt), fmt), want)


def test_non_finite_inputs_saturate():      # reading of a point the paper is silent on
    fmt = Format(3, 7)
    c = orc.encode(np.array([np.inf, -np.inf, np.nan], dtype=np.float32), fmt)
    q = orc.decode(c, fmt)
    assert q[0] == fmt.max and q[1] == -fmt.max and abs(q[2]) == fmt.max


# ------------------------------------------------------------------ P4: library special cases
def _all_finite_f32_sample(scale_lo, scale_hi, n, seed):
    rng = np.random.default_rng(seed)
    mags = np.exp2(rng.uniform(scale_lo, scale_hi, size=n))
    return (mags * rng.choice([-1.0, 1.0], size=n)).astype(np.float32)


def test_e5m10_is_ieee_half():
    fmt = Format(5, 10)
    codes = valid_codes(fmt)
    e = (codes >> 10) & 31
    sub = codes[e < 31].astype(np.uint16)                 # every finite binary16
    assert np.array_equal(orc.decode(sub, fmt), sub.view(np.float16).astype(np.float32))
    x = _all_finite_f32_sample(-30, 15.99, 300000, 21)
    x = np.concatenate([x, sub.view(np.float16).astype(np.float32)])
    # exact ties between neighbouring halves
    h = sub.view(np.float16).astype(np.float64)
    h = np.sort(h[np.isfinite(h)])
    ties = ((h[:-1] + h[1:]) / 2).astype(np.float32)
    x = np.concatenate([x, ties])
    x = x[np.abs(x) < 65520]
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16).astype(np.uint32)
    assert np.array_equal(orc.encode(x, fmt), want)


def test_e8m7_is_bfloat16():
    fmt = Format(8, 7)
    x = _all_finite_f32_sample(-140, 127, 300000, 22)
    x = np.concatenate([x, synth.normal_f32(100000, 0.05, 23)])
    t = torch.from_numpy(x).to(torch.bfloat16)
    keep = torch.isfinite(t.float()).numpy()
    want = t.view(torch.int16).numpy().view(np.uint16).astype(np.uint32)
    got = orc.encode(x, fmt)
    assert np.array_equal(got[keep], want[keep])
    assert np.array_equal(orc.decode(got[keep], fmt), t.float().numpy()[keep])


def test_e4m3_is_ocp_fp8_below_its_nan_code():
    fmt = Format(4, 3)
    x = _all_finite_f32_sample(-14, 8.8, 200000, 24)
    x = np.concatenate([x, np.arange(-448, 449, dtype=np.float32) / 1.0,
                        np.arange(-4096, 4097, dtype=np.float32) * np.float32(2.0 ** -13)])
    x = x[np.abs(x) <= 448]
    t = torch.from_numpy(x).to(torch.float8_e4m3fn)
    want = t.view(torch.uint8).numpy().astype(np.uint32)
    assert np.array_equal(orc.encode(x, fmt), want)
    assert np.array_equal(orc.decode(want, fmt), t.float().numpy())


def test_e5m2_is_ocp_fp8_below_its_inf_code():
    fmt = Format(5, 2)
    x = _all_finite_f32_sample(-20, 15.8, 200000, 25)
    x = x[np.abs(x) < 61440]
    t = torch.from_numpy(x).to(torch.float8_e5m2)
    want = t.view(torch.uint8).numpy().astype(np.uint32)
    assert np.array_equal(orc.encode(x, fmt), want)
    assert np.array_equal(orc.decode(want, fmt), t.float().numpy())


# ------------------------------------------------------------------ P8: packing
def numpy_pack(codes: np.ndarray, bits: int) -> np.ndarray:
    """Independent packer: expand to one bit per byte, LSB first, let numpy pack little-endian."""
    b = ((codes[:, None].astype(np.uint64) >> np.arange(bits, dtype=np.uint64)) & 1).astype(np.uint8)
    stream = np.packbits(b.ravel(), bitorder="little")
    pad = (-stream.size) % 16
    return np.concatenate([stream, np.zeros(pad, dtype=np.uint8)])


@pytest.mark.parametrize("bits", list(range(2, 33)))
def test_pack_unpack_identity_and_layout(bits):
    rng = np.random.default_rng(bits)
    for n in (1, 31, 33, 64, 257, 2048 + 37):
        codes = rng.integers(0, 1 << bits, size=n, dtype=np.uint64).astype(np.uint32)
        p = orc.pack(codes, bits)
        assert p.size % 16 == 0 and p.size == orc.packed_bytes(n, bits)
        assert p.size - (n * bits + 7) // 8 < 16
        assert np.array_equal(p, numpy_pack(codes, bits))      # layout + zero padding
        assert np.array_equal(orc.unpack(p, n, bits), codes)


def test_pack_little_endian_dwords():
    # stream bit i is bit (i mod 32) of little-endian dword i // 32
    codes = np.array([0x5, 0x3, 0x7FF], dtype=np.uint32)        # 11-bit codes
    p = orc.pack(codes, 11)
    dw = p.view("<u4")
    assert dw[0] == (0x5 | (0x3 << 11) | ((0x7FF << 22) & 0xFFFFFFFF))
    assert dw[1] == (0x7FF >> 10)
