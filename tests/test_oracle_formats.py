"""Pins for the oracle's number formats and phi (Sec. 2.1, Eq. 1, Eq. 2).

Nothing here re-types the oracle's own formula: values come from the paper's
stated constants (tests/golden), from torch's float8 decoder/caster, or from
exact rational arithmetic.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from tests import indep
from workloads import bf16_bits_to_f32

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _golden_constants():
    out = {}
    for line in open(os.path.join(GOLD, "formats.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def test_e2m1_value_set_matches_paper_constants():
    g = _golden_constants()
    vals = [oracle.e2m1_value(c) for c in range(16)]
    assert len(set(vals)) == g["e2m1_distinct_values"]          # +0 and -0 coincide
    assert max(vals) == g["e2m1_max"] and min(vals) == -g["e2m1_max"]
    # E2M1 = 1 sign, 2 exponent, 1 mantissa bit: magnitudes are m/2 (e=0) and (1+m/2)*2^(e-1)
    want = sorted({(m / 2 if e == 0 else (1 + m / 2) * 2.0 ** (e - 1))
                   for e in range(4) for m in range(2)})
    assert sorted(set(abs(v) for v in vals)) == want


def test_e4m3_table_matches_torch_decoder():
    g = _golden_constants()
    grid = indep.e4m3_grid_torch()
    mine = np.array([oracle.e4m3_value(b) for b in range(0x7F)])
    assert np.array_equal(mine, grid)
    assert mine.max() == g["e4m3_scale_max"]
    assert mine[1] == 2.0 ** -9 and np.all(np.diff(mine) > 0)


def test_scale_hand_cases():
    for line in open(os.path.join(GOLD, "scale_hand_cases.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        amax, scale, byte = line.split()[:3]
        b = oracle.e4m3_from_amax(float(amax))
        assert b == int(byte, 16), line
        assert oracle.e4m3_value(b) == float(scale), line


def test_scale_rounding_exact_over_bf16_amax():
    """Every positive bf16 amax in a wide range: RNE_E4M3(amax/6) decided on rationals."""
    grid = indep.e4m3_grid_exact()
    # bf16 bit patterns: exponents from 2^-12 up past saturation, all 128 mantissas (strided)
    bits = np.array([(e << 7) | m for e in range(127 - 12, 127 + 13) for m in range(0, 128, 3)],
                    dtype=np.uint16)
    for a in bf16_bits_to_f32(bits):
        want = indep.nearest_even_index(Fraction(float(a)) / 6, grid)
        assert oracle.e4m3_from_amax(float(a)) == want, float(a)


def test_scale_rounding_matches_torch_cast_when_quotient_is_exact():
    """amax = 6*v with v exactly representable: torch's RNE cast of v is the answer."""
    rng = np.random.default_rng(0)
    v = (rng.integers(1, 1 << 12, 4000) * 2.0 ** rng.integers(-20, -3, 4000)).astype(np.float32)
    v = v[v <= 448.0]
    tb = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = np.array([oracle.e4m3_from_amax(6.0 * float(x)) for x in v])
    assert np.array_equal(mine, tb)


def test_e2m1_ties_and_neighbours():
    # ties go to the code with even mantissa: 0, 1, 1, 2, 2, 4, 4; above 5 -> 6
    ties = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    V = oracle.E2M1_VALUES
    for s in (1.0, 0.171875, 448.0, 2.0 ** -9):
        for t, want in ties.items():
            assert V[oracle.e2m1_round(t * s, s)] == want
            up = np.nextafter(t * s, np.inf); dn = np.nextafter(t * s, -np.inf)
            lo = max(v for v in V if v < t); hi = min(v for v in V if v > t)
            assert V[oracle.e2m1_round(up, s)] == hi and V[oracle.e2m1_round(dn, s)] == lo
        assert V[oracle.e2m1_round(1e9 * s, s)] == 6.0         # saturates
        assert V[oracle.e2m1_round(0.0, s)] == 0.0


def test_e2m1_round_exact_random():
    rng = np.random.default_rng(1)
    grid = indep.e4m3_grid_exact()
    for _ in range(3000):
        sb = int(rng.integers(1, 0x7F))
        x = float(bf16_bits_to_f32(np.array([rng.integers(0, 0x7F80)], dtype=np.uint16))[0])
        s = grid[sb]
        want = indep.nearest_even_index(Fraction(x) / s, indep.E2M1)
        assert oracle.e2m1_round(x, float(s)) == want


def test_phi_round_trip_all_values_all_scales():
    """phi^-1(phi(s*v)) = s*v for the 15 values and every positive scale, when the block holds 6s."""
    V = np.array([oracle.e2m1_value(c) for c in range(16)])
    for sb in range(1, 0x7F):
        s = oracle.e4m3_value(sb)
        blk = np.zeros((1, 16), np.float32)
        blk[0, :16] = (V * s).astype(np.float32)       # includes +6s and -6s
        assert np.array_equal(blk[0].astype(np.float64), V * s)   # exact in fp32
        packed, scales, xf = oracle.phi(blk)
        assert scales[0, 0] == sb
        assert np.array_equal(xf[0].astype(np.float64), V * s)
        codes = np.stack([packed[0] & 15, packed[0] >> 4], -1).reshape(-1)
        assert np.array_equal(codes & 7, np.arange(16) & 7)
        # sign bit copied from the input, also for -0
        assert np.array_equal(codes >> 3, np.signbit(blk[0]).astype(np.uint8))


def test_phi_matches_exact_rational_phi_on_random_bf16_blocks():
    rng = np.random.default_rng(2)
    bits = rng.integers(0, 1 << 16, size=(300, 16)).astype(np.uint16)
    bits[(bits & 0x7F80) == 0x7F80] = 0x3F80                       # no inf/nan
    x = bf16_bits_to_f32(bits)
    x[::3] *= 2.0 ** -20                                              # some tiny blocks
    x = np.clip(x, -3e4, 3e4).astype(np.float32)
    packed, scales, xf = oracle.phi(x)
    for r in range(x.shape[0]):
        codes, sb, deq = indep.phi_block_exact(list(x[r]))
        got = np.stack([packed[r] & 15, packed[r] >> 4], -1).reshape(-1)
        assert scales[r, 0] == sb
        assert list(got) == codes
        assert [Fraction(float(v)) for v in xf[r]] == deq


def test_phi_numpy_twin_agrees_on_gaussian_rows():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((64, 128)).astype(np.float32)
    x[:, 5] *= 20
    assert np.array_equal(oracle.fake_quant(x).astype(np.float64), indep.fake_quant_np(x))


def test_phi_power_of_two_homogeneity_and_error_bound():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((32, 64)).astype(np.float32)
    xf = oracle.fake_quant(x)
    for k in (-3, 2, 5):
        assert np.array_equal(oracle.fake_quant(x * np.float32(2.0 ** k)), xf * np.float32(2.0 ** k))
    _, scales, _ = oracle.phi(x)
    s = np.array([oracle.e4m3_value(int(b)) for b in scales.reshape(-1)]).reshape(scales.shape)
    s = np.repeat(s, 16, axis=-1)
    # un-saturated elements are within half the largest E2M1 gap (2) times s
    unsat = np.abs(x) <= 6 * s
    assert np.all(np.abs(x - xf)[unsat] <= 1.0 * s[unsat] + 1e-12)
    # the scale is within one E4M3 half-step (1/16 relative) of amax/6
    amax = np.abs(x).reshape(32, 4, 16).max(-1)
    sc = s[:, ::16]
    assert np.all(np.abs(sc - amax / 6) <= sc / 16 + 1e-12)


def test_phi_zero_block_and_underflow_block():
    x = np.zeros((2, 16), np.float32)
    x[1, :] = 1e-4                       # amax/6 < 2^-10: the scale rounds to 0
    packed, scales, xf = oracle.phi(x)
    assert not scales.any() and not xf.any() and not packed.any()


def test_packed_nibble_order():
    x = np.zeros((1, 16), np.float32)
    x[0, 0] = 6.0     # element 0 -> low nibble of byte 0
    x[0, 1] = -3.0    # element 1 -> high nibble of byte 0
    packed, scales, _ = oracle.phi(x)
    assert packed[0, 0] == (7 | ((8 | 5) << 4)) and scales[0, 0] == 0x38


@pytest.mark.parametrize("mode", [0, 1])
def test_scale_mode_literal_eq1(mode):
    """scale_mode 1 keeps Eq. 1's un-rounded scale: the block max is then reproduced exactly."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((8, 16)).astype(np.float32)
    xf = oracle.fake_quant(x, scale_mode=mode)
    amax_in = np.abs(x).max(-1); amax_out = np.abs(xf).max(-1)
    if mode == 1:
        assert np.allclose(amax_out, amax_in, rtol=1e-6)
    else:
        assert np.all(np.abs(amax_out - amax_in) <= amax_in / 16 * 1.0001)
