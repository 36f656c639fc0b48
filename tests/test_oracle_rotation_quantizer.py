"""Pins for the oracle's rotation and round-to-nearest quantizer (CPU only).

Nothing here compares the oracle with itself: every expectation is a hand-worked
row, a mathematical invariant, or an independently constructed matrix.
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def sylvester(d):
    """Hadamard matrix by the Kronecker recursion (independent of the oracle's parity rule)."""
    h = np.array([[1.0]])
    while h.shape[0] < d:
        h = np.kron(np.array([[1.0, 1.0], [1.0, -1.0]]), h)
    return h


# ---------------------------------------------------------------- rotation ----
@pytest.mark.parametrize("d", [2, 4, 8, 64, 128])
def test_rotation_matches_kronecker_construction(oracle, d):
    rng = np.random.default_rng(d)
    x = rng.standard_normal(d)
    np.testing.assert_allclose(oracle.hadamard(x), sylvester(d) @ x, rtol=0, atol=1e-12)


def test_rotation_hand_worked_d4(oracle):
    # H4 [1,2,3,4]: row sums with signs ++++, +-+-, ++--, +--+
    np.testing.assert_array_equal(oracle.hadamard([1, 2, 3, 4]), [10, -2, -4, 0])


@pytest.mark.parametrize("d", [64, 128])
def test_rotation_is_orthogonal_and_preserves_scores(oracle, d):
    # Preliminaries, "Hadamard rotation": H^T H = I and (Hq)^T (Hk) = q^T k.
    rng = np.random.default_rng(7)
    q, k = rng.standard_normal(d), rng.standard_normal(d)
    hq, hk = oracle.hadamard(q) / np.sqrt(d), oracle.hadamard(k) / np.sqrt(d)
    np.testing.assert_allclose(oracle.hadamard(hq) / np.sqrt(d), q, atol=1e-13)
    assert abs(hq @ hk - q @ k) < 1e-12
    assert abs(hq @ hq - q @ q) < 1e-12  # ||Hq|| = ||q|| (appendix on the rotated correction)
    e0 = np.zeros(d)
    e0[0] = np.sqrt(d)
    np.testing.assert_allclose(oracle.hadamard(np.ones(d)) / np.sqrt(d), e0, atol=1e-13)


def test_rotation_rejects_non_power_of_two(oracle):
    with pytest.raises(ValueError):
        oracle.hadamard(np.ones(48))


# --------------------------------------------------------------- quantizer ----
def _load_rows():
    rows = []
    with open(os.path.join(GOLDEN, "rtn_hand_rows.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            bits, x, codes, scale, zero = [p.strip() for p in line.split("|")]
            rows.append((int(bits), [float(t) for t in x.split()], [int(t) for t in codes.split()],
                         float(scale), float(zero)))
    return rows


@pytest.mark.parametrize("bits,x,codes,scale,zero", _load_rows())
def test_quantizer_hand_worked_rows(oracle, bits, x, codes, scale, zero):
    c, s, z = oracle.quantize(np.array([x]), bits, rotate=False)
    assert c[0].tolist() == codes
    assert s[0, 0] == np.float32(scale)
    assert z[0, 0] == np.float32(zero)


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("d", [64, 128])
def test_quantizer_error_bound_after_rotation(oracle, bits, d):
    # |x^ - x| <= step/2 (sentence after Eq. 1); the stored step is rounded to
    # float after the codes are chosen, which adds at most L * 2^-24 * step.
    rng = np.random.default_rng(bits * 1000 + d)
    x = rng.standard_normal((257, d))
    x[:, 5] *= 10.0
    L = 2 ** bits - 1
    codes, scale, zero = oracle.quantize(x, bits)
    y = np.stack([oracle.hadamard(r) for r in x]) / np.sqrt(d)
    err = np.abs(oracle.dequantize(codes, scale, zero) - y)
    bound = 0.5 * scale.astype(np.float64) * (1 + L * 2.0 ** -22)
    assert np.all(err <= bound)
    assert codes.min() == 0 and codes.max() == L
    assert np.all(codes.min(axis=1) == 0)         # the minimum of every row maps to code 0
    assert np.mean(codes.max(axis=1) == L) > 0.99  # the maximum maps to L (bar exact ties)
    # the bound is tight: some element comes close to step/2
    assert np.max(err / scale) > 0.45


def test_quantizer_error_is_roughly_uniform(oracle):
    # Noise model (Eq. 5): error ~ U(-step/2, step/2): mean 0, variance step^2/12.
    rng = np.random.default_rng(11)
    x = rng.standard_normal((4096, 128))
    codes, scale, zero = oracle.quantize(x, 4)
    y = np.stack([oracle.hadamard(r) for r in x]) / np.sqrt(128)
    e = (oracle.dequantize(codes, scale, zero) - y) / scale
    assert abs(e.mean()) < 2e-3
    assert abs(e.var() - 1.0 / 12.0) < 2e-3


@pytest.mark.parametrize("bits", [2, 4])
def test_quantizer_grid_points_are_lossless(oracle, bits):
    L = 2 ** bits - 1
    rng = np.random.default_rng(3)
    grid = rng.integers(0, L + 1, size=(64, 16)).astype(np.float64)
    grid[:, 0], grid[:, 1] = 0, L
    x = (grid - 2.0) * 0.375  # step 0.375, zero-point 2
    codes, scale, zero = oracle.quantize(x, bits, rotate=False)
    np.testing.assert_array_equal(codes, grid.astype(np.uint8))
    assert np.all(scale == np.float32(0.375)) and np.all(zero == 2.0)
    np.testing.assert_array_equal(oracle.dequantize(codes, scale, zero), x)


def test_quantizer_power_of_two_scaling(oracle):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((32, 128))
    c1, s1, z1 = oracle.quantize(x, 2)
    c2, s2, z2 = oracle.quantize(x * 2.0 ** -7, 2)
    np.testing.assert_array_equal(c1, c2)
    np.testing.assert_array_equal(z1, z2)
    np.testing.assert_array_equal(s1 * np.float32(2.0 ** -7), s2)


def test_quantizer_degenerate_rows(oracle):
    d = 8
    zero_row = np.zeros((1, d))
    c, s, z = oracle.quantize(zero_row, 2, rotate=False)
    assert not c.any() and s[0, 0] == 0 and z[0, 0] == 0
    const = np.full((1, d), 2.5)
    c, s, z = oracle.quantize(const, 2, rotate=False)
    # a nonzero constant sits on the top grid point: exact up to the float rounding of the stored step
    np.testing.assert_allclose(oracle.dequantize(c, s, z), const, rtol=2.0 ** -23, atol=0)
    assert np.all(c == 3) and z[0, 0] == 0
    neg = np.full((1, d), -1.25)
    c, s, z = oracle.quantize(neg, 2, rotate=False)
    np.testing.assert_allclose(oracle.dequantize(c, s, z), neg, rtol=2.0 ** -23, atol=0)
    assert np.all(c == 0) and z[0, 0] == 3


def test_quantizer_one_signed_row_has_zero_point_outside_code_range(oracle):
    # The range is the tight [min, max]; nothing forces it to contain 0, so z can leave [0, L].
    x = np.array([[10.0, 10.5, 11.0, 11.5, 12.0, 13.0, 10.25, 12.75]])
    c, s, z = oracle.quantize(x, 2, rotate=False)
    assert z[0, 0] == -10.0 and s[0, 0] == 1.0
    assert np.all(np.abs(oracle.dequantize(c, s, z) - x) <= 0.5)


def test_quantizer_groups_are_independent(oracle):
    rng = np.random.default_rng(9)
    x = rng.standard_normal((16, 128))
    c, s, z = oracle.quantize(x, 2, group=32, rotate=False)
    for j in range(4):
        cj, sj, zj = oracle.quantize(x[:, 32 * j:32 * j + 32], 2, rotate=False)
        np.testing.assert_array_equal(c[:, 32 * j:32 * j + 32], cj)
        np.testing.assert_array_equal(s[:, j], sj[:, 0])
        np.testing.assert_array_equal(z[:, j], zj[:, 0])


def test_quantizer_rotation_happens_before_rounding(oracle):
    # Quantizing x with rotation == quantizing H x without, up to the 1/sqrt(d) in the stored step.
    rng = np.random.default_rng(13)
    x = rng.standard_normal((8, 64))
    u = np.stack([oracle.hadamard(r) for r in x])
    c1, s1, z1 = oracle.quantize(x, 2, rotate=True)
    c2, s2, z2 = oracle.quantize(u, 2, rotate=False)
    np.testing.assert_array_equal(c1, c2)
    np.testing.assert_array_equal(z1, z2)
    np.testing.assert_array_equal(s1, (s2.astype(np.float64) * 0.125).astype(np.float32))


def test_effective_bitwidth_values_printed_in_the_paper():
    # B_eff = B + 24/g for an FP8 scale and a BF16 zero-point per group.
    with open(os.path.join(GOLDEN, "effective_bits.txt")) as f:
        rows = [l.split("#")[0].split() for l in f if l.split("#")[0].strip()]
    for bits, g, printed in rows:
        assert round(int(bits) + 24.0 / int(g), 2) == pytest.approx(float(printed), abs=0.006)
