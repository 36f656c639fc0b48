"""Pins for the oracle's group-wise quantizer with FP8-E4M3 scales and BF16 zero-points.

The 8-bit format is pinned to PyTorch's independent implementation of float8_e4m3fn (decode of all
256 encodings, nearest rounding) rather than to the oracle's own formula; the quantizer is pinned to
the properties Eq. 1 of the paper promises (range covered, |error| <= step / 2) and to the storage
arithmetic of the effective-bitwidth formula."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26266_amd import workloads as wl


def _e4m3_table():
    vals = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    return vals


def test_e4m3_ceil_against_torch_table():
    table = _e4m3_table()
    pos = np.sort(table[(table > 0) & np.isfinite(table)])
    assert pos[0] == 2.0 ** -9 and pos[-1] == 448.0 and len(pos) == 126
    rng = np.random.default_rng(7)
    xs = np.concatenate([np.exp(rng.uniform(np.log(1e-4), np.log(600.0), 4000)), pos, pos * (1 + 1e-12),
                         pos * (1 - 1e-12)])
    for x in xs:
        v, byte = oracle.e4m3_ceil(float(x))
        want = pos[np.searchsorted(pos, x, side="left")] if x <= 448.0 else 448.0
        assert v == want, (x, v, want)
        assert table[byte] == v                      # the encoding decodes (by torch's table) to the value
        # consistent with nearest rounding: the nearest value is this one or the one below it
        near = float(torch.tensor([min(x, 448.0)], dtype=torch.float32).to(torch.float8_e4m3fn).float()[0])
        assert near <= v


def test_bf16_round_against_torch():
    rng = np.random.default_rng(3)
    xs = np.concatenate([np.arange(-600, 601, dtype=np.float64), rng.integers(-70000, 70000, 2000).astype(np.float64)])
    got = np.array([oracle.bf16_round(float(x)) for x in xs])
    want = torch.tensor(xs, dtype=torch.float32).to(torch.bfloat16).float().numpy().astype(np.float64)
    assert np.array_equal(got, want)
    assert oracle.bf16_round(257.0) == 256.0 and oracle.bf16_round(259.0) == 260.0   # ties to even


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("group", [32, 64, 128])
def test_fp8meta_quantizer_covers_range_and_bounds_error(bits, group):
    rng = np.random.default_rng(11)
    d = 128
    x = wl.round_to_bf16((rng.standard_normal((300, d)) * np.exp(rng.uniform(-3, 3, (300, 1)))).astype(np.float32))
    codes, scale, zero = oracle.quantize(x, bits, group, True, True)
    L = 2 ** bits - 1
    table = _e4m3_table()
    assert np.all(np.isin(scale.astype(np.float64), table))                     # stored scales are E4M3 values
    assert np.array_equal(zero, torch.tensor(zero).to(torch.bfloat16).float().numpy())  # stored zeros are BF16
    assert codes.min() >= 0 and codes.max() <= L
    u = np.stack([oracle.hadamard(r) for r in x.astype(np.float64)]) * 0.08838834764831845
    xhat = oracle.dequantize(codes, scale, zero)
    G = d // group
    step = np.repeat(scale.astype(np.float64), group, axis=1)
    assert np.all(np.abs(xhat - u) <= 0.5 * step * (1 + 1e-9))                  # Eq. 1's bound with the stored step
    ug = u.reshape(300, G, group)
    rng_ = ug.max(axis=2) - ug.min(axis=2)
    s = scale.astype(np.float64)
    assert np.all(s * L >= rng_ * (1 - 1e-12))                                  # the grid covers [min, max] ...
    pos = np.sort(table[(table > 0) & np.isfinite(table)])
    below = pos[np.maximum(np.searchsorted(pos, s, side="left") - 1, 0)]
    tight = (s > pos[0]) & (s < 448.0)
    assert np.all((below * L < rng_)[tight])                                    # ... and no smaller E4M3 step would
    # min maps to code 0; the stored step exceeds the exact one by less than one E4M3 spacing (1/8), so
    # max still lands within one code of L / 1.125
    cg = codes.reshape(300, G, group)
    assert np.all(np.take_along_axis(cg, ug.argmin(axis=2)[..., None], axis=2) == 0)
    assert np.all(np.take_along_axis(cg, ug.argmax(axis=2)[..., None], axis=2) >= round(L / 1.125) - 1)


def test_fp8meta_groups_are_independent_and_finer_groups_help():
    rng = np.random.default_rng(5)
    x = wl.round_to_bf16(rng.standard_normal((64, 128)).astype(np.float32))
    u = np.stack([oracle.hadamard(r) for r in x.astype(np.float64)]) * 0.08838834764831845
    err = {}
    for g in (128, 64, 32):
        c, s, z = oracle.quantize(x, 2, g, True, True)
        err[g] = float(np.mean((oracle.dequantize(c, s, z) - u) ** 2))
    assert err[32] < err[64] < err[128]
    # a group is quantized from its own range only: changing one group's content through a rotation-
    # free call leaves the other groups' codes and metadata alone
    y = x.astype(np.float64).copy()
    c0, s0, z0 = oracle.quantize(y, 2, 32, False, True)
    y[:, 32:64] *= 3.0
    c1, s1, z1 = oracle.quantize(y, 2, 32, False, True)
    keep = np.r_[0:32, 64:128]
    assert np.array_equal(c0[:, keep], c1[:, keep])
    assert np.array_equal(s0[:, [0, 2, 3]], s1[:, [0, 2, 3]]) and np.array_equal(z0[:, [0, 2, 3]], z1[:, [0, 2, 3]])


def test_fp8meta_degenerate_groups():
    x = np.zeros((3, 128))
    x[1, :] = 2.0           # constant row: after rotation only channel 0 is non-zero
    x[2, 5] = 1.0
    c, s, z = oracle.quantize(x, 2, 32, True, True)
    assert np.all(c[0] == 0) and np.all(s[0] == 0) and np.all(z[0] == 0)
    # row 1: groups 1..3 are all-zero after rotation, group 0 holds the single value 2*sqrt(128)/sqrt(128)...
    assert np.all(s[1, 1:] == 0) and s[1, 0] > 0
    xhat = oracle.dequantize(c, s, z)
    u = np.stack([oracle.hadamard(r) for r in x]) * 0.08838834764831845
    step = np.repeat(s.astype(np.float64), 32, axis=1)
    assert np.all(np.abs(xhat - u) <= 0.5 * step + 1e-12)


def test_effective_bitwidth_of_the_format():
    # "Effective bitwidth": B + 24 / g with one 8-bit scale and one 16-bit zero-point per group
    for bits, g, want in ((2, 32, 2.75), (2, 128, 2.1875), (4, 64, 4.375)):
        d = 128
        assert (d * bits + (8 + 16) * (d // g)) / d == want


def _hand_groups():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "fp8meta_hand_groups.txt")
    rows = []
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        bits, x, codes, step, zero, plain = [f.strip() for f in line.split("|")]
        rows.append((int(bits), np.array(x.split(), dtype=np.float64), np.array(codes.split(), dtype=np.int64),
                     float(step), float(zero), np.array(plain.split(), dtype=np.int64)))
    return rows


def test_bf16_zero_point_beyond_256_hand_worked():
    """Zero-points above 256 in magnitude are not BF16 values: the stored one is rounded (8 significant bits,
    ties to even) and the codes are taken with the stored one.  Expected values are worked by hand in the
    golden file; a quantizer that took the codes with the unrounded zero-point would give its last column."""
    rows = _hand_groups()
    assert len(rows) >= 5
    for bits, x, codes, step, zero, plain in rows:
        g = len(x)
        got_codes, got_scale, got_zero = oracle.quantize(x[None, :], bits, g, False, True)
        assert abs(zero) > 256
        assert got_scale[0, 0] == np.float32(step), (x, got_scale)
        assert got_zero[0, 0] == np.float32(zero), (x, got_zero)
        assert np.array_equal(got_codes[0].astype(np.int64), codes), (x, got_codes)
        assert not np.array_equal(codes, plain)          # the rounding of the zero-point is visible in the codes
        # the same group without the 8-bit/16-bit metadata keeps the integer zero-point and the plain codes
        # (steps here are exact in E4M3 or, where they are not, the row says so by its stored step)
        if step * (2 ** bits - 1) == x.max() - x.min():
            c32, s32, z32 = oracle.quantize(x[None, :], bits, g, False, False)
            assert np.array_equal(c32[0].astype(np.int64), plain) and s32[0, 0] == np.float32(step)
            assert abs(z32[0, 0] - zero) >= 1


def test_error_bound_fails_only_where_the_zero_point_is_rounded():
    """|error| <= step / 2 holds whenever the BF16 zero-point is exact (|z| <= 256) and can fail beyond it: the
    second hand-worked group reconstructs every value as 1008 (error up to 2 with a step of 0.5)."""
    bits, x, codes, step, zero, _ = _hand_groups()[1]
    got_codes, got_scale, got_zero = oracle.quantize(x[None, :], bits, len(x), False, True)
    xhat = oracle.dequantize(got_codes, got_scale, got_zero)[0]
    assert np.array_equal(xhat, np.full(4, 1008.0)) and np.max(np.abs(xhat - x)) == 2.0
    rng = np.random.default_rng(21)
    for _ in range(200):
        off = rng.uniform(-60, 60)
        xs = wl.round_to_bf16((rng.standard_normal(32) + off).astype(np.float32)).astype(np.float64)
        c, s, z = oracle.quantize(xs[None, :], 2, 32, False, True)
        if abs(z[0, 0]) <= 256:
            assert np.all(np.abs(oracle.dequantize(c, s, z)[0] - xs) <= 0.5 * s[0, 0] * (1 + 1e-9))
