"""Pins for the oracle's per-channel key quantizer and the scalar correction it leads to (CPU only;
appendix "Per-Channel Quantization Correction").  Expectations: a hand-worked block, the per-token
quantizer applied to the transposed block (a different routine, the same definition with the roles of
tokens and channels exchanged), the error bound per channel, and closed forms for the shared b."""
import math

import numpy as np
import pytest
from scipy.special import softmax


def test_hand_worked_block(oracle):
    # 4 tokens x 2 channels, 2 bits, no rotation.  Channel 0: values 0, 1, 2, 3 -> step 1, zero 0, codes
    # 0..3.  Channel 1: values -1, 0.5, 2, -0.25 -> range 3, step 1, inv 1, z = -rint(-1) = 1,
    # codes rint(v) + 1 = 0, 1 (rint(0.5) = 0: ties to even), 3, 1 (rint(-0.25) = -0).
    x = np.array([[0.0, -1.0], [1.0, 0.5], [2.0, 2.0], [3.0, -0.25]])
    codes, scale, zero = oracle.quantize_per_channel(x, 2, rotate=False)
    assert codes.tolist() == [[0, 0], [1, 1], [2, 3], [3, 1]]
    assert scale.tolist() == [1.0, 1.0] and zero.tolist() == [0.0, 1.0]
    # a constant non-zero channel is widened to include 0; an all-zero channel has step 0
    x = np.array([[2.0, 0.0], [2.0, 0.0], [2.0, 0.0]])
    codes, scale, zero = oracle.quantize_per_channel(x, 2, rotate=False)
    assert codes.tolist() == [[3, 0]] * 3 and scale[1] == 0.0 and scale[0] == np.float32(2.0 / 3.0) and zero[0] == 0.0


def test_equals_the_per_token_quantizer_on_the_transposed_block(oracle):
    rng = np.random.default_rng(41)
    for bits in (2, 4):
        x = rng.standard_normal((37, 16)) * np.exp(rng.standard_normal((1, 16)))
        codes, scale, zero = oracle.quantize_per_channel(x, bits, rotate=False)
        tc, ts, tz = oracle.quantize(np.ascontiguousarray(x.T), bits, rotate=False)     # rows = channels
        assert np.array_equal(codes, tc.T) and np.array_equal(scale, ts[:, 0]) and np.array_equal(zero, tz[:, 0])


def test_rotated_error_bound_and_range(oracle):
    rng = np.random.default_rng(42)
    d, rows = 64, 50
    h = np.array([[1.0]])
    while h.shape[0] < d:
        h = np.kron(np.array([[1.0, 1.0], [1.0, -1.0]]), h)
    x = rng.standard_normal((rows, d))
    x[:, 5] *= 10.0
    for bits in (2, 4):
        L = 2 ** bits - 1
        codes, scale, zero = oracle.quantize_per_channel(x, bits)
        y = x @ h / math.sqrt(d)
        yhat = (codes.astype(np.float64) - zero[None, :]) * scale[None, :].astype(np.float64)
        assert np.all(np.abs(yhat - y) <= 0.5 * scale[None, :] * (1 + 1e-6) + 1e-12)
        assert np.all(codes.min(axis=0) == 0) and np.all(codes.max(axis=0) == L)       # range covered per channel
        assert np.allclose(scale, (y.max(axis=0) - y.min(axis=0)) / L, rtol=1e-6)


def test_shared_correction_is_one_scalar_per_query_and_block(oracle):
    """Per-channel steps do not depend on the key, so every cached key of the block gets the same b =
    sigma^2/24 sum_c q~_c^2 step_c^2 and the cached block's odds against the current block shrink by e^-b."""
    rng = np.random.default_rng(43)
    d, m, ns, nr = 16, 5, 30, 7
    q, kr, vr = rng.standard_normal((m, d)), rng.standard_normal((nr, d)), rng.standard_normal((nr, d))
    kc, vc = rng.standard_normal((ns, d)), rng.standard_normal((ns, d))
    codes, scale, zero = oracle.quantize_per_channel(kc, 2, rotate=False)
    khat = (codes.astype(np.float64) - zero[None, :]) * scale[None, :].astype(np.float64)
    steps = np.repeat(scale[None, :].astype(np.float64), ns, axis=0)
    _, mass0 = oracle.attention(q, khat, steps, vc, kr, vr, correction=0, rotate=False)
    _, mass1 = oracle.attention(q, khat, steps, vc, kr, vr, correction=1, rotate=False)
    b = (q ** 2 * scale[None, :].astype(np.float64) ** 2).sum(axis=1) / (24.0 * d)
    odds0, odds1 = mass0 / (1 - mass0), mass1 / (1 - mass1)
    assert np.allclose(odds1, odds0 * np.exp(-b), rtol=1e-11)
    # exact form: sum over channels of log(sinh(a)/a), a = q_c step_c / (2 sqrt(d))
    _, mass2 = oracle.attention(q, khat, steps, vc, kr, vr, correction=2, rotate=False)
    a = q * scale[None, :].astype(np.float64) / (2.0 * math.sqrt(d))
    b2 = np.log(np.sinh(a) / a).sum(axis=1)
    assert np.allclose(mass2 / (1 - mass2), odds0 * np.exp(-b2), rtol=1e-10)
    assert np.all(b2 <= b)


def test_whole_path_with_key_blocks(oracle):
    """chunk_attention with per-channel key blocks: textbook attention over the dequantized keys, written
    with numpy here, with one b per (query, block)."""
    from paper_2605_26266_amd import workloads as wl
    w = wl.WORKLOADS["tiny"]
    kc, vc = wl.chunk_kv(w, 0)
    k2, v2 = wl.chunk_kv(w, 1, n_tokens=40)
    kc, vc = np.concatenate([kc, k2]), np.concatenate([vc, v2])
    kr, vr = wl.chunk_kv(w, 2, n_tokens=33)
    q = wl.chunk_q(w)[:9]
    d = w.head_dim
    out, mass, quant = oracle.chunk_attention(q, kc, vc, kr, vr, 2, 1, key_blocks=[64, 40])
    h = np.array([[1.0]])
    while h.shape[0] < d:
        h = np.kron(np.array([[1.0, 1.0], [1.0, -1.0]]), h)
    hn = h / math.sqrt(d)
    qd = q[:, 0, :].astype(np.float64)
    qr = qd @ hn
    s_parts, t0 = [], 0
    for n in (64, 40):
        c_, s_, z_ = oracle.quantize_per_channel(kc[t0:t0 + n, 0, :], 2)
        assert np.array_equal(quant[0]["k_codes"][t0:t0 + n], c_) and np.array_equal(quant[0]["k_scale"][t0], s_)
        khat = (c_.astype(np.float64) - z_[None, :]) * s_[None, :].astype(np.float64)
        b = (qr ** 2 * s_[None, :].astype(np.float64) ** 2).sum(axis=1) / (24.0 * d)
        s_parts.append(qr @ khat.T / math.sqrt(d) - b[:, None])
        t0 += n
    s = np.concatenate(s_parts + [qd @ kr[:, 0, :].astype(np.float64).T / math.sqrt(d)], axis=1)
    p = softmax(s, axis=1)
    assert np.allclose(mass[0], p[:, :104].sum(axis=1), rtol=1e-11)
    vcodes, vs, vz = quant[0]["v_codes"], quant[0]["v_scale"], quant[0]["v_zero"]
    vhat = (vcodes.astype(np.float64) - vz) * vs.astype(np.float64)
    want = (p[:, :104] @ vhat) @ hn.T + p[:, 104:] @ vr[:, 0, :].astype(np.float64)
    assert np.allclose(out[:, 0, :], want, rtol=1e-10, atol=1e-12)
