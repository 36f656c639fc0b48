"""Pins for the oracle's bias correction and corrected chunk attention (CPU only).

Expectations come from closed forms, quadrature, Monte-Carlo, textbook softmax
attention written independently with numpy/scipy, hand-worked tiny cases and
invariants -- never from a second call of the oracle routine under test.
"""
import math

import numpy as np
import pytest
from scipy.special import softmax


def sylvester(d):
    h = np.array([[1.0]])
    while h.shape[0] < d:
        h = np.kron(np.array([[1.0, 1.0], [1.0, -1.0]]), h)
    return h


# --------------------------------------------------------------- correction ----
def test_log_sinhc_against_direct_formula_and_limits(oracle):
    for a in [0.05, 0.3, 1.0, 2.5, 7.0, 30.0]:
        assert oracle.log_sinhc(a) == pytest.approx(math.log(math.sinh(a) / a), rel=1e-12)
        assert oracle.log_sinhc(-a) == oracle.log_sinhc(a)
    assert oracle.log_sinhc(0.0) == 0.0
    # small argument: a^2/6 - a^4/180 (series of log(sinh a / a))
    a = 1e-4
    assert oracle.log_sinhc(a) == pytest.approx(a * a / 6 - a ** 4 / 180, rel=1e-12)
    # large argument does not overflow: log(sinh a / a) -> a - log(2a)
    assert oracle.log_sinhc(2000.0) == pytest.approx(2000.0 - math.log(4000.0), rel=1e-14)


def test_scalar_moment_by_quadrature(oracle):
    # E[e^{t eps}], eps ~ U(-D/2, D/2), equals sinh(tD/2)/(tD/2) (appendix, scalar MGF).
    x, w = np.polynomial.legendre.leggauss(64)
    for t, D in [(1.0, 0.7), (0.3, 5.0), (2.0, 3.0)]:
        mean = 0.5 * np.sum(w * np.exp(t * x * D / 2))
        assert math.log(mean) == pytest.approx(oracle.correction([t], [D], 1.0, 2), rel=1e-12)


def test_scalar_monte_carlo_jensen_bias_and_second_order_restoration(oracle):
    # Single score, delta ~ U(-D/2, D/2): the mean of e^{s+delta} exceeds e^s, and
    # subtracting the Taylor b = D^2/24 restores it up to the fourth-order term -D^4/2880.
    rng = np.random.default_rng(2024)
    s = 0.8
    for D in [0.5, 1.5]:
        delta = rng.uniform(-D / 2, D / 2, size=10_000_000)
        raw = np.exp(s + delta).mean()
        b = oracle.correction([1.0], [D], 1.0, 1)
        assert b == pytest.approx(D * D / 24, rel=1e-14)
        assert raw > math.exp(s) * (1 + 0.5 * (D * D / 24))
        fixed = np.exp(s + delta - b).mean()
        se = np.exp(delta).std() / math.sqrt(delta.size)
        assert abs(math.log(fixed / math.exp(s)) - (-D ** 4 / 2880)) < 5 * se + D ** 6 / 1e5
        assert abs(fixed - math.exp(s)) < 0.1 * abs(raw - math.exp(s))
        # the exact form removes the bias altogether
        exact = np.exp(s + delta - oracle.correction([1.0], [D], 1.0, 2)).mean()
        assert abs(math.log(exact / math.exp(s))) < 5 * se


def test_taylor_is_half_the_score_noise_variance(oracle):
    # sigma_i^2 = 1/(12 d) sum q_c^2 D_c^2 (Eq. 7) and b ~ sigma_i^2 / 2.
    rng = np.random.default_rng(5)
    d = 16
    q = rng.standard_normal(d)
    D = rng.uniform(0.2, 1.0, size=d)
    eps = rng.uniform(-0.5, 0.5, size=(400_000, d)) * D
    delta = eps @ q / math.sqrt(d)
    b = oracle.correction(q, D, 1 / math.sqrt(d), 1)
    assert b == pytest.approx(np.sum(q * q * D * D) / (24 * d), rel=1e-13)
    assert delta.var() / 2 == pytest.approx(b, rel=2e-2)
    # and the exact multi-channel form equals log E[e^delta]
    assert math.log(np.exp(delta).mean()) == pytest.approx(oracle.correction(q, D, 1 / math.sqrt(d), 2), rel=3e-2)


def test_taylor_overestimates_exact_within_fourth_order(oracle):
    rng = np.random.default_rng(6)
    d = 128
    sigma = 1 / math.sqrt(d)
    for scale in [0.1, 1.0, 4.0]:
        q = rng.standard_normal(d) * scale
        D = rng.uniform(0.5, 2.0)
        bt = oracle.correction(q, [D], sigma, 1)
        be = oracle.correction(q, [D], sigma, 2)
        alpha = 0.5 * sigma * q * D
        assert 0 <= be <= bt
        assert bt - be <= np.sum(alpha ** 4) / 180 * (1 + 1e-9)


def test_correction_sign_monotonicity_and_zero_step(oracle):
    rng = np.random.default_rng(8)
    q = rng.standard_normal(64)
    prev = 0.0
    for D in [0.0, 0.1, 0.5, 1.0, 3.0]:
        for mode in (1, 2):
            assert oracle.correction(q, [D], 0.125, mode) >= 0
        b = oracle.correction(q, [D], 0.125, 1)
        assert b >= prev
        prev = b
    assert oracle.correction(q, [0.0], 0.125, 1) == 0.0
    assert oracle.correction(q, [0.0], 0.125, 2) == 0.0
    assert oracle.correction(q, [1.0], 0.125, 0) == 0.0


def test_single_group_correction_is_rotation_invariant_but_grouped_is_not(oracle):
    rng = np.random.default_rng(9)
    d = 128
    q = rng.standard_normal(d)
    q[3] *= 10
    hq = sylvester(d) @ q / math.sqrt(d)
    b_q = oracle.correction(q, [0.7], 1 / math.sqrt(d), 1)
    b_hq = oracle.correction(hq, [0.7], 1 / math.sqrt(d), 1)
    assert b_q == pytest.approx(b_hq, rel=1e-12)          # ||Hq||^2 = ||q||^2
    assert b_q == pytest.approx(0.49 * (q @ q) / (24 * d), rel=1e-12)
    steps = np.array([0.2, 0.9, 0.4, 1.3])
    g_q = oracle.correction(q, steps, 1 / math.sqrt(d), 1)
    g_hq = oracle.correction(hq, steps, 1 / math.sqrt(d), 1)
    assert abs(g_q - g_hq) > 1e-3 * g_q                    # per-group norms differ after mixing
    manual = sum(steps[j] ** 2 * np.sum(hq[32 * j:32 * j + 32] ** 2) for j in range(4)) / (24 * d)
    assert g_hq == pytest.approx(manual, rel=1e-12)


# ---------------------------------------------------------------- attention ----
def textbook(q, k, v, sigma, bias=None):
    s = sigma * q @ k.T
    if bias is not None:
        s = s - bias
    p = softmax(s, axis=1)
    return p @ v, p


def test_hand_worked_two_cached_one_current(oracle):
    # d = 2, sigma = 1, one query [1, 0]; cached keys [1,0], [0,1] with steps 0; current key [0,0].
    # scores (1, 0 | 0): p = (e, 1, 1)/(e + 2).
    q = np.array([[1.0, 0.0]])
    kh = np.array([[1.0, 0.0], [0.0, 1.0]])
    vh = np.array([[1.0, 2.0], [3.0, 4.0]])
    kr = np.array([[0.0, 0.0]])
    vr = np.array([[5.0, 6.0]])
    out, mass = oracle.attention(q, kh, np.zeros((2, 1)), vh, kr, vr, sigma=1.0, correction=1, rotate=False)
    z = math.e + 2
    np.testing.assert_allclose(out[0], [(math.e * 1 + 3 + 5) / z, (math.e * 2 + 4 + 6) / z], rtol=1e-14)
    assert mass[0] == pytest.approx((math.e + 1) / z, rel=1e-14)
    # now give the first cached key step 2: b = sigma^2 * 4 * ||q||^2 / 24 = 1/6 on that score only
    out, mass = oracle.attention(q, kh, np.array([[2.0], [0.0]]), vh, kr, vr, sigma=1.0, correction=1, rotate=False)
    e1 = math.exp(1 - 1 / 6)
    z = e1 + 2
    np.testing.assert_allclose(out[0], [(e1 * 1 + 3 + 5) / z, (e1 * 2 + 4 + 6) / z], rtol=1e-14)
    assert mass[0] == pytest.approx((e1 + 1) / z, rel=1e-14)


@pytest.mark.parametrize("d", [64, 128])
def test_zero_step_reduces_to_textbook_attention(oracle, d):
    rng = np.random.default_rng(d)
    m, ns, nr = 9, 37, 13
    q, k, v = rng.standard_normal((m, d)), rng.standard_normal((ns + nr, d)), rng.standard_normal((ns + nr, d))
    sigma = 1 / math.sqrt(d)
    ref, p = textbook(q, k, v, sigma)
    for corr in (0, 1, 2):
        out, mass = oracle.attention(q, k[:ns], np.zeros((ns, 1)), v[:ns], k[ns:], v[ns:], correction=corr, rotate=False)
        np.testing.assert_allclose(out, ref, atol=1e-13)
        np.testing.assert_allclose(mass, p[:, :ns].sum(1), atol=1e-13)
    # rotated basis: cached keys/values given as K Hn, V Hn; queries/current in the original basis
    hn = sylvester(d) / math.sqrt(d)
    out, mass = oracle.attention(q, k[:ns] @ hn, np.zeros((ns, 1)), v[:ns] @ hn, k[ns:], v[ns:], correction=1, rotate=True)
    np.testing.assert_allclose(out, ref, atol=1e-12)
    np.testing.assert_allclose(mass, p[:, :ns].sum(1), atol=1e-12)


def test_correction_is_subtracted_from_cached_scores_only(oracle):
    rng = np.random.default_rng(21)
    d, m, ns, nr = 64, 5, 23, 11
    sigma = 0.2
    q, k, v = rng.standard_normal((m, d)), rng.standard_normal((ns + nr, d)), rng.standard_normal((ns + nr, d))
    step = rng.uniform(0.3, 2.0, size=(ns, 1))
    bias = np.zeros((m, ns + nr))
    bias[:, :ns] = sigma ** 2 * (step[:, 0] ** 2)[None, :] * np.sum(q * q, axis=1)[:, None] / 24
    ref, p = textbook(q, k, v, sigma, bias)
    out, mass = oracle.attention(q, k[:ns], step, v[:ns], k[ns:], v[ns:], sigma=sigma, correction=1, rotate=False)
    np.testing.assert_allclose(out, ref, atol=1e-13)
    np.testing.assert_allclose(mass, p[:, :ns].sum(1), atol=1e-13)
    off, mass_off = oracle.attention(q, k[:ns], step, v[:ns], k[ns:], v[ns:], sigma=sigma, correction=0, rotate=False)
    assert np.all(mass <= mass_off)          # b >= 0 can only move mass off the cache
    assert np.all(mass < mass_off - 1e-6)


def test_empty_cache_and_empty_current_block(oracle):
    rng = np.random.default_rng(22)
    d = 64
    q, k, v = rng.standard_normal((4, d)), rng.standard_normal((10, d)), rng.standard_normal((10, d))
    ref, _ = textbook(q, k, v, 0.125)
    out, mass = oracle.attention(q, np.zeros((0, d)), np.zeros((0, 1)), np.zeros((0, d)), k, v)
    np.testing.assert_allclose(out, ref, atol=1e-13)
    assert np.all(mass == 0)
    out, mass = oracle.attention(q, k, np.zeros((10, 1)), v, np.zeros((0, d)), np.zeros((0, d)), rotate=False)
    np.testing.assert_allclose(out, ref, atol=1e-13)
    np.testing.assert_allclose(mass, 1.0, atol=1e-15)
    with pytest.raises(ValueError):
        oracle.attention(q, np.zeros((0, d)), np.zeros((0, 1)), np.zeros((0, d)), np.zeros((0, d)), np.zeros((0, d)))


def test_cached_token_permutation_invariance(oracle):
    rng = np.random.default_rng(23)
    d, ns = 64, 40
    q, kr, vr = rng.standard_normal((6, d)), rng.standard_normal((7, d)), rng.standard_normal((7, d))
    kh, vh, st = rng.standard_normal((ns, d)), rng.standard_normal((ns, d)), rng.uniform(0.1, 1, (ns, 1))
    perm = rng.permutation(ns)
    a, ma = oracle.attention(q, kh, st, vh, kr, vr)
    b, mb = oracle.attention(q, kh[perm], st[perm], vh[perm], kr, vr)
    np.testing.assert_allclose(a, b, atol=1e-13)
    np.testing.assert_allclose(ma, mb, atol=1e-13)


def test_shared_steps_shift_the_cached_block_uniformly(oracle):
    # Per-channel quantization (appendix): steps that do not depend on the key give one scalar b
    # per query, so relative weights inside the cached block do not change; only P_S moves.
    rng = np.random.default_rng(24)
    d, ns, nr = 64, 12, 5
    sigma = 0.125
    q = rng.standard_normal((3, d))
    kh, vh = rng.standard_normal((ns, d)), np.eye(ns, d)          # values pick out the weights
    kr, vr = rng.standard_normal((nr, d)), np.zeros((nr, d))
    st = np.full((ns, 1), 0.8)
    on, m_on = oracle.attention(q, kh, st, vh, kr, vr, sigma=sigma, correction=1, rotate=False)
    off, m_off = oracle.attention(q, kh, st, vh, kr, vr, sigma=sigma, correction=0, rotate=False)
    w_on, w_off = on[:, :ns], off[:, :ns]
    np.testing.assert_allclose(w_on / w_on.sum(1, keepdims=True), w_off / w_off.sum(1, keepdims=True), atol=1e-13)
    b = sigma ** 2 * 0.64 * np.sum(q * q, axis=1) / 24
    # odds of the cached block shrink by exactly e^{-b}
    np.testing.assert_allclose((m_on / (1 - m_on)) / (m_off / (1 - m_off)), np.exp(-b), rtol=1e-12)


def test_monte_carlo_attention_stealing_and_its_repair(oracle):
    # Additive uniform key noise (Eq. 5-6): averaged over draws the cached mass is inflated
    # (Jensen bias, Eq. 8-9) and the corrected mass returns to the clean value (Eq. 11).
    rng = np.random.default_rng(25)
    d, m, ns, nr = 64, 8, 24, 24
    sigma = 1 / math.sqrt(d)
    q = rng.standard_normal((m, d)) * 2.0
    k, v = rng.standard_normal((ns + nr, d)), rng.standard_normal((ns + nr, d))
    step = np.full((ns, 1), 1.5)
    _, p = textbook(q, k, v, sigma)
    clean = p[:, :ns].sum(1)
    # Z_R is noise-free, so the odds P_S/(1-P_S) = Z_S/Z_R are linear in the cached partition sum.
    odds = lambda mass: mass / (1 - mass)
    raw, fixed, exact = np.zeros(m), np.zeros(m), np.zeros(m)
    draws = 1500
    for _ in range(draws):
        kh = k[:ns] + rng.uniform(-0.75, 0.75, size=(ns, d))
        raw += odds(oracle.attention(q, kh, step, v[:ns], k[ns:], v[ns:], correction=0, rotate=False)[1])
        fixed += odds(oracle.attention(q, kh, step, v[:ns], k[ns:], v[ns:], correction=1, rotate=False)[1])
        exact += odds(oracle.attention(q, kh, step, v[:ns], k[ns:], v[ns:], correction=2, rotate=False)[1])
    raw, fixed, exact = raw / draws, fixed / draws, exact / draws
    clean = odds(clean)
    assert np.all(raw > 1.1 * clean)                        # stealing: E[Z^_S] > Z_S
    assert np.all(np.abs(exact - clean) < 0.1 * (raw - clean))   # exact b: unbiased partition sum
    assert np.all(np.abs(fixed - clean) < 0.2 * (raw - clean))   # Taylor b: unbiased to second order
    assert np.all(fixed <= exact)                           # ... and never under-corrects


def test_whole_path_direction_on_the_tiny_config(oracle):
    # Soft expectation from the analysis section: on rotated INT2 keys the cached mass is inflated
    # relative to unquantized keys, much less at INT4, and the correction moves it back.
    from paper_2605_26266_amd import workloads as wl
    w = wl.WORKLOADS["tiny"]
    kc = np.concatenate([wl.chunk_kv(w, c)[0] for c in range(w.cached_chunks)])
    vc = np.concatenate([wl.chunk_kv(w, c)[1] for c in range(w.cached_chunks)])
    kr, vr = wl.chunk_kv(w, w.cached_chunks)
    q = wl.chunk_q(w)
    _, p = textbook(q[:, 0].astype(np.float64), np.concatenate([kc, kr])[:, 0].astype(np.float64),
                    np.concatenate([vc, vr])[:, 0].astype(np.float64), 1 / 8)
    clean = p[:, :kc.shape[0]].sum(1)
    _, raw2, _ = oracle.chunk_attention(q, kc, vc, kr, vr, 2, correction=0)
    _, fix2, _ = oracle.chunk_attention(q, kc, vc, kr, vr, 2, correction=1)
    _, raw4, _ = oracle.chunk_attention(q, kc, vc, kr, vr, 4, correction=0)
    steal2, steal4 = np.mean(raw2[0] - clean), np.mean(raw4[0] - clean)
    assert steal2 > 0 and steal2 > 3 * abs(steal4)
    assert abs(np.mean(fix2[0] - clean)) < steal2


def test_causal_mask_against_textbook_masked_softmax(oracle):
    """The causal option against an independent numpy statement of masked softmax attention (no
    quantization error: step 0), with and without a cached prefix, m == nr and m < nr."""
    rng = np.random.default_rng(21)
    d = 16
    for (m, ns, nr) in ((7, 5, 7), (4, 0, 9), (6, 3, 10)):
        q, kr, vr = rng.standard_normal((m, d)), rng.standard_normal((nr, d)), rng.standard_normal((nr, d))
        ks, vs = rng.standard_normal((ns, d)), rng.standard_normal((ns, d))
        out, mass = oracle.attention(q, ks, np.zeros((ns, 1)), vs, kr, vr, correction=1, rotate=False, causal=True)
        s = np.concatenate([q @ ks.T, q @ kr.T], axis=1) / np.sqrt(d)
        vis = np.ones((m, ns + nr), dtype=bool)
        for r in range(m):
            vis[r, ns + r + nr - m + 1:] = False
        s = np.where(vis, s, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        want = p @ np.concatenate([vs, vr])
        assert np.allclose(out, want, rtol=1e-12, atol=1e-12)
        assert np.allclose(mass, p[:, :ns].sum(axis=1), rtol=1e-12, atol=1e-14)
    # the last query row sees every key: identical to the unmasked call
    full, _ = oracle.attention(q, ks, np.zeros((ns, 1)), vs, kr, vr, correction=1, rotate=False)
    assert np.allclose(out[-1], full[-1], rtol=1e-13)


def test_grouped_query_heads_share_the_cache(oracle):
    rng = np.random.default_rng(4)
    from paper_2605_26266_amd import workloads as wl
    d, m, ns, nr = 64, 5, 40, 6
    q = wl.round_to_bf16(rng.standard_normal((m, 6, d)).astype(np.float32))
    kc, vc = (wl.round_to_bf16(rng.standard_normal((ns, 2, d)).astype(np.float32)) for _ in range(2))
    kr, vr = (wl.round_to_bf16(rng.standard_normal((nr, 2, d)).astype(np.float32)) for _ in range(2))
    out, mass, quant = oracle.chunk_attention(q, kc, vc, kr, vr, 2, 1)
    assert len(quant) == 2 and out.shape == (m, 6, d) and mass.shape == (6, m)
    for h in range(6):
        o1, m1, _ = oracle.chunk_attention(q[:, h:h + 1], kc[:, h // 3:h // 3 + 1], vc[:, h // 3:h // 3 + 1],
                                           kr[:, h // 3:h // 3 + 1], vr[:, h // 3:h // 3 + 1], 2, 1)
        assert np.array_equal(o1[:, 0], out[:, h]) and np.array_equal(m1[0], mass[h])


def test_randomised_rotation_against_dense_matrices(oracle):
    """Sign vector of the randomised Hadamard rotation: the cache basis is x -> Hn (signs * x).  With the
    cached keys / values rotated by an explicit dense matrix here and no quantization error (step 0), the
    result must be textbook attention in the original basis: a sign dropped on the query, on the output,
    or applied after the Hadamard matrix instead of before it breaks the equality."""
    rng = np.random.default_rng(33)
    d, m, ns, nr = 32, 6, 11, 4
    signs = np.where(rng.random(d) < 0.5, -1.0, 1.0)
    assert 0 < (signs < 0).sum() < d
    rot = np.diag(signs) @ (sylvester(d) / np.sqrt(d))          # row vector x -> x @ rot
    q, ks, vs = rng.standard_normal((m, d)), rng.standard_normal((ns, d)), rng.standard_normal((ns, d))
    kr, vr = rng.standard_normal((nr, d)), rng.standard_normal((nr, d))
    out, mass = oracle.attention(q, ks @ rot, np.zeros((ns, 1)), vs @ rot, kr, vr, correction=1, signs=signs)
    p = softmax(np.concatenate([q @ ks.T, q @ kr.T], axis=1) / np.sqrt(d), axis=1)
    assert np.allclose(out, p @ np.concatenate([vs, vr]), rtol=1e-11, atol=1e-12)
    assert np.allclose(mass, p[:, :ns].sum(axis=1), rtol=1e-12)
    # without the signs the same call is wrong (the pin above is not vacuous)
    bad, _ = oracle.attention(q, ks @ rot, np.zeros((ns, 1)), vs @ rot, kr, vr, correction=1)
    assert not np.allclose(bad, out, atol=1e-3)


def test_randomised_rotation_in_the_quantizer(oracle):
    """Codes written with a sign vector decode to within half a step of the densely rotated input, per
    rotated channel, and un-rotate to the input within the same bound times sqrt(d)."""
    rng = np.random.default_rng(34)
    d, rows = 64, 9
    signs = np.where(rng.random(d) < 0.5, -1.0, 1.0)
    rot = np.diag(signs) @ (sylvester(d) / np.sqrt(d))
    x = rng.standard_normal((rows, d)) * np.exp(rng.standard_normal((1, d)))     # uneven channels
    for bits in (2, 4):
        codes, scale, zero = oracle.quantize(x, bits, signs=signs)
        y = x @ rot
        yhat = (codes.astype(np.float64) - zero.astype(np.float64)) * scale.astype(np.float64)
        assert np.all(np.abs(yhat - y) <= 0.5 * scale.astype(np.float64) * (1 + 1e-6) + 1e-9)
        assert np.all(np.abs(yhat @ rot.T - x).max(axis=1) <= 0.5 * scale[:, 0] * np.sqrt(d) * (1 + 1e-6))
        plain, _, _ = oracle.quantize(x, bits)
        assert not np.array_equal(plain, codes)
    # all-plus signs are the plain rotation, bit for bit
    a = oracle.quantize(x, 2, signs=np.ones(d))
    b = oracle.quantize(x, 2)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
