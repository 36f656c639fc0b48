"""Pins for the oracle's attention-level diagnostics (CPU only): attention-stealing masses, the
Jensen-Shannon divergence between quantized and unquantized attention weights, and the output MSE.

Expectations come from scipy / numpy statements of the definitions on explicitly built probability
vectors, from special cases with a known value, and from the direction of the effects that the paper
reports for INT2 -- never from a second call of the routine under test.
"""
import math

import numpy as np
import pytest
from scipy.spatial.distance import jensenshannon
from scipy.special import softmax


def sylvester(d):
    h = np.array([[1.0]])
    while h.shape[0] < d:
        h = np.kron(np.array([[1.0, 1.0], [1.0, -1.0]]), h)
    return h


def test_against_scipy_on_explicit_distributions(oracle):
    """No rotation: the caller's k^ is used as is, so both probability rows can be written with numpy."""
    rng = np.random.default_rng(5)
    d, m, ns, nr = 16, 7, 13, 5
    q = rng.standard_normal((m, d))
    kref, vref = rng.standard_normal((ns, d)), rng.standard_normal((ns, d))
    khat = kref + 0.3 * rng.uniform(-0.5, 0.5, (ns, d))
    vhat = vref + 0.3 * rng.uniform(-0.5, 0.5, (ns, d))
    kr, vr = rng.standard_normal((nr, d)), rng.standard_normal((nr, d))
    step = rng.uniform(0.2, 0.6, (ns, 1))
    for correction in (0, 1):
        diag = oracle.diagnostics(q, khat, step, vhat, kref, vref, kr, vr, correction=correction, rotate=False)
        s_ref = np.concatenate([q @ kref.T, q @ kr.T], axis=1) / math.sqrt(d)
        b = correction * step[:, 0][None, :] ** 2 * (q ** 2).sum(axis=1)[:, None] / (24 * d)
        s_hat = np.concatenate([q @ khat.T / math.sqrt(d) - b, q @ kr.T / math.sqrt(d)], axis=1)
        p, ph = softmax(s_ref, axis=1), softmax(s_hat, axis=1)
        assert np.allclose(diag[:, 0], p[:, :ns].sum(axis=1), rtol=1e-12)
        assert np.allclose(diag[:, 1], ph[:, :ns].sum(axis=1), rtol=1e-12)
        want_jsd = np.array([jensenshannon(p[r], ph[r]) ** 2 for r in range(m)])   # scipy returns the square root
        assert np.allclose(diag[:, 2], want_jsd, rtol=1e-9, atol=1e-15)
        o, oh = p @ np.concatenate([vref, vr]), ph @ np.concatenate([vhat, vr])
        assert np.allclose(diag[:, 3], ((oh - o) ** 2).mean(axis=1), rtol=1e-11)


def test_rotated_basis_and_signs_against_dense_matrices(oracle):
    rng = np.random.default_rng(6)
    d, m, ns, nr = 32, 4, 9, 6
    signs = np.where(rng.random(d) < 0.5, -1.0, 1.0)
    rot = np.diag(signs) @ (sylvester(d) / math.sqrt(d))
    q, kref, vref = rng.standard_normal((m, d)), rng.standard_normal((ns, d)), rng.standard_normal((ns, d))
    kr, vr = rng.standard_normal((nr, d)), rng.standard_normal((nr, d))
    khat_rot = kref @ rot + 0.2 * rng.uniform(-0.5, 0.5, (ns, d))     # noise added in the rotated basis
    vhat_rot = vref @ rot + 0.2 * rng.uniform(-0.5, 0.5, (ns, d))
    diag = oracle.diagnostics(q, khat_rot, np.zeros((ns, 1)), vhat_rot, kref, vref, kr, vr, correction=1, signs=signs)
    p = softmax(np.concatenate([q @ kref.T, q @ kr.T], axis=1) / math.sqrt(d), axis=1)
    ph = softmax(np.concatenate([q @ (khat_rot @ rot.T).T, q @ kr.T], axis=1) / math.sqrt(d), axis=1)
    assert np.allclose(diag[:, 1], ph[:, :ns].sum(axis=1), rtol=1e-11)
    assert np.allclose(diag[:, 2], [jensenshannon(p[r], ph[r]) ** 2 for r in range(m)], rtol=1e-8, atol=1e-15)
    o, oh = p @ np.concatenate([vref, vr]), ph @ np.concatenate([vhat_rot @ rot.T, vr])
    assert np.allclose(diag[:, 3], ((oh - o) ** 2).mean(axis=1), rtol=1e-10)


def test_special_cases(oracle):
    rng = np.random.default_rng(7)
    d, m, ns, nr = 16, 3, 6, 4
    q, k, v = rng.standard_normal((m, d)), rng.standard_normal((ns, d)), rng.standard_normal((ns, d))
    kr, vr = rng.standard_normal((nr, d)), rng.standard_normal((nr, d))
    # identical caches, step 0: nothing differs
    diag = oracle.diagnostics(q, k, np.zeros((ns, 1)), v, k, v, kr, vr, rotate=False)
    assert np.array_equal(diag[:, 0], diag[:, 1]) and np.all(diag[:, 2] == 0.0) and np.all(diag[:, 3] == 0.0)
    # a uniform shift of all cached scores by -c moves mass but not the within-block shape:
    # one cached key, one current key, shift c  ->  closed forms for P^_S and the two-point JSD
    q1, k1, kr1 = np.ones((1, d)), np.zeros((1, d)), np.zeros((1, d))
    v1, vr1 = np.ones((1, d)), -np.ones((1, d))
    step = np.array([[2.0]])
    c = (1.0 / d) * 4.0 * d / 24.0                     # sigma^2 step^2 ||q||^2 / 24 with sigma = 1/sqrt(d)
    diag = oracle.diagnostics(q1, k1, step, v1, k1, v1, kr1, vr1, correction=1, rotate=False)
    ph = 1.0 / (1.0 + math.exp(c))
    assert diag[0, 0] == pytest.approx(0.5, rel=1e-14) and diag[0, 1] == pytest.approx(ph, rel=1e-13)
    mix = 0.5 * (0.5 + ph)
    jsd = 0.5 * (0.5 * math.log(0.5 / mix) + 0.5 * math.log(0.5 / (1 - mix))) \
        + 0.5 * (ph * math.log(ph / mix) + (1 - ph) * math.log((1 - ph) / (1 - mix)))
    assert diag[0, 2] == pytest.approx(jsd, rel=1e-10)
    assert diag[0, 3] == pytest.approx((2 * ph - 1.0) ** 2, rel=1e-12)     # o = 0, o^ = ph - (1 - ph) per channel
    # disjoint supports reach the upper bound log 2
    big = 60.0 * math.sqrt(d)
    kq = np.concatenate([np.full((1, d), big / d), np.zeros((1, d))])      # reference: all mass on cached key 0
    kh = np.concatenate([np.zeros((1, d)), np.full((1, d), big / d)])      # quantized: all mass on cached key 1
    diag = oracle.diagnostics(q1, kh, np.zeros((2, 1)), np.zeros((2, d)), kq, np.zeros((2, d)), kr1, vr1,
                              correction=0, rotate=False)
    assert diag[0, 2] == pytest.approx(math.log(2.0), rel=1e-12)


def test_direction_of_the_effects_at_int2(oracle):
    """What the paper reports for 2-bit keys (attention stealing and its repair; appendices on JSD and output
    MSE): without the correction the cached block gains mass on average, the correction shrinks
    that shift and lowers both the divergence and the output error."""
    from paper_2605_26266_amd import workloads as wl
    w = wl.WORKLOADS["small"]
    heads = range(2)
    kc, vc = wl.chunk_kv(w, 0, heads=heads, n_tokens=512)
    kr, vr = wl.chunk_kv(w, 1, heads=heads, n_tokens=256)
    q = wl.chunk_q(w, heads=heads)[:48]
    off = oracle.chunk_diagnostics(q, kc, vc, kr, vr, 2, correction=0)
    on = oracle.chunk_diagnostics(q, kc, vc, kr, vr, 2, correction=1)
    assert np.array_equal(off[:, :, 0], on[:, :, 0])                       # the reference side does not move
    steal_off, steal_on = (off[:, :, 1] - off[:, :, 0]).mean(), (on[:, :, 1] - on[:, :, 0]).mean()
    assert steal_off > 0.0
    assert abs(steal_on) < 0.6 * steal_off      # the mean shift shrinks (the ratio Z_S / Z is not linear in Z_S, so it need not vanish)
    assert on[:, :, 2].mean() < off[:, :, 2].mean()
    assert on[:, :, 3].mean() < off[:, :, 3].mean()
    assert np.all(off[:, :, 2] <= math.log(2.0)) and np.all(off[:, :, 2] >= 0.0)
