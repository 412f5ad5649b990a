"""Pins for the oracle's mask-based MVDR (Eq. 6-9 of the paper and the reference-channel reading)."""

import numpy as np

from oracle import gss_oracle as o


def _cn(rng, shape):
    return (rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) / np.sqrt(2)


def _hpd(rng, F, D):
    A = _cn(rng, (F, D, D))
    return A @ A.conj().swapaxes(-1, -2) + 0.2 * np.eye(D)


def test_covariances_by_loops_and_sum_rule():
    rng = np.random.default_rng(0)
    F, T, D, K = 2, 7, 3, 3
    Y = _cn(rng, (F, T, D))
    g = rng.random((K, F, T))
    g /= g.sum(0, keepdims=True)
    g[:, :, 3] = 0.0                                   # a frame with no active class
    pk, pb = o.masked_covariances(Y, g, 1)
    for f in range(F):
        ak = np.zeros((D, D), complex)
        ab = np.zeros((D, D), complex)
        for t in range(T):
            outer = np.array([[Y[f, t, i] * np.conj(Y[f, t, j]) for j in range(D)] for i in range(D)])
            ak += g[1, f, t] * outer
            ab += (g[0, f, t] + g[2, f, t]) * outer
        assert np.allclose(pk[f], ak) and np.allclose(pb[f], ab)
    # Phi_k + Phi_bg = sum over frames with an active class of y y^H
    keep = np.ones(T, bool)
    keep[3] = False
    tot = np.einsum("fti,ftj->fij", Y[:, keep], Y[:, keep].conj())
    assert np.allclose(pk + pb, tot)
    assert np.allclose(pk, pk.conj().swapaxes(-1, -2))
    assert np.linalg.eigvalsh(pk).min() > -1e-12 and np.linalg.eigvalsh(pb).min() > -1e-12


def test_distortionless_for_rank1_target():
    """Phi_k = s^2 v v^H, any PD Phi_bg: column r of H equals Phi_bg^-1 v conj(v_r) / (v^H Phi_bg^-1 v),
    the classical steering-vector MVDR, so h_r^H v = v_r."""
    rng = np.random.default_rng(1)
    F, D = 4, 5
    v = _cn(rng, (F, D))
    phi_k = 2.7 * np.einsum("fi,fj->fij", v, v.conj())
    phi_bg = _hpd(rng, F, D)
    H = o.souden_filters(phi_k, phi_bg)
    for f in range(F):
        lam, V = np.linalg.eigh(phi_bg[f])
        binv_v = V @ ((V.conj().T @ v[f]) / lam)
        for r in range(D):
            closed = binv_v * np.conj(v[f, r]) / np.vdot(v[f], binv_v)
            assert np.allclose(H[f, :, r], closed, atol=1e-10)
            assert abs(np.vdot(H[f, :, r], v[f]) - v[f, r]) < 1e-10


def test_identity_background_closed_form_and_loading():
    rng = np.random.default_rng(2)
    F, D = 3, 4
    v = _cn(rng, (F, D))
    phi_k = np.einsum("fi,fj->fij", v, v.conj())
    eye = np.broadcast_to(np.eye(D, dtype=complex), (F, D, D)).copy()
    H = o.souden_filters(phi_k, o.load_background(eye))
    for r in range(D):
        assert np.allclose(H[:, :, r], v * np.conj(v[:, r:r + 1]) / np.sum(np.abs(v) ** 2, -1, keepdims=True), atol=1e-12)
    # loading adds DELTA_BF * tr/D to the diagonal only
    pb = _hpd(rng, F, D)
    lo = o.load_background(pb)
    assert np.allclose(lo - pb, (o.DELTA_BF * np.trace(pb, axis1=1, axis2=2).real / D)[:, None, None] * np.eye(D))


def test_filter_scale_invariance_and_unit_trace():
    rng = np.random.default_rng(3)
    F, D = 3, 4
    pk, pb = _hpd(rng, F, D), _hpd(rng, F, D)
    H = o.souden_filters(pk, pb)
    H2 = o.souden_filters(7.0 * pk, 0.03 * pb)
    assert np.allclose(H, H2, atol=1e-12)               # so the 1/T of Eq. (6), (7) cancels
    assert np.allclose(np.einsum("frr->f", H), 1.0)     # G / tr G has unit trace


def test_filter_D2_adjugate_formula():
    rng = np.random.default_rng(4)
    pk, pb = _hpd(rng, 5, 2), _hpd(rng, 5, 2)
    H = o.souden_filters(pk, pb)
    for f in range(5):
        a, b, c, d = pb[f, 0, 0], pb[f, 0, 1], pb[f, 1, 0], pb[f, 1, 1]
        inv = np.array([[d, -b], [-c, a]]) / (a * d - b * c)
        G = inv @ pk[f]
        assert np.allclose(H[f], G / np.trace(G).real, atol=1e-12)


def test_zero_target_gives_zero_output():
    rng = np.random.default_rng(5)
    Y = _cn(rng, (2, 9, 3))
    g = np.zeros((2, 2, 9))
    g[1] = 1.0
    X, ref, h = o.mvdr(Y, g, 0)
    assert np.all(X == 0) and np.all(h == 0) and ref == 0


def test_no_background_gives_zero_filter():
    """R7: a frequency whose background covariance is exactly zero (every frame belongs to the target with mask 1,
    or the bin is silent) has no solution of Eq. (8): the filter and the output are zero there, and the other
    frequencies are what they are without that bin."""
    rng = np.random.default_rng(11)
    F, T, D, K = 3, 40, 4, 2
    Y = (rng.standard_normal((F, T, D)) + 1j * rng.standard_normal((F, T, D))) / np.sqrt(2)
    gamma = rng.random((K, F, T))
    gamma /= gamma.sum(axis=0, keepdims=True)
    gamma[0, 1] = 1.0
    gamma[1, 1] = 0.0                                   # bin 1: all of it is target
    X, ref, h = o.mvdr(Y, gamma, 0)
    assert np.all(h[1] == 0) and np.all(X[1] == 0)
    keep = [0, 2]
    X2, ref2, h2 = o.mvdr(Y[keep], gamma[:, keep], 0, ref)
    assert np.allclose(X[keep], X2, rtol=0, atol=1e-12) and np.allclose(h[keep], h2, rtol=0, atol=1e-12)
    # and a single frame with the target's mask at one: nothing but zeros, no exception
    X1, _, h1 = o.mvdr(Y[:, :1], np.stack([np.ones((F, 1)), np.zeros((F, 1))]), 0)
    assert np.all(X1 == 0) and np.all(h1 == 0)


def test_reference_channel_brute_force_and_dead_mic():
    rng = np.random.default_rng(6)
    F, T, D = 6, 400, 4
    v = _cn(rng, (F, D))
    v[:, 2] = 0.0                                        # microphone 2 does not pick up the target at all
    u = _cn(rng, (F, D))
    lab = rng.random((F, T)) < 0.5
    Y = np.where(lab[..., None], v[:, None, :] * _cn(rng, (F, T, 1)) * 2.0, u[:, None, :] * _cn(rng, (F, T, 1)))
    Y = Y + 0.05 * _cn(rng, (F, T, D))
    g = np.stack([lab.astype(float), 1.0 - lab])
    X, ref, h = o.mvdr(Y, g, 0)
    assert ref != 2
    pk, pb = o.masked_covariances(Y, g, 0)
    pbl = o.load_background(pb)
    H = o.souden_filters(pk, pbl)
    scores = []
    for r in range(D):
        num = den = 0.0
        for f in range(F):
            hr = H[f, :, r]
            num += np.vdot(hr, pk[f] @ hr).real
            den += np.vdot(hr, pbl[f] @ hr).real
        scores.append(num / den)
    assert ref == int(np.argmax(scores))
    assert np.allclose(scores, o.reference_channel_scores(H, pk, pbl))
    # forcing the reference is honoured, and the output is h^H y (Eq. 9) by loops
    X1, ref1, h1 = o.mvdr(Y, g, 0, ref=1)
    assert ref1 == 1 and np.allclose(h1, H[:, :, 1])
    for f in (0, 3):
        for t in (0, 17):
            assert abs(X1[f, t] - sum(np.conj(h1[f, d]) * Y[f, t, d] for d in range(D))) < 1e-12


def test_mvdr_suppresses_interferer():
    """Oracle masks for two directional sources: the output must keep the target's reference-channel
    image and attenuate the interferer by a large factor."""
    rng = np.random.default_rng(7)
    F, T, D = 4, 600, 5
    v, u = _cn(rng, (F, D)), _cn(rng, (F, D))
    lab = rng.random((F, T)) < 0.5
    s = _cn(rng, (F, T))
    Y = np.where(lab[..., None], v[:, None, :] * s[..., None], u[:, None, :] * s[..., None]) + 0.01 * _cn(rng, (F, T, D))
    g = np.stack([lab.astype(float), 1.0 - lab])
    X, ref, h = o.mvdr(Y, g, 0, ref=0)
    tgt = np.abs(X[lab] - (v[:, 0][:, None] * s)[lab])
    assert np.sqrt(np.mean(tgt ** 2)) < 0.05 * np.sqrt(np.mean(np.abs((v[:, 0][:, None] * s)[lab]) ** 2))
    assert np.sqrt(np.mean(np.abs(X[~lab]) ** 2)) < 0.05 * np.sqrt(np.mean(np.abs((u[:, 0][:, None] * s)[~lab]) ** 2))


def test_batch_wrapper():
    rng = np.random.default_rng(8)
    Y = _cn(rng, (2, 3, 12, 2)).astype(np.complex64)
    g = rng.random((2, 2, 3, 12))
    g /= g.sum(1, keepdims=True)
    X, ref = o.mvdr_batch(Y, g, np.array([12, 7]), np.array([0, 1]), np.array([-1, 1]))
    X1, r1, _ = o.mvdr(Y[1, :, :7], g[1, :, :, :7], 1, 1)
    assert np.allclose(X[1, :, :7], X1) and np.all(X[1, :, 7:] == 0) and ref[1] == 1


# ---------------------------------------------------------------- reference channel per frequency (R16)
def test_per_frequency_reference_by_loops():
    """The per-frequency choice written out with loops; where every frequency prefers the same channel it is
    the per-segment choice; a fixed reference channel is used as given."""
    rng = np.random.default_rng(21)
    F, T, D, K = 6, 40, 4, 3
    Y = _cn(rng, (F, T, D))
    g = rng.random((K, F, T))
    g /= g.sum(0, keepdims=True)
    X, ref_f, h = o.mvdr_per_frequency_ref(Y, g, 1)
    pk, pb = o.masked_covariances(Y, g, 1)
    pbl = o.load_background(pb)
    H = o.souden_filters(pk, pbl)
    for f in range(F):
        best, best_score = 0, -1.0
        for r in range(D):
            hr = H[f, :, r]
            sc = np.vdot(hr, pk[f] @ hr).real / np.vdot(hr, pbl[f] @ hr).real
            if sc > best_score:
                best, best_score = r, sc
        assert ref_f[f] == best
        assert np.allclose(h[f], H[f, :, best])
        for t in range(T):
            assert abs(X[f, t] - np.vdot(H[f, :, best], Y[f, t])) < 1e-12
    # forcing every frequency to the per-segment channel reproduces the per-segment beamformer
    Xs, ref_s, _ = o.mvdr(Y, g, 1)
    Xf, rf, _ = o.mvdr_per_frequency_ref(Y, g, 1, ref=np.full(F, ref_s))
    assert np.all(rf == ref_s) and np.allclose(Xf, Xs)
    # mixed: negative entries are chosen, the others kept
    given = np.array([2, -1, 0, -1, 3, 1])
    _, rmix, _ = o.mvdr_per_frequency_ref(Y, g, 1, ref=given)
    assert np.all(rmix[given >= 0] == given[given >= 0]) and np.all(rmix[given < 0] == ref_f[given < 0])


def test_per_frequency_reference_follows_a_microphone_that_is_dead_in_a_band():
    """Two-source toy: microphone 0 hears the target in the lower half of the band only, microphone 1 in the
    upper half only.  One channel per segment has to give up half of the band; one per frequency picks the
    live microphone in each half and is distortionless there (h^H v = v_ref)."""
    rng = np.random.default_rng(22)
    F, T, D = 8, 400, 3
    v = _cn(rng, (F, D))
    v[:4, 1] = 0.0                                   # mic 1 dead below, mic 0 dead above
    v[4:, 0] = 0.0
    v[:, 2] *= 0.05                                  # mic 2 hears the target only faintly
    s = _cn(rng, (F, T))
    n = 0.3 * _cn(rng, (F, T, D))
    Y = s[:, :, None] * v[:, None, :] + n
    g = np.zeros((2, F, T))
    g[0] = 0.9
    g[1] = 0.1
    _, ref_f, h = o.mvdr_per_frequency_ref(Y, g, 0)
    assert np.all(ref_f[:4] == 0) and np.all(ref_f[4:] == 1)
    phi_k = np.einsum("fi,fj->fij", v, v.conj())
    H = o.souden_filters(phi_k, o.load_background(np.einsum("fti,ftj->fij", n, n.conj())))
    for f in range(F):
        r = ref_f[f]
        assert abs(np.vdot(H[f, :, r], v[f]) - v[f, r]) < 1e-9
