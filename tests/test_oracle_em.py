"""Pins for the oracle's cACGMM EM (Eq. 2-5 of the paper and the M-step reading).

None of these tests re-types the oracle's own formula or re-calls its library
routine: each one checks against a closed form, an invariant of the model, a
different numerical route (eigendecomposition, explicit 2x2 algebra, Python
loops) or a statistical limit.
"""

import math

import numpy as np
import pytest

from oracle import gss_oracle as o


def _cn(rng, shape):
    return (rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) / np.sqrt(2)


def _random_hpd(rng, shape, D):
    A = _cn(rng, shape + (D, D))
    return A @ A.conj().swapaxes(-1, -2) + 0.1 * np.eye(D)


def _toy(rng, F=5, T=60, D=3, K=3):
    Y = _cn(rng, (F, T, D)) * np.exp(rng.standard_normal((F, T, 1)))
    act = (rng.random((K, T)) < 0.6).astype(np.uint8)
    act[K - 1] = 1
    return Y, act


# ---------------------------------------------------------------- Eq. (2)
def test_unit_norm_and_zero_frame():
    rng = np.random.default_rng(0)
    Y = _cn(rng, (4, 7, 5)) * 1e3
    Y[1, 2] = 0.0
    Yn = o.unit_normalise(Y)
    n = np.linalg.norm(Yn, axis=-1)
    assert np.allclose(np.delete(n.ravel(), 1 * 7 + 2), 1.0, atol=1e-14)
    assert np.all(Yn[1, 2] == 0.0)
    # direction is preserved: Yn is a positive multiple of Y
    r = Yn[0, 0] / Y[0, 0]
    assert np.allclose(r.imag, 0, atol=1e-18) and np.all(r.real > 0) and np.allclose(r, r[0])


def test_masks_invariant_to_per_bin_complex_scaling():
    rng = np.random.default_rng(1)
    Y, act = _toy(rng)
    c = _cn(rng, Y.shape[:2] + (1,)) * 10.0
    g1 = o.cacgmm_em(Y, act, 4)
    g2 = o.cacgmm_em(Y * c, act, 4)
    assert np.max(np.abs(g1 - g2)) < 1e-10


# ---------------------------------------------------------------- Eq. (4): quadratic form and log-det
def test_quadratic_form_logdet_vs_eigendecomposition_D2_and_closed_form():
    rng = np.random.default_rng(2)
    F, K, T, D = 6, 3, 11, 2
    B = _random_hpd(rng, (F, K), D)
    Yn = o.unit_normalise(_cn(rng, (F, T, D)))
    q, logdet = o.quadratic_forms(Yn, B)
    for f in range(F):
        for k in range(K):
            lam, V = np.linalg.eigh(B[f, k])
            a, b, c, d = B[f, k, 0, 0], B[f, k, 0, 1], B[f, k, 1, 0], B[f, k, 1, 1]
            det = (a * d - b * c).real
            assert abs(logdet[f, k] - math.log(det)) < 1e-12
            assert abs(logdet[f, k] - np.sum(np.log(lam))) < 1e-12
            inv = np.array([[d, -b], [-c, a]]) / (a * d - b * c)      # adjugate formula
            for t in range(T):
                y = Yn[f, t]
                q_eig = sum(abs(np.vdot(V[:, i], y)) ** 2 / lam[i] for i in range(D))
                q_adj = np.vdot(y, inv @ y).real
                assert abs(q[k, f, t] - q_eig) < 1e-11 * max(1, q_eig)
                assert abs(q[k, f, t] - q_adj) < 1e-11 * max(1, q_adj)


def test_quadratic_form_vs_eigendecomposition_D5():
    rng = np.random.default_rng(3)
    F, K, T, D = 3, 2, 9, 5
    B = _random_hpd(rng, (F, K), D)
    Yn = o.unit_normalise(_cn(rng, (F, T, D)))
    q, logdet = o.quadratic_forms(Yn, B)
    lam, V = np.linalg.eigh(B)
    proj = np.einsum("fkdi,ftd->kfti", V.conj(), Yn)
    q_eig = np.sum(np.abs(proj) ** 2 / lam.transpose(1, 0, 2)[:, :, None, :], axis=-1)
    assert np.allclose(q, q_eig, rtol=1e-11)
    assert np.allclose(logdet, np.log(lam).sum(-1), atol=1e-11)


def test_quadratic_form_clamped_on_zero_frame():
    B = np.eye(3, dtype=complex)[None, None]
    Yn = np.zeros((1, 2, 3), dtype=complex)
    q, _ = o.quadratic_forms(Yn, B)
    assert np.all(q == o.EPS_Q)


# ---------------------------------------------------------------- Eq. (3), (5): posteriors
def test_posteriors_sum_to_one_and_respect_activity():
    rng = np.random.default_rng(4)
    Y, act = _toy(rng, K=4)
    act[3] = (rng.random(act.shape[1]) < 0.7)          # allow frames with no active class
    act[:, 5] = 0
    g = o.cacgmm_em(Y, act, 3)
    any_active = act.any(axis=0)
    s = g.sum(axis=0)
    assert np.allclose(s[:, any_active], 1.0, atol=1e-12)
    assert np.all(s[:, ~any_active] == 0.0)
    assert np.all(g[np.broadcast_to((act == 0)[:, None, :], g.shape)] == 0.0)
    assert np.all(g >= 0) and np.all(g <= 1 + 1e-15)


def test_single_active_class_gives_one():
    rng = np.random.default_rng(5)
    Y, act = _toy(rng, K=3)
    act[:] = 0
    act[2] = 1
    act[0, :20] = 1
    g = o.cacgmm_em(Y, act, 5)
    assert np.all(g[2, :, 20:] == 1.0)
    # K = 1: every mask is one for any number of iterations
    g1 = o.cacgmm_em(Y, np.ones((1, Y.shape[1]), np.uint8), 7)
    assert np.all(g1 == 1.0)


def test_e_step_matches_direct_density_evaluation():
    """gamma_k = pi_tfk A(y;B_k) / sum_k' pi_tfk' A(y;B_k') evaluated literally from Eq. (3)-(5) with loops,
    including the printed constant of Eq. (4), which must cancel."""
    rng = np.random.default_rng(6)
    F, T, D, K = 2, 8, 3, 3
    B = _random_hpd(rng, (F, K), D)
    pi = rng.random((F, K)) + 0.1
    pi /= pi.sum(1, keepdims=True)
    act = np.array([[1] * 8, [1, 0, 1, 0, 1, 1, 0, 1], [0, 1, 1, 0, 0, 1, 1, 1]], dtype=np.uint8)
    Yn = o.unit_normalise(_cn(rng, (F, T, D)))
    g, _ = o.e_step(Yn, B, pi, act)
    const = (1.0 / (2 * math.pi)) ** D * math.factorial(D - 1)
    for f in range(F):
        for t in range(T):
            y = Yn[f, t]
            dens = []
            for k in range(K):
                lam, V = np.linalg.eigh(B[f, k])
                qk = sum(abs(np.vdot(V[:, i], y)) ** 2 / lam[i] for i in range(D))
                dens.append(const / np.prod(lam) * qk ** (-D))
            w = np.array([pi[f, k] * act[k, t] for k in range(K)])
            w = w / w.sum()
            post = w * np.array(dens)
            post /= post.sum()
            assert np.allclose(g[:, f, t], post, atol=1e-12)


def test_density_scale_invariance_in_B():
    """A(y; cB) = A(y; B): rescaling any B between the M- and the E-step must not move gamma."""
    rng = np.random.default_rng(7)
    Y, act = _toy(rng, K=3)
    Yn = o.unit_normalise(Y)
    F, T, D = Yn.shape
    g0 = o.initial_posteriors(act, F)
    B, pi, _ = o.m_step(Yn, g0, np.ones_like(g0))
    g1, _ = o.e_step(Yn, B, pi, act)
    B2 = B.copy()
    B2[:, 1] *= 37.5
    B2[:, 0] *= 0.01
    g2, _ = o.e_step(Yn, B2, pi, act)
    assert np.max(np.abs(g1 - g2)) < 1e-10


# ---------------------------------------------------------------- M-step
def test_m_step_hermitian_positive_definite_and_trace():
    rng = np.random.default_rng(8)
    Y, act = _toy(rng, F=4, T=40, D=4, K=3)
    Yn = o.unit_normalise(Y)
    g = o.initial_posteriors(act, 4)
    B, pi, N = o.m_step(Yn, g, np.ones_like(g))
    assert np.max(np.abs(B - B.conj().swapaxes(-1, -2))) == 0.0
    lam = np.linalg.eigvalsh(B)
    assert lam.min() >= o.DELTA * (1 - 1e-9)
    assert np.allclose(np.trace(B, axis1=-2, axis2=-1).real, 4 * (1 + o.DELTA), rtol=1e-12)
    assert np.allclose(pi.sum(1), 1.0)
    assert np.allclose(N, g.sum(axis=2).T)


def test_m_step_trace_identity():
    """tr(B_old^-1 * D * R / N) = D for any gamma when q = y^H B_old^-1 y (no reference needed)."""
    rng = np.random.default_rng(9)
    F, T, D, K = 3, 50, 4, 3
    Yn = o.unit_normalise(_cn(rng, (F, T, D)))
    B_old = _random_hpd(rng, (F, K), D)
    gamma = rng.random((K, F, T))
    q, _ = o.quadratic_forms(Yn, B_old)
    R, N = o.weighted_scatter(Yn, gamma, q)
    lam, V = np.linalg.eigh(B_old)
    Binv = np.einsum("fkij,fkj,fklj->fkil", V, 1.0 / lam, V.conj())
    tr = np.einsum("fkij,fkji->fk", Binv, D * R / N[:, :, None, None])
    assert np.allclose(tr.real, D, rtol=1e-11) and np.allclose(tr.imag, 0, atol=1e-11)


def test_m_step_scatter_by_loops():
    rng = np.random.default_rng(10)
    F, T, D, K = 2, 6, 3, 2
    Yn = o.unit_normalise(_cn(rng, (F, T, D)))
    gamma = rng.random((K, F, T))
    q = rng.random((K, F, T)) + 0.5
    R, N = o.weighted_scatter(Yn, gamma, q)
    for f in range(F):
        for k in range(K):
            acc = np.zeros((D, D), complex)
            for t in range(T):
                for i in range(D):
                    for j in range(D):
                        acc[i, j] += gamma[k, f, t] / q[k, f, t] * Yn[f, t, i] * np.conj(Yn[f, t, j])
            assert np.allclose(R[f, k], acc, atol=1e-13)
            assert abs(N[f, k] - sum(gamma[k, f])) < 1e-12


def test_dead_class_gets_identity():
    rng = np.random.default_rng(11)
    Y, act = _toy(rng, F=2, T=30, D=3, K=3)
    act[1] = 0
    Yn = o.unit_normalise(Y)
    g = o.initial_posteriors(act, 2)
    B, pi, N = o.m_step(Yn, g, np.ones_like(g))
    assert np.allclose(B[:, 1], (1 + o.DELTA) * np.eye(3))
    assert np.all(pi[:, 1] == 0)
    g2 = o.cacgmm_em(Y, act, 4)
    assert np.all(g2[1] == 0) and np.all(np.isfinite(g2))


def test_single_class_converges_to_shape_of_true_covariance():
    """K = 1 is the classical fixed-point (Tyler-type) scatter estimator: for y = z/|z|, z ~ CN(0, Sigma),
    B * D / tr B -> Sigma * D / tr Sigma as T grows (tolerance ~ 1/sqrt(T))."""
    rng = np.random.default_rng(12)
    D, T = 3, 40000
    A = _cn(rng, (D, D))
    Sigma = A @ A.conj().T + 0.3 * np.eye(D)
    L = np.linalg.cholesky(Sigma)
    z = (_cn(rng, (T, D)) @ L.T)[None]                              # [1, T, D], covariance Sigma
    g, B, pi = o.cacgmm_em(z, np.ones((1, T), np.uint8), 40, return_params=True)
    est = B[0, 0] - o.DELTA * np.eye(D)
    est = est * D / np.trace(est).real
    ref = Sigma * D / np.trace(Sigma).real
    assert np.max(np.abs(est - ref)) < 6.0 / math.sqrt(T) * np.max(np.abs(ref))


# ---------------------------------------------------------------- whole EM: equivariances
def test_em_equivariances():
    rng = np.random.default_rng(13)
    Y, act = _toy(rng, F=6, T=50, D=4, K=4)
    F, T, D = Y.shape
    g = o.cacgmm_em(Y, act, 5)
    # classes
    pk = rng.permutation(4)
    assert np.max(np.abs(o.cacgmm_em(Y, act[pk], 5) - g[pk])) < 1e-10
    # frames (no temporal model)
    pt = rng.permutation(T)
    assert np.max(np.abs(o.cacgmm_em(Y[:, pt], act[:, pt], 5) - g[:, :, pt])) < 1e-10
    # per-frequency unitary mixing of the channels
    U = np.linalg.qr(_cn(rng, (F, D, D)))[0]
    YU = np.einsum("fij,ftj->fti", U, Y)
    assert np.max(np.abs(o.cacgmm_em(YU, act, 5) - g)) < 1e-9
    # frequencies are independent
    sel = [4, 1]
    assert np.max(np.abs(o.cacgmm_em(Y[sel], act, 5) - g[:, sel])) < 1e-12
    # padded frames (zero activity) change nothing and come back as zeros
    Yp = np.concatenate([Y, _cn(rng, (F, 9, D))], axis=1)
    ap = np.concatenate([act, np.zeros((4, 9), np.uint8)], axis=1)
    gp = o.cacgmm_em(Yp, ap, 5)
    assert np.max(np.abs(gp[:, :, :T] - g)) < 1e-12 and np.all(gp[:, :, T:] == 0)


def test_batch_wrapper_pads_with_zeros():
    rng = np.random.default_rng(14)
    Y = _cn(rng, (2, 3, 20, 2)).astype(np.complex64)
    act = np.ones((2, 2, 20), np.uint8)
    act[:, 0, ::3] = 0
    T_len = np.array([20, 13], dtype=np.int32)
    g = o.cacgmm_em_batch(Y, act, T_len, 3)
    assert np.all(g[1, :, :, 13:] == 0)
    assert np.allclose(g[1, :, :, :13], o.cacgmm_em(Y[1, :, :13], act[1, :, :13], 3))
    assert np.allclose(g[0], o.cacgmm_em(Y[0], act[0], 3))


def test_likelihood_non_decreasing_uniform_weights():
    rng = np.random.default_rng(15)
    F, T, D, K = 3, 200, 3, 2
    v = _cn(rng, (K, F, D))
    lab = rng.integers(0, K, size=(F, T))
    Y = v[lab, np.arange(F)[:, None]] * _cn(rng, (F, T, 1)) + 0.3 * _cn(rng, (F, T, D))
    act = np.ones((K, T), np.uint8)
    Yn = o.unit_normalise(Y)
    gamma = o.initial_posteriors(act, F) + 0.05 * rng.random((K, F, T))   # break the symmetric start
    gamma /= gamma.sum(0, keepdims=True)
    q = np.ones_like(gamma)
    prev = -np.inf
    for _ in range(12):
        B, pi, _ = o.m_step(Yn, gamma, q, weight_mode=0)
        ll = o.log_likelihood(Yn, B, pi, act)
        assert ll >= prev - 1e-6 * abs(prev if np.isfinite(prev) else 1.0)
        prev = ll
        gamma, q = o.e_step(Yn, B, pi, act)


def test_recovers_generating_labels_with_guidance():
    """Two directional sources with disjoint-but-overlapping activity and a weak noise class: the class
    with the largest mask must be the generating source on (nearly) all source-dominated bins."""
    rng = np.random.default_rng(16)
    F, T, D = 8, 300, 4
    v = _cn(rng, (2, F, D))
    v /= np.linalg.norm(v, axis=-1, keepdims=True)
    act = np.zeros((3, T), np.uint8)
    act[0, :200] = 1
    act[1, 100:] = 1
    act[2] = 1
    lab = np.where(np.arange(T) < 100, 0, np.where(np.arange(T) >= 200, 1, rng.integers(0, 2, size=(F, T))))
    Y = v[lab, np.arange(F)[:, None]] * (3.0 * _cn(rng, (F, T, 1))) + 0.05 * _cn(rng, (F, T, D))
    g = o.cacgmm_em(Y, act, 15)
    est = g[:2].argmax(axis=0)
    assert np.mean(est == lab) > 0.97


def test_weight_modes_differ_and_validate():
    rng = np.random.default_rng(17)
    Y, act = _toy(rng)
    g1 = o.cacgmm_em(Y, act, 3, weight_mode=1)
    g0 = o.cacgmm_em(Y, act, 3, weight_mode=0)
    assert np.max(np.abs(g1 - g0)) > 1e-4
    with pytest.raises(ValueError):
        o.cacgmm_em(Y, act, 1, weight_mode=2)


def test_zero_iterations_returns_normalised_activity():
    rng = np.random.default_rng(18)
    Y, act = _toy(rng, K=3)
    g = o.cacgmm_em(Y, act, 0)
    cnt = np.maximum(act.sum(0), 1)
    assert np.allclose(g, np.broadcast_to((act / cnt)[:, None, :], g.shape))
