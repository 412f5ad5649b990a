"""Pins for the WPE oracle: checks against what the definition and the mathematics fix, none of which
re-types the oracle's own formulas (weighted least squares through a library QR/SVD solver, a scalar closed
form, the signal model that delayed linear prediction inverts, invariances, brute-force loops)."""

import numpy as np

from oracle import wpe_oracle as w
from paper_2212_05271_amd import synth


def _cn(rng, shape):
    return (rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) / np.sqrt(2)


def test_stacking_by_loops():
    rng = np.random.default_rng(0)
    T, D, L, delay = 9, 3, 4, 2
    y = _cn(rng, (T, D))
    yt = w.stack_delayed(y, L, delay)
    assert yt.shape == (T, D * L)
    for t in range(T):
        for tau in range(L):
            for d in range(D):
                src = t - delay - tau
                want = y[src, d] if src >= 0 else 0.0
                assert yt[t, tau * D + d] == want


def test_one_step_is_weighted_least_squares():
    """One iteration minimises sum_t |y_{t,d} - g_d^H ytilde_t|^2 / lambda_t: the library's lstsq on the
    row-scaled system must give the same prediction (loading 1e-10 is far below the comparison's level)."""
    rng = np.random.default_rng(1)
    T, D, L, delay = 300, 3, 4, 2
    y = _cn(rng, (T, D)) * (0.2 + rng.random((T, 1)))
    x = w.wpe_bin(y, L, delay, iters=1)
    lam = np.mean(np.abs(y) ** 2, axis=1)
    sw = 1.0 / np.sqrt(lam)
    yt = np.zeros((T, D * L), complex)
    for t in range(T):
        for tau in range(L):
            if t - delay - tau >= 0:
                yt[t, tau * D:(tau + 1) * D] = y[t - delay - tau]
    coef, *_ = np.linalg.lstsq(yt * sw[:, None], y * sw[:, None], rcond=None)
    want = y - yt @ coef
    assert np.abs(x - want).max() < 1e-8 * np.abs(y).max()


def test_single_channel_single_tap_closed_form():
    rng = np.random.default_rng(2)
    T, delay = 50, 3
    y = _cn(rng, (T, 1))
    lam = np.abs(y[:, 0]) ** 2
    lam = np.maximum(lam, 1e-10 * lam.max())
    num = sum(y[t - delay, 0] * np.conj(y[t, 0]) / lam[t] for t in range(delay, T))
    den = sum(abs(y[t - delay, 0]) ** 2 / lam[t] for t in range(delay, T))
    g = num / (den * (1 + 1e-10))
    want = y.copy()
    for t in range(delay, T):
        want[t, 0] = y[t, 0] - np.conj(g) * y[t - delay, 0]
    x = w.wpe_bin(y, taps=1, delay=delay, iters=1)
    assert np.abs(x - want).max() < 1e-12


def test_normal_equations_hold_after_the_last_iteration():
    """The residual is orthogonal (in the lambda-weighted sense) to every delayed observation."""
    rng = np.random.default_rng(3)
    T, D, L, delay = 400, 4, 5, 2
    y = _cn(rng, (T, D)) * (0.1 + rng.random((T, 1)))
    x2 = w.wpe_bin(y, L, delay, iters=2)
    x3 = w.wpe_bin(y, L, delay, iters=3)
    lam = w.variance(x2)                          # the weights the third iteration used
    yt = w.stack_delayed(y, L, delay)
    resid = (yt.T / lam) @ x3.conj()
    scale = np.abs((yt.T / lam) @ y.conj()).max()
    assert np.abs(resid).max() < 1e-7 * scale


def test_recovers_the_autoregressive_model():
    """On data that follow y_t = s_t + sum_tau A_tau y_{t-delay-tau} with a white-in-time dry signal, the
    output approaches s_t and G^H approaches [A_0 A_1 ...] (statistical error ~ sqrt(D L / T))."""
    F, T, D, order, delay = 3, 6000, 3, 3, 2
    Y, S, A = synth.reverberant_stft(F=F, T=T, D=D, order=order, delay=delay, seed=5)
    Y = Y.astype(np.complex128)
    X = w.wpe(Y, taps=order, delay=delay, iters=3)
    err_in = np.linalg.norm(Y - S) / np.linalg.norm(S)
    err_out = np.linalg.norm(X - S) / np.linalg.norm(S)
    assert err_in > 0.15
    assert err_out < 0.2 * err_in
    for f in range(F):
        yt = w.stack_delayed(Y[f], order, delay)
        G = w.filter_from_variance(Y[f], yt, w.variance(S[f]))
        GH = G.conj().T                                             # [D, D*order]
        for tau in range(order):
            blk = GH[:, tau * D:(tau + 1) * D]
            assert np.abs(blk - A[f, tau]).max() < 0.1 * np.abs(A[f, 0]).max() + 0.02


def test_invariances():
    rng = np.random.default_rng(4)
    T, D, L, delay = 200, 3, 3, 2
    y = _cn(rng, (T, D)) * (0.1 + rng.random((T, 1)))
    x = w.wpe_bin(y, L, delay, 3)
    c = 3.7 * np.exp(0.4j)
    assert np.abs(w.wpe_bin(c * y, L, delay, 3) - c * x).max() < 1e-9            # complex scale
    perm = np.array([2, 0, 1])
    assert np.abs(w.wpe_bin(y[:, perm], L, delay, 3) - x[:, perm]).max() < 1e-9  # channel order
    M = _cn(rng, (D, D)) + 2 * np.eye(D)                                         # any invertible mixing commutes
    xm = w.wpe_bin(y @ M.T, L, delay, 1)                                         # with the prediction step once
    lam = np.mean(np.abs(y @ M.T) ** 2, axis=1)                                  # the weights are kept equal
    yt = w.stack_delayed(y, L, delay)
    G = w.filter_from_variance(y, yt, np.maximum(lam, 1e-10 * lam.max()), load_rel=0.0)
    assert np.abs(xm - (y - yt @ G.conj()) @ M.T).max() < 1e-6
    assert np.array_equal(x[:delay], y[:delay])                                  # no past, nothing predicted


def test_degenerate_inputs():
    y0 = np.zeros((20, 3), complex)
    assert np.array_equal(w.wpe_bin(y0), y0)                          # silence stays silence
    rng = np.random.default_rng(6)
    y = _cn(rng, (2, 3))
    assert np.array_equal(w.wpe_bin(y, taps=4, delay=2), y)           # no frame has a past
    assert np.array_equal(w.wpe_bin(y, iters=0), y)
    assert w.wpe_bin(np.zeros((0, 3), complex)).shape == (0, 3)
    Y = _cn(rng, (2, 30, 2))
    X = w.wpe(Y, taps=3, delay=2, iters=2, T_valid=20)
    assert np.array_equal(X[:, 20:], np.zeros((2, 10, 2)))
    assert np.abs(X[:, :20] - w.wpe(Y[:, :20], 3, 2, 2)).max() == 0.0  # padding frames play no part
    z = y0.copy()
    z[5] = 1.0                                                        # a single non-zero frame: floor at work
    out = w.wpe_bin(z, taps=2, delay=2, iters=2)
    assert np.all(np.isfinite(out))
