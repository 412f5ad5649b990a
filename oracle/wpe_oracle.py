"""Float64 CPU oracle for weighted-prediction-error (WPE) dereverberation.

TEST INFRASTRUCTURE ONLY: the plain definition that the HIP kernels are checked against.  Only the
test-suite may import it; the product path never does, and it shares no code with the HIP path.

arXiv 2212.05271, Section 2.1, removes the late reverberation X^tail of its signal model (the equation
above Eq. (2)) with the WPE algorithm of the works it cites there and prints no formula for it.  What is
computed here is that published algorithm (Nakatani et al., "Speech dereverberation based on
variance-normalized delayed linear prediction", 2010) in its usual offline, per-frequency, multichannel
form, with the symbols used in that literature:

  for every frequency bin, with y_t in C^D the observation, Delta the prediction delay, L the number of taps,

    ytilde_t = [y_{t-Delta}; y_{t-Delta-1}; ...; y_{t-Delta-L+1}]  in C^{D L}   (zero before the first frame)
    x_t      = y_t                                                             (start)
    repeat `iters` times:
      lambda_t = (1/D) sum_d |x_{t,d}|^2                 time-varying variance of the desired signal
      R = sum_t ytilde_t ytilde_t^H / lambda_t           (D L x D L)
      P = sum_t ytilde_t y_t^H      / lambda_t           (D L x D)
      G = R^{-1} P                                       prediction filter
      x_t = y_t - G^H ytilde_t                           y minus the predicted late reverberation

Readings (neither paper fixes them; they are part of the definition used on both sides):

  W1  lambda_t is floored at EPS_POWER_REL times its maximum over the segment's frames; a bin whose
      frames are all zero is returned unchanged.
  W2  R gets the diagonal loading LOAD_REL * tr(R) / (D L); a bin with tr(R) = 0 (no frame has a
      past) is returned unchanged.
  W3  Frames at t >= T_valid do not exist: they contribute nothing, they are no one's past, and their
      output is zero.
  W4  Defaults of the callers: L = 10 taps, Delta = 2, 3 iterations.

Component a = tau * D + d of ytilde_t is y_{t-Delta-tau, d}.
"""

from __future__ import annotations

import numpy as np

EPS_POWER_REL = 1e-10
LOAD_REL = 1e-10


def stack_delayed(y: np.ndarray, taps: int, delay: int) -> np.ndarray:
    """y [T, D] -> ytilde [T, D*taps]; component tau*D + d of row t is y[t - delay - tau, d], zero before t = 0."""
    T, D = y.shape
    out = np.zeros((T, taps * D), dtype=np.complex128)
    for tau in range(taps):
        shift = delay + tau
        if shift < T:
            out[shift:, tau * D:(tau + 1) * D] = y[:T - shift]
    return out


def variance(x: np.ndarray) -> np.ndarray:
    """lambda_t of the current estimate x [T, D], floored as reading W1 says (all zeros -> zeros)."""
    lam = np.mean(np.abs(x) ** 2, axis=1)
    top = lam.max() if lam.size else 0.0
    return np.maximum(lam, EPS_POWER_REL * top)


def filter_from_variance(y: np.ndarray, yt: np.ndarray, lam: np.ndarray, load_rel: float = LOAD_REL):
    """One weighted least-squares step: returns G [D*taps, D], or None when the bin is left unchanged."""
    N = yt.shape[1]
    if not np.any(lam > 0):
        return None
    w = 1.0 / lam
    R = (yt.T * w) @ yt.conj()            # R[a,b] = sum_t w_t ytilde_a conj(ytilde_b)
    P = (yt.T * w) @ y.conj()             # P[a,d] = sum_t w_t ytilde_a conj(y_d)
    tr = float(np.real(np.trace(R)))
    if not tr > 0.0:
        return None
    R = R + (load_rel * tr / N) * np.eye(N)
    return np.linalg.solve(R, P)


def wpe_bin(y: np.ndarray, taps: int = 10, delay: int = 2, iters: int = 3) -> np.ndarray:
    """WPE of one frequency bin.  y [T, D] complex -> x [T, D] complex128."""
    y = np.asarray(y, dtype=np.complex128)
    x = y.copy()
    if y.shape[0] == 0:
        return x
    yt = stack_delayed(y, taps, delay)
    for _ in range(iters):
        G = filter_from_variance(y, yt, variance(x))
        if G is None:
            return y.copy()
        x = y - yt @ G.conj()             # x_{t,d} = y_{t,d} - sum_a conj(G[a,d]) ytilde_{t,a}
    return x


def wpe(Y: np.ndarray, taps: int = 10, delay: int = 2, iters: int = 3, T_valid: int | None = None) -> np.ndarray:
    """Y [F, T, D] complex -> dereverberated [F, T, D] complex128; frames at t >= T_valid come back as zero."""
    F, T, D = Y.shape
    Tv = T if T_valid is None else max(0, min(int(T_valid), T))
    out = np.zeros((F, T, D), dtype=np.complex128)
    for f in range(F):
        out[f, :Tv] = wpe_bin(Y[f, :Tv], taps, delay, iters)
    return out
