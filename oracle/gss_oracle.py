"""Float64 CPU oracle for the guided-source-separation (GSS) hot path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP kernels are checked against.  Only the test-suite, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path never does, and it
shares no code with the HIP path.

Everything is complex128 / float64 NumPy, vectorised over the frequency axis
and otherwise written step by step in the order and notation of the paper
(arXiv 2212.05271, Section 2):

  * unit normalisation                       Eq. (2)
  * cACG density / cACGMM                    Eq. (3), (4)
  * activity-guided, time-varying weights    Eq. (5)
  * EM: E-step posteriors = masks            Section 2.2 (last paragraph)
  * masked spatial covariances               Eq. (6), (7)
  * Souden MVDR filter + reference channel   Eq. (8) and the sentence after it
  * beamformer output                        Eq. (9)
  * STFT / inverse STFT around it            Section 3 (list of ported operations)
  * segment + context -> frame bookkeeping   Section 2.2 ("context window"), Section 3 (ii)

The paper does not print the M-step, the initialisation, any regularisation,
the reference-channel rule in formula form, or the STFT parameters.  The
readings taken here (the constants below are part of the algorithm's
definition, not numerical noise):

  R1  M-step: the cACGMM fixed-point update
        B_{f,k} = D * sum_t (gamma_{k,f,t} / q_{k,f,t}) y y^H / sum_t gamma_{k,f,t},
      q = y^H B_old^{-1} y, one fixed-point step per EM iteration.
  R2  Initialisation: gamma^0 = activity normalised over the classes, q^0 = 1
      (i.e. B^0 = I), each iteration is an M-step followed by an E-step.
  R3  Mixture weights: weight_mode 1: pi_{f,k} proportional to sum_t gamma;
      weight_mode 0: pi uniform.  log pi is floored at log(1e-30).
  R4  Regularisation of B: Hermitise, rescale to trace D, add DELTA * I.  A class
      with (numerically) zero trace gets B = I.
  R5  The constant factor of Eq. (4) is common to all classes and is dropped.
  R6  The beamformer (Eq. 6-9) uses whatever Y it is handed (no normalisation
      inside); the EM normalises internally (Eq. 2).
  R7  Phi_bg gets relative diagonal loading DELTA_BF * tr(Phi_bg) / D; the
      filter's denominator is Re tr(G) + EPS_TRACE.  A frequency without any
      background energy (tr Phi_bg = 0: Eq. (8) has no solution) gets the zero filter.
  R8  One reference channel per segment: the channel r maximising
      sum_f Re(h_r^H Phi_k h_r) / sum_f Re(h_r^H Phi_bg h_r), lowest index on ties.
  R9  Frames without any active class have gamma = 0 for every class.
  R10 A zero-energy frame normalises to the zero vector; q is clamped to EPS_Q.
  R11 STFT: periodic Hann window of n_fft samples, hop n_fft/4, the signal
      zero-padded by n_fft - hop on both sides, T = ceil(N / hop) + 3 frames;
      inverse = irfft * window / (sum of squared windows over the shifts), overlap-add.
  R12 Segment bounds (plus context) are snapped outward to hop multiples and
      clipped to the recording; frame activity is sampled at the sample nearest
      the window centre.
  R13 A fixed number of iterations, no early exit.
  R16 Reference channel per frequency (speakers that move; Section 3, "Segment
      batching", says one reference channel suits a recording only when the
      speakers are stationary): the channel r maximising, for that frequency
      alone, Re(h_r^H Phi_k h_r) / Re(h_r^H Phi_bg h_r), lowest index on ties.
  R17 Block-wise processing for speakers that move (Section 1 cites block-online
      GSS; the paper gives no formula): a segment is cut into consecutive blocks
      of `block` samples (the last one shorter); block b is enhanced from the
      span [block start - history, block end) only, i.e. as a segment of its own
      with left context `history` and no right context, with its own masks,
      filter and reference channel.  Nothing after the block's last frame is used.
"""

from __future__ import annotations

import numpy as np

# ---- constants of the algorithm (see R4, R7, R10 above) --------------------
EPS_NORM_SQ = 1e-20   # floor on ||y||^2 in Eq. (2)
EPS_N = 1e-10         # floor on sum_t gamma, and on a trace
EPS_Q = 1e-10         # floor on the quadratic form y^H B^-1 y
EPS_PI = 1e-30        # floor inside log(pi)
DELTA = 1e-6          # diagonal loading of B after scaling to trace D
DELTA_BF = 1e-6       # relative diagonal loading of Phi_bg
EPS_TRACE = 1e-20     # added to Re tr(Phi_bg^-1 Phi_k)
EPS_SNR = 1e-300      # floor on the background power in the reference-channel ratio


# ---------------------------------------------------------------------------
# Eq. (2): unit normalisation (the WPE tail estimate is taken to be zero)
# ---------------------------------------------------------------------------
def unit_normalise(Y):
    """Y[..., D] complex -> Y / max(||Y||, 1e-10) along the channel axis. Eq. (2), R10."""
    Y = np.asarray(Y, dtype=np.complex128)
    n2 = np.sum(Y.real ** 2 + Y.imag ** 2, axis=-1, keepdims=True)
    return Y / np.sqrt(np.maximum(n2, EPS_NORM_SQ))


# ---------------------------------------------------------------------------
# Section 2.2: cACGMM EM guided by speaker activity
# ---------------------------------------------------------------------------
def initial_posteriors(activity, F):
    """gamma^0[k, f, t] = a[k, t] / max(1, sum_k a[k, t])   (R2)."""
    a = (np.asarray(activity) != 0).astype(np.float64)          # [K, T]
    g = a / np.maximum(a.sum(axis=0, keepdims=True), 1.0)
    return np.repeat(g[:, None, :], F, axis=1)                    # [K, F, T]


def weighted_scatter(Yn, gamma, q):
    """N[f,k] = sum_t gamma and R[f,k] = sum_t (gamma / q) y y^H, the sufficient statistics of R1."""
    N = gamma.sum(axis=2).T                                       # [F, K]
    w = gamma / q                                                 # [K, F, T]
    R = np.einsum("kft,fti,ftj->fkij", w, Yn, Yn.conj())
    return R, N


def regularise_scatter(B):
    """R4: Hermitise, rescale to trace D (identity if the trace vanishes), add DELTA * I."""
    D = B.shape[-1]
    eye = np.eye(D, dtype=np.complex128)
    B = 0.5 * (B + B.conj().swapaxes(-1, -2))
    tr = np.trace(B, axis1=-2, axis2=-1).real
    dead = tr <= EPS_N
    B[dead] = eye
    tr = np.where(dead, float(D), tr)
    B = B * (D / tr)[..., None, None]
    return B + DELTA * eye


def m_step(Yn, gamma, q, weight_mode=1):
    """Parameters of the component model from the posteriors (R1, R3, R4).

    Yn[F,T,D] unit-normalised, gamma[K,F,T], q[K,F,T].
    Returns B[F,K,D,D], pi[F,K], N[F,K].
    """
    F, T, D = Yn.shape
    K = gamma.shape[0]
    R, N = weighted_scatter(Yn, gamma, q)
    B = regularise_scatter(D * R / np.maximum(N, EPS_N)[:, :, None, None])
    if weight_mode == 1:
        pi = N / np.maximum(N.sum(axis=1, keepdims=True), EPS_N)
    elif weight_mode == 0:
        pi = np.full((F, K), 1.0 / K)
    else:
        raise ValueError("weight_mode must be 0 or 1")
    return B, pi, N


def quadratic_forms(Yn, B):
    """q[k,f,t] = max(Re(y^H B_{f,k}^{-1} y), EPS_Q) and log det B_{f,k}.  Eq. (4), R10."""
    # solve B x = y for every frame:  B[F,K,D,D], rhs[F,1,D,T] -> x[F,K,D,T]
    rhs = Yn.transpose(0, 2, 1)[:, None, :, :]
    x = np.linalg.solve(B, np.broadcast_to(rhs, B.shape[:2] + rhs.shape[2:]))
    q = np.einsum("ftd,fkdt->kft", Yn.conj(), x).real
    sign, logdet = np.linalg.slogdet(B)
    return np.maximum(q, EPS_Q), logdet.real


def e_step(Yn, B, pi, activity):
    """State posteriors under Eq. (3)-(5).  Returns gamma[K,F,T], q[K,F,T]."""
    F, T, D = Yn.shape
    a = (np.asarray(activity) != 0)                               # [K, T]
    q, logdet = quadratic_forms(Yn, B)
    logpi = np.log(np.maximum(pi, EPS_PI))                        # [F, K]
    # log of pi_k * A(y; B_k) without the class-independent constant (R5)
    ell = (logpi - logdet).T[:, :, None] - D * np.log(q)          # [K, F, T]
    act = a[:, None, :]                                           # [K, 1, T]
    ell_m = np.where(act, ell, -np.inf)
    mx = ell_m.max(axis=0, keepdims=True)
    mx = np.where(np.isfinite(mx), mx, 0.0)                       # frames with no active class (R9)
    e = np.where(act, np.exp(ell_m - mx), 0.0)
    Z = e.sum(axis=0, keepdims=True)
    gamma = np.where(Z > 0.0, e / np.where(Z > 0.0, Z, 1.0), 0.0)
    return gamma, q


def cacgmm_em(Y, activity, iters, weight_mode=1, return_params=False):
    """Guided cACGMM EM for one segment.

    Y[F,T,D] complex (any scale), activity[K,T] in {0,1}, `iters` M+E iterations.
    Returns the masks gamma[K,F,T] (float64); with return_params also (B, pi).
    """
    Y = np.asarray(Y)
    F, T, D = Y.shape
    K = np.asarray(activity).shape[0]
    Yn = unit_normalise(Y)
    gamma = initial_posteriors(activity, F)
    q = np.ones((K, F, T))
    B = np.broadcast_to(np.eye(D, dtype=np.complex128), (F, K, D, D)).copy()
    pi = np.full((F, K), 1.0 / K)
    for _ in range(int(iters)):
        B, pi, _ = m_step(Yn, gamma, q, weight_mode)
        gamma, q = e_step(Yn, B, pi, activity)
    if return_params:
        return gamma, B, pi
    return gamma


def cacgmm_em_batch(Y, activity, T_len, iters, weight_mode=1):
    """Padded batch: Y[S,F,Tmax,D], activity[S,K,Tmax], T_len[S] (or None).

    Every segment is run on its own first T_len[s] frames; frames at or beyond
    T_len[s] come back as exact zeros.
    """
    Y = np.asarray(Y)
    S, F, Tmax, D = Y.shape
    K = np.asarray(activity).shape[1]
    gamma = np.zeros((S, K, F, Tmax))
    for s in range(S):
        T = Tmax if T_len is None else int(T_len[s])
        if T > 0:
            gamma[s, :, :, :T] = cacgmm_em(Y[s, :, :T], np.asarray(activity)[s, :, :T], iters, weight_mode)
    return gamma


def log_likelihood(Yn, B, pi, activity):
    """sum_{f,t} log sum_k pi_{t,f,k} A(y;B_k) up to the constant of Eq. (4); frames with no active class skipped."""
    F, T, D = Yn.shape
    a = (np.asarray(activity) != 0)
    q, logdet = quadratic_forms(Yn, B)
    w = pi.T[:, :, None] * a[:, None, :]                          # [K,F,T] numerator of Eq. (5)
    den = w.sum(axis=0, keepdims=True)
    ok = den[0] > 0
    w = w / np.where(den > 0, den, 1.0)
    dens = np.exp(-logdet.T[:, :, None] - D * np.log(q))
    mix = (w * dens).sum(axis=0)
    return float(np.log(mix[ok]).sum())


# ---------------------------------------------------------------------------
# Section 2.3: mask-based MVDR
# ---------------------------------------------------------------------------
def masked_covariances(Y, gamma, target):
    """Phi_k[F,D,D], Phi_bg[F,D,D] of Eq. (6), (7) without the common 1/T."""
    Y = np.asarray(Y, dtype=np.complex128)
    g_t = np.asarray(gamma, dtype=np.float64)[target]             # [F, T]
    g_bg = np.asarray(gamma, dtype=np.float64).sum(axis=0) - g_t
    phi_k = np.einsum("ft,fti,ftj->fij", g_t, Y, Y.conj())
    phi_bg = np.einsum("ft,fti,ftj->fij", g_bg, Y, Y.conj())
    return phi_k, phi_bg


def load_background(phi_bg):
    """Phi_bg + DELTA_BF * tr(Phi_bg)/D * I   (R7)."""
    D = phi_bg.shape[-1]
    tr = np.trace(phi_bg, axis1=-2, axis2=-1).real
    return phi_bg + (DELTA_BF * tr / D)[:, None, None] * np.eye(D)


def souden_filters(phi_k, phi_bg_loaded):
    """H[F, D(channel), D(ref)]: column r is the filter of Eq. (8) for reference channel r; zero where the
    background covariance is zero (R7)."""
    D = phi_k.shape[-1]
    none = ~(np.trace(phi_bg_loaded, axis1=-2, axis2=-1).real > 0.0)
    G = np.linalg.solve(np.where(none[:, None, None], np.eye(D), phi_bg_loaded), phi_k)
    G[none] = 0.0
    tr = np.trace(G, axis1=-2, axis2=-1).real
    return G / (tr + EPS_TRACE)[:, None, None]


def reference_channel_scores(H, phi_k, phi_bg_loaded):
    """score[r] = sum_f Re(h_r^H Phi_k h_r) / sum_f Re(h_r^H Phi_bg h_r)   (R8)."""
    num = np.einsum("fir,fij,fjr->r", H.conj(), phi_k, H).real
    den = np.einsum("fir,fij,fjr->r", H.conj(), phi_bg_loaded, H).real
    return num / np.maximum(den, EPS_SNR)


def reference_channel_scores_per_frequency(H, phi_k, phi_bg_loaded):
    """score[f, r] = Re(h_r^H Phi_k h_r) / Re(h_r^H Phi_bg h_r) at frequency f   (R16)."""
    num = np.einsum("fir,fij,fjr->fr", H.conj(), phi_k, H).real
    den = np.einsum("fir,fij,fjr->fr", H.conj(), phi_bg_loaded, H).real
    return num / np.maximum(den, EPS_SNR)


def mvdr_per_frequency_ref(Y, gamma, target, ref=None):
    """Mask-based Souden MVDR with one reference channel per frequency (R16).

    Y[F,T,D], gamma[K,F,T], target class index, ref[F] channels (None = choose all; an entry < 0 = choose
    that frequency's).  Returns X[F,T] complex128, ref[F] (int), h[F,D].
    """
    Y = np.asarray(Y, dtype=np.complex128)
    F = Y.shape[0]
    phi_k, phi_bg = masked_covariances(Y, gamma, target)
    phi_bg_l = load_background(phi_bg)
    H = souden_filters(phi_k, phi_bg_l)
    chosen = np.argmax(reference_channel_scores_per_frequency(H, phi_k, phi_bg_l), axis=1)   # lowest index on ties
    if ref is None:
        ref_f = chosen
    else:
        ref_f = np.where(np.asarray(ref) < 0, chosen, np.asarray(ref))
    ref_f = ref_f.astype(np.int64)
    h = H[np.arange(F), :, ref_f]
    X = np.einsum("fd,ftd->ft", h.conj(), Y)
    return X, ref_f, h


def mvdr(Y, gamma, target, ref=None):
    """Mask-based Souden MVDR for one segment.

    Y[F,T,D], gamma[K,F,T], target class index, ref channel (None/-1 = choose by R8).
    Returns X[F,T] complex128, ref (int), h[F,D].
    """
    Y = np.asarray(Y, dtype=np.complex128)
    phi_k, phi_bg = masked_covariances(Y, gamma, target)
    phi_bg_l = load_background(phi_bg)
    H = souden_filters(phi_k, phi_bg_l)
    if ref is None or int(ref) < 0:
        ref = int(np.argmax(reference_channel_scores(H, phi_k, phi_bg_l)))  # argmax = lowest index on ties
    ref = int(ref)
    h = H[:, :, ref]
    X = np.einsum("fd,ftd->ft", h.conj(), Y)                       # Eq. (9)
    return X, ref, h


def mvdr_batch(Y, gamma, T_len, target, ref):
    """Padded batch version of mvdr(); ref[s] < 0 means choose.  Returns X[S,F,Tmax], ref[S]."""
    Y = np.asarray(Y)
    S, F, Tmax, D = Y.shape
    X = np.zeros((S, F, Tmax), dtype=np.complex128)
    ref_out = np.zeros(S, dtype=np.int32)
    for s in range(S):
        T = Tmax if T_len is None else int(T_len[s])
        r = -1 if ref is None else int(ref[s])
        if T > 0:
            X[s, :, :T], ref_out[s], _ = mvdr(Y[s, :, :T], np.asarray(gamma)[s, :, :, :T], int(target[s]), r)
        else:
            ref_out[s] = max(r, 0)
    return X, ref_out


# ---------------------------------------------------------------------------
# STFT / inverse STFT (R11)
# ---------------------------------------------------------------------------
def hann_periodic(n_fft):
    n = np.arange(n_fft, dtype=np.float64)
    return 0.5 - 0.5 * np.cos(2.0 * np.pi * n / n_fft)


def stft_num_frames(N, hop):
    return -(-int(N) // int(hop)) + 3


def stft(x, n_fft=1024, hop=256):
    """x[..., N] real -> Y[..., F, T] complex128, F = n_fft/2 + 1, T = ceil(N/hop) + 3."""
    x = np.asarray(x, dtype=np.float64)
    N = x.shape[-1]
    T = stft_num_frames(N, hop)
    pad = n_fft - hop
    total = (T - 1) * hop + n_fft
    xp = np.zeros(x.shape[:-1] + (total,), dtype=np.float64)
    xp[..., pad:pad + N] = x
    w = hann_periodic(n_fft)
    out = np.empty(x.shape[:-1] + (n_fft // 2 + 1, T), dtype=np.complex128)
    for t in range(T):
        out[..., t] = np.fft.rfft(xp[..., t * hop:t * hop + n_fft] * w, axis=-1)
    return out


def istft(X, N, n_fft=1024, hop=256):
    """X[..., F, T] -> x[..., N]: weighted overlap-add inverse of stft()."""
    X = np.asarray(X, dtype=np.complex128)
    T = X.shape[-1]
    pad = n_fft - hop
    total = (T - 1) * hop + n_fft
    w = hann_periodic(n_fft)
    wsq = sum(np.roll(w, m * hop) ** 2 for m in range(n_fft // hop))   # constant (1.5 for Hann, hop = n_fft/4)
    ws = w / wsq
    y = np.zeros(X.shape[:-2] + (total,), dtype=np.float64)
    for t in range(T):
        y[..., t * hop:t * hop + n_fft] += np.fft.irfft(X[..., t], n=n_fft, axis=-1) * ws
    return y[..., pad:pad + N]


def stft_channels_last(x, n_fft=1024, hop=256):
    """x[D, N] -> Y[F, T, D], the layout the EM and the beamformer take."""
    return np.ascontiguousarray(np.moveaxis(stft(x, n_fft, hop), 0, -1))


# ---------------------------------------------------------------------------
# Segment + context -> sample / frame bookkeeping (R12).  Integers only.
# ---------------------------------------------------------------------------
def segment_frames(seg_start, seg_end, n_samples, ctx_left, ctx_right, hop=256):
    """One target segment [seg_start, seg_end) in samples of a recording of n_samples.

    Returns a dict of Python ints:
      ext_start, ext_end : the context-extended span, snapped outward to hop multiples, clipped
      frame0, n_frames   : its frames in the recording's STFT (R11 numbering), n_frames = span/hop + 3
      cut_start, cut_end : the target region as sample offsets inside the span's inverse STFT
    """
    s, e, n = int(seg_start), int(seg_end), int(n_samples)
    a = max(s - int(ctx_left), 0)
    b = min(e + int(ctx_right), n)
    ext_start = (a // hop) * hop
    ext_end = min(-(-b // hop) * hop, -(-n // hop) * hop)
    frame0 = ext_start // hop
    n_frames = (ext_end - ext_start) // hop + 3
    return dict(ext_start=ext_start, ext_end=ext_end, frame0=frame0, n_frames=n_frames,
                cut_start=s - ext_start, cut_end=e - ext_start)


def frame_activity(act_samples, frame0, n_frames, hop=256):
    """Frame-level activity of one class from its sample-level 0/1 activity.

    Frame t (recording numbering) is centred on sample (t - 1) * hop; the activity is
    read at that sample clamped into [0, N - 1].
    """
    act = np.asarray(act_samples)
    N = act.shape[-1]
    out = np.zeros(act.shape[:-1] + (n_frames,), dtype=np.uint8)
    for i in range(n_frames):
        c = (frame0 + i - 1) * hop
        c = min(max(c, 0), N - 1)
        out[..., i] = (act[..., c] != 0)
    return out


# ---------------------------------------------------------------------------
# Block-wise processing of a segment (R17).  The bookkeeping is integers only.
# ---------------------------------------------------------------------------
def block_spans(seg_start, seg_end, block):
    """Consecutive blocks [b0, b1) of `block` samples that tile the segment [seg_start, seg_end)."""
    s, e, n = int(seg_start), int(seg_end), int(block)
    return [(b, min(b + n, e)) for b in range(s, e, n)]


def enhance_blocks(x, act_samples, seg_start, seg_end, target, block, history, iters, weight_mode=1, hop=256):
    """One segment of the recording x[D, N], block by block (R17): every block is its own segment with left
    context `history` samples and no right context: STFT of the recording, the block's frames, EM, MVDR with
    the block's own reference channel, inverse STFT, cut to the block.  act_samples[n_spk, N]; the classes are
    the speakers plus a noise class that is always active.  Returns the enhanced segment (float64) and the
    list of (block start, block end, reference channel)."""
    x = np.asarray(x, dtype=np.float64)
    N = x.shape[1]
    Yrec = stft_channels_last(x).astype(np.complex64)       # the precision in which the stages hand it over
    out = np.zeros(int(seg_end) - int(seg_start))
    info = []
    for b0, b1 in block_spans(seg_start, seg_end, block):
        fr = segment_frames(b0, b1, N, history, 0, hop)
        f0, nf = fr["frame0"], fr["n_frames"]
        Ys = Yrec[:, f0:f0 + nf]
        act = np.concatenate([frame_activity(act_samples, f0, nf, hop), np.ones((1, nf), np.uint8)])
        g = cacgmm_em(Ys, act, iters, weight_mode)
        X, ref, _ = mvdr(Ys, g, target)
        xb = istft(X, (nf - 3) * hop, 4 * hop, hop)[fr["cut_start"]:fr["cut_end"]]
        out[b0 - int(seg_start):b1 - int(seg_start)] = xb
        info.append((b0, b1, ref))
    return out, info
