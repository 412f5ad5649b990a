"""Seeded synthetic inputs with the shapes of the paper's workloads.

This module only *draws inputs* (multichannel STFT tensors, speaker
activities, time-domain recordings, segment lists).  It holds none of the
method's arithmetic: no normalisation, EM, covariance, beamformer or STFT code
lives here, so it can feed both the HIP path and the CPU oracle.

The public corpora the paper measures on (LibriCSS, AMI, AliMeeting, CHiME-6)
are not available; these generators take their shapes: 16 kHz audio, 513
frequency bins, 2 to 24 channels, a context-extended segment of a few hundred
to ~1900 frames, up to four speakers plus a noise class, sparse overlap
(Table 1 of the paper: roughly 20 % of speech time with two speakers).

Every tensor is generated in float64 from numpy's PCG64 with
seed = 1000 * config + segment_index and cast ONCE to complex64 / float32 /
uint8; both sides consume the identical cast arrays.
"""

from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

FS = 16000
N_FFT = 1024
HOP = 256
C_SOUND = 343.0


@dataclass
class Segment:
    """One context-extended segment in the STFT domain."""
    name: str
    Y: np.ndarray            # complex64 [F, T, D]
    activity: np.ndarray     # uint8 [K, T]; the noise class is the last row (all ones)
    iters: int
    target: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def shape(self):
        F, T, D = self.Y.shape
        return F, T, D, self.activity.shape[0]


def _rng(config, index=0):
    return np.random.default_rng(1000 * int(config) + int(index))


def _cn(rng, shape):
    """Circular complex standard normal, E|z|^2 = 1."""
    return (rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) / np.sqrt(2.0)


def _sources(rng, K, F, T, sigma=1.5):
    """s[k,f,t] ~ CN(0, exp(sigma * g)), g ~ N(0,1) i.i.d. per T-F bin (sparse, speech-like dynamics)."""
    g = rng.standard_normal((K, F, T))
    return np.exp(0.5 * sigma * g) * _cn(rng, (K, F, T))


def _mix(v, s, act):
    """sum_k v[k,f,:] * s[k,f,t] * act[k,t]  ->  [F,T,D]."""
    return np.einsum("kfd,kft,kt->ftd", v, s, act.astype(np.float64))


def _scale_to_snr(speech, noise, snr_db):
    ps = np.mean(np.abs(speech) ** 2)
    pn = np.mean(np.abs(noise) ** 2)
    return noise * np.sqrt(ps / (pn * 10.0 ** (snr_db / 10.0)))


def _freqs_hz(F, n_fft=N_FFT):
    """Centre frequencies of the first F bins of an n_fft-point STFT (bins spread over 0..8 kHz when F < 513)."""
    return np.arange(F) * (FS / 2.0) / max(F - 1, 1)


# ---------------------------------------------------------------------------
# activities
# ---------------------------------------------------------------------------
def markov_activity(rng, n_spk, T, mean_on=125.0, p_active=0.21, overlap_range=(0.15, 0.25), max_tries=200):
    """Per-speaker two-state Markov on/off chains.

    Mean on-run `mean_on` frames (2 s at hop 256); the off-rate follows from the
    stationary active fraction `p_active`.  Redrawn until every speaker is active
    at least once and, for n_spk >= 2 and overlap_range given, the fraction of
    frames with >= 2 speakers lies inside overlap_range.
    """
    p_off = 1.0 / mean_on                                    # on -> off
    p_on = p_off * p_active / (1.0 - p_active)               # off -> on
    best = None
    for _ in range(max_tries):
        u = rng.random((n_spk, T))
        act = np.zeros((n_spk, T), dtype=np.uint8)
        state = rng.random(n_spk) < p_active
        for t in range(T):
            flip = np.where(state, u[:, t] < p_off, u[:, t] < p_on)
            state = np.where(flip, ~state, state)
            act[:, t] = state
        if not act.any(axis=1).all():
            continue
        best = act
        if n_spk < 2 or overlap_range is None:
            break
        ov = float(np.mean(act.sum(axis=0) >= 2))
        if overlap_range[0] <= ov <= overlap_range[1]:
            break
    if best is None:                                         # very short segment: force one run per speaker
        best = np.zeros((n_spk, T), dtype=np.uint8)
        for k in range(n_spk):
            a = (k * T) // n_spk
            best[k, a:max(a + 1, ((k + 1) * T) // n_spk)] = 1
    return best


# ---------------------------------------------------------------------------
# array geometries and spatial models
# ---------------------------------------------------------------------------
def circular_array(D=8, radius=0.10):
    phi = 2.0 * np.pi * np.arange(D) / D
    return np.stack([radius * np.cos(phi), radius * np.sin(phi)], axis=1)      # [D, 2] metres


def plane_wave_steering(pos, theta, freqs):
    """v[k,f,m] = exp(j 2 pi f <pos_m, u(theta_k)> / c) / sqrt(D)   (far field)."""
    u = np.stack([np.cos(theta), np.sin(theta)], axis=1)                       # [K, 2]
    delay = pos @ u.T / C_SOUND                                                # [D, K] seconds
    ph = 2.0 * np.pi * freqs[None, :, None] * delay.T[:, None, :]              # [K, F, D]
    return np.exp(1j * ph) / np.sqrt(pos.shape[0])


def diffuse_noise(rng, pos, freqs, T, floor=0.01):
    """n[f,t,:] = C_f w, C_f C_f^H = Gamma_f + floor * I, Gamma_f[i,j] = sinc(2 f d_ij / c) (spherically isotropic)."""
    D = pos.shape[0]
    dist = np.linalg.norm(pos[:, None, :] - pos[None, :, :], axis=-1)
    gam = np.sinc(2.0 * freqs[:, None, None] * dist[None] / C_SOUND) + floor * np.eye(D)
    C = np.linalg.cholesky(gam)                                                # [F, D, D]
    w = _cn(rng, (len(freqs), T, D))
    return np.einsum("fij,ftj->fti", C, w)


def multi_array_geometry(rng, n_arrays=6, mics=4, spacing=0.05, room=4.0):
    centres = rng.uniform(0.0, room, size=(n_arrays, 2))
    orient = rng.uniform(0.0, 2.0 * np.pi, size=n_arrays)
    off = (np.arange(mics) - (mics - 1) / 2.0) * spacing
    pos = centres[:, None, :] + off[None, :, None] * np.stack([np.cos(orient), np.sin(orient)], axis=1)[:, None, :]
    return pos.reshape(n_arrays * mics, 2), np.repeat(np.arange(n_arrays), mics)


# ---------------------------------------------------------------------------
# the STFT-domain configurations
# ---------------------------------------------------------------------------
def config0(F=513, T=200, index=0):
    """2 channels, 2 speakers + noise, random steering vectors, white noise at 10 dB, 10 iterations."""
    rng = _rng(0, index)
    D, n_spk = 2, 2
    v = _cn(rng, (n_spk, F, D))
    v /= np.linalg.norm(v, axis=-1, keepdims=True)
    act = np.zeros((n_spk + 1, T), dtype=np.uint8)
    act[0, : (140 * T) // 200] = 1
    act[1, (90 * T) // 200:] = 1
    act[2, :] = 1
    s = _sources(rng, n_spk, F, T)
    speech = _mix(v, s, act[:n_spk])
    noise = _scale_to_snr(speech, _cn(rng, (F, T, D)), 10.0)
    Y = (speech + noise).astype(np.complex64)
    return Segment("c0", Y, act, iters=10, target=0, meta=dict(config=0, index=index))


def _array_segment(name, config, index, rng, pos, F, T, n_spk, K, iters, snr_db, gains=None, clock=None):
    freqs = _freqs_hz(F)
    theta = rng.uniform(0.0, 2.0 * np.pi, size=n_spk)
    v = plane_wave_steering(pos, theta, freqs)                                 # [n_spk, F, D]
    if gains is not None:
        v = v * gains[None, None, :]
    if clock is not None:
        v = v * np.exp(-2j * np.pi * freqs[None, :, None] * clock[None, None, :])
    act_spk = markov_activity(rng, n_spk, T, overlap_range=(0.15, 0.25) if n_spk == 4 else None)
    s = _sources(rng, n_spk, F, T)
    speech = _mix(v, s, act_spk)
    noise = _scale_to_snr(speech, diffuse_noise(rng, pos, freqs, T), snr_db)
    Y = (speech + noise).astype(np.complex64)
    act = np.zeros((K, T), dtype=np.uint8)
    act[:n_spk] = act_spk
    act[K - 1] = 1                                                             # noise class, always active
    return Segment(name, Y, act, iters=iters, target=0,
                   meta=dict(config=config, index=index, n_spk=n_spk, theta=theta))


def config1(F=513, T=1560, index=0):
    """8-mic circular array (r = 10 cm), 4 speakers + noise, diffuse noise at 5 dB, 20 iterations."""
    rng = _rng(1, index)
    return _array_segment("c1", 1, index, rng, circular_array(8, 0.10), F, T, n_spk=4, K=5, iters=20, snr_db=5.0)


def config2_plan(S=64, t_min=125, t_max=1875):
    """Segment lengths and speaker counts of the 64-segment batch (drawn from seed 2000)."""
    rng = _rng(2, 0)
    T = rng.integers(t_min, t_max + 1, size=S)
    n_spk = rng.integers(1, 5, size=S)
    return T.astype(np.int32), n_spk.astype(np.int32)


def config2_segment(index, T, n_spk, F=513):
    """One segment of the batch: the generators of config 1 with a per-segment seed; K padded to 5."""
    rng = _rng(2, index + 1)
    seg = _array_segment(f"c2[{index}]", 2, index, rng, circular_array(8, 0.10), F, int(T),
                         n_spk=int(n_spk), K=5, iters=15, snr_db=5.0)
    return seg


def config3(F=513, T=1500, index=0):
    """24 channels = 6 four-mic linear sub-arrays with per-array gain and clock offset, diffuse noise at 0 dB."""
    rng = _rng(3, index)
    pos, arr = multi_array_geometry(rng)
    gain = rng.uniform(0.5, 1.5, size=6)[arr]
    clock = rng.uniform(-2e-3, 2e-3, size=6)[arr]
    return _array_segment("c3", 3, index, rng, pos, F, T, n_spk=4, K=5, iters=20, snr_db=0.0,
                          gains=gain, clock=clock)


def pad_batch(segments):
    """Stack segments of one bucket into the padded batch layout the library takes.

    Returns Y[S,F,Tmax,D] complex64 (zeros in the padding), activity[S,K,Tmax] uint8 (zeros in the
    padding), T_len[S] int32, target[S] int32.
    """
    S = len(segments)
    F, _, D, K = segments[0].shape
    Tmax = max(s.Y.shape[1] for s in segments)
    Y = np.zeros((S, F, Tmax, D), dtype=np.complex64)
    act = np.zeros((S, K, Tmax), dtype=np.uint8)
    T_len = np.zeros(S, dtype=np.int32)
    target = np.zeros(S, dtype=np.int32)
    for i, s in enumerate(segments):
        T = s.Y.shape[1]
        Y[i, :, :T] = s.Y
        act[i, :, :T] = s.activity
        T_len[i] = T
        target[i] = s.target
    return Y, act, T_len, target


def buckets_by_length(T, n_buckets=4):
    """Indices of the segments sorted by length and cut into n_buckets equal groups (longest first)."""
    order = np.argsort(-np.asarray(T), kind="stable")
    return [list(map(int, b)) for b in np.array_split(order, n_buckets) if len(b)]


# ---------------------------------------------------------------------------
# time-domain recording + diarization-style segments (the full-pipeline configuration)
# ---------------------------------------------------------------------------
def _band_noise(rng, n, lo=100.0, hi=7000.0):
    """White noise band-limited to [lo, hi] Hz by zeroing rfft bins (block-wise to bound memory)."""
    out = np.empty(n)
    blk = 1 << 20
    for a in range(0, n, blk):
        m = min(blk, n - a)
        spec = np.fft.rfft(rng.standard_normal(m))
        fr = np.fft.rfftfreq(m, 1.0 / FS)
        spec[(fr < lo) | (fr > hi)] = 0.0
        out[a:a + m] = np.fft.irfft(spec, n=m)
    return out


def _rir(rng, delay_samples, rt60):
    n = int(rt60 * FS)
    t = np.arange(n) / FS
    tail = rng.standard_normal(n) * 10.0 ** (-3.0 * t / rt60) * 0.1
    h = np.zeros(delay_samples + n)
    h[delay_samples] = 1.0
    h[delay_samples:] += tail
    return h


def diarization_segments(rng, n_samples, n_spk=4, n_segments=1200, dur_range=(1.0, 20.0)):
    """Segment list (start, end, speaker) tiling the recording in time order, consecutive segments of
    different speakers overlapping by a random fraction so that ~15 % of speech time is overlapped."""
    durs = rng.uniform(dur_range[0], dur_range[1], size=n_segments)
    durs = durs * (n_samples / FS) / durs.sum() * 1.12          # stretch/shrink so the list spans the recording
    starts, ends, spk = [], [], []
    t = 0.0
    prev = -1
    for d in durs:
        k = int(rng.integers(0, n_spk))
        if k == prev:
            k = (k + 1) % n_spk
        ov = min(rng.uniform(0.0, 0.25) * d, t)
        a = int((t - ov) * FS)
        b = min(int((t - ov + d) * FS), n_samples)
        if b - a < HOP:
            break
        starts.append(a); ends.append(b); spk.append(k)
        t = t - ov + d
        prev = k
        if b >= n_samples:
            break
    return (np.asarray(starts, dtype=np.int64), np.asarray(ends, dtype=np.int64), np.asarray(spk, dtype=np.int32))


def meeting(duration_s=3600.0, n_segments=1200, D=8, n_spk=4, snr_db=5.0, index=0):
    """Synthetic meeting: x[D, N] float32, sample-level activity[n_spk, N] uint8, segment list.

    Each speaker is band-limited noise with a 4 Hz amplitude envelope, gated by its diarization
    segments, convolved with exponentially decaying random RIRs (RT60 0.3-0.6 s) whose direct-path
    delays follow the 10 cm circular array; spatially diffuse noise (per-channel white noise mixed
    through a low-order coherence model) is added at `snr_db`.
    """
    from scipy.signal import oaconvolve

    rng = _rng(4, index)
    N = int(duration_s * FS)
    starts, ends, spk = diarization_segments(rng, N, n_spk, n_segments)
    act = np.zeros((n_spk, N), dtype=np.uint8)
    for a, b, k in zip(starts, ends, spk):
        act[k, a:b] = 1
    pos = circular_array(D, 0.10)
    theta = rng.uniform(0.0, 2.0 * np.pi, size=n_spk)
    u = np.stack([np.cos(theta), np.sin(theta)], axis=1)
    x = np.zeros((D, N))
    tt = np.arange(N) / FS
    for k in range(n_spk):
        env = 0.5 + 0.5 * np.sin(2.0 * np.pi * 4.0 * tt + rng.uniform(0, 2 * np.pi))
        src = _band_noise(rng, N) * env * act[k]
        rt60 = rng.uniform(0.3, 0.6)
        for m in range(D):
            delay = int(round(-(pos[m] @ u[k]) / C_SOUND * FS)) + 8      # plane-wave delay over the array, in samples
            x[m] += oaconvolve(src, _rir(rng, max(delay, 0), rt60))[:N]
    # diffuse-ish noise: white noise per channel mixed through the broadband coherence of the array
    dist = np.linalg.norm(pos[:, None, :] - pos[None, :, :], axis=-1)
    C = np.linalg.cholesky(np.sinc(2.0 * 1000.0 * dist / C_SOUND) + 0.01 * np.eye(D))
    noise = np.zeros((D, N))
    blk = 1 << 22
    for a in range(0, N, blk):
        m = min(blk, N - a)
        noise[:, a:a + m] = C @ rng.standard_normal((D, m))
    ps = np.mean(x ** 2)
    pn = np.mean(noise ** 2)
    x += noise * np.sqrt(ps / (pn * 10.0 ** (snr_db / 10.0)))
    x /= np.max(np.abs(x)) * 1.05
    return x.astype(np.float32), act, (starts, ends, spk)


def reverberant_stft(F=513, T=1560, D=8, order=6, delay=2, decay=0.55, seed=0, n_spk=2):
    """Synthetic reverberant multichannel STFT for dereverberation tests and timing.

    Per bin, a dry signal s_t (speech-like: complex Gaussian sources with a slowly varying, on/off envelope,
    mixed by random steering vectors, plus a weak white floor) is passed through a multichannel
    autoregression  y_t = s_t + sum_{tau < order} A_tau y_{t-delay-tau},  with random D x D matrices A_tau
    whose size decays with tau and is scaled so the recursion is stable.  This is the signal model that
    delayed linear prediction inverts exactly; it stands in for room reverberation of recorded meetings.
    Returns (Y [F,T,D] complex64, S_dry [F,T,D] complex128, A [F,order,D,D] complex128).
    """
    rng = np.random.default_rng([4242, seed])
    env = np.zeros((n_spk, T))
    for k in range(n_spk):
        on = markov_activity(rng, 1, T, mean_on=60.0, p_active=0.5)[0].astype(np.float64)
        slow = np.exp(0.8 * np.cumsum(rng.standard_normal(T)) / np.sqrt(np.arange(1, T + 1)))
        env[k] = on * slow + 1e-3
    v = _cn(rng, (F, n_spk, D))
    src = _cn(rng, (F, n_spk, T)) * np.sqrt(env)[None]
    S = np.einsum("fkd,fkt->ftd", v, src) + 0.03 * _cn(rng, (F, T, D))
    A = _cn(rng, (F, order, D, D)) * (decay ** np.arange(order))[None, :, None, None]
    gain = np.linalg.norm(A, ord=2, axis=(-2, -1)).sum(axis=1)          # sum of spectral norms per bin
    A *= (0.7 / gain)[:, None, None, None]                                # sum < 1: the recursion is stable
    Y = np.zeros((F, T, D), dtype=np.complex128)
    for t in range(T):
        acc = S[:, t].copy()
        for tau in range(order):
            tp = t - delay - tau
            if tp >= 0:
                acc += np.einsum("fij,fj->fi", A[:, tau], Y[:, tp])
        Y[:, t] = acc
    return Y.astype(np.complex64), S, A
