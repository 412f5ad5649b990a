"""Pins for the oracle's STFT / inverse STFT and the segment -> frame bookkeeping."""

import numpy as np

from oracle import gss_oracle as o


def test_stft_against_direct_dft_small():
    rng = np.random.default_rng(0)
    n_fft, hop, N = 16, 4, 37
    x = rng.standard_normal(N)
    Y = o.stft(x, n_fft, hop)
    T = -(-N // hop) + 3
    assert Y.shape == (n_fft // 2 + 1, T)
    pad = n_fft - hop
    for t in range(T):
        for f in range(n_fft // 2 + 1):
            acc = 0j
            for n in range(n_fft):
                i = t * hop + n - pad
                xv = x[i] if 0 <= i < N else 0.0
                w = 0.5 - 0.5 * np.cos(2 * np.pi * n / n_fft)
                acc += xv * w * np.exp(-2j * np.pi * f * n / n_fft)
            assert abs(Y[f, t] - acc) < 1e-12


def test_stft_frame_count_and_span():
    for N in (1, 255, 256, 257, 1000, 4096):
        Y = o.stft(np.ones(N), 1024, 256)
        assert Y.shape == (513, -(-N // 256) + 3)
        assert o.stft_num_frames(N, 256) == Y.shape[1]


def test_istft_inverts_stft():
    rng = np.random.default_rng(1)
    for N in (700, 4096, 5000):
        x = rng.standard_normal((2, N))
        xr = o.istft(o.stft(x), N)
        assert np.max(np.abs(xr - x)) < 1e-12


def test_bin_centred_sinusoid():
    """Amplitude-A cosine at bin b: |Y[b]| = A * sum(w)/2 = 256 A, |Y[b +- 1]| = 128 A, other bins 0 (Hann)."""
    N, b, A = 8192, 37, 0.7
    n = np.arange(N)
    x = A * np.cos(2 * np.pi * b * n / 1024 + 0.3)
    Y = np.abs(o.stft(x))
    t = 10                                               # an interior frame
    assert abs(Y[b, t] - 256 * A) < 1e-9
    assert abs(Y[b - 1, t] - 128 * A) < 1e-9 and abs(Y[b + 1, t] - 128 * A) < 1e-9
    rest = np.delete(Y[:, t], [b - 1, b, b + 1])
    assert rest.max() < 1e-9


def test_parseval_per_frame():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(3000)
    Y = o.stft(x)
    w = 0.5 - 0.5 * np.cos(2 * np.pi * np.arange(1024) / 1024)
    xp = np.concatenate([np.zeros(768), x, np.zeros(4096)])
    for t in (0, 3, 7):
        frame = xp[t * 256:t * 256 + 1024] * w
        e_time = np.sum(frame ** 2)
        e_freq = (np.abs(Y[0, t]) ** 2 + np.abs(Y[512, t]) ** 2 + 2 * np.sum(np.abs(Y[1:512, t]) ** 2)) / 1024
        assert abs(e_time - e_freq) < 1e-9 * max(1.0, e_time)


def test_channels_last_layout():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, 2000))
    Y = o.stft_channels_last(x)
    assert Y.shape == (513, o.stft_num_frames(2000, 256), 3)
    assert np.allclose(Y[:, :, 1], o.stft(x[1]))


# ---------------------------------------------------------------- segment -> frame bookkeeping
def _reference_segment(s, e, n, cl, cr, hop):
    """Sample-by-sample reference: mark the context-extended span, grow it to whole hops inside the
    hop-rounded recording, and list the STFT frames whose support touches it."""
    n_round = -(-n // hop) * hop
    mark = np.zeros(n_round, bool)
    for i in range(n):
        if s - cl <= i < e + cr:
            mark[i] = True
    idx = np.nonzero(mark)[0]
    first_blk, last_blk = idx[0] // hop, idx[-1] // hop
    ext_start, ext_end = first_blk * hop, (last_blk + 1) * hop
    n_fft = 4 * hop
    T_rec = n_round // hop + 3
    frames = [t for t in range(T_rec)
              if (t - 3) * hop < ext_end and (t - 3) * hop + n_fft > ext_start]
    return ext_start, ext_end, frames


def test_segment_frames_exhaustive_small():
    hop = 4
    for n in (5, 8, 13, 16):
        for s in range(n):
            for e in range(s + 1, n + 1):
                for cl, cr in ((0, 0), (3, 2), (6, 9)):
                    r = o.segment_frames(s, e, n, cl, cr, hop)
                    es, ee, frames = _reference_segment(s, e, n, cl, cr, hop)
                    assert (r["ext_start"], r["ext_end"]) == (es, ee)
                    assert r["frame0"] == frames[0] and r["n_frames"] == len(frames)
                    assert frames == list(range(frames[0], frames[0] + len(frames)))
                    assert r["n_frames"] == o.stft_num_frames(ee - es, hop)
                    assert r["cut_start"] == s - es and r["cut_end"] == e - es
                    assert 0 <= r["cut_start"] < r["cut_end"] <= ee - es


def test_sliced_recording_stft_reconstructs_span():
    """Frames [frame0, frame0 + n_frames) of the recording's STFT, inverted on their own, give back the
    recording on the extended span (interior samples are covered by all of their four frames)."""
    rng = np.random.default_rng(4)
    n = 9000
    x = rng.standard_normal(n)
    Y = o.stft(x)
    r = o.segment_frames(3100, 5200, n, 700, 900)
    Ys = Y[:, r["frame0"]:r["frame0"] + r["n_frames"]]
    span = r["ext_end"] - r["ext_start"]
    xs = o.istft(Ys, span)
    assert np.max(np.abs(xs - x[r["ext_start"]:r["ext_end"]])) < 1e-12
    assert np.allclose(xs[r["cut_start"]:r["cut_end"]], x[3100:5200])


def test_frame_activity_reads_the_sample_the_window_weighs_most():
    """Independent pin of the frame -> sample rule: a unit impulse at sample c is sent through the oracle's
    STFT; for every frame the sample whose impulse gives that frame the most energy is the sample the frame's
    analysis window weighs most (its centre, or the nearest sample of the recording when the centre falls
    outside).  frame_activity must read exactly that sample: an activity that is on at that sample only
    lights the frame, and an activity that is off at that sample only leaves it dark."""
    n_fft, hop = 16, 4
    for N in (37, 40, 9):
        T = o.stft_num_frames(N, hop)
        energy = np.zeros((N, T))
        for c in range(N):
            x = np.zeros(N)
            x[c] = 1.0
            energy[c] = np.sum(np.abs(o.stft(x, n_fft, hop)) ** 2, axis=0)
        for t in range(T):
            if energy[:, t].max() == 0.0:                   # the frame's support touches the recording only where
                continue                                    # the window is zero: nothing to read
            best = np.flatnonzero(energy[:, t] >= energy[:, t].max() * (1 - 1e-12))
            assert len(best) == 1, (N, t, best)             # the heaviest sample is unique
            c = int(best[0])
            only = np.zeros(N, np.uint8)
            only[c] = 1
            assert o.frame_activity(only, 0, T, hop)[t] == 1, (N, t, c)
            assert o.frame_activity(1 - only, 0, T, hop)[t] == 0, (N, t, c)
            # the same frame addressed through a frame range that starts later
            if t >= 2:
                assert o.frame_activity(only, t - 2, 3, hop).tolist()[2] == 1
        # an impulse on a window centre lights one frame only; one in between lights none (nearest-centre sampling
        # of a one-sample event), so every interior sample is read by at most one frame
        reads = np.zeros(N, int)
        for c in range(N):
            only = np.zeros(N, np.uint8)
            only[c] = 1
            reads[c] = int(o.frame_activity(only, 0, T, hop).sum())
        assert np.all(reads[1:N - 1] <= 1) and reads.sum() == T


def test_frame_activity_samples_window_centre():
    hop = 4
    act = np.zeros(40, np.uint8)
    act[10:22] = 1
    fa = o.frame_activity(act, 0, 13, hop)
    expect = [int(act[min(max((t - 1) * hop, 0), 39)]) for t in range(13)]
    assert fa.tolist() == expect
    fa2 = o.frame_activity(np.stack([act, 1 - act]), 2, 5, hop)
    assert fa2.shape == (2, 5) and fa2[0].tolist() == expect[2:7] and np.all(fa2[0] + fa2[1] == 1)


# ---------------------------------------------------------------- block-wise processing (R17)
def test_block_spans_tile_the_segment():
    for s, e, n in ((0, 10, 3), (5, 6, 4), (7, 39, 8), (100, 164, 64), (3, 20, 100)):
        spans = o.block_spans(s, e, n)
        covered = np.zeros(e - s, int)
        for b0, b1 in spans:
            assert s <= b0 < b1 <= e and b1 - b0 <= n
            covered[b0 - s:b1 - s] += 1
        assert np.all(covered == 1)
        assert all(b1 - b0 == n for b0, b1 in spans[:-1])


def test_block_processing_is_causal_and_reduces_to_the_segment():
    """(i) One block that spans the whole segment, with the left context as history, is the ordinary
    per-segment result with no right context.  (ii) Causality: audio that comes after a block's last frame
    does not change that block's output (here: everything from 768 samples after the block's end on is
    replaced), while audio inside its history does."""
    rng = np.random.default_rng(31)
    D, N = 3, 12000
    act = np.zeros((2, N), np.uint8)
    act[0, 1000:9000] = 1
    act[1, 5000:12000] = 1
    src = rng.standard_normal((2, N)) * act
    A = rng.standard_normal((D, 2))
    x = A @ src + 0.05 * rng.standard_normal((D, N))
    s0, s1, hist, iters = 2048, 9216, 1536, 4
    # (i)
    whole, info = o.enhance_blocks(x, act, s0, s1, 0, s1 - s0, hist, iters)
    assert len(info) == 1
    fr = o.segment_frames(s0, s1, N, hist, 0)
    Ys = o.stft_channels_last(x).astype(np.complex64)[:, fr["frame0"]:fr["frame0"] + fr["n_frames"]]
    a = np.concatenate([o.frame_activity(act, fr["frame0"], fr["n_frames"]), np.ones((1, fr["n_frames"]), np.uint8)])
    X, ref, _ = o.mvdr(Ys, o.cacgmm_em(Ys, a, iters), 0)
    direct = o.istft(X, (fr["n_frames"] - 3) * 256)[fr["cut_start"]:fr["cut_end"]]
    assert info[0][2] == ref and np.max(np.abs(whole - direct)) < 1e-12
    # (ii)
    block = 2560
    base, binfo = o.enhance_blocks(x, act, s0, s1, 0, block, hist, iters)
    assert [b[:2] for b in binfo] == o.block_spans(s0, s1, block) and len(binfo) == 3
    b0, b1, _ = binfo[0]
    x2 = x.copy()
    x2[:, b1 + 768:] = rng.standard_normal((D, N - b1 - 768))        # beyond the reach of the block's last frame
    changed, _ = o.enhance_blocks(x2, act, s0, s1, 0, block, hist, iters)
    assert np.max(np.abs(changed[:b1 - s0] - base[:b1 - s0])) < 1e-12
    assert np.max(np.abs(changed[b1 - s0:] - base[b1 - s0:])) > 1e-3
    x3 = x.copy()
    x3[:, b0 - hist:b0 - hist + 512] *= 3.0                           # inside the first block's history
    changed3, _ = o.enhance_blocks(x3, act, s0, s1, 0, block, hist, iters)
    assert np.max(np.abs(changed3[:b1 - s0] - base[:b1 - s0])) > 1e-6
