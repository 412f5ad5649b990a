"""Host logic of the recording-level drivers: batch planning and super-segment packing (no GPU)."""

import numpy as np

from paper_2212_05271_amd import pipeline, synth


def _segments(n=60, seconds=200):
    rng = np.random.default_rng(7)
    return synth.diarization_segments(rng, 16000 * seconds, n_segments=n)


def test_plan_batches_covers_everything_within_budget():
    n_frames = np.array([1800, 300, 950, 1200, 40, 1799, 640], dtype=np.int32)
    batches = pipeline.plan_batches(n_frames, max_batch_frames=4000)
    assert sorted(i for b in batches for i in b) == list(range(len(n_frames)))
    for b in batches:
        tmax = max(n_frames[i] for i in b)
        assert len(b) == 1 or len(b) * tmax <= 4000
        assert all(n_frames[b[0]] >= n_frames[i] for i in b)          # longest first: pads to the first


def test_super_segments_same_speaker_time_order_and_cap():
    st, en, spk = _segments()
    cap = 20 * 16000
    supers = pipeline.plan_super_segments(st, en, spk, cap)
    assert sorted(i for m in supers for i in m) == list(range(len(st)))       # every segment exactly once
    for m in supers:
        assert len(set(int(spk[i]) for i in m)) == 1
        assert all(st[m[j]] <= st[m[j + 1]] for j in range(len(m) - 1))
        dur = sum(int(en[i] - st[i]) for i in m)
        assert len(m) == 1 or dur <= cap
    # greedy: a super-segment could not have taken its speaker's next segment
    for m in supers:
        later = [i for i in range(len(st)) if spk[i] == spk[m[0]] and st[i] > st[m[-1]]]
        if later:
            nxt = min(later, key=lambda i: st[i])
            assert sum(int(en[i] - st[i]) for i in m) + int(en[nxt] - st[nxt]) > cap


def test_super_segments_one_per_batch_option():
    st, en, spk = _segments(n=12, seconds=60)
    supers = pipeline.plan_super_segments(st, en, spk, 0)
    assert sorted(m[0] for m in supers) == list(range(len(st))) and all(len(m) == 1 for m in supers)


def test_super_segment_pieces_context_once_and_clipped():
    st = np.array([16000, 80000, 200000], dtype=np.int64)
    en = np.array([48000, 120000, 230000], dtype=np.int64)
    N = 240000
    ps, pe, member_of = pipeline.super_segment_pieces([0, 1, 2], st, en, N, 32000, 32000)
    assert member_of == [-1, 0, 1, 2, -1]
    assert ps.tolist() == [0, 16000, 80000, 200000, 230000]                    # left context clipped at 0
    assert pe.tolist() == [16000, 48000, 120000, 230000, 240000]               # right context clipped at N
    ps, pe, member_of = pipeline.super_segment_pieces([1], st, en, N, 0, 0)
    assert member_of == [1] and ps.tolist() == [80000] and pe.tolist() == [120000]


def test_merge_runs_no_frame_twice():
    from paper_2212_05271_amd.pipeline import merge_runs
    hop = 256
    # context | member (touching), a gap, two back-to-back members, an isolated span
    es = np.array([0, 2560, 10240, 12800, 30720]) 
    ee = np.array([2560, 5120, 12800, 15360, 33280])
    runs = merge_runs(es, ee, hop)
    assert [r[2] for r in runs] == [[0, 1], [2, 3], [4]]
    assert runs[0][:2] == (0, 5120 // hop + 3) and runs[1][:2] == (10240 // hop, (15360 - 10240) // hop + 3)
    for f0, nf, idx in runs:
        for p in idx:                                   # every span's own frames lie inside its run
            assert f0 <= es[p] // hop and ee[p] // hop + 3 <= f0 + nf
    assert sum(r[1] for r in runs) < sum((e - s) // hop + 3 for s, e in zip(es, ee))
    assert merge_runs([], [], hop) == []
