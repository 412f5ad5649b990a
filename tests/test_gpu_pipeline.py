"""Full-size batch (config 2) and the recording-level pipeline (config 4, at reduced duration) on the GPU
against the oracle, on sampled segments / bins that the oracle can finish in seconds."""

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL_GAMMA = 1e-3
TOL_X = 1e-4


@pytest.fixture(scope="module")
def env():
    import torch
    from oracle import gss_oracle as o
    from paper_2212_05271_amd import binding as gss
    from paper_2212_05271_amd import pipeline, synth
    ctx = gss.Context(0)
    yield dict(torch=torch, o=o, gss=gss, synth=synth, ctx=ctx, pipeline=pipeline)
    ctx.close()


def test_config2_full_size_batch(env):
    """64 segments, T in [125, 1875], 1-4 speakers + noise (K padded to 5), 15 iterations, bucketed by length
    into 4 padded batches: the launch configuration of the batched workload.  The oracle checks the shortest,
    the longest and one middle segment of every bucket on six frequency bins, the first and the last included
    (segments and bins are independent)."""
    t, o, gss, synth, ctx = env["torch"], env["o"], env["gss"], env["synth"], env["ctx"]
    T, ns = synth.config2_plan()
    buckets = synth.buckets_by_length(T, 4)
    bins = np.array([0, 5, 130, 300, 500, 512])
    for bi, idx in enumerate(buckets):
        segs = [synth.config2_segment(i, T[i], ns[i]) for i in idx]
        Y, act, T_len, target = synth.pad_batch(segs)
        Yd = t.from_numpy(Y).cuda()
        Td = t.from_numpy(T_len).cuda()
        g = gss.gss_cacgmm_em(ctx, Yd, t.from_numpy(act).cuda(), Td, 15)
        ref = t.zeros(len(idx), dtype=t.int32).cuda()
        X = gss.gss_mvdr(ctx, Yd, g, t.from_numpy(target).cuda(), ref, Td)
        t.cuda.synchronize()
        by_len = np.argsort([sg.Y.shape[1] for sg in segs], kind="stable")
        for pick in sorted({int(by_len[0]), int(by_len[-1]), len(idx) // 2 + (bi % 3)}):
            seg = segs[pick]
            Ts = seg.Y.shape[1]
            go = o.cacgmm_em(seg.Y[bins], seg.activity, 15)
            gg = g[pick].cpu().numpy()
            assert np.max(np.abs(gg[:, bins, :Ts] - go)) <= TOL_GAMMA
            assert np.all(gg[:, :, Ts:] == 0)
            Xo, _, _ = o.mvdr(seg.Y[bins], gg[:, bins, :Ts].astype(np.float64), 0, ref=0)
            Xg = X[pick].cpu().numpy()
            assert np.linalg.norm(Xg[bins, :Ts] - Xo) <= TOL_X * np.linalg.norm(Xo)
            assert np.all(Xg[:, Ts:] == 0)
        del Yd, g, X


def test_recording_pipeline_reduced_meeting(env):
    """Config 4 at reduced duration: a 60 s, 8-channel synthetic meeting with 16 diarization segments, 7.5 s of
    context per side: STFT of the recording once, segments as frame ranges, batched EM (15 iterations) + MVDR +
    iSTFT, target regions cut out.  Two segments are re-done end to end by the oracle."""
    t, o, gss, synth, ctx, pipeline = (env[k] for k in ("torch", "o", "gss", "synth", "ctx", "pipeline"))
    x, act_s, (st, en, spk) = synth.meeting(duration_s=60.0, n_segments=16)
    D, N = x.shape
    ctx_s = 120_000
    xd = t.from_numpy(x).cuda()
    outs, fr = pipeline.enhance_recording(ctx, xd, act_s, st, en, spk, ctx_s, ctx_s, iters=15)
    t.cuda.synchronize()
    assert len(outs) == len(st)
    for i in range(len(st)):
        assert outs[i].shape[0] == int(en[i] - st[i])
        ref = o.segment_frames(int(st[i]), int(en[i]), N, ctx_s, ctx_s)
        for key in ("ext_start", "ext_end", "frame0", "n_frames", "cut_start", "cut_end"):
            assert int(fr[key][i]) == ref[key]
    Yrec = o.stft_channels_last(x).astype(np.complex64)
    order = np.argsort(fr["n_frames"])
    for i in (int(order[0]), int(order[len(order) // 2])):
        f0, nf = int(fr["frame0"][i]), int(fr["n_frames"][i])
        Ys = Yrec[:, f0:f0 + nf]
        act = np.concatenate([o.frame_activity(act_s, f0, nf), np.ones((1, nf), np.uint8)])
        go = o.cacgmm_em(Ys, act, 15)
        Xo, ro, _ = o.mvdr(Ys, go, int(spk[i]))
        xo = o.istft(Xo, (nf - 3) * 256)[int(fr["cut_start"][i]):int(fr["cut_end"][i])]
        xg = outs[i].cpu().numpy()
        assert int(fr["ref"][i]) == ro
        assert np.linalg.norm(xg - xo) <= TOL_X * np.linalg.norm(xo)


def test_recording_pipeline_with_wpe(env):
    """The 60 s meeting with dereverberation switched on (10 taps, delay 2, 3 iterations): WPE -> EM -> MVDR ->
    iSTFT of the shortest segment re-done end to end by the oracles (the dereverberated STFT rounded to
    complex64, the precision in which the stages hand it over)."""
    from oracle import wpe_oracle as w
    t, o, gss, synth, ctx, pipeline = (env[k] for k in ("torch", "o", "gss", "synth", "ctx", "pipeline"))
    x, act_s, (st, en, spk) = synth.meeting(duration_s=60.0, n_segments=16)
    D, N = x.shape
    ctx_s = 48_000
    xd = t.from_numpy(x).cuda()
    outs, fr = pipeline.enhance_recording(ctx, xd, act_s, st, en, spk, ctx_s, ctx_s, iters=15, wpe_taps=10)
    t.cuda.synchronize()
    plain, _ = pipeline.enhance_recording(ctx, xd, act_s, st, en, spk, ctx_s, ctx_s, iters=15)
    Yrec = o.stft_channels_last(x).astype(np.complex64)
    i = int(np.argsort(fr["n_frames"])[0])
    f0, nf = int(fr["frame0"][i]), int(fr["n_frames"][i])
    Ys = w.wpe(Yrec[:, f0:f0 + nf].astype(np.complex128), 10, 2, 3).astype(np.complex64)
    act = np.concatenate([o.frame_activity(act_s, f0, nf), np.ones((1, nf), np.uint8)])
    go = o.cacgmm_em(Ys, act, 15)
    Xo, ro, _ = o.mvdr(Ys, go, int(spk[i]))
    xo = o.istft(Xo, (nf - 3) * 256)[int(fr["cut_start"][i]):int(fr["cut_end"][i])]
    xg = outs[i].cpu().numpy()
    assert int(fr["ref"][i]) == ro
    assert np.linalg.norm(xg - xo) <= TOL_X * np.linalg.norm(xo)
    assert np.linalg.norm(xg - plain[i].cpu().numpy()) > 1e-2 * np.linalg.norm(xo)   # and it does change the output


def test_super_segment_batching_reduced_meeting(env):
    """Super-segment batching (Section 3, "Segment batching") on the 60 s meeting: same-speaker segments
    concatenated along time with one context window per super-segment, shared statistics, every member
    inverted and cut on its own.  One super-segment with several members is re-done end to end by the oracle
    from the same concatenation rule."""
    t, o, gss, synth, ctx, pipeline = (env[k] for k in ("torch", "o", "gss", "synth", "ctx", "pipeline"))
    x, act_s, (st, en, spk) = synth.meeting(duration_s=60.0, n_segments=16)
    D, N = x.shape
    ctx_s = 32_000
    xd = t.from_numpy(x).cuda()
    outs, info = pipeline.enhance_recording_super(ctx, xd, act_s, st, en, spk, ctx_s, ctx_s, max_batch_s=10.0, iters=15)
    t.cuda.synchronize()
    assert sorted(i for m in info["supers"] for i in m) == list(range(len(st)))
    for i in range(len(st)):
        assert outs[i].shape[0] == int(en[i] - st[i])
    multi = [b for b, m in enumerate(info["supers"]) if len(m) > 1]
    assert multi, "the test meeting must produce a super-segment with more than one member"
    b = multi[0]
    members = info["supers"][b]
    ps, pe, member_of = pipeline.super_segment_pieces(members, st, en, N, ctx_s, ctx_s)
    Yrec = o.stft_channels_last(x).astype(np.complex64)
    frames = [o.segment_frames(int(s), int(e), N, 0, 0) for s, e in zip(ps, pe)]
    # spans that touch in time form one run of consecutive frames: no recording frame is used twice
    used = set()
    run_list = []                                       # [first frame, last frame + 1]
    for f in frames:
        fa, fb = f["frame0"], f["frame0"] + f["n_frames"]
        if run_list and f["ext_start"] <= run_list[-1][2]:
            run_list[-1][1] = max(run_list[-1][1], fb)
            run_list[-1][2] = max(run_list[-1][2], f["ext_end"])
        else:
            run_list.append([fa, fb, f["ext_end"]])
    for fa, fb, _ in run_list:
        for q in range(fa, fb):
            used.add(q)
    assert len(used) == sum(fb - fa for fa, fb, _ in run_list)   # no frame twice, unless members overlap in time
    Ys = np.concatenate([Yrec[:, fa:fb] for fa, fb, _ in run_list], axis=1)
    act = np.concatenate([o.frame_activity(act_s, fa, fb - fa) for fa, fb, _ in run_list], axis=1)
    act = np.concatenate([act, np.ones((1, act.shape[1]), np.uint8)])
    assert Ys.shape[1] == int(info["T"][b])
    assert len(run_list) < len(frames), "the context and the first member must have merged"
    go = o.cacgmm_em(Ys, act, 15)
    Xo, ro, _ = o.mvdr(Ys, go, int(spk[members[0]]))
    assert int(info["ref"][b]) == ro
    starts = np.concatenate([[0], np.cumsum([r[1] - r[0] for r in run_list])])
    for f, i in zip(frames, member_of):
        nf = f["n_frames"]
        if i >= 0:
            r = next(q for q, (fa, fb, _) in enumerate(run_list) if fa <= f["frame0"] and f["frame0"] + nf <= fb)
            off = int(starts[r]) + f["frame0"] - run_list[r][0]
            xo = o.istft(Xo[:, off:off + nf], (nf - 3) * 256)[f["cut_start"]:f["cut_end"]]
            xg = outs[i].cpu().numpy()
            assert np.linalg.norm(xg - xo) <= TOL_X * np.linalg.norm(xo)

def test_recording_pipeline_full_hour(env):
    """Config 4 at full size: a one-hour, 8-channel synthetic meeting with 1200 diarization segments and 7.5 s of
    context per side through the pipeline driver (STFT of the recording once, padded batches of EM (15
    iterations) + MVDR + iSTFT).  Every output has its segment's length and is finite; the bookkeeping matches
    the oracle's for every segment; one interior segment is re-done end to end by the oracle, whose STFT is
    taken over that segment's span plus the 768 samples on either side that its frames reach into."""
    t, o, gss, synth, ctx, pipeline = (env[k] for k in ("torch", "o", "gss", "synth", "ctx", "pipeline"))
    x, act_s, (st, en, spk) = synth.meeting(duration_s=3600.0, n_segments=1200)
    D, N = x.shape
    ctx_s = 120_000
    xd = t.from_numpy(x).cuda()
    outs, fr = pipeline.enhance_recording(ctx, xd, act_s, st, en, spk, ctx_s, ctx_s, iters=15)
    t.cuda.synchronize()
    assert len(outs) == 1200 and ctx.get_status() == 0
    for i in range(len(st)):
        assert outs[i].shape[0] == int(en[i] - st[i])
        ref = o.segment_frames(int(st[i]), int(en[i]), N, ctx_s, ctx_s)
        for key in ("ext_start", "ext_end", "frame0", "n_frames", "cut_start", "cut_end"):
            assert int(fr[key][i]) == ref[key]
    assert all(bool(t.isfinite(v).all()) for v in outs[::50])
    # the shortest segment whose extended span stays 768 samples clear of both ends of the recording
    inner = [i for i in range(len(st)) if fr["ext_start"][i] >= 768 and fr["ext_end"][i] + 768 <= N]
    i = min(inner, key=lambda k: int(fr["n_frames"][k]))
    s0, e0 = int(fr["ext_start"][i]) - 768, int(fr["ext_end"][i]) + 768
    f0, nf = int(fr["frame0"][i]), int(fr["n_frames"][i])
    Ysub = o.stft_channels_last(x[:, s0:e0]).astype(np.complex64)       # its frame u is recording frame u + s0 / 256
    u0 = f0 - s0 // 256
    assert u0 == 3 and u0 + nf <= Ysub.shape[1]
    Ys = Ysub[:, u0:u0 + nf]
    act = np.concatenate([o.frame_activity(act_s, f0, nf), np.ones((1, nf), np.uint8)])
    go = o.cacgmm_em(Ys, act, 15)
    Xo, ro, _ = o.mvdr(Ys, go, int(spk[i]))
    xo = o.istft(Xo, (nf - 3) * 256)[int(fr["cut_start"][i]):int(fr["cut_end"][i])]
    xg = outs[i].cpu().numpy()
    assert int(fr["ref"][i]) == ro
    assert np.linalg.norm(xg - xo) <= TOL_X * np.linalg.norm(xo)


def test_block_processing_reduced_meeting(env):
    """Block-wise processing (every block of a segment enhanced from its own past only, own reference channel) on
    the 60 s meeting: block table and two segments end to end against the oracle's block loop."""
    t, o, gss, synth, ctx, pipeline = (env[k] for k in ("torch", "o", "gss", "synth", "ctx", "pipeline"))
    x, act_s, (st, en, spk) = synth.meeting(duration_s=60.0, n_segments=16)
    D, N = x.shape
    block, hist, iters = 32_000, 48_000, 8
    xd = t.from_numpy(x).cuda()
    outs, info = pipeline.enhance_recording_blocks(ctx, xd, act_s, st, en, spk, block, hist, iters=iters)
    t.cuda.synchronize()
    assert len(outs) == len(st)
    rows = 0
    for i in range(len(st)):
        assert outs[i].shape[0] == int(en[i] - st[i])
        spans = o.block_spans(int(st[i]), int(en[i]), block)
        mine = np.flatnonzero(info["segment"] == i)
        assert [(int(info["start"][m]), int(info["end"][m])) for m in mine] == spans
        rows += len(spans)
    assert rows == len(info["segment"])
    longest = int(np.argmax(en - st))
    shortest = int(np.argmin(en - st))
    for i in (longest, shortest):
        xo, binfo = o.enhance_blocks(x, act_s, int(st[i]), int(en[i]), int(spk[i]), block, hist, iters)
        mine = np.flatnonzero(info["segment"] == i)
        assert [int(info["ref"][m]) for m in mine] == [b[2] for b in binfo]
        xg = outs[i].cpu().numpy()
        assert np.linalg.norm(xg - xo) <= TOL_X * np.linalg.norm(xo)
    assert len(o.block_spans(int(st[longest]), int(en[longest]), block)) > 1
