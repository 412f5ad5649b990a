"""Per-configuration timing of the EM + MVDR path on one MI355X (the other configurations next to bench.py's).

    python -m paper_2212_05271_amd.measure_configs [--meeting-s 300]

For each synthetic configuration (the same seeded generators the parity tests use): stream time of
gss_cacgmm_em and gss_mvdr with the inputs resident in HBM, audio seconds per second over the two, EM
iterations and time-frequency-bin-iterations per second, and the algorithmic fp64 rate of the EM
((3 + 4K) D^2 + 3D + 30K flops per bin and iteration) against the 78.6 TFLOP/s vector peak.  The padded
batch (config 2) is reported per length bucket and in total; the recording pipeline (config 4) runs on a
meeting of --meeting-s seconds with the same segment statistics and reports recording seconds per second
end to end (STFT once, batches of EM + MVDR + iSTFT, cuts), with per-segment context and with
super-segment batching.
"""

from __future__ import annotations

import argparse
import time

import numpy as np

FS, HOP = 16000, 256
PEAK_TFLOPS_F64 = 78.6


def _timeit(torch, fn, n):
    fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / n


def measure_batch(torch, gss, ctx, name, Y, act, T_len, iters, target=None, reps=3):
    S, F, T, D = Y.shape
    K = act.shape[1]
    Yd = torch.from_numpy(Y).cuda()
    ad = torch.from_numpy(act).cuda()
    Td = None if T_len is None else torch.from_numpy(T_len).cuda()
    tgt = torch.zeros(S, dtype=torch.int32).cuda() if target is None else torch.from_numpy(target).cuda()
    ref = torch.zeros(S, dtype=torch.int32).cuda()
    g = gss.gss_cacgmm_em(ctx, Yd, ad, Td, iters)
    X = gss.gss_mvdr(ctx, Yd, g, tgt, ref, Td)
    t_em = _timeit(torch, lambda: gss.gss_cacgmm_em(ctx, Yd, ad, Td, iters, out=g), reps)
    t_mv = _timeit(torch, lambda: gss.gss_mvdr(ctx, Yd, g, tgt, ref, Td, out=X), reps)
    frames = T * S if T_len is None else int(T_len.sum())
    flops = ((3 + 4 * K) * D * D + 3 * D + 30 * K) * F * frames * iters
    return dict(name=name, S=S, T=T, D=D, K=K, iters=iters, frames=frames, em_ms=t_em * 1e3, mvdr_ms=t_mv * 1e3,
                audio_s=frames * HOP / FS, flops=flops, bins_iters=F * frames * iters)


def row(r):
    t = (r["em_ms"] + r["mvdr_ms"]) * 1e-3
    tf = r["flops"] / (r["em_ms"] * 1e-3) / 1e12
    return (f"| {r['name']} | {r['S']} | {r['T']} | {r['D']} | {r['K']} | {r['iters']} | {r['em_ms']:.2f} | "
            f"{r['mvdr_ms']:.3f} | {r['audio_s'] / t:,.0f} | {r['iters'] / (r['em_ms'] * 1e-3):,.0f} | "
            f"{r['bins_iters'] / (r['em_ms'] * 1e-3):.3g} | {tf:.1f} | {100 * tf / PEAK_TFLOPS_F64:.0f} % |")


def sub_records(torch, gss, ctx, synth):
    """EM + MVDR stream time of configurations 0-3 (config 2 per length bucket and in total) as a list of dicts:
    the sub-records of bench.py's JSON line."""
    recs = []

    def rec(r):
        tf = r["flops"] / (r["em_ms"] * 1e-3) / 1e12
        t = (r["em_ms"] + r["mvdr_ms"]) * 1e-3
        return dict(config=r["name"], S=r["S"], Tmax=r["T"], D=r["D"], K=r["K"], em_iters=r["iters"],
                    em_ms=round(r["em_ms"], 3), mvdr_ms=round(r["mvdr_ms"], 3), audio_s_per_s=round(r["audio_s"] / t, 1),
                    em_iters_per_s=round(r["S"] * r["iters"] / (r["em_ms"] * 1e-3), 1),
                    em_alg_tflops=round(tf, 2), em_frac_of_fp64_peak=round(tf / PEAK_TFLOPS_F64, 4))

    for name, seg in (("c0", synth.config0()), ("c1", synth.config1()), ("c3", synth.config3())):
        recs.append(rec(measure_batch(torch, gss, ctx, name, seg.Y[None], seg.activity[None], None, seg.iters)))
    for r in config2_rows(torch, gss, ctx, synth):
        recs.append(rec(r))
    return recs


def config2_rows(torch, gss, ctx, synth, progress=None):
    """Config 2 three ways: each of its four length buckets as a padded batch of its own, their sum, and all 64
    segments in one ragged batch (the kernels skip what lies beyond a segment's length, so nothing is gained by
    bucketing; the one call is the faster way)."""
    rows = []
    T, ns = synth.config2_plan()
    all_segs = [synth.config2_segment(i, T[i], ns[i]) for i in range(len(T))]
    tot = None
    for bi, idx in enumerate(synth.buckets_by_length(T, 4)):
        segs = [all_segs[i] for i in idx]
        Y, act, T_len, target = synth.pad_batch(segs)
        r = measure_batch(torch, gss, ctx, f"c2 bucket {bi}", Y, act, T_len, 15, target)
        rows.append(r)
        if progress:
            progress(r)
        if tot is None:
            tot = dict(r, name="c2 four buckets, summed")
        else:
            for k in ("S", "frames", "em_ms", "mvdr_ms", "audio_s", "flops", "bins_iters"):
                tot[k] += r[k]
            tot["T"] = max(tot["T"], r["T"])
        del Y, act
    rows.append(tot)
    if progress:
        progress(tot)
    Y, act, T_len, target = synth.pad_batch(all_segs)
    del all_segs
    r = measure_batch(torch, gss, ctx, "c2 one call, 64 ragged segments", Y, act, T_len, 15, target)
    rows.append(r)
    if progress:
        progress(r)
    return rows


def sweeps(torch, gss, ctx, synth):
    """The axes of the paper's ablations (Section 5.3) as speed and mask-change sweeps on config 1: EM
    iterations, number of channels, noise class on/off, class-weight mode.  No recognition scores: the
    corpora are not available; what can be reported is the time and how far the masks still move."""
    seg = synth.config1()
    F, T, D, K = seg.shape
    Yd = torch.from_numpy(seg.Y[None]).cuda()
    ad = torch.from_numpy(seg.activity[None]).cuda()
    audio = T * HOP / FS
    g_ref = gss.gss_cacgmm_em(ctx, Yd, ad, None, 20)
    print("| EM iterations | EM ms | audio-s/s (EM) | max abs mask change vs 20 iterations | mean |")
    print("|---:|---:|---:|---:|---:|")
    for it in (1, 2, 3, 5, 10, 15, 20):
        g = gss.gss_cacgmm_em(ctx, Yd, ad, None, it)
        t = _timeit(torch, lambda: gss.gss_cacgmm_em(ctx, Yd, ad, None, it, out=g), 3)
        d = (g - g_ref).abs()
        print(f"| {it} | {t * 1e3:.3f} | {audio / t:,.0f} | {d.max().item():.3f} | {d.mean().item():.4f} |", flush=True)
    print()
    print("| channels | EM ms (20 it.) | MVDR ms | audio-s/s (EM+MVDR) |")
    print("|---:|---:|---:|---:|")
    tgt = torch.zeros(1, dtype=torch.int32).cuda()
    ref = torch.zeros(1, dtype=torch.int32).cuda()
    for d_sub in (2, 4, 6, 8):
        Ys = Yd[..., :d_sub].contiguous()
        g = gss.gss_cacgmm_em(ctx, Ys, ad, None, 20)
        X = gss.gss_mvdr(ctx, Ys, g, tgt, ref)
        te = _timeit(torch, lambda: gss.gss_cacgmm_em(ctx, Ys, ad, None, 20, out=g), 3)
        tm = _timeit(torch, lambda: gss.gss_mvdr(ctx, Ys, g, tgt, ref, out=X), 3)
        print(f"| {d_sub} | {te * 1e3:.3f} | {tm * 1e3:.3f} | {audio / (te + tm):,.0f} |", flush=True)
    print()
    print("| variant | classes | EM ms (20 it.) | max abs change of the speaker masks vs default |")
    print("|---|---:|---:|---:|")
    an = ad[:, :K - 1].contiguous()                                   # without the noise class
    gn = gss.gss_cacgmm_em(ctx, Yd, an, None, 20)
    tn = _timeit(torch, lambda: gss.gss_cacgmm_em(ctx, Yd, an, None, 20, out=gn), 3)
    gu = gss.gss_cacgmm_em(ctx, Yd, ad, None, 20, 0)
    tu = _timeit(torch, lambda: gss.gss_cacgmm_em(ctx, Yd, ad, None, 20, 0, out=gu), 3)
    t0 = _timeit(torch, lambda: gss.gss_cacgmm_em(ctx, Yd, ad, None, 20, out=g_ref), 3)
    print(f"| default (noise class, weights from the masks) | {K} | {t0 * 1e3:.3f} | 0 |")
    print(f"| no noise class | {K - 1} | {tn * 1e3:.3f} | {(gn - g_ref[:, :K - 1]).abs().max().item():.3f} |")
    print(f"| uniform class weights (weight_mode 0) | {K} | {tu * 1e3:.3f} | "
          f"{(gu[:, :K - 1] - g_ref[:, :K - 1]).abs().max().item():.3f} |")
    print()
    # context duration and dereverberation on/off, on a 10-minute meeting through the super-segment pipeline
    from . import pipeline
    dur = 600.0
    x, act_s, (st, en, spk) = synth.meeting(duration_s=dur, n_segments=200)
    xd = torch.from_numpy(x).cuda()
    print("| context per side (s) | WPE | ms (10-minute meeting, super-segments, 15 it.) | audio processed (s) | recording-s/s | "
          "relative change of the enhanced segments vs 15 s, no WPE |")
    print("|---:|---|---:|---:|---:|---:|")
    base_out = None
    rows = []
    for c_s, taps in ((15.0, 0), (5.0, 0), (10.0, 0), (20.0, 0), (15.0, 10)):
        c = int(c_s * FS)

        def run():
            return pipeline.enhance_recording_super(ctx, xd, act_s, st, en, spk, c, c, max_batch_s=50.0, iters=15,
                                                    wpe_taps=taps)

        run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        outs, info = run()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        flat = torch.cat(outs)
        if base_out is None:
            base_out = flat
        rel = ((flat - base_out).norm() / base_out.norm()).item()
        proc = float(np.sum(info["T"])) * HOP / FS
        rows.append((c_s, taps, dt, proc, rel))
    for c_s, taps, dt, proc, rel in sorted(rows, key=lambda r: (r[1], r[0])):
        print(f"| {c_s:.0f} | {'10 taps, delay 2, 3 it.' if taps else 'off'} | {dt * 1e3:.1f} | {proc:.0f} | {dur / dt:,.0f} | {rel:.3f} |",
              flush=True)


def wpe_rows(torch, gss, ctx, synth, large=False):
    """gss_wpe on a reverberant stand-in of config 1's shape (513 x 1560 x 8; large: config 3's, 513 x 1500 x
    24), 10 taps, delay 2: time per call, audio seconds per second, and the algorithmic fp64 rate of the
    covariance kernel (8 flops per complex multiply-add, N(N+1)/2 + N D entries per frame, N = D taps)."""
    Y, _, _ = synth.reverberant_stft(F=513, T=1500, D=24, seed=3) if large else synth.reverberant_stft(F=513, T=1560, D=8, seed=0)
    F, T, D = Y.shape
    taps, delay = 10, 2
    N = D * taps
    Yd = torch.from_numpy(Y[None]).cuda()
    X = gss.gss_wpe(ctx, Yd, None, taps, delay, 3)
    audio = T * HOP / FS
    print(f"{D} channels, {T} frames:")
    print("| WPE iterations | ms | audio-s/s | covariance kernel: launches, mean us, TFLOP/s (alg.), of 78.6 |")
    print("|---:|---:|---:|---|")
    for it in (1, 2, 3):
        t = _timeit(torch, lambda: gss.gss_wpe(ctx, Yd, None, taps, delay, it, out=X), 5)
        ctx.profile_enable(True)
        gss.gss_wpe(ctx, Yd, None, taps, delay, it, out=X)
        ms, n = ctx.profile_get(2)
        ctx.profile_enable(False)
        flops = (N * (N + 1) // 2 + N * D) * 8 * F * T
        tf = flops / (ms / n * 1e-3) / 1e12
        print(f"| {it} | {t * 1e3:.3f} | {audio / t:,.0f} | {n}, {ms / n * 1e3:.1f}, {tf:.1f}, {100 * tf / PEAK_TFLOPS_F64:.0f} % |",
              flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--meeting-s", type=float, default=300.0, help="duration of the config-4 meeting (0 = skip)")
    ap.add_argument("--sweeps", action="store_true",
                    help="only the parameter sweeps on config 1 (iterations, channels, noise class, weight mode)")
    ap.add_argument("--wpe", action="store_true", help="only the dereverberation timing (config 1's shape)")
    ap.add_argument("--wpe-large", action="store_true", help="only the dereverberation timing at config 3's shape (24 channels)")
    ap.add_argument("--config", choices=("c0", "c1", "c2", "c3"), default=None,
                    help="only this configuration (for a kernel trace of its own)")
    a = ap.parse_args()

    import torch
    from . import binding as gss
    from . import pipeline, synth

    ctx = gss.Context(0)
    if a.sweeps:
        sweeps(torch, gss, ctx, synth)
        ctx.close()
        return
    if a.wpe or a.wpe_large:
        wpe_rows(torch, gss, ctx, synth, large=a.wpe_large)
        ctx.close()
        return
    print("| config | S | Tmax | D | K | iters | EM ms | MVDR ms | audio-s/s (EM+MVDR) | EM iters/s | bin-iters/s | "
          "EM TFLOP/s (alg.) | of 78.6 |")
    print("|---|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|")
    for name, make in (("c0", synth.config0), ("c1", synth.config1), ("c3", synth.config3)):
        if a.config in (None, name):
            seg = make()
            print(row(measure_batch(torch, gss, ctx, name, seg.Y[None], seg.activity[None], None, seg.iters)), flush=True)
    if a.config in (None, "c2"):
        config2_rows(torch, gss, ctx, synth, progress=lambda r: print(row(r), flush=True))

    if a.meeting_s > 0 and a.config is None:
        n_seg = max(4, int(round(1200 * a.meeting_s / 3600.0)))
        x, act_s, (st, en, spk) = synth.meeting(duration_s=a.meeting_s, n_segments=n_seg)
        xd = torch.from_numpy(x).cuda()
        ctx_samples = int(7.5 * FS)

        def run():
            return pipeline.enhance_recording(ctx, xd, act_s, st, en, spk, ctx_samples, ctx_samples, iters=15)

        def timed(fn):
            """Median wall time of three calls after a warm-up call (the allocator settles), and the last result."""
            fn()
            torch.cuda.synchronize()
            ts = []
            for _ in range(3):
                t0 = time.perf_counter()
                res = fn()
                torch.cuda.synchronize()
                ts.append(time.perf_counter() - t0)
            return sorted(ts)[1], res

        dt, (outs, fr) = timed(run)
        proc = float(np.sum(fr["n_frames"])) * HOP / FS
        def run_super():
            return pipeline.enhance_recording_super(ctx, xd, act_s, st, en, spk, ctx_samples, ctx_samples,
                                                    max_batch_s=50.0, iters=15)

        del outs
        dts, (_, info) = timed(run_super)
        procs = float(np.sum(info["T"])) * HOP / FS
        print(f"\nc4 pipeline: {a.meeting_s:.0f} s meeting, 8 channels, {n_seg} segments with 7.5 s of context per side "
              f"({proc:.0f} s of audio processed), 15 iterations: {dt * 1e3:.1f} ms end to end = "
              f"{a.meeting_s / dt:,.0f} recording-s/s, {proc / dt:,.0f} processed audio-s/s "
              f"(includes the host-side batch assembly)")
        print(f"the same with super-segments (same-speaker segments concatenated up to 50 s, one context window each: "
              f"{len(info['supers'])} super-segments, {procs:.0f} s of audio processed): {dts * 1e3:.1f} ms = "
              f"{a.meeting_s / dts:,.0f} recording-s/s")

        def run_super_wpe():
            return pipeline.enhance_recording_super(ctx, xd, act_s, st, en, spk, ctx_samples, ctx_samples,
                                                    max_batch_s=50.0, iters=15, wpe_taps=10, wpe_delay=2, wpe_iters=3)

        dtw, _ = timed(run_super_wpe)
        print(f"super-segments with dereverberation (WPE, 10 taps, delay 2, 3 iterations) before the mask estimation: "
              f"{dtw * 1e3:.1f} ms = {a.meeting_s / dtw:,.0f} recording-s/s (WPE adds {(dtw - dts) * 1e3:.1f} ms)")
    ctx.close()


if __name__ == "__main__":
    main()
