#!/usr/bin/env python3
"""Benchmark of the GSS hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload (config 4, the largest single-GPU configuration): one synthetic one-hour, 8-channel, 16 kHz meeting
with 4 speakers and 1200 diarization segments (1-20 s each), every segment extended by 7.5 s of context on
either side.  One step = one pass of the whole hot path over the recording through the C ABI, inputs resident
in HBM before the timed region: gss_stft of the recording, then per batch of segments (read in place as frame
ranges of that STFT) gss_cacgmm_em_frames (15 iterations, K = 5 classes) -> gss_mvdr_frames -> gss_istft, and
the cut of every target region.

Prints ONE JSON line: processed audio-seconds per second (context included, since it is processed) over the
whole step, recording seconds per second, the roofline figures of the dominant kernel (the accumulating EM
pass; its launches are timed with HIP events on their stream inside the library during a second run of the
same K steps), the other configurations as sub-records (EM + MVDR stream time), and the CPU oracle timed on
the host on a stated sample.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FS, HOP = 16000, 256
# Published MI355X vector peak for the arithmetic type of the EM kernels (fp64 FMA): 78.6 TFLOP/s.
PEAK_TFLOPS_F64 = 78.6
# HBM bytes per launch of the dominant kernel on the one-hour meeting, written by
# `python -m paper_2212_05271_amd.profile_summary traffic` from rocprofv3 --pmc runs of this script (FETCH_SIZE /
# WRITE_SIZE, scaled by the copy-kernel calibration).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "em_pass_hbm_traffic.md")


def em_pass_flops_per_bin(D, K):
    """Algorithmic flops of one EM iteration per time-frequency bin: (3 + 4K) D^2 + 3 D + 30 K."""
    return (3 + 4 * K) * D * D + 3 * D + 30 * K


def cpu_baseline(x, act_s, st, en, spk, fr, ctx_samples, iters, budget_s):
    """The float64 oracle, as it stands, on a sample of the same workload: the shortest segments in turn, every
    8th frequency bin, STFT of the segment's span -> EM -> MVDR -> iSTFT, until the time budget is used."""
    import numpy as np
    import psutil
    from oracle import gss_oracle as o

    proc = psutil.Process()
    c0 = proc.cpu_times()
    t0 = time.perf_counter()
    N = x.shape[1]
    # segments whose span stays 768 samples (the reach of their outermost frames) clear of both ends of the
    # recording: the oracle then needs the STFT of that span only
    inner = [i for i in np.argsort(fr["n_frames"], kind="stable")
             if fr["ext_start"][i] >= 768 and fr["ext_end"][i] + 768 <= N]
    done_frames, n_done, bins_step = 0, 0, 8
    F = 513
    fs = np.arange(0, F, bins_step)
    for i in inner:
        s0, e0 = int(fr["ext_start"][i]) - 768, int(fr["ext_end"][i]) + 768
        f0, nf = int(fr["frame0"][i]), int(fr["n_frames"][i])
        Ysub = o.stft_channels_last(x[:, s0:e0]).astype(np.complex64)   # its frame u is recording frame u + s0 / 256
        u0 = f0 - s0 // HOP
        Ys = Ysub[:, u0:u0 + nf]
        act = np.concatenate([o.frame_activity(act_s, f0, nf), np.ones((1, nf), np.uint8)])
        g = o.cacgmm_em(Ys[fs], act, iters)
        X, _, _ = o.mvdr(Ys[fs], g, int(spk[i]))
        Xfull = np.zeros((F, nf), dtype=np.complex128)
        Xfull[fs] = X
        o.istft(Xfull, (nf - 3) * HOP)
        done_frames += nf
        n_done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    wall = time.perf_counter() - t0
    c1 = proc.cpu_times()
    cpu = (c1.user + c1.system) - (c0.user + c0.system)
    frac = len(fs) / F
    return dict(value=done_frames * HOP / FS * frac / wall, unit="audio-s/s", cores=max(1, int(round(cpu / wall))),
                kind="oracle", seconds=round(wall, 2), cpu_seconds=round(cpu, 2),
                sample=f"the {n_done} shortest of the 1200 segments ({done_frames} frames with context), every "
                       f"{bins_step}th frequency bin ({len(fs)} of {F}): STFT of the span, {iters} EM iterations, "
                       f"MVDR, iSTFT; rate scaled by the bin fraction (bins and segments are independent)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="time budget of the oracle baseline (0 = skip)")
    ap.add_argument("--no-subconfigs", action="store_true", help="skip the sub-records of configurations 0-3")
    ap.add_argument("--meeting-s", type=float, default=3600.0, help="duration of the meeting (config 4 = 3600)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run three 256 MiB device-to-device copies (the known-size kernel that the "
                         "FETCH_SIZE / WRITE_SIZE counters are scaled by) and exit")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (segments are independent and would be sharded without any "
              "communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2212_05271_amd import binding as gss
    from paper_2212_05271_amd import measure_configs, pipeline, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    if a.copy_calibration:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 256 << 20, "bytes_written": 256 << 20, "copies": 3}}))
        return
    ctx = gss.Context(0)

    # set-up (untimed): the synthetic meeting, resident in HBM
    n_seg = max(4, int(round(1200 * a.meeting_s / 3600.0)))
    x, act_s, (st, en, spk) = synth.meeting(duration_s=a.meeting_s, n_segments=n_seg)
    D, N = x.shape
    K, iters, F = act_s.shape[0] + 1, 15, 513
    ctx_samples = int(7.5 * FS)
    xd = torch.from_numpy(x).to(dev)
    torch.cuda.synchronize()

    def step():
        return pipeline.enhance_recording(ctx, xd, act_s, st, en, spk, ctx_samples, ctx_samples, iters=iters)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        outs, fr = step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / a.steps * 1e3
    frames = int(np.sum(fr["n_frames"]))
    audio_s = frames * HOP / FS
    value = audio_s * a.steps / elapsed
    status = ctx.get_status()
    peak_gb = torch.cuda.max_memory_allocated() / 1e9
    del outs

    # second run of the same K steps: the launches of the dominant kernel bracketed by HIP events on their stream
    ctx.profile_enable(True)
    ctx.profile_get(0), ctx.profile_get(1)
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    pass_ms, pass_n = ctx.profile_get(0)
    fac_ms, fac_n = ctx.profile_get(1)
    ctx.profile_enable(False)

    flops_total = em_pass_flops_per_bin(D, K) * F * frames * iters * a.steps
    achieved = flops_total / (pass_ms * 1e-3) / 1e12
    traffic = None
    if os.path.exists(TRAFFIC_FILE) and abs(a.meeting_s - 3600.0) < 1e-6:
        import re
        m = re.search(r"^bytes per launch \(FETCH_SIZE \+ WRITE_SIZE, calibrated\): (\d+)", open(TRAFFIC_FILE).read(), re.M)
        if m:
            traffic = int(m.group(1))
    roofline = dict(bound="alu", kernel="em_whole_small<8,5> (all EM iterations of a batch of segments in one launch: one "
                    "wavefront per segment and frequency)", achieved=round(achieved, 3), peak=PEAK_TFLOPS_F64, unit="TFLOP/s",
                    frac=round(achieved / PEAK_TFLOPS_F64, 4), traffic=traffic,
                    flops_per_launch=round(flops_total / max(pass_n, 1)), avg_launch_us=round(pass_ms / max(pass_n, 1) * 1e3, 2),
                    launches=pass_n,
                    note="algorithmic flops ((3 + 4K) D^2 + 3D + 30K per time-frequency bin and iteration, K = 5 classes, "
                         "15 iterations; the final mask pass and the factorisations inside the kernel are not counted) "
                         "over the summed duration of the launches; fp64 vector FMA peak (the kernel's arithmetic; packed "
                         "fp32 is switched off for this library).  The kernel skips the classes that are inactive in a "
                         "whole 64-frame tile, so it executes fewer flops than the formula counts.")

    out = {
        "metric": "audio_sec_per_sec_cacgmm_em_mvdr",
        "value": round(value, 2),
        "unit": "audio-s/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": f"config 4: one synthetic {a.meeting_s:.0f} s, 8-channel, 16 kHz meeting, 4 speakers + noise "
                               f"class (K=5), {n_seg} segments of 1-20 s each with 7.5 s of context per side; step = STFT of "
                               "the recording + per batch EM (15 iterations) + MVDR + iSTFT + cut; value counts the audio "
                               "processed, context included",
                   "F": F, "D": D, "K": K, "em_iters": iters, "segments": n_seg, "frames_processed": frames,
                   "audio_s_processed": round(audio_s, 1), "recording_s": a.meeting_s},
        "recording_s_per_s": round(a.meeting_s * a.steps / elapsed, 1),
        "em_iters_per_s": round(n_seg * iters * a.steps / elapsed, 1),
        "tf_bin_iters_per_s": round(F * frames * iters * a.steps / elapsed, 1),
        "em_kernel_ms_per_step": {"em": round(pass_ms / a.steps, 2), "separate_factor_launches": round(fac_ms / a.steps, 2),
                                  "note": "from the second, event-instrumented run of the same steps"},
        "peak_device_memory_gb": round(peak_gb, 2),
        "status_word": status,
        "roofline": roofline,
    }
    if not a.no_subconfigs:
        out["other_configs"] = measure_configs.sub_records(torch, gss, ctx, synth)
    if a.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(x, act_s, st, en, spk, fr, ctx_samples, iters, a.cpu_seconds)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
