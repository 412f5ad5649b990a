#!/usr/bin/env python3
"""Benchmark of the GSS hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step = one pass of the whole hot path over the workload: gss_stft -> gss_cacgmm_em (20 iterations)
-> gss_mvdr -> gss_istft, all through the C ABI, inputs resident in HBM before the timed region.

Workload (config 1): a single long segment, 8-channel circular array, F = 513, T = 1560 frames (10 s
target + 15 s context = 24.96 s of audio), 4 speakers + noise class (K = 5), diffuse noise at 5 dB.  The
configuration is defined in the STFT domain; its time-domain input is obtained once, at set-up, by
inverting each channel of the synthetic STFT, so that the timed step can start from samples.

Prints ONE JSON line: audio-seconds per second over the whole step, the EM iterations per second, the
roofline figures of the dominant kernel (the accumulating EM pass, timed with HIP events on its stream in
a second run of the same K steps), and the CPU oracle timed on the host on a stated sample.
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
# HBM bytes per launch of the accumulating EM pass on this workload, from rocprofv3 --pmc runs
# (FETCH_SIZE + WRITE_SIZE in KiB, each scaled by the copy-kernel calibration).
EM_PASS_TRAFFIC_BYTES = (53273 + 1322) * 1024   # profiles/em_config1_hbm_traffic.md


def em_pass_flops(F, T, D, K):
    """Algorithmic flops of one EM iteration: (3 + 4K) D^2 + 3 D + 30 K per time-frequency bin."""
    return ((3 + 4 * K) * D * D + 3 * D + 30 * K) * F * T


def cpu_baseline(seg, x_np, n_iters, bins_step):
    """The float64 oracle, as it stands, on every bins_step-th frequency bin of the same workload."""
    import numpy as np
    import psutil
    from oracle import gss_oracle as o

    proc = psutil.Process()
    c0 = proc.cpu_times()
    t0 = time.perf_counter()
    Y = o.stft_channels_last(x_np[0]).astype(np.complex64)          # the stage boundary type
    fs = np.arange(0, Y.shape[0], bins_step)
    g = o.cacgmm_em(Y[fs], seg.activity, n_iters)
    X, ref, _ = o.mvdr(Y[fs], g, seg.target)
    Xfull = np.zeros(Y.shape[:2], dtype=np.complex128)
    Xfull[fs] = X
    o.istft(Xfull, x_np.shape[-1])
    wall = time.perf_counter() - t0
    c1 = proc.cpu_times()
    cpu = (c1.user + c1.system) - (c0.user + c0.system)
    audio_s = seg.Y.shape[1] * HOP / FS
    frac = len(fs) / Y.shape[0]
    return dict(value=audio_s * frac / wall, unit="audio-s/s", cores=max(1, int(round(cpu / wall))),
                kind="oracle", seconds=round(wall, 2), cpu_seconds=round(cpu, 2),
                sample=f"every {bins_step}th frequency bin ({len(fs)} of {Y.shape[0]}) of the same segment, all "
                       f"{n_iters} EM iterations + MVDR; STFT/iSTFT on all bins; rate scaled by the bin fraction")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--cpu-bins-step", type=int, default=2, help="oracle baseline runs every n-th bin (0 = skip)")
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
    from paper_2212_05271_amd import synth

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

    seg = synth.config1()
    F, T, D, K = seg.shape
    iters = seg.iters
    N = (T - 3) * HOP
    audio_s = T * HOP / FS

    # set-up (untimed): time-domain input from the synthetic STFT, channel by channel
    Yc = torch.from_numpy(np.ascontiguousarray(np.moveaxis(seg.Y, 2, 0))).to(dev)          # [D, F, T]
    x = gss.gss_istft(ctx, Yc, N).reshape(1, D, N).contiguous()
    act = torch.from_numpy(seg.activity[None]).to(dev)
    target = torch.zeros(1, dtype=torch.int32, device=dev)
    ref = torch.full((1,), -1, dtype=torch.int32, device=dev)
    Y = torch.empty((1, F, T, D), dtype=torch.complex64, device=dev)
    gamma = torch.empty((1, K, F, T), dtype=torch.float32, device=dev)
    X = torch.empty((1, F, T), dtype=torch.complex64, device=dev)
    xh = torch.empty((1, N), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()

    def step(events=None):
        ref.fill_(-1)
        if events is not None:
            events[0].record()
        gss.gss_stft(ctx, x, out=Y)
        if events is not None:
            events[1].record()
        gss.gss_cacgmm_em(ctx, Y, act, None, iters, 1, out=gamma)
        if events is not None:
            events[2].record()
        gss.gss_mvdr(ctx, Y, gamma, target, ref, out=X)
        if events is not None:
            events[3].record()
        gss.gss_istft(ctx, X, N, out=xh)
        if events is not None:
            events[4].record()

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / a.steps * 1e3
    value = audio_s * a.steps / elapsed

    # second run of the same K steps: stage times (torch events on the current stream, which is the stream
    # the library launches on) and the dominant kernel's launches bracketed by HIP events inside the library
    ctx.profile_enable(True)
    ctx.profile_get(0), ctx.profile_get(1)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(a.steps)]
    for i in range(a.steps):
        step(evs[i])
    torch.cuda.synchronize()
    pass_ms, pass_n = ctx.profile_get(0)
    fac_ms, fac_n = ctx.profile_get(1)
    ctx.profile_enable(False)
    stage = [sum(e[j].elapsed_time(e[j + 1]) for e in evs) / a.steps for j in range(4)]
    em_ms = stage[1]

    flops = em_pass_flops(F, T, D, K)
    pass_avg_ms = pass_ms / max(pass_n, 1)
    achieved = flops / (pass_avg_ms * 1e-3) / 1e12
    roofline = dict(bound="alu", kernel="em_pass_small<8,5> (accumulating EM pass, one launch per EM iteration)",
                    achieved=round(achieved, 3), peak=PEAK_TFLOPS_F64, unit="TFLOP/s",
                    frac=round(achieved / PEAK_TFLOPS_F64, 4), traffic=EM_PASS_TRAFFIC_BYTES,
                    flops_per_launch=flops, avg_launch_us=round(pass_avg_ms * 1e3, 2), launches=pass_n,
                    note="fp64 vector FMA peak; packed fp32 is switched off for this library, and fp64 FMA issues "
                         "at the unpacked-fp32 rate")

    out = {
        "metric": "audio_sec_per_sec_cacgmm_em_mvdr",
        "value": round(value, 2),
        "unit": "audio-s/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": "config 1: single long segment, 8-ch circular array, F=513, T=1560 (24.96 s audio), "
                               "4 speakers + noise (K=5), diffuse noise 5 dB, 20 EM iterations, MVDR target 0; "
                               "step = STFT + EM + MVDR + iSTFT",
                   "F": F, "T": T, "D": D, "K": K, "em_iters": iters, "segments": 1},
        "em_iters_per_s": round(iters / (em_ms * 1e-3), 1),
        "tf_bin_iters_per_s": round(F * T * iters / (em_ms * 1e-3), 1),
        "stage_ms": {"stft": round(stage[0], 4), "em": round(stage[1], 4), "mvdr": round(stage[2], 4),
                     "istft": round(stage[3], 4)},
        "em_factor_avg_us": round(fac_ms / max(fac_n, 1) * 1e3, 2),
        "roofline": roofline,
    }
    if a.cpu_bins_step > 0:
        out["cpu_baseline"] = cpu_baseline(seg, x.cpu().numpy(), iters, a.cpu_bins_step)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
