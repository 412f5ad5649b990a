"""Recording-level driver over the C-ABI calls: STFT of the whole recording once, context-extended
segments cut out of it as frame ranges, bucketed by length and padded into batches, then
gss_cacgmm_em -> gss_mvdr -> gss_istft per batch and the target region cut out of each result.

Only orchestration and memory plumbing (slicing, padding, copies) happen here, with torch as the
allocator; every step of the method runs in the library's kernels.  The bookkeeping integers come from
gss_frames_from_segments / gss_frame_activity.
"""

from __future__ import annotations

import numpy as np

from . import binding as gss

HOP = 256
N_FFT = 1024


def plan_batches(n_frames, max_batch_frames=200_000, max_segments=64):
    """Sort segments by length (longest first) and cut the order into batches whose padded size
    (segments x longest) stays below max_batch_frames.  Returns a list of index lists."""
    order = np.argsort(-np.asarray(n_frames), kind="stable")
    batches, cur = [], []
    for i in order:
        tmax = n_frames[cur[0]] if cur else n_frames[i]
        if cur and ((len(cur) + 1) * tmax > max_batch_frames or len(cur) >= max_segments):
            batches.append(cur)
            cur = []
        cur.append(int(i))
    if cur:
        batches.append(cur)
    return batches


def enhance_recording(ctx, x, act_samples, seg_start, seg_end, seg_spk, ctx_left, ctx_right, iters=15,
                      weight_mode=1, max_batch_frames=200_000, Yrec=None):
    """x[D, N] float32 CUDA tensor, act_samples[n_spk, N] uint8 (host), segments (host arrays).

    Classes per segment: the n_spk speakers in recording order plus a noise class that is always active
    (K = n_spk + 1); the target class is the segment's speaker.  Returns a list of 1-D float32 CUDA
    tensors (the enhanced target region of every segment) and a dict of bookkeeping arrays.
    """
    import torch

    D, N = x.shape
    n_spk = act_samples.shape[0]
    K = n_spk + 1
    if Yrec is None:
        Yrec = gss.gss_stft(ctx, x.reshape(1, D, N).contiguous())          # [1, F, Trec, D]
    F = Yrec.shape[1]
    fr = gss.gss_frames_from_segments(seg_start, seg_end, N, ctx_left, ctx_right, HOP)
    n_seg = len(seg_start)
    outputs = [None] * n_seg
    refs = np.zeros(n_seg, dtype=np.int32)
    for batch in plan_batches(fr["n_frames"], max_batch_frames):
        S = len(batch)
        Tmax = int(max(fr["n_frames"][i] for i in batch))
        Y = torch.zeros((S, F, Tmax, D), dtype=torch.complex64, device=x.device)
        act = np.zeros((S, K, Tmax), dtype=np.uint8)
        T_len = np.zeros(S, dtype=np.int32)
        for b, i in enumerate(batch):
            f0, nf = int(fr["frame0"][i]), int(fr["n_frames"][i])
            Y[b, :, :nf] = Yrec[0, :, f0:f0 + nf]
            act[b, :n_spk, :nf] = gss.gss_frame_activity(act_samples, f0, nf, HOP)
            act[b, n_spk, :nf] = 1
            T_len[b] = nf
        act_d = torch.from_numpy(act).to(x.device)
        T_d = torch.from_numpy(T_len).to(x.device)
        tgt = torch.from_numpy(np.asarray([seg_spk[i] for i in batch], dtype=np.int32)).to(x.device)
        ref = torch.full((S,), -1, dtype=torch.int32, device=x.device)
        gamma = gss.gss_cacgmm_em(ctx, Y, act_d, T_d, iters, weight_mode)
        X = gss.gss_mvdr(ctx, Y, gamma, tgt, ref, T_d)
        xh = gss.gss_istft(ctx, X, (Tmax - 3) * HOP)
        ref_h = ref.cpu().numpy()
        for b, i in enumerate(batch):
            outputs[i] = xh[b, int(fr["cut_start"][i]):int(fr["cut_end"][i])]
            refs[i] = ref_h[b]
    fr["ref"] = refs
    return outputs, fr
