"""Recording-level drivers over the C-ABI calls: STFT of the whole recording once, segments cut out of it as
frame ranges, bucketed by length and padded into batches, then gss_cacgmm_em -> gss_mvdr -> gss_istft per
batch and the target region cut out of each result.

enhance_recording         every segment on its own, extended by its own context (padded batching);
enhance_recording_super   segments of one speaker concatenated along time into super-segments that share
                          one context window and one set of statistics (arXiv 2212.05271, Section 3,
                          "Segment batching"); the super-segments are then batched with padding like above.

Only orchestration and memory plumbing (slicing, padding, copies) happen here, with torch as the
allocator; every step of the method runs in the library's kernels.  The bookkeeping integers come from
gss_frames_from_segments / gss_frame_activity.
"""

from __future__ import annotations

import numpy as np

from . import binding as gss

HOP = 256
N_FFT = 1024


def plan_batches(n_frames, max_batch_frames=400_000, max_segments=128):
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
                      weight_mode=1, max_batch_frames=400_000, Yrec=None, wpe_taps=0, wpe_delay=2, wpe_iters=3):
    """x[D, N] float32 CUDA tensor, act_samples[n_spk, N] uint8 (host), segments (host arrays).

    Classes per segment: the n_spk speakers in recording order plus a noise class that is always active
    (K = n_spk + 1); the target class is the segment's speaker.  The recording is transformed once; a segment
    (with its context) is a frame range of that STFT and is handed to the library as such
    (gss_cacgmm_em_frames / gss_mvdr_frames): nothing is copied or padded on the way in.  wpe_taps > 0
    dereverberates every segment's STFT (context included) with gss_wpe before the masks are estimated; masks
    and beamformer then work on the dereverberated copy (Section 2.1).  Returns a list of 1-D float32 CUDA
    tensors (the enhanced target region of every segment) and a dict of bookkeeping arrays.
    """
    import torch

    D, N = x.shape
    n_spk = act_samples.shape[0]
    K = n_spk + 1
    if Yrec is None:
        Yrec = gss.gss_stft(ctx, x.reshape(1, D, N).contiguous())          # [1, F, Trec, D]
    Yr = Yrec[0]
    F = Yr.shape[0]
    fr = gss.gss_frames_from_segments(seg_start, seg_end, N, ctx_left, ctx_right, HOP)
    n_seg = len(seg_start)
    outputs = [None] * n_seg
    # frame-level activity of the whole recording once; a segment's rows are a slice of it
    act_rec = gss.gss_frame_activity(act_samples, 0, Yr.shape[1], HOP)
    batches = plan_batches(fr["n_frames"], max_batch_frames)
    ref_all = torch.full((n_seg,), -1, dtype=torch.int32, device=x.device)
    order = np.concatenate([np.asarray(b, dtype=np.int64) for b in batches]) if batches else np.zeros(0, np.int64)
    frame0_d = torch.from_numpy(np.ascontiguousarray(fr["frame0"][order])).to(x.device)
    tlen_d = torch.from_numpy(np.ascontiguousarray(fr["n_frames"][order])).to(x.device)
    tgt_d = torch.from_numpy(np.ascontiguousarray(np.asarray(seg_spk, dtype=np.int32)[order])).to(x.device)
    pos = 0
    for batch in batches:
        S = len(batch)
        Tmax = int(max(fr["n_frames"][i] for i in batch))
        act = np.zeros((S, K, Tmax), dtype=np.uint8)
        for b, i in enumerate(batch):
            f0, nf = int(fr["frame0"][i]), int(fr["n_frames"][i])
            act[b, :n_spk, :nf] = act_rec[:, f0:f0 + nf]
            act[b, n_spk, :nf] = 1
        act_d = torch.from_numpy(act).to(x.device)
        f0_d, T_d, tgt = frame0_d[pos:pos + S], tlen_d[pos:pos + S], tgt_d[pos:pos + S]
        ref = torch.full((S,), -1, dtype=torch.int32, device=x.device)
        if wpe_taps > 0:
            Y = torch.zeros((S, F, Tmax, D), dtype=torch.complex64, device=x.device)
            for b, i in enumerate(batch):
                f0, nf = int(fr["frame0"][i]), int(fr["n_frames"][i])
                Y[b, :, :nf] = Yr[:, f0:f0 + nf]
            Y = gss.gss_wpe(ctx, Y, T_d, wpe_taps, wpe_delay, wpe_iters)
            gamma = gss.gss_cacgmm_em(ctx, Y, act_d, T_d, iters, weight_mode)
            X = gss.gss_mvdr(ctx, Y, gamma, tgt, ref, T_d)
        else:
            gamma = gss.gss_cacgmm_em_frames(ctx, Yr, f0_d, act_d, T_d, iters, weight_mode)
            X = gss.gss_mvdr_frames(ctx, Yr, f0_d, gamma, tgt, ref, T_d)
        xh = gss.gss_istft(ctx, X, (Tmax - 3) * HOP)
        ref_all[pos:pos + S] = ref
        for b, i in enumerate(batch):
            outputs[i] = xh[b, int(fr["cut_start"][i]):int(fr["cut_end"][i])]
        pos += S
    refs = np.zeros(n_seg, dtype=np.int32)
    refs[order] = ref_all.cpu().numpy()
    fr["ref"] = refs
    return outputs, fr


def block_spans(seg_start, seg_end, block):
    """Consecutive blocks of `block` samples that tile [seg_start, seg_end) (the last one may be shorter)."""
    s, e, n = int(seg_start), int(seg_end), int(block)
    if n <= 0:
        raise ValueError("block must be positive")
    return [(b, min(b + n, e)) for b in range(s, e, n)]


def enhance_recording_blocks(ctx, x, act_samples, seg_start, seg_end, seg_spk, block, history, iters=15,
                             weight_mode=1, max_batch_frames=400_000, Yrec=None):
    """Block-wise processing for speakers that move (Section 3, "Segment batching", keeps one set of statistics
    and one reference channel per batch for stationary speakers only; Section 1 cites block-online GSS): every
    segment is cut into consecutive blocks of `block` samples, and every block is enhanced as a segment of its
    own from the span [block start - history, block end): own masks, own filter, own reference channel, nothing
    after the block's last frame.  The blocks of all segments are independent, so they are batched together
    like any other segments.  Returns (outputs, info): outputs[i] the enhanced segment i (its blocks joined),
    info the block table (segment, start, end, reference channel)."""
    import torch

    b0s, b1s, owner = [], [], []
    for i in range(len(seg_start)):
        for b0, b1 in block_spans(seg_start[i], seg_end[i], block):
            b0s.append(b0); b1s.append(b1); owner.append(i)
    b0s, b1s = np.asarray(b0s, np.int64), np.asarray(b1s, np.int64)
    spk_b = np.asarray([seg_spk[i] for i in owner], dtype=np.int32)
    outs_b, fr = enhance_recording(ctx, x, act_samples, b0s, b1s, spk_b, int(history), 0, iters=iters,
                                   weight_mode=weight_mode, max_batch_frames=max_batch_frames, Yrec=Yrec)
    outputs = []
    pos = 0
    for i in range(len(seg_start)):
        n = sum(1 for o_ in owner if o_ == i)
        outputs.append(torch.cat(outs_b[pos:pos + n]) if n > 1 else outs_b[pos])
        pos += n
    info = dict(segment=np.asarray(owner, np.int32), start=b0s, end=b1s, ref=fr["ref"], frames=fr)
    return outputs, info


def plan_super_segments(seg_start, seg_end, seg_spk, max_batch_samples):
    """Packs the segments of each speaker, in time order, into super-segments: a super-segment takes the
    speaker's next segment as long as the summed duration of its members stays within max_batch_samples
    (a segment longer than that forms a super-segment alone; max_batch_samples <= 0 makes every segment a
    super-segment of its own: the option for non-stationary speakers of Section 3, segment batching).  Returns a list of index lists, ordered by the start of
    their first member."""
    seg_start = np.asarray(seg_start, dtype=np.int64)
    seg_end = np.asarray(seg_end, dtype=np.int64)
    seg_spk = np.asarray(seg_spk)
    supers = []
    for spk in np.unique(seg_spk):
        idx = [int(i) for i in np.flatnonzero(seg_spk == spk)]
        idx.sort(key=lambda i: (int(seg_start[i]), int(seg_end[i]), i))
        cur, dur = [], 0
        for i in idx:
            d = int(seg_end[i] - seg_start[i])
            if cur and (max_batch_samples <= 0 or dur + d > max_batch_samples):
                supers.append(cur)
                cur, dur = [], 0
            cur.append(i)
            dur += d
        if cur:
            supers.append(cur)
    supers.sort(key=lambda m: (int(seg_start[m[0]]), m[0]))
    return supers


def super_segment_pieces(members, seg_start, seg_end, n_samples, ctx_left, ctx_right):
    """Sample spans of one super-segment, in order: one context span before its first member, the members
    themselves (no context of their own), one context span after its last member; spans are clipped to the
    recording and empty ones dropped.  Returns (starts, ends, member_of) with member_of = segment index or -1
    for a context span."""
    first, last = members[0], members[-1]
    starts, ends, member_of = [], [], []
    lo = max(0, int(seg_start[first]) - int(ctx_left))
    if lo < int(seg_start[first]):
        starts.append(lo); ends.append(int(seg_start[first])); member_of.append(-1)
    for i in members:
        starts.append(int(seg_start[i])); ends.append(int(seg_end[i])); member_of.append(int(i))
    hi = min(int(n_samples), int(seg_end[last]) + int(ctx_right))
    if hi > int(seg_end[last]):
        starts.append(int(seg_end[last])); ends.append(hi); member_of.append(-1)
    return np.asarray(starts, np.int64), np.asarray(ends, np.int64), member_of


def merge_runs(ext_start, ext_end, hop=HOP):
    """Hop-snapped spans in time order -> runs of consecutive frames.  Spans that touch or overlap are merged
    (a span that starts at or before the end of the run so far extends it), so that every frame of the recording
    appears at most once per run.  Returns a list of (first frame, number of frames, indices of the spans in the
    run); a run of samples [a, b) is covered by the frames a / hop .. b / hop + 2."""
    runs = []
    cur_a = cur_b = None
    idx = []
    for p, (a, b) in enumerate(zip(ext_start, ext_end)):
        a, b = int(a), int(b)
        if cur_a is not None and a <= cur_b:
            cur_b = max(cur_b, b)
            idx.append(p)
        else:
            if cur_a is not None:
                runs.append((cur_a // hop, (cur_b - cur_a) // hop + 3, idx))
            cur_a, cur_b, idx = a, b, [p]
    if cur_a is not None:
        runs.append((cur_a // hop, (cur_b - cur_a) // hop + 3, idx))
    return runs


def enhance_recording_super(ctx, x, act_samples, seg_start, seg_end, seg_spk, ctx_left, ctx_right,
                            max_batch_s=50.0, iters=15, weight_mode=1, max_batch_frames=400_000, Yrec=None,
                            wpe_taps=0, wpe_delay=2, wpe_iters=3):
    """Super-segment batching.  Arguments as enhance_recording; max_batch_s bounds the summed member
    duration of a super-segment (seconds at 16 kHz).

    Every span of a super-segment (context, members, context) is snapped to the frame range that covers it
    (the bookkeeping of a stand-alone segment without context).  Spans that touch or overlap in time (the
    context before the first member and that member, back-to-back members, ...) are merged into one run of
    frames, so that no recording frame enters the statistics twice and the frames of a run are consecutive in
    time; the runs are concatenated along time, the EM and the beamformer see the concatenation as one
    segment (one set of class parameters, one filter and one reference channel), and every member's own
    frames (a slice of its run) of the beamformed STFT are inverted on their own and cut to the member.
    Returns (outputs, info) with outputs[i] the enhanced segment i and info holding the super-segment
    membership, lengths, runs and reference channels.
    """
    import torch

    D, N = x.shape
    n_spk = act_samples.shape[0]
    K = n_spk + 1
    if Yrec is None:
        Yrec = gss.gss_stft(ctx, x.reshape(1, D, N).contiguous())          # [1, F, Trec, D]
    F = Yrec.shape[1]
    n_seg = len(seg_start)
    supers = plan_super_segments(seg_start, seg_end, seg_spk, int(round(max_batch_s * 16000)))
    plans = []
    for members in supers:
        ps, pe, member_of = super_segment_pieces(members, seg_start, seg_end, N, ctx_left, ctx_right)
        fr = gss.gss_frames_from_segments(ps, pe, N, 0, 0, HOP)
        runs = merge_runs(fr["ext_start"], fr["ext_end"], HOP)
        plans.append(dict(members=members, member_of=member_of, fr=fr, runs=runs,
                          T=int(sum(r[1] for r in runs))))
    outputs = [None] * n_seg
    super_ref = np.zeros(len(supers), dtype=np.int32)
    Yr = Yrec[0]
    Trec = Yr.shape[1]
    # frame-level activity of the whole recording once; a run's rows are a slice of it
    act_rec = gss.gss_frame_activity(act_samples, 0, Trec, HOP)
    for batch in plan_batches([p["T"] for p in plans], max_batch_frames):
        S = len(batch)
        Tmax = max(plans[b]["T"] for b in batch)
        # recording frame of every frame of the concatenations (padding: frame 0, zeroed below); the runs are
        # gathered with one indexed copy per super-segment
        src = np.zeros((S, Tmax), dtype=np.int64)
        act = np.zeros((S, K, Tmax), dtype=np.uint8)
        T_len = np.zeros(S, dtype=np.int32)
        for bi, b in enumerate(batch):
            off = 0
            for f0, nf, _ in plans[b]["runs"]:
                src[bi, off:off + nf] = np.arange(f0, f0 + nf)
                act[bi, :n_spk, off:off + nf] = act_rec[:, f0:f0 + nf]
                off += nf
            act[bi, n_spk, :off] = 1
            T_len[bi] = off
        src_d = torch.from_numpy(src).to(x.device)
        Y = torch.empty((S, F, Tmax, D), dtype=torch.complex64, device=x.device)
        for bi in range(S):
            torch.index_select(Yr, 1, src_d[bi], out=Y[bi])
            Y[bi, :, int(T_len[bi]):] = 0
        T_d = torch.from_numpy(T_len).to(x.device)
        tgt = torch.from_numpy(np.asarray([seg_spk[plans[b]["members"][0]] for b in batch], dtype=np.int32)).to(x.device)
        ref = torch.full((S,), -1, dtype=torch.int32, device=x.device)
        if wpe_taps > 0:                                  # the concatenation is dereverberated as one segment
            Y = gss.gss_wpe(ctx, Y, T_d, wpe_taps, wpe_delay, wpe_iters)
        gamma = gss.gss_cacgmm_em(ctx, Y, torch.from_numpy(act).to(x.device), T_d, iters, weight_mode)
        X = gss.gss_mvdr(ctx, Y, gamma, tgt, ref, T_d)
        del Y, gamma
        ref_h = ref.cpu().numpy()
        members = []                                # (segment index, position in X's [S * Tmax] frame axis, frames, cut)
        for bi, b in enumerate(batch):
            super_ref[b] = ref_h[bi]
            fr, runs = plans[b]["fr"], plans[b]["runs"]
            run_off = np.concatenate([[0], np.cumsum([r[1] for r in runs])])
            for p, i in enumerate(plans[b]["member_of"]):
                if i < 0:
                    continue
                # the member's own frames: a slice of the run that holds its span
                f0, nf = int(fr["frame0"][p]), int(fr["n_frames"][p])
                r = next(q for q, run in enumerate(runs) if p in run[2])
                off = int(run_off[r]) + f0 - runs[r][0]
                members.append((i, bi * Tmax + off, nf, int(fr["cut_start"][p]), int(fr["cut_end"][p])))
        # every member's slice is inverted on its own, in padded batches of similar length, each gathered from the
        # beamformed STFT (frequency-major copy, one zero frame appended for the padding) with one indexed copy
        Xf = torch.zeros((F, S * Tmax + 1), dtype=torch.complex64, device=x.device)
        Xf[:, :S * Tmax].view(F, S, Tmax).copy_(X.permute(1, 0, 2))
        del X
        for mb in plan_batches([m[2] for m in members], max_batch_frames, max_segments=1024):
            Tm = max(members[m][2] for m in mb)
            idx = np.full((len(mb), Tm), S * Tmax, dtype=np.int64)
            for q, m in enumerate(mb):
                idx[q, :members[m][2]] = np.arange(members[m][1], members[m][1] + members[m][2])
            idx_d = torch.from_numpy(idx.reshape(-1)).to(x.device)
            Xp = Xf.index_select(1, idx_d).view(F, len(mb), Tm).permute(1, 0, 2).contiguous()
            xh = gss.gss_istft(ctx, Xp, (Tm - 3) * HOP)
            for q, m in enumerate(mb):
                i, _, _, c0, c1 = members[m]
                outputs[i] = xh[q, c0:c1]
        del Xf
    info = dict(supers=supers, T=np.asarray([p["T"] for p in plans], dtype=np.int32), ref=super_ref,
                pieces=[(p["member_of"], p["fr"]) for p in plans], runs=[p["runs"] for p in plans])
    return outputs, info
