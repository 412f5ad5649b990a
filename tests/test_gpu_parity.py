"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle on the same seeded
inputs.  Tolerances are the ones stated for this build: masks max|d gamma| <= 1e-3 after the configured
EM iterations, beamformed STFT relative L2 error <= 1e-4, integer/index handling and structural zeros
bit-exact.  STFT / iSTFT (fp32 arithmetic against an fp64 reference): relative L2 <= 1e-5.
"""

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL_GAMMA = 1e-3
TOL_X = 1e-4
TOL_STFT = 1e-5


@pytest.fixture(scope="module")
def env():
    import torch
    from oracle import gss_oracle as o
    from paper_2212_05271_amd import binding as gss
    from paper_2212_05271_amd import synth
    ctx = gss.Context(0)
    yield dict(torch=torch, o=o, gss=gss, synth=synth, ctx=ctx)
    ctx.close()


def _cn(rng, shape):
    return (rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) / np.sqrt(2)


def _gpu_em(env, Y, act, T_len, iters, weight_mode=1):
    t = env["torch"]
    Yd = t.from_numpy(np.ascontiguousarray(Y)).cuda()
    ad = t.from_numpy(np.ascontiguousarray(act)).cuda()
    Td = None if T_len is None else t.from_numpy(np.asarray(T_len, dtype=np.int32)).cuda()
    g = env["gss"].gss_cacgmm_em(env["ctx"], Yd, ad, Td, iters, weight_mode)
    t.cuda.synchronize()
    return g.cpu().numpy()


def _gpu_mvdr(env, Y, gamma, T_len, target, ref):
    t = env["torch"]
    Yd = t.from_numpy(np.ascontiguousarray(Y)).cuda()
    gd = t.from_numpy(np.ascontiguousarray(gamma, dtype=np.float32)).cuda()
    Td = None if T_len is None else t.from_numpy(np.asarray(T_len, dtype=np.int32)).cuda()
    tg = t.from_numpy(np.asarray(target, dtype=np.int32)).cuda()
    rf = t.from_numpy(np.asarray(ref, dtype=np.int32)).cuda()
    X = env["gss"].gss_mvdr(env["ctx"], Yd, gd, tg, rf, Td)
    t.cuda.synchronize()
    return X.cpu().numpy(), rf.cpu().numpy()


def _check_segment(env, seg, fsel=None, weight_mode=1, iters=None):
    """EM + MVDR of one segment against the oracle (on the frequency bins in fsel)."""
    o = env["o"]
    iters = seg.iters if iters is None else iters
    g = _gpu_em(env, seg.Y[None], seg.activity[None], None, iters, weight_mode)[0]
    F = seg.Y.shape[0]
    fs = np.arange(F) if fsel is None else np.asarray(fsel)
    go = o.cacgmm_em(seg.Y[fs], seg.activity, iters, weight_mode)
    dg = float(np.max(np.abs(g[:, fs] - go)))
    assert dg <= TOL_GAMMA, f"{seg.name}: max|d gamma| = {dg}"
    assert np.all(g[np.broadcast_to((seg.activity == 0)[:, None, :], g.shape)] == 0.0)
    # beamformer on the oracle's masks, reference channel forced to the oracle's choice
    Xo, ro, _ = o.mvdr(seg.Y[fs], go, seg.target)
    Xg, rg = _gpu_mvdr(env, seg.Y[None][:, fs], go[None].astype(np.float32), None, [seg.target], [ro])
    rel = float(np.linalg.norm(Xg[0] - Xo) / np.linalg.norm(Xo))
    assert rel <= TOL_X, f"{seg.name}: rel L2(X) = {rel}"
    assert int(rg[0]) == ro
    return dg, rel


# ---------------------------------------------------------------------------------------------
# EM + MVDR on the configurations
# ---------------------------------------------------------------------------------------------
def test_config0_full(env):
    _check_segment(env, env["synth"].config0())


def test_config0_small_ragged(env):
    _check_segment(env, env["synth"].config0(F=33, T=77))


def test_config1_small(env):
    _check_segment(env, env["synth"].config1(F=33, T=200))


def test_config1_full_size_every_bin(env):
    """Full-size single long segment (F = 513, T = 1560, D = 8, K = 5, 20 iterations), in the launch
    configuration the benchmark times; the oracle runs all 513 bins."""
    seg = env["synth"].config1()
    o = env["o"]
    g = _gpu_em(env, seg.Y[None], seg.activity[None], None, seg.iters)[0]
    go = np.concatenate([o.cacgmm_em(seg.Y[f0:f0 + 57], seg.activity, seg.iters) for f0 in range(0, 513, 57)], axis=1)
    assert go.shape == g.shape
    assert np.max(np.abs(g - go)) <= TOL_GAMMA
    s = g.sum(axis=0)
    assert np.all(np.abs(s - 1.0) < 1e-5)                      # the noise class is always active
    Xg, rg = _gpu_mvdr(env, seg.Y[None], g[None], None, [0], [-1])
    Xo, ro, _ = o.mvdr(seg.Y, g.astype(np.float64), 0)        # whole tensor: the covariances are cheap on the CPU
    assert int(rg[0]) == ro
    assert np.linalg.norm(Xg[0] - Xo) / np.linalg.norm(Xo) <= TOL_X


def test_weight_mode_uniform_and_zero_iterations(env):
    seg = env["synth"].config1(F=17, T=150)
    _check_segment(env, seg, weight_mode=0)
    g = _gpu_em(env, seg.Y[None], seg.activity[None], None, 0)[0]
    go = env["o"].cacgmm_em(seg.Y, seg.activity, 0)
    assert np.max(np.abs(g - go)) < 1e-7


@pytest.mark.parametrize("D,K", [(1, 2), (2, 3), (3, 2), (4, 4), (5, 3), (6, 2), (7, 5), (8, 8), (8, 1)])
def test_channel_and_class_counts(env, D, K):
    rng = np.random.default_rng(100 * D + K)
    F, T = 9, 150
    Y = (_cn(rng, (F, T, D)) * np.exp(rng.standard_normal((F, T, 1)))).astype(np.complex64)
    act = (rng.random((K, T)) < 0.6).astype(np.uint8)
    act[K - 1] = 1
    g = _gpu_em(env, Y[None], act[None], None, 6)[0]
    go = env["o"].cacgmm_em(Y, act, 6)
    assert np.max(np.abs(g - go)) <= TOL_GAMMA
    if D >= 2 and K >= 2:
        Xo, ro, _ = env["o"].mvdr(Y, go, 0)
        Xg, rg = _gpu_mvdr(env, Y[None], go[None], None, [0], [ro])
        assert np.linalg.norm(Xg[0] - Xo) / np.linalg.norm(Xo) <= TOL_X


@pytest.mark.parametrize("D", [1, 2, 3, 4, 5, 6, 7, 8])
def test_every_small_instantiation(env, D):
    """Every (D, K) instantiation of the chunked kernels (one pass and one factor launch per iteration; forced
    through the context option, few channels would take the whole-EM kernel here) for D <= 8, K = 1..8, on two
    problems of 10 tiles with a ragged tail: few problems on many workgroup slots, so every problem is cut into
    chunks and the factor kernel adds several partial sums."""
    env["ctx"].get_status()                                            # clear what earlier tests raised
    gss, ctx = env["gss"], env["ctx"]
    ctx.set_option(gss.GSS_OPT_EM_WHOLE_MIN_PROBLEMS, 1 << 40)
    try:
        for K in range(1, 9):
            rng = np.random.default_rng(10 * D + K)
            F, T = 2, 600
            Y = (_cn(rng, (F, T, D)) * np.exp(rng.standard_normal((F, T, 1)))).astype(np.complex64)
            act = (rng.random((K, T)) < 0.5).astype(np.uint8)
            act[K - 1] = 1
            T_len = np.array([T - 13], dtype=np.int32)
            g = _gpu_em(env, Y[None], act[None], T_len, 3)[0]
            go = env["o"].cacgmm_em_batch(Y[None], act[None], T_len, 3)[0]
            assert np.max(np.abs(g - go)) <= TOL_GAMMA, (D, K)
            assert np.all(g[:, :, T - 13:] == 0)
    finally:
        ctx.set_option(gss.GSS_OPT_EM_WHOLE_MIN_PROBLEMS, -1)
    assert env["ctx"].get_status() == 0


@pytest.mark.parametrize("D", [1, 2, 3, 4, 5, 6, 7, 8])
def test_every_whole_em_instantiation(env, D):
    """The one-wavefront-per-problem kernel (whole EM of a problem in one wavefront, factorisation included),
    forced through the context option, for every (D, K): a ragged batch of three segments with weights from the
    masks and uniform, degenerate frames included; and the same bits on a second run."""
    env["ctx"].get_status()                                            # clear what earlier tests raised
    gss, ctx = env["gss"], env["ctx"]
    ctx.set_option(gss.GSS_OPT_EM_WHOLE_MIN_PROBLEMS, 0)
    try:
        for K in range(1, 9):
            rng = np.random.default_rng(50 * D + K)
            S, F, T = 3, 3, 333
            Y = (_cn(rng, (S, F, T, D)) * np.exp(rng.standard_normal((S, F, T, 1)))).astype(np.complex64)
            Y[1, :, 40] = 0                                              # a zero-energy frame
            act = (rng.random((S, K, T)) < 0.5).astype(np.uint8)
            act[:, K - 1] = 1
            act[2, :, 100:110] = 0                                       # frames without any active class
            if K > 1:
                act[0, 0] = 0                                            # a class that is never active
            T_len = np.array([T, 150, T - 13], dtype=np.int32)
            for wm in (1, 0):
                g = _gpu_em(env, Y, act, T_len, 4, wm)
                go = env["o"].cacgmm_em_batch(Y, act, T_len, 4, wm)
                assert np.max(np.abs(g - go)) <= TOL_GAMMA, (D, K, wm)
                for s_ in range(S):
                    assert np.all(g[s_, :, :, T_len[s_]:] == 0)
            assert np.array_equal(g, _gpu_em(env, Y, act, T_len, 4, 0))
        assert env["ctx"].get_status() == 16                            # the zero-energy frame, nothing else
    finally:
        ctx.set_option(gss.GSS_OPT_EM_WHOLE_MIN_PROBLEMS, -1)


@pytest.mark.parametrize("D", [1, 2, 3, 4])
def test_every_tiny_problem_instantiation(env, D):
    """Few problems of at most 4 tiles and at most 4 channels take the whole-EM kernel with four wavefronts per
    problem (one tile each, frames resident in registers) by default: every (D, K), a ragged batch of two segments
    (4 and 2 tiles of 4: two wavefronts of the second segment own padding only), weights from the masks and
    uniform, a zero-energy frame, frames without any active class, a class that is never active; the same bits on
    a second run; and agreement with the one-wavefront kernel (forced through the context option) far inside the
    tolerance."""
    env["ctx"].get_status()                                            # clear what earlier tests raised
    gss, ctx = env["gss"], env["ctx"]
    for K in range(1, 9):
        rng = np.random.default_rng(70 * D + K)
        S, F, T = 2, 3, 200
        Y = (_cn(rng, (S, F, T, D)) * np.exp(rng.standard_normal((S, F, T, 1)))).astype(np.complex64)
        Y[0, :, 40] = 0
        act = (rng.random((S, K, T)) < 0.5).astype(np.uint8)
        act[:, K - 1] = 1
        act[1, :, 20:30] = 0
        if K > 1:
            act[0, 0] = 0
        T_len = np.array([T, 70], dtype=np.int32)
        for wm in (1, 0):
            g = _gpu_em(env, Y, act, T_len, 4, wm)
            go = env["o"].cacgmm_em_batch(Y, act, T_len, 4, wm)
            assert np.max(np.abs(g - go)) <= TOL_GAMMA, (D, K, wm)
            for s_ in range(S):
                assert np.all(g[s_, :, :, T_len[s_]:] == 0)
        assert np.array_equal(g, _gpu_em(env, Y, act, T_len, 4, 0))
        ctx.set_option(gss.GSS_OPT_EM_WHOLE_MIN_PROBLEMS, 0)
        try:
            g1 = _gpu_em(env, Y, act, T_len, 4, 0)
        finally:
            ctx.set_option(gss.GSS_OPT_EM_WHOLE_MIN_PROBLEMS, -1)
        assert np.max(np.abs(g - g1)) <= 1e-5, (D, K)
    assert env["ctx"].get_status() == 16                                # the zero-energy frame, nothing else


@pytest.mark.parametrize("D", [1, 2, 3, 4])
def test_few_channels_four_wavefronts_many_tiles(env, D):
    """Few problems of more than 4 tiles at up to 4 channels: where the per-lane accumulators fit in registers
    (D * D * K <= 80) the default is the whole-EM kernel with four wavefronts per problem, each walking every
    fourth tile with the next tile requested ahead.  Every such (D, K): a ragged batch (13 and 6 tiles of 13,
    the last one partly filled; in the short segment two wavefronts get one tile and two get two), tiles without
    any active class, a zero-energy frame, both weight modes, the same bits on a second run, and agreement with
    the one-wavefront kernel and the chunked kernels (forced through the context option) far inside the
    tolerance."""
    env["ctx"].get_status()                                            # clear what earlier tests raised
    gss, ctx = env["gss"], env["ctx"]
    for K in range(1, 9):
        rng = np.random.default_rng(170 * D + K)
        S, F, T = 2, 3, 800
        Y = (_cn(rng, (S, F, T, D)) * np.exp(rng.standard_normal((S, F, T, 1)))).astype(np.complex64)
        Y[0, :, 300] = 0
        act = (rng.random((S, K, T)) < 0.5).astype(np.uint8)
        act[:, K - 1] = 1
        act[:, :, 128:256] = 0                         # two tiles in which nothing is active
        if K > 1:
            act[0, 0] = 0
            act[1, 1 % K, :500] = 0
        T_len = np.array([T, 370], dtype=np.int32)
        for wm in (1, 0):
            g = _gpu_em(env, Y, act, T_len, 4, wm)
            go = env["o"].cacgmm_em_batch(Y, act, T_len, 4, wm)
            assert np.max(np.abs(g - go)) <= TOL_GAMMA, (D, K, wm)
            for s_ in range(S):
                assert np.all(g[s_, :, :, T_len[s_]:] == 0)
        assert np.array_equal(g, _gpu_em(env, Y, act, T_len, 4, 0))
        for forced in (0, 1 << 40):
            ctx.set_option(gss.GSS_OPT_EM_WHOLE_MIN_PROBLEMS, forced)
            try:
                g1 = _gpu_em(env, Y, act, T_len, 4, 0)
            finally:
                ctx.set_option(gss.GSS_OPT_EM_WHOLE_MIN_PROBLEMS, -1)
            assert np.max(np.abs(g - g1)) <= 1e-5, (D, K, forced)
    assert env["ctx"].get_status() == 16                                # the zero-energy frame, nothing else


@pytest.mark.parametrize("D,mode", [(8, 0), (8, 1 << 40), (6, -1), (4, -1), (18, -1), (24, -1), (32, -1)])
def test_rank_deficient_classes(env, D, mode):
    """Classes with fewer active frames than channels have rank-deficient scatter matrices: B is then the 1e-6
    loading plus a low-rank part, its condition number is about 1e7 and its inverse has entries of 1e6, and the
    quadratic forms of the class's own frames come out of a cancellation of such terms.  That is accurate only
    if the coefficients are those of the Hermitian part of the computed inverse (one triangle of it mirrored was
    off by up to 1e-4 relative in q, 1e-2 and more in the masks after a few iterations): every M-step implementation
    (whole-EM kernel, chunked kernels, large arrays).  Two cases: five frames in all with two classes of three frames
    each that contest one frame, and a long segment with one class of three frames; tolerance as everywhere."""
    gss, ctx = env["gss"], env["ctx"]
    rng = np.random.default_rng(900 + D)
    ctx.get_status()
    ctx.set_option(gss.GSS_OPT_EM_WHOLE_MIN_PROBLEMS, mode)
    try:
        F, T, K = 4, 5, 2
        Y = (_cn(rng, (F, T, D)) * np.exp(rng.standard_normal((F, T, 1)))).astype(np.complex64)
        act = np.zeros((K, T), dtype=np.uint8)
        act[0, :3] = 1
        act[1, 2:5] = 1
        for iters in (1, 2, 4):
            g = _gpu_em(env, Y[None], act[None], None, iters, 0)[0]
            go = env["o"].cacgmm_em(Y, act, iters, 0)
            assert np.max(np.abs(g - go)) <= 1e-5, (D, iters)
        F, T, K = 3, 300, 3
        Y = (_cn(rng, (F, T, D)) * np.exp(rng.standard_normal((F, T, 1)))).astype(np.complex64)
        act = np.zeros((K, T), dtype=np.uint8)
        act[K - 1] = 1
        act[0, 10:200] = 1
        act[1, 250:253] = 1
        g = _gpu_em(env, Y[None], act[None], None, 4)[0]
        go = env["o"].cacgmm_em(Y, act, 4)
        assert np.max(np.abs(g - go)) <= 1e-5
        assert np.all(g[np.broadcast_to((act == 0)[:, None, :], g.shape)] == 0)
    finally:
        ctx.set_option(gss.GSS_OPT_EM_WHOLE_MIN_PROBLEMS, -1)
    assert ctx.get_status() == 0


@pytest.mark.parametrize("D", [10, 20, 26, 32])
def test_every_large_instantiation(env, D):
    """Every (class count, items-per-lane) instantiation of the large-array kernels: K = 1..8 at one channel
    count out of each items-per-lane range, problems cut into chunks."""
    env["ctx"].get_status()                                            # clear what earlier tests raised
    for K in range(1, 9):
        rng = np.random.default_rng(10 * D + K)
        F, T = 2, 330
        Y = (_cn(rng, (F, T, D)) * np.exp(rng.standard_normal((F, T, 1)))).astype(np.complex64)
        act = (rng.random((K, T)) < 0.5).astype(np.uint8)
        act[K - 1] = 1
        T_len = np.array([T - 9], dtype=np.int32)
        g = _gpu_em(env, Y[None], act[None], T_len, 3)[0]
        go = env["o"].cacgmm_em_batch(Y[None], act[None], T_len, 3)[0]
        assert np.max(np.abs(g - go)) <= TOL_GAMMA, (D, K)
        assert np.all(g[:, :, T - 9:] == 0)
    assert env["ctx"].get_status() == 0


@pytest.mark.parametrize("D,K,T", [(9, 3, 100), (11, 2, 70), (12, 5, 150), (14, 2, 60), (16, 2, 70), (21, 3, 90),
                                   (23, 3, 90), (24, 5, 200), (29, 2, 80), (32, 4, 130)])
def test_large_arrays(env, D, K, T):
    """9 <= D <= 32 channels (run-time D kernels; the rows of the packed triangle end in coefficient groups of
    every length 1..8, and the channel counts cover every remainder of D modulo 8 between them and the tests above)."""
    rng = np.random.default_rng(1000 + D)
    F = 5
    v = _cn(rng, (K, F, D))
    lab = rng.integers(0, K, size=(F, T))
    Y = (v[lab, np.arange(F)[:, None]] * _cn(rng, (F, T, 1)) * np.exp(rng.standard_normal((F, T, 1)))
         + 0.3 * _cn(rng, (F, T, D))).astype(np.complex64)
    act = (rng.random((K, T)) < 0.7).astype(np.uint8)
    act[K - 1] = 1
    T_len = np.array([T - 7], dtype=np.int32)
    g = _gpu_em(env, Y[None], act[None], T_len, 6)[0]
    go = env["o"].cacgmm_em_batch(Y[None], act[None], T_len, 6)[0]
    assert np.max(np.abs(g - go)) <= TOL_GAMMA
    assert np.all(g[:, :, T - 7:] == 0)
    Xo, ro = env["o"].mvdr_batch(Y[None], go[None], T_len, [0], [-1])
    Xg, rg = _gpu_mvdr(env, Y[None], go[None], T_len, [0], ro)
    assert np.linalg.norm(Xg - Xo) <= TOL_X * np.linalg.norm(Xo)
    Xa, ra = _gpu_mvdr(env, Y[None], go[None], T_len, [0], [-1])
    assert int(ra[0]) == int(ro[0])


def test_config3_full_size_sampled_bins(env):
    """24-channel multi-array segment (F = 513, T = 1500, K = 5, 20 iterations); oracle on every 64th bin."""
    seg = env["synth"].config3()
    o = env["o"]
    g = _gpu_em(env, seg.Y[None], seg.activity[None], None, seg.iters)[0]
    fs = np.arange(0, 513, 64)
    go = o.cacgmm_em(seg.Y[fs], seg.activity, seg.iters)
    assert np.max(np.abs(g[:, fs] - go)) <= TOL_GAMMA
    Xo, ro, _ = o.mvdr(seg.Y[fs], go, 0)
    Xg, rg = _gpu_mvdr(env, seg.Y[None][:, fs], go[None], None, [0], [ro])
    assert np.linalg.norm(Xg[0] - Xo) <= TOL_X * np.linalg.norm(Xo)


def test_padded_batch_ragged_lengths(env):
    """Batch of segments of different lengths and speaker counts, padded with masks (config-2 style)."""
    synth, o = env["synth"], env["o"]
    Ts = [190, 64, 131, 1, 77, 200]
    ns = [4, 1, 2, 3, 4, 2]
    segs = [synth.config2_segment(i, Ts[i], ns[i], F=11) for i in range(len(Ts))]
    Y, act, T_len, target = synth.pad_batch(segs)
    T_len[3] = 0                                               # an empty segment in the batch
    rng = np.random.default_rng(5)
    Yj = Y.copy()
    for i, T in enumerate(T_len):                              # junk in the padding must not matter
        Yj[i, :, T:] = _cn(rng, Yj[i, :, T:].shape).astype(np.complex64)
    g = _gpu_em(env, Yj, act, T_len, 15)
    go = o.cacgmm_em_batch(Y, act, T_len, 15)
    assert np.max(np.abs(g - go)) <= TOL_GAMMA
    for i, T in enumerate(T_len):
        assert np.all(g[i, :, :, T:] == 0.0)
    ref_o = np.full(len(Ts), -1, dtype=np.int32)
    Xo, ro = o.mvdr_batch(Y, go, T_len, target, ref_o)
    Xg, rg = _gpu_mvdr(env, Yj, go.astype(np.float32), T_len, target, ro)
    for i, T in enumerate(T_len):
        assert np.all(Xg[i, :, T:] == 0)
        if T > 0:
            assert np.linalg.norm(Xg[i, :, :T] - Xo[i, :, :T]) <= TOL_X * np.linalg.norm(Xo[i, :, :T])


def test_degenerate_frames(env):
    """Zero-energy frames (flagged in the status word), frames with no active class, a class that is never active."""
    rng = np.random.default_rng(7)
    F, T, D, K = 6, 130, 4, 4
    Y = _cn(rng, (F, T, D)).astype(np.complex64)
    Y[:, 10] = 0
    Y[2, 64:70] = 0
    act = (rng.random((K, T)) < 0.7).astype(np.uint8)
    act[:, 20:25] = 0
    act[2] = 0
    env["ctx"].get_status()                                    # clear whatever earlier tests raised
    g = _gpu_em(env, Y[None], act[None], None, 8)[0]
    go = env["o"].cacgmm_em(Y, act, 8)
    assert np.all(np.isfinite(g))
    assert np.max(np.abs(g - go)) <= TOL_GAMMA
    assert np.all(g[:, :, 20:25] == 0) and np.all(g[2] == 0)
    assert env["ctx"].get_status() == 16                       # GSS_STATUS_ZERO_FRAME and nothing else
    # without the zero-energy frames the status word stays clear; a zero frame in the padding does not count
    Y2 = _cn(rng, (1, F, T, D)).astype(np.complex64)
    Y2[:, :, 100:] = 0
    g = _gpu_em(env, Y2, act[None], [100], 3)
    assert np.all(g[:, :, :, 100:] == 0) and env["ctx"].get_status() == 0


def test_bitwise_determinism_and_frequency_independence(env):
    seg = env["synth"].config1(F=20, T=333)
    g1 = _gpu_em(env, seg.Y[None], seg.activity[None], None, 10)
    g2 = _gpu_em(env, seg.Y[None], seg.activity[None], None, 10)
    assert np.array_equal(g1, g2)
    sel = [3, 17, 4]
    g3 = _gpu_em(env, seg.Y[None][:, sel], seg.activity[None], None, 10)
    assert np.array_equal(g3[0], g1[0][:, sel])
    perm = [4, 0, 2, 1, 3]
    g4 = _gpu_em(env, seg.Y[None], seg.activity[None][:, perm], None, 10)
    assert np.max(np.abs(g4[0] - g1[0][perm])) <= 1e-6


def test_equivariances_on_the_gpu(env):
    """The invariances that pin the oracle, re-run through the kernels (they catch indexing mistakes that a
    matching oracle would share): frames permuted, channels permuted (a unitary map), every frame rescaled by
    its own complex number, padding appended.  Rounding order changes, so the comparison is to 1e-6."""
    seg = env["synth"].config1(F=12, T=400)
    rng = np.random.default_rng(5)
    Y, a = seg.Y, seg.activity
    g = _gpu_em(env, Y[None], a[None], None, 10)[0]
    pt = rng.permutation(Y.shape[1])
    gp = _gpu_em(env, np.ascontiguousarray(Y[:, pt])[None], np.ascontiguousarray(a[:, pt])[None], None, 10)[0]
    assert np.max(np.abs(gp - g[:, :, pt])) <= 1e-6
    pd = rng.permutation(Y.shape[2])
    gd = _gpu_em(env, np.ascontiguousarray(Y[:, :, pd])[None], a[None], None, 10)[0]
    assert np.max(np.abs(gd - g)) <= 1e-6
    c = (rng.uniform(0.5, 2.0, Y.shape[:2]) * np.exp(2j * np.pi * rng.uniform(size=Y.shape[:2]))).astype(np.complex64)
    gs = _gpu_em(env, (Y * c[:, :, None]).astype(np.complex64)[None], a[None], None, 10)[0]
    assert np.max(np.abs(gs - g)) <= 1e-5            # the rescaled input is rounded to complex64 again
    Tp = Y.shape[1] + 77
    Ypad = np.zeros((1, Y.shape[0], Tp, Y.shape[2]), np.complex64)
    Ypad[0, :, :Y.shape[1]] = Y
    apad = np.zeros((1, a.shape[0], Tp), np.uint8)
    apad[0, :, :Y.shape[1]] = a
    gpad = _gpu_em(env, Ypad, apad, np.array([Y.shape[1]], np.int32), 10)[0]
    assert np.array_equal(gpad[:, :, :Y.shape[1]], g) and np.all(gpad[:, :, Y.shape[1]:] == 0)


def test_reference_channel_choice(env):
    """Auto mode returns the oracle's channel whenever the oracle's best and second-best scores differ by
    more than 1e-4 relative; a fixed channel is honoured."""
    o = env["o"]
    for seed in range(4):
        rng = np.random.default_rng(40 + seed)
        F, T, D = 12, 300, 6
        v, u = _cn(rng, (F, D)), _cn(rng, (F, D))
        v[:, seed % D] *= 3.0
        lab = rng.random((F, T)) < 0.5
        s = _cn(rng, (F, T))
        Y = (np.where(lab[..., None], v[:, None, :] * s[..., None], u[:, None, :] * s[..., None])
             + 0.1 * _cn(rng, (F, T, D))).astype(np.complex64)
        g = np.stack([lab, ~lab]).astype(np.float32)
        phi_k, phi_bg = o.masked_covariances(Y, g, 0)
        pbl = o.load_background(phi_bg)
        H = o.souden_filters(phi_k, pbl)
        sc = np.sort(o.reference_channel_scores(H, phi_k, pbl))[::-1]
        Xo, ro, _ = o.mvdr(Y, g, 0)
        Xg, rg = _gpu_mvdr(env, Y[None], g[None], None, [0], [-1])
        if (sc[0] - sc[1]) > 1e-4 * sc[0]:
            assert int(rg[0]) == ro
        Xf, rf = _gpu_mvdr(env, Y[None], g[None], None, [0], [2])
        Xo2, _, _ = o.mvdr(Y, g, 0, ref=2)
        assert int(rf[0]) == 2 and np.linalg.norm(Xf[0] - Xo2) <= TOL_X * np.linalg.norm(Xo2)


def test_mvdr_target_class_and_literal_normalised_input(env):
    """Target other than 0, and the paper's literal reading (beamformer fed the unit-normalised Y)."""
    o = env["o"]
    seg = env["synth"].config1(F=15, T=260)
    go = o.cacgmm_em(seg.Y, seg.activity, 5)
    Yn = o.unit_normalise(seg.Y).astype(np.complex64)
    for tgt, Yin in ((2, seg.Y), (0, Yn)):
        Xo, ro, _ = o.mvdr(Yin, go, tgt)
        Xg, rg = _gpu_mvdr(env, Yin[None], go[None], None, [tgt], [ro])
        assert np.linalg.norm(Xg[0] - Xo) <= TOL_X * np.linalg.norm(Xo)


# ---------------------------------------------------------------------------------------------
# STFT / inverse STFT and the chained pipeline
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("S,D,N", [(1, 2, 5000), (2, 3, 4096), (1, 9, 2500), (1, 1, 255)])
def test_stft_istft(env, S, D, N):
    t, o, gss = env["torch"], env["o"], env["gss"]
    rng = np.random.default_rng(N + D)
    x = rng.standard_normal((S, D, N)).astype(np.float32)
    Y = gss.gss_stft(env["ctx"], t.from_numpy(x).cuda()).cpu().numpy()
    Yo = np.stack([o.stft_channels_last(x[s]) for s in range(S)])
    assert Y.shape == Yo.shape
    assert np.linalg.norm(Y - Yo) <= TOL_STFT * np.linalg.norm(Yo)
    T = Yo.shape[2]
    X = (rng.standard_normal((S, 513, T)) + 1j * rng.standard_normal((S, 513, T))).astype(np.complex64)
    xr = gss.gss_istft(env["ctx"], t.from_numpy(X).cuda(), N).cpu().numpy()
    xo = np.stack([o.istft(X[s], N) for s in range(S)])
    assert np.linalg.norm(xr - xo) <= TOL_STFT * np.linalg.norm(xo)
    back = gss.gss_istft(env["ctx"], t.from_numpy(np.ascontiguousarray(Y[..., 0])).cuda(), N).cpu().numpy()
    assert np.linalg.norm(back - x[:, 0]) <= TOL_STFT * np.linalg.norm(x[:, 0])


def test_full_chain_time_domain(env):
    """x -> STFT -> EM -> MVDR -> iSTFT on the GPU against the same chain in the oracle (the oracle's STFT
    is rounded to complex64, the type of the boundary between the stages)."""
    t, o, gss = env["torch"], env["o"], env["gss"]
    rng = np.random.default_rng(11)
    D, N, K = 4, 12000, 3
    T = o.stft_num_frames(N, 256)
    src = rng.standard_normal((2, N)) * (np.sin(2 * np.pi * 3.0 * np.arange(N) / 16000.0)[None] ** 2 + 0.1)
    act_s = np.zeros((K, N), np.uint8)
    act_s[0, : 2 * N // 3] = 1
    act_s[1, N // 3:] = 1
    act_s[2] = 1
    mix = rng.standard_normal((2, D))
    x = ((mix.T @ (src * act_s[:2])) + 0.05 * rng.standard_normal((D, N))).astype(np.float32)
    act = gss.gss_frame_activity(act_s, 0, T)
    assert np.array_equal(act, o.frame_activity(act_s, 0, T))
    ctx = env["ctx"]
    Y = gss.gss_stft(ctx, t.from_numpy(x[None]).cuda())
    g = gss.gss_cacgmm_em(ctx, Y, t.from_numpy(act[None]).cuda(), None, 10)
    ref = t.full((1,), -1, dtype=t.int32).cuda()
    X = gss.gss_mvdr(ctx, Y, g, t.zeros(1, dtype=t.int32).cuda(), ref)
    xh = gss.gss_istft(ctx, X, N).cpu().numpy()[0]
    Yo = o.stft_channels_last(x).astype(np.complex64)
    go = o.cacgmm_em(Yo, act, 10)
    Xo, ro, _ = o.mvdr(Yo, go, 0)
    xo = o.istft(Xo, N)
    assert int(ref.item()) == ro
    assert np.max(np.abs(g.cpu().numpy()[0] - go)) <= TOL_GAMMA
    assert np.linalg.norm(X.cpu().numpy()[0] - Xo) <= TOL_X * np.linalg.norm(Xo)
    assert np.linalg.norm(xh - xo) <= TOL_X * np.linalg.norm(xo)


# ---------------------------------------------------------------------------------------------
# error handling through the ABI
# ---------------------------------------------------------------------------------------------
def test_argument_errors(env):
    t, gss, ctx = env["torch"], env["gss"], env["ctx"]
    Y = t.zeros((1, 3, 10, 2), dtype=t.complex64).cuda()
    act = t.ones((1, 2, 10), dtype=t.uint8).cuda()
    with pytest.raises(gss.GssError) as e:
        gss.gss_cacgmm_em(ctx, Y, act, None, -1)
    assert e.value.code == gss.GSS_EINVAL
    with pytest.raises(gss.GssError) as e:
        gss.gss_cacgmm_em(ctx, Y, act, None, 1, weight_mode=3)
    assert e.value.code == gss.GSS_EINVAL
    act9 = t.ones((1, 9, 10), dtype=t.uint8).cuda()
    with pytest.raises(gss.GssError) as e:
        gss.gss_cacgmm_em(ctx, Y, act9, None, 1)
    assert e.value.code == gss.GSS_EUNSUPPORTED
    Y33 = t.zeros((1, 3, 10, 33), dtype=t.complex64).cuda()   # more channels than GSS_MAX_D
    with pytest.raises(gss.GssError) as e:
        gss.gss_cacgmm_em(ctx, Y33, act, None, 1)
    assert e.value.code == gss.GSS_EUNSUPPORTED
    x = t.zeros((1, 2, 1000)).cuda()
    with pytest.raises(gss.GssError) as e:
        gss.gss_stft(ctx, x, n_fft=512, hop=128)
    assert e.value.code == gss.GSS_EUNSUPPORTED
    with pytest.raises(TypeError):
        gss.gss_cacgmm_em(ctx, Y.cpu(), act, None, 1)
    # an out-of-range target is clamped and flagged, never faults
    g = gss.gss_cacgmm_em(ctx, Y, act, None, 1)
    ref = t.zeros(1, dtype=t.int32).cuda()
    gss.gss_mvdr(ctx, Y, g, t.full((1,), 7, dtype=t.int32).cuda(), ref)
    assert ctx.get_status() & 4
    # a reference channel beyond the array is flagged and replaced by the chosen one, never read as an index
    ref = t.full((1,), 9, dtype=t.int32).cuda()
    D = Y.shape[-1]
    gss.gss_mvdr(ctx, Y, g, t.zeros(1, dtype=t.int32).cuda(), ref)
    assert ctx.get_status() & 32 and 0 <= int(ref.item()) < D


# ---------------------------------------------------------------------------------------------
# segments as frame ranges of one recording's STFT
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("D", [4, 8, 12])
def test_frames_entry_points(env, D):
    """gss_cacgmm_em_frames / gss_mvdr_frames read segments in place out of a recording's STFT: the same bits
    as the dense entry points on copies of those frame ranges, and the oracle's values; a range that runs past
    the end of the recording is clipped, never read."""
    t, gss, ctx, o = env["torch"], env["gss"], env["ctx"], env["o"]
    rng = np.random.default_rng(900 + D)
    F, Trec, K, iters = 7, 700, 3, 5
    Yrec = (_cn(rng, (F, Trec, D)) * np.exp(rng.standard_normal((F, Trec, 1)))).astype(np.complex64)
    frame0 = np.array([0, 130, 417, 600], dtype=np.int64)
    T_len = np.array([200, 77, 283, 150], dtype=np.int32)          # the last one would end at frame 750 > Trec
    S, Tmax = len(frame0), 283
    act = (rng.random((S, K, Tmax)) < 0.6).astype(np.uint8)
    act[:, K - 1] = 1
    for s in range(S):
        act[s, :, T_len[s]:] = 0
    Yd = t.from_numpy(Yrec).cuda()
    f0d, Td, ad = t.from_numpy(frame0).cuda(), t.from_numpy(T_len).cuda(), t.from_numpy(act).cuda()
    g = gss.gss_cacgmm_em_frames(ctx, Yd, f0d, ad, Td, iters)
    tgt = t.zeros(S, dtype=t.int32).cuda()
    ref = t.full((S,), -1, dtype=t.int32).cuda()
    X = gss.gss_mvdr_frames(ctx, Yd, f0d, g, tgt, ref, Td)
    t.cuda.synchronize()
    # dense copies (the clipped length of the last segment is what the recording holds: 100 frames)
    T_eff = np.minimum(T_len, Trec - frame0).astype(np.int32)
    Yp = np.zeros((S, F, Tmax, D), np.complex64)
    for s in range(S):
        Yp[s, :, :T_eff[s]] = Yrec[:, frame0[s]:frame0[s] + T_eff[s]]
    gd = gss.gss_cacgmm_em(ctx, t.from_numpy(Yp).cuda(), ad, t.from_numpy(T_eff).cuda(), iters)
    ref2 = t.full((S,), -1, dtype=t.int32).cuda()
    Xd = gss.gss_mvdr(ctx, t.from_numpy(Yp).cuda(), gd, tgt, ref2, t.from_numpy(T_eff).cuda())
    t.cuda.synchronize()
    assert t.equal(g, gd) and t.equal(X, Xd) and t.equal(ref, ref2)
    gn = g.cpu().numpy()
    for s in range(S):
        go = o.cacgmm_em(Yp[s, :, :T_eff[s]], act[s, :, :T_eff[s]], iters)
        assert np.max(np.abs(gn[s, :, :, :T_eff[s]] - go)) <= TOL_GAMMA
        assert np.all(gn[s, :, :, T_eff[s]:] == 0)
        Xo, ro, _ = o.mvdr(Yp[s, :, :T_eff[s]], go, 0)
        Xg, rg = _gpu_mvdr(env, Yp[s:s + 1, :, :T_eff[s]], go[None], None, [0], [ro])
        assert np.linalg.norm(Xg[0] - Xo) <= TOL_X * np.linalg.norm(Xo)


def test_reference_channel_per_frequency(env):
    """gss_mvdr_ex with one reference channel per frequency: the chosen channels agree with the oracle's wherever
    its two best scores differ by more than 1e-4 relative; with the channels forced to the oracle's the beamformed
    STFT matches; a given channel is kept; dense batch and frame ranges of a recording alike."""
    t, gss, ctx, o = env["torch"], env["gss"], env["ctx"], env["o"]
    for D in (4, 8, 12):
        rng = np.random.default_rng(1200 + D)
        S, F, T, K = 2, 33, 200, 3
        Y = (_cn(rng, (S, F, T, D)) * np.exp(rng.standard_normal((S, F, T, 1)))).astype(np.complex64)
        g = rng.random((S, K, F, T)).astype(np.float32)
        g /= g.sum(1, keepdims=True)
        T_len = np.array([T, 150], dtype=np.int32)
        Yd, gd, Td = t.from_numpy(Y).cuda(), t.from_numpy(g).cuda(), t.from_numpy(T_len).cuda()
        tgt = t.from_numpy(np.array([1, 0], dtype=np.int32)).cuda()
        ref = t.full((S, F), -1, dtype=t.int32).cuda()
        X = gss.gss_mvdr_ex(ctx, Yd, gd, tgt, ref, Td, ref_mode=gss.GSS_REF_PER_FREQUENCY)
        t.cuda.synchronize()
        ref_g = ref.cpu().numpy()
        for s_ in range(S):
            Ts = int(T_len[s_])
            gs = g[s_, :, :, :Ts].astype(np.float64)
            Xo, ro, _ = o.mvdr_per_frequency_ref(Y[s_, :, :Ts], gs, int(tgt[s_].item()))
            pk, pb = o.masked_covariances(Y[s_, :, :Ts], gs, int(tgt[s_].item()))
            pbl = o.load_background(pb)
            sc = np.sort(o.reference_channel_scores_per_frequency(o.souden_filters(pk, pbl), pk, pbl), axis=1)
            clear = (sc[:, -1] - sc[:, -2]) > 1e-4 * sc[:, -1]
            assert clear.sum() > F // 2 and np.all(ref_g[s_][clear] == ro[clear])
            # X with the oracle's channels
            rf = t.from_numpy(np.stack([ro if q == s_ else np.zeros(F, np.int64) for q in range(S)]).astype(np.int32)).cuda()
            Xf = gss.gss_mvdr_ex(ctx, Yd, gd, tgt, rf, Td, ref_mode=gss.GSS_REF_PER_FREQUENCY)
            t.cuda.synchronize()
            assert np.array_equal(rf.cpu().numpy()[s_], ro.astype(np.int32))
            Xg = Xf[s_].cpu().numpy()
            assert np.linalg.norm(Xg[:, :Ts] - Xo) <= TOL_X * np.linalg.norm(Xo)
            assert np.all(Xg[:, Ts:] == 0)
        # the per-segment mode of the general call is gss_mvdr
        r1 = t.full((S,), -1, dtype=t.int32).cuda()
        r2 = t.full((S,), -1, dtype=t.int32).cuda()
        Xa = gss.gss_mvdr_ex(ctx, Yd, gd, tgt, r1, Td)
        Xb = gss.gss_mvdr(ctx, Yd, gd, tgt, r2, Td)
        assert t.equal(Xa, Xb) and t.equal(r1, r2)
    del X
