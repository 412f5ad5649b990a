"""The no-allocation variant of the EM entry point (static scratch array per GPU) against the ordinary entry
point, through the C ABI: two calls in a row, the second on a smaller input, plus the size limit."""

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _problem(rng, S, F, T, D, K):
    Y = ((rng.standard_normal((S, F, T, D)) + 1j * rng.standard_normal((S, F, T, D)))
         * np.exp(rng.standard_normal((S, F, T, 1)))).astype(np.complex64)
    act = (rng.random((S, K, T)) < 0.6).astype(np.uint8)
    act[:, K - 1] = 1
    T_len = rng.integers(T // 2, T + 1, size=S).astype(np.int32)
    T_len[0] = T
    return Y, act, T_len


def test_noalloc_matches_allocating_entry_point_twice():
    import torch
    from oracle import gss_oracle as o
    from paper_2212_05271_amd import binding as gss

    rng = np.random.default_rng(77)
    with gss.Context(0) as ctx:
        # first a larger problem (several chunks per problem and a ragged tail), then a smaller one that reuses
        # the front of the same static array, then a 12-channel one (the kernels for more than 8 channels)
        for (S, F, T, D, K, iters) in ((3, 65, 700, 8, 5, 6), (2, 17, 150, 4, 3, 4), (1, 9, 200, 12, 3, 3)):
            Y, act, T_len = _problem(rng, S, F, T, D, K)
            Yd, ad, Td = (torch.from_numpy(a).cuda() for a in (Y, act, T_len))
            g_ref = gss.gss_cacgmm_em(ctx, Yd, ad, Td, iters)
            torch.cuda.synchronize()
            out = torch.full((S, K, F, T), -7.0, dtype=torch.float32, device="cuda")
            before = ctx.scratch_bytes()
            gss.gss_cacgmm_em_noalloc(ctx, Yd, ad, Td, iters, out=out)
            torch.cuda.synchronize()
            assert ctx.scratch_bytes() == before                   # the context's own scratch was not touched
            a, b = out.cpu().numpy(), g_ref.cpu().numpy()
            assert np.max(np.abs(a - b)) <= 1e-3                    # the stated tolerance for masks ...
            assert np.array_equal(a, b)                            # ... and in fact the same kernels, bit for bit
            go = o.cacgmm_em_batch(Y[:1, :5], act[:1], T_len[:1], iters)
            assert np.max(np.abs(a[:1, :, :5] - go)) <= 1e-3
        assert ctx.get_status() == 0


def test_noalloc_rejects_what_does_not_fit():
    import torch
    from paper_2212_05271_amd import binding as gss

    with gss.Context(0) as ctx:
        S, F, T, D, K = 40, 513, 64, 8, 5                          # coefficients alone: 40*513*5*64*8 B = 52 MB, with
        Y = torch.zeros((S, F, T, D), dtype=torch.complex64, device="cuda")   # the partial sums beyond 64 MiB
        act = torch.ones((S, K, T), dtype=torch.uint8, device="cuda")
        out = torch.full((S, K, F, T), -7.0, dtype=torch.float32, device="cuda")
        with pytest.raises(gss.GssError) as e:
            gss.gss_cacgmm_em_noalloc(ctx, Y, act, None, 2, out=out)
        assert e.value.code == gss.GSS_ETOOBIG
        torch.cuda.synchronize()
        assert bool((out == -7.0).all())                           # nothing was written
        # the context still works afterwards, through both entry points
        g = gss.gss_cacgmm_em(ctx, Y[:1], act[:1], None, 1)
        gss.gss_cacgmm_em_noalloc(ctx, Y[:1], act[:1], None, 1, out=out[:1])
        torch.cuda.synchronize()
        assert torch.equal(g, out[:1])
