"""The entry point that allocates nothing (`ssgd_full_gradient_static`) against the one it is a variant of
(`ssgd_full_gradient`), through the C ABI: same kernels, same launch shape, so the values agree bit for bit.
Two calls in a row share the library's static scratch array; the second works on a smaller data set, so
whatever the first left behind must not show."""
import numpy as np
import pytest

from paper_2003_10579_amd import synth

pytestmark = pytest.mark.gpu


def _context(ssgd, torch, kind, N, d, classes, seed, updates):
    if kind == "lsq":
        X, y, _ = synth.lsq_data(N, d, seed)
    else:
        X, y = synth.mixture_data(N, d, classes, seed=seed)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context(kind, Xd, yd, 6, 2, 16, "k_async", ssgd.delay_dist("exp", 1.0), 0.05, seed=seed, classes=classes,
                       replicas=2)
    ctx.run(updates)            # parameters away from zero
    return ctx, (Xd, yd)


def test_static_scratch_entry_point_matches_the_allocating_one():
    import torch
    from paper_2003_10579_amd import ssgd
    assert torch.cuda.is_available(), "this test needs the GPU"
    ssgd.lib()
    big, keep_big = _context(ssgd, torch, "softmax", 20000, 3072, 10, 3, 25)      # 2.3 M floats of scratch memory
    small, keep_small = _context(ssgd, torch, "softmax", 1001, 132, 3, 4, 25)     # 17 k floats: far inside the first call's
    tiny, keep_tiny = _context(ssgd, torch, "lsq", 300, 64, 1, 5, 10)
    for ctx in (big, small, tiny, big):
        for replica in (0, 1):
            out = torch.full((ctx.nw + 8,), float("nan"), dtype=torch.float32, device="cuda")
            ctx.full_gradient_static(out, replica)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            ref = ctx.full_gradient(replica)
            assert np.all(np.isfinite(got[:ctx.nw])) and np.linalg.norm(ref) > 0
            assert np.array_equal(got[:ctx.nw].view(np.uint32), ref.view(np.uint32))
            assert np.all(np.isnan(got[ctx.nw:]))          # nothing written past |w|
    for ctx in (big, small, tiny):
        ctx.close()


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2003_10579_amd import ssgd
    ssgd.lib()
    # 16 floats per sample: 300 000 samples need more than the 4 Mi floats of the static array
    X, y, _ = synth.lsq_data(300000, 4, 1)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context("lsq", Xd, yd, 4, 2, 8, "k_sync", ssgd.delay_dist("exp", 1.0), 0.01, seed=1)
    out = torch.zeros(ctx.nw, dtype=torch.float32, device="cuda")
    with pytest.raises(ssgd.SsgdError) as ei:
        ctx.full_gradient_static(out)
    assert ei.value.status == ssgd.EINVAL and "static array" in str(ei.value)
    assert np.all(np.isfinite(ctx.full_gradient()))         # the allocating entry point still takes it
    ctx.close()
    # a shape neither entry point is built for
    X, y, _ = synth.lsq_data(100, 6, 1)
    ctx = ssgd.Context("lsq", torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(), 4, 2, 8, "k_sync",
                       ssgd.delay_dist("exp", 1.0), 0.01, seed=1)
    with pytest.raises(ssgd.SsgdError) as ei:
        ctx.full_gradient_static(torch.zeros(ctx.nw, dtype=torch.float32, device="cuda"))
    assert ei.value.status == ssgd.EINVAL
    ctx.close()
