"""The entry point that allocates nothing (choco_metrics_noalloc) against choco_metrics.

Two calls in a row on one GPU share the library's own scratch array; the second call works
on a smaller state, so anything the first call left behind in the array would show.
"""
import numpy as np
import pytest

from paper_1907_09356_amd import binding as B
from paper_1907_09356_amd import synth

pytestmark = pytest.mark.gpu


def make_ctx(n, d, seed, steps):
    import torch
    X0 = synth.normal_state(n, d, seed=seed)
    X = torch.from_numpy(np.ascontiguousarray(X0)).to("cuda:0")
    ld = (d + 3) // 4 * 4
    if ld != d:
        Xp = torch.zeros((n, ld), dtype=torch.float32, device="cuda:0")
        Xp[:, :d] = X
        X = Xp
    ctx = B.Choco(X, d, *synth.ring_csr(n), 0.3, B.Q_SIGN, seed=seed)
    grads = synth.GradientStream(n, d, seed=seed + 1)
    for _ in range(steps):
        g = torch.zeros_like(X)
        g[:, :d] = torch.from_numpy(grads.next()).to("cuda:0")
        ctx.step(g, 0.05)
    return ctx, X


def check(ctx, out):
    import torch
    out.fill_(-1.0)
    ctx.metrics_noalloc(out)          # enqueues only
    want = ctx.metrics()              # same stream, waits
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for name, g in zip(("consensus", "mean_norm", "psi"), got):
        w = want[name]
        assert np.isfinite(g) and abs(g - w) <= 1e-13 * abs(w), (name, g, w)


def test_noalloc_metrics_match_on_two_calls_the_second_smaller():
    import torch
    out = torch.empty(3, dtype=torch.float64, device="cuda:0")
    big, Xb = make_ctx(8, 300_001, seed=3, steps=2)      # 1024 blocks: every slot of the array is written
    small, Xs = make_ctx(5, 1000, seed=4, steps=3)        # 4 blocks: most of the array keeps the first call's sums
    try:
        check(big, out)
        check(small, out)
        check(big, out)
        # the two calls back to back on one stream with no wait in between
        out2 = torch.empty(3, dtype=torch.float64, device="cuda:0")
        big.metrics_noalloc(out)
        small.metrics_noalloc(out2)
        torch.cuda.synchronize()
        wb, ws = big.metrics(), small.metrics()
        for o, w in ((out, wb), (out2, ws)):
            g = o.cpu().numpy()
            assert abs(g[0] - w["consensus"]) <= 1e-13 * w["consensus"]
            assert abs(g[2] - w["psi"]) <= 1e-13 * w["psi"]
    finally:
        big.close()
        small.close()


def test_noalloc_rejects_bad_arguments():
    import torch
    ctx, X = make_ctx(3, 64, seed=1, steps=0)
    try:
        out = torch.empty(4, dtype=torch.float64, device="cuda:0")
        assert B.lib().choco_metrics_noalloc(ctx.ctx, None) == B.E_INVAL
        assert B.lib().choco_metrics_noalloc(None, out.data_ptr()) == B.E_INVAL
        assert B.lib().choco_metrics_noalloc(ctx.ctx, out.data_ptr() + 4) == B.E_INVAL   # not 8-byte aligned
    finally:
        ctx.close()


def test_noalloc_rejects_a_vector_above_its_maximum():
    # d = 2^28 + 4 with one worker: 1 GiB of state, 1 GiB of workspace
    import torch
    n, d = 1, (1 << 28) + 4
    X = torch.zeros((n, d), dtype=torch.float32, device="cuda:0")
    ctx = B.Choco(X, d, np.array([0, 1]), np.array([0]), np.array([1.0], dtype=np.float32), 0.5, B.Q_IDENTITY)
    try:
        out = torch.zeros(3, dtype=torch.float64, device="cuda:0")
        assert B.lib().choco_metrics_noalloc(ctx.ctx, out.data_ptr()) == B.E_UNSUPPORTED
        m = ctx.metrics()                      # the ordinary call still serves this size
        assert m["consensus"] == 0.0
    finally:
        ctx.close()
