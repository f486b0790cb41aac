"""GPU parity: the HIP path against the CPU oracle, element by element, through the C ABI.

Bar: kept index sets, sign bits, quantisation levels and the per-worker norms/scales are
bit-exact; X, Xhat and S agree to 1e-6 relative L2 per step (they are in fact required to
be bit-identical here, because both sides round every operation in the same order).
"""
import numpy as np
import pytest

from paper_1907_09356_amd import binding as B
from paper_1907_09356_amd import synth
from tests.parity_util import Pair, rel_l2

pytestmark = pytest.mark.gpu

ORDERS = [B.ORDER_COMPRESS_THEN_MIX, B.ORDER_MIX_THEN_COMPRESS]

COMPRESSORS = {
    "identity": dict(compressor=B.Q_IDENTITY),
    "sign": dict(compressor=B.Q_SIGN),
    "qsgd16": dict(compressor=B.Q_QSGD, levels=16),
    "qsgd2_unbiased": dict(compressor=B.Q_QSGD, levels=2, qsgd_biased=0),
    "qsgd_b16": dict(compressor=B.Q_QSGD, levels=32768),
    "topk": dict(compressor=B.Q_TOPK),
    "randk": dict(compressor=B.Q_RANDK),
    "randk_rescaled": dict(compressor=B.Q_RANDK, randk_rescale=1),
}


def topo_for(n):
    if n == 9:
        return synth.torus_csr(3, 3)
    if n == 64:
        return synth.torus_csr(8, 8)
    return synth.ring_csr(n)


SPARSE_MIXES = [B.MIX_INCREMENTAL_S, B.MIX_DIRECT]
MIX_NAME = {B.MIX_AUTO: "auto", B.MIX_INCREMENTAL_S: "incremental", B.MIX_DIRECT: "direct"}


def run(n, d, comp, order, steps=6, mix_form=None, gamma=0.2, frac=0.01, seed=5, lr=0.05,
        force=False, x0=None):
    """mix_form=None: the library's choice for the dense operators; for top_a / random_a BOTH
    evaluations of the mix, one run each (the library's choice is one of the two)."""
    kw = dict(COMPRESSORS[comp])
    sparse = kw["compressor"] in (B.Q_TOPK, B.Q_RANDK)
    if mix_form is None:
        if sparse:
            for m in SPARSE_MIXES:
                run(n, d, comp, order, steps, m, gamma, frac, seed, lr, force, x0)
            return
        mix_form = B.MIX_AUTO
    if sparse:
        kw["k"] = max(1, int(frac * d))
    X0 = synth.normal_state(n, d, seed=seed) if x0 is None else x0
    pair = Pair(X0, topo_for(n), gamma, order=order, mix_form=mix_form, seed=1234 + seed, **kw)
    grads = synth.GradientStream(n, d, seed=seed + 1)
    try:
        for t in range(steps):
            if force:
                pair.force_state()
            det = pair.gossip_step()
            pair.check(det, tag="%s n=%d d=%d order=%d mix=%s step %d" % (comp, n, d, order, MIX_NAME[mix_form], t))
            pair.sgd_step(grads.next(), lr)
    finally:
        pair.close()


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("comp", list(COMPRESSORS))
@pytest.mark.parametrize("n,d", [(8, 4096), (9, 2000), (8, 70001), (3, 1027), (64, 5000)])
def test_step_parity_free_running(n, d, comp, order):
    # several 256-wide tiles, ragged tails (d not a multiple of 4 or 256), ring and torus
    run(n, d, comp, order)


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("comp", ["sign", "qsgd16", "topk", "randk"])
def test_step_parity_teacher_forced(comp, order):
    run(8, 10000, comp, order, steps=4, force=True)


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("comp", ["topk", "randk"])
def test_sparse_operators_with_both_mix_forms(comp, order):
    run(8, 6000, comp, order)


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("comp", ["identity", "sign", "qsgd16", "topk", "randk"])
def test_more_workers_than_the_lds_tile_holds(comp, order):
    # n > 64: the direct mix reads neighbour rows from global memory instead of LDS
    run(70, 1030, comp, order, steps=3)


@pytest.mark.parametrize("mix", SPARSE_MIXES)
@pytest.mark.parametrize("d,k", [(1, 1), (3, 2), (5, 5), (300, 1), (300, 300), (4096, 2048)])
@pytest.mark.parametrize("comp", ["topk", "randk"])
def test_select_extreme_k(comp, d, k, mix):
    kw = dict(COMPRESSORS[comp])
    pair = Pair(synth.normal_state(4, d, seed=d + k), synth.ring_csr(4), 0.3, k=k, seed=9, mix_form=mix, **kw)
    try:
        for t in range(3):
            det = pair.gossip_step()
            pair.check(det, tag="%s d=%d k=%d step %d" % (comp, d, k, t))
    finally:
        pair.close()


@pytest.mark.parametrize("mix", SPARSE_MIXES)
@pytest.mark.parametrize("order", ORDERS)
def test_topk_ties_and_zeros(order, mix):
    # integer-valued state: thousands of equal magnitudes, so the tie rule (lower index
    # first) decides most of the selection; all-zero rows as well
    rng = np.random.default_rng(3)
    n, d, k = 5, 3000, 100
    X0 = rng.integers(-3, 4, size=(n, d)).astype(np.float32)
    X0[2] = 0.0
    X0[3, ::2] = -0.0
    pair = Pair(X0, synth.ring_csr(n), 0.25, compressor=B.Q_TOPK, k=k, order=order, mix_form=mix)
    try:
        for t in range(5):
            det = pair.gossip_step()
            pair.check(det, tag="ties step %d" % t)
    finally:
        pair.close()


@pytest.mark.parametrize("comp", ["topk", "randk"])
def test_select_when_one_digit_overflows_the_candidate_list(comp):
    # every |v| equal and d far above the candidate capacity: the select has to finish by
    # scanning the row itself
    n, d, k = 3, 40000, 10
    X0 = np.full((n, d), 1.5, dtype=np.float32)
    X0[:, 1::3] = -1.5
    kw = dict(COMPRESSORS[comp])
    pair = Pair(X0, synth.ring_csr(n), 0.25, k=k, seed=2, **kw)
    try:
        det = pair.gossip_step()
        pair.check(det, tag="overflow")
        if comp == "topk":
            assert np.array_equal(det["sel"], np.tile(np.arange(k), (n, 1)))
            assert np.all(pair.gpu.last_scalars()[:, 3] == 2)   # row-scan mode was taken
        det = pair.gossip_step()
        pair.check(det, tag="overflow step 2")
    finally:
        pair.close()


@pytest.mark.parametrize("mix", SPARSE_MIXES)
@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("comp,k", [("topk", 8000), ("randk", 12000), ("randk_rescaled", 12000)])
def test_long_candidate_lists_take_the_multi_block_select(comp, k, order, mix):
    # k + slack above 16384 candidates per worker: histogram parts, parallel emission, finish
    n, d = 4, 200000
    kw = dict(COMPRESSORS[comp])
    pair = Pair(synth.normal_state(n, d, seed=6), synth.ring_csr(n), 0.2, k=k, order=order, seed=5, mix_form=mix, **kw)
    grads = synth.GradientStream(n, d, seed=7)
    try:
        for t in range(5):
            det = pair.step(grads.next(), 0.05)
            pair.check(det, tag="multi-block %s step %d" % (comp, t))
    finally:
        pair.close()


def test_multi_block_select_with_crowded_threshold_bin_and_overflow():
    # integer-valued state (thousands of ties around the threshold) and a constant state (one
    # key for the whole row) with k large enough for the multi-block select: its finish kernel
    # has to take the digit-by-digit path on the list, resp. the row scan
    n, d, k = 3, 120000, 9000
    rng = np.random.default_rng(8)
    for X0 in (rng.integers(-4, 5, size=(n, d)).astype(np.float32),
               np.full((n, d), -2.5, dtype=np.float32)):
        pair = Pair(X0, synth.ring_csr(n), 0.25, compressor=B.Q_TOPK, k=k)
        try:
            for t in range(3):
                det = pair.gossip_step()
                pair.check(det, tag="multi-block ties step %d" % t)
        finally:
            pair.close()


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("comp", list(COMPRESSORS))
@pytest.mark.parametrize("n", [1, 2])
def test_single_and_two_workers(n, comp, order):
    # degenerate graphs: one node (W = [1]) and two nodes (complete graph, weights 1/2)
    run(n, 3000, comp, order, steps=3)


@pytest.mark.parametrize("graph", ["hub", "complete"])
@pytest.mark.parametrize("comp", ["sign", "topk", "randk"])
def test_rows_of_w_longer_than_the_mix_kernel_stages(comp, graph):
    # the tile mix keeps up to 16 neighbours of a row in a lane group and reads longer rows from
    # memory: a hub of degree 30 among short rows (both paths in one workgroup), and the complete
    # graph on 20 nodes (every row long)
    if graph == "hub":
        n = 40
        adj = synth.irregular_graph(n, 30, seed=5)
        assert adj.sum(1).max() == 30 and adj.sum(1).min() < 15
        topo = synth.metropolis_csr(adj)
    else:
        n = 20
        topo = synth.complete_csr(n)
    kw = dict(COMPRESSORS[comp])
    if kw["compressor"] in (B.Q_TOPK, B.Q_RANDK):
        kw["k"] = 30
    d = 3000
    pair = Pair(synth.normal_state(n, d, seed=12), topo, 0.3, seed=14, **kw)
    grads = synth.GradientStream(n, d, seed=13)
    try:
        if kw["compressor"] in (B.Q_TOPK, B.Q_RANDK):
            assert pair.mix == B.MIX_DIRECT      # the fused tile pass
        for t in range(4):
            det = pair.step(grads.next(), 0.05)
            pair.check(det, tag="%s graph %s step %d" % (graph, comp, t))
    finally:
        pair.close()


@pytest.mark.parametrize("mix", SPARSE_MIXES)
@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("comp", ["sign", "qsgd16", "topk", "randk"])
def test_irregular_graph_with_local_degree_weights(comp, order, mix):
    # 32 nodes, maximum degree 14, weights 1/(1 + max(deg i, deg j)) with the remainder on the
    # self loop: rows of different lengths and different weights per edge
    adj = synth.irregular_graph(32, 14, seed=3)
    assert adj.sum(1).max() == 14
    topo = synth.metropolis_csr(adj)
    kw = dict(COMPRESSORS[comp])
    if kw["compressor"] in (B.Q_TOPK, B.Q_RANDK):
        kw["k"] = 40
        kw["mix_form"] = mix
    elif mix != SPARSE_MIXES[0]:
        pytest.skip("the dense operators have one form of the mix")
    n, d = 32, 4000
    pair = Pair(synth.normal_state(n, d, seed=2), topo, 0.3, order=order, seed=4, **kw)
    grads = synth.GradientStream(n, d, seed=3)
    try:
        for t in range(5):
            det = pair.step(grads.next(), 0.05)
            pair.check(det, tag="irregular %s step %d" % (comp, t))
    finally:
        pair.close()


@pytest.mark.parametrize("comp", ["sign", "qsgd16"])
def test_norm_finalise_kernel_for_long_rows(comp):
    # more than 256 group sums per row (d > 2^20): the norm tree's last level runs in its own
    # kernel instead of inside the apply kernel
    kw = dict(COMPRESSORS[comp])
    n, d = 2, (1 << 20) + 4096 * 3 + 77
    pair = Pair(synth.normal_state(n, d, seed=9), synth.ring_csr(n), 0.3, seed=1, **kw)
    grads = synth.GradientStream(n, d, seed=10)
    try:
        for t in range(2):
            det = pair.step(grads.next(), 0.05)
            pair.check(det, tag="long rows %s step %d" % (comp, t))
    finally:
        pair.close()


def test_guess_survives_a_sudden_change_of_scale():
    # the first digit of the threshold jumps by many bins between steps in both directions
    n, d, k = 4, 20000, 200
    pair = Pair(synth.normal_state(n, d, seed=1), synth.ring_csr(n), 0.2, compressor=B.Q_TOPK, k=k)
    try:
        rng = np.random.default_rng(0)
        for t, scale in enumerate([1.0, 1.0, 1e-4, 1e-4, 1e5, 1.0, 1.0]):
            G = (rng.standard_normal((n, d)) * scale).astype(np.float32)
            pair.sgd_step(G, 1.0)
            det = pair.gossip_step()
            pair.check(det, tag="scale jump step %d" % t)
    finally:
        pair.close()


def test_guess_fails_again_and_again_on_long_rows():
    # rows above 2^21 entries repair a failed guess in one launch whose workgroups count themselves
    # in per worker: several failures in one run (the scale of the difference jumps both ways), and
    # enough workers that each gets fewer workgroups than the usual 64
    n, d, k = 20, 2_100_003, 2100
    pair = Pair(synth.normal_state(n, d, seed=3), synth.ring_csr(n), 0.2, compressor=B.Q_TOPK, k=k)
    try:
        rng = np.random.default_rng(1)
        for t, scale in enumerate([1.0, 1e-4, 1e5, 1.0, 1e-3]):
            G = (rng.standard_normal((n, d)) * scale).astype(np.float32)
            det = pair.step(G, 1.0)
            pair.check(det, tag="long rows, scale jump, step %d" % t)
        assert np.all(pair.gpu.last_scalars()[:, 4] >= 2)    # steps so far that needed the fallback, per worker
    finally:
        pair.close()


def test_zero_state_and_zero_norm():
    n, d = 4, 1000
    for comp in ("sign", "qsgd16", "topk"):
        kw = dict(COMPRESSORS[comp])
        if comp == "topk":
            kw["k"] = 10
        pair = Pair(np.zeros((n, d), dtype=np.float32), synth.ring_csr(n), 0.3, **kw)
        try:
            for t in range(2):
                det = pair.gossip_step()
                pair.check(det, tag="zero %s" % comp)
        finally:
            pair.close()


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("comp", list(COMPRESSORS))
@pytest.mark.parametrize("n,d,mix_form", [(8, 70001, B.MIX_AUTO), (9, 2000, B.MIX_AUTO), (70, 1030, B.MIX_AUTO),
                                          (8, 70001, B.MIX_INCREMENTAL_S), (9, 2000, B.MIX_INCREMENTAL_S),
                                          (70, 1030, B.MIX_DIRECT), (8, 6000, B.MIX_DIRECT)])
def test_fused_step_equals_sgd_then_gossip(n, d, mix_form, comp, order):
    # MIX_AUTO: the direct form up to 64 workers, incremental neighbour sums above
    kw = dict(COMPRESSORS[comp])
    sparse = kw["compressor"] in (B.Q_TOPK, B.Q_RANDK)
    if mix_form != B.MIX_AUTO and not sparse:
        pytest.skip("the dense operators have one form of the mix")
    if sparse:
        kw["k"] = max(1, d // 100)
    pair = Pair(synth.normal_state(n, d, seed=3), topo_for(n), 0.2, order=order, mix_form=mix_form,
                seed=77, **kw)
    grads = synth.GradientStream(n, d, seed=4)
    try:
        for t in range(5):
            det = pair.step(grads.next(), 0.05)
            pair.check(det, tag="fused %s n=%d d=%d order=%d step %d" % (comp, n, d, order, t))
    finally:
        pair.close()


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("comp", ["identity", "sign", "qsgd16", "topk", "randk", "randk_rescaled"])
@pytest.mark.parametrize("n,d,mix_form", [(8, 70001, B.MIX_AUTO), (70, 1030, B.MIX_AUTO), (8, 70001, B.MIX_INCREMENTAL_S),
                                          (8, 6000, B.MIX_DIRECT)])
def test_fused_momentum_step_equals_momentum_then_gossip(n, d, mix_form, comp, order):
    # Algorithm 2: v <- (g + lambda x) + beta v; x <- x - eta v, then the gossip step
    kw = dict(COMPRESSORS[comp])
    sparse = kw["compressor"] in (B.Q_TOPK, B.Q_RANDK)
    if mix_form != B.MIX_AUTO and not sparse:
        pytest.skip("the dense operators have one form of the mix")
    if sparse:
        kw["k"] = max(1, d // 100)
    pair = Pair(synth.normal_state(n, d, seed=3), topo_for(n), 0.2, order=order, mix_form=mix_form,
                seed=78, **kw)
    grads = synth.GradientStream(n, d, seed=5)
    try:
        for t in range(5):
            det = pair.step_momentum(grads.next(), 0.05, 0.9, 1e-4)
            pair.check(det, tag="fused momentum %s n=%d d=%d order=%d step %d" % (comp, n, d, order, t))
    finally:
        pair.close()


def test_sgd_and_momentum_steps_match():
    import torch
    from oracle import choco_ref as ref
    n, d = 6, 12345
    X0 = synth.normal_state(n, d, seed=2)
    pair = Pair(X0, synth.ring_csr(n), 0.3, compressor=B.Q_IDENTITY)
    try:
        rng = np.random.default_rng(1)
        V = np.zeros_like(X0)
        M = torch.zeros_like(pair.X)
        for t in range(4):
            G = rng.standard_normal((n, d)).astype(np.float32)
            Gd = torch.zeros_like(pair.X)
            Gd[:, :d] = torch.from_numpy(G).cuda()
            pair.gpu.momentum_step(Gd, M, 0.05, 0.9, 1e-4)
            pair.ref.momentum_step(V, G, 0.05, 0.9, 1e-4)
            pair.gpu.sync()
            assert np.array_equal(pair.X[:, :d].cpu().numpy(), pair.ref.X)
            assert np.array_equal(M[:, :d].cpu().numpy(), V)
            pair.sgd_step(G, 0.01)
            pair.gpu.sync()
            assert np.array_equal(pair.X[:, :d].cpu().numpy(), pair.ref.X)
    finally:
        pair.close()


def test_metrics_match():
    n, d = 9, 5000
    pair = Pair(synth.normal_state(n, d, seed=4), synth.torus_csr(3, 3), 0.3, compressor=B.Q_SIGN)
    try:
        for _ in range(3):
            pair.gossip_step()
        g, r = pair.gpu.metrics(), pair.ref.metrics()
        for key in ("consensus", "mean_norm", "psi"):
            assert abs(g[key] - r[key]) <= 1e-10 * abs(r[key])
    finally:
        pair.close()


@pytest.mark.parametrize("comp", ["sign", "qsgd16", "topk", "randk"])
def test_same_call_twice_is_bitwise_repeatable(comp):
    import torch
    n, d = 8, 30000
    outs = []
    for _ in range(2):
        kw = dict(COMPRESSORS[comp])
        if kw["compressor"] in (B.Q_TOPK, B.Q_RANDK):
            kw["k"] = 300
        X = torch.from_numpy(synth.normal_state(n, d, seed=8)).cuda().contiguous()
        ctx = B.Choco(X, d, *synth.ring_csr(n), 0.3, seed=3, **kw)
        for _ in range(5):
            ctx.gossip_step()
        ctx.sync()
        outs.append((X.cpu().numpy().copy(), ctx.xhat().cpu().numpy().copy()))
        ctx.close()
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("mix", SPARSE_MIXES)
def test_resume_from_step_counter(mix):
    # random operators are keyed by (seed, t, worker, index): restoring (X, Xhat, S, t)
    # continues a run exactly
    import torch
    n, d, k = 4, 5000, 50
    topo = synth.ring_csr(n)
    X = torch.from_numpy(synth.normal_state(n, d, seed=3)).cuda().contiguous()
    a = B.Choco(X, d, *topo, 0.2, B.Q_RANDK, k=k, seed=11, mix_form=mix)
    for _ in range(3):
        a.gossip_step()
    a.sync()
    X2 = X.clone()
    b = B.Choco(X2, d, *topo, 0.2, B.Q_RANDK, k=k, seed=11, mix_form=mix)
    b.xhat().copy_(a.xhat())
    assert (a.nsum() is None) == (mix == B.MIX_DIRECT)    # the direct form keeps no third vector
    if a.nsum() is not None:
        b.nsum().copy_(a.nsum())
    b.set_step(a.get_step())
    for _ in range(2):
        a.gossip_step()
        b.gossip_step()
    a.sync()
    b.sync()
    assert torch.equal(X, X2) and torch.equal(a.xhat(), b.xhat())
    a.close()
    b.close()


@pytest.mark.parametrize("mix", SPARSE_MIXES)
def test_long_run_statistics_small_workload(mix):
    # the small BASELINE workload: ring of 8, d = 4096, top-1% (k = 41), gamma = 0.05,
    # 200 gossip steps from distinct x_i; consensus error per step and the mean agree
    # with the oracle to 1e-4 (free running)
    n, d, k = 8, 4096, 41
    pair = Pair(synth.normal_state(n, d, seed=20190709), synth.ring_csr(n), 0.05,
                compressor=B.Q_TOPK, k=k, mix_form=mix)
    try:
        for t in range(200):
            pair.gpu.gossip_step()
            pair.ref.gossip_step()
            if t % 20 == 19 or t == 0:
                g, r = pair.gpu.metrics(), pair.ref.metrics()
                assert abs(g["consensus"] - r["consensus"]) <= 1e-4 * r["consensus"]
                assert abs(g["mean_norm"] - r["mean_norm"]) <= 1e-4 * r["mean_norm"]
        X, Xhat, S = pair.gpu_state()
        assert rel_l2(X, pair.ref.X) <= 1e-6
    finally:
        pair.close()


def test_long_run_choco_sgd_sign_1000_steps():
    # datacenter-shaped workload scaled down in d: ring of 8, sign, gamma = 0.4, lr = 0.1,
    # shared x0 ~ N(0, 0.05^2), non-IID synthetic gradients, 1000 steps of (sgd, gossip)
    n, d = 8, 2700
    X0 = synth.normal_state(n, d, seed=7, std=0.05, shared=True)
    pair = Pair(X0, synth.ring_csr(n), 0.4, compressor=B.Q_SIGN)
    grads = synth.GradientStream(n, d, seed=8, noise_std=0.01, bias_std=0.001)
    try:
        for t in range(1000):
            pair.sgd_step(grads.next(), 0.1)
            pair.gpu.gossip_step()
            pair.ref.gossip_step()
        g, r = pair.gpu.metrics(), pair.ref.metrics()
        assert abs(g["consensus"] - r["consensus"]) <= 1e-4 * r["consensus"]
        assert abs(g["mean_norm"] - r["mean_norm"]) <= 1e-4 * r["mean_norm"]
    finally:
        pair.close()


def test_logistic_regression_workload_2000_steps():
    # CHOCO-SGD on synthetic L2-regularised logistic regression: 9 workers on a 3 x 3 torus
    # (weights 1/5), d = 2000, 1000 samples per worker, minibatch 32, scaled sign,
    # lr = 0.1 / (1 + t / 100), 2000 fused iterations.  The gradients are taken at the
    # oracle's iterates; as long as the two sides agree bit for bit (checked on the way)
    # they are the GPU's iterates too.
    n, d = 9, 2000
    prob = synth.LogisticProblem(n, d, samples=1000, seed=5, lam=1e-4, batch=32)
    X0 = np.zeros((n, d), dtype=np.float32)
    pair = Pair(X0, synth.torus_csr(3, 3), 0.1, compressor=B.Q_SIGN)
    loss0 = prob.loss(X0.mean(0))
    try:
        for t in range(2000):
            G = prob.gradient(pair.ref.X, t)
            det = pair.step(G, 0.1 / (1.0 + t / 100.0))
            if t % 250 == 249 or t < 3:
                pair.check(det, tag="logistic step %d" % t)
        g, r = pair.gpu.metrics(), pair.ref.metrics()
        assert abs(g["consensus"] - r["consensus"]) <= 1e-4 * r["consensus"]
        assert abs(g["mean_norm"] - r["mean_norm"]) <= 1e-4 * r["mean_norm"]
        X, _, _ = pair.gpu_state()
        assert prob.loss(X.mean(0)) < loss0 - 0.002        # it did learn (unit-norm features, decaying lr: slowly)
        spread = np.linalg.norm(X - X.mean(0), axis=1).max()
        assert spread < 0.2 * np.linalg.norm(X.mean(0))    # and the workers agree
    finally:
        pair.close()


@pytest.mark.parametrize("comp", ["sign", "qsgd16", "topk", "randk"])
@pytest.mark.parametrize("order", ORDERS)
def test_row_stride_wider_than_the_vector(comp, order):
    # ld rounded up to 64 floats (rows 256-byte aligned, the layout the benchmark uses) and
    # then some: the pad columns are read but never counted, selected or sent
    n, d = 6, 5003
    X0 = synth.normal_state(n, d, seed=41)
    kw = dict(COMPRESSORS[comp])
    if kw["compressor"] in (B.Q_TOPK, B.Q_RANDK):
        kw["k"] = 50
    pair = Pair(X0, synth.ring_csr(n), 0.3, order=order, seed=3, ld_align=64, **kw)
    assert pair.ld == 5056
    grads = synth.GradientStream(n, d, seed=9, noise_std=0.05, bias_std=0.02)
    for t in range(3):
        det = pair.step(grads.next(), 0.1)
        pair.check(det, tag="%s wide rows step %d" % (comp, t))
    assert not pair.gpu.xhat()[:, d:].any() and not pair.X[:, d:].any()
    msgs = pair.gpu.pack_messages()
    dense = pair.gpu.unpack_messages(msgs)
    pair.gpu.sync()
    assert not dense[:, d:].any()
    pair.close()


@pytest.mark.parametrize("mix", SPARSE_MIXES)
@pytest.mark.parametrize("order", ORDERS)
def test_random_masks_selected_ahead_or_not_are_the_same(order, mix):
    # random_a on short rows selects the next step's mask on a second stream; switching that
    # off, on again, moving the step counter and timing the kernels must not change a bit
    n, d, k = 6, 30011, 300
    X0 = synth.normal_state(n, d, seed=51)
    pair = Pair(X0, synth.ring_csr(n), 0.3, order=order, seed=8, compressor=B.Q_RANDK, k=k, randk_rescale=1,
                mix_form=mix)
    grads = synth.GradientStream(n, d, seed=12, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(12):
            if t == 3:
                pair.gpu.set_lookahead(False)
            if t == 6:
                pair.gpu.set_lookahead(True)
            if t == 8:
                pair.gpu.set_profiling(True)
            if t == 10:
                pair.gpu.set_profiling(False)
            if t == 9:       # jump ahead: a mask selected for step 9 must not be used for step 40
                pair.gpu.set_step(40)
                pair.ref.t = 40
            det = pair.step(grads.next(), 0.05)
            pair.check(det, tag="lookahead step %d" % t)
    finally:
        pair.close()


@pytest.mark.parametrize("d,k", [(30011, 300), (400_003, 2000)])
def test_random_masks_selected_ahead_in_batches(d, k):
    # the masks are drawn four steps at a time, a batch ahead: whole batches used up one after the
    # other, and batches cut short at their first, a middle and their last step by a moved step
    # counter (forwards, into the middle of a batch, backwards), by the look-ahead switched off and
    # on and by timed steps; with the bitmap of short rows and with the bit map in global memory,
    # where a batch that is dropped half used leaves marks to clear
    n = 3
    X0 = synth.normal_state(n, d, seed=53)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=10, compressor=B.Q_RANDK, k=k)
    grads = synth.GradientStream(n, d, seed=14, noise_std=0.05, bias_std=0.02)
    moves = {14: 21, 19: 100, 24: 7, 29: 29}          # step of the test -> counter set before it
    off, on = {17, 31, 36}, {18, 33, 37}
    timed_on, timed_off = {26}, {27}
    try:
        for step in range(44):
            if step in moves:
                pair.gpu.set_step(moves[step])
                pair.ref.t = moves[step]
            if step in off:
                pair.gpu.set_lookahead(False)
            if step in on:
                pair.gpu.set_lookahead(True)
            if step in timed_on:
                pair.gpu.set_profiling(True)
            if step in timed_off:
                pair.gpu.set_profiling(False)
            det = pair.step(grads.next(), 0.05)
            pair.check(det, tag="batched lookahead step %d (t = %d)" % (step, pair.ref.t - 1))
    finally:
        pair.close()


@pytest.mark.parametrize("mix", SPARSE_MIXES)
def test_random_masks_selected_ahead_on_rows_without_a_bitmap(mix):
    # above 327,680 entries the kept entries are marked in a bit map in global memory; it exists twice and a
    # mask that was drawn ahead and then dropped (set_step) has its marks cleared again
    n, d, k = 3, 400_003, 3000
    X0 = synth.normal_state(n, d, seed=52)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=9, compressor=B.Q_RANDK, k=k, mix_form=mix)
    grads = synth.GradientStream(n, d, seed=13, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(9):
            if t == 3:
                pair.gpu.set_lookahead(False)
            if t == 5:
                pair.gpu.set_lookahead(True)
            if t == 7:
                pair.gpu.set_step(70)
                pair.ref.t = 70
            if t % 2 == 0:
                det = pair.step(grads.next(), 0.05)
                pair.check(det, tag="lookahead, bit map, step %d" % t)
                continue
            # separate calls, and the message encoder, which marks and clears the same map
            from oracle import choco_ref as ref
            pair.sgd_step(grads.next(), 0.05)
            v = pair.ref.X - pair.ref.Xhat
            tt = pair.ref.t
            det = pair.gossip_step()
            pair.check(det, tag="lookahead, bit map, step %d" % t)
            msgs = pair.gpu.pack_messages()
            dense = pair.gpu.unpack_messages(msgs)
            pair.gpu.sync()
            got = msgs.cpu().numpy().view(np.uint32)
            for i in range(n):
                q, want = ref.pack_message(B.Q_RANDK, v[i], k=k, seed=9, t=tt, worker=i)
                assert np.array_equal(got[i], want)
                assert np.array_equal(dense[i, :d].cpu().numpy(), q)
    finally:
        pair.close()
