"""GPU parity at the full sizes of the benchmark workloads, in the launch configuration
bench.py times (same n, d, k, operator, topology; non-temporal streaming path for the large
states).  Every output is compared with the oracle, element by element."""
import numpy as np
import pytest

from paper_1907_09356_amd import binding as B
from paper_1907_09356_amd import synth
from tests.parity_util import Pair

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


MIXES = [B.MIX_INCREMENTAL_S, B.MIX_DIRECT]   # the library's own choice for these shapes is the second


class GradientPool:
    """Two gradient buffers g = b_i + eps (the distribution of synth.GradientStream), made once in
    float32 and handed out in turn, as bench.py does: at 8 x 28 M entries a fresh float64 draw per
    step costs more than the oracle's step."""

    def __init__(self, n, d, seed, noise_std, bias_std):
        rng = np.random.default_rng(seed)
        self.bufs = []
        bias = None
        if bias_std > 0:
            bias = rng.standard_normal((n, d), dtype=np.float32) * np.float32(bias_std)
        for _ in range(2):
            g = rng.standard_normal((n, d), dtype=np.float32) * np.float32(noise_std)
            if bias is not None:
                g += bias
            self.bufs.append(g)
        self.t = 0

    def next(self):
        g = self.bufs[self.t & 1]
        self.t += 1
        return g


# The inputs of a shape are the same in every test of it: made once, kept for the shapes used
# last (the large ones take seconds to draw, a dozen tests share them).  Nothing writes to them.
_INPUTS = {}


def inputs(n, d, bias_std):
    key = (n, d, bias_std)
    if key not in _INPUTS:
        while len(_INPUTS) >= 2:
            _INPUTS.pop(next(iter(_INPUTS)))
        X0 = synth.normal_state(n, d, seed=20190709, std=0.05, shared=True)
        _INPUTS[key] = (X0, GradientPool(n, d, seed=11, noise_std=0.01, bias_std=bias_std))
    else:
        _INPUTS[key] = _INPUTS.pop(key)     # most recently used last
    X0, grads = _INPUTS[key]
    grads.t = 0
    return X0, grads


def run(n, d, topo, steps, gamma, lr, bias_std, fused=True, layers=None, momentum=False, **kw):
    """fused=True drives choco_step (momentum=True: choco_step_momentum), the calls bench.py
    times; False the two separate calls."""
    X0, grads = inputs(n, d, bias_std)
    pair = Pair(X0, topo, gamma, seed=7, layers=layers, **kw)
    try:
        for t in range(steps):
            if momentum:
                det = pair.step_momentum(grads.next(), lr, 0.9, 1e-4)   # also compares the momentum memory
            elif fused:
                det = pair.step(grads.next(), lr)
            else:
                pair.sgd_step(grads.next(), lr)
                det = pair.gossip_step()
            pair.check(det, tag="full size step %d" % t)
        return pair.gpu.last_scalars() if layers is None else pair.gpu.layer_scalars()
    finally:
        pair.close()


@pytest.mark.parametrize("mix", MIXES)
def test_large_model_shape_topk(mix):
    # n = 8 ring, d = 28,000,000, top-k 0.1 %: step 0 takes the histogram fallback, the
    # later steps the guessed-threshold path; with the neighbour sums kept incrementally
    # (scatter) and with the direct mix (the update of xhat rides on the tile pass)
    steps = 3 if mix == B.MIX_DIRECT else 2
    scal = run(8, 28_000_000, synth.ring_csr(8), steps, 0.01, 0.05, 0.0, compressor=B.Q_TOPK, k=28_000, mix_form=mix)
    assert np.all(scal[:, 3] == 0)


@pytest.mark.parametrize("mix", MIXES)
def test_large_model_shape_topk_in_the_printed_order(mix):
    # Algorithm 1 as printed (mix, then compress): with incremental sums ONE pass over the rows
    # does local update, mix and candidate selection (the 4-vectors-per-thread, non-temporal
    # instantiation that only rows above 2^21 entries take)
    run(8, 28_000_000, synth.ring_csr(8), 2, 0.01, 0.05, 0.0, compressor=B.Q_TOPK, k=28_000,
        order=B.ORDER_MIX_THEN_COMPRESS, mix_form=mix)


@pytest.mark.parametrize("mix", MIXES)
def test_large_model_shape_topk_with_momentum(mix):
    # Algorithm 2 fused into the first pass (choco_step_momentum), 40 B/entry
    run(8, 28_000_000, synth.ring_csr(8), 2, 0.01, 0.05, 0.0, momentum=True, compressor=B.Q_TOPK, k=28_000,
        mix_form=mix)


def test_large_model_shape_randk():
    # the masks of step 1 on are drawn ahead on the second stream; the update of xhat and the
    # deferred local update ride on the tile pass
    run(8, 28_000_000, synth.ring_csr(8), 3, 0.01, 0.05, 0.0, compressor=B.Q_RANDK, k=28_000)


def test_large_model_shape_qsgd():
    run(8, 28_000_000, synth.ring_csr(8), 2, 0.01, 0.05, 0.0, compressor=B.Q_QSGD, levels=16)


@pytest.mark.parametrize("mix", MIXES)
@pytest.mark.parametrize("comp", [B.Q_TOPK, B.Q_RANDK])
@pytest.mark.parametrize("topo", ["ring", "torus"])
def test_peer_to_peer_shape(comp, topo, mix):
    csr = synth.ring_csr(64) if topo == "ring" else synth.torus_csr(8, 8)
    run(64, 270_000, csr, 4, 0.02, 0.1, 0.001, compressor=comp, k=2700, mix_form=mix)


@pytest.mark.parametrize("comp", [B.Q_TOPK, B.Q_RANDK])
def test_peer_to_peer_shape_in_the_printed_order(comp):
    run(64, 270_000, synth.torus_csr(8, 8), 3, 0.02, 0.1, 0.001, compressor=comp, k=2700,
        order=B.ORDER_MIX_THEN_COMPRESS)


@pytest.mark.parametrize("fused", [True, False])
def test_datacenter_shape_sign(fused):
    run(8, 270_000, synth.ring_csr(8), 10, 0.4, 0.1, 0.001, fused=fused, compressor=B.Q_SIGN)


def test_large_model_shape_topk_separate_calls():
    run(8, 28_000_000, synth.ring_csr(8), 1, 0.01, 0.05, 0.0, fused=False, compressor=B.Q_TOPK, k=28_000)


@pytest.mark.parametrize("n,comp,mix", [(8, B.Q_SIGN, B.MIX_AUTO), (64, B.Q_SIGN, B.MIX_AUTO),
                                        (64, B.Q_TOPK, B.MIX_DIRECT), (64, B.Q_TOPK, B.MIX_INCREMENTAL_S),
                                        (64, B.Q_RANDK, B.MIX_DIRECT), (64, B.Q_RANDK, B.MIX_INCREMENTAL_S)])
def test_layer_wise_shapes(n, comp, mix):
    # the 65 layers of the 0.27 M-parameter model (d = 272,474), 1 % of every layer
    layers = synth.layer_table(synth.resnet20_like_lengths(), fraction=0.01)
    d = synth.layers_dim(layers)
    scal = run(n, d, synth.ring_csr(n), 3, 0.4 if comp == B.Q_SIGN else 0.02, 0.1, 0.001, layers=layers,
               compressor=comp, mix_form=mix)
    if comp == B.Q_RANDK:
        big = layers[1] > 10240
        assert np.all(scal[:, big, 3] == 1)     # the bracket around the expected order statistic held


@pytest.mark.parametrize("n,kw", [(8, dict(compressor=B.Q_SIGN)), (64, dict(compressor=B.Q_TOPK, k=2700)),
                                  (64, dict(compressor=B.Q_RANDK, k=2700))])
def test_messages_at_full_size(n, kw):
    from oracle import choco_ref as ref
    d = 270_000
    X0 = synth.normal_state(n, d, seed=20190709, std=0.05, shared=True)
    pair = Pair(X0, synth.ring_csr(n), 0.1, seed=7, **kw)
    grads = synth.GradientStream(n, d, seed=11, noise_std=0.01, bias_std=0.001)
    try:
        for t in range(2):
            pair.sgd_step(grads.next(), 0.1)
            v = pair.ref.X - pair.ref.Xhat
            det = pair.gossip_step()
            pair.check(det, tag="step %d" % t)
            msgs = pair.gpu.pack_messages()
            dense = pair.gpu.unpack_messages(msgs)
            pair.gpu.sync()
            got = msgs.cpu().numpy().view(np.uint32)
            dense = dense.cpu().numpy()
            for i in range(0, n, max(1, n // 8)):      # every worker at n = 8, a sample of 8 at n = 64
                q, want = ref.pack_message(kw["compressor"], v[i], k=kw.get("k", 1), seed=7, t=t, worker=i)
                if kw["compressor"] == B.Q_TOPK:
                    a = got[i].reshape(-1, 2)
                    a = a[np.argsort(a[:, 0], kind="stable")]
                    assert np.array_equal(a.reshape(-1), want)
                else:
                    assert np.array_equal(got[i], want)
                assert np.array_equal(dense[i, :d], q)
    finally:
        pair.close()


def long_run(n, d, topo, steps, gamma, lr, layers=None, **kw):
    """Free-running fused iterations at full size; the long-run statistics to 1e-4 and (the
    two sides never having parted) the final state bit for bit."""
    X0, grads = inputs(n, d, 0.001)
    pair = Pair(X0, topo, gamma, seed=7, layers=layers, **kw)
    try:
        for t in range(steps):
            det = pair.step(grads.next(), lr)
        pair.check(det, tag="after %d steps" % steps)
        g, r = pair.gpu.metrics(), pair.ref.metrics()
        assert abs(g["consensus"] - r["consensus"]) <= 1e-4 * r["consensus"]
        assert abs(g["mean_norm"] - r["mean_norm"]) <= 1e-4 * r["mean_norm"]
    finally:
        pair.close()


def test_datacenter_shape_sign_1000_steps():
    long_run(8, 270_000, synth.ring_csr(8), 1000, 0.4, 0.1, compressor=B.Q_SIGN)


@pytest.mark.parametrize("mix", MIXES)
def test_peer_to_peer_ring_topk_40_steps(mix):
    long_run(64, 270_000, synth.ring_csr(64), 40, 0.02, 0.1, compressor=B.Q_TOPK, k=2700, mix_form=mix)


def test_peer_to_peer_torus_randk_40_steps():
    # the masks of steps 4..39 are all drawn ahead on the second stream, four steps at a time
    long_run(64, 270_000, synth.torus_csr(8, 8), 40, 0.02, 0.1, compressor=B.Q_RANDK, k=2700)


@pytest.mark.parametrize("comp", [B.Q_TOPK, B.Q_RANDK])
def test_peer_to_peer_layer_wise_30_steps(comp):
    # the 65 layers of the 0.27 M-parameter model, free-running: long layers streamed in shared
    # launches, short ones in the layer kernel, the fused direct mix; random_a draws ahead in batches
    layers = synth.layer_table(synth.resnet20_like_lengths(), fraction=0.01)
    d = synth.layers_dim(layers)
    long_run(64, d, synth.ring_csr(64), 30, 0.02, 0.1, layers=layers, compressor=comp)


def test_layer_wise_sign_on_the_language_model_sizes():
    # layers of up to 21.6 M entries (5,281 group sums: the third tree level wraps 20 times)
    layers = synth.layer_table(synth.lstm_like_lengths(), fraction=0.001)
    d = synth.layers_dim(layers)
    run(8, d, synth.ring_csr(8), 2, 0.01, 0.05, 0.0, layers=layers, compressor=B.Q_SIGN)


@pytest.mark.parametrize("comp,mix", [(B.Q_TOPK, B.MIX_DIRECT), (B.Q_TOPK, B.MIX_INCREMENTAL_S),
                                      (B.Q_RANDK, B.MIX_DIRECT)])
def test_layer_wise_selection_on_the_language_model_sizes(comp, mix):
    # 0.1 % of every layer; the 21.6 M-entry layer takes the guessed-threshold select on its own,
    # the 1.69 M-entry layers take it in launches that they share, the biases the layer kernel
    layers = synth.layer_table(synth.lstm_like_lengths(), fraction=0.001)
    d = synth.layers_dim(layers)
    run(8, d, synth.ring_csr(8), 2, 0.01, 0.05, 0.0, layers=layers, compressor=comp, mix_form=mix)


def test_random_k_messages_of_the_large_model_shape():
    # d = 28 M, k = 28,000: ranks through the bit map in global memory (27,344 chunks per worker)
    from oracle import choco_ref as ref
    n, d, k = 8, 28_000_000, 28_000
    X0, grads = inputs(n, d, 0.0)
    pair = Pair(X0, synth.ring_csr(n), 0.01, seed=7, compressor=B.Q_RANDK, k=k)
    try:
        pair.sgd_step(grads.next(), 0.05)
        v = pair.ref.X - pair.ref.Xhat
        det = pair.gossip_step()
        pair.check(det, tag="step 0")
        msgs = pair.gpu.pack_messages()
        dense = pair.gpu.unpack_messages(msgs)
        pair.gpu.sync()
        got = msgs.cpu().numpy().view(np.uint32)
        for i in (0, 5):
            q, want = ref.pack_message(B.Q_RANDK, v[i], k=k, seed=7, t=0, worker=i)
            assert np.array_equal(got[i], want)
            assert np.array_equal(dense[i, :d].cpu().numpy(), q)
    finally:
        pair.close()
