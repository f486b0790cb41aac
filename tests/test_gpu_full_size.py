"""GPU parity at the full sizes of the benchmark workloads, in the launch configuration
bench.py times (same n, d, k, operator, topology; non-temporal streaming path for the large
states).  Every output is compared with the oracle, element by element."""
import numpy as np
import pytest

from paper_1907_09356_amd import binding as B
from paper_1907_09356_amd import synth
from tests.parity_util import Pair

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def run(n, d, topo, steps, gamma, lr, bias_std, **kw):
    X0 = synth.normal_state(n, d, seed=20190709, std=0.05, shared=True)
    pair = Pair(X0, topo, gamma, seed=7, **kw)
    grads = synth.GradientStream(n, d, seed=11, noise_std=0.01, bias_std=bias_std)
    try:
        for t in range(steps):
            pair.sgd_step(grads.next(), lr)
            det = pair.gossip_step()
            pair.check(det, tag="full size step %d" % t)
        return pair.gpu.last_scalars()
    finally:
        pair.close()


def test_large_model_shape_topk():
    # n = 8 ring, d = 28,000,000, top-k 0.1 %: step 0 takes the histogram fallback, the
    # later steps the guessed-threshold path
    scal = run(8, 28_000_000, synth.ring_csr(8), 3, 0.01, 0.05, 0.0, compressor=B.Q_TOPK, k=28_000)
    assert np.all(scal[:, 3] == 0)


def test_large_model_shape_qsgd():
    run(8, 28_000_000, synth.ring_csr(8), 1, 0.01, 0.05, 0.0, compressor=B.Q_QSGD, levels=16)


@pytest.mark.parametrize("comp", [B.Q_TOPK, B.Q_RANDK])
@pytest.mark.parametrize("topo", ["ring", "torus"])
def test_peer_to_peer_shape(comp, topo):
    csr = synth.ring_csr(64) if topo == "ring" else synth.torus_csr(8, 8)
    run(64, 270_000, csr, 4, 0.02, 0.1, 0.001, compressor=comp, k=2700)


def test_datacenter_shape_sign():
    run(8, 270_000, synth.ring_csr(8), 10, 0.4, 0.1, 0.001, compressor=B.Q_SIGN)
