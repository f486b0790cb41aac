"""Steps replayed from a captured HIP graph.  The operators that do not take the step counter
as a launch argument (sign, top_a) may be captured by the caller once the library keeps all of
its work on the caller's stream; every replay must leave the state the eager calls would."""
import numpy as np
import pytest
import torch

from paper_1907_09356_amd import binding as B, synth
from tests.parity_util import Pair

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,kw", [("sign", dict(compressor=B.Q_SIGN)),
                                     ("topk", dict(compressor=B.Q_TOPK, k=50)),
                                     ("topk_sums", dict(compressor=B.Q_TOPK, k=50, mix_form=B.MIX_INCREMENTAL_S))])
def test_replayed_steps_match_eager_steps(name, kw):
    n, d, steps_in_graph = 6, 5003, 3
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        X0 = synth.normal_state(n, d, seed=61)
        pair = Pair(X0, synth.torus_csr(2, 3), 0.3, seed=3, **kw)
        grads = synth.GradientStream(n, d, seed=62, noise_std=0.05, bias_std=0.02)
        try:
            det = pair.step(grads.next(), 0.05)            # eager steps first (top_a: a threshold guess exists)
            pair.check(det, tag="%s eager step 0" % name)
            det = pair.step(grads.next(), 0.05)
            pair.check(det, tag="%s eager step 1" % name)
            G = grads.next()
            Gd = torch.zeros((n, pair.ld), dtype=torch.float32, device=pair.X.device)
            Gd[:, :d] = torch.from_numpy(np.ascontiguousarray(G, dtype=np.float32)).to(pair.X.device)
            pair.gpu.sync()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):     # recorded, not run
                for _ in range(steps_in_graph):
                    pair.gpu.step(Gd, 0.05)
            side.synchronize()
            for replay in range(3):
                graph.replay()
                side.synchronize()
                for _ in range(steps_in_graph):
                    pair.ref.sgd_step(G, 0.05)
                    det = pair.ref.gossip_step(want_details=True)
                pair.check(det, tag="%s replay %d" % (name, replay))
                # the program's own eager work between the replays
                det = pair.step(grads.next(), 0.05)
                pair.check(det, tag="%s eager step after replay %d" % (name, replay))
        finally:
            pair.close()
