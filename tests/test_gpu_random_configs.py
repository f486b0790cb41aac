"""GPU parity on randomly drawn configurations: sizes, topologies, operators, orders, mix forms,
layer tables and call sequences come from a seeded generator, so that corners nobody thought of
get a turn (every case is reproducible from its number)."""
import numpy as np
import pytest

from paper_1907_09356_amd import binding as B
from paper_1907_09356_amd import synth
from tests.parity_util import Pair

pytestmark = pytest.mark.gpu


def draw_case(case):
    rng = np.random.default_rng(1000 + case)
    comp = [B.Q_TOPK, B.Q_RANDK, B.Q_SIGN, B.Q_QSGD][case % 4]
    sparse = comp in (B.Q_TOPK, B.Q_RANDK)
    n = int(rng.choice([1, 2, 3, 5, 8, 9, 12, 16, 17]))
    topo_kind = rng.choice(["ring", "torus", "irregular"]) if n >= 4 else "ring"
    if topo_kind == "torus":
        side = {4: (2, 2), 5: (1, 5), 8: (2, 4), 9: (3, 3), 12: (3, 4), 16: (4, 4), 17: (1, 17)}
        a, b = side.get(n, (1, n))
        topo = synth.torus_csr(a, b) if a > 1 and b > 1 else synth.ring_csr(n)
    elif topo_kind == "irregular":
        topo = synth.metropolis_csr(synth.irregular_graph(n, min(n - 1, 6), seed=case))
    else:
        topo = synth.ring_csr(n)
    kw = dict(compressor=comp, order=int(rng.choice([B.ORDER_COMPRESS_THEN_MIX, B.ORDER_MIX_THEN_COMPRESS])),
              seed=int(rng.integers(0, 2 ** 40)))
    layered = bool(rng.random() < 0.4)
    layers = None
    if layered:
        nl = int(rng.integers(1, 9))
        lengths = [int(x) for x in rng.choice([1, 2, 3, 5, 17, 255, 256, 257, 768, 769, 1000, 2561, 3072, 3073, 4099, 10240, 10241, 12000], size=nl)]
        if rng.random() < 0.25:
            lengths[int(rng.integers(0, nl))] = int(rng.choice([40961, 45000, 70001]))   # a long layer
        start, length, k = synth.layer_table(lengths, fraction=float(rng.choice([0.01, 0.05, 0.3])))
        if sparse and nl > 1 and rng.random() < 0.3:
            k[int(rng.integers(0, nl))] = 0
            if k.sum() == 0:
                k[0] = 1
        layers = (start, length, k)
        d = synth.layers_dim(layers)
    else:
        d = int(rng.choice([1, 3, 4, 5, 63, 64, 257, 1000, 4097, 30011, 65536, 100003]))
        if sparse:
            kw["k"] = int(max(1, min(d, rng.choice([1, 2, d // 100 + 1, d // 10 + 1, d]))))
        if sparse and rng.random() < 0.5:
            kw["mix_form"] = int(rng.choice([B.MIX_INCREMENTAL_S, B.MIX_DIRECT]))
    if comp == B.Q_QSGD:
        kw["levels"] = int(rng.choice([1, 2, 3, 16, 255]))
        kw["qsgd_biased"] = int(rng.integers(0, 2))
    if comp == B.Q_RANDK:
        kw["randk_rescale"] = int(rng.integers(0, 2))
    # top_a / random_a layer by layer, default order: MIX_AUTO is the direct form; every other
    # case takes the neighbour sums instead
    if layers is not None and comp in (B.Q_TOPK, B.Q_RANDK) and kw["order"] == B.ORDER_COMPRESS_THEN_MIX and case % 2 == 1:
        kw["mix_form"] = B.MIX_INCREMENTAL_S
    ld_align = int(rng.choice([4, 4, 64]))
    calls = [str(c) for c in rng.choice(["step", "separate", "gossip", "momentum"], size=4)]
    return dict(n=n, d=d, topo=topo, kw=kw, layers=layers, ld_align=ld_align, calls=calls,
                gamma=float(rng.choice([0.05, 0.3, 0.9])), std=float(rng.choice([1.0, 0.05, 1e-3])))


@pytest.mark.parametrize("case", range(160))
def test_random_configuration(case):
    c = draw_case(case)
    n, d = c["n"], c["d"]
    X0 = synth.normal_state(n, d, seed=case, std=c["std"])
    inside = np.ones(d, dtype=bool)
    if c["layers"] is not None:
        inside[:] = False
        for a, ln in zip(c["layers"][0], c["layers"][1]):
            inside[a:a + ln] = True
        X0[:, ~inside] = 0.0
    pair = Pair(X0, c["topo"], c["gamma"], layers=c["layers"], ld_align=c["ld_align"], **c["kw"])
    grads = synth.GradientStream(n, d, seed=case + 7, noise_std=0.05 * c["std"], bias_std=0.02 * c["std"])
    tag = "case %d %s" % (case, {k: v for k, v in c.items() if k not in ("topo", "layers")})
    try:
        for t, call in enumerate(c["calls"]):
            G = grads.next()
            G[:, ~inside] = 0.0
            if call == "step":
                det = pair.step(G, 0.1)
            elif call == "separate":
                pair.sgd_step(G, 0.1)
                det = pair.gossip_step()
            elif call == "momentum":
                det = pair.step_momentum(G, 0.05, 0.9, 1e-4)
            else:
                det = pair.gossip_step()
            pair.check(det, tag="%s, call %d (%s)" % (tag, t, call))
    finally:
        pair.close()


def draw_large_case(case):
    """Shapes that fill the chip (and run the look-ahead selection beside real work)."""
    rng = np.random.default_rng(5000 + case)
    comp = [B.Q_RANDK, B.Q_TOPK, B.Q_RANDK, B.Q_SIGN, B.Q_QSGD][case % 5]
    n = int(rng.choice([32, 48, 64]))
    topo = synth.ring_csr(n) if rng.random() < 0.5 else synth.torus_csr(8, n // 8)
    kw = dict(compressor=comp, seed=int(rng.integers(0, 2 ** 40)),
              order=int(rng.choice([B.ORDER_COMPRESS_THEN_MIX, B.ORDER_MIX_THEN_COMPRESS])))
    layers = None
    if rng.random() < 0.6:
        nl = int(rng.integers(8, 40))
        lengths = [int(x) for x in rng.choice([16, 64, 432, 2304, 4608, 9216, 18432, 36864, 40960], size=nl)]
        if rng.random() < 0.3:
            lengths[0] = int(rng.choice([41000, 147456]))
        layers = synth.layer_table(lengths, fraction=float(rng.choice([0.01, 0.03])))
        d = synth.layers_dim(layers)
    else:
        d = int(rng.choice([100_003, 270_000, 327_680, 327_684, 400_001]))
        if comp in (B.Q_TOPK, B.Q_RANDK):
            kw["k"] = max(1, d // int(rng.choice([100, 1000])))
    if comp == B.Q_QSGD:
        kw["levels"] = int(rng.choice([4, 16]))
    if comp == B.Q_RANDK:
        kw["randk_rescale"] = int(rng.integers(0, 2))
    # top_a / random_a layer by layer, default order: MIX_AUTO is the direct form; every other
    # case takes the neighbour sums instead
    if layers is not None and comp in (B.Q_TOPK, B.Q_RANDK) and kw["order"] == B.ORDER_COMPRESS_THEN_MIX and case % 2 == 1:
        kw["mix_form"] = B.MIX_INCREMENTAL_S
    return dict(n=n, d=d, topo=topo, kw=kw, layers=layers)


@pytest.mark.parametrize("case", range(12))
def test_random_configuration_that_fills_the_chip(case):
    c = draw_large_case(case)
    n, d = c["n"], c["d"]
    X0 = synth.normal_state(n, d, seed=case, std=0.05)
    inside = np.ones(d, dtype=bool)
    if c["layers"] is not None:
        inside[:] = False
        for a, ln in zip(c["layers"][0], c["layers"][1]):
            inside[a:a + ln] = True
        X0[:, ~inside] = 0.0
    pair = Pair(X0, c["topo"], 0.05, layers=c["layers"], ld_align=64, **c["kw"])
    grads = synth.GradientStream(n, d, seed=case + 7, noise_std=0.01, bias_std=0.001)
    try:
        for t in range(4):
            G = grads.next()
            G[:, ~inside] = 0.0
            det = pair.step(G, 0.1)
            pair.check(det, tag="large case %d (n=%d, d=%d, %s) step %d" % (case, n, d, c["kw"], t))
    finally:
        pair.close()


def draw_generic_layers_case(case):
    """Layer tables as a flat parameter vector has them: layers that start anywhere, gaps, entries
    before the first and after the last layer; nothing outside the layers is zeroed."""
    rng = np.random.default_rng(9000 + case)
    comp = [B.Q_TOPK, B.Q_RANDK, B.Q_SIGN, B.Q_QSGD][case % 4]
    sparse = comp in (B.Q_TOPK, B.Q_RANDK)
    n = int(rng.choice([1, 2, 3, 5, 8, 17]))
    topo = synth.ring_csr(n)
    nl = int(rng.integers(1, 12))
    lengths = [int(x) for x in rng.choice([1, 1, 2, 3, 5, 6, 17, 255, 257, 767, 769, 1000, 2559, 3071, 3073, 4099, 10239, 12000], size=nl)]
    if rng.random() < 0.25:
        lengths[int(rng.integers(0, nl))] = int(rng.choice([40958, 40961, 52001]))
    aligned = rng.random() < 0.25           # every fourth table keeps the 4-entry alignment (with non-zero padding)
    start, pos = [], int(rng.integers(0, 6)) * (0 if aligned else 1)
    for ln in lengths:
        if aligned:
            pos = (pos + 3) // 4 * 4
        start.append(pos)
        pos += ln + (0 if aligned else int(rng.choice([0, 0, 0, 1, 2, 3, 7])))
    d = pos + (0 if aligned else int(rng.integers(0, 9)))
    length = np.asarray(lengths, dtype=np.int64)
    k = np.maximum(1, np.floor(float(rng.choice([0.01, 0.05, 0.3])) * length).astype(np.int64))
    if sparse and nl > 1 and rng.random() < 0.3:
        k[int(rng.integers(0, nl))] = 0
        if k.sum() == 0:
            k[0] = 1
    kw = dict(compressor=comp, order=int(rng.choice([B.ORDER_COMPRESS_THEN_MIX, B.ORDER_MIX_THEN_COMPRESS])),
              seed=int(rng.integers(0, 2 ** 40)))
    if comp == B.Q_QSGD:
        kw["levels"] = int(rng.choice([1, 2, 3, 16, 255]))
        kw["qsgd_biased"] = int(rng.integers(0, 2))
    if comp == B.Q_RANDK:
        kw["randk_rescale"] = int(rng.integers(0, 2))
    # top_a / random_a layer by layer, default order: MIX_AUTO is the direct form; every other
    # case takes the neighbour sums instead
    if length is not None and comp in (B.Q_TOPK, B.Q_RANDK) and kw["order"] == B.ORDER_COMPRESS_THEN_MIX and case % 2 == 1:
        kw["mix_form"] = B.MIX_INCREMENTAL_S
    calls = [str(c) for c in rng.choice(["step", "separate", "gossip", "momentum"], size=3)]
    return dict(n=n, d=d, topo=topo, kw=kw, layers=(np.asarray(start, dtype=np.int64), length, k),
                ld_align=int(rng.choice([4, 64])), calls=calls, gamma=float(rng.choice([0.05, 0.3, 0.9])))


@pytest.mark.parametrize("case", range(60))
def test_random_generic_layer_table(case):
    c = draw_generic_layers_case(case)
    n, d = c["n"], c["d"]
    X0 = synth.normal_state(n, d, seed=case + 100)
    pair = Pair(X0, c["topo"], c["gamma"], layers=c["layers"], ld_align=c["ld_align"], **c["kw"])
    grads = synth.GradientStream(n, d, seed=case + 107, noise_std=0.05, bias_std=0.02)
    tag = "generic case %d %s starts %s lengths %s" % (case, c["kw"], c["layers"][0].tolist(), c["layers"][1].tolist())
    try:
        for t, call in enumerate(c["calls"]):
            G = grads.next()
            if call == "step":
                det = pair.step(G, 0.1)
            elif call == "separate":
                pair.sgd_step(G, 0.1)
                det = pair.gossip_step()
            elif call == "momentum":
                det = pair.step_momentum(G, 0.05, 0.9, 1e-4)
            else:
                det = pair.gossip_step()
            pair.check(det, tag="%s, call %d (%s)" % (tag, t, call))
    finally:
        pair.close()
