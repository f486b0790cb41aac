"""GPU parity of layer-wise compression (Section 5: the operator is applied to every layer
on its own) against the oracle: kept sets, codes, per-layer norms and scales and the whole
state, bit for bit."""
import numpy as np
import pytest

from paper_1907_09356_amd import binding, synth
from tests.parity_util import Pair

pytestmark = pytest.mark.gpu

OPERATORS = [
    ("topk", dict(compressor=binding.Q_TOPK)),
    ("randk", dict(compressor=binding.Q_RANDK)),
    ("randk_rescaled", dict(compressor=binding.Q_RANDK, randk_rescale=1)),
    ("sign", dict(compressor=binding.Q_SIGN)),
    ("qsgd16", dict(compressor=binding.Q_QSGD, levels=16)),
    ("qsgd2_unbiased", dict(compressor=binding.Q_QSGD, levels=2, qsgd_biased=0)),
]
ORDERS = [binding.ORDER_COMPRESS_THEN_MIX, binding.ORDER_MIX_THEN_COMPRESS]
# order of the step and form of the mix: what MIX_AUTO picks in either order (top_a / random_a:
# the direct form with its fused pass, and the neighbour sums in the printed order) and, for
# top_a / random_a, the neighbour sums in the default order too
FORMS = [
    pytest.param(binding.ORDER_COMPRESS_THEN_MIX, binding.MIX_AUTO, id="compress_mix"),
    pytest.param(binding.ORDER_MIX_THEN_COMPRESS, binding.MIX_AUTO, id="mix_compress"),
    pytest.param(binding.ORDER_COMPRESS_THEN_MIX, binding.MIX_INCREMENTAL_S, id="compress_mix_sums"),
]
SPARSE_OPS = (binding.Q_TOPK, binding.Q_RANDK)


def form(q, order, mix_form):
    if mix_form != binding.MIX_AUTO and q["compressor"] not in SPARSE_OPS:
        pytest.skip("sign and gsgd layer by layer have the direct form only")
    return dict(order=order, mix_form=mix_form)

# every size class of the layer kernel (up to 768 / 3,072 / 10,240 entries) and the streaming
# select above it, ragged lengths, one-entry and sub-vector layers, chunk and group boundaries
# of the norm tree
MIXED_LENGTHS = [432, 16, 1, 3, 2304, 255, 256, 257, 768, 769, 2560, 2561, 3072, 3073, 4097, 9216, 10240, 10241,
                 36864, 7, 40960, 10]


def mixed_layers(fraction=0.01):
    start, length, k = synth.layer_table(MIXED_LENGTHS, fraction=fraction)
    k[1] = 0            # a silent layer
    k[3] = length[3]    # a layer sent whole
    return start, length, k


def padded_state(n, layers, seed, std=1.0):
    d = synth.layers_dim(layers)
    X = synth.normal_state(n, d, seed=seed, std=std)
    inside = np.zeros(d, dtype=bool)
    for a, ln in zip(layers[0], layers[1]):
        inside[a:a + ln] = True
    X[:, ~inside] = 0.0
    return X, inside


@pytest.mark.parametrize("order,mix_form", FORMS)
@pytest.mark.parametrize("name,q", OPERATORS)
def test_layered_gossip_steps(name, q, order, mix_form):
    layers = mixed_layers()
    n = 5
    X0, _ = padded_state(n, layers, seed=11)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=5, layers=layers, **form(q, order, mix_form), **q)
    for t in range(4):
        det = pair.gossip_step()
        pair.check(det, tag="%s step %d" % (name, t))
    pair.close()


@pytest.mark.parametrize("order,mix_form", FORMS)
@pytest.mark.parametrize("name,q", OPERATORS)
def test_layered_fused_iterations(name, q, order, mix_form):
    layers = mixed_layers(fraction=0.05)
    n = 6
    X0, inside = padded_state(n, layers, seed=12)
    pair = Pair(X0, synth.torus_csr(2, 3), 0.2, seed=6, layers=layers, **form(q, order, mix_form), **q)
    grads = synth.GradientStream(n, pair.d, seed=3, noise_std=0.05, bias_std=0.02)
    for t in range(4):
        G = grads.next()
        G[:, ~inside] = 0.0
        det = pair.step(G, 0.1)
        pair.check(det, tag="%s fused step %d" % (name, t))
    pair.close()


@pytest.mark.parametrize("mix_form", [binding.MIX_AUTO, binding.MIX_INCREMENTAL_S])
@pytest.mark.parametrize("name,q", [OPERATORS[0], OPERATORS[1], OPERATORS[3]])
def test_layered_momentum_iterations(name, q, mix_form):
    layers = mixed_layers(fraction=0.02)
    n = 4
    X0, inside = padded_state(n, layers, seed=13)
    pair = Pair(X0, synth.ring_csr(n), 0.25, seed=7, layers=layers,
                **form(q, binding.ORDER_COMPRESS_THEN_MIX, mix_form), **q)
    grads = synth.GradientStream(n, pair.d, seed=4, noise_std=0.05, bias_std=0.02)
    for t in range(3):
        G = grads.next()
        G[:, ~inside] = 0.0
        det = pair.step_momentum(G, 0.05, 0.9, 1e-4)
        pair.check(det, tag="%s momentum step %d" % (name, t))
    pair.close()


@pytest.mark.parametrize("order,mix_form", FORMS)
def test_layered_topk_ties_go_to_the_lower_index(order, mix_form):
    # few distinct magnitudes, many exact zeros: the threshold key is shared by far more
    # entries than may be kept, in every size class
    lengths = [100, 2500, 9000, 30000]
    layers = synth.layer_table(lengths, fraction=0.3)
    d = synth.layers_dim(layers)
    n = 3
    rng = np.random.default_rng(5)
    X0 = rng.integers(-2, 3, size=(n, d)).astype(np.float32) * 0.5
    pair = Pair(X0, synth.ring_csr(n), 0.5, compressor=binding.Q_TOPK, order=order, mix_form=mix_form, layers=layers)
    for t in range(3):
        det = pair.gossip_step()
        pair.check(det, tag="ties step %d" % t)
    scal = pair.gpu.layer_scalars()
    assert np.any(scal[:, :, 2] > scal[:, :, 1])      # the tie rule really was exercised
    pair.close()


def test_layered_zero_difference_sends_zeros():
    # x = xhat after a full-precision round: norms are 0, gsgd sends level 0 everywhere
    layers = synth.layer_table([40, 3000], fraction=0.1)
    d = synth.layers_dim(layers)
    X0 = np.zeros((3, d), dtype=np.float32)
    for q in (dict(compressor=binding.Q_QSGD, levels=4), dict(compressor=binding.Q_SIGN),
              dict(compressor=binding.Q_TOPK)):
        pair = Pair(X0, synth.ring_csr(3), 0.4, layers=layers, **q)
        det = pair.gossip_step()
        pair.check(det, tag="zero state")
        pair.close()


@pytest.mark.parametrize("name,q", [OPERATORS[0], OPERATORS[2], OPERATORS[3], OPERATORS[4]])
def test_layers_of_the_small_image_model(name, q):
    # the layer sizes of Section 5's 0.27 M-parameter model, 1 % per layer, on the ring of
    # Table 1 (n = 8)
    layers = synth.layer_table(synth.resnet20_like_lengths(), fraction=0.01)
    n = 8
    X0, inside = padded_state(n, layers, seed=14, std=0.1)
    pair = Pair(X0, synth.ring_csr(n), 0.05, seed=8, layers=layers, **q)
    grads = synth.GradientStream(n, pair.d, seed=5)
    for t in range(3):
        G = grads.next()
        G[:, ~inside] = 0.0
        det = pair.step(G, 0.1)
        pair.check(det, tag="%s resnet-like step %d" % (name, t))
    pair.close()


@pytest.mark.parametrize("order,mix_form", FORMS)
@pytest.mark.parametrize("name,q", [OPERATORS[3], OPERATORS[4]])
def test_dense_layers_of_any_length(name, q, order, mix_form):
    # sign / gsgd stream the rows with per-layer norms: layers far above what one workgroup
    # could hold, with more than 256 group sums (the third tree level wraps), next to tiny ones
    lengths = [5, 1_200_001, 16, 100_003, 4096, 4097, 36864]
    layers = synth.layer_table(lengths, fraction=0.01)
    n = 3
    X0, inside = padded_state(n, layers, seed=15)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=4, layers=layers, **form(q, order, mix_form), **q)
    grads = synth.GradientStream(n, pair.d, seed=7, noise_std=0.05, bias_std=0.02)
    for t in range(3):
        G = grads.next()
        G[:, ~inside] = 0.0
        det = pair.step(G, 0.1)
        pair.check(det, tag="%s long layers step %d" % (name, t))
    pair.close()


def test_dense_layers_with_more_workers_than_the_lds_tile_holds():
    layers = synth.layer_table([300, 5000, 70], fraction=0.01)
    n = 70
    X0, inside = padded_state(n, layers, seed=16)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=4, layers=layers, compressor=binding.Q_SIGN)
    for t in range(2):
        det = pair.gossip_step()
        pair.check(det, tag="sign, 70 workers, step %d" % t)
    pair.close()


@pytest.mark.parametrize("name,q", [OPERATORS[0], OPERATORS[1], OPERATORS[3], OPERATORS[4]])
def test_layers_with_a_wider_row_stride(name, q):
    layers = synth.layer_table([432, 16, 2304, 37, 9216, 10], fraction=0.02)
    n = 4
    X0, inside = padded_state(n, layers, seed=17)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=4, layers=layers, ld_align=64, **q)
    assert pair.ld > pair.d + 3
    grads = synth.GradientStream(n, pair.d, seed=7, noise_std=0.05, bias_std=0.02)
    for t in range(3):
        G = grads.next()
        G[:, ~inside] = 0.0
        det = pair.step(G, 0.1)
        pair.check(det, tag="%s wide rows step %d" % (name, t))
    assert not pair.gpu.xhat()[:, pair.d:].any()
    pair.close()


@pytest.mark.parametrize("order,mix_form", FORMS)
def test_layered_random_masks_selected_ahead_or_not_are_the_same(order, mix_form):
    # layer-wise random_a draws the next step's masks on a second stream; switching that off
    # and on, moving the step counter (a mask drawn for step 9 is dropped, its marks with it)
    # and timing the kernels must not change a bit
    layers = mixed_layers(fraction=0.03)
    n = 6
    X0, inside = padded_state(n, layers, seed=21)
    pair = Pair(X0, synth.ring_csr(n), 0.3, order=order, mix_form=mix_form, seed=9, layers=layers, compressor=binding.Q_RANDK,
                randk_rescale=1)
    grads = synth.GradientStream(n, pair.d, seed=13, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(13):
            if t == 3:
                pair.gpu.set_lookahead(False)
            if t == 6:
                pair.gpu.set_lookahead(True)
            if t == 8:
                pair.gpu.set_profiling(True)
            if t == 10:
                pair.gpu.set_profiling(False)
            if t == 9 or t == 12:   # 12: dropped while the look-ahead is on and a mask is pending
                pair.gpu.set_step(40 + t)
                pair.ref.t = 40 + t
            G = grads.next()
            G[:, ~inside] = 0.0
            det = pair.step(G, 0.05)
            pair.check(det, tag="layered lookahead step %d" % t)
    finally:
        pair.close()


# layers above CHOCO_MAX_LAYER_LEN take the guessed-threshold select of the whole-vector path,
# one layer after the other: a one-block select (41,000 / 50,000 / 300,000), a list long enough
# for the multi-block select (600,000 at 3 %), beside layers of every short class
LONG_LENGTHS = [432, 50000, 7, 41000, 2561, 600000, 10, 300000, 12000]
SPARSE = [OPERATORS[0], OPERATORS[1], OPERATORS[2]]


def long_layers(fraction=0.03):
    start, length, k = synth.layer_table(LONG_LENGTHS, fraction=fraction)
    k[3] = length[3]    # a long layer sent whole
    return start, length, k


@pytest.mark.parametrize("order,mix_form", FORMS)
@pytest.mark.parametrize("name,q", SPARSE)
def test_long_layers_fused_iterations(name, q, order, mix_form):
    layers = long_layers()
    n = 4
    X0, inside = padded_state(n, layers, seed=31)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=15, layers=layers, **form(q, order, mix_form), **q)
    grads = synth.GradientStream(n, pair.d, seed=14, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(4):
            G = grads.next()
            G[:, ~inside] = 0.0
            if t == 2:      # separate calls in between
                pair.sgd_step(G, 0.1)
                det = pair.gossip_step()
            else:
                det = pair.step(G, 0.1)
            pair.check(det, tag="%s long layers step %d" % (name, t))
        scal = pair.gpu.layer_scalars()
        if q["compressor"] == binding.Q_RANDK:
            assert np.all(scal[:, [1, 5, 7], 3] == 1)   # the guess from the key distribution held
    finally:
        pair.close()


def test_long_layers_random_masks_selected_ahead_over_several_batches():
    # a selection made ahead is spread over two streams of the library (layers with launches of
    # their own; layers that share launches and the layer kernel): eleven steps cross two batch
    # boundaries, with the look-ahead switched off and on and the step counter moved in between
    layers = long_layers(fraction=0.02)
    n = 3
    X0, inside = padded_state(n, layers, seed=35)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=19, layers=layers, compressor=binding.Q_RANDK)
    grads = synth.GradientStream(n, pair.d, seed=18, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(11):
            if t == 5:
                pair.gpu.set_lookahead(False)
            if t == 6:
                pair.gpu.set_lookahead(True)
            if t == 9:      # in the middle of a batch: what was selected for the old counter is dropped
                pair.gpu.set_step(101)
                pair.ref.t = 101
            G = grads.next()
            G[:, ~inside] = 0.0
            det = pair.step(G, 0.1)
            pair.check(det, tag="long layers selected ahead, step %d" % t)
    finally:
        pair.close()


@pytest.mark.parametrize("mix_form", [binding.MIX_AUTO, binding.MIX_INCREMENTAL_S])
@pytest.mark.parametrize("name,q", [OPERATORS[0], OPERATORS[1]])
def test_long_layers_momentum_with_a_silent_long_layer(name, q, mix_form):
    start, length, k = long_layers(fraction=0.01)
    k[1] = 0            # a long layer that sends nothing still takes its local update
    layers = (start, length, k)
    n = 3
    X0, inside = padded_state(n, layers, seed=32)
    pair = Pair(X0, synth.ring_csr(n), 0.25, seed=16, layers=layers,
                **form(q, binding.ORDER_COMPRESS_THEN_MIX, mix_form), **q)
    grads = synth.GradientStream(n, pair.d, seed=15, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(3):
            G = grads.next()
            G[:, ~inside] = 0.0
            det = pair.step_momentum(G, 0.05, 0.9, 1e-4)
            pair.check(det, tag="%s silent long layer step %d" % (name, t))
    finally:
        pair.close()


@pytest.mark.parametrize("name,q", [OPERATORS[0], OPERATORS[1]])
def test_a_layer_long_enough_for_the_histogram_fallback(name, q):
    # above 2^21 entries a failed guess (top_a: the first step) is repaired by the sampled
    # histogram and a rebuilt list instead of a scan of the layer
    layers = synth.layer_table([100, 2_200_000, 45000], fraction=0.001)
    n = 3
    X0, inside = padded_state(n, layers, seed=33)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=17, layers=layers, **q)
    grads = synth.GradientStream(n, pair.d, seed=16, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(3):
            G = grads.next()
            G[:, ~inside] = 0.0
            det = pair.step(G, 0.1)
            pair.check(det, tag="%s 2.2 M-entry layer step %d" % (name, t))
    finally:
        pair.close()


@pytest.mark.parametrize("polls", ["0", None])
@pytest.mark.parametrize("layered", [True, False])
@pytest.mark.parametrize("name,q", [OPERATORS[0], OPERATORS[1]])
def test_fallback_workgroups_that_stop_waiting_leave_the_select_to_scan_the_row(name, q, layered, polls, monkeypatch):
    # the workgroups of the fallback launch wait for the one that places the new guess, in a
    # bounded poll; with a bound of zero polls (set from the host) every one of them gives up at
    # once, the list is marked as not to be trusted and the exact select scans the row: same result
    # (polls = None: the library's own bound; the list is rebuilt from the histogram)
    if polls is not None:
        monkeypatch.setenv("CHOCO_FALLBACK_SPIN_LIMIT", polls)
    n = 3
    if layered:
        layers = synth.layer_table([100, 2_200_000, 45000], fraction=0.001)
        X0, inside = padded_state(n, layers, seed=36)
        pair = Pair(X0, synth.ring_csr(n), 0.3, seed=20, layers=layers, **q)
    else:
        d = 2_300_003
        X0, inside = synth.normal_state(n, d, seed=36), np.ones(d, dtype=bool)
        pair = Pair(X0, synth.ring_csr(n), 0.3, seed=20, k=2300, **q)
    grads = synth.GradientStream(n, pair.d, seed=19, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(3):
            G = grads.next()
            G[:, ~inside] = 0.0
            det = pair.step(G, 0.1)
            pair.check(det, tag="%s fallback without the wait, step %d" % (name, t))
            if not layered and t == 0 and q["compressor"] == binding.Q_TOPK:
                # top_a has no guess at the first step: the fallback ran (counted once per worker)
                # and ended in the row scan (mode 2), or the select took the rebuilt list (mode 0)
                scal = pair.gpu.last_scalars()
                assert np.all(scal[:, 4] >= 1)
                assert np.all(scal[:, 3] == (2 if polls == "0" else 0))
    finally:
        pair.close()


def test_long_layer_topk_ties_go_to_the_lower_index():
    layers = synth.layer_table([3000, 120000], fraction=0.2)
    d = synth.layers_dim(layers)
    n = 3
    rng = np.random.default_rng(6)
    X0 = rng.integers(-2, 3, size=(n, d)).astype(np.float32) * 0.5
    pair = Pair(X0, synth.ring_csr(n), 0.5, compressor=binding.Q_TOPK, layers=layers)
    try:
        for t in range(3):
            det = pair.gossip_step()
            pair.check(det, tag="long layer ties step %d" % t)
    finally:
        pair.close()


# --------------------------------------------------------------------------
# Entries outside the layers, and tables as a model's flat parameter vector has them
# --------------------------------------------------------------------------
@pytest.mark.parametrize("order,mix_form", FORMS)
@pytest.mark.parametrize("name,q", OPERATORS)
def test_padding_between_layers_may_hold_anything(name, q, order, mix_form):
    # aligned table (layers start on multiples of 4), but x and g are NOT zero in the padding
    # entries: they are never compressed or sent (q = 0 there), yet the local update and the
    # mix treat them like any entry - exactly what the oracle does with entries in no slice
    layers = mixed_layers(fraction=0.05)
    n = 5
    d = synth.layers_dim(layers)
    X0 = synth.normal_state(n, d, seed=21)          # padding entries as random as the rest
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=5, layers=layers, **form(q, order, mix_form), **q)
    grads = synth.GradientStream(n, d, seed=22, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(4):
            det = pair.step(grads.next(), 0.1)
            pair.check(det, tag="%s non-zero padding step %d" % (name, t))
        inside = np.zeros(d, dtype=bool)
        for a, ln in zip(layers[0], layers[1]):
            inside[a:a + ln] = True
        assert (~inside).any() and not pair.gpu.xhat()[:, :d].cpu().numpy()[:, ~inside].any()
    finally:
        pair.close()


def generic_table(lengths, gaps, fraction=0.05, lead=0, tail=0):
    """(start, length, k), d for layers laid out with the given gaps after each (no alignment)."""
    start, pos = [], lead
    for ln, g in zip(lengths, gaps):
        start.append(pos)
        pos += ln + g
    length = np.asarray(lengths, dtype=np.int64)
    k = np.maximum(1, np.floor(fraction * length).astype(np.int64))
    return (np.asarray(start, dtype=np.int64), length, k), pos + tail


# layers that start anywhere: back to back without padding, several inside one 16-byte piece,
# gaps of 1..9 entries, every size class of the layer kernel, a vector that begins before the
# first layer and goes on after the last
GENERIC_LENGTHS = [5, 1, 2, 1, 433, 17, 2561, 3, 10241, 255, 40957, 7, 9001, 64]
GENERIC_GAPS = [0, 0, 0, 3, 0, 1, 0, 0, 9, 0, 2, 0, 0, 0]


@pytest.mark.parametrize("order,mix_form", FORMS)
@pytest.mark.parametrize("name,q", OPERATORS)
def test_layer_tables_without_alignment(name, q, order, mix_form):
    layers, d = generic_table(GENERIC_LENGTHS, GENERIC_GAPS, lead=3, tail=6)
    layers[2][1] = 0 if q["compressor"] in (binding.Q_TOPK, binding.Q_RANDK) else layers[2][1]   # a silent layer
    assert any(s % 4 for s in layers[0])
    n = 5
    X0 = synth.normal_state(n, d, seed=23)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=6, layers=layers, **form(q, order, mix_form), **q)
    grads = synth.GradientStream(n, d, seed=24, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(4):
            if t % 2:
                pair.sgd_step(grads.next(), 0.1)
                det = pair.gossip_step()
            else:
                det = pair.step(grads.next(), 0.1)      # the local update becomes a pass of its own
            pair.check(det, tag="%s generic table step %d" % (name, t))
    finally:
        pair.close()


@pytest.mark.parametrize("mix_form", [binding.MIX_AUTO, binding.MIX_INCREMENTAL_S])
@pytest.mark.parametrize("name,q", [OPERATORS[0], OPERATORS[1], OPERATORS[3], OPERATORS[4]])
def test_layer_tables_without_alignment_long_layers_and_momentum(name, q, mix_form):
    # layers above 10,240 entries that start off a 16-byte boundary take the streaming select on a
    # piece of the row whose first entries belong to the layer before
    layers, d = generic_table([30, 70001, 3, 41000, 5000, 90000], [0, 0, 1, 0, 0, 0], fraction=0.01, lead=1, tail=2)
    n = 4
    X0 = synth.normal_state(n, d, seed=25)
    pair = Pair(X0, synth.ring_csr(n), 0.25, seed=7, layers=layers,
                **form(q, binding.ORDER_COMPRESS_THEN_MIX, mix_form), **q)
    grads = synth.GradientStream(n, d, seed=26, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(4):
            det = pair.step_momentum(grads.next(), 0.05, 0.9, 1e-4) if t < 2 else pair.step(grads.next(), 0.05)
            pair.check(det, tag="%s generic long layers step %d" % (name, t))
    finally:
        pair.close()


@pytest.mark.parametrize("lead", [1, 3])
def test_long_layers_off_alignment_end_on_a_block_boundary(lead):
    # long layers whose lengths are whole numbers of 2048- and 4096-entry pieces of the streaming
    # pass, started 1 and 3 entries off a 16-byte boundary: their last entries fall into one more
    # piece.  From the second step on the gradient makes those entries the largest of their layers,
    # so a pass that stops a piece short loses kept entries.  One layer takes the multi-block select with launches of its own (3 % of
    # 606,208), the others share launches.
    lengths = [606208, 12288, 20480, 40960]
    layers, d = generic_table(lengths, [0, 0, 5, 0], fraction=0.03, lead=lead, tail=2)
    n = 3
    X0 = synth.normal_state(n, d, seed=35)
    pair = Pair(X0, synth.ring_csr(n), 0.25, seed=8, layers=layers, compressor=binding.Q_TOPK)
    grads = synth.GradientStream(n, d, seed=36, noise_std=0.05, bias_std=0.02)
    ends = np.asarray([a + ln - 1 for a, ln in zip(layers[0], layers[1])])
    try:
        for t in range(4):
            G = grads.next()
            if t >= 1:      # (step 0 scans the rows themselves: no threshold guess yet)
                G[:, ends] = -1000.0 * (t + 1)
                G[:, ends - 1] = 800.0 * (t + 1)
            det = pair.step(G, 0.05)
            pair.check(det, tag="block-boundary layers step %d" % t)
            if t >= 1:
                assert np.all(np.isin(ends, det["sel"][0]))     # (the oracle keeps them, so the parity check bites)
    finally:
        pair.close()


@pytest.mark.parametrize("name,q", OPERATORS)
def test_messages_of_a_layer_table_without_alignment(name, q):
    from oracle import choco_ref as ref
    layers, d = generic_table([5, 1, 2, 433, 17, 2561, 3, 4099], [0, 0, 3, 0, 1, 0, 0, 0], lead=2, tail=5)
    n = 4
    X0 = synth.normal_state(n, d, seed=27)
    pair = Pair(X0, synth.ring_csr(n), 0.3, seed=9, layers=layers, **q)
    grads = synth.GradientStream(n, d, seed=28, noise_std=0.05, bias_std=0.02)
    try:
        for t in range(2):
            pair.sgd_step(grads.next(), 0.1)
            v = pair.ref.X - pair.ref.Xhat
            want = [ref.pack_layers(q["compressor"], v[i], layers, levels=q.get("levels", 1),
                                    qsgd_biased=q.get("qsgd_biased", 1), randk_rescale=q.get("randk_rescale", 0),
                                    seed=pair.ref.seed, t=t, worker=i) for i in range(n)]
            det = pair.gossip_step()
            pair.check(det, tag="%s step %d" % (name, t))
            msgs = pair.gpu.pack_messages()
            got = msgs.cpu().numpy().view(np.uint32)
            dense = pair.gpu.unpack_messages(msgs)
            pair.gpu.sync()
            dense = dense.cpu().numpy()
            for i in range(n):
                if q["compressor"] == binding.Q_TOPK:
                    a = got[i].reshape(-1, 2)
                    b = want[i][1].reshape(-1, 2)
                    assert np.array_equal(a[np.argsort(a[:, 0], kind="stable")], b[np.argsort(b[:, 0], kind="stable")])
                else:
                    assert np.array_equal(got[i], want[i][1]), "%s: worker %d message differs" % (name, i)
                assert np.array_equal(dense[i, :d], want[i][0])
    finally:
        pair.close()
