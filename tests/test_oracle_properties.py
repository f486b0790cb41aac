"""Property tests of the oracle on randomly drawn inputs (hypothesis): what Appendix C and
Section 3 fix for every vector, every size and every seed, not only for the hand-picked cases
of the pin tests."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import choco_ref as ref

SETTINGS = dict(max_examples=60, deadline=None)


def vector(seed, d, kind):
    rng = np.random.default_rng(seed)
    v = rng.standard_normal(d).astype(np.float32)
    if kind == 1:                      # few distinct magnitudes and exact zeros: ties everywhere
        v = (rng.integers(-2, 3, size=d) * 0.5).astype(np.float32)
    elif kind == 2:                    # one entry carries almost all of the norm
        v *= np.float32(1e-4)
        v[int(rng.integers(0, d))] = np.float32(3.0)
    return v


@settings(**SETTINGS)
@given(seed=st.integers(0, 2 ** 31), d=st.integers(1, 700), kind=st.integers(0, 2), frac=st.floats(0.0, 1.0))
def test_sparsifiers_keep_exactly_k_entries_and_satisfy_the_compression_bound(seed, d, kind, frac):
    # Appendix C: top_a and random_a keep k entries as they are; ||Q(v) - v||^2 <= (1 - k/d) ||v||^2
    # for top_a on every vector (Definition 1 with omega = k/d; for random_a it holds in expectation)
    v = vector(seed, d, kind)
    k = max(1, min(d, int(round(frac * d))))
    top = ref.compress(ref.TOPK, v, k=k)
    rnd = ref.compress(ref.RANDK, v, k=k, seed=seed, t=3, worker=1)
    q_top, sel_top, q_rnd, sel_rnd = top["q"], top["sel"], rnd["q"], rnd["sel"]
    for q, sel in ((q_top, sel_top), (q_rnd, sel_rnd)):
        sel = np.asarray(sel)
        assert sel.size == k and np.unique(sel).size == k
        kept = np.zeros(d, dtype=bool)
        kept[sel] = True
        assert np.array_equal(q[kept], v[kept]) and not q[~kept].any()
    err = float(np.sum((q_top.astype(np.float64) - v) ** 2))
    assert err <= (1.0 - k / d) * float(np.sum(v.astype(np.float64) ** 2)) * (1 + 1e-12) + 1e-30
    # the k kept magnitudes are the k largest, ties to the lower index
    order = np.lexsort((np.arange(d), -np.abs(v)))
    assert np.array_equal(np.sort(np.asarray(sel_top)), np.sort(order[:k]))


@settings(**SETTINGS)
@given(seed=st.integers(0, 2 ** 31), d=st.integers(1, 700), kind=st.integers(0, 2),
       comp=st.sampled_from(["topk", "randk", "sign", "qsgd"]), levels=st.sampled_from([1, 2, 3, 16, 255]),
       frac=st.floats(0.0, 1.0), biased=st.integers(0, 1), rescale=st.integers(0, 1))
def test_a_packed_message_decodes_to_the_operator_output(seed, d, kind, comp, levels, frac, biased, rescale):
    # whatever the receiver decodes is Q(v), and the message has the size the format states
    v = vector(seed, d, kind)
    c = {"topk": ref.TOPK, "randk": ref.RANDK, "sign": ref.SIGN, "qsgd": ref.QSGD}[comp]
    k = max(1, min(d, int(round(frac * d))))
    kw = dict(k=k, levels=levels, qsgd_biased=biased, randk_rescale=rescale, seed=seed, t=5, worker=2)
    try:
        q, msg = ref.pack_message(c, v, **kw)
    except ValueError:
        # gsgd: more entries at level s than the message has index slots for (documented limit)
        assert comp == "qsgd"
        return
    assert msg.size == ref.message_words(c, d, k=k, levels=levels)
    assert np.array_equal(ref.compress(c, v, **kw)["q"], q)
    back = ref.unpack_message(c, d, msg, **kw)
    assert np.array_equal(back, q)
    assert 32 * msg.size >= ref.paper_message_bits(c, d, k=k, levels=levels) - 32


@settings(max_examples=25, deadline=None)
@given(seed=st.integers(0, 2 ** 31), n=st.integers(2, 7), d=st.integers(1, 300),
       comp=st.sampled_from(["topk", "randk", "sign", "qsgd"]), order=st.integers(0, 1), form=st.integers(0, 1))
def test_a_gossip_step_preserves_the_average_of_the_iterates(seed, n, d, comp, order, form):
    # Section 3: W is doubly stochastic, so every gossip step leaves the worker average where it
    # was, whatever the operator, the order of the two halves and the evaluation of the mix
    rng = np.random.default_rng(seed)
    X0 = rng.standard_normal((n, d)).astype(np.float32)
    row_ptr = np.arange(0, 3 * n + 1, 3, dtype=np.int32) if n >= 3 else np.arange(0, 2 * n + 1, 2, dtype=np.int32)
    if n >= 3:
        col = np.array([sorted({(i - 1) % n, i, (i + 1) % n}) for i in range(n)], dtype=np.int32).reshape(-1)
        w = np.full(col.size, 1.0 / 3.0, dtype=np.float32)
    else:
        col = np.array([0, 1, 0, 1], dtype=np.int32)
        w = np.full(4, 0.5, dtype=np.float32)
    c = {"topk": ref.TOPK, "randk": ref.RANDK, "sign": ref.SIGN, "qsgd": ref.QSGD}[comp]
    st_ = ref.RefState(X0, row_ptr, col, w, gamma=0.3, compressor=c, k=max(1, d // 3), levels=4,
                       order=[ref.COMPRESS_THEN_MIX, ref.MIX_THEN_COMPRESS][order],
                       mix_form=[ref.INCREMENTAL_S, ref.DIRECT][form], seed=seed)
    mean0 = X0.astype(np.float64).mean(axis=0)
    for _ in range(3):
        st_.gossip_step()
    mean = st_.X.astype(np.float64).mean(axis=0)
    scale = max(1.0, float(np.abs(X0).max()))
    assert np.max(np.abs(mean - mean0)) <= 2e-5 * scale


@settings(max_examples=40, deadline=None)
@given(seed=st.integers(0, 2 ** 31), lengths=st.lists(st.integers(1, 200), min_size=1, max_size=6),
       comp=st.sampled_from(["topk", "randk", "sign", "qsgd"]), frac=st.floats(0.0, 1.0))
def test_layer_by_layer_is_the_operator_on_every_slice_and_its_messages_decode(seed, lengths, comp, frac):
    # Section 5: the operator is applied to every layer on its own; a worker's message is the
    # layers' messages one after the other
    start, pos = [], 0
    for ln in lengths:
        start.append(pos)
        pos = (pos + ln + 3) // 4 * 4
    d = start[-1] + lengths[-1]
    k = [max(1, min(ln, int(round(frac * ln)))) for ln in lengths]
    layers = (np.array(start, dtype=np.int64), np.array(lengths, dtype=np.int64), np.array(k, dtype=np.int64))
    v = vector(seed, d, 0)
    for a, ln in zip(start, lengths):       # the padding between layers is never sent
        v[a + ln:(a + ln + 3) // 4 * 4] = 0.0
    c = {"topk": ref.TOPK, "randk": ref.RANDK, "sign": ref.SIGN, "qsgd": ref.QSGD}[comp]
    kw = dict(levels=3, seed=seed, t=4, worker=1)
    try:
        q, msg = ref.pack_layers(c, v, layers, **kw)
    except ValueError:
        assert comp == "qsgd"
        return
    assert msg.size == ref.layers_message_words(c, layers, 3)
    assert np.array_equal(ref.unpack_layers(c, d, msg, layers, **kw), q)
    if comp in ("topk", "sign"):            # no randomness: the slice alone gives the same
        for a, ln, kl in zip(start, lengths, k):
            alone = ref.compress(c, v[a:a + ln], k=kl)["q"]
            assert np.array_equal(q[a:a + ln], alone)
