"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU.  Each check is chosen so that a plausible
mistake in the oracle (a dropped term, a wrong sign or index, a transposed
operand, a wrong tie rule) fails at least one of them.
"""
import math
import os

import numpy as np
import pytest

from oracle import choco_ref as ref
from paper_1907_09356_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------
# random numbers
# --------------------------------------------------------------------------
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        vals = [int(x, 16) for x in r]
        out = ref.philox4x32_10(vals[0:4], vals[4:6])
        assert [int(x) for x in out] == vals[6:10]


def test_random_word_counter_layout():
    # word e of worker i at step t on a stream = output (e mod 4) of the block
    # with counter (e // 4, i, t mod 2^32, stream | (t >> 32) << 8), key = seed halves
    seed = 0x0123456789ABCDEF
    for (t, i, e, stream) in [(0, 0, 0, 1), (5, 3, 1027, 2), ((7 << 32) | 9, 63, 2**31 - 1, 1)]:
        blk = ref.philox4x32_10(
            [e >> 2, i, t & 0xFFFFFFFF, stream | ((t >> 32) << 8)],
            [seed & 0xFFFFFFFF, seed >> 32])
        assert ref.random_word(seed, t, i, e, stream) == int(blk[e & 3])


def test_random_words_look_uniform():
    words = np.array([ref.random_word(11, 3, 2, e, ref.STREAM_DITHER) for e in range(20000)],
                     dtype=np.float64) / 2.0**32
    assert abs(words.mean() - 0.5) < 4 * math.sqrt(1 / 12 / 20000)
    hist, _ = np.histogram(words, bins=16, range=(0, 1))
    expected = 20000 / 16
    chi2 = ((hist - expected) ** 2 / expected).sum()
    assert chi2 < 45.0  # 15 dof, p ~ 1e-4


# --------------------------------------------------------------------------
# canonical fp64 sum
# --------------------------------------------------------------------------
@pytest.mark.parametrize("d", [1, 3, 255, 256, 257, 4096, 70001])
def test_canonical_sum_exact_on_integers(d):
    rng = np.random.default_rng(d)
    terms = rng.integers(0, 1000, size=d).astype(np.float64)
    assert ref.canonical_sum(terms) == float(terms.astype(np.int64).sum())


def test_canonical_sum_close_to_exact():
    rng = np.random.default_rng(1)
    terms = np.abs(rng.standard_normal(100003))
    exact = math.fsum(terms)
    got = ref.canonical_sum(terms)
    assert abs(got - exact) <= 64 * np.finfo(np.float64).eps * exact
    # the tree is a fixed association: permuting inputs may change low bits, but
    # summing the same array twice may not
    assert got == ref.canonical_sum(terms.copy())


# --------------------------------------------------------------------------
# The norm tree against a correctly rounded sum.  Appendix C writes ||x||_1 (sign) and
# ||x||_2 (gsgd_b) and says nothing about how they are accumulated; the oracle sums over a
# fixed tree.  What the operators USE of a norm are three fp32 numbers (c, r, step), and
# from them every sign magnitude and every level.  These pins show that, over the classes
# of vectors and the sizes the GPU parity tests run on, those numbers are bit for bit the
# ones a correctly rounded sum (math.fsum) of the same terms gives, so the shape of the
# tree decides nothing that is compared.
# --------------------------------------------------------------------------
NORM_PIN_SIZES = [1, 2, 3, 5, 63, 64, 255, 256, 257, 1023, 4095, 4096, 4097, 10000, 65536, 65537,
                  270_000, 272_474, 1_048_577, 2_800_000]
NORM_PIN_KINDS = ["gauss_1", "gauss_0.05", "gauss_1e-3", "integers", "zeros", "dominant", "mixed_scales"]


def norm_pin_vector(kind, d, seed):
    rng = np.random.default_rng(seed)
    if kind.startswith("gauss_"):
        return (rng.standard_normal(d) * float(kind[6:])).astype(np.float32)
    if kind == "integers":
        return rng.integers(-9, 10, size=d).astype(np.float32)
    if kind == "zeros":
        return np.zeros(d, dtype=np.float32)
    if kind == "dominant":          # one entry carries (nearly) the whole norm
        v = (rng.standard_normal(d) * 1e-4).astype(np.float32)
        v[int(rng.integers(0, d))] = np.float32(-1000.0)
        return v
    if kind == "mixed_scales":      # blocks of very different magnitude: cancellation-free but ill-scaled
        v = rng.standard_normal(d)
        v *= 10.0 ** rng.integers(-6, 4, size=d)
        return v.astype(np.float32)
    raise ValueError(kind)


def scales_from_exact_sums(v, levels, biased):
    """(c, r, step) of Appendix C with the two norms summed exactly and rounded once."""
    d = v.size
    v64 = v.astype(np.float64)
    l1 = math.fsum(np.abs(v64))
    l2sq = math.fsum(v64 * v64)          # a product of two fp32 numbers is exact in fp64
    c = np.float32(l1 / d)
    nrm = math.sqrt(l2sq)
    s = float(levels)
    tau = 1.0 + min(d / (s * s), math.sqrt(d) / s) if biased else 1.0
    if nrm > 0.0:
        return c, np.float32(s / nrm), np.float32(nrm / (tau * s))
    return c, np.float32(0.0), np.float32(0.0)


def bits32(x):
    return int(np.asarray(x, dtype=np.float32).view(np.uint32))


@pytest.mark.parametrize("kind", NORM_PIN_KINDS)
def test_norm_tree_gives_the_scalars_of_a_correctly_rounded_sum(kind):
    differing = []
    for d in NORM_PIN_SIZES:
        for rep in range(2 if d > 100_000 else 4):
            v = norm_pin_vector(kind, d, seed=1000 * d + rep)
            for levels, biased in ((16, 1), (4, 0)):
                c, r, step = scales_from_exact_sums(v, levels, biased)
                sg = ref.compress(ref.SIGN, v)
                qs = ref.compress(ref.QSGD, v, levels=levels, qsgd_biased=biased, seed=9, t=rep, worker=1)
                got = (np.float32(sg["scal"][1]), np.float32(qs["scal"][2]), np.float32(qs["scal"][3]))
                if (bits32(got[0]), bits32(got[1]), bits32(got[2])) != (bits32(c), bits32(r), bits32(step)):
                    differing.append((kind, d, rep, levels, biased))
                    continue
                # every sign magnitude is that c, every gsgd magnitude a level times that step
                assert np.array_equal(np.abs(sg["q"]), np.full(d, c, dtype=np.float32))
                assert np.array_equal(np.abs(qs["q"]), np.abs(qs["codes"]).astype(np.float32) * step)
    # an input on which the tree and the exact sum round to different fp32 scalars would have
    # to be listed and explained in the design notes; none is known
    assert differing == []


@pytest.mark.parametrize("kind", ["gauss_1", "gauss_0.05", "gauss_1e-3", "dominant", "mixed_scales"])
def test_gsgd_levels_are_those_of_a_correctly_rounded_norm(kind):
    # levels recomputed entry by entry in numpy fp32 from the exactly summed norm and the
    # (separately pinned) random words: floor(|v| r + u), u = (word >> 8) 2^-24
    for d in (1, 7, 256, 4097, 20000):
        v = norm_pin_vector(kind, d, seed=77 + d)
        for levels, biased in ((16, 1), (2, 0)):
            _, r, _ = scales_from_exact_sums(v, levels, biased)
            seed, t, worker = 123456789, 3, 2
            words = np.array([ref.random_word(seed, t, worker, e, ref.STREAM_DITHER) for e in range(d)],
                             dtype=np.uint64)
            u = (words >> np.uint64(8)).astype(np.float32) * np.float32(1.0 / 16777216.0)
            a = np.abs(v) * r                         # one fp32 product
            lev = np.floor(a + u).astype(np.int32)    # one fp32 sum
            want = np.where(v < 0, -lev, lev)
            if not float(np.abs(v).max()) > 0.0:
                want[:] = 0
            out = ref.compress(ref.QSGD, v, levels=levels, qsgd_biased=biased, seed=seed, t=t, worker=worker)
            assert np.array_equal(out["codes"], want)


def test_norm_tree_at_the_language_model_size():
    # one worker's difference vector at the largest benchmark size (d = 28,000,000, entries of
    # the spread of the synthetic state): scalars of the tree = scalars of the exact sum
    d = 28_000_000
    v = (np.random.default_rng(2019).standard_normal(d) * 0.05).astype(np.float32)
    c, r, step = scales_from_exact_sums(v, 16, 1)
    sg = ref.compress(ref.SIGN, v)
    assert bits32(sg["scal"][1]) == bits32(c)
    del sg
    qs = ref.compress(ref.QSGD, v, levels=16, qsgd_biased=1, seed=7, t=0, worker=0)
    assert bits32(qs["scal"][2]) == bits32(r) and bits32(qs["scal"][3]) == bits32(step)
    # relative distance of the tree from the exact sums: a few units in the last place of fp64
    v64 = v.astype(np.float64)
    assert abs(qs["scal"][0] - math.fsum(v64 * v64)) <= 8 * np.finfo(np.float64).eps * qs["scal"][0]


def test_norm_tree_is_insensitive_to_its_shape():
    # the same terms summed left to right, pairwise and by the tree agree to a few ulps of
    # fp64 -- 2^29 times finer than the fp32 rounding of the scalars that are compared
    rng = np.random.default_rng(5)
    for d in (1000, 65537, 1_000_003):
        terms = np.abs(rng.standard_normal(d) * 0.05).astype(np.float32).astype(np.float64)
        exact = math.fsum(terms)
        tree = ref.canonical_sum(terms)
        seq = 0.0
        for x in terms[:200000]:
            seq += float(x)
        eps = np.finfo(np.float64).eps
        assert abs(tree - exact) <= 4 * eps * exact
        assert abs(float(np.sum(terms)) - exact) <= 64 * eps * exact      # numpy's pairwise sum
        assert abs(seq - math.fsum(terms[:200000])) <= 200000 * eps * seq  # (sequential: the loose one)


# --------------------------------------------------------------------------
# compression operators (Appendix C)
# --------------------------------------------------------------------------
def brute_topk(v, k):
    order = sorted(range(len(v)), key=lambda e: (-abs(float(v[e])), e))
    return sorted(order[:k])


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_topk_brute_force_with_ties(dtype):
    rng = np.random.default_rng(7)
    cases = [
        np.array([0, 0, 0, 0, 0, 0], dtype=dtype),
        np.array([1, -1, 1, -1, 1, -1, 0.5], dtype=dtype),
        np.array([-0.0, 0.0, 3, -3, 2, 2, -2, 1e-30, -1e-30], dtype=dtype),
        np.array([5, 4, 3, 2, 1], dtype=dtype),
        np.array([1, 2, 3, 4, 5], dtype=dtype),
    ]
    for _ in range(40):
        d = int(rng.integers(1, 64))
        cases.append(rng.integers(-3, 4, size=d).astype(dtype))       # many ties
        cases.append(rng.standard_normal(d).astype(dtype))
    for v in cases:
        for k in sorted({1, max(1, len(v) // 3), len(v)}):
            out = ref.compress(ref.TOPK, v, k=k)
            want = brute_topk(v, k)
            assert out["sel"].tolist() == want
            q = np.zeros_like(v)
            q[want] = v[want]
            assert np.array_equal(out["q"], q)
            # Definition 1 with delta = k/d holds for every single call
            lhs = float(np.sum((out["q"].astype(np.float64) - v.astype(np.float64)) ** 2))
            rhs = (1 - k / len(v)) * float(np.sum(v.astype(np.float64) ** 2))
            assert lhs <= rhs * (1 + 1e-12) + 1e-300


def test_topk_k_equals_d_is_identity():
    v = np.random.default_rng(3).standard_normal(257).astype(np.float32)
    out = ref.compress(ref.TOPK, v, k=257)
    assert np.array_equal(out["q"], v)


def test_randk_is_the_k_smallest_words():
    d, k, seed, t, i = 300, 17, 99, 12, 5
    v = np.random.default_rng(0).standard_normal(d).astype(np.float32)
    out = ref.compress(ref.RANDK, v, k=k, seed=seed, t=t, worker=i)
    words = [ref.random_word(seed, t, i, e, ref.STREAM_RANDK) for e in range(d)]
    want = sorted(sorted(range(d), key=lambda e: (words[e], e))[:k])
    assert out["sel"].tolist() == want
    assert len(set(want)) == k
    q = np.zeros_like(v)
    q[want] = v[want]
    assert np.array_equal(out["q"], q)
    # the unbiased version rescales the kept entries by d/k
    out2 = ref.compress(ref.RANDK, v, k=k, seed=seed, t=t, worker=i, randk_rescale=1)
    assert np.array_equal(out2["sel"], out["sel"])
    assert np.array_equal(out2["q"][want], np.float32(d / k) * v[want])


def test_randk_statistics():
    # each coordinate is kept with probability k/d, so E||Q(v)-v||^2 = (1-k/d)||v||^2
    # with equality, and E[(d/k) v.u] = v for the unbiased version
    d, k, draws = 40, 10, 6000
    v = np.random.default_rng(5).standard_normal(d)
    counts = np.zeros(d)
    err = np.zeros(draws)
    mean_unbiased = np.zeros(d)
    for t in range(draws):
        out = ref.compress(ref.RANDK, v, k=k, seed=2024, t=t, worker=t % 7)
        counts[out["sel"]] += 1
        err[t] = np.sum((out["q"] - v) ** 2)
        mean_unbiased += (d / k) * out["q"]
    p = k / d
    z = (counts - draws * p) / math.sqrt(draws * p * (1 - p))
    assert np.abs(z).max() < 4.5
    target = (1 - p) * np.sum(v ** 2)
    assert abs(err.mean() - target) < 5 * err.std() / math.sqrt(draws)
    mean_unbiased /= draws
    sd = np.abs(v) * math.sqrt((1 - p) / p / draws)
    assert np.all(np.abs(mean_unbiased - v) < 5 * sd + 1e-12)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_sign_closed_form(dtype):
    rng = np.random.default_rng(11)
    for d in (1, 5, 256, 1000):
        v = rng.standard_normal(d).astype(dtype)
        if d >= 5:
            v[2] = 0.0
            v[3] = -0.0
        out = ref.compress(ref.SIGN, v)
        v64 = v.astype(np.float64)
        c = np.abs(v64).sum() / d
        q = out["q"].astype(np.float64)
        tol = 1e-6 if dtype == np.float32 else 1e-13
        assert np.allclose(np.abs(q), c, rtol=tol, atol=0)
        assert len(np.unique(np.abs(out["q"]))) == 1
        # one bit per entry: negative iff v < 0 (zeros of either sign map to +c)
        assert np.array_equal(out["codes"], np.where(v < 0, -1, 1))
        assert np.array_equal(np.signbit(out["q"]), v < 0)
        # ||Q(v)-v||^2 = ||v||^2 - ||v||_1^2/d, i.e. delta = ||v||_1^2/(d ||v||_2^2)
        lhs = np.sum((q - v64) ** 2)
        rhs = np.sum(v64 ** 2) - np.abs(v64).sum() ** 2 / d
        assert abs(lhs - rhs) <= 10 * tol * np.sum(v64 ** 2)
        assert abs(out["scal"][0] - np.abs(v64).sum()) <= 1e-12 * np.abs(v64).sum()


def test_qsgd_level_probabilities_and_unbiasedness():
    d, s, draws = 24, 4, 8000
    v = np.random.default_rng(2).standard_normal(d)
    nrm = np.linalg.norm(v)
    a = s * np.abs(v) / nrm
    up = np.zeros(d)
    mean_q = np.zeros(d)
    for t in range(draws):
        out = ref.compress(ref.QSGD, v, levels=s, qsgd_biased=0, seed=77, t=t, worker=1)
        lev = np.abs(out["codes"])
        assert np.all((lev == np.floor(a)) | (lev == np.floor(a) + 1))
        assert np.array_equal(np.sign(out["codes"][lev > 0]), np.sign(v[lev > 0]).astype(int))
        assert np.allclose(out["q"], np.sign(v) * lev * nrm / s, rtol=1e-12, atol=1e-300)
        up += (lev == np.floor(a) + 1)
        mean_q += out["q"]
    frac = a - np.floor(a)
    sd = np.sqrt(frac * (1 - frac) / draws)
    assert np.all(np.abs(up / draws - frac) < 5 * sd + 1e-9)       # P(round up) = frac
    assert np.all(np.abs(mean_q / draws - v) < 5 * sd * nrm / s + 1e-9)  # E Q(v) = v


def test_qsgd_biased_scaling_and_contraction():
    d, s = 64, 2
    rng = np.random.default_rng(4)
    v = rng.standard_normal(d)
    tau = 1 + min(d / s ** 2, math.sqrt(d) / s)
    errs = []
    for t in range(3000):
        ub = ref.compress(ref.QSGD, v, levels=s, qsgd_biased=0, seed=5, t=t)
        b = ref.compress(ref.QSGD, v, levels=s, qsgd_biased=1, seed=5, t=t)
        assert np.array_equal(ub["codes"], b["codes"])        # same dither, same levels
        assert np.allclose(b["q"] * tau, ub["q"], rtol=1e-12)  # only the scale differs
        errs.append(np.sum((b["q"] - v) ** 2))
    errs = np.array(errs)
    bound = (1 - 1 / tau) * np.sum(v ** 2)
    assert errs.mean() <= bound + 4 * errs.std() / math.sqrt(len(errs))


def test_qsgd_limits():
    v = np.random.default_rng(8).standard_normal(50)
    # many levels: Q(v) -> v / tau with tau -> 1
    s = 1 << 20
    out = ref.compress(ref.QSGD, v, levels=s, qsgd_biased=1, seed=1, t=0)
    tau = 1 + min(50 / s ** 2, math.sqrt(50) / s)
    assert np.allclose(out["q"], v / tau, atol=2 * np.linalg.norm(v) / s)
    # zero vector -> zero
    z = ref.compress(ref.QSGD, np.zeros(9, dtype=np.float32), levels=16, seed=1, t=0)
    assert np.all(z["q"] == 0) and np.all(z["codes"] == 0)
    # one entry carrying the whole norm reaches the top level s
    e = np.zeros(5)
    e[3] = -2.5
    o = ref.compress(ref.QSGD, e, levels=16, qsgd_biased=0, seed=1, t=0)
    assert o["codes"][3] == -16 and o["q"][3] == -2.5


def test_identity_operator():
    v = np.random.default_rng(0).standard_normal(33).astype(np.float32)
    assert np.array_equal(ref.compress(ref.IDENTITY, v)["q"], v)


# --------------------------------------------------------------------------
# topologies (Assumption 1 and the topology table)
# --------------------------------------------------------------------------
def test_topology_spectral_gaps_match_the_paper():
    for line in open(os.path.join(GOLDEN, "topology_spectral_gaps.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        name, n, printed = line.split()
        n = int(n)
        side = int(round(math.sqrt(n)))
        csr = synth.ring_csr(n) if name == "ring" else synth.torus_csr(side, side)
        W = synth.csr_to_dense(*csr)
        assert np.allclose(W, W.T) and np.allclose(W.sum(0), 1, atol=1e-6)
        assert np.allclose(W.sum(1), 1, atol=1e-6)
        lam = np.sort(np.abs(np.linalg.eigvalsh(W)))[::-1]
        rho = 1 - lam[1]
        digits = len(printed.split(".")[1])
        assert abs(rho - float(printed)) <= 0.5 * 10 ** (-digits) + 1e-4, (name, n, rho)


# --------------------------------------------------------------------------
# the gossip step (Algorithm 1 without its gradient step; Appendix A matrix form)
# --------------------------------------------------------------------------
ALL_Q = [
    dict(compressor=ref.IDENTITY),
    dict(compressor=ref.TOPK, k=5),
    dict(compressor=ref.RANDK, k=5),
    dict(compressor=ref.RANDK, k=5, randk_rescale=1),
    dict(compressor=ref.SIGN),
    dict(compressor=ref.QSGD, levels=4),
    dict(compressor=ref.QSGD, levels=4, qsgd_biased=0),
]


def make_state(n, d, dtype, topo, **kw):
    X = synth.normal_state(n, d, seed=123, dtype=dtype)
    return ref.RefState(X, *topo, **kw)


@pytest.mark.parametrize("order", [ref.COMPRESS_THEN_MIX, ref.MIX_THEN_COMPRESS])
@pytest.mark.parametrize("mix_form", [ref.INCREMENTAL_S, ref.DIRECT])
@pytest.mark.parametrize("q", ALL_Q)
def test_average_is_preserved(order, mix_form, q):
    # Assumption 3, first property: X+ 11^T/n = X 11^T/n for any Q and gamma
    for dtype, tol in ((np.float64, 1e-13), (np.float32, 2e-6)):
        # weights rounded to the state's precision: the incremental form needs rows
        # of W that sum to one as exactly as that precision allows
        st = make_state(9, 50, dtype, synth.torus_csr(3, 3, wdtype=dtype), gamma=0.37,
                        order=order, mix_form=mix_form, seed=6, **q)
        mean0 = st.X.astype(np.float64).mean(0)
        for _ in range(25):
            st.gossip_step()
            mean = st.X.astype(np.float64).mean(0)
            # rounding scales with the largest magnitudes that were added up
            scale = max(1.0, np.linalg.norm(mean0), float(np.abs(st.Xhat).max()))
            assert np.linalg.norm(mean - mean0) <= 5 * tol * scale


@pytest.mark.parametrize("mix_form", [ref.INCREMENTAL_S, ref.DIRECT])
def test_identity_gamma_one_is_exact_averaging(mix_form):
    # Appendix A, "Example: exact averaging": X+ = X W.  With Q = identity and
    # gamma = 1 the compress-then-mix order gives it from any state; the
    # printed order gives it from the second step on (once xhat = x).
    for dtype, tol in ((np.float64, 1e-13), (np.float32, 2e-6)):
        topo = synth.ring_csr(8, wdtype=dtype)   # rows sum to one to the state's precision
        W = synth.csr_to_dense(*topo)
        st = make_state(8, 40, dtype, topo, gamma=1.0, compressor=ref.IDENTITY,
                        order=ref.COMPRESS_THEN_MIX, mix_form=mix_form)
        for _ in range(4):
            before = st.X.astype(np.float64)
            want = W @ before
            st.gossip_step()
            assert np.linalg.norm(st.X - want) <= tol * np.linalg.norm(want)
            # xhat absorbed x - xhat, so it now equals the x the step started from
            assert np.linalg.norm(st.Xhat - before) <= tol * np.linalg.norm(before)
        st = make_state(8, 40, dtype, topo, gamma=1.0, compressor=ref.IDENTITY,
                        order=ref.MIX_THEN_COMPRESS, mix_form=mix_form)
        x0 = st.X.copy()
        st.gossip_step()
        assert np.array_equal(st.X, x0)           # xhat = 0: the first mix is a no-op
        assert np.allclose(st.Xhat, x0)
        for _ in range(3):
            want = W @ st.X.astype(np.float64)
            st.gossip_step()
            assert np.linalg.norm(st.X - want) <= tol * np.linalg.norm(want)


def test_asymmetric_weights_are_not_transposed():
    # an irregular graph has w_ij that differ per row; mixing must use row i of
    # W for worker i.  Checked against a dense matrix product.
    adj = np.zeros((6, 6), dtype=bool)
    for a, b in [(0, 1), (0, 2), (0, 3), (1, 2), (3, 4), (4, 5)]:
        adj[a, b] = adj[b, a] = True
    topo = synth.metropolis_csr(adj)
    W = synth.csr_to_dense(*topo)
    assert np.allclose(W, W.T) and np.allclose(W.sum(1), 1)
    st = make_state(6, 30, np.float64, topo, gamma=1.0, compressor=ref.IDENTITY,
                    mix_form=ref.DIRECT)
    want = W @ st.X
    st.gossip_step()
    assert np.allclose(st.X, want, rtol=0, atol=1e-7)  # w is stored as float32


def replica_simulation(X0, W, gamma, k, steps, grads, lr):
    """Algorithm 1 exactly as printed, node by node: every node keeps its own
    replica of xhat_j for itself and each neighbour and only ever reads its own
    memory plus received messages.  Pure Python floats, top_a as Q."""
    n, d = X0.shape
    nbrs = [[j for j in range(n) if W[i, j] != 0] for i in range(n)]
    x = [list(map(float, X0[i])) for i in range(n)]
    rep = [{j: [0.0] * d for j in nbrs[i]} for i in range(n)]
    for t in range(steps):
        for i in range(n):                                   # mixing step
            for e in range(d):
                acc = 0.0
                for j in nbrs[i]:
                    acc += float(W[i, j]) * (rep[i][j][e] - rep[i][i][e])
                x[i][e] += gamma * acc
        msgs = []
        for i in range(n):                                   # compression
            v = [x[i][e] - rep[i][i][e] for e in range(d)]
            keep = sorted(range(d), key=lambda e: (-abs(v[e]), e))[:k]
            msgs.append({e: v[e] for e in keep})
        for i in range(n):                                   # exchange, update of the replicas
            for j in nbrs[i]:
                for e, val in msgs[j].items():
                    rep[i][j][e] += val
        for i in range(n):                                   # local gradient step
            for e in range(d):
                x[i][e] -= lr * float(grads[t][i, e])
    return np.array(x), np.array([rep[i][i] for i in range(n)])


def test_printed_algorithm_against_node_local_replicas():
    n, d, k, steps = 6, 12, 3, 15
    adj = np.zeros((n, n), dtype=bool)
    for a, b in [(0, 1), (1, 2), (2, 3), (3, 4), (4, 5), (5, 0), (0, 3)]:
        adj[a, b] = adj[b, a] = True
    topo = synth.metropolis_csr(adj)
    W = synth.csr_to_dense(*topo)
    X0 = synth.normal_state(n, d, seed=9, dtype=np.float64)
    rng = np.random.default_rng(10)
    grads = [rng.standard_normal((n, d)) for _ in range(steps)]
    want_x, want_xhat = replica_simulation(X0, W, 0.3, k, steps, grads, 0.05)
    for mix_form, tol in ((ref.DIRECT, 1e-12), (ref.INCREMENTAL_S, 1e-10)):
        st = ref.RefState(X0, *topo, gamma=0.3, compressor=ref.TOPK, k=k,
                          order=ref.MIX_THEN_COMPRESS, mix_form=mix_form)
        for t in range(steps):
            st.gossip_step()
            st.sgd_step(grads[t], 0.05)
        assert np.allclose(st.X, want_x, rtol=0, atol=tol)
        assert np.allclose(st.Xhat, want_xhat, rtol=0, atol=tol)


@pytest.mark.parametrize("q", ALL_Q[1:])
@pytest.mark.parametrize("order", [ref.COMPRESS_THEN_MIX, ref.MIX_THEN_COMPRESS])
def test_neighbour_sums_track_their_definition(q, order):
    # S_i = sum_j w_ij xhat_j at all times (the "three vectors" remark), and the
    # two mix forms stay within rounding of each other
    topo = synth.torus_csr(3, 3)
    W = synth.csr_to_dense(*topo)
    a = make_state(9, 64, np.float32, topo, gamma=0.2, order=order,
                   mix_form=ref.INCREMENTAL_S, seed=3, **q)
    b = make_state(9, 64, np.float32, topo, gamma=0.2, order=order, mix_form=ref.DIRECT,
                   seed=3, **q)
    for _ in range(50):
        # teacher-forced: both forms start every step from the same state, because a
        # free-running pair drifts apart by whole quantisation steps once one rounding
        # difference flips a discrete decision
        b.X[...] = a.X
        b.Xhat[...] = a.Xhat
        a.gossip_step()
        b.gossip_step()
        want = W @ a.Xhat.astype(np.float64)
        assert np.linalg.norm(a.S - want) <= 2e-6 * max(np.linalg.norm(want), 1e-3)
        assert np.linalg.norm(a.X.astype(np.float64) - b.X) <= 1e-6 * np.linalg.norm(b.X)
        # in the printed order Q reads the freshly mixed x, so a last-bit difference
        # between the forms can move one stochastic rounding across its threshold:
        # allow isolated whole-level flips for gsgd, none for the other operators
        gap = np.abs(a.Xhat.astype(np.float64) - b.Xhat)
        flipped = int((gap > 1e-5 * np.abs(b.Xhat).max()).sum())
        assert flipped <= (2 if q["compressor"] == ref.QSGD else 0)
        gap[gap > 1e-5 * np.abs(b.Xhat).max()] = 0.0
        assert np.linalg.norm(gap) <= 1e-6 * np.linalg.norm(b.Xhat)


def test_mix_forms_agree_on_long_run_statistics():
    # 1000 free-running steps: consensus error and mean agree to 1e-4 between the
    # incremental and the direct form.  Run with Q = identity and a small gamma so that
    # the comparison is between roundings of one linear recursion that is still above
    # the fp32 floor; with a discrete Q the two runs separate by whole quantisation
    # steps and only the teacher-forced comparison above is meaningful.
    topo = synth.ring_csr(8)
    runs = []
    for mix_form in (ref.INCREMENTAL_S, ref.DIRECT):
        st = make_state(8, 512, np.float32, topo, gamma=0.03, compressor=ref.IDENTITY,
                        mix_form=mix_form)
        for _ in range(1000):
            st.gossip_step()
        runs.append((st.metrics(), st.X.astype(np.float64).mean(0)))
    (ma, xa), (mb, xb) = runs
    assert mb["consensus"] > 1e-7
    assert abs(ma["consensus"] - mb["consensus"]) <= 1e-4 * mb["consensus"]
    assert np.linalg.norm(xa - xb) <= 1e-4 * np.linalg.norm(xb)


def theoretical_gamma(W, delta):
    """Theorem 4.1: gamma = rho^2 delta / (16 rho + rho^2 + 4 beta^2 + 2 rho beta^2 - 8 rho delta)."""
    lam = np.sort(np.abs(np.linalg.eigvalsh(W)))[::-1]
    rho = 1 - lam[1]
    beta = np.linalg.norm(np.eye(len(W)) - W, 2)
    return rho ** 2 * delta / (16 * rho + rho ** 2 + 4 * beta ** 2 + 2 * rho * beta ** 2
                               - 8 * rho * delta), rho


def test_lyapunov_function_decays_linearly():
    # Assumption 3 / Appendix A: Psi(X+, Y+) <= (1 - c) Psi(X, Y), c = rho^2 delta / 82,
    # at the theoretical stepsize, for the deterministic top_a (delta = k/d) from
    # arbitrary (X, Y); checked per step along a trajectory in fp64.
    n, d, k = 4, 16, 4
    topo = synth.ring_csr(n)
    W = synth.csr_to_dense(*topo)
    gamma, rho = theoretical_gamma(W, k / d)
    c = rho ** 2 * (k / d) / 82
    st = ref.RefState(synth.normal_state(n, d, seed=1, dtype=np.float64), *topo, gamma=gamma,
                      compressor=ref.TOPK, k=k, order=ref.MIX_THEN_COMPRESS, mix_form=ref.DIRECT)
    st.Xhat[...] = synth.normal_state(n, d, seed=2, dtype=np.float64)   # arbitrary Y
    psi = st.metrics()["psi"]
    for _ in range(300):
        st.gossip_step()
        new = st.metrics()["psi"]
        assert new <= (1 - c) * psi * (1 + 1e-12)
        psi = new


@pytest.mark.parametrize("order", [ref.COMPRESS_THEN_MIX, ref.MIX_THEN_COMPRESS])
def test_consensus_error_decays_log_linearly_at_practical_stepsize(order):
    # the small BASELINE workload: ring of 8, d = 4096, top-1%, gamma = 0.05
    n, d, k = 8, 4096, 41
    st = ref.RefState(synth.normal_state(n, d, seed=20190709, dtype=np.float32),
                      *synth.ring_csr(n), gamma=0.05, compressor=ref.TOPK, k=k, order=order)
    errs = []
    for _ in range(200):
        st.gossip_step()
        errs.append(st.metrics()["consensus"])
    errs = np.array(errs)
    assert abs(errs[0] - d * (1 - 1 / n)) < 0.1 * d        # starts near d (1 - 1/n)
    t = np.arange(len(errs))
    slope, icpt = np.polyfit(t, np.log(errs), 1)
    resid = np.log(errs) - (slope * t + icpt)
    r2 = 1 - resid.var() / np.log(errs).var()
    assert slope < 0 and r2 > 0.99
    assert errs[-1] < errs[0]


def test_error_feedback_form_emits_the_same_messages():
    # Appendix E (Algorithm 4): v = x^(t) - x^(t-1) + m, q = Q(v), m <- v - q, with
    # m^(t) = x^(t-1) - xhat^(t), is Algorithm 1 rewritten.  The rewrite is run
    # here in numpy (fp64) with the oracle's Q and must choose the same entries.
    n, d, k, gamma, lr = 5, 40, 6, 0.25, 0.1
    topo = synth.ring_csr(n, wdtype=np.float64)
    W = synth.csr_to_dense(*topo)
    X0 = synth.normal_state(n, d, seed=4, dtype=np.float64)
    rng = np.random.default_rng(12)
    grads = [rng.standard_normal((n, d)) for _ in range(20)]
    st = ref.RefState(X0, *topo, gamma=gamma, compressor=ref.TOPK, k=k,
                      order=ref.MIX_THEN_COMPRESS, mix_form=ref.DIRECT)
    x = X0.copy()
    x_prev = np.zeros_like(x)
    m = np.zeros_like(x)
    xhat = np.zeros_like(x)
    for t in range(20):
        det = st.gossip_step(want_details=True)
        x = x + gamma * (W @ xhat - xhat)
        v = x - x_prev + m
        q = np.zeros_like(x)
        for i in range(n):
            out = ref.compress(ref.TOPK, v[i], k=k)
            assert out["sel"].tolist() == det["sel"][i].tolist()
            q[i] = out["q"]
        m = v - q
        xhat = xhat + q
        x_prev = x.copy()
        assert np.allclose(xhat, st.Xhat, atol=1e-12)
        assert np.allclose(x, st.X, atol=1e-12)
        st.sgd_step(grads[t], lr)
        x = x - lr * grads[t]


# --------------------------------------------------------------------------
# local updates and metrics
# --------------------------------------------------------------------------
def test_sgd_and_momentum_steps():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((3, 17)).astype(np.float32)
    G = rng.standard_normal((3, 17)).astype(np.float32)
    st = ref.RefState(X, *synth.ring_csr(3), gamma=0.1, compressor=ref.IDENTITY)
    st.sgd_step(G, 0.125)                                      # Algorithm 1, local gradient step
    assert np.array_equal(st.X, X - np.float32(0.125) * G)
    # Algorithm 2: v <- (g + lambda x) + beta v ; x <- x - eta v, against numpy in fp64
    X64 = X.astype(np.float64)
    V = np.zeros_like(X64)
    st = ref.RefState(X64, *synth.ring_csr(3), gamma=0.1, compressor=ref.IDENTITY)
    Vw = np.zeros_like(X64)
    x = X64.copy()
    for _ in range(5):
        g = rng.standard_normal(X.shape)
        V = (g + 1e-4 * x) + 0.9 * V
        x = x - 0.05 * V
        st.momentum_step(Vw, g, 0.05, 0.9, 1e-4)
    assert np.allclose(st.X, x, atol=1e-14) and np.allclose(Vw, V, atol=1e-14)


def test_metrics_against_numpy():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((7, 33))
    st = ref.RefState(X, *synth.ring_csr(7), gamma=0.1, compressor=ref.IDENTITY)
    st.Xhat[...] = rng.standard_normal((7, 33))
    m = st.metrics()
    xbar = X.mean(0)
    assert math.isclose(m["consensus"], ((X - xbar) ** 2).sum() / 7, rel_tol=1e-12)
    assert math.isclose(m["mean_norm"], np.linalg.norm(xbar), rel_tol=1e-12)
    assert math.isclose(m["psi"], ((X - xbar) ** 2).sum() + ((X - st.Xhat) ** 2).sum(),
                        rel_tol=1e-12)


# --------------------------------------------------------------------------
# layer-wise compression (Section 5: the operator is applied to every layer on its own)
# --------------------------------------------------------------------------
LAYER_Q = [
    dict(compressor=ref.TOPK),
    dict(compressor=ref.RANDK),
    dict(compressor=ref.RANDK, randk_rescale=1),
    dict(compressor=ref.SIGN),
    dict(compressor=ref.QSGD, levels=4),
    dict(compressor=ref.QSGD, levels=4, qsgd_biased=0),
]


def test_layer_sizes_of_the_small_model():
    # Section 5: the image model has 0.27 million parameters; Table 1 prints 1.04 MB for
    # the uncompressed fp32 vector, i.e. 4 d bytes in MiB
    lengths = synth.resnet20_like_lengths()
    d = int(lengths.sum())
    assert round(d / 1e6, 2) == 0.27
    assert round(4 * d / 2**20, 2) == 1.04
    start, length, k = synth.layer_table(lengths, fraction=0.01)
    assert np.all(start % 4 == 0) and np.all(start[1:] >= start[:-1] + length[:-1])
    assert synth.layers_dim((start, length, k)) == d     # only the last layer is ragged


@pytest.mark.parametrize("q", LAYER_Q)
@pytest.mark.parametrize("order", [ref.COMPRESS_THEN_MIX, ref.MIX_THEN_COMPRESS])
def test_one_layer_is_the_whole_vector(q, order):
    n, d, k = 5, 300, 17
    X = synth.normal_state(n, d, seed=4)
    topo = synth.ring_csr(n)
    flat = ref.RefState(X, *topo, gamma=0.3, k=k, order=order, seed=9, **q)
    lay = ref.RefState(X, *topo, gamma=0.3, order=order, seed=9,
                       layers=([0], [d], [k]), **q)
    for _ in range(4):
        a = flat.gossip_step(want_details=True)
        b = lay.gossip_step(want_details=True)
        for name in ("sel", "codes"):
            assert (a[name] is None) == (b[name] is None)
            if a[name] is not None:
                assert np.array_equal(a[name], b[name])
        assert np.array_equal(a["scal"], b["scal"][:, 0, :])
        assert np.array_equal(flat.X, lay.X) and np.array_equal(flat.Xhat, lay.Xhat)
        assert np.array_equal(flat.S, lay.S)


@pytest.mark.parametrize("q", [dict(compressor=ref.TOPK), dict(compressor=ref.SIGN)])
def test_layers_of_deterministic_operators_are_compressed_alone(q):
    # each slice gets exactly what the operator gives for that slice as a vector of its own
    # (own norm, own length in the scale, own k); entries in no layer are never sent
    n = 3
    start = np.array([0, 12, 40, 300], dtype=np.int64)
    length = np.array([10, 28, 257, 45], dtype=np.int64)   # gaps at 10..11 and 297..299
    k = np.array([3, 1, 40, 0], dtype=np.int64)
    d = 350                                                # and a tail 345..349 in no layer
    X = synth.normal_state(n, d, seed=8, dtype=np.float64)
    st = ref.RefState(X, *synth.ring_csr(n, wdtype=np.float64), gamma=0.2,
                      layers=(start, length, k), **q)
    st.gossip_step()
    covered = np.zeros(d, dtype=bool)
    for i in range(n):
        for l in range(4):
            sl = slice(start[l], start[l] + length[l])
            covered[sl] = True
            if q["compressor"] == ref.TOPK and k[l] == 0:
                assert not st.Xhat[i, sl].any()
                continue
            alone = ref.compress(q["compressor"], X[i, sl], k=int(max(k[l], 1)))
            assert np.array_equal(st.Xhat[i, sl], alone["q"])   # xhat was 0, so xhat = q
    assert not st.Xhat[:, ~covered].any()


def test_random_layers_use_the_words_of_their_global_coordinates():
    # random_a per layer: the k[l] smallest words among the layer's own coordinates win,
    # each coordinate drawing the word of its index in the whole vector
    n, seed = 2, 77
    start = np.array([0, 20, 100], dtype=np.int64)
    length = np.array([18, 80, 61], dtype=np.int64)
    k = np.array([4, 9, 61], dtype=np.int64)
    d = 161
    X = synth.normal_state(n, d, seed=3)
    st = ref.RefState(X, *synth.ring_csr(n), gamma=0.2, compressor=ref.RANDK, seed=seed,
                      layers=(start, length, k))
    for t in range(3):
        det = st.gossip_step(want_details=True)
        for i in range(n):
            want = []
            for l in range(3):
                es = np.arange(start[l], start[l] + length[l])
                words = np.array([ref.random_word(seed, t, i, int(e), ref.STREAM_RANDK) for e in es])
                order = np.lexsort((es, words))
                want.extend(sorted(es[order[:k[l]]]))
            assert list(det["sel"][i]) == want


def test_quantised_layers_have_their_own_norm_and_tau():
    # gsgd_b per layer, formula of Appendix C retyped for a slice: norm and tau from the
    # slice, dither word from the global coordinate
    n, s, seed = 2, 4, 5
    start = np.array([0, 8], dtype=np.int64)
    length = np.array([7, 33], dtype=np.int64)
    d = 41
    X = synth.normal_state(n, d, seed=12, dtype=np.float64)
    X[:, 8:] *= 100.0                                     # very different norms
    st = ref.RefState(X, *synth.ring_csr(n, wdtype=np.float64), gamma=0.1, compressor=ref.QSGD,
                      levels=s, seed=seed, layers=(start, length, [0, 0]))
    det = st.gossip_step(want_details=True)
    for i in range(n):
        for l in range(2):
            sl = slice(start[l], start[l] + length[l])
            v = X[i, sl]
            nrm = math.sqrt(float((v * v).sum()))
            dl = int(length[l])
            tau = 1.0 + min(dl / s**2, math.sqrt(dl) / s)
            assert det["scal"][i, l, 1] == pytest.approx(nrm, rel=1e-14)
            for j, e in enumerate(range(start[l], start[l] + length[l])):
                u = (ref.random_word(seed, 0, i, e, ref.STREAM_DITHER) >> 8) / 2.0**24
                level = math.floor(s * abs(v[j]) / nrm + u)
                want = math.copysign(level * nrm / (tau * s), v[j])
                assert abs(det["codes"][i, e]) == level
                assert st.Xhat[i, e] == pytest.approx(want, rel=1e-12, abs=1e-300)
    assert not st.Xhat[:, 7].any()     # the gap


@pytest.mark.parametrize("q", LAYER_Q)
def test_layered_steps_keep_the_average_and_converge(q):
    # Assumption 3 does not depend on how Q is built: the average is preserved, and with
    # a contractive operator per layer the consensus error still decays (Theorem 2 applies
    # with the smallest per-layer delta)
    lengths = [40, 5, 130, 64]
    layers = synth.layer_table(lengths, fraction=0.25)
    d = synth.layers_dim(layers)
    n = 6
    X = synth.normal_state(n, d, seed=21, dtype=np.float64)
    inside = np.zeros(d, dtype=bool)
    for a, ln in zip(layers[0], layers[1]):
        inside[a:a + ln] = True
    X[:, ~inside] = 0.0      # padding between layers is never sent, so it must not differ
    st = ref.RefState(X, *synth.ring_csr(n, wdtype=np.float64), gamma=0.05, seed=2, layers=layers, **q)
    mean0 = st.X.mean(0)
    c0 = st.metrics()["consensus"]
    for _ in range(600):
        st.gossip_step()
    m = st.metrics()
    assert np.linalg.norm(st.X.mean(0) - mean0) <= 1e-11 * max(1.0, float(np.abs(st.Xhat).max()))
    unbiased = q.get("randk_rescale") or q.get("qsgd_biased") == 0
    if not unbiased:
        assert m["consensus"] < 1e-3 * c0


# --------------------------------------------------------------------------
# messages on the wire (Appendix C: the size stated with each operator)
# --------------------------------------------------------------------------
def test_message_sizes_match_the_printed_tables():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "message_sizes.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 10
    for source, d, op, par, mb in rows:
        d, mb = int(d), float(mb)
        if op == "identity":
            bits = ref.paper_message_bits(ref.IDENTITY, d)
        elif op == "sign":
            bits = ref.paper_message_bits(ref.SIGN, d)
        elif op == "qsgd_bits":
            bits = ref.paper_message_bits(ref.QSGD, d, levels=2 ** (int(par) - 1))
        else:
            bits = ref.paper_message_bits(ref.TOPK, d, k=int(math.floor(float(par) * d)))
        digits = len(mb.__repr__().split(".")[1])
        assert abs(bits / 8 / 2**20 - mb) <= 0.6 * 10.0 ** -digits, (source, op, par)


def test_message_bit_counts():
    # Appendix C: d + 32 (sign), 2*32*k (top_a), 32*k (random_a), b bits per entry (gsgd_b)
    assert ref.paper_message_bits(ref.SIGN, 1000) == 1032
    assert ref.paper_message_bits(ref.TOPK, 1000, k=10) == 640
    assert ref.paper_message_bits(ref.RANDK, 1000, k=10) == 320
    assert ref.paper_message_bits(ref.QSGD, 1000, levels=8) == 4 * 1000 + 32
    assert ref.paper_message_bits(ref.IDENTITY, 1000) == 32000
    # the byte layout meets those counts up to word padding (and the four index slots of gsgd)
    for d in (32, 64, 4096):
        assert 32 * ref.message_words(ref.SIGN, d) == ref.paper_message_bits(ref.SIGN, d)
        assert (32 * ref.message_words(ref.QSGD, d, levels=8)
                == ref.paper_message_bits(ref.QSGD, d, levels=8) + 4 * 32)
    assert 32 * ref.message_words(ref.TOPK, 1000, k=7) == ref.paper_message_bits(ref.TOPK, 1000, k=7)
    assert 32 * ref.message_words(ref.RANDK, 1000, k=7) == ref.paper_message_bits(ref.RANDK, 1000, k=7)
    assert ref.message_words(ref.SIGN, 33) == 1 + 2


WIRE_Q = [
    (ref.IDENTITY, {}),
    (ref.TOPK, dict(k=9)),
    (ref.RANDK, dict(k=9, seed=5, t=3, worker=2)),
    (ref.RANDK, dict(k=9, seed=5, t=3, worker=2, randk_rescale=1)),
    (ref.SIGN, {}),
    (ref.QSGD, dict(levels=16, seed=8, t=1, worker=4)),
    (ref.QSGD, dict(levels=2, seed=8, qsgd_biased=0)),
    (ref.QSGD, dict(levels=3, seed=8)),
    (ref.QSGD, dict(levels=1, seed=8)),
]


@pytest.mark.parametrize("d", [9, 31, 32, 33, 1000])
@pytest.mark.parametrize("comp,kw", WIRE_Q)
def test_receiver_recovers_q_from_the_message(comp, kw, d):
    v = synth.normal_state(1, d, seed=d)[0]
    v[d // 2] = 0.0
    want = ref.compress(comp, v, **kw)["q"]
    q, msg = ref.pack_message(comp, v, **kw)
    assert np.array_equal(q, want)
    got = ref.unpack_message(comp, d, msg, **kw)
    if comp == ref.QSGD:
        # a zero level is sent without its sign: -0.0 arrives as +0.0
        assert np.array_equal(got, want) and not np.signbit(got[got == 0]).any()
    else:
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))   # also the sign of zeros


def test_message_layouts_bit_by_bit():
    d, s = 77, 8
    v = synth.normal_state(1, d, seed=1)[0]
    W = (d + 31) // 32

    def bits_of(words):   # bit e%32 of word e/32
        return np.unpackbits(words.view(np.uint8), bitorder="little")[:d].astype(bool)

    # sign: the scale, then one bit per entry
    det = ref.compress(ref.SIGN, v)
    _, msg = ref.pack_message(ref.SIGN, v)
    assert msg[:1].view(np.float32)[0] == np.float32(det["scal"][1])
    assert np.array_equal(bits_of(msg[1:1 + W]), v < 0)
    # gsgd: step, four index slots, the sign plane, then magnitude bits lowest first
    det = ref.compress(ref.QSGD, v, levels=s, seed=2)
    _, msg = ref.pack_message(ref.QSGD, v, levels=s, seed=2)
    assert msg[:1].view(np.float32)[0] == np.float32(det["scal"][3])
    assert np.all(msg[1:5] == 0xFFFFFFFF)
    planes = msg[5:].reshape(4, W)                      # 1 + bit_length(s - 1) = 4 planes
    assert np.array_equal(bits_of(planes[0]), det["codes"] < 0)
    level = sum(bits_of(planes[1 + p]).astype(int) << p for p in range(3))
    assert np.array_equal(level, np.abs(det["codes"]))
    # top_a: (index, value) pairs by ascending index; random_a: the values alone
    det = ref.compress(ref.TOPK, v, k=5)
    _, msg = ref.pack_message(ref.TOPK, v, k=5)
    assert np.array_equal(msg[0::2], det["sel"].astype(np.uint32))
    assert np.array_equal(msg[1::2].view(np.float32), v[det["sel"]])
    det = ref.compress(ref.RANDK, v, k=5, seed=4, t=6, worker=1, randk_rescale=1)
    _, msg = ref.pack_message(ref.RANDK, v, k=5, seed=4, t=6, worker=1, randk_rescale=1)
    assert np.array_equal(msg.view(np.float32), det["q"][det["sel"]])


def test_at_most_four_entries_can_reach_the_top_level():
    # floor(|v| r + u) = s needs |v| r >= s - u > s - 1, i.e. |v| / ||v|| > 1 - 1/s >= 1/2 for s >= 2
    # (s = 1 has a magnitude bit for its top level): the squares of four shares of one half are
    # the whole norm, so a fifth cannot exist.  Vectors built to come close: 1 to 5 equal large
    # entries over a small floor; the message's four index slots always suffice.
    rng = np.random.default_rng(12)
    worst = 0
    for s in (2, 4, 16):
        for big in (1, 2, 3, 4, 5):
            for rep in range(60):
                d = int(rng.integers(big, 40))
                v = (rng.standard_normal(d) * 1e-6).astype(np.float32)
                v[rng.choice(d, size=big, replace=False)] = np.float32(rng.choice([-3.0, 3.0]))
                out = ref.compress(ref.QSGD, v, levels=s, qsgd_biased=int(rep & 1), seed=rep, t=rep, worker=big)
                top = int((np.abs(out["codes"]) == s).sum())
                worst = max(worst, top)
                assert top <= 4
                ref.pack_message(ref.QSGD, v, levels=s, qsgd_biased=int(rep & 1), seed=rep, t=rep, worker=big)
    assert worst >= 1      # the construction does reach the top level


def test_gsgd_level_s_travels_through_the_index_slots():
    # one entry holds almost the whole norm: floor(s |v| / ||v|| + u) reaches s, which the
    # magnitude bits (0 .. s-1) cannot hold
    s = 4
    v = np.full(50, 1e-4, dtype=np.float32)
    v[17] = -3.0
    hits = 0
    for t in range(20):
        det = ref.compress(ref.QSGD, v, levels=s, seed=1, t=t)
        q, msg = ref.pack_message(ref.QSGD, v, levels=s, seed=1, t=t)
        if abs(det["codes"][17]) == s:
            hits += 1
            assert msg[1] == 17 and np.all(msg[2:5] == 0xFFFFFFFF)
        assert np.array_equal(ref.unpack_message(ref.QSGD, 50, msg, levels=s, seed=1, t=t), det["q"])
    assert hits >= 10
    # s = 2: up to three entries can get there at once
    v = np.zeros(40, dtype=np.float32)
    v[[3, 20, 33]] = [0.575, -0.575, 0.575]
    seen = 0
    for t in range(200):
        det = ref.compress(ref.QSGD, v, levels=2, seed=3, t=t)
        q, msg = ref.pack_message(ref.QSGD, v, levels=2, seed=3, t=t)
        over = np.flatnonzero(np.abs(det["codes"]) == 2)
        seen = max(seen, over.size)
        assert list(msg[1:1 + over.size]) == list(over)
        assert np.array_equal(ref.unpack_message(ref.QSGD, 40, msg, levels=2, seed=3, t=t), det["q"])
    assert seen >= 2


@pytest.mark.parametrize("comp,kw", [(ref.TOPK, {}), (ref.RANDK, dict(seed=5, t=3, worker=2)),
                                      (ref.SIGN, {}), (ref.QSGD, dict(levels=8, seed=8, t=1, worker=4))])
def test_layered_messages_are_the_layers_messages_one_after_the_other(comp, kw):
    start = np.array([0, 12, 40, 300], dtype=np.int64)
    length = np.array([10, 28, 257, 45], dtype=np.int64)
    k = np.array([3, 0, 40, 5], dtype=np.int64)
    d = 350
    v = synth.normal_state(1, d, seed=2)[0]
    q, msg = ref.pack_layers(comp, v, (start, length, k), **kw)
    # q is what a layered step sends (checked against one) ...
    st = ref.RefState(v[None, :], [0, 1], [0], [1.0], gamma=0.5, compressor=comp, layers=(start, length, k),
                      levels=kw.get("levels", 1), seed=kw.get("seed", 0))
    st.t = kw.get("t", 0)
    if kw.get("worker", 0) == 0:
        st.gossip_step()
        assert np.array_equal(st.Xhat[0], q)
    # ... the message is the concatenation of the per-layer messages (top_a positions global) ...
    off = 0
    sparse = comp in (ref.TOPK, ref.RANDK)
    for l in range(4):
        if sparse and k[l] == 0:
            continue
        sl = slice(start[l], start[l] + length[l])
        ql, ml = ref.pack_message(comp, v[sl], k=int(k[l]) if sparse else 1, **kw) if not kw.get("seed") else (None, None)
        words = ref.message_words(comp, int(length[l]), int(k[l]) if sparse else 0, kw.get("levels", 1))
        if ml is not None:          # operators without random words: the slice alone gives the same message
            ml = ml.copy()
            if comp == ref.TOPK:
                ml[0::2] += np.uint32(start[l])
            assert np.array_equal(msg[off:off + words], ml)
        off += words
    assert off == msg.size == ref.layers_message_words(comp, (start, length, k), kw.get("levels", 1))
    # ... and the receiver gets q back
    back = ref.unpack_layers(comp, d, msg, (start, length, k), **kw)
    assert np.array_equal(back, q)
    inside = np.zeros(d, dtype=bool)
    for a, ln in zip(start, length):
        inside[a:a + ln] = True
    assert not q[~inside].any()
