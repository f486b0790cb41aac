"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1907_09356_amd import binding as B
from paper_1907_09356_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "choco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(choco_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 15
    raw = ctypes.CDLL(B.LIB_PATH)
    for name in names:
        assert hasattr(raw, name), "missing export " + name
    assert sorted(B.EXPORTS) == names


def test_strerror():
    assert B.strerror(B.OK) == "ok"
    for code in (B.E_INVAL, B.E_NOMEM, B.E_HIP, B.E_UNSUPPORTED, -99):
        assert isinstance(B.strerror(code), str) and B.strerror(code)


def cfg(**over):
    topo = over.pop("topo", synth.ring_csr(8))
    kw = dict(n=8, d=1000, gamma=0.1, compressor=B.Q_TOPK, k=10)
    kw.update(over)
    return B.make_config(kw.pop("n"), kw.pop("d"), *topo, kw.pop("gamma"), kw.pop("compressor"), **kw)


def test_workspace_bytes_scales_with_the_state():
    c, keep = cfg()
    small = B.workspace_bytes(c)
    c2, keep2 = cfg(d=100000, k=1000)
    big = B.workspace_bytes(c2)
    assert small >= 2 * 8 * 1000 * 4 and big >= 2 * 8 * 100000 * 4
    c3, keep3 = cfg(d=100000, compressor=B.Q_SIGN)
    assert B.workspace_bytes(c3) < big     # direct mix form keeps no S array


@pytest.mark.parametrize("over", [
    dict(n=0), dict(d=0), dict(d=2 ** 31), dict(d=2 ** 31 - 2 ** 19 + 1, k=5), dict(ld=1001), dict(ld=996), dict(gamma=0.0),
    dict(gamma=-1.0), dict(gamma=float("nan")), dict(gamma=float("inf")), dict(compressor=7),
    dict(k=0), dict(k=1001), dict(compressor=B.Q_QSGD, levels=0), dict(order=2), dict(mix_form=3),
])
def test_bad_scalars_are_rejected(over):
    c, keep = cfg(**over)
    out = ctypes.c_size_t()
    assert B.lib().choco_workspace_bytes(ctypes.byref(c), ctypes.byref(out)) == B.E_INVAL


def test_largest_vector_is_accepted():
    c, keep = cfg(d=2 ** 31 - 2 ** 19, k=5)
    out = ctypes.c_size_t()
    assert B.lib().choco_workspace_bytes(ctypes.byref(c), ctypes.byref(out)) == B.OK
    assert out.value > 8 * 4 * (2 ** 31 - 2 ** 19)


def test_auto_mix_form_keeps_no_third_vector_up_to_64_workers():
    # MIX_AUTO: the direct form wherever the LDS tile of all rows exists; incremental
    # neighbour sums (a third n x d array) above 64 workers and for top_a in the printed order
    def ws(**over):
        c, keep = cfg(d=100000, k=1000, **over)
        return B.workspace_bytes(c)
    state = 8 * 100000 * 4
    assert ws(mix_form=B.MIX_INCREMENTAL_S) - ws(mix_form=B.MIX_DIRECT) >= state - 4096
    assert abs(ws() - ws(mix_form=B.MIX_DIRECT)) < 4096
    assert abs(ws(order=B.ORDER_MIX_THEN_COMPRESS) - ws(mix_form=B.MIX_INCREMENTAL_S,
                                                        order=B.ORDER_MIX_THEN_COMPRESS)) < 4096
    assert abs(ws(compressor=B.Q_RANDK, order=B.ORDER_MIX_THEN_COMPRESS)
               - ws(compressor=B.Q_RANDK, mix_form=B.MIX_DIRECT, order=B.ORDER_MIX_THEN_COMPRESS)) < 4096


def test_unsupported_combination_is_reported():
    c, keep = cfg(compressor=B.Q_SIGN, mix_form=B.MIX_INCREMENTAL_S)
    out = ctypes.c_size_t()
    assert B.lib().choco_workspace_bytes(ctypes.byref(c), ctypes.byref(out)) == B.E_UNSUPPORTED


def init_code(c, x=0x1000, ws=0x10000, nbytes=1 << 40):
    ctx = ctypes.c_void_p(1)
    rc = B.lib().choco_init(ctypes.byref(c), x, ws, nbytes, ctypes.byref(ctx))
    assert ctx.value is None
    return rc


def test_bad_mixing_matrices_are_rejected_before_any_device_work():
    # the pointers below are never dereferenced: validation fails first
    rp, col, w = synth.ring_csr(8)
    bad = []
    w2 = w.copy(); w2[0] = 0.5                       # row does not sum to one / asymmetric
    bad.append((rp, col, w2))
    w3 = w.copy(); w3[1] = -w3[1]                    # negative weight
    bad.append((rp, col, w3))
    col2 = col.copy(); col2[0], col2[1] = col2[1], col2[0]   # columns not ascending
    bad.append((rp, col2, w))
    col3 = col.copy(); col3[2] = 99                  # column out of range
    bad.append((rp, col3, w))
    rp2 = rp.copy(); rp2[0] = 1
    bad.append((rp2, col, w))
    # no self loop: a 4-cycle with weights 1/2 on the two neighbours only
    rp4 = np.array([0, 2, 4, 6, 8], dtype=np.int32)
    col4 = np.array([1, 3, 0, 2, 1, 3, 0, 2], dtype=np.int32)
    w4 = np.full(8, 0.5, dtype=np.float32)
    c4, k4 = B.make_config(4, 100, rp4, col4, w4, 0.1, B.Q_SIGN)
    assert init_code(c4) == B.E_INVAL
    # asymmetric pattern: 0 lists 1 but 1 does not list 0
    rp5 = np.array([0, 2, 3], dtype=np.int32)
    col5 = np.array([0, 1, 1], dtype=np.int32)
    w5 = np.array([0.5, 0.5, 1.0], dtype=np.float32)
    c5, k5 = B.make_config(2, 100, rp5, col5, w5, 0.1, B.Q_SIGN)
    assert init_code(c5) == B.E_INVAL
    for topo in bad:
        c, keep = cfg(topo=topo)
        assert init_code(c) == B.E_INVAL


def test_null_pointers_alignment_and_small_workspace():
    c, keep = cfg()
    assert init_code(c, x=0) == B.E_INVAL
    assert init_code(c, ws=0) == B.E_INVAL
    assert init_code(c, x=0x1004) == B.E_INVAL       # X must be 16-byte aligned
    assert init_code(c, ws=0x10010) == B.E_INVAL     # workspace must be 256-byte aligned
    assert init_code(c, nbytes=B.workspace_bytes(c) - 1) == B.E_NOMEM
    c2, keep2 = B.make_config(8, 1000, None, None, None, 0.1, B.Q_SIGN)
    assert init_code(c2) == B.E_INVAL
    L = B.lib()
    assert L.choco_gossip_step(None) == B.E_INVAL
    assert L.choco_sgd_step(None, 0x1000, 0.1) == B.E_INVAL
    assert L.choco_destroy(None) == B.OK


# layer tables are validated on the host before any device work
def layer_code(d, start, length, k, **over):
    c, keep = cfg(d=d, layers=(start, length, k), **over)
    out = ctypes.c_size_t()
    return B.lib().choco_workspace_bytes(ctypes.byref(c), ctypes.byref(out))


def test_layer_tables_are_validated():
    assert layer_code(1000, [0, 400], [400, 600], [4, 6]) == B.OK
    assert layer_code(1000, [0, 400], [398, 600], [4, 6]) == B.OK          # start padded to 4
    assert layer_code(1000, [0, 400], [400, 600], None, compressor=B.Q_SIGN) == B.OK
    assert layer_code(1000, [0, 400], [400, 600], None) == B.E_INVAL       # top_a needs k per layer
    # any disjoint ascending slices are a layer table: no alignment, gaps allowed
    assert layer_code(1000, [0, 398], [398, 602], [4, 6]) == B.OK          # starts anywhere
    assert layer_code(1000, [0, 404], [400, 596], [4, 6]) == B.OK          # a gap between layers
    assert layer_code(1000, [0, 400], [400, 500], [4, 6]) == B.OK          # the vector goes on after the last layer
    assert layer_code(1000, [4, 400], [396, 600], [4, 6]) == B.OK          # ... and begins before the first
    assert layer_code(1000, [1, 3, 7], [2, 4, 993], [1, 1, 9]) == B.OK     # several layers inside one 16-byte piece
    assert layer_code(1000, [0, 400], [400, 601], [4, 6]) == B.E_INVAL     # runs past d
    assert layer_code(1000, [0, 399], [400, 601], [4, 6]) == B.E_INVAL     # overlap
    assert layer_code(1000, [400, 0], [600, 400], [6, 4]) == B.E_INVAL     # not ascending
    assert layer_code(1000, [0, 400], [400, 600], [401, 6]) == B.E_INVAL   # k above the length
    assert layer_code(1000, [0, 400], [400, 600], [0, 0]) == B.E_INVAL     # nothing ever sent
    assert layer_code(1000, [0, 400], [400, 600], [0, 6]) == B.OK          # one silent layer is fine
    assert layer_code(1000, [0, 400], [400, 0], [4, 0]) == B.E_INVAL


def test_layer_limits_are_reported_as_unsupported():
    limit = 10240    # CHOCO_MAX_LAYER_LEN: longer top_a / random_a layers take the streaming select
    assert layer_code(limit + 8, [0, 8], [8, limit], [1, 10]) == B.OK
    assert layer_code(limit + 9, [0, 8], [8, limit + 1], [1, 10]) == B.OK
    assert layer_code(limit + 9, [0, 8], [8, limit + 1], [1, 0]) == B.OK       # a long silent layer
    assert layer_code(limit + 9, [0, 8], [8, limit + 1], None, compressor=B.Q_SIGN) == B.OK   # dense: any length
    # top_a / random_a layer by layer: the direct form where its fused pass exists (default order)
    assert layer_code(1000, [0, 400], [400, 600], [4, 6], mix_form=B.MIX_DIRECT) == B.OK
    assert layer_code(1000, [0, 400], [400, 600], [4, 6], mix_form=B.MIX_INCREMENTAL_S) == B.OK
    assert layer_code(1000, [0, 400], [400, 600], [4, 6], mix_form=B.MIX_DIRECT,
                      order=B.ORDER_MIX_THEN_COMPRESS) == B.E_UNSUPPORTED
    assert layer_code(1000, [0, 400], [400, 600], None, compressor=B.Q_SIGN, mix_form=B.MIX_DIRECT) == B.E_UNSUPPORTED
    assert layer_code(1000, [0, 400], [400, 600], None, compressor=B.Q_IDENTITY) == B.E_UNSUPPORTED


def test_long_layers_bring_candidate_lists_into_the_workspace():
    start, length, k = synth.layer_table([30000, 70000], fraction=0.01)
    short = synth.layer_table([10000] * 10, fraction=0.01)
    c1, keep1 = cfg(d=100000, layers=(start, length, k))
    c2, keep2 = cfg(d=100000, layers=short)
    assert B.workspace_bytes(c1) > B.workspace_bytes(c2)


def test_layered_workspace_needs_no_candidate_lists():
    c, keep = cfg(d=100000, k=1000)
    flat = B.workspace_bytes(c)
    start, length, k = synth.layer_table([10000] * 10, fraction=0.01)
    c2, keep2 = cfg(d=100000, layers=(start, length, k))
    assert B.workspace_bytes(c2) < flat


def test_random_k_workspace_holds_the_selections_made_ahead():
    # random_a selects four steps ahead on rows up to 2^21 entries (eight copies of the kept lists
    # and maps), one step ahead above (two copies); top_a keeps one copy
    n, d, k = 8, 100_000, 1000
    base, _ = cfg(n=n, d=d, k=k, compressor=B.Q_TOPK)
    rk, _ = cfg(n=n, d=d, k=k, compressor=B.Q_RANDK)
    lists = n * k * 4                               # kept indices of one step
    bitmap = n * ((d + 31) // 32) * 4               # kept-entry bitmap of one step
    extra = B.workspace_bytes(rk) - B.workspace_bytes(base)
    assert extra >= 7 * (lists + bitmap)            # (random_a also keeps Qv, the kept values by entry)
    d2 = (1 << 21) + 4
    base2, _ = cfg(n=n, d=d2, k=k, compressor=B.Q_TOPK, mix_form=B.MIX_INCREMENTAL_S)
    rk2, _ = cfg(n=n, d=d2, k=k, compressor=B.Q_RANDK, mix_form=B.MIX_INCREMENTAL_S)
    extra2 = B.workspace_bytes(rk2) - B.workspace_bytes(base2)
    keptmap = n * ((d2 + 31) // 32) * 4
    assert lists + keptmap <= extra2 < 3 * (lists + keptmap)


def test_paper_message_bits_is_host_arithmetic():
    # Appendix C: d + 32 (sign), 2*32*k (top_a), 32*k (random_a), b bits per entry (gsgd_b)
    assert B.paper_message_bits(B.Q_SIGN, 272474) == 272474 + 32
    assert B.paper_message_bits(B.Q_TOPK, 272474, k=2724) == 64 * 2724
    assert B.paper_message_bits(B.Q_RANDK, 272474, k=2724) == 32 * 2724
    assert B.paper_message_bits(B.Q_QSGD, 1000, levels=128) == 8 * 1000 + 32
    assert B.paper_message_bits(B.Q_IDENTITY, 1000) == 32000
    out = ctypes.c_int64()
    assert B.lib().choco_paper_message_bits(B.Q_TOPK, 100, 0, 1, ctypes.byref(out)) == B.E_INVAL
    assert B.lib().choco_paper_message_bits(9, 100, 1, 1, ctypes.byref(out)) == B.E_INVAL
