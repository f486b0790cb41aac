"""ctypes/numpy front end of the CPU oracle (oracle/choco_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports it.  It holds
no arithmetic of its own: every number comes out of the compiled oracle.
"""
import ctypes
import os

import numpy as np

from . import build as _build

IDENTITY, TOPK, RANDK, SIGN, QSGD = 0, 1, 2, 3, 4
COMPRESS_THEN_MIX, MIX_THEN_COMPRESS = 0, 1
INCREMENTAL_S, DIRECT = 0, 1
STREAM_RANDK, STREAM_DITHER = 1, 2

_lib = None

_i32p = ctypes.POINTER(ctypes.c_int32)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_f64p = ctypes.POINTER(ctypes.c_double)


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if (not os.path.exists(path)
                or os.path.getmtime(path) < os.path.getmtime(_build.SRC)):
            _build.build()
        _lib = ctypes.CDLL(path)
        _lib.choco_ref_random_word.restype = ctypes.c_uint32
        _lib.choco_ref_random_word.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32,
                                               ctypes.c_int64, ctypes.c_int32]
        _lib.choco_ref_canonical_sum.restype = ctypes.c_double
        _lib.choco_ref_canonical_sum.argtypes = [ctypes.c_int64, _f64p]
        _lib.choco_ref_paper_message_bits.restype = ctypes.c_int64
        _lib.choco_ref_paper_message_bits.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64,
                                                      ctypes.c_int32]
        _lib.choco_ref_message_words.restype = ctypes.c_int64
        _lib.choco_ref_message_words.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64,
                                                 ctypes.c_int32]
        f32p = ctypes.POINTER(ctypes.c_float)
        _lib.choco_ref_pack_message.restype = ctypes.c_int
        _lib.choco_ref_pack_message.argtypes = [ctypes.c_int32, ctypes.c_int64, f32p, ctypes.c_int64,
                                                ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32, f32p,
                                                _u32p]
        _lib.choco_ref_unpack_message.restype = ctypes.c_int
        _lib.choco_ref_unpack_message.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64,
                                                  ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                  ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32,
                                                  _u32p, f32p]
        _lib.choco_ref_layers_message_words.restype = ctypes.c_int64
        _lib.choco_ref_layers_message_words.argtypes = [ctypes.c_int32, ctypes.c_int32, _i64p, _i64p,
                                                        ctypes.c_int32]
        _lib.choco_ref_pack_layers.restype = ctypes.c_int
        _lib.choco_ref_pack_layers.argtypes = [ctypes.c_int32, ctypes.c_int64, f32p, ctypes.c_int32, _i64p,
                                               _i64p, _i64p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                               ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32, f32p, _u32p]
        _lib.choco_ref_unpack_layers.restype = ctypes.c_int
        _lib.choco_ref_unpack_layers.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, _i64p, _i64p,
                                                 _i64p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                 ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32, _u32p, f32p]
        for suf, real in (("f32", ctypes.c_float), ("f64", ctypes.c_double)):
            rp = ctypes.POINTER(real)
            f = getattr(_lib, "choco_ref_compress_" + suf)
            f.restype = ctypes.c_int
            f.argtypes = [ctypes.c_int32, ctypes.c_int64, rp, ctypes.c_int64, ctypes.c_int32,
                          ctypes.c_int32, ctypes.c_int32, ctypes.c_uint64, ctypes.c_uint64,
                          ctypes.c_int32, rp, _i32p, _i32p, _f64p]
            f = getattr(_lib, "choco_ref_gossip_step_" + suf)
            f.restype = ctypes.c_int
            f.argtypes = [ctypes.c_int32, ctypes.c_int64, _i32p, _i32p, rp, real,
                          ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                          ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_uint64,
                          ctypes.c_uint64, rp, rp, rp, _i32p, _i32p, _f64p]
            f = getattr(_lib, "choco_ref_gossip_step_layers_" + suf)
            f.restype = ctypes.c_int
            f.argtypes = [ctypes.c_int32, ctypes.c_int64, _i32p, _i32p, rp, real,
                          ctypes.c_int32, ctypes.c_int32, _i64p, _i64p, _i64p, ctypes.c_int32,
                          ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                          ctypes.c_uint64, ctypes.c_uint64, rp, rp, rp, _i32p, _i32p, _f64p]
            f = getattr(_lib, "choco_ref_sgd_step_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int32, ctypes.c_int64, rp, rp, real]
            f = getattr(_lib, "choco_ref_momentum_step_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int32, ctypes.c_int64, rp, rp, rp, real, real, real]
            f = getattr(_lib, "choco_ref_metrics_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int32, ctypes.c_int64, rp, rp, _f64p, _f64p, _f64p]
    return _lib


def _suffix(dtype):
    dtype = np.dtype(dtype)
    if dtype == np.float32:
        return "f32", ctypes.c_float
    if dtype == np.float64:
        return "f64", ctypes.c_double
    raise TypeError("oracle state must be float32 or float64, got %s" % dtype)


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype)) if a is not None else None


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().choco_ref_philox4x32_10(_ptr(ctr, ctypes.c_uint32), _ptr(key, ctypes.c_uint32),
                                  _ptr(out, ctypes.c_uint32))
    return out


def random_word(seed, t, worker, e, stream):
    return int(lib().choco_ref_random_word(seed, t, worker, e, stream))


def canonical_sum(terms):
    terms = np.ascontiguousarray(terms, dtype=np.float64)
    return float(lib().choco_ref_canonical_sum(terms.size, _ptr(terms, ctypes.c_double)))


def compress(compressor, v, k=1, levels=1, qsgd_biased=1, randk_rescale=0, seed=0, t=0, worker=0):
    """Q(v) for one vector.  Returns dict(q, sel, codes, scal)."""
    v = np.ascontiguousarray(v)
    suf, real = _suffix(v.dtype)
    d = v.size
    q = np.empty_like(v)
    sparse = compressor in (TOPK, RANDK)
    sel = np.empty(k, dtype=np.int32) if sparse else None
    codes = np.zeros(d, dtype=np.int32) if compressor in (SIGN, QSGD) else None
    scal = np.zeros(4, dtype=np.float64)
    rc = getattr(lib(), "choco_ref_compress_" + suf)(
        compressor, d, _ptr(v, real), k, levels, qsgd_biased, randk_rescale, seed, t, worker,
        _ptr(q, real), _ptr(sel, ctypes.c_int32), _ptr(codes, ctypes.c_int32),
        _ptr(scal, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle rejected the compressor arguments")
    return dict(q=q, sel=sel, codes=codes, scal=scal)


def paper_message_bits(compressor, d, k=0, levels=1):
    """Bits per message as Appendix C counts them."""
    return int(lib().choco_ref_paper_message_bits(compressor, d, k, levels))


def message_words(compressor, d, k=0, levels=1):
    """32-bit words of one message in this build's byte layout."""
    return int(lib().choco_ref_message_words(compressor, d, k, levels))


def pack_message(compressor, v, k=1, levels=1, qsgd_biased=1, randk_rescale=0, seed=0, t=0, worker=0):
    """(q, message words) for one float32 vector v: q = Q(v) and its encoding."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    q = np.empty_like(v)
    msg = np.zeros(message_words(compressor, v.size, k, levels), dtype=np.uint32)
    rc = lib().choco_ref_pack_message(compressor, v.size, _ptr(v, ctypes.c_float), k, levels,
                                      qsgd_biased, randk_rescale, seed, t, worker,
                                      _ptr(q, ctypes.c_float), _ptr(msg, ctypes.c_uint32))
    if rc != 0:
        raise ValueError("oracle could not pack the message (%d)" % rc)
    return q, msg


def unpack_message(compressor, d, msg, k=1, levels=1, qsgd_biased=1, randk_rescale=0, seed=0, t=0,
                   worker=0):
    """The receiver's q from the message (and the shared seed, step and sender for random_a)."""
    msg = np.ascontiguousarray(msg, dtype=np.uint32)
    q = np.empty(d, dtype=np.float32)
    rc = lib().choco_ref_unpack_message(compressor, d, k, levels, qsgd_biased, randk_rescale, seed, t,
                                        worker, _ptr(msg, ctypes.c_uint32), _ptr(q, ctypes.c_float))
    if rc != 0:
        raise ValueError("oracle could not unpack the message")
    return q


def _layer_arrays(layers):
    start, length, k = layers
    start = np.ascontiguousarray(start, dtype=np.int64)
    length = np.ascontiguousarray(length, dtype=np.int64)
    k = np.zeros_like(start) if k is None else np.ascontiguousarray(k, dtype=np.int64)
    return start, length, k


def layers_message_words(compressor, layers, levels=1):
    start, length, k = _layer_arrays(layers)
    return int(lib().choco_ref_layers_message_words(compressor, start.size, _ptr(length, ctypes.c_int64),
                                                    _ptr(k, ctypes.c_int64), levels))


def pack_layers(compressor, v, layers, levels=1, qsgd_biased=1, randk_rescale=0, seed=0, t=0, worker=0):
    """(q, message words) with the operator applied layer by layer: the layers' messages one
    after the other."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    start, length, k = _layer_arrays(layers)
    q = np.empty_like(v)
    msg = np.zeros(layers_message_words(compressor, (start, length, k), levels), dtype=np.uint32)
    rc = lib().choco_ref_pack_layers(compressor, v.size, _ptr(v, ctypes.c_float), start.size,
                                     _ptr(start, ctypes.c_int64), _ptr(length, ctypes.c_int64),
                                     _ptr(k, ctypes.c_int64), levels, qsgd_biased, randk_rescale, seed, t,
                                     worker, _ptr(q, ctypes.c_float), _ptr(msg, ctypes.c_uint32))
    if rc != 0:
        raise ValueError("oracle could not pack the layered message (%d)" % rc)
    return q, msg


def unpack_layers(compressor, d, msg, layers, levels=1, qsgd_biased=1, randk_rescale=0, seed=0, t=0,
                  worker=0):
    msg = np.ascontiguousarray(msg, dtype=np.uint32)
    start, length, k = _layer_arrays(layers)
    q = np.empty(d, dtype=np.float32)
    rc = lib().choco_ref_unpack_layers(compressor, d, start.size, _ptr(start, ctypes.c_int64),
                                       _ptr(length, ctypes.c_int64), _ptr(k, ctypes.c_int64), levels,
                                       qsgd_biased, randk_rescale, seed, t, worker,
                                       _ptr(msg, ctypes.c_uint32), _ptr(q, ctypes.c_float))
    if rc != 0:
        raise ValueError("oracle could not unpack the layered message")
    return q


class RefState:
    """State (X, Xhat, S, t) of all n workers, stepped by the oracle."""

    def __init__(self, X, row_ptr, col_idx, w, gamma, compressor, k=1, levels=1, qsgd_biased=1,
                 randk_rescale=0, order=COMPRESS_THEN_MIX, mix_form=INCREMENTAL_S, seed=0,
                 layers=None):
        """layers = (start, length, k) arrays: the operator is applied to each slice
        [start, start + length) on its own, keeping k[l] entries of slice l (top_a /
        random_a; ignored by the others).  None: the whole vector is one layer."""
        self.X = np.array(X, order="C", copy=True)
        self.suf, self.real = _suffix(self.X.dtype)
        self.n, self.d = self.X.shape
        self.Xhat = np.zeros_like(self.X)   # xhat_i^(0) = 0 (Algorithm 1, input line)
        self.S = np.zeros_like(self.X)
        self.row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
        self.col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
        self.w = np.ascontiguousarray(w, dtype=self.X.dtype)
        self.gamma = float(gamma)
        self.compressor, self.k, self.levels = int(compressor), int(k), int(levels)
        self.qsgd_biased, self.randk_rescale = int(qsgd_biased), int(randk_rescale)
        self.order, self.mix_form, self.seed = int(order), int(mix_form), int(seed)
        self.t = 0
        self.layers = None
        if layers is not None:
            self.layers = tuple(np.ascontiguousarray(a, dtype=np.int64) for a in layers)
            assert len(self.layers) == 3 and len({a.size for a in self.layers}) == 1

    def _layered_step(self, want_details):
        sparse = self.compressor in (TOPK, RANDK)
        start, length, k = self.layers
        nseg = start.size
        ktot = int(k.sum()) if sparse else 0
        sel = codes = scal = None
        if want_details:
            if sparse:
                sel = np.empty((self.n, ktot), dtype=np.int32)
            if self.compressor in (SIGN, QSGD):
                codes = np.zeros((self.n, self.d), dtype=np.int32)
            scal = np.zeros((self.n, nseg, 4), dtype=np.float64)
        rc = getattr(lib(), "choco_ref_gossip_step_layers_" + self.suf)(
            self.n, self.d, _ptr(self.row_ptr, ctypes.c_int32), _ptr(self.col_idx, ctypes.c_int32),
            _ptr(self.w, self.real), self.gamma, self.compressor, nseg,
            _ptr(start, ctypes.c_int64), _ptr(length, ctypes.c_int64), _ptr(k, ctypes.c_int64),
            self.levels, self.qsgd_biased, self.randk_rescale, self.order, self.mix_form,
            self.seed, self.t, _ptr(self.X, self.real), _ptr(self.Xhat, self.real),
            _ptr(self.S, self.real), _ptr(sel, ctypes.c_int32), _ptr(codes, ctypes.c_int32),
            _ptr(scal, ctypes.c_double))
        if rc != 0:
            raise ValueError("oracle rejected the step arguments")
        self.t += 1
        return dict(sel=sel, codes=codes, scal=scal)

    def gossip_step(self, want_details=False):
        if self.layers is not None:
            return self._layered_step(want_details)
        sparse = self.compressor in (TOPK, RANDK)
        sel = codes = scal = None
        if want_details:
            if sparse:
                sel = np.empty((self.n, self.k), dtype=np.int32)
            if self.compressor in (SIGN, QSGD):
                codes = np.zeros((self.n, self.d), dtype=np.int32)
            scal = np.zeros((self.n, 4), dtype=np.float64)
        rc = getattr(lib(), "choco_ref_gossip_step_" + self.suf)(
            self.n, self.d, _ptr(self.row_ptr, ctypes.c_int32), _ptr(self.col_idx, ctypes.c_int32),
            _ptr(self.w, self.real), self.gamma, self.compressor, self.k, self.levels,
            self.qsgd_biased, self.randk_rescale, self.order, self.mix_form, self.seed, self.t,
            _ptr(self.X, self.real), _ptr(self.Xhat, self.real), _ptr(self.S, self.real),
            _ptr(sel, ctypes.c_int32), _ptr(codes, ctypes.c_int32), _ptr(scal, ctypes.c_double))
        if rc != 0:
            raise ValueError("oracle rejected the step arguments")
        self.t += 1
        return dict(sel=sel, codes=codes, scal=scal)

    def sgd_step(self, G, lr):
        G = np.ascontiguousarray(G, dtype=self.X.dtype)
        assert G.shape == self.X.shape
        getattr(lib(), "choco_ref_sgd_step_" + self.suf)(
            self.n, self.d, _ptr(self.X, self.real), _ptr(G, self.real), float(lr))

    def momentum_step(self, V, G, lr, beta, lam):
        G = np.ascontiguousarray(G, dtype=self.X.dtype)
        assert V.dtype == self.X.dtype and V.flags.c_contiguous and V.shape == self.X.shape
        getattr(lib(), "choco_ref_momentum_step_" + self.suf)(
            self.n, self.d, _ptr(self.X, self.real), _ptr(V, self.real), _ptr(G, self.real),
            float(lr), float(beta), float(lam))

    def metrics(self):
        c = ctypes.c_double()
        m = ctypes.c_double()
        p = ctypes.c_double()
        getattr(lib(), "choco_ref_metrics_" + self.suf)(
            self.n, self.d, _ptr(self.X, self.real), _ptr(self.Xhat, self.real),
            ctypes.byref(c), ctypes.byref(m), ctypes.byref(p))
        return dict(consensus=c.value, mean_norm=m.value, psi=p.value)
