"""ctypes binding of include/choco.h: argument marshalling only.

Every step of the path runs in the HIP library; torch is used here for device
memory and the stream handle.  There is no CPU fallback: if libchoco.so is
missing, loading fails with an error that says how to build it.
"""
import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libchoco.so")

OK, E_INVAL, E_NOMEM, E_HIP, E_UNSUPPORTED = 0, -1, -2, -3, -4
Q_IDENTITY, Q_TOPK, Q_RANDK, Q_SIGN, Q_QSGD = 0, 1, 2, 3, 4
ORDER_COMPRESS_THEN_MIX, ORDER_MIX_THEN_COMPRESS = 0, 1
MIX_AUTO, MIX_INCREMENTAL_S, MIX_DIRECT = 0, 1, 2

EXPORTS = [
    "choco_workspace_bytes", "choco_init", "choco_gossip_step", "choco_sgd_step", "choco_step",
    "choco_momentum_step", "choco_step_momentum", "choco_metrics", "choco_xhat", "choco_nsum", "choco_last_selection",
    "choco_set_capture", "choco_last_scalars", "choco_layer_scalars", "choco_get_step", "choco_set_step", "choco_sync",
    "choco_destroy", "choco_strerror", "choco_last_hip_error", "choco_set_profiling",
    "choco_profile_report", "choco_paper_message_bits", "choco_message_bytes", "choco_pack_messages",
    "choco_unpack_messages", "choco_set_lookahead", "choco_metrics_noalloc", "choco_get_mix_form", "choco_last_message",
]


class ChocoConfig(ctypes.Structure):
    _fields_ = [
        ("n", ctypes.c_int32),
        ("d", ctypes.c_int64),
        ("ld", ctypes.c_int64),
        ("row_ptr_host", ctypes.POINTER(ctypes.c_int32)),
        ("col_idx_host", ctypes.POINTER(ctypes.c_int32)),
        ("w_host", ctypes.POINTER(ctypes.c_float)),
        ("gamma", ctypes.c_float),
        ("compressor", ctypes.c_int32),
        ("k", ctypes.c_int64),
        ("levels", ctypes.c_int32),
        ("qsgd_biased", ctypes.c_int32),
        ("randk_rescale", ctypes.c_int32),
        ("order", ctypes.c_int32),
        ("mix_form", ctypes.c_int32),
        ("seed", ctypes.c_uint64),
        ("stream", ctypes.c_void_p),
        ("nlayers", ctypes.c_int32),
        ("layer_start_host", ctypes.POINTER(ctypes.c_int64)),
        ("layer_len_host", ctypes.POINTER(ctypes.c_int64)),
        ("layer_k_host", ctypes.POINTER(ctypes.c_int64)),
    ]


class ChocoError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (what, strerror(code), code))


_lib = None


def lib():
    """The loaded HIP library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "HIP library %s is missing; build it with "
                "`python -c 'import __graft_entry__ as g; g.build()'` "
                "(there is no CPU fallback)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, cfgp = ctypes.c_void_p, ctypes.POINTER(ChocoConfig)
        L.choco_workspace_bytes.argtypes = [cfgp, ctypes.POINTER(ctypes.c_size_t)]
        L.choco_init.argtypes = [cfgp, vp, vp, ctypes.c_size_t, ctypes.POINTER(vp)]
        L.choco_gossip_step.argtypes = [vp]
        L.choco_sgd_step.argtypes = [vp, vp, ctypes.c_float]
        L.choco_step.argtypes = [vp, vp, ctypes.c_float]
        L.choco_momentum_step.argtypes = [vp, vp, vp, ctypes.c_float, ctypes.c_float, ctypes.c_float]
        L.choco_step_momentum.argtypes = [vp, vp, vp, ctypes.c_float, ctypes.c_float, ctypes.c_float]
        dp = ctypes.POINTER(ctypes.c_double)
        L.choco_metrics.argtypes = [vp, dp, dp, dp]
        L.choco_metrics_noalloc.argtypes = [vp, vp]
        L.choco_xhat.argtypes = [vp, ctypes.POINTER(vp)]
        L.choco_nsum.argtypes = [vp, ctypes.POINTER(vp)]
        L.choco_last_selection.argtypes = [vp, vp, vp]
        L.choco_set_capture.argtypes = [vp, vp]
        L.choco_last_message.argtypes = [vp, ctypes.c_int32, vp, vp, vp, ctypes.POINTER(ctypes.c_float)]
        L.choco_last_scalars.argtypes = [vp, dp]
        L.choco_layer_scalars.argtypes = [vp, dp]
        L.choco_paper_message_bits.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                               ctypes.POINTER(ctypes.c_int64)]
        L.choco_message_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
        L.choco_pack_messages.argtypes = [vp, vp]
        L.choco_unpack_messages.argtypes = [vp, vp, vp]
        L.choco_get_mix_form.argtypes = [vp, ctypes.POINTER(ctypes.c_int32)]
        L.choco_get_step.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64)]
        L.choco_set_step.argtypes = [vp, ctypes.c_uint64]
        L.choco_sync.argtypes = [vp]
        L.choco_set_lookahead.argtypes = [vp, ctypes.c_int]
        L.choco_set_profiling.argtypes = [vp, ctypes.c_int]
        L.choco_profile_report.argtypes = [vp, ctypes.c_char_p, ctypes.c_size_t]
        L.choco_destroy.argtypes = [vp]
        L.choco_strerror.argtypes = [ctypes.c_int]
        L.choco_strerror.restype = ctypes.c_char_p
        L.choco_last_hip_error.argtypes = [vp]
        for name in EXPORTS:
            if name != "choco_strerror":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(code):
    return lib().choco_strerror(code).decode()


def _check(code, what):
    if code != OK:
        raise ChocoError(code, what)


def make_config(n, d, row_ptr, col_idx, w, gamma, compressor, k=1, levels=1, qsgd_biased=1,
                randk_rescale=0, order=ORDER_COMPRESS_THEN_MIX, mix_form=MIX_AUTO, seed=0, ld=0,
                stream=None, layers=None):
    """Fill a choco_config.  Returns (config, keepalive) - the numpy arrays the
    config points into must outlive the calls that read it.  layers = (start, length, k)
    arrays switches layer-wise compression on (k may be None for SIGN / QSGD)."""
    row_ptr = None if row_ptr is None else np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = None if col_idx is None else np.ascontiguousarray(col_idx, dtype=np.int32)
    w = None if w is None else np.ascontiguousarray(w, dtype=np.float32)
    cfg = ChocoConfig()
    cfg.n, cfg.d, cfg.ld = int(n), int(d), int(ld)
    cfg.row_ptr_host = None if row_ptr is None else row_ptr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    cfg.col_idx_host = None if col_idx is None else col_idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    cfg.w_host = None if w is None else w.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
    cfg.gamma = float(gamma)
    cfg.compressor, cfg.k, cfg.levels = int(compressor), int(k), int(levels)
    cfg.qsgd_biased, cfg.randk_rescale = int(qsgd_biased), int(randk_rescale)
    cfg.order, cfg.mix_form, cfg.seed = int(order), int(mix_form), int(seed)
    cfg.stream = stream
    keep = [row_ptr, col_idx, w]
    cfg.nlayers = 0
    if layers is not None:
        i64p = ctypes.POINTER(ctypes.c_int64)
        start, length, lk = layers
        start = np.ascontiguousarray(start, dtype=np.int64)
        length = np.ascontiguousarray(length, dtype=np.int64)
        assert start.size == length.size
        cfg.nlayers = int(start.size)
        cfg.layer_start_host = start.ctypes.data_as(i64p)
        cfg.layer_len_host = length.ctypes.data_as(i64p)
        keep += [start, length]
        if lk is not None:
            lk = np.ascontiguousarray(lk, dtype=np.int64)
            assert lk.size == start.size
            cfg.layer_k_host = lk.ctypes.data_as(i64p)
            keep.append(lk)
    return cfg, tuple(keep)


def paper_message_bits(compressor, d, k=1, levels=1):
    """Bits of one message as Appendix C counts them."""
    out = ctypes.c_int64(0)
    _check(lib().choco_paper_message_bits(int(compressor), int(d), int(k), int(levels), ctypes.byref(out)),
           "choco_paper_message_bits")
    return out.value


def workspace_bytes(cfg):
    out = ctypes.c_size_t(0)
    _check(lib().choco_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)), "choco_workspace_bytes")
    return out.value


class Choco:
    """All n workers on one GPU.  X is a contiguous float32 CUDA tensor of shape
    (n, ld) with ld a multiple of 4 and ld >= d; it is updated in place."""

    def __init__(self, X, d, row_ptr, col_idx, w, gamma, compressor, **kw):
        import torch
        assert X.is_cuda and X.dtype == torch.float32 and X.is_contiguous() and X.dim() == 2
        self.torch = torch
        self.X = X
        self.n, self.ld = X.shape
        self.d = int(d)
        stream = kw.pop("stream", None)
        if stream is None:
            stream = torch.cuda.current_stream(X.device).cuda_stream
        self.cfg, self._keep = make_config(self.n, self.d, row_ptr, col_idx, w, gamma, compressor,
                                           ld=self.ld, stream=stream, **kw)
        nbytes = workspace_bytes(self.cfg)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=X.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        self._ws_off = self._ws_ptr - base
        ctx = ctypes.c_void_p()
        _check(lib().choco_init(ctypes.byref(self.cfg), X.data_ptr(), self._ws_ptr, nbytes,
                                ctypes.byref(ctx)), "choco_init")
        self.ctx = ctx
        self.k = int(self.cfg.k)
        self.nlayers = int(self.cfg.nlayers)
        if self.nlayers and compressor in (Q_TOPK, Q_RANDK):
            self.k = int(np.asarray(kw["layers"][2], dtype=np.int64).sum())   # pairs per worker
        self._capture = None

    def close(self):
        if getattr(self, "ctx", None):
            lib().choco_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def gossip_step(self):
        _check(lib().choco_gossip_step(self.ctx), "choco_gossip_step")

    def sgd_step(self, G, lr):
        assert G.is_cuda and G.is_contiguous() and G.shape == self.X.shape and G.dtype == self.X.dtype
        _check(lib().choco_sgd_step(self.ctx, G.data_ptr(), float(lr)), "choco_sgd_step")

    def step(self, G, lr):
        """sgd_step(G, lr) followed by gossip_step(), fused where the operator allows."""
        assert G.is_cuda and G.is_contiguous() and G.shape == self.X.shape and G.dtype == self.X.dtype
        _check(lib().choco_step(self.ctx, G.data_ptr(), float(lr)), "choco_step")

    def momentum_step(self, G, M, lr, beta, lam):
        for T in (G, M):
            assert T.is_cuda and T.is_contiguous() and T.shape == self.X.shape and T.dtype == self.X.dtype
        _check(lib().choco_momentum_step(self.ctx, G.data_ptr(), M.data_ptr(), float(lr), float(beta),
                                         float(lam)), "choco_momentum_step")

    def step_momentum(self, G, M, lr, beta, lam):
        """momentum_step(G, M, ...) followed by gossip_step(), fused where the operator allows."""
        for T in (G, M):
            assert T.is_cuda and T.is_contiguous() and T.shape == self.X.shape and T.dtype == self.X.dtype
        _check(lib().choco_step_momentum(self.ctx, G.data_ptr(), M.data_ptr(), float(lr), float(beta),
                                         float(lam)), "choco_step_momentum")

    def metrics(self):
        c, m, p = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        _check(lib().choco_metrics(self.ctx, ctypes.byref(c), ctypes.byref(m), ctypes.byref(p)),
               "choco_metrics")
        return dict(consensus=c.value, mean_norm=m.value, psi=p.value)

    def metrics_noalloc(self, out):
        """The three figures of metrics() written to `out` (3 float64 on the device); no wait."""
        assert out.is_cuda and out.is_contiguous() and out.dtype == self.torch.float64 and out.numel() == 3
        _check(lib().choco_metrics_noalloc(self.ctx, out.data_ptr()), "choco_metrics_noalloc")

    def _view(self, ptr):
        off = ptr - self.workspace.data_ptr()
        nbytes = self.n * self.ld * 4
        return self.workspace[off:off + nbytes].view(self.torch.float32).view(self.n, self.ld)

    def xhat(self):
        p = ctypes.c_void_p()
        _check(lib().choco_xhat(self.ctx, ctypes.byref(p)), "choco_xhat")
        return self._view(p.value)

    def nsum(self):
        p = ctypes.c_void_p()
        _check(lib().choco_nsum(self.ctx, ctypes.byref(p)), "choco_nsum")
        return None if not p.value else self._view(p.value)

    def last_selection(self):
        torch = self.torch
        idx = torch.empty((self.n, self.k), dtype=torch.int32, device=self.X.device)
        val = torch.empty((self.n, self.k), dtype=torch.float32, device=self.X.device)
        _check(lib().choco_last_selection(self.ctx, idx.data_ptr(), val.data_ptr()),
               "choco_last_selection")
        return idx, val

    def last_message(self, worker):
        """What `worker` sent in the last gossip step: dict(idx, val) for top_a / random_a,
        dict(bits, scale) for sign / gsgd (bits: int32 CUDA tensor (planes, ceil(d/32)))."""
        torch = self.torch
        comp = int(self.cfg.compressor)
        if comp in (Q_TOPK, Q_RANDK):
            idx = torch.empty(self.k, dtype=torch.int32, device=self.X.device)
            val = torch.empty(self.k, dtype=torch.float32, device=self.X.device)
            _check(lib().choco_last_message(self.ctx, int(worker), idx.data_ptr(), val.data_ptr(), None, None),
                   "choco_last_message")
            return dict(idx=idx, val=val)
        planes = 1
        if comp == Q_QSGD:
            planes = 1 + max(1, (int(self.cfg.levels) - 1).bit_length())
        bits = torch.empty((planes, (self.d + 31) // 32), dtype=torch.int32, device=self.X.device)
        scale = ctypes.c_float()
        _check(lib().choco_last_message(self.ctx, int(worker), None, None, bits.data_ptr(),
                                        None if self.nlayers else ctypes.byref(scale)), "choco_last_message")
        return dict(bits=bits, scale=scale.value)

    def set_capture(self, codes):
        """codes: int32 CUDA tensor (n, ld) or None."""
        if codes is not None:
            assert codes.is_cuda and codes.is_contiguous() and codes.shape == self.X.shape
            assert codes.dtype == self.torch.int32
        self._capture = codes
        _check(lib().choco_set_capture(self.ctx, None if codes is None else codes.data_ptr()),
               "choco_set_capture")

    def last_scalars(self):
        out = np.zeros((self.n, 6), dtype=np.float64)
        _check(lib().choco_last_scalars(self.ctx, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double))),
               "choco_last_scalars")
        return out

    def layer_scalars(self):
        out = np.zeros((self.n, self.nlayers, 4), dtype=np.float64)
        _check(lib().choco_layer_scalars(self.ctx, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double))),
               "choco_layer_scalars")
        return out

    def message_bytes(self):
        out = ctypes.c_size_t(0)
        _check(lib().choco_message_bytes(self.ctx, ctypes.byref(out)), "choco_message_bytes")
        return out.value

    def pack_messages(self):
        """The messages of the last gossip step: uint32 CUDA tensor (n, words per message)."""
        torch = self.torch
        words = self.message_bytes() // 4
        msgs = torch.empty((self.n, words), dtype=torch.int32, device=self.X.device)
        _check(lib().choco_pack_messages(self.ctx, msgs.data_ptr()), "choco_pack_messages")
        return msgs

    def unpack_messages(self, msgs):
        """Dense q (n, ld) decoded from messages as pack_messages returns them."""
        assert msgs.is_cuda and msgs.is_contiguous() and msgs.dtype == self.torch.int32
        assert msgs.shape == (self.n, self.message_bytes() // 4)
        q = self.torch.empty_like(self.X)
        _check(lib().choco_unpack_messages(self.ctx, msgs.data_ptr(), q.data_ptr()), "choco_unpack_messages")
        return q

    def mix_form(self):
        """MIX_INCREMENTAL_S or MIX_DIRECT: what the library resolved MIX_AUTO to."""
        m = ctypes.c_int32()
        _check(lib().choco_get_mix_form(self.ctx, ctypes.byref(m)), "choco_get_mix_form")
        return m.value

    def get_step(self):
        t = ctypes.c_uint64()
        _check(lib().choco_get_step(self.ctx, ctypes.byref(t)), "choco_get_step")
        return t.value

    def set_step(self, t):
        _check(lib().choco_set_step(self.ctx, int(t)), "choco_set_step")

    def set_lookahead(self, on):
        _check(lib().choco_set_lookahead(self.ctx, 1 if on else 0), "choco_set_lookahead")

    def sync(self):
        _check(lib().choco_sync(self.ctx), "choco_sync")

    def set_profiling(self, on):
        _check(lib().choco_set_profiling(self.ctx, 1 if on else 0), "choco_set_profiling")

    def profile_report(self):
        """{kernel name: (launches, total milliseconds)} since profiling was switched on."""
        buf = ctypes.create_string_buffer(8192)
        _check(lib().choco_profile_report(self.ctx, buf, len(buf)), "choco_profile_report")
        out = {}
        for line in buf.value.decode().splitlines():
            name, count, ms = line.split()
            out[name] = (int(count), float(ms))
        return out
