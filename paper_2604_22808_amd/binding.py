"""ctypes binding of libfreqattn.so: the same entry points as include/freqattn.h, argument marshalling only.

Device tensors are torch tensors (torch is used for device memory and streams, nothing else); every computation
happens inside the library.  Loading fails loudly when the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfreqattn.so")

OK, EINVAL, ENOMEM, EHIP, EUNSUPPORTED, ERANGE = 0, 1, 2, 3, 4, 5
F32, BF16 = 0, 1
LAUNCH_FUSED, LAUNCH_SEPARATE = 0, 1
PATH_AUTO, PATH_GENERIC, PATH_MFMA, PATH_TABLES_ONLY = 0, 1, 2, 3
TRANSFORM_DCT, TRANSFORM_HAAR = 0, 1


class Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "heads", "head_dim", "T", "H", "W", "dtype")]


class BandCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("low_num", "low_den", "mid_num", "mid_den", "low_compress", "mid_block",
                                         "mid_diag", "mid_stride", "mid_block0", "high_window", "n_summary")] + \
               [("softmax_scale", C.c_float), ("transform", C.c_int32), ("mid2_num", C.c_int32), ("mid2_den", C.c_int32)]


EXPORTS = {
    "freqattn_create": (C.c_int, [C.POINTER(Shape), C.POINTER(BandCfg), C.c_int32, C.POINTER(C.c_void_p)]),
    "freqattn_forward": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(BandCfg),
                                   C.POINTER(C.c_int32), C.c_void_p, C.c_void_p]),
    "freqattn_forward_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(BandCfg),
                                          C.POINTER(C.c_int32), C.c_void_p, C.c_void_p]),
    "freqattn_forward_projected": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.POINTER(BandCfg), C.POINTER(C.c_int32), C.c_void_p, C.c_void_p]),
    "freqattn_destroy": (None, [C.c_void_p]),
    "freqattn_last_error": (C.c_char_p, [C.c_void_p]),
    "freqattn_set_launch_mode": (C.c_int, [C.c_void_p, C.c_int32]),
    "freqattn_get_path": (C.c_int32, [C.c_void_p]),
    "freqattn_set_exchange_fusion": (C.c_int, [C.c_void_p, C.c_int32]),
    "freqattn_set_alloc_prediction": (C.c_int, [C.c_void_p, C.c_int32]),
    "freqattn_band_sizes": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64)]),
    "freqattn_band_index": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]),
    "freqattn_mid_blocks": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int64)]),
    "freqattn_mid2_blocks": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int64)]),
    "freqattn_dct_matrix": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_double)]),
    "freqattn_get_v_box": (C.c_int32, [C.c_void_p]),
    "freqattn_summary_weights": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_float)]),
    "freqattn_read_spectral": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_float), C.c_void_p]),
    "freqattn_route_fixed": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]),
    "freqattn_load_balance": (C.c_int, [C.POINTER(C.c_float), C.c_int32, C.c_float, C.POINTER(C.c_float)]),
    "freqattn_route_mlp": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_int32,
                                     C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float),
                                     C.POINTER(C.c_float), C.POINTER(C.c_int32), C.POINTER(C.c_float),
                                     C.POINTER(C.c_float), C.c_void_p]),
    "freqattn_forward_routed": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(BandCfg), C.c_float,
                                          C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float),
                                          C.POINTER(C.c_float), C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float),
                                          C.c_void_p]),
    "freqattn_dense_forward": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "freqattn_set_stage_timing": (C.c_int, [C.c_void_p, C.c_int32]),
    "freqattn_stage_times": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_float),
                                       C.POINTER(C.c_int32)]),
    "freqattn_workspace_bytes": (C.c_int64, [C.c_void_p]),
    "freqattn_check_range": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), C.c_void_p]),
    "freqattn_measure_peaks": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p]),
}

_lib = None


def lib():
    """The loaded library; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(or python paper_2604_22808_amd/build.py) first")
        # torch ships its own HIP runtime (same soname): load it first so that the library binds to the runtime
        # that owns torch's device memory and streams instead of bringing a second one into the process.
        import torch  # noqa: F401
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


class FreqAttnError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"freqattn status {status}: {msg}")
        self.status = status


def _ptr(t):
    return C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_cfg(**kw) -> BandCfg:
    base = dict(low_num=1, low_den=4, mid_num=1, mid_den=2, low_compress=4, mid_block=64, mid_diag=1, mid_stride=8,
                mid_block0=1, high_window=256, n_summary=16, softmax_scale=0.0, transform=0, mid2_num=0, mid2_den=1)
    base.update(kw)
    return BandCfg(**base)


class Context:
    """Owns one freqattn_ctx.  Methods carry the names of the C entry points without the prefix."""

    def __init__(self, batch, heads, head_dim, grid, dtype, cfg: BandCfg, path=PATH_AUTO):
        self.shape = Shape(batch, heads, head_dim, grid[0], grid[1], grid[2], dtype)
        self.cfg = cfg
        self._h = C.c_void_p()
        st = lib().freqattn_create(C.byref(self.shape), C.byref(cfg), path, C.byref(self._h))
        if st != OK:
            raise FreqAttnError(st, lib().freqattn_last_error(None).decode())

    def _check(self, st):
        if st != OK:
            raise FreqAttnError(st, lib().freqattn_last_error(self._h).decode())

    def destroy(self):
        if self._h:
            lib().freqattn_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def _check_tensors(self, who, **tensors):
        """The library sees raw addresses only: a tensor on the host, of another type, shape or layout would make its
        kernels read or write out of bounds, so every device tensor is checked here before its pointer is taken."""
        import torch
        s = self.shape
        want_shape = (s.batch, s.heads, s.T * s.H * s.W, s.head_dim)
        want_dtype = torch.bfloat16 if s.dtype == BF16 else torch.float32
        for name, t in tensors.items():
            if not isinstance(t, torch.Tensor):
                raise TypeError(f"{who}: {name} must be a torch tensor")
            if not t.is_cuda:
                raise ValueError(f"{who}: {name} must be a device tensor")
            if t.dtype != want_dtype:
                raise ValueError(f"{who}: {name} has dtype {t.dtype}, the context was created for {want_dtype}")
            if tuple(t.shape) != want_shape:
                raise ValueError(f"{who}: {name} has shape {tuple(t.shape)}, expected {want_shape}")
            if not t.is_contiguous():
                raise ValueError(f"{who}: {name} must be contiguous")

    # ---- hot path
    def forward(self, q, k, v, head_alloc, out, cfg=None):
        self._check_tensors("forward", q=q, k=k, v=v, out=out)
        ha = np.ascontiguousarray(head_alloc, dtype=np.int32)
        if ha.shape != (self.shape.heads,):
            raise ValueError(f"forward: head_alloc must hold {self.shape.heads} entries, got shape {ha.shape}")
        cfg = cfg or self.cfg
        self._check(lib().freqattn_forward(self._h, _ptr(q), _ptr(k), _ptr(v), C.byref(cfg),
                                           ha.ctypes.data_as(C.POINTER(C.c_int32)), _ptr(out), _stream()))
        return out

    def forward_projected(self, x, wq, wk, wv, wo, head_alloc, out, cfg=None):
        import torch
        s = self.shape
        hd = s.heads * s.head_dim
        if not isinstance(x, torch.Tensor) or x.dim() != 3:
            raise ValueError("forward_projected: x must be a [batch, N, d_model] tensor")
        d_model = int(x.shape[2])
        want = {"x": (s.batch, s.T * s.H * s.W, d_model), "out": (s.batch, s.T * s.H * s.W, d_model),
                "wq": (d_model, hd), "wk": (d_model, hd), "wv": (d_model, hd), "wo": (hd, d_model)}
        for name, t in (("x", x), ("out", out), ("wq", wq), ("wk", wk), ("wv", wv), ("wo", wo)):
            if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.bfloat16 or not t.is_contiguous() \
                    or tuple(t.shape) != want[name]:
                raise ValueError(f"forward_projected: {name} must be a contiguous bf16 device tensor of shape {want[name]}")
        ha = np.ascontiguousarray(head_alloc, dtype=np.int32)
        if ha.shape != (s.heads,):
            raise ValueError(f"forward_projected: head_alloc must hold {s.heads} entries")
        cfg = cfg or self.cfg
        self._check(lib().freqattn_forward_projected(self._h, _ptr(x), d_model, _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo),
                                                     C.byref(cfg), ha.ctypes.data_as(C.POINTER(C.c_int32)), _ptr(out),
                                                     _stream()))
        return out

    def forward_static(self, q, k, v, head_alloc, out, cfg=None):
        self._check_tensors("forward_static", q=q, k=k, v=v, out=out)
        ha = np.ascontiguousarray(head_alloc, dtype=np.int32)
        if ha.shape != (self.shape.heads,):
            raise ValueError(f"forward_static: head_alloc must hold {self.shape.heads} entries, got shape {ha.shape}")
        cfg = cfg or self.cfg
        self._check(lib().freqattn_forward_static(self._h, _ptr(q), _ptr(k), _ptr(v), C.byref(cfg),
                                                  ha.ctypes.data_as(C.POINTER(C.c_int32)), _ptr(out), _stream()))
        return out

    @staticmethod
    def _router_weights(who, w1, b1, w2, b2):
        f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
        w1, b1, w2, b2 = f(w1), f(b1), f(w2), f(b2)
        hidden = int(w1.shape[1]) if w1.ndim == 2 else -1
        if w1.shape != (256, hidden) or b1.shape != (hidden,) or w2.shape != (hidden, 3) or b2.shape != (3,) or hidden < 1:
            raise ValueError(f"{who}: router weights must be w1 [256, hidden], b1 [hidden], w2 [hidden, 3], b2 [3]")
        return hidden, w1, b1, w2, b2

    def forward_routed(self, q, k, v, t, w1, b1, w2, b2, out, cfg=None):
        self._check_tensors("forward_routed", q=q, k=k, v=v, out=out)
        hidden, w1, b1, w2, b2 = self._router_weights("forward_routed", w1, b1, w2, b2)
        alloc = np.zeros(self.shape.heads, np.int32)
        pi = np.zeros(3, np.float32)
        P = lambda a: a.ctypes.data_as(C.POINTER(C.c_float))
        cfg = cfg or self.cfg
        self._check(lib().freqattn_forward_routed(self._h, _ptr(q), _ptr(k), _ptr(v), C.byref(cfg), float(t), hidden,
                                                  P(w1), P(b1), P(w2), P(b2), _ptr(out),
                                                  alloc.ctypes.data_as(C.POINTER(C.c_int32)), P(pi), _stream()))
        return alloc, pi

    def dense_forward(self, q, k, v, out):
        self._check_tensors("dense_forward", q=q, k=k, v=v, out=out)
        self._check(lib().freqattn_dense_forward(self._h, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _stream()))
        return out

    def route_mlp(self, q, k, v, t, w1, b1, w2, b2):
        self._check_tensors("route_mlp", q=q, k=k, v=v)
        hidden, w1, b1, w2, b2 = self._router_weights("route_mlp", w1, b1, w2, b2)
        alloc = np.zeros(self.shape.heads, np.int32)
        pi = np.zeros(3, np.float32)
        stats = np.zeros(192, np.float32)
        P = lambda a: a.ctypes.data_as(C.POINTER(C.c_float))
        self._check(lib().freqattn_route_mlp(self._h, _ptr(q), _ptr(k), _ptr(v), float(t), hidden, P(w1), P(b1), P(w2),
                                             P(b2), alloc.ctypes.data_as(C.POINTER(C.c_int32)), P(pi), P(stats),
                                             _stream()))
        return alloc, pi, stats

    # ---- options and introspection
    def set_launch_mode(self, mode):
        self._check(lib().freqattn_set_launch_mode(self._h, mode))

    def set_exchange_fusion(self, enabled):
        self._check(lib().freqattn_set_exchange_fusion(self._h, 1 if enabled else 0))

    def set_alloc_prediction(self, enabled):
        self._check(lib().freqattn_set_alloc_prediction(self._h, 1 if enabled else 0))

    def get_path(self):
        return lib().freqattn_get_path(self._h)

    def check_range(self):
        """Synchronises; raises FreqAttnError (ERANGE) if a forward since the last check left the fp16 range."""
        flag = C.c_int32(0)
        self._check(lib().freqattn_check_range(self._h, C.byref(flag), _stream()))
        return int(flag.value)

    def workspace_bytes(self):
        return lib().freqattn_workspace_bytes(self._h)

    def measure_peaks(self):
        """(bytes/s of a plain streaming copy, flop/s of an MFMA loop) on this machine; synchronises."""
        cp, mf = C.c_double(0.0), C.c_double(0.0)
        self._check(lib().freqattn_measure_peaks(self._h, C.byref(cp), C.byref(mf), _stream()))
        return cp.value, mf.value

    @property
    def n_bands(self):
        return 4 if self.cfg.mid2_num > 0 else 3

    def band_sizes(self):
        n = (C.c_int64 * 4)()
        self._check(lib().freqattn_band_sizes(self._h, n))
        return [int(x) for x in n][:self.n_bands]

    def band_index(self, band):
        out = np.zeros(self.band_sizes()[band], np.int32)
        self._check(lib().freqattn_band_index(self._h, band, out.ctypes.data_as(C.POINTER(C.c_int32))))
        return out

    def _blocks(self, fn, band):
        nnz = C.c_int64()
        self._check(fn(self._h, None, None, C.byref(nnz)))
        nb = -(-self.band_sizes()[band] // self.cfg.mid_block)
        rp = np.zeros(nb + 1, np.int32)
        ci = np.zeros(nnz.value, np.int32)
        self._check(fn(self._h, rp.ctypes.data_as(C.POINTER(C.c_int32)), ci.ctypes.data_as(C.POINTER(C.c_int32)),
                       C.byref(nnz)))
        return rp, ci

    def mid_blocks(self):
        return self._blocks(lib().freqattn_mid_blocks, 1)

    def mid2_blocks(self):
        if self.n_bands < 4:
            return np.zeros(1, np.int32), np.zeros(0, np.int32)
        return self._blocks(lib().freqattn_mid2_blocks, 3)

    def get_v_box(self):
        return int(lib().freqattn_get_v_box(self._h))

    def summary_weights(self, band):
        m = min(self.cfg.n_summary, int(self.band_sizes()[band]))
        n = self.shape.T * self.shape.H * self.shape.W
        out = np.zeros((m, n), np.float32)
        self._check(lib().freqattn_summary_weights(self._h, band, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def dct_matrix(self, axis):
        n = (self.shape.T, self.shape.H, self.shape.W)[axis]
        out = np.zeros((n, n), np.float64)
        self._check(lib().freqattn_dct_matrix(self._h, axis, out.ctypes.data_as(C.POINTER(C.c_double))))
        return out

    def read_spectral(self, which, slice_, band):
        out = np.zeros((self.band_sizes()[band], self.shape.head_dim), np.float32)
        self._check(lib().freqattn_read_spectral(self._h, which, slice_, band, out.ctypes.data_as(C.POINTER(C.c_float)),
                                                 _stream()))
        return out

    def set_stage_timing(self, enabled):
        self._check(lib().freqattn_set_stage_timing(self._h, int(enabled)))

    def stage_times(self):
        names = (C.c_char_p * 16)()
        ms = (C.c_float * 16)()
        n = C.c_int32()
        self._check(lib().freqattn_stage_times(self._h, 16, names, ms, C.byref(n)))
        return [(names[i].decode(), float(ms[i])) for i in range(n.value)]


def load_balance(pi_heads, lam):
    p = np.ascontiguousarray(pi_heads, dtype=np.float32)
    if p.ndim != 2 or p.shape[1] != 3:
        raise ValueError("load_balance: pi_heads must be [heads, 3]")
    out = C.c_float(0.0)
    st = lib().freqattn_load_balance(p.ctypes.data_as(C.POINTER(C.c_float)), p.shape[0], float(lam), C.byref(out))
    if st != OK:
        raise FreqAttnError(st, "freqattn_load_balance: bad arguments")
    return float(out.value)


def route_fixed(heads, n_low, n_mid, n_high):
    out = np.zeros(heads, np.int32)
    st = lib().freqattn_route_fixed(heads, n_low, n_mid, n_high, out.ctypes.data_as(C.POINTER(C.c_int32)))
    if st != OK:
        raise FreqAttnError(st, "freqattn_route_fixed: bad arguments")
    return out
