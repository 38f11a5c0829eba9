"""Python face of the CPU oracle (``sjd_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, the smoke check and the benchmark's CPU-baseline leg may import this package; the
product package never does.  Everything here is argument marshalling around the C functions; the
arithmetic lives in the C file, whose header cites the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np

from . import build as _build


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_blocks", "n_layers", "width", "n_heads", "mlp_ratio", "seq_len", "token_dim")] + \
               [("reverse_mask", C.c_uint32), ("mask_nearest", C.c_int32)]


def _as_cfg(cfg) -> _Cfg:
    return _Cfg(cfg.n_blocks, cfg.n_layers, cfg.width, cfg.n_heads, cfg.mlp_ratio, cfg.seq_len,
                cfg.token_dim, cfg.reverse_mask, int(getattr(cfg, "mask_nearest", 0)))


class Oracle:
    """One arithmetic flavour of the oracle: ``Oracle("f32")`` or ``Oracle("f64")``."""

    def __init__(self, real: str = "f32"):
        assert real in ("f32", "f64")
        path = _build.lib_path(real)
        if not os.path.exists(path):
            _build.build(force=False)
        self.lib = C.CDLL(path)
        self.real = real
        self.dtype = np.float32 if real == "f32" else np.float64
        self._rp = C.POINTER(C.c_float if real == "f32" else C.c_double)
        self.lib.orc_block_floats.restype = C.c_size_t
        assert self.lib.orc_real_bytes() == np.dtype(self.dtype).itemsize

    # -- helpers
    def _r(self, a) -> np.ndarray:
        return np.ascontiguousarray(a, dtype=self.dtype)

    def _p(self, a: Optional[np.ndarray]):
        return None if a is None else a.ctypes.data_as(self._rp)

    @staticmethod
    def _w(blob: np.ndarray):
        assert blob.dtype == np.float32 and blob.flags.c_contiguous
        return blob.ctypes.data_as(C.POINTER(C.c_float))

    def num_threads(self) -> int:
        return int(self.lib.orc_num_threads())

    # -- one sample, one block
    def cond(self, cfg, blob, j, x) -> Tuple[np.ndarray, np.ndarray]:
        x = self._r(x)
        mu = np.empty_like(x); al = np.empty_like(x)
        rc = self.lib.orc_cond(C.byref(_as_cfg(cfg)), self._w(blob), j, self._p(x), self._p(mu), self._p(al))
        assert rc == 0
        return mu, al

    def forward_block(self, cfg, blob, j, x) -> np.ndarray:
        x = self._r(x); y = np.empty_like(x)
        assert self.lib.orc_forward_block(C.byref(_as_cfg(cfg)), self._w(blob), j, self._p(x), self._p(y)) == 0
        return y

    def forward_block_logdet(self, cfg, blob, j, x) -> Tuple[np.ndarray, float]:
        """eq. 4 for one sample and log |det dy/dx| of the block (= -sum alpha)."""
        x = self._r(x); y = np.empty_like(x); ld = np.zeros(1, self.dtype)
        assert self.lib.orc_forward_block_logdet(C.byref(_as_cfg(cfg)), self._w(blob), j, self._p(x), self._p(y),
                                                 self._p(ld)) == 0
        return y, float(ld[0])

    def sequential_inverse_block_naive(self, cfg, blob, j, z, fill: float = 0.0) -> np.ndarray:
        z = self._r(z); x = np.empty_like(z)
        assert self.lib.orc_sequential_inverse_block_naive(C.byref(_as_cfg(cfg)), self._w(blob), j, self._p(z),
                                                           self._p(x), C.c_double(fill)) == 0
        return x

    def sequential_inverse_block(self, cfg, blob, j, z) -> np.ndarray:
        z = self._r(z); x = np.empty_like(z)
        assert self.lib.orc_sequential_inverse_block(C.byref(_as_cfg(cfg)), self._w(blob), j, self._p(z),
                                                     self._p(x)) == 0
        return x

    def jacobi_map(self, cfg, blob, j, z, x_prev) -> np.ndarray:
        z = self._r(z); xp = self._r(x_prev); xn = np.empty_like(z)
        assert self.lib.orc_jacobi_map(C.byref(_as_cfg(cfg)), self._w(blob), j, self._p(z), self._p(xp),
                                       self._p(xn)) == 0
        return xn

    def jacobi_inverse_block(self, cfg, blob, j, z, tau, *, x0=None, criterion=0, max_iters=0,
                             want_trace=False, want_iterates=False):
        """Returns (x, iters[, trace][, iterates])."""
        z = self._r(z); x = np.empty_like(z)
        cap = cfg.seq_len if not (0 < max_iters < cfg.seq_len) else max_iters
        x0a = None if x0 is None else self._r(x0)
        trace = np.zeros(cap, self.dtype) if want_trace else None
        its = np.zeros((cap,) + z.shape, self.dtype) if want_iterates else None
        it = self.lib.orc_jacobi_inverse_block(C.byref(_as_cfg(cfg)), self._w(blob), j, self._p(z), self._p(x0a),
                                               C.c_double(tau), criterion, max_iters, self._p(x), self._p(trace),
                                               self._p(its))
        assert it >= 1
        out = [x, it]
        if want_trace:
            out.append(trace[:it])
        if want_iterates:
            out.append(its[:it])
        return tuple(out)

    # -- batch
    def sample(self, cfg, blob, z, jacobi_mask, tau, *, criterion=0, init=0, max_iters=0):
        """Returns (x [B,T,D], iters [K,B] int32, last_delta [K,B])."""
        z = self._r(z)
        B = z.shape[0]
        x = np.empty_like(z)
        iters = np.zeros((cfg.n_blocks, B), np.int32)
        deltas = np.zeros((cfg.n_blocks, B), self.dtype)
        rc = self.lib.orc_sample(C.byref(_as_cfg(cfg)), self._w(blob), self._p(z), self._p(x), B,
                                 C.c_uint32(jacobi_mask & 0xFFFFFFFF), C.c_double(tau), criterion, init, max_iters,
                                 iters.ctypes.data_as(C.POINTER(C.c_int32)), self._p(deltas))
        assert rc == 0
        return x, iters, deltas

    def forward(self, cfg, blob, x) -> np.ndarray:
        x = self._r(x); z = np.empty_like(x)
        assert self.lib.orc_forward(C.byref(_as_cfg(cfg)), self._w(blob), self._p(x), self._p(z), x.shape[0]) == 0
        return z

    def forward_logdet(self, cfg, blob, x) -> Tuple[np.ndarray, np.ndarray]:
        """Whole forward map (blocks K-1 .. 0) and its log-determinant per sample."""
        x = self._r(x); z = np.empty_like(x); ld = np.zeros(x.shape[0], self.dtype)
        assert self.lib.orc_forward_logdet(C.byref(_as_cfg(cfg)), self._w(blob), self._p(x), self._p(z), self._p(ld),
                                           x.shape[0]) == 0
        return z, ld

    # -- primitives
    def layernorm(self, x, g, b) -> np.ndarray:
        x = self._r(x); y = np.empty_like(x)
        g = np.ascontiguousarray(g, np.float32); b = np.ascontiguousarray(b, np.float32)
        self.lib.orc_layernorm(self._p(x), self._w(g), self._w(b), x.shape[0], x.shape[1], self._p(y))
        return y

    def linear(self, a, Wm, bias) -> np.ndarray:
        a = self._r(a)
        Wm = np.ascontiguousarray(Wm, np.float32); bias = np.ascontiguousarray(bias, np.float32)
        y = np.empty((a.shape[0], Wm.shape[1]), self.dtype)
        self.lib.orc_linear(self._p(a), self._w(Wm), self._w(bias), a.shape[0], Wm.shape[0], Wm.shape[1], self._p(y))
        return y

    def gelu(self, x) -> np.ndarray:
        x = self._r(x); y = np.empty_like(x)
        self.lib.orc_gelu(self._p(x), x.size, self._p(y))
        return y

    def causal_attention(self, q, k, v, H) -> np.ndarray:
        q = self._r(q); k = self._r(k); v = self._r(v); o = np.empty_like(q)
        self.lib.orc_causal_attention(self._p(q), self._p(k), self._p(v), q.shape[0], q.shape[1], H, self._p(o))
        return o
