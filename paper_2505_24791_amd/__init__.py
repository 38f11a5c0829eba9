"""Thin Python binding of the HIP library ``libsjd.so`` (see ``include/sjd.h``).

Argument marshalling only: every step of selective Jacobi decoding runs in the library's kernels.
PyTorch is used for device memory and streams.  There is no CPU path: importing works anywhere,
but creating a ``Flow`` without the built library or without an MI355X raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsjd.so")

SJD_OK, SJD_EINVAL, SJD_ENOMEM, SJD_EHIP, SJD_ENONFINITE, SJD_ESTATE = 0, -1, -2, -3, -4, -5
SJD_MAX_BLOCKS = 32
DTYPE_F32, DTYPE_BF16, DTYPE_F16 = 0, 1, 2
(PROF_GEMM, PROF_ATTENTION, PROF_EPILOGUE, PROF_DECODE_GEMM, PROF_DECODE_ATTN, PROF_OTHER, PROF_DECODE_FUSED,
 PROF_GEMM_RESID, PROF_GEMM_FC1, PROF_DECODE_RESID, PROF_GEMM_HEAD, PROF_DECODE_FC1, PROF_DECODE_HEAD) = range(13)
PROF_FAMILIES = 13
PROF_NAMES = ("gemm_qkv", "attention", "epilogue", "decode_qkv", "decode_attn", "other", "decode_fused", "gemm_resid",
              "gemm_fc1", "decode_resid", "gemm_head", "decode_fc1", "decode_head")
PROF_GEMM_ALL = (PROF_GEMM, PROF_GEMM_RESID, PROF_GEMM_FC1, PROF_GEMM_HEAD)            # every whole-sequence projection
PROF_DECODE_GEMM_ALL = (PROF_DECODE_GEMM, PROF_DECODE_RESID, PROF_DECODE_FC1, PROF_DECODE_HEAD)   # every single-token projection

EXPORTS = ("sjd_flow_create", "sjd_flow_load_weights", "sjd_jacobi_inverse_block", "sjd_sequential_inverse_block",
           "sjd_sample", "sjd_conditioner", "sjd_op_linear_h16", "sjd_jacobi_trace_block", "sjd_forward_block",
           "sjd_forward", "sjd_flow_set_mask_nearest", "sjd_flow_set_sequential_path", "sjd_flow_set_sequential_cus", "sjd_flow_set_projection_path",
           "sjd_op_panel_linear_h16", "sjd_op_panel_linear_h16_noalloc", "sjd_op_attention_h16", "sjd_profile_enable", "sjd_profile_read", "sjd_flow_device_bytes",
           "sjd_last_error", "sjd_flow_destroy")


class SjdConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_blocks", "n_layers", "width", "n_heads", "mlp_ratio", "seq_len",
                                         "token_dim", "max_batch", "dtype")] + [("reverse_mask", C.c_uint32)]


class SjdJacobiOpts(C.Structure):
    _fields_ = [("tau", C.c_float), ("criterion", C.c_int32), ("init", C.c_int32), ("max_iters", C.c_int32),
                ("drop_converged", C.c_int32), ("refine_below", C.c_float)]


class SjdStats(C.Structure):
    _fields_ = [("block_iters", C.c_int32 * SJD_MAX_BLOCKS), ("mean_sample_iters", C.c_float * SJD_MAX_BLOCKS),
                ("block_ms", C.c_float * SJD_MAX_BLOCKS)]


class SjdProfile(C.Structure):
    _fields_ = [("ms", C.c_double * PROF_FAMILIES), ("launches", C.c_int64 * PROF_FAMILIES),
                ("flops", C.c_double * PROF_FAMILIES), ("bytes", C.c_double * PROF_FAMILIES)]


class SjdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"sjd error {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Loads libsjd.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2505_24791_amd.build` "
                           "(or __graft_entry__.build()) first; this package has no CPU fallback")
    lib = C.CDLL(LIB_PATH)
    vp, i32p, fp = C.c_void_p, C.POINTER(C.c_int32), C.c_void_p
    lib.sjd_flow_create.argtypes = [C.POINTER(SjdConfig), C.POINTER(vp)]
    lib.sjd_flow_load_weights.argtypes = [vp, vp, C.c_size_t]
    lib.sjd_jacobi_inverse_block.argtypes = [vp, C.c_int, fp, fp, C.c_int, C.POINTER(SjdJacobiOpts), i32p, i32p, vp]
    lib.sjd_sequential_inverse_block.argtypes = [vp, C.c_int, fp, fp, C.c_int, vp]
    lib.sjd_sample.argtypes = [vp, fp, fp, C.c_int, C.c_uint32, C.POINTER(SjdJacobiOpts), C.POINTER(SjdStats), i32p, vp]
    lib.sjd_conditioner.argtypes = [vp, C.c_int, fp, fp, fp, C.c_int, vp]
    lib.sjd_jacobi_trace_block.argtypes = [vp, C.c_int, vp, vp, vp, C.c_int, C.POINTER(SjdJacobiOpts),
                                           C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_int32),
                                           C.POINTER(C.c_int32), vp]
    lib.sjd_forward_block.argtypes = [vp, C.c_int, vp, vp, vp, C.c_int, C.c_int, vp]
    lib.sjd_forward.argtypes = [vp, vp, vp, vp, C.c_int, vp]
    lib.sjd_flow_set_sequential_path.argtypes = [vp, C.c_int]
    lib.sjd_flow_set_sequential_cus.argtypes = [vp, C.c_int]
    lib.sjd_flow_set_mask_nearest.argtypes = [vp, C.c_int]
    lib.sjd_op_linear_h16.argtypes = [C.c_int, C.c_int, vp, vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, vp]
    lib.sjd_op_attention_h16.argtypes = [C.c_int, vp, vp, C.c_int, C.c_int, C.c_int, vp]
    lib.sjd_profile_enable.argtypes = [vp, C.c_uint32]
    lib.sjd_profile_read.argtypes = [vp, C.POINTER(SjdProfile), C.c_int]
    lib.sjd_flow_device_bytes.argtypes = [vp]
    lib.sjd_flow_device_bytes.restype = C.c_size_t
    lib.sjd_last_error.restype = C.c_char_p
    lib.sjd_flow_destroy.argtypes = [vp]
    lib.sjd_flow_destroy.restype = None
    for name in EXPORTS:
        if name not in ("sjd_flow_device_bytes", "sjd_last_error", "sjd_flow_destroy"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int, allow_nonfinite: bool = False) -> int:
    if rc == SJD_OK or (allow_nonfinite and rc == SJD_ENONFINITE):
        return rc
    raise SjdError(rc, load_library().sjd_last_error().decode())


@dataclass
class JacobiOpts:
    tau: float = 1e-3
    criterion: int = 0
    init: int = 0
    max_iters: int = 0
    drop_converged: int = 1
    refine_below: float = 0.0

    def c(self) -> SjdJacobiOpts:
        return SjdJacobiOpts(self.tau, self.criterion, self.init, self.max_iters, self.drop_converged,
                             self.refine_below)


def _stream_ptr() -> Optional[int]:
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, shape=None) -> C.c_void_p:
    import torch
    assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous(), "need a contiguous float32 CUDA tensor"
    if shape is not None:
        assert tuple(t.shape) == tuple(shape), (tuple(t.shape), tuple(shape))
    return C.c_void_p(t.data_ptr())


def op_linear_h16(a, wt, bias, M, N, K, epilogue, *, resid=None, kernel=0):
    """``sjd_op_linear_h16`` on torch tensors: a [M,K] and wt [N_pad,K] in float16 or bfloat16 (same
    type), bias [N] float32; returns c [M,N] (16-bit) or, for epilogue 2, updates ``resid`` in place."""
    import torch
    lib = load_library()
    assert a.is_cuda and wt.is_cuda and a.dtype == wt.dtype and a.is_contiguous() and wt.is_contiguous()
    assert wt.shape[0] % 256 == 0 and wt.shape[0] >= N and wt.shape[1] == K and tuple(a.shape) == (M, K)
    dtype = DTYPE_F16 if a.dtype == torch.float16 else DTYPE_BF16
    c = None
    if epilogue == 2:
        assert resid is not None and resid.dtype == torch.float32 and tuple(resid.shape) == (M, N) and resid.is_contiguous()
    else:
        c = torch.empty((M, N), dtype=a.dtype, device=a.device)
    _check(lib.sjd_op_linear_h16(dtype, kernel, C.c_void_p(a.data_ptr()), C.c_void_p(wt.data_ptr()),
                                 C.c_void_p(bias.data_ptr()), C.c_void_p(resid.data_ptr()) if resid is not None else None,
                                 C.c_void_p(c.data_ptr()) if c is not None else None, M, N, K, epilogue, _stream_ptr()))
    return resid if epilogue == 2 else c


def op_panel_linear_h16(a, wt, bias, M, N, epilogue, *, K=512, ln_g=None, ln_b=None, resid=None, noalloc=False):
    """``sjd_op_panel_linear_h16`` on torch tensors.  epilogue 0 / 1 (K = 512): a [M,512] float32, ln_g / ln_b
    [512] float32, returns c [M,N] in wt's type; epilogue 2: a [M,K] 16-bit, updates ``resid`` in place."""
    import torch
    lib = load_library()
    assert a.is_cuda and wt.is_cuda and a.is_contiguous() and wt.is_contiguous() and tuple(a.shape) == (M, K)
    assert wt.shape[0] >= N and wt.shape[1] == K and wt.dtype in (torch.float16, torch.bfloat16)
    dtype = DTYPE_F16 if wt.dtype == torch.float16 else DTYPE_BF16
    c = None
    if epilogue == 2:
        assert a.dtype == wt.dtype
        assert resid is not None and resid.dtype == torch.float32 and tuple(resid.shape) == (M, N) and resid.is_contiguous()
    else:
        assert a.dtype == torch.float32 and ln_g is not None and ln_b is not None
        c = torch.empty((M, N), dtype=wt.dtype, device=a.device)
    ptr = lambda t: C.c_void_p(t.data_ptr()) if t is not None else None
    fn = lib.sjd_op_panel_linear_h16_noalloc if noalloc else lib.sjd_op_panel_linear_h16
    _check(fn(dtype, ptr(a), ptr(ln_g), ptr(ln_b), ptr(wt), ptr(bias), ptr(resid), ptr(c), M, N, K, epilogue, _stream_ptr()))
    return resid if epilogue == 2 else c


def op_attention_h16(qkv, n_samples, T, H):
    """``sjd_op_attention_h16`` on a torch tensor: qkv [n_samples*T, 3*H*64] float16, bfloat16 or float32;
    returns o [n_samples*T, H*64] of the same type."""
    import torch
    lib = load_library()
    assert qkv.is_cuda and qkv.is_contiguous() and tuple(qkv.shape) == (n_samples * T, 3 * H * 64)
    dtype = {torch.float16: DTYPE_F16, torch.bfloat16: DTYPE_BF16, torch.float32: DTYPE_F32}[qkv.dtype]
    o = torch.empty((n_samples * T, H * 64), dtype=qkv.dtype, device=qkv.device)
    _check(lib.sjd_op_attention_h16(dtype, C.c_void_p(qkv.data_ptr()), C.c_void_p(o.data_ptr()), n_samples, T, H,
                                    _stream_ptr()))
    return o


class Flow:
    """A flow on the current device.  ``cfg`` needs the attributes of ``workloads.FlowConfig``."""

    def __init__(self, cfg, max_batch: Optional[int] = None, dtype: Optional[int] = None):
        self.lib = load_library()
        self.cfg = cfg
        self.max_batch = int(max_batch if max_batch is not None else cfg.batch)
        # 16-bit workloads default to IEEE-half operands: their bf16-valued weights convert exactly and
        # the activations keep three more mantissa bits, which the stopping rule needs (tau ~ 1e-3)
        self.dtype = (DTYPE_F16 if cfg.bf16 else DTYPE_F32) if dtype is None else dtype
        c = SjdConfig(cfg.n_blocks, cfg.n_layers, cfg.width, cfg.n_heads, cfg.mlp_ratio, cfg.seq_len, cfg.token_dim,
                      self.max_batch, self.dtype, cfg.reverse_mask)
        h = C.c_void_p()
        _check(self.lib.sjd_flow_create(C.byref(c), C.byref(h)))
        self._h = h

    def close(self) -> None:
        if getattr(self, "_h", None):
            self.lib.sjd_flow_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def device_bytes(self) -> int:
        return int(self.lib.sjd_flow_device_bytes(self._h))

    def load_weights(self, blob: np.ndarray) -> None:
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        _check(self.lib.sjd_flow_load_weights(self._h, C.c_void_p(blob.ctypes.data), blob.nbytes))

    def _shape(self, batch):
        return (batch, self.cfg.seq_len, self.cfg.token_dim)

    def conditioner(self, block: int, x):
        import torch
        B = x.shape[0]
        mu = torch.empty_like(x); al = torch.empty_like(x)
        _check(self.lib.sjd_conditioner(self._h, block, _dev(x, self._shape(B)), _dev(mu), _dev(al), B, _stream_ptr()))
        return mu, al

    def jacobi_inverse_block(self, block: int, z, opts: JacobiOpts, allow_nonfinite: bool = False, x0=None):
        """Returns (x, iters_per_sample int32 [B], passes_launched, rc).  With opts.init == 2 the first
        iterate is ``x0`` (copied, not modified)."""
        import torch
        B = z.shape[0]
        x = torch.empty_like(z) if x0 is None else x0.detach().clone().contiguous()
        iters = np.zeros(B, np.int32)
        passes = C.c_int32(0)
        o = opts.c()
        rc = _check(self.lib.sjd_jacobi_inverse_block(self._h, block, _dev(z, self._shape(B)), _dev(x), B, C.byref(o),
                                                      iters.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(passes),
                                                      _stream_ptr()), allow_nonfinite)
        return x, iters, int(passes.value), rc

    def jacobi_trace_block(self, block: int, z, opts: JacobiOpts, x_ref=None, x0=None):
        """Jacobi decoding with the per-pass record.  Returns (x, iters [B], passes, delta [passes, B],
        err [passes, B] or None)."""
        import torch
        B = z.shape[0]
        T = self.cfg.seq_len
        cap = opts.max_iters if 0 < opts.max_iters < T else T
        x = torch.empty_like(z) if x0 is None else x0.detach().clone().contiguous()
        iters = np.zeros(B, np.int32)
        passes = C.c_int32(0)
        delta = np.zeros((cap, B), np.float32)
        err = np.zeros((cap, B), np.float32) if x_ref is not None else None
        o = opts.c()
        fp = C.POINTER(C.c_float)
        _check(self.lib.sjd_jacobi_trace_block(
            self._h, block, _dev(z, self._shape(B)), _dev(x), _dev(x_ref, self._shape(B)) if x_ref is not None else None,
            B, C.byref(o), delta.ctypes.data_as(fp), err.ctypes.data_as(fp) if err is not None else None,
            iters.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(passes), _stream_ptr()))
        n = int(passes.value)
        return x, iters, n, delta[:n], (err[:n] if err is not None else None)

    def forward_block(self, block: int, x, logdet=None, accumulate: bool = False):
        """eq. 4 for one block.  Returns (y, logdet [B] float32 device tensor)."""
        import torch
        B = x.shape[0]
        y = torch.empty_like(x)
        if logdet is None:
            logdet = torch.zeros(B, dtype=torch.float32, device=x.device)
        _check(self.lib.sjd_forward_block(self._h, block, _dev(x, self._shape(B)), _dev(y), C.c_void_p(logdet.data_ptr()),
                                          1 if accumulate else 0, B, _stream_ptr()))
        return y, logdet

    def forward(self, x):
        """The whole forward map (blocks K-1 .. 0).  Returns (z, logdet [B])."""
        import torch
        B = x.shape[0]
        z = torch.empty_like(x)
        logdet = torch.zeros(B, dtype=torch.float32, device=x.device)
        _check(self.lib.sjd_forward(self._h, _dev(x, self._shape(B)), _dev(z), C.c_void_p(logdet.data_ptr()), B,
                                    _stream_ptr()))
        return z, logdet

    def sequential_inverse_block(self, block: int, z):
        import torch
        B = z.shape[0]
        x = torch.empty_like(z)
        _check(self.lib.sjd_sequential_inverse_block(self._h, block, _dev(z, self._shape(B)), _dev(x), B, _stream_ptr()))
        return x

    def sample(self, z, jacobi_mask: int, opts: JacobiOpts, out=None, want_iters: bool = True,
               allow_nonfinite: bool = False):
        """Returns (x, stats dict, iters int32 [K, B] or None)."""
        import torch
        B = z.shape[0]
        x = torch.empty_like(z) if out is None else out
        K = self.cfg.n_blocks
        stats = SjdStats()
        iters = np.zeros((K, B), np.int32) if want_iters else None
        ip = iters.ctypes.data_as(C.POINTER(C.c_int32)) if want_iters else None
        o = opts.c()
        _check(self.lib.sjd_sample(self._h, _dev(z, self._shape(B)), _dev(x, self._shape(B)), B,
                                   C.c_uint32(jacobi_mask & 0xFFFFFFFF), C.byref(o), C.byref(stats), ip, _stream_ptr()),
               allow_nonfinite)
        st = {"block_iters": list(stats.block_iters[:K]), "mean_sample_iters": list(stats.mean_sample_iters[:K]),
              "block_ms": list(stats.block_ms[:K])}
        return x, st, iters

    def set_mask_nearest(self, o: int) -> None:
        """Masked-dependency probe (eq. 6): attention ignores the o nearest preceding positions; 0 = off."""
        _check(self.lib.sjd_flow_set_mask_nearest(self._h, o))

    def set_sequential_path(self, path: int) -> None:
        """0 automatic, 1 per-step launches (graph replay), 2 persistent kernel, 3 the same with a plain launch."""
        _check(self.lib.sjd_flow_set_sequential_path(self._h, path))

    def set_projection_path(self, path: int) -> None:
        """0 automatic, 1 tile kernels + LayerNorm launches, 2 activation-stationary kernels (16-bit, width 512)."""
        _check(self.lib.sjd_flow_set_projection_path(self._h, path))

    def set_sequential_cus(self, n_cus: int) -> None:
        """Workgroups of the persistent sequential kernel: 0 = one per CU of the device, else a multiple of 32."""
        _check(self.lib.sjd_flow_set_sequential_cus(self._h, n_cus))

    def profile_enable(self, families) -> None:
        """Family indices (PROF_*); PROF_GEMM / PROF_DECODE_GEMM stand for every whole-sequence / single-token
        projection family."""
        mask = 0
        for f in families:
            mask |= 1 << f
            if f == PROF_GEMM:
                for g in PROF_GEMM_ALL:
                    mask |= 1 << g
            if f == PROF_DECODE_GEMM:
                for g in PROF_DECODE_GEMM_ALL:
                    mask |= 1 << g
        _check(self.lib.sjd_profile_enable(self._h, mask))

    def profile_read(self, reset: bool = True) -> dict:
        p = SjdProfile()
        _check(self.lib.sjd_profile_read(self._h, C.byref(p), 1 if reset else 0))
        out = {PROF_NAMES[i]: {"ms": p.ms[i], "launches": int(p.launches[i]), "flops": p.flops[i], "bytes": p.bytes[i]}
               for i in range(PROF_FAMILIES)}
        # all whole-sequence projections together, all single-token projections together
        out["gemm"] = {k: sum(out[PROF_NAMES[g]][k] for g in PROF_GEMM_ALL) for k in ("ms", "launches", "flops", "bytes")}
        out["decode_gemm"] = {k: sum(out[PROF_NAMES[g]][k] for g in PROF_DECODE_GEMM_ALL)
                              for k in ("ms", "launches", "flops", "bytes")}
        return out
