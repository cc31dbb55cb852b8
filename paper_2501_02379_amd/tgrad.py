"""ctypes binding of libtgrad.so: the same entry points as include/tgrad.h.

Argument marshalling only.  PyTorch supplies device memory and the stream; every
arithmetic step of the optimizer runs in the library's HIP kernels.  There is no
CPU fallback: if the library is missing, `load()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

MAX_NDIM = 6
TGRAD_C64, TGRAD_CBF16 = 0, 1
TGRAD_SELECT_TOPK_MAG = 0
TGRAD_SELECT_RANDOM = 1
TGRAD_ORDER_US_LR, TGRAD_ORDER_LR_US, TGRAD_ORDER_SUM = 0, 1, 2

TGRAD_OK = 0
TGRAD_ERR_INVALID_ARG = -1
TGRAD_ERR_UNSUPPORTED = -2
TGRAD_ERR_NOT_READY = -3
TGRAD_ERR_HIP = -4
TGRAD_ERR_TOO_SMALL = -5
TGRAD_ERR_NOT_CONVERGED = -6

STATE_STEP, STATE_INDICES, STATE_CORE_M, STATE_CORE_V = 0, 1, 2, 3
STATE_SPARSE_M, STATE_SPARSE_V, STATE_SPARSE_G, STATE_CORE_G = 4, 5, 6, 7
STATE_GRAM0, STATE_FACTOR0, STATE_EIG_INFO0 = 32, 64, 96

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtgrad.so")

EXPORTS = (
    "tgrad_query_sizes", "tgrad_init", "tgrad_refresh_factors", "tgrad_step", "tgrad_step_static", "tgrad_get_state", "tgrad_check",
    "tgrad_set_state", "tgrad_set_profiling", "tgrad_get_kernel_times", "tgrad_calibration_copy",
    "tgrad_calibration_mfma", "tgrad_calibration_tile_stream",
    "tgrad_destroy", "tgrad_strerror",
)


class tgrad_config(C.Structure):
    _fields_ = [
        ("ndim", C.c_int32),
        ("shape", C.c_int64 * MAX_NDIM),
        ("rank", C.c_int32 * MAX_NDIM),
        ("k_sparse", C.c_int64),
        ("grad_dtype", C.c_int32),
        ("weight_dtype", C.c_int32),
        ("lr", C.c_float),
        ("beta1", C.c_float),
        ("beta2", C.c_float),
        ("eps", C.c_float),
        ("alpha", C.c_float),
        ("lambda_", C.c_float),
        ("weight_decay", C.c_float),
        ("refresh_every", C.c_int32),
        ("hooi_sweeps", C.c_int32),
        ("select_rule", C.c_int32),
        ("select_seed", C.c_uint64),
        ("order", C.c_int32),
        ("warm_restart", C.c_int32),
        ("eig_max_sweeps", C.c_int32),
    ]


class TgradError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, strerror(status), status))


_lib = None


def load():
    """dlopen libtgrad.so (built by paper_2501_02379_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libtgrad.so is not built: run `python -m paper_2501_02379_amd.build` "
            "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    lib.tgrad_query_sizes.argtypes = [C.POINTER(tgrad_config), C.POINTER(sz), C.POINTER(sz)]
    lib.tgrad_init.argtypes = [C.POINTER(vp), C.POINTER(tgrad_config), vp, vp, vp]
    lib.tgrad_refresh_factors.argtypes = [vp, vp]
    lib.tgrad_step.argtypes = [vp, vp, vp]
    lib.tgrad_step_static.argtypes = [C.POINTER(tgrad_config), vp, C.c_int64, vp, vp, vp]
    lib.tgrad_get_state.argtypes = [vp, i32, vp, sz]
    lib.tgrad_set_state.argtypes = [vp, i32, vp, sz]
    lib.tgrad_check.argtypes = [vp, C.POINTER(C.c_int64)]
    lib.tgrad_set_profiling.argtypes = [vp, i32]
    lib.tgrad_get_kernel_times.argtypes = [vp, C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                           C.POINTER(C.c_int64), i32]
    lib.tgrad_calibration_copy.argtypes = [vp, vp, sz, vp]
    lib.tgrad_calibration_mfma.argtypes = [C.c_int, C.c_int64, vp, vp, C.POINTER(C.c_double)]
    lib.tgrad_calibration_tile_stream.argtypes = [vp, sz, C.c_int, C.c_int, vp, C.POINTER(C.c_int64)]
    lib.tgrad_destroy.argtypes = [vp]
    lib.tgrad_strerror.argtypes = [i32]
    lib.tgrad_strerror.restype = C.c_char_p
    for name in EXPORTS:
        if name != "tgrad_strerror":
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load().tgrad_strerror(int(status)).decode()


def make_config(shape: Sequence[int], rank: Sequence[int], k_sparse: int, *, grad_dtype=TGRAD_C64,
                weight_dtype=TGRAD_C64, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, alpha=1.0,
                lam=1.0, weight_decay=0.0, refresh_every=1, hooi_sweeps=0,
                select_rule=TGRAD_SELECT_TOPK_MAG, select_seed=0, warm_restart=False,
                order=TGRAD_ORDER_US_LR, eig_max_sweeps=0) -> tgrad_config:
    cfg = tgrad_config()
    cfg.ndim = len(shape)
    if len(shape) <= MAX_NDIM and len(rank) == len(shape):
        for n, (i, r) in enumerate(zip(shape, rank)):
            cfg.shape[n] = int(i)
            cfg.rank[n] = int(r)
    cfg.k_sparse = int(k_sparse)
    cfg.grad_dtype = grad_dtype
    cfg.weight_dtype = weight_dtype
    cfg.lr, cfg.beta1, cfg.beta2, cfg.eps = lr, beta1, beta2, eps
    cfg.alpha, cfg.lambda_, cfg.weight_decay = alpha, lam, weight_decay
    cfg.refresh_every, cfg.hooi_sweeps, cfg.select_rule = refresh_every, hooi_sweeps, select_rule
    cfg.select_seed = int(select_seed) & 0xFFFFFFFFFFFFFFFF
    cfg.warm_restart = int(warm_restart)
    cfg.order = int(order)
    cfg.eig_max_sweeps = int(eig_max_sweeps)
    return cfg


def tgrad_query_sizes(cfg: tgrad_config):
    """-> (status, state_bytes, workspace_bytes)"""
    a, b = C.c_size_t(0), C.c_size_t(0)
    rc = load().tgrad_query_sizes(C.byref(cfg), C.byref(a), C.byref(b))
    return rc, a.value, b.value


def _ptr(t) -> int:
    return int(t.data_ptr())


class Context:
    """One weight tensor's optimizer context; owns the torch buffers behind state/workspace."""

    def __init__(self, cfg: tgrad_config, device="cuda:0", stream=None):
        import torch
        self.lib = load()
        self.cfg = cfg
        rc, sb, wb = tgrad_query_sizes(cfg)
        if rc != TGRAD_OK:
            raise TgradError(rc, "tgrad_query_sizes")
        self.state_bytes, self.workspace_bytes = sb, wb
        self.device = torch.device(device)
        self.state_buf = torch.empty(sb, dtype=torch.uint8, device=self.device)
        self.ws_buf = torch.empty(wb, dtype=torch.uint8, device=self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.handle = C.c_void_p(None)
        with torch.cuda.device(self.device):
            rc = self.lib.tgrad_init(C.byref(self.handle), C.byref(cfg), _ptr(self.state_buf),
                                     _ptr(self.ws_buf), C.c_void_p(self.stream.cuda_stream))
        if rc != TGRAD_OK:
            raise TgradError(rc, "tgrad_init")
        self.shape = tuple(int(cfg.shape[n]) for n in range(cfg.ndim))
        self.rank = tuple(int(cfg.rank[n]) for n in range(cfg.ndim))
        self.k = int(cfg.k_sparse)

    # ---- the three calls of the hot path -------------------------------------------------
    def tgrad_refresh_factors(self, grad) -> None:
        rc = self.lib.tgrad_refresh_factors(self.handle, _ptr(grad))
        if rc != TGRAD_OK:
            raise TgradError(rc, "tgrad_refresh_factors")

    def tgrad_step(self, weight, grad) -> None:
        rc = self.lib.tgrad_step(self.handle, _ptr(weight), _ptr(grad))
        if rc != TGRAD_OK:
            raise TgradError(rc, "tgrad_step")

    # ---- state ---------------------------------------------------------------------------
    def _item_array(self, what: int) -> np.ndarray:
        C_ = int(np.prod(self.rank))
        if what == STATE_STEP:
            return np.zeros(1, dtype=np.int64)
        if what == STATE_INDICES:
            return np.zeros(self.k, dtype=np.int64)
        if what in (STATE_CORE_M, STATE_CORE_G):
            return np.zeros(C_, dtype=np.complex64).reshape(self.rank)
        if what == STATE_CORE_V:
            return np.zeros(C_, dtype=np.float32).reshape(self.rank)
        if what in (STATE_SPARSE_M, STATE_SPARSE_G):
            return np.zeros(self.k, dtype=np.complex64)
        if what == STATE_SPARSE_V:
            return np.zeros(self.k, dtype=np.float32)
        if STATE_FACTOR0 <= what < STATE_FACTOR0 + len(self.shape):
            n = what - STATE_FACTOR0
            return np.zeros((self.shape[n], self.rank[n]), dtype=np.complex64)
        if STATE_EIG_INFO0 <= what < STATE_EIG_INFO0 + len(self.shape):
            return np.zeros(3, dtype=np.int32)
        if STATE_GRAM0 <= what < STATE_GRAM0 + len(self.shape):
            n = what - STATE_GRAM0
            return np.zeros((self.shape[n], self.shape[n]), dtype=np.complex128)
        raise TgradError(TGRAD_ERR_INVALID_ARG, "state selector")

    def tgrad_get_state(self, what: int) -> np.ndarray:
        out = self._item_array(what)
        rc = self.lib.tgrad_get_state(self.handle, what, out.ctypes.data_as(C.c_void_p), out.nbytes)
        if rc != TGRAD_OK:
            raise TgradError(rc, "tgrad_get_state")
        return out

    def tgrad_check(self) -> int:
        """Non-finite gradient entries seen by the last refresh."""
        n = C.c_int64(-1)
        rc = self.lib.tgrad_check(self.handle, C.byref(n))
        if rc != TGRAD_OK:
            raise TgradError(rc, "tgrad_check")
        return int(n.value)

    def tgrad_set_state(self, what: int, value) -> None:
        ref = self._item_array(what)
        arr = np.ascontiguousarray(np.asarray(value).astype(ref.dtype).reshape(ref.shape))
        rc = self.lib.tgrad_set_state(self.handle, what, arr.ctypes.data_as(C.c_void_p), arr.nbytes)
        if rc != TGRAD_OK:
            raise TgradError(rc, "tgrad_set_state")

    @property
    def t(self) -> int:
        return int(self.tgrad_get_state(STATE_STEP)[0])

    # ---- per-kernel timing ----------------------------------------------------------------
    def tgrad_set_profiling(self, enabled: bool) -> None:
        rc = self.lib.tgrad_set_profiling(self.handle, 1 if enabled else 0)
        if rc != TGRAD_OK:
            raise TgradError(rc, "tgrad_set_profiling")

    def tgrad_get_kernel_times(self) -> dict:
        cap = 64
        names = (C.c_char_p * cap)()
        ms = (C.c_double * cap)()
        cnt = (C.c_int64 * cap)()
        n = self.lib.tgrad_get_kernel_times(self.handle, names, ms, cnt, cap)
        if n < 0:
            raise TgradError(n, "tgrad_get_kernel_times")
        return {names[i].decode(): {"total_ms": ms[i], "launches": int(cnt[i])} for i in range(n)}

    def tgrad_destroy(self) -> None:
        if self.handle:
            self.lib.tgrad_destroy(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.tgrad_destroy()
        except Exception:
            pass


STATIC_WORKSPACE_BYTES = 32 << 20


def tgrad_step_static(cfg: tgrad_config, state, t: int, weight, grad, stream=None) -> None:
    """The allocation-free step: `state` is the caller's state buffer (a torch uint8 tensor of
    state_bytes, zero-filled before t = 0); scratch is the library's fixed per-GPU array."""
    import torch
    st = stream if stream is not None else torch.cuda.current_stream(weight.device)
    with torch.cuda.device(weight.device):
        rc = load().tgrad_step_static(C.byref(cfg), _ptr(state), int(t), _ptr(weight), _ptr(grad),
                                      C.c_void_p(st.cuda_stream))
    if rc != TGRAD_OK:
        raise TgradError(rc, "tgrad_step_static")


def tgrad_calibration_copy(dst, src, stream=None) -> None:
    """Plain copy kernel of known size (dst, src: torch tensors of equal byte length)."""
    import torch
    nbytes = dst.numel() * dst.element_size()
    if nbytes != src.numel() * src.element_size():
        raise TgradError(TGRAD_ERR_INVALID_ARG, "tgrad_calibration_copy")
    st = stream if stream is not None else torch.cuda.current_stream(dst.device)
    rc = load().tgrad_calibration_copy(_ptr(dst), _ptr(src), nbytes, C.c_void_p(st.cuda_stream))
    if rc != TGRAD_OK:
        raise TgradError(rc, "tgrad_calibration_copy")


def tgrad_calibration_tile_stream(buf, tile_bytes: int, tiles_per_slab: int, stream=None) -> int:
    """The update kernel's access pattern without arithmetic on `buf` (a torch tensor, rewritten with
    itself); returns the bytes one launch reads (it writes as many)."""
    import torch
    st = stream if stream is not None else torch.cuda.current_stream(buf.device)
    n = C.c_int64(0)
    rc = load().tgrad_calibration_tile_stream(_ptr(buf), buf.numel() * buf.element_size(), int(tile_bytes),
                                              int(tiles_per_slab), C.c_void_p(st.cuda_stream), C.byref(n))
    if rc != TGRAD_OK:
        raise TgradError(rc, "tgrad_calibration_tile_stream")
    return int(n.value)


def tgrad_calibration_mfma(kind: int, iterations: int, sink, stream=None) -> float:
    """Register-resident matrix-core loop (kind 0: float32, 1: float64); returns the launch's flops."""
    import torch
    st = stream if stream is not None else torch.cuda.current_stream(sink.device)
    flops = C.c_double(0.0)
    rc = load().tgrad_calibration_mfma(int(kind), int(iterations), _ptr(sink), C.c_void_p(st.cuda_stream),
                                       C.byref(flops))
    if rc != TGRAD_OK:
        raise TgradError(rc, "tgrad_calibration_mfma")
    return float(flops.value)


def to_device_grad(g: np.ndarray, device="cuda:0"):
    """Upload a gradient (complex64, or uint16 bf16 pairs with a trailing axis of 2)."""
    import torch
    g = np.ascontiguousarray(g)
    if g.dtype == np.complex64:
        return torch.from_numpy(g.view(np.float32).reshape(g.shape + (2,))).to(device)
    if g.dtype == np.uint16:
        return torch.from_numpy(g.view(np.int16)).to(device)
    raise TypeError("gradient must be complex64 or uint16 bf16 pairs")


def to_device_weight(w: np.ndarray, device="cuda:0"):
    """Upload weights: complex64, or uint16 bf16 (re, im) pairs with a trailing axis of 2 (for a
    context made with weight_dtype=TGRAD_CBF16)."""
    import torch
    if np.asarray(w).dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(w).view(np.int16)).to(device)
    w = np.ascontiguousarray(w, dtype=np.complex64)
    return torch.from_numpy(w.view(np.float32).reshape(w.shape + (2,))).to(device)


def weight_to_host(w_dev) -> np.ndarray:
    """complex64 array, or uint16 bf16 pairs (trailing axis 2) for half-precision weights."""
    a = np.ascontiguousarray(w_dev.detach().cpu().numpy())
    if a.dtype == np.int16:
        return a.view(np.uint16)
    return a.view(np.complex64).reshape(a.shape[:-1])
