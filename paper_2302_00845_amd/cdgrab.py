"""ctypes binding of libcdgrab.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks their
dtype / shape / contiguity, and passes raw device pointers through the C ABI.
There is no fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # loaded first so that the HIP runtime torch ships is the one in the process

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcdgrab.so")
_lib = None

CDGRAB_OK, CDGRAB_EINVAL, CDGRAB_ENOMEM, CDGRAB_EHIP, CDGRAB_EGEN = 0, -1, -2, -3, -4

GEN_FN = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                          ctypes.c_void_p, ctypes.c_void_p)


class CdgrabError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("cdgrab error %d: %s" % (code, text))
        self.code = code


class _Options(ctypes.Structure):
    _fields_ = [("device", ctypes.c_int32), ("block_pairs", ctypes.c_int32),
                ("stream", ctypes.c_void_p), ("timing", ctypes.c_int32),
                ("pass1_groups", ctypes.c_int32), ("apply_mode", ctypes.c_int32),
                ("gram_mode", ctypes.c_int32), ("apply_groups", ctypes.c_int32)]


class Timing(ctypes.Structure):
    _fields_ = [("generator_ms", ctypes.c_double), ("balance_ms", ctypes.c_double),
                ("pass1_ms", ctypes.c_double), ("reduce_ms", ctypes.c_double),
                ("resolve_ms", ctypes.c_double), ("pass2_ms", ctypes.c_double),
                ("finish_ms", ctypes.c_double), ("blocks", ctypes.c_int64),
                ("block_pairs", ctypes.c_int32), ("pass1_groups", ctypes.c_int32)]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


class Plan(ctypes.Structure):
    _fields_ = [("pairs", ctypes.c_int64), ("blocks", ctypes.c_int64),
                ("block_pairs", ctypes.c_int32), ("vector_width", ctypes.c_int32),
                ("tile_elems", ctypes.c_int32), ("fused_apply", ctypes.c_int32),
                ("pass1_groups", ctypes.c_int32), ("pass2_groups", ctypes.c_int32),
                ("gram_ahead", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("workspace_bytes", ctypes.c_int64), ("staging_bytes", ctypes.c_int64),
                ("bytes_per_example", ctypes.c_double)]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libcdgrab.so (built by ``python -m paper_2302_00845_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_2302_00845_amd.build` "
            "(there is no fallback path)" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    P, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    lib.cdgrab_create.argtypes = [ctypes.POINTER(P), ctypes.POINTER(_Options)]
    lib.cdgrab_create.restype = ctypes.c_int
    lib.cdgrab_destroy.argtypes = [P]
    lib.cdgrab_destroy.restype = ctypes.c_int
    lib.cdgrab_last_error.argtypes = [P]
    lib.cdgrab_last_error.restype = ctypes.c_char_p
    lib.cdgrab_plan_epoch.argtypes = [i64, i64, i64, i32, i32, i64, ctypes.POINTER(Plan)]
    lib.cdgrab_plan_epoch.restype = ctypes.c_int
    lib.cdgrab_pergrad.argtypes = [P, i64, i64, i64, P, P, P, P]
    lib.cdgrab_pergrad.restype = ctypes.c_int
    lib.cdgrab_balance_epoch.argtypes = [P, i64, i64, i64, P, P, P, P, P, P, P, P, P]
    lib.cdgrab_balance_epoch.restype = ctypes.c_int
    lib.cdgrab_reorder.argtypes = [P, i64, i64, P, P, P]
    lib.cdgrab_reorder.restype = ctypes.c_int
    lib.cdgrab_balance_epoch_randomized.argtypes = [P, i64, i64, i64, P, P, P, P, P, P, P]
    lib.cdgrab_balance_epoch_randomized.restype = ctypes.c_int
    lib.cdgrab_balance_epoch_stale_mean.argtypes = [P, i64, i64, P, P, P, P, P, P, P]
    lib.cdgrab_balance_epoch_stale_mean.restype = ctypes.c_int
    lib.cdgrab_balance_epoch_independent.argtypes = [P, i64, i64, i64, P, P, P, P]
    lib.cdgrab_balance_epoch_independent.restype = ctypes.c_int
    lib.cdgrab_train_epoch_softmax.argtypes = [P, i64, i64, i64, i64, P, P, P, P, P, ctypes.c_float,
                                               ctypes.c_float, P, P, P, P]
    lib.cdgrab_train_epoch_softmax.restype = ctypes.c_int
    lib.cdgrab_train_softmax.argtypes = [P, i64, i64, i64, i64, P, P, P, P, P, ctypes.c_float,
                                         ctypes.c_float, i64, P, P]
    lib.cdgrab_train_softmax.restype = ctypes.c_int
    lib.cdgrab_herding_bound.argtypes = [P, i64, i64, i64, P, P, P]
    lib.cdgrab_herding_bound.restype = ctypes.c_int
    lib.cdgrab_balance_epoch_static.argtypes = [P, i64, i64, i64, P, P, P, P, P, P, P]
    lib.cdgrab_balance_epoch_static.restype = ctypes.c_int
    lib.cdgrab_get_timing.argtypes = [P, ctypes.POINTER(Timing)]
    lib.cdgrab_get_timing.restype = ctypes.c_int
    _lib = lib
    return lib


def cdgrab_plan_epoch(m: int, n: int, d: int, block_pairs: int = 0, streamed: bool = False,
                      base_align: int = 16) -> dict:
    """Host-only blocking plan (cdgrab_plan_epoch)."""
    lib = load_library()
    plan = Plan()
    rc = lib.cdgrab_plan_epoch(m, n, d, block_pairs, 1 if streamed else 0, base_align,
                               ctypes.byref(plan))
    if rc != CDGRAB_OK:
        raise CdgrabError(rc, "cdgrab_plan_epoch rejected m=%d n=%d d=%d block_pairs=%d" % (m, n, d, block_pairs))
    return plan.as_dict()


def _ptr(t: Optional[torch.Tensor], dtype, shape, name, device) -> Optional[int]:
    if t is None:
        return None
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if t.device != device:
        raise ValueError("%s must live on %s, got %s" % (name, device, t.device))
    return t.data_ptr()


class Handle:
    """Owns a cdgrab_handle (workspace + stream binding) on one GPU."""

    def __init__(self, device: int = 0, block_pairs: int = 0, timing: int = 0,
                 pass1_groups: int = 0, stream: Optional[torch.cuda.Stream] = None,
                 apply_mode: int = 0, gram_mode: int = 0, apply_groups: int = 0):
        self._lib = load_library()
        self.device = torch.device("cuda", device)
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        self.stream = stream
        opt = _Options(device=device, block_pairs=block_pairs, stream=stream.cuda_stream,
                       timing=timing, pass1_groups=pass1_groups,
                       apply_mode=apply_mode, gram_mode=gram_mode, apply_groups=apply_groups)
        h = ctypes.c_void_p()
        rc = self._lib.cdgrab_create(ctypes.byref(h), ctypes.byref(opt))
        if rc != CDGRAB_OK:
            raise CdgrabError(rc, self._lib.cdgrab_last_error(None).decode())
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.cdgrab_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != CDGRAB_OK:
            raise CdgrabError(rc, self._lib.cdgrab_last_error(self._h).decode())

    def timing(self) -> dict:
        t = Timing()
        self._check(self._lib.cdgrab_get_timing(self._h, ctypes.byref(t)))
        return t.as_dict()


def cdgrab_pergrad(h: Handle, X: torch.Tensor, y: torch.Tensor, W: torch.Tensor,
                   G_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Per-example softmax cross-entropy gradients G[N][(in_dim+1)*classes]."""
    N, in_dim = X.shape
    classes = W.shape[1]
    if G_out is None:
        G_out = torch.empty((N, (in_dim + 1) * classes), dtype=torch.float32, device=h.device)
    h._check(h._lib.cdgrab_pergrad(
        h._h, N, in_dim, classes,
        _ptr(X, torch.float32, (N, in_dim), "X", h.device),
        _ptr(y, torch.int32, (N,), "y", h.device),
        _ptr(W, torch.float32, (in_dim + 1, classes), "W", h.device),
        _ptr(G_out, torch.float32, (N, (in_dim + 1) * classes), "G_out", h.device)))
    return G_out


def cdgrab_balance_epoch(h: Handle, m: int, n: int, d: int,
                         grads: Optional[torch.Tensor] = None,
                         gen=None, gen_ctx: Optional[int] = None,
                         perm_in: Optional[torch.Tensor] = None,
                         want_r32: bool = True, want_r64: bool = False,
                         want_dots: bool = False) -> dict:
    """One epoch of coordinated pair balancing.

    ``grads`` is a [m][n][d] fp32 GPU tensor, or ``gen`` is a C function pointer
    (cdgrab_gen_fn, e.g. taken from another shared library with ctypes) with its
    context pointer ``gen_ctx``.  Returns the output tensors in a dict.
    """
    dev = h.device
    half = n // 2 if n >= 0 else 0
    signs = torch.empty((max(m, 0), max(half, 0)), dtype=torch.int8, device=dev)
    perm = torch.empty((max(m, 0), max(n, 0)), dtype=torch.int32, device=dev)
    r32 = torch.empty((max(d, 0),), dtype=torch.float32, device=dev) if want_r32 else None
    r64 = torch.empty((max(d, 0),), dtype=torch.float64, device=dev) if want_r64 else None
    dots = torch.empty((max(m, 0), max(half, 0)), dtype=torch.float64, device=dev) if want_dots else None
    gptr = _ptr(grads, torch.float32, (m, n, d), "grads", dev) if grads is not None else None
    gen_ptr = ctypes.cast(gen, ctypes.c_void_p) if gen is not None else None
    h._check(h._lib.cdgrab_balance_epoch(
        h._h, m, n, d, gptr, gen_ptr, gen_ctx,
        _ptr(perm_in, torch.int32, (m, n), "perm_in", dev),
        signs.data_ptr(), perm.data_ptr(),
        r32.data_ptr() if r32 is not None else None,
        r64.data_ptr() if r64 is not None else None,
        dots.data_ptr() if dots is not None else None))
    return {"signs": signs, "perm": perm, "r32": r32, "r64": r64, "dots": dots}


def cdgrab_balance_epoch_static(h: Handle, grads: torch.Tensor, out: dict,
                                perm_in: Optional[torch.Tensor] = None) -> dict:
    """cdgrab_balance_epoch on the library's static workspace (dense input, rows of at most
    CDGRAB_STATIC_MAX_D elements).  The call allocates nothing: ``out`` holds the caller's
    output tensors ``signs`` [m][n/2] int8 and ``perm`` [m][n] int32, and optionally ``r32``
    [d] float32, ``r64`` [d] float64, ``dots`` [m][n/2] float64."""
    m, n, d = grads.shape
    dev = h.device
    h._check(h._lib.cdgrab_balance_epoch_static(
        h._h, m, n, d, _ptr(grads, torch.float32, (m, n, d), "grads", dev),
        _ptr(perm_in, torch.int32, (m, n), "perm_in", dev),
        _ptr(out["signs"], torch.int8, (m, n // 2), "signs", dev),
        _ptr(out["perm"], torch.int32, (m, n), "perm", dev),
        _ptr(out.get("r32"), torch.float32, (d,), "r32", dev),
        _ptr(out.get("r64"), torch.float64, (d,), "r64", dev),
        _ptr(out.get("dots"), torch.float64, (m, n // 2), "dots", dev)))
    return out


def cdgrab_reorder(h: Handle, signs: torch.Tensor, perm_in: Optional[torch.Tensor] = None) -> torch.Tensor:
    """General reorder from per-example +-1 signs [m][n] (int8)."""
    m, n = signs.shape
    out = torch.empty((m, n), dtype=torch.int32, device=h.device)
    h._check(h._lib.cdgrab_reorder(
        h._h, m, n, _ptr(signs, torch.int8, (m, n), "signs", h.device),
        _ptr(perm_in, torch.int32, (m, n), "perm_in", h.device), out.data_ptr()))
    return out


def cdgrab_herding_bound(h: Handle, z: torch.Tensor, perm: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Parallel herding objective of z[m][n][d] (indexed by example id) visited in
    the orders perm[m][n]; returns a one-element float64 GPU tensor."""
    m, n, d = z.shape
    out = torch.empty((1,), dtype=torch.float64, device=h.device)
    h._check(h._lib.cdgrab_herding_bound(
        h._h, m, n, d, _ptr(z, torch.float32, (m, n, d), "z", h.device),
        _ptr(perm, torch.int32, (m, n), "perm", h.device), out.data_ptr()))
    return out


def cdgrab_train_epoch_softmax(h: Handle, X: torch.Tensor, y: torch.Tensor, W: torch.Tensor,
                               perm_in: Optional[torch.Tensor] = None,
                               velocity: Optional[torch.Tensor] = None, lr: float = 0.1,
                               momentum: float = 0.0, want_grads: bool = False,
                               want_loss: bool = True) -> dict:
    """One CD-GraB training epoch of the softmax-regression model; W (and velocity)
    are updated in place.  X[m][n][in_dim], y[m][n]."""
    m, n, in_dim = X.shape
    classes = W.shape[1]
    d = (in_dim + 1) * classes
    dev = h.device
    signs = torch.empty((m, n // 2), dtype=torch.int8, device=dev)
    perm = torch.empty((m, n), dtype=torch.int32, device=dev)
    grads = torch.empty((m, n, d), dtype=torch.float32, device=dev) if want_grads else None
    loss = torch.empty((m, n), dtype=torch.float32, device=dev) if want_loss else None
    h._check(h._lib.cdgrab_train_epoch_softmax(
        h._h, m, n, in_dim, classes,
        _ptr(X, torch.float32, (m, n, in_dim), "X", dev), _ptr(y, torch.int32, (m, n), "y", dev),
        _ptr(perm_in, torch.int32, (m, n), "perm_in", dev),
        _ptr(W, torch.float32, (in_dim + 1, classes), "W", dev),
        _ptr(velocity, torch.float32, (d,), "velocity", dev), lr, momentum,
        signs.data_ptr(), perm.data_ptr(),
        grads.data_ptr() if grads is not None else None,
        loss.data_ptr() if loss is not None else None))
    return {"signs": signs, "perm": perm, "grads": grads, "loss": loss}


def cdgrab_train_softmax(h: Handle, X: torch.Tensor, y: torch.Tensor, W: torch.Tensor,
                         perm: torch.Tensor, epochs: int,
                         velocity: Optional[torch.Tensor] = None, lr: float = 0.1,
                         momentum: float = 0.0, want_loss: bool = True) -> dict:
    """`epochs` CD-GraB training epochs with the permutations carried over; W, velocity
    and perm[m][n] (first order in, next order out) are updated in place."""
    m, n, in_dim = X.shape
    classes = W.shape[1]
    d = (in_dim + 1) * classes
    dev = h.device
    signs = torch.empty((m, n // 2), dtype=torch.int8, device=dev)
    loss = torch.empty((epochs, m, n), dtype=torch.float32, device=dev) if want_loss else None
    h._check(h._lib.cdgrab_train_softmax(
        h._h, m, n, in_dim, classes,
        _ptr(X, torch.float32, (m, n, in_dim), "X", dev), _ptr(y, torch.int32, (m, n), "y", dev),
        _ptr(perm, torch.int32, (m, n), "perm", dev),
        _ptr(W, torch.float32, (in_dim + 1, classes), "W", dev),
        _ptr(velocity, torch.float32, (d,), "velocity", dev), lr, momentum, epochs,
        signs.data_ptr(), loss.data_ptr() if loss is not None else None))
    return {"signs": signs, "perm": perm, "loss": loss}


def cdgrab_balance_epoch_independent(h: Handle, grads: torch.Tensor,
                                     perm_in: Optional[torch.Tensor] = None) -> dict:
    """ID-GraB (PairBal): m independent one-worker walks over grads[m][n][d]."""
    m, n, d = grads.shape
    signs = torch.empty((m, n // 2), dtype=torch.int8, device=h.device)
    perm = torch.empty((m, n), dtype=torch.int32, device=h.device)
    h._check(h._lib.cdgrab_balance_epoch_independent(
        h._h, m, n, d, _ptr(grads, torch.float32, (m, n, d), "grads", h.device),
        _ptr(perm_in, torch.int32, (m, n), "perm_in", h.device), signs.data_ptr(), perm.data_ptr()))
    return {"signs": signs, "perm": perm}


def cdgrab_balance_epoch_stale_mean(h: Handle, grads: torch.Tensor,
                                    stale_mean: Optional[torch.Tensor] = None,
                                    perm_in: Optional[torch.Tensor] = None) -> dict:
    """Centralized GraB balancing of grads[n][d] centred by a stale mean."""
    n, d = grads.shape
    dev = h.device
    signs = torch.empty((n,), dtype=torch.int8, device=dev)
    perm = torch.empty((n,), dtype=torch.int32, device=dev)
    mean = torch.empty((d,), dtype=torch.float32, device=dev)
    r64 = torch.empty((d,), dtype=torch.float64, device=dev)
    h._check(h._lib.cdgrab_balance_epoch_stale_mean(
        h._h, n, d, _ptr(grads, torch.float32, (n, d), "grads", dev),
        _ptr(stale_mean, torch.float32, (d,), "stale_mean", dev),
        _ptr(perm_in, torch.int32, (n,), "perm_in", dev),
        signs.data_ptr(), perm.data_ptr(), mean.data_ptr(), r64.data_ptr()))
    return {"signs": signs, "perm": perm, "mean": mean, "r64": r64}


def cdgrab_balance_epoch_randomized(h: Handle, grads: torch.Tensor, uniforms: torch.Tensor,
                                    perm_in: Optional[torch.Tensor] = None) -> dict:
    """cdgrab_balance_epoch with the randomized sign rule; uniforms[m][n/2] in [0,1)."""
    m, n, d = grads.shape
    dev = h.device
    signs = torch.empty((m, n // 2), dtype=torch.int8, device=dev)
    perm = torch.empty((m, n), dtype=torch.int32, device=dev)
    r64 = torch.empty((d,), dtype=torch.float64, device=dev)
    dots = torch.empty((m, n // 2), dtype=torch.float64, device=dev)
    h._check(h._lib.cdgrab_balance_epoch_randomized(
        h._h, m, n, d, _ptr(grads, torch.float32, (m, n, d), "grads", dev),
        _ptr(uniforms, torch.float32, (m, n // 2), "uniforms", dev),
        _ptr(perm_in, torch.int32, (m, n), "perm_in", dev),
        signs.data_ptr(), perm.data_ptr(), r64.data_ptr(), dots.data_ptr()))
    return {"signs": signs, "perm": perm, "r64": r64, "dots": dots}
