"""CPU oracle for the CD-GraB pair-balancing path -- TEST INFRASTRUCTURE ONLY.

A ctypes wrapper around ``cdgrab_oracle.c`` (plain C, double precision, written
from the paper's algorithm statements).  Only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package.  It shares nothing with
the HIP library and never imports it.

Each wrapper keeps the name of the C function it calls; see the C file's header
for which passage of the paper each one follows and which readings were taken.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cdgrab_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    lib = ctypes.CDLL(_LIB)
    i64, dbl = ctypes.c_int64, ctypes.c_double
    P = ctypes.c_void_p
    lib.oracle_greedy_balance.argtypes = [i64, P, P, P, P, P]
    lib.oracle_greedy_balance.restype = ctypes.c_int
    lib.oracle_pair_balance.argtypes = [i64, P, P, P, P, ctypes.c_int, P, P, P]
    lib.oracle_pair_balance.restype = ctypes.c_int
    lib.oracle_server_epoch.argtypes = [i64, i64, i64, P, P, P, P, P, P, P, P]
    lib.oracle_server_epoch.restype = ctypes.c_int
    lib.oracle_stream_pairs.argtypes = [i64, P, i64, P, P, P, P, P, P]
    lib.oracle_stream_pairs.restype = ctypes.c_int
    lib.oracle_reorder.argtypes = [i64, P, P, P]
    lib.oracle_reorder.restype = ctypes.c_int
    lib.oracle_softmax_pergrad.argtypes = [i64, i64, i64, P, P, P, P]
    lib.oracle_softmax_pergrad.restype = ctypes.c_int
    lib.oracle_softmax_loss.argtypes = [i64, i64, P, ctypes.c_int32, P]
    lib.oracle_softmax_loss.restype = dbl
    lib.oracle_parallel_herding.argtypes = [i64, i64, i64, P, P]
    lib.oracle_parallel_herding.restype = dbl
    lib.oracle_train_epoch_softmax.argtypes = [i64, i64, i64, i64, P, P, P, P, P, dbl, dbl, P, P]
    lib.oracle_train_epoch_softmax.restype = ctypes.c_int
    lib.oracle_randomized_epoch.argtypes = [i64, i64, i64, P, P, P, P, P, P, P]
    lib.oracle_randomized_epoch.restype = ctypes.c_int
    lib.oracle_grab_stale_mean.argtypes = [i64, i64, P, P, P, P, P, P, P, P, P, P]
    lib.oracle_grab_stale_mean.restype = ctypes.c_int
    _lib = lib
    return lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def greedy_balance(r: np.ndarray, c: np.ndarray):
    """One greedy step on double vectors; updates ``r`` in place.

    Returns (s, t, ||r||_before, ||c||) with s the sign given to c.
    """
    assert r.dtype == np.float64 and r.flags.c_contiguous
    c = _c(c, np.float64)
    t, nr, nc = (ctypes.c_double() for _ in range(3))
    s = _load().oracle_greedy_balance(r.size, _p(r), _p(c), ctypes.byref(t),
                                      ctypes.byref(nr), ctypes.byref(nc))
    return s, t.value, nr.value, nc.value


def server_epoch(z: np.ndarray, perm_in: np.ndarray | None = None):
    """One epoch over z[m][n][d] (fp32).  Returns a dict with
    eps [m][n/2] int8, r [d] float64, perm [m][n] int32,
    t, norm_r, norm_c [m][n/2] float64 (t = <r, z2 - z1> when the pair was decided).
    """
    z = _c(z, np.float32)
    m, n, d = z.shape
    if perm_in is not None:
        perm_in = _c(perm_in, np.int32)
        assert perm_in.shape == (m, n)
    eps = np.zeros((m, n // 2), np.int8)
    r = np.zeros(d, np.float64)
    perm = np.zeros((m, n), np.int32)
    t = np.zeros((m, n // 2), np.float64)
    nr = np.zeros_like(t)
    nc = np.zeros_like(t)
    rc = _load().oracle_server_epoch(m, n, d, _p(z), _p(perm_in), _p(eps), _p(r),
                                     _p(perm), _p(t), _p(nr), _p(nc))
    if rc != 0:
        raise ValueError("oracle_server_epoch rejected the sizes m=%d n=%d d=%d" % (m, n, d))
    return {"eps": eps, "r": r, "perm": perm, "t": t, "norm_r": nr, "norm_c": nc}


def stream_pairs(r: np.ndarray, rows: np.ndarray, eps_in: np.ndarray | None = None):
    """Advance running sum ``r`` (float64, in place) over rows[count][2][d] (fp32).

    With ``eps_in`` the given exported signs are imposed (replay).  Returns
    (eps, t, norm_r, norm_c) per pair.
    """
    assert r.dtype == np.float64 and r.flags.c_contiguous
    rows = _c(rows, np.float32)
    count, two, d = rows.shape
    assert two == 2 and d == r.size
    if eps_in is not None:
        eps_in = _c(eps_in, np.int8)
        assert eps_in.shape == (count,)
    eps = np.zeros(count, np.int8)
    t = np.zeros(count, np.float64)
    nr = np.zeros(count, np.float64)
    nc = np.zeros(count, np.float64)
    rc = _load().oracle_stream_pairs(d, _p(r), count, _p(rows), _p(eps_in), _p(eps),
                                     _p(t), _p(nr), _p(nc))
    if rc != 0:
        raise ValueError("oracle_stream_pairs failed")
    return eps, t, nr, nc


def reorder(signs: np.ndarray, perm_in: np.ndarray | None = None) -> np.ndarray:
    """Alg. "Reordering Vectors based on Balanced Signs" for one worker."""
    signs = _c(signs, np.int8)
    n = signs.size
    if perm_in is not None:
        perm_in = _c(perm_in, np.int32)
        assert perm_in.shape == (n,)
    out = np.zeros(n, np.int32)
    rc = _load().oracle_reorder(n, _p(signs), _p(perm_in), _p(out))
    if rc != 0:
        raise ValueError("oracle_reorder: signs must be +1 or -1")
    return out


def softmax_pergrad(X: np.ndarray, y: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Per-example softmax cross-entropy gradients, [N][(in_dim+1)*classes] fp32."""
    X = _c(X, np.float32)
    y = _c(y, np.int32)
    W = _c(W, np.float32)
    N, in_dim = X.shape
    assert W.shape[0] == in_dim + 1
    classes = W.shape[1]
    G = np.zeros((N, (in_dim + 1) * classes), np.float32)
    rc = _load().oracle_softmax_pergrad(N, in_dim, classes, _p(X), _p(y), _p(W), _p(G))
    if rc != 0:
        raise ValueError("oracle_softmax_pergrad failed (label out of range?)")
    return G


def softmax_loss(x: np.ndarray, y: int, W64: np.ndarray) -> float:
    """Cross-entropy loss of one example with double weights W64[(in_dim+1)][classes]."""
    x = _c(x, np.float32)
    W64 = _c(W64, np.float64)
    in_dim = x.size
    assert W64.shape[0] == in_dim + 1
    return _load().oracle_softmax_loss(in_dim, W64.shape[1], _p(x), int(y), _p(W64))


def parallel_herding(z: np.ndarray, perm: np.ndarray | None = None) -> float:
    """Parallel herding objective of z[m][n][d] visited in order perm[m][n]."""
    z = _c(z, np.float32)
    m, n, d = z.shape
    if perm is not None:
        perm = _c(perm, np.int32)
        assert perm.shape == (m, n)
    return _load().oracle_parallel_herding(m, n, d, _p(z), _p(perm))


def train_epoch_softmax(X: np.ndarray, y: np.ndarray, perm_in: np.ndarray | None, W: np.ndarray,
                        v: np.ndarray | None, lr: float, momentum: float):
    """One training epoch of m simulated workers (see the C function).  X[m][n][in_dim],
    y[m][n]; W, v double arrays, not modified.  Returns dict W, v (double), rows
    [m][n][d] fp32, loss [m][n], and the balancing of those rows (eps, perm, r)."""
    X = _c(X, np.float32)
    y = _c(y, np.int32)
    m, n, in_dim = X.shape
    W = np.array(W, dtype=np.float64, order="C").copy()
    classes = W.shape[1]
    v = np.zeros(W.size) if v is None else np.array(v, dtype=np.float64).reshape(-1).copy()
    if perm_in is not None:
        perm_in = _c(perm_in, np.int32)
    rows = np.zeros((m, n, W.size), np.float32)
    loss = np.zeros((m, n), np.float64)
    rc = _load().oracle_train_epoch_softmax(m, n, in_dim, classes, _p(X), _p(y), _p(perm_in), _p(W),
                                            _p(v), float(lr), float(momentum), _p(rows), _p(loss))
    if rc != 0:
        raise ValueError("oracle_train_epoch_softmax failed")
    bal = server_epoch(rows, perm_in)
    return {"W": W, "v": v, "rows": rows, "loss": loss, "eps": bal["eps"], "perm": bal["perm"], "r": bal["r"]}


def grab_stale_mean(g: np.ndarray, stale_mean: np.ndarray | None = None, perm_in: np.ndarray | None = None):
    """Centralized GraB balancing of g[n][d] centred by stale_mean.  Returns dict with
    s [n] int8, r [d], perm [n], mean [d], t, norm_r, norm_z [n]."""
    g = _c(g, np.float32)
    n, d = g.shape
    if stale_mean is not None:
        stale_mean = _c(stale_mean, np.float32)
    if perm_in is not None:
        perm_in = _c(perm_in, np.int32)
    s = np.zeros(n, np.int8)
    r = np.zeros(d)
    perm = np.zeros(n, np.int32)
    mean = np.zeros(d)
    t, nr, nz = np.zeros(n), np.zeros(n), np.zeros(n)
    rc = _load().oracle_grab_stale_mean(n, d, _p(g), _p(stale_mean), _p(perm_in), _p(s), _p(r), _p(perm),
                                        _p(mean), _p(t), _p(nr), _p(nz))
    if rc != 0:
        raise ValueError("oracle_grab_stale_mean failed")
    return {"s": s, "r": r, "perm": perm, "mean": mean, "t": t, "norm_r": nr, "norm_z": nz}


def randomized_epoch(z: np.ndarray, u: np.ndarray, perm_in: np.ndarray | None = None):
    """Server walk with the RandomizedBalance subroutine and the given uniform draws
    u[m][n/2].  Returns dict eps, r, perm, t (t = <r, z2 - z1> at decision time)."""
    z = _c(z, np.float32)
    u = _c(u, np.float32)
    m, n, d = z.shape
    assert u.shape == (m, n // 2)
    if perm_in is not None:
        perm_in = _c(perm_in, np.int32)
    eps = np.zeros((m, n // 2), np.int8)
    r = np.zeros(d)
    perm = np.zeros((m, n), np.int32)
    t = np.zeros((m, n // 2))
    rc = _load().oracle_randomized_epoch(m, n, d, _p(z), _p(u), _p(perm_in), _p(eps), _p(r), _p(perm), _p(t))
    if rc != 0:
        raise ValueError("oracle_randomized_epoch failed")
    return {"eps": eps, "r": r, "perm": perm, "t": t}
