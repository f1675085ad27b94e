"""Bandwidth probes for bench.py (see hbm_probe.hip): kernels of known HBM traffic.

Not part of the method and not part of the balancing library; they give the
practical read ceiling of the device and a copy of known size for scaling
rocprofv3's traffic counters.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(_HERE, "libhbm_probe.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

_lib = None


def build(force: bool = True) -> None:
    src = os.path.join(_HERE, "hbm_probe.hip")
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(src):
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
                        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", LIB, src],
                       check=True)


def _load():
    global _lib
    if _lib is None:
        import torch  # noqa: F401  (the HIP runtime torch ships must be the one in the process)
        if not os.path.exists(LIB):
            raise FileNotFoundError("%s is missing: run workloads.hbm_probe.build()" % LIB)
        lib = ctypes.CDLL(LIB)
        lib.hbm_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p,
                                       ctypes.POINTER(ctypes.c_double)]
        lib.hbm_probe_read.restype = ctypes.c_int
        lib.hbm_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int,
                                       ctypes.c_void_p, ctypes.POINTER(ctypes.c_double)]
        lib.hbm_probe_copy.restype = ctypes.c_int
        _lib = lib
    return _lib


def read_bandwidth(nbytes: int = 2 << 30, reps: int = 5, device: str = "cuda:0") -> float:
    """GB/s of a plain streaming read over a zero-filled scratch buffer of nbytes."""
    import torch
    buf = torch.zeros(nbytes // 4, dtype=torch.float32, device=device)
    out = ctypes.c_double()
    rc = _load().hbm_probe_read(buf.data_ptr(), buf.numel() * 4, reps,
                                torch.cuda.current_stream().cuda_stream, ctypes.byref(out))
    if rc != 0:
        raise RuntimeError("hbm_probe_read failed with %d" % rc)
    del buf
    return out.value


def copy_bandwidth(nbytes: int = 1 << 30, reps: int = 3, device: str = "cuda:0") -> float:
    """GB/s (read + written) of a plain device copy of nbytes; its HBM traffic is 2 * nbytes
    per launch, which is what the traffic counters of a profiled run are scaled against."""
    import torch
    src = torch.ones(nbytes // 4, dtype=torch.float32, device=device)
    dst = torch.empty_like(src)
    out = ctypes.c_double()
    rc = _load().hbm_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel() * 4, reps,
                                torch.cuda.current_stream().cuda_stream, ctypes.byref(out))
    if rc != 0:
        raise RuntimeError("hbm_probe_copy failed with %d" % rc)
    del src, dst
    return out.value
