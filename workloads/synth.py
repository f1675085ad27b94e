"""Python side of the counter-based streaming generator (see synth_core.h).

``SynthRows`` draws the small seeded tables with numpy (shared mean, per-row
log-normal scale, per-block log-uniform scale), keeps a host copy and -- when a
GPU is present -- a device copy, and exposes

  * ``fill_pairs_host`` / ``sample_host``: the gcc build of the generator, and
  * ``device_callback``: a (function pointer, context pointer) pair for the
    balancing library's generator argument, backed by the hipcc build.

Both builds come from the one header and produce identical bits.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
HOST_LIB = os.path.join(_HERE, "libsynth_host.so")
HIP_LIB = os.path.join(_HERE, "libsynth_hip.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build(force: bool = True) -> None:
    core = os.path.join(_HERE, "synth_core.h")
    src_c = os.path.join(_HERE, "synth_host.c")
    src_hip = os.path.join(_HERE, "synth_hip.hip")

    def stale(lib, src):
        return force or not os.path.exists(lib) or os.path.getmtime(lib) < max(
            os.path.getmtime(src), os.path.getmtime(core))

    if stale(HOST_LIB, src_c):
        subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
                        "-fno-fast-math", "-Wall", "-o", HOST_LIB, src_c, "-lm"], check=True)
    if stale(HIP_LIB, src_hip):
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
                        "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
                        "-packed-fp32-ops", "-o", HIP_LIB, src_hip], check=True)


class _Params(ctypes.Structure):
    _fields_ = [("seed", ctypes.c_uint64), ("m", ctypes.c_int64), ("n", ctypes.c_int64),
                ("d", ctypes.c_int64), ("mu", ctypes.c_void_p), ("row_scale", ctypes.c_void_p),
                ("block_scale", ctypes.c_void_p), ("block_len", ctypes.c_int64),
                ("n_block_scales", ctypes.c_int32), ("zero_threshold", ctypes.c_uint32)]


_host = None
_hip = None


def _host_lib():
    global _host
    if _host is None:
        build(force=False) if not os.path.exists(HOST_LIB) else None
        lib = ctypes.CDLL(HOST_LIB)
        lib.synth_fill_pairs_host.argtypes = [ctypes.POINTER(_Params), ctypes.c_int64, ctypes.c_int64,
                                              ctypes.c_void_p]
        lib.synth_fill_pairs_host.restype = ctypes.c_int
        lib.synth_sample_host.argtypes = [ctypes.POINTER(_Params), ctypes.c_void_p, ctypes.c_int64,
                                          ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        lib.synth_sample_host.restype = ctypes.c_int
        lib.synth_mix_host.argtypes = [ctypes.c_uint64]
        lib.synth_mix_host.restype = ctypes.c_uint64
        _host = lib
    return _host


def _hip_lib():
    global _hip
    if _hip is None:
        import torch  # noqa: F401  (the HIP runtime torch ships must be the one in the process)
        if not os.path.exists(HIP_LIB):
            raise FileNotFoundError("%s is missing: run workloads.synth.build()" % HIP_LIB)
        lib = ctypes.CDLL(HIP_LIB)
        lib.synth_fill_pairs_device.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                                ctypes.c_void_p, ctypes.c_void_p]
        lib.synth_fill_pairs_device.restype = ctypes.c_int
        lib.synth_set_drain.argtypes = [ctypes.c_void_p, ctypes.c_int64]
        lib.synth_set_drain.restype = ctypes.c_int
        lib.synth_set_streaming_stores.argtypes = [ctypes.c_int]
        lib.synth_set_streaming_stores.restype = ctypes.c_int
        _hip = lib
    return _hip


def mix(x: int) -> int:
    """The generator's 64-bit mixing function (for its statistical tests)."""
    return int(_host_lib().synth_mix_host(ctypes.c_uint64(x & (2 ** 64 - 1))))


_drain_buf = None


def set_input_drain(enabled: bool, device: str = "cuda:0", megabytes: int = 384) -> None:
    """After every device fill, read a zero-filled scratch buffer larger than the
    GPU's last-level cache (256 MB Infinity Cache + L2), so that the rows just
    written have reached HBM before the consumer starts.  The drain runs inside the
    generator's own (separately timed) work."""
    global _drain_buf
    import torch
    lib = _hip_lib()
    if enabled:
        if _drain_buf is None:
            _drain_buf = torch.zeros(megabytes * (1 << 20) // 4, dtype=torch.float32, device=device)
        lib.synth_set_drain(_drain_buf.data_ptr(), _drain_buf.numel())
    else:
        lib.synth_set_drain(None, 0)


STORE_MODES = {"plain": 0, "streaming": 1, "auto": 2}


def set_store_mode(mode: str = "auto") -> None:
    """How the device generator writes its rows: "plain" (ordinary stores), "streaming"
    (non-temporal stores) or "auto" (the default: streaming for blocks larger than the
    last-level cache, plain for blocks that fit it).  The values are the same in every
    mode; only the cache hint of the stores differs."""
    rc = _hip_lib().synth_set_streaming_stores(STORE_MODES[mode])
    if rc != 0:
        raise ValueError("bad store mode %r" % mode)


class SynthRows:
    """Rows g[worker][position][element] of one streaming workload."""

    def __init__(self, seed: int, m: int, n: int, d: int, block_scales: int = 0,
                 zero_fraction: float = 0.0, mean_scale: float = 0.1, row_sigma: float = 0.5):
        self.seed, self.m, self.n, self.d = seed, m, n, d
        rng = np.random.default_rng(seed)
        self.mu = (mean_scale * rng.standard_normal(d)).astype(np.float32)
        self.row_scale = np.exp(row_sigma * rng.standard_normal(m * n)).astype(np.float32)
        self.n_block_scales = int(block_scales)
        if block_scales:
            # log-uniform over [1e-3, 1]
            self.block_scale = (10.0 ** rng.uniform(-3.0, 0.0, block_scales)).astype(np.float32)
            self.block_len = -(-d // block_scales)
        else:
            self.block_scale = None
            self.block_len = d
        self.zero_threshold = int(round(zero_fraction * 65536))
        self._host_params = _Params(
            seed, m, n, d, self.mu.ctypes.data, self.row_scale.ctypes.data,
            self.block_scale.ctypes.data if block_scales else None, self.block_len,
            self.n_block_scales, self.zero_threshold)
        self._dev = None

    # ---- host build -----------------------------------------------------
    def fill_pairs_host(self, first_pair: int, count: int) -> np.ndarray:
        out = np.empty((count, 2, self.d), np.float32)
        rc = _host_lib().synth_fill_pairs_host(ctypes.byref(self._host_params), first_pair, count,
                                               out.ctypes.data)
        if rc != 0:
            raise ValueError("synth_fill_pairs_host failed")
        return out

    def sample_host(self, row_ids, elems) -> np.ndarray:
        row_ids = np.ascontiguousarray(row_ids, np.int64)
        elems = np.ascontiguousarray(elems, np.int64)
        out = np.empty((row_ids.size, elems.size), np.float32)
        rc = _host_lib().synth_sample_host(ctypes.byref(self._host_params), row_ids.ctypes.data,
                                           row_ids.size, elems.ctypes.data, elems.size, out.ctypes.data)
        if rc != 0:
            raise ValueError("synth_sample_host: index out of range")
        return out

    def dense_host(self) -> np.ndarray:
        """All rows as z[m][n][d] (small shapes only)."""
        pairs = self.fill_pairs_host(0, self.m * self.n // 2)          # [k*m+i][2][d]
        z = pairs.reshape(self.n // 2, self.m, 2, self.d).transpose(1, 0, 2, 3)
        return np.ascontiguousarray(z.reshape(self.m, self.n, self.d))

    # ---- device build ---------------------------------------------------
    def device_callback(self, device: str = "cuda:0"):
        """(function pointer, context pointer) for cdgrab_balance_epoch's generator."""
        import torch
        lib = _hip_lib()
        if self._dev is None:
            mu = torch.from_numpy(self.mu).to(device)
            rs = torch.from_numpy(self.row_scale).to(device)
            bs = torch.from_numpy(self.block_scale).to(device) if self.n_block_scales else None
            params = _Params(self.seed, self.m, self.n, self.d, mu.data_ptr(), rs.data_ptr(),
                             bs.data_ptr() if bs is not None else None, self.block_len,
                             self.n_block_scales, self.zero_threshold)
            self._dev = (mu, rs, bs, params)
        params = self._dev[3]
        return lib.synth_fill_pairs_device, ctypes.addressof(params)

    def fill_pairs_device(self, first_pair: int, count: int, device: str = "cuda:0"):
        """A staging block [count][2][d] generated on the GPU (torch tensor)."""
        import torch
        fn, ctx = self.device_callback(device)
        out = torch.empty((count, 2, self.d), dtype=torch.float32, device=device)
        rc = fn(ctx, first_pair, count, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise RuntimeError("synth_fill_pairs_device failed with %d" % rc)
        return out


def from_workload(w, seed: int, n: int | None = None, d: int | None = None) -> SynthRows:
    """SynthRows for one of workloads.CONFIGS (optionally with n or d reduced)."""
    return SynthRows(seed, w.m, n if n is not None else w.n, d if d is not None else w.d,
                     block_scales=w.block_scales, zero_fraction=w.zero_fraction)
