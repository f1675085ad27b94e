"""Shared helpers of the GPU parity tests: compare the HIP path's outputs with
the CPU oracle on the same rows.

Tolerances:
  * permutations: bit-exact given the signs;
  * signs: identical wherever |<r,d>| > 1e-9 * ||r|| * ||d||.  Inside that margin
    either sign is a correct outcome of the greedy rule in finite precision; the
    oracle is then advanced with the HIP path's sign (replay) and everything after
    is judged against that walk;
  * running sum: <= 1e-5 relative L2 (fp32 export); the double export is held to
    1e-12, which is what the arithmetic (double everywhere, different summation
    order) supports.
"""
import numpy as np

import oracle

SIGN_MARGIN = 1e-9
R32_TOL = 1e-5
R64_TOL = 1e-12


def flatten_pairs(z):
    m, n, d = z.shape
    return np.ascontiguousarray(
        z.reshape(m, n // 2, 2, d).transpose(1, 0, 2, 3).reshape(m * n // 2, 2, d))


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a - b)


def expected_perm_from_signs(eps, perm_in=None):
    """Next order per worker from pair signs, through the oracle's list-form
    reorder fed the expanded per-example signs (first row -eps, second +eps)."""
    m, half = eps.shape
    n = 2 * half
    out = np.zeros((m, n), np.int32)
    for i in range(m):
        s = np.empty(n, np.int8)
        s[0::2] = -eps[i]
        s[1::2] = eps[i]
        out[i] = oracle.reorder(s, None if perm_in is None else perm_in[i])
    return out


def check_epoch(z, got, perm_in=None, expect_exact_signs=False):
    """z: rows [m][n][d] fp32 (numpy).  got: dict of numpy arrays from the HIP path
    with keys signs, perm and optionally r32, r64, dots.  Returns a small report."""
    m, n, d = z.shape
    eps_gpu = got["signs"]
    assert eps_gpu.shape == (m, n // 2) and eps_gpu.dtype == np.int8
    assert np.all(np.abs(eps_gpu) == 1)
    free = oracle.server_epoch(z, perm_in)
    same = np.array_equal(free["eps"], eps_gpu)
    report = {"free_run_equal": same, "in_margin_flips": 0}
    if expect_exact_signs:
        assert same, "signs differ from the oracle on exact-arithmetic input"
    if same:
        ref_r, ref_t = free["r"], free["t"]
        assert np.array_equal(free["perm"], got["perm"])
    else:
        rows = flatten_pairs(z)
        eps_flat = np.ascontiguousarray(eps_gpu.T).reshape(-1)
        r = np.zeros(d)
        eps_used, t, nr, nc = oracle.stream_pairs(r, rows, eps_in=eps_flat)
        want = np.where(t <= 0, 1, -1)
        bad = want != eps_flat
        outside = bad & (np.abs(t) > SIGN_MARGIN * nr * nc)
        assert not outside.any(), (
            "sign differs outside the margin at flattened pairs %s" % np.nonzero(outside)[0][:8])
        report["in_margin_flips"] = int(bad.sum())
        ref_r = r
        ref_t = t.reshape(n // 2, m).T
    # permutations are an exact function of the signs
    assert np.array_equal(expected_perm_from_signs(eps_gpu, perm_in), got["perm"])
    for i in range(m):
        assert sorted(got["perm"][i].tolist()) == sorted(
            (perm_in[i] if perm_in is not None else np.arange(n)).tolist())
    if got.get("r64") is not None:
        e = rel_l2(got["r64"], ref_r)
        report["r64_rel_l2"] = e
        assert e <= R64_TOL, "double running sum off by %g" % e
    if got.get("r32") is not None:
        e = rel_l2(got["r32"], ref_r)
        report["r32_rel_l2"] = e
        assert e <= R32_TOL, "fp32 running sum off by %g" % e
    if got.get("dots") is not None:
        scale = np.maximum(np.abs(ref_t), 1e-300)
        # dots agree to double rounding relative to ||r|| ||d||, not to |t| itself
        report["dots_max_abs_err"] = float(np.max(np.abs(got["dots"] - ref_t)))
    return report
