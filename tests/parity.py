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


def replay_pairs(rows, eps_flat, r=None):
    """The oracle's walk over rows[P][2][d] with the given exported signs imposed.
    Returns (r, t, norm_r, norm_c): the running sum after the walk and, per pair, the
    inner product the oracle saw when that pair was decided and the two norms.  Before
    the first pair where the imposed sign is not the oracle's own choice this IS the
    oracle's free run; after it, it is the walk every later decision is judged against."""
    rows = np.ascontiguousarray(rows, np.float32)
    if r is None:
        r = np.zeros(rows.shape[2])
    _, t, nr, nc = oracle.stream_pairs(r, rows, eps_in=np.ascontiguousarray(eps_flat, np.int8))
    return r, t, nr, nc


def judge_greedy(t, nr, nc, eps_flat):
    """Greedy rule on a replayed walk: every imposed sign must be the rule's choice
    (+1 iff t <= 0) or lie inside the margin.  Returns the number of in-margin flips."""
    want = np.where(t <= 0, 1, -1)
    bad = want != eps_flat
    outside = bad & (np.abs(t) > SIGN_MARGIN * nr * nc)
    assert not outside.any(), (
        "sign differs outside the margin at flattened pairs %s" % np.nonzero(outside)[0][:8])
    return int(bad.sum())


class GeneratedWalk:
    """Walks the oracle over rows the GPU generator produces, block by block: the rows of
    the next chunk are generated on the GPU and copied to pinned host memory while the
    oracle (one CPU thread) works on the current one.  The HIP path's signs are imposed
    (replay), so the walk is the oracle's free run up to the first in-margin difference
    and the reference for everything after it."""

    def __init__(self, gen, chunk_pairs, device="cuda:0"):
        import torch
        self.torch = torch
        self.gen = gen
        self.chunk = int(chunk_pairs)
        self.device = device
        n = self.chunk * 2 * gen.d
        self.dev_buf = [torch.empty(n, dtype=torch.float32, device=device) for _ in range(2)]
        self.pin_buf = [torch.empty(n, dtype=torch.float32, pin_memory=True) for _ in range(2)]
        self.events = [torch.cuda.Event() for _ in range(2)]
        self.fn, self.ctx = gen.device_callback(device)

    def _issue(self, slot, first, cnt):
        torch = self.torch
        rc = self.fn(self.ctx, first, cnt, self.dev_buf[slot].data_ptr(),
                     torch.cuda.current_stream().cuda_stream)
        assert rc == 0, "generator failed with %d" % rc
        k = cnt * 2 * self.gen.d
        self.pin_buf[slot][:k].copy_(self.dev_buf[slot][:k], non_blocking=True)
        self.events[slot].record()

    def run(self, first_pair, count, eps_flat, r=None):
        """Replays flattened pairs first_pair .. first_pair+count-1 with signs eps_flat[count].
        Returns (r, t, norm_r, norm_c)."""
        d = self.gen.d
        if r is None:
            r = np.zeros(d)
        t_all, nr_all, nc_all = [], [], []
        starts = list(range(first_pair, first_pair + count, self.chunk))
        if starts:
            self._issue(0, starts[0], min(self.chunk, first_pair + count - starts[0]))
        for q, first in enumerate(starts):
            cnt = min(self.chunk, first_pair + count - first)
            slot = q & 1
            if q + 1 < len(starts):
                nxt = starts[q + 1]
                self._issue(slot ^ 1, nxt, min(self.chunk, first_pair + count - nxt))
            self.events[slot].synchronize()
            rows = self.pin_buf[slot][:cnt * 2 * d].numpy().reshape(cnt, 2, d)
            off = first - first_pair
            _, t, nr, nc = oracle.stream_pairs(r, rows, eps_in=eps_flat[off:off + cnt])
            t_all.append(t); nr_all.append(nr); nc_all.append(nc)
        return r, np.concatenate(t_all), np.concatenate(nr_all), np.concatenate(nc_all)
