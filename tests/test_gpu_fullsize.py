"""Full-size checks in the launch configuration the benchmark times.

The oracle cannot walk a whole ResNet-18- or GPT-2-sized epoch in test time, so
at full d it (a) walks a prefix of the epoch that spans more than one block and a
ragged tail, fed the same bytes, and (b) checks properties of the whole epoch
that hold at any size: the running sum at sampled coordinates equals the signed
sum of the differences regenerated element by element on the host, every
permutation is the exact function of the signs, and the recorded dots agree in
sign with the decisions.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from workloads import synth
from parity import check_epoch, expected_perm_from_signs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2302_00845_amd as p
    return p


def _prefix_parity(lib, name, n, bb):
    w = workloads.CONFIGS[name]
    g = synth.from_workload(w, 31, n=n)
    fn, ctx = g.device_callback()
    h = lib.Handle(block_pairs=bb)
    out = lib.cdgrab_balance_epoch(h, w.m, n, w.d, gen=fn, gen_ctx=ctx, want_r64=True, want_dots=True)
    torch.cuda.synchronize()
    got = {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}
    pairs = w.m * n // 2
    # oracle walks the same bytes, one staging block at a time
    r = np.zeros(w.d)
    eps_o, t_o, nr_o, nc_o = [], [], [], []
    step = 16
    for first in range(0, pairs, step):
        cnt = min(step, pairs - first)
        rows = g.fill_pairs_device(first, cnt).cpu().numpy()
        gpu_eps = np.ascontiguousarray(got["signs"].T).reshape(-1)[first:first + cnt]
        e, t, nr, nc = oracle.stream_pairs(r, rows, eps_in=gpu_eps)     # replay the HIP path's signs
        eps_o.append(e); t_o.append(t); nr_o.append(nr); nc_o.append(nc)
        del rows
    t = np.concatenate(t_o); nr = np.concatenate(nr_o); nc = np.concatenate(nc_o)
    gpu_eps = np.ascontiguousarray(got["signs"].T).reshape(-1)
    bad = (np.where(t <= 0, 1, -1) != gpu_eps) & (np.abs(t) > 1e-9 * nr * nc)
    assert not bad.any(), "sign outside the margin at pairs %s" % np.nonzero(bad)[0]
    err = np.linalg.norm(got["r64"] - r) / np.linalg.norm(r)
    assert err <= 1e-12, err
    np.testing.assert_allclose(np.ascontiguousarray(got["dots"].T).reshape(-1), t,
                               rtol=0, atol=1e-9 * float(np.max(nr * nc)))
    assert np.array_equal(expected_perm_from_signs(got["signs"]), got["perm"])
    return int((np.where(t <= 0, 1, -1) != gpu_eps).sum())


def test_c4_full_d_prefix_two_blocks_and_tail(lib):
    # m=32, d=11.2M, n=6 -> 96 pairs = three full blocks of 32 ... use Bb=32 with n=5? n must be even:
    # n=4 -> 64 pairs (2 blocks); with Bb=16 the same epoch is 4 blocks.
    flips = _prefix_parity(lib, "c4_resnet18", 4, 32)
    print("in-margin flips:", flips)


def test_c5_full_d_block_and_ragged_tail(lib):
    # m=8, d=124M, n=6 -> 24 pairs: one block of 16 and a tail of 8 at Bb=16
    flips = _prefix_parity(lib, "c5_gpt2s", 6, 16)
    print("in-margin flips:", flips)


@pytest.mark.parametrize("name", ["c3_stream_1m", "c4_resnet18", "c5_gpt2s"])
def test_whole_epoch_properties(lib, name):
    """The benchmark's configuration (full n, full d, default launch plan) of each
    streamed workload: properties that hold at any size, and the running sum at
    sampled coordinates against rows regenerated element by element on the host."""
    w = workloads.CONFIGS[name]
    g = synth.from_workload(w, 2302)
    fn, ctx = g.device_callback()
    h = lib.Handle(timing=1)
    perm_in = workloads.random_perms(2302, w.m, w.n)
    out = lib.cdgrab_balance_epoch(h, w.m, w.n, w.d, gen=fn, gen_ctx=ctx,
                                   perm_in=torch.from_numpy(perm_in).cuda(), want_r64=True, want_dots=True)
    torch.cuda.synchronize()
    signs = out["signs"].cpu().numpy()
    dots = out["dots"].cpu().numpy()
    assert np.all(np.abs(signs) == 1)
    assert np.array_equal(signs, np.where(dots <= 0, 1, -1))
    assert signs[0, 0] == 1 and dots[0, 0] == 0.0          # first pair: r = 0 -> tie -> +1
    assert np.array_equal(expected_perm_from_signs(signs, perm_in), out["perm"].cpu().numpy())
    # running sum at sampled coordinates = signed sum of regenerated differences
    rng = np.random.default_rng(0)
    blk = g.block_len
    elems = np.unique(np.concatenate([[0, 1, w.d - 1, blk - 1, min(blk, w.d - 1)],
                                      rng.integers(0, w.d, 59)])).astype(np.int64)
    all_rows = np.arange(w.m * w.n, dtype=np.int64)
    vals = g.sample_host(all_rows, elems).astype(np.float64).reshape(w.m, w.n, -1)
    diffs = vals[:, 1::2] - vals[:, 0::2]                  # [m][n/2][elems]
    want = (signs[:, :, None].astype(np.float64) * diffs).sum((0, 1))
    got = out["r64"].cpu().numpy()[elems]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12 * np.abs(diffs).sum((0, 1)).max())
    # the balanced sum stays far below a random-sign walk's worst case
    assert np.abs(got).max() < 50 * np.sqrt(w.m * w.n / 2) * np.abs(diffs).std()
    r32 = out["r32"].cpu().numpy()[elems]
    np.testing.assert_allclose(r32, want, rtol=1e-6, atol=1e-6 * np.abs(want).max())
    print(name, h.timing())
