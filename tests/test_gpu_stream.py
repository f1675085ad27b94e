"""GPU tests of the streamed (generator-fed) form of cdgrab_balance_epoch, at
reduced and at full d, against the CPU oracle fed the same bytes."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from workloads import synth
from parity import check_epoch, rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2302_00845_amd as p
    return p


def dense_from_device(rows_src, pairs):
    """z[m][n][d] (numpy) from the GPU generator's staging layout, block by block."""
    m, n, d = rows_src.m, rows_src.n, rows_src.d
    blk = rows_src.fill_pairs_device(0, pairs)
    torch.cuda.synchronize()
    rows = blk.cpu().numpy()                               # [k*m+i][2][d]
    return np.ascontiguousarray(
        rows.reshape(n // 2, m, 2, d).transpose(1, 0, 2, 3).reshape(m, n, d))


@pytest.mark.parametrize("kw", [dict(), dict(block_scales=64), dict(zero_fraction=0.2),
                                dict(block_scales=64, zero_fraction=0.2)])
@pytest.mark.parametrize("d", [4096, 1001, 70_003])
def test_device_generator_is_bit_identical_to_host(kw, d):
    g = synth.SynthRows(11, 3, 6, d, **kw)
    dev = g.fill_pairs_device(2, 5).cpu().numpy()
    host = g.fill_pairs_host(2, 5)
    assert np.array_equal(dev.view(np.uint32), host.view(np.uint32))


def test_device_generator_large_d_samples():
    w = workloads.CONFIGS["c4_resnet18"]
    g = synth.from_workload(w, 5, n=4)
    blk = g.fill_pairs_device(32, 2)                       # pairs 32,33: worker 0,1, pair 1
    elems = np.array([0, 1, 174_999, 175_000, 5_600_001, 11_199_999], np.int64)
    got = blk.cpu().numpy()[:, :, elems]
    rows = np.array([0 * 4 + 2, 0 * 4 + 3, 1 * 4 + 2, 1 * 4 + 3], np.int64)
    want = g.sample_host(rows, elems).reshape(2, 2, -1)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("name,n,bb", [("c3_stream_1m", 8, 0), ("c3_stream_1m", 6, 16)])
def test_streamed_epoch_reduced_n(lib, name, n, bb):
    w = workloads.CONFIGS[name]
    g = synth.from_workload(w, 21, n=n)
    fn, ctx = g.device_callback()
    h = lib.Handle(block_pairs=bb)
    perm_in = workloads.random_perms(3, w.m, n)
    out = lib.cdgrab_balance_epoch(h, w.m, n, w.d, gen=fn, gen_ctx=ctx,
                                   perm_in=torch.from_numpy(perm_in).cuda(), want_r64=True, want_dots=True)
    torch.cuda.synchronize()
    got = {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}
    z = dense_from_device(g, w.m * n // 2)
    rep = check_epoch(z, got, perm_in)
    # streamed and dense input give the same bits
    h2 = lib.Handle(block_pairs=bb)
    out2 = lib.cdgrab_balance_epoch(h2, w.m, n, w.d, grads=torch.from_numpy(z).cuda(),
                                    perm_in=torch.from_numpy(perm_in).cuda(), want_r64=True)
    torch.cuda.synchronize()
    assert torch.equal(out2["signs"], out["signs"]) and torch.equal(out2["r64"], out["r64"])
    assert torch.equal(out2["perm"], out["perm"])
    print(rep)


def test_generator_error_is_reported(lib):
    import ctypes
    from paper_2302_00845_amd.cdgrab import GEN_FN

    @GEN_FN
    def failing(ctx, first, count, staging, stream):
        return 7

    h = lib.Handle()
    with pytest.raises(lib.CdgrabError) as ei:
        lib.cdgrab_balance_epoch(h, 2, 4, 64, gen=failing, gen_ctx=None)
    assert ei.value.code == -4
