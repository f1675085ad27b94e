"""The entry point that allocates nothing (cdgrab_balance_epoch_static) against the
ordinary one: two calls in a row through the C ABI, the second on a smaller input, on the
library's static workspace, which keeps the first call's contents."""
import numpy as np
import pytest
import torch

import workloads
from parity import check_epoch

pytestmark = pytest.mark.gpu


def _outputs(m, n, d, dev):
    return {"signs": torch.empty((m, n // 2), dtype=torch.int8, device=dev),
            "perm": torch.empty((m, n), dtype=torch.int32, device=dev),
            "r32": torch.empty((d,), dtype=torch.float32, device=dev),
            "r64": torch.empty((d,), dtype=torch.float64, device=dev),
            "dots": torch.empty((m, n // 2), dtype=torch.float64, device=dev)}


def _np(out):
    return {k: v.cpu().numpy() for k, v in out.items() if v is not None}


def test_static_workspace_matches_ordinary_entry_point_twice():
    import paper_2302_00845_amd as pkg
    dev = torch.device("cuda", 0)
    # the ordinary entry point in the launch form the static one uses
    # (per-block Gram, at most 128 workgroups in the dot/Gram pass): bit-identical outputs
    ref_h = pkg.Handle(gram_mode=1, pass1_groups=128)
    h = pkg.Handle()
    shapes = [(8, 96, 20_000, 3), (3, 10, 1001, 4)]   # the second is smaller, odd d, one short block
    for m, n, d, seed in shapes:
        z = workloads.heavy_rows(seed, m, n, d)
        zd = torch.from_numpy(z).to(dev)
        perm_in = torch.from_numpy(workloads.random_perms(seed, m, n)).to(dev)
        ref = pkg.cdgrab_balance_epoch(ref_h, m, n, d, grads=zd, perm_in=perm_in, want_r64=True, want_dots=True)
        out = _outputs(m, n, d, dev)
        for t in out.values():
            t.fill_(77)                                   # every output must be overwritten
        before = torch.cuda.memory_allocated()
        pkg.cdgrab_balance_epoch_static(h, zd, out, perm_in=perm_in)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        got, want = _np(out), _np(ref)
        assert np.array_equal(got["signs"], want["signs"])
        assert np.array_equal(got["perm"], want["perm"])
        assert np.array_equal(got["r64"], want["r64"])
        assert np.array_equal(got["r32"], want["r32"])
        assert np.array_equal(got["dots"], want["dots"])
        # and against the oracle, to the bar of every other epoch test
        check_epoch(z, got, perm_in.cpu().numpy())
    # exact-arithmetic rows: identical to the ordinary entry point's default plan too, ties included
    z = workloads.integer_rows(5, 4, 40, 777)
    zd = torch.from_numpy(z).to(dev)
    out = _outputs(4, 40, 777, dev)
    pkg.cdgrab_balance_epoch_static(h, zd, out)
    ref = pkg.cdgrab_balance_epoch(pkg.Handle(), 4, 40, 777, grads=zd, want_r64=True, want_dots=True)
    torch.cuda.synchronize()
    for k in ("signs", "perm", "r64", "dots"):
        assert np.array_equal(out[k].cpu().numpy(), ref[k].cpu().numpy()), k
    check_epoch(z, _np(out), expect_exact_signs=True)


def test_static_workspace_rejects_long_rows_and_generators():
    import paper_2302_00845_amd as pkg
    dev = torch.device("cuda", 0)
    h = pkg.Handle()
    d = 131072 + 4
    zd = torch.zeros((1, 2, d), dtype=torch.float32, device=dev)
    with pytest.raises(pkg.CdgrabError) as ei:
        pkg.cdgrab_balance_epoch_static(h, zd, _outputs(1, 2, d, dev))
    assert ei.value.code == -1 and "131072" in str(ei.value)
    lib = pkg.load_library()
    assert lib.cdgrab_balance_epoch_static(h._h, 1, 2, 8, None, None, None, None, None, None, None) == -1
    # the handle still serves ordinary calls afterwards
    z = workloads.tiny_epoch(1, 2, 8, 64)
    out = pkg.cdgrab_balance_epoch(h, 2, 8, 64, grads=torch.from_numpy(z).to(dev), want_r64=True)
    torch.cuda.synchronize()
    check_epoch(z, _np(out))
