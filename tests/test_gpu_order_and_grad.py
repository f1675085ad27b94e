"""GPU parity tests of cdgrab_reorder and cdgrab_pergrad against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from parity import rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2302_00845_amd as p
    return p


@pytest.mark.parametrize("m,n", [(1, 1), (1, 2), (3, 7), (4, 256), (5, 257), (2, 1000), (16, 3750), (1, 48816)])
@pytest.mark.parametrize("with_perm", [False, True])
def test_reorder_matches_oracle(lib, m, n, with_perm):
    signs = workloads.random_signs(m * 1000 + n, m, n)
    perm_in = workloads.random_perms(n, m, n) if with_perm else None
    h = lib.Handle()
    out = lib.cdgrab_reorder(h, torch.from_numpy(signs).cuda(),
                             torch.from_numpy(perm_in).cuda() if with_perm else None).cpu().numpy()
    for i in range(m):
        want = oracle.reorder(signs[i], perm_in[i] if with_perm else None)
        assert np.array_equal(out[i], want)


def test_reorder_all_one_sign(lib):
    h = lib.Handle()
    n = 300
    for s in (1, -1):
        signs = np.full((2, n), s, np.int8)
        out = lib.cdgrab_reorder(h, torch.from_numpy(signs).cuda()).cpu().numpy()
        want = np.arange(n) if s == 1 else np.arange(n)[::-1]
        assert np.array_equal(out[0], want) and np.array_equal(out[1], want)


def test_reorder_rejects_bad_sign(lib):
    h = lib.Handle()
    signs = np.ones((2, 10), np.int8)
    signs[1, 3] = 0
    with pytest.raises(lib.CdgrabError) as ei:
        lib.cdgrab_reorder(h, torch.from_numpy(signs).cuda())
    assert ei.value.code == -1


@pytest.mark.parametrize("N,in_dim,classes", [(1, 1, 1), (5, 7, 4), (64, 784, 10), (257, 784, 10), (33, 100, 70),
                                               (9, 2000, 12), (300, 33, 300), (9000, 30, 3), (5, 6000, 7), (3, 16000, 3)])
def test_pergrad_matches_oracle(lib, N, in_dim, classes):
    X, y, W = workloads.softmax_problem(N, N, in_dim, classes)
    if classes > 1 and in_dim <= 2000:
        W = (W * 20).astype(np.float32)       # logits of order one; with long features they already are
    h = lib.Handle()
    G = lib.cdgrab_pergrad(h, torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(),
                           torch.from_numpy(W).cuda()).cpu().numpy()
    want = oracle.softmax_pergrad(X, y, W)
    if classes == 1:
        assert np.all(np.abs(G) <= 1e-6)                  # softmax of one class: delta = 0
        return
    for e in range(N):
        assert rel_l2(G[e], want[e]) <= 1e-5
    assert rel_l2(G, want) <= 1e-5


def test_pergrad_empty_and_errors(lib):
    h = lib.Handle()
    X = torch.zeros((0, 5), dtype=torch.float32, device="cuda")
    y = torch.zeros((0,), dtype=torch.int32, device="cuda")
    W = torch.zeros((6, 3), dtype=torch.float32, device="cuda")
    assert lib.cdgrab_pergrad(h, X, y, W).shape == (0, 18)
    with pytest.raises(TypeError):
        lib.cdgrab_pergrad(h, X.double(), y, W)
    big = torch.zeros((2, 20000), dtype=torch.float32, device="cuda")         # one example exceeds LDS
    with pytest.raises(lib.CdgrabError) as ei:
        lib.cdgrab_pergrad(h, big, torch.zeros(2, dtype=torch.int32, device="cuda"),
                           torch.zeros((20001, 3), dtype=torch.float32, device="cuda"))
    assert ei.value.code == -1


def test_config2_softmax_end_to_end(lib):
    """Config 2 at full size: 60 000 per-example gradients of the 784->10 softmax
    regression on the GPU (<= 1e-5 rel. L2 per example against the double oracle),
    then one balanced epoch on those gradients, judged against the oracle walking
    the same bytes."""
    from parity import check_epoch
    w = workloads.CONFIGS["c2_softmax"]
    N = w.m * w.n
    X, y, W = workloads.softmax_problem(7, N)
    h = lib.Handle()
    G = lib.cdgrab_pergrad(h, torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(),
                           torch.from_numpy(W).cuda())
    perm_in = workloads.random_perms(8, w.m, w.n)
    out = lib.cdgrab_balance_epoch(h, w.m, w.n, w.d, grads=G.view(w.m, w.n, w.d),
                                   perm_in=torch.from_numpy(perm_in).cuda(), want_r64=True, want_dots=True)
    torch.cuda.synchronize()
    Gh = G.cpu().numpy()
    want = oracle.softmax_pergrad(X, y, W)
    num = np.linalg.norm(Gh.astype(np.float64) - want, axis=1)
    den = np.linalg.norm(want.astype(np.float64), axis=1)
    assert np.all(num <= 1e-5 * den)
    got = {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}
    rep = check_epoch(Gh.reshape(w.m, w.n, w.d), got, perm_in)
    print(rep)
