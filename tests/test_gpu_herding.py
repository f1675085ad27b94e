"""GPU tests of cdgrab_herding_bound against the CPU oracle, and the paper's
synthetic herding study at reduced scale: repeated balance + reorder on fixed
vectors drives the parallel herding objective far below random orders'."""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2302_00845_amd as p
    return p


def gpu_bound(lib, h, z, perm=None):
    zt = torch.from_numpy(z).cuda() if isinstance(z, np.ndarray) else z
    pt = torch.from_numpy(perm).cuda() if isinstance(perm, np.ndarray) else perm
    return float(lib.cdgrab_herding_bound(h, zt, pt).cpu()[0])


def test_closed_form_cases(lib):
    h = lib.Handle()
    z = np.array([[[1.0], [-1.0]], [[2.0], [-2.0]]], np.float32)
    assert gpu_bound(lib, h, z) == 3.0
    assert gpu_bound(lib, h, z, np.array([[0, 1], [1, 0]], np.int32)) == 1.0
    assert gpu_bound(lib, h, z + 5.0) == 3.0
    one = np.array([[[3.0, -4.0]]], np.float32)              # a single vector: prefix is 0
    assert gpu_bound(lib, h, one) == 0.0


@pytest.mark.parametrize("m,n,d", [(1, 1, 1), (3, 7, 5), (4, 64, 1024), (5, 400, 16), (16, 50, 7850),
                                   (2, 3000, 3), (8, 33, 300), (5, 20000, 16), (100, 1000, 16), (3, 70001, 8),
                                   (2, 999, 512), (7, 130, 516), (1, 300000, 1)])
@pytest.mark.parametrize("with_perm", [False, True])
def test_matches_oracle(lib, m, n, d, with_perm):
    h = lib.Handle()
    z = workloads.heavy_rows(m * 7 + n, m, n, d)
    perm = workloads.random_perms(n, m, n) if with_perm else None
    want = oracle.parallel_herding(z, perm)
    got = gpu_bound(lib, h, z, perm)
    assert abs(got - want) <= 1e-9 * max(want, 1e-30)


@pytest.mark.parametrize("m,n,d,exact", [
    (5, 24, 300, False),        # one block per worker: m one-worker epochs back to back
    (7, 200, 300, False),       # two blocks: the walks run side by side, the worker as a grid coordinate
    (3, 2100, 40, True),        # seventeen blocks, a ragged last one, exact ties
    (4, 300, 1001, True),       # odd row length: scalar loads, rows of later workers unaligned
    (16, 468, 7850, False),     # config 2's row length
    (2, 66000, 8, True),        # 516 blocks: more than one batch of Gram matrices, the last tile carried over
    (70, 130, 16, False)])
def test_independent_walks_match_oracle(lib, m, n, d, exact):
    """ID-GraB (PairBal): worker i's signs and order are those of a one-worker walk over its
    own rows, whether the library runs the m walks one after the other or side by side."""
    from parity import judge_greedy, replay_pairs, flatten_pairs, expected_perm_from_signs
    z = workloads.integer_rows(9, m, n, d, 4) if exact else workloads.heavy_rows(9, m, n, d)
    perm_in = workloads.random_perms(4, m, n)
    h = lib.Handle()
    out = lib.cdgrab_balance_epoch_independent(h, torch.from_numpy(z).cuda(), torch.from_numpy(perm_in).cuda())
    signs, perm = out["signs"].cpu().numpy(), out["perm"].cpu().numpy()
    for i in range(m):
        ref = oracle.server_epoch(z[i:i + 1], perm_in[i:i + 1])
        if not np.array_equal(ref["eps"][0], signs[i]):
            assert not exact
            # a near-tie decided the other way: judge worker i's walk by replay
            _, t, nr, nc = replay_pairs(flatten_pairs(z[i:i + 1]), signs[i])
            judge_greedy(t, nr, nc, signs[i])
    assert np.array_equal(perm, expected_perm_from_signs(signs, perm_in))
    # a coordinated epoch on the same handle afterwards is unaffected
    g = lib.cdgrab_balance_epoch(h, m, n, d, grads=torch.from_numpy(z).cuda(), want_r64=True, want_dots=True)
    from parity import check_epoch
    check_epoch(z, {k: (v.cpu().numpy() if v is not None else None) for k, v in g.items()})


def _run_orders(lib, h, z, epochs, coordinated):
    m, n, d = z.shape
    perm = torch.arange(n, dtype=torch.int32, device="cuda").repeat(m, 1).contiguous()
    for _ in range(epochs):
        idx = perm.long().unsqueeze(-1).expand(m, n, d)
        visited = torch.gather(z, 1, idx).contiguous()
        if coordinated:
            perm = lib.cdgrab_balance_epoch(h, m, n, d, grads=visited, perm_in=perm, want_r32=False)["perm"]
        else:
            perm = lib.cdgrab_balance_epoch_independent(h, visited, perm)["perm"]
    return perm


def test_coordination_matters_with_many_workers(lib):
    """The ablation's point (Sec. 5 and App. E): with many workers, independent
    balancing loses to coordinated balancing on the parallel herding objective."""
    h = lib.Handle()
    N, d, m = 1 << 15, 16, 64
    vec = workloads.herding_vectors(5, N, d)
    z = torch.from_numpy(vec.reshape(m, N // m, d)).cuda()
    coord = gpu_bound(lib, h, z, _run_orders(lib, h, z, 8, True))
    indep = gpu_bound(lib, h, z, _run_orders(lib, h, z, 8, False))
    rand = np.mean([gpu_bound(lib, h, z, workloads.random_perms(s, m, N // m)) for s in range(3)])
    print("m=%d coordinated %.2f independent %.2f random %.2f" % (m, coord, indep, rand))
    assert coord < 0.5 * indep and indep < rand


def test_herding_bound_over_worker_counts(lib):
    """The shape of App. E's figure at reduced scale (60 000 vectors, 16 dimensions, the
    paper's worker counts): coordinated balancing stays flat and lowest as m grows, while
    independent per-worker balancing climbs towards random orders.  Measured: coordinated
    2.5 / 2.2 / 2.1 / 2.4 / 2.1, independent 5.6 / 8.6 / 10.0 / 14.9 / 18.2, random about 80."""
    h = lib.Handle()
    N, d = 60000, 16
    vec = workloads.herding_vectors(11, N, d)
    coord, indep, rand = [], [], []
    for m in (5, 10, 20, 50, 100):
        z = torch.from_numpy(vec.reshape(m, N // m, d)).cuda()
        coord.append(gpu_bound(lib, h, z, _run_orders(lib, h, z, 8, True)))
        indep.append(gpu_bound(lib, h, z, _run_orders(lib, h, z, 8, False)))
        rand.append(gpu_bound(lib, h, z, workloads.random_perms(m, m, N // m)))
    print("coordinated", ["%.2f" % b for b in coord], "independent", ["%.2f" % b for b in indep],
          "random", ["%.1f" % b for b in rand])
    assert max(coord) < 1.5 * min(coord)                       # flat in m
    assert all(c < 0.6 * i for c, i in zip(coord, indep))      # and lowest
    assert indep[-1] > 2.0 * indep[0] and indep[2] > indep[0]  # independent balancing degrades with m
    assert all(i < r for i, r in zip(indep, rand))


def test_synthetic_herding_study_reduced(lib):
    """App. E's synthetic study, scaled down (2^16 unit vectors in 16 dimensions
    instead of 10^6): CD-GraB's orders reach a parallel herding bound far below that
    of random orders, for few and for many workers."""
    h = lib.Handle()
    N, d = 1 << 16, 16
    vec = workloads.herding_vectors(3, N, d)
    for m in (4, 32):
        n = N // m
        z = torch.from_numpy(vec.reshape(m, n, d)).cuda()
        rand = [gpu_bound(lib, h, z, workloads.random_perms(s, m, n)) for s in range(3)]
        perm = torch.arange(n, dtype=torch.int32, device="cuda").repeat(m, 1).contiguous()
        bounds = [gpu_bound(lib, h, z, perm)]
        for epoch in range(8):
            idx = perm.long().unsqueeze(-1).expand(m, n, d)
            visited = torch.gather(z, 1, idx).contiguous()        # rows in visiting order
            out = lib.cdgrab_balance_epoch(h, m, n, d, grads=visited, perm_in=perm, want_r32=False)
            perm = out["perm"]
            bounds.append(gpu_bound(lib, h, z, perm))
        final_perm = perm.cpu().numpy()
        for i in range(m):
            assert np.array_equal(np.sort(final_perm[i]), np.arange(n))
        # cross-check the evaluator on the final orders
        want = oracle.parallel_herding(vec.reshape(m, n, d), final_perm)
        assert abs(bounds[-1] - want) <= 1e-9 * want
        print("m=%d random %.2f  epochs %s" % (m, np.mean(rand), ["%.2f" % b for b in bounds]))
        assert bounds[-1] < 0.25 * min(rand)
        assert min(bounds[1:]) < bounds[0]


@pytest.mark.parametrize("n,d,exact", [(1, 1, True), (7, 3, True), (33, 100, True), (100, 1000, True),
                                       (64, 5000, False), (257, 300, False)])
def test_stale_mean_balance_matches_oracle(lib, n, d, exact):
    """Centralized GraB balancing (single vectors centred by a stale mean)."""
    h = lib.Handle()
    rng = np.random.default_rng(n + d)
    if exact:
        g = rng.integers(-6, 7, size=(n, d)).astype(np.float32)
        mu = rng.integers(-2, 3, size=d).astype(np.float32)
    else:
        g = workloads.heavy_rows(n, 1, n, d)[0]
        mu = g.mean(0).astype(np.float32) + 0.01 * rng.standard_normal(d).astype(np.float32)
    perm_in = rng.permutation(n).astype(np.int32)
    out = lib.cdgrab_balance_epoch_stale_mean(h, torch.from_numpy(g).cuda(), torch.from_numpy(mu).cuda(),
                                              torch.from_numpy(perm_in).cuda())
    ref = oracle.grab_stale_mean(g, mu, perm_in)
    s = out["signs"].cpu().numpy()
    if np.array_equal(s, ref["s"]):
        ref_r = ref["r"]
        assert np.array_equal(out["perm"].cpu().numpy(), ref["perm"])
    else:
        assert not exact
        # a near-tie may be decided differently: advance the oracle with the HIP path's signs
        # and judge every decision and the running sum against that walk.  Vector j enters the
        # pair walk as the pair (g_j, stale mean), whose difference is -z_j and whose exported
        # sign is -s_j; the rule s_j = +1 iff ||r + z_j|| < ||r - z_j|| reads, in the walk's
        # terms, eps = +1 iff t <= 0.
        from parity import judge_greedy, replay_pairs
        rows = np.stack([g, np.broadcast_to(mu, g.shape)], axis=1)
        ref_r, t, nr, nz = replay_pairs(rows, -s)
        print("in-margin flips:", judge_greedy(t, nr, nz, -s))
    np.testing.assert_allclose(out["r64"].cpu().numpy(), ref_r, rtol=0,
                               atol=1e-12 * max(1.0, np.abs(ref_r).max()))
    assert np.array_equal(out["perm"].cpu().numpy(), oracle.reorder(s, perm_in))
    np.testing.assert_allclose(out["mean"].cpu().numpy(), ref["mean"], rtol=1e-6, atol=1e-7)
    # no stale mean given = zero mean
    out0 = lib.cdgrab_balance_epoch_stale_mean(h, torch.from_numpy(g).cuda())
    ref0 = oracle.grab_stale_mean(g)
    if exact:
        assert np.array_equal(out0["signs"].cpu().numpy(), ref0["s"])


def _run_stale_mean_orders(lib, h, z, epochs):
    """ID-GraB (Bal): every worker balances its own vectors, centred by the mean of its
    previous epoch (zero before the first), with no shared state."""
    m, n, d = z.shape
    perm = torch.arange(n, dtype=torch.int32, device="cuda").repeat(m, 1).contiguous()
    stale = [None] * m
    for _ in range(epochs):
        idx = perm.long().unsqueeze(-1).expand(m, n, d)
        visited = torch.gather(z, 1, idx).contiguous()
        nxt = torch.empty_like(perm)
        for i in range(m):
            out = lib.cdgrab_balance_epoch_stale_mean(h, visited[i], stale[i], perm[i].contiguous())
            nxt[i] = out["perm"]
            stale[i] = out["mean"]
        perm = nxt
    return perm


@pytest.mark.timeout(900)
def test_synthetic_herding_study_at_paper_scale(lib):
    """App. E's synthetic study as the paper states it: one million vectors from Unif(0,1)^16,
    zero-centred and scaled to unit length, split evenly over m = 5, 10, 20, 50, 100 workers,
    three seeds; orders from CD-GraB (coordinated pair balancing), ID-GraB (PairBal)
    (independent pair balancing), ID-GraB (Bal) (independent balancing with a stale mean) and
    random orders (D-RR), compared on the parallel herding objective.  The paper reports a
    figure, so only its qualitative content can be checked: coordinated balancing is lowest
    and flat in m, the uncoordinated variants grow with m."""
    h = lib.Handle()
    N, d, epochs = 1_000_000, 16, 8
    ms = (5, 10, 20, 50, 100)
    table = {}
    for seed in range(3):
        vec = workloads.herding_vectors(100 + seed, N, d)
        coord, pair, bal, rand = [], [], [], []
        for m in ms:
            n = N // m
            z = torch.from_numpy(vec.reshape(m, n, d)).cuda()
            perm_c = _run_orders(lib, h, z, epochs, True)
            coord.append(gpu_bound(lib, h, z, perm_c))
            pair.append(gpu_bound(lib, h, z, _run_orders(lib, h, z, epochs, False)))
            # the stale-mean variant costs a call per worker and epoch: fewer epochs, first seed only
            if seed == 0:
                bal.append(gpu_bound(lib, h, z, _run_stale_mean_orders(lib, h, z, 4)))
            rand.append(gpu_bound(lib, h, z, workloads.random_perms(seed * 1000 + m, m, n)))
            if seed == 0:
                # the evaluator itself, at this size, against the oracle
                want = oracle.parallel_herding(vec.reshape(m, n, d), perm_c.cpu().numpy())
                assert abs(coord[-1] - want) <= 1e-9 * want
            del z
        table[seed] = (coord, pair, bal, rand)
        print("seed %d  CD-GraB %s | ID-GraB (PairBal) %s | ID-GraB (Bal) %s | random %s" % (
            seed, ["%.2f" % b for b in coord], ["%.2f" % b for b in pair], ["%.2f" % b for b in bal],
            ["%.0f" % b for b in rand]))
        assert max(coord) < 2.0 * min(coord)                          # flat in m
        assert all(c < p for c, p in zip(coord, pair))                # lowest
        assert coord[-1] < 0.5 * pair[-1]
        assert pair[-1] > 2.0 * pair[0] and pair[2] > pair[0]         # uncoordinated: grows with m
        assert all(c < 0.2 * r for c, r in zip(coord, rand))
        if bal:
            assert all(c < b for c, b in zip(coord, bal)) and bal[-1] > bal[0]
