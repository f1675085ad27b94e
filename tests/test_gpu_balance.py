"""GPU parity tests of cdgrab_balance_epoch (dense input) against the CPU oracle.
Every call goes through the C ABI via the ctypes binding."""
import os

import numpy as np
import pytest
import torch

import workloads
from conftest import GOLDEN, load_hand_cases
from parity import check_epoch

pytestmark = pytest.mark.gpu

HAND = load_hand_cases(os.path.join(GOLDEN, "hand_cases.txt"))


@pytest.fixture(scope="module")
def lib():
    import paper_2302_00845_amd as p
    return p


def run_epoch(p, z, perm_in=None, block_pairs=0, pass1_groups=0, apply_mode=0, gram_mode=0, apply_groups=0):
    m, n, d = z.shape
    h = p.Handle(block_pairs=block_pairs, pass1_groups=pass1_groups, apply_mode=apply_mode, gram_mode=gram_mode,
                 apply_groups=apply_groups)
    zt = torch.from_numpy(z).cuda()
    pt = torch.from_numpy(perm_in).cuda() if perm_in is not None else None
    out = p.cdgrab_balance_epoch(h, m, n, d, grads=zt, perm_in=pt, want_r32=True, want_r64=True,
                                 want_dots=True)
    torch.cuda.synchronize()
    got = {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}
    h.close()
    return got


@pytest.mark.parametrize("case", HAND, ids=[c["name"] for c in HAND])
@pytest.mark.parametrize("bb", [16, 32, 64])
def test_hand_cases(lib, case, bb):
    got = run_epoch(lib, case["rows"], block_pairs=bb)
    assert got["signs"].tolist() == case["eps"].tolist()
    assert got["r64"].tolist() == case["r"].tolist()
    assert got["perm"].tolist() == case["perm"].tolist()


@pytest.mark.parametrize("bb", [16, 32, 64])
@pytest.mark.parametrize("seed,m,n,d,maxabs", [
    (0, 1, 2, 1, 3), (1, 1, 8, 3, 2), (2, 3, 6, 4, 2), (3, 4, 10, 7, 5), (4, 5, 4, 1, 1),
    (5, 2, 16, 2, 1), (6, 7, 12, 33, 9), (7, 4, 64, 1024, 8), (8, 3, 50, 777, 4),
    (9, 16, 8, 130, 2), (10, 33, 6, 258, 3), (11, 2, 70, 4100, 8), (12, 5, 60, 1500, 3),
])
def test_exact_integer_inputs_bitwise(lib, bb, seed, m, n, d, maxabs):
    """Small-integer rows: all arithmetic is exact, so signs (ties included),
    running sum and permutations must equal the oracle bit for bit.  Shapes cover
    d < one tile, d not a multiple of 4 or 2, several tiles, ragged last block."""
    z = workloads.integer_rows(seed, m, n, d, maxabs)
    perm_in = workloads.random_perms(seed + 50, m, n)
    got = run_epoch(lib, z, perm_in, block_pairs=bb)
    rep = check_epoch(z, got, perm_in, expect_exact_signs=True)
    assert rep["r64_rel_l2"] == 0.0
    assert rep["dots_max_abs_err"] == 0.0


@pytest.mark.parametrize("bb", [16, 32, 64])
def test_config1_tiny_epoch(lib, bb):
    z = workloads.tiny_epoch(1234)                       # m=4, n=64, d=1024
    got = run_epoch(lib, z, block_pairs=bb)
    rep = check_epoch(z, got)
    assert rep["in_margin_flips"] == 0 or not rep["free_run_equal"]


@pytest.mark.parametrize("m,n,d", [(4, 64, 1024), (32, 16, 5000), (8, 40, 65536 + 12), (1, 256, 3000),
                                   (3, 34, 7850)])
def test_heavy_tailed_rows(lib, m, n, d):
    z = workloads.heavy_rows(77, m, n, d)
    got = run_epoch(lib, z)
    check_epoch(z, got)


@pytest.mark.parametrize("m,n,d,bb", [(4, 64, 1024, 16), (3, 50, 777, 32), (8, 40, 65536 + 12, 32),
                                      (16, 30, 130, 64), (2, 70, 4100, 0)])
def test_fused_and_separate_passes_agree(lib, m, n, d, bb):
    """Applying a block inside the next block's dot/Gram launch and applying it with
    its own launch are the same computation: bit-identical on exact input, and both
    within the oracle's tolerances on heavy-tailed rows."""
    zi = workloads.integer_rows(m + n, m, n, d, 6)
    a = run_epoch(lib, zi, block_pairs=bb, apply_mode=2)
    b = run_epoch(lib, zi, block_pairs=bb, apply_mode=1)
    for k in ("signs", "perm", "r64", "dots"):
        assert np.array_equal(a[k], b[k]), k
    check_epoch(zi, a, expect_exact_signs=True)
    z = workloads.heavy_rows(m * n, m, n, d)
    check_epoch(z, run_epoch(lib, z, block_pairs=bb, apply_mode=2))
    check_epoch(z, run_epoch(lib, z, block_pairs=bb, apply_mode=1))


@pytest.mark.parametrize("m,n,d,bb,groups", [
    (4, 64, 1024, 16, 0), (3, 50, 777, 32, 0), (8, 40, 65536 + 12, 32, 0), (16, 30, 130, 64, 0),
    (2, 70, 30000, 0, 1),        # one workgroup: 30 groups per thread, two slabs of 15
    (3, 22, 100001, 32, 2),      # odd row length (scalar loads), ragged last block, three slabs
    (2, 36, 262144 + 8, 16, 0),  # 65 538 groups on 257 workgroups: the last thread row is partly empty
    (1, 4, 1, 0, 0)])
def test_resident_apply_matches_flat_apply(lib, m, n, d, bb, groups):
    """The apply kernel for long rows (a resident grid, sums held in registers, the running
    sum updated in one burst per slab) adds the same terms in the same order as the flat
    one: every output is bit-identical, also on rows that are not exactly representable."""
    for z in (workloads.integer_rows(m + d, m, n, d, 5), workloads.heavy_rows(m * n + 1, m, n, d)):
        a = run_epoch(lib, z, block_pairs=bb, apply_mode=3, apply_groups=groups)
        b = run_epoch(lib, z, block_pairs=bb, apply_mode=4)
        for k in ("signs", "perm", "r64", "r32", "dots"):
            assert np.array_equal(a[k], b[k]), k
        check_epoch(z, a)


def test_resident_apply_unaligned_rows(lib):
    """Rows that start at an 8-byte (not 16-byte) boundary take the two-float loads."""
    m, n, d = 2, 12, 20002
    z = workloads.heavy_rows(9, m, n, d)
    buf = torch.zeros(m * n * d + 2, dtype=torch.float32, device="cuda")
    view = buf[2:].view(m, n, d)
    view.copy_(torch.from_numpy(z))
    outs = []
    for mode in (3, 4):
        h = lib.Handle(apply_mode=mode, apply_groups=3)
        out = lib.cdgrab_balance_epoch(h, m, n, d, grads=view, want_r64=True, want_dots=True)
        torch.cuda.synchronize()
        outs.append({k: v.cpu().numpy() for k, v in out.items() if v is not None})
    for k in ("signs", "perm", "r64", "dots"):
        assert np.array_equal(outs[0][k], outs[1][k]), k
    check_epoch(z, outs[0])


@pytest.mark.parametrize("m,n,d,bb", [(4, 64, 1024, 16), (3, 50, 777, 32), (8, 40, 65536 + 12, 32),
                                      (16, 30, 130, 64), (2, 70, 4100, 0), (5, 6, 3, 16), (1, 4, 1, 0)])
def test_grams_ahead_and_per_block_agree(lib, m, n, d, bb):
    """The Gram matrices do not depend on the running sum, so computing them for many
    blocks ahead (one launch) and computing each inside its block's own launch are the
    same computation: bit-identical on exact input, both within the oracle's tolerances on
    heavy-tailed rows.  (The long-row case forces the ahead form where it is not the default.)"""
    zi = workloads.integer_rows(m + n + 1, m, n, d, 6)
    perm = workloads.random_perms(2, m, n)
    a = run_epoch(lib, zi, perm_in=perm, block_pairs=bb, gram_mode=2)
    b = run_epoch(lib, zi, perm_in=perm, block_pairs=bb, gram_mode=1)
    for k in ("signs", "perm", "r64", "dots"):
        assert np.array_equal(a[k], b[k]), k
    check_epoch(zi, a, perm, expect_exact_signs=True)
    z = workloads.heavy_rows(m * n + 1, m, n, d)
    check_epoch(z, run_epoch(lib, z, block_pairs=bb, gram_mode=2))
    check_epoch(z, run_epoch(lib, z, block_pairs=bb, gram_mode=1))


def test_grams_ahead_is_refused_for_long_rows(lib):
    h = lib.Handle(gram_mode=2)
    z = torch.zeros((1, 4, 131072 + 4), dtype=torch.float32, device="cuda")
    with pytest.raises(lib.CdgrabError) as ei:
        lib.cdgrab_balance_epoch(h, 1, 4, z.shape[2], grads=z)
    assert ei.value.code == -1


def test_grams_ahead_over_several_batches(lib):
    """More blocks than one ahead-launch covers (512): the last block of a batch is the
    previous block of the next batch's first."""
    m, n, d = 3, 2 * 16 * 180, 37                     # 8640 pairs = 540 blocks of 16
    zi = workloads.integer_rows(77, m, n, d, 3)
    a = run_epoch(lib, zi, block_pairs=16, gram_mode=2)
    b = run_epoch(lib, zi, block_pairs=16, gram_mode=1)
    for k in ("signs", "perm", "r64", "dots"):
        assert np.array_equal(a[k], b[k]), k
    check_epoch(zi, a, expect_exact_signs=True)


def _random_cases(count):
    rng = np.random.default_rng(20230200845)
    cases = []
    for _ in range(count):
        m = int(rng.integers(1, 12))
        n = 2 * int(rng.integers(1, 40))
        d = int(rng.choice([1, 2, 3, 17, 63, 64, 65, 127, 130, 255, 1000, 4097, 20000]))
        bb = int(rng.choice([0, 16, 32, 64]))
        apply_mode = int(rng.integers(0, 3))
        gram_mode = int(rng.integers(0, 3))
        cases.append((m, n, d, bb, apply_mode, gram_mode))
    return cases


_WIDE_CASES = [(300, 4, 50, 0, 0, 0), (300, 4, 50, 32, 2, 1), (97, 6, 300, 16, 1, 1), (1, 600, 33, 0, 0, 0),
               (64, 2, 1000, 64, 0, 2), (1000, 2, 7, 0, 0, 0)]


@pytest.mark.parametrize("m,n,d,bb,apply_mode,gram_mode", _random_cases(32) + _WIDE_CASES)
def test_seeded_random_shapes_exact(lib, m, n, d, bb, apply_mode, gram_mode):
    """Seeded draw of shapes and launch forms on exact-arithmetic inputs (plus a few with many
    workers, where a block spans several steps, or a single one): whatever the block size, apply
    form and Gram form, signs, order and running sum equal the oracle's bit for bit."""
    zi = workloads.integer_rows(m * 1000 + n + d, m, n, d, 5)
    perm = workloads.random_perms(d, m, n)
    got = run_epoch(lib, zi, perm_in=perm, block_pairs=bb, apply_mode=apply_mode, gram_mode=gram_mode)
    check_epoch(zi, got, perm, expect_exact_signs=True)


def test_unaligned_base_pointer(lib):
    """A gradient array that starts 4 bytes into an allocation takes the scalar-load path."""
    m, n, d = 3, 10, 1001
    z = workloads.integer_rows(21, m, n, d, 5)
    buf = torch.zeros(m * n * d + 1, dtype=torch.float32, device="cuda")
    view = buf[1:].view(m, n, d)
    view.copy_(torch.from_numpy(z))
    h = lib.Handle()
    out = lib.cdgrab_balance_epoch(h, m, n, d, grads=view, want_r64=True, want_dots=True)
    torch.cuda.synchronize()
    got = {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}
    check_epoch(z, got, expect_exact_signs=True)


def test_identical_rows_all_ties(lib):
    m, n, d = 3, 8, 100
    z = np.tile(np.arange(d, dtype=np.float32), (m, n, 1))
    got = run_epoch(lib, z)
    assert np.all(got["signs"] == 1)
    assert np.all(got["r64"] == 0)
    want = list(range(1, n, 2)) + list(range(n - 2, -1, -2))
    for i in range(m):
        assert got["perm"][i].tolist() == want


def test_deterministic_and_group_count_invariant_on_exact_input(lib):
    z = workloads.heavy_rows(5, 8, 32, 20000)
    a = run_epoch(lib, z)
    b = run_epoch(lib, z)
    for k in ("signs", "perm", "r64", "dots"):
        assert np.array_equal(a[k], b[k]), k                     # run-to-run bit identical
    zi = workloads.integer_rows(6, 8, 32, 20000, 4)
    c = run_epoch(lib, zi, pass1_groups=7)
    e = run_epoch(lib, zi, pass1_groups=300)
    for k in ("signs", "perm", "r64", "dots"):
        assert np.array_equal(c[k], e[k]), k                     # exact input: grid does not matter


def test_own_stream_and_handle_reuse_across_shapes(lib):
    """One handle on a stream of its own (default priority), reused for epochs of different
    shapes and forms (the workspace grows and shrinks its use), with work of another
    handle on the default stream in between: every epoch equals the oracle's."""
    stream = torch.cuda.Stream()
    h = lib.Handle(stream=stream)
    h0 = lib.Handle()
    for seed, (m, n, d) in enumerate([(4, 32, 700), (2, 8, 50000), (8, 64, 64), (1, 2, 1), (3, 20, 9001)]):
        zi = workloads.integer_rows(100 + seed, m, n, d, 5)
        zt = torch.from_numpy(zi).cuda()
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            out = lib.cdgrab_balance_epoch(h, m, n, d, grads=zt, want_r64=True, want_dots=True)
        other = lib.cdgrab_balance_epoch(h0, m, n, d, grads=zt, want_r64=True)    # default stream, concurrently
        stream.synchronize()
        torch.cuda.synchronize()
        got = {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}
        check_epoch(zi, got, expect_exact_signs=True)
        assert torch.equal(other["signs"], out["signs"]) and torch.equal(other["r64"], out["r64"])


@pytest.mark.parametrize("gram_mode,d", [(0, 1000), (1, 1000), (0, 70_000)])
def test_epoch_can_be_captured_in_a_graph(lib, gram_mode, d):
    """On a handle whose workspace is warm (one eager epoch of the same shape) the epoch
    enqueues kernels and device-to-device copies only -- no allocation, no synchronisation,
    no memset node -- so a caller may capture it in a HIP graph.  Every replay, with eager
    epochs in between, reproduces the eager result bit for bit."""
    m, n = 4, 64
    zi = workloads.integer_rows(5, m, n, d, 5)
    perm_np = workloads.random_perms(6, m, n)
    zt, perm = torch.from_numpy(zi).cuda(), torch.from_numpy(perm_np).cuda()
    s = torch.cuda.Stream()
    h = lib.Handle(stream=s, gram_mode=gram_mode)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        ref = lib.cdgrab_balance_epoch(h, m, n, d, grads=zt, perm_in=perm, want_r64=True, want_dots=True)
    s.synchronize()
    check_epoch(zi, {k: (v.cpu().numpy() if v is not None else None) for k, v in ref.items()}, perm_np,
                expect_exact_signs=True)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        out = lib.cdgrab_balance_epoch(h, m, n, d, grads=zt, perm_in=perm, want_r64=True, want_dots=True)
    torch.cuda.synchronize()
    for _ in range(3):
        for k in ("signs", "perm", "r64", "dots"):
            out[k].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in ("signs", "perm", "r64", "dots"):
            assert torch.equal(out[k], ref[k]), k
        with torch.cuda.stream(s):                       # eager work on the same handle between replays
            lib.cdgrab_balance_epoch(h, m, n, d, grads=zt, perm_in=perm)
        s.synchronize()


def test_argument_errors(lib):
    h = lib.Handle()
    z = torch.zeros((2, 3, 4), dtype=torch.float32, device="cuda")
    with pytest.raises(lib.CdgrabError) as ei:
        lib.cdgrab_balance_epoch(h, 2, 3, 4, grads=z)            # odd n
    assert ei.value.code == -1
    with pytest.raises(lib.CdgrabError):
        lib.cdgrab_balance_epoch(h, 2, 4, 4)                      # neither grads nor generator
    with pytest.raises(lib.CdgrabError):
        lib.Handle(block_pairs=24)


def test_overlapping_orders_are_refused(lib):
    """perm_in and perm_out of one call must be two buffers: the permutation kernels read
    one while other threads write the other."""
    h = lib.Handle()
    raw = lib.load_library()
    m, n, d = 2, 8, 16
    z = torch.from_numpy(workloads.tiny_epoch(2, m, n, d)).cuda()
    signs = torch.empty((m, n // 2), dtype=torch.int8, device="cuda")
    perm = torch.from_numpy(workloads.random_perms(2, m, n)).cuda()
    other = torch.empty_like(perm)
    P = perm.data_ptr()
    rc = raw.cdgrab_balance_epoch(h._h, m, n, d, z.data_ptr(), None, None, P, signs.data_ptr(), P,
                                  None, None, None)
    assert rc == -1 and b"overlap" in raw.cdgrab_last_error(h._h)
    # a partial overlap (perm_out starting inside perm_in) as well
    rc = raw.cdgrab_balance_epoch(h._h, m, n, d, z.data_ptr(), None, None, P, signs.data_ptr(), P + 4 * n,
                                  None, None, None)
    assert rc == -1
    ex = torch.ones((m, n), dtype=torch.int8, device="cuda")
    assert raw.cdgrab_reorder(h._h, m, n, ex.data_ptr(), P, P) == -1
    assert raw.cdgrab_reorder(h._h, m, n, ex.data_ptr(), P, other.data_ptr()) == 0
    g1 = z.view(m * n, d)
    s1 = torch.empty((m * n,), dtype=torch.int8, device="cuda")
    p1 = perm.view(-1)
    assert raw.cdgrab_balance_epoch_stale_mean(h._h, m * n, d, g1.data_ptr(), None, p1.data_ptr(), s1.data_ptr(),
                                               p1.data_ptr(), None, None) == -1
    mean = torch.zeros(d, dtype=torch.float32, device="cuda")
    assert raw.cdgrab_balance_epoch_stale_mean(h._h, m * n, d, g1.data_ptr(), mean.data_ptr(), None,
                                               s1.data_ptr(), other.view(-1).data_ptr(), mean.data_ptr(),
                                               None) == -1
    # two buffers: fine
    rc = raw.cdgrab_balance_epoch(h._h, m, n, d, z.data_ptr(), None, None, P, signs.data_ptr(),
                                  other.data_ptr(), None, None, None)
    assert rc == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("m,n,d,bb", [(1, 4, 1, 0), (4, 40, 300, 16), (3, 70, 5000, 32), (16, 20, 130, 64)])
def test_randomized_rule_matches_oracle(lib, m, n, d, bb):
    """RandomizedBalance with caller-supplied draws against the oracle fed the same draws."""
    import oracle
    from parity import expected_perm_from_signs
    rng = np.random.default_rng(m * n + d)
    v = rng.standard_normal((m, n, d))
    z = (v / (2 * np.linalg.norm(v, axis=2, keepdims=True))).astype(np.float32)
    u = rng.random((m, n // 2)).astype(np.float32)
    perm_in = workloads.random_perms(1, m, n)
    h = lib.Handle(block_pairs=bb)
    out = lib.cdgrab_balance_epoch_randomized(h, torch.from_numpy(z).cuda(), torch.from_numpy(u).cuda(),
                                              torch.from_numpy(perm_in).cuda())
    ref = oracle.randomized_epoch(z, u, perm_in)
    eps = out["signs"].cpu().numpy()
    if np.array_equal(eps, ref["eps"]):
        ref_r, ref_t = ref["r"], ref["t"]
        assert np.array_equal(out["perm"].cpu().numpy(), ref["perm"])
    else:
        # a draw within rounding of its threshold may decide differently: the oracle is advanced
        # with the HIP path's signs and every decision, the dots and the running sum are judged
        # against that walk (p = (1 + t)/2 with t = <r, z2 - z1>; exported sign -1 iff u < p)
        from parity import flatten_pairs, replay_pairs
        flat_gpu = np.ascontiguousarray(eps.T).reshape(-1)
        ref_r, t, nr, nc = replay_pairs(flatten_pairs(z), flat_gpu)
        uf = np.ascontiguousarray(u.T).reshape(-1).astype(np.float64)
        want = np.where(uf < 0.5 * (1.0 + t), -1, 1)
        bad = want != flat_gpu
        assert np.all(np.abs(uf[bad] - 0.5 * (1.0 + t[bad])) <= 1e-9 * np.maximum(1.0, nr[bad] * nc[bad]))
        print("draws within rounding of their threshold:", int(bad.sum()))
        ref_t = t.reshape(n // 2, m).T
    np.testing.assert_allclose(out["r64"].cpu().numpy(), ref_r, atol=1e-12)
    np.testing.assert_allclose(out["dots"].cpu().numpy(), ref_t, atol=1e-12)
    assert np.array_equal(out["perm"].cpu().numpy(), expected_perm_from_signs(eps, perm_in))
    # the greedy entry point is unaffected by an earlier randomized call on the same handle
    g = lib.cdgrab_balance_epoch(h, m, n, d, grads=torch.from_numpy(z).cuda(), want_r64=True, want_dots=True)
    got = {k: (val.cpu().numpy() if val is not None else None) for k, val in g.items()}
    check_epoch(z, got)
