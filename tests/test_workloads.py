"""CPU checks of the seeded input generators (statistics and structure only:
the generators hold none of the method's arithmetic)."""
import numpy as np
import pytest
from scipy import stats

import workloads
from workloads import synth


def test_mixer_avalanche_and_balance():
    rng = np.random.default_rng(0)
    xs = [int(v) for v in rng.integers(0, 2 ** 63, 200)] + list(range(64))
    flips = np.zeros((64, 64))
    for x in xs:
        base = synth.mix(x)
        for b in range(64):
            diff = base ^ synth.mix(x ^ (1 << b))
            flips[b] += [(diff >> o) & 1 for o in range(64)]
    rate = flips / len(xs)
    assert rate.min() > 0.33 and rate.max() < 0.67        # every input bit moves every output bit
    # consecutive counters give balanced bits
    words = np.array([synth.mix(i) for i in range(4096)], dtype=np.uint64)
    ones = np.array([((words >> np.uint64(o)) & np.uint64(1)).mean() for o in range(64)])
    assert np.all(np.abs(ones - 0.5) < 0.04)


def test_student_t3_noise_distribution():
    g = synth.SynthRows(3, 2, 4, 100_000)
    rows = g.fill_pairs_host(0, 4)                         # [p][which][d]
    T = []
    for p in range(4):
        for which in range(2):
            rid = (p % g.m) * g.n + 2 * (p // g.m) + which
            T.append((rows[p, which].astype(np.float64) - g.mu) / g.row_scale[rid])
    T = np.concatenate(T)
    assert stats.kstest(T, stats.t(3).cdf).statistic < 0.004
    q = np.quantile(T, [0.05, 0.25, 0.75, 0.95, 0.999])
    np.testing.assert_allclose(q, stats.t(3).ppf([0.05, 0.25, 0.75, 0.95, 0.999]), rtol=0.08)
    # heavy tail: far more mass beyond 6 than a normal has
    assert (np.abs(T) > 6).mean() > 5e-3
    # neighbouring elements and neighbouring rows are uncorrelated
    a = np.clip(T[:100_000], -5, 5)
    assert abs(np.corrcoef(a[:-1], a[1:])[0, 1]) < 0.02
    b = np.clip(T[100_000:200_000], -5, 5)
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.02


def test_tables_block_scales_and_zero_mask():
    g = synth.SynthRows(5, 3, 6, 64_000, block_scales=64, zero_fraction=0.2)
    assert g.block_len == 1000 and g.block_scale.shape == (64,)
    assert g.block_scale.min() >= 1e-3 and g.block_scale.max() <= 1.0
    z = g.dense_host()
    zero = (z == 0)
    assert abs(zero.mean() - 0.2) < 0.005                  # Bernoulli(0.2) exact zeros
    assert abs(zero[0, 0].mean() - 0.2) < 0.01 and not np.array_equal(zero[0, 0], zero[0, 1])
    # per-block scale: typical magnitude of a block follows its scale
    nz = np.where(zero, np.nan, np.abs(z))
    med = np.nanmedian(nz.reshape(-1, 64, 1000), axis=(0, 2))
    ratio = med / g.block_scale
    assert ratio.max() / ratio.min() < 1.25
    # log-normal(0.5) row scales
    big = synth.SynthRows(6, 32, 512, 8)
    ls = np.log(big.row_scale)
    assert abs(ls.mean()) < 0.02 and abs(ls.std() - 0.5) < 0.02
    assert abs(big.mu.std() - 0.1) < 0.08


def test_element_addressing_is_consistent():
    g = synth.SynthRows(7, 4, 6, 999, block_scales=64, zero_fraction=0.2)
    z = g.dense_host()
    rows = np.array([0, 5, 6, 23], np.int64)               # row id = worker*n + position
    elems = np.array([0, 1, 17, 500, 998], np.int64)
    got = g.sample_host(rows, elems)
    want = z.reshape(-1, 999)[rows][:, elems]
    assert np.array_equal(got, want)
    # pair p -> worker p % m, positions 2*(p//m), 2*(p//m)+1
    blk = g.fill_pairs_host(5, 3)
    for q, p in enumerate(range(5, 8)):
        i, k = p % 4, p // 4
        assert np.array_equal(blk[q, 0], z[i, 2 * k]) and np.array_equal(blk[q, 1], z[i, 2 * k + 1])
    # same seed -> same bits, other seed -> other rows
    assert np.array_equal(synth.SynthRows(7, 4, 6, 999, 64, 0.2).dense_host(), z)
    assert not np.array_equal(synth.SynthRows(8, 4, 6, 999, 64, 0.2).dense_host(), z)
    with pytest.raises(ValueError):
        g.sample_host(np.array([24]), np.array([0]))


def test_numpy_generators_shapes_and_seeding():
    z = workloads.tiny_epoch(1)
    assert z.shape == (4, 64, 1024) and z.dtype == np.float32
    assert np.array_equal(z, workloads.tiny_epoch(1)) and not np.array_equal(z, workloads.tiny_epoch(2))
    assert abs(z.std() - 1.0) < 0.02
    X, y, W = workloads.softmax_problem(0, 1000)
    assert X.shape == (1000, 784) and 0 <= X.min() and X.max() < 1 and abs(X.mean() - 0.5) < 0.01
    assert set(np.unique(y)) == set(range(10)) and W.shape == (785, 10) and abs(W.std() - 0.01) < 1e-3
    zi = workloads.integer_rows(0, 2, 4, 8, 3)
    assert np.array_equal(zi, np.round(zi)) and np.abs(zi).max() <= 3
    p = workloads.random_perms(0, 3, 10)
    assert all(sorted(r.tolist()) == list(range(10)) for r in p)
    c = workloads.CONFIGS
    assert (c["c4_resnet18"].m, c["c4_resnet18"].n, c["c4_resnet18"].d) == (32, 512, 11_200_000)
    assert all(w.n % 2 == 0 for w in c.values())
