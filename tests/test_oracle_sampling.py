"""Pins for the oracle's Philox generator, size allocation, weights and masks."""
import os
from math import comb

import numpy as np
import pytest

from oracle import philox, sampling

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat():
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        yield v[:4], v[4:6], v[6:]


def test_philox_known_answers():
    for ctr, key, out in _kat():
        assert list(philox.philox4x32_10(ctr, key)) == out
        arr = philox.philox4x32_10_array(*ctr, *key)
        assert [int(x) for x in arr] == out


def test_philox_scalar_and_array_agree_on_random_counters():
    rng = np.random.default_rng(0)
    c = rng.integers(0, 1 << 32, size=(4, 200), dtype=np.uint64)
    k0, k1 = 0x12345678, 0x9ABCDEF0
    o = philox.philox4x32_10_array(c[0], c[1], c[2], c[3], k0, k1)
    for i in range(200):
        assert tuple(int(x[i]) for x in o) == philox.philox4x32_10(c[:, i], (k0, k1))


def test_philox_is_a_bijection_of_the_counter_low_bits():
    # distinct counters under one key give distinct outputs (it is a permutation)
    outs = {philox.philox4x32_10((i, 0, 0, 0), (5, 6)) for i in range(2000)}
    assert len(outs) == 2000


def test_rho_sum_closed_form():
    for line in open(os.path.join(GOLDEN, "allocation_cases.txt")):
        if line.startswith("#"):
            continue
        n, ns, total, k1 = line.split()
        n = int(n)
        s = sum(sampling.rho(n, i) for i in range(1, n))
        harmonic = sum(1.0 / i for i in range(1, n))
        assert s == pytest.approx(2 * (n - 1) * harmonic / n, rel=1e-13)
        assert s == pytest.approx(float(total), rel=1e-12)


def test_allocation_figure_case_n30_k25000():
    plan = sampling.allocation(30, 25000)
    assert not plan["enumerate"] and plan["k"] == 25000 and plan["K"] == 12499
    assert plan["T"] == pytest.approx(7.659197342001644, rel=1e-13)
    # real-valued k_1 = k rho_1 / sum rho = 3264.05; the integer plan splits the
    # K sampled pairs, so class 1 (sizes 1 and 29) gets K*2rho_1/T pairs
    assert abs(int(plan["q"][1]) - 12499 * 2 * sampling.rho(30, 1) / plan["T"]) <= 1
    assert int(plan["q"][1]) == 3264
    assert int(plan["q"].sum()) == 12499
    assert np.all(np.diff(plan["b"]) >= 0) and plan["b"][-1] == 12499
    # the middle class (15, 15) is a single size: half the per-size mass of its neighbours' pair mass
    assert int(plan["q"][15]) == pytest.approx(12499 * sampling.rho(30, 15) / plan["T"], abs=1)


@pytest.mark.parametrize("n,ns", [(5, 10), (25, 64), (26, 1001), (100, 2000), (1001, 20000), (7, 100000)])
def test_allocation_invariants(n, ns):
    plan = sampling.allocation(n, ns)
    if plan["enumerate"]:
        assert plan["k"] == 1 << n
        return
    assert plan["k"] == 2 * (ns // 2)
    assert int(plan["q"].sum()) == plan["K"]
    assert np.all(plan["q"] >= 0)
    # proportionality: each class within one pair of its real-valued share
    H = n // 2
    share = np.array([0.0] + [sampling.rho(n, s) * (1 if 2 * s == n else 2) for s in range(1, H + 1)])
    share = plan["K"] * share / share.sum()
    assert np.all(np.abs(plan["q"] - share) <= 1.0 + 1e-9)


def test_weights_carry_class_mass_and_equal_kernel_under_enumeration():
    n = 10
    Z, w, sz = sampling.sample(n, 1 << n, 1, 0)
    assert Z.shape == (1 << n, 1)
    for s in range(1, n):
        kernel = (n - 1) / (comb(n, s) * s * (n - s))      # the kernel-weight equation
        sel = sz == s
        assert sel.sum() == comb(n, s)
        assert np.allclose(w[sel], kernel, rtol=1e-7)
    assert w[0] == 0 and w[1] == 0 and sz[0] == 0 and sz[1] == n
    # sampled mode: rows of one size share rho_s
    n = 41
    Z, w, sz = sampling.sample(n, 6000, 9, 4)
    for s in range(1, n):
        sel = sz == s
        if sel.any():
            assert w[sel].astype(np.float64).sum() == pytest.approx(sampling.rho(n, s), rel=1e-6)


def test_enumeration_rows_are_all_coalitions_once():
    n = 9
    Z, w, sz = sampling.sample(n, 1 << n, 3, 7)
    assert sorted(int(z) for z in Z[:, 0]) == list(range(1 << n))
    assert np.all(Z[0::2, 0] ^ Z[1::2, 0] == (1 << n) - 1)
    assert Z[0, 0] == 0 and Z[1, 0] == (1 << n) - 1


@pytest.mark.parametrize("n,ns", [(30, 2000), (64, 1000), (65, 1000), (130, 3001), (1000, 400)])
def test_mask_invariants(n, ns):
    Z, w, sz = sampling.sample(n, ns, 1234567890123, 42)
    plan = sampling.allocation(n, ns)
    k, K = plan["k"], plan["K"]
    bits = sampling.unpack_rows(Z, n)
    assert Z.shape == (k, (n + 63) // 64)
    assert np.array_equal(bits.sum(axis=1), sz)
    assert not bits[0].any() and bits[1].all()
    assert np.array_equal(bits[0::2], ~bits[1::2])
    r = np.arange(1, K + 1)
    assert np.array_equal(sz[2::2], sampling.pair_sizes(plan["b"], r))
    assert np.all(np.diff(sz[2::2]) >= 0)                 # pairs laid out by size
    assert int(bits[2:].sum()) == n * K                   # each pair holds n edges in total
    # padding bits are zero in both members
    if n % 64:
        pad = ~np.uint64((1 << (n % 64)) - 1)
        assert not np.any(Z[:, -1] & pad)


def test_masks_are_the_smallest_keys_with_low_index_ties():
    # direct restatement on one pair with python sorting of (key, column)
    n, ns, seed, tag = 37, 500, 99, 5
    Z, w, sz = sampling.sample(n, ns, seed, tag)
    bits = sampling.unpack_rows(Z, n)
    for r in (1, 17, 200, 249):
        keys = []
        for j in range(n):
            out = philox.philox4x32_10((j // 4, r, 0, tag), (seed & 0xFFFFFFFF, seed >> 32))
            keys.append((out[j % 4], j))
        chosen = sorted(keys)[: sz[2 * r]]
        expect = np.zeros(n, bool)
        expect[[j for _, j in chosen]] = True
        assert np.array_equal(bits[2 * r], expect)


def test_shard_independence():
    n, ns = 77, 1200
    Z, w, sz = sampling.sample(n, ns, 5, 1)
    for r0, r1 in [(0, 10), (10, 333), (333, 600)]:
        Zp, wp, szp = sampling.sample(n, ns, 5, 1, pair_range=(r0, r1))
        assert np.array_equal(Zp, Z[2 * r0:2 * r1])
        assert np.array_equal(wp, w[2 * r0:2 * r1])
        assert np.array_equal(szp, sz[2 * r0:2 * r1])


def test_different_tag_or_seed_gives_different_masks():
    a = sampling.sample(50, 400, 5, 1)[0]
    assert not np.array_equal(a, sampling.sample(50, 400, 5, 2)[0])
    assert not np.array_equal(a, sampling.sample(50, 400, 6, 1)[0])
    assert not np.array_equal(a, sampling.sample(50, 400, 5 + (1 << 32), 1)[0])


def test_column_frequencies_are_uniform():
    # within a size class every column is equally likely: chi-square on size-s rows
    n, ns = 40, 40000
    Z, w, sz = sampling.sample(n, ns, 2024, 11)
    bits = sampling.unpack_rows(Z, n)
    small = bits[2::2]
    counts = small.sum(axis=0).astype(np.float64)
    expected = small.sum() / n
    chi2 = ((counts - expected) ** 2 / expected).sum()
    # 39 degrees of freedom: mean 39, sd ~8.8 (variance is smaller than
    # multinomial because rows have fixed size; the bound is generous)
    assert chi2 < 39 + 6 * 8.9


def test_gram_closed_form_under_enumeration():
    # with kernel weights, Z^T W Z = a I + b 11^T,
    # diag = ((n-1)/n) H_{n-1}, off-diag = ((n-1)/n)(H_{n-1} - 1)
    n = 12
    Z, w, sz = sampling.sample(n, 1 << n, 0, 0)
    B = sampling.unpack_rows(Z, n).astype(np.float64)
    G = B[2:].T @ (w[2:, None].astype(np.float64) * B[2:])
    Hn = sum(1.0 / i for i in range(1, n))
    assert np.allclose(np.diag(G), (n - 1) / n * Hn, rtol=1e-6)
    off = G[~np.eye(n, dtype=bool)]
    assert np.allclose(off, (n - 1) / n * (Hn - 1.0), rtol=1e-6)
    assert np.diag(G)[0] == pytest.approx(2.7682209, rel=1e-6)
    assert off[0] == pytest.approx(1.8515542, rel=1e-6)


# ---------------------------------------------------------------- saturated size classes (option)
def test_unranking_is_the_lexicographic_order_of_subsets():
    import itertools
    for n, s in [(5, 1), (5, 2), (6, 3), (9, 4), (12, 2)]:
        want = [list(c) for c in itertools.combinations(range(n), s)]
        got = [sampling.unrank_subset(n, s, j) for j in range(len(want))]
        assert got == want


@pytest.mark.parametrize("n,ns", [(30, 25000), (200, 3000), (12, 1000), (9, 510), (1010, 20000)])
def test_saturated_classes_are_enumerated_once_with_the_kernel_weight(n, ns):
    from math import comb
    plain = sampling.allocation(n, ns)
    plan = sampling.allocation(n, ns, saturate=True)
    up = plan["enum_upto"]
    assert up >= 1 and plain["enum_upto"] == 0
    assert int(plan["q"].sum()) == plan["K"] and np.all(np.diff(plan["b"]) >= 0)
    # the first class that stays sampled was allotted fewer pairs than it has coalitions; the enumerated ones had enough
    assert plan["q"][up + 1] < comb(n, up + 1) or 2 * (up + 1) >= n
    assert plain["q"][1] >= comb(n, 1)
    Z, w, sz = sampling.sample(n, ns, 7, 3, saturate=True)
    bits = sampling.unpack_rows(Z, n)
    for s in range(1, up + 1):
        assert plan["q"][s] == comb(n, s)
        for size in (s, n - s):
            rows = bits[sz == size]
            assert len(rows) == comb(n, s) and len({r.tobytes() for r in rows}) == comb(n, s)   # every subset once
            # the Shapley kernel weight itself: (n-1) / (C(n,s) s (n-s))
            assert np.all(w[sz == size] == np.float32((n - 1) / (comb(n, s) * s * (n - s))))
    # complements and sizes as in every plan; sampled classes keep their whole mass
    assert np.array_equal(bits[0::2], ~bits[1::2])
    for s in range(up + 1, min(up + 4, n // 2)):
        if plan["q"][s] > 0:
            assert abs(w[sz == s].astype(np.float64).sum() - sampling.rho(n, s)) < 1e-5 * sampling.rho(n, s)
    # pairs of the sampled classes are drawn as without the option (same keys, same pair index): only the sizes moved
    with pytest.raises(ValueError):
        sampling.allocation(n, ns, weighting="uniform", saturate=True)


def test_saturation_brings_the_estimate_closer_to_exact_shapley():
    """9 players, 510 rows: without the option the 254 pairs are drawn with replacement from 255 pairs of
    coalitions; with it the classes 1..3 are enumerated and only the size-4 class (125 of its 126 pairs) is
    sampled (with replacement), so most of the sampling error is gone."""
    from oracle import shapley, solve
    n = 9
    rng = np.random.default_rng(3)
    a, c = rng.standard_normal(n), rng.standard_normal(n)
    f = lambda bits: float(np.tanh(bits @ a) + 0.5 * np.sin(bits @ c))     # interactions of every order
    vals = np.array([f(np.array([(m >> j) & 1 for j in range(n)], dtype=np.float64)) for m in range(1 << n)])
    exact = shapley.exact_shapley(vals, n)
    err = {}
    for sat in (False, True):
        e = []
        for seed in range(6):
            Z, w, sz = sampling.sample(n, 510, seed, 1, saturate=sat)
            bits = sampling.unpack_rows(Z, n)
            idx = (bits.astype(np.int64) << np.arange(n)).sum(axis=1)
            e.append(np.abs(solve.solve_lstsq(bits, w, vals[idx]) - exact).max())
        err[sat] = np.mean(e)
    assert err[True] < 0.6 * err[False]
