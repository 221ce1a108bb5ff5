"""Pins for the CPU oracle: each test fixes the oracle to something other than itself.

Citations are to the paper's Section 3.1 (objective, E-step, M-step, codes, reconstruction),
Section 3.2 / Eq. 1 / Table 1 (size accounting) and Appendix B.1 (iteration count).
None of these tests needs a GPU.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads


# ------------------------------------------------------------------ E-step: exact rational brute force

def _exact_top2(X, C):
    """All N*K squared distances as exact rationals (floats are dyadic rationals), sorted by (D, k)."""
    out = []
    for x in X:
        xs = [Fraction(float(v)) for v in x]
        ds = []
        for k, c in enumerate(C):
            D = sum((a - Fraction(float(b))) ** 2 for a, b in zip(xs, c))
            ds.append((D, k))
        ds.sort()
        out.append(ds[:2])
    return out


@pytest.mark.parametrize("d", [4, 8, 16, 3, 5, 6, 7, 9])  # the paper's g runs over 4..9 (Table 1 and its ablations)
@pytest.mark.parametrize("seed", [0, 1])
def test_assign_top2_equals_exact_rational_bruteforce(d, seed):
    X, C = workloads.make_small(N=40, d=d, K=7, seed=100 + seed)
    # plant exact ties: a duplicated centroid, and a vector exactly half-way between two centroids
    C[5] = C[2]
    X[3] = (C[0] + C[1]) / 2  # exact in fp32: fp16-representable operands
    X[4] = C[6]               # a zero distance
    k1, D1, k2, D2 = oracle.assign_top2(X, C)
    ref = _exact_top2(X, C)
    for i, ((Da, ka), (Db, kb)) in enumerate(ref):
        assert k1[i] == ka and k2[i] == kb, (i, k1[i], k2[i], ka, kb)
        assert D1[i] == pytest.approx(float(Da), rel=1e-14, abs=0)
        assert D2[i] == pytest.approx(float(Db), rel=1e-14, abs=0)
    assert D1[4] == 0.0
    # duplicated centroid: whenever 2 or 5 wins, it is 2 (lowest index on ties)
    assert not np.any(k1 == 5)


def test_assign_single_centroid_has_no_runner_up():
    X, C = workloads.make_small(N=16, d=4, K=1, seed=3)
    k1, D1, k2, D2 = oracle.assign_top2(X, C)
    assert np.all(k1 == 0) and np.all(k2 == np.iinfo(np.uint32).max) and np.all(np.isinf(D2))
    np.testing.assert_allclose(D1, ((X.astype(np.float64) - C[0].astype(np.float64)) ** 2).sum(1), rtol=1e-15)


# ------------------------------------------------------------------ E-step: kd-tree library query

@pytest.mark.parametrize("d,N,K", [(4, 30000, 1024), (8, 8000, 512), (16, 3000, 300), (6, 9000, 500), (9, 5000, 400)])
def test_assign_top2_matches_kdtree(d, N, K):
    from scipy.spatial import cKDTree

    X, C = workloads.make_small(N=N, d=d, K=K, seed=7 + d)
    k1, D1, k2, D2 = oracle.assign_top2(X, C)
    dist, nn = cKDTree(C.astype(np.float64)).query(X.astype(np.float64), k=2)
    np.testing.assert_allclose(np.sqrt(D1), dist[:, 0], rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(np.sqrt(D2), dist[:, 1], rtol=1e-12, atol=1e-300)
    clear = (D2 - D1) > 1e-12 * D2
    assert clear.mean() > 0.9
    assert np.array_equal(k1[clear], nn[clear, 0].astype(np.uint32))
    # the runner-up index is compared only through its distance (a tie for second place may reorder it)
    d2 = ((X.astype(np.float64) - C[k2].astype(np.float64)) ** 2).sum(1)
    np.testing.assert_allclose(d2, dist[:, 1] ** 2, rtol=1e-12, atol=1e-300)
    # vectors that ARE centroids (the seeded subset) sit at distance exactly zero
    assert (D1 == 0.0).sum() >= K


# ------------------------------------------------------------------ M-step

def test_update_is_the_grouped_mean_and_keeps_empty_clusters():
    X, C = workloads.make_small(N=5000, d=8, K=37, seed=11)
    rng = np.random.default_rng(5)
    idx = rng.integers(0, 30, size=X.shape[0]).astype(np.uint32)  # clusters 30..36 stay empty
    out, counts = oracle.update(X, idx, C)
    n = np.bincount(idx, minlength=37)
    assert np.array_equal(counts, n.astype(np.uint32))
    for j in range(8):
        s = np.bincount(idx, weights=X[:, j].astype(np.float64), minlength=37)
        want = (s[:30] / n[:30]).astype(np.float32)
        got = out[:30, j]
        # bincount may add in another order: allow one fp32 ulp around the fp64 mean
        assert np.all(np.abs(got.astype(np.float64) - want) <= np.spacing(np.abs(want)).astype(np.float64))
    assert np.array_equal(out[30:], C[30:])  # empty: previous centroid kept, bit for bit


def test_update_of_identical_members_is_that_vector_exactly():
    rng = np.random.default_rng(2)
    pool = (rng.standard_normal((9, 4)) * 0.02).astype(np.float16).astype(np.float32)
    idx = rng.integers(0, 9, size=4000).astype(np.uint32)
    idx[:9] = np.arange(9)
    X = pool[idx]
    out, counts = oracle.update(X, idx, np.zeros_like(pool))
    assert np.array_equal(out, pool)
    assert counts.sum() == 4000


def test_update_hand_worked_example():
    # two clusters on a line, worked by hand: means (1+2+6)/3 = 3 and (10+20)/2 = 15
    X = np.array([[1, 0, 0, 0], [10, 0, 0, 0], [2, 0, 0, 0], [20, 4, 0, 0], [6, 3, 0, 0]], np.float32)
    idx = np.array([0, 1, 0, 1, 0], np.uint32)
    out, counts = oracle.update(X, idx, np.full((3, 4), 7, np.float32))
    assert np.array_equal(out, np.array([[3, 1, 0, 0], [15, 2, 0, 0], [7, 7, 7, 7]], np.float32))
    assert counts.tolist() == [3, 2, 0]


# ------------------------------------------------------------------ Lloyd loop

def test_fit_equals_manual_composition_and_history_is_the_objective():
    X, C0 = workloads.make_small(N=6000, d=4, K=64, seed=21)
    C, idx, J, hist = oracle.kmeans_fit(X, C0, 6)
    Cm = C0.copy()
    for t in range(6):
        k1, D1, _, _ = oracle.assign_top2(X, Cm)
        assert hist[t] == pytest.approx(float(D1.sum()), rel=1e-13)
        assert hist[t] == pytest.approx(oracle.inertia(X, Cm, k1), rel=1e-13)
        Cm, _ = oracle.update(X, k1, Cm)
    assert np.array_equal(Cm, C)
    k1, D1, _, _ = oracle.assign_top2(X, C)
    assert np.array_equal(k1, idx)
    assert J == hist[6] == pytest.approx(float(D1.sum()), rel=1e-13)


@pytest.mark.parametrize("d,K", [(4, 256), (8, 100), (16, 33), (6, 77), (9, 50)])
def test_inertia_never_increases(d, K):
    X, C0 = workloads.make_small(N=20000, d=d, K=K, seed=31 + d)
    C0[1] = C0[0]  # a duplicate seed: cluster 1 is empty at the first E-step and must keep its value
    C, idx, J, hist = oracle.kmeans_fit(X, C0, 12)
    assert np.all(np.diff(hist) <= 1e-12 * hist[:-1]), hist
    assert hist[-1] < 0.9 * hist[0]
    k1, _, _, _ = oracle.assign_top2(X, C0)
    assert not np.any(k1 == 1)
    C1, _, _, _ = oracle.kmeans_fit(X, C0, 1)
    assert np.array_equal(C1[1], C0[1]) and not np.array_equal(C1[0], C0[0])


def test_single_cluster_is_the_global_mean():
    X, _ = workloads.make_small(N=5000, d=8, K=1, seed=41)
    C0 = np.full((1, 8), 0.5, np.float32)
    C, idx, J, hist = oracle.kmeans_fit(X, C0, 3)
    mean = X.astype(np.float64).mean(0)
    assert np.all(np.abs(C[0].astype(np.float64) - mean) <= np.spacing(np.abs(mean).astype(np.float32)))
    assert np.all(idx == 0)
    want = ((X.astype(np.float64) - C[0].astype(np.float64)) ** 2).sum()
    assert J == pytest.approx(want, rel=1e-12)
    # sum of squares about the mean = N * d * (population variance averaged over components)
    assert J == pytest.approx(X.shape[0] * X.astype(np.float64).var(0).sum(), rel=1e-6)


def test_every_vector_its_own_centroid_gives_zero_inertia():
    X, _ = workloads.make_small(N=300, d=4, K=1, seed=43)
    C, idx, J, hist = oracle.kmeans_fit(X, X.copy(), 4)
    assert J == 0.0 and np.all(hist == 0.0)
    assert np.array_equal(C[idx], X)
    # duplicates (if any) resolve to their first occurrence
    first = np.array([np.flatnonzero((X == x).all(1))[0] for x in X], np.uint32)
    assert np.array_equal(idx, first)


def test_zero_inertia_when_every_distinct_vector_is_a_centroid():
    rng = np.random.default_rng(47)
    pool = np.unique((rng.standard_normal((50, 4)) * 0.02).astype(np.float16).astype(np.float32), axis=0)
    X = pool[rng.integers(0, len(pool), size=7000)]
    extra = (rng.standard_normal((14, 4)) * 5 + 40).astype(np.float16).astype(np.float32)  # far away, stay empty
    C0 = np.concatenate([extra[:7], pool, extra[7:]])
    C, idx, J, hist = oracle.kmeans_fit(X, C0, 5)
    assert J == 0.0 and np.all(hist == 0.0)
    assert np.array_equal(C, C0)  # members equal their centroid, empty clusters keep theirs
    assert np.array_equal(oracle.decode(C, idx), X)


def test_fixed_point_and_resume_by_chaining():
    X, C0 = workloads.make_small(N=3000, d=4, K=5, seed=53)
    Ca, ia, Ja, ha = oracle.kmeans_fit(X, C0, 60)
    Cb, ib, Jb, hb = oracle.kmeans_fit(X, Ca, 1)
    if np.array_equal(ia, ib):  # converged: a further step changes nothing
        assert np.array_equal(Ca, Cb) and Ja == Jb
    C1, _, _, _ = oracle.kmeans_fit(X, C0, 4)
    C2, i2, J2, _ = oracle.kmeans_fit(X, C1, 3)
    C7, i7, J7, _ = oracle.kmeans_fit(X, C0, 7)
    assert np.array_equal(C2, C7) and np.array_equal(i2, i7) and J2 == J7


def test_library_lloyd_agrees_on_tie_free_data():
    from sklearn.cluster import KMeans

    rng = np.random.default_rng(59)
    centers = rng.standard_normal((12, 4)) * 4
    X = (centers[rng.integers(0, 12, 4000)] + 0.3 * rng.standard_normal((4000, 4))).astype(np.float32)
    C0 = X[rng.choice(4000, 12, replace=False)].copy()
    C, idx, J, hist = oracle.kmeans_fit(X, C0, 8)
    assert np.bincount(idx, minlength=12).min() > 0
    km = KMeans(n_clusters=12, init=C0.astype(np.float64), n_init=1, max_iter=8, tol=0.0, algorithm="lloyd")
    km.fit(X.astype(np.float64))
    # the library re-labels once after its last update, as the oracle does; it may stop early when converged
    assert np.array_equal(km.labels_.astype(np.uint32), idx) or km.n_iter_ < 8
    k1, D1, _, _ = oracle.assign_top2(X, km.cluster_centers_.astype(np.float32))
    assert float(D1.sum()) == pytest.approx(km.inertia_, rel=1e-5)
    if km.n_iter_ == 8:
        np.testing.assert_allclose(C, km.cluster_centers_, rtol=1e-5, atol=1e-6)
        assert J == pytest.approx(km.inertia_, rel=1e-6)


# ------------------------------------------------------------------ reconstruction

def test_decode_is_a_row_gather_and_inertia_is_the_reconstruction_error():
    X, C0 = workloads.make_small(N=9000, d=16, K=128, seed=61)
    C, idx, J, _ = oracle.kmeans_fit(X, C0, 3)
    W = oracle.decode(C, idx)
    assert W.dtype == np.float32 and W.shape == X.shape
    assert W.tobytes() == C[idx].tobytes()
    assert J == pytest.approx(((X.astype(np.float64) - W.astype(np.float64)) ** 2).sum(), rel=1e-12)
    # reshaped back to the matrix: row-major view, as the paper's layer does with .view(in_features, -1)
    R = 90
    assert np.array_equal(W.reshape(R, -1), C[idx.reshape(R, -1)].reshape(R, -1))


# ------------------------------------------------------------------ size accounting (Eq. 1, Table 1)

def _rows(golden_dir):
    with open(os.path.join(golden_dir, "table1_bits_per_parameter.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                yield line.split()


def test_bits_per_parameter_reproduces_table_1(golden_dir):
    seen = 0
    for d_in, d_out, g, n, codes_m, cb_m, cb_pct, bits in _rows(golden_dir):
        d_in, d_out, g, n = int(d_in), int(d_out), int(g), int(n)
        k, cb = oracle.parameter_counts(d_in, d_out, g, n)
        b = oracle.bits_per_parameter(d_in, d_out, g, n)
        assert round(b, 2) == float(bits)
        assert b == pytest.approx(16 / g + 16 * g * n / (d_in * d_out), rel=1e-15)  # right-hand form of Eq. 1
        if codes_m != "-":
            assert round(k / 1e6, 2) == float(codes_m)
            assert round(cb / 1e6, 2) == float(cb_m)
            # the printed percentage is the ratio of the two PRINTED (rounded) figures, 0.26M / 16.78M etc.
            total_m = round(d_in * d_out / 1e6, 2)
            assert total_m == 16.78
            assert round(100 * round(cb / 1e6, 2) / total_m, 2) == float(cb_pct)
            assert abs(100 * cb / (d_in * d_out) - float(cb_pct)) < 0.03
        seen += 1
    assert seen == 4


def test_code_bits_per_weight_of_the_benchmark_configs():
    want = {1: 2.0, 2: 3.0, 3: 4.0, 4: 2.0, 5: 1.0}
    for w in workloads.WORKLOADS.values():
        assert oracle.code_bits_per_weight(w.K, w.d) == want[w.number] == w.code_bits_per_weight
        # codes term of Eq. 1 with 16-bit codes is 16/g; packed codes cost log2(n)/g <= 16/g for n <= 2^16
        assert oracle.code_bits_per_weight(w.K, w.d) <= 16 / w.d
