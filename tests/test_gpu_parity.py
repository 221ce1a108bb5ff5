"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Sizes here are ones the oracle finishes in seconds while still spanning several centroid tiles,
several workgroups and ragged tails. Full-size configurations are in test_gpu_fullsize.py.
"""
import numpy as np
import pytest

import oracle
import workloads
from tests import parity

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def g():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_helpers

    return gpu_helpers


@pytest.fixture(params=[0, 1, 2, 3], ids=["auto", "direct", "fp32-mfma", "auto-unpruned"])
def mode(request, g):
    """Runs a test once per E-step selection: 0 = automatic (fp16 MFMA for these fp16-representable inputs when
    K >= 128, norm-window pruning when K >= 8192 or in long fits of many vectors), 1 = direct form only,
    2 = fp32 MFMA + guard band + refinement, 3 = automatic without pruning."""
    import paper_2503_13089_amd as cc

    cc.set_assign_mode(request.param)
    yield request.param
    cc.set_assign_mode(0)


SHAPES = [  # (N, d, K): ragged in N (not a multiple of 256/512/1024) and in K (not a multiple of any tile)
    (70001, 4, 1500),
    (30011, 8, 777),
    (20003, 16, 515),
    (4099, 4, 4099),   # K == N: every vector is a centroid
    (513, 8, 1),       # a single centroid
    (1, 4, 1),         # the smallest legal problem
    (65536, 4, 256),   # cfg1's shape
    (40003, 4, 9001),  # K large enough for the norm-window pruning of the automatic mode
    (20011, 8, 8200),
    # sub-vector lengths other than 4, 8, 16 (the paper's g runs over 4..9): zero-padded inside the library
    (30007, 6, 700),
    (20011, 5, 8300),
    (9001, 9, 300),
    (5003, 7, 129),
    (777, 3, 50),
    (6007, 12, 200),
]


@pytest.mark.parametrize("N,d,K", SHAPES)
def test_decode_is_bit_exact(g, N, d, K):
    rng = np.random.default_rng(N + d + K)
    C = rng.standard_normal((K, d)).astype(np.float32)
    C.view(np.uint32)[::7] ^= 0x7  # arbitrary bit patterns, not just "nice" floats
    idx = rng.integers(0, K, size=N).astype(np.uint32)
    print(f"decode N={N} d={d} K={K}", flush=True)
    out = g.gpu_decode(C, idx)
    assert out.tobytes() == oracle.decode(C, idx).tobytes()


def test_decode_clamps_out_of_range_codes(g):
    C = np.arange(40, dtype=np.float32).reshape(10, 4)
    idx = np.array([0, 9, 10, 4000000000, 3], np.uint32)
    out = g.gpu_decode(C, idx)
    assert np.array_equal(out, C[[0, 9, 9, 9, 3]])


@pytest.mark.parametrize("N,d,K", SHAPES)
def test_assign_lockstep(g, mode, N, d, K):
    X, C0 = workloads.make_small(N, d, K, seed=1000 + N)
    # centroids after one oracle step: general fp32 values rather than copies of inputs
    k0, _, _, _ = oracle.assign_top2(X, C0)
    C, _ = oracle.update(X, k0, C0)
    for cents in (C0, C):
        k1, D1, k2, D2 = oracle.assign_top2(X, cents)
        print(f"assign N={N} d={d} K={K}", flush=True)
        idx, J = g.gpu_assign(X, cents)
        parity.check_assignment(X, cents, idx, k1, D1, D2)
        parity.check_inertia(J, float(D1.sum()))
        idx2, none = g.gpu_assign(X, cents, want_inertia=False)
        assert none is None and np.array_equal(idx, idx2)


def test_assign_general_fp32_inputs(g, mode):
    """Inputs that are not fp16 numbers: the automatic selection must fall back to the fp32 kernels."""
    X, C0 = workloads.make_small(60001, 8, 1300, seed=4242, fp16_round=False)
    k0, _, _, _ = oracle.assign_top2(X, C0)
    C, _ = oracle.update(X, k0, C0)
    k1, D1, _, D2 = oracle.assign_top2(X, C)
    idx, J = g.gpu_assign(X, C)
    parity.check_assignment(X, C, idx, k1, D1, D2)
    parity.check_inertia(J, float(D1.sum()))


@pytest.mark.parametrize("N,d,K", SHAPES)
def test_lloyd_iter_equals_assign_then_update(g, mode, N, d, K):
    import paper_2503_13089_amd as cc

    X, C0 = workloads.make_small(N, d, K, seed=7000 + N)
    Xd = g.dev(X)
    ws = g.workspace(N, d, K)
    idx_a, J_a = g.gpu_assign(Xd, C0, ws=ws)
    C_a, counts_a, _ = g.gpu_update(Xd, idx_a, C0, ws=ws)
    Cd = g.dev(C0)
    idx_d = torch.empty(N, dtype=torch.uint32, device="cuda")
    counts_d = torch.empty(K, dtype=torch.uint32, device="cuda")
    J_d = torch.zeros(1, dtype=torch.float64, device="cuda")
    print(f"lloyd_iter N={N} d={d} K={K}", flush=True)
    cc.lloyd_iter(Xd, Cd, idx_d, J_d, counts_d, ws)
    torch.cuda.synchronize()
    assert np.array_equal(idx_d.cpu().numpy(), idx_a)
    assert np.array_equal(counts_d.cpu().numpy(), counts_a)
    assert Cd.cpu().numpy().tobytes() == C_a.tobytes()
    assert float(J_d.item()) == J_a
    # and against the oracle's M-step on those codes
    want, counts = oracle.update(X, idx_a, C0)
    assert C_a.tobytes() == want.tobytes() and np.array_equal(counts_a, counts)


def test_assign_exact_ties_take_the_lowest_index(g, mode):
    X, C = workloads.make_small(5000, 4, 64, seed=77)
    C[40] = C[3]
    C[63] = C[3]
    idx, _ = g.gpu_assign(X, C)
    k1, D1, _, D2 = oracle.assign_top2(X, C)
    assert (k1 == 3).any() and not np.isin(idx, [40, 63]).any()
    assert np.array_equal(idx, k1) or parity.check_assignment(X, C, idx, k1, D1, D2) >= 0


@pytest.mark.parametrize("N,d,K", SHAPES)
def test_update_lockstep(g, N, d, K):
    X, C0 = workloads.make_small(N, d, K, seed=2000 + N)
    k1, _, _, _ = oracle.assign_top2(X, C0)
    if K > 8:
        k1[k1 == 5] = 6  # force an empty cluster
    want, counts = oracle.update(X, k1, C0)
    print(f"update N={N} d={d} K={K}", flush=True)
    got, gcounts, stats = g.gpu_update(X, k1, C0)
    assert np.array_equal(gcounts, counts)
    assert stats.skipped_vectors == 0
    # fp16-representable inputs: the fixed-point sums are exact, so the means match bit for bit
    assert stats.fixed_point_exp >= 24
    assert got.tobytes() == want.tobytes()
    if K > 8:
        assert np.array_equal(got[5], C0[5])


@pytest.mark.parametrize("N,d,K", [(1048576 + 1235, 4, 5000), (1048576 + 77, 8, 65536), (1100003, 16, 2049), (1048576, 4, 70),
                                   (1200001, 6, 9001)])
def test_update_by_slices_matches_the_oracle(g, N, d, K):
    """From 2^20 vectors on the M-step runs by cluster slices (LDS accumulators, one pass over the codes per slice):
    ragged vector ranges, a last slice that is not full, slices that no vector falls into, codes out of range."""
    rng = np.random.default_rng(N + K)
    X = (rng.standard_normal((N, d)) * 0.02).astype(np.float16).astype(np.float32)
    idx = rng.integers(0, K, size=N).astype(np.uint32)
    idx[rng.integers(0, N, size=N // 3)] = rng.integers(0, max(1, K // 50))   # a crowded low slice
    empty = np.unique(rng.integers(0, K, size=5))
    idx[np.isin(idx, empty)] = (empty[0] + 1) % K if K > 1 else 0              # some clusters without members
    prev = rng.standard_normal((K, d)).astype(np.float32)
    print(f"update by slices N={N} d={d} K={K}", flush=True)
    want, counts = oracle.update(X, idx, prev)
    got, gcounts, stats = g.gpu_update(X, idx, prev)
    assert stats.skipped_vectors == 0 and np.array_equal(gcounts, counts)
    assert got.tobytes() == want.tobytes()
    # codes >= K are skipped and counted
    bad = idx.copy()
    where = rng.choice(N, size=11, replace=False)
    bad[where] = K + rng.integers(0, 1000, size=11).astype(np.uint32)
    keep = np.ones(N, bool)
    keep[where] = False
    want2, counts2 = oracle.update(X[keep], idx[keep], prev)
    got2, gcounts2, stats2 = g.gpu_update(X, bad, prev)
    assert stats2.skipped_vectors == 11 and np.array_equal(gcounts2, counts2)
    assert got2.tobytes() == want2.tobytes()


def test_update_general_fp32_inputs_and_bad_codes(g):
    X, C0 = workloads.make_small(50000, 8, 300, seed=5, fp16_round=False)
    X[:100] *= 1e-6   # a wide dynamic range
    X[100:110] *= 300
    k1, _, _, _ = oracle.assign_top2(X, C0)
    want, counts = oracle.update(X, k1, C0)
    got, gcounts, stats = g.gpu_update(X, k1, C0)
    assert np.array_equal(gcounts, counts)
    parity.check_centroids(got, want, X)
    bad = k1.copy()
    bad[7] = 300
    bad[9] = 2**31
    keep = np.ones(len(bad), bool)
    keep[[7, 9]] = False
    want2, counts2 = oracle.update(X[keep], k1[keep], C0)
    got2, gcounts2, stats2 = g.gpu_update(X, bad, C0)
    assert stats2.skipped_vectors == 2
    assert np.array_equal(gcounts2, counts2)
    parity.check_centroids(got2, want2, X)


@pytest.mark.parametrize("N,d,K,iters", [(65536, 4, 256, 10), (30011, 8, 777, 5), (20003, 16, 515, 4), (3000, 4, 3000, 2),
                                         (50021, 4, 8500, 4), (30011, 6, 500, 4), (20003, 9, 8200, 3)])
def test_fit_trajectory_following(g, mode, N, d, K, iters):
    """Free-running GPU fit, every step verified: the oracle checks each assignment against the GPU's
    own centroids, adopts the GPU's choice on near-ties, and recomputes the update."""
    if (N, d, K) == (65536, 4, 256):
        X, C0 = workloads.make_inputs(workloads.by_number(1))
    else:
        X, C0 = workloads.make_small(N, d, K, seed=3000 + N)
    Xd = g.dev(X)
    ws = g.workspace(N, d, K)
    C = C0.copy()
    near_total = 0
    for t in range(iters):
        print(f"trajectory N={N} d={d} K={K} step {t}", flush=True)
        idx_t, J_t = g.gpu_assign(Xd, C, ws=ws)
        k1, D1, _, D2 = oracle.assign_top2(X, C)
        near_total += parity.check_assignment(X, C, idx_t, k1, D1, D2)
        parity.check_inertia(J_t, oracle.inertia(X, C, idx_t))
        want_next, _ = oracle.update(X, idx_t, C)
        C_next, idx_next, J_next, stats = g.gpu_fit(X, C, 1, ws=ws, Xd=Xd)
        assert stats.assign_calls == 2
        assert C_next.tobytes() == want_next.tobytes()  # exact sums on fp16-representable inputs
        idx_chk, J_chk = g.gpu_assign(Xd, C_next, ws=ws)
        assert np.array_equal(idx_next, idx_chk) and J_next == J_chk
        C = C_next
    # one call with iters=T gives the same bits as T chained calls with iters=1
    C_T, idx_T, J_T, _ = g.gpu_fit(X, C0, iters, ws=ws, Xd=Xd)
    assert C_T.tobytes() == C.tobytes()
    assert np.array_equal(idx_T, idx_next) and J_T == J_next
    # and again (determinism)
    C_T2, idx_T2, J_T2, _ = g.gpu_fit(X, C0, iters, Xd=Xd)
    assert C_T2.tobytes() == C_T.tobytes() and np.array_equal(idx_T2, idx_T) and J_T2 == J_T
    print(f"near-tie divergences adopted: {near_total}")


def test_fit_end_to_end_cfg1(g, mode):
    w = workloads.by_number(1)
    X, C0 = workloads.make_inputs(w)
    C_or, idx_or, J_or, hist = oracle.kmeans_fit(X, C0, w.iters)
    C, idx, J, stats = g.gpu_fit(X, C0, w.iters)
    assert stats.assign_calls == w.iters + 1
    parity.check_inertia(J, J_or)
    assert J == pytest.approx(oracle.inertia(X, C, idx), rel=1e-6)
    out = g.gpu_decode(C, idx)
    assert out.tobytes() == C[idx].tobytes()
    assert J == pytest.approx(((X.astype(np.float64) - out) ** 2).sum(), rel=1e-6)
    # centroid agreement is guaranteed only if no near-tie was resolved differently along the way
    same = np.array_equal(idx, idx_or)
    if same:
        parity.check_centroids(C, C_or, X)
    frac = np.mean(np.linalg.norm(C - C_or, axis=1) <= 1e-4 * np.linalg.norm(C_or, axis=1) + 1e-9)
    print(f"cfg1 end-to-end: identical codes={same}, centroids within tolerance={frac:.4f}")
    assert frac > 0.95


def test_fit_iters_zero_and_aliasing(g, mode):
    X, C0 = workloads.make_small(9000, 4, 100, seed=9)
    C, idx, J, stats = g.gpu_fit(X, C0, 0)
    assert C.tobytes() == C0.tobytes() and stats.assign_calls == 1
    k1, D1, _, D2 = oracle.assign_top2(X, C0)
    parity.check_assignment(X, C0, idx, k1, D1, D2)
    parity.check_inertia(J, float(D1.sum()))
    # centroids aliasing init_centroids
    import paper_2503_13089_amd as cc

    Xd, Cd = g.dev(X), g.dev(C0)
    ws = g.workspace(9000, 4, 100)
    idx_d = torch.empty(9000, dtype=torch.uint32, device="cuda")
    cc.kmeans_fit(Xd, 100, 3, Cd, Cd, idx_d, None, ws)
    torch.cuda.synchronize()
    C3, idx3, _, _ = g.gpu_fit(X, C0, 3)
    assert Cd.cpu().numpy().tobytes() == C3.tobytes() and np.array_equal(idx_d.cpu().numpy(), idx3)


def test_zero_inertia_when_every_distinct_vector_is_a_centroid(g, mode):
    rng = np.random.default_rng(47)
    pool = np.unique((rng.standard_normal((200, 8)) * 0.02).astype(np.float16).astype(np.float32), axis=0)
    X = pool[rng.integers(0, len(pool), size=50000)]
    C, idx, J, _ = g.gpu_fit(X, pool, 3)
    assert J == 0.0
    assert np.array_equal(g.gpu_decode(C, idx), X)


@pytest.mark.parametrize("N,d,K", [(60013, 4, 9000), (30007, 8, 8192), (25013, 16, 8300)])
def test_pruned_estep_is_bit_identical_whatever_the_hint(g, N, d, K):
    """The automatic mode visits only a norm window of the codebook, sized from the codes a previous call left in
    the workspace. The hint may be fresh, stale or absent: the codes must be the same bits as without pruning."""
    import paper_2503_13089_amd as cc

    X, C0 = workloads.make_small(N, d, K, seed=8800 + N)
    k0, _, _, _ = oracle.assign_top2(X, C0)
    C1, _ = oracle.update(X, k0, C0)
    rng = np.random.default_rng(1)
    C2 = (C1 * rng.uniform(0.5, 1.5, size=(K, 1))).astype(np.float32)  # very different norms: a useless hint for C1
    Xd = g.dev(X)
    try:
        cc.set_assign_mode(3)
        ref_idx, ref_J = g.gpu_assign(Xd, C1)
        cc.set_assign_mode(0)
        ws = g.workspace(N, d, K)
        fresh_idx, fresh_J = g.gpu_assign(Xd, C1, ws=ws)      # no hint yet: whole codebook
        hinted_idx, hinted_J = g.gpu_assign(Xd, C1, ws=ws)    # hint = the exact codes: tightest windows
        st = cc.read_stats(ws)
        assert 0 < st.scored_stages <= st.total_stages
        g.gpu_assign(Xd, C2, ws=ws)                           # leaves codes for another codebook behind
        stale_idx, stale_J = g.gpu_assign(Xd, C1, ws=ws)      # stale hint
        Xs = g.dev(X[::-1].copy())                            # other vectors on the same workspace: misaligned hint
        g.gpu_assign(Xs, C2, ws=ws)
        mis_idx, mis_J = g.gpu_assign(Xd, C1, ws=ws)
    finally:
        cc.set_assign_mode(0)
    for name, idx, J in (("fresh", fresh_idx, fresh_J), ("hinted", hinted_idx, hinted_J), ("stale", stale_idx, stale_J),
                         ("misaligned", mis_idx, mis_J)):
        assert np.array_equal(idx, ref_idx), name
        assert J == pytest.approx(ref_J, rel=1e-12), name  # same terms, summed in norm order instead of input order
    k1, D1, _, D2 = oracle.assign_top2(X, C1)
    parity.check_assignment(X, C1, ref_idx, k1, D1, D2)
    if d == 4:
        assert st.scored_stages < 0.9 * st.total_stages  # at 4 dimensions the windows really are narrower


@pytest.mark.parametrize("N,d,K,iters", [(530011, 4, 300, 6), (524288, 8, 1025, 5), (540001, 6, 256, 5)])
def test_windowed_fit_with_a_small_codebook(g, N, d, K, iters):
    """With at least 2^19 vectors and 5 iterations a fit takes the windowed E-step and the incremental M-step from
    256 centroids on. Its codes and centroids must be the bits of the whole-codebook fit, and the final assignment
    must be the oracle's argmin for the final centroids."""
    import paper_2503_13089_amd as cc

    X, C0 = workloads.make_small(N, d, K, seed=4100 + K)
    Xd = g.dev(X)
    try:
        cc.set_assign_mode(3)
        C_ref, idx_ref, J_ref, _ = g.gpu_fit(X, C0, iters, Xd=Xd)
        cc.set_assign_mode(0)
        ws = g.workspace(N, d, K)
        C, idx, J, st = g.gpu_fit(X, C0, iters, ws=ws, Xd=Xd)
        C_short, _, _, st_short = g.gpu_fit(X, C0, iters - 1 if iters == 5 else 4, Xd=Xd)  # below 5 iterations: no windows
    finally:
        cc.set_assign_mode(0)
    assert 0 < st.scored_stages < st.total_stages
    assert st_short.scored_stages == st_short.total_stages or st_short.total_stages == 0
    assert C.tobytes() == C_ref.tobytes() and np.array_equal(idx, idx_ref)
    assert J == pytest.approx(J_ref, rel=1e-12)
    k1, D1, _, D2 = oracle.assign_top2(X, C)
    parity.check_assignment(X, C, idx, k1, D1, D2)
    parity.check_inertia(J, oracle.inertia(X, C, idx))
    # the oracle's own trajectory from the same start: same objective within the near-tie allowance
    _, _, J_or, _ = oracle.kmeans_fit(X, C0, iters)
    assert J == pytest.approx(J_or, rel=1e-3)


def _awkward_vectors(N, d, rng):
    """fp16-representable vectors built to stress the window logic: seven orders of magnitude in norm, exact zeros,
    vectors along +-e = (1,..,1)/sqrt(d) (cosine +-1), duplicates, and one huge outlier."""
    scale = 10.0 ** rng.uniform(-6, 0, size=(N, 1))
    X = (rng.standard_normal((N, d)) * scale).astype(np.float16).astype(np.float32)
    X[::97] = 0.0
    X[5::101] = np.float32(0.03125)        # exactly along e
    X[7::103] = np.float32(-0.0078125)     # exactly along -e
    X[11::107] = X[3]                      # duplicates
    X[13] = np.float32(2048.0)
    return np.ascontiguousarray(X)


@pytest.mark.parametrize("d,fp16", [(4, True), (8, True), (4, False)])
def test_pruned_estep_on_awkward_data(g, d, fp16):
    """Pruned (automatic) and unpruned runs must agree bit for bit, and with the oracle, on data with extreme norm
    ranges, zero vectors, vectors exactly along the projection direction, duplicates and an outlier; with fp16 = False
    the values are perturbed off the fp16 grid so that the fp32 MFMA variant runs under the same windows."""
    import paper_2503_13089_amd as cc

    rng = np.random.default_rng(31 + d)
    N, K = 70003, 8704
    X = _awkward_vectors(N, d, rng)
    if not fp16:
        X = (X * np.float32(1.0001)).astype(np.float32)
    C0 = np.ascontiguousarray(X[rng.choice(N, K, replace=False)])
    k0, _, _, _ = oracle.assign_top2(X, C0)
    C1, _ = oracle.update(X, k0, C0)
    Xd = g.dev(X)
    try:
        cc.set_assign_mode(3)
        ref = {}
        for name, C in (("init", C0), ("step", C1)):
            ref[name] = g.gpu_assign(Xd, C)
        cc.set_assign_mode(0)
        ws = g.workspace(N, d, K)
        for name, C in (("init", C0), ("step", C1), ("init", C0), ("step", C1), ("step", C1)):
            idx, J = g.gpu_assign(Xd, C, ws=ws)
            assert np.array_equal(idx, ref[name][0]), name
            assert J == pytest.approx(ref[name][1], rel=1e-12)
        # a whole fit: pruned (bootstrap, hints, M-step by sorting) against unpruned (fused atomics), bit for bit
        Cp, ip, Jp, stp = g.gpu_fit(X, C0, 4, ws=ws, Xd=Xd)
        cc.set_assign_mode(3)
        Cu, iu, Ju, _ = g.gpu_fit(X, C0, 4, Xd=Xd)
    finally:
        cc.set_assign_mode(0)
    assert Cp.tobytes() == Cu.tobytes() and np.array_equal(ip, iu) and Jp == pytest.approx(Ju, rel=1e-12)
    assert 0 < stp.scored_stages <= stp.total_stages
    for name, C in (("init", C0), ("step", C1)):
        k1, D1, _, D2 = oracle.assign_top2(X, C)
        parity.check_assignment(X, C, ref[name][0], k1, D1, D2)


@pytest.mark.parametrize("d", [4, 8])
def test_pruned_estep_with_norms_and_cosines_on_key_boundaries(g, d):
    """Small-integer lattice points scaled by powers of two: norms that are exactly the lower edge of a norm key or
    shell, cosines exactly on the edge of a cosine bucket, and exact ties everywhere. The window bounds carry only
    rounding-level slack, so this is where an off-by-one-cell would show: pruned and unpruned runs must agree bit
    for bit, and with the oracle."""
    import paper_2503_13089_amd as cc

    rng = np.random.default_rng(91 + d)
    N, K = 120000, 8704
    scale = np.exp2(rng.integers(-6, 1, size=(N, 1))).astype(np.float32)
    X = np.ascontiguousarray(rng.integers(-3, 4, size=(N, d)).astype(np.float32) * scale)
    distinct = np.unique(X, axis=0)
    assert len(distinct) >= K
    C0 = np.ascontiguousarray(distinct[rng.choice(len(distinct), K, replace=False)])
    k0, _, _, _ = oracle.assign_top2(X, C0)
    C1, _ = oracle.update(X, k0, C0)
    Xd = g.dev(X)
    try:
        ws = g.workspace(N, d, K)
        for C in (C0, C1):
            cc.set_assign_mode(3)
            ref, Jref = g.gpu_assign(Xd, C)
            cc.set_assign_mode(0)
            for _ in range(2):  # cold (guessed windows), then with the codes of the first call as the hint
                idx, J = g.gpu_assign(Xd, C, ws=ws)
                assert np.array_equal(idx, ref)
                assert J == pytest.approx(Jref, rel=1e-12)
            k1, D1, _, D2 = oracle.assign_top2(X, C)
            parity.check_assignment(X, C, ref, k1, D1, D2)
            if C is C0:  # lattice centroids: every distance is exact in fp32, so even the ties must match (lowest index)
                assert np.array_equal(ref, k1)
    finally:
        cc.set_assign_mode(0)


@pytest.mark.parametrize("case", ["centroids near the origin", "centroids far out", "one shell apart"])
def test_cold_estep_when_no_centroid_is_near_the_guess(g, case):
    """The first E-step on a workspace without codes guesses where each vector's neighbours are (a window around its
    own norm and projection). When the centroids lie somewhere else entirely - every guessed window empty - the guess
    only costs time: the codes are still the argmin over all centroids, bit for bit those of the unpruned run."""
    import paper_2503_13089_amd as cc

    rng = np.random.default_rng(77)
    N, d, K = 50021, 4, 8200
    X = (rng.standard_normal((N, d)) * 0.05).astype(np.float16).astype(np.float32)
    C = (rng.standard_normal((K, d))).astype(np.float32)
    if case == "centroids near the origin":
        C *= np.float32(1e-4)
    elif case == "centroids far out":
        C *= np.float32(30.0)
    else:  # all centroids on one thin shell just outside every guessed window of the bulk
        C = (C / np.linalg.norm(C, axis=1, keepdims=True) * 0.5).astype(np.float32)
    Xd = g.dev(X)
    try:
        cc.set_assign_mode(3)
        ref_idx, ref_J = g.gpu_assign(Xd, C)
        cc.set_assign_mode(0)
        ws = g.workspace(N, d, K)
        idx, J = g.gpu_assign(Xd, C, ws=ws)        # cold: guessed windows, then real ones
        idx2, J2 = g.gpu_assign(Xd, C, ws=ws)      # hinted
    finally:
        cc.set_assign_mode(0)
    assert np.array_equal(idx, ref_idx) and np.array_equal(idx2, ref_idx)
    assert J == pytest.approx(ref_J, rel=1e-12) and J2 == pytest.approx(ref_J, rel=1e-12)
    k1, D1, _, D2 = oracle.assign_top2(X, C)
    parity.check_assignment(X, C, idx, k1, D1, D2)


@pytest.mark.parametrize("d,K", [(4, 1300), (8, 700), (16, 300), (4, 8300)])
def test_bf16_weights_take_the_fp16_kernels(g, d, K):
    """bf16 weights are fp16 numbers except where they are tiny (below 2^-17 a bf16 number generally is not). Such
    inputs still go to the fp16 matrix-core kernels, whose guard band then carries what the operand lost; codes and
    objective must be those of the fp32 kernels and of the oracle."""
    import paper_2503_13089_amd as cc
    from oracle import layer as olayer

    rng = np.random.default_rng(500 + d)
    N = 60013
    X = olayer.bf16_round((rng.standard_normal((N, d)) * 0.02).astype(np.float32))
    X[::7, 0] = olayer.bf16_round((rng.standard_normal(len(X[::7])) * 1e-7).astype(np.float32))
    X[3::11, d - 1] = olayer.bf16_round((rng.standard_normal(len(X[3::11])) * 1e-12).astype(np.float32))
    X[5::13] = olayer.bf16_round((rng.standard_normal((len(X[5::13]), d)) * 3e-6).astype(np.float32))  # whole tiny vectors
    assert not np.array_equal(X.astype(np.float16).astype(np.float32), X)
    C0 = np.ascontiguousarray(X[rng.choice(N, K, replace=False)])
    k0, _, _, _ = oracle.assign_top2(X, C0)
    C1, _ = oracle.update(X, k0, C0)
    Xd = g.dev(X)
    ws = g.workspace(N, d, K)
    try:
        for C in (C0, C1):
            cc.set_assign_mode(0)
            idx, J = g.gpu_assign(Xd, C, ws=ws)
            assert cc.read_stats(ws).fp16_inputs == 1
            cc.set_assign_mode(2)
            idx32, J32 = g.gpu_assign(Xd, C)
            assert np.array_equal(idx, idx32) and J == pytest.approx(J32, rel=1e-12)
            k1, D1, _, D2 = oracle.assign_top2(X, C)
            parity.check_assignment(X, C, idx, k1, D1, D2)
            parity.check_inertia(J, float(D1.sum()))
        cc.set_assign_mode(0)
        Cf, idf, Jf, _ = g.gpu_fit(X, C0, 3, ws=ws, Xd=Xd)
        cc.set_assign_mode(2)
        Cg, idg, Jg, _ = g.gpu_fit(X, C0, 3, Xd=Xd)
    finally:
        cc.set_assign_mode(0)
    assert np.array_equal(idf, idg) and Cf.tobytes() == Cg.tobytes() and Jf == pytest.approx(Jg, rel=1e-12)
    # values of the fp16 normal range that are not fp16 numbers still send the call to the fp32 kernels
    X2 = X.copy()
    X2[1, 0] = np.float32(0.0200001)
    g.gpu_assign(g.dev(X2), C1, ws=ws)
    assert cc.read_stats(ws).fp16_inputs == 0


@pytest.mark.parametrize("d", [8, 16, 6, 12])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_many_near_ties_at_longer_vectors(g, d, seed):
    """At d = 8 and 16 the fp16 kernel splits a centroid component into two parts and carries the 2^-22 residual in
    its guard band. Vectors on a coarse lattice and centroids that are means of a few of them make exact ties and
    near-ties by the thousand, where a band that is too narrow shows as a wrong code: the codes must be those of the
    fp32 kernels and of the oracle, for the initial centroids and after an update, with and without windows."""
    import paper_2503_13089_amd as cc

    rng = np.random.default_rng(9000 + 10 * d + seed)
    N, K = 90001, 8300 if seed == 1 else 1900
    scale = np.float32(2.0 ** -(4 + seed))
    X = (rng.integers(-24, 25, size=(N, d)).astype(np.float32) * scale)
    X[::5] *= np.float32(0.125)       # a second, finer lattice: short and long vectors side by side
    C0 = np.ascontiguousarray(X[rng.choice(N, K, replace=False)])
    k0, _, _, _ = oracle.assign_top2(X, C0)
    C1, _ = oracle.update(X, k0, C0)
    Xd = g.dev(X)
    ws = g.workspace(N, d, K)
    try:
        for C in (C0, C1):
            k1, D1, _, D2 = oracle.assign_top2(X, C)
            cc.set_assign_mode(2)
            idx32, J32 = g.gpu_assign(Xd, C)
            for m in (0, 3):
                cc.set_assign_mode(m)
                idx, J = g.gpu_assign(Xd, C, ws=ws)
                assert cc.read_stats(ws).fp16_inputs == 1
                assert np.array_equal(idx, idx32), (m, int((idx != idx32).sum()))
                assert J == pytest.approx(J32, rel=1e-12)
                parity.check_assignment(X, C, idx, k1, D1, D2)
    finally:
        cc.set_assign_mode(0)


@pytest.mark.parametrize("seed", range(10))
def test_random_problem_fits_agree_with_and_without_windows(g, seed):
    """Seeded random shapes (d = 1..16, a few hundred to twelve thousand centroids, short and long fits, fp16- and
    bf16-valued vectors): the automatic path - windows, guessed bootstrap, incremental M-step where they apply -
    must return the bits of the whole-codebook path, and codes that are the oracle's argmin for the final centroids."""
    import paper_2503_13089_amd as cc
    from oracle import layer as olayer

    rng = np.random.default_rng(424200 + seed)
    d = int(rng.choice([1, 2, 3, 4, 4, 5, 6, 7, 8, 9, 12, 16]))
    big = seed % 3 == 0
    N = int(rng.integers(530000, 700000)) if big else int(rng.integers(9000, 150000))
    K = int(rng.integers(256, 2500)) if big else int(rng.choice([rng.integers(130, 4000), rng.integers(8192, 11000)]))
    K = min(K, N)
    iters = int(rng.integers(2, 8))
    X, C0 = workloads.make_small(N, d, K, seed=int(rng.integers(1 << 30)))
    if seed % 4 == 1:
        X = olayer.bf16_round(X * np.float32(1e-3))
        C0 = np.ascontiguousarray(X[rng.choice(N, K, replace=False)])
    print(f"random problem N={N} d={d} K={K} iters={iters}", flush=True)
    Xd = g.dev(X)
    try:
        cc.set_assign_mode(3)
        Cr, ir, Jr, _ = g.gpu_fit(X, C0, iters, Xd=Xd)
        cc.set_assign_mode(0)
        Cp, ip, Jp, _ = g.gpu_fit(X, C0, iters, Xd=Xd)
    finally:
        cc.set_assign_mode(0)
    assert Cp.tobytes() == Cr.tobytes() and np.array_equal(ip, ir)
    assert Jp == pytest.approx(Jr, rel=1e-12)
    k1, D1, _, D2 = oracle.assign_top2(X, Cp)
    parity.check_assignment(X, Cp, ip, k1, D1, D2)
    parity.check_inertia(Jp, oracle.inertia(X, Cp, ip))


def test_more_than_65536_clusters(g, mode):
    """K above the 16-bit code range: the M-step cannot use its bucket formulation there (the sums are accumulated
    by the E-step kernel, or by atomics), with and without the window pruning of the automatic mode."""
    import paper_2503_13089_amd as cc

    N, d, K = 90001, 4, 66001
    X, C0 = workloads.make_small(N, d, K, seed=4242)
    Xd = g.dev(X)
    ws = g.workspace(N, d, K)
    print(f"large K N={N} d={d} K={K}", flush=True)
    idx_a, J_a = g.gpu_assign(Xd, C0, ws=ws)
    k1, D1, _, D2 = oracle.assign_top2(X, C0)
    parity.check_assignment(X, C0, idx_a, k1, D1, D2)
    parity.check_inertia(J_a, float(D1.sum()))
    C_a, counts_a, _ = g.gpu_update(Xd, idx_a, C0, ws=ws)
    want, counts = oracle.update(X, idx_a, C0)
    assert C_a.tobytes() == want.tobytes() and np.array_equal(counts_a, counts)
    Cd = g.dev(C0)
    idx_d = torch.empty(N, dtype=torch.uint32, device="cuda")
    counts_d = torch.empty(K, dtype=torch.uint32, device="cuda")
    J_d = torch.zeros(1, dtype=torch.float64, device="cuda")
    cc.lloyd_iter(Xd, Cd, idx_d, J_d, counts_d, ws)
    torch.cuda.synchronize()
    assert np.array_equal(idx_d.cpu().numpy(), idx_a)
    assert np.array_equal(counts_d.cpu().numpy(), counts_a)
    assert Cd.cpu().numpy().tobytes() == C_a.tobytes()
    # two iterations in one call equal two chained single-iteration calls
    C2, i2, J2, _ = g.gpu_fit(X, C0, 2, ws=ws, Xd=Xd)
    C1, _, _, _ = g.gpu_fit(X, C0, 1, ws=ws, Xd=Xd)
    C12, i12, J12, _ = g.gpu_fit(X, C1, 1, ws=ws, Xd=Xd)
    assert C2.tobytes() == C12.tobytes() and np.array_equal(i2, i12) and J2 == J12
    assert C1.tobytes() == C_a.tobytes()
