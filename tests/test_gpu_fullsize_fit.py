"""Parity of the job that bench.py times: whole fits of the benchmark configurations at their stated sizes and
iteration counts (Section 3.1 E-step / M-step and the definition of q; Appendix B.1 for the iteration count), in the
automatic launch configuration: windowed E-steps chained through the codes of the previous iteration and, from the
third iteration on, the M-step that moves only the vectors whose code changed.

A free-running oracle fit of these sizes takes hours and would differ legitimately after the first near-tie, so the
fit of T iterations is pinned from both ends instead:
  - the same fit with every E-step over the whole codebook and every M-step recomputed (assign mode 3) must give the
    same centroid, code and objective bytes;
  - the last Lloyd iteration is replayed by the oracle: fit(T-1) -> cc_assign -> oracle.update (O(N d), exact) must be
    the centroids of fit(T) byte for byte; the same at an early iteration whose M-step is already incremental;
  - the returned codes are the oracle's argmin over all K for a seeded sample of vectors, the objective is the
    oracle's for the returned (centroids, codes) over all N, and decode is the oracle's gather.
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
    import paper_2503_13089_amd as cc
    from tests import gpu_helpers

    cc.set_assign_mode(0)
    return gpu_helpers


def _replay_last_iteration(g, X, Xd, C0, T, ws, C_T):
    """fit(T).centroids == oracle M-step of (cc_assign against fit(T-1).centroids)."""
    C_prev, idx_prev, _, _ = g.gpu_fit(X, C0, T - 1, ws=ws, Xd=Xd)
    a, _ = g.gpu_assign(Xd, C_prev, ws=ws)
    assert np.array_equal(a, idx_prev)  # the codes a fit returns are the E-step of its next iteration
    want, _ = oracle.update(X, a, C_prev)
    assert C_T.tobytes() == want.tobytes(), f"iteration {T} of the fit is not the oracle's M-step of its E-step"
    return idx_prev


@pytest.mark.parametrize("number", [3, 2, 5, 4])
def test_benchmark_fit_at_full_size_and_length(g, number):
    import paper_2503_13089_amd as cc

    w = workloads.by_number(number)
    T = w.iters
    print(f"{w.name}: generating", flush=True)
    X, C0 = workloads.make_inputs(w)
    N, d, K = X.shape[0], w.d, w.K
    Xd = g.dev(X)
    ws = g.workspace(N, d, K)
    try:
        cc.set_assign_mode(0)
        print(f"{w.name}: fit({T}), automatic mode", flush=True)
        C, idx, J, st = g.gpu_fit(X, C0, T, ws=ws, Xd=Xd)
        assert st.assign_calls == T + 1 and st.fp16_inputs == 1
        assert 0 < st.scored_stages < st.total_stages   # the windows really pruned
        print(f"{w.name}: scored {st.scored_stages / st.total_stages:.4f} of the codebook, refined "
              f"{st.refined_vectors}; fit({T}) again with whole-codebook E-steps", flush=True)
        cc.set_assign_mode(3)
        C_ref, idx_ref, J_ref, st_ref = g.gpu_fit(X, C0, T, ws=ws, Xd=Xd)
        assert st_ref.scored_stages == st_ref.total_stages or st_ref.total_stages == 0
        cc.set_assign_mode(0)
        assert C.tobytes() == C_ref.tobytes()
        assert np.array_equal(idx, idx_ref)
        assert J == pytest.approx(J_ref, rel=1e-12)  # same terms, summed in key order instead of input order
        del C_ref, idx_ref
        print(f"{w.name}: oracle replay of iteration {T}", flush=True)
        idx_before = _replay_last_iteration(g, X, Xd, C0, T, ws, C)
        moved_last = float(np.mean(idx_before != idx))
        # an early iteration whose M-step is already the incremental one (the third of a windowed fit; a codebook
        # below 8192 entries only takes the windows in fits of five iterations or more)
        t_mid = 3 if K >= 8192 else 5
        print(f"{w.name}: oracle replay of iteration {t_mid}", flush=True)
        C_mid, _, _, st_mid = g.gpu_fit(X, C0, t_mid, ws=ws, Xd=Xd)
        assert 0 < st_mid.scored_stages < st_mid.total_stages
        _replay_last_iteration(g, X, Xd, C0, t_mid, ws, C_mid)
    finally:
        cc.set_assign_mode(0)
    print(f"{w.name}: returned codes against the oracle (sample x all K), objective, decode", flush=True)
    assert idx.max() < K
    rng = np.random.default_rng(1700 + number)
    sel = np.sort(rng.choice(N, size=4096, replace=False))
    k1, D1, _, D2 = oracle.assign_top2(X[sel], C)
    near = parity.check_assignment(X[sel], C, idx[sel], k1, D1, D2)
    J_or = oracle.inertia(X, C, idx)
    parity.check_inertia(J, J_or)
    out = g.gpu_decode(C, idx)
    assert out.tobytes() == oracle.decode(C, idx).tobytes()
    # objective = reconstruction error of the decoded matrix (Section 3.1)
    assert J == pytest.approx(float(((X.astype(np.float64) - out) ** 2).sum()), rel=1e-5)
    print(f"{w.name}: J={J:.6e} (oracle {J_or:.6e}); near-ties in the sample: {near}; codes changed by the last "
          f"iteration: {moved_last:.4f}")


def _lattice_problem(m, N, seed):
    """Centroids on every point of an m^4 integer lattice (shuffled), vectors on the centres of its cells: each vector
    has 16 nearest centroids at exactly the same distance, so every decision is a tie inside the guard band."""
    rng = np.random.default_rng(seed)
    s = np.float32(2.0 ** -6)
    grid = np.stack(np.meshgrid(*([np.arange(m)] * 4), indexing="ij"), -1).reshape(-1, 4).astype(np.float32)
    C = np.ascontiguousarray(grid[rng.permutation(len(grid))] * s)
    cells = np.stack(np.meshgrid(*([np.arange(m - 1)] * 4), indexing="ij"), -1).reshape(-1, 4).astype(np.float32) + 0.5
    X = np.ascontiguousarray(cells[rng.integers(0, len(cells), size=N)] * s)
    return X, C


@pytest.mark.parametrize("mode", [0, 3], ids=["windowed", "whole-codebook"])
def test_refine_list_overflow_takes_the_direct_pass(g, mode):
    """More guard-band vectors than the refine list holds (N/8 + 4096): the E-step must fall back to the direct-form
    pass over everything, and a Lloyd iteration must rebuild its cluster sums from those codes."""
    import paper_2503_13089_amd as cc

    N = 60013
    X, C = _lattice_problem(10, N, seed=31)
    K = C.shape[0]
    k1, D1, _, D2 = oracle.assign_top2(X, C)
    assert np.all(D2 == D1)  # every vector is an exact tie
    Xd = g.dev(X)
    ws = g.workspace(N, 4, K)
    try:
        cc.set_assign_mode(mode)
        print(f"refine overflow, mode {mode}: assign", flush=True)
        idx, J = g.gpu_assign(Xd, C, ws=ws)
        st = cc.read_stats(ws)
        assert st.refined_vectors > N // 8 + 4096, st.refined_vectors
        assert np.array_equal(idx, k1)  # exact ties go to the lowest centroid index
        parity.check_inertia(J, float(D1.sum()))
        print(f"refine overflow, mode {mode}: one Lloyd iteration", flush=True)
        Cd = g.dev(C)
        idx_d = torch.empty(N, dtype=torch.uint32, device="cuda")
        counts_d = torch.empty(K, dtype=torch.uint32, device="cuda")
        cc.lloyd_iter(Xd, Cd, idx_d, None, counts_d, ws)
        torch.cuda.synchronize()
        st = cc.read_stats(ws)
        assert st.refined_vectors > N // 8 + 4096
    finally:
        cc.set_assign_mode(0)
    want, counts = oracle.update(X, k1, C)
    assert np.array_equal(idx_d.cpu().numpy(), k1)
    assert np.array_equal(counts_d.cpu().numpy(), counts)
    assert Cd.cpu().numpy().tobytes() == want.tobytes()


def _cascade_problem(seed):
    """32768 independent cells, far apart along three coordinates, each holding the same one-dimensional system of
    40 vectors and 2 centroids along the first coordinate: groups of 2, 4, 32, 1, 1 vectors at -23, 10, 20, 21, 24 and
    centroids starting at 21 and 24. Lloyd moves the boundary between the two centroids from 22.5 to 20.4 (one vector
    changes code) and then to 19.6, which puts the group of 32 on its other side: 80 % of all codes change in the third
    E-step, 10 % in the fourth."""
    rng = np.random.default_rng(seed)
    cells = np.stack(np.meshgrid(*([np.arange(32)] * 3), indexing="ij"), -1).reshape(-1, 3).astype(np.float32) * 128.0
    pos = np.repeat(np.array([-23, 10, 20, 21, 24], np.float32), [2, 4, 32, 1, 1])
    X = np.empty((len(cells), len(pos), 4), np.float32)
    X[:, :, 0] = pos[None, :]
    X[:, :, 1:] = cells[:, None, :]
    X = X.reshape(-1, 4)[rng.permutation(len(cells) * len(pos))]
    C0 = np.empty((len(cells), 2, 4), np.float32)
    C0[:, 0, 0], C0[:, 1, 0] = 21.0, 24.0
    C0[:, :, 1:] = cells[:, None, :]
    C0 = C0.reshape(-1, 4)[rng.permutation(len(cells) * 2)]
    assert np.array_equal(X.astype(np.float16).astype(np.float32), X)
    return np.ascontiguousarray(X), np.ascontiguousarray(C0)


def test_incremental_mstep_when_most_codes_change_in_one_iteration(g):
    """The M-step of a windowed fit moves only the vectors whose code changed, two records each; here 80 % of them
    change between the second and the third E-step, at K = 65536 (the largest codebook of that path). The vectors'
    large common offsets also put most decisions inside the guard band, so the refine list overflows as well."""
    import paper_2503_13089_amd as cc

    X, C0 = _cascade_problem(seed=5)
    N, d, K = X.shape[0], 4, C0.shape[0]
    assert K == 65536
    Xd = g.dev(X)
    ws = g.workspace(N, d, K)
    fits = {}
    try:
        for t in (1, 2, 3, 4, 6):
            cc.set_assign_mode(0)
            print(f"cascade: fit({t})", flush=True)
            fits[t] = g.gpu_fit(X, C0, t, ws=ws, Xd=Xd)
            assert 0 < fits[t][3].scored_stages < fits[t][3].total_stages
        cc.set_assign_mode(3)
        print("cascade: fit(6) with whole-codebook E-steps", flush=True)
        C_ref, idx_ref, J_ref, _ = g.gpu_fit(X, C0, 6, ws=ws, Xd=Xd)
    finally:
        cc.set_assign_mode(0)
    C6, idx6, J6, st6 = fits[6]
    assert C6.tobytes() == C_ref.tobytes() and np.array_equal(idx6, idx_ref) and J6 == pytest.approx(J_ref, rel=1e-12)
    # fit(t).idx is the E-step of iteration t + 1: the third E-step (the first one followed by an incremental M-step)
    moved = float(np.mean(fits[1][1] != fits[2][1]))
    moved_next = float(np.mean(fits[2][1] != fits[3][1]))
    print(f"cascade: codes changed in the third E-step {moved:.3f}, in the fourth {moved_next:.3f}; refined "
          f"{st6.refined_vectors}", flush=True)
    assert moved > 0.5
    assert st6.refined_vectors > 7 * (N // 8 + 4096)  # every E-step overflowed the list
    # iterations 3 and 4 replayed by the oracle's M-step
    for t in (3, 4):
        want, _ = oracle.update(X, fits[t - 1][1], fits[t - 1][0])
        assert fits[t][0].tobytes() == want.tobytes(), f"iteration {t}"
    # and the result is the oracle's: codes over all K on a sample, objective over all N
    rng = np.random.default_rng(6)
    sel = np.sort(rng.choice(N, size=8192, replace=False))
    k1, D1, _, D2 = oracle.assign_top2(X[sel], C6)
    parity.check_assignment(X[sel], C6, idx6[sel], k1, D1, D2)
    parity.check_inertia(J6, oracle.inertia(X, C6, idx6))
