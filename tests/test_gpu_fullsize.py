"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (automatic E-step
selection). The oracle cannot evaluate N x K distances for the large configurations in seconds, so:
  - cfg2 (N = 4.2M, K = 4096) is checked exhaustively for one Lloyd step;
  - cfg3/4/5 (K = 65536) check a seeded sample of vectors against the oracle over ALL K centroids,
    plus properties over all N vectors that hold at any size: every code is in range, no randomly
    drawn centroid is closer than the chosen one, the update equals the oracle's M-step on the
    GPU's codes (O(N d) on the CPU, exact), the objective equals the oracle's for those codes,
    and decode is the bit-exact gather.
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


def _sqdist(X, C, idx):
    return ((X.astype(np.float64) - C[idx].astype(np.float64)) ** 2).sum(1)


def _check_step_sampled(g, X, Xd, C, ws, rng, sample):
    N, d = X.shape
    K = C.shape[0]
    idx, J = g.gpu_assign(Xd, C, ws=ws)
    assert idx.max() < K
    # sampled vectors against the oracle over all K
    sel = np.sort(rng.choice(N, size=sample, replace=False))
    k1, D1, _, D2 = oracle.assign_top2(X[sel], C)
    near = parity.check_assignment(X[sel], C, idx[sel], k1, D1, D2)
    # all vectors: randomly drawn centroids are never closer than the chosen one
    Dg = _sqdist(X, C, idx)
    for _ in range(2):
        r = rng.integers(0, K, size=N)
        assert np.all(Dg <= _sqdist(X, C, r) * (1 + parity.NEAR_TIE) + 1e-300)
    parity.check_inertia(J, float(Dg.sum()))
    parity.check_inertia(J, oracle.inertia(X, C, idx))
    return idx, J, near


@pytest.mark.parametrize("number", [3, 5, 4])
def test_large_configs_one_lloyd_step(g, number):
    w = workloads.by_number(number)
    print(f"generating {w.name}", flush=True)
    X, C0 = workloads.make_inputs(w)
    N, d, K = X.shape[0], w.d, w.K
    rng = np.random.default_rng(900 + number)
    Xd = g.dev(X)
    ws = g.workspace(N, d, K)
    print(f"{w.name}: assign against the initial centroids", flush=True)
    idx0, J0, near0 = _check_step_sampled(g, X, Xd, C0, ws, rng, sample=4096)
    print(f"{w.name}: update", flush=True)
    want, counts = oracle.update(X, idx0, C0)
    got, gcounts, stats = g.gpu_update(Xd, idx0, C0, ws=ws)
    assert np.array_equal(gcounts, counts) and stats.skipped_vectors == 0
    assert got.tobytes() == want.tobytes()
    print(f"{w.name}: assign against the updated centroids", flush=True)
    idx1, J1, near1 = _check_step_sampled(g, X, Xd, got, ws, rng, sample=4096)
    assert J1 <= J0
    print(f"{w.name}: fit(iters=1) reproduces the step; decode", flush=True)
    C1, idx_f, J_f, st = g.gpu_fit(X, C0, 1, ws=ws, Xd=Xd)
    assert C1.tobytes() == got.tobytes() and np.array_equal(idx_f, idx1) and J_f == J1
    out = g.gpu_decode(C1, idx_f)
    assert out.tobytes() == oracle.decode(C1, idx_f).tobytes()
    print(f"{w.name}: J0={J0:.6e} J1={J1:.6e} near-ties in samples={near0 + near1} refined={st.refined_vectors}")


def test_cfg2_exhaustive_lloyd_step(g):
    w = workloads.by_number(2)
    X, C0 = workloads.make_inputs(w)
    N, d, K = X.shape[0], w.d, w.K
    Xd = g.dev(X)
    ws = g.workspace(N, d, K)
    C = C0
    for step in range(2):
        print(f"cfg2 exhaustive step {step}", flush=True)
        k1, D1, _, D2 = oracle.assign_top2(X, C)
        idx, J = g.gpu_assign(Xd, C, ws=ws)
        near = parity.check_assignment(X, C, idx, k1, D1, D2)
        parity.check_inertia(J, oracle.inertia(X, C, idx))
        want, counts = oracle.update(X, idx, C)
        got, gcounts, _ = g.gpu_update(Xd, idx, C, ws=ws)
        assert np.array_equal(gcounts, counts) and got.tobytes() == want.tobytes()
        print(f"  near-tie divergences: {near}")
        C = got
    out = g.gpu_decode(C, idx)
    assert out.tobytes() == oracle.decode(C, idx).tobytes()
