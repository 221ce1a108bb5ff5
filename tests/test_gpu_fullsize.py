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


def test_layer_path_at_full_size(g):
    """The layer's data path at the benchmark matrix taken as a linear layer (in = 4096, out = 11008, g = 4,
    K = 65536, bf16), in the configuration bench.py times. The numpy oracle handles these sizes for the pure data
    movement (whole arrays compared bit for bit); sums and products are checked on sampled outputs in fp64."""
    import paper_2503_13089_amd as cc
    from oracle import layer as L

    w = workloads.by_number(3)
    in_features, out_features, gdim, K = w.rows, w.cols, w.d, w.K
    rng = np.random.default_rng(77)
    n = L.num_codes(in_features, out_features, gdim)
    print("layer path full size: reshape", flush=True)
    W = torch.from_numpy((rng.standard_normal((out_features, in_features)) * 0.02).astype(np.float32)).to(torch.bfloat16)
    Wd = W.cuda()
    X = torch.empty((n, gdim), dtype=torch.float32, device="cuda")
    cc.layer_vectors(Wd, gdim, X)
    assert X.cpu().numpy().tobytes() == L.prepare_matrix(W.float().numpy(), gdim).tobytes()
    del X
    print("layer path full size: reconstruction", flush=True)
    book = torch.from_numpy((rng.standard_normal((K, gdim)) * 0.02).astype(np.float32)).to(torch.bfloat16).cuda()
    codes_np = rng.integers(0, K, size=n).astype(np.uint16)
    codes = torch.from_numpy(codes_np.view(np.int16)).cuda().view(torch.uint16)
    rebuilt = torch.empty((in_features, out_features), dtype=torch.bfloat16, device="cuda")
    cc.layer_weight(book, codes, in_features, out_features, rebuilt)
    bookh = book.float().cpu().numpy()
    want = L.layer_weight(bookh, codes_np, in_features, out_features)
    assert rebuilt.float().cpu().numpy().tobytes() == want.tobytes()
    print("layer path full size: 4-bit codebook", flush=True)
    C32 = (rng.standard_normal((K, gdim)) * 0.02).astype(np.float32)
    q, s = L.quantize_codebook(C32, 4)
    qbook = torch.empty(K * gdim // 2, dtype=torch.uint8, device="cuda")
    scale = torch.zeros(1, dtype=torch.float32, device="cuda")
    cc.codebook_quantize(torch.from_numpy(C32).cuda(), 4, qbook, scale, torch.zeros(4, dtype=torch.uint8, device="cuda"))
    assert scale.item() == s and np.array_equal(qbook.cpu().numpy(), L.pack_int4(q))
    cc.layer_weight_q(qbook, 4, scale, K, gdim, codes, in_features, out_features, rebuilt)
    want_q = L.layer_weight(L.dequantize_codebook(q, s, "bf16"), codes_np, in_features, out_features)
    assert rebuilt.float().cpu().numpy().tobytes() == want_q.tobytes()
    print("layer path full size: forward (sampled outputs)", flush=True)
    M = 3
    x = torch.from_numpy(rng.standard_normal((M, in_features)).astype(np.float32)).to(torch.bfloat16).cuda()
    xh = x.float().cpu().numpy().astype(np.float64)
    cols = np.sort(rng.choice(out_features, size=64, replace=False))
    y = torch.empty((M, out_features), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(cc.layer_forward_workspace_bytes(M, in_features, out_features),
                         cc.layer_forward_q_workspace_bytes(M, in_features, out_features), 256), dtype=torch.uint8, device="cuda")
    cc.layer_forward(x, book, codes, out_features, None, y, ws)
    got = y.float().cpu().numpy().astype(np.float64)[:, cols]
    ref = xh @ want.astype(np.float64)[:, cols]
    mag = np.abs(xh) @ np.abs(want.astype(np.float64))[:, cols]
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + in_features * 2.0 ** -24 * mag)
    cc.layer_forward_q(x, qbook, 4, scale, K, gdim, codes, out_features, None, y, ws)
    got = y.float().cpu().numpy().astype(np.float64)[:, cols]
    Q = L.layer_weight(q.astype(np.float64), codes_np, in_features, out_features)[:, cols]
    ref = float(s) * (xh @ Q)
    mag = float(s) * (np.abs(xh) @ (np.abs(Q) + 8.0))
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + in_features * 2.0 ** -24 * mag)
    print("layer path full size: codebook gradient", flush=True)
    wsz = torch.empty(cc.workspace_bytes(n, gdim, K), dtype=torch.uint8, device="cuda")
    grad = torch.empty((K, gdim), dtype=torch.float32, device="cuda")
    cc.layer_codebook_grad(Wd.t().contiguous(), codes, K, gdim, grad, wsz)
    Gh = W.float().numpy().T
    wantg = L.gather_backward(Gh, codes_np, K, gdim)
    assert np.array_equal(grad.cpu().numpy(), wantg.astype(np.float32))  # exact sums of bf16 values, one rounding
    del wsz
    print("layer path full size: codebook gradient from the prepared order", flush=True)
    plan = torch.empty(cc.layer_grad_plan_bytes(n, K), dtype=torch.uint8, device="cuda")
    pws = torch.empty(cc.layer_grad_plan_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    cc.layer_grad_plan(codes, K, plan, pws)
    gws = torch.empty(cc.layer_codebook_grad_planned_workspace_bytes(n, K, gdim), dtype=torch.uint8, device="cuda")
    grad2 = torch.empty_like(grad)
    cc.layer_codebook_grad_planned(Wd.t().contiguous(), K, gdim, plan, grad2, gws)
    assert np.array_equal(grad2.cpu().numpy(), wantg.astype(np.float32))
