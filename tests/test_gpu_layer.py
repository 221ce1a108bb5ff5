"""GPU parity of the layer data path (include/cluscomp.h, "compressed linear layer") against oracle/layer.py:
bit-exact for data movement and format conversion, fp64-derived tolerances for sums."""
import numpy as np
import pytest
import torch

import oracle
from oracle import layer as L

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cc():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2503_13089_amd as cc

    return cc


TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _dev(a, dt=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dt is not None:
        t = t.to(dt)
    return t.cuda()


# (out_features, in_features, g): ragged against the 64 x 64 transpose tiles, with and without padding columns
LAYER_SHAPES = [(256, 192, 4), (250, 131, 4), (129, 67, 6), (100, 300, 9), (64, 64, 8), (7, 5, 7), (1, 1, 3), (513, 70, 5)]


def test_constructor_arithmetic(cc):
    for out_features, g in [(4096, 4), (4096, 6), (4096, 9), (11008, 7), (10, 4), (7, 7)]:
        assert cc.layer_deficiency(out_features, g) == L.deficiency(out_features, g)
        assert cc.layer_num_codes(123, out_features, g) == L.num_codes(123, out_features, g)


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("out_features,in_features,g", LAYER_SHAPES)
def test_layer_vectors_bit_exact(cc, out_features, in_features, g, dt):
    rng = np.random.default_rng(out_features * 7 + in_features + g)
    W = _dev(rng.standard_normal((out_features, in_features)).astype(np.float32), TORCH_DT[dt])
    n = L.num_codes(in_features, out_features, g)
    X = torch.full((n, g), 7.0, dtype=torch.float32, device="cuda")  # padding must be overwritten with zeros
    print(f"layer_vectors {out_features}x{in_features} g={g} {dt}", flush=True)
    cc.layer_vectors(W, g, X)
    want = L.prepare_matrix(W.float().cpu().numpy(), g)
    assert X.cpu().numpy().tobytes() == want.tobytes()


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_layer_pack_formats(cc, dt):
    rng = np.random.default_rng(5)
    K, g, n = 3001, 6, 50021
    C = rng.standard_normal((K, g)).astype(np.float32) * np.float32(10.0) ** rng.integers(-12, 6, (K, g)).astype(np.float32)
    C[0, :4] = [1.00390625, 1.01171875, 65520.0, 3.4e38]  # bf16 ties; fp16 overflow; bf16 overflow
    C[1, :3] = [0.0, -0.0, 5.9e-8]
    idx = rng.integers(0, K, size=n).astype(np.uint32)
    idx[7] = K + 5  # clamped
    book = torch.empty((K, g), dtype=TORCH_DT[dt], device="cuda")
    codes = torch.empty(n, dtype=torch.uint16, device="cuda")
    cc.layer_pack(_dev(C), book, _dev(idx.view(np.int32)).view(torch.uint32), codes)
    want = L.bf16_round(C) if dt == "bf16" else L.fp16_round(C)
    got = book.float().cpu().numpy()
    assert got.tobytes() == want.tobytes()
    want_codes = np.minimum(idx, K - 1).astype(np.uint16)
    assert np.array_equal(codes.cpu().view(torch.int16).numpy().view(np.uint16), want_codes)
    # either half alone
    book2 = torch.empty_like(book)
    cc.layer_pack(_dev(C), book2, None, None)
    assert torch.equal(book2.view(torch.int16), book.view(torch.int16))
    codes2 = torch.empty_like(codes)
    cc.layer_pack(None, None, _dev(idx.view(np.int32)).view(torch.uint32), codes2, K=K)
    assert torch.equal(codes2.view(torch.int16), codes.view(torch.int16))


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("out_features,in_features,g", LAYER_SHAPES)
def test_layer_weight_bit_exact(cc, out_features, in_features, g, dt):
    rng = np.random.default_rng(out_features + 3 * in_features + g)
    K = 977
    book = _dev(rng.standard_normal((K, g)).astype(np.float32), TORCH_DT[dt])
    n = L.num_codes(in_features, out_features, g)
    codes_np = rng.integers(0, K, size=n).astype(np.uint16)
    codes_np[0] = 60000  # >= K: clamped to K - 1
    codes = _dev(codes_np.view(np.int16)).view(torch.uint16)
    W = torch.zeros((in_features, out_features), dtype=TORCH_DT[dt], device="cuda")
    print(f"layer_weight {out_features}x{in_features} g={g} {dt}", flush=True)
    cc.layer_weight(book, codes, in_features, out_features, W)
    ref_codes = np.minimum(codes_np, K - 1)
    want = L.layer_weight(book.float().cpu().numpy(), ref_codes, in_features, out_features)
    assert W.float().cpu().numpy().tobytes() == want.tobytes()


def test_cluster_then_rebuild_round_trip(cc):
    """vectors -> fit -> pack -> weight: the rebuilt weight equals the oracle's reconstruction from the same
    (codebook, codes), and with K = N every vector is its own centroid, so the bf16 weight comes back exactly."""
    from tests import gpu_helpers as g_

    rng = np.random.default_rng(9)
    out_features, in_features, g = 150, 64, 4
    W = torch.from_numpy(rng.standard_normal((out_features, in_features)).astype(np.float32)).to(torch.bfloat16).cuda()
    n = L.num_codes(in_features, out_features, g)
    X = torch.empty((n, g), dtype=torch.float32, device="cuda")
    cc.layer_vectors(W, g, X)
    Xh = X.cpu().numpy()
    C, idx, J, _ = g_.gpu_fit(Xh, Xh.copy(), 0)  # K = N, init = the vectors themselves
    assert J == 0.0
    book = torch.empty((n, g), dtype=torch.bfloat16, device="cuda")
    codes = torch.empty(n, dtype=torch.uint16, device="cuda")
    cc.layer_pack(_dev(C), book, _dev(idx.view(np.int32)).view(torch.uint32), codes)
    back = torch.empty((in_features, out_features), dtype=torch.bfloat16, device="cuda")
    cc.layer_weight(book, codes, in_features, out_features, back)
    assert torch.equal(back, W.t().contiguous())


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("out_features,in_features,g,K", [(256, 192, 4, 500), (250, 131, 4, 9000), (129, 67, 6, 300),
                                                          (100, 300, 9, 64), (513, 300, 5, 8200), (7, 5, 7, 3),
                                                          (600, 512, 8, 65536)])
def test_codebook_grad(cc, out_features, in_features, g, K, dt):
    rng = np.random.default_rng(out_features + in_features + g + K)
    G = _dev(rng.standard_normal((in_features, out_features)).astype(np.float32) * 1e-3, TORCH_DT[dt])
    n = L.num_codes(in_features, out_features, g)
    codes_np = rng.integers(0, K, size=n).astype(np.uint16) if K < 65536 else rng.integers(0, K, size=n).astype(np.uint16)
    codes = _dev(codes_np.view(np.int16)).view(torch.uint16)
    out = torch.full((K, g), 3.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(cc.workspace_bytes(max(n, K), g, K), dtype=torch.uint8, device="cuda")
    print(f"codebook_grad {out_features}x{in_features} g={g} K={K} {dt}", flush=True)
    cc.layer_codebook_grad(G, codes, K, g, out, ws)
    Gh = G.float().cpu().numpy()
    want = L.gather_backward(Gh, codes_np, K, g)
    got = out.cpu().numpy().astype(np.float64)
    # per entry: fixed-point grid 2^-38 max|G| per term (exact for 16-bit inputs) + one fp32 rounding of the sum
    absG = L.gather_backward(np.abs(Gh), codes_np, K, g)
    counts = L.gather_backward(np.ones_like(Gh), codes_np, K, g)
    tol = 2.0 ** -24 * absG + counts * 2.0 ** -38 * np.abs(Gh).max() + 1e-45
    assert np.all(np.abs(got - want) <= tol), float(np.max(np.abs(got - want) / tol))
    if dt != "f32":
        assert np.array_equal(got, want.astype(np.float32).astype(np.float64))  # exact sums, one rounding
    # deterministic
    out2 = torch.empty_like(out)
    cc.layer_codebook_grad(G, codes, K, g, out2, ws)
    assert torch.equal(out.view(torch.int32), out2.view(torch.int32))


@pytest.mark.parametrize("out_features,in_features,g,K,dt", [(2052, 2049, 4, 65536, "bf16"), (2052, 2049, 4, 5000, "f16"),
                                                             (4104, 2049, 8, 40000, "bf16"), (4112, 4099, 16, 3000, "f16")])
def test_codebook_grad_of_a_large_16_bit_layer_is_summed_in_place(cc, out_features, in_features, g, K, dt):
    """From 2^20 sub-vectors on, a 16-bit gradient whose sub-vectors are whole runs of g numbers is read where it lies
    (no fp32 copy): the exact sums, rounded once, as for every other layer - also with codes beyond K (left out), with
    a code array that is only 2-byte aligned (the copying route takes over) and on a second call."""
    rng = np.random.default_rng(out_features + in_features + g + K)
    G = _dev(rng.standard_normal((in_features, out_features)).astype(np.float32) * 1e-3, TORCH_DT[dt])
    n = L.num_codes(in_features, out_features, g)
    assert n >= 1 << 20 and n % 128 != 0  # the last round of the last range is ragged
    codes_np = rng.integers(0, K, size=n).astype(np.uint16)
    codes_np[codes_np == 7] = 8                       # an empty cluster
    beyond = rng.choice(n, size=50, replace=False) if K < 65536 else np.empty(0, dtype=np.int64)
    codes_np[beyond] = 65535 if K < 65535 else 0
    buf = torch.empty(n + 1, dtype=torch.int16, device="cuda")
    buf[:n] = torch.from_numpy(codes_np.view(np.int16)).cuda()
    codes = buf[:n].view(torch.uint16)
    out = torch.full((K, g), 3.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(cc.workspace_bytes(n, g, K), dtype=torch.uint8, device="cuda")
    print(f"codebook_grad in place {out_features}x{in_features} g={g} K={K} {dt}", flush=True)
    cc.layer_codebook_grad(G, codes, K, g, out, ws)
    Gh = G.float().cpu().numpy().copy()
    kept = codes_np.copy()
    if beyond.size:   # the definition over the entries whose code names a cluster
        Gh.reshape(n, g)[beyond] = 0.0
        kept[beyond] = 0
    want = L.gather_backward(Gh, kept, K, g)
    got = out.cpu().numpy()
    assert np.array_equal(got, want.astype(np.float32))
    assert np.all(got[7] == 0.0)
    out2 = torch.empty_like(out)
    cc.layer_codebook_grad(G, codes, K, g, out2, ws)
    assert torch.equal(out.view(torch.int32), out2.view(torch.int32))
    # the same codes one element further on: 2-byte aligned only
    buf[1:] = torch.from_numpy(codes_np.view(np.int16)).cuda()
    out3 = torch.empty_like(out)
    print("  the same through the copying route", flush=True)
    cc.layer_codebook_grad(G, buf[1:].view(torch.uint16), K, g, out3, ws)
    assert torch.equal(out.view(torch.int32), out3.view(torch.int32))


def test_codebook_grad_in_place_keeps_a_non_finite_entry_out_of_the_sums_and_flags_it(cc):
    """Finite gradients are the caller's precondition; one that is not must neither poison its cluster's sum (its
    conversion to the fixed-point grid would be undefined) nor go unnoticed."""
    rng = np.random.default_rng(77)
    out_features, in_features, g, K = 2052, 2049, 4, 30000
    Gh = (rng.standard_normal((in_features, out_features)).astype(np.float32) * 1e-3)
    G = _dev(Gh, torch.bfloat16)
    G[1000, 1001] = float("inf")
    G[5, 7] = float("nan")
    n = L.num_codes(in_features, out_features, g)
    codes_np = rng.integers(0, K, size=n).astype(np.uint16)
    codes = _dev(codes_np.view(np.int16)).view(torch.uint16)
    out = torch.empty((K, g), dtype=torch.float32, device="cuda")
    ws = torch.empty(cc.workspace_bytes(n, g, K), dtype=torch.uint8, device="cuda")
    print("codebook_grad in place with an inf and a nan among the gradients", flush=True)
    cc.layer_codebook_grad(G, codes, K, g, out, ws)
    torch.cuda.synchronize()
    assert cc.read_stats(ws).nonfinite_inputs == 1
    clean = G.float().cpu().numpy().copy()
    clean[1000, 1001] = 0.0
    clean[5, 7] = 0.0
    want = L.gather_backward(clean, codes_np, K, g)
    assert np.array_equal(out.cpu().numpy(), want.astype(np.float32))


def _plan(cc, codes, K):
    n = codes.numel()
    plan = torch.empty(cc.layer_grad_plan_bytes(n, K), dtype=torch.uint8, device="cuda")
    ws = torch.empty(cc.layer_grad_plan_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    cc.layer_grad_plan(codes, K, plan, ws)
    return plan


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("out_features,in_features,g,K", [(256, 192, 4, 500), (250, 131, 4, 9000), (129, 67, 6, 300),
                                                          (100, 300, 9, 64), (513, 300, 5, 8200), (7, 5, 7, 3),
                                                          (600, 512, 8, 65536), (1024, 1536, 4, 3), (640, 333, 16, 2),
                                                          (2048, 1024, 8, 1)])
def test_codebook_grad_planned(cc, out_features, in_features, g, K, dt):
    """The gradient from a prepared order of the codes: against the definition, against the unplanned entry point,
    and the same bits on a second call. The last cases have clusters of 10^5..10^6 members (many work items each)."""
    rng = np.random.default_rng(out_features + in_features + g + K)
    G = _dev(rng.standard_normal((in_features, out_features)).astype(np.float32) * 1e-3, TORCH_DT[dt])
    n = L.num_codes(in_features, out_features, g)
    codes_np = rng.integers(0, K, size=n).astype(np.uint16)
    if K > 100:
        codes_np[codes_np == 7] = 8  # an empty cluster
    codes = _dev(codes_np.view(np.int16)).view(torch.uint16)
    print(f"codebook_grad_planned {out_features}x{in_features} g={g} K={K} {dt}", flush=True)
    plan = _plan(cc, codes, K)
    out = torch.full((K, g), 3.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(cc.layer_codebook_grad_planned_workspace_bytes(n, K, g), dtype=torch.uint8, device="cuda")
    cc.layer_codebook_grad_planned(G, K, g, plan, out, ws)
    Gh = G.float().cpu().numpy()
    want = L.gather_backward(Gh, codes_np, K, g)
    got = out.cpu().numpy().astype(np.float64)
    # fp64 accumulation (count * 2^-53 * sum|terms|), then one rounding to fp32
    absG = L.gather_backward(np.abs(Gh), codes_np, K, g)
    counts = L.gather_backward(np.ones_like(Gh), codes_np, K, g)
    tol = 2.0 ** -24 * np.abs(want) + counts * 2.0 ** -52 * absG + 1e-45
    assert np.all(np.abs(got - want) <= tol), float(np.max(np.abs(got - want) / tol))
    if K > 100:
        assert np.all(got[7] == 0.0)
    if dt != "f32":
        # 16-bit terms of this spread add up exactly in fp64: the rounded exact sum, as the unplanned entry point gives
        assert np.array_equal(got, want.astype(np.float32).astype(np.float64))
        out1 = torch.empty_like(out)
        ws1 = torch.empty(cc.workspace_bytes(max(n, K), g, K), dtype=torch.uint8, device="cuda")
        cc.layer_codebook_grad(G, codes, K, g, out1, ws1)
        assert torch.equal(out.view(torch.int32), out1.view(torch.int32))
    out2 = torch.empty_like(out)
    cc.layer_codebook_grad_planned(G, K, g, plan, out2, ws)
    assert torch.equal(out.view(torch.int32), out2.view(torch.int32))


def test_codebook_grad_planned_leaves_out_codes_beyond_k_and_rejects_a_foreign_plan(cc):
    rng = np.random.default_rng(5)
    in_features, out_features, g, K = 96, 200, 4, 50
    G = _dev(rng.standard_normal((in_features, out_features)).astype(np.float32), torch.bfloat16)
    n = L.num_codes(in_features, out_features, g)
    codes_np = rng.integers(0, 64, size=n).astype(np.uint16)  # codes 50..63 have no cluster
    codes = _dev(codes_np.view(np.int16)).view(torch.uint16)
    plan = _plan(cc, codes, K)
    out = torch.empty((K, g), dtype=torch.float32, device="cuda")
    ws = torch.empty(cc.layer_codebook_grad_planned_workspace_bytes(n, K, g), dtype=torch.uint8, device="cuda")
    cc.layer_codebook_grad_planned(G, K, g, plan, out, ws)
    want = L.gather_backward(G.float().cpu().numpy(), codes_np, 64, g)[:K]
    assert np.array_equal(out.cpu().numpy(), want.astype(np.float32))
    # a plan for another codebook size: detected on the device
    other = _plan(cc, codes, 64)
    big = torch.empty(max(other.numel(), plan.numel()), dtype=torch.uint8, device="cuda")
    big[:other.numel()] = other
    cc.layer_codebook_grad_planned(G, K, g, big, out, ws)
    assert torch.isnan(out).all()


FORWARD_CASES = [  # (M, in_features, out_features, g, K, bias)
    (1, 256, 192, 4, 500, False),
    (7, 512, 250, 4, 9000, True),     # padding columns, ragged column tile
    (33, 136, 129, 6, 300, True),     # in_features not a multiple of the 64-wide step; codes straddle column tiles
    (64, 128, 100, 9, 64, False),
    (130, 320, 513, 5, 8200, True),   # three row tiles of 128/2/...; odd g
    (32, 1024, 1024, 8, 65536, True),
    (5, 64, 70, 7, 3, False),
    (200, 4096, 256, 4, 65536, False),
    # few rows: M <= 4 with g = 4 takes a kernel of its own (one lane per code column, a register block per row count);
    # the same kind of shape with g = 8 or more rows stays with the tile kernel
    (2, 136, 200, 8, 300, True),      # in_features not a multiple of the 16 rows a round of the 8 waves takes
    (3, 1048, 1000, 4, 65536, False),
    (4, 4096, 1280, 4, 65536, True),  # several slices of in_features
    (2, 24, 516, 4, 300, False),
    (3, 40, 250, 4, 900, True),       # padding columns in the last code column
    (4, 8, 12, 4, 7, True),           # fewer pairs of in-features than waves
    (8, 520, 516, 8, 4096, True),     # padding columns (516 = 64 * 8 + 4)
    (9, 264, 333, 4, 1000, True),     # padding columns, ragged last block of code columns
    (12, 72, 68, 4, 50, False),
    (16, 4096, 256, 8, 65536, False),
    # prefill-sized batches: the weight is rebuilt and multiplied by the library's matrix-core product
    (128, 2048, 2048, 4, 65536, True),
    (256, 512, 768, 4, 65536, True),
    (1000, 1024, 520, 8, 4096, False),
    (384, 1536, 1000, 6, 30000, True),
]


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("M,in_features,out_features,g,K,with_bias", FORWARD_CASES)
def test_layer_forward(cc, M, in_features, out_features, g, K, with_bias, dt):
    rng = np.random.default_rng(M + in_features + out_features + g)
    T = TORCH_DT[dt]
    x = _dev(rng.standard_normal((M, in_features)).astype(np.float32), T)
    book = _dev(rng.standard_normal((K, g)).astype(np.float32) * 0.05, T)
    bias = _dev(rng.standard_normal(out_features).astype(np.float32), T) if with_bias else None
    n = L.num_codes(in_features, out_features, g)
    codes_np = rng.integers(0, K, size=n).astype(np.uint16)
    codes = _dev(codes_np.view(np.int16)).view(torch.uint16)
    y = torch.full((M, out_features), 9.0, dtype=T, device="cuda")
    nbytes = cc.layer_forward_workspace_bytes(M, in_features, out_features)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    print(f"layer_forward M={M} {in_features}->{out_features} g={g} K={K} {dt} ws={nbytes}", flush=True)
    cc.layer_forward(x, book, codes, out_features, bias, y, ws)
    xh, bh = x.float().cpu().numpy(), book.float().cpu().numpy()
    biash = bias.float().cpu().numpy() if with_bias else None
    want = L.layer_forward(xh, bh, codes_np, in_features, out_features, biash)
    # products of two 16-bit values are exact in fp32; the fp32 accumulation of in_features terms (in whatever
    # order) is off by at most in_features * 2^-24 * sum|terms|; then one rounding to the 16-bit output format
    mag = L.layer_forward(np.abs(xh), np.abs(bh), codes_np, in_features, out_features,
                          np.abs(biash) if with_bias else None)
    half_ulp = 2.0 ** -8 if dt == "bf16" else 2.0 ** -11
    got = y.float().cpu().numpy().astype(np.float64)
    tol = half_ulp * np.abs(want) + in_features * 2.0 ** -24 * mag + (2.0 ** -24 if dt == "f16" else 1e-38)
    bad = np.abs(got - want) > tol
    assert not bad.any(), (int(bad.sum()), float(np.max(np.abs(got - want) / tol)))
    # same inputs, same bits
    y2 = torch.empty_like(y)
    cc.layer_forward(x, book, codes, out_features, bias, y2, ws)
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))


@pytest.mark.parametrize("M", [40, 2048])
def test_layer_forward_prefill_at_model_size(cc, M):
    """A prefill batch, and a wide decoding batch, through an MLP-sized layer (the rebuilt-weight route): sampled rows of y against the definition, and the same bits on a second call."""
    rng = np.random.default_rng(77)
    in_features, out_features, g, K = 4096, 11008, 4, 65536
    T = torch.bfloat16
    x = _dev(rng.standard_normal((M, in_features)).astype(np.float32), T)
    book = _dev(rng.standard_normal((K, g)).astype(np.float32) * 0.02, T)
    bias = _dev(rng.standard_normal(out_features).astype(np.float32), T)
    n = L.num_codes(in_features, out_features, g)
    codes_np = rng.integers(0, K, size=n).astype(np.uint16)
    codes = _dev(codes_np.view(np.int16)).view(torch.uint16)
    y = torch.full((M, out_features), 9.0, dtype=T, device="cuda")
    nbytes = cc.layer_forward_workspace_bytes(M, in_features, out_features)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    print(f"layer_forward M={M} {in_features}->{out_features} ws={nbytes}", flush=True)
    cc.layer_forward(x, book, codes, out_features, bias, y, ws)
    rows = np.concatenate([[0, M - 1], rng.choice(M, size=min(30, M), replace=False)])
    xh = x.float().cpu().numpy()[rows]
    bh, biash = book.float().cpu().numpy(), bias.float().cpu().numpy()
    want = L.layer_forward(xh, bh, codes_np, in_features, out_features, biash)
    mag = L.layer_forward(np.abs(xh), np.abs(bh), codes_np, in_features, out_features, np.abs(biash))
    got = y.float().cpu().numpy()[rows].astype(np.float64)
    tol = 2.0 ** -8 * np.abs(want) + in_features * 2.0 ** -24 * mag + 1e-38
    bad = np.abs(got - want) > tol
    assert not bad.any(), (int(bad.sum()), float(np.max(np.abs(got - want) / tol)))
    y2 = torch.empty_like(y)
    cc.layer_forward(x, book, codes, out_features, bias, y2, ws)
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("M,in_features,out_features,g,K", [(192, 1024, 2560, 4, 65536), (300, 200, 300, 4, 500),
                                                            (129, 4096, 130, 8, 4096), (513, 72, 1000, 6, 300),
                                                            # the shortest contractions: one operand block, not even that
                                                            (300, 8, 40, 4, 100), (257, 24, 33, 3, 50), (128, 16, 257, 4, 9),
                                                            # several row tiles with a ragged last one, column tiles likewise
                                                            (777, 264, 515, 5, 2000)])
def test_layer_forward_many_rows_meets_the_definition_and_reads_out_weight_rows(cc, M, in_features, out_features, g, K, dt):
    """The rebuilt-weight route (rebuild into matrix-core operands + the product, the contraction split over workgroups
    where the tiles are few, in_features not a multiple of the operand's 16, ragged edges in both directions): every
    output against the definition, the same bits on a second call, and one-hot inputs must return rows of the
    reconstructed weight exactly (no arithmetic error possible)."""
    rng = np.random.default_rng(M + in_features)
    T = TORCH_DT[dt]
    x = _dev(rng.standard_normal((M, in_features)).astype(np.float32), T)
    book = _dev(rng.standard_normal((K, g)).astype(np.float32) * 0.02, T)
    bias = _dev(rng.standard_normal(out_features).astype(np.float32), T)
    n = L.num_codes(in_features, out_features, g)
    codes_np = rng.integers(0, K, size=n).astype(np.uint16)
    codes = _dev(codes_np.view(np.int16)).view(torch.uint16)
    nbytes = cc.layer_forward_workspace_bytes(M, in_features, out_features)
    assert nbytes >= in_features * out_features * 2   # room for the rebuilt weight: this is the many-rows route
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    print(f"layer_forward (many rows) M={M} {in_features}->{out_features} g={g} K={K} {dt} ws={nbytes}", flush=True)
    y = torch.full((M, out_features), 9.0, dtype=T, device="cuda")
    cc.layer_forward(x, book, codes, out_features, bias, y, ws)
    xh, bh, biash = x.float().cpu().numpy(), book.float().cpu().numpy(), bias.float().cpu().numpy()
    want = L.layer_forward(xh, bh, codes_np, in_features, out_features, biash)
    mag = L.layer_forward(np.abs(xh), np.abs(bh), codes_np, in_features, out_features, np.abs(biash))
    got = y.float().cpu().numpy().astype(np.float64)
    half_ulp = 2.0 ** -8 if dt == "bf16" else 2.0 ** -11
    tol = half_ulp * np.abs(want) + in_features * 2.0 ** -24 * mag + (2.0 ** -24 if dt == "f16" else 1e-38)
    assert np.all(np.abs(got - want) <= tol), float(np.max(np.abs(got - want) / tol))
    y2 = torch.empty_like(y)
    cc.layer_forward(x, book, codes, out_features, bias, y2, ws)
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))
    # one-hot rows of x: row m of y is row pick[m] of the weight, bit for bit
    pick = rng.integers(0, in_features, size=M)
    onehot = np.zeros((M, in_features), np.float32)
    onehot[np.arange(M), pick] = 1.0
    cc.layer_forward(_dev(onehot, T), book, codes, out_features, None, y, ws)
    W = torch.empty((in_features, out_features), dtype=T, device="cuda")
    cc.layer_weight(book, codes, in_features, out_features, W)
    assert torch.equal(y.view(torch.int16), W[torch.from_numpy(pick).cuda()].view(torch.int16))


def test_layer_forward_reads_out_single_weight_rows(cc):
    """One-hot inputs: y must equal rows of the reconstructed weight exactly (no arithmetic error possible)."""
    rng = np.random.default_rng(2)
    in_features, out_features, g, K = 128, 200, 4, 1000
    book = _dev(rng.standard_normal((K, g)).astype(np.float32), torch.bfloat16)
    n = L.num_codes(in_features, out_features, g)
    codes = _dev(rng.integers(0, K, size=n).astype(np.uint16).view(np.int16)).view(torch.uint16)
    x = torch.eye(in_features, dtype=torch.bfloat16, device="cuda")
    y = torch.empty((in_features, out_features), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(cc.layer_forward_workspace_bytes(in_features, in_features, out_features), 256), dtype=torch.uint8,
                     device="cuda")
    cc.layer_forward(x, book, codes, out_features, None, y, ws)
    W = torch.empty_like(y)
    cc.layer_weight(book, codes, in_features, out_features, W)
    assert torch.equal(y.view(torch.int16), W.view(torch.int16))


# ------------------------------------------------------------------ uniformly quantised codebook

def _quantize_on_gpu(cc, C, bits):
    K, g = C.shape
    nbytes = K * g if bits == 8 else (K * g + 1) // 2
    qbook = torch.zeros(nbytes + 16, dtype=torch.uint8, device="cuda")[:nbytes]
    scale = torch.zeros(1, dtype=torch.float32, device="cuda")
    scratch = torch.zeros(4, dtype=torch.uint8, device="cuda")
    cc.codebook_quantize(_dev(C), bits, qbook, scale, scratch)
    return qbook, scale


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("K,g", [(65536, 4), (3001, 6), (500, 9), (7, 5), (1, 1), (4096, 8)])
def test_codebook_quantize_bit_exact(cc, K, g, bits):
    rng = np.random.default_rng(K + g + bits)
    C = (rng.standard_normal((K, g)) * 0.02).astype(np.float32)
    C[0, 0] = 0.25  # the extreme entry defines the scale
    qbook, scale = _quantize_on_gpu(cc, C, bits)
    q, s = L.quantize_codebook(C, bits)
    assert scale.cpu().numpy()[0] == s
    want = q.reshape(-1).view(np.uint8) if bits == 8 else L.pack_int4(q)
    assert np.array_equal(qbook.cpu().numpy(), want)
    # all-zero codebook
    qz, sz = _quantize_on_gpu(cc, np.zeros((K, g), np.float32), bits)
    assert sz.item() == 0.0 and not qz.any().item()


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("out_features,in_features,g,K", [(256, 192, 4, 65536), (250, 131, 4, 9000), (129, 67, 6, 300),
                                                          (100, 300, 9, 64), (513, 70, 5, 8200), (64, 64, 8, 65536),
                                                          (7, 5, 7, 3)])
def test_layer_weight_q_bit_exact(cc, out_features, in_features, g, K, dt, bits):
    """Covers codebooks that fit LDS (<= 128 KB) and ones that do not (65536 x 4 at 8 bits, 65536 x 8)."""
    rng = np.random.default_rng(out_features + in_features + g + K + bits)
    C = (rng.standard_normal((K, g)) * 0.02).astype(np.float32)
    q, s = L.quantize_codebook(C, bits)
    qbook, scale = _quantize_on_gpu(cc, C, bits)
    n = L.num_codes(in_features, out_features, g)
    codes_np = rng.integers(0, K, size=n).astype(np.uint16)
    codes = _dev(codes_np.view(np.int16)).view(torch.uint16)
    W = torch.zeros((in_features, out_features), dtype=TORCH_DT[dt], device="cuda")
    print(f"layer_weight_q {out_features}x{in_features} g={g} K={K} {dt} bits={bits}", flush=True)
    cc.layer_weight_q(qbook, bits, scale, K, g, codes, in_features, out_features, W)
    want = L.layer_weight(L.dequantize_codebook(q, s, dt), codes_np, in_features, out_features)
    assert W.float().cpu().numpy().tobytes() == want.tobytes()


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("M,in_features,out_features,g,K,with_bias",
                         FORWARD_CASES + [(3, 2048, 1024, 4, 65536, True),
                                          # 16 < M <= 64 with g = 4 / 8 and an LDS-sized codebook: matrix cores + LDS codebook
                                          (40, 512, 320, 4, 65536, True), (64, 264, 200, 8, 9000, False),
                                          (17, 1024, 1024, 4, 30000, True), (33, 72, 70, 4, 100, False),
                                          # a wide decoding batch on a layer of 2^25 weights: rebuilt integer weight + matrix-core product
                                          (24, 4096, 8448, 4, 65536, True),
                                          # many rows on the shortest contractions and ragged tiles
                                          (300, 8, 40, 4, 100, True), (257, 24, 33, 3, 50, False), (777, 264, 515, 5, 2000, True)])
def test_layer_forward_q(cc, M, in_features, out_features, g, K, with_bias, dt, bits):
    rng = np.random.default_rng(M + in_features + out_features + g + bits)
    T = TORCH_DT[dt]
    x = _dev(rng.standard_normal((M, in_features)).astype(np.float32), T)
    C = (rng.standard_normal((K, g)) * 0.05).astype(np.float32)
    q, s = L.quantize_codebook(C, bits)
    qbook, scale = _quantize_on_gpu(cc, C, bits)
    bias = _dev(rng.standard_normal(out_features).astype(np.float32), T) if with_bias else None
    n = L.num_codes(in_features, out_features, g)
    codes_np = rng.integers(0, K, size=n).astype(np.uint16)
    codes = _dev(codes_np.view(np.int16)).view(torch.uint16)
    y = torch.full((M, out_features), 9.0, dtype=T, device="cuda")
    nbytes = cc.layer_forward_q_workspace_bytes(M, in_features, out_features)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    print(f"layer_forward_q M={M} {in_features}->{out_features} g={g} K={K} {dt} bits={bits} ws={nbytes}", flush=True)
    cc.layer_forward_q(x, qbook, bits, scale, K, g, codes, out_features, bias, y, ws)
    # definition: y = s * (x . Q) + bias with Q rebuilt from the integers q; fp64 here
    xh = x.float().cpu().numpy()
    biash = bias.float().cpu().numpy() if with_bias else None
    want = float(s) * L.layer_forward(xh, q.astype(np.float64), codes_np, in_features, out_features)
    # fp32 accumulation of exact products, possibly taken with the storage offset 2^(bits-1) left in
    mag = float(s) * L.layer_forward(np.abs(xh), np.abs(q.astype(np.float64)) + 2.0 ** (bits - 1), codes_np, in_features,
                                     out_features)
    if with_bias:
        want = want + biash.astype(np.float64)[None, :]
        mag = mag + np.abs(biash.astype(np.float64))[None, :]
    half_ulp = 2.0 ** -8 if dt == "bf16" else 2.0 ** -11
    got = y.float().cpu().numpy().astype(np.float64)
    tol = half_ulp * np.abs(want) + in_features * 2.0 ** -24 * mag + (2.0 ** -24 if dt == "f16" else 1e-38)
    bad = np.abs(got - want) > tol
    assert not bad.any(), (int(bad.sum()), float(np.max(np.abs(got - want) / tol)))
    y2 = torch.empty_like(y)
    cc.layer_forward_q(x, qbook, bits, scale, K, g, codes, out_features, bias, y2, ws)
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))


# ------------------------------------------------------------------ one layer in one call

@pytest.mark.parametrize("out_features,in_features,g,K,iters,dt", [(256, 192, 4, 500, 3, "bf16"), (250, 131, 6, 300, 2, "f16"),
                                                                   (700, 512, 4, 9000, 2, "bf16"), (64, 40, 9, 17, 0, "f32")])
def test_layer_compress_equals_the_chain_of_calls(cc, out_features, in_features, g, K, iters, dt):
    from tests import gpu_helpers as g_

    rng = np.random.default_rng(out_features + in_features + g + K)
    W = _dev((rng.standard_normal((out_features, in_features)) * 0.02).astype(np.float32), TORCH_DT[dt])
    n = L.num_codes(in_features, out_features, g)
    ids_np = rng.choice(n, size=K, replace=False).astype(np.uint32)
    ids = _dev(ids_np.view(np.int32)).view(torch.uint32)
    book = torch.empty((K, g), dtype=torch.bfloat16, device="cuda")
    codes = torch.empty(n, dtype=torch.uint16, device="cuda")
    J = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = torch.empty(cc.layer_compress_workspace_bytes(out_features, in_features, g, K), dtype=torch.uint8, device="cuda")
    print(f"layer_compress {out_features}x{in_features} g={g} K={K} iters={iters} {dt}", flush=True)
    cc.layer_compress(W, g, iters, ids, book, codes, J, ws)
    # the same thing step by step
    X = torch.empty((n, g), dtype=torch.float32, device="cuda")
    cc.layer_vectors(W, g, X)
    Xh = X.cpu().numpy()
    C, idx, Jc, _ = g_.gpu_fit(Xh, np.ascontiguousarray(Xh[ids_np]), iters)
    book2 = torch.empty_like(book)
    codes2 = torch.empty_like(codes)
    cc.layer_pack(_dev(C), book2, _dev(idx.view(np.int32)).view(torch.uint32), codes2)
    assert torch.equal(book.view(torch.int16), book2.view(torch.int16))
    assert torch.equal(codes.view(torch.int16), codes2.view(torch.int16))
    assert J.item() == Jc
    # and against the oracle end to end (free-running on both sides; these small problems have no near-ties)
    Co, idxo, Jo, _ = oracle.kmeans_fit(L.prepare_matrix(W.float().cpu().numpy(), g), Xh[ids_np], iters)
    assert Jc == pytest.approx(Jo, rel=1e-5)
    assert np.array_equal(idx, idxo)


def test_model_driver_matches_single_calls(cc):
    """The streaming driver (copies overlapped with clustering, shared workspace) returns what separate
    cc_layer_compress calls return, layer by layer."""
    rng = np.random.default_rng(3)
    shapes = [(192, 128), (250, 128), (128, 320), (192, 128)]
    layers = [("layer%d" % i, torch.from_numpy((rng.standard_normal(s) * 0.02).astype(np.float32)).to(torch.bfloat16).pin_memory())
              for i, s in enumerate(shapes)]
    g, K, iters, seed = 4, 300, 3, 11
    got = list(cc.compress_model(layers, g, K, iters, seed))
    assert [r.name for r in got] == [n for n, _ in layers]
    for pos, ((name, w), r) in enumerate(zip(layers, got)):
        out_features, in_features = w.shape
        n = L.num_codes(in_features, out_features, g)
        from paper_2503_13089_amd.driver import init_ids

        ids = init_ids(n, K, seed + pos).cuda().view(torch.uint32)
        book = torch.empty((K, g), dtype=torch.bfloat16, device="cuda")
        codes = torch.empty(n, dtype=torch.uint16, device="cuda")
        J = torch.zeros(1, dtype=torch.float64, device="cuda")
        ws = torch.empty(cc.layer_compress_workspace_bytes(out_features, in_features, g, K), dtype=torch.uint8, device="cuda")
        cc.layer_compress(w.cuda(), g, iters, ids, book, codes, J, ws)
        assert torch.equal(r.codebook.view(torch.int16), book.cpu().view(torch.int16))
        assert torch.equal(r.codes.view(torch.int16), codes.cpu().view(torch.int16))
        assert r.inertia == J.item() and (r.in_features, r.out_features) == (in_features, out_features)
