"""Pins of the layer oracle (oracle/layer.py) against things other than itself: element-by-element brute force on tiny
inputs, torch's CPU library routines (embedding, matmul, bfloat16 conversion, autograd), the constructor arithmetic of
the paper's layer listing, and round trips."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import layer


@pytest.mark.parametrize("out_features,g,expect", [(4096, 4, 0), (4096, 6, 2), (4096, 9, 8), (11008, 7, 3), (10, 4, 2), (7, 7, 0)])
def test_deficiency_and_code_count_follow_the_listing_constructor(out_features, g, expect):
    assert layer.deficiency(out_features, g) == expect
    assert (out_features + expect) % g == 0 and 0 <= expect < g
    assert layer.num_codes(5, out_features, g) == 5 * (out_features + expect) // g


def test_code_counts_of_table_1():
    # Table 1 (4096 x 4096): 4.19 M, 2.80 M and 1.86 M codes for g = 4, 6, 9
    assert round(layer.num_codes(4096, 4096, 4) / 1e6, 2) == 4.19
    assert round(layer.num_codes(4096, 4096, 6) / 1e6, 2) == 2.80
    assert round(layer.num_codes(4096, 4096, 9) / 1e6, 2) == 1.87  # with padding; the table's 1.86 is 4096*4096/9
    assert round(4096 * 4096 / 9 / 1e6, 2) == 1.86


@pytest.mark.parametrize("out_features,in_features,g", [(10, 3, 4), (12, 5, 4), (7, 2, 3), (9, 4, 9), (5, 1, 8)])
def test_prepare_matrix_elementwise(out_features, in_features, g):
    rng = np.random.default_rng(out_features * 31 + g)
    W = rng.standard_normal((out_features, in_features)).astype(np.float32)
    X = layer.prepare_matrix(W, g)
    width = out_features + layer.deficiency(out_features, g)
    assert X.shape == (in_features * width // g, g) and X.dtype == np.float32
    flat = X.reshape(-1)
    for r in range(in_features):
        for c in range(width):
            want = W[c, r] if c < out_features else 0.0
            assert flat[r * width + c] == want


@pytest.mark.parametrize("out_features,in_features,g", [(10, 3, 4), (12, 5, 4), (7, 6, 3), (64, 9, 9)])
def test_identity_codebook_round_trip(out_features, in_features, g):
    """Every vector its own centroid: reconstruction returns the transposed weight exactly."""
    rng = np.random.default_rng(7)
    W = rng.standard_normal((out_features, in_features)).astype(np.float32)
    X = layer.prepare_matrix(W, g)
    codes = np.arange(X.shape[0], dtype=np.uint32)
    back = layer.layer_weight(X, codes, in_features, out_features)
    assert back.tobytes() == np.ascontiguousarray(W.T).tobytes()


def test_layer_weight_matches_torch_embedding_view_slice():
    rng = np.random.default_rng(11)
    K, g, in_features, out_features = 50, 6, 9, 20
    C = rng.standard_normal((K, g)).astype(np.float32)
    codes = rng.integers(0, K, size=layer.num_codes(in_features, out_features, g)).astype(np.uint32)
    vectors = torch.nn.functional.embedding(torch.from_numpy(codes.astype(np.int64)), torch.from_numpy(C))
    want = vectors.view(in_features, -1)[:, :out_features].contiguous().numpy()
    assert layer.layer_weight(C, codes, in_features, out_features).tobytes() == want.tobytes()


def test_bf16_round_matches_torch_and_known_cases():
    rng = np.random.default_rng(3)
    a = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 20000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, np.inf, -np.inf, 1e-45, -1e-40, 3.3895314e38, 65504.0], np.float32),
        # exact ties: 1 + 2^-8 (rounds to even: 1.0), 1 + 3*2^-8 (rounds to 1 + 2^-6), largest finite (overflows to inf)
        np.array([1.00390625, 1.01171875, 3.4028235e38], np.float32),
    ])
    got = layer.bf16_round(a)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert got.tobytes() == want.tobytes()
    assert got[-3] == 1.0 and got[-2] == np.float32(1.015625) and np.isinf(got[-1])
    assert np.isnan(layer.bf16_round(np.array([np.nan], np.float32))[0])
    # 8 significant bits: every bf16 value survives, and the error is at most half a unit in the last place
    assert np.array_equal(layer.bf16_round(got), got)
    finite = np.isfinite(got) & (np.abs(a) > 1e-30)
    assert np.all(np.abs(got[finite] - a[finite]) <= np.abs(a[finite]) * 2.0 ** -8)


def test_layer_forward_matches_torch_fp64_matmul():
    rng = np.random.default_rng(5)
    K, g, in_features, out_features, M = 40, 4, 12, 18, 7
    C = rng.standard_normal((K, g)).astype(np.float32)
    codes = rng.integers(0, K, size=layer.num_codes(in_features, out_features, g)).astype(np.uint32)
    x = rng.standard_normal((M, in_features)).astype(np.float32)
    b = rng.standard_normal(out_features).astype(np.float32)
    W = torch.from_numpy(C).double()[torch.from_numpy(codes.astype(np.int64))].view(in_features, -1)[:, :out_features]
    want = torch.matmul(torch.from_numpy(x).double(), W) + torch.from_numpy(b).double()
    got = layer.layer_forward(x, C, codes, in_features, out_features, b)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-13, atol=1e-13)
    # one-hot inputs read out single rows of the reconstructed weight
    eye = np.eye(in_features, dtype=np.float32)
    assert np.array_equal(layer.layer_forward(eye, C, codes, in_features, out_features),
                          layer.layer_weight(C.astype(np.float64), codes, in_features, out_features))


@pytest.mark.parametrize("g,out_features", [(4, 16), (6, 20), (9, 30)])
def test_gather_backward_matches_autograd_and_bruteforce(g, out_features):
    rng = np.random.default_rng(13 + g)
    K, in_features = 23, 8
    C = torch.from_numpy(rng.standard_normal((K, g))).requires_grad_(True)  # fp64
    codes = rng.integers(0, K, size=layer.num_codes(in_features, out_features, g)).astype(np.uint32)
    G = rng.standard_normal((in_features, out_features))
    W = C[torch.from_numpy(codes.astype(np.int64))].view(in_features, -1)[:, :out_features]
    (W * torch.from_numpy(G)).sum().backward()
    got = layer.gather_backward(G, codes, K, g)
    np.testing.assert_allclose(got, C.grad.numpy(), rtol=1e-13, atol=1e-14)
    # element by element
    width = out_features + layer.deficiency(out_features, g)
    brute = np.zeros((K, g))
    for r in range(in_features):
        for c in range(out_features):
            brute[int(codes[(r * width + c) // g]), (r * width + c) % g] += G[r, c]
    np.testing.assert_allclose(got, brute, rtol=1e-13, atol=1e-14)
    # total mass is preserved, unused clusters get exactly zero
    assert got.sum() == pytest.approx(G.sum(), rel=1e-12)
    unused = np.setdiff1d(np.arange(K), codes)
    assert np.all(got[unused] == 0.0)


def _half_grid():
    """Every finite non-negative IEEE half value built from the format's definition: subnormals m * 2^-24
    (m = 0..1023), normals (1024 + m) * 2^(e - 25) for biased exponents e = 1..30."""
    vals = [Fraction(m, 2 ** 24) for m in range(1024)]
    for e in range(1, 31):
        vals += [Fraction(1024 + m) * Fraction(2) ** (e - 25) for m in range(1024)]
    return vals


def test_fp16_round_is_round_to_nearest_even_on_the_half_grid():
    """Pins oracle.layer.fp16_round without calling numpy's own half conversion: the nearest point of the half grid
    (constructed from the format's definition) in exact rational arithmetic, ties to the even mantissa, overflow to
    infinity from 65520 on; and torch's conversion as a second, independent routine."""
    import bisect

    grid = _half_grid()
    assert grid[-1] == 65504 and grid[1] == Fraction(1, 2 ** 24) and grid[1024] == Fraction(1, 2 ** 14)
    rng = np.random.default_rng(61)
    a = np.concatenate([
        (rng.standard_normal(3000) * 10.0 ** rng.integers(-9, 5, size=3000)).astype(np.float32),
        # exact ties between neighbouring half values, at several exponents, and the neighbourhood of the overflow
        np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -24 * 1.5, 2.0 ** -24 * 2.5, 2.0 ** -25, 2.0 ** -26,
                  65504.0, 65519.996, 65520.0, 70000.0, 0.0, 2.0 ** -14 - 2.0 ** -25, 1e-8, 3.0e38], np.float32)])
    a = np.concatenate([a, -a])
    got = layer.fp16_round(a)
    for x, y in zip(a.tolist(), got.tolist()):
        fx = abs(Fraction(x))
        if fx >= Fraction(65520):
            want = float("inf")
        else:
            i = bisect.bisect_left(grid, fx)
            cands = [j for j in (i - 1, i) if 0 <= j < len(grid)]
            best = min(cands, key=lambda j: (abs(grid[j] - fx), j % 2))  # even index = even mantissa (the grid is contiguous)
            want = float(grid[best])
        assert abs(y) == want and (y == 0 or (y < 0) == (x < 0)), (x, y, want)
    want_t = torch.from_numpy(a).to(torch.float16).to(torch.float32).numpy()
    assert got.tobytes() == want_t.tobytes()
    assert np.array_equal(layer.fp16_round(got[np.isfinite(got)]), got[np.isfinite(got)])  # idempotent


# ------------------------------------------------------------------ uniformly quantised codebook

@pytest.mark.parametrize("bits", [8, 4])
def test_quantize_codebook_grid_properties(bits):
    rng = np.random.default_rng(17 + bits)
    C = (rng.standard_normal((500, 4)) * 0.02).astype(np.float32)
    C[3, 1] = 0.31  # the extreme value
    q, s = layer.quantize_codebook(C, bits)
    qmax = 2 ** (bits - 1) - 1
    assert q.dtype == np.int8 and q.min() >= -qmax and q.max() == qmax and q[3, 1] == qmax
    assert s == np.float32(np.float32(0.31) / np.float32(qmax))
    # nearest grid point: error at most half a step (plus the rounding of the fp32 quotient)
    err = np.abs(q.astype(np.float64) * float(s) - C.astype(np.float64))
    assert err.max() <= 0.5 * float(s) * (1 + 1e-6)
    # odd symmetry, and grid points are fixed points
    qn, sn = layer.quantize_codebook(-C, bits)
    assert sn == s and np.array_equal(qn, -q)
    grid = (np.arange(-qmax, qmax + 1, dtype=np.float32) * s).reshape(-1, 1)
    qg, sg = layer.quantize_codebook(grid, bits)
    assert sg == s and np.array_equal(qg.reshape(-1), np.arange(-qmax, qmax + 1))
    # all-zero codebook: scale 0, codes 0, no division by zero
    q0, s0 = layer.quantize_codebook(np.zeros((3, 4), np.float32), bits)
    assert s0 == 0.0 and not q0.any()


@pytest.mark.parametrize("bits", [8, 4])
def test_quantize_codebook_matches_exact_rational_rounding(bits):
    """Away from ties (where the fp32 quotient could round either way) the integer is the exact nearest one."""
    from fractions import Fraction

    rng = np.random.default_rng(23 + bits)
    C = (rng.standard_normal((40, 3)) * 0.1).astype(np.float32)
    q, s = layer.quantize_codebook(C, bits)
    qmax = 2 ** (bits - 1) - 1
    checked = 0
    for c, got in zip(C.reshape(-1), q.reshape(-1)):
        t = Fraction(float(c)) / Fraction(float(s))
        lo = t.numerator // t.denominator
        frac = t - lo
        if abs(frac - Fraction(1, 2)) < Fraction(1, 10 ** 5):
            continue
        want = lo + (1 if frac > Fraction(1, 2) else 0)
        want = max(-(qmax + 1), min(qmax, want))
        assert got == want
        checked += 1
    assert checked > 100


def test_dequantize_and_nibble_packing():
    rng = np.random.default_rng(29)
    q = rng.integers(-8, 8, size=(33, 5)).astype(np.int8)
    packed = layer.pack_int4(q)
    assert packed.size == (q.size + 1) // 2
    assert np.array_equal(layer.unpack_int4(packed, q.size).reshape(q.shape), q)
    # element 0 in the low nibble of byte 0, element 1 in its high nibble; -1 is 0xF
    assert layer.pack_int4(np.array([-1, 2, 7, -8], np.int8)).tolist() == [0x2F, 0x87]
    s = np.float32(0.0123)
    d = layer.dequantize_codebook(q, s, "bf16")
    want = torch.from_numpy(q.astype(np.float32) * s).to(torch.bfloat16).to(torch.float32).numpy()
    assert d.tobytes() == want.tobytes()
    d16 = layer.dequantize_codebook(q, s, "f16")
    assert d16.tobytes() == (q.astype(np.float32) * s).astype(np.float16).astype(np.float32).tobytes()
