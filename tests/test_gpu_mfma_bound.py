"""Pins the one undocumented hardware property the default E-step depends on (Section 3.1: the codes must be the
true argmin, so every fast score needs a proven error bound): how far the fp32 result of
v_mfma_f32_32x32x16_f16 - chained and preset as the E-step kernel uses it - can be from the exact sum of its exact
products and its C operand.

The guard band of the fp16 E-step assumes |result - exact| <= 8 * 2^-24 * S, where S adds, for every nonzero product
a * b, max(|a|, 2^-14) * max(|b|, 2^-14) (the matrix core aligns products by the exponent fields of their factors, so an
fp16 subnormal factor weighs 2^-14 however small it is), plus |c| for the C operand. Here the instruction runs on
adversarial operand sets - the operand layouts of the kernel for d = 4, 8, 16 over eight decades of magnitude and
several centroid scales, heavy cancellation, subnormal factors, wide random exponents, every number of occupied
slots - and each of the 1024 results of a tile is compared with the exact sum (integer arithmetic on the host).
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

ULPS_ASSUMED = 8.0          # kAccumUlps in the kernel
U = 2.0 ** -24
A14 = 2.0 ** -14


def f16(v):
    return np.asarray(v, np.float64).astype(np.float16).astype(np.float64)


def exact_and_weight(A, B, C):
    """Exact C[m] + sum_q A[m][q] B[n][q] for fp16-valued A, B (float64 arrays) and the inflated sum of |terms|.
    Every product is a multiple of 2^-48 below 2^32 in magnitude; split at 2^-8 both halves sum exactly in int64."""
    P = A[:, :, None, :] * B[:, None, :, :]                       # exact in float64 (22-bit products)
    hi = np.rint(P * 2.0 ** 8)
    lo = (P - hi * 2.0 ** -8) * 2.0 ** 48
    assert np.all(lo == np.rint(lo)) and np.abs(lo).max(initial=0) < 2.0 ** 41 and np.abs(hi).max(initial=0) < 2.0 ** 41
    s_hi = hi.astype(np.int64).sum(-1)
    s_lo = lo.astype(np.int64).sum(-1)
    exact = s_hi.astype(np.float64) * 2.0 ** -8 + s_lo.astype(np.float64) * 2.0 ** -48 + C[:, :, None]
    W = (np.maximum(np.abs(A), A14)[:, :, None, :] * np.maximum(np.abs(B), A14)[:, None, :, :] * (P != 0)).sum(-1)
    return exact, W + np.abs(C)[:, :, None]


def run(cc, A, B, C):
    T = A.shape[0]
    Ad = torch.from_numpy(A.astype(np.float16)).cuda()
    Bd = torch.from_numpy(B.astype(np.float16)).cuda()
    Cd = torch.from_numpy(C.astype(np.float32)).cuda()
    D = torch.empty((T, 32, 32), dtype=torch.float32, device="cuda")
    cc.mfma_f16_probe(Ad, Bd, Cd, D)
    torch.cuda.synchronize()
    return D.cpu().numpy().astype(np.float64)


def kernel_like(d, scale, sigma_log2, rng, tiles):
    """Operands laid out as the E-step lays them out: rows of A = centroids near the vectors, split into fp16 parts
    (three for d = 4, with the norm in three more slots against fixed multipliers; two for d = 8, 16 with the norm as
    the C operand), rows of B = -2 x."""
    sigma = 2.0 ** sigma_log2
    parts = 3 if d == 4 else 2
    S = 16 if d <= 8 else 32
    A = np.zeros((tiles, 32, S)); B = np.zeros((tiles, 32, S)); C = np.zeros((tiles, 32))
    x = f16(rng.standard_normal((tiles, 32, d)) * scale)
    c = (x + rng.standard_normal((tiles, 32, d)) * scale * 0.1).astype(np.float32).astype(np.float64)
    rest = (c * sigma).astype(np.float32).astype(np.float64)
    for p in range(parts):
        h = f16(rest)
        A[:, :, p * d:(p + 1) * d] = h
        rest = rest - h
        B[:, :, p * d:(p + 1) * d] = f16(-2.0 * x)
    norm = ((c ** 2).sum(-1) * sigma).astype(np.float32).astype(np.float64)
    if d == 4:
        g0 = f16(norm / 256.0); r1 = norm - g0 * 256.0
        g1 = f16(r1 * 8.0); r2 = r1 - g1 * 0.125
        g2 = f16(r2 * 16384.0)
        A[:, :, 12], A[:, :, 13], A[:, :, 14] = g0, g1, g2
        B[:, :, 12], B[:, :, 13], B[:, :, 14] = 256.0, 0.125, 2.0 ** -14
    else:
        C = norm
    return A, B, C


def cancellation(S, rng, tiles):
    """Pairs of slots whose products cancel to the last few bits, magnitudes spread over 2^+-10 across the slots."""
    A = np.zeros((tiles, 32, S)); B = np.zeros((tiles, 32, S))
    mag = 2.0 ** rng.integers(-10, 11, size=(tiles, 32, S // 2))
    a = f16(rng.uniform(1.0, 2.0, size=(tiles, 32, S // 2)) * mag)
    A[:, :, 0::2] = a
    A[:, :, 1::2] = -f16(a * (1.0 + rng.choice([0.0, 2.0 ** -10, -2.0 ** -10], size=a.shape)))
    b = f16(rng.uniform(1.0, 2.0, size=(tiles, 32, S // 2)) * 2.0 ** rng.integers(-6, 7, size=(tiles, 32, S // 2)))
    B[:, :, 0::2] = b
    B[:, :, 1::2] = b
    C = f16(rng.standard_normal((tiles, 32))) * rng.choice([0.0, 1.0, 1024.0], size=(tiles, 32))
    return A, B, C


def subnormals(S, rng, tiles):
    """fp16 subnormal factors (multiples of 2^-24 below 2^-14) against normal ones, and against each other."""
    sub = lambda shape: rng.integers(-1023, 1024, size=shape) * 2.0 ** -24
    A = sub((tiles, 32, S)).astype(np.float64)
    B = f16(rng.standard_normal((tiles, 32, S)) * 2.0 ** rng.integers(-14, 9, size=(tiles, 32, S)))
    mix = rng.random((tiles, 32, S)) < 0.3
    A[mix] = f16(rng.standard_normal(int(mix.sum())))
    B[rng.random((tiles, 32, S)) < 0.2] = 2.0 ** -20
    C = np.zeros((tiles, 32))
    return A, B, C


def wide_exponents(S, rng, tiles, nonzero):
    """Random signs and exponents over the whole fp16 range, `nonzero` occupied slots per row."""
    def draw(shape):
        v = rng.uniform(1.0, 2.0, size=shape) * 2.0 ** rng.integers(-24, 15, size=shape) * rng.choice([-1.0, 1.0], size=shape)
        return f16(v)
    A, B = draw((tiles, 32, S)), draw((tiles, 32, S))
    keep = np.zeros(S, bool)
    keep[rng.permutation(S)[:nonzero]] = True
    A[:, :, ~keep] = 0.0
    C = f16(rng.standard_normal((tiles, 32))) * 2.0 ** rng.integers(-10, 20, size=(tiles, 32))
    return A, B, C


def test_fp16_matrix_core_accumulation_stays_inside_the_assumed_bound():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2503_13089_amd as cc

    rng = np.random.default_rng(20250313)
    sets = []
    for d in (4, 8, 16):
        for scale in (1.0, 1e-1, 1e-2, 1e-3, 1e-4, 3e-5, 1e-5, 1e-6):
            for sl in (18, 13, 8, 3, -3):
                if scale * 2.0 ** sl > 8000.0 or d * (5 * scale) ** 2 * 2.0 ** sl > 2.0 ** 23:
                    continue  # the kernel never scales its centroids out of the fp16 range
                sets.append((f"kernel layout d={d} scale={scale:g} sigma=2^{sl}", kernel_like(d, scale, sl, rng, 8)))
    for S in (16, 32):
        sets.append((f"cancellation, {S} slots", cancellation(S, rng, 32)))
        sets.append((f"subnormal factors, {S} slots", subnormals(S, rng, 32)))
        for nz in (1, 2, 3, 7, 12, 15, 16, 24, 31, 32):
            if nz <= S:
                sets.append((f"wide exponents, {nz} of {S} slots", wide_exponents(S, rng, 8, nz)))
    worst_all, outputs = 0.0, 0
    for name, (A, B, C) in sets:
        print(name, flush=True)
        D = run(cc, A, B, C)
        exact, W = exact_and_weight(A, B, C)
        err = np.abs(D - exact)
        ratio = float((err / (U * W + 1e-300)).max())
        worst_all = max(worst_all, ratio)
        outputs += D.size
        assert np.all(err <= ULPS_ASSUMED * U * W), f"{name}: error {ratio:.2f} x 2^-24 x inflated sum of |terms|"
    print(f"{outputs} results, worst error = {worst_all:.2f} x 2^-24 x S (the kernels assume {ULPS_ASSUMED:g})")
    assert worst_all <= 0.75 * ULPS_ASSUMED, "the margin on the assumed accumulation bound is nearly used up"


def test_probe_reproduces_exact_small_integer_products():
    """Sanity of the probe itself: small integers multiply and add exactly, so D must equal the integer result."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2503_13089_amd as cc

    rng = np.random.default_rng(3)
    for S in (16, 32):
        A = rng.integers(-8, 9, size=(4, 32, S)).astype(np.float64)
        B = rng.integers(-8, 9, size=(4, 32, S)).astype(np.float64)
        C = rng.integers(-100, 101, size=(4, 32)).astype(np.float64)
        D = run(cc, A, B, C)
        assert np.array_equal(D, np.einsum("tmq,tnq->tmn", A, B) + C[:, :, None])
