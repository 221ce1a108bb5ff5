"""Per-call options of the clustering calls (the `_ex` entry points): the E-step selection never changes a result
(Section 3.1 defines the codes as the argmin, whatever computes it), a profile only observes, and the finite-input
precondition is reported instead of silently producing sums with Inf or NaN in them."""
import numpy as np
import pytest

import oracle
from tests import parity

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def cc():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2503_13089_amd as m

    m.set_assign_mode(0)
    return m


def _problem(N, d, K, seed):
    rng = np.random.default_rng(seed)
    X = (rng.standard_normal((N, d)) * 0.02).astype(np.float16).astype(np.float32)
    C = X[rng.choice(N, size=K, replace=False)].copy()
    return X, C


def test_assign_mode_is_a_per_call_choice_and_every_choice_returns_the_same_codes(cc):
    N, d, K = 70001, 4, 1000
    X, C = _problem(N, d, K, 5)
    Xd, Cd = torch.from_numpy(X).cuda(), torch.from_numpy(C).cuda()
    ws = torch.empty(cc.workspace_bytes(N, d, K), dtype=torch.uint8, device="cuda")
    got = {}
    for mode in (0, 1, 2, 3):
        print(f"cc_assign_ex mode {mode}", flush=True)
        idx = torch.empty(N, dtype=torch.uint32, device="cuda")
        J = torch.zeros(1, dtype=torch.float64, device="cuda")
        cc.assign(Xd, Cd, idx, J, ws, assign_mode=mode)
        torch.cuda.synchronize()
        got[mode] = (idx.cpu().numpy().copy(), float(J.item()))
    k1, D1, _, D2 = oracle.assign_top2(X, C)
    for mode in (0, 1, 2, 3):
        parity.check_assignment(X, C, got[mode][0], k1, D1, D2)   # every choice against the definition
        parity.check_inertia(got[mode][1], float(D1.sum()))
    for mode in (1, 2, 3):
        assert np.array_equal(got[mode][0], got[0][0]), mode      # and against each other: same codes
    # the option is an argument of the call, not state: a call without it takes the binding's default again
    idx = torch.empty(N, dtype=torch.uint32, device="cuda")
    cc.assign(Xd, Cd, idx, None, ws)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), got[0][0])


def test_profile_counts_the_kernels_of_the_calls_it_is_given_and_changes_nothing(cc):
    N, d, K, T = 600000, 4, 4096, 6   # large and long enough for the windowed E-steps and the incremental M-step
    X, C0 = _problem(N, d, K, 9)
    Xd, C0d = torch.from_numpy(X).cuda(), torch.from_numpy(C0).cuda()
    ws = torch.empty(cc.workspace_bytes(N, d, K), dtype=torch.uint8, device="cuda")

    def fit(profile):
        C = torch.empty_like(C0d)
        idx = torch.empty(N, dtype=torch.uint32, device="cuda")
        J = torch.zeros(1, dtype=torch.float64, device="cuda")
        cc.kmeans_fit(Xd, K, T, C0d, C, idx, J, ws, profile=profile)
        torch.cuda.synchronize()
        return C.cpu().numpy(), idx.cpu().numpy(), float(J.item())

    print("fit without a profile", flush=True)
    plain = fit(None)
    prof = cc.Profile(max_records=512)
    print("fit with a profile", flush=True)
    observed = fit(prof)
    assert plain[0].tobytes() == observed[0].tobytes() and np.array_equal(plain[1], observed[1]) and plain[2] == observed[2]
    ms, launches, dropped = prof.read()
    print(ms, launches, dropped, flush=True)
    assert dropped == 0
    # T E-steps + the final one (+ at most one bootstrap pass over guessed windows), one M-step call per iteration
    assert T + 1 <= launches["estep_f16"] <= T + 2
    assert launches["mstep"] >= T and launches["order"] >= 1
    # fp16 inputs: the fp32 variant is launched beside the fp16 one and switched off by its device-side gate - its
    # launches are counted, its time is that of an empty kernel
    assert launches["estep_direct"] == 0 and ms["estep_f32"] < 0.25 * ms["estep_f16"]
    for slot, n in launches.items():
        assert (ms[slot] > 0.0) == (n > 0), slot
    assert ms["estep_f16"] < 1000.0
    # reading empties it
    ms2, launches2, dropped2 = prof.read()
    assert sum(launches2.values()) == 0 and dropped2 == 0 and sum(ms2.values()) == 0.0
    prof.close()

    # a slot mask restricts what is recorded; a profile that is too small drops records and says how many
    only = cc.Profile(max_records=512, slots=("mstep",))
    fit(only)
    ms, launches, dropped = only.read()
    assert launches["mstep"] >= T and sum(launches.values()) == launches["mstep"] and dropped == 0
    only.close()
    small = cc.Profile(max_records=3)
    third = fit(small)
    ms, launches, dropped = small.read()
    assert sum(launches.values()) == 3 and dropped > 0
    assert third[0].tobytes() == plain[0].tobytes()
    small.close()


@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
def test_non_finite_inputs_are_flagged_and_kept_out_of_the_sums(cc, bad):
    N, d, K = 40000, 4, 300
    X, C0 = _problem(N, d, K, 11)
    Xd = torch.from_numpy(X).cuda()
    C0d = torch.from_numpy(C0).cuda()
    ws = torch.empty(cc.workspace_bytes(N, d, K), dtype=torch.uint8, device="cuda")
    C = torch.empty_like(C0d)
    idx = torch.empty(N, dtype=torch.uint32, device="cuda")
    cc.kmeans_fit(Xd, K, 2, C0d, C, idx, None, ws)
    torch.cuda.synchronize()
    assert cc.read_stats(ws).nonfinite_inputs == 0
    clean = C.cpu().numpy().copy()

    Xb = X.copy()
    Xb[12345, 2] = bad
    Xbd = torch.from_numpy(Xb).cuda()
    print(f"fit with one {bad} among the inputs", flush=True)
    cc.kmeans_fit(Xbd, K, 2, C0d, C, idx, None, ws)
    torch.cuda.synchronize()
    st = cc.read_stats(ws)
    assert st.nonfinite_inputs == 1
    codes = idx.cpu().numpy()
    assert codes.max() < K
    got = C.cpu().numpy()
    assert np.isfinite(got).all()    # the bad component never reached a sum
    # one vector out of 40000 moved: all but a few clusters are the clean run's, bit for bit
    changed = np.flatnonzero((got != clean).any(axis=1))
    assert changed.size <= 30, changed.size

    # stand-alone M-step: the flag is set there too, and the other components of the vector still count
    a = codes.copy()
    out = torch.empty_like(C0d)
    counts = torch.empty(K, dtype=torch.uint32, device="cuda")
    cc.update(Xbd, torch.from_numpy(a.astype(np.uint32)).cuda(), C0d, out, counts, ws)
    torch.cuda.synchronize()
    assert cc.read_stats(ws).nonfinite_inputs == 1
    Xz = Xb.copy()
    Xz[12345, 2] = 0.0
    want, want_counts = oracle.update(Xz, a, C0)
    k = a[12345]
    others = np.arange(K) != k
    assert out.cpu().numpy()[others].tobytes() == want[others].tobytes()
    assert np.array_equal(counts.cpu().numpy(), want_counts)
    # the cluster of the bad vector: its finite components are summed, the bad one contributes nothing
    row = out.cpu().numpy()[k]
    assert np.array_equal(row[[0, 1, 3]], want[k][[0, 1, 3]]) and row[2] == want[k][2]
