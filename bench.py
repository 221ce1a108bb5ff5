"""Benchmark of the clustering hot path on one MI355X.

The timed job is the whole path through the C ABI: one cc_kmeans_fit of `steps` Lloyd iterations (each an E-step
and an M-step; the fit ends with the E-step and objective of the returned codebook) followed by one cc_decode. One
"step" is one Lloyd iteration of that job. The job is repeated (5 times by default, each repetition exactly `steps`
iterations, each bracketed by a device synchronisation) and the headline is steps / median wall time, on the
4096x11008, d=4, K=65536 workload with all inputs resident in HBM.

`roofline` prices the dominant kernel of that same timed region - the E-step's scoring kernel as the fit launches it
(windowed: it visits only the part of the codebook the triangle-inequality windows leave) - from HIP events that the
library records around exactly those launches (cc_profile) and the number of (vector, centroid) pairs they scored
(cc_stats). The whole-codebook kernels, the M-step and decode are measured after the timed region and reported under
`kernels`; whole fits of the other benchmark configurations under `other_configs`; the CPU oracle timed on this
box's host cores on a bounded sample of the same workload under `cpu_baseline`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--repeats R] [--no-cpu-baseline]
                    [--only fit|estep_whole|estep_f32|update|decode|layer_forward|layer_forward_m1|layer_grad]   (one part per process, for counter runs)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_PEAK_TFLOPS = 157.3   # MI355X fp32 vector = fp32 matrix peak
F16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 matrix peak
HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
VALU_ISSUE_PEAK = 1024 * 2.4e9 / 4   # wave-instructions/s: 1024 SIMDs, one 64-lane VALU instruction per 4 cycles

# HBM bytes per launch from rocprofv3 counter runs of `bench.py --only <kernel>` (FETCH_SIZE and WRITE_SIZE in KiB per
# dispatch, averaged over the kernel's launches, each scaled by what the same counter reads for a plain device copy of
# known size; the summaries and the factors are in profiles/pmc_*.md). Keyed by (workload, kernel).
# cfg3 figures from profiles/pmc_bench_cfg3.md: FETCH_SIZE x 1.988, WRITE_SIZE x 0.994 (a device copy of 180.4 MB
# reads 44,300 KiB x 2 dispatches on FETCH_SIZE and writes 88,580 KiB x 2 on WRITE_SIZE).
_KIB = 1024.0
MEASURED_TRAFFIC_BYTES = {
    ("cfg3_4096x11008_d4_k65536", "fit_estep"): (147500 * 1.988 + 97360 * 0.994) * _KIB,     # windowed kernel, mean of 44 launches
    ("cfg3_4096x11008_d4_k65536", "estep_whole"): (283040 * 1.988 + 88480 * 0.994) * _KIB,
    ("cfg3_4096x11008_d4_k65536", "update"): ((110200 + 18450) * 1.988 + (36860 + 3328) * 0.994) * _KIB,  # both kernels
    ("cfg3_4096x11008_d4_k65536", "decode"): (26120 * 1.988 + 176100 * 0.994) * _KIB,
}


def cpu_baseline(w, X, C0, sample_log2=20):
    """The oracle as it stands, timed on this host: one E-step over the first 2^sample_log2 vectors against
    all K centroids, scaled linearly in N (its cost is exactly proportional to N), plus one full-N M-step."""
    import numpy as np

    import oracle

    n = min(1 << sample_log2, X.shape[0])
    t0 = time.perf_counter()
    k1, _, _, _ = oracle.assign_top2(X[:n], C0)
    t_assign = time.perf_counter() - t0
    idx_full = np.resize(k1, X.shape[0])
    t0 = time.perf_counter()
    oracle.update(X, idx_full, C0)
    t_update = time.perf_counter() - t0
    t_iter = t_assign * (X.shape[0] / n) + t_update
    return {
        "value": 1.0 / t_iter, "unit": "Lloyd iter/s", "cores": oracle.threads(), "kind": "oracle",
        "build": "gcc -O2 -fopenmp (the oracle as the tests use it, not tuned)",
        "sample": f"E-step on the first {n} of {X.shape[0]} vectors x all {w.K} centroids "
                  f"({t_assign:.2f} s, scaled by N/n) + one full-N M-step ({t_update:.2f} s)",
    }


# (blocks, [(name, out_features, in_features)]) of decoder-only models, linear layers of one block
MODEL_SHAPES = {
    "llama7b": (32, [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                     ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]),
    "llama70b": (80, [("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192), ("o", 8192, 8192),
                      ("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672)]),
}


def model_job(cc, torch, args):
    """Clusters every linear layer of a model-shaped list of synthetic bf16 weights (one pinned host matrix per
    distinct shape, reused for every block: the values do not matter for the time, the copies are real) with the
    settings of the paper's Appendix B.1 (20 iterations) and prints one JSON line."""
    blocks, shapes = MODEL_SHAPES[args.model]
    gen = torch.Generator().manual_seed(20250313)
    host = {}
    for _, o, i in shapes:
        if (o, i) not in host:
            host[(o, i)] = (torch.randn((o, i), generator=gen) * 0.02).to(torch.bfloat16).pin_memory()
    layers = [("block%d.%s" % (b, n), host[(o, i)]) for b in range(blocks) for n, o, i in shapes]
    params = sum(o * i for _, o, i in shapes) * blocks
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    total_inertia = 0.0
    count = 0
    for r in cc.compress_model(layers, args.model_g, args.model_k, args.steps, seed=1, keep_outputs=True):
        total_inertia += r.inertia
        count += 1
        if count % 56 == 0:
            print("[model] %d / %d layers, %.1f s" % (count, len(layers), time.perf_counter() - t0), file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    print(json.dumps({
        "metric": "whole-model clustering time (all linear layers, host weights in, codebooks + codes out)",
        "value": wall, "unit": "s", "higher_is_better": False, "n_gpus": 1, "data": "synthetic",
        "config": {"workload": args.model, "layers": len(layers), "parameters": params, "g": args.model_g,
                   "K": args.model_k, "iters": args.steps, "weights": "bf16, pinned host memory"},
        "layers_per_s": len(layers) / wall, "sum_of_objectives": total_inertia,
    }))


def layer_kernels(cc, torch, timed, w, ws, idx, Cd):
    """The layer's data path on the benchmark matrix taken as a linear weight [out = cols, in = rows] (so that its
    transpose is the clustered matrix): reshape, storage formats, reconstruction, codebook gradient, forward."""
    in_features, out_features, g, K = w.rows, w.cols, w.d, w.K
    n = cc.layer_num_codes(in_features, out_features, g)
    bf = torch.bfloat16
    weight = (torch.randn(out_features, in_features, device="cuda") * 0.02).to(bf)
    vectors = torch.empty(n, g, dtype=torch.float32, device="cuda")
    book = torch.empty(K, g, dtype=bf, device="cuda")
    codes = torch.empty(n, dtype=torch.uint16, device="cuda")
    cc.layer_pack(Cd, book, idx, codes)
    rebuilt = torch.empty(in_features, out_features, dtype=bf, device="cuda")
    grad = torch.empty(K, g, dtype=torch.float32, device="cuda")
    res = {}

    def entry(name, ms, nbytes, bound="hbm"):
        res[name] = {"bound": bound, "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "bytes_per_launch": nbytes, "avg_ms": ms}

    entry("layer_vectors", timed(lambda: cc.layer_vectors(weight, g, vectors), reps=10), in_features * out_features * 6.0)
    entry("layer_weight", timed(lambda: cc.layer_weight(book, codes, in_features, out_features, rebuilt), reps=10),
          2.0 * n + 2.0 * K * g + 2.0 * in_features * out_features)
    entry("layer_codebook_grad", timed(lambda: cc.layer_codebook_grad(rebuilt, codes, K, g, grad, ws)),
          2.0 * in_features * out_features + 2.0 * n + 4.0 * K * g)
    # the training form: the order of the (fixed) codes prepared once, then one pass over the gradient per step
    plan = torch.empty(cc.layer_grad_plan_bytes(n, K), dtype=torch.uint8, device="cuda")
    pws = torch.empty(cc.layer_grad_plan_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    plan_ms = timed(lambda: cc.layer_grad_plan(codes, K, plan, pws))
    gws = torch.empty(cc.layer_codebook_grad_planned_workspace_bytes(n, K, g), dtype=torch.uint8, device="cuda")
    entry("layer_codebook_grad_planned", timed(lambda: cc.layer_codebook_grad_planned(rebuilt, K, g, plan, grad, gws), reps=10),
          2.0 * in_features * out_features + 4.0 * n + 4.0 * K * g)
    res["layer_codebook_grad_planned"]["plan_build_ms"] = plan_ms
    del plan, pws, gws
    fwd = {}
    for M in (1, 32):
        x = torch.randn(M, in_features, device="cuda").to(bf)
        y = torch.empty(M, out_features, dtype=bf, device="cuda")
        fws = torch.empty(max(cc.layer_forward_workspace_bytes(M, in_features, out_features), 256), dtype=torch.uint8,
                          device="cuda")
        ms = timed(lambda: cc.layer_forward(x, book, codes, out_features, None, y, fws), reps=10)
        dense_ms = timed(lambda: torch.matmul(x, rebuilt, out=y), reps=10)
        # algorithmic traffic: the codes, the codebook once, x and y; the dense product reads the whole 16-bit weight
        nbytes = 2.0 * n + 2.0 * K * g + 2.0 * M * (in_features + out_features)
        fwd["M%d" % M] = {"avg_ms": ms, "GB/s": nbytes / (ms * 1e-3) / 1e9, "bytes_per_launch": nbytes,
                          "dense_matmul_on_rebuilt_weight_ms": dense_ms}
    # prefill-sized batch: weight rebuilt once (transposed) + the library's own matrix-core product (a contraction:
    # priced against the bf16 MFMA peak; the rebuild is inside the time)
    M = 2048
    x = torch.randn(M, in_features, device="cuda").to(bf)
    y = torch.empty(M, out_features, dtype=bf, device="cuda")
    fws = torch.empty(max(cc.layer_forward_workspace_bytes(M, in_features, out_features), 256), dtype=torch.uint8,
                      device="cuda")
    ms = timed(lambda: cc.layer_forward(x, book, codes, out_features, None, y, fws), reps=10)
    flop = 2.0 * M * in_features * out_features
    fwd["M%d" % M] = {"avg_ms": ms, "bound": "mfma", "achieved": flop / (ms * 1e-3) / 1e12, "peak": 2500.0,
                      "unit": "TFLOP/s", "frac": flop / (ms * 1e-3) / 1e12 / 2500.0, "flop_per_launch": flop,
                      "framework_matmul_on_a_ready_weight_ms": timed(lambda: torch.matmul(x, rebuilt, out=y), reps=10)}
    res["layer_forward"] = fwd
    # the paper's inference variant: codebook quantised to 4 bits (128 KB: held in LDS by persistent workgroups)
    qbook = torch.empty(K * g // 2, dtype=torch.uint8, device="cuda")
    scale = torch.zeros(1, dtype=torch.float32, device="cuda")
    scratch = torch.zeros(4, dtype=torch.uint8, device="cuda")
    cc.codebook_quantize(Cd, 4, qbook, scale, scratch)
    entry("layer_weight_q4", timed(lambda: cc.layer_weight_q(qbook, 4, scale, K, g, codes, in_features, out_features, rebuilt),
                                   reps=10), 2.0 * n + 0.5 * K * g + 2.0 * in_features * out_features)
    fq = {}
    for M in (1, 8):
        x = torch.randn(M, in_features, device="cuda").to(bf)
        y = torch.empty(M, out_features, dtype=bf, device="cuda")
        fws = torch.empty(max(cc.layer_forward_q_workspace_bytes(M, in_features, out_features), 256), dtype=torch.uint8,
                          device="cuda")
        ms = timed(lambda: cc.layer_forward_q(x, qbook, 4, scale, K, g, codes, out_features, None, y, fws), reps=10)
        nbytes = 2.0 * n + 0.5 * K * g + 2.0 * M * (in_features + out_features)
        fq["M%d" % M] = {"avg_ms": ms, "GB/s": nbytes / (ms * 1e-3) / 1e9, "bytes_per_launch": nbytes}
    res["layer_forward_q4"] = fq
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--repeats", type=int, default=5, help="repetitions of the timed job (each exactly --steps iterations)")
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--no-layer-kernels", action="store_true")
    ap.add_argument("--assign-mode", type=int, default=0)
    ap.add_argument("--only", choices=["fit", "estep_whole", "estep_f32", "update", "decode", "layer_forward", "layer_forward_m1",
                                       "layer_grad"], default=None,
                    help="run just this part a few times and exit (for rocprofv3 counter runs; prints no JSON)")
    ap.add_argument("--model", choices=sorted(MODEL_SHAPES), default=None,
                    help="instead of the default benchmark: cluster every linear layer of a model of this shape "
                         "(synthetic weights) through the streaming driver and report the whole-model time")
    ap.add_argument("--model-g", type=int, default=4)
    ap.add_argument("--model-k", type=int, default=65500)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (matrices are independent, so "
              "a multi-GPU job is one such process per GPU). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import statistics

    import torch

    import paper_2503_13089_amd as cc
    import workloads

    cc.load_library()  # raises if the HIP library has not been built: there is no fallback
    if args.model:
        model_job(cc, torch, args)
        return
    w = next(v for k, v in workloads.WORKLOADS.items() if k.startswith(args.workload))
    mode = args.assign_mode
    torch.cuda.set_device(0)
    X, C0 = workloads.make_inputs(w)
    N, d, K = X.shape[0], w.d, w.K
    Xd = torch.from_numpy(X).cuda()
    Cd = torch.from_numpy(C0).cuda()
    ws = torch.empty(cc.workspace_bytes(N, d, K), dtype=torch.uint8, device="cuda")
    idx = torch.empty(N, dtype=torch.uint32, device="cuda")
    J = torch.zeros(1, dtype=torch.float64, device="cuda")
    out = torch.empty_like(Xd)
    C0d = Cd.clone()
    # device time of the E-step scoring kernels inside the timed fits (two event records per launch)
    prof = cc.Profile(max_records=64 * (args.steps + 4), slots=("estep_f16", "estep_f32", "estep_direct"))

    def job(iters, profile=None):
        cc.kmeans_fit(Xd, K, iters, C0d, Cd, idx, J, ws, assign_mode=mode, profile=profile)
        cc.decode(Cd, idx, out)

    if args.only:
        only_job(cc, torch, args, w, Xd, Cd, C0d, idx, J, out, ws)
        return

    if args.warmup > 0:
        job(args.warmup)
    walls, prof_ms, prof_n = [], dict.fromkeys(cc.PROFILE_SLOTS, 0.0), dict.fromkeys(cc.PROFILE_SLOTS, 0)
    scored = total = refined = assigns = 0
    for _ in range(max(1, args.repeats)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        job(args.steps, prof)
        torch.cuda.synchronize()
        walls.append(time.perf_counter() - t0)
        ms, launches, dropped = prof.read()
        assert dropped == 0
        st = cc.read_stats(ws)
        for k in ms:
            prof_ms[k] += ms[k]
            prof_n[k] += launches[k]
        scored += st.scored_stages
        total += st.total_stages
        refined += st.refined_vectors
        assigns += st.assign_calls
    wall = statistics.median(walls)
    ms_per_step = wall * 1e3 / args.steps
    final_objective = float(J.item())

    # the dominant kernel of the timed region: the E-step scoring kernel that ran (the other variants return at once)
    slot = max(("estep_f16", "estep_f32", "estep_direct"), key=lambda k: prof_ms[k])
    launches_per_job = prof_n[slot] / len(walls)
    launch_ms = prof_ms[slot] / max(1, prof_n[slot])
    # (vector, centroid) pairs scored per launch: with windows, the stages (32 centroids) each 512-vector tile scored
    pairs_per_launch = (scored * 32.0 * 512.0 / prof_n[slot]) if total else float(N) * K
    flop_per_launch = 2.0 * d * pairs_per_launch
    km = 1 if d <= 8 else 2            # fp16 MFMAs per (32 centroids x 32 vectors) tile: 16 k slots each
    if slot == "estep_f16":
        bound, peak, unit = "mfma", F16_MFMA_PEAK_TFLOPS, "TFLOP/s"
        kernel = "assign_mfma_f16_kernel (E-step scoring, fp16 matrix cores)" + (", windowed" if total else "")
    elif slot == "estep_f32":
        bound, peak, unit = "mfma", FP32_PEAK_TFLOPS, "TFLOP/s"
        kernel = "assign_mfma_kernel (E-step scoring, fp32 matrix cores)" + (", windowed" if total else "")
    else:
        bound, peak, unit = "alu", FP32_PEAK_TFLOPS, "TFLOP/s"
        kernel = "assign_direct_kernel (E-step, direct form on the vector ALUs)"
    achieved = flop_per_launch / (launch_ms * 1e-3) / 1e12

    def timed(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def kernel_ms(fn, slot_name, reps=3):
        """Device time per launch of one of the library's kernels inside fn (a profile's event records)."""
        p = cc.Profile(max_records=64, slots=(slot_name,))
        fn(None)
        for _ in range(reps):
            fn(p)
        ms, launches, _ = p.read()
        p.close()
        return ms[slot_name] / max(1, launches[slot_name])

    # after the timed region: the whole-codebook scoring kernels (what the E-step costs without windows), one
    # stand-alone Lloyd iteration, the stand-alone M-step and decode
    whole_ms = kernel_ms(lambda p: cc.assign(Xd, Cd, idx, None, ws, assign_mode=3 if mode == 0 else mode, profile=p),
                         "estep_direct" if (mode == 1 or K < 128) else ("estep_f32" if mode == 2 else "estep_f16"))
    f32_ms = kernel_ms(lambda p: cc.assign(Xd, Cd, idx, None, ws, assign_mode=2, profile=p), "estep_f32", reps=2) if K >= 128 else None
    Cc = Cd.clone()
    iter_ms = timed(lambda: cc.lloyd_iter(Xd, Cc, idx, J, None, ws, assign_mode=mode))
    cc.assign(Xd, Cd, idx, None, ws, assign_mode=mode)
    Cn = torch.empty_like(Cd)
    update_ms = kernel_ms(lambda p: cc.update(Xd, idx, Cd, Cn, None, ws, profile=p), "mstep", reps=5)
    decode_ms = timed(lambda: cc.decode(Cd, idx, out), reps=10)

    layer = None
    if w.d == 4 and K <= 65536 and not args.no_layer_kernels:
        layer = layer_kernels(cc, torch, timed, w, ws, idx, Cd)

    assign_flop = 2.0 * d * N * K
    update_bytes = 4.0 * d * N + 4.0 * N + 4.0 * K * (d + 1)
    decode_bytes = 4.0 * N + 4.0 * K * d + 4.0 * d * N

    def hbm(nbytes, ms, name):
        return {"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "bytes_per_launch": nbytes, "avg_ms": ms,
                "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, name))}

    kernels = {
        # the same scoring kernel over the whole codebook: 2 d N K algorithmic flop, bought as 16 k slots per pair and
        # MFMA on the fp16 matrix cores (d = 4: 3 fp16 parts x 4 products + 3 norm slots)
        "estep_whole_codebook": {
            "bound": "mfma", "avg_ms": whole_ms, "flop_per_launch": assign_flop,
            "achieved": assign_flop / (whole_ms * 1e-3) / 1e12, "unit": "TFLOP/s",
            "peak": F16_MFMA_PEAK_TFLOPS if mode in (0, 3) and K >= 128 else FP32_PEAK_TFLOPS,
            "frac": assign_flop / (whole_ms * 1e-3) / 1e12 / (F16_MFMA_PEAK_TFLOPS if mode in (0, 3) and K >= 128 else FP32_PEAK_TFLOPS),
            "issued_mfma_slot_frac": (2.0 * 16 * km * N * K / (whole_ms * 1e-3) / 1e12 / F16_MFMA_PEAK_TFLOPS
                                      if mode in (0, 3) and K >= 128 else None),
            "valu_issue_frac": N * K / 128.0 / (whole_ms * 1e-3) / VALU_ISSUE_PEAK,
            "fp32_peak_equivalent": assign_flop / (whole_ms * 1e-3) / 1e12 / FP32_PEAK_TFLOPS,
            "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, "estep_whole")),
        },
        "update": hbm(update_bytes, update_ms, "update"),
        "decode": hbm(decode_bytes, decode_ms, "decode"),
    }
    if f32_ms is not None:
        # the like-for-like "% of FP32 peak": the same algorithm on v_mfma_f32_32x32x2_f32
        kernels["estep_whole_codebook_fp32_mfma"] = {
            "bound": "mfma", "avg_ms": f32_ms, "flop_per_launch": assign_flop, "achieved": assign_flop / (f32_ms * 1e-3) / 1e12,
            "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": assign_flop / (f32_ms * 1e-3) / 1e12 / FP32_PEAK_TFLOPS,
            "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, "estep_f32"))}

    line = {
        "metric": "Lloyd iter/s (assign+update) at 4096x11008,d=4,K=65536; % FP32 peak",
        "value": args.steps / wall, "unit": "Lloyd iter/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "rows": w.rows, "cols": w.cols, "d": d, "N": N, "K": K,
                   "step": "one Lloyd iteration inside cc_kmeans_fit(iters=steps); the timed job also holds the "
                           "fit's final E-step + objective and one cc_decode",
                   "timing": "median wall time of %d repetitions of the job" % len(walls),
                   "job_wall_ms": {"median": wall * 1e3, "min": min(walls) * 1e3, "max": max(walls) * 1e3},
                   "arithmetic": ("scores from exact fp16 x fp16 products of the inputs with the centroids split into "
                                  "fp16 parts, fp32 accumulation, fp32 direct-form distances for every decision; "
                                  "cluster sums in 64-bit fixed point" if mode in (0, 3) else "fp32"),
                   "assign_mode": mode, "final_objective": final_objective,
                   "scored_codebook_fraction": (scored / total if total else 1.0),
                   "refined_vectors_per_assign": refined / max(1, assigns)},
        # the dominant kernel of the timed region, per launch, averaged over all its launches in the timed fits
        "roofline": {"bound": bound, "kernel": kernel, "achieved": achieved, "peak": peak, "unit": unit,
                     "frac": achieved / peak, "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, "fit_estep")),
                     "flop_per_launch": flop_per_launch, "pairs_per_launch": pairs_per_launch, "avg_ms": launch_ms,
                     "launches_per_job": launches_per_job,
                     "ms_per_step_in_this_kernel": launch_ms * launches_per_job / args.steps,
                     "work": "2 d flop per (vector, centroid) pair actually scored: scored stages x 32 centroids x "
                             "512 vectors, summed over the launches (cc_stats), not the whole N x K"},
        # the same launches against the unit that binds the fp16 variant: one v_min3_f32 per two scores on the vector ALUs
        "roofline_alu": {"bound": "alu", "kernel": kernel, "achieved": pairs_per_launch / 128.0 / (launch_ms * 1e-3) / 1e9,
                         "peak": VALU_ISSUE_PEAK / 1e9, "unit": "G wave-instr/s",
                         "frac": pairs_per_launch / 128.0 / (launch_ms * 1e-3) / VALU_ISSUE_PEAK, "traffic": None},
        "standalone_lloyd_iter_ms": iter_ms,
        "kernels": kernels,
    }
    if slot == "estep_f16":
        line["roofline"]["issued_mfma_slot_frac"] = 2.0 * 16 * km * pairs_per_launch / (launch_ms * 1e-3) / 1e12 / F16_MFMA_PEAK_TFLOPS
    if layer is not None:
        line["layer_kernels"] = layer
    del ws, out, Xd
    torch.cuda.empty_cache()
    if not args.no_other_configs and args.workload == "cfg3":
        line["other_configs"] = other_configs(cc, torch, workloads, w, mode)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, X, C0)
    print(json.dumps(line))


def other_configs(cc, torch, workloads, skip, mode):
    """Whole fits (iterations as listed for each configuration, + final E-step + objective) and decode of the other
    benchmark configurations: median wall time of three runs after one warm-up."""
    import statistics

    res = {}
    for w in sorted(workloads.WORKLOADS.values(), key=lambda v: v.number):
        if w.name == skip.name:
            continue
        X, C0 = workloads.make_inputs(w)
        N, d, K = X.shape[0], w.d, w.K
        Xd, C0d = torch.from_numpy(X).cuda(), torch.from_numpy(C0).cuda()
        del X
        Cd = torch.empty_like(C0d)
        ws = torch.empty(cc.workspace_bytes(N, d, K), dtype=torch.uint8, device="cuda")
        idx = torch.empty(N, dtype=torch.uint32, device="cuda")
        J = torch.zeros(1, dtype=torch.float64, device="cuda")
        out = torch.empty_like(Xd)
        walls = []
        for r in range(4):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            cc.kmeans_fit(Xd, K, w.iters, C0d, Cd, idx, J, ws, assign_mode=mode)
            cc.decode(Cd, idx, out)
            torch.cuda.synchronize()
            if r > 0:
                walls.append(time.perf_counter() - t0)
        st = cc.read_stats(ws)
        wall = statistics.median(walls)
        res[w.name] = {"iters": w.iters, "job_wall_ms": wall * 1e3, "lloyd_iter_per_s": w.iters / wall,
                       "final_objective": float(J.item()),
                       "scored_codebook_fraction": st.scored_stages / st.total_stages if st.total_stages else 1.0}
        del Xd, C0d, Cd, ws, idx, out
        torch.cuda.empty_cache()
    return res


def only_job(cc, torch, args, w, Xd, Cd, C0d, idx, J, out, ws):
    """One part of the benchmark, a few launches, nothing else: what a rocprofv3 counter run is pointed at."""
    K = w.K
    if args.only == "layer_forward":
        # the benchmark matrix as a linear layer (in = rows, out = cols) at a prefill batch of 2048 rows
        bf = torch.bfloat16
        in_features, out_features, g = w.rows, w.cols, w.d
        n = cc.layer_num_codes(in_features, out_features, g)
        book = (torch.randn(K, g, device="cuda") * 0.02).to(bf)
        codes = torch.randint(0, K, (n,), device="cuda", dtype=torch.int32).to(torch.uint16)
        x = torch.randn(2048, in_features, device="cuda").to(bf)
        y = torch.empty(2048, out_features, dtype=bf, device="cuda")
        fws = torch.empty(cc.layer_forward_workspace_bytes(2048, in_features, out_features), dtype=torch.uint8, device="cuda")
        for _ in range(5):
            cc.layer_forward(x, book, codes, out_features, None, y, fws)
    elif args.only in ("layer_forward_m1", "layer_grad"):
        # the benchmark matrix as a linear layer: one row of x through the fused forward pass, or the codebook gradient
        # of a bf16 weight gradient
        bf = torch.bfloat16
        in_features, out_features, g = w.rows, w.cols, w.d
        n = cc.layer_num_codes(in_features, out_features, g)
        book = (torch.randn(K, g, device="cuda") * 0.02).to(bf)
        codes = torch.randint(0, K, (n,), device="cuda", dtype=torch.int32).to(torch.uint16)
        if args.only == "layer_forward_m1":
            x = torch.randn(1, in_features, device="cuda").to(bf)
            y = torch.empty(1, out_features, dtype=bf, device="cuda")
            fws = torch.empty(max(cc.layer_forward_workspace_bytes(1, in_features, out_features), 256), dtype=torch.uint8, device="cuda")
            for _ in range(5):
                cc.layer_forward(x, book, codes, out_features, None, y, fws)
        else:
            gw = (torch.randn(in_features, out_features, device="cuda") * 1e-3).to(bf)
            grad = torch.empty(K, g, dtype=torch.float32, device="cuda")
            for _ in range(5):
                cc.layer_codebook_grad(gw, codes, K, g, grad, ws)
    elif args.only == "fit":
        for _ in range(2):
            cc.kmeans_fit(Xd, K, args.steps, C0d, Cd, idx, J, ws, assign_mode=args.assign_mode)
    else:
        cc.kmeans_fit(Xd, K, 3, C0d, Cd, idx, J, ws, assign_mode=args.assign_mode)  # realistic centroids and codes
        Cn = torch.empty_like(Cd)
        for _ in range(3):
            if args.only == "estep_whole":
                cc.assign(Xd, Cd, idx, None, ws, assign_mode=3)
            elif args.only == "estep_f32":
                cc.assign(Xd, Cd, idx, None, ws, assign_mode=2)
            elif args.only == "update":
                cc.update(Xd, idx, Cd, Cn, None, ws)
            elif args.only == "decode":
                cc.decode(Cd, idx, out)
    # a plain device copy of known size (N d 4 bytes read and as many written): scales FETCH_SIZE / WRITE_SIZE
    out.copy_(Xd)
    torch.cuda.synchronize()


if __name__ == "__main__":
    main()
