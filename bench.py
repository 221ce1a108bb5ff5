"""Benchmark of the clustering hot path on one MI355X.

One "step" is one Lloyd iteration of the whole path through the C ABI, on centroids chained from the
previous step: cc_lloyd_iter (E-step + objective + M-step, the unit cc_kmeans_fit repeats) and cc_decode
(reconstruction). The stand-alone cc_update is timed once outside the steps for its own roofline line.
The headline value is Lloyd iterations per second on the 4096x11008, d=4, K=65536 workload with all
inputs resident in HBM. The JSON line also carries the roofline position of the dominant kernel (the
E-step) and the CPU oracle timed on this machine's host cores on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--no-cpu-baseline]
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
HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
VALU_ISSUE_PEAK = 1024 * 2.4e9 / 4   # wave-instructions/s: 1024 SIMDs, one 64-lane VALU instruction per 4 cycles

# HBM bytes per launch of the E-step kernel from rocprofv3 counters (profiles/pmc_bench_cfg3.md):
# FETCH_SIZE 295,033 KiB x 2.000 + WRITE_SIZE 88,484 KiB x 1.000, scale factors from a device copy of known size.
MEASURED_TRAFFIC_BYTES = {("cfg3_4096x11008_d4_k65536", 0): (295033 * 2.0 + 88484 * 1.0) * 1024}


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
    # prefill-sized batch: weight rebuilt once + the GEMM library (a contraction: priced against the bf16 MFMA peak)
    M = 2048
    x = torch.randn(M, in_features, device="cuda").to(bf)
    y = torch.empty(M, out_features, dtype=bf, device="cuda")
    fws = torch.empty(max(cc.layer_forward_workspace_bytes(M, in_features, out_features), 256), dtype=torch.uint8,
                      device="cuda")
    untuned_ms = timed(lambda: cc.layer_forward(x, book, codes, out_features, None, y, fws), reps=10)
    # start-up step of a serving process: time the library's candidate algorithms for this product once
    tws = torch.empty(cc.layer_forward_tune_workspace_bytes(M, in_features, out_features), dtype=torch.uint8, device="cuda")
    cc.layer_forward_tune(M, in_features, out_features, bf, False, False, tws)
    del tws
    ms = timed(lambda: cc.layer_forward(x, book, codes, out_features, None, y, fws), reps=10)
    flop = 2.0 * M * in_features * out_features
    fwd["M%d" % M] = {"avg_ms": ms, "bound": "mfma", "achieved": flop / (ms * 1e-3) / 1e12, "peak": 2500.0,
                      "unit": "TFLOP/s", "frac": flop / (ms * 1e-3) / 1e12 / 2500.0, "flop_per_launch": flop,
                      "avg_ms_with_the_library's_first_algorithm": untuned_ms,
                      "dense_matmul_on_rebuilt_weight_ms": timed(lambda: torch.matmul(x, rebuilt, out=y), reps=10)}
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
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--assign-mode", type=int, default=0)
    ap.add_argument("--model", choices=sorted(MODEL_SHAPES), default=None,
                    help="instead of the default benchmark: cluster every linear layer of a model of this shape "
                         "(synthetic weights) through the streaming driver and report the whole-model time")
    ap.add_argument("--model-g", type=int, default=4)
    ap.add_argument("--model-k", type=int, default=65500)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of the input matrix (known size) so that a counter run "
                         "can scale FETCH_SIZE / WRITE_SIZE against it")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (matrices are independent, so "
              "a multi-GPU job is one such process per GPU). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2503_13089_amd as cc
    import workloads

    cc.load_library()  # raises if the HIP library has not been built: there is no fallback
    if args.model:
        model_job(cc, torch, args)
        return
    w = next(v for k, v in workloads.WORKLOADS.items() if k.startswith(args.workload))
    cc.set_assign_mode(args.assign_mode)
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

    def job(iters):
        cc.kmeans_fit(Xd, K, iters, C0d, Cd, idx, J, ws)
        cc.decode(Cd, idx, out)

    if args.warmup > 0:
        job(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    job(args.steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    final_objective = float(J.item())
    fit_stats = cc.read_stats(ws)

    # outside the timed region: the E-step alone over the whole codebook (dominant kernel), one hinted (pruned)
    # Lloyd iteration, the stand-alone M-step and decode
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

    brute_mode = 3 if args.assign_mode == 0 else args.assign_mode
    cc.set_assign_mode(brute_mode)
    assign_ms = timed(lambda: cc.assign(Xd, Cd, idx, None, ws))
    stats = cc.read_stats(ws)
    cc.set_assign_mode(args.assign_mode)
    Cc = Cd.clone()
    iter_ms = timed(lambda: cc.lloyd_iter(Xd, Cc, idx, J, None, ws))
    Cn = torch.empty_like(Cd)
    update_ms = timed(lambda: cc.update(Xd, idx, Cd, Cn, None, ws))
    decode_ms = timed(lambda: cc.decode(Cd, idx, out), reps=10)

    layer = layer_kernels(cc, torch, timed, w, ws, idx, Cd) if w.d == 4 and K <= 65536 else None

    if args.calibrate_copy:
        out.copy_(Xd)  # N*d*4 bytes read and as many written
        torch.cuda.synchronize()

    assign_flop = 2.0 * d * N * K
    update_bytes = 4.0 * d * N + 4.0 * N + 4.0 * K * (d + 1)
    decode_bytes = 4.0 * N + 4.0 * K * d + 4.0 * d * N
    achieved = assign_flop / (assign_ms * 1e-3) / 1e12  # whole codebook scored: no pruning in this measurement
    line = {
        "metric": "Lloyd iter/s (assign+update) at 4096x11008,d=4,K=65536; % FP32 peak",
        "value": args.steps / wall, "unit": "Lloyd iter/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if args.assign_mode != 0 else "f32 (scores from exact fp16x3 products on the fp16 MFMA, fp32 accumulate)",
        "data": "synthetic",
        "config": {"workload": w.name, "rows": w.rows, "cols": w.cols, "d": d, "N": N, "K": K,
                   "step": "one Lloyd iteration inside cc_kmeans_fit(iters=steps); the timed region also holds the "
                           "fit's final E-step + objective and one cc_decode",
                   "assign_mode": args.assign_mode, "final_objective": final_objective,
                   "scored_codebook_fraction": (fit_stats.scored_stages / fit_stats.total_stages
                                                if fit_stats.total_stages else 1.0)},
        "roofline": {"bound": "mfma" if args.assign_mode != 1 else "alu",
                     "kernel": "assign (E-step), whole codebook scored (cc_set_assign_mode(%d))" % brute_mode,
                     "achieved": achieved, "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / FP32_PEAK_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, args.assign_mode)),
                     "flop_per_launch": assign_flop, "avg_ms": assign_ms},
        # the same kernel against the unit that actually bounds the fp16-MFMA variant: one v_min3_f32 per two scores
        "roofline_alu": {"bound": "alu", "kernel": "assign (E-step)", "achieved": N * K / 128.0 / (assign_ms * 1e-3) / 1e9,
                         "peak": VALU_ISSUE_PEAK / 1e9, "unit": "G wave-instr/s",
                         "frac": N * K / 128.0 / (assign_ms * 1e-3) / VALU_ISSUE_PEAK, "traffic": None},
        # what the matrix cores really execute in the default variant: 16 k-slots per (vector, centroid) pair and MFMA
        # (d = 4: 3 fp16 parts x d products + 3 norm slots = one MFMA; d = 8, 16: 2 parts x d = one, two MFMAs),
        # against the dense fp16 MFMA peak
        "roofline_mfma_f16": ({"bound": "mfma", "kernel": "assign (E-step), whole codebook scored",
                               "achieved": 2.0 * 16 * (1 if d <= 8 else 2) * N * K / (assign_ms * 1e-3) / 1e12,
                               "peak": 2500.0, "unit": "TFLOP/s",
                               "frac": 2.0 * 16 * ((3 * d + 3 + 15) // 16 if d != 16 else 3) * N * K / (assign_ms * 1e-3) / 1e12 / 2500.0,
                               "traffic": None} if args.assign_mode in (0, 3) else None),
        "standalone_lloyd_iter_ms": iter_ms,
        "other_kernels": {
            "update": {"bound": "hbm", "achieved": update_bytes / (update_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                       "unit": "GB/s", "frac": update_bytes / (update_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "bytes_per_launch": update_bytes, "avg_ms": update_ms},
            "decode": {"bound": "hbm", "achieved": decode_bytes / (decode_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                       "unit": "GB/s", "frac": decode_bytes / (decode_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "bytes_per_launch": decode_bytes, "avg_ms": decode_ms},
        },
        "refined_vectors_per_assign": stats.refined_vectors / max(1, stats.assign_calls),
    }
    if layer is not None:
        line["layer_kernels"] = layer
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, X, C0)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
