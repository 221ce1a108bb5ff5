"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header
declares, sizes its workspace, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2503_13089_amd as cc
from paper_2503_13089_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "cluscomp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cc_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = cc.load_library()
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert cc.version().startswith("cluscomp-gfx950")


def test_workspace_query():
    assert cc.workspace_bytes(65536, 4, 256) > 0
    big = cc.workspace_bytes(11272192, 4, 65536)
    assert 11272192 * 4 <= big < 1.5e9  # at least the per-vector distance array; about 1.2 GB at this size
    assert cc.workspace_bytes(65536, 4, 256) % 256 == 0
    # the M-step's record buffer holds two records (vector + 16 bytes) per vector - an incremental update writes a
    # plus and a minus record for every vector whose code changed, and all of them may change - next to the ordered
    # copy of the vectors, two code arrays, the permutation and the distances
    for N, d, K in [(11272192, 4, 65536), (1 << 20, 8, 300), (70001, 16, 65536)]:
        assert cc.workspace_bytes(N, d, K) >= 2 * N * (4 * d + 16) + N * 4 * d + 4 * N * 4
    for N, d, K in [(0, 4, 1), (10, 17, 2), (10, 0, 2), (10, 4, 0), (10, 4, 11), (1 << 32, 4, 8), (1 << 26, 4, (1 << 24) + 1)]:
        assert cc.workspace_bytes(N, d, K) == 0


A16 = ctypes.c_void_p(0x1000)      # fake, aligned, never dereferenced: every case below fails validation first
A4 = ctypes.c_void_p(0x1004)
MISALIGNED = ctypes.c_void_p(0x1001)


def _fit(lib, vectors=A16, N=1000, d=4, K=8, iters=1, init=A16, cent=A16, idx=A4, inertia=None, ws=A16, wsb=0):
    return lib.cc_kmeans_fit(vectors, N, d, K, iters, init, cent, idx, inertia, ws, wsb, None)


def test_fit_rejects_bad_arguments_without_launching():
    lib = cc.load_library()
    assert _fit(lib, vectors=None) == -1 and "NULL" in cc.last_error()
    assert _fit(lib, idx=None) == -1
    assert _fit(lib, d=17) == -2 and "d = 17" in cc.last_error()
    assert _fit(lib, N=0) == -2
    assert _fit(lib, K=0) == -2
    assert _fit(lib, K=1001) == -2 and "exceeds N" in cc.last_error()
    assert _fit(lib, N=1 << 32) == -2
    assert _fit(lib, iters=-1) == -3
    assert _fit(lib, vectors=MISALIGNED) == -4
    assert _fit(lib, ws=None) == -1
    assert _fit(lib, ws=ctypes.c_void_p(0x1010)) == -4
    assert _fit(lib, ws=ctypes.c_void_p(0x1100), wsb=cc.workspace_bytes(1000, 4, 8) - 1) == -5
    assert "needed" in cc.last_error()


def test_other_entry_points_reject_bad_arguments():
    lib = cc.load_library()
    assert lib.cc_assign(None, 10, 4, A16, 2, A4, None, A16, 0, None) == -1
    assert lib.cc_assign(A16, 10, 4, A16, 20, A4, None, A16, 0, None) == -2
    assert lib.cc_assign(A16, 10, 4, MISALIGNED, 2, A4, None, A16, 0, None) == -4
    assert lib.cc_assign(A16, 10, 4, A16, 2, A4, None, ctypes.c_void_p(0x1100), 16, None) == -5
    assert lib.cc_update(A16, 10, 4, None, A16, 2, A16, None, A16, 0, None) == -1
    assert lib.cc_update(A16, 10, 24, A4, A16, 2, A16, None, A16, 0, None) == -2
    assert lib.cc_update(A16, 10, 4, A4, A16, 2, A16, None, ctypes.c_void_p(0x1100), 16, None) == -5
    assert lib.cc_decode(None, 2, 4, A4, 10, A16, None) == -1
    assert lib.cc_decode(A16, 2, 17, A4, 10, A16, None) == -2
    assert lib.cc_decode(A16, 0, 4, A4, 10, A16, None) == -2
    assert lib.cc_decode(A16, 2, 4, A4, 10, MISALIGNED, None) == -4
    assert lib.cc_read_stats(None, 0, None, None) == -1


def test_options_and_profile_arguments():
    """The *_ex entry points take per-call options; nothing about the E-step selection is process-wide."""
    lib = cc.load_library()
    o = binding._COptions()
    o.struct_bytes, o.assign_mode = ctypes.sizeof(binding._COptions), 7
    assert _fit_ex(lib, o) == -2 and "assign mode 7" in cc.last_error()
    o.assign_mode = -1
    assert _fit_ex(lib, o) == -2
    o.struct_bytes, o.assign_mode = 4, 0
    assert _fit_ex(lib, o) == -2 and "struct_bytes" in cc.last_error()
    o.struct_bytes = ctypes.sizeof(binding._COptions)
    assert _fit_ex(lib, o, K=0) == -2 and "K == 0" in cc.last_error()      # valid options: the usual checks follow
    assert lib.cc_assign_ex(A16, 10, 4, A16, 20, A4, None, A16, 0, None, None) == -2   # NULL options = defaults
    assert lib.cc_update_ex(A16, 10, 4, None, A16, 2, A16, None, A16, 0, None, ctypes.byref(o)) == -1
    assert lib.cc_lloyd_iter_ex(A16, 10, 4, A16, 2, None, None, None, A16, 0, None, ctypes.byref(o)) == -1
    h = ctypes.c_void_p()
    assert lib.cc_profile_create(0, 1, ctypes.byref(h)) == -2
    assert lib.cc_profile_create(16, 0, ctypes.byref(h)) == -2 and lib.cc_profile_create(16, 1 << 6, ctypes.byref(h)) == -2
    assert lib.cc_profile_create(16, 1, None) == -1
    assert lib.cc_profile_read(None, None, None, None) == -1
    lib.cc_profile_destroy(None)
    with pytest.raises(cc.CCError):
        cc.set_assign_mode(9)
    prev = cc.set_assign_mode(1)
    assert cc.set_assign_mode(prev) == 1


def _fit_ex(lib, options, K=8):
    return lib.cc_kmeans_fit_ex(A16, 1000, 4, K, 1, A16, A16, A4, None, A16, 0, None, ctypes.byref(options))


def test_layer_entry_points_reject_bad_arguments():
    lib = cc.load_library()
    F32, F16, BF16 = 0, 1, 2
    assert lib.cc_layer_deficiency(4096, 6) == 2 and lib.cc_layer_deficiency(4096, 4) == 0
    assert lib.cc_layer_num_codes(4096, 4096, 9) == 4096 * 456
    assert lib.cc_layer_vectors(None, F16, 8, 8, 4, A16, None) == -1
    assert lib.cc_layer_vectors(A16, F16, 8, 8, 0, A16, None) == -2
    assert lib.cc_layer_vectors(A16, F16, 8, 8, 17, A16, None) == -2
    assert lib.cc_layer_vectors(A16, 5, 8, 8, 4, A16, None) == -2
    assert lib.cc_layer_vectors(A16, F16, 8, 8, 4, MISALIGNED, None) == -4
    assert lib.cc_layer_pack(None, 10, 4, None, F16, None, 0, None, None) == -1
    assert lib.cc_layer_pack(A16, 10, 4, None, F16, None, 0, None, None) == -1  # half a pair
    assert lib.cc_layer_pack(A16, 70000, 4, A16, F16, None, 0, None, None) == -2 and "16-bit codes" in cc.last_error()
    assert lib.cc_layer_pack(A16, 10, 4, A16, F32, None, 0, None, None) == -2
    assert lib.cc_layer_pack(None, 10, 4, None, F16, A4, 0, A16, None) == -2
    assert lib.cc_layer_weight(A16, BF16, 10, 4, None, 8, 8, A16, None) == -1
    assert lib.cc_layer_weight(A16, BF16, 0, 4, A16, 8, 8, A16, None) == -2
    assert lib.cc_layer_weight(A16, BF16, 10, 4, A16, 0, 8, A16, None) == -2
    assert lib.cc_layer_weight(A16, BF16, 10, 4, A16, 8, 8, MISALIGNED, None) == -4
    assert lib.cc_layer_codebook_grad(A16, F32, 8, 8, A16, 10, 4, None, A16, 0, None) == -1
    assert lib.cc_layer_codebook_grad(A16, F32, 8, 8, A16, 10, 4, A16, None, 0, None) == -1
    assert lib.cc_layer_codebook_grad(A16, F32, 8, 8, A16, 10, 4, A16, ctypes.c_void_p(0x1100), 16, None) == -5
    assert lib.cc_layer_codebook_grad(A16, F32, 8, 8, A16, 10, 4, A16, ctypes.c_void_p(0x1010), 1 << 30, None) == -4


def test_forward_and_quantised_entry_points_reject_bad_arguments():
    lib = cc.load_library()
    F32, F16, BF16 = 0, 1, 2
    WS = ctypes.c_void_p(0x1100)
    assert lib.cc_layer_forward_workspace_bytes(0, 64, 64) == 0
    assert lib.cc_layer_forward_workspace_bytes(1, 4096, 4096) % 256 == 0 and lib.cc_layer_forward_workspace_bytes(1, 4096, 4096) > 0
    assert lib.cc_layer_forward(None, 1, A16, BF16, 10, 4, A16, 64, 64, None, A16, WS, 1 << 30, None) == -1
    assert lib.cc_layer_forward(A16, 0, A16, BF16, 10, 4, A16, 64, 64, None, A16, WS, 1 << 30, None) == -2
    assert lib.cc_layer_forward(A16, 1, A16, F32, 10, 4, A16, 64, 64, None, A16, WS, 1 << 30, None) == -2  # 16-bit only
    assert lib.cc_layer_forward(A16, 1, A16, BF16, 10, 4, A16, 60, 64, None, A16, WS, 1 << 30, None) == -2
    assert "multiple of 8" in cc.last_error()
    assert lib.cc_layer_forward(A16, 1, A16, BF16, 10, 4, A16, 64, 64, None, MISALIGNED, WS, 1 << 30, None) == -4
    assert lib.cc_layer_forward(A16, 1, A16, BF16, 10, 4, A16, 4096, 4096, None, A16, None, 0, None) == -1
    assert lib.cc_layer_forward(A16, 1, A16, BF16, 10, 4, A16, 4096, 4096, None, A16, WS, 16, None) == -5
    assert lib.cc_codebook_quantize(None, 10, 4, 4, A16, A16, A16, None) == -1
    assert lib.cc_codebook_quantize(A16, 10, 4, 3, A16, A16, A16, None) == -2 and "bits = 3" in cc.last_error()
    assert lib.cc_codebook_quantize(A16, 70000, 4, 4, A16, A16, A16, None) == -2
    assert lib.cc_layer_weight_q(A16, 4, A16, 10, 4, A16, 8, 8, F32, A16, None) == -2
    assert lib.cc_layer_weight_q(A16, 2, A16, 10, 4, A16, 8, 8, BF16, A16, None) == -2
    assert lib.cc_layer_weight_q(A16, 4, None, 10, 4, A16, 8, 8, BF16, A16, None) == -1
    assert lib.cc_layer_forward_q_workspace_bytes(1, 4096, 4096) >= lib.cc_layer_forward_workspace_bytes(1, 4096, 4096)
    # prefill-sized batches: room for the rebuilt weight (whole matrix-core operands: columns padded to 32, in-features
    # to 16) and for fp32 partial tiles where the contraction is split; the quantised route also holds the integer
    # codebook in 16 bits (2 MiB)
    big = lib.cc_layer_forward_workspace_bytes(2048, 4096, 4096)
    assert big >= 4096 * 4096 * 2 and big % 256 == 0
    big_q = lib.cc_layer_forward_q_workspace_bytes(2048, 4096, 4096)
    assert big_q == big + (2 << 20)
    assert lib.cc_layer_forward_workspace_bytes(4096, 4104, 4100) >= 4128 * 4112 * 2
    assert lib.cc_layer_forward_workspace_bytes(128, 4096, 4096) > 4096 * 4096 * 2 + 128 * 4096 * 4
    assert lib.cc_layer_forward(A16, 2048, A16, BF16, 10, 4, A16, 4096, 4096, None, A16, WS, 16, None) == -5
    assert lib.cc_layer_forward_q(A16, 1, A16, 4, A16, 10, 4, A16, 64, 64, None, A16, BF16, None, 0, None) == -1
    assert lib.cc_layer_forward_q(A16, 1, A16, 5, A16, 10, 4, A16, 64, 64, None, A16, BF16, WS, 1 << 30, None) == -2
    assert lib.cc_layer_forward_q(A16, 1, A16, 4, A16, 10, 4, A16, 64, 64, None, A16, BF16, WS, 16, None) == -5


def test_planned_gradient_entry_points_reject_bad_arguments():
    lib = cc.load_library()
    BF16 = 2
    P = ctypes.c_void_p(0x1100)
    n = 96 * 50  # codes of a 96 x 200 layer at g = 4
    assert lib.cc_layer_grad_plan_bytes(0, 10) == 0 and lib.cc_layer_grad_plan_bytes(n, 70000) == 0
    need = lib.cc_layer_grad_plan_bytes(n, 50)
    assert need >= 4 * n + 2 * 4 * 51 and need % 256 == 0
    assert lib.cc_layer_grad_plan_workspace_bytes(n) >= 8 * n
    assert lib.cc_layer_codebook_grad_planned_workspace_bytes(n, 50, 4) >= 50 * 4 * 8
    assert lib.cc_layer_codebook_grad_planned_workspace_bytes(n, 50, 17) == 0
    assert lib.cc_layer_grad_plan(None, n, 50, P, 1 << 30, P, 1 << 30, None) == -1
    assert lib.cc_layer_grad_plan(A16, 0, 50, P, 1 << 30, P, 1 << 30, None) == -2
    assert lib.cc_layer_grad_plan(A16, n, 70000, P, 1 << 30, P, 1 << 30, None) == -2
    assert lib.cc_layer_grad_plan(A16, n, 50, MISALIGNED, 1 << 30, P, 1 << 30, None) == -4
    assert lib.cc_layer_grad_plan(A16, n, 50, P, need - 1, P, 1 << 30, None) == -5
    assert lib.cc_layer_grad_plan(A16, n, 50, P, need, P, 16, None) == -5
    assert lib.cc_layer_codebook_grad_planned(None, BF16, 96, 200, 50, 4, P, need, A16, P, 1 << 30, None) == -1
    assert lib.cc_layer_codebook_grad_planned(A16, BF16, 96, 200, 50, 17, P, need, A16, P, 1 << 30, None) == -2
    assert lib.cc_layer_codebook_grad_planned(A16, BF16, 96, 200, 50, 4, P, need - 1, A16, P, 1 << 30, None) == -5
    assert "plan has" in cc.last_error()
    assert lib.cc_layer_codebook_grad_planned(A16, BF16, 96, 200, 50, 4, P, need, A16, P, 16, None) == -5
    assert lib.cc_layer_codebook_grad_planned(MISALIGNED, BF16, 96, 200, 50, 4, P, need, A16, P, 1 << 30, None) == -4


def test_binding_refuses_host_tensors():
    import torch

    x = torch.zeros(16, 4)
    with pytest.raises(TypeError):
        cc.decode(x, torch.zeros(16, dtype=torch.int32), x)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching a device."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    proc = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                          timeout=120)
    assert proc.returncode == 2
    assert "one GPU" in proc.stderr and proc.stdout.strip() == ""


def test_build_refuses_a_hand_scheduled_kernel_that_spills():
    """The product kernel of the prefill route places its memory waits by hand; the build reads the compiler's
    resource report and must fail if that kernel ever needs scratch memory."""
    from paper_2503_13089_amd import build as b

    head = "f.hip:1:1: remark: Function Name: _ZN2cc12_GLOBAL__N_116gemm_frag_kernelILi2EEEvPKt [-Rpass-analysis=kernel-resource-usage]\n"
    ok = head + "f.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-R]\nf.hip:1:1: remark:     VGPRs Spill: 0 [-R]\n"
    b._check_no_spills("/x/layer_gemm.hip", ok)
    other = "f.hip:1:1: remark: Function Name: some_other_kernel [-R]\nf.hip:1:1: remark:     VGPRs Spill: 9 [-R]\n"
    b._check_no_spills("/x/layer_gemm.hip", ok + other)          # only the listed kernels are held to it
    b._check_no_spills("/x/decode.hip", other)                    # files without such kernels are not checked
    with pytest.raises(RuntimeError, match="spills"):
        b._check_no_spills("/x/layer_gemm.hip", ok.replace("Spill: 0", "Spill: 4"))
    with pytest.raises(RuntimeError, match="scratch"):
        b._check_no_spills("/x/layer_gemm.hip", ok.replace("lane]: 0", "lane]: 16"))
    with pytest.raises(RuntimeError, match="no resource report"):
        b._check_no_spills("/x/layer_gemm.hip", other)
