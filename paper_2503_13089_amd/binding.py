"""ctypes binding of libcluscomp.so: argument marshalling only (same names as the C entry points).

torch supplies device memory (`data_ptr()`) and the current HIP stream; nothing is computed here.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcluscomp.so")
_lib = None

EXPORTS = (
    "cc_workspace_bytes", "cc_kmeans_fit", "cc_assign", "cc_lloyd_iter", "cc_update", "cc_decode",
    "cc_kmeans_fit_ex", "cc_assign_ex", "cc_lloyd_iter_ex", "cc_update_ex",
    "cc_profile_create", "cc_profile_read", "cc_profile_destroy",
    "cc_read_stats", "cc_mfma_f16_probe", "cc_last_error", "cc_version",
    "cc_layer_deficiency", "cc_layer_num_codes", "cc_layer_vectors", "cc_layer_pack", "cc_layer_weight",
    "cc_layer_codebook_grad", "cc_layer_forward", "cc_layer_forward_workspace_bytes",
    "cc_layer_grad_plan_bytes", "cc_layer_grad_plan_workspace_bytes", "cc_layer_grad_plan",
    "cc_layer_codebook_grad_planned_workspace_bytes", "cc_layer_codebook_grad_planned",
    "cc_layer_compress", "cc_layer_compress_workspace_bytes", "cc_codebook_quantize", "cc_layer_weight_q", "cc_layer_forward_q", "cc_layer_forward_q_workspace_bytes",
)


class CCError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"cluscomp status {status}: {message}")
        self.status = status


class _CStats(ctypes.Structure):
    _fields_ = [("refined_vectors", ctypes.c_uint64), ("skipped_vectors", ctypes.c_uint64),
                ("assign_calls", ctypes.c_uint64), ("scored_stages", ctypes.c_uint64),
                ("total_stages", ctypes.c_uint64), ("fixed_point_exp", ctypes.c_int32),
                ("fp16_inputs", ctypes.c_uint32), ("nonfinite_inputs", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class _COptions(ctypes.Structure):
    _fields_ = [("struct_bytes", ctypes.c_uint32), ("assign_mode", ctypes.c_int32), ("profile", ctypes.c_void_p)]


PROFILE_SLOTS = ("estep_f16", "estep_f32", "estep_direct", "refine", "mstep", "order")


@dataclass
class Stats:
    refined_vectors: int
    skipped_vectors: int
    assign_calls: int
    scored_stages: int
    total_stages: int
    fixed_point_exp: int
    fp16_inputs: int = 0
    nonfinite_inputs: int = 0


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the built HIP library; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2503_13089_amd.build` "
            "(or __graft_entry__.build()); this package has no CPU fallback")
    # PyTorch ships a HIP runtime of its own, and the tensors passed in live in that runtime's context: it has
    # to be the one this process loads first, so that the library binds to it and not to a second copy
    import torch  # noqa: F401

    lib = ctypes.CDLL(_LIB_PATH)
    u64, u32, i32, vp, sz = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
    lib.cc_workspace_bytes.argtypes = [u64, u32, u32]
    lib.cc_workspace_bytes.restype = sz
    lib.cc_kmeans_fit.argtypes = [vp, u64, u32, u32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.cc_kmeans_fit.restype = ctypes.c_int
    lib.cc_assign.argtypes = [vp, u64, u32, vp, u32, vp, vp, vp, sz, vp]
    lib.cc_assign.restype = ctypes.c_int
    lib.cc_lloyd_iter.argtypes = [vp, u64, u32, vp, u32, vp, vp, vp, vp, sz, vp]
    lib.cc_lloyd_iter.restype = ctypes.c_int
    lib.cc_update.argtypes = [vp, u64, u32, vp, vp, u32, vp, vp, vp, sz, vp]
    lib.cc_update.restype = ctypes.c_int
    lib.cc_decode.argtypes = [vp, u32, u32, vp, u64, vp, vp]
    lib.cc_decode.restype = ctypes.c_int
    lib.cc_read_stats.argtypes = [vp, sz, ctypes.POINTER(_CStats), vp]
    lib.cc_read_stats.restype = ctypes.c_int
    op = ctypes.POINTER(_COptions)
    lib.cc_kmeans_fit_ex.argtypes = lib.cc_kmeans_fit.argtypes + [op]
    lib.cc_kmeans_fit_ex.restype = ctypes.c_int
    lib.cc_assign_ex.argtypes = lib.cc_assign.argtypes + [op]
    lib.cc_assign_ex.restype = ctypes.c_int
    lib.cc_lloyd_iter_ex.argtypes = lib.cc_lloyd_iter.argtypes + [op]
    lib.cc_lloyd_iter_ex.restype = ctypes.c_int
    lib.cc_update_ex.argtypes = lib.cc_update.argtypes + [op]
    lib.cc_update_ex.restype = ctypes.c_int
    lib.cc_profile_create.argtypes = [u32, u32, ctypes.POINTER(vp)]
    lib.cc_profile_create.restype = ctypes.c_int
    lib.cc_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(u32), ctypes.POINTER(u32)]
    lib.cc_profile_read.restype = ctypes.c_int
    lib.cc_profile_destroy.argtypes = [vp]
    lib.cc_profile_destroy.restype = None
    lib.cc_layer_deficiency.argtypes = [u32, u32]
    lib.cc_layer_deficiency.restype = u32
    lib.cc_layer_num_codes.argtypes = [u64, u64, u32]
    lib.cc_layer_num_codes.restype = u64
    lib.cc_layer_vectors.argtypes = [vp, ctypes.c_int, u32, u32, u32, vp, vp]
    lib.cc_layer_vectors.restype = ctypes.c_int
    lib.cc_layer_pack.argtypes = [vp, u32, u32, vp, ctypes.c_int, vp, u64, vp, vp]
    lib.cc_layer_pack.restype = ctypes.c_int
    lib.cc_layer_weight.argtypes = [vp, ctypes.c_int, u32, u32, vp, u32, u32, vp, vp]
    lib.cc_layer_weight.restype = ctypes.c_int
    lib.cc_layer_grad_plan_bytes.argtypes = [u64, u32]
    lib.cc_layer_grad_plan_bytes.restype = sz
    lib.cc_layer_grad_plan_workspace_bytes.argtypes = [u64]
    lib.cc_layer_grad_plan_workspace_bytes.restype = sz
    lib.cc_layer_grad_plan.argtypes = [vp, u64, u32, vp, sz, vp, sz, vp]
    lib.cc_layer_grad_plan.restype = ctypes.c_int
    lib.cc_layer_codebook_grad_planned_workspace_bytes.argtypes = [u64, u32, u32]
    lib.cc_layer_codebook_grad_planned_workspace_bytes.restype = sz
    lib.cc_layer_codebook_grad_planned.argtypes = [vp, ctypes.c_int, u32, u32, u32, u32, vp, sz, vp, vp, sz, vp]
    lib.cc_layer_codebook_grad_planned.restype = ctypes.c_int
    lib.cc_layer_forward_workspace_bytes.argtypes = [u64, u32, u32]
    lib.cc_layer_forward_workspace_bytes.restype = sz
    lib.cc_layer_forward.argtypes = [vp, u64, vp, ctypes.c_int, u32, u32, vp, u32, u32, vp, vp, vp, sz, vp]
    lib.cc_layer_forward.restype = ctypes.c_int
    lib.cc_layer_compress_workspace_bytes.argtypes = [u32, u32, u32, u32]
    lib.cc_layer_compress_workspace_bytes.restype = sz
    lib.cc_layer_compress.argtypes = [vp, ctypes.c_int, u32, u32, u32, u32, i32, vp, vp, ctypes.c_int, vp, vp, vp, sz, vp]
    lib.cc_layer_compress.restype = ctypes.c_int
    lib.cc_codebook_quantize.argtypes = [vp, u32, u32, ctypes.c_int, vp, vp, vp, vp]
    lib.cc_codebook_quantize.restype = ctypes.c_int
    lib.cc_layer_weight_q.argtypes = [vp, ctypes.c_int, vp, u32, u32, vp, u32, u32, ctypes.c_int, vp, vp]
    lib.cc_layer_weight_q.restype = ctypes.c_int
    lib.cc_layer_forward_q_workspace_bytes.argtypes = [u64, u32, u32]
    lib.cc_layer_forward_q_workspace_bytes.restype = sz
    lib.cc_layer_forward_q.argtypes = [vp, u64, vp, ctypes.c_int, vp, u32, u32, vp, u32, u32, vp, vp, ctypes.c_int, vp, sz, vp]
    lib.cc_layer_forward_q.restype = ctypes.c_int
    lib.cc_layer_codebook_grad.argtypes = [vp, ctypes.c_int, u32, u32, vp, u32, u32, vp, vp, sz, vp]
    lib.cc_layer_codebook_grad.restype = ctypes.c_int
    lib.cc_mfma_f16_probe.argtypes = [vp, vp, vp, vp, u32, u32, vp]
    lib.cc_mfma_f16_probe.restype = ctypes.c_int
    lib.cc_last_error.restype = ctypes.c_char_p
    lib.cc_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def last_error() -> str:
    return load_library().cc_last_error().decode()


def version() -> str:
    return load_library().cc_version().decode()


def _check(status: int):
    if status != 0:
        raise CCError(status, last_error())


def _ptr(t, dtype, what):
    """Device pointer of a contiguous CUDA(HIP) tensor of the expected dtype, or None."""
    import torch

    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what}: expected a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{what}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _idx_dtype():
    import torch

    return torch.uint32


# What the *_ex entry points are called with when a caller of this module does not say: cc_options are per call in
# the library; this default lives here, in the binding, so that a test can run unchanged code under each E-step kernel.
_default_assign_mode = 0


def set_assign_mode(mode: int) -> int:
    """Sets the cc_options::assign_mode that calls through this module pass from now on; returns the previous one."""
    global _default_assign_mode
    if mode not in (0, 1, 2, 3):
        raise CCError(-2, f"unknown assign mode {mode}")
    prev, _default_assign_mode = _default_assign_mode, mode
    return prev


class Profile:
    """cc_profile: device time of the library's kernels inside the calls it is passed to (`profile=`)."""

    def __init__(self, max_records: int = 256, slots=PROFILE_SLOTS):
        mask = 0
        for name in slots:
            mask |= 1 << PROFILE_SLOTS.index(name)
        self._h = ctypes.c_void_p()
        _check(load_library().cc_profile_create(max_records, mask, ctypes.byref(self._h)))

    def read(self):
        """Waits for the recorded kernels; returns ({slot: ms}, {slot: launches}, dropped) and empties the profile."""
        n = len(PROFILE_SLOTS)
        ms, launches, dropped = (ctypes.c_double * n)(), (ctypes.c_uint32 * n)(), ctypes.c_uint32()
        _check(load_library().cc_profile_read(self._h, ms, launches, ctypes.byref(dropped)))
        return ({k: float(ms[i]) for i, k in enumerate(PROFILE_SLOTS)},
                {k: int(launches[i]) for i, k in enumerate(PROFILE_SLOTS)}, int(dropped.value))

    def close(self):
        if self._h:
            load_library().cc_profile_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _options(assign_mode, profile):
    o = _COptions()
    o.struct_bytes = ctypes.sizeof(_COptions)
    o.assign_mode = _default_assign_mode if assign_mode is None else assign_mode
    o.profile = profile._h if profile is not None else None
    return ctypes.byref(o)


def workspace_bytes(N: int, d: int, K: int) -> int:
    return int(load_library().cc_workspace_bytes(N, d, K))


def kmeans_fit(vectors, K: int, iters: int, init_centroids, centroids, idx, inertia, workspace, assign_mode=None,
               profile=None) -> None:
    """cc_kmeans_fit_ex on the current stream. vectors [N,d] f32, init/centroids [K,d] f32, idx [N] uint32,
    inertia [1] f64 or None, workspace uint8 [>= workspace_bytes]. Asynchronous."""
    import torch

    N, d = vectors.shape
    lib = load_library()
    _check(lib.cc_kmeans_fit_ex(_ptr(vectors, torch.float32, "vectors"), N, d, K, iters,
                             _ptr(init_centroids, torch.float32, "init_centroids"),
                             _ptr(centroids, torch.float32, "centroids"), _ptr(idx, _idx_dtype(), "idx"),
                             _ptr(inertia, torch.float64, "inertia"), _ptr(workspace, torch.uint8, "workspace"),
                             workspace.numel(), _stream(), _options(assign_mode, profile)))


def assign(vectors, centroids, idx, inertia, workspace, assign_mode=None, profile=None) -> None:
    import torch

    N, d = vectors.shape
    K = centroids.shape[0]
    _check(load_library().cc_assign_ex(_ptr(vectors, torch.float32, "vectors"), N, d,
                                    _ptr(centroids, torch.float32, "centroids"), K, _ptr(idx, _idx_dtype(), "idx"),
                                    _ptr(inertia, torch.float64, "inertia"), _ptr(workspace, torch.uint8, "workspace"),
                                    workspace.numel(), _stream(), _options(assign_mode, profile)))


def lloyd_iter(vectors, centroids, idx, inertia, counts, workspace, assign_mode=None, profile=None) -> None:
    """cc_lloyd_iter_ex: one E-step + M-step; `centroids` is updated in place."""
    import torch

    N, d = vectors.shape
    K = centroids.shape[0]
    _check(load_library().cc_lloyd_iter_ex(_ptr(vectors, torch.float32, "vectors"), N, d,
                                        _ptr(centroids, torch.float32, "centroids"), K, _ptr(idx, _idx_dtype(), "idx"),
                                        _ptr(inertia, torch.float64, "inertia"), _ptr(counts, _idx_dtype(), "counts"),
                                        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(),
                                        _options(assign_mode, profile)))


def update(vectors, idx, prev_centroids, centroids, counts, workspace, profile=None) -> None:
    import torch

    N, d = vectors.shape
    K = prev_centroids.shape[0]
    _check(load_library().cc_update_ex(_ptr(vectors, torch.float32, "vectors"), N, d, _ptr(idx, _idx_dtype(), "idx"),
                                    _ptr(prev_centroids, torch.float32, "prev_centroids"), K,
                                    _ptr(centroids, torch.float32, "centroids"), _ptr(counts, _idx_dtype(), "counts"),
                                    _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(),
                                    _options(None, profile)))


def decode(centroids, idx, out) -> None:
    import torch

    K, d = centroids.shape
    N = idx.shape[0]
    _check(load_library().cc_decode(_ptr(centroids, torch.float32, "centroids"), K, d, _ptr(idx, _idx_dtype(), "idx"),
                                    N, _ptr(out, torch.float32, "out"), _stream()))


def read_stats(workspace) -> Stats:
    import torch

    st = _CStats()
    _check(load_library().cc_read_stats(_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                                        ctypes.byref(st), _stream()))
    return Stats(int(st.refined_vectors), int(st.skipped_vectors), int(st.assign_calls), int(st.scored_stages),
                 int(st.total_stages), int(st.fixed_point_exp), int(st.fp16_inputs), int(st.nonfinite_inputs))


def mfma_f16_probe(A, B, C, D) -> None:
    """cc_mfma_f16_probe: A, B float16 [tiles, 32, 16 * km], C float32 [tiles, 32], D float32 [tiles, 32, 32] (out)."""
    import torch

    tiles, rows, slots = A.shape
    if rows != 32 or slots not in (16, 32) or B.shape != A.shape or C.shape != (tiles, 32) or D.shape != (tiles, 32, 32):
        raise ValueError("A, B: [tiles, 32, 16 or 32]; C: [tiles, 32]; D: [tiles, 32, 32]")
    _check(load_library().cc_mfma_f16_probe(_ptr(A, torch.float16, "A"), _ptr(B, torch.float16, "B"),
                                            _ptr(C, torch.float32, "C"), _ptr(D, torch.float32, "D"), tiles, slots // 16,
                                            _stream()))


# ---- the compressed linear layer ---------------------------------------------------------------------

def _dtype_code(t) -> int:
    """cc_dtype of a tensor's element type."""
    import torch

    codes = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}
    if t.dtype not in codes:
        raise TypeError(f"unsupported element type {t.dtype}")
    return codes[t.dtype]


def _any_ptr(t, what):
    return _ptr(t, t.dtype, what) if t is not None else None


def layer_deficiency(out_features: int, g: int) -> int:
    return load_library().cc_layer_deficiency(out_features, g)


def layer_num_codes(in_features: int, out_features: int, g: int) -> int:
    return load_library().cc_layer_num_codes(in_features, out_features, g)


def layer_vectors(weight, g: int, vectors) -> None:
    import torch

    out_features, in_features = weight.shape
    _check(load_library().cc_layer_vectors(_any_ptr(weight, "weight"), _dtype_code(weight), out_features, in_features, g,
                                           _ptr(vectors, torch.float32, "vectors"), _stream()))


def layer_pack(centroids, codebook, idx, codes, K: int | None = None) -> None:
    """Either pair (centroids, codebook) / (idx, codes) may be None; K is needed when only codes are packed."""
    import torch

    K, g = (centroids.shape if centroids is not None else (K, 1))
    _check(load_library().cc_layer_pack(_ptr(centroids, torch.float32, "centroids"), K, g, _any_ptr(codebook, "codebook"),
                                        _dtype_code(codebook) if codebook is not None else 1,
                                        _ptr(idx, _idx_dtype(), "idx"), idx.numel() if idx is not None else 0,
                                        _ptr(codes, torch.uint16, "codes"), _stream()))


def layer_weight(codebook, codes, in_features: int, out_features: int, weight) -> None:
    import torch

    K, g = codebook.shape
    if weight.dtype != codebook.dtype:
        raise TypeError("weight and codebook must share one element type")
    _check(load_library().cc_layer_weight(_any_ptr(codebook, "codebook"), _dtype_code(codebook), K, g,
                                          _ptr(codes, torch.uint16, "codes"), in_features, out_features,
                                          _any_ptr(weight, "weight"), _stream()))


def layer_codebook_grad(grad_weight, codes, K: int, g: int, grad_codebook, workspace) -> None:
    import torch

    in_features, out_features = grad_weight.shape
    _check(load_library().cc_layer_codebook_grad(_any_ptr(grad_weight, "grad_weight"), _dtype_code(grad_weight), in_features,
                                                 out_features, _ptr(codes, torch.uint16, "codes"), K, g,
                                                 _ptr(grad_codebook, torch.float32, "grad_codebook"),
                                                 _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()))


def layer_grad_plan_bytes(num_codes: int, K: int) -> int:
    return load_library().cc_layer_grad_plan_bytes(num_codes, K)


def layer_grad_plan_workspace_bytes(num_codes: int) -> int:
    return load_library().cc_layer_grad_plan_workspace_bytes(num_codes)


def layer_grad_plan(codes, K: int, plan, workspace) -> None:
    """Orders the code positions by cluster into `plan` (uint8 device tensor), once per layer."""
    import torch

    _check(load_library().cc_layer_grad_plan(_ptr(codes, torch.uint16, "codes"), codes.numel(), K,
                                             _ptr(plan, torch.uint8, "plan"), plan.numel(),
                                             _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()))


def layer_codebook_grad_planned_workspace_bytes(num_codes: int, K: int, g: int) -> int:
    return load_library().cc_layer_codebook_grad_planned_workspace_bytes(num_codes, K, g)


def layer_codebook_grad_planned(grad_weight, K: int, g: int, plan, grad_codebook, workspace) -> None:
    import torch

    in_features, out_features = grad_weight.shape
    _check(load_library().cc_layer_codebook_grad_planned(_any_ptr(grad_weight, "grad_weight"), _dtype_code(grad_weight),
                                                         in_features, out_features, K, g, _ptr(plan, torch.uint8, "plan"),
                                                         plan.numel(), _ptr(grad_codebook, torch.float32, "grad_codebook"),
                                                         _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                                                         _stream()))


def layer_forward_workspace_bytes(M: int, in_features: int, out_features: int) -> int:
    return load_library().cc_layer_forward_workspace_bytes(M, in_features, out_features)


def layer_forward(x, codebook, codes, out_features: int, bias, y, workspace) -> None:
    import torch

    M, in_features = x.shape
    K, g = codebook.shape
    if x.dtype != codebook.dtype or y.dtype != codebook.dtype or (bias is not None and bias.dtype != codebook.dtype):
        raise TypeError("x, codebook, bias and y must share one element type")
    _check(load_library().cc_layer_forward(_any_ptr(x, "x"), M, _any_ptr(codebook, "codebook"), _dtype_code(codebook), K, g,
                                           _ptr(codes, torch.uint16, "codes"), in_features, out_features,
                                           _any_ptr(bias, "bias"), _any_ptr(y, "y"),
                                           _ptr(workspace, torch.uint8, "workspace"),
                                           workspace.numel() if workspace is not None else 0, _stream()))


def layer_compress_workspace_bytes(out_features: int, in_features: int, g: int, K: int) -> int:
    return load_library().cc_layer_compress_workspace_bytes(out_features, in_features, g, K)


def layer_compress(weight, g: int, iters: int, init_ids, codebook, codes, inertia, workspace) -> None:
    import torch

    out_features, in_features = weight.shape
    K = codebook.shape[0]
    _check(load_library().cc_layer_compress(_any_ptr(weight, "weight"), _dtype_code(weight), out_features, in_features, g, K,
                                            iters, _ptr(init_ids, _idx_dtype(), "init_ids"), _any_ptr(codebook, "codebook"),
                                            _dtype_code(codebook), _ptr(codes, torch.uint16, "codes"),
                                            _ptr(inertia, torch.float64, "inertia"),
                                            _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()))


# ---- uniformly quantised codebook --------------------------------------------------------------------

def codebook_quantize(centroids, bits: int, qbook, scale, scratch) -> None:
    """qbook: uint8 tensor of K*g (8 bits) or ceil(K*g/2) (4 bits) bytes; scale: 1 float32; scratch: >= 4 bytes."""
    import torch

    K, g = centroids.shape
    _check(load_library().cc_codebook_quantize(_ptr(centroids, torch.float32, "centroids"), K, g, bits,
                                               _ptr(qbook, torch.uint8, "qbook"), _ptr(scale, torch.float32, "scale"),
                                               _ptr(scratch, torch.uint8, "scratch"), _stream()))


def layer_weight_q(qbook, bits: int, scale, K: int, g: int, codes, in_features: int, out_features: int, weight) -> None:
    import torch

    _check(load_library().cc_layer_weight_q(_ptr(qbook, torch.uint8, "qbook"), bits, _ptr(scale, torch.float32, "scale"), K, g,
                                            _ptr(codes, torch.uint16, "codes"), in_features, out_features,
                                            _dtype_code(weight), _any_ptr(weight, "weight"), _stream()))


def layer_forward_q_workspace_bytes(M: int, in_features: int, out_features: int) -> int:
    return load_library().cc_layer_forward_q_workspace_bytes(M, in_features, out_features)


def layer_forward_q(x, qbook, bits: int, scale, K: int, g: int, codes, out_features: int, bias, y, workspace) -> None:
    import torch

    M, in_features = x.shape
    if y.dtype != x.dtype or (bias is not None and bias.dtype != x.dtype):
        raise TypeError("x, bias and y must share one element type")
    _check(load_library().cc_layer_forward_q(_any_ptr(x, "x"), M, _ptr(qbook, torch.uint8, "qbook"), bits,
                                             _ptr(scale, torch.float32, "scale"), K, g, _ptr(codes, torch.uint16, "codes"),
                                             in_features, out_features, _any_ptr(bias, "bias"), _any_ptr(y, "y"),
                                             _dtype_code(x), _ptr(workspace, torch.uint8, "workspace"),
                                             workspace.numel() if workspace is not None else 0, _stream()))
