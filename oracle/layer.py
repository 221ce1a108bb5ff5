"""Plain numpy definitions of the ClusComp linear layer's data path (the paper's layer listing and the
reshape footnote of Section 3.1), in fp64 wherever arithmetic happens.

TEST INFRASTRUCTURE, NOT THE PRODUCT: slow, obvious, written from the paper's description; only tests,
the smoke check and the CPU-baseline leg of the benchmark may import it.

Layout conventions (Section 3.1 footnote + layer listing)
  - The framework's linear weight is stored [out_features, in_features]. The matrix that is clustered is
    its transpose W[in_features, out_features], row-major, whose rows are cut into vectors of length g.
  - When g does not divide out_features, every row is zero-padded by `deficiency` columns, so the codes
    number in_features * (out_features + deficiency) / g, and reconstruction drops the padding again.
  - Storage: codebook in a 16-bit float format, codes as unsigned 16-bit integers (Section 3.2).
"""
from __future__ import annotations

import numpy as np


def deficiency(out_features: int, g: int) -> int:
    """Zero columns appended to each row so that g divides the row length (layer listing, constructor)."""
    r = out_features % g
    return 0 if r == 0 else g - r


def num_codes(in_features: int, out_features: int, g: int) -> int:
    """Number of codes of one layer (layer listing, constructor)."""
    return in_features * (out_features + deficiency(out_features, g)) // g


def prepare_matrix(weight, g: int):
    """Vectors to cluster from a linear weight stored [out_features, in_features] (Section 3.1 footnote):
    transpose, zero-pad each row to a multiple of g, cut rows into vectors of length g."""
    weight = np.asarray(weight)
    out_features, in_features = weight.shape
    pad = deficiency(out_features, g)
    rows = np.zeros((in_features, out_features + pad), dtype=np.float32)
    rows[:, :out_features] = weight.T
    return rows.reshape(-1, g)


def bf16_round(a):
    """fp32 -> bfloat16 (round to nearest, ties to even), returned as the fp32 value it represents.
    bfloat16 is the top 16 bits of the fp32 pattern; NaN stays NaN."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lower = bits & 0xFFFF
    upper = bits >> 16
    round_up = (lower > 0x8000) | ((lower == 0x8000) & ((upper & 1) == 1))
    upper = upper + round_up.astype(np.uint64)
    out = ((upper & 0xFFFF) << 16).astype(np.uint32)
    nan = np.isnan(a)
    out[nan] = 0x7FC00000
    return out.view(np.float32).reshape(a.shape)


def fp16_round(a):
    """fp32 -> IEEE half (round to nearest even), returned as fp32."""
    with np.errstate(over="ignore"):  # values beyond the half range round to infinity, as the format prescribes
        return np.asarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


def layer_weight(codebook, codes, in_features: int, out_features: int):
    """Reconstructed weight W[in_features, out_features] (layer listing, forward: gather the codebook rows
    by code, view as in_features rows, drop the padding columns). Pure data movement."""
    codebook = np.asarray(codebook)
    g = codebook.shape[1]
    pad = deficiency(out_features, g)
    width = out_features + pad
    vectors = codebook[np.asarray(codes, dtype=np.int64)]          # [num_codes, g]
    return np.ascontiguousarray(vectors.reshape(in_features, width)[:, :out_features])


def layer_forward(x, codebook, codes, in_features: int, out_features: int, bias=None):
    """y = x W (+ bias) in fp64 with W = layer_weight(...) (layer listing, forward)."""
    W = layer_weight(np.asarray(codebook, dtype=np.float64), codes, in_features, out_features)
    y = np.asarray(x, dtype=np.float64) @ W
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    return y


def gather_backward(grad_weight, codes, num_clusters: int, g: int):
    """Gradient of a scalar loss with respect to the codebook, given its gradient with respect to the
    reconstructed weight (the codebook is the only trainable tensor of the layer, Section 3.2/3.3):
    every weight entry is a copy of one codebook entry, so the codebook gradient is the sum of the
    gradients of its copies; padding columns are cut away in the forward pass and contribute nothing."""
    grad_weight = np.asarray(grad_weight, dtype=np.float64)
    in_features, out_features = grad_weight.shape
    width = out_features + deficiency(out_features, g)
    padded = np.zeros((in_features, width), dtype=np.float64)
    padded[:, :out_features] = grad_weight
    G = np.zeros((num_clusters, g), dtype=np.float64)
    np.add.at(G, np.asarray(codes, dtype=np.int64), padded.reshape(-1, g))  # unbuffered: repeated codes accumulate
    return G


# ---- uniformly quantised codebook (the paper's inference-only variant: Section 2's symmetric uniform grid
# applied to the codebook, Section 4.4 / the codebook-quantisation appendix) ------------------------------

def quantize_codebook(codebook, bits: int):
    """Symmetric uniform quantisation of a whole codebook with one scale: q = clamp(round(c / s), -2^(b-1),
    2^(b-1) - 1), round = to nearest (ties to even), s = max|c| / (2^(b-1) - 1), so that the grid spans the
    codebook's range. (The background formula prints 2^b - 1 under the scale, which together with its own
    clamp would clip everything above half the range; the reading taken here is the one under which the
    clamp is a safeguard only.) The paper does not fix the arithmetic: scale and quotient are taken in fp32,
    the precision of the device code, because they decide integers. Returns (q as int8, s as float32)."""
    c = np.ascontiguousarray(codebook, dtype=np.float32)
    qmax = np.float32(2 ** (bits - 1) - 1)
    s = np.float32(np.max(np.abs(c)) / qmax) if c.size else np.float32(0.0)
    if s == 0.0 or not np.isfinite(s):
        return np.zeros(c.shape, dtype=np.int8), np.float32(0.0)
    q = np.rint(np.divide(c, s, dtype=np.float32))
    q = np.clip(q, -(2 ** (bits - 1)), 2 ** (bits - 1) - 1)
    return q.astype(np.int8), s


def dequantize_codebook(q, scale, fmt: str = "bf16"):
    """c_hat = q * s in fp32, then rounded to the 16-bit format the layer computes in (returned as fp32)."""
    v = np.multiply(np.asarray(q, dtype=np.float32), np.float32(scale), dtype=np.float32)
    return bf16_round(v) if fmt == "bf16" else fp16_round(v)


def pack_int4(q):
    """Two's-complement nibbles in element order: element e sits in byte e // 2, low nibble first."""
    flat = (np.asarray(q, dtype=np.int8).reshape(-1).astype(np.int16) & 0xF).astype(np.uint8)
    if flat.size % 2:
        flat = np.concatenate([flat, np.zeros(1, np.uint8)])
    return (flat[0::2] | (flat[1::2] << 4)).astype(np.uint8)


def unpack_int4(packed, count: int):
    p = np.asarray(packed, dtype=np.uint8)
    nib = np.empty(p.size * 2, dtype=np.int16)
    nib[0::2] = p & 0xF
    nib[1::2] = p >> 4
    nib = np.where(nib >= 8, nib - 16, nib)
    return nib[:count].astype(np.int8)
