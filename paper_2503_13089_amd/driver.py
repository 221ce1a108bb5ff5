"""Whole-model driver: streams the linear layers of a model through cc_layer_compress, one after the other, with
the host-to-device copy of the next weight overlapped with the clustering of the current one.

Orchestration only (buffers, two HIP streams, events); every computation is a call into libcluscomp.so.
Matrices are independent (Section 3.1, Remark), so this loop is also the unit that scales out: one such
process per GPU, each with its own share of the layers.
"""
from __future__ import annotations

from dataclasses import dataclass

from . import binding as _b


@dataclass
class CompressedLayer:
    name: str
    in_features: int
    out_features: int
    codebook: object  # torch tensor [K, g], 16-bit, on the host
    codes: object     # torch tensor [num_codes], uint16, on the host
    inertia: float


def init_ids(num_vectors: int, K: int, seed: int):
    """K distinct vector indices, seeded (host tensor, int32 bit patterns of the uint32 indices)."""
    import numpy as np
    import torch

    sel = np.random.default_rng(seed).choice(num_vectors, size=K, replace=False).astype(np.uint32)
    return torch.from_numpy(sel.view(np.int32))


def compress_model(layers, g: int, K: int, iters: int = 20, seed: int = 0, keep_outputs: bool = True):
    """layers: iterable of (name, weight) with weight a host tensor [out_features, in_features] (fp32, fp16 or
    bf16; pinned memory makes the copies asynchronous). Yields one CompressedLayer per layer, in order.
    The starting centroids of a layer are a sample without replacement of its vectors, drawn from
    numpy.random.default_rng(seed + position of the layer)."""
    import torch

    _b.load_library()
    dev = torch.device("cuda")
    copy_stream = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    staged = [None, None]       # device copies of the weights in flight
    ready = [None, None]        # events: copy finished
    ws = None
    pending = None

    def stage(slot, weight):
        with torch.cuda.stream(copy_stream):
            if staged[slot] is not None:
                copy_stream.wait_event(consumed[slot])  # the previous tenant of this slot has been read
            if staged[slot] is None or staged[slot].shape != weight.shape or staged[slot].dtype != weight.dtype:
                staged[slot] = torch.empty(weight.shape, dtype=weight.dtype, device=dev)
            staged[slot].copy_(weight, non_blocking=True)
            ev = torch.cuda.Event()
            ev.record(copy_stream)
            ready[slot] = ev

    consumed = [torch.cuda.Event(), torch.cuda.Event()]
    it = iter(layers)
    try:
        cur = next(it)
    except StopIteration:
        return
    stage(0, cur[1])
    pos = 0
    while cur is not None:
        slot = pos % 2
        nxt = next(it, None)
        if nxt is not None:
            stage(1 - slot, nxt[1])
        name, weight = cur
        out_features, in_features = weight.shape
        n = _b.layer_num_codes(in_features, out_features, g)
        k = min(K, n)
        need = _b.layer_compress_workspace_bytes(out_features, in_features, g, k)
        if ws is None or ws.numel() < need:
            ws = torch.empty(need, dtype=torch.uint8, device=dev)
        ids = init_ids(n, k, seed + pos).to(dev, non_blocking=True).view(torch.uint32)
        book = torch.empty((k, g), dtype=torch.bfloat16, device=dev)
        codes = torch.empty(n, dtype=torch.uint16, device=dev)
        inertia = torch.zeros(1, dtype=torch.float64, device=dev)
        main.wait_event(ready[slot])
        _b.layer_compress(staged[slot], g, iters, ids, book, codes, inertia, ws)
        consumed[slot].record(main)
        computed = torch.cuda.Event()
        computed.record(main)
        if pending is not None:
            yield pending()
        done = torch.cuda.Event()
        # the results go back on the copy stream, behind the weight that is already on its way, so that neither the
        # next layer's clustering nor the host (which would otherwise wait on the main stream to read the objective)
        # is held up by them
        inertia_h = torch.empty(1, dtype=torch.float64, pin_memory=True)
        book_h = torch.empty(book.shape, dtype=book.dtype, pin_memory=True) if keep_outputs else None
        codes_h = torch.empty(codes.shape, dtype=codes.dtype, pin_memory=True) if keep_outputs else None
        with torch.cuda.stream(copy_stream):
            copy_stream.wait_event(computed)
            inertia_h.copy_(inertia, non_blocking=True)
            if keep_outputs:
                book_h.copy_(book, non_blocking=True)
                codes_h.copy_(codes, non_blocking=True)
            done.record(copy_stream)
        for t in (book, codes, inertia):
            t.record_stream(copy_stream)  # the allocator must not hand the memory out again before the copies ran

        def finish(name=name, i=in_features, o=out_features, b=book_h, c=codes_h, j=inertia_h, done=done):
            done.synchronize()
            return CompressedLayer(name, i, o, b, c, float(j[0]))

        pending = finish
        cur = nxt
        pos += 1
    if pending is not None:
        yield pending()
