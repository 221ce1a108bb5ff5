"""Thin numpy <-> device wrappers around the C-ABI binding for the GPU tests."""
import numpy as np
import torch

import paper_2503_13089_amd as cc


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def workspace(N, d, K):
    nbytes = cc.workspace_bytes(N, d, K)
    assert nbytes > 0
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")


def gpu_assign(X, C, want_inertia=True, ws=None):
    N, d = X.shape
    Xd, Cd = (X if torch.is_tensor(X) else dev(X)), (C if torch.is_tensor(C) else dev(C))
    ws = workspace(N, d, Cd.shape[0]) if ws is None else ws
    idx = torch.empty(N, dtype=torch.uint32, device="cuda")
    J = torch.zeros(1, dtype=torch.float64, device="cuda") if want_inertia else None
    cc.assign(Xd, Cd, idx, J, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), (float(J.item()) if want_inertia else None)


def gpu_update(X, idx, prev, ws=None):
    N, d = X.shape
    Xd = X if torch.is_tensor(X) else dev(X)
    Pd = prev if torch.is_tensor(prev) else dev(prev)
    K = Pd.shape[0]
    ws = workspace(N, d, K) if ws is None else ws
    out = torch.empty_like(Pd)
    counts = torch.empty(K, dtype=torch.uint32, device="cuda")
    cc.update(Xd, dev(np.asarray(idx, np.uint32)), Pd, out, counts, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), counts.cpu().numpy(), cc.read_stats(ws)


def gpu_decode(C, idx):
    Cd = C if torch.is_tensor(C) else dev(C)
    idx_d = idx if torch.is_tensor(idx) else dev(np.asarray(idx, np.uint32))
    out = torch.empty((idx_d.shape[0], Cd.shape[1]), dtype=torch.float32, device="cuda")
    cc.decode(Cd, idx_d, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_fit(X, C0, iters, ws=None, Xd=None):
    N, d = X.shape
    Xd = dev(X) if Xd is None else Xd
    C0d = dev(C0)
    K = C0d.shape[0]
    ws = workspace(N, d, K) if ws is None else ws
    C = torch.empty_like(C0d)
    idx = torch.empty(N, dtype=torch.uint32, device="cuda")
    J = torch.zeros(1, dtype=torch.float64, device="cuda")
    cc.kmeans_fit(Xd, K, iters, C0d, C, idx, J, ws)
    torch.cuda.synchronize()
    return C.cpu().numpy(), idx.cpu().numpy(), float(J.item()), cc.read_stats(ws)
