"""Shared helpers of the GPU parity tests: device buffers via torch, layer set-up."""
import numpy as np
import torch

import paper_2408_11746_amd as mst

DEV = "cuda:0"
TOL = 1e-4          # max|gpu - ref| / max|ref| per output tensor, fp32 values


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    m = np.abs(ref).max() if ref.size else 0.0
    if m == 0.0:
        return float(np.abs(got).max()) if got.size else 0.0
    return float(np.abs(got - ref).max() / m)


class Rig:
    """One layer on the GPU with its workspace."""

    def __init__(self, W, M, T, cap=None):
        O, I = W.shape
        self.O, self.I, self.T = O, I, T
        cap = int(cap if cap is not None else min(O * I, max(int(M.sum()) * 2, 64)))
        self.layer = mst.Layer(O, I, cap, DEV)
        self.ws = torch.empty(mst.mst_workspace_bytes(O, I, cap, T), dtype=torch.uint8, device=DEV)
        self.layer.load_dense(dev(W.astype(np.float32)), dev(M.astype(np.uint8)), self.ws)
        torch.cuda.synchronize()

    def fwd(self, X, act=mst.MST_F32):
        T = X.shape[0]
        Y = torch.full((T, self.O), float("nan"), dtype=torch.float32, device=DEV)
        mst.mst_sparse_fc_fwd(self.layer, dev(X), Y, T, act)
        torch.cuda.synchronize()
        return Y.cpu().numpy()

    def bwd_input(self, dY, act=mst.MST_F32):
        T = dY.shape[0]
        dX = torch.full((T, self.I), float("nan"), dtype=torch.float32, device=DEV)
        mst.mst_sparse_fc_bwd_input(self.layer, dev(dY), dX, T, act)
        torch.cuda.synchronize()
        return dX.cpu().numpy()

    def bwd_weight(self, dY, X, act=mst.MST_F32):
        T = X.shape[0]
        dW = torch.full((max(self.layer.nnz, 1),), float("nan"), dtype=torch.float32, device=DEV)
        mst.mst_sparse_fc_bwd_weight(self.layer, dev(dY), dev(X), dW, T, self.ws, act)
        torch.cuda.synchronize()
        return dW.cpu().numpy()[: self.layer.nnz]

    def export(self):
        W = torch.empty((self.O, self.I), dtype=torch.float32, device=DEV)
        M = torch.empty((self.O, self.I), dtype=torch.uint8, device=DEV)
        self.layer.export_dense(W, M)
        torch.cuda.synchronize()
        return W.cpu().numpy(), M.cpu().numpy()

    def indices(self):
        out = torch.empty(max(self.layer.nnz, 1), dtype=torch.int32, device=DEV)
        self.layer.indices(out)
        torch.cuda.synchronize()
        return out.cpu().numpy()[: self.layer.nnz]
