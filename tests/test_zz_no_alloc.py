"""The entry point that allocates nothing (mst_sparse_fc_bwd_weight_static: the SDDMM's partial
sums in a device array inside the library) against mst_sparse_fc_bwd_weight with a caller
workspace: two calls in a row, the second on a smaller input, both bit for bit; and the
oracle's weight gradient within tolerance.  Sizes beyond the array are refused."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth
from oracle import products as opr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, TOL, DEV, dev, rel_err  # noqa: E402


def _both(rig, dY, X, T, act=mst.MST_F32):
    nnz = rig.layer.nnz
    a = torch.full((nnz,), float("nan"), dtype=torch.float32, device=DEV)
    b = torch.full((nnz,), float("nan"), dtype=torch.float32, device=DEV)
    mst.mst_sparse_fc_bwd_weight_static(rig.layer, dY, X, a, T, act)
    # the existing entry point pinned to the kernels the static one always runs (left to itself
    # it may form the gradient by a dense contraction: equal within tolerance, not bit for bit)
    rig.layer.set_path(mst.MST_PATH_SPARSE)
    mst.mst_sparse_fc_bwd_weight(rig.layer, dY, X, b, T, rig.ws, act)
    rig.layer.set_path(mst.MST_PATH_AUTO)
    torch.cuda.synchronize()
    return a.cpu().numpy(), b.cpu().numpy()


def test_static_scratch_entry_point_twice_second_call_smaller():
    assert mst.mst_static_scratch_bytes() == 64 << 20
    # first call: the single-layer workload (768 -> 3072, density 0.05, 512 tokens)
    I, O, T = 768, 3072, 512
    W, M = synth.make_layer(5, 1, I, O, 0.05)
    X, dY = synth.make_activations(5, 1, T, I, O)
    rig = Rig(W, M, T, cap=int(M.sum()) * 3 // 2)
    got, want = _both(rig, dev(dY), dev(X), T)
    np.testing.assert_array_equal(got, want)
    assert rel_err(got, opr.fc_bwd_weight(dY, X, M)) <= TOL
    # second call: a smaller, ragged layer and batch; the array still holds the first call's sums
    I2, O2, T2 = 200, 333, 130
    W2, M2 = synth.make_layer(5, 2, I2, O2, 0.1, "powerlaw")
    X2, dY2 = synth.make_activations(5, 2, T2, I2, O2)
    rig2 = Rig(W2, M2, T2)
    got2, want2 = _both(rig2, dev(dY2), dev(X2), T2)
    np.testing.assert_array_equal(got2, want2)
    assert rel_err(got2, opr.fc_bwd_weight(dY2, X2, M2)) <= TOL
    # and the first layer again with bfloat16 activations
    Xf, dYf, xb, yb = synth.make_activations(5, 1, T, I, O, "bf16")
    got3, want3 = _both(rig, dev(yb.view(np.int16)), dev(xb.view(np.int16)), T, mst.MST_BF16)
    np.testing.assert_array_equal(got3, want3)
    assert rel_err(got3, opr.fc_bwd_weight(dYf, Xf, M)) <= TOL


def test_static_scratch_refuses_what_does_not_fit():
    I, O = 768, 3072
    W, M = synth.make_layer(5, 3, I, O, 0.05)
    rig = Rig(W, M, 128, cap=int(M.sum()) * 3 // 2)
    T = 8192                                    # 64 planes of partial sums: far beyond 64 MiB
    X = torch.zeros((T, I), dtype=torch.float32, device=DEV)
    dY = torch.zeros((T, O), dtype=torch.float32, device=DEV)
    dW = torch.zeros(rig.layer.nnz, dtype=torch.float32, device=DEV)
    with pytest.raises(mst.MstError) as e:
        mst.mst_sparse_fc_bwd_weight_static(rig.layer, dY, X, dW, T)
    assert e.value.code == -3
