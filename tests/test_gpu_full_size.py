"""Parity at the benchmark's full sizes and launch configuration (config C2: GPT-2-small
block, density 0.10, T = 8192, fp32; plus the bf16 medium fc1 of C4 and a power-law layer
of C3).  The oracle computes sampled outputs one by one; properties that hold at any size
(adjoint identities, bit-exact masks against the oracle on the same score bits) cover the rest."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth
from oracle import mixed_growing as omg
from oracle import products as opr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, TOL, dev, rel_err, DEV  # noqa: E402


from gpu_util import sampled_check as _sampled_check  # noqa: E402


@pytest.mark.parametrize("name,I,O", [("fc1", 768, 3072), ("fc2", 3072, 768), ("qkv", 768, 2304), ("proj", 768, 768)])
def test_c2_layer_products_sampled(name, I, O):
    T, d = 8192, 0.10
    print("case", name, I, O, flush=True)
    W, M = synth.make_layer(2024, 7, I, O, d)
    X, dY = synth.make_activations(2024, 7, T, I, O)
    rig = Rig(W, M, T, cap=int(M.sum()) * 3 // 2)
    Y = rig.fwd(X)
    _sampled_check("fwd", Y, lambda t, o: opr.fc_fwd_at(X, W, M, t, o), (T, O))
    dX = rig.bwd_input(dY)
    _sampled_check("bwd_input", dX, lambda t, i: opr.fc_bwd_input_at(dY, W, M, t, i), (T, I))
    dW = rig.bwd_weight(dY, X)
    flat = np.flatnonzero(M.reshape(-1))
    rng = np.random.default_rng(1)
    pick = np.unique(np.concatenate([[0, flat.size - 1], rng.integers(0, flat.size, 1500)]))
    ref = np.array([opr.dense_grad_at(dY, X, int(f // I), int(f % I)) for f in flat[pick]])
    assert np.abs(dW[pick] - ref).max() / np.abs(ref).max() <= TOL
    # the one-call backward, as the benchmark times it: the same input gradient (bit for bit from the
    # sparse kernels; on the dense path the call may cut the contraction range with its workspace,
    # another order of additions), the
    # weight gradient at the sampled positions
    dX1 = torch.full((T, I), float("nan"), dtype=torch.float32, device=DEV)
    dW1 = torch.full((rig.layer.nnz,), float("nan"), dtype=torch.float32, device=DEV)
    mst.mst_sparse_fc_bwd(rig.layer, dev(dY), dev(X), dX1, dW1, T, rig.ws)
    torch.cuda.synchronize()
    if rig.layer.uses_dense(mst.MST_F32, T):
        assert np.abs(dX1.cpu().numpy() - dX).max() <= 2e-6 * np.abs(dX).max()
    else:
        np.testing.assert_array_equal(dX1.cpu().numpy(), dX)
    dW1 = dW1.cpu().numpy()
    assert np.abs(dW1[pick] - ref).max() / np.abs(ref).max() <= TOL
    assert rel_err(dW1, dW) <= 1e-5                   # the two weight gradients differ in summation order only
    # adjoint identities tie the three full-size outputs together (fp64 reductions of fp32 outputs)
    a = float((dY.astype(np.float64) * Y).sum())
    b = float((dX.astype(np.float64) * X).sum())
    c = float((dW.astype(np.float64) * W[M != 0]).sum())
    assert abs(a - b) <= 1e-4 * abs(a) + 1e-3 and abs(a - c) <= 1e-4 * abs(a) + 1e-3


def test_c2_fc1_mask_update_full_size_bit_exact():
    I, O, T, d = 768, 3072, 8192, 0.10
    W, M = synth.make_layer(2024, 8, I, O, d)
    X, dY = synth.make_activations(2024, 8, T, I, O)
    rig = Rig(W, M, T, cap=int(M.sum()) * 3 // 2)
    G = torch.empty((O, I), dtype=torch.float32, device=DEV)
    Xd, dYd = dev(X), dev(dY)
    mst.mst_dense_grad(dYd, Xd, G, T, O, I, mst.MST_F32, rig.ws)
    torch.cuda.synchronize()
    Gh = G.cpu().numpy()
    rng = np.random.default_rng(3)
    for o, i in zip(rng.integers(0, O, 300), rng.integers(0, I, 300)):
        ref = opr.dense_grad_at(dY, X, int(o), int(i))
        assert abs(Gh[o, i] - ref) <= TOL * 400.0          # |G| is O(sqrt(T)) ~ 90; max|G| ~ 400
    st = mst.mst_mask_update(rig.layer, dYd, Xd, T, d, 0.3, 0.25, 77, rig.ws)
    torch.cuda.synchronize()
    ref = omg.update(W, M, Gh, d, 0.3, 0.25, 77)
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, ref["M"])
    np.testing.assert_array_equal(We, ref["W"])
    assert st["n_prune"] == 70779 and st["nnz_after"] == int(M.sum())


def test_c4_bf16_medium_fc1_sampled():
    I, O, T, d = 1024, 4096, 16384, 0.05
    W, M = synth.make_layer(2024, 9, I, O, d)
    Xf, dYf, xb, yb = synth.make_activations(2024, 9, T, I, O, "bf16")
    rig = Rig(W, M, T, cap=int(M.sum()) * 3 // 2)
    Y = rig.fwd(xb.view(np.int16), mst.MST_BF16)
    _sampled_check("fwd bf16", Y, lambda t, o: opr.fc_fwd_at(Xf, W, M, t, o), (T, O), n=800)
    flat = np.flatnonzero(M.reshape(-1))
    pick = np.unique(np.random.default_rng(2).integers(0, flat.size, 600))
    ref = np.array([opr.dense_grad_at(dYf, Xf, int(f // I), int(f % I)) for f in flat[pick]])
    # at this density and batch the automatic choice for bf16 is the MFMA gradient read at
    # the active positions; the SDDMM is checked as well by pinning the sparse path
    for path in (mst.MST_PATH_AUTO, mst.MST_PATH_SPARSE):
        rig.layer.set_path(path)
        dW = rig.bwd_weight(yb.view(np.int16), xb.view(np.int16), mst.MST_BF16)
        assert np.abs(dW[pick] - ref).max() / np.abs(ref).max() <= TOL, path


def test_c3_powerlaw_layer_sampled():
    I, O, T, d = 768, 3072, 16384, 0.02
    W, M = synth.make_layer(2024, 10, I, O, d, "powerlaw")
    X, dY = synth.make_activations(2024, 10, T, I, O)
    lens = M.sum(axis=1)
    assert lens.max() == I and np.median(lens) <= 4
    rig = Rig(W, M, T, cap=int(M.sum()) * 3 // 2)
    Y = rig.fwd(X)
    full = int(np.argmax(lens))
    _sampled_check("fwd powerlaw", Y, lambda t, o: opr.fc_fwd_at(X, W, M, t, o), (T, O), n=800)
    for t in (0, 5000, T - 1):                       # a completely full row and an empty one
        assert abs(Y[t, full] - opr.fc_fwd_at(X, W, M, t, full)) <= TOL * np.abs(Y).max()
    empty = np.flatnonzero(lens == 0)
    if empty.size:
        assert not Y[:, empty[0]].any()
    dX = rig.bwd_input(dY)
    _sampled_check("bwd_input powerlaw", dX, lambda t, i: opr.fc_bwd_input_at(dY, W, M, t, i), (T, I), n=800)
