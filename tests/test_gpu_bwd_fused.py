"""GPU parity of mst_sparse_fc_bwd (both gradients of the backward pass from one walk of the
transposed view) against the CPU oracle and against the two separate entry points."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth
from oracle import products as opr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, TOL, dev, rel_err, DEV  # noqa: E402

# (T, I, O, density, mask)
CASES = [
    (300, 200, 333, 0.10, "uniform"),       # nothing a multiple of 4 / 64 / 128
    (129, 768, 768, 0.05, "uniform"),       # one token past a tile
    (512, 768, 3072, 0.05, "uniform"),      # short batch: the chunk range is split over workgroups
    (200, 130, 1100, 0.10, "uniform"),      # short batch, ragged, 9 chunks split unevenly
    (640, 3072, 768, 0.10, "uniform"),      # many row slabs, 6 chunks
    (1, 5, 3, 0.6, "uniform"),              # single token, tiny
    (2100, 200, 3850, 0.05, "uniform"),     # ragged everywhere, 31 chunks
    (700, 768, 768, 0.06, "powerlaw"),      # long rows spread over quads, empty rows
]
SHAPES = [(0, 0), (8, 3), (8, 4), (8, 5), (16, 1), (16, 2)]


def _run(rig, dYd, Xd, T, I, act):
    dX = torch.full((T, I), float("nan"), dtype=torch.float32, device=DEV)
    dW = torch.full((max(rig.layer.nnz, 1),), float("nan"), dtype=torch.float32, device=DEV)
    mst.mst_sparse_fc_bwd(rig.layer, dYd, Xd, dX, dW, T, rig.ws, act)
    torch.cuda.synchronize()
    return dX.cpu().numpy(), dW.cpu().numpy()[: rig.layer.nnz]


@pytest.mark.parametrize("T,I,O,density,mask", CASES)
def test_both_gradients_match_oracle_in_every_launch_shape(T, I, O, density, mask):
    print("case", T, I, O, density, mask, flush=True)
    W, M = synth.make_layer(41, 1, I, O, density, mask)
    X, dY = synth.make_activations(41, 1, T, I, O)
    rig = Rig(W, M, T)
    rig.layer.set_path(mst.MST_PATH_SPARSE)
    ref_dX, ref_dW = opr.fc_bwd_input(dY, W, M), opr.fc_bwd_weight(dY, X, M)
    sep_dX = rig.bwd_input(dY)
    first = None
    try:
        for shape in SHAPES:
            mst.mst_bwd_force_shape(*shape)
            dX, dW = _run(rig, dev(dY), dev(X), T, I, mst.MST_F32)
            assert rel_err(dX, ref_dX) <= TOL and rel_err(dW, ref_dW) <= TOL, shape
            if shape != (0, 0):
                # a given launch shape forms the separate call's sums, bit for bit (the automatic choice may
                # split the chunk range of a short batch, which regroups the input gradient's sum)
                np.testing.assert_array_equal(dX, sep_dX)
            else:
                assert rel_err(dX, sep_dX) <= 1e-6
            if first is None:
                first = dW
            np.testing.assert_array_equal(dW, first)             # the weight gradient is the same in every shape
    finally:
        mst.mst_bwd_force_shape(0, 0)


def test_bf16_activations():
    T, I, O = 520, 264, 392
    W, M = synth.make_layer(42, 2, I, O, 0.04)                   # below the density of the bf16 dense weight gradient
    X, dY, xb, yb = synth.make_activations(42, 2, T, I, O, "bf16")
    rig = Rig(W, M, T)
    rig.layer.set_path(mst.MST_PATH_SPARSE)
    try:
        for shape in SHAPES[1:]:
            mst.mst_bwd_force_shape(*shape)
            dX, dW = _run(rig, dev(yb.view(np.int16)), dev(xb.view(np.int16)), T, I, mst.MST_BF16)
            assert rel_err(dX, opr.fc_bwd_input(dY, W, M)) <= TOL
            assert rel_err(dW, opr.fc_bwd_weight(dY, X, M)) <= TOL
    finally:
        mst.mst_bwd_force_shape(0, 0)


@pytest.mark.parametrize("density,path", [(0.01, mst.MST_PATH_AUTO), (0.5, mst.MST_PATH_AUTO), (0.2, mst.MST_PATH_DENSE),
                                          (0.0, mst.MST_PATH_AUTO), (1.0, mst.MST_PATH_SPARSE)])
def test_paths_that_use_the_separate_kernels_or_degenerate_layers(density, path):
    T, I, O = 200, 136, 96
    W, M = synth.make_layer(43, 3, I, O, density)
    X, dY = synth.make_activations(43, 3, T, I, O)
    rig = Rig(W, M, T, cap=O * I)
    rig.layer.set_path(path)
    dX, dW = _run(rig, dev(dY), dev(X), T, I, mst.MST_F32)
    assert rel_err(dX, opr.fc_bwd_input(dY, W, M)) <= TOL
    if rig.layer.nnz:
        assert rel_err(dW, opr.fc_bwd_weight(dY, X, M)) <= TOL


def test_argument_errors():
    W, M = synth.make_layer(44, 4, 64, 48, 0.1)
    rig = Rig(W, M, 16)
    X = torch.zeros((16, 64), device=DEV)
    dY = torch.zeros((16, 48), device=DEV)
    dX = torch.zeros((16, 64), device=DEV)
    dW = torch.zeros((rig.layer.nnz,), device=DEV)
    small = torch.empty(64, dtype=torch.uint8, device=DEV)
    with pytest.raises(mst.MstError) as e:
        mst.mst_sparse_fc_bwd(rig.layer, dY, X, dX, dW, 16, small)
    assert e.value.code == -3
    with pytest.raises(mst.MstError):
        mst.mst_sparse_fc_bwd(rig.layer, dY, X, None, dW, 16, rig.ws)
    with pytest.raises(mst.MstError):
        mst.mst_sparse_fc_bwd(rig.layer, dY, X, dX, dW, 0, rig.ws)
    for bad in [(8, 2), (16, 3), (4, 4), (8, 0)]:
        with pytest.raises(mst.MstError):
            mst.mst_bwd_force_shape(*bad)


@pytest.mark.parametrize("density,act,walk", [(0.045, "f32", True), (0.065, "f32", True), (0.09, "f32", False),
                                              (0.025, "bf16", True), (0.04, "bf16", False)])
def test_automatic_path_of_the_one_call_backward(density, act, walk):
    """On the automatic path the one-call backward takes the shared walk below its own cross-over
    density (0.07 with fp32, 0.03 with bfloat16 activations on whole tiles, T >= 2048) and the two
    dense contractions above it, whatever the separate calls would choose; mst_layer_uses_dense(.., 2)
    says which; both sides agree with the oracle."""
    T, I, O = 2048, 256, 512
    W, M = synth.make_layer(47, 3, I, O, density)
    if act == "f32":
        X, dY = synth.make_activations(47, 3, T, I, O)
        Xd, dYd, a = dev(X), dev(dY), mst.MST_F32
    else:
        X, dY, xb, yb = synth.make_activations(47, 3, T, I, O, "bf16")
        Xd, dYd, a = dev(xb.view(np.int16)), dev(yb.view(np.int16)), mst.MST_BF16
    rig = Rig(W, M, T)
    assert rig.layer.uses_dense(a, T, 2) == (not walk)
    dX, dW = _run(rig, dYd, Xd, T, I, a)
    assert rel_err(dX, opr.fc_bwd_input(dY, W, M)) <= TOL and rel_err(dW, opr.fc_bwd_weight(dY, X, M)) <= TOL
    rig.layer.set_path(mst.MST_PATH_SPARSE)
    sX, sW = _run(rig, dYd, Xd, T, I, a)
    if walk:                                        # the same kernels: the same bits
        np.testing.assert_array_equal(dX, sX)
        np.testing.assert_array_equal(dW, sW)
    else:
        assert rel_err(dX, sX) <= TOL and rel_err(dW, sW) <= TOL
