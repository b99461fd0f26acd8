"""Seeded random layers (shape, density, mask kind, launch shape, path) through the C ABI
against the oracle: the three products, the one-call backward, a Mixed-Growing update from given scores
(bit-exact mask and weights) and the products again on the updated layer."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth
from oracle import mixed_growing as omg
from oracle import products as opr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, TOL, dev, rel_err, DEV  # noqa: E402

BWD_SHAPES = [(0, 0), (8, 3), (16, 1)]


def _bwd_one_call(rig, dY, X, T, I, shape):
    """Both gradients through mst_sparse_fc_bwd in a given launch shape."""
    dX = torch.full((T, I), float("nan"), dtype=torch.float32, device=DEV)
    dW = torch.full((max(rig.layer.nnz, 1),), float("nan"), dtype=torch.float32, device=DEV)
    try:
        mst.mst_bwd_force_shape(*shape)
        mst.mst_sparse_fc_bwd(rig.layer, dev(dY), dev(X), dX, dW, T, rig.ws)
        torch.cuda.synchronize()
    finally:
        mst.mst_bwd_force_shape(0, 0)
    return dX.cpu().numpy(), dW.cpu().numpy()[: rig.layer.nnz]

LAUNCH_SHAPES = [(128, 2), (128, 3), (128, 4), (64, 2), (64, 3), (64, 4), (64, 6), (64, 8), (0, 0)]


def _random_case(rng):
    T = int(rng.choice([1, 7, 64, 65, 130, 257, 500]))
    I, O = int(rng.integers(1, 700)), int(rng.integers(1, 700))
    d = float(rng.choice([0.0, 0.01, 0.03, 0.1, 0.3, 0.6, 1.0]))
    kind = str(rng.choice(["uniform", "powerlaw", "rows"]))
    seed = int(rng.integers(1, 10 ** 6))
    if kind == "rows":            # a few full rows, many empty rows, the rest uniform
        M = (rng.random((O, I)) < d).astype(np.uint8)
        M[rng.random(O) < 0.5] = 0
        M[rng.random(O) < 0.08] = 1
        W = (synth.normal(seed, 5, (O, I), 0.02) * M).astype(np.float32)
    else:
        W, M = synth.make_layer(seed, 1, I, O, d, kind)
    X, dY = synth.make_activations(seed, 1, T, I, O)
    shape = LAUNCH_SHAPES[int(rng.integers(0, len(LAUNCH_SHAPES)))]
    path = int(rng.choice([mst.MST_PATH_AUTO, mst.MST_PATH_SPARSE, mst.MST_PATH_SPARSE, mst.MST_PATH_DENSE]))
    d2 = float(rng.choice([d, min(1.0, d * 2 + 0.01), d / 2]))
    return T, I, O, d, kind, seed, W, M, X, dY, shape, path, d2


@pytest.mark.parametrize("stream_seed", [1, 2, 3])
def test_random_layers(stream_seed):
    rng = np.random.default_rng(stream_seed)
    for case in range(14):
        T, I, O, d, kind, seed, W, M, X, dY, shape, path, d2 = _random_case(rng)
        print("case", stream_seed, case, T, I, O, d, kind, shape, path, int(M.sum()), flush=True)
        rig = Rig(W, M, T, cap=O * I)
        rig.layer.set_path(path)
        try:
            mst.mst_spmm_force_shape(*shape)
            assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, M)) <= TOL
            assert rel_err(rig.bwd_input(dY), opr.fc_bwd_input(dY, W, M)) <= TOL
        finally:
            mst.mst_spmm_force_shape(0, 0)
        if M.sum() > 0:
            assert rel_err(rig.bwd_weight(dY, X), opr.fc_bwd_weight(dY, X, M)) <= TOL
        dX1, dW1 = _bwd_one_call(rig, dY, X, T, I, BWD_SHAPES[case % 3])
        assert rel_err(dX1, opr.fc_bwd_input(dY, W, M)) <= TOL
        if M.sum() > 0:
            assert rel_err(dW1, opr.fc_bwd_weight(dY, X, M)) <= TOL
        G = synth.normal(seed, 77, (O, I))
        mst.mst_mask_update_from_scores(rig.layer, dev(G), d2, 0.3, 0.25, seed, rig.ws)
        torch.cuda.synchronize()
        ref = omg.update(W, M, G, d2, 0.3, 0.25, seed)
        We, Me = rig.export()
        np.testing.assert_array_equal(Me, ref["M"])
        np.testing.assert_array_equal(We, ref["W"])
        assert rel_err(rig.fwd(X), opr.fc_fwd(X, ref["W"], ref["M"])) <= TOL
        assert rel_err(rig.bwd_input(dY), opr.fc_bwd_input(dY, ref["W"], ref["M"])) <= TOL
        if ref["M"].sum() > 0:
            assert rel_err(rig.bwd_weight(dY, X), opr.fc_bwd_weight(dY, X, ref["M"])) <= TOL
        dX1, dW1 = _bwd_one_call(rig, dY, X, T, I, BWD_SHAPES[(case + 1) % 3])
        assert rel_err(dX1, opr.fc_bwd_input(dY, ref["W"], ref["M"])) <= TOL
        if ref["M"].sum() > 0:
            assert rel_err(dW1, opr.fc_bwd_weight(dY, X, ref["M"])) <= TOL
