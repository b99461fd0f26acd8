"""The index views are built when a sparse kernel will walk them.

An update of a layer that the dense MFMA contractions serve (density above the cross-over at
the batch size of the last product call) rebuilds vals / flat / rowptr and writes the new
weights into the layer's dense copy in place; the views stay unbuilt.  Calls that carry a
workspace build them when the sparse kernels are due; Y and dX (no workspace) run the dense
product meanwhile.  Every state is compared with the oracle: masks and weights after
Algorithm 1 bit for bit, the products (App. Eq. (1) and its gradients) within tolerance."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth
from oracle import mixed_growing as omg
from oracle import products as opr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, TOL, DEV, dev, rel_err  # noqa: E402


def _check_products(tag, rig, W, M, X, dY, Xd, dYd, T):
    Y = rig.fwd(X)
    dX = rig.bwd_input(dY)
    nnz = rig.layer.nnz
    dX2 = torch.full((T, rig.I), float("nan"), dtype=torch.float32, device=DEV)
    dW2 = torch.full((max(nnz, 1),), float("nan"), dtype=torch.float32, device=DEV)
    mst.mst_sparse_fc_bwd(rig.layer, dYd, Xd, dX2, dW2, T, rig.ws)
    torch.cuda.synchronize()
    dW = rig.bwd_weight(dY, X)
    e = (rel_err(Y, opr.fc_fwd(X, W, M)), rel_err(dX, opr.fc_bwd_input(dY, W, M)),
         rel_err(dX2.cpu().numpy(), opr.fc_bwd_input(dY, W, M)),
         rel_err(dW2.cpu().numpy()[:nnz], opr.fc_bwd_weight(dY, X, M)), rel_err(dW, opr.fc_bwd_weight(dY, X, M)))
    print(tag, "errors fwd / dX / bwd.dX / bwd.dW / dW:", e, flush=True)
    assert max(e) <= TOL, (tag, e)


def _update(rig, W, M, Gd, Gh, d, seed):
    st = mst.mst_mask_update_from_scores(rig.layer, Gd, d, 0.3, 0.25, seed, rig.ws)
    torch.cuda.synchronize()
    ref = omg.update(W, M, Gh, d, 0.3, 0.25, seed)
    c = ref["counts"]
    assert (st["n_prune"], st["n_grad"], st["n_rand"], st["nnz_after"]) == \
        (c["n_prune"], c["n_grad"], c["n_rand"], c["nnz_target"])
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, ref["M"])
    np.testing.assert_array_equal(We, ref["W"])
    np.testing.assert_array_equal(rig.indices(), np.flatnonzero(ref["M"].reshape(-1)))
    return ref["W"], ref["M"]


def test_views_follow_the_path_across_updates():
    I, O, T = 384, 640, 2048                       # whole 128-tiles (the fast dense kernels), not whole 256-tiles; long batch
    W, M = synth.make_layer(77, 1, I, O, 0.5)
    X, dY = synth.make_activations(77, 1, T, I, O)
    Xd, dYd = dev(X), dev(dY)
    rig = Rig(W, M, T, cap=O * I)
    L = rig.layer
    Gd = torch.empty((O, I), dtype=torch.float32, device=DEV)
    mst.mst_dense_grad(dYd, Xd, Gd, T, O, I, mst.MST_F32, None)
    torch.cuda.synchronize()
    Gh = Gd.cpu().numpy()

    # loaded: views built whatever the density; the product calls tell the layer batch size and type
    assert L.format_stats()["row_view_slots"] > 0
    _check_products("loaded d=0.5", rig, W, M, X, dY, Xd, dYd, T)
    assert L.uses_dense(mst.MST_F32, T) and L.uses_dense(mst.MST_F32, T, True)

    # 0.5 -> 0.2: stays on the dense contractions, views left unbuilt, dense copy updated in place
    W, M = _update(rig, W, M, Gd, Gh, 0.2, 901)
    fs = L.format_stats()
    assert fs["row_view_slots"] == 0 and fs["col_view_slots"] == 0 and fs["nnz"] == int(M.sum())
    _check_products("d=0.2 dense, unbuilt", rig, W, M, X, dY, Xd, dYd, T)
    assert L.format_stats()["row_view_slots"] == 0                     # nothing above needed them

    # the entry point without a workspace cannot build them
    dWs = torch.zeros(L.nnz, dtype=torch.float32, device=DEV)
    with pytest.raises(mst.MstError):
        mst.mst_sparse_fc_bwd_weight_static(L, dYd, Xd, dWs, 128)

    # the caller's optimiser changes the values: hand-over, then the dense copy takes them
    vals = L.values()
    vals.mul_(1.5)
    L.sync_values()
    W = (W * np.float32(1.5)).astype(np.float32)
    _check_products("d=0.2 after a value change", rig, W, M, X, dY, Xd, dYd, T)

    # pinned to the sparse kernels: Y and dX have no workspace and stay dense until a call with one
    L.set_path(mst.MST_PATH_SPARSE)
    assert L.uses_dense(mst.MST_F32, T)
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, M)) <= TOL
    dW = rig.bwd_weight(dY, X)                                         # builds both views from mask + dense copy
    assert rel_err(dW, opr.fc_bwd_weight(dY, X, M)) <= TOL
    assert L.format_stats()["row_view_slots"] >= L.nnz and not L.uses_dense(mst.MST_F32, T)
    _check_products("d=0.2 sparse kernels", rig, W, M, X, dY, Xd, dYd, T)
    mst.mst_sparse_fc_bwd_weight_static(L, dYd, Xd, dWs, 128)          # fine now
    torch.cuda.synchronize()
    assert rel_err(dWs.cpu().numpy(), opr.fc_bwd_weight(dY[:128], X[:128], M)) <= TOL
    # an update of a pinned layer builds its views at once
    W, M = _update(rig, W, M, Gd, Gh, 0.15, 902)
    assert L.format_stats()["row_view_slots"] >= L.nnz
    _check_products("d=0.15 pinned sparse", rig, W, M, X, dY, Xd, dYd, T)
    L.set_path(mst.MST_PATH_AUTO)

    # 0.15 -> 0.3 on the automatic path: dense again; the dense copy is stale (views were rebuilt
    # without it), so the update clears it first
    W, M = _update(rig, W, M, Gd, Gh, 0.3, 903)
    assert L.format_stats()["row_view_slots"] == 0
    _check_products("d=0.3 dense again", rig, W, M, X, dY, Xd, dYd, T)

    # 0.3 -> 0.02: below the cross-over, the update builds the views itself
    W, M = _update(rig, W, M, Gd, Gh, 0.02, 904)
    assert L.format_stats()["row_view_slots"] >= L.nnz and not L.uses_dense(mst.MST_F32, T)
    _check_products("d=0.02 sparse", rig, W, M, X, dY, Xd, dYd, T)

    # and back up: 0.02 -> 0.1
    W, M = _update(rig, W, M, Gd, Gh, 0.1, 905)
    assert L.format_stats()["row_view_slots"] == 0 and L.uses_dense(mst.MST_F32, T)
    _check_products("d=0.1 dense", rig, W, M, X, dY, Xd, dYd, T)


def test_first_update_before_any_product_call_builds_the_views():
    """A layer that has seen no product call gives the update nothing to judge the path by."""
    I, O, T = 256, 384, 256
    W, M = synth.make_layer(78, 1, I, O, 0.6)
    X, dY = synth.make_activations(78, 1, T, I, O)
    rig = Rig(W, M, T, cap=O * I)
    Gh = opr.dense_grad(dY, X).astype(np.float32)
    W, M = _update(rig, W, M, dev(Gh), Gh, 0.4, 11)
    assert rig.layer.format_stats()["row_view_slots"] >= rig.layer.nnz
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, M)) <= TOL


@pytest.mark.parametrize("O,I", [(7, 5), (37, 131), (3, 3000), (2500, 3), (9, 4099), (1, 1)])
def test_canonical_arrays_after_a_dense_path_update_of_a_ragged_layer(O, I):
    """vals / flat of a layer whose views stay unbuilt are the ordered compaction of the mask taken as
    one sequence of O*I positions: shapes whose rows do not align with anything."""
    T = 64
    W, M = synth.make_layer(300 + O, 1, I, O, 0.7)
    X, dY = synth.make_activations(300 + O, 1, T, I, O)
    rig = Rig(W, M, T, cap=O * I)
    L = rig.layer
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, M)) <= TOL            # the call tells the layer its batch
    Gh = opr.dense_grad(dY, X).astype(np.float32)
    W, M = _update(rig, W, M, dev(Gh), Gh, 0.5, 17)
    nnz = int(M.sum())
    if nnz > 0.3 * O * I and O * I > 1:                                # (an update that changes nothing rebuilds nothing)
        assert L.format_stats()["row_view_slots"] == 0                 # canonical arrays only
    np.testing.assert_array_equal(L.values().cpu().numpy()[:nnz], W.reshape(-1)[np.flatnonzero(M.reshape(-1))])
    _check_products("ragged %dx%d" % (O, I), rig, W, M, X, dY, dev(X), dev(dY), T)
