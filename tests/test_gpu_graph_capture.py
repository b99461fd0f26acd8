"""The product calls under HIP graph capture.

mst_sparse_fc_fwd and mst_sparse_fc_bwd only launch kernels on the caller's stream (clears are
fill kernels, nothing is allocated, nothing is read back), so a training loop may record them
into a graph.  Each graph is replayed several times with eager work and synchronisations in
between, on inputs that change between replays, and every replay is compared with the eager
result bit for bit and with the oracle within tolerance."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth
from oracle import products as opr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, TOL, DEV, dev, rel_err  # noqa: E402


@pytest.mark.parametrize("density,path,mask", [(0.03, mst.MST_PATH_AUTO, "uniform"), (0.5, mst.MST_PATH_AUTO, "uniform"),
                                               (0.2, mst.MST_PATH_SPARSE, "uniform"),
                                               (0.05, mst.MST_PATH_SPARSE, "powerlaw")])
def test_forward_and_backward_replay_from_a_graph(density, path, mask):
    I, O, T = 384, 640, 2048
    W, M = synth.make_layer(91, 1, I, O, density, mask)
    if mask == "powerlaw":                          # the forward is then two launches: sparse kernel + heavy rows' dense pass
        mst.mst_heavy_rows(2)
    try:
        rig = Rig(W, M, T, cap=int(M.sum()) * 2)
    finally:
        mst.mst_heavy_rows(1)
    L = rig.layer
    L.set_path(path)
    assert (L.format_stats()["heavy_rows"] > 0) == (mask == "powerlaw")
    nnz = L.nnz
    X = torch.empty((T, I), dtype=torch.float32, device=DEV)
    dY = torch.empty((T, O), dtype=torch.float32, device=DEV)
    Y = torch.zeros((T, O), dtype=torch.float32, device=DEV)
    dX = torch.zeros((T, I), dtype=torch.float32, device=DEV)
    dW = torch.zeros((nnz,), dtype=torch.float32, device=DEV)

    def calls(stream):
        mst.mst_sparse_fc_fwd(L, X, Y, T, mst.MST_F32, stream)
        mst.mst_sparse_fc_bwd(L, dY, X, dX, dW, T, rig.ws, mst.MST_F32, stream)

    def fill(seed):
        Xh, dYh = synth.make_activations(91, seed, T, I, O)
        X.copy_(dev(Xh))
        dY.copy_(dev(dYh))
        return Xh, dYh

    # eager first: builds whatever the calls cache (dense weight copy, views) outside the capture
    fill(10)
    calls(torch.cuda.current_stream())
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        calls(torch.cuda.current_stream())
    torch.cuda.synchronize()

    for rep in range(3):
        Xh, dYh = fill(20 + rep)
        graph.replay()
        torch.cuda.synchronize()
        got = (Y.cpu().numpy().copy(), dX.cpu().numpy().copy(), dW.cpu().numpy().copy())
        # the program's own eager work between replays: the same calls, outputs poisoned first
        for t_ in (Y, dX, dW):
            t_.fill_(float("nan"))
        calls(torch.cuda.current_stream())
        torch.cuda.synchronize()
        eager = (Y.cpu().numpy(), dX.cpu().numpy(), dW.cpu().numpy())
        for name, g, e in zip(("Y", "dX", "dW"), got, eager):
            np.testing.assert_array_equal(g, e, err_msg="%s, replay %d" % (name, rep))
        refs = (opr.fc_fwd(Xh, W, M), opr.fc_bwd_input(dYh, W, M), opr.fc_bwd_weight(dYh, Xh, M))
        errs = [rel_err(g, r) for g, r in zip(got, refs)]
        print("density", density, "replay", rep, "errors", errs, flush=True)
        assert max(errs) <= TOL

    # the caller's optimiser changes the values and hands them over OUTSIDE the graph: the hand-over
    # itself refreshes whatever the recorded products read (index views, dense weight copy)
    graph.replay()
    torch.cuda.synchronize()
    Y1 = Y.cpu().numpy().copy()
    L.values().mul_(2.0)
    L.sync_values()
    graph.replay()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(Y.cpu().numpy(), 2.0 * Y1)          # doubling is exact in fp32
