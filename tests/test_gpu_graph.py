"""The product calls allocate nothing and enqueue only kernels, so a caller may record them
into a HIP graph.  Replays are interleaved with eager work and compared with the eager result."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, dev, DEV  # noqa: E402


def test_products_replay_from_a_hip_graph():
    T, I, O = 512, 768, 3072
    W, M = synth.make_layer(41, 1, I, O, 0.05)
    X, dY = synth.make_activations(41, 1, T, I, O)
    rig = Rig(W, M, T)
    Xd, dYd = dev(X), dev(dY)
    Y = torch.empty((T, O), dtype=torch.float32, device=DEV)
    dX = torch.empty((T, I), dtype=torch.float32, device=DEV)
    dW = torch.empty(rig.layer.nnz, dtype=torch.float32, device=DEV)
    dX2, dW2 = torch.empty_like(dX), torch.empty_like(dW)

    def step():
        mst.mst_sparse_fc_fwd(rig.layer, Xd, Y, T)
        mst.mst_sparse_fc_bwd_input(rig.layer, dYd, dX, T)
        mst.mst_sparse_fc_bwd_weight(rig.layer, dYd, Xd, dW, T, rig.ws)
        mst.mst_sparse_fc_bwd(rig.layer, dYd, Xd, dX2, dW2, T, rig.ws)      # both gradients in one call
        rig.layer.sync_values()

    step()
    torch.cuda.synchronize()
    ref = (Y.clone(), dX.clone(), dW.clone(), dX2.clone(), dW2.clone())

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    with torch.cuda.graph(g, stream=side):
        step()
    for rep in range(3):
        for buf in (Y, dX, dW, dX2, dW2):
            buf.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip((Y, dX, dW, dX2, dW2), ref):
            assert torch.equal(got, want), rep     # bit-identical to the eager run
        # eager work between the replays
        Xd.mul_(1.0)
        step()
        torch.cuda.synchronize()
