"""Parity at the full size of the schedule-sweep workload: the GPT-2-large fully-connected set
(1280 -> 3840 / 1280 / 5120, 5120 -> 1280) at T = 8192 tokens, fp32, at the densities the
sweep passes through (Sec. 3.1: dense start, ultra-sparse phase, restoration).  Densities
1.0, 0.5 and 0.1 run the masked dense MFMA path, 0.02 the sparse kernels, in the launch
configuration the benchmark times (automatic path and launch shape); 0.1 runs a second time
pinned to the sparse kernels.  Outputs are compared
with the oracle at >= 10^4 sampled positions per tensor (plus the longest / shortest rows
and columns); the adjoint identities cover the complete outputs; masks after a fused
Mixed-Growing update (Algorithm 1) are compared in full, bit for bit; the update phase of the
whole block runs as the benchmark issues it (one call for the four layers, a stream each)."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth
from oracle import mixed_growing as omg
from oracle import products as opr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, TOL, DEV, check_layer_products, dev, sampled_check  # noqa: E402

T = 8192
LARGE = synth.LAYER_SETS["large"]


@pytest.mark.parametrize("name,I,O", LARGE)
def test_large_layer_products_at_every_sweep_density(name, I, O):
    lid = 30 + [n for n, _, _ in LARGE].index(name)
    X, dY = synth.make_activations(2024, lid, T, I, O)
    Xd, dYd = dev(X), dev(dY)
    for d in (1.0, 0.5, 0.1, 0.02):
        print("case", name, I, O, "density", d, flush=True)
        W, M = synth.make_layer(2024, lid, I, O, d)
        rig = Rig(W, M, T, cap=int(M.sum()))
        check_layer_products("%s d=%.2f" % (name, d), rig, W, M, X, dY, Xd, dYd, mst.MST_F32, n=10000)
        assert rig.layer.uses_dense(mst.MST_F32, T) == (d >= 0.1)
        if d == 0.1:
            rig.layer.set_path(mst.MST_PATH_SPARSE)
            check_layer_products("%s d=%.2f sparse" % (name, d), rig, W, M, X, dY, Xd, dYd, mst.MST_F32, n=3000)
        del rig
        torch.cuda.empty_cache()


@pytest.mark.parametrize("name,I,O", LARGE)
def test_large_dense_gradient_with_the_split_grid(name, I, O):
    """mst_dense_grad at the sweep's shapes (the workspace makes it split the token range)."""
    print("case", name, I, O, flush=True)
    lid = 40 + [n for n, _, _ in LARGE].index(name)
    X, dY = synth.make_activations(2024, lid, T, I, O)
    G = torch.full((O, I), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(8 * O * I * 4, dtype=torch.uint8, device=DEV)
    mst.mst_dense_grad(dev(dY), dev(X), G, T, O, I, mst.MST_F32, ws)
    torch.cuda.synchronize()
    sampled_check("G " + name, G.cpu().numpy(), lambda o, i: opr.dense_grad_at(dY, X, o, i), (O, I), n=10000, seed=4)
    # the 100-tile shapes (fc1, fc2) run five workgroups per two tiles; with that schedule switched off
    # (plain k ranges) the result is the same up to summation order
    try:
        mst.mst_gemm_force_fp32_mfma(-52)
        G3 = torch.full((O, I), float("nan"), dtype=torch.float32, device=DEV)
        mst.mst_dense_grad(dev(dY), dev(X), G3, T, O, I, mst.MST_F32, ws)
        torch.cuda.synchronize()
    finally:
        mst.mst_gemm_force_fp32_mfma(52)
    a3 = G3.cpu().numpy()
    assert np.abs(G.cpu().numpy() - a3).max() <= 1e-5 * np.abs(a3).max()
    if O * I == 5120 * 1280:
        assert not np.array_equal(G.cpu().numpy(), a3)             # the two schedules really differ
    # without a workspace (one pass over all tokens) the result is the same up to summation order
    G2 = torch.full((O, I), float("nan"), dtype=torch.float32, device=DEV)
    mst.mst_dense_grad(dev(dY), dev(X), G2, T, O, I, mst.MST_F32, None)
    torch.cuda.synchronize()
    a, b = G.cpu().numpy(), G2.cpu().numpy()
    assert np.abs(a - b).max() <= 1e-5 * np.abs(a).max()


def test_large_fc1_fused_updates_along_the_sweep_are_bit_exact():
    """The 1280 -> 5120 layer (N = 6.55 M positions) driven dense -> 0.5 -> 0.1 -> 0.02 -> 0.1 by the
    fused update itself, as the sweep does: every mask, the surviving weights and the index
    list equal the oracle's update run on the GPU's own score bits; the score is within
    tolerance of the oracle's at sampled positions."""
    I, O = 1280, 5120
    N = O * I
    X, dY = synth.make_activations(2024, 50, T, I, O)
    Xd, dYd = dev(X), dev(dY)
    W = synth.normal(2024, 50002, (O, I), 0.02)
    M = np.ones((O, I), np.uint8)
    rig = Rig(W, M, T, cap=N)
    # the score buffer of the fused update, formed by the same product with the same split
    G = torch.empty((O, I), dtype=torch.float32, device=DEV)
    gws = torch.empty(8 * N * 4, dtype=torch.uint8, device=DEV)
    mst.mst_dense_grad(dYd, Xd, G, T, O, I, mst.MST_F32, gws)
    torch.cuda.synchronize()
    Gh = G.cpu().numpy()
    sampled_check("G fc1", Gh, lambda o, i: opr.dense_grad_at(dY, X, o, i), (O, I), n=3000, seed=5)
    seed = 2 ** 40 + 17
    for step, d in enumerate((0.5, 0.1, 0.02, 0.1)):
        print("update to density", d, flush=True)
        nnz_before = rig.layer.nnz
        dWg = torch.full((nnz_before,), float("nan"), dtype=torch.float32, device=DEV)
        # the sweep's call: weight gradient and update from one dense gradient
        st = mst.mst_sparse_fc_bwd_weight_update(rig.layer, dYd, Xd, dWg, T, d, 0.3, 0.25, seed + step, rig.ws)
        torch.cuda.synchronize()
        ref = omg.update(W, M, Gh, d, 0.3, 0.25, seed + step)
        c = ref["counts"]
        assert (st["n_prune"], st["n_grad"], st["n_rand"]) == (c["n_prune"], c["n_grad"], c["n_rand"])
        assert st["nnz_after"] == c["nnz_target"] == rig.layer.nnz
        We, Me = rig.export()
        np.testing.assert_array_equal(Me, ref["M"])
        np.testing.assert_array_equal(We, ref["W"])
        np.testing.assert_array_equal(rig.indices(), np.flatnonzero(ref["M"].reshape(-1)))
        if c["n_grad"] > 0:
            # the weight gradient of the positions active before the update = the score bits there
            np.testing.assert_array_equal(dWg.cpu().numpy(), Gh.reshape(-1)[np.flatnonzero(M.reshape(-1))])
        W, M = ref["W"], ref["M"]
    # the layer still computes with the topology it ended on
    Y = rig.fwd(X)
    sampled_check("fwd after the sweep", Y, lambda t, o: opr.fc_fwd_at(X, W, M, t, o), (T, O), n=2000, seed=6)


def test_large_block_update_phase_as_the_benchmark_issues_it():
    """The update phase of a sweep step in the benchmark's launch configuration: the four layers
    of the block, per layer on a stream of its own the weight gradient read from the score
    buffer, then ONE mst_mask_update_from_scores_multi call that runs the four updates side by
    side (three side streams and the main one).  Ultra-sparse direction (0.1 -> 0.02) and back
    (0.02 -> 0.1): every layer's mask, weights and index list equal the oracle's Algorithm 1."""
    main = torch.cuda.current_stream()
    streams = [torch.cuda.Stream() for _ in LARGE[:-1]] + [main]
    rigs, Ws, Ms, Gs, Gd, seeds = [], [], [], [], [], []
    for j, (name, I, O) in enumerate(LARGE):
        W, M = synth.make_layer(4100 + j, 1, I, O, 0.10)
        Ws.append(W); Ms.append(M)
        Gs.append(synth.normal(4100 + j, 77, (O, I), 1.0))
        Gd.append(dev(Gs[-1]))
        rigs.append(Rig(W, M, T, cap=O * I))
        seeds.append(2 ** 50 + 101 * j)
    torch.cuda.synchronize()
    for rnd, d in enumerate((0.02, 0.10)):
        print("block update to density", d, flush=True)
        dWs = []
        for j, rig in enumerate(rigs):
            dW = torch.full((rig.layer.nnz,), float("nan"), dtype=torch.float32, device=DEV)
            streams[j].wait_stream(main)
            mst.mst_gather_active(rig.layer, Gd[j], dW, streams[j])
            dWs.append(dW)
        sts = mst.mst_mask_update_from_scores_multi([r.layer for r in rigs], Gd, [d] * len(rigs), 0.3, 0.25,
                                                    [s + rnd for s in seeds], [r.ws for r in rigs], streams)
        torch.cuda.synchronize()
        for j, rig in enumerate(rigs):
            np.testing.assert_array_equal(dWs[j].cpu().numpy(), Gs[j].reshape(-1)[np.flatnonzero(Ms[j].reshape(-1))])
            ref = omg.update(Ws[j], Ms[j], Gs[j], d, 0.3, 0.25, seeds[j] + rnd)
            c = ref["counts"]
            assert (sts[j]["n_prune"], sts[j]["n_grad"], sts[j]["n_rand"], sts[j]["nnz_after"]) == \
                (c["n_prune"], c["n_grad"], c["n_rand"], c["nnz_target"])
            We, Me = rig.export()
            np.testing.assert_array_equal(Me, ref["M"], err_msg=LARGE[j][0])
            np.testing.assert_array_equal(We, ref["W"], err_msg=LARGE[j][0])
            np.testing.assert_array_equal(rig.indices(), np.flatnonzero(ref["M"].reshape(-1)))
            Ws[j], Ms[j] = ref["W"], ref["M"]
    # the layers compute with the topology they ended on (dense path at 0.1)
    j = 1
    X, _ = synth.make_activations(4100, 9, T, LARGE[j][1], LARGE[j][2])
    Y = rigs[j].fwd(X)
    sampled_check("fwd after the block updates", Y, lambda t, o: opr.fc_fwd_at(X, Ws[j], Ms[j], t, o),
                  (T, LARGE[j][2]), n=2000, seed=8)
