"""GPU parity of the Mixed-Growing update (Algorithm 1) against the CPU oracle.

Masks, index sets and weights must be bit-exact for a given score buffer; the fused
entry point (score computed on the matrix cores) is checked in three steps: its score
is within tolerance of the oracle's, the mask it produces equals the oracle's mask on
the GPU's own score bits, and the number of positions that differ from the oracle-score
mask is reported (near-threshold near-ties only)."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth
from oracle import mixed_growing as omg
from oracle import products as opr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, TOL, dev, rel_err, DEV  # noqa: E402


def _scores(seed, O, I, quantise=None):
    G = synth.normal(seed, 77, (O, I))
    if quantise:
        G = (np.round(G * quantise) / quantise).astype(np.float32)
    return G


def _update_and_compare(W, M, G, d_t, zeta, R, seed, cap=None):
    O, I = W.shape
    rig = Rig(W, M, 1, cap=cap if cap is not None else O * I)
    st = mst.mst_mask_update_from_scores(rig.layer, dev(G), d_t, zeta, R, seed, rig.ws)
    torch.cuda.synchronize()
    ref = omg.update(W, M, G, d_t, zeta, R, seed)
    c = ref["counts"]
    assert st["n_prune"] == c["n_prune"] and st["n_grad"] == c["n_grad"] and st["n_rand"] == c["n_rand"]
    assert st["nnz_after"] == c["nnz_target"] == rig.layer.nnz
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, ref["M"])              # bit-exact mask
    np.testing.assert_array_equal(We, ref["W"])              # kept values untouched, grown / pruned = 0
    np.testing.assert_array_equal(rig.indices(), np.flatnonzero(ref["M"].reshape(-1)))
    return rig, ref


@pytest.mark.parametrize("O,I,density", [(333, 200, 0.1), (768, 768, 0.05), (130, 4100, 0.02)])
@pytest.mark.parametrize("quantise", [None, 4])
def test_update_from_scores_is_bit_exact(O, I, density, quantise):
    print("case", O, I, density, quantise, flush=True)
    W, M = synth.make_layer(21, 1, I, O, density)
    if quantise:                                   # many equal magnitudes, zeros and equal scores
        W = (np.round(W * 50 * quantise) / (50 * quantise)).astype(np.float32) * M
    G = _scores(21, O, I, quantise)
    _update_and_compare(W, M, G, density, 0.3, 0.25, seed=12345)


@pytest.mark.parametrize("d_t,zeta,R", [(0.05, 0.3, 0.0), (0.05, 0.3, 1.0), (0.02, 0.3, 0.25), (0.2, 0.3, 0.25),
                                        (0.05, 1.0, 0.5), (1.0, 0.3, 0.25), (0.0, 0.3, 0.25), (0.05, 0.0, 0.25)])
def test_update_special_cases(d_t, zeta, R):
    print("case", d_t, zeta, R, flush=True)
    O, I = 256, 384
    W, M = synth.make_layer(22, 2, I, O, 0.05)
    G = _scores(22, O, I)
    _update_and_compare(W, M, G, d_t, zeta, R, seed=2 ** 63 + 11)


def test_warmup_jump_from_dense_and_restoration_to_dense():
    O, I = 192, 320
    W = synth.normal(23, 5, (O, I), 0.02)
    ones = np.ones((O, I), np.uint8)
    G = _scores(23, O, I)
    rig, ref = _update_and_compare(W, ones, G, 0.53152, 0.3, 0.25, seed=5)      # pure prune
    assert ref["counts"]["n_grow"] == 0
    # chain a second and third update on the same layer object: down to 4 %, then back to dense
    W1, M1 = ref["W"], ref["M"]
    st = mst.mst_mask_update_from_scores(rig.layer, dev(G), 0.04, 0.3, 0.25, 6, rig.ws)
    ref2 = omg.update(W1, M1, G, 0.04, 0.3, 0.25, 6)
    torch.cuda.synchronize()
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, ref2["M"]); np.testing.assert_array_equal(We, ref2["W"])
    st = mst.mst_mask_update_from_scores(rig.layer, dev(G), 1.0, 0.3, 0.25, 7, rig.ws)
    ref3 = omg.update(ref2["W"], ref2["M"], G, 1.0, 0.3, 0.25, 7)
    torch.cuda.synchronize()
    We, Me = rig.export()
    assert st["n_prune"] == 0 and Me.all()
    np.testing.assert_array_equal(Me, ref3["M"]); np.testing.assert_array_equal(We, ref3["W"])


def test_products_after_update_use_the_new_topology():
    T, I, O = 260, 384, 256
    W, M = synth.make_layer(24, 3, I, O, 0.08)
    X, dY = synth.make_activations(24, 3, T, I, O)
    G = opr.dense_grad(dY, X).astype(np.float32)
    rig = Rig(W, M, T, cap=O * I)
    mst.mst_mask_update_from_scores(rig.layer, dev(G), 0.08, 0.3, 0.25, 99, rig.ws)
    ref = omg.update(W, M, G, 0.08, 0.3, 0.25, 99)
    # give the grown weights a value, as an optimiser step would, then resync
    vals = rig.layer.values()
    vals.add_(0.003)
    rig.layer.sync_values()
    W2 = ref["W"].copy()
    W2[ref["M"] != 0] += np.float32(0.003)
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W2, ref["M"])) <= TOL
    assert rel_err(rig.bwd_input(dY), opr.fc_bwd_input(dY, W2, ref["M"])) <= TOL
    assert rel_err(rig.bwd_weight(dY, X), opr.fc_bwd_weight(dY, X, ref["M"])) <= TOL


def test_powerlaw_layer_update():
    O, I = 768, 768
    W, M = synth.make_layer(25, 4, I, O, 0.02, "powerlaw")
    G = _scores(25, O, I)
    _update_and_compare(W, M, G, 0.02, 0.3, 0.25, seed=31337)


def test_capacity_is_enforced_before_anything_runs():
    O, I = 64, 64
    W, M = synth.make_layer(26, 5, I, O, 0.1)
    rig = Rig(W, M, 1, cap=int(M.sum()) + 5)
    with pytest.raises(mst.MstError) as e:
        mst.mst_mask_update_from_scores(rig.layer, dev(_scores(26, O, I)), 0.5, 0.3, 0.25, 1, rig.ws)
    assert e.value.code == -4
    _, Me = rig.export()
    np.testing.assert_array_equal(Me, M)          # untouched


@pytest.mark.parametrize("act", ["f32", "bf16"])
def test_fused_update_three_step_check(act):
    T, I, O = 1024, 768, 768
    W, M = synth.make_layer(27, 6, I, O, 0.05)
    if act == "f32":
        X, dY = synth.make_activations(27, 6, T, I, O)
        Xd, dYd, code = dev(X), dev(dY), mst.MST_F32
    else:
        X, dY, xb, yb = synth.make_activations(27, 6, T, I, O, "bf16")
        Xd, dYd, code = dev(xb.view(np.int16)), dev(yb.view(np.int16)), mst.MST_BF16
    rig = Rig(W, M, T, cap=O * I // 4)
    # step 1: the score the update will use is within tolerance of the oracle's
    Gg = torch.empty((O, I), dtype=torch.float32, device=DEV)
    mst.mst_dense_grad(dYd, Xd, Gg, T, O, I, code, rig.ws)
    torch.cuda.synchronize()
    G_gpu = Gg.cpu().numpy()
    G_ref = opr.dense_grad(dY, X)
    assert rel_err(G_gpu, G_ref) <= TOL
    # step 2: fused update == oracle update on the GPU's own score bits
    st = mst.mst_mask_update(rig.layer, dYd, Xd, T, 0.05, 0.3, 0.25, 4242, rig.ws, code)
    torch.cuda.synchronize()
    ref = omg.update(W, M, G_gpu, 0.05, 0.3, 0.25, 4242)
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, ref["M"])
    np.testing.assert_array_equal(We, ref["W"])
    # step 3: against the oracle's own score only near-ties at the threshold may differ
    ref64 = omg.update(W, M, G_ref.astype(np.float32), 0.05, 0.3, 0.25, 4242)
    differ = int((Me != ref64["M"]).sum())
    print("positions differing from the oracle-score mask:", differ, "of", st["n_grow"], "grown")
    assert differ <= max(4, st["n_grow"] // 100)


def test_schedule_sweep_chain_matches_oracle_and_switches_paths():
    """Densities 1.0 -> 0.5 -> 0.1 -> 0.02 -> 0.1 -> 0.5, every transition produced by the
    update itself (the large-model sweep at reduced width): masks stay bit-exact against the
    oracle chain and the products stay within tolerance on the dense (MFMA) and sparse paths."""
    T, I, O = 384, 320, 512
    W = synth.normal(31, 1, (O, I), 0.02)
    M = np.ones((O, I), np.uint8)
    X, dY = synth.make_activations(31, 1, T, I, O)
    G = opr.dense_grad(dY, X).astype(np.float32)
    rig = Rig(W, M, T, cap=O * I)
    Gd = dev(G)
    Wc, Mc = W.copy(), M.copy()
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, Wc, Mc)) <= TOL            # dense start: MFMA path
    for step, d in enumerate([0.5, 0.1, 0.02, 0.1, 0.5]):
        st = mst.mst_mask_update_from_scores(rig.layer, Gd, d, 0.3, 0.25, 1000 + step, rig.ws)
        ref = omg.update(Wc, Mc, G, d, 0.3, 0.25, 1000 + step)
        torch.cuda.synchronize()
        We, Me = rig.export()
        np.testing.assert_array_equal(Me, ref["M"])
        np.testing.assert_array_equal(We, ref["W"])
        assert st["nnz_after"] == omg.target_count(O * I, d)
        Wc, Mc = ref["W"], ref["M"]
        # train the surviving and grown weights a little so later prunes see non-zero values
        vals = rig.layer.values()
        vals.add_(0.001 * (step + 1))
        rig.layer.sync_values()
        Wc = Wc.copy()
        Wc[Mc != 0] += np.float32(0.001 * (step + 1))
        assert rel_err(rig.fwd(X), opr.fc_fwd(X, Wc, Mc)) <= TOL
        assert rel_err(rig.bwd_input(dY), opr.fc_bwd_input(dY, Wc, Mc)) <= TOL
        assert rel_err(rig.bwd_weight(dY, X), opr.fc_bwd_weight(dY, X, Mc)) <= TOL


@pytest.mark.parametrize("lam", [0.5, 0.037, 4.0])
@pytest.mark.parametrize("quantise", [None, 4])
def test_prune_score_with_gradient_term_is_bit_exact(lam, quantise):
    # the other prune criterion of the scheme table: smallest |w| + lambda |grad|
    print("case", lam, quantise, flush=True)
    O, I, density = 300, 520, 0.08
    W, M = synth.make_layer(26, 3, I, O, density)
    if quantise:
        W = (np.round(W * 50 * quantise) / (50 * quantise)).astype(np.float32) * M
    G = _scores(26, O, I, quantise)
    rig = Rig(W, M, 1, cap=O * I)
    rig.layer.set_prune_lambda(lam)
    st = mst.mst_mask_update_from_scores(rig.layer, dev(G), density, 0.3, 0.25, 99, rig.ws)
    torch.cuda.synchronize()
    ref = omg.update(W, M, G, density, 0.3, 0.25, 99, prune_lambda=float(np.float32(lam)))
    plain = omg.update(W, M, G, density, 0.3, 0.25, 99)
    assert ref["prune"].tolist() != plain["prune"].tolist()          # the criterion changes the prune set here
    assert st["n_prune"] == ref["counts"]["n_prune"]
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, ref["M"])
    np.testing.assert_array_equal(We, ref["W"])
    # back to the magnitude criterion on the same layer object
    rig.layer.set_prune_lambda(0.0)
    mst.mst_mask_update_from_scores(rig.layer, dev(G), density, 0.3, 0.25, 100, rig.ws)
    torch.cuda.synchronize()
    ref2 = omg.update(ref["W"], ref["M"], G, density, 0.3, 0.25, 100)
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, ref2["M"])
    np.testing.assert_array_equal(We, ref2["W"])


def test_prune_lambda_rejects_bad_values():
    W, M = synth.make_layer(27, 1, 64, 48, 0.1)
    rig = Rig(W, M, 1)
    for bad in (-1.0, float("nan"), float("inf")):
        with pytest.raises(mst.MstError):
            rig.layer.set_prune_lambda(bad)


@pytest.mark.parametrize("act", ["f32", "bf16"])
@pytest.mark.parametrize("d_now,d_next,zeta,R", [(0.05, 0.05, 0.3, 0.25), (0.5, 0.3, 0.3, 0.25), (0.1, 0.1, 0.3, 1.0),
                                                  (0.05, 0.05, 0.0, 0.25)])
def test_weight_gradient_and_update_from_one_dense_gradient(act, d_now, d_next, zeta, R):
    print("case", act, d_now, d_next, zeta, R, flush=True)
    T, I, O = 512, 640, 384
    W, M = synth.make_layer(28, 7, I, O, d_now)
    if act == "f32":
        X, dY = synth.make_activations(28, 7, T, I, O)
        Xd, dYd, code = dev(X), dev(dY), mst.MST_F32
    else:
        X, dY, xb, yb = synth.make_activations(28, 7, T, I, O, "bf16")
        Xd, dYd, code = dev(xb.view(np.int16)), dev(yb.view(np.int16)), mst.MST_BF16
    rig = Rig(W, M, T, cap=O * I)
    Gg = torch.empty((O, I), dtype=torch.float32, device=DEV)
    mst.mst_dense_grad(dYd, Xd, Gg, T, O, I, code, rig.ws)
    torch.cuda.synchronize()
    G_gpu = Gg.cpu().numpy()
    nnz0 = rig.layer.nnz
    dW = torch.full((nnz0,), float("nan"), dtype=torch.float32, device=DEV)
    st = mst.mst_sparse_fc_bwd_weight_update(rig.layer, dYd, Xd, dW, T, d_next, zeta, R, 777, rig.ws, code)
    torch.cuda.synchronize()
    # the weight gradient at the positions active before the update
    assert rel_err(dW.cpu().numpy(), opr.fc_bwd_weight(dY, X, M)) <= TOL
    # the update, on the GPU's own score bits
    ref = omg.update(W, M, G_gpu, d_next, zeta, R, 777)
    assert st["n_prune"] == ref["counts"]["n_prune"] and st["n_grad"] == ref["counts"]["n_grad"]
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, ref["M"])
    np.testing.assert_array_equal(We, ref["W"])
    np.testing.assert_array_equal(rig.indices(), np.flatnonzero(ref["M"].reshape(-1)))


def test_gradient_term_of_the_prune_score_with_random_growth_only():
    # R = 1 (nothing grows by gradient) with lambda > 0: the fused update still has to form the gradient
    T, I, O = 256, 320, 192
    W, M = synth.make_layer(29, 8, I, O, 0.1)
    X, dY = synth.make_activations(29, 8, T, I, O)
    rig = Rig(W, M, T, cap=O * I)
    rig.layer.set_prune_lambda(0.01)
    Gg = torch.empty((O, I), dtype=torch.float32, device=DEV)
    mst.mst_dense_grad(dev(dY), dev(X), Gg, T, O, I, mst.MST_F32, rig.ws)
    torch.cuda.synchronize()
    G_gpu = Gg.cpu().numpy()
    Gg.zero_()                                          # nothing stale may be picked up
    mst.mst_mask_update(rig.layer, dev(dY), dev(X), T, 0.1, 0.3, 1.0, 5, rig.ws)
    torch.cuda.synchronize()
    ref = omg.update(W, M, G_gpu, 0.1, 0.3, 1.0, 5, prune_lambda=float(np.float32(0.01)))
    assert ref["counts"]["n_grad"] == 0
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, ref["M"])
    np.testing.assert_array_equal(We, ref["W"])


def test_several_layers_in_one_call_on_their_own_streams():
    """mst_mask_update_from_scores_multi: the layers' update chains run side by side on different streams;
    every layer ends as the single-layer call (and the oracle's Algorithm 1) leaves it, bit for bit."""
    shapes = [(333, 200, 0.10, 0.05), (768, 512, 0.05, 0.12), (130, 4100, 0.30, 0.02), (64, 64, 0.5, 0.5)]
    rigs, Ws, Ms, Gs, Gd, seeds = [], [], [], [], [], []
    for j, (O, I, d0, _) in enumerate(shapes):
        W, M = synth.make_layer(600 + j, 1, I, O, d0)
        Ws.append(W); Ms.append(M)
        Gs.append(_scores(600 + j, O, I, 4 if j == 1 else None))
        Gd.append(dev(Gs[-1]))
        rigs.append(Rig(W, M, 1, cap=O * I))
        seeds.append(2 ** 63 + 17 * j)
    streams = [torch.cuda.Stream() for _ in shapes[:-1]] + [torch.cuda.current_stream()]
    targets = [s[3] for s in shapes]
    for rnd in range(2):                                     # twice: the second call starts from the first one's topology
        sts = mst.mst_mask_update_from_scores_multi([r.layer for r in rigs], Gd, targets, 0.3, 0.25, seeds,
                                                    [r.ws for r in rigs], streams)
        torch.cuda.synchronize()
        for j, rig in enumerate(rigs):
            ref = omg.update(Ws[j], Ms[j], Gs[j], targets[j], 0.3, 0.25, seeds[j])
            c = ref["counts"]
            assert (sts[j]["n_prune"], sts[j]["n_grad"], sts[j]["n_rand"], sts[j]["nnz_after"]) == \
                (c["n_prune"], c["n_grad"], c["n_rand"], c["nnz_target"])
            We, Me = rig.export()
            np.testing.assert_array_equal(Me, ref["M"])
            np.testing.assert_array_equal(We, ref["W"])
            np.testing.assert_array_equal(rig.indices(), np.flatnonzero(ref["M"].reshape(-1)))
            Ws[j], Ms[j] = ref["W"], ref["M"]
        targets = [0.08, 0.05, 0.02, 0.9]
    # nothing runs when any layer's arguments are refused: a layer twice, a density out of range
    before = [r.export() for r in rigs]
    with pytest.raises(mst.MstError):
        mst.mst_mask_update_from_scores_multi([rigs[0].layer, rigs[0].layer], Gd[:2], [0.1, 0.1], 0.3, 0.25, seeds[:2],
                                              [rigs[0].ws, rigs[1].ws], streams[:2])
    with pytest.raises(mst.MstError):
        mst.mst_mask_update_from_scores_multi([r.layer for r in rigs], Gd, [0.1, 0.1, 1.5, 0.1], 0.3, 0.25, seeds,
                                              [r.ws for r in rigs], streams)
    torch.cuda.synchronize()
    for r, (W0, M0) in zip(rigs, before):
        We, Me = r.export()
        np.testing.assert_array_equal(Me, M0)
        np.testing.assert_array_equal(We, W0)
