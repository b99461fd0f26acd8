"""Parity at full size of the two remaining benchmark workloads.

* GPT-2-small block at the ultra-sparse density 0.02 with power-law row lengths (exponent
  1.5: a few completely full rows, most rows nearly empty), T = 16384, fp32: all four
  layers, every product call incl. the one-call backward and the weight gradient.
* GPT-2-medium block at density 0.05 with bfloat16 activations and fp32 accumulation,
  T = 16384: the layers the other full-size file does not cover, on the automatic path
  (dense bf16 MFMA contractions at this density) and pinned to the sparse kernels, and a
  fused Mixed-Growing update (Algorithm 1) whose dense gradient runs on the bf16 matrix cores.

Sampled outputs (>= 10^4 per tensor plus the longest / shortest rows and columns) against
the oracle, adjoint identities over the complete outputs, masks in full."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth
from oracle import mixed_growing as omg
from oracle import products as opr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, TOL, DEV, check_layer_products, dev, sampled_check  # noqa: E402

T = 16384


@pytest.mark.parametrize("name,I,O", synth.LAYER_SETS["small"])
def test_powerlaw_block_layer_every_product(name, I, O):
    print("case", name, I, O, flush=True)
    lid = 60 + [n for n, _, _ in synth.LAYER_SETS["small"]].index(name)
    W, M = synth.make_layer(2024, lid, I, O, 0.02, "powerlaw")
    lens = M.sum(axis=1)
    assert lens.max() == I and np.median(lens) <= 4          # full rows next to nearly empty ones
    X, dY = synth.make_activations(2024, lid, T, I, O)
    rig = Rig(W, M, T, cap=int(M.sum()) * 3 // 2)
    Y, dX, dW = check_layer_products("powerlaw " + name, rig, W, M, X, dY, dev(X), dev(dY), mst.MST_F32, n=10000)
    empty = np.flatnonzero(lens == 0)
    if empty.size:
        assert not Y[:, empty].any()                          # empty rows give exact zeros


@pytest.mark.parametrize("name,I,O", [l for l in synth.LAYER_SETS["medium"] if l[0] != "fc1"])
def test_medium_bf16_layer_every_product(name, I, O):
    print("case", name, I, O, flush=True)
    lid = 70 + [n for n, _, _ in synth.LAYER_SETS["medium"]].index(name)
    W, M = synth.make_layer(2024, lid, I, O, 0.05)
    Xf, dYf, xb, yb = synth.make_activations(2024, lid, T, I, O, "bf16")
    Xd, dYd = dev(xb.view(np.int16)), dev(yb.view(np.int16))
    rig = Rig(W, M, T, cap=int(M.sum()) * 3 // 2)
    # automatic choice at this density: Y and dX as two-product bf16 MFMA contractions (bfloat16
    # activations x fp32 weights split hi + lo), weight gradient as the bf16 MFMA product read
    # at the active positions
    _, dX_auto, dW_auto = check_layer_products("bf16 auto " + name, rig, W, M, Xf, dYf, Xd, dYd, mst.MST_BF16,
                                               n=10000)
    # pinned to the sparse kernels: both gradients from one walk of the transposed view
    rig.layer.set_path(mst.MST_PATH_SPARSE)
    _, dX_sp, dW_sp = check_layer_products("bf16 sparse " + name, rig, W, M, Xf, dYf, Xd, dYd, mst.MST_BF16,
                                           n=3000)
    assert rig.layer.nnz > 0 and not rig.layer.uses_dense(mst.MST_BF16, T)
    rig.layer.set_path(mst.MST_PATH_AUTO)
    assert rig.layer.uses_dense(mst.MST_BF16, T) and rig.layer.uses_dense(mst.MST_BF16, T, True)
    assert np.abs(dX_sp - dX_auto).max() <= 2e-5 * np.abs(dX_auto).max()   # split weights: 2^-17 per term
    assert np.abs(dW_sp - dW_auto).max() <= 1e-5 * np.abs(dW_auto).max()


def test_medium_bf16_fc1_fused_update_full_size():
    I, O, d = 1024, 4096, 0.05
    W, M = synth.make_layer(2024, 80, I, O, d)
    Xf, dYf, xb, yb = synth.make_activations(2024, 80, T, I, O, "bf16")
    Xd, dYd = dev(xb.view(np.int16)), dev(yb.view(np.int16))
    rig = Rig(W, M, T, cap=int(M.sum()) * 3 // 2)
    G = torch.full((O, I), float("nan"), dtype=torch.float32, device=DEV)
    gws = torch.empty(8 * O * I * 4, dtype=torch.uint8, device=DEV)
    mst.mst_dense_grad(dYd, Xd, G, T, O, I, mst.MST_BF16, gws)
    torch.cuda.synchronize()
    Gh = G.cpu().numpy()
    # step 1: the score (bf16 MFMA, fp32 accumulation) against the oracle on the same bf16 values
    sampled_check("G bf16", Gh, lambda o, i: opr.dense_grad_at(dYf, Xf, o, i), (O, I), n=10000, seed=7)
    # step 2: the fused update's mask equals the oracle's update on the GPU's own score bits
    st = mst.mst_mask_update(rig.layer, dYd, Xd, T, d, 0.3, 0.25, 4242, rig.ws, mst.MST_BF16)
    torch.cuda.synchronize()
    ref = omg.update(W, M, Gh, d, 0.3, 0.25, 4242)
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, ref["M"])
    np.testing.assert_array_equal(We, ref["W"])
    c = ref["counts"]
    assert (st["n_prune"], st["n_grad"], st["n_rand"]) == (c["n_prune"], c["n_grad"], c["n_rand"])
    assert st["nnz_after"] == int(M.sum()) == rig.layer.nnz
    # step 3: against the mask from the oracle's own (fp64) score only near-threshold positions differ
    Go = opr.dense_grad(dYf, Xf).astype(np.float32)
    ref_o = omg.update(W, M, Go, d, 0.3, 0.25, 4242)
    differ = int((ref_o["M"] != ref["M"]).sum())
    print("positions that differ from the oracle-score mask:", differ, "of", c["n_grad"], "grown by gradient", flush=True)
    assert differ <= max(8, c["n_grow"] // 100)
    # the updated layer computes with its new topology
    Y = torch.full((T, O), float("nan"), dtype=torch.float32, device=DEV)
    mst.mst_sparse_fc_fwd(rig.layer, Xd, Y, T, mst.MST_BF16)
    torch.cuda.synchronize()
    sampled_check("fwd after update", Y.cpu().numpy(), lambda t, o: opr.fc_fwd_at(Xf, ref["W"], ref["M"], t, o),
                  (T, O), n=2000, seed=8)
