"""GPU parity of the three products and the dense gradient against the CPU oracle.

Bar: max|gpu - oracle| / max|oracle| <= 1e-4 per output tensor (fp32 values)."""
import numpy as np
import pytest

import paper_2408_11746_amd as mst
import synth
from oracle import products as opr

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import Rig, TOL, dev, rel_err, DEV  # noqa: E402


def _case(seed, T, I, O, density, mask="uniform"):
    W, M = synth.make_layer(seed, 1, I, O, density, mask)
    X, dY = synth.make_activations(seed, 1, T, I, O)
    return W, M, X, dY


# (T, I, O, density): several token tiles, several chunks, ragged tails in every dimension
SHAPES = [
    (300, 200, 333, 0.10),      # nothing a multiple of 4 / 64 / 128
    (129, 768, 768, 0.05),      # one token past a tile
    (512, 768, 3072, 0.05),     # the 768 -> 3072 layer at 512 tokens
    (640, 3072, 768, 0.02),     # long contraction (24 chunks)
    (64, 130, 70, 0.5),
    (1, 5, 3, 0.6),             # single token, tiny
    (2100, 200, 3850, 0.05),    # ragged everywhere and large enough for whole-block wavefronts
]


@pytest.mark.parametrize("T,I,O,density", SHAPES)
def test_products_match_oracle(T, I, O, density):
    print("case", T, I, O, density, flush=True)
    W, M, X, dY = _case(11, T, I, O, density)
    rig = Rig(W, M, T)
    assert rig.layer.nnz == int(M.sum())
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, M)) <= TOL
    assert rel_err(rig.bwd_input(dY), opr.fc_bwd_input(dY, W, M)) <= TOL
    assert rel_err(rig.bwd_weight(dY, X), opr.fc_bwd_weight(dY, X, M)) <= TOL


SPMM_SHAPES = [(128, 2), (128, 3), (128, 4), (64, 2), (64, 3), (64, 4), (64, 6), (64, 8)]


@pytest.mark.parametrize("tokens,quads", SPMM_SHAPES)
def test_every_spmm_launch_shape_matches_oracle_and_each_other(tokens, quads):
    """Each launch shape of the SpMM kernel, pinned, on inputs ragged in every dimension
    (tokens past a tile, rows past a slab of every width, a partial last chunk); all
    shapes add a row's entries in the same order, so they agree bit for bit."""
    T, I, O, density = 333, 410, 1100, 0.08
    print("case", tokens, quads, T, I, O, density, flush=True)
    W, M, X, dY = _case(21, T, I, O, density)
    rig = Rig(W, M, T)
    try:
        mst.mst_spmm_force_shape(128, 4)
        y_ref, dx_ref = rig.fwd(X), rig.bwd_input(dY)
        mst.mst_spmm_force_shape(tokens, quads)
        y, dx = rig.fwd(X), rig.bwd_input(dY)
    finally:
        mst.mst_spmm_force_shape(0, 0)
    assert rel_err(y, opr.fc_fwd(X, W, M)) <= TOL
    assert rel_err(dx, opr.fc_bwd_input(dY, W, M)) <= TOL
    np.testing.assert_array_equal(y, y_ref)
    np.testing.assert_array_equal(dx, dx_ref)


def test_spmm_force_shape_rejects_unknown_shapes():
    for tokens, quads in [(128, 6), (64, 5), (32, 4), (0, 4), (64, 0)]:
        with pytest.raises(mst.MstError):
            mst.mst_spmm_force_shape(tokens, quads)
    mst.mst_spmm_force_shape(0, 0)


def test_long_rows_spread_over_a_quad():
    """Blocks of 16 rows built by hand so that the format spreads 1, 4, 1 (too few empty
    rows for the second long row) and 0 long rows over whole quads, next to ordinary
    blocks; all products and the layer round trip against the oracle."""
    rng = np.random.default_rng(5)
    T, I, O = 200, 300, 80
    M = (rng.random((O, I)) < 0.04).astype(np.uint8)
    M[0:16] = 0
    M[3] = 1                                   # block 0: one full row, a few short rows, many empty
    M[5, ::7] = 1
    M[9, 10:14] = 1
    M[16:32] = 0
    for r in (17, 20, 22, 31):                 # block 1: four long rows, twelve empty
        M[r, rng.random(I) < 0.7] = 1
    M[32:48] = (rng.random((16, I)) < 0.05)
    M[33] = 1
    M[40, : I // 2] = 1                        # block 2: two long rows, exactly four empty rows
    M[[34, 35, 36, 37]] = 0
    M[48:64] = (rng.random((16, I)) < 0.05)    # block 3: a full row, no empty row
    M[50] = 1
    M[48:64, 0] = 1
    W = (synth.normal(9, 77, (O, I), 0.02) * M).astype(np.float32)
    X, dY = synth.make_activations(9, 1, T, I, O)
    rig = Rig(W, M, T)
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, M)) <= TOL
    assert rel_err(rig.bwd_input(dY), opr.fc_bwd_input(dY, W, M)) <= TOL
    assert rel_err(rig.bwd_weight(dY, X), opr.fc_bwd_weight(dY, X, M)) <= TOL
    for shape in ((128, 2), (64, 3), (64, 8)):
        try:
            mst.mst_spmm_force_shape(*shape)
            assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, M)) <= TOL, shape
        finally:
            mst.mst_spmm_force_shape(0, 0)
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, M)
    np.testing.assert_array_equal(We, W)
    # the transposed problem puts the long rows into the col view
    rigT = Rig(np.ascontiguousarray(W.T), np.ascontiguousarray(M.T), T)
    Xt, dYt = synth.make_activations(9, 2, T, O, I)
    assert rel_err(rigT.bwd_input(dYt), opr.fc_bwd_input(dYt, W.T, M.T)) <= TOL
    assert rel_err(rigT.bwd_weight(dYt, Xt), opr.fc_bwd_weight(dYt, Xt, M.T)) <= TOL


def test_load_export_roundtrip_and_canonical_order():
    W, M, _, _ = _case(3, 8, 200, 333, 0.1)
    rig = Rig(W, M, 8)
    We, Me = rig.export()
    np.testing.assert_array_equal(Me, M)
    np.testing.assert_array_equal(We, W * M)
    np.testing.assert_array_equal(rig.indices(), np.flatnonzero(M.reshape(-1)))
    np.testing.assert_array_equal(rig.layer.values().cpu().numpy(), W[M != 0])


def test_garbage_behind_the_mask_is_ignored():
    W, M, X, dY = _case(4, 70, 96, 80, 0.2)
    W2 = W.copy()
    W2[M == 0] = 1e6
    rig = Rig(W2, M, 70)
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, M)) <= TOL
    We, _ = rig.export()
    np.testing.assert_array_equal(We, W * M)


def test_powerlaw_rows_and_full_rows():
    W, M, X, dY = _case(5, 256, 768, 768, 0.02, mask="powerlaw")
    assert M.sum(axis=1).max() >= 500        # some nearly full rows
    rig = Rig(W, M, 256)
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, M)) <= TOL
    assert rel_err(rig.bwd_input(dY), opr.fc_bwd_input(dY, W, M)) <= TOL
    assert rel_err(rig.bwd_weight(dY, X), opr.fc_bwd_weight(dY, X, M)) <= TOL


def test_degenerate_layers():
    T, I, O = 140, 136, 72
    X, dY = synth.make_activations(6, 1, T, I, O)
    W = synth.normal(6, 9, (O, I), 0.02)
    # empty layer: outputs are exactly zero
    rig = Rig(W, np.zeros((O, I), np.uint8), T)
    assert rig.layer.nnz == 0
    assert not rig.fwd(X).any() and not rig.bwd_input(dY).any()
    assert rig.bwd_weight(dY, X).size == 0
    # fully dense layer through the sparse kernels
    ones = np.ones((O, I), np.uint8)
    rig = Rig(W, ones, T, cap=O * I)
    rig.layer.set_path(mst.MST_PATH_SPARSE)
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, ones)) <= TOL
    assert rel_err(rig.bwd_input(dY), opr.fc_bwd_input(dY, W, ones)) <= TOL
    assert rel_err(rig.bwd_weight(dY, X), opr.fc_bwd_weight(dY, X, ones)) <= TOL
    # a single active weight
    one = np.zeros((O, I), np.uint8)
    one[71, 135] = 1
    rig = Rig(W, one, T)
    Y = rig.fwd(X)
    assert rel_err(Y, opr.fc_fwd(X, W, one)) <= TOL and not Y[:, :71].any()
    assert rel_err(rig.bwd_weight(dY, X), opr.fc_bwd_weight(dY, X, one)) <= TOL


def test_dense_path_matches_oracle():
    T, I, O = 200, 136, 264
    W, M, X, dY = _case(7, T, I, O, 0.6)
    rig = Rig(W, M, T, cap=O * I)
    rig.layer.set_path(mst.MST_PATH_DENSE)
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W, M)) <= TOL
    assert rel_err(rig.bwd_input(dY), opr.fc_bwd_input(dY, W, M)) <= TOL
    assert rel_err(rig.bwd_weight(dY, X), opr.fc_bwd_weight(dY, X, M)) <= TOL
    # auto picks the dense kernels at this density and must agree with the sparse ones
    rig.layer.set_path(mst.MST_PATH_AUTO)
    Ya = rig.fwd(X)
    rig.layer.set_path(mst.MST_PATH_SPARSE)
    assert rel_err(Ya, rig.fwd(X)) <= TOL


@pytest.mark.parametrize("T,I,O", [(300, 200, 333), (1024, 768, 768), (130, 64, 2304)])
def test_dense_grad_matches_oracle(T, I, O):
    X, dY = synth.make_activations(8, 2, T, I, O)
    G = torch.full((O, I), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(mst.mst_workspace_bytes(O, I, 16, T), dtype=torch.uint8, device=DEV)
    mst.mst_dense_grad(dev(dY), dev(X), G, T, O, I, mst.MST_F32, ws)
    torch.cuda.synchronize()
    ref = opr.dense_grad(dY, X)
    assert rel_err(G.cpu().numpy(), ref) <= TOL
    G2 = torch.full((O, I), float("nan"), dtype=torch.float32, device=DEV)
    mst.mst_dense_grad(dev(dY), dev(X), G2, T, O, I, mst.MST_F32, None)     # no split workspace
    torch.cuda.synchronize()
    assert rel_err(G2.cpu().numpy(), ref) <= TOL


def test_bf16_activations_fp32_accumulate():
    T, I, O = 260, 1024, 512
    W, M = synth.make_layer(9, 1, I, O, 0.05)
    Xf, dYf, xb, yb = synth.make_activations(9, 1, T, I, O, "bf16")
    rig = Rig(W, M, T)
    xb_d, yb_d = dev(xb.view(np.int16)), dev(yb.view(np.int16))
    Y = torch.empty((T, O), dtype=torch.float32, device=DEV)
    dX = torch.empty((T, I), dtype=torch.float32, device=DEV)
    dW = torch.empty(rig.layer.nnz, dtype=torch.float32, device=DEV)
    G = torch.empty((O, I), dtype=torch.float32, device=DEV)
    mst.mst_sparse_fc_fwd(rig.layer, xb_d, Y, T, mst.MST_BF16)
    mst.mst_sparse_fc_bwd_input(rig.layer, yb_d, dX, T, mst.MST_BF16)
    mst.mst_sparse_fc_bwd_weight(rig.layer, yb_d, xb_d, dW, T, rig.ws, mst.MST_BF16)
    mst.mst_dense_grad(yb_d, xb_d, G, T, O, I, mst.MST_BF16, rig.ws)
    torch.cuda.synchronize()
    # the oracle sees exactly the bf16-rounded inputs, widened to fp64
    assert rel_err(Y.cpu().numpy(), opr.fc_fwd(Xf, W, M)) <= TOL
    assert rel_err(dX.cpu().numpy(), opr.fc_bwd_input(dYf, W, M)) <= TOL
    assert rel_err(dW.cpu().numpy(), opr.fc_bwd_weight(dYf, Xf, M)) <= TOL
    assert rel_err(G.cpu().numpy(), opr.dense_grad(dYf, Xf)) <= TOL


@pytest.mark.parametrize("T,I,O", [(333, 130, 203), (1000, 264, 72), (70, 8, 8)])
def test_bf16_dense_grad_ragged_shapes(T, I, O):
    """The bf16 MFMA gradient where rows are not multiples of eight elements (element-wise
    edge loads), tiles are partial and the k range does not fill a step."""
    Xf, dYf, xb, yb = synth.make_activations(12, 3, T, I, O, "bf16")
    G = torch.full((O, I), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(mst.mst_workspace_bytes(O, I, 16, T), dtype=torch.uint8, device=DEV)
    mst.mst_dense_grad(dev(yb.view(np.int16)), dev(xb.view(np.int16)), G, T, O, I, mst.MST_BF16, ws)
    torch.cuda.synchronize()
    assert rel_err(G.cpu().numpy(), opr.dense_grad(dYf, Xf)) <= TOL


def test_results_are_bit_reproducible():
    W, M, X, dY = _case(10, 384, 256, 384, 0.1)
    rig = Rig(W, M, 384)
    a = (rig.fwd(X), rig.bwd_input(dY), rig.bwd_weight(dY, X))
    b = (rig.fwd(X), rig.bwd_input(dY), rig.bwd_weight(dY, X))
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_sync_values_after_optimizer_step():
    W, M, X, dY = _case(12, 200, 256, 192, 0.1)
    rig = Rig(W, M, 200)
    vals = rig.layer.values()
    vals.mul_(0.5).add_(0.01)                     # caller's optimiser updates in place
    rig.layer.sync_values()
    W2 = W.copy()
    W2[M != 0] = W[M != 0] * np.float32(0.5) + np.float32(0.01)
    assert rel_err(rig.fwd(X), opr.fc_fwd(X, W2, M)) <= TOL
    assert rel_err(rig.bwd_input(dY), opr.fc_bwd_input(dY, W2, M)) <= TOL


def test_argument_errors_launch_nothing():
    W, M, X, dY = _case(13, 16, 32, 32, 0.2)
    rig = Rig(W, M, 16)
    Y = torch.empty((16, 32), dtype=torch.float32, device=DEV)
    with pytest.raises(mst.MstError):
        mst.mst_sparse_fc_fwd(rig.layer, dev(X), Y, 0)                       # T < 1
    small = torch.empty(64, dtype=torch.uint8, device=DEV)
    dW = torch.empty(rig.layer.nnz, dtype=torch.float32, device=DEV)
    with pytest.raises(mst.MstError) as e:
        mst.mst_sparse_fc_bwd_weight(rig.layer, dev(dY), dev(X), dW, 16, small)
    assert e.value.code == -3
    with pytest.raises(mst.MstError) as e:                                    # capacity exceeded
        tiny = mst.Layer(32, 32, 4, DEV)
        tiny.load_dense(dev(W), dev(M), rig.ws)
    assert e.value.code == -4


def test_gather_active_format_stats_and_lds_probe():
    O, I, T = 200, 333, 64
    W, M = synth.make_layer(31, 1, I, O, 0.07)
    rig = Rig(W, M, T)
    G = synth.normal(31, 5, (O, I))
    dW = torch.full((rig.layer.nnz,), float("nan"), dtype=torch.float32, device=DEV)
    mst.mst_gather_active(rig.layer, dev(G), dW)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(dW.cpu().numpy(), G[M != 0])          # ascending flat index
    fs = rig.layer.format_stats()
    nnz = int(M.sum())
    assert fs["nnz"] == nnz
    # every view stores each active weight once plus padding; padding is bounded by the format
    # (longest of four rows per 128-index chunk, even step counts)
    for v, (R, K) in (("row", (O, I)), ("col", (I, O))):
        slots = fs[v + "_view_slots"]
        assert slots >= nnz and slots % 8 == 0
        assert 0.0 < fs[v + "_view_efficiency"] <= 1.0
        assert abs(fs[v + "_view_efficiency"] - nnz / slots) < 1e-12
    # an exact count of the row view's slots from the mask: per chunk and quad of the ranked rows
    out = torch.empty(4 * 1024, dtype=torch.float32, device=DEV)
    for width in (4, 8, 16):
        mst.mst_probe_lds_read(out, width, 10, 4)
    torch.cuda.synchronize()
    assert np.isfinite(out.cpu().numpy()).all()
    with pytest.raises(mst.MstError):
        mst.mst_probe_lds_read(out, 5, 10, 4)


@pytest.mark.parametrize("T,I,O", [(512, 256, 384), (1024, 768, 768), (256, 128, 1280), (512, 256, 768), (768, 512, 256)])
def test_dense_products_on_the_bf16_split_kernel(T, I, O):
    """Shapes of whole tiles: the dense fp32 products (dense gradient; forward and input
    gradient of a dense layer) take the kernel that splits every fp32 operand into two
    bfloat16 values and adds three bf16 MFMA products.  Against the oracle within the fp32
    tolerance, and against the plain fp32 MFMA kernel (pinned by the hook)."""
    print("case", T, I, O, flush=True)
    X, dY = synth.make_activations(41, 2, T, I, O)
    # values over several orders of magnitude in every operand, so that hi + lo matters
    X = (X * np.exp2(synth.normal(41, 7, X.shape) * 3)).astype(np.float32)
    W = synth.normal(41, 3, (O, I), 0.02)
    M = np.ones((O, I), np.uint8)
    rig = Rig(W, M, T, cap=O * I)
    Xd, dYd = dev(X), dev(dY)
    res = {}
    try:
        for mode in (128, 256, 1):          # split kernel with either workgroup tile (where the shape allows), fp32 MFMA
            mst.mst_gemm_force_fp32_mfma(mode)
            G = torch.full((O, I), float("nan"), dtype=torch.float32, device=DEV)
            mst.mst_dense_grad(dYd, Xd, G, T, O, I, mst.MST_F32, rig.ws)
            torch.cuda.synchronize()
            res[mode] = (G.cpu().numpy(), rig.fwd(X), rig.bwd_input(dY))
    finally:
        mst.mst_gemm_force_fp32_mfma(0)
    refs = (opr.dense_grad(dY, X), opr.fc_fwd(X, W, M), opr.fc_bwd_input(dY, W, M))
    for name, got128, got256, got_f32, ref in zip(("G", "Y", "dX"), res[128], res[256], res[1], refs):
        e0, e2, e1 = rel_err(got128, ref), rel_err(got256, ref), rel_err(got_f32, ref)
        print(name, "split-128 err %.3g  split-256 err %.3g  fp32-mfma err %.3g" % (e0, e2, e1), flush=True)
        assert e0 <= TOL and e1 <= TOL and e2 <= TOL
        # hi + lo carries 16 significant bits: at most 3 * 2^-18 = 1.1e-5 of a product is lost
        assert e0 <= 2e-5 and e2 <= 2e-5
        assert not np.array_equal(got128, got_f32) or e0 == 0.0         # the kernels really differ


@pytest.mark.parametrize("T,I,O,tile", [(256, 320, 128, 160), (512, 320, 640, 160), (768, 128, 160, 160), (1024, 640, 320, 160),
                                        (256, 192, 128, 192), (512, 384, 768, 192), (768, 64, 192, 192), (1024, 768, 576, 192)])
def test_dense_products_on_the_narrow_workgroup_tiles(T, I, O, tile):
    """Forward (output O wide) and input gradient (output I wide) of a dense layer pinned to the
    256 x 160 or the 256 x 192 workgroup tile of the split kernel where the output width is a
    multiple of it (the other product falls back to another tile), against the oracle."""
    print("case", T, I, O, tile, flush=True)
    X, dY = synth.make_activations(45, 2, T, I, O)
    X = (X * np.exp2(synth.normal(45, 7, X.shape) * 3)).astype(np.float32)
    W = synth.normal(45, 3, (O, I), 0.02)
    M = np.ones((O, I), np.uint8)
    rig = Rig(W, M, T, cap=O * I)
    rig.layer.set_path(mst.MST_PATH_DENSE)
    tiles = {}
    try:
        mst.mst_gemm_force_fp32_mfma(tile)
        Y = rig.fwd(X)
        tiles["Y"] = mst.mst_gemm_last_tile()
        dX = rig.bwd_input(dY)
        tiles["dX"] = mst.mst_gemm_last_tile()
        mst.mst_gemm_force_fp32_mfma(128)
        Y128, dX128 = rig.fwd(X), rig.bwd_input(dY)
    finally:
        mst.mst_gemm_force_fp32_mfma(0)
    for name, got, got128, ref, width, depth in (("Y", Y, Y128, opr.fc_fwd(X, W, M), O, I),
                                                 ("dX", dX, dX128, opr.fc_bwd_input(dY, W, M), I, O)):
        e = rel_err(got, ref)
        print(name, "width", width, "tile", tiles[name], "err %.3g" % e, flush=True)
        assert e <= 2e-5
        if width % tile == 0 and depth % 64 == 0:
            assert tiles[name] == tile                   # the pinned tile really ran
            if width % 128 == 0:
                np.testing.assert_array_equal(got, got128)   # every tile adds a result's terms in the same order


@pytest.mark.parametrize("T,I,O", [(64, 256, 256), (128, 256, 512), (1088, 512, 256), (2048, 768, 768)])
def test_bf16_dense_gradient_on_both_workgroup_tiles(T, I, O):
    """G = dY^T X with bfloat16 operands on whole 256 x 256 tiles: the two-stage 256-tile kernel
    (one, two, an odd and a split number of k steps) and the 128-tile kernel, each against
    the oracle on the same bfloat16 values; the products are exact in fp32, so the two
    kernels differ only by the order of fp32 additions."""
    print("case", T, I, O, flush=True)
    Xf, dYf, xb, yb = synth.make_activations(43, 5, T, I, O, "bf16")
    Xd, dYd = dev(xb.view(np.int16)), dev(yb.view(np.int16))
    ref = opr.dense_grad(dYf, Xf)
    ws = torch.empty(8 * O * I * 4, dtype=torch.uint8, device=DEV)
    got = {}
    try:
        for mode in (128, 256):
            for w in (None, ws):
                mst.mst_gemm_force_fp32_mfma(mode)
                G = torch.full((O, I), float("nan"), dtype=torch.float32, device=DEV)
                mst.mst_dense_grad(dYd, Xd, G, T, O, I, mst.MST_BF16, w)
                torch.cuda.synchronize()
                got[(mode, w is not None)] = G.cpu().numpy()
    finally:
        mst.mst_gemm_force_fp32_mfma(0)
    for key, g in got.items():
        e = rel_err(g, ref)
        print(key, "err %.3g" % e, flush=True)
        assert e <= 2e-6                      # fp32 accumulation of exact products
    assert rel_err(got[(256, False)], got[(128, False)]) <= 2e-6


@pytest.mark.parametrize("T,I,O", [(256, 256, 512), (512, 768, 256), (768, 32, 256), (1024, 288, 768)])
def test_dense_products_with_bf16_activations_on_the_256_tile(T, I, O):
    """Y and dX of a dense-path layer with bfloat16 activations on whole 256 x 256 tiles: the
    activations go to the matrix cores as they are, the fp32 weights as bf16 hi + lo (two
    products per term).  Against the oracle on the same bfloat16 values, and against the fp32
    MFMA kernel that serves ragged shapes (pinned by the hook)."""
    print("case", T, I, O, flush=True)
    W = synth.normal(47, 3, (O, I), 0.02)
    W = (W * np.exp2(synth.normal(47, 8, W.shape) * 3)).astype(np.float32)     # weights over several orders of magnitude
    M = synth.make_layer(47, 1, I, O, 0.5)[1]
    Xf, dYf, xb, yb = synth.make_activations(47, 1, T, I, O, "bf16")
    rig = Rig(W * M, M, T, cap=O * I)
    rig.layer.set_path(mst.MST_PATH_DENSE)

    def run():
        Y = torch.full((T, O), float("nan"), dtype=torch.float32, device=DEV)
        dX = torch.full((T, I), float("nan"), dtype=torch.float32, device=DEV)
        mst.mst_sparse_fc_fwd(rig.layer, dev(xb.view(np.int16)), Y, T, mst.MST_BF16)
        ty = mst.mst_gemm_last_tile()
        mst.mst_sparse_fc_bwd_input(rig.layer, dev(yb.view(np.int16)), dX, T, mst.MST_BF16)
        tx = mst.mst_gemm_last_tile()
        torch.cuda.synchronize()
        return Y.cpu().numpy(), dX.cpu().numpy(), ty, tx

    try:
        Y, dX, ty, tx = run()
        mst.mst_gemm_force_fp32_mfma(1)
        Y32, dX32, _, _ = run()
    finally:
        mst.mst_gemm_force_fp32_mfma(0)
    # Y is O wide with depth I, dX is I wide with depth O: whole tiles and a depth that is a multiple of 32
    assert ty == (256 if O % 256 == 0 and I % 32 == 0 else 0)
    assert tx == (256 if I % 256 == 0 and O % 32 == 0 else 0)
    for name, got, got32, ref in (("Y", Y, Y32, opr.fc_fwd(Xf, W, M)), ("dX", dX, dX32, opr.fc_bwd_input(dYf, W, M))):
        e, e32 = rel_err(got, ref), rel_err(got32, ref)
        print(name, "err %.3g  fp32-mfma err %.3g" % (e, e32), flush=True)
        assert e <= 2e-5 and e32 <= TOL
