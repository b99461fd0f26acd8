"""Pins for oracle.products: brute force, reduction to a plain product, adjoint identities."""
import numpy as np
import pytest

from oracle import products as pr


def _tiny(seed, T=3, I=5, O=4, density=0.5):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((T, I)).astype(np.float32)
    dY = rng.standard_normal((T, O)).astype(np.float32)
    W = rng.standard_normal((O, I)).astype(np.float32)
    M = (rng.random((O, I)) < density).astype(np.uint8)
    return X, dY, W, M


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_python_loops(seed):
    X, dY, W, M = _tiny(seed)
    T, I = X.shape
    O = W.shape[0]
    Y = [[0.0] * O for _ in range(T)]
    dX = [[0.0] * I for _ in range(T)]
    dW = []
    G = [[0.0] * I for _ in range(O)]
    for t in range(T):
        for o in range(O):
            for i in range(I):
                if M[o, i]:
                    Y[t][o] += float(X[t, i]) * float(W[o, i])
                    dX[t][i] += float(dY[t, o]) * float(W[o, i])
    for o in range(O):
        for i in range(I):
            s = 0.0
            for t in range(T):
                s += float(dY[t, o]) * float(X[t, i])
            G[o][i] = s
    for f in range(O * I):                  # ascending flat index o*I + i
        if M[f // I, f % I]:
            dW.append(G[f // I][f % I])
    np.testing.assert_allclose(pr.fc_fwd(X, W, M), np.array(Y), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(pr.fc_bwd_input(dY, W, M), np.array(dX), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(pr.dense_grad(dY, X), np.array(G), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(pr.fc_bwd_weight(dY, X, M), np.array(dW), rtol=1e-13, atol=1e-14)
    assert pr.fc_fwd(X, W, M).dtype == np.float64


def test_density_one_is_plain_matmul_and_density_zero_is_zero():
    X, dY, W, _ = _tiny(7, T=6, I=9, O=5)
    ones = np.ones_like(W, dtype=np.uint8)
    np.testing.assert_allclose(pr.fc_fwd(X, W, ones), X.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-14)
    np.testing.assert_allclose(pr.fc_bwd_input(dY, W, ones), dY.astype(np.float64) @ W.astype(np.float64), rtol=1e-14)
    assert pr.fc_bwd_weight(dY, X, ones).shape == (W.size,)
    zeros = np.zeros_like(ones)
    assert not pr.fc_fwd(X, W, zeros).any() and not pr.fc_bwd_input(dY, W, zeros).any()
    assert pr.fc_bwd_weight(dY, X, zeros).size == 0


def test_masked_out_weights_do_not_matter():
    X, dY, W, M = _tiny(3, T=4, I=8, O=6)
    W2 = W.copy()
    W2[M == 0] = 1e6                        # garbage behind the mask must be invisible
    np.testing.assert_array_equal(pr.fc_fwd(X, W, M), pr.fc_fwd(X, W2, M))
    np.testing.assert_array_equal(pr.fc_bwd_input(dY, W, M), pr.fc_bwd_input(dY, W2, M))


def test_adjoint_identities_tie_the_three_products():
    X, dY, W, M = _tiny(11, T=17, I=13, O=7, density=0.3)
    Y = pr.fc_fwd(X, W, M)
    dX = pr.fc_bwd_input(dY, W, M)
    dW = pr.fc_bwd_weight(dY, X, M)
    a = float((dY.astype(np.float64) * Y).sum())
    b = float((dX * X).sum())
    c = float((dW * W.astype(np.float64)[M != 0]).sum())
    assert a == pytest.approx(b, rel=1e-12) and a == pytest.approx(c, rel=1e-12)


def test_linearity_and_single_entry_probe():
    X, dY, W, M = _tiny(5, T=4, I=6, O=3)
    X2 = np.roll(X, 1, axis=0)
    np.testing.assert_allclose(pr.fc_fwd(X + X2, W, M), pr.fc_fwd(X, W, M) + pr.fc_fwd(X2, W, M), atol=1e-6)
    # one active weight at (o, i) = (2, 4): Y[:, 2] = w * X[:, 4], dX[:, 4] = w * dY[:, 2]
    W1 = np.zeros_like(W); M1 = np.zeros_like(M)
    W1[2, 4] = 0.5; M1[2, 4] = 1
    Y = pr.fc_fwd(X, W1, M1)
    np.testing.assert_allclose(Y[:, 2], 0.5 * X[:, 4].astype(np.float64))
    assert not np.delete(Y, 2, axis=1).any()
    dX = pr.fc_bwd_input(dY, W1, M1)
    np.testing.assert_allclose(dX[:, 4], 0.5 * dY[:, 2].astype(np.float64))
    assert not np.delete(dX, 4, axis=1).any()
    np.testing.assert_allclose(pr.fc_bwd_weight(dY, X, M1), [np.dot(dY[:, 2].astype(np.float64), X[:, 4])])


def test_elementwise_probes_agree_with_full_products():
    X, dY, W, M = _tiny(9, T=8, I=10, O=7)
    Y, dX, G = pr.fc_fwd(X, W, M), pr.fc_bwd_input(dY, W, M), pr.dense_grad(dY, X)
    for (t, o, i) in [(0, 0, 0), (7, 6, 9), (3, 2, 5)]:
        assert pr.fc_fwd_at(X, W, M, t, o) == pytest.approx(Y[t, o], rel=1e-13, abs=1e-14)
        assert pr.fc_bwd_input_at(dY, W, M, t, i) == pytest.approx(dX[t, i], rel=1e-13, abs=1e-14)
        assert pr.dense_grad_at(dY, X, o, i) == pytest.approx(G[o, i], rel=1e-13, abs=1e-14)
