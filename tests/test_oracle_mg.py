"""Pins for oracle.mixed_growing (Algorithm 1): counts, RandK keys, selections, invariants."""
import random
import struct

import numpy as np
import pytest

from oracle import mixed_growing as mg


# ----------------------------------------------------------------- counts

def test_counts_worked_examples(golden):
    for row in golden("mg_counts_768x3072.txt"):
        N, nnz = int(row[0]), int(row[1])
        d, z, R = float(row[2]), float(row[3]), float(row[4])
        want = dict(zip(["nnz_target", "n_prune", "n_grow", "n_rand", "n_grad"], map(int, row[5:])))
        assert mg.counts(N, nnz, d, z, R) == want


def test_counts_conserve_and_stay_in_range():
    rnd = random.Random(0)
    for _ in range(3000):
        N = rnd.randint(1, 5000)
        nnz = rnd.randint(0, N)
        d, z, R = rnd.random(), rnd.random(), rnd.random()
        if rnd.random() < 0.1:
            d = rnd.choice([0.0, 1.0])
        if rnd.random() < 0.1:
            z = rnd.choice([0.0, 1.0])
        c = mg.counts(N, nnz, d, z, R)
        assert nnz - c["n_prune"] + c["n_grow"] == c["nnz_target"]         # lands on the target
        assert abs(c["nnz_target"] / N - d) <= 0.5 / N + 1e-12              # density equals schedule
        assert 0 <= c["n_prune"] <= nnz and 0 <= c["n_grow"] <= N - nnz
        assert c["n_rand"] + c["n_grad"] == c["n_grow"] and c["n_rand"] >= 0 and c["n_grad"] >= 0
        assert c["n_rand"] == int(c["n_grow"] * R)


def test_counts_same_target_keeps_count_and_uses_zeta():
    c = mg.counts(10000, 1000, 0.1, 0.3, 0.25)
    assert c == dict(nnz_target=1000, n_prune=300, n_grow=300, n_rand=75, n_grad=225)


# ----------------------------------------------------------------- RandK keys

def test_randk_key_is_splitmix64(golden):
    want = [int(r[0]) for r in golden("splitmix64_seed1234567.txt")]
    got = mg.randk_key(1234567, np.arange(len(want)))
    assert [int(x) for x in got] == want
    # scalar re-derivation in Python integers for other seeds / indices
    def ref(seed, f):
        m = (1 << 64) - 1
        z = (seed + (f + 1) * 0x9E3779B97F4A7C15) & m
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
        return z ^ (z >> 31)
    for seed in (0, 1, 2 ** 63 + 5, 2 ** 64 - 1):
        fs = [0, 1, 77, 2 ** 31, 6553599]
        assert [int(x) for x in mg.randk_key(seed, np.array(fs))] == [ref(seed, f) for f in fs]


def test_abs_bits_orders_like_magnitude():
    v = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-30, -2.5, 2.5, 3.0, -1e38], dtype=np.float32)
    b = mg.abs_bits(v)
    assert b[0] == b[1] == 0 and b[5] == b[6]
    order = np.argsort(b, kind="stable")
    assert list(np.abs(v[order])) == sorted(np.abs(v).tolist())


# ----------------------------------------------------------------- selections

def _abs32(x):
    return struct.unpack("<I", struct.pack("<f", abs(float(x))))[0]


def _brute_force(W, M, G, d, z, R, seed):
    """Algorithm 1 with Python's sorted() on explicit (score, flat index) tuples."""
    O, I = W.shape
    N = O * I
    act = [f for f in range(N) if M[f // I, f % I]]
    ina = [f for f in range(N) if not M[f // I, f % I]]
    c = mg.counts(N, len(act), d, z, R)
    prune = sorted(act, key=lambda f: (_abs32(W[f // I, f % I]), f))[: c["n_prune"]]
    grad = sorted(ina, key=lambda f: (-_abs32(G[f // I, f % I]), f))[: c["n_grad"]]
    gs = set(grad)
    rest = [f for f in ina if f not in gs]
    m = (1 << 64) - 1
    def key(f):
        zz = (seed + (f + 1) * 0x9E3779B97F4A7C15) & m
        zz = ((zz ^ (zz >> 30)) * 0xBF58476D1CE4E5B9) & m
        zz = ((zz ^ (zz >> 27)) * 0x94D049BB133111EB) & m
        return zz ^ (zz >> 31)
    rand = sorted(rest, key=lambda f: (key(f), f))[: c["n_rand"]]
    return sorted(prune), sorted(grad), sorted(rand)


def _layer(seed, O, I, density, quantise=None):
    rng = np.random.default_rng(seed)
    M = (rng.random((O, I)) < density).astype(np.uint8)
    W = rng.standard_normal((O, I)).astype(np.float32)
    G = rng.standard_normal((O, I)).astype(np.float32)
    if quantise:                      # many exact duplicates and zeros -> ties everywhere
        W = (np.round(W * quantise) / quantise).astype(np.float32)
        G = (np.round(G * quantise) / quantise).astype(np.float32)
    W *= M
    return W, M, G


@pytest.mark.parametrize("seed,quant", [(0, None), (1, 2), (2, 1), (3, 4)])
@pytest.mark.parametrize("d_t,zeta,R", [(0.3, 0.3, 0.25), (0.2, 0.5, 0.5), (0.45, 0.2, 0.0), (0.3, 1.0, 1.0)])
def test_update_equals_brute_force_on_tiny_layers(seed, quant, d_t, zeta, R):
    W, M, G = _layer(seed, 6, 7, 0.3, quant)
    out = mg.update(W, M, G, d_t, zeta, R, seed=99 + seed)
    p, g, r = _brute_force(W, M, G, d_t, zeta, R, 99 + seed)
    assert out["prune"].tolist() == p
    assert out["grad"].tolist() == g
    assert out["rand"].tolist() == r


def _check_invariants(W, M, G, out, d_t):
    I = W.shape[1]
    Mb = M.reshape(-1) != 0
    Mn = out["M"].reshape(-1) != 0
    c = out["counts"]
    p, g, r = set(out["prune"].tolist()), set(out["grad"].tolist()), set(out["rand"].tolist())
    assert int(Mn.sum()) == c["nnz_target"] == mg.target_count(Mb.size, d_t)
    assert len(p) == c["n_prune"] and len(g) == c["n_grad"] and len(r) == c["n_rand"]
    assert all(Mb[f] for f in p) and not any(Mb[f] for f in g | r)
    assert not (p & g) and not (p & r) and not (g & r)
    assert all(not Mn[f] for f in p) and all(Mn[f] for f in g | r)
    kept = [f for f in np.flatnonzero(Mb) if f not in p]
    Wf, Gf = W.reshape(-1), G.reshape(-1)
    if p and kept:      # every pruned weight is smaller (in the total order) than every kept one
        assert max((_abs32(Wf[f]), f) for f in p) < min((_abs32(Wf[f]), f) for f in kept)
    unchosen = [f for f in np.flatnonzero(~Mb) if f not in g]
    if g and unchosen:  # every gradient-grown position beats every unchosen candidate
        assert max((-_abs32(Gf[f]), f) for f in g) < min((-_abs32(Gf[f]), f) for f in unchosen)
    Wn = out["W"].reshape(-1)
    assert all(Wn[f] == 0 for f in p | g | r) and not Wn[~Mn].any()
    assert all(Wn[f] == Wf[f] for f in kept)


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("d_t", [0.1, 0.12, 0.05, 0.6, 1.0, 0.0])
def test_update_invariants(seed, d_t):
    W, M, G = _layer(seed, 24, 40, 0.1, quantise=8 if seed % 2 else None)
    out = mg.update(W, M, G, d_t, 0.3, 0.25, seed)
    _check_invariants(W, M, G, out, d_t)


def test_special_cases_rigl_set_and_no_op():
    W, M, G = _layer(5, 16, 32, 0.2)
    d = M.mean()
    rigl = mg.update(W, M, G, d, 0.3, 0.0, 1)       # R = 0: gradient growth only
    setm = mg.update(W, M, G, d, 0.3, 1.0, 1)       # R = 1: random growth only
    assert rigl["rand"].size == 0 and rigl["grad"].size == rigl["counts"]["n_grow"]
    assert setm["grad"].size == 0 and setm["rand"].size == setm["counts"]["n_grow"]
    assert rigl["prune"].tolist() == setm["prune"].tolist()
    assert int(rigl["M"].sum()) == int(M.sum()) == int(setm["M"].sum())   # count preserved
    same = mg.update(W, M, G, d, 0.0, 0.25, 1)      # zeta = 0, same density: nothing moves
    np.testing.assert_array_equal(same["M"], M)
    np.testing.assert_array_equal(same["W"], W)


def test_zero_valued_active_weight_is_pruned_first():
    W, M, G = _layer(6, 8, 8, 0.5)
    act = np.flatnonzero(M.reshape(-1))
    W.reshape(-1)[act[5]] = 0.0                      # e.g. grown by the previous update
    W.reshape(-1)[act[9]] = -0.0
    out = mg.update(W, M, G, M.mean(), 2.0 / act.size + 1e-9, 0.5, 3)
    assert out["prune"].tolist() == [act[5], act[9]]


def test_random_growth_is_uniform_over_candidates():
    O, I = 8, 16
    rng = np.random.default_rng(0)
    M = (rng.random((O, I)) < 0.25).astype(np.uint8)
    W = rng.standard_normal((O, I)).astype(np.float32) * M
    G = np.zeros((O, I), dtype=np.float32)
    cand = np.flatnonzero(M.reshape(-1) == 0)
    hits = np.zeros(O * I)
    trials = 4000
    for s in range(trials):
        out = mg.update(W, M, G, M.mean(), 0.5, 1.0, seed=s * 7919 + 13)
        hits[out["rand"]] += 1
    k = out["counts"]["n_rand"]
    assert hits[M.reshape(-1) != 0].sum() == 0
    expect = trials * k / cand.size
    chi2 = float(((hits[cand] - expect) ** 2 / (expect * (1 - k / cand.size))).sum())
    dof = cand.size - 1
    assert abs(chi2 - dof) < 6 * (2 * dof) ** 0.5    # ~6 sigma band


# ----------------------------------------------------------------- the other prune criterion

def test_prune_lambda_zero_is_the_magnitude_criterion():
    W, M, G = _layer(5, 9, 11, 0.4)
    a = mg.update(W, M, G, 0.35, 0.3, 0.25, 77)
    b = mg.update(W, M, G, 0.35, 0.3, 0.25, 77, prune_lambda=0.0)
    for k in ("prune", "grad", "rand"):
        np.testing.assert_array_equal(a[k], b[k])


@pytest.mark.parametrize("lam", [0.25, 1.0, 3.0])
def test_prune_lambda_brute_force_on_dyadic_values(lam):
    # multiples of 1/8 below 16 and a dyadic lambda: |w| + lambda |g| is exact in fp32 and in
    # Python floats alike, so sorting Python tuples is an independent statement of the order
    rng = np.random.default_rng(9)
    O, I = 7, 9
    M = (rng.random((O, I)) < 0.5).astype(np.uint8)
    W = (rng.integers(-40, 41, (O, I)) / 8.0).astype(np.float32) * M
    G = (rng.integers(-40, 41, (O, I)) / 8.0).astype(np.float32)
    N = O * I
    act = [f for f in range(N) if M.flat[f]]
    c = mg.counts(N, len(act), 0.45, 0.4, 0.5)
    want = sorted(sorted(act, key=lambda f: (abs(float(W.flat[f])) + lam * abs(float(G.flat[f])), f))[: c["n_prune"]])
    got = mg.update(W, M, G, 0.45, 0.4, 0.5, 3, prune_lambda=lam)
    assert got["prune"].tolist() == want
    # the growth sets do not depend on the prune criterion
    ref = mg.update(W, M, G, 0.45, 0.4, 0.5, 3)
    np.testing.assert_array_equal(got["grad"], ref["grad"])
    np.testing.assert_array_equal(got["rand"], ref["rand"])
    assert got["prune"].tolist() != ref["prune"].tolist()          # the criterion matters on this input


def test_prune_lambda_large_ranks_by_gradient_alone():
    W, M, G = _layer(6, 10, 12, 0.5)
    act = np.flatnonzero(M.reshape(-1))
    got = mg.update(W, M, G, 0.5, 0.3, 0.0, 1, prune_lambda=2.0 ** 40)
    order = sorted(act.tolist(), key=lambda f: (_abs32(G.flat[f]), f))
    assert got["prune"].tolist() == sorted(order[: got["counts"]["n_prune"]])


def test_prune_score_rounds_product_then_sum():
    # 3 * (1 + 2^-23) needs 25 bits: the product rounds to 3 + 2^-21 (ties to even) before 1 is added
    w = np.array([1.0], np.float32)
    g = np.array([1.0 + 2.0 ** -23], np.float32)
    bits = mg.prune_score_bits(w, g, 3.0)
    prod = np.float32(3.0) * g[0]
    assert bits.view(np.float32)[0] == np.float32(np.float32(1.0) + prod)
    assert float(prod) == 3.0 + 2.0 ** -21
