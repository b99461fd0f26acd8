"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and its host arithmetic (schedule, count lines) equals the oracle's."""
import os
import random
import re

import pytest

import paper_2408_11746_amd as mst
from paper_2408_11746_amd import binding
from oracle import mixed_growing as omg
from oracle import schedule as osc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "mst.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(mst_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert len(names) >= 20 and "mst_sparse_fc_fwd" in names and "mst_schedule_density" in names
    L = mst.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names          # the binding covers the whole header
    assert b"gfx950" in L.mst_version()


def test_five_named_entry_points_exist_in_binding():
    for n in ["mst_sparse_fc_fwd", "mst_sparse_fc_bwd_input", "mst_sparse_fc_bwd_weight", "mst_mask_update",
              "mst_schedule_density"]:
        assert callable(getattr(mst, n))


def test_schedule_matches_oracle_everywhere_it_changes():
    for kw in [dict(), dict(S_M=0.9, N=4, Delta_W=10, T_U=33, Delta_R=7, zeta=[0.3, 0.25, 0.2, 0.1, 0.05]),
               dict(S_M=0.5, N=1, Delta_W=5, T_U=0, Delta_R=5, zeta=[0.5, 0.1])]:
        cfg = mst.ScheduleCfg(**kw)
        ocfg = osc.ScheduleCfg(S_M=cfg.S_M, N=cfg.N, Delta_W=cfg.Delta_W, T_U=cfg.T_U, Delta_R=cfg.Delta_R,
                               zeta=list(cfg.zeta))
        total = ocfg.T_W + ocfg.T_U + ocfg.T_R + 50
        steps = set(range(0, total, max(1, total // 997))) | {0, total - 1}
        for b in osc.zeta_boundaries(ocfg):
            steps |= {max(0, b - 1), b, b + 1}
        for k in range(ocfg.N + 1):
            steps |= {k * ocfg.Delta_W, max(0, k * ocfg.Delta_W - 1)}
        for t in sorted(steps):
            d, z = mst.mst_schedule_density(cfg, t)
            assert d == pytest.approx(osc.density(ocfg, t), abs=1e-15), t
            assert z == pytest.approx(osc.zeta(ocfg, t), abs=1e-15), t


def test_schedule_rejects_bad_arguments():
    with pytest.raises(mst.MstError):
        mst.mst_schedule_density(mst.ScheduleCfg(), -1)
    with pytest.raises(mst.MstError):
        mst.mst_schedule_density(mst.ScheduleCfg(zeta=[0.3]), 5)
    with pytest.raises(mst.MstError):
        mst.mst_schedule_density(mst.ScheduleCfg(S_M=1.5), 5)


def test_update_counts_match_oracle():
    rnd = random.Random(1)
    cases = [(2359296, 117965, 0.05, 0.3, 0.25), (2359296, 2359296, 0.53152, 0.3, 0.25),
             (2359296, 2341177, 1.0, 0.3, 0.25), (10, 0, 0.5, 0.3, 0.5), (10, 10, 0.0, 0.0, 0.0)]
    for _ in range(2000):
        N = rnd.randint(1, 10 ** 7)
        cases.append((N, rnd.randint(0, N), rnd.random(), rnd.random(), rnd.random()))
    for N, nnz, d, z, R in cases:
        got = mst.mst_update_counts(N, nnz, d, z, R)
        want = omg.counts(N, nnz, d, z, R)
        assert got["nnz_after"] == want["nnz_target"] and got["nnz_before"] == nnz
        for k in ("n_prune", "n_grow", "n_rand", "n_grad"):
            assert got[k] == want[k], (N, nnz, d, z, R, k)


def test_size_queries_and_argument_errors():
    assert mst.mst_layer_device_bytes(0, 5, 1) == 0
    assert mst.mst_layer_device_bytes(70000, 5, 1) == 0
    assert mst.mst_layer_device_bytes(8, 8, 65) == 0            # capacity above O*I
    a = mst.mst_layer_device_bytes(768, 768, 1000)
    b = mst.mst_layer_device_bytes(768, 768, 100000)
    assert 0 < a < b
    assert mst.mst_workspace_bytes(768, 768, 1000, 128) < mst.mst_workspace_bytes(768, 768, 1000, 8192)
    with pytest.raises(mst.MstError):
        mst.mst_update_counts(10, 11, 0.5, 0.3, 0.25)
    with pytest.raises(mst.MstError):
        mst.mst_update_counts(10, 5, 1.5, 0.3, 0.25)
    # null handles / pointers are rejected on the host before anything touches a GPU
    L = mst.lib()
    assert L.mst_sparse_fc_fwd(None, None, None, 4, 0, None) == -1
    assert L.mst_layer_load_dense(None, None, None, None, 0, None) == -1
    assert L.mst_mask_update(None, None, None, 4, 0, 0.1, 0.3, 0.25, 1, None, 0, None, None) == -1
    assert L.mst_sparse_fc_bwd(None, None, None, None, None, 4, 0, None, 0, None) == -1
    assert L.mst_sparse_fc_bwd_weight_update(None, None, None, None, 4, 0, 0.1, 0.3, 0.25, 1, None, 0, None, None) == -1
    assert L.mst_strided_attention_mask(None, 8, 4, None) == -1
    assert L.mst_layer_set_prune_lambda(None, 0.5) == -1
    assert L.mst_bwd_force_shape(8, 2) == -1 and L.mst_bwd_force_shape(16, 3) == -1 and L.mst_bwd_force_shape(0, 0) == 0
    assert L.mst_spmm_force_shape(128, 6) == -1 and L.mst_spmm_force_shape(0, 0) == 0
    assert L.mst_heavy_rows(3) == -1 and L.mst_heavy_rows(-1) == -1 and L.mst_heavy_rows(2) == 0 and L.mst_heavy_rows(1) == 0
    # the several-layer update: a negative count or missing arrays; an empty set of layers is fine
    assert L.mst_mask_update_from_scores_multi(-1, None, None, None, 0.3, 0.25, None, None, None, None, None) == -1
    assert L.mst_mask_update_from_scores_multi(2, None, None, None, 0.3, 0.25, None, None, None, None, None) == -1
    assert L.mst_mask_update_from_scores_multi(0, None, None, None, 0.3, 0.25, None, None, None, None, None) == 0


def test_product_package_never_imports_the_oracle():
    import subprocess
    import sys
    code = ("import sys; sys.path.insert(0, %r); import paper_2408_11746_amd as m; m.lib(); "
            "bad = [k for k in sys.modules if k == 'oracle' or k.startswith('oracle.')]; "
            "assert not bad, bad; print('clean')" % ROOT)
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True)
    assert out.returncode == 0 and "clean" in out.stdout, out.stderr
    for name in ("binding.py", "build.py", "__init__.py"):
        src = open(os.path.join(ROOT, "paper_2408_11746_amd", name)).read()
        assert "oracle" not in src


def test_calls_on_a_layer_that_was_never_loaded_return_state_error():
    """mst_layer_create does no device work and the caller's buffer is uninitialised: until
    mst_layer_load_dense has succeeded, every call that would read the layer's device arrays
    must refuse on the host (MST_ERR_STATE) before anything is launched.  No GPU is needed:
    the pointers are never dereferenced."""
    import ctypes as C
    L = mst.lib()
    O, I, cap, T = 64, 96, 512, 32
    nbytes = mst.mst_layer_device_bytes(O, I, cap)
    wsb = mst.mst_workspace_bytes(O, I, cap, T)
    assert nbytes > 0 and wsb > 0
    fake = 0x10000                      # non-null, 16-byte aligned, never touched
    h = C.c_void_p()
    assert L.mst_layer_create(C.byref(h), O, I, cap, fake, nbytes) == 0
    try:
        st = binding.UpdateStats()
        assert L.mst_layer_nnz(h) == 0
        assert L.mst_sparse_fc_fwd(h, fake, fake, T, 0, None) == -4
        assert L.mst_sparse_fc_bwd_input(h, fake, fake, T, 0, None) == -4
        assert L.mst_sparse_fc_bwd_weight(h, fake, fake, fake, T, 0, fake, wsb, None) == -4
        assert L.mst_sparse_fc_bwd(h, fake, fake, fake, fake, T, 0, fake, wsb, None) == -4
        assert L.mst_mask_update_from_scores(h, fake, 0.1, 0.3, 0.25, 1, fake, wsb, C.byref(st), None) == -4
        assert L.mst_mask_update(h, fake, fake, T, 0, 0.1, 0.3, 0.25, 1, fake, wsb, C.byref(st), None) == -4
        assert L.mst_sparse_fc_bwd_weight_update(h, fake, fake, fake, T, 0, 0.1, 0.3, 0.25, 1, fake, wsb,
                                                 C.byref(st), None) == -4
        assert L.mst_layer_export_dense(h, fake, fake, None) == -4
        assert L.mst_layer_sync_values(h, None) == -4
        assert L.mst_layer_indices(h, fake, None) == -4
        p, n = C.c_void_p(), C.c_int64()
        assert L.mst_layer_values(h, C.byref(p), C.byref(n)) == -4
        # argument errors still come first
        assert L.mst_sparse_fc_fwd(h, None, fake, T, 0, None) == -1
    finally:
        L.mst_layer_destroy(h)
