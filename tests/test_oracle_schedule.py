"""Pins for oracle.schedule (Sec. 3.1 cubic schedules, Sec. 3.2 piecewise cosine)."""
import math

import pytest

from oracle import schedule as sc


def test_stage_values_match_hand_computed_table(golden):
    cfg = sc.ScheduleCfg()
    for phase, k, step, d in golden("sv_stage_densities.txt"):
        if phase == "mean":
            continue
        assert sc.density(cfg, int(step)) == pytest.approx(float(d), abs=1e-12), (phase, k, step)


def test_step_average_density(golden):
    cfg = sc.ScheduleCfg()
    want = [float(r[3]) for r in golden("sv_stage_densities.txt") if r[0] == "mean"][0]
    got = sum(sc.density(cfg, t) for t in range(0, 140000, 1)) / 140000
    assert got == pytest.approx(want, abs=1e-12)
    assert want == pytest.approx(34400 / 140000, abs=1e-15)


def test_end_points_and_phase_lengths():
    cfg = sc.ScheduleCfg()
    assert cfg.T_W == 10000 and cfg.T_R == 10000          # T_W = N * Delta_W as stated
    assert sc.density(cfg, 0) == 1.0                        # starts dense
    assert sc.density(cfg, cfg.T_W) == pytest.approx(0.04, abs=1e-15)
    assert sc.density(cfg, cfg.T_W + cfg.T_U - 1) == pytest.approx(0.04, abs=1e-15)
    assert sc.density(cfg, cfg.T_W + cfg.T_U + cfg.T_R) == 1.0
    assert sc.density(cfg, 10 ** 7) == 1.0


@pytest.mark.parametrize("N,dw,dr,tu,sm", [(5, 2000, 2000, 100000, 0.96), (4, 10, 7, 33, 0.9), (1, 5, 5, 0, 0.5)])
def test_stagewise_monotone_with_N_stages(N, dw, dr, tu, sm):
    cfg = sc.ScheduleCfg(S_M=sm, N=N, Delta_W=dw, T_U=tu, Delta_R=dr, zeta=[0.3] * (N + 1))
    warm = [sc.density(cfg, t) for t in range(cfg.T_W)]
    rest = [sc.density(cfg, cfg.T_W + cfg.T_U + t) for t in range(cfg.T_R)]
    assert all(a >= b for a, b in zip(warm, warm[1:]))      # dense -> sparse
    assert all(a <= b for a, b in zip(rest, rest[1:]))      # sparse -> dense
    assert len(set(warm)) == N and len(set(rest)) == N      # N stages, constant within a stage
    for k in range(N):
        assert len(set(warm[k * dw:(k + 1) * dw])) == 1
        assert len(set(rest[k * dr:(k + 1) * dr])) == 1
    # "symmetric to the warm-up": restoration stage k mirrors warm-up stage k about (1 + d_min)/2
    for k in range(N):
        assert warm[k * dw] + rest[k * dr] == pytest.approx(1.0 + (1.0 - sm), abs=1e-12)


def test_cubic_shape_not_linear_or_quadratic():
    # (1 - k/N)^3 with N = 2: middle stage must be d_min + (1-d_min)/8
    cfg = sc.ScheduleCfg(S_M=0.8, N=2, Delta_W=10, T_U=10, Delta_R=10, zeta=[0.3] * 3)
    assert sc.density(cfg, 10) == pytest.approx(0.2 + 0.8 / 8, abs=1e-15)
    assert sc.density(cfg, 30 + 10) == pytest.approx(1.0 - 0.8 / 8, abs=1e-15)


def test_zeta_boundaries_and_cosine():
    cfg = sc.ScheduleCfg()
    b = sc.zeta_boundaries(cfg)
    assert b == [0, 110000, 112000, 114000, 116000, 118000, 120000]   # T_0 .. T_{N+1}
    for i in range(1, len(b)):
        lo, hi = b[i - 1], b[i]
        assert sc.zeta(cfg, lo) == pytest.approx(0.3, abs=1e-15)      # restarts at zeta_i
        assert sc.zeta(cfg, (lo + hi) // 2) == pytest.approx(0.15, abs=1e-12)   # cos(pi/2) = 0
        assert sc.zeta(cfg, hi - 1) < 1e-6 * 0.3 * (110000 / (hi - lo)) ** 2 + 1e-6
        q = lo + (hi - lo) // 4                                         # quarter point: (1 + cos(pi/4))/2
        assert sc.zeta(cfg, q) == pytest.approx(0.15 * (1 + math.sqrt(0.5)), abs=1e-12)
    assert sc.zeta(cfg, 120000) == 0.0 and sc.zeta(cfg, 139999) == 0.0


def test_zeta_decaying_magnitudes_and_monotone_within_period():
    mags = [0.3, 0.25, 0.2, 0.15, 0.1, 0.05]
    cfg = sc.ScheduleCfg(zeta=mags)
    b = sc.zeta_boundaries(cfg)
    for i in range(1, len(b)):
        assert sc.zeta(cfg, b[i - 1]) == pytest.approx(mags[i - 1], abs=1e-15)
        vals = [sc.zeta(cfg, t) for t in range(b[i - 1], b[i], max(1, (b[i] - b[i - 1]) // 50))]
        assert all(x > y for x, y in zip(vals, vals[1:]))
        assert all(0.0 <= v <= mags[i - 1] for v in vals)


def test_bad_arguments():
    cfg = sc.ScheduleCfg()
    with pytest.raises(ValueError):
        sc.density(cfg, -1)
    with pytest.raises(ValueError):
        sc.zeta(sc.ScheduleCfg(zeta=[0.3]), 5)
