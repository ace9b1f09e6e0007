"""Pins of the oracle's second solver: the paper's own choice (Section 3.1), a non-smooth Newton
method whose every iteration is solved by a Krylov method, here preconditioned conjugate
residuals with a fixed iteration count.  Same rows, biases and friction coefficient as the
block-Jacobi solver, so both have to meet at the same solution where that solution is unique, and
the Newton solver has to obey the same closed forms (Section 3.1: restitution 0, mu = 1,
speculative contacts)."""
import numpy as np
import pytest

import oracle
import scenes
from helpers import angular_momentum, free_params, linear_momentum, single_scene

G = 9.81
SOLVE_ONLY = oracle.PH_CONTACTS | oracle.PH_SOLVE


def newton(krylov=8, **kw):
    p = free_params(**kw)
    p.solver, p.krylov_iters, p.newton_reg = 1, krylov, 0.0     # (undamped Newton steps: the closed forms are met exactly)
    return p


def test_hanging_chain_carries_its_weight_without_sag_where_jacobi_stretches():
    """Eight links hanging from the world at rest.  20 Jacobi sweeps per substep leave part of the
    weight unsupported every substep, and the feedback term holds the chain at a stretched
    equilibrium (millimetres); two Newton iterations of 16 inner iterations solve the 48 rows of the
    chain exactly (a Krylov method is exact after as many iterations as the operator has distinct
    eigenvalues), so nothing moves at all."""
    rob = scenes.make_chain(n_links=8, seg_len=0.3, mass=0.5)
    z_rest = scenes.rest_state(rob, 1)[0, -1, 2]
    sag = {}
    for name, p, its in (("jacobi", free_params(contacts=0), 20), ("newton", newton(16, contacts=0), 2)):
        o = oracle.OracleSim(single_scene(rob, params=p))
        o.set_state(scenes.rest_state(rob, 1))
        for _ in range(240):
            o.step(None, 1 / 60, 4, its)
        sag[name] = z_rest - o.get_state()[0, -1, 2]
        if name == "newton":
            assert np.abs(o.get_state()[0, :, 7:13]).max() < 1e-12
    assert sag["jacobi"] > 2e-3
    assert abs(sag["newton"]) < 1e-10


def test_newton_iterate_reaches_the_fixed_point_of_the_jacobi_sweeps():
    """A swinging chain (bilateral rows only: one solution): the velocities after one substep of
    three Newton iterations equal those after 200000 Jacobi sweeps, and the joint residual of the last
    Newton iterate is at rounding level."""
    rob = scenes.make_chain(n_links=4)
    st = scenes.rest_state(rob, 1)
    rng = np.random.default_rng(2)
    st[0, :, 7:13] = rng.uniform(-1, 1, (4, 6))
    out = {}
    for name, p, its in (("jacobi", free_params(contacts=0), 200000), ("newton", newton(30, contacts=0), 3)):
        o = oracle.OracleSim(single_scene(rob, params=p))
        o.set_state(st)
        o.start_trace(0, 8192)
        o.substep_phases(None, 1 / 240, its, oracle.PH_FORCES | oracle.PH_SOLVE)
        out[name] = o.get_state()[0, :, 7:13].copy()
        if name == "newton":
            tr = o.trace()
            assert len(tr) == 3 and tr["bilateral_max"][0] > 0.1 and tr["bilateral_max"][-1] < 1e-10
    np.testing.assert_allclose(out["newton"], out["jacobi"], atol=1e-8)


def test_resting_sphere_gets_m_g_h_and_a_dropped_one_does_not_rebound():
    rob = scenes.make_single(radius=0.1, pos=(0.0, 0.0, 0.3), mass=2.0)
    o = oracle.OracleSim(single_scene(rob, params=newton(8)))
    o.set_state(scenes.rest_state(rob, 1))
    touched, vz = False, []
    for _ in range(120):
        o.step(None, 1 / 60, 2, 3)
        c = o.get_contacts()[0, 0]
        touched |= bool(c["active"] and c["d"] <= 1e-4)
        if touched:
            vz.append(o.get_state()[0, 0, 9])
    assert touched and max(vz) < 1e-9
    o.start_trace(0, 64)
    o.step(None, 1 / 60, 1, 3)
    # (the trace records the iterate at the start of every Newton iteration: the last record is the
    #  iterate the third iteration starts from)
    assert o.trace()["sum_lambda_n"][-1] == pytest.approx(2.0 * G / 60, rel=1e-9)
    assert o.get_state()[0, 0, 2] == pytest.approx(0.1, abs=1e-6)


@pytest.mark.parametrize("depth,v_expected", [(0.005, 0.24), (0.050, 2.0)])
def test_penetration_bias_and_its_cap_are_the_same_rows_as_for_jacobi(depth, v_expected):
    r, h = 0.1, 1.0 / 240.0
    sc = single_scene(scenes.make_single(radius=r, pos=(0.0, 0.0, r - depth)), params=newton(8, gravity=(0.0, 0.0, 0.0)))
    o = oracle.OracleSim(sc)
    o.set_state(scenes.rest_state(sc.robot, 1))
    o.substep_phases(None, h, 2, SOLVE_ONLY)
    assert o.get_state()[0, 0, 9] == pytest.approx(v_expected, rel=1e-12)


def test_closing_speculative_contact_leaves_gap_over_h():
    h, r, d = 1.0 / 120.0, 0.1, 0.010
    sc = single_scene(scenes.make_single(radius=r, pos=(0.0, 0.0, r + d)), params=newton(8, gravity=(0.0, 0.0, 0.0)))
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(sc.robot, 1)
    st[0, 0, 9] = -2.0
    o.set_state(st)
    o.step(None, h, 1, 2)
    assert o.get_state()[0, 0, 9] == pytest.approx(-d / h, rel=1e-12)


def _lying_capsule(params, v0=0.0):
    rob = scenes.make_single(radius=0.05, seg_len=0.4, axis=0, pos=(0, 0, 0.05), mass=1.0)
    o = oracle.OracleSim(single_scene(rob, params=params))
    st = scenes.rest_state(rob)
    st[0, 0, 7] = v0
    o.set_state(st)
    return rob, o


def test_sliding_capsule_decelerates_at_mu_g_then_stays():
    """Smooth isotropic Coulomb friction (Section 3.1) with mu = 1: while it slides at more than a
    few mm/s the friction force is mu m g to within the smoothing (|v| / sqrt(v^2 + eps^2), eps =
    1 mm/s); once stopped it creeps at less than eps."""
    rob, o = _lying_capsule(newton(24), v0=2.0)
    dt, vs = 1 / 60, []
    for _ in range(24):
        o.step(None, dt, 4, 6)
        vs.append(o.get_state()[0, 0, 7])
    vs = np.array(vs)
    assert vs[5] == pytest.approx(2.0 - G * 6 * dt, rel=2e-5)
    assert abs(vs[-1]) < 1e-3 and abs(o.get_state()[0, 0, 10:13]).max() < 1e-6
    assert o.get_state()[0, 0, 2] == pytest.approx(0.05, abs=1e-9)


@pytest.mark.parametrize("deg,sticks", [(35.0, True), (55.0, False)])
def test_tilted_gravity_sticks_iff_tan_theta_below_mu(deg, sticks):
    th = np.radians(deg)
    rob, o = _lying_capsule(newton(24, gravity=(G * np.sin(th), 0.0, -G * np.cos(th))))
    for _ in range(60):
        o.step(None, 1 / 60, 4, 6)
    s = o.get_state()[0, 0]
    if sticks:
        # held, up to the creep of the smoothed law (of the order of its eps = 1 mm/s)
        assert abs(s[7]) < 4e-3 and abs(s[0]) < 4e-3
    else:
        assert s[7] == pytest.approx(G * (np.sin(th) - np.cos(th)), rel=0.01)


def test_hinge_driven_by_constant_torque_stops_at_its_limit():
    rob = scenes.make_chain(n_links=1, seg_len=0.4, mass=1.0, lo=-0.5, hi=0.8, gear=2.0)
    o = oracle.OracleSim(single_scene(rob, params=newton(12, contacts=0, gravity=(0, 0, 0))))
    o.set_state(scenes.rest_state(rob))
    for _ in range(120):
        o.step(np.array([[1.0]]), 1 / 60, 4, 3)
    assert 0.8 - 1e-6 < o.joint_angles()[0, 0, 0] < 0.8 + 1e-3
    assert abs(o.get_obs()[0][0, 11 + 1]) < 1e-6
    for _ in range(120):
        o.step(np.array([[-1.0]]), 1 / 60, 4, 3)
    assert -0.5 - 1e-3 < o.joint_angles()[0, 0, 0] < -0.5 + 1e-6


def _humanoid_free(gyro=1):
    rob = scenes.make_humanoid()
    sc = single_scene(rob, params=newton(8, contacts=0, gravity=(0, 0, 0), gyroscopic=gyro))
    o = oracle.OracleSim(sc)
    o.reset(3)
    return rob, o


def test_momenta_are_conserved_by_the_newton_solve():
    """Every impulse acts with equal and opposite sign at one shared point, whatever the inner
    solve returns: linear momentum over whole steps, angular momentum exactly at fixed pose."""
    rob, o = _humanoid_free()
    p0 = linear_momentum(rob, o.get_state()[0])
    for k in range(20):
        o.step(0.2 * scenes.actions_for_step(11, k, 1, rob.n_dofs), 1 / 60, 4, 3)
    scale = (rob.mass[:, None] * np.abs(o.get_state()[0][:, 7:10])).sum()
    assert scale > 1.0
    np.testing.assert_allclose(linear_momentum(rob, o.get_state()[0]), p0, atol=1e-11 * scale)
    rob, o = _humanoid_free(gyro=0)
    for k in range(5):
        o.step(0.2 * scenes.actions_for_step(5, k, 1, rob.n_dofs), 1 / 60, 2, 3)
    L0 = angular_momentum(rob, o.get_state()[0])
    o.substep_phases(0.2 * scenes.actions_for_step(5, 99, 1, rob.n_dofs), 1 / 240, 3, oracle.PH_FORCES | oracle.PH_SOLVE)
    np.testing.assert_allclose(angular_momentum(rob, o.get_state()[0]), L0, atol=1e-11 * (np.abs(L0).max() + 1.0))


def test_standing_humanoid_joints_hold_better_than_with_jacobi_and_runs_stay_finite():
    """Humanoids dropped from the reset pose with small random torques (5 % of the benchmark's):
    until they have landed and settled, the joints' anchor points separate by millimetres under 20
    Jacobi sweeps and by a fraction of that under 3 x 8 Newton / Krylov iterations.  (At the
    benchmark's full +-100 N m the limbs spin at the 64 rad/s cap and both solvers show
    centimetres: there the anchor error is the second-order term of the rotation update, r (w h)^2
    / 2 = 7 mm per substep for a 0.2 m limb, which no velocity-level solve removes.)"""
    sep = {}
    for name, solver, its in (("jacobi", 0, 20), ("newton", 1, 3)):
        sc, cfg = scenes.config_scene(2, num_envs=16)
        sc.params.solver, sc.params.krylov_iters = solver, 8
        o = oracle.OracleSim(sc, threads=8)
        o.reset(cfg["seed"])
        e = []
        for s in range(150):
            o.start_trace(env=s % 16, cap=4096)
            o.step(0.05 * scenes.actions_for_step(cfg["seed"], s, 16, 21), cfg["dt"], 4, its)
            e.append(o.trace()["pos_err_max"].max())
        assert np.isfinite(o.get_state()).all()
        sep[name] = np.median(e[100:])
    assert sep["jacobi"] > 2e-3 and sep["newton"] < 0.6 * sep["jacobi"]


def test_envs_are_independent_and_deterministic_under_the_newton_solver():
    sc, cfg = scenes.config_scene(3, num_envs=6)
    sc.params.solver, sc.params.krylov_iters = 1, 8
    outs = []
    for threads in (1, 4):
        o = oracle.OracleSim(sc, threads=threads)
        o.reset(cfg["seed"])
        for s in range(40):
            o.step(scenes.actions_for_step(cfg["seed"], s, 6, 21), cfg["dt"], 4, 3)
        outs.append(o.get_state())
    assert np.array_equal(outs[0], outs[1]) and np.isfinite(outs[0]).all()
    one = scenes.config_scene(3, num_envs=6)[0]
    one.params.solver, one.params.krylov_iters = 1, 8
    one.num_envs, one.env_origins = 1, sc.env_origins[4:5].copy()
    o = oracle.OracleSim(one)
    full = oracle.OracleSim(sc); full.reset(cfg["seed"])
    o.set_state(full.get_state()[4:5])
    for s in range(40):
        o.step(scenes.actions_for_step(cfg["seed"], s, 6, 21)[4:5], cfg["dt"], 4, 3)
    assert np.array_equal(o.get_state()[0], outs[0][4])


def _one_substep(rob, p, state, its, warm_from=None, share=1.0, dt=1 / 240):
    """Velocities and kept impulses after one substep from `state`; with warm_from = (lam_j, lam_s)
    the rows start from `share` of those impulses."""
    o = oracle.OracleSim(single_scene(rob, params=p))
    o.set_state(state)
    if warm_from is not None:
        o.set_warm_start(share)
        o.set_warm(*warm_from)
        o.set_warm_flags(-np.ones((1, o.J, 3), np.int32), np.ones((1, o.S), np.int32))
    o.substep_phases(None, dt, its, oracle.PH_ALL)
    return o.get_state()[0, :, 7:13].copy(), o.get_warm()


def test_newton_warm_start_is_the_first_iterate_chain():
    """The kept impulses times the share are the Newton method's first iterate (the paper names no
    starting point; zero is the other choice).  A swinging chain has one solution: started from that
    solution's own impulses a single Newton iteration with a single inner iteration - which from zero
    is far from solved - finds nothing left to do and returns the solved velocities; started from
    half of them it does not."""
    rob = scenes.make_chain(n_links=4)
    st = scenes.rest_state(rob, 1)
    st[0, :, 7:13] = np.random.default_rng(5).uniform(-1, 1, (4, 6))
    solved, kept = _one_substep(rob, newton(30, contacts=0), st, 3)
    weak = newton(1, contacts=0)
    cold, _ = _one_substep(rob, weak, st, 1)
    warm, kept_again = _one_substep(rob, weak, st, 1, warm_from=kept)
    half, _ = _one_substep(rob, weak, st, 1, warm_from=kept, share=0.5)
    assert np.abs(cold - solved).max() > 1e-2
    np.testing.assert_allclose(warm, solved, atol=1e-9)
    np.testing.assert_allclose(kept_again[0], kept[0], atol=1e-9)
    assert np.abs(half - solved).max() > 1e-3


def test_newton_warm_start_is_the_first_iterate_contact_with_friction():
    """The same for a capsule held on a tilted plane by friction (normal and both friction rows
    carry impulses): from the solved impulses one weak iteration stays at the solution."""
    th = np.radians(35.0)
    p = newton(24, gravity=(G * np.sin(th), 0.0, -G * np.cos(th)))
    rob, o = _lying_capsule(p)
    for _ in range(30):
        o.step(None, 1 / 60, 4, 6)
    st = o.get_state()
    solved, kept = _one_substep(rob, p, st, 60)      # (the friction law's compliance settles slowly)
    assert np.abs(kept[1][0, :, 0]).max() > 1e-3 and np.abs(kept[1][0, :, 1:]).max() > 1e-4    # normal and friction impulses
    weak = newton(1, gravity=(G * np.sin(th), 0.0, -G * np.cos(th)))
    cold, _ = _one_substep(rob, weak, st, 1)
    warm, _ = _one_substep(rob, weak, st, 1, warm_from=kept)
    assert np.abs(cold - solved).max() > 1e-3
    np.testing.assert_allclose(warm, solved, atol=1e-9)
