"""Pins for the CPU oracle's dynamics: closed forms and invariants that hold
whatever the implementation looks like (Section 3.1 constants: gravity, mu = 1,
restitution 0, velocity-level implicit stepping)."""
import numpy as np
import pytest

import oracle
import scenes
from helpers import (angular_momentum, free_params, linear_momentum, single_scene)

G = 9.81


def test_free_fall_matches_discrete_closed_form():
    # semi-implicit Euler: v_n = v_0 - g h n ; z_n = z_0 + n h v_0 - g h^2 n(n+1)/2
    rob = scenes.make_single(radius=0.05, seg_len=0.2, axis=0, pos=(0.0, 0.0, 50.0))
    sc = single_scene(rob, params=free_params(contacts=0))
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(rob)
    st[0, 0, 7:10] = (1.5, -0.5, 3.0)
    o.set_state(st)
    dt, sub, n_steps = 1.0 / 60.0, 4, 25
    for _ in range(n_steps):
        o.step(None, dt, sub, 3)
    h, n = dt / sub, sub * n_steps
    s = o.get_state()[0, 0]
    assert s[9] == pytest.approx(3.0 - G * h * n, abs=1e-12)
    assert s[2] == pytest.approx(50.0 + n * h * 3.0 - 0.5 * G * h * h * n * (n + 1), abs=1e-11)
    assert s[0] == pytest.approx(n * h * 1.5, abs=1e-12)
    assert s[1] == pytest.approx(-n * h * 0.5, abs=1e-12)
    # and the continuous parabola is approached at first order in h
    t = n * h
    assert abs(s[2] - (50.0 + 3.0 * t - 0.5 * G * t * t)) < 0.6 * G * h * t


def test_spin_about_symmetry_axis_is_steady_and_quaternion_stays_unit():
    rob = scenes.make_single(radius=0.05, seg_len=0.3, axis=2, pos=(0, 0, 5.0))
    sc = single_scene(rob, params=free_params(contacts=0, gravity=(0, 0, 0)))
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(rob)
    st[0, 0, 10:13] = (0, 0, 7.0)
    o.set_state(st)
    for _ in range(50):
        o.step(None, 1 / 60, 2, 1)
    s = o.get_state()[0, 0]
    np.testing.assert_allclose(s[10:13], (0, 0, 7.0), atol=1e-12)
    assert np.linalg.norm(s[3:7]) == pytest.approx(1.0, abs=1e-14)
    # rotated about z only: x,y components of the quaternion stay zero
    assert abs(s[4]) < 1e-14 and abs(s[5]) < 1e-14


def _humanoid_free(gyro=1, N=1):
    rob = scenes.make_humanoid()
    sc = single_scene(rob, params=free_params(contacts=0, gravity=(0, 0, 0), gyroscopic=gyro),
                      num_envs=N)
    o = oracle.OracleSim(sc)
    o.reset(3)
    return rob, sc, o


def test_internal_torques_and_solver_conserve_linear_momentum():
    rob, sc, o = _humanoid_free()
    p0 = linear_momentum(rob, o.get_state()[0])
    for k in range(20):
        a = scenes.actions_for_step(11, k, 1, rob.n_dofs)
        o.step(a, 1 / 60, 4, 10)
    p1 = linear_momentum(rob, o.get_state()[0])
    scale = (rob.mass[:, None] * np.abs(o.get_state()[0][:, 7:10])).sum()
    assert scale > 1.0      # the robot is actually flailing
    np.testing.assert_allclose(p1, p0, atol=1e-11 * scale)


def test_torques_and_solver_conserve_angular_momentum_exactly_at_fixed_pose():
    # forces + solve phases only (positions frozen), gyroscopic term off: joint
    # torques are equal and opposite and solver impulses act at one shared point
    rob, sc, o = _humanoid_free(gyro=0)
    for k in range(5):          # get into a generic moving configuration first
        o.step(scenes.actions_for_step(5, k, 1, rob.n_dofs), 1 / 60, 2, 5)
    L0 = angular_momentum(rob, o.get_state()[0])
    a = scenes.actions_for_step(5, 99, 1, rob.n_dofs)
    o.substep_phases(a, 1 / 240, 25, oracle.PH_FORCES | oracle.PH_SOLVE)
    L1 = angular_momentum(rob, o.get_state()[0])
    scale = np.abs(L0).max() + 1.0
    np.testing.assert_allclose(L1, L0, atol=1e-11 * scale)


def test_angular_momentum_drift_over_whole_steps_is_first_order_in_h():
    def drift(sub):
        rob, sc, o = _humanoid_free(gyro=1)
        st = o.get_state()
        rng = np.random.default_rng(0)
        st[0, :, 10:13] = rng.uniform(-3, 3, (rob.n_bodies, 3))   # tumbling start, no torques
        o.set_state(st)
        o.substep_phases(None, 1e-9, 200, oracle.PH_SOLVE)        # make joint velocities consistent
        L0 = angular_momentum(rob, o.get_state()[0])
        for _ in range(30):
            o.step(None, 1 / 60, sub, 40)
        return np.linalg.norm(angular_momentum(rob, o.get_state()[0]) - L0), np.linalg.norm(L0)
    d1, n0 = drift(4)
    d2, _ = drift(8)
    assert n0 > 0.5
    assert d1 < 0.2 * n0
    assert 1.5 < d1 / d2 < 2.7


def test_free_asymmetric_body_needs_the_gyroscopic_term():
    # a tumbling capsule: |L| stays put to first order with the gyroscopic term
    # and drifts at zeroth order without it
    def run(gyro, sub):
        rob = scenes.make_single(radius=0.05, seg_len=0.5, axis=0, pos=(0, 0, 5.0))
        sc = single_scene(rob, params=free_params(contacts=0, gravity=(0, 0, 0), gyroscopic=gyro))
        o = oracle.OracleSim(sc)
        st = scenes.rest_state(rob)
        st[0, 0, 10:13] = (4.0, 3.0, 0.0)
        o.set_state(st)
        L0 = angular_momentum(rob, o.get_state()[0])
        for _ in range(60):
            o.step(None, 1 / 60, sub, 1)
        return np.linalg.norm(angular_momentum(rob, o.get_state()[0]) - L0) / np.linalg.norm(L0)
    assert run(1, 4) < 0.05
    assert 1.5 < run(1, 4) / run(1, 8) < 2.7
    assert run(0, 4) > 0.5


def test_joint_residual_decays_monotonically_on_resting_chain_and_vanishes():
    rob = scenes.make_chain(n_links=4)
    sc = single_scene(rob, params=free_params(contacts=0))
    o = oracle.OracleSim(sc)
    o.set_state(scenes.rest_state(rob))
    o.start_trace(0, 4096)
    o.step(None, 1 / 60, 1, 80)
    tr = o.trace()
    rms = tr["bilateral_rms"]
    assert len(rms) == 80 and rms[0] > 1e-3
    assert np.all(np.diff(rms) <= 1e-15)
    assert rms[-1] < 0.05 * rms[0]
    o.set_state(scenes.rest_state(rob))
    o.start_trace(0, 4096)
    o.step(None, 1 / 60, 1, 3000)
    assert o.trace()["bilateral_max"][-1] < 1e-12
    # a resting chain with converged joints does not move
    s = o.get_state()[0]
    assert np.abs(s[:, 7:13]).max() < 1e-10


def test_single_hinge_small_angle_period():
    L, m, r = 0.5, 0.8, 0.03
    rob = scenes.make_chain(n_links=1, seg_len=L, radius=r, mass=m, top=(0, 0, 2.0))
    _, i_ax, i_tr = scenes.capsule_mass_inertia(r, L, mass=m)
    lc = L / 2
    T_exact = 2 * np.pi * np.sqrt((i_tr + m * lc * lc) / (m * G * lc))
    sc = single_scene(rob, params=free_params(contacts=0))
    th0 = 0.05
    periods = []
    for sub in (8, 16):
        o = oracle.OracleSim(sc)
        ang = np.zeros((1, 3)); ang[0, 0] = th0
        st = scenes.posed_state(rob, rob.rest_pos[0], np.array([1.0, 0, 0, 0]), ang)[None]
        o.set_state(st)
        h = 1 / 60 / sub
        th, t = [], []
        for k in range(int(2.2 * T_exact * 60)):
            o.step(None, 1 / 60, sub, 30)
            th.append(o.joint_angles()[0, 0, 0]); t.append((k + 1) / 60)
        th, t = np.array(th), np.array(t)
        # downward zero crossings, linearly interpolated
        idx = np.where((th[:-1] > 0) & (th[1:] <= 0))[0]
        tc = t[idx] + (t[idx + 1] - t[idx]) * th[idx] / (th[idx] - th[idx + 1])
        assert len(tc) >= 2
        periods.append(tc[1] - tc[0])
    assert periods[1] == pytest.approx(T_exact, rel=0.02)
    assert abs(periods[1] - T_exact) <= abs(periods[0] - T_exact) + 1e-4


def _settle_sphere(iters=30, steps=90, mu=1.0):
    rob = scenes.make_single(radius=0.1, seg_len=0.0, pos=(0, 0, 0.3), mass=2.0)
    sc = single_scene(rob, params=free_params(mu=mu))
    o = oracle.OracleSim(sc)
    o.set_state(scenes.rest_state(rob))
    return rob, o


def test_resting_sphere_normal_impulse_balances_gravity_and_no_rebound():
    rob, o = _settle_sphere()
    dt, sub = 1 / 60, 2
    vz_after_touch, touched = [], False
    for _ in range(120):
        o.step(None, dt, sub, 30)
        s = o.get_state()[0, 0]
        if o.get_contacts()[0, 0]["d"] <= 1e-4 and o.get_contacts()[0, 0]["active"]:
            touched = True
        if touched:
            vz_after_touch.append(s[9])
    assert touched
    assert max(vz_after_touch) < 1e-6          # restitution 0: never moves up again
    o.start_trace(0, 64)
    o.step(None, dt, 1, 30)
    tr = o.trace()
    assert tr["sum_lambda_n"][-1] == pytest.approx(2.0 * G * dt, rel=1e-6)
    z = o.get_state()[0, 0, 2]
    assert 0.1 - 1e-3 < z < 0.1 + 1e-6          # rests on the surface


def _lying_capsule(params, v0=0.0):
    rob = scenes.make_single(radius=0.05, seg_len=0.4, axis=0, pos=(0, 0, 0.05), mass=1.0)
    sc = single_scene(rob, params=params)
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(rob)
    st[0, 0, 7] = v0
    o.set_state(st)
    return rob, o


def test_sliding_capsule_decelerates_at_mu_g_and_friction_stays_in_cone():
    rob, o = _lying_capsule(free_params(), v0=2.0)
    o.start_trace(0, 100000)
    dt, vs = 1 / 60, []
    for _ in range(24):
        o.step(None, dt, 4, 40)
        vs.append(o.get_state()[0, 0, 7])
    vs = np.array(vs)
    t = dt * np.arange(1, len(vs) + 1)
    sliding = vs > 0.3
    slope = np.polyfit(t[sliding], vs[sliding], 1)[0]
    assert slope == pytest.approx(-1.0 * G, rel=0.03)
    assert abs(vs[-1]) < 1e-3                     # at rest after v0/(mu g) = 0.2 s
    assert o.trace()["cone_excess"].max() <= 1e-12


@pytest.mark.parametrize("deg,sticks", [(35.0, True), (55.0, False)])
def test_tilted_gravity_sticks_iff_tan_theta_below_mu(deg, sticks):
    th = np.radians(deg)
    g = (G * np.sin(th), 0.0, -G * np.cos(th))
    rob, o = _lying_capsule(free_params(gravity=g))
    for _ in range(60):
        o.step(None, 1 / 60, 4, 60)
    s = o.get_state()[0, 0]
    if sticks:
        assert abs(s[0]) < 5e-3 and abs(s[7]) < 1e-2
    else:
        a = G * (np.sin(th) - 1.0 * np.cos(th))
        assert s[7] == pytest.approx(a * 1.0, rel=0.05)


def test_hinge_driven_by_constant_torque_stops_at_its_limit():
    rob = scenes.make_chain(n_links=1, seg_len=0.4, mass=1.0, lo=-0.5, hi=0.8, gear=2.0)
    sc = single_scene(rob, params=free_params(contacts=0, gravity=(0, 0, 0)))
    o = oracle.OracleSim(sc)
    o.set_state(scenes.rest_state(rob))
    for _ in range(120):
        o.step(np.array([[1.0]]), 1 / 60, 4, 30)
    th = o.joint_angles()[0, 0, 0]
    assert 0.8 - 1e-3 < th < 0.8 + 0.03
    rate = o.get_obs()[0][0, 11 + 1]
    assert abs(rate) < 1e-2
    for _ in range(120):
        o.step(np.array([[-1.0]]), 1 / 60, 4, 30)
    assert -0.5 - 0.03 < o.joint_angles()[0, 0, 0] < -0.5 + 1e-3


def test_envs_are_independent_permutable_and_deterministic():
    sc8, cfg = scenes.config_scene(3, num_envs=8)
    o8 = oracle.OracleSim(sc8, threads=4)
    o8.reset(9)
    s0 = o8.get_state()
    acts = [scenes.actions_for_step(1, k, 8, sc8.robot.n_dofs) for k in range(6)]
    for a in acts:
        o8.step(a, cfg["dt"], cfg["substeps"], cfg["iterations"])
    ref = o8.get_state()
    # env 5 alone
    sc1, _ = scenes.config_scene(3, num_envs=8)
    sc1.num_envs = 1
    sc1.env_origins = sc8.env_origins[5:6].copy()
    o1 = oracle.OracleSim(sc1)
    o1.set_state(s0[5:6])
    for a in acts:
        o1.step(a[5:6], cfg["dt"], cfg["substeps"], cfg["iterations"])
    assert np.array_equal(o1.get_state()[0], ref[5])
    # permuted order
    perm = np.array([3, 1, 7, 0, 2, 6, 5, 4])
    scp, _ = scenes.config_scene(3, num_envs=8)
    scp.env_origins = sc8.env_origins[perm].copy()
    op = oracle.OracleSim(scp, threads=2)
    op.set_state(s0[perm])
    for a in acts:
        op.step(a[perm], cfg["dt"], cfg["substeps"], cfg["iterations"])
    assert np.array_equal(op.get_state(), ref[perm])


@pytest.mark.parametrize("k,n_envs,steps", [(2, 6, 1000), (4, 6, 1000), (1, 8, 300)])
def test_long_random_action_runs_stay_finite_and_unit(k, n_envs, steps):
    sc, cfg = scenes.config_scene(k, num_envs=n_envs)
    o = oracle.OracleSim(sc, threads=8)
    if cfg["fallen"]:
        o.set_state(scenes.fallen_states(sc, cfg["seed"]))
    else:
        o.reset(cfg["seed"])
    for s in range(steps):
        o.step(scenes.actions_for_step(cfg["seed"], s, n_envs, sc.robot.n_dofs),
               cfg["dt"], cfg["substeps"], cfg["iterations"])
    st = o.get_state()
    assert np.isfinite(st).all()
    np.testing.assert_allclose(np.linalg.norm(st[:, :, 3:7], axis=2), 1.0, atol=1e-12)
    assert np.abs(st[:, :, 0:3]).max() < 60.0          # nobody is flung away
    assert np.linalg.norm(st[:, :, 10:13], axis=2).max() <= 64.0 + 1e-9
    _, _, done = o.get_obs()
    if steps >= 1000:
        assert done.all()                                # 1000-frame cap (Section 4.1)
