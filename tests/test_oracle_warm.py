"""Pins for the oracle's warm start (rows start a substep from a share of the impulses they ended
the previous one with; a stiffness gain within the Jacobi scheme of Section 3.1): static closed
forms the kept impulses must converge to, conservation laws that the extra impulses must not
break, and the reason for having it (a lower residual at the same number of sweeps)."""
import numpy as np
import pytest

import oracle
import scenes
from helpers import angular_momentum, free_params, linear_momentum, single_scene

G = 9.81


def test_share_zero_is_the_plain_solver():
    rob = scenes.make_humanoid()
    out = []
    for share in (None, 0.0):
        sc = single_scene(rob, num_envs=2)
        o = oracle.OracleSim(sc)
        if share is not None:
            o.set_warm_start(share)
        o.reset(3)
        for k in range(6):
            o.step(scenes.actions_for_step(2, k, 2, rob.n_dofs), 1 / 60, 2, 6)
        out.append(o.get_state())
    assert np.array_equal(out[0], out[1])
    lj, ls = o.get_warm()       # the impulses are kept either way; share 0 does not use them
    assert np.abs(lj).max() > 0


def test_injected_static_impulses_cancel_the_load_exactly():
    # a chain at rest under gravity: joint k carries the weight of the links below it.  Started
    # from exactly these impulses (share 1), a substep with no sweep at all leaves it at rest.
    n, mass = 4, 0.5
    rob = scenes.make_chain(n_links=n, mass=mass)
    h = 1 / 120
    sc = single_scene(rob, params=free_params(contacts=0, warm_start=1.0))
    o = oracle.OracleSim(sc)
    o.set_state(scenes.rest_state(rob))
    lj = np.zeros((1, n, 6))
    lj[0, :, 2] = [h * G * mass * (n - k) for k in range(n)]
    o.set_warm(lj, np.zeros((1, o.S, 3)))
    o.substep_phases(None, h, 0, oracle.PH_FORCES | oracle.PH_SOLVE)
    assert np.abs(o.get_state()[0][:, 7:13]).max() < 1e-15
    # without them the links fall
    o.set_state(scenes.rest_state(rob))
    o.substep_phases(None, h, 0, oracle.PH_FORCES | oracle.PH_SOLVE)
    np.testing.assert_allclose(o.get_state()[0][:, 9], -G * h, rtol=1e-12)
    # a motor torque is cancelled by the limit row started from gear * u * h (hinge about y,
    # the joint's first axis: row 3), whichever limit is the nearer one
    gear = 2.0
    rob1 = scenes.make_chain(n_links=1, seg_len=0.4, mass=1.0, lo=-0.5, hi=0.8, gear=gear)
    sc1 = single_scene(rob1, params=free_params(contacts=0, gravity=(0, 0, 0), warm_start=1.0))
    o1 = oracle.OracleSim(sc1)
    for u, th in ((1.0, 0.7), (-1.0, -0.4)):
        o1.set_state(_hinge_state(rob1, th))
        lj1 = np.zeros((1, 1, 6)); lj1[0, 0, 3] = gear * h
        o1.set_warm(lj1, np.zeros((1, o1.S, 3)))
        o1.substep_phases(np.array([[u]]), h, 0, oracle.PH_FORCES | oracle.PH_SOLVE)
        assert np.abs(o1.get_state()[0][:, 7:13]).max() < 1e-14


def _hinge_state(rob, th):
    """One-link chain hinged to the world about y at its top end, turned by th."""
    st = scenes.rest_state(rob)
    anchor = st[0, 0, :3] + np.array([0.0, 0.0, 0.2])
    q = np.array([np.cos(th / 2), 0.0, np.sin(th / 2), 0.0])
    R = np.array([[np.cos(th), 0, np.sin(th)], [0, 1, 0], [-np.sin(th), 0, np.cos(th)]])
    st[0, 0, :3] = anchor + R @ np.array([0.0, 0.0, -0.2])
    st[0, 0, 3:7] = q
    return st


def test_hanging_chain_steady_state():
    # at rest the kept vertical impulses equal the static tension h g (mass below), and the sweeps
    # only have to supply the share that was not kept: the sag that drives them shrinks to
    # (1 - share) of the cold start's
    n, mass = 4, 0.5
    rob = scenes.make_chain(n_links=n, mass=mass)
    dt, sub, its = 1 / 60, 2, 4
    h = dt / sub
    want = np.array([h * G * mass * (n - k) for k in range(n)])
    z_rest = scenes.rest_state(rob)[0][-1, 2]
    sag = {}
    for share in (0.0, 0.5, 0.9):
        sc = single_scene(rob, params=free_params(contacts=0, warm_start=share))
        o = oracle.OracleSim(sc)
        o.set_state(scenes.rest_state(rob))
        for _ in range(400):
            o.step(None, dt, sub, its)
        lam, st = o.get_warm()[0][0], o.get_state()[0]
        np.testing.assert_allclose(lam[:, 2], want, rtol=1e-9)
        assert np.abs(lam[:, [0, 1, 3, 4, 5]]).max() < 1e-9    # nothing sideways, no torque, limits idle
        assert np.abs(st[:, 7:13]).max() < 1e-10
        sag[share] = z_rest - st[-1, 2]
    assert sag[0.0] > 0.01
    assert sag[0.5] == pytest.approx(0.5 * sag[0.0], rel=1e-6)
    assert sag[0.9] == pytest.approx(0.1 * sag[0.0], rel=1e-6)


def test_limit_row_settles_at_the_motor_impulse():
    # a hinge pressed against its upper limit by a constant torque: the limit row balances it
    gear = 2.0
    rob = scenes.make_chain(n_links=1, seg_len=0.4, mass=1.0, lo=-0.5, hi=0.8, gear=gear)
    sc = single_scene(rob, params=free_params(contacts=0, gravity=(0, 0, 0), warm_start=0.9))
    o = oracle.OracleSim(sc)
    o.set_state(scenes.rest_state(rob))
    dt, sub = 1 / 60, 4
    for _ in range(240):
        o.step(np.array([[1.0]]), dt, sub, 6)
    assert 0.8 - 1e-3 < o.joint_angles()[0, 0, 0] < 0.8 + 0.03
    # the hinge axis is the joint's first axis: angular row 0 (row 3 of the joint) is the limit row
    assert o.get_warm()[0][0, 0, 3] == pytest.approx(gear * dt / sub, rel=1e-6)
    # pressed the other way it leaves the limit; at the lower one the kept impulse is that
    # limit's, again positive
    for _ in range(240):
        o.step(np.array([[-1.0]]), dt, sub, 6)
    assert -0.5 - 0.03 < o.joint_angles()[0, 0, 0] < -0.5 + 1e-3
    assert o.get_warm()[0][0, 0, 3] == pytest.approx(gear * dt / sub, rel=1e-6)


def test_resting_sphere_starts_from_the_impulse_that_carries_it():
    m = 2.0
    rob = scenes.make_single(radius=0.1, seg_len=0.0, pos=(0, 0, 0.12), mass=m)
    dt = 1 / 60
    viol = {}
    for share in (0.0, 1.0):
        sc = single_scene(rob, params=free_params(warm_start=share))
        o = oracle.OracleSim(sc)
        o.set_state(scenes.rest_state(rob))
        for _ in range(90):
            o.step(None, dt, 1, 3)
        lj, ls = o.get_warm()
        assert ls[0, 0, 0] == pytest.approx(m * G * dt, rel=1e-6)      # normal row: m g h
        assert np.abs(ls[0, 0, 1:]).max() < 1e-12
        o.start_trace(0, 16)
        o.step(None, dt, 1, 3)
        viol[share] = o.trace()["onesided_viol"][0]
    # the first sweep sees the approach speed g h when started cold, nothing when warm
    assert viol[0.0] == pytest.approx(G * dt, rel=1e-6)
    assert viol[1.0] < 1e-9
    # set_state and reset drop what is kept
    o.set_state(scenes.rest_state(rob))
    assert np.abs(o.get_warm()[1]).max() == 0
    for _ in range(30):
        o.step(None, dt, 1, 3)
    assert np.abs(o.get_warm()[1]).max() > 0
    o.reset(1)
    assert np.abs(o.get_warm()[1]).max() == 0


def test_momentum_is_conserved_with_warm_start():
    rob = scenes.make_humanoid()
    sc = single_scene(rob, params=free_params(contacts=0, gravity=(0, 0, 0), gyroscopic=0, warm_start=0.9))
    o = oracle.OracleSim(sc)
    o.reset(3)
    p0 = linear_momentum(rob, o.get_state()[0])
    for k in range(20):
        o.step(scenes.actions_for_step(11, k, 1, rob.n_dofs), 1 / 60, 4, 10)
    st = o.get_state()[0]
    scale = (rob.mass[:, None] * np.abs(st[:, 7:10])).sum()
    assert scale > 1.0 and np.abs(o.get_warm()[0]).max() > 1e-3
    np.testing.assert_allclose(linear_momentum(rob, st), p0, atol=1e-11 * scale)
    # at a fixed pose (forces and solve only) the angular momentum is kept as well: the kept
    # impulses act at the same shared points as the solver's
    L0 = angular_momentum(rob, st)
    o.substep_phases(scenes.actions_for_step(5, 99, 1, rob.n_dofs), 1 / 240, 25, oracle.PH_FORCES | oracle.PH_SOLVE)
    np.testing.assert_allclose(angular_momentum(rob, o.get_state()[0]), L0, atol=1e-11 * (np.abs(L0).max() + 1.0))


def test_warm_start_lowers_residual_and_penetration_at_equal_sweeps():
    n = 8
    res, pen = {}, {}
    for share in (0.0, 0.8):
        sc, cfg = scenes.config_scene(3, num_envs=n)
        sc.params.warm_start = share
        o = oracle.OracleSim(sc)
        o.reset(5)
        its = 10
        r, p = [], []
        for t in range(90):
            u = 0.3 * scenes.actions_for_step(cfg["seed"], t, n, sc.robot.n_dofs)
            o.start_trace(0, 4 * its + 8)
            o.step(u, cfg["dt"], cfg["substeps"], its)
            if t >= 30:
                r.append(o.trace()["bilateral_rms"][its - 1::its].mean())
                c = o.get_contacts()
                act = c["active"] == 1
                p.append((-c["d"][act]).clip(0).max() if act.any() else 0.0)
        res[share], pen[share] = np.mean(r), np.mean(p)
    assert res[0.8] < 0.9 * res[0.0]
    assert pen[0.8] < 0.8 * pen[0.0]
