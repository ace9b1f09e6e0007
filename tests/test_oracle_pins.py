"""Closed-form pins of the oracle's solver details that no invariant test reaches: the weighted
mass splitting, the penetration branch of the contact bias, damping and the angular-velocity
cap, the two rules that drop a kept impulse, and the generator behind every seeded draw.
Each expected number is worked out by hand from the stated rule (Section 3.1 of the paper:
speculative unilateral contacts, restitution 0; the rest are this build's readings), so a wrong
sign, factor or operand in the oracle fails here."""
import numpy as np
import pytest

import oracle
import scenes
from scenes import robots
from helpers import free_params, single_scene

SOLVE_ONLY = oracle.PH_CONTACTS | oracle.PH_SOLVE


def _pinned_sphere(r, m, z):
    """A sphere whose centre a joint with three locked axes pins to the world."""
    bld = robots._Builder("pinned_sphere")
    b = bld.body("ball", r, 0.0, 0, (0.0, 0.0, z), mass=m)
    bld.joint(-1, b, (0.0, 0.0, z), [], 0.0)
    return bld.build(root_body=0, feet=(0,), term_height=-1e9, alive_bonus=0.0)


# gap -> share of the body the contact block gets: 1 up to half the margin (0.01), then a straight
# ramp down to 0 at the margin (0.02)
@pytest.mark.parametrize("d,w", [(0.004, 1.0), (0.010, 1.0), (0.012, 0.8), (0.015, 0.5), (0.019, 0.1)])
def test_one_sweep_gives_the_weighted_average_of_the_joint_copy_and_the_contact_copy(d, w):
    """Body shared by a joint block (weight 1) and a contact block (weight w).  From the snapshot
    v = (0, 0, -3) the joint block alone brings its copy to rest, the contact block alone brings its
    copy to the speculative bound -d/h; the body gets (1 * 0 + w * (-d/h)) / (1 + w)."""
    r, m, h = 0.1, 2.0, 1.0 / 120.0
    sc = single_scene(_pinned_sphere(r, m, r + d), params=free_params(gravity=(0.0, 0.0, 0.0)))
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(sc.robot, 1)
    st[0, 0, 9] = -3.0
    o.set_state(st)
    o.substep_phases(None, h, 1, SOLVE_ONLY)
    rec = o.get_contacts()[0, 0]
    assert rec["active"] == 1 and rec["w"] == pytest.approx(w, abs=1e-12)
    v = o.get_state()[0, 0, 7:13]
    assert v[2] == pytest.approx(-(d / h) * w / (1.0 + w), rel=1e-12)
    assert np.abs(np.delete(v, 2)).max() < 1e-14
    # and the floor of the ramp: a contact at the very edge of the margin still gets 1e-6
    if d == 0.019:
        st[0, 0, 2] = r + 0.02 - 1e-10
        o.set_state(st)
        o.substep_phases(None, h, 1, SOLVE_ONLY)
        assert o.get_contacts()[0, 0]["w"] == pytest.approx(1e-6, rel=1e-9)


def test_two_equal_blocks_split_the_body_in_halves_and_converge_to_the_joint():
    """The same body with the contact at full weight: after one sweep half way between rest and
    the bound, and the sweeps converge to rest (the bilateral joint wins over the one-sided bound)."""
    r, m, h, d = 0.1, 2.0, 1.0 / 120.0, 0.004
    sc = single_scene(_pinned_sphere(r, m, r + d), params=free_params(gravity=(0.0, 0.0, 0.0)))
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(sc.robot, 1)
    st[0, 0, 9] = -3.0
    o.set_state(st)
    o.substep_phases(None, h, 1, SOLVE_ONLY)
    assert o.get_state()[0, 0, 9] == pytest.approx(-0.5 * d / h, rel=1e-12)
    o.set_state(st)
    o.substep_phases(None, h, 60, SOLVE_ONLY)
    assert abs(o.get_state()[0, 0, 9]) < 1e-12


def test_mid_segment_block_fades_towards_the_segment_ends():
    """A capsule across a ridge whose crest meets the segment at 5 % of its length: the
    mid-segment slot's share is (0.05 - 0.001) / 0.1 of what the gap alone would give (1 here)."""
    t = scenes.make_flat_heightfield(nx=16, ny=16, cell=0.1)
    t.heights[:, 8] = 0.2                                     # crest along y at x = 0.8
    r, seg, d = 0.05, 0.4, 0.005
    rob = scenes.make_single(radius=r, seg_len=seg, axis=0, pos=(0.78 + seg / 2, 0.75, 0.2 + r + d))
    sc = single_scene(rob, terrain=t, params=free_params(gravity=(0.0, 0.0, 0.0)))
    o = oracle.OracleSim(sc)
    o.set_state(scenes.rest_state(rob, 1).astype(np.float32).astype(np.float64))
    c = o.generate_contacts()[0]
    mid = c[2]
    assert mid["active"] == 1 and mid["kind"] == 3
    assert mid["d"] == pytest.approx(d, abs=1e-6) and mid["n"][2] == pytest.approx(1.0, abs=1e-9)
    assert mid["w"] == pytest.approx(0.49, abs=2e-6)
    # the same capsule with the crest under its middle: no fade
    st = scenes.rest_state(rob, 1)
    st[0, 0, 0] = 0.8
    o.set_state(st.astype(np.float32).astype(np.float64))
    assert o.generate_contacts()[0, 2]["w"] == pytest.approx(1.0, abs=1e-12)


@pytest.mark.parametrize("depth,v_expected", [(0.005, 0.24), (0.050, 2.0)])
def test_penetrating_sphere_separates_at_beta_depth_over_h_capped_by_the_depenetration_speed(depth, v_expected):
    """beta_c = 0.2, h = 1/240 s, cap 2 m/s: 5 mm deep -> 0.2 * 0.005 * 240 = 0.24 m/s;
    50 mm deep -> 2.4 m/s, capped at exactly 2.  A sphere that already leaves faster is left alone."""
    r, h = 0.1, 1.0 / 240.0
    sc = single_scene(scenes.make_single(radius=r, pos=(0.0, 0.0, r - depth)), params=free_params(gravity=(0.0, 0.0, 0.0)))
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(sc.robot, 1)
    o.set_state(st)
    o.substep_phases(None, h, 4, SOLVE_ONLY)
    assert o.get_contacts()[0, 0]["d"] == pytest.approx(-depth, abs=1e-15)
    assert o.get_state()[0, 0, 9] == pytest.approx(v_expected, rel=1e-12)
    st[0, 0, 9] = 3.0
    o.set_state(st)
    o.substep_phases(None, h, 4, SOLVE_ONLY)
    assert o.get_state()[0, 0, 9] == pytest.approx(3.0, rel=1e-15)


def test_damping_divides_the_velocities_by_one_plus_h_c_every_substep():
    h, n, c_lin, c_ang = 1.0 / 90.0, 7, 3.0, 5.0
    p = free_params(gravity=(0.0, 0.0, 0.0), contacts=0, lin_damping=c_lin, ang_damping=c_ang)
    sc = single_scene(scenes.make_single(radius=0.1, pos=(0.0, 0.0, 1.0)), params=p)
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(sc.robot, 1)
    v0, w0 = np.array([1.0, -2.0, 0.5]), np.array([0.3, 0.2, -0.1])
    st[0, 0, 7:10], st[0, 0, 10:13] = v0, w0
    o.set_state(st)
    o.step(None, n * h, n, 0)
    s = o.get_state()[0, 0]
    np.testing.assert_allclose(s[7:10], v0 / (1.0 + h * c_lin) ** n, rtol=1e-13)
    np.testing.assert_allclose(s[10:13], w0 / (1.0 + h * c_ang) ** n, rtol=1e-13)
    # positions integrate the damped velocities: x_n = x_0 + h * sum_k v_k
    x_n = np.array([0.0, 0.0, 1.0]) + h * sum(v0 / (1.0 + h * c_lin) ** k for k in range(1, n + 1))
    np.testing.assert_allclose(s[0:3], x_n, rtol=1e-13)


def test_angular_velocity_cap_keeps_the_direction_and_comes_after_the_damping():
    h = 1.0 / 90.0
    direction = np.array([1.0, 2.0, 2.0]) / 3.0
    for c_ang, w_in, w_out in ((0.0, 100.0, 64.0), (5.0, 100.0, 64.0), (5.0, 66.0, 66.0 / (1.0 + 5.0 * h)), (0.0, 63.0, 63.0)):
        p = free_params(gravity=(0.0, 0.0, 0.0), contacts=0, ang_damping=c_ang, max_ang_vel=64.0)
        sc = single_scene(scenes.make_single(radius=0.1, pos=(0.0, 0.0, 1.0)), params=p)
        o = oracle.OracleSim(sc)
        st = scenes.rest_state(sc.robot, 1)
        st[0, 0, 10:13] = w_in * direction
        o.set_state(st)
        o.step(None, h, 1, 0)
        w = o.get_state()[0, 0, 10:13]
        assert np.linalg.norm(w) == pytest.approx(w_out, rel=1e-13)
        np.testing.assert_allclose(w / np.linalg.norm(w), direction, atol=1e-14)
        # the orientation has turned by the capped rate: angle = 2 atan(h |w| / 2) for this update rule
        q = o.get_state()[0, 0, 3:7]
        assert 2.0 * np.arctan2(np.linalg.norm(q[1:]), q[0]) == pytest.approx(2.0 * np.arctan(0.5 * h * w_out), rel=1e-12)


def test_kept_limit_impulse_is_dropped_when_the_row_stands_for_the_other_limit():
    """One link hinged to the world, hanging at angle 0 between the limits -0.6 and +0.4: the limit
    row stands for the upper limit (the nearer one).  With no sweep at all the step applies
    share x kept impulse as a torque about the hinge axis: delta omega_y = -0.8 * 0.3 / I_yy when the
    kept impulse stood for the upper limit (or for 'the nearer one'), nothing when it stood for the
    lower one."""
    rob = scenes.make_chain(n_links=1, lo=-0.6, hi=0.4)
    p = free_params(gravity=(0.0, 0.0, 0.0), contacts=0, warm_start=0.8)
    sc = single_scene(rob, params=p)
    I_yy = rob.inertia[0, 1]
    lam = np.zeros((1, 1, 6)); lam[0, 0, 3] = 0.3
    got = {}
    for side in (1, -1, 0):
        o = oracle.OracleSim(sc)
        o.set_state(scenes.rest_state(rob, 1))
        o.set_warm(lam, np.zeros((1, o.S, 3)))
        o.set_warm_flags(np.full((1, 1, 3), side), np.ones((1, o.S)))
        o.substep_phases(None, 1.0 / 120.0, 0, oracle.PH_SOLVE)
        got[side] = o.get_state()[0, 0, 7:13].copy()
    want = np.zeros(6); want[4] = -0.8 * 0.3 / I_yy
    np.testing.assert_allclose(got[1], want, atol=1e-13)
    np.testing.assert_allclose(got[-1], want, atol=1e-13)
    np.testing.assert_allclose(got[0], np.zeros(6), atol=1e-15)
    # what is handed on: the limit the row stands for now, with the impulse it started from
    kept_j, _ = o.get_warm()
    assert kept_j[0, 0, 3] == 0.0


def test_kept_contact_impulse_is_dropped_when_the_slot_was_not_active_in_the_previous_substep():
    """A sphere 1 mm above the plane with a kept normal impulse of 0.5 N s: with no sweep the step
    applies share x kept / m upwards if the slot was active in the previous substep, nothing else."""
    r, m = 0.1, 2.0
    p = free_params(gravity=(0.0, 0.0, 0.0), warm_start=0.8)
    sc = single_scene(scenes.make_single(radius=r, pos=(0.0, 0.0, r + 0.001), mass=m), params=p)
    got = {}
    for was_on in (1, 0):
        o = oracle.OracleSim(sc)
        o.set_state(scenes.rest_state(sc.robot, 1))
        ls = np.zeros((1, o.S, 3)); ls[0, 0, 0] = 0.5
        o.set_warm(np.zeros((1, 0, 6)), ls)
        o.set_warm_flags(np.zeros((1, 0, 3)), np.full((1, o.S), was_on))
        o.substep_phases(None, 1.0 / 120.0, 0, SOLVE_ONLY)
        got[was_on] = o.get_state()[0, 0, 9]
    assert got[1] == pytest.approx(0.8 * 0.5 / m, rel=1e-13)
    assert got[0] == 0.0


def test_uniform_generator_reproduces_the_published_splitmix64_outputs():
    """Every seeded draw (reset noise, pushes, targets) is the top 24 bits of one SplitMix64 output
    (Steele, Lea and Flood 2014; the reference generator's first three outputs from state 0 are
    0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F).  uniform(seed, 0, 0) mixes `seed`
    plus one increment, so seeds 0, g and 2 g (g = the generator's increment) walk that sequence."""
    g = 0x9E3779B97F4A7C15
    ref = (0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F)
    for k, z in enumerate(ref):
        assert oracle.uniform((k * g) & (2 ** 64 - 1), 0, 0) == (z >> 40) / 2.0 ** 24
    # env and index enter as odd multiples added to the seed: distinct streams, all in [0, 1)
    u = np.array([[oracle.uniform(7, e, i) for i in range(64)] for e in range(64)])
    assert u.min() >= 0.0 and u.max() < 1.0 and len(np.unique(u)) == u.size
    assert abs(u.mean() - 0.5) < 0.02 and abs(np.corrcoef(u[:-1].ravel(), u[1:].ravel())[0, 1]) < 0.05
