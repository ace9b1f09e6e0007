"""Pins for the oracle's capsule-capsule contacts (Section 3.1: contacts among bodies as
unilateral constraints with Coulomb friction, restitution 0; Section 4.1: inter-agent
collisions): closest points against brute force and closed forms, perfectly inelastic
collisions, momentum conservation of an isolated pair, self- against inter-agent path,
a resting stack."""
import numpy as np
import pytest

import oracle
import scenes
from helpers import free_params, single_scene, linear_momentum, angular_momentum


def _brute_d2(P0, P1, Q0, Q1, n=401):
    u = np.linspace(0.0, 1.0, n)
    a = P0[None, :] + u[:, None] * (P1 - P0)[None, :]
    b = Q0[None, :] + u[:, None] * (Q1 - Q0)[None, :]
    return ((a[:, None, :] - b[None, :, :]) ** 2).sum(2).min()


def test_segment_segment_against_dense_sampling():
    rng = np.random.default_rng(5)
    for k in range(300):
        P0, P1, Q0, Q1 = (rng.uniform(-1, 1, 3).astype(np.float32).astype(np.float64) for _ in range(4))
        if k % 7 == 0:
            Q1 = Q0 + (P1 - P0) * rng.uniform(0.3, 2.0)      # parallel
        if k % 11 == 0:
            P1 = P0.copy()                                   # a sphere
        d2, s, t = oracle.segment_segment_f32(P0, P1, Q0, Q1)
        assert 0.0 <= s <= 1.0 and 0.0 <= t <= 1.0
        # the reported parameters give the reported distance ...
        cp, cq = P0 + s * (P1 - P0), Q0 + t * (Q1 - Q0)
        assert abs(((cp - cq) ** 2).sum() - d2) < 1e-5
        # ... and no sampled pair of points is closer (sampling error of a 401 x 401 grid)
        ref = _brute_d2(P0, P1, Q0, Q1)
        assert d2 <= ref + 1e-5
        assert d2 >= ref - 0.02


def test_segment_segment_closed_forms():
    # crossing segments touch
    d2, s, t = oracle.segment_segment_f32([-1, 0, 0], [1, 0, 0], [0, -1, 0], [0, 1, 0])
    assert d2 == 0.0 and s == 0.5 and t == 0.5
    # skew segments: distance along the common normal
    d2, s, t = oracle.segment_segment_f32([-1, 0, 0], [1, 0, 0], [0.5, -1, 0.25], [0.5, 3, 0.25])
    assert d2 == pytest.approx(0.0625, rel=1e-6) and s == pytest.approx(0.75) and t == pytest.approx(0.25)
    # end point against end point
    d2, s, t = oracle.segment_segment_f32([0, 0, 0], [1, 0, 0], [2, 1, 0], [3, 1, 0])
    assert d2 == pytest.approx(2.0) and s == 1.0 and t == 0.0
    # point against segment interior (textbook point-line distance)
    d2, s, t = oracle.segment_segment_f32([0.25, 2, 0], [0.25, 2, 0], [0, 0, 0], [1, 0, 0])
    assert d2 == pytest.approx(4.0) and t == pytest.approx(0.25)
    # swapping the segments swaps the parameters
    a = oracle.segment_segment_f32([0, 0, 0], [1, 0.2, 0], [0.3, 1, 0.1], [0.9, 0.4, -0.3])
    b = oracle.segment_segment_f32([0.3, 1, 0.1], [0.9, 0.4, -0.3], [0, 0, 0], [1, 0.2, 0])
    assert a[0] == pytest.approx(b[0], rel=1e-5) and a[1] == pytest.approx(b[2], abs=1e-5)


def _two_spheres(m0, m1, gap=0.05, r=0.1, group=False):
    """Two free spheres on the x axis far above the ground, no gravity."""
    p = free_params(gravity=(0.0, 0.0, 0.0), self_collide=1)
    if not group:
        rob = scenes.make_loose([(r, 0.0, 0, (0.0, 0.0, 5.0), m0), (r, 0.0, 0, (2 * r + gap, 0.0, 5.0), m1)])
        return rob, single_scene(rob, params=p)
    assert m0 == m1
    p.self_collide, p.group_size = 0, 2
    rob = scenes.make_single(radius=r, pos=(0.0, 0.0, 5.0), mass=m0)
    sc = single_scene(rob, params=p, num_envs=2)
    sc.env_origins[1, 0] = 2 * r + gap
    return rob, sc


@pytest.mark.parametrize("m0,m1", [(1.0, 1.0), (1.0, 3.0), (5.0, 0.5)])
def test_head_on_collision_is_perfectly_inelastic(m0, m1):
    """Restitution 0: after the impact both spheres move with the centre-of-mass velocity and the
    surfaces touch; before it (gap larger than what one substep closes) nothing changes."""
    rob, sc = _two_spheres(m0, m1)
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(rob)
    st[0, 0, 7], st[0, 1, 7] = 1.0, -0.5
    o.set_state(st)
    vcm = (m0 * 1.0 - m1 * 0.5) / (m0 + m1)
    h = 1.0 / 240.0
    o.substep_phases(None, h, 4)               # gap 0.05 > 1.5 * h: speculative row inactive
    s = o.get_state()
    assert s[0, 0, 7] == pytest.approx(1.0, abs=1e-12) and s[0, 1, 7] == pytest.approx(-0.5, abs=1e-12)
    for _ in range(40):
        o.substep_phases(None, h, 4)
    s = o.get_state()
    assert s[0, 0, 7] == pytest.approx(vcm, abs=1e-9) and s[0, 1, 7] == pytest.approx(vcm, abs=1e-9)
    assert s[0, 1, 0] - s[0, 0, 0] - 0.2 == pytest.approx(0.0, abs=1e-9)
    assert np.abs(s[0, :, 8:13]).max() < 1e-12
    pc = o.get_pair_contacts()
    assert len(pc) == 1 and (pc[0]["body_a"], pc[0]["body_b"]) == (0, 1)
    assert np.allclose(pc[0]["n"], [-1.0, 0.0, 0.0]) and pc[0]["d"] == pytest.approx(0.0, abs=1e-9)


def test_isolated_pair_conserves_linear_and_angular_momentum():
    """Off-centre capsule hits with friction: the contact impulses are internal forces."""
    rng = np.random.default_rng(11)
    p = free_params(gravity=(0.0, 0.0, 0.0), self_collide=1, gyroscopic=0)
    hits = 0
    for trial in range(40):
        rob = scenes.make_loose([(0.08, 0.5, 0, (0.0, 0.0, 5.0), 1.3), (0.05, 0.4, 1, (0.1, 0.05, 6.0), 0.7)])
        sc = single_scene(rob, params=p)
        st = scenes.rest_state(rob)
        st[0, 1, 2] = 5.14
        q = rng.normal(size=(2, 4)) * 0.3 + np.array([1.0, 0, 0, 0])
        st[0, :, 3:7] = q / np.linalg.norm(q, axis=1, keepdims=True)
        st[0, :, 7:13] = rng.normal(size=(2, 6)) * np.array([0.5, 0.5, 0.5, 2, 2, 2])
        st[0, 1, 9] -= 4.0
        o = oracle.OracleSim(sc)
        o.set_state(st)
        P0, L0 = linear_momentum(rob, st[0]), angular_momentum(rob, st[0])
        o.substep_phases(None, 1.0 / 240.0, 30, oracle.PH_CONTACTS | oracle.PH_FORCES | oracle.PH_SOLVE)
        s1 = o.get_state()
        pc = o.get_pair_contacts()
        if len(pc) == 0 or np.abs(s1[0, :, 7:13] - st[0, :, 7:13]).max() < 1e-2:
            continue                                    # no record, or a speculative row that stayed idle
        hits += 1
        assert np.allclose(linear_momentum(rob, s1[0]), P0, atol=1e-12)
        assert np.allclose(angular_momentum(rob, s1[0]), L0, atol=1e-12)
        # the relative normal velocity at the contact satisfies the speculative bound
        c = pc[0]
        va = s1[0, 0, 7:10] + np.cross(s1[0, 0, 10:13], c["ra"])
        vb = s1[0, 1, 7:10] + np.cross(s1[0, 1, 10:13], c["rb"])
        bound = -c["d"] * 240.0 if c["d"] >= 0 else 0.0
        assert c["n"] @ (va - vb) >= bound - 1e-6
    assert hits >= 10


def test_contact_geometry_of_two_capsules():
    """Crossed capsules one above the other: closed-form distance, normal and contact points
    (to the single precision of the segment parameters)."""
    rob = scenes.make_loose([(0.08, 0.6, 0, (0.0, 0.0, 5.0), 1.0), (0.05, 0.4, 1, (0.1, -0.05, 6.0), 1.0)])
    sc = single_scene(rob, params=free_params(gravity=(0.0, 0.0, 0.0), self_collide=1))
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(rob)
    st[0, 1, 2] = 5.14
    o.set_state(st)
    pc = o.generate_pair_contacts()
    assert len(pc) == 1
    c = pc[0]
    assert c["d"] == pytest.approx(0.14 - 0.13, abs=2e-6)
    assert np.allclose(c["n"], [0, 0, -1.0], atol=2e-6)          # from B (above) to A
    # one contact point, midway between the top of A and the bottom of B at the crossing
    assert np.allclose(c["ra"], [0.1, 0.0, 0.085], atol=2e-6)
    assert np.allclose(c["rb"], [0.0, 0.05, -0.055], atol=2e-6)
    assert c["s"] == pytest.approx((0.1 + 0.3) / 0.6, abs=1e-6) and c["t"] == pytest.approx(0.25 / 0.4 * 1.0, abs=1e-6)
    # outside the margin: no record
    st[0, 1, 2] += 0.011
    o.set_state(st)
    assert len(o.generate_pair_contacts()) == 0


def test_inter_agent_contact_equals_self_contact_of_the_merged_robot():
    """Two one-sphere agents of one interaction group behave exactly like one robot made of the
    same two free spheres with self-collision on."""
    rob2, sc2 = _two_spheres(1.0, 1.0)
    rob1, scg = _two_spheres(1.0, 1.0, group=True)
    a, b = oracle.OracleSim(sc2), oracle.OracleSim(scg)
    st = scenes.rest_state(rob2)
    st[0, 0, 7:10], st[0, 1, 7:10] = (1.0, 0.2, 0.0), (-0.5, 0.0, 0.1)
    a.set_state(st)
    sg = np.zeros((2, 1, 13))
    sg[:, 0] = st[0]
    sg[1, 0, 0] -= scg.env_origins[1, 0]
    b.set_state(sg)
    for _ in range(30):
        a.substep_phases(None, 1.0 / 240.0, 6)
        b.substep_phases(None, 1.0 / 240.0, 6)
    sa, sb = a.get_state(), b.get_state()
    sb[1, 0, 0] += scg.env_origins[1, 0]
    assert np.allclose(sa[0], sb[:, 0], atol=1e-12)
    assert len(b.get_pair_contacts()) == 1
    # agents of different groups never see each other
    scg.params.group_size = 1
    c = oracle.OracleSim(scg)
    c.set_state(sg)
    for _ in range(30):
        c.substep_phases(None, 1.0 / 240.0, 6)
    assert len(c.get_pair_contacts()) == 0
    assert c.get_state()[0, 0, 7] == pytest.approx(1.0)


def test_sphere_resting_on_a_grounded_sphere_stays_put():
    """Stack under gravity: ground contact and sphere-sphere contact share the lower body; after
    settling both spheres are at rest with touching surfaces."""
    r = 0.1
    rob = scenes.make_loose([(r, 0.0, 0, (0.0, 0.0, r), 2.0), (r, 0.0, 0, (0.0, 0.0, 1.0), 1.0)])
    sc = single_scene(rob, params=free_params(self_collide=1))
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(rob)
    st[0, 1, 2] = 3 * r + 0.002
    o.set_state(st)
    for _ in range(240):
        o.step(None, 1.0 / 60.0, 4, 20)
    s = o.get_state()
    assert np.abs(s[0, :, 7:10]).max() < 2e-3
    assert s[0, 0, 2] == pytest.approx(r, abs=2e-3)
    assert s[0, 1, 2] - s[0, 0, 2] == pytest.approx(2 * r, abs=2e-3)
    assert np.abs(s[0, :, 0:2]).max() < 1e-6


def _sphere_cluster(n_envs, seed):
    rob = scenes.make_loose([(0.1, 0.0, 0, (3.0 * k, 0.0, 5.0), 1.0) for k in range(16)])
    sc = scenes.make_scene(rob, scenes.make_plane(), n_envs,
                           params=scenes.SimParams(gravity=(0.0, 0.0, 0.0), self_collide=1))
    rng = np.random.default_rng(seed)
    st = np.repeat(scenes.rest_state(rob), n_envs, axis=0)
    st[:, :, 0:3] = np.array([0.0, 0.0, 5.0]) + rng.normal(size=(n_envs, 16, 3)) * 0.02
    return rob, sc, st.astype(np.float32).astype(np.float64)


def test_bounded_contact_store_keeps_the_closest_contacts_of_a_block():
    """Sixteen overlapping spheres per agent, 120 touching pairs each.  With room for 50 contacts
    per block of two agents, each block keeps exactly the 50 with the smallest centre distance
    (worked out here from the positions in double precision; the distances on either side of the
    cut are far enough apart for single precision to order them the same way), in the order the unbounded list has them; a
    bound that is not reached changes nothing."""
    rob, sc, st = _sphere_cluster(4, 5)
    h = 1.0 / 240.0
    free = oracle.OracleSim(sc, threads=1)
    free.set_state(st); free.step(None, h, 1, 3)
    all_c = free.get_pair_contacts()
    assert len(all_c) == 4 * 120
    # closed form for spheres: gap = |x_a - x_b| - 2 r
    x = st[:, :, 0:3]
    gap = np.linalg.norm(x[all_c["env_a"], all_c["body_a"]] - x[all_c["env_b"], all_c["body_b"]], axis=1) - 0.2
    np.testing.assert_allclose(all_c["d"], gap, atol=1e-12)
    np.testing.assert_allclose(all_c["gap32"], gap, atol=1e-6)
    keep = np.zeros(len(all_c), bool)
    for blk in range(2):
        idx = np.flatnonzero(all_c["env_a"] // 2 == blk)
        srt = idx[np.argsort(gap[idx])]
        assert gap[srt[50]] - gap[srt[49]] > 1e-6   # the cut falls where single precision orders as double does
        keep[srt[:50]] = True
    capped = oracle.OracleSim(sc, threads=1)
    capped.set_pair_cap(50, 2)
    capped.set_state(st); capped.step(None, h, 1, 3)
    kept = capped.get_pair_contacts()
    assert len(kept) == 100
    for f in ("env_a", "body_a", "env_b", "body_b"):
        assert np.array_equal(kept[f], all_c[f][keep]), f
    assert capped.set_pair_cap(0, 1) == 4 * 120 - 100
    assert np.abs(capped.get_state() - free.get_state()).max() > 1e-6   # fewer contacts, another step
    # a bound that is not reached: bit for bit the unbounded step, also in several threads
    roomy = oracle.OracleSim(sc, threads=4)
    roomy.set_pair_cap(240, 2)
    roomy.set_state(st); roomy.step(None, h, 1, 3)
    assert np.array_equal(roomy.get_state(), free.get_state())
    assert roomy.set_pair_cap(0, 1) == 0


def test_bounded_contact_store_breaks_equal_gaps_by_the_smaller_key():
    """Four spheres at the corners of a square of side 0.15 touch along the four sides with exactly
    equal gaps (the diagonals, 0.212 apart against 0.2 + the 0.01 margin, do not): room for two keeps the two pairs with the
    smallest (agent, agent, body, body) keys, (0,1) and (0,2)."""
    rob = scenes.make_loose([(0.1, 0.0, 0, (3.0 * k, 0.0, 5.0), 1.0) for k in range(4)])
    sc = scenes.make_scene(rob, scenes.make_plane(), 1,
                           params=scenes.SimParams(gravity=(0.0, 0.0, 0.0), self_collide=1, contact_margin=0.01))
    st = scenes.rest_state(rob)
    st[0, :, 0:3] = np.array([[0.0, 0.0, 5.0], [0.15, 0.0, 5.0], [0.0, 0.15, 5.0], [0.15, 0.15, 5.0]])
    ref = oracle.OracleSim(sc, threads=1)
    ref.set_state(st)
    c = ref.generate_pair_contacts()
    assert sorted(zip(c["body_a"].tolist(), c["body_b"].tolist())) == [(0, 1), (0, 2), (1, 3), (2, 3)]
    assert len(set(c["gap32"].tolist())) == 1
    ref.set_pair_cap(2, 1)
    ref.step(None, 1.0 / 240.0, 1, 2)
    k = ref.get_pair_contacts()
    assert list(zip(k["body_a"].tolist(), k["body_b"].tolist())) == [(0, 1), (0, 2)]


# ---- interaction groups chosen from positions (agents that wander meet their actual neighbours)

def _sphere_agents(n, origins, group):
    p = free_params(gravity=(0.0, 0.0, 0.0), self_collide=0)
    p.group_size = group
    rob = scenes.make_single(radius=0.1, pos=(0.0, 0.0, 5.0), mass=1.0)
    sc = single_scene(rob, params=p, num_envs=n)
    sc.env_origins[:] = np.asarray(origins, np.float64)
    return rob, sc


def test_agents_grouped_by_hand_equal_the_merged_robot_whatever_their_numbers():
    """Agents 0 and 3 of four, put into one group by a permutation, behave exactly like one robot
    made of the same two free spheres with self-collision on (and like agents 0 and 1 of the
    consecutive grouping); agents 1 and 2, far away, form the other group.  In their own order
    (0,1 | 2,3) agents 0 and 3 pass through each other."""
    rob2, sc2 = _two_spheres(1.0, 1.0)
    org = [(0.0, 0.0, 0.0), (40.0, 0.0, 0.0), (80.0, 0.0, 0.0), (0.25, 0.0, 0.0)]
    rob1, sc4 = _sphere_agents(4, org, 2)
    a, b, c = oracle.OracleSim(sc2), oracle.OracleSim(sc4), oracle.OracleSim(sc4)
    st = scenes.rest_state(rob2)
    st[0, 0, 7:10], st[0, 1, 7:10] = (1.0, 0.2, 0.0), (-0.5, 0.0, 0.1)
    a.set_state(st)
    s4 = np.repeat(scenes.rest_state(rob1), 4, axis=0)
    s4[0, 0, 7:10], s4[3, 0, 7:10] = st[0, 0, 7:10], st[0, 1, 7:10]
    s4[1, 0, 7:10] = (0.0, 0.3, 0.0)   # a bystander that just drifts
    b.set_state(s4); c.set_state(s4)
    b.set_groups([0, 3, 2, 1])
    assert b.get_groups().tolist() == [0, 3, 2, 1]
    for _ in range(30):
        a.substep_phases(None, 1.0 / 240.0, 6)
        b.step(None, 1.0 / 240.0, 1, 6)
        c.step(None, 1.0 / 240.0, 1, 6)
    sa, sb, sc_ = a.get_state(), b.get_state(), c.get_state()
    sb[3, 0, 0] += 0.25
    assert np.allclose(sa[0, 0], sb[0, 0], atol=1e-12) and np.allclose(sa[0, 1], sb[3, 0], atol=1e-12)
    pc = b.get_pair_contacts()
    assert len(pc) == 1 and (pc["env_a"][0], pc["env_b"][0]) == (0, 3)    # reported by agent number
    assert sb[1, 0, 8] == pytest.approx(0.3) and sb[1, 0, 1] == pytest.approx(0.3 * 30 / 240.0)
    # their own order: nobody meets anybody
    assert len(c.get_pair_contacts()) == 0 and sc_[0, 0, 7] == pytest.approx(1.0)
    # not a permutation
    with pytest.raises(ValueError):
        b.set_groups([0, 0, 1, 2])
    # back to their own order
    b.set_groups(None)
    assert b.get_groups().tolist() == [0, 1, 2, 3]


def test_regrouping_orders_the_agents_along_the_hilbert_curve_of_their_cells():
    """What defines the curve: it visits every cell of an aligned 2^k x 2^k block once, and
    consecutive cells share an edge.  One agent per cell of the 8 x 8 block of 2 m cells whose
    corner is (16 m, -32 m) (negative coordinates included), numbered at random, reach 0 (nobody
    is anybody's neighbour: the groups are consecutive agents of the order).  A second agent in
    one of the cells comes right after the first one (equal cells: by agent number)."""
    rng = np.random.default_rng(4)
    cells = np.stack(np.meshgrid(np.arange(8), np.arange(8)), -1).reshape(64, 2)
    num = rng.permutation(64)
    org = np.zeros((65, 3))
    org[num, 0:2] = cells * 2.0 + np.array([16.0, -32.0]) + rng.uniform(0.05, 1.95, size=(64, 2))
    org[64, 0:2] = np.floor(org[num[20], 0:2] / 2.0) * 2.0 + 1.0   # in the cell of agent num[20], not on top of it
    rob, sc = _sphere_agents(65, org, 2)
    o = oracle.OracleSim(sc)
    o.set_state(np.repeat(scenes.rest_state(rob), 65, axis=0))
    o.regroup(2.0, 0.0)
    order = o.get_groups()
    assert sorted(order.tolist()) == list(range(65))
    k = order.tolist().index(64)
    assert order[k - 1] == num[20]
    walk = np.floor(org[np.delete(order, k), 0:2] / 2.0).astype(int)
    assert len({tuple(c) for c in walk}) == 64
    assert np.all(np.abs(np.diff(walk, axis=0)).sum(1) == 1)
    # the position counts, not the origin: every agent moved by one block along x walks through
    # the neighbouring block the same way (edge by edge; the block itself may be turned)
    st = o.get_state()
    st[:, 0, 0] += 16.0
    o.set_state(st)
    o.regroup(2.0, 0.0)
    order2 = o.get_groups()
    walk2 = np.floor((org[order2[order2 != 64], 0:2] + np.array([16.0, 0.0])) / 2.0).astype(int)
    assert walk2[:, 0].min() == 16 and len({tuple(c) for c in walk2}) == 64
    assert np.all(np.abs(np.diff(walk2, axis=0)).sum(1) == 1)
    # floor, not truncation: an agent at x = -0.1 lies in cell -1, not in cell 0 with the one at +0.1
    rob2, sc2 = _sphere_agents(3, [(0.1, 0.5, 0.0), (-0.1, 0.5, 0.0), (0.3, 0.5, 0.0)], 2)
    o2 = oracle.OracleSim(sc2)
    o2.set_state(np.repeat(scenes.rest_state(rob2), 3, axis=0))
    o2.regroup(2.0, 0.0)
    g = o2.get_groups().tolist()
    assert abs(g.index(0) - g.index(2)) == 1 and g.index(1) in (0, 2)


def test_regrouping_puts_wandering_neighbours_into_one_group():
    """Sixty-four agents numbered at random over a field in tight clumps of four, 30 m between
    clumps.  In their own order almost every close pair is split between groups; after regrouping
    with cells larger than a clump and smaller than the clump distance every clump that does not
    straddle a cell border is one group (counted by brute force here), and a step then finds
    contacts between clump mates only."""
    rng = np.random.default_rng(11)
    centres = np.stack(np.meshgrid(np.arange(4) * 30.0 + 7.0, np.arange(4) * 30.0 + 9.0), -1).reshape(16, 2)
    pts = np.repeat(centres, 4, axis=0) + np.tile(np.array([[0, 0], [0.19, 0], [0, 0.19], [0.19, 0.19]]), (16, 1))
    perm = rng.permutation(64)
    org = np.zeros((64, 3)); org[perm, 0:2] = pts          # agent perm[k] stands at point k
    rob, sc = _sphere_agents(64, org, 4)
    o = oracle.OracleSim(sc)
    o.set_state(np.repeat(scenes.rest_state(rob), 64, axis=0))
    near, split = o.count_near_pairs(0.5)
    assert near == 16 * 6 and split > 80
    o.regroup(8.0, 0.5)
    groups = o.get_groups().reshape(16, 4)
    clump_of = np.empty(64, int); clump_of[perm] = np.arange(64) // 4
    assert all(len(set(clump_of[g])) == 1 for g in groups)
    assert o.count_near_pairs(0.5) == (96, 0)
    o.step(None, 1.0 / 240.0, 1, 4)
    pc = o.get_pair_contacts()
    assert len(pc) == 16 * 4    # the four sides of each square touch (0.19 < 0.2), the diagonals do not
    assert np.array_equal(clump_of[pc["env_a"]], clump_of[pc["env_b"]])


def test_regrouping_grows_groups_from_neighbours_inside_a_window():
    """Eight agents in one cell (one window), reach 1 m.  Along x: agents 0..7 at
    0, 10, 0.5, 10.4, 20, 30, 20.9, 0.9 (order inside the cell: by number).
    Groups of 2.  Clusters: 0 takes its first free neighbour 2 (7, also within reach, comes later
    in the order) and is full; 1 takes 3; 4 takes 6; 5 and 7 have no free neighbour.  Layout:
    [0 2] [1 3] [4 6] then the free agents [5 7].
    Groups of 4.  Clusters: {0, 2, 7} (7 is a neighbour of both), {1, 3}, {4, 6}.  Layout: 0 2 7,
    then {1, 3} does not fit any more: the gap is closed with the free agent 5, [0 2 7 5]; then
    [1 3 4 6]."""
    xs = [0.0, 10.0, 0.5, 10.4, 20.0, 30.0, 20.9, 0.9]
    rob, sc = _sphere_agents(8, [(x, 1.0, 0.0) for x in xs], 2)
    o = oracle.OracleSim(sc)
    o.set_state(np.repeat(scenes.rest_state(rob), 8, axis=0))
    o.regroup(100.0, 1.0)
    assert o.get_groups().tolist() == [0, 2, 1, 3, 4, 6, 5, 7]
    assert o.count_near_pairs(1.0) == (5, 2)     # 0-2, 0-7, 2-7, 1-3, 4-6; apart: 0-7, 2-7
    sc.params.group_size = 4
    o4 = oracle.OracleSim(sc)
    o4.set_state(np.repeat(scenes.rest_state(rob), 8, axis=0))
    o4.regroup(100.0, 1.0)
    assert o4.get_groups().tolist() == [0, 2, 7, 5, 1, 3, 4, 6]
    assert o4.count_near_pairs(1.0) == (5, 0)
    # Agents 0..4 in a row 0.9 m apart plus a far pair 5, 6, groups of 4: clusters {0,1,2,3}
    # (full; 4's only neighbour 3 is taken, so 4 stays free) and {5, 6}.  Layout [0 1 2 3] [5 6 4]
    rob7, sc7 = _sphere_agents(7, [(0.9 * k, 1.0, 0.0) for k in range(5)] + [(50.0, 1.0, 0.0), (50.5, 1.0, 0.0)], 4)
    o7 = oracle.OracleSim(sc7)
    o7.set_state(np.repeat(scenes.rest_state(rob7), 7, axis=0))
    o7.regroup(1000.0, 1.0)
    assert o7.get_groups().tolist() == [0, 1, 2, 3, 5, 6, 4]
    # groups of 3 on the same row: clusters {0,1,2}, {3,4}, {5,6}; {5,6} does not fit behind {3,4},
    # no free agent: its first member closes the gap: [0 1 2] [3 4 5] [6]
    sc7.params.group_size = 3
    o3 = oracle.OracleSim(sc7)
    o3.set_state(np.repeat(scenes.rest_state(rob7), 7, axis=0))
    o3.regroup(1000.0, 1.0)
    assert o3.get_groups().tolist() == [0, 1, 2, 3, 4, 5, 6]
