"""GPU parity of the capsule-capsule contacts (within an agent and between the agents of an
interaction group) against the fp64 oracle: contact sets and segment parameters bit for bit on
identical fp32 states, free-running states within the same bars as the terrain-only tests."""
import numpy as np
import pytest

import oracle
import scenes

pytestmark = pytest.mark.gpu

TOL_1, TOL_10 = 1e-4, 1e-3


def _P():
    import paper_1810_05762_amd as P
    return P


def rel_err(g, o):
    out = []
    for sl in (slice(0, 3), slice(3, 7), slice(7, 10), slice(10, 13)):
        d = np.abs(g[:, :, sl] - o[:, :, sl]).reshape(g.shape[0], -1).max(1)
        n = np.maximum(1.0, np.abs(o[:, :, sl]).reshape(g.shape[0], -1).max(1))
        out.append(d / n)
    return np.stack(out, 1).max(1)


def _key(r):
    return np.lexsort((r["body_b"], r["env_b"], r["body_a"], r["env_a"]))


def assert_same_pair_sets(pg, po):
    """Same contacts (as sets), same single-precision segment parameters."""
    assert len(pg) == len(po), (len(pg), len(po))
    pg, po = pg[_key(pg)], po[_key(po)]
    for f in ("env_a", "body_a", "env_b", "body_b"):
        assert np.array_equal(pg[f], po[f]), f
    assert np.array_equal(pg["s"].view(np.uint32) & 0x7fffffff, po["s"].view(np.uint32) & 0x7fffffff)
    assert np.array_equal(pg["t"].view(np.uint32) & 0x7fffffff, po["t"].view(np.uint32) & 0x7fffffff)
    np.testing.assert_allclose(pg["d"], po["d"], atol=2e-6)
    np.testing.assert_allclose(pg["w"], po["w"], atol=2e-3)   # (margin - d) / (margin / 2) with d to 2e-6


def _loose_pairs_scene(n_envs, seed):
    """Two free capsules per env in random poses, no gravity; axis distance 0.09 .. 0.16 m
    (radii 0.08 + 0.05: from 4 cm of overlap to 3 cm of clearance; a distance near zero would
    leave the contact normal undefined)."""
    from scipy.spatial.transform import Rotation
    rob = scenes.make_loose([(0.08, 0.5, 0, (0.0, 0.0, 5.0), 1.3), (0.05, 0.4, 1, (0.0, 0.0, 6.0), 0.7)])
    p = scenes.SimParams(gravity=(0.0, 0.0, 0.0), self_collide=1)
    sc = scenes.make_scene(rob, scenes.make_plane(), n_envs, params=p)
    rng = np.random.default_rng(seed)
    st = np.repeat(scenes.rest_state(rob), n_envs, axis=0)
    for e in range(n_envs):
        while True:
            q = rng.normal(size=(2, 4))
            q /= np.linalg.norm(q, axis=1, keepdims=True)
            x1 = st[e, 0, 0:3] + rng.normal(size=3) * 0.15
            ends = []
            for b, x in ((0, st[e, 0, 0:3]), (1, x1)):
                ax = Rotation.from_quat([q[b, 1], q[b, 2], q[b, 3], q[b, 0]]).as_matrix()[:, int(rob.axis[b])]
                ends += [x - rob.half_len[b] * ax, x + rob.half_len[b] * ax]
            d2, _, _ = oracle.segment_segment_f32(*ends)
            if 0.09 ** 2 < d2 < 0.16 ** 2:
                break
        st[e, :, 3:7] = q
        st[e, 1, 0:3] = x1
    st[:, :, 7:13] = rng.normal(size=(n_envs, 2, 6)) * np.array([0.5, 0.5, 0.5, 2, 2, 2])
    return rob, sc, st.astype(np.float32).astype(np.float64)


def test_two_capsules_contact_set_and_one_step_parity():
    P = _P()
    n = 203
    rob, sc, st = _loose_pairs_scene(n, 3)
    sim, ref = P.Sim(sc), oracle.OracleSim(sc, threads=8)
    sim.set_state(st); ref.set_state(st)
    sim.record_contacts(True)
    h = float(np.float32(1.0 / 240.0))
    sim.step(None, h, 1, 20); ref.step(None, h, 1, 20)
    pg, dropped = sim.get_pair_contacts()
    po = ref.get_pair_contacts()
    assert dropped == 0
    assert 40 < len(po) < n                      # some touch, some do not
    assert_same_pair_sets(pg, po)
    e = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
    print(f"two capsules: {len(po)} contacts, 1 substep max rel err {e.max():.2e}")
    assert e.max() <= TOL_1
    # the contacts did change the motion
    moved = np.abs(ref.get_state()[:, :, 7:13] - st[:, :, 7:13]).reshape(n, -1).max(1)
    assert (moved > 1e-2).sum() > 20
    sim.check(); sim.close()


def test_head_on_spheres_match_the_closed_form():
    """Perfectly inelastic impact: both spheres end with the centre-of-mass velocity."""
    P = _P()
    rob = scenes.make_loose([(0.1, 0.0, 0, (0.0, 0.0, 5.0), 1.0), (0.1, 0.0, 0, (0.25, 0.0, 5.0), 3.0)])
    sc = scenes.make_scene(rob, scenes.make_plane(), 5, params=scenes.SimParams(gravity=(0.0, 0.0, 0.0), self_collide=1))
    sim = P.Sim(sc)
    st = np.repeat(scenes.rest_state(rob), 5, axis=0)
    st[:, 0, 7], st[:, 1, 7] = 1.0, -0.5
    sim.set_state(st)
    for _ in range(12):
        sim.step(None, 1.0 / 60.0, 4, 4)
    s = sim.get_state().cpu().numpy()
    vcm = (1.0 * 1.0 - 3.0 * 0.5) / 4.0
    assert np.allclose(s[:, :, 7], vcm, atol=1e-5)
    assert np.allclose(s[:, 1, 0] - s[:, 0, 0], 0.2, atol=1e-5)
    sim.close()


def _humanoid_scene(n_envs, group, spacing, terrain="plane", self_collide=1):
    rob = scenes.make_humanoid()
    p = scenes.SimParams(self_collide=self_collide, group_size=group)
    t = scenes.make_plane() if terrain == "plane" else scenes.make_heightfield(seed=1003)
    return rob, scenes.make_scene(rob, t, n_envs, seed=21, params=p, spacing=spacing if group > 1 else None)


@pytest.mark.parametrize("group,terrain,n_envs", [(1, "plane", 37), (4, "plane", 38), (16, "plane", 40), (4, "heightfield", 38)])
def test_humanoids_with_collisions(group, terrain, n_envs):
    """Falling humanoids (random actions) with self-collision, in groups standing 0.6 m apart:
    contact sets of every substep on teacher-forced states, then ten free-running steps."""
    P = _P()
    rob, sc = _humanoid_scene(n_envs, group, 0.6, terrain)
    sim, ref = P.Sim(sc), oracle.OracleSim(sc, threads=8)
    sim.reset(5)
    sim.record_contacts(True)
    dt, sub, its = float(np.float32(1.0 / 60.0)), 4, 20
    h = dt / sub
    total = inter = 0
    for s in range(50):
        a = scenes.actions_for_step(9, s, n_envs, rob.n_dofs)
        if s % 5 == 4:
            # one substep on identical states: sets bit for bit, state to the one-step bar
            ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
            sim.step(a, h, 1, its); ref.step(a, h, 1, its)
            pg, dropped = sim.get_pair_contacts()
            po = ref.get_pair_contacts()
            assert dropped == 0
            assert_same_pair_sets(pg, po)
            cg, co = sim.get_contacts(), ref.get_contacts()
            assert all(np.array_equal(cg[f], co[f]) for f in ("active", "kind", "feat"))
            e = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
            assert e.max() <= TOL_1, (s, e.max())
            total += len(po); inter += int((po["env_a"] != po["env_b"]).sum())
        else:
            sim.step(a, dt, sub, its)
    assert total > 20
    if group > 1:
        assert inter > 5
    # free run from a contact-rich state
    ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    errs = {}
    for s in range(10):
        a = scenes.actions_for_step(9, 50 + s, n_envs, rob.n_dofs)
        sim.step(a, dt, sub, its); ref.step(a, dt, sub, its)
        if s in (0, 9):
            errs[s + 1] = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
    print(f"group {group} {terrain}: {total} pair contacts sampled ({inter} between agents); 1 step max {errs[1].max():.2e}, "
          f"10 steps median {np.median(errs[10]):.2e} p95 {np.quantile(errs[10], .95):.2e} max {errs[10].max():.2e}")
    assert errs[1].max() <= TOL_1
    # (contact sets are compared on the teacher-forced substeps above; in the free run every env
    #  has to stay within the ten-step tolerance, whatever its contact sets did)
    assert np.median(errs[10]) <= TOL_1 and errs[10].max() <= TOL_10
    sim.check(); sim.close()


@pytest.mark.parametrize("group,terrain,n_envs", [(4, "plane", 38), (1, "heightfield", 37), (16, "plane", 40)])
def test_humanoids_with_collisions_and_warm_start(group, terrain, n_envs):
    """Collisions and the warm start together (capsule-capsule contacts start every substep without
    impulses, joints and terrain slots from 0.8 of what they ended the last one with): substeps on
    identical states with identical kept impulses agree in contact sets, state and kept impulses;
    then ten free-running steps."""
    import dataclasses
    P = _P()
    rob, sc = _humanoid_scene(n_envs, group, 0.6, terrain)
    sc.params = dataclasses.replace(sc.params, warm_start=0.8)
    sim, ref = P.Sim(sc), oracle.OracleSim(sc, threads=8)
    sim.reset(5)
    sim.record_contacts(True)
    dt, sub, its = float(np.float32(1.0 / 60.0)), 4, 20
    h = dt / sub

    def kept():
        lj, ls = sim.get_kept_impulses()
        return lj.cpu().numpy().astype(np.float64), ls.cpu().numpy().astype(np.float64)

    def sync_ref():
        # same fp32 state, nothing kept on either side (set_state clears it)
        st = sim.get_state()
        sim.set_state(st)
        ref.set_state(st.cpu().numpy().astype(np.float64))

    total = 0
    for s in range(40):
        a = scenes.actions_for_step(9, s, n_envs, rob.n_dofs)
        if s % 5 == 4:
            # two substeps from identical states: the second one starts from kept impulses
            sync_ref()
            for rep in range(2):
                sim.step(a, h, 1, its); ref.step(a, h, 1, its)
                pg, dropped = sim.get_pair_contacts()
                po = ref.get_pair_contacts()
                assert dropped == 0
                if rep == 0:
                    assert_same_pair_sets(pg, po)   # (identical states only before the first substep)
                total += len(po)
            e = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
            assert e.max() <= TOL_1, (s, e.max())
            (gj, gs), (oj, os_) = kept(), ref.get_warm()
            scale = max(1.0, np.abs(oj).max(), np.abs(os_).max())
            assert max(np.abs(gj - oj).max(), np.abs(gs - os_).max()) / scale <= 1e-4
        else:
            sim.step(a, dt, sub, its)
    assert total > 20
    sync_ref()
    errs = {}
    for s in range(10):
        a = scenes.actions_for_step(9, 40 + s, n_envs, rob.n_dofs)
        sim.step(a, dt, sub, its); ref.step(a, dt, sub, its)
        if s in (0, 9):
            errs[s + 1] = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
    print(f"warm, group {group} {terrain}: {total} pair contacts sampled; 1 step max {errs[1].max():.2e}, "
          f"10 steps median {np.median(errs[10]):.2e} p95 {np.quantile(errs[10], .95):.2e} max {errs[10].max():.2e}")
    assert errs[1].max() <= TOL_1
    assert np.median(errs[10]) <= TOL_1 and errs[10].max() <= TOL_10
    sim.check(); sim.close()


def test_distant_groups_do_not_interact_and_variant_matches_plain_kernel():
    """With collisions compiled in but nothing close enough to touch, the states equal those of the
    plain kernel up to rounding (two instantiations of the kernel: the compiler may contract
    multiply-adds differently; the extra phase changes nothing else)."""
    P = _P()
    n = 35
    rob = scenes.make_humanoid()
    sc0 = scenes.make_scene(rob, scenes.make_plane(), n, seed=4, params=scenes.SimParams())
    sc1 = scenes.make_scene(rob, scenes.make_plane(), n, seed=4, params=scenes.SimParams(group_size=4))   # agents 5 m apart
    a0, a1 = P.Sim(sc0), P.Sim(sc1)
    a0.reset(3); a1.reset(3)
    a1.record_contacts(True)
    for s in range(8):
        a = scenes.actions_for_step(2, s, n, rob.n_dofs)
        a0.step(a, 1.0 / 60.0, 4, 20); a1.step(a, 1.0 / 60.0, 4, 20)
    assert len(a1.get_pair_contacts()[0]) == 0
    e = rel_err(a1.get_state().cpu().numpy().astype(np.float64), a0.get_state().cpu().numpy().astype(np.float64))
    assert e.max() <= TOL_1
    a0.close(); a1.close()


def test_parallel_and_degenerate_capsule_pairs():
    """Parallel capsules (the search starts from the middle of the first segment), a sphere
    against a capsule and a sphere against a sphere, side by side and touching."""
    P = _P()
    rob = scenes.make_loose([(0.05, 0.4, 0, (0.0, 0.0, 5.0), 1.0), (0.05, 0.3, 0, (0.05, 0.0, 6.0), 1.0),
                             (0.06, 0.0, 0, (0.0, 1.0, 5.0), 0.5), (0.04, 0.0, 0, (0.0, 1.0, 6.0), 0.8),
                             (0.05, 0.4, 2, (1.0, 0.0, 5.0), 1.0), (0.07, 0.0, 0, (1.0, 0.0, 6.0), 0.6)])
    sc = scenes.make_scene(rob, scenes.make_plane(), 19, params=scenes.SimParams(gravity=(0.0, 0.0, 0.0), self_collide=1))
    st = np.repeat(scenes.rest_state(rob), 19, axis=0)
    st[:, 1, 2] = 5.0 + 0.095          # parallel to body 0, 5 mm of overlap
    st[:, 3, 2] = 5.0 + 0.105          # sphere on sphere, 5 mm of clearance
    st[:, 5, 2] = 5.0 + 0.2 + 0.125    # sphere on the end of an upright capsule, 5 mm of clearance
    st[:, 1, 9], st[:, 3, 9], st[:, 5, 9] = -0.5, -2.0, -2.5
    sim, ref = P.Sim(sc), oracle.OracleSim(sc, threads=4)
    sim.set_state(st); ref.set_state(st)
    sim.record_contacts(True)
    h = float(np.float32(1.0 / 240.0))
    for k in range(6):
        ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))    # identical states every substep
        sim.step(None, h, 1, 10); ref.step(None, h, 1, 10)
        pg, dropped = sim.get_pair_contacts()
        po = ref.get_pair_contacts()
        assert dropped == 0 and len(po) == 3 * 19
        assert_same_pair_sets(pg, po)
        if k == 0:
            assert np.all(po["s"][po["body_a"] == 0] == 0.5)      # exactly parallel: middle of the first segment
        e = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
        assert e.max() <= TOL_1
    assert set(zip(po["body_a"].tolist(), po["body_b"].tolist())) == {(0, 1), (2, 3), (4, 5)}
    sim.check(); sim.close()


@pytest.mark.parametrize("E", [1, 2])
def test_more_contacts_than_a_workgroup_holds_keeps_the_closest(E):
    """Sixteen overlapping spheres per env: 120 touching pairs each against room for 96 per
    workgroup (of one env, and of two: 240 against 96, the key's env fields in play).  The 96 with
    the smallest (single-precision gap, key) stay, the same ones as in the oracle with the same
    bound, whichever wavefront found which pair first; the step then agrees to the one-step bar."""
    P = _P()
    rng = np.random.default_rng(2)
    rob = scenes.make_loose([(0.1, 0.0, 0, (3.0 * k, 0.0, 5.0), 1.0) for k in range(16)])
    n = 3 * E
    sc = scenes.make_scene(rob, scenes.make_plane(), n, params=scenes.SimParams(gravity=(0.0, 0.0, 0.0), self_collide=1))
    assert len(rob.collide_pairs) == 120
    st = np.repeat(scenes.rest_state(rob), n, axis=0)
    st[:, :, 0:3] = np.array([0.0, 0.0, 5.0]) + rng.normal(size=(n, 16, 3)) * 0.02
    st = st.astype(np.float32).astype(np.float64)
    cap = P.binding.SIM_PAIR_CAP
    sim, ref = P.Sim(sc), oracle.OracleSim(sc, threads=1)
    sim.set_envs_per_block(E)
    assert sim.launch_info()["envs_per_block"] == E
    ref.set_pair_cap(cap, E)
    sim.set_state(st); ref.set_state(st)
    sim.record_contacts(True)
    h = float(np.float32(1.0 / 240.0))
    for rep in range(2):   # twice: the second substep starts from what the first left in the workgroup's memory
        sim.step(None, h, 1, 4); ref.step(None, h, 1, 4)
        pg, dropped = sim.get_pair_contacts()
        po = ref.get_pair_contacts()
        assert len(pg) == 3 * cap and dropped == (rep + 1) * 3 * (120 * E - cap)
        assert_same_pair_sets(pg, po)
        e = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
        assert e.max() <= TOL_1, e.max()
        ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    assert ref.set_pair_cap(0, 1) == 2 * 3 * (120 * E - cap)
    sim.check(); sim.close()


def test_envs_per_block_must_hold_whole_groups():
    P = _P()
    rob, sc = _humanoid_scene(24, 4, 1.0)
    sim = P.Sim(sc)
    assert sim.launch_info()["envs_per_block"] % 4 == 0
    with pytest.raises(P.SimError):
        sim.set_envs_per_block(6)
    sim.set_envs_per_block(8)
    sim.step(None, 1.0 / 60.0, 2, 4)
    sim.check(); sim.close()


def test_task_logic_with_interacting_agents():
    """Pushes, grace period and auto-reset together with collisions in groups of 4: an agent that
    is reset reappears in its rest pose next to its neighbours.  Frame by frame from identical
    states: counters, episodes and done flags equal the oracle's (away from the fall threshold),
    states within the one-step bar, nothing dropped."""
    P = _P()
    n = 44
    rob, sc = _humanoid_scene(n, 4, 0.7, "plane")
    tp = scenes.TaskParams(fall_grace_frames=3, target_period=11, push_min_frames=5, push_max_frames=9, auto_reset=1,
                           push_min_newton=20.0, push_max_newton=50.0, seed=4)
    sim, ref = P.Sim(sc), oracle.OracleSim(sc, threads=8)
    sim.reset(8)
    ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    sim.set_task(tp); ref.set_task(tp)
    sim.record_contacts(True)
    dt = float(np.float32(1.0 / 60.0))
    steps = np.zeros(n, np.int32)
    episodes = contacts = 0
    for f in range(60):
        a = scenes.actions_for_step(3, f, n, rob.n_dofs)
        ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
        cg, tg, _ = sim.get_task_state()
        ref.set_task_state(cg.cpu().numpy(), tg.cpu().numpy().astype(np.float64))
        ref.set_step_count(steps); sim.set_step_count(steps)
        og, rg, dg = [x.cpu().numpy().copy() for x in sim.step_obs(a, dt, 4, 20)]
        ref.step(a, dt, 4, 20)
        oo, ro, do = ref.get_obs()
        same = dg == do
        assert same.mean() > 0.95, f
        assert np.array_equal(sim.get_task_state()[0].cpu().numpy()[same], ref.get_task_state()[0][same]), f
        e = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
        assert e[same].max() <= 2e-4, (f, e[same].max())
        pg, dropped = sim.get_pair_contacts()
        assert dropped == 0
        # (records of the fourth substep, whose start states already differ by rounding: the same
        # contacts with nearly the same segment parameters, apart from an occasional borderline one)
        po = ref.get_pair_contacts()
        kg = {(r["env_a"], r["body_a"], r["env_b"], r["body_b"]) for r in pg}
        ko = {(r["env_a"], r["body_a"], r["env_b"], r["body_b"]) for r in po}
        assert len(kg ^ ko) <= 1 + len(ko) // 20, (f, kg ^ ko)
        contacts += len(pg)
        episodes += int(do.sum())
        steps = np.where(dg == 1, 0, steps + 1).astype(np.int32)
    assert episodes > n // 2 and contacts > 50
    sim.check(); sim.close()


def test_full_size_collision_variant_sampled_groups_match_the_oracle():
    """4096 humanoids on the heightfield in groups of 4 standing 1 m apart, in the launch shape
    `bench.py --self-collide --group-size 4 --spacing 1.0` times; 16 sampled groups (64 envs) are
    recomputed by the oracle."""
    P = _P()
    n, group = 4096, 4
    rob, sc = _humanoid_scene(n, group, 1.0, "heightfield")
    sim = P.Sim(sc)
    sim.reset(5)
    sim.record_contacts(True)
    dt, sub, its = float(np.float32(1.0 / 60.0)), 4, 20
    for s in range(40):
        sim.step(scenes.actions_for_step(9, s, n, rob.n_dofs), dt, sub, its)
    groups = np.random.default_rng(1).choice(n // group, 16, replace=False)
    groups[:2] = (0, n // group - 1)
    pick = (groups[:, None] * group + np.arange(group)[None, :]).reshape(-1)
    _, small = _humanoid_scene(len(pick), group, 1.0, "heightfield")
    small.env_origins = sc.env_origins[pick].copy()
    ref = oracle.OracleSim(small, threads=8)
    ref.set_state(sim.get_state().cpu().numpy()[pick].astype(np.float64))
    errs = {}
    for s in range(10):
        a = scenes.actions_for_step(9, 40 + s, n, rob.n_dofs)
        sim.step(a, dt, sub, its); ref.step(a[pick], dt, sub, its)
        if s in (0, 9):
            errs[s + 1] = np.asarray(rel_err(sim.get_state().cpu().numpy()[pick].astype(np.float64), ref.get_state())).reshape(len(pick), -1).max(1)
    pg, dropped = sim.get_pair_contacts(cap=400000)
    info = sim.launch_info()
    print(f"full size, groups of 4: {len(pg)} capsule contacts in all, 1 step {errs[1].max():.2e}, 10 steps median {np.median(errs[10]):.2e} max {errs[10].max():.2e}")
    assert info["envs_per_block"] == 16 and dropped == 0 and len(pg) > n // 2
    assert errs[1].max() <= TOL_1
    assert np.median(errs[10]) <= TOL_1 and errs[10].max() <= TOL_10       # every sampled env
    g = sim.get_state().cpu().numpy()
    assert np.isfinite(g).all()
    sim.check(); sim.close()
