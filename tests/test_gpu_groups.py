"""GPU parity of the interaction groups chosen from positions (one shared scene: Section 3.1, last
paragraph; colliding agents of the flagrun tasks: Section 4.1) against the fp64 oracle: the order
of the agents and the pair counts bit for bit, stepping with regrouped agents to the same bars as
with consecutive groups, and the indexing by agent checked against a scene stored in another order."""
import dataclasses

import numpy as np
import pytest

import oracle
import scenes
from helpers import gate_after_10_steps, rel_err4
from test_gpu_pairs import assert_same_pair_sets, rel_err, TOL_1, TOL_10

pytestmark = pytest.mark.gpu


def _P():
    import paper_1810_05762_amd as P
    return P


def _crowd_scene(n, group, side, terrain="plane", seed=3, warm=0.0, min_dist=0.55):
    """n humanoids standing at random in a square of `side` metres (at least min_dist apart), numbered
    in no spatial order: consecutive numbers are mostly far apart."""
    rob = scenes.make_humanoid()
    p = scenes.SimParams(self_collide=1, group_size=group, warm_start=warm)
    t = scenes.make_plane() if terrain == "plane" else scenes.make_heightfield(seed=1003)
    sc = scenes.make_scene(rob, t, n, seed=21, params=p)
    rng = np.random.default_rng(seed)
    pts, tries = [], 0
    while len(pts) < n:
        tries += 1
        assert tries < 5000 * n, "the square is too small for that many agents"
        c = rng.uniform(0.0, side, size=2)
        if all(np.hypot(*(c - q)) >= min_dist for q in pts):
            pts.append(c)
    base = np.asarray(t.origin[:2], np.float64) + 9.0 if terrain != "plane" else np.zeros(2)   # well inside the field
    org = np.zeros((n, 3))
    org[:, 0:2] = np.array(pts) + base
    if terrain != "plane":
        org[:, 2] = [scenes.terrain_height_max_near(t, x, y, 0.5) for x, y in org[:, 0:2]]
    sc.env_origins = org.astype(np.float32).astype(np.float64)
    return rob, sc


def test_order_of_the_agents_and_pair_counts_equal_the_oracle():
    P = _P()
    n = 333
    rob, sc = _crowd_scene(n, 4, 14.0)
    sim, ref = P.Sim(sc), oracle.OracleSim(sc, threads=8)
    sim.reset(5)
    ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    assert np.array_equal(sim.get_groups(), np.arange(n))
    near0 = sim.count_near_pairs(1.0)
    assert near0 == ref.count_near_pairs(1.0) and near0[0] > 100 and near0[1] > 0.9 * near0[0]
    for cell in (2.0, 0.7, 50.0):
        sim.regroup(cell, 1.0); ref.regroup(cell, 1.0)
        pe = sim.get_groups()
        assert sorted(pe.tolist()) == list(range(n))
        assert np.array_equal(pe, ref.get_groups()), cell
        assert sim.count_near_pairs(1.0) == ref.count_near_pairs(1.0)
    sim.regroup(2.0, 1.0); ref.regroup(2.0, 1.0)
    near1 = sim.count_near_pairs(1.0)
    print(f"pairs within 1 m: {near0[0]}, kept apart by the groups: {near0[1]} in number order, {near1[1]} after regrouping")
    assert near1[0] == near0[0] and near1[1] < 0.75 * near0[1]
    sim.set_groups(None)
    assert np.array_equal(sim.get_groups(), np.arange(n))
    sim.close()


@pytest.mark.parametrize("group,terrain,warm", [(4, "plane", 0.0), (16, "plane", 0.0), (4, "heightfield", 0.8)])
def test_crowd_with_regrouping_every_few_steps(group, terrain, warm):
    """A crowd of falling humanoids, regrouped every five steps on both sides: the orders agree
    (from the GPU's own fp32 state), single substeps from identical states agree in contact sets
    (reported by agent number) and state, then ten free steps with one regrouping in between."""
    P = _P()
    n = 118
    rob, sc = _crowd_scene(n, group, 7.0, terrain, warm=warm)
    sim, ref = P.Sim(sc), oracle.OracleSim(sc, threads=8)
    sim.reset(5)
    sim.record_contacts(True)
    dt, sub, its = float(np.float32(1.0 / 60.0)), 4, 20
    h = dt / sub
    total = inter = far = 0

    def sync_ref():
        st = sim.get_state()
        sim.set_state(st)                                  # (also clears what the warm start keeps)
        ref.set_state(st.cpu().numpy().astype(np.float64))

    for s in range(40):
        a = scenes.actions_for_step(9, s, n, rob.n_dofs)
        if s % 5 == 0:
            sync_ref()
            sim.regroup(1.5, 1.2); ref.regroup(1.5, 1.2)
            assert np.array_equal(sim.get_groups(), ref.get_groups())
        if s % 5 == 4:
            sync_ref()
            sim.step(a, h, 1, its); ref.step(a, h, 1, its)
            pg, dropped = sim.get_pair_contacts()
            po = ref.get_pair_contacts()
            assert dropped == 0
            assert_same_pair_sets(pg, po)
            cg, co = sim.get_contacts(), ref.get_contacts()
            assert all(np.array_equal(cg[f], co[f]) for f in ("active", "kind", "feat"))
            e = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
            assert e.max() <= TOL_1, (s, e.max())
            total += len(po)
            between = po["env_a"] != po["env_b"]
            inter += int(between.sum())
            far += int((np.abs(po["env_a"] - po["env_b"])[between] >= group).sum())
        else:
            sim.step(a, dt, sub, its)
    # agents met, and mostly agents whose numbers are further apart than a consecutive group reaches
    assert inter > 10 and far > 0.5 * inter, (total, inter, far)
    # ten free steps, substep by substep so that every contact set is seen: an agent whose sets
    # ever differed (equal distances within rounding pick another terrain feature, a capsule pair
    # at the margin), and from then on everybody who shares a group with it, is on another branch
    sync_ref()
    errs = {}
    forked = np.zeros(n, bool)
    for s in range(10):
        a = scenes.actions_for_step(9, 40 + s, n, rob.n_dofs)
        if s == 5:
            # both sides would regroup from their own states, which differ by rounding: the orders
            # may differ where an agent stands on a cell border, so the oracle takes the GPU's order
            sim.regroup(1.5, 1.2)
            ref.set_groups(sim.get_groups())
        for _ in range(sub):
            sim.step(a, h, 1, its); ref.step(a, h, 1, its)
            cg, co = sim.get_contacts(), ref.get_contacts()
            forked |= np.any([(cg[f] != co[f]).any(1) for f in ("active", "kind", "feat")], axis=0)
            pg, po = sim.get_pair_contacts()[0], ref.get_pair_contacts()
            ids = lambda r: set(zip(r["env_a"].tolist(), r["body_a"].tolist(), r["env_b"].tolist(), r["body_b"].tolist()))
            for ea, _ba, eb, _bb in ids(pg) ^ ids(po):
                forked[ea] = forked[eb] = True
            members = sim.get_groups()
            for g0 in range(0, n, group):
                m = members[g0:g0 + group]
                if forked[m].any():
                    forked[m] = True
        if s in (0, 9):
            errs[s + 1] = rel_err4(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
    print(f"crowd, group {group} {terrain}: {total} pair contacts sampled ({inter} between agents, {far} beyond number distance {group}); "
          f"1 step max {errs[1].max():.2e}")
    assert errs[1].max() <= TOL_1
    # (on the heightfield most fallen humanoids meet equal distances to two terrain features
    #  sooner or later, and a fork counts for the whole group from then on)
    gate_after_10_steps(errs[10], forked, label=f"crowd, group {group} {terrain}: ", min_same=8 if terrain != "plane" else None,
                        interacting=True)
    assert np.median(errs[10].max(1)) <= TOL_1
    sim.check(); sim.close()


def test_places_by_hand_equal_the_same_scene_stored_in_that_order():
    """Scene A holds the agents in the order of a random permutation of scene B's; B with that
    permutation as its places runs the very same workgroups as A in its own order: states,
    observations, rewards and contact records agree bit for bit, agent for agent (heightfield,
    warm start, height-map observation; actions permuted alike)."""
    P = _P()
    n, group = 52, 4
    rob, scb = _crowd_scene(n, group, 5.0, "heightfield", warm=0.8)
    scb.params = dataclasses.replace(scb.params, height_map=1)
    perm = np.random.default_rng(8).permutation(n).astype(np.int32)     # place k of B holds agent perm[k]
    sca = dataclasses.replace(scb, env_origins=scb.env_origins[perm].copy())
    A, Bs = P.Sim(sca), P.Sim(scb)
    Bs.reset(3)
    stb = Bs.get_state()
    A.set_state(stb[perm.astype(np.int64)].contiguous())
    Bs.set_state(stb)
    Bs.set_groups(perm)
    assert np.array_equal(Bs.get_groups(), perm)
    A.record_contacts(True); Bs.record_contacts(True)
    for s in range(12):
        act = scenes.actions_for_step(4, s, n, rob.n_dofs)
        oa, ra, da = A.step_obs(act[perm], 1.0 / 60.0, 4, 20)
        ob, rb, db = Bs.step_obs(act, 1.0 / 60.0, 4, 20)
        assert np.array_equal(oa.cpu().numpy(), ob.cpu().numpy()[perm]), s
        assert np.array_equal(ra.cpu().numpy(), rb.cpu().numpy()[perm]) and np.array_equal(da.cpu().numpy(), db.cpu().numpy()[perm])
    assert np.array_equal(A.get_state().cpu().numpy(), Bs.get_state().cpu().numpy()[perm])
    ca, cb = A.get_contacts(), Bs.get_contacts()
    assert all(np.array_equal(ca[f], cb[f][perm]) for f in ca.dtype.names)
    pa, _ = A.get_pair_contacts()
    pb, _ = Bs.get_pair_contacts()
    assert len(pa) == len(pb) and len(pa) > 0
    assert np.array_equal(perm[pa["env_a"]], pb["env_a"]) and np.array_equal(perm[pa["env_b"]], pb["env_b"])
    for f in ("body_a", "body_b", "s", "t", "d", "w"):
        assert np.array_equal(pa[f], pb[f])
    ja, sa_ = (x.cpu().numpy() for x in A.get_kept_impulses())
    jb, sb_ = (x.cpu().numpy() for x in Bs.get_kept_impulses())
    assert np.array_equal(ja, jb[perm]) and np.array_equal(sa_, sb_[perm]) and np.abs(ja).max() > 0
    A.close(); Bs.close()


def test_group_calls_check_their_arguments():
    P = _P()
    rob, sc = _crowd_scene(20, 4, 4.0)
    sim = P.Sim(sc)
    with pytest.raises(P.SimError):
        sim.set_groups(np.zeros(20, np.int32))                   # not a permutation
    with pytest.raises(P.SimError):
        sim.set_groups(np.arange(20, dtype=np.int32) + 1)        # out of range
    assert np.array_equal(sim.get_groups(), np.arange(20))       # nothing was taken over
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(P.SimError):
            sim.regroup(bad, 1.0)
    for bad in (-1.0, float("nan"), float("inf")):
        with pytest.raises(P.SimError):
            sim.regroup(1.0, bad)
    sim.close()
    lone = P.Sim(scenes.make_scene(rob, scenes.make_plane(), 20, params=scenes.SimParams(self_collide=1)))
    with pytest.raises(P.SimError):
        lone.regroup(1.0, 1.0)
    lone.close()


def test_regrouping_and_step_captured_in_one_graph_replay_like_eager_calls():
    """sim_regroup enqueues kernels only (no allocation, no clearing call, no synchronisation), so
    it can be captured in a HIP graph together with the step that follows it: every replay, with
    eager calls on the same sim in between, equals the eager pair of calls bit for bit, places
    included."""
    import torch
    P = _P()
    n = 96
    rob, sc = _crowd_scene(n, 4, 9.0, warm=0.8)

    def make():
        sim = P.Sim(sc); sim.reset(7)
        return sim

    dt = float(np.float32(1.0 / 60.0))
    acts = [torch.as_tensor(scenes.actions_for_step(5, s, n, rob.n_dofs)).cuda() for s in range(12)]
    eager, graphed = make(), make()
    abuf = acts[0].clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.regroup(1.5, 1.2)
        graphed.step_obs(abuf, dt, 4, 20)
    assert torch.equal(graphed.get_state(), eager.get_state())      # capturing runs nothing
    for k in range(12):
        abuf.copy_(acts[k])
        g.replay()
        torch.cuda.synchronize()
        eager.regroup(1.5, 1.2)
        eo, er, ed = eager.step_obs(acts[k], dt, 4, 20)
        assert torch.equal(graphed.obs, eo) and torch.equal(graphed.reward, er) and torch.equal(graphed.done, ed), k
        assert torch.equal(graphed.get_state(), eager.get_state())
        assert np.array_equal(graphed.get_groups(), eager.get_groups())
    assert not np.array_equal(eager.get_groups(), np.arange(n))
    graphed.check(); eager.check()
    graphed.close(); eager.close()


def test_full_size_crowd_regrouped_order_and_sampled_groups_match_the_oracle():
    """4096 humanoids in one square on the plane at 0.3 agents per square metre, numbered in no
    spatial order, in the launch shape `bench.py --crowd 0.3` times.  After the robots have fallen
    over each other: the whole order of the agents and the pair counts equal the oracle's bit for
    bit; then 24 sampled groups (those with the most contacts between agents among them) are
    recomputed by the oracle as a small scene holding their agents in place order."""
    P = _P()
    n, group = 4096, 4
    rob = scenes.make_humanoid()
    p = scenes.SimParams(self_collide=1, group_size=group)
    sc = scenes.make_scene(rob, scenes.make_plane(), n, seed=21, params=p)
    sc.env_origins = scenes.crowd_origins(n, 0.3, 1002)
    sim = P.Sim(sc)
    sim.reset(5)
    sim.record_contacts(True)
    dt, sub, its = float(np.float32(1.0 / 60.0)), 4, 20
    for s in range(60):
        if s % 10 == 0:
            sim.regroup(2.4, 1.2)
        sim.step(scenes.actions_for_step(9, s, n, rob.n_dofs), dt, sub, its)
    # order and counts of the whole crowd
    full = oracle.OracleSim(sc, threads=8)
    full.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    sim.regroup(2.4, 1.2); full.regroup(2.4, 1.2)
    places = sim.get_groups()
    assert np.array_equal(places, full.get_groups())
    near = sim.count_near_pairs(1.2)
    assert near == full.count_near_pairs(1.2) and near[0] > 500 and near[1] < 0.25 * near[0]
    # sampled groups, stepped by the oracle on their own
    sim.step(scenes.actions_for_step(9, 60, n, rob.n_dofs), dt, sub, its)
    pg, dropped = sim.get_pair_contacts(cap=400000)
    place_of = np.empty(n, np.int64); place_of[places] = np.arange(n)
    between = pg[pg["env_a"] != pg["env_b"]]
    busy = np.bincount(place_of[between["env_a"]] // group, minlength=n // group)
    groups = np.argsort(-busy, kind="stable")[:20].tolist() + [0, 1, n // group - 2, n // group - 1]
    pick = np.concatenate([places[g * group:(g + 1) * group] for g in groups])
    small = scenes.make_scene(rob, scenes.make_plane(), len(pick), seed=21, params=p)
    small.env_origins = sc.env_origins[pick].copy()
    ref = oracle.OracleSim(small, threads=8)
    ref.set_state(sim.get_state().cpu().numpy()[pick].astype(np.float64))
    errs = {}
    for s in range(10):
        a = scenes.actions_for_step(9, 61 + s, n, rob.n_dofs)
        sim.step(a, dt, sub, its); ref.step(a[pick], dt, sub, its)
        if s in (0, 9):
            errs[s + 1] = rel_err(sim.get_state().cpu().numpy()[pick].astype(np.float64), ref.get_state())
    print(f"full-size crowd: {near[0]} agent pairs within 1.2 m, {near[1]} of them in different groups; {len(pg)} capsule contacts, "
          f"{len(between)} between agents, {busy[groups[0]]} in the busiest group; sampled groups: 1 step {errs[1].max():.2e}, "
          f"10 steps median {np.median(errs[10]):.2e} max {errs[10].max():.2e}")
    assert sim.launch_info()["envs_per_block"] == 16 and dropped == 0 and len(between) > 500 and busy[groups[0]] >= 3
    assert errs[1].max() <= TOL_1
    assert np.median(errs[10]) <= TOL_1 and errs[10].max() <= TOL_10
    sim.check(); sim.close()
