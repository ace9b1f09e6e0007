"""GPU parity of the task logic around the step (Section 4.1): pushes, grace period, flagrun
targets, episode limit and the reset of finished envs, against the oracle through the C ABI.
Integer outcomes (counters, push frames, episode indices, done away from its threshold) must be
equal; forces, targets and reset states agree to fp32 rounding."""
import dataclasses

import numpy as np
import pytest

import oracle
import scenes
from test_gpu_parity import rel_err

pytestmark = pytest.mark.gpu
DT = float(np.float32(1.0 / 60.0))


def _P():
    import paper_1810_05762_amd as P
    return P


def test_pushes_match_the_oracle_on_free_bodies():
    P = _P()
    n = 300
    rob = scenes.make_single(radius=0.1, pos=(0.0, 0.0, 1.0), mass=2.0)
    sc = scenes.make_scene(rob, scenes.make_plane(), n,
                           params=scenes.SimParams(gravity=(0.0, 0.0, 0.0), contacts=0, max_ang_vel=1e30))
    tp = scenes.TaskParams(fall_grace_frames=10 ** 6, target_period=0, push_min_frames=3, push_max_frames=7,
                           auto_reset=0, push_min_newton=2.0, push_max_newton=4.0, seed=5)
    sim = P.Sim(sc); sim.set_state(scenes.rest_state(rob, n)); sim.set_task(tp)
    ref = oracle.OracleSim(sc); ref.set_state(scenes.rest_state(rob, n)); ref.set_task(tp)
    n_push = 0
    for f in range(40):
        sim.step(None, DT, 2, 4); ref.step(None, DT, 2, 4)
        c, _, push = sim.get_task_state()
        assert np.array_equal(c.cpu().numpy(), ref.get_task_state()[0])
        pg, po = push.cpu().numpy(), ref.get_last_push()
        assert np.array_equal(np.abs(pg).sum(1) > 0, np.abs(po).sum(1) > 0)
        assert np.abs(pg - po).max() < 2e-6 * 4.0
        n_push += int((np.abs(po).sum(1) > 0).sum())
    assert n_push > 5 * n
    assert np.abs(sim.get_state().cpu().numpy()[:, 0, 7:10] - ref.get_state()[:, 0, 7:10]).max() < 1e-5
    sim.close()


def test_grace_targets_and_auto_reset_match_the_oracle_step_by_step():
    """Humanoids on the heightfield under random actions fall within a second; with a grace of 3
    frames and auto-reset most envs go through several episodes in 70 frames."""
    P = _P()
    n = 96
    sc, cfg = scenes.config_scene(3, num_envs=n)
    tp = scenes.TaskParams(fall_grace_frames=3, target_period=11, push_min_frames=5, push_max_frames=9, auto_reset=1,
                           target_reach=1.0, target_radius=100.0, push_min_newton=20.0, push_max_newton=50.0, seed=21)
    sim = P.Sim(sc); sim.reset(cfg["seed"]); sim.set_task(tp)
    ref = oracle.OracleSim(sc, threads=8)
    ref.set_state(sim.get_state().cpu().numpy().astype(np.float64)); ref.set_task(tp)
    c0, t0, _ = sim.get_task_state()
    assert np.array_equal(c0.cpu().numpy(), ref.get_task_state()[0])
    assert np.abs(t0.cpu().numpy() - ref.get_task_state()[1]).max() < 1e-3     # fp32 cos/sin at 100 m
    steps = np.zeros(n, np.int32)
    episodes_ended = redraws = pushes = 0
    term = sc.robot.term_height
    for f in range(70):
        # both sides continue from the GPU's state of the previous frame
        ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
        c, t, _ = sim.get_task_state()
        ref.set_task_state(c.cpu().numpy(), t.cpu().numpy().astype(np.float64))
        ref.set_step_count(steps); sim.set_step_count(steps)
        act = scenes.actions_for_step(cfg["seed"], f, n, sc.robot.n_dofs)
        og, rg, dg = [x.cpu().numpy().copy() for x in sim.step_obs(act, DT, cfg["substeps"], cfg["iterations"])]
        ref.step(act, DT, cfg["substeps"], cfg["iterations"])
        oo, ro, do = ref.get_obs()
        cg, tg, pg = [x.cpu().numpy() for x in sim.get_task_state()]
        co, to = ref.get_task_state()
        po = ref.get_last_push()
        assert np.abs(pg - po).max() < 1e-4 and np.array_equal(np.abs(pg).sum(1) > 0, np.abs(po).sum(1) > 0)
        pushes += int((np.abs(po).sum(1) > 0).sum())
        # the height decides an integer: compare away from the threshold (the oracle's obs[0] of an env
        # that was reset is already the new episode's, so take the pre-reset height from done itself)
        same = dg == do
        assert same.mean() > 0.97, f
        ok = same
        assert np.array_equal(cg[ok], co[ok]), f
        assert np.abs(tg[ok] - to[ok]).max() < 2e-3
        ended = ok & (do == 1)
        episodes_ended += int(ended.sum())
        redraws += int((co[ok, 1] == 0).sum())
        sg, so = sim.get_state().cpu().numpy().astype(np.float64), ref.get_state()
        e = rel_err(sg, so).max(1)
        assert e[ended].max(initial=0.0) < 1e-5                          # the reset recipe, fp32 against fp64
        assert np.quantile(e[ok & ~ended], 0.95) < 1e-4 and e[ok & ~ended].max() < 1e-3
        assert np.abs(og[ended] - oo[ended]).max(initial=0.0) < 2e-4     # first observation of the new episode
        assert np.abs(rg[ok] - ro[ok]).max() < 0.25 and np.median(np.abs(rg[ok] - ro[ok])) < 1e-4
        steps = np.where(dg == 1, 0, steps + 1).astype(np.int32)
    assert episodes_ended > n and redraws > 3 * n and pushes > 3 * n
    sim.close()


def test_task_outcomes_do_not_depend_on_the_narrow_launch_shapes():
    P = _P()
    sc, cfg = scenes.config_scene(3, num_envs=50)
    tp = scenes.TaskParams(fall_grace_frames=2, target_period=7, push_min_frames=4, push_max_frames=6, auto_reset=1, seed=3)
    outs = []
    for epb in (8, 5):
        sim = P.Sim(sc); sim.set_envs_per_block(epb); sim.reset(2); sim.set_task(tp)
        for f in range(50):
            obs, rew, done = sim.step_obs(scenes.actions_for_step(6, f, 50, 21), DT, 4, 20)
        outs.append([x.cpu().numpy().copy() for x in (obs, rew, done, sim.get_state(), *sim.get_task_state())])
        sim.close()
    assert all(np.array_equal(a, b) for a, b in zip(*outs))
    assert (outs[0][4][:, 3] >= 1).mean() > 0.8             # nearly every env has finished an episode


def test_task_description_is_validated_and_can_be_switched_off():
    P = _P()
    sc, cfg = scenes.config_scene(0, num_envs=16)
    sim = P.Sim(sc); sim.reset(1)
    for bad in (dict(push_min_frames=0, push_max_frames=5), dict(push_min_frames=9, push_max_frames=5),
                dict(fall_grace_frames=-1), dict(target_radius=-1.0), dict(push_min_newton=3.0, push_max_newton=1.0)):
        with pytest.raises(P.SimError) as ei:
            sim.set_task(dataclasses.replace(scenes.TaskParams(), **bad))
        assert ei.value.code == -1
    a = P.Sim(sc); a.reset(1)
    sim.set_task(scenes.TaskParams(target_period=0)); sim.set_task(None)     # on (targets kept), then off: same as never on
    for f in range(5):
        act = scenes.actions_for_step(1, f, 16, 8)
        sim.step(act, DT, 2, 8); a.step(act, DT, 2, 8)
    assert np.array_equal(sim.get_state().cpu().numpy(), a.get_state().cpu().numpy())
    assert all(np.array_equal(x.cpu().numpy(), y.cpu().numpy()) for x, y in zip(sim.get_obs(), a.get_obs()))
    sim.close(); a.close()
