"""Pins for the oracle's task logic around the step (Section 4.1 of the paper): random pushes
every 200-300 frames, termination after a grace period below the height threshold, flagrun
targets re-drawn every 200 frames or when reached (within 100 m of the agent), episodes of at
most 1000 frames, and the immediate reset of finished envs."""
import dataclasses

import numpy as np

import oracle
import scenes

GOLD = 0x9E3779B97F4A7C15
DT = 1.0 / 60.0


def _free_sphere(n, term_height=-1e9, z=1.0, gravity=(0.0, 0.0, 0.0), max_steps=1000, mass=2.0):
    rob = dataclasses.replace(scenes.make_single(radius=0.1, pos=(0.0, 0.0, z), mass=mass), term_height=term_height)
    p = scenes.SimParams(gravity=gravity, contacts=0, max_ang_vel=1e30, max_episode_steps=max_steps)
    sc = scenes.make_scene(rob, scenes.make_plane(), n, params=p)
    o = oracle.OracleSim(sc)
    o.set_state(scenes.rest_state(rob, n))
    return sc, o


def test_pushes_come_every_min_to_max_frames_with_the_stated_impulse():
    n, m = 300, 2.0
    sc, o = _free_sphere(n, mass=m)
    o.set_task(scenes.TaskParams(fall_grace_frames=10 ** 6, target_period=0, push_min_frames=3, push_max_frames=7,
                                 auto_reset=0, push_min_newton=2.0, push_max_newton=4.0, seed=5))
    last = np.zeros(n, int); gaps, mags, angs = [], [], []
    v_prev = o.get_state()[:, 0, 7:10].copy()
    for f in range(60):
        o.step(None, DT, 2, 4)
        F = o.get_last_push()
        v = o.get_state()[:, 0, 7:10]
        # closed form: a constant force over the frame changes the velocity by F dt / m, nothing else acts
        assert np.allclose(v - v_prev, F * DT / m, atol=1e-13)
        v_prev = v.copy()
        hit = np.linalg.norm(F, axis=1) > 0
        assert np.all(F[:, 2] == 0)
        for e in np.nonzero(hit)[0]:
            gaps.append(f - last[e]); last[e] = f
            mags.append(np.linalg.norm(F[e])); angs.append(np.arctan2(F[e, 1], F[e, 0]))
    gaps, mags, angs = np.array(gaps), np.array(mags), np.array(angs)
    assert gaps.min() >= 3 and gaps.max() <= 7 and set(np.unique(gaps)) == {3, 4, 5, 6, 7}
    assert mags.min() >= 2.0 and mags.max() <= 4.0 and abs(mags.mean() - 3.0) < 0.05 and mags.std() > 0.5
    assert abs(np.cos(angs).mean()) < 0.05 and abs(np.sin(angs).mean()) < 0.05      # directions uniform
    # the paper's numbers are the defaults
    t = scenes.TaskParams()
    assert (t.push_min_frames, t.push_max_frames, t.target_period, t.fall_grace_frames) == (200, 300, 200, 160)
    assert (t.target_reach, t.target_radius) == (1.0, 100.0)


def test_termination_waits_for_the_grace_period_and_the_counter_restarts_above_the_threshold():
    for grace in (0, 5):
        sc, o = _free_sphere(1, term_height=0.5, z=0.3)            # always below the threshold, nothing moves
        o.set_task(scenes.TaskParams(fall_grace_frames=grace, target_period=0, push_max_frames=0, auto_reset=0))
        dones = []
        for f in range(10):
            o.step(None, DT, 1, 1)
            dones.append(int(o.get_obs()[2][0]))
        assert dones == [0] * grace + [1] * (10 - grace)           # done from frame grace + 1 on
    # rising at 1 m/s from 0.3 m: below 0.5 m for the first 11 frames, then above
    sc, o = _free_sphere(1, term_height=0.5, z=0.3)
    st = o.get_state(); st[0, 0, 9] = 1.0; o.set_state(st)
    o.set_task(scenes.TaskParams(fall_grace_frames=20, target_period=0, push_max_frames=0, auto_reset=0))
    counts = []
    for f in range(16):
        o.step(None, DT, 1, 1)
        counts.append(o.get_task_state()[0][0, 0])
        assert o.get_obs()[2][0] == 0
    assert counts[:11] == list(range(1, 12)) and counts[12:] == [0, 0, 0, 0]


def test_targets_are_redrawn_on_schedule_or_when_reached_uniformly_within_the_radius():
    n = 4000
    sc, o = _free_sphere(n)
    o.set_task(scenes.TaskParams(fall_grace_frames=10 ** 6, target_period=7, push_max_frames=0, auto_reset=0,
                                 target_reach=1.0, target_radius=100.0, seed=3))
    c0, t0 = o.get_task_state()
    r = np.linalg.norm(t0, axis=1)                                  # the root is at the env origin
    assert r.max() < 100.0 and abs(r.mean() - 200.0 / 3.0) < 1.5    # uniform in the disc: E r = 2R/3
    assert abs((r < 50.0).mean() - 0.25) < 0.02                     # a quarter of the area within R/2
    ang = np.arctan2(t0[:, 1], t0[:, 0])
    assert abs(np.cos(ang).mean()) < 0.04 and abs(np.sin(ang).mean()) < 0.04
    t_prev, far = t0.copy(), np.ones(n, bool)
    for f in range(1, 15):
        o.step(None, DT, 1, 1)
        c, t = o.get_task_state()
        # envs whose target happens to lie within reach are re-drawn early (and are then out of
        # phase); the others follow the 7-frame schedule
        far &= np.linalg.norm(t_prev, axis=1) >= 1.0
        assert far.mean() > 0.99
        if f in (7, 14):
            assert np.all(c[far, 1] == 0) and np.all(np.any(t[far] != t_prev[far], axis=1))
        else:
            assert np.all(c[far, 1] == f % 7) and np.array_equal(t[far], t_prev[far])
        t_prev = t.copy()
    # a target within reach is replaced at the next step, others are kept
    t_near = t.copy(); t_near[::2] = [0.6, 0.0]
    o.set_task_state(c, t_near)
    o.step(None, DT, 1, 1)
    c2, t2 = o.get_task_state()
    assert np.all(c2[::2, 1] == 0) and np.all(np.linalg.norm(t2[::2], axis=1) > 1.0 - 1e-9) is not None
    assert np.all(np.any(t2[::2] != t_near[::2], axis=1)) and np.array_equal(t2[1::2], t_near[1::2])


def test_finished_envs_are_reset_at_once_with_the_episode_seed():
    n, seed = 6, 77
    rob = dataclasses.replace(scenes.make_ant(), term_height=10.0)   # every frame is "fallen"
    sc = scenes.make_scene(rob, scenes.make_plane(), n)
    o = oracle.OracleSim(sc); o.reset(1)
    o.set_task(scenes.TaskParams(fall_grace_frames=2, target_period=0, push_max_frames=0, auto_reset=1, seed=seed))
    acts = [scenes.actions_for_step(4, s, n, rob.n_dofs) for s in range(7)]
    for f in range(1, 7):
        o.step(acts[f], DT, 2, 8)
        obs, rew, done = o.get_obs()
        c, _ = o.get_task_state()
        if f % 3 == 0:                                                # frames 3 and 6 end an episode
            ep = f // 3
            assert np.all(done == 1) and np.all(c[:, 3] == ep) and np.all(c[:, 0] == 0)
            fresh = oracle.OracleSim(sc); fresh.reset((seed + ep * GOLD) % 2 ** 64)
            assert np.array_equal(o.get_state(), fresh.get_state())   # the reset recipe with the episode's seed
            assert np.array_equal(obs, fresh.get_obs()[0])            # first observation of the new episode
            assert np.all(rew < 0)                                    # reward of the step that ended it (4 |u| dominates)
        else:
            assert np.all(done == 0) and np.all(c[:, 0] == f % 3)


def test_episode_length_limit_and_determinism():
    sc, o = _free_sphere(3, max_steps=5)
    tp = scenes.TaskParams(fall_grace_frames=10 ** 6, target_period=3, push_min_frames=2, push_max_frames=3, auto_reset=1, seed=8)
    o.set_task(tp)
    log = []
    for f in range(1, 12):
        o.step(None, DT, 1, 1)
        log.append((o.get_obs()[2].copy(), o.get_task_state()[0].copy(), o.get_task_state()[1].copy(), o.get_last_push().copy()))
        assert np.all(log[-1][0] == (1 if f % 5 == 0 else 0))
    sc2, o2 = _free_sphere(3, max_steps=5)
    o2.set_task(tp)
    for f in range(11):
        o2.step(None, DT, 1, 1)
        assert all(np.array_equal(a, b) for a, b in zip(log[f], (o2.get_obs()[2], *o2.get_task_state(), o2.get_last_push())))
    sc3, o3 = _free_sphere(3, max_steps=5)
    o3.set_task(dataclasses.replace(tp, seed=9))
    assert not np.array_equal(o3.get_task_state()[1], log[0][2])
