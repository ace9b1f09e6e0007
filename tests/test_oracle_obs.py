"""Pins for the oracle's observation vector (Table 2, "Ours": 76 numbers for the
humanoid), reward (Eq. 1-3), episode rules (Section 4.1) and seeded reset."""
import numpy as np
import pytest
from scipy.spatial.transform import Rotation

import oracle
import scenes
from helpers import free_params, rot_of, single_scene


def _recompute_obs_reward(scene, state, u, contacts, target, steps):
    """Independent numpy/scipy recomputation from a downloaded state."""
    rob = scene.robot
    D, F = rob.n_dofs, len(rob.feet)
    obs = np.zeros(11 + 3 * D + F)
    s = state[rob.root_body]
    Rr = rot_of(s[3:7])
    yaw, pitch, roll = Rr.as_euler("ZYX")
    height = s[2]
    if scene.terrain.kind == scenes.HEIGHTFIELD:
        t = scene.terrain
        wx, wy = s[0] + scene.env_origins[0, 0], s[1] + scene.env_origins[0, 1]
        ux, uy = (wx - t.origin[0]) / t.cell, (wy - t.origin[1]) / t.cell
        i, j = int(np.floor(ux)), int(np.floor(uy))
        fx, fy = ux - i, uy - j
        h = t.heights.astype(np.float64)
        if fx >= fy:   # barycentric interpolation on triangle (i,j),(i+1,j),(i+1,j+1)
            th = (1 - fx) * h[j, i] + (fx - fy) * h[j, i + 1] + fy * h[j + 1, i + 1]
        else:
            th = (1 - fy) * h[j, i] + fx * h[j + 1, i + 1] + (fy - fx) * h[j + 1, i]
        height = s[2] + scene.env_origins[0, 2] - th
    obs[0:3] = height, roll, pitch
    obs[3:6], obs[6:9] = s[7:10], s[10:13]
    to_t = np.asarray(target) - s[0:2]
    psi = np.arctan2(to_t[1], to_t[0]) - yaw
    obs[9:11] = np.sin(psi), np.cos(psi)
    n_lim = 0
    for j in range(rob.n_joints):
        a, b = rob.j_parent[j], rob.j_child[j]
        Ra = rot_of(state[a][3:7]) if a >= 0 else Rotation.identity()
        wa = state[a][10:13] if a >= 0 else np.zeros(3)
        phi = (Ra.inv() * rot_of(state[b][3:7])).as_rotvec()
        for k in range(3):
            if rob.j_mode[j, k] != scenes.HINGE:
                continue
            ai = rob.j_act[j, k]
            th = rob.j_axes[j, k] @ phi
            obs[11 + ai] = th
            obs[11 + D + ai] = Ra.apply(rob.j_axes[j, k]) @ (state[b][10:13] - wa)
            obs[11 + 2 * D + ai] = u[ai]
            n_lim += min(th - rob.j_lo[j, k], rob.j_hi[j, k] - th) <= 0
    # slots are laid out body by body: capsule 2 (+1 on a field), sphere 1
    per = [((3 if scene.terrain.kind == scenes.HEIGHTFIELD else 2) if rob.half_len[b] > 0 else 1)
           for b in range(rob.n_bodies)]
    start = np.concatenate([[0], np.cumsum(per)])
    n_feet = 0
    for f, fb in enumerate(rob.feet):
        c = contacts[start[fb]:start[fb + 1]]
        flag = bool(((c["active"] == 1) & (c["d"] <= 0.005)).any())
        obs[11 + 3 * D + f] = flag
        n_feet += flag
    speed = s[7:9] @ to_t / np.linalg.norm(to_t)
    ct = np.cos(psi)
    r_head = 1.0 if ct > 0.8 else ct / 0.8
    r_stand = 1.0 if Rr.apply([0, 0, 1.0])[2] > 0.93 else 0.0
    rew = (rob.alive_bonus + speed + 0.5 * r_head + 0.05 * r_stand - 4.0 * np.abs(u).sum()
           - 0.5 * (u ** 2).sum() - 0.2 * n_lim - 1.0 * n_feet)
    done = height < rob.term_height or steps >= scene.params.max_episode_steps
    return obs, rew, done


def test_observation_sizes_match_table_2():
    sc, _ = scenes.config_scene(2, num_envs=1)
    assert oracle.OracleSim(sc).obs_dim == 76        # 1+2+3+3+2+21+21+21+2
    sc, _ = scenes.config_scene(0, num_envs=1)
    assert oracle.OracleSim(sc).obs_dim == 39        # same groups, 8 DoF and 4 feet


@pytest.mark.parametrize("k", [0, 2, 3])
def test_obs_reward_done_match_independent_recomputation(k):
    sc, cfg = scenes.config_scene(k, num_envs=1)
    o = oracle.OracleSim(sc)
    o.reset(17)
    tgt = np.array([[3.0, -4.0]])
    o.set_targets(tgt)
    saw_foot = saw_limit = False
    for s in range(140):
        a = 1.4 * scenes.actions_for_step(3, s, 1, sc.robot.n_dofs)     # some get clipped
        o.step(a, cfg["dt"], cfg["substeps"], cfg["iterations"])
        if s % 7 and s < 120:
            continue
        obs, rew, done = o.get_obs()
        u = np.clip(a[0].astype(np.float64), -1, 1)
        eo, er, ed = _recompute_obs_reward(sc, o.get_state()[0], u, o.get_contacts()[0], tgt[0], s + 1)
        np.testing.assert_allclose(obs[0], eo, atol=1e-9)
        assert rew[0] == pytest.approx(er, abs=1e-9)
        assert bool(done[0]) == bool(ed)
        saw_foot |= eo[-len(sc.robot.feet):].any()
    assert saw_foot


def test_reward_of_upright_still_robot_facing_its_target():
    sc, _ = scenes.config_scene(2, num_envs=1)
    o = oracle.OracleSim(sc)
    o.set_state(scenes.rest_state(sc.robot))
    o.set_targets(np.array([[50.0, 0.0]]))
    obs, rew, done = o.get_obs()          # no step yet: u = 0, nothing in contact (1.4 m up)
    # R_alive + 0.5 * 1 + 0.05 * 1 - 0.2 * N_joints; knees/elbows rest exactly on a limit (4 DoF)
    assert rew[0] == pytest.approx(2.0 + 0.5 + 0.05 - 0.2 * 4, abs=1e-12)
    assert obs[0, 0] == pytest.approx(1.7) and not done[0]
    np.testing.assert_allclose(obs[0, 1:9], 0, atol=1e-15)
    np.testing.assert_allclose(obs[0, 9:11], (0, 1), atol=1e-15)
    # facing away: heading term becomes cos/0.8 = -1.25
    o.set_targets(np.array([[-50.0, 0.0]]))
    assert o.get_obs()[1][0] == pytest.approx(2.0 - 0.5 * 1.25 + 0.05 - 0.8, abs=1e-12)
    # moving toward the target at 2 m/s adds S = 2
    st = scenes.rest_state(sc.robot); st[0, :, 7] = -2.0
    o.set_state(st)
    assert o.get_obs()[1][0] == pytest.approx(2.0 + 2.0 - 0.5 * 1.25 + 0.05 - 0.8, abs=1e-12)


def test_fall_threshold_and_frame_cap_set_done():
    sc, _ = scenes.config_scene(2, num_envs=2)
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(sc.robot, 2)
    st[1, :, 2] -= 1.05            # torso at 0.65 < 0.7
    o.set_state(st)
    assert list(o.get_obs()[2]) == [0, 1]
    o.set_state(scenes.rest_state(sc.robot, 2))
    o.set_step_count([999, 5])
    o.step(None, 1 / 60, 1, 1)
    assert list(o.get_obs()[2]) == [1, 0]


def test_reset_noise_is_seeded_bounded_and_kinematically_consistent():
    sc, _ = scenes.config_scene(2, num_envs=64)
    o = oracle.OracleSim(sc)
    o.reset(123)
    a = o.get_state()
    o.reset(123)
    assert np.array_equal(a, o.get_state())
    o.reset(124)
    b = o.get_state()
    assert not np.array_equal(a, b)
    rob = sc.robot
    off = a[:, 0, 0:3] - rob.rest_pos[0]
    assert np.abs(off).max() <= 0.05 and np.abs(off).max() > 0.03
    th = o.joint_angles()
    hinge = rob.j_mode == scenes.HINGE
    assert np.abs(th[:, hinge]).max() <= 0.05 + 1e-12
    assert np.abs(th[:, ~hinge]).max() < 1e-12
    assert (th[:, hinge] >= rob.j_lo[hinge] - 1e-12).all() and (th[:, hinge] <= rob.j_hi[hinge] + 1e-12).all()
    # joint angular velocities: one uniform rate per hinge axis, read back by the observation
    D = rob.n_dofs
    obs = o.get_obs()[0]
    want = np.zeros((64, D))
    for env in range(64):
        for j in range(rob.n_joints):
            for k in range(3):
                if rob.j_mode[j, k] == scenes.HINGE:
                    want[env, rob.j_act[j, k]] = 0.05 * (2 * oracle.uniform(123, env, 256 + 3 * j + k) - 1)
    o.reset(123)
    np.testing.assert_allclose(o.get_obs()[0][:, 11 + D:11 + 2 * D], want, atol=1e-12)
    assert 0.03 < np.abs(want).max() <= 0.05
    # the body the joint tree hangs from keeps the common velocity and does not turn
    top = [b for b in range(rob.n_bodies) if b not in set(rob.j_child)]
    assert len(top) == 1
    assert np.abs(a[:, top[0], 10:13]).max() == 0 and 0.03 < np.abs(a[:, top[0], 7:10]).max() <= 0.05
    # anchors coincide and share one velocity, locked axes do not turn: the state is assembled,
    # so the bilateral rows see no error and no residual before the first sweep
    o.start_trace(0, 8)
    o.substep_phases(None, 1 / 240, 1, oracle.PH_SOLVE)
    assert o.trace()["pos_err_max"][0] < 1e-12
    assert o.trace()["bilateral_max"][0] < 1e-12
    o.reset(124)
    b = o.get_state()
    # masked reset touches only the chosen envs
    mask = np.zeros(64, np.uint8); mask[3] = 1
    o.reset(999, mask)
    c = o.get_state()
    assert np.array_equal(c[:3], b[:3]) and np.array_equal(c[4:], b[4:]) and not np.array_equal(c[3], b[3])


def test_uniform_generator_is_uniform_and_keyed():
    u = np.array([[oracle.uniform(5, e, i) for i in range(64)] for e in range(256)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert u.mean() == pytest.approx(0.5, abs=0.01)
    assert u.var() == pytest.approx(1 / 12, abs=0.005)
    assert abs(np.corrcoef(u[:, 0], u[:, 1])[0, 1]) < 0.2
    assert oracle.uniform(5, 1, 2) != oracle.uniform(6, 1, 2) != oracle.uniform(5, 2, 1)
    # values are multiples of 2^-24, so fp32 holds them exactly
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)
