"""The oracle against the numbers the paper prints (fixtures under tests/golden/, each with
its citation): observation layout of the humanoid, reward coefficients and thresholds, the task
rules of Section 4.1, the physics constants of Section 3.1."""
import os

import numpy as np
import pytest
from scipy.spatial.transform import Rotation

import oracle
import scenes
from helpers import free_params, single_scene

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def test_observation_layout_of_the_humanoid():
    g = golden("observation_humanoid_ours.txt")
    assert sum(v for k, v in g.items() if k != "total") == g["total"]
    rob = scenes.make_humanoid()
    sc = single_scene(rob, num_envs=3)
    o = oracle.OracleSim(sc)
    assert o.obs_dim == g["total"] == rob.obs_dim
    assert rob.n_dofs == g["joint_angles"] == g["joint_angle_velocities"] == g["actuator_forces"]
    assert len(rob.feet) == g["feet_in_contact"]
    # the blocks sit in the table's order: height, roll/pitch, velocity, angular velocity, heading,
    # joint angles, joint velocities, actuator forces (= the clipped actions), feet flags
    o.reset(seed=4)
    u = np.random.default_rng(0).uniform(-1.5, 1.5, (3, rob.n_dofs))
    o.substep_phases(u, 1.0 / 240.0, 0, phases=0)        # loads the actions, moves nothing
    obs, rew, done = o.get_obs()
    st = o.get_state()
    n_root = int(g["root_body_height"] + g["root_body_rotation_roll_pitch"] + g["root_body_velocity"]
                 + g["root_body_angular_velocity"] + g["root_body_heading_sin_cos"])
    D = rob.n_dofs
    assert n_root == 11
    assert np.allclose(obs[:, 0], st[:, rob.root_body, 2])
    assert np.allclose(obs[:, 3:6], st[:, rob.root_body, 7:10]) and np.allclose(obs[:, 6:9], st[:, rob.root_body, 10:13])
    assert np.allclose(obs[:, 9] ** 2 + obs[:, 10] ** 2, 1.0)
    assert np.allclose(obs[:, n_root:n_root + D], o.joint_angles()[:, :, :].reshape(3, -1)[:, _hinge_columns(rob)])
    assert np.allclose(obs[:, n_root + 2 * D:n_root + 3 * D], np.clip(u, -1, 1))
    assert set(np.unique(obs[:, n_root + 3 * D:])) <= {0.0, 1.0}


def _hinge_columns(rob):
    """Columns of the flattened [J][3] joint-angle array in action order."""
    cols = np.zeros(rob.n_dofs, int)
    for j in range(rob.n_joints):
        for k in range(3):
            if rob.j_mode[j, k] == scenes.HINGE:
                cols[rob.j_act[j, k]] = 3 * j + k
    return cols


def _reward(o):
    return o.get_obs()[1].copy()


def test_reward_coefficients_and_thresholds():
    g = golden("reward_terms.txt")
    assert scenes.make_ant().alive_bonus == g["alive_bonus_ant"]
    rob = scenes.make_humanoid()
    assert rob.alive_bonus == g["alive_bonus_humanoid"]
    sc = single_scene(rob, params=free_params(contacts=0), num_envs=1)
    o = oracle.OracleSim(sc)
    st = scenes.rest_state(rob)
    st[0, :, 2] += 1.0                                   # in the air: no foot contact
    D = rob.n_dofs

    def reward(state, u=None, target=(1000.0, 0.0)):
        o.set_state(state)
        o.set_targets(np.array([target]))
        o.substep_phases(np.zeros((1, D)) if u is None else u, 1.0 / 240.0, 0, phases=0)
        return float(_reward(o)[0])

    # at rest, upright, facing the target, no joint at a limit apart from those the rest pose has
    n_lim = int(sum(min(0.0 - rob.j_lo[j, k], rob.j_hi[j, k] - 0.0) <= 0 for j in range(rob.n_joints)
                    for k in range(3) if rob.j_mode[j, k] == scenes.HINGE))
    base = reward(st)
    assert base == pytest.approx(g["alive_bonus_humanoid"] + g["heading_bonus"] + g["standing_bonus"]
                                 - g["joint_at_limit_cost"] * n_lim)
    # speed toward the target enters with weight 1
    sv = st.copy(); sv[0, rob.root_body, 7] = 0.7
    assert reward(sv) - base == pytest.approx(g["speed_toward_target"] * 0.7)
    # actions: 4 |u|_1 (torque over maximum torque is the action) + 0.5 |u|_2^2
    u = np.zeros((1, D)); u[0, 3], u[0, 7] = 0.5, -0.25
    assert reward(st, u) - base == pytest.approx(-g["torque_cost_l1_over_max_torque"] * 0.75
                                                 - g["control_cost_l2_squared"] * (0.25 + 0.0625))
    # heading: full bonus above cos 0.8, cos / 0.8 below
    for cos_t in (0.9, 0.8, 0.4, -0.5):
        tgt = 50.0 * np.array([cos_t, np.sqrt(1 - cos_t ** 2)])
        want = 1.0 if cos_t > g["heading_full_above_cos"] else cos_t / g["heading_full_above_cos"]
        assert reward(st, target=tuple(tgt)) - base == pytest.approx(g["heading_bonus"] * (want - 1.0), abs=1e-9)
    # standing: indicator of the torso's z axis above cos 0.93
    for tilt_cos, on in ((0.95, 1.0), (0.91, 0.0)):
        q = Rotation.from_euler("y", np.arccos(tilt_cos)).as_quat()     # x, y, z, w
        tilted = st.copy()
        tilted[0, :, 3:7] = [q[3], q[0], q[1], q[2]]
        got = reward(tilted)
        # tilting about y turns the heading as well: compare with the same pose's heading term only
        obs = o.get_obs()[0][0]
        head = 1.0 if obs[10] > g["heading_full_above_cos"] else obs[10] / g["heading_full_above_cos"]
        assert got == pytest.approx(g["alive_bonus_humanoid"] + g["heading_bonus"] * head + g["standing_bonus"] * on
                                    - g["joint_at_limit_cost"] * n_lim, abs=1e-9)


def test_task_rules_and_terrain_map_size():
    g = golden("section_4_1_task_numbers.txt")
    t = scenes.TaskParams()
    assert t.fall_grace_frames == g["fallen_grace_frames_flagrun"]
    assert t.target_period == g["target_redraw_period_frames"]
    assert t.target_reach == g["target_reached_within_m"] and t.target_radius == g["target_within_m"]
    assert (t.push_min_frames, t.push_max_frames) == (g["push_interval_min_frames"], g["push_interval_max_frames"])
    assert scenes.SimParams().max_episode_steps == g["episode_limit_frames"]
    rob = scenes.make_humanoid()
    p = scenes.SimParams(height_map=1)
    sc = scenes.make_scene(rob, scenes.make_flat_heightfield(nx=64, ny=64, cell=0.1), 2, params=p)
    o = oracle.OracleSim(sc)
    assert o.obs_dim - rob.obs_dim == g["height_map_rows"] * g["height_map_cols"]


def test_physics_constants():
    g = golden("section_3_1_physics_constants.txt")
    assert scenes.SimParams().mu == g["friction_coefficient"]
    assert g["time_step_s"] == pytest.approx(1.0 / 120.0)
    # restitution 0: a sphere dropped on the plane does not come back up
    rob = scenes.make_single(radius=0.1, pos=(0.0, 0.0, 0.3), mass=1.0)
    sc = single_scene(rob, params=free_params(gravity=(0.0, 0.0, -g["gravity_m_s2"])))
    o = oracle.OracleSim(sc)
    o.set_state(scenes.rest_state(rob))
    vmax_after = 0.0
    landed = False
    for _ in range(120):
        o.step(None, g["time_step_s"], 1, 8)
        s = o.get_state()[0, 0]
        if s[2] < 0.1 + 0.021:
            landed = True
        if landed:
            vmax_after = max(vmax_after, s[9])
    assert landed and vmax_after <= g["restitution"] + 1e-9
    # free fall before the impact: v = -g t exactly for the discrete scheme
    o.set_state(scenes.rest_state(rob))
    o.step(None, g["time_step_s"], 1, 8)
    assert o.get_state()[0, 0, 9] == pytest.approx(-g["gravity_m_s2"] * g["time_step_s"])
