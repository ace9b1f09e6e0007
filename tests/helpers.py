"""Small independent numpy helpers for the tests (momenta, rotations)."""
import numpy as np
from scipy.spatial.transform import Rotation

import scenes


def rot_of(q_wxyz):
    q = np.asarray(q_wxyz, np.float64)
    return Rotation.from_quat([q[1], q[2], q[3], q[0]])


def linear_momentum(robot, state_env):
    return (robot.mass[:, None] * state_env[:, 7:10]).sum(0)


def angular_momentum(robot, state_env):
    """About the env origin: sum of x x m v + R I R^T w."""
    L = np.zeros(3)
    for b in range(robot.n_bodies):
        s = state_env[b]
        R = rot_of(s[3:7]).as_matrix()
        Iw = R @ np.diag(robot.inertia[b]) @ R.T
        L += np.cross(s[0:3], robot.mass[b] * s[7:10]) + Iw @ s[10:13]
    return L


def free_params(**kw):
    """Parameters for invariant tests: no angular-velocity cap, no damping."""
    p = scenes.SimParams(max_ang_vel=1e30)
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def single_scene(robot, terrain=None, params=None, num_envs=1):
    terrain = terrain or scenes.make_plane()
    sc = scenes.make_scene(robot, terrain, num_envs, params=params or scenes.SimParams())
    sc.env_origins[:] = 0.0
    return sc
