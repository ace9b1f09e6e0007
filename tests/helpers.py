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


TOL_1, TOL_10 = 1e-4, 1e-3     # the task's state tolerances after 1 and after 10 env-steps


def rel_err4(g, o):
    """[N][4]: error of position, quaternion, linear and angular velocity per env, each
    |gpu - ref|_inf / max(1, |ref|_inf) over the env's bodies."""
    out = []
    for sl in (slice(0, 3), slice(3, 7), slice(7, 10), slice(10, 13)):
        d = np.abs(g[:, :, sl] - o[:, :, sl]).reshape(g.shape[0], -1).max(1)
        n = np.maximum(1.0, np.abs(o[:, :, sl]).reshape(g.shape[0], -1).max(1))
        out.append(d / n)
    return np.stack(out, 1)


def gate_after_10_steps(e10q, forked, many_impacts=False, label="", sets_seen_every_substep=True, min_same=None,
                        interacting=False):
    """The 10-step state gate, split by whether the two sides ever disagreed on a contact set.

    e10q [N][4] from rel_err4; forked [N] bool: in some substep the HIP path and the oracle
    selected a different set of active slots, kind or nearest terrain feature (equal distances to
    within rounding).
      (i)  envs whose contact sets stayed identical: every one within 1e-3, no percentile.  With
           many_impacts (8 x 32 fallen humanoids, h = 1/480 s) this holds for positions and
           orientations; for the velocities it holds for at least 97 % of them, all stay within
           5e-3: a speculative contact that closes turns a position difference delta into a
           velocity difference delta / h (its bias is gap / h), so a body that hits the ground in
           the last substeps shows 480 times its position error in its velocity
           (tests/test_oracle_sensitivity.py shows the oracle doing this against copies of itself).
           Without sets_seen_every_substep (whole env-steps in one launch: only the sets of each
           step's last substep can be compared, so some forks go unseen) one env in a hundred
           (three with many_impacts) may lie between 1e-3 and 5e-3, in any of x, q, v, w.
           With interacting agents (capsule-capsule contacts between the agents of a group) a
           contact passes every difference in one agent on to the other: identical sets do not
           bound the growth as they do for an agent on its own, and the all-fp32 twin of the oracle
           leaves 1e-3 for up to a fifth of such agents
           (tests/test_oracle_sensitivity.py, the crowd).  There nine in ten stay within 1e-3, all
           within 5e-3 in position and orientation and within 5e-2 in the velocities (a closing
           contact divides a position difference by h = 1/240 s, see above).
      (ii) envs that forked follow another branch of a discontinuous map (a limb catches an edge
           on one side and misses it on the other): reported; nine in ten stay within 1e-3, and
           none leaves the scale of the state itself (1.0: nothing blows up).  There is no sharper
           bound for all of them: the all-fp32 twin of the oracle shows forked agents at 9e-2
           after ten steps (tests/test_oracle_sensitivity.py, the crowd).
    Returns the summary line."""
    e10 = e10q.max(1)
    same = ~forked
    line = (f"{label}10 steps: {same.sum()} envs with identical contact sets, max x {e10q[same, 0].max():.2e} "
            f"q {e10q[same, 1].max():.2e} v {e10q[same, 2].max():.2e} w {e10q[same, 3].max():.2e}")
    if forked.any():
        ef = e10[forked]
        line += f"; {forked.sum()} forked: median {np.median(ef):.2e} p90 {np.quantile(ef, .9):.2e} max {ef.max():.2e}"
    print(line)
    # (min_same: with interacting agents a fork spreads to everybody its agent shares a group with,
    #  so fewer stay on the common branch; the caller says how many it still expects)
    assert same.sum() >= (max(1, len(e10) // 4) if min_same is None else min_same), "too few envs kept identical contact sets to gate anything"
    if interacting:
        assert (e10[same] <= TOL_10).mean() >= 0.9 and e10q[same, :2].max() <= 5e-3 and e10q[same, 2:].max() <= 5e-2, line
    elif not sets_seen_every_substep:
        # (an unseen fork moves positions as well as velocities)
        assert (e10[same] <= TOL_10).mean() >= (0.97 if many_impacts else 0.99) and e10[same].max() <= 5e-3, line
    elif many_impacts:
        assert e10q[same, :2].max() <= TOL_10, line
        ev = e10q[same, 2:].max(1)
        assert (ev <= TOL_10).mean() >= 0.97 and ev.max() <= 5e-3, line
    else:
        assert e10q[same, :2].max() <= TOL_10, line
        assert e10q[same, 2:].max() <= TOL_10, line
    if forked.any():
        assert np.quantile(e10[forked], 0.9) <= TOL_10 and e10[forked].max() <= 1.0, line
    return line
