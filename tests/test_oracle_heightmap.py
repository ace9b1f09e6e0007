"""Pins for the oracle's 15 x 11 height-map observation (Section 4.1, complex terrain task).

The paper fixes the size (15 x 11), that the map follows the centre of mass and that it is denser
near the robot.  The pins recover the sample positions from the observation itself on linear
terrains (where the terrain height is an exact linear function of position) and check those
facts, the heading alignment, the mass weighting of the centre and the border behaviour."""
import numpy as np
from scipy.spatial.transform import Rotation

import oracle
import scenes

ROWS, COLS = 15, 11


def _sim(terrain, state, origin=(10.0, 10.0, 0.0)):
    rob = scenes.make_humanoid()
    sc = scenes.make_scene(rob, terrain, 1, params=scenes.SimParams(height_map=1))
    sc.env_origins[0] = origin
    o = oracle.OracleSim(sc)
    o.set_state(state[None])
    obs, _, _ = o.get_obs()
    base = 11 + 3 * rob.n_dofs + len(rob.feet)
    assert obs.shape[1] == base + ROWS * COLS
    return rob, obs[0, base:].reshape(ROWS, COLS), obs[0, :base]


def _com(rob, state):
    return (rob.mass[:, None] * state[:, 0:3]).sum(0) / rob.mass.sum()


def _pose(yaw=0.0, z=1.4, bend=0.0):
    rob = scenes.make_humanoid()
    q = Rotation.from_euler("z", yaw).as_quat()  # x,y,z,w
    ang = np.zeros((rob.n_joints, 3)); ang[:, 1] = bend
    return scenes.posed_state(rob, np.array([0.0, 0.0, z]), np.array([q[3], q[0], q[1], q[2]]), ang)


def test_flat_field_gives_minus_centre_height_everywhere():
    st = _pose(yaw=0.7, bend=0.2)
    rob, hm, _ = _sim(scenes.make_flat_heightfield(nx=300, ny=300, cell=0.1, height=0.37), st)
    assert np.allclose(hm, 0.37 - _com(rob, st)[2], atol=1e-6)
    # plane terrain: height 0 under every sample
    rob, hm, _ = _sim(scenes.make_plane(), st)
    assert np.allclose(hm, -_com(rob, st)[2], atol=1e-12)


def _offsets():
    """Sample offsets recovered from unit slopes along x and y at zero yaw."""
    st = _pose()
    rob, hx, _ = _sim(scenes.make_tilted_heightfield(nx=300, ny=300, cell=0.1, slope_x=0.25), st)
    _, hy, _ = _sim(scenes.make_tilted_heightfield(nx=300, ny=300, cell=0.1, slope_y=0.25), st)
    c = _com(rob, st)
    f = (hx + c[2]) / 0.25 - (10.0 + c[0])       # forward offset of each sample
    l = (hy + c[2]) / 0.25 - (10.0 + c[1])       # leftward offset
    return f, l


def test_grid_is_rectangular_centred_on_the_com_and_denser_near_the_robot():
    f, l = _offsets()
    assert np.allclose(f, f[:, :1], atol=1e-5) and np.allclose(l, l[:1, :], atol=1e-5)   # rectangular
    fr, lc = f[:, 0], l[0, :]
    assert abs(fr[4]) < 1e-5 and abs(lc[5]) < 1e-5                                      # a sample under the centre
    assert np.all(np.diff(fr) > 0) and np.all(np.diff(lc) > 0)
    # spacing grows away from the centre sample in all four directions
    assert np.all(np.diff(np.diff(fr[4:])) > 0) and np.all(np.diff(np.diff(fr[4::-1] * -1)) > 0)
    assert np.all(np.diff(np.diff(lc[5:])) > 0)
    assert np.allclose(lc[5:], -lc[5::-1], atol=1e-5)                                   # symmetric sideways
    assert fr[-1] > 5.0 and -1.5 < fr[0] < -0.5 and 1.0 < lc[-1] < 2.0                   # looks further ahead


def test_grid_turns_with_the_heading():
    f, l = _offsets()
    for yaw in (0.9, -2.2):
        st = _pose(yaw=yaw)
        rob, hm, base = _sim(scenes.make_tilted_heightfield(nx=300, ny=300, cell=0.1, slope_x=0.25, slope_y=-0.1), st)
        c = _com(rob, st)
        wx = 10.0 + c[0] + np.cos(yaw) * f - np.sin(yaw) * l
        wy = 10.0 + c[1] + np.sin(yaw) * f + np.cos(yaw) * l
        assert np.allclose(hm, 0.25 * wx - 0.1 * wy - c[2], atol=2e-5)


def test_centre_is_mass_weighted():
    st = _pose(bend=0.6)            # bent limbs: the centre of mass is not the root body
    rob = scenes.make_humanoid()
    c = _com(rob, st)
    assert np.linalg.norm(c[:2] - st[rob.root_body, :2]) > 0.01
    f, l = _offsets()
    _, hm, _ = _sim(scenes.make_tilted_heightfield(nx=300, ny=300, cell=0.1, slope_x=0.25, slope_y=0.15), st)
    assert np.allclose(hm, 0.25 * (10 + c[0] + f) + 0.15 * (10 + c[1] + l) - c[2], atol=2e-5)


def test_samples_beyond_the_field_read_the_border():
    f, l = _offsets()
    st = _pose()
    ter = scenes.make_tilted_heightfield(nx=300, ny=300, cell=0.1, slope_x=0.25)
    rob, hm, _ = _sim(ter, st, origin=(27.0, 10.0, 0.0))      # field ends at x = 29.9
    c = _com(rob, st)
    wx = np.minimum(27.0 + c[0] + f, 29.9)
    assert np.allclose(hm, 0.25 * wx - c[2], atol=2e-5)
    assert (27.0 + c[0] + f).max() > 31.0
