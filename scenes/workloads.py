"""Workload recipes: the five benchmark/parity configurations, seeded actions,
env placement and hand-built initial states.  Inputs only.

State interchange format used everywhere outside the simulators' private
layouts: ``state[N][B][13]`` = position(3), quaternion(w,x,y,z), linear
velocity(3), angular velocity(3); positions are env-local (relative to the
env's origin), velocities are world-frame.
"""
from dataclasses import dataclass, field
import numpy as np

from .robots import Robot, make_ant, make_humanoid, HINGE
from .terrain import (Terrain, make_plane, make_heightfield, terrain_height_max_near,
                      PLANE, HEIGHTFIELD)


@dataclass
class SimParams:
    gravity: tuple = (0.0, 0.0, -9.81)
    mu: float = 1.0
    contact_margin: float = 0.02
    beta_joint: float = 0.2
    beta_contact: float = 0.2
    max_depen_vel: float = 2.0
    lin_damping: float = 0.0
    ang_damping: float = 0.0
    max_ang_vel: float = 64.0
    gyroscopic: int = 1
    contacts: int = 1
    reset_noise: float = 0.05
    max_episode_steps: int = 1000
    height_map: int = 0            # 1: append the 15 x 11 terrain height map to the observation
    self_collide: int = 0          # 1: capsules of one robot collide (pairs: robots.collision_pairs)
    group_size: int = 1            # agents per interaction group (inter-agent collisions inside it)
    warm_start: float = 0.0        # share (0..1) of the previous substep's impulses the rows start from
    solver: int = 0                # 0: block projected Jacobi; 1: non-smooth Newton with a Krylov inner solve
    krylov_iters: int = 8          # conjugate-residual iterations per Newton iteration (solver 1)
    newton_reg: float = 0.1        # damping of the Newton step: this share of the operator's diagonal is added to it (solver 1)


@dataclass
class TaskParams:
    """Task logic around the step (Section 4.1 of the paper); the defaults are the flagrun tasks'
    numbers.  "A few newtons" is read as 1 to 5 N."""
    enabled: int = 1
    fall_grace_frames: int = 160
    target_period: int = 200
    push_min_frames: int = 200
    push_max_frames: int = 300
    auto_reset: int = 1
    target_reach: float = 1.0
    target_radius: float = 100.0
    push_min_newton: float = 1.0
    push_max_newton: float = 5.0
    seed: int = 0


@dataclass
class Scene:
    robot: Robot
    terrain: Terrain
    num_envs: int
    env_origins: np.ndarray        # [N][3] world position of each env's origin
    params: SimParams = field(default_factory=SimParams)
    name: str = ""


def env_grid_origins(num_envs, spacing=5.0):
    side = int(np.ceil(np.sqrt(num_envs)))
    idx = np.arange(num_envs)
    o = np.zeros((num_envs, 3), np.float64)
    o[:, 0] = (idx % side) * spacing
    o[:, 1] = (idx // side) * spacing
    return o


def env_field_origins(terrain, num_envs, seed, border=4.0, clear_radius=0.5):
    """Seeded uniform xy positions inside the heightfield (all envs share it and
    never interact); z is the highest sample within `clear_radius`."""
    rng = np.random.Generator(np.random.Philox(key=int(seed) + 77))
    ex, ey = terrain.extent
    border = min(border, 0.25 * min(ex, ey))
    o = np.zeros((num_envs, 3), np.float64)
    o[:, 0] = terrain.origin[0] + rng.uniform(border, ex - border, num_envs)
    o[:, 1] = terrain.origin[1] + rng.uniform(border, ey - border, num_envs)
    for e in range(num_envs):
        o[e, 2] = terrain_height_max_near(terrain, o[e, 0], o[e, 1], clear_radius)
    # keep origins fp32-representable so both simulators see identical numbers
    return o.astype(np.float32).astype(np.float64)


def env_group_origins(terrain, num_envs, group_size, spacing, seed):
    """Origins for interacting agents: consecutive `group_size` agents stand on a small square
    grid `spacing` apart (Section 4.1: the initial spacing sets how often agents collide); the
    groups themselves are placed like non-interacting envs."""
    n_groups = (num_envs + group_size - 1) // group_size
    base = env_grid_origins(n_groups, spacing=50.0) if terrain.kind == PLANE else env_field_origins(
        terrain, n_groups, seed, border=8.0)
    side = int(np.ceil(np.sqrt(group_size)))
    o = np.zeros((num_envs, 3), np.float64)
    for e in range(num_envs):
        g, k = divmod(e, group_size)
        o[e, 0] = base[g, 0] + ((k % side) - 0.5 * (side - 1)) * spacing
        o[e, 1] = base[g, 1] + ((k // side) - 0.5 * (side - 1)) * spacing
        o[e, 2] = 0.0 if terrain.kind == PLANE else terrain_height_max_near(terrain, o[e, 0], o[e, 1], 0.5)
    return o.astype(np.float32).astype(np.float64)


def crowd_origins(num_envs, density, seed, min_dist=0.5, base=(0.0, 0.0)):
    """Origins for agents that share one scene (Section 3.1, last paragraph): a square with
    `density` agents per square metre, one agent per cell of a jittered grid (no two closer than
    about min_dist), numbered in no spatial order, so that consecutive numbers are mostly far
    apart.  z = 0 (the caller lifts them onto a heightfield)."""
    rng = np.random.Generator(np.random.Philox(key=int(seed) + 991))
    side = float(np.sqrt(num_envs / density))
    k = int(np.ceil(np.sqrt(num_envs)))
    cell = side / k
    idx = rng.permutation(k * k)[:num_envs]
    jit = max(cell - min_dist, 0.0)
    o = np.zeros((num_envs, 3), np.float64)
    o[:, 0] = base[0] + (idx % k + 0.5) * cell + rng.uniform(-0.5, 0.5, num_envs) * jit
    o[:, 1] = base[1] + (idx // k + 0.5) * cell + rng.uniform(-0.5, 0.5, num_envs) * jit
    return o.astype(np.float32).astype(np.float64)


def make_scene(robot, terrain, num_envs, seed=0, params=None, name="", spacing=None):
    """`spacing` (with params.group_size > 1) places the agents of a group that far apart."""
    params = params or SimParams()
    if params.group_size > 1 and spacing is not None:
        origins = env_group_origins(terrain, num_envs, params.group_size, spacing, seed)
    elif terrain.kind == PLANE:
        origins = env_grid_origins(num_envs)
    else:
        origins = env_field_origins(terrain, num_envs, seed)
    return Scene(robot=robot, terrain=terrain, num_envs=int(num_envs), env_origins=origins,
                 params=params or SimParams(), name=name)


# name, robot, terrain, N, dt, substeps, iterations, steps
CONFIGS = [
    dict(name="ant16_plane", robot="ant", terrain="plane", num_envs=16,
         dt=1.0 / 60.0, substeps=2, iterations=8, steps=100, fallen=False),
    dict(name="ant1024_plane", robot="ant", terrain="plane", num_envs=1024,
         dt=1.0 / 60.0, substeps=4, iterations=16, steps=1000, fallen=False),
    dict(name="humanoid1024_plane", robot="humanoid", terrain="plane", num_envs=1024,
         dt=1.0 / 60.0, substeps=4, iterations=20, steps=1000, fallen=False),
    dict(name="humanoid4096_heightfield", robot="humanoid", terrain="heightfield", num_envs=4096,
         dt=1.0 / 60.0, substeps=4, iterations=20, steps=1000, fallen=False),
    dict(name="humanoid8192_heightfield_fallen", robot="humanoid", terrain="heightfield",
         num_envs=8192, dt=1.0 / 60.0, substeps=8, iterations=32, steps=1000, fallen=True),
]

_HF_CACHE = {}


def config_scene(k, num_envs=None):
    """Scene + stepping parameters of benchmark configuration k (base seed 1000+k).
    `num_envs` overrides the env count (parity tests run the same recipe smaller)."""
    cfg = dict(CONFIGS[k])
    seed = 1000 + k
    robot = make_ant() if cfg["robot"] == "ant" else make_humanoid()
    if cfg["terrain"] == "plane":
        terrain = make_plane()
    else:
        if "hf" not in _HF_CACHE:
            _HF_CACHE["hf"] = make_heightfield(seed=1003)
        terrain = _HF_CACHE["hf"]
    n = int(num_envs) if num_envs is not None else cfg["num_envs"]
    cfg["num_envs"] = n
    cfg["seed"] = seed
    scene = make_scene(robot, terrain, n, seed=seed, name=cfg["name"])
    return scene, cfg


def actions_for_step(seed, step, num_envs, n_dofs):
    """Uniform [-1,1) actions for one step, fp32 [N][D]; any step can be drawn
    on its own (counter-based generator keyed by seed, advanced by step)."""
    rng = np.random.Generator(np.random.Philox(key=int(seed), counter=[0, 0, int(step), 0]))
    return rng.uniform(-1.0, 1.0, (num_envs, n_dofs)).astype(np.float32)


def targets_for_step(seed, step, num_envs, period=200, distance=100.0):
    """Per-env target positions (env-local xy) re-drawn every `period` steps."""
    epoch = int(step) // int(period)
    rng = np.random.Generator(np.random.Philox(key=int(seed) + 31, counter=[0, 0, epoch, 0]))
    ang = rng.uniform(0.0, 2.0 * np.pi, num_envs)
    return np.stack([distance * np.cos(ang), distance * np.sin(ang)], axis=1).astype(np.float32)


# ---- hand-built states (plain rigid-transform bookkeeping, no dynamics) ----

def _qmul(a, b):
    aw, ax, ay, az = a
    bw, bx, by, bz = b
    return np.array([aw * bw - ax * bx - ay * by - az * bz,
                     aw * bx + ax * bw + ay * bz - az * by,
                     aw * by - ax * bz + ay * bw + az * bx,
                     aw * bz + ax * by - ay * bx + az * bw])


def _qrot(q, v):
    w, x, y, z = q
    u = np.array([x, y, z])
    return v + 2.0 * np.cross(u, np.cross(u, v) + w * v)


def _qexp(phi):
    a = float(np.linalg.norm(phi))
    if a < 1e-12:
        return np.array([1.0, 0.5 * phi[0], 0.5 * phi[1], 0.5 * phi[2]])
    s = np.sin(0.5 * a) / a
    return np.array([np.cos(0.5 * a), s * phi[0], s * phi[1], s * phi[2]])


def rest_state(robot, num_envs=1):
    B = robot.n_bodies
    s = np.zeros((num_envs, B, 13), np.float64)
    s[:, :, 0:3] = robot.rest_pos[None]
    s[:, :, 3] = 1.0
    return s


def posed_state(robot, base_pos, base_quat, joint_angles):
    """Place all bodies from a pose of body 0 and per-joint rotation vectors
    (joint_angles[J][3] along each joint's own axes)."""
    B = robot.n_bodies
    x = np.zeros((B, 3))
    q = np.zeros((B, 4))
    placed = np.zeros(B, bool)
    x[0], q[0], placed[0] = base_pos, base_quat, True
    for j in range(robot.n_joints):
        a, b = int(robot.j_parent[j]), int(robot.j_child[j])
        phi = robot.j_axes[j].T @ joint_angles[j]
        if a < 0:
            qa, xa, la = np.array([1.0, 0, 0, 0]), np.zeros(3), robot.j_anchor[j]
        else:
            assert placed[a], "joints must be listed parents-first"
            qa, xa, la = q[a], x[a], robot.j_anchor[j] - robot.rest_pos[a]
        lb = robot.j_anchor[j] - robot.rest_pos[b]
        q[b] = _qmul(qa, _qexp(phi))
        q[b] /= np.linalg.norm(q[b])
        x[b] = xa + _qrot(qa, la) - _qrot(q[b], lb)
        placed[b] = True
    s = np.zeros((B, 13))
    s[:, 0:3], s[:, 3:7] = x, q
    return s


def fallen_states(scene, seed, drop=(0.3, 1.0), near_radius=1.5):
    """Random fallen poses: uniform random base orientation, joint angles uniform
    within limits, lowest surface point `drop` metres above the highest terrain
    sample within `near_radius` of the env origin.  Returns fp32-rounded
    state[N][B][13]."""
    robot, N = scene.robot, scene.num_envs
    rng = np.random.Generator(np.random.Philox(key=int(seed) + 501))
    out = np.zeros((N, robot.n_bodies, 13))
    hinge = robot.j_mode == HINGE
    for e in range(N):
        qb = rng.normal(size=4)
        qb /= np.linalg.norm(qb)
        ang = np.where(hinge, rng.uniform(robot.j_lo, robot.j_hi), 0.0)
        s = posed_state(robot, robot.rest_pos[0], qb, ang)
        low = np.inf
        for b in range(robot.n_bodies):
            u = np.zeros(3)
            u[robot.axis[b]] = 1.0
            d = _qrot(s[b, 3:7], u) * robot.half_len[b]
            low = min(low, s[b, 2] - abs(d[2]) - robot.radius[b])
        ox, oy, oz = scene.env_origins[e]
        top = terrain_height_max_near(scene.terrain, ox, oy, near_radius) - oz
        s[:, 2] += (top + rng.uniform(*drop)) - low
        out[e] = s
    return out.astype(np.float32).astype(np.float64)
