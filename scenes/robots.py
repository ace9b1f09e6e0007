"""Robot description tables (inputs only: geometry, mass properties, joints).

Conventions: z is up, x forward, y left.  Every body frame is world-aligned in
the rest pose, a capsule's segment runs along one of its body axes, inertia is
diagonal in the body frame.  A joint has an anchor point given in the rest pose
and three orthonormal axes expressed in the parent frame; each axis is either
locked or a limited, actuated hinge.  Joints are listed parents-first so a
kinematic traversal can place children in list order starting from body 0.
A parent index of -1 attaches the child to the static world.
"""
from dataclasses import dataclass, field
import math
import numpy as np

LOCK, HINGE = 0, 1


def capsule_mass_inertia(radius, seg_len, density=None, mass=None):
    """Mass and (axial, transverse) inertia of a solid capsule.

    Cylinder of length ``seg_len`` plus two hemispherical caps of ``radius``.
    Give either a density or the total mass.  ``seg_len == 0`` is a sphere.
    """
    r, L = float(radius), float(seg_len)
    vol_c = math.pi * r * r * L
    vol_h = (2.0 / 3.0) * math.pi * r ** 3
    vol = vol_c + 2.0 * vol_h
    rho = float(density) if mass is None else float(mass) / vol
    m_c, m_h = rho * vol_c, rho * vol_h
    i_ax = m_c * r * r / 2.0 + 2.0 * m_h * (2.0 * r * r / 5.0)
    i_tr = (m_c * (L * L / 12.0 + r * r / 4.0)
            + 2.0 * m_h * (2.0 * r * r / 5.0 + L * L / 4.0 + 3.0 * L * r / 8.0))
    return m_c + 2.0 * m_h, i_ax, i_tr


@dataclass
class Robot:
    name: str
    radius: np.ndarray          # [B]
    half_len: np.ndarray        # [B]  0 for a sphere
    axis: np.ndarray            # [B]  int32 body axis (0,1,2) the segment runs along
    mass: np.ndarray            # [B]
    inertia: np.ndarray         # [B,3] body-frame diagonal
    rest_pos: np.ndarray        # [B,3] env-local rest position of the body centre
    j_parent: np.ndarray        # [J] int32, -1 = world
    j_child: np.ndarray         # [J] int32
    j_anchor: np.ndarray        # [J,3] rest-pose anchor (env-local)
    j_axes: np.ndarray          # [J,3,3] rows are e_0,e_1,e_2 in the parent frame
    j_mode: np.ndarray          # [J,3] int32 LOCK / HINGE
    j_lo: np.ndarray            # [J,3]
    j_hi: np.ndarray            # [J,3]
    j_gear: np.ndarray          # [J,3]
    j_act: np.ndarray           # [J,3] int32 action index, -1 for locked axes
    root_body: int = 0
    feet: tuple = ()
    term_height: float = 0.0
    alive_bonus: float = 0.0
    body_names: list = field(default_factory=list)

    @property
    def n_bodies(self):
        return int(self.radius.shape[0])

    @property
    def n_joints(self):
        return int(self.j_parent.shape[0])

    @property
    def n_dofs(self):
        return int((self.j_mode == HINGE).sum())

    def n_slots(self, heightfield):
        """End-sphere slots (1 per sphere, 2 per capsule) plus one mid-segment
        slot per capsule on a heightfield."""
        caps = int((self.half_len > 0).sum())
        sph = self.n_bodies - caps
        return sph + caps * (3 if heightfield else 2)

    @property
    def obs_dim(self):
        return 11 + 3 * self.n_dofs + len(self.feet)

    @property
    def collide_pairs(self):
        """int32 [P, 2]: body pairs that may touch when self-collision is on (collision_pairs)."""
        return collision_pairs(self)


def collision_pairs(robot, clearance=0.03, samples=33):
    """Body pairs of one robot that may collide with each other: all pairs that no joint connects
    and whose capsules are more than `clearance` apart in the rest pose (capsules that touch or
    overlap by construction, such as neighbours along a limb, are filtered out).  The rest-pose
    gap is taken from `samples` points along each segment.  Returns int32 [P, 2], first < second."""
    B = robot.n_bodies
    joined = {(min(int(a), int(b)), max(int(a), int(b))) for a, b in zip(robot.j_parent, robot.j_child)}
    u = np.linspace(-1.0, 1.0, samples)
    pts = []
    for b in range(B):
        ax = np.zeros(3)
        ax[int(robot.axis[b])] = robot.half_len[b]
        pts.append(robot.rest_pos[b][None, :] + u[:, None] * ax[None, :])
    out = []
    for a in range(B):
        for b in range(a + 1, B):
            if (a, b) in joined:
                continue
            d = np.linalg.norm(pts[a][:, None, :] - pts[b][None, :, :], axis=2).min()
            if d - robot.radius[a] - robot.radius[b] > clearance:
                out.append((a, b))
    return np.array(out, np.int32).reshape(-1, 2)


class _Builder:
    def __init__(self, name):
        self.name = name
        self.bodies = []
        self.joints = []
        self.n_act = 0

    def body(self, name, r, seg_len, axis, centre, density=None, mass=None):
        m, i_ax, i_tr = capsule_mass_inertia(r, seg_len, density=density, mass=mass)
        inertia = [i_tr, i_tr, i_tr]
        inertia[axis] = i_ax
        if seg_len == 0:
            inertia = [i_ax] * 3
        self.bodies.append((name, r, seg_len / 2.0, axis, m, inertia, list(centre)))
        return len(self.bodies) - 1

    def joint(self, parent, child, anchor, hinges, gear):
        """hinges: list of (axis_vector, lo, hi); remaining axes are locked and
        completed to a right-handed orthonormal triad."""
        axes = [np.asarray(h[0], dtype=np.float64) for h in hinges]
        basis = [np.array(v, dtype=np.float64) for v in ((1, 0, 0), (0, 1, 0), (0, 0, 1))]
        for cand in basis:
            if len(axes) == 3:
                break
            if all(abs(float(cand @ a)) < 1e-9 for a in axes):
                axes.append(cand)
        mode = [HINGE] * len(hinges) + [LOCK] * (3 - len(hinges))
        lo = [h[1] for h in hinges] + [0.0] * (3 - len(hinges))
        hi = [h[2] for h in hinges] + [0.0] * (3 - len(hinges))
        act = []
        for _ in hinges:
            act.append(self.n_act)
            self.n_act += 1
        act += [-1] * (3 - len(hinges))
        g = [gear] * len(hinges) + [0.0] * (3 - len(hinges))
        self.joints.append((parent, child, list(anchor), np.stack(axes), mode, lo, hi, g, act))

    def build(self, **kw):
        b, j = self.bodies, self.joints
        f64 = np.float64
        return Robot(
            name=self.name,
            radius=np.array([x[1] for x in b], f64),
            half_len=np.array([x[2] for x in b], f64),
            axis=np.array([x[3] for x in b], np.int32),
            mass=np.array([x[4] for x in b], f64),
            inertia=np.array([x[5] for x in b], f64).reshape(-1, 3),
            rest_pos=np.array([x[6] for x in b], f64).reshape(-1, 3),
            j_parent=np.array([x[0] for x in j], np.int32),
            j_child=np.array([x[1] for x in j], np.int32),
            j_anchor=np.array([x[2] for x in j], f64).reshape(-1, 3),
            j_axes=np.array([x[3] for x in j], f64).reshape(-1, 3, 3),
            j_mode=np.array([x[4] for x in j], np.int32).reshape(-1, 3),
            j_lo=np.array([x[5] for x in j], f64).reshape(-1, 3),
            j_hi=np.array([x[6] for x in j], f64).reshape(-1, 3),
            j_gear=np.array([x[7] for x in j], f64).reshape(-1, 3),
            j_act=np.array([x[8] for x in j], np.int32).reshape(-1, 3),
            body_names=[x[0] for x in b],
            **kw,
        )


def make_ant(init_height=0.75, gear=15.0):
    """Torso sphere (r 0.25, 1 kg) and four two-capsule legs (segment 0.4,
    r 0.08, 0.2 kg each) along +x, +y, -x, -y; hip hinge about z, knee hinge
    about z x d (positive bends the leg down); limits +-0.7 rad."""
    bld = _Builder("ant")
    z0 = init_height
    torso = bld.body("torso", 0.25, 0.0, 2, (0, 0, z0), mass=1.0)
    dirs = [(1, 0, 0), (0, 1, 0), (-1, 0, 0), (0, -1, 0)]
    feet = []
    for k, d in enumerate(dirs):
        d = np.array(d, dtype=np.float64)
        ax = 0 if d[0] != 0 else 1
        up = bld.body(f"leg{k}_upper", 0.08, 0.4, ax, tuple(0.45 * d + (0, 0, z0)), mass=0.2)
        lo = bld.body(f"leg{k}_lower", 0.08, 0.4, ax, tuple(0.85 * d + (0, 0, z0)), mass=0.2)
        zc = np.cross((0, 0, 1.0), d)
        bld.joint(torso, up, tuple(0.25 * d + (0, 0, z0)), [((0, 0, 1.0), -0.7, 0.7)], gear)
        bld.joint(up, lo, tuple(0.65 * d + (0, 0, z0)), [(zc, -0.7, 0.7)], gear)
        feet.append(lo)
    return bld.build(root_body=torso, feet=tuple(feet), term_height=0.3, alive_bonus=0.5)


def make_humanoid(init_height=1.4, gear=100.0, density=1000.0):
    """13-capsule stick figure, 12 joints, 21 limited hinge DoF (abdomen 3,
    shoulders 2x2, elbows 1x2, hips 3x2, knees 1x2, ankles 2x2), neck locked."""
    bld = _Builder("humanoid")
    z0 = init_height
    X, Y, Z = (1.0, 0, 0), (0, 1.0, 0), (0, 0, 1.0)

    def at(x, y, z):
        return (x, y, z + z0)

    pelvis = bld.body("pelvis", 0.09, 0.14, 1, at(0, 0, 0), density)
    torso = bld.body("torso", 0.09, 0.25, 2, at(0, 0, 0.30), density)
    head = bld.body("head", 0.09, 0.10, 2, at(0, 0, 0.66), density)
    bld.joint(pelvis, torso, at(0, 0, 0.10),
              [(X, -0.6, 0.6), (Y, -1.0, 0.5), (Z, -0.7, 0.7)], gear)
    bld.joint(torso, head, at(0, 0, 0.52), [], gear)
    for side, sy in (("R", -1.0), ("L", 1.0)):
        ua = bld.body(f"upper_arm_{side}", 0.04, 0.24, 2, at(0, 0.20 * sy, 0.33), density)
        la = bld.body(f"lower_arm_{side}", 0.04, 0.22, 2, at(0, 0.20 * sy, 0.10), density)
        bld.joint(torso, ua, at(0, 0.20 * sy, 0.45), [(X, -1.2, 1.2), (Y, -1.5, 1.5)], gear)
        bld.joint(ua, la, at(0, 0.20 * sy, 0.21), [(Y, -2.0, 0.0)], gear)
    feet = []
    for side, sy in (("R", -1.0), ("L", 1.0)):
        th = bld.body(f"thigh_{side}", 0.06, 0.35, 2, at(0, 0.10 * sy, -0.225), density)
        sh = bld.body(f"shin_{side}", 0.05, 0.30, 2, at(0, 0.10 * sy, -0.55), density)
        ft = bld.body(f"foot_{side}", 0.04, 0.16, 0, at(0.04, 0.10 * sy, -0.75), density)
        bld.joint(pelvis, th, at(0, 0.10 * sy, -0.05),
                  [(X, -0.5, 0.5), (Y, -1.6, 0.6), (Z, -0.6, 0.6)], gear)
        bld.joint(th, sh, at(0, 0.10 * sy, -0.40), [(Y, 0.0, 2.0)], gear)
        bld.joint(sh, ft, at(0, 0.10 * sy, -0.70), [(Y, -0.7, 0.7), (X, -0.4, 0.4)], gear)
        feet.append(ft)
    return bld.build(root_body=torso, feet=tuple(feet), term_height=0.7, alive_bonus=2.0)


def make_chain(n_links=3, seg_len=0.3, radius=0.03, mass=0.5, top=(0.0, 0.0, 2.0),
               direction=(0.0, 0.0, -1.0), hinge_axis=(0.0, 1.0, 0.0), lo=-3.0, hi=3.0,
               gear=1.0, world_anchor=True):
    """Pendulum chain of capsules along an axis-aligned direction, each link
    hinged to the previous one (the first to the world if ``world_anchor``)."""
    bld = _Builder("chain")
    d = np.array(direction, dtype=np.float64)
    ax = int(np.argmax(np.abs(d)))
    top = np.array(top, dtype=np.float64)
    gap = radius * 0.0
    prev = -1
    for k in range(n_links):
        a = top + d * (k * (seg_len + gap))
        c = a + d * (seg_len / 2.0)
        b = bld.body(f"link{k}", radius, seg_len, ax, tuple(c), mass=mass)
        if k > 0 or world_anchor:
            bld.joint(prev, b, tuple(a), [(hinge_axis, lo, hi)], gear)
        prev = b
    return bld.build(root_body=0, feet=(), term_height=-1e9, alive_bonus=0.0)


def make_single(radius=0.1, seg_len=0.0, axis=0, pos=(0.0, 0.0, 1.0), mass=1.0):
    """One free body (sphere if seg_len == 0, else a capsule), no joints."""
    bld = _Builder("single")
    bld.body("body", radius, seg_len, axis, pos, mass=mass)
    return bld.build(root_body=0, feet=(0,), term_height=-1e9, alive_bonus=0.0)


def make_loose(bodies):
    """Free bodies without joints: ``bodies`` is a list of (radius, seg_len, axis, pos, mass)."""
    bld = _Builder("loose")
    for k, (r, L, ax, pos, m) in enumerate(bodies):
        bld.body(f"body{k}", r, L, ax, pos, mass=m)
    return bld.build(root_body=0, feet=(0,), term_height=-1e9, alive_bonus=0.0)


def make_star(n_legs=6, hub_radius=0.2, seg_len=0.3, radius=0.05, height=0.6, gear=5.0):
    """Sphere hub with ``n_legs`` horizontal capsules hinged to it about z: the hub belongs to
    ``n_legs`` joints (more than any body of the ant or the humanoid).  Legs point along +-x / +-y
    in turn, staggered in height so that they do not coincide."""
    bld = _Builder("star")
    hub = bld.body("hub", hub_radius, 0.0, 0, (0.0, 0.0, height), mass=2.0)
    dirs = [(1, 0), (0, 1), (-1, 0), (0, -1)]
    for k in range(n_legs):
        dx, dy = dirs[k % 4]
        z = height + 0.08 * (k // 4) - 0.04 * ((k // 4) % 2)
        a = np.array([dx * hub_radius, dy * hub_radius, z])
        c = a + np.array([dx, dy, 0.0]) * (seg_len / 2.0)
        leg = bld.body(f"leg{k}", radius, seg_len, 0 if dx else 1, tuple(c), mass=0.3)
        bld.joint(hub, leg, tuple(a), [((0.0, 0.0, 1.0), -0.6, 0.6)], gear)
    return bld.build(root_body=0, feet=(), term_height=-1e9, alive_bonus=0.0)


def make_raft(n_links=13, seg_len=0.25, radius=0.05, clearance=0.01, gear=2.0):
    """Free chain of capsules lying along x just above the ground: every end sphere is within
    the contact margin from the first substep on (many simultaneous contacts per env)."""
    bld = _Builder("raft")
    prev = -1
    x = 0.0
    for k in range(n_links):
        c = (x + seg_len / 2.0, 0.0, radius + clearance)
        b = bld.body(f"link{k}", radius, seg_len, 0, c, mass=0.4)
        if prev >= 0:
            bld.joint(prev, b, (x, 0.0, radius + clearance), [((0.0, 1.0, 0.0), -0.5, 0.5)], gear)
        prev = b
        x += seg_len
    return bld.build(root_body=n_links // 2, feet=(0, n_links - 1), term_height=-1e9, alive_bonus=0.0)
