"""ctypes binding of include/sim.h.  Same names as the C entry points; the `Sim`
class below only bundles a handle with its workspace tensor."""
import ctypes as C
import os

import numpy as np

from . import build as _build

SIM_PAIR_CAP = 96
SIM_MAX_FEET = 4
_LIB = None


class SimError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"sim error {code}: {msg}")
        self.code = code


class BodyDesc(C.Structure):
    _fields_ = [("axis", C.c_int32), ("pad", C.c_int32), ("radius", C.c_double), ("half_len", C.c_double),
                ("mass", C.c_double), ("inertia", C.c_double * 3), ("rest_pos", C.c_double * 3)]


class JointDesc(C.Structure):
    _fields_ = [("parent", C.c_int32), ("child", C.c_int32), ("anchor", C.c_double * 3),
                ("axes", (C.c_double * 3) * 3), ("mode", C.c_int32 * 3), ("act", C.c_int32 * 3),
                ("lo", C.c_double * 3), ("hi", C.c_double * 3), ("gear", C.c_double * 3)]


class SimDesc(C.Structure):
    _fields_ = [
        ("n_bodies", C.c_int32), ("n_joints", C.c_int32),
        ("bodies", C.POINTER(BodyDesc)), ("joints", C.POINTER(JointDesc)),
        ("root_body", C.c_int32), ("n_feet", C.c_int32), ("foot_bodies", C.c_int32 * SIM_MAX_FEET),
        ("term_height", C.c_double), ("alive_bonus", C.c_double),
        ("max_episode_steps", C.c_int32), ("terrain_kind", C.c_int32),
        ("hf_nx", C.c_int32), ("hf_ny", C.c_int32),
        ("hf_cell", C.c_double), ("hf_origin", C.c_double * 2),
        ("hf_heights", C.POINTER(C.c_float)), ("env_origins", C.POINTER(C.c_double)),
        ("gravity", C.c_double * 3), ("mu", C.c_double), ("contact_margin", C.c_double),
        ("beta_joint", C.c_double), ("beta_contact", C.c_double), ("max_depen_vel", C.c_double),
        ("lin_damping", C.c_double), ("ang_damping", C.c_double), ("max_ang_vel", C.c_double),
        ("reset_noise", C.c_double), ("gyroscopic", C.c_int32), ("contacts", C.c_int32),
        ("height_map", C.c_int32),
        ("n_collide_pairs", C.c_int32), ("collide_pairs", C.POINTER(C.c_int32)), ("group_size", C.c_int32),
        ("warm_start", C.c_double),
        ("solver", C.c_int32), ("krylov_iterations", C.c_int32), ("newton_reg", C.c_double),
    ]


class TaskDesc(C.Structure):
    _fields_ = [("enabled", C.c_int32), ("fall_grace_frames", C.c_int32), ("target_period", C.c_int32),
                ("push_min_frames", C.c_int32), ("push_max_frames", C.c_int32), ("auto_reset", C.c_int32),
                ("target_reach", C.c_double), ("target_radius", C.c_double),
                ("push_min_newton", C.c_double), ("push_max_newton", C.c_double), ("seed", C.c_uint64)]


PAIR_CONTACT_DTYPE = np.dtype([("env_a", np.int32), ("body_a", np.int32), ("env_b", np.int32),
                               ("body_b", np.int32), ("s", np.float32), ("t", np.float32),
                               ("d", np.float32), ("w", np.float32)])
CONTACT_DTYPE = np.dtype([("active", np.int32), ("kind", np.int32), ("feat", np.int32),
                          ("d", np.float32), ("n", np.float32, 3), ("rc", np.float32, 3),
                          ("w", np.float32), ("pad", np.int32)])

_SYMBOLS = {
    "sim_default_params": [C.POINTER(SimDesc)],
    "sim_builtin_robot": [C.c_int32, C.POINTER(SimDesc)],
    "sim_workspace_bytes": [C.POINTER(SimDesc), C.c_int, C.POINTER(C.c_size_t)],
    "sim_create": [C.POINTER(SimDesc), C.c_int, C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)],
    "sim_create_static": [C.POINTER(SimDesc), C.c_int, C.POINTER(C.c_void_p)],
    "sim_destroy": [C.c_void_p],
    "sim_num_envs": [C.c_void_p], "sim_num_bodies": [C.c_void_p], "sim_num_slots": [C.c_void_p],
    "sim_obs_dim": [C.c_void_p], "sim_act_dim": [C.c_void_p],
    "sim_reset": [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p],
    "sim_step": [C.c_void_p, C.c_void_p, C.c_float, C.c_int, C.c_int, C.c_void_p],
    "sim_step_obs": [C.c_void_p, C.c_void_p, C.c_float, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_get_obs": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_set_task": [C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_get_task_state": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_get_kept_impulses": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_set_task_state": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_set_targets": [C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_get_state": [C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_set_state": [C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_set_step_count": [C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_record_contacts": [C.c_void_p, C.c_int],
    "sim_get_contacts": [C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_generate_contacts": [C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_get_pair_contacts": [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p],
    "sim_regroup": [C.c_void_p, C.c_float, C.c_float, C.c_void_p],
    "sim_set_groups": [C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_get_groups": [C.c_void_p, C.c_void_p, C.c_void_p],
    "sim_count_near_pairs": [C.c_void_p, C.c_float, C.c_void_p, C.c_void_p],
    "sim_check": [C.c_void_p, C.c_void_p],
    "sim_launch_info": [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_size_t)],
    "sim_set_envs_per_block": [C.c_void_p, C.c_int],
    "sim_last_error": [],
}


def load_library():
    """Loads libsim355.so (built in-tree).  Builds it only if it is absent; there
    is no fallback implementation: a missing or unloadable library is an error."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(_build.LIB_PATH):
        _build.build(force=True)
    L = C.CDLL(_build.LIB_PATH)
    for name, args in _SYMBOLS.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = C.c_char_p if name == "sim_last_error" else C.c_int
    _LIB = L
    return L


def lib():
    return load_library()


def sim_last_error():
    return lib().sim_last_error().decode()


def _chk(rc):
    if rc < 0:
        raise SimError(rc, sim_last_error())
    return rc


SIM_ROBOT_ANT, SIM_ROBOT_HUMANOID = 1, 2


def sim_default_params():
    """A SimDesc with the library's default parameters and no robot, terrain or origins."""
    d = SimDesc()
    _chk(lib().sim_default_params(C.byref(d)))
    return d


def sim_builtin_robot(kind, desc=None):
    """Points desc (a fresh default one if None) at the library's built-in robot tables."""
    d = sim_default_params() if desc is None else desc
    _chk(lib().sim_builtin_robot(int(kind), C.byref(d)))
    return d


def make_desc(scene):
    """scenes.Scene -> (SimDesc, keepalive list)."""
    r, t, p = scene.robot, scene.terrain, scene.params
    bodies = (BodyDesc * r.n_bodies)()
    for b in range(r.n_bodies):
        bd = bodies[b]
        bd.axis, bd.radius, bd.half_len, bd.mass = int(r.axis[b]), r.radius[b], r.half_len[b], r.mass[b]
        for c in range(3):
            bd.inertia[c], bd.rest_pos[c] = r.inertia[b, c], r.rest_pos[b, c]
    joints = (JointDesc * max(r.n_joints, 1))()
    for j in range(r.n_joints):
        jd = joints[j]
        jd.parent, jd.child = int(r.j_parent[j]), int(r.j_child[j])
        for c in range(3):
            jd.anchor[c] = r.j_anchor[j, c]
            jd.mode[c], jd.act[c] = int(r.j_mode[j, c]), int(r.j_act[j, c])
            jd.lo[c], jd.hi[c], jd.gear[c] = r.j_lo[j, c], r.j_hi[j, c], r.j_gear[j, c]
            for k in range(3):
                jd.axes[c][k] = r.j_axes[j, c, k]
    heights = np.ascontiguousarray(t.heights, dtype=np.float32)
    origins = np.ascontiguousarray(scene.env_origins, dtype=np.float64)
    d = SimDesc()
    d.n_bodies, d.n_joints = r.n_bodies, r.n_joints
    d.bodies, d.joints = bodies, joints
    d.root_body, d.n_feet = r.root_body, len(r.feet)
    for i, f in enumerate(r.feet):
        d.foot_bodies[i] = int(f)
    d.term_height, d.alive_bonus, d.max_episode_steps = r.term_height, r.alive_bonus, p.max_episode_steps
    d.terrain_kind, d.hf_nx, d.hf_ny, d.hf_cell = t.kind, t.nx, t.ny, t.cell
    d.hf_origin[0], d.hf_origin[1] = t.origin
    d.hf_heights = heights.ctypes.data_as(C.POINTER(C.c_float))
    d.env_origins = origins.ctypes.data_as(C.POINTER(C.c_double))
    for c in range(3):
        d.gravity[c] = p.gravity[c]
    d.mu, d.contact_margin, d.beta_joint, d.beta_contact = p.mu, p.contact_margin, p.beta_joint, p.beta_contact
    d.max_depen_vel, d.lin_damping, d.ang_damping = p.max_depen_vel, p.lin_damping, p.ang_damping
    d.max_ang_vel, d.reset_noise = p.max_ang_vel, p.reset_noise
    d.gyroscopic, d.contacts = p.gyroscopic, p.contacts
    d.height_map = int(getattr(p, "height_map", 0))
    pairs = np.ascontiguousarray(r.collide_pairs if getattr(p, "self_collide", 0) else np.zeros((0, 2)), dtype=np.int32)
    d.n_collide_pairs = int(pairs.shape[0])
    d.collide_pairs = pairs.ctypes.data_as(C.POINTER(C.c_int32)) if d.n_collide_pairs else None
    d.group_size = int(getattr(p, "group_size", 1))
    d.warm_start = float(getattr(p, "warm_start", 0.0))
    d.solver = int(getattr(p, "solver", 0))
    d.krylov_iterations = int(getattr(p, "krylov_iters", 8))
    d.newton_reg = float(getattr(p, "newton_reg", 0.0))
    return d, [bodies, joints, heights, origins, pairs]


# ---- plain functions, one per C entry point (pointers are ints / torch data_ptr) ----

def sim_workspace_bytes(desc, num_envs):
    out = C.c_size_t(0)
    _chk(lib().sim_workspace_bytes(C.byref(desc), int(num_envs), C.byref(out)))
    return int(out.value)


def sim_create(desc, num_envs, workspace_ptr, workspace_bytes):
    h = C.c_void_p(None)
    _chk(lib().sim_create(C.byref(desc), int(num_envs), workspace_ptr, workspace_bytes, C.byref(h)))
    return h


def sim_create_static(desc, num_envs):
    h = C.c_void_p(None)
    _chk(lib().sim_create_static(C.byref(desc), int(num_envs), C.byref(h)))
    return h


def sim_destroy(h):
    return _chk(lib().sim_destroy(h))


def sim_reset(h, env_mask_ptr, seed, stream):
    return _chk(lib().sim_reset(h, env_mask_ptr, int(seed), stream))


def sim_step(h, actions_ptr, dt, substeps, iterations, stream):
    return _chk(lib().sim_step(h, actions_ptr, float(dt), int(substeps), int(iterations), stream))


def sim_step_obs(h, actions_ptr, dt, substeps, iterations, obs_ptr, reward_ptr, done_ptr, stream):
    return _chk(lib().sim_step_obs(h, actions_ptr, float(dt), int(substeps), int(iterations), obs_ptr, reward_ptr,
                                   done_ptr, stream))


def sim_set_task(h, task, stream):
    """task: an object with the fields of sim_task_desc_t (e.g. scenes.TaskParams) or None."""
    if task is None:
        return _chk(lib().sim_set_task(h, None, stream))
    t = TaskDesc()
    for name, _ in TaskDesc._fields_:
        setattr(t, name, getattr(task, name))
    return _chk(lib().sim_set_task(h, C.addressof(t), stream))


def sim_get_kept_impulses(h, joint_rows_ptr, slot_rows_ptr, stream):
    return _chk(lib().sim_get_kept_impulses(h, joint_rows_ptr, slot_rows_ptr, stream))


def sim_get_task_state(h, counters_ptr, targets_ptr, push_ptr, stream):
    return _chk(lib().sim_get_task_state(h, counters_ptr, targets_ptr, push_ptr, stream))


def sim_set_task_state(h, counters_ptr, targets_ptr, stream):
    return _chk(lib().sim_set_task_state(h, counters_ptr, targets_ptr, stream))


def sim_get_obs(h, obs_ptr, reward_ptr, done_ptr, stream):
    return _chk(lib().sim_get_obs(h, obs_ptr, reward_ptr, done_ptr, stream))


def sim_set_targets(h, target_ptr, stream):
    return _chk(lib().sim_set_targets(h, target_ptr, stream))


def sim_get_state(h, state_ptr, stream):
    return _chk(lib().sim_get_state(h, state_ptr, stream))


def sim_set_state(h, state_ptr, stream):
    return _chk(lib().sim_set_state(h, state_ptr, stream))


def sim_set_step_count(h, counts_ptr, stream):
    return _chk(lib().sim_set_step_count(h, counts_ptr, stream))


def sim_record_contacts(h, enable):
    return _chk(lib().sim_record_contacts(h, int(enable)))


def sim_get_contacts(h, recs_ptr, stream):
    return _chk(lib().sim_get_contacts(h, recs_ptr, stream))


def sim_generate_contacts(h, recs_ptr, stream):
    return _chk(lib().sim_generate_contacts(h, recs_ptr, stream))


def sim_get_pair_contacts(h, recs_ptr, cap, count_ptr, stream):
    return _chk(lib().sim_get_pair_contacts(h, recs_ptr, int(cap), count_ptr, stream))


def sim_regroup(h, cell, reach, stream):
    return _chk(lib().sim_regroup(h, float(cell), float(reach), stream))


def sim_set_groups(h, place_env_ptr, stream):
    return _chk(lib().sim_set_groups(h, place_env_ptr, stream))


def sim_get_groups(h, place_env_ptr, stream):
    return _chk(lib().sim_get_groups(h, place_env_ptr, stream))


def sim_count_near_pairs(h, reach, counts_ptr, stream):
    return _chk(lib().sim_count_near_pairs(h, float(reach), counts_ptr, stream))


def sim_check(h, stream):
    return _chk(lib().sim_check(h, stream))


def sim_launch_info(h):
    t, e, l = C.c_int32(0), C.c_int32(0), C.c_size_t(0)
    _chk(lib().sim_launch_info(h, C.byref(t), C.byref(e), C.byref(l)))
    return {"threads_per_block": t.value, "envs_per_block": e.value, "lds_bytes": l.value}


def sim_set_envs_per_block(h, e):
    return _chk(lib().sim_set_envs_per_block(h, int(e)))


class Sim:
    """A simulator handle plus the torch tensor that backs its workspace."""

    def __init__(self, scene, device="cuda:0", static_workspace=False):
        """static_workspace: keep the workspace in the library's own device array
        (sim_create_static) instead of a torch tensor."""
        import torch
        self.torch = torch
        if not torch.cuda.is_available():
            raise RuntimeError("paper_1810_05762_amd needs a GPU: there is no CPU path")
        self.device = torch.device(device)
        self.desc, self._keep = make_desc(scene)
        self.N = int(scene.num_envs)
        nbytes = sim_workspace_bytes(self.desc, self.N)
        with torch.cuda.device(self.device):
            if static_workspace:
                self.workspace, self._ws_ptr = None, None
                self.h = sim_create_static(self.desc, self.N)
            else:
                self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
                base = self.workspace.data_ptr()
                self._ws_ptr = (base + 255) & ~255
                self.h = sim_create(self.desc, self.N, self._ws_ptr, nbytes)
        L = lib()
        self.B, self.S = L.sim_num_bodies(self.h), L.sim_num_slots(self.h)
        self.J = int(scene.robot.n_joints)
        self.obs_dim, self.act_dim = L.sim_obs_dim(self.h), L.sim_act_dim(self.h)
        f32 = dict(dtype=torch.float32, device=self.device)
        self.obs = torch.zeros(self.N, self.obs_dim, **f32)
        self.reward = torch.zeros(self.N, **f32)
        self.done = torch.zeros(self.N, dtype=torch.uint8, device=self.device)
        self._delivered = False

    def close(self):
        if getattr(self, "h", None):
            self.torch.cuda.synchronize(self.device)
            sim_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self):
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def _dev(self, a, dtype):
        t = self.torch
        if isinstance(a, t.Tensor):
            return a.to(device=self.device, dtype=dtype).contiguous()
        # (a copy: torch refuses to wrap arrays that are not writable, e.g. broadcast views)
        return t.as_tensor(np.array(a, order="C", copy=True), dtype=dtype).to(self.device)

    def reset(self, seed=0, mask=None):
        m = None if mask is None else self._dev(mask, self.torch.uint8)
        sim_reset(self.h, None if m is None else m.data_ptr(), seed, self._stream())
        self._delivered = False

    def step(self, actions, dt, substeps, iterations):
        a = None if actions is None else self._dev(actions, self.torch.float32)
        if a is not None and tuple(a.shape) != (self.N, self.act_dim):
            raise ValueError(f"actions must be [{self.N}][{self.act_dim}]")
        sim_step(self.h, None if a is None else a.data_ptr(), dt, substeps, iterations, self._stream())
        self._delivered = False

    def step_obs(self, actions, dt, substeps, iterations):
        a = None if actions is None else self._dev(actions, self.torch.float32)
        if a is not None and tuple(a.shape) != (self.N, self.act_dim):
            raise ValueError(f"actions must be [{self.N}][{self.act_dim}]")
        sim_step_obs(self.h, None if a is None else a.data_ptr(), dt, substeps, iterations, self.obs.data_ptr(),
                     self.reward.data_ptr(), self.done.data_ptr(), self._stream())
        self._delivered = True     # the step wrote into self.obs / reward / done; the library kept no copy
        return self.obs, self.reward, self.done

    def set_task(self, task):
        sim_set_task(self.h, task, self._stream())

    def get_kept_impulses(self):
        """Warm start: joint row impulses [N][J][6] and terrain slot impulses [N][S][3] kept for the next substep."""
        t = self.torch
        lj = t.zeros(self.N, self.J, 6, dtype=t.float32, device=self.device)
        ls = t.zeros(self.N, self.S, 3, dtype=t.float32, device=self.device)
        sim_get_kept_impulses(self.h, lj.data_ptr(), ls.data_ptr(), self._stream())
        return lj, ls

    def get_task_state(self):
        t = self.torch
        c = t.empty(self.N, 4, dtype=t.int32, device=self.device)
        tg = t.empty(self.N, 2, dtype=t.float32, device=self.device)
        p = t.empty(self.N, 3, dtype=t.float32, device=self.device)
        sim_get_task_state(self.h, c.data_ptr(), tg.data_ptr(), p.data_ptr(), self._stream())
        return c, tg, p

    def set_task_state(self, counters, targets):
        c = self._dev(np.asarray(counters, np.int32).reshape(self.N, 4), self.torch.int32)
        tg = self._dev(np.asarray(targets, np.float32).reshape(self.N, 2), self.torch.float32)
        sim_set_task_state(self.h, c.data_ptr(), tg.data_ptr(), self._stream())

    def get_obs(self):
        if self._delivered:
            return self.obs, self.reward, self.done
        sim_get_obs(self.h, self.obs.data_ptr(), self.reward.data_ptr(), self.done.data_ptr(), self._stream())
        return self.obs, self.reward, self.done

    def set_targets(self, xy):
        t = self._dev(xy, self.torch.float32)
        if t.numel() != self.N * 2:
            raise ValueError("targets must be [N][2]")
        sim_set_targets(self.h, t.data_ptr(), self._stream())

    def get_state(self):
        s = self.torch.empty(self.N, self.B, 13, dtype=self.torch.float32, device=self.device)
        sim_get_state(self.h, s.data_ptr(), self._stream())
        return s

    def set_state(self, state):
        s = self._dev(state, self.torch.float32)
        if s.numel() != self.N * self.B * 13:
            raise ValueError("state must be [N][B][13]")
        sim_set_state(self.h, s.data_ptr(), self._stream())
        self._delivered = False

    def set_step_count(self, counts):
        c = self._dev(np.broadcast_to(np.asarray(counts, np.int32), (self.N,)), self.torch.int32)
        sim_set_step_count(self.h, c.data_ptr(), self._stream())

    def record_contacts(self, enable=True):
        sim_record_contacts(self.h, 1 if enable else 0)

    def _recs(self, fn):
        buf = self.torch.empty(self.N * self.S * CONTACT_DTYPE.itemsize, dtype=self.torch.uint8, device=self.device)
        fn(self.h, buf.data_ptr(), self._stream())
        return buf.cpu().numpy().view(CONTACT_DTYPE).reshape(self.N, self.S)

    def get_contacts(self):
        return self._recs(sim_get_contacts)

    def generate_contacts(self):
        return self._recs(sim_generate_contacts)

    def get_pair_contacts(self, cap=4096):
        """(records, dropped): capsule-capsule contacts of the last substep of the last step."""
        buf = self.torch.zeros(cap * PAIR_CONTACT_DTYPE.itemsize, dtype=self.torch.uint8, device=self.device)
        cnt = self.torch.zeros(2, dtype=self.torch.int32, device=self.device)
        sim_get_pair_contacts(self.h, buf.data_ptr(), cap, cnt.data_ptr(), self._stream())
        n, dropped = (int(v) for v in cnt.cpu().numpy())
        return buf.cpu().numpy().view(PAIR_CONTACT_DTYPE)[:min(n, cap)].copy(), dropped

    def regroup(self, cell, reach):
        """Interaction groups from the agents' positions: order along the Hilbert curve through a grid of
        `cell` metres, then groups of agents within `reach` of each other inside windows of that order."""
        sim_regroup(self.h, cell, reach, self._stream())

    def set_groups(self, place_env):
        """place_env[N]: the agent at every place (a permutation); None: every agent at its own."""
        if place_env is None:
            sim_set_groups(self.h, None, self._stream())
            return
        pe = self.torch.as_tensor(np.array(place_env, np.int32, copy=True)).to(self.device)
        sim_set_groups(self.h, pe.data_ptr(), self._stream())

    def get_groups(self):
        pe = self.torch.zeros(self.N, dtype=self.torch.int32, device=self.device)
        sim_get_groups(self.h, pe.data_ptr(), self._stream())
        return pe.cpu().numpy()

    def count_near_pairs(self, reach):
        """(agent pairs whose roots are within `reach`, those of them in different groups)"""
        c = self.torch.zeros(2, dtype=self.torch.int64, device=self.device)
        sim_count_near_pairs(self.h, reach, c.data_ptr(), self._stream())
        return tuple(int(v) for v in c.cpu().numpy())

    def check(self):
        sim_check(self.h, self._stream())

    def launch_info(self):
        return sim_launch_info(self.h)

    def set_envs_per_block(self, e):
        sim_set_envs_per_block(self.h, e)
