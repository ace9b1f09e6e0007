"""ctypes wrapper around the fp64 CPU oracle (oracle/oracle.c).

TEST INFRASTRUCTURE ONLY: import this from tests, the smoke check and the
benchmark's CPU-baseline leg, never from the product package.  It takes the same
`scenes.Scene` input description as the HIP binding but shares no code with it.
"""
import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile oracle.c with gcc (no FMA contraction, OpenMP over envs)."""
    src = os.path.join(_HERE, "oracle.c")
    hdr = os.path.join(_HERE, "oracle.h")
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
        return _LIB_PATH
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC",
           "-shared", "-Wall", "-Wno-misleading-indentation", "-o", _LIB_PATH, src, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


class _Desc(C.Structure):
    _d = C.POINTER(C.c_double)
    _i = C.POINTER(C.c_int32)
    _fields_ = [
        ("n_bodies", C.c_int32), ("n_joints", C.c_int32), ("n_dofs", C.c_int32), ("n_feet", C.c_int32),
        ("radius", _d), ("half_len", _d), ("axis", _i), ("mass", _d), ("inertia", _d), ("rest_pos", _d),
        ("j_parent", _i), ("j_child", _i), ("j_anchor", _d), ("j_axes", _d), ("j_mode", _i),
        ("j_lo", _d), ("j_hi", _d), ("j_gear", _d), ("j_act", _i),
        ("root_body", C.c_int32), ("feet", _i), ("term_height", C.c_double), ("alive_bonus", C.c_double),
        ("terrain_kind", C.c_int32), ("hf_nx", C.c_int32), ("hf_ny", C.c_int32),
        ("hf_cell", C.c_double), ("hf_origin", C.c_double * 2), ("hf_heights", C.POINTER(C.c_float)),
        ("env_origins", _d),
        ("gravity", C.c_double * 3), ("mu", C.c_double), ("margin", C.c_double),
        ("beta_joint", C.c_double), ("beta_contact", C.c_double), ("max_depen_vel", C.c_double),
        ("lin_damping", C.c_double), ("ang_damping", C.c_double), ("max_ang_vel", C.c_double),
        ("reset_noise", C.c_double),
        ("gyroscopic", C.c_int32), ("contacts", C.c_int32), ("max_episode_steps", C.c_int32),
        ("height_map", C.c_int32),
        ("n_collide_pairs", C.c_int32), ("collide_pairs", _i), ("group_size", C.c_int32),
    ]


class Contact(C.Structure):
    _fields_ = [("active", C.c_int32), ("kind", C.c_int32), ("feat", C.c_int32), ("pad", C.c_int32),
                ("d", C.c_double), ("n", C.c_double * 3), ("rc", C.c_double * 3), ("w", C.c_double)]


PAIR_CONTACT_DTYPE = np.dtype([("env_a", np.int32), ("body_a", np.int32), ("env_b", np.int32),
                               ("body_b", np.int32), ("s", np.float32), ("t", np.float32),
                               ("d", np.float64), ("n", np.float64, 3), ("ra", np.float64, 3),
                               ("rb", np.float64, 3), ("w", np.float64), ("gap32", np.float32),
                               ("pad", np.int32)])
CONTACT_DTYPE = np.dtype([("active", np.int32), ("kind", np.int32), ("feat", np.int32), ("pad", np.int32),
                          ("d", np.float64), ("n", np.float64, 3), ("rc", np.float64, 3),
                          ("w", np.float64)])
TRACE_DTYPE = np.dtype([("bilateral_rms", np.float64), ("bilateral_max", np.float64),
                        ("onesided_viol", np.float64), ("sum_lambda_n", np.float64),
                        ("cone_excess", np.float64), ("pos_err_max", np.float64)])

PH_CONTACTS, PH_FORCES, PH_SOLVE, PH_INTEGRATE, PH_ALL = 1, 2, 4, 8, 15


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = C.CDLL(_LIB_PATH)
    vp, dp, ip = C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int32)
    L.oracle_create.restype = vp
    L.oracle_create.argtypes = [C.POINTER(_Desc), C.c_int32]
    L.oracle_destroy.argtypes = [vp]
    L.oracle_n_slots.argtypes = [vp]
    L.oracle_obs_dim.argtypes = [vp]
    L.oracle_set_threads.argtypes = [vp, C.c_int32]
    L.oracle_get_threads.argtypes = [vp]
    L.oracle_set_warm_start.argtypes = [vp, C.c_double]
    L.oracle_set_solver.argtypes = [vp, C.c_int32, C.c_int32, C.c_double]
    L.oracle_set_pair_cap.argtypes = [vp, C.c_int32, C.c_int32]
    L.oracle_set_pair_cap.restype = C.c_int64
    L.oracle_regroup.argtypes = [vp, C.c_double, C.c_double]
    L.oracle_set_groups.argtypes = [vp, ip]
    L.oracle_set_groups.restype = C.c_int32
    L.oracle_get_groups.argtypes = [vp, ip]
    L.oracle_count_near_pairs.argtypes = [vp, C.c_double, C.c_void_p]
    L.oracle_get_warm.argtypes = [vp, dp, dp]
    L.oracle_set_warm.argtypes = [vp, dp, dp]
    L.oracle_set_warm_flags.argtypes = [vp, ip, ip]
    L.oracle_reset.argtypes = [vp, C.c_void_p, C.c_uint64]
    L.oracle_set_state.argtypes = [vp, dp]
    L.oracle_get_state.argtypes = [vp, dp]
    L.oracle_set_targets.argtypes = [vp, dp]
    L.oracle_set_step_count.argtypes = [vp, ip]
    L.oracle_step.argtypes = [vp, dp, C.c_double, C.c_int32, C.c_int32]
    L.oracle_substep_phases.argtypes = [vp, dp, C.c_double, C.c_int32, C.c_int32]
    L.oracle_get_obs.argtypes = [vp, dp, dp, C.c_void_p]
    L.oracle_get_contacts.argtypes = [vp, C.c_void_p]
    L.oracle_generate_contacts.argtypes = [vp, C.c_int32, C.c_void_p]
    L.oracle_set_trace.argtypes = [vp, C.c_int32, C.c_void_p, C.c_int32]
    L.oracle_trace_count.argtypes = [vp]
    L.oracle_joint_angles.argtypes = [vp, dp]
    L.oracle_set_task.argtypes = [vp, C.c_void_p]
    L.oracle_get_task_state.argtypes = [vp, ip, dp]
    L.oracle_set_task_state.argtypes = [vp, ip, dp]
    L.oracle_get_last_push.argtypes = [vp, dp]
    L.oracle_get_pair_contacts.argtypes = [vp, C.c_void_p, C.c_int32]
    L.oracle_generate_pair_contacts.argtypes = [vp, C.c_void_p, C.c_int32]
    fp = C.POINTER(C.c_float)
    L.oracle_segment_segment_f32.restype = C.c_float
    L.oracle_segment_segment_f32.argtypes = [fp, fp, fp, fp, fp, fp]
    L.oracle_uniform.restype = C.c_double
    L.oracle_uniform.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
    _lib = L
    return L


def uniform(seed, env, idx):
    return float(_load().oracle_uniform(seed, env, idx))


def segment_segment_f32(P0, P1, Q0, Q1):
    """(d2, s, t) of the oracle's single-precision segment-segment closest points."""
    a = [np.ascontiguousarray(x, dtype=np.float32) for x in (P0, P1, Q0, Q1)]
    s, t = C.c_float(), C.c_float()
    fp = C.POINTER(C.c_float)
    d2 = _load().oracle_segment_segment_f32(*[x.ctypes.data_as(fp) for x in a], C.byref(s), C.byref(t))
    return float(d2), float(s.value), float(t.value)


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


class _Task(C.Structure):
    _fields_ = [("enabled", C.c_int32), ("fall_grace_frames", C.c_int32), ("target_period", C.c_int32),
                ("push_min_frames", C.c_int32), ("push_max_frames", C.c_int32), ("auto_reset", C.c_int32),
                ("target_reach", C.c_double), ("target_radius", C.c_double),
                ("push_min_newton", C.c_double), ("push_max_newton", C.c_double), ("seed", C.c_uint64)]


class OracleSim:
    """fp64 reference simulator for a `scenes.Scene`."""

    def __init__(self, scene, threads=1):
        L = _load()
        self._L = L
        r, t, p = scene.robot, scene.terrain, scene.params
        f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
        i32 = lambda a: np.ascontiguousarray(a, dtype=np.int32)
        keep = dict(
            radius=f64(r.radius), half_len=f64(r.half_len), axis=i32(r.axis), mass=f64(r.mass),
            inertia=f64(r.inertia), rest_pos=f64(r.rest_pos), j_parent=i32(r.j_parent),
            j_child=i32(r.j_child), j_anchor=f64(r.j_anchor), j_axes=f64(r.j_axes), j_mode=i32(r.j_mode),
            j_lo=f64(r.j_lo), j_hi=f64(r.j_hi), j_gear=f64(r.j_gear), j_act=i32(r.j_act),
            feet=i32(np.array(list(r.feet) + [0], dtype=np.int32)),
            heights=np.ascontiguousarray(t.heights, dtype=np.float32),
            env_origins=f64(scene.env_origins),
            pairs=i32(r.collide_pairs if getattr(p, "self_collide", 0) else np.zeros((0, 2), np.int32)),
        )
        self._keep = keep
        d = _Desc()
        d.n_bodies, d.n_joints, d.n_dofs, d.n_feet = r.n_bodies, r.n_joints, r.n_dofs, len(r.feet)
        for k in ("radius", "half_len", "mass", "inertia", "rest_pos", "j_anchor", "j_axes", "j_lo",
                  "j_hi", "j_gear", "env_origins"):
            setattr(d, k, _dp(keep[k]))
        for k in ("axis", "j_parent", "j_child", "j_mode", "j_act", "feet"):
            setattr(d, k, _ip(keep[k]))
        d.root_body, d.term_height, d.alive_bonus = r.root_body, r.term_height, r.alive_bonus
        d.terrain_kind, d.hf_nx, d.hf_ny, d.hf_cell = t.kind, t.nx, t.ny, t.cell
        d.hf_origin[0], d.hf_origin[1] = t.origin
        d.hf_heights = keep["heights"].ctypes.data_as(C.POINTER(C.c_float))
        for i in range(3):
            d.gravity[i] = p.gravity[i]
        d.mu, d.margin, d.beta_joint, d.beta_contact = p.mu, p.contact_margin, p.beta_joint, p.beta_contact
        d.max_depen_vel, d.lin_damping, d.ang_damping = p.max_depen_vel, p.lin_damping, p.ang_damping
        d.max_ang_vel, d.reset_noise = p.max_ang_vel, p.reset_noise
        d.gyroscopic, d.contacts, d.max_episode_steps = p.gyroscopic, p.contacts, p.max_episode_steps
        d.height_map = int(getattr(p, "height_map", 0))
        d.n_collide_pairs = int(keep["pairs"].shape[0])
        d.collide_pairs = _ip(keep["pairs"]) if d.n_collide_pairs else None
        d.group_size = int(getattr(p, "group_size", 1))
        self.N, self.B, self.J, self.D = scene.num_envs, r.n_bodies, r.n_joints, r.n_dofs
        self._h = L.oracle_create(C.byref(d), self.N)
        if not self._h:
            raise RuntimeError("oracle_create failed (model too large)")
        self.S = L.oracle_n_slots(self._h)
        self.obs_dim = L.oracle_obs_dim(self._h)
        self._trace = None
        L.oracle_set_threads(self._h, int(threads))
        L.oracle_set_warm_start(self._h, float(getattr(p, "warm_start", 0.0)))
        L.oracle_set_solver(self._h, int(getattr(p, "solver", 0)), int(getattr(p, "krylov_iters", 8)),
                            float(getattr(p, "newton_reg", 0.0)))

    def __del__(self):
        if getattr(self, "_h", None):
            self._L.oracle_destroy(self._h)
            self._h = None

    def set_threads(self, n):
        self._L.oracle_set_threads(self._h, int(n))

    def set_warm_start(self, share):
        """Rows start each substep from `share` (0..1) of their impulse at the end of the previous one."""
        self._L.oracle_set_warm_start(self._h, float(share))

    def set_solver(self, kind, krylov_iters=8, reg=0.0):
        """kind 0: block projected Jacobi; 1: non-smooth Newton with `krylov_iters` conjugate-residual
        iterations per Newton iteration (the `iterations` of step() then count Newton iterations)."""
        self._L.oracle_set_solver(self._h, int(kind), int(krylov_iters), float(reg))

    def set_pair_cap(self, cap, envs_per_unit):
        """Bounded contact store: every block of `envs_per_unit` consecutive agents keeps at most
        `cap` capsule-capsule contacts per substep, those with the smallest (single-precision gap,
        key).  cap <= 0 lifts the bound.  Returns the number removed since the last call."""
        return int(self._L.oracle_set_pair_cap(self._h, int(cap), int(envs_per_unit)))

    def regroup(self, cell, reach):
        """Interaction groups from the agents' positions: order along the Hilbert curve through a grid
        of `cell` metres; inside windows of that order, groups of agents within `reach` of each other."""
        self._L.oracle_regroup(self._h, float(cell), float(reach))

    def set_groups(self, place_env):
        """place_env[N]: a permutation of the agents, groups are consecutive places (None: identity)."""
        if place_env is None:
            rc = self._L.oracle_set_groups(self._h, None)
        else:
            pe = np.ascontiguousarray(place_env, np.int32).reshape(self.N)
            rc = self._L.oracle_set_groups(self._h, pe.ctypes.data_as(C.POINTER(C.c_int32)))
        if rc != 0:
            raise ValueError("place_env is not a permutation of the agents")

    def get_groups(self):
        pe = np.zeros(self.N, np.int32)
        self._L.oracle_get_groups(self._h, pe.ctypes.data_as(C.POINTER(C.c_int32)))
        return pe

    def count_near_pairs(self, reach):
        """(agent pairs whose roots are within `reach`, those of them in different groups)"""
        c = np.zeros(2, np.int64)
        self._L.oracle_count_near_pairs(self._h, float(reach), c.ctypes.data)
        return int(c[0]), int(c[1])

    def set_warm(self, lam_j, lam_s):
        lj = np.ascontiguousarray(lam_j, np.float64).reshape(self.N, self.J, 6)
        ls = np.ascontiguousarray(lam_s, np.float64).reshape(self.N, self.S, 3)
        self._L.oracle_set_warm(self._h, _dp(lj), _dp(ls))

    def set_warm_flags(self, limit_side, slot_was_active):
        """Bookkeeping of the kept impulses: which limit a hinge row's stood for ([N][J][3]: 0 lower,
        1 upper, -1 whichever is nearer now) and whether a slot was active in the previous substep."""
        sd = np.ascontiguousarray(limit_side, np.int32).reshape(self.N, self.J, 3)
        on = np.ascontiguousarray(slot_was_active, np.int32).reshape(self.N, self.S)
        self._L.oracle_set_warm_flags(self._h, _ip(sd), _ip(on))

    def get_warm(self):
        """Impulses kept for the next substep: joints [N][J][6], terrain slots [N][S][3]."""
        lj = np.zeros((self.N, self.J, 6)); ls = np.zeros((self.N, self.S, 3))
        self._L.oracle_get_warm(self._h, _dp(lj), _dp(ls))
        return lj, ls

    def reset(self, seed=0, mask=None):
        m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
        self._L.oracle_reset(self._h, None if m is None else m.ctypes.data, int(seed))

    def set_state(self, state):
        s = np.ascontiguousarray(state, dtype=np.float64).reshape(self.N, self.B, 13)
        self._L.oracle_set_state(self._h, _dp(s))

    def get_state(self):
        s = np.empty((self.N, self.B, 13), np.float64)
        self._L.oracle_get_state(self._h, _dp(s))
        return s

    def set_targets(self, xy):
        t = np.ascontiguousarray(xy, dtype=np.float64).reshape(self.N, 2)
        self._L.oracle_set_targets(self._h, _dp(t))

    def set_task(self, task):
        """task: scenes.TaskParams or None (off).  Initialises the per-env task state."""
        if task is None:
            self._L.oracle_set_task(self._h, None)
            return
        t = _Task()
        for name, _ in _Task._fields_:
            setattr(t, name, getattr(task, name))
        self._L.oracle_set_task(self._h, C.addressof(t))

    def get_task_state(self):
        c = np.zeros((self.N, 4), np.int32)
        t = np.zeros((self.N, 2), np.float64)
        self._L.oracle_get_task_state(self._h, _ip(c), _dp(t))
        return c, t

    def set_task_state(self, counters, targets):
        c = np.ascontiguousarray(counters, dtype=np.int32).reshape(self.N, 4)
        t = np.ascontiguousarray(targets, dtype=np.float64).reshape(self.N, 2)
        self._L.oracle_set_task_state(self._h, _ip(c), _dp(t))

    def get_last_push(self):
        p = np.zeros((self.N, 3), np.float64)
        self._L.oracle_get_last_push(self._h, _dp(p))
        return p

    def set_step_count(self, counts):
        c = np.ascontiguousarray(np.broadcast_to(np.asarray(counts, np.int32), (self.N,)))
        self._L.oracle_set_step_count(self._h, _ip(c))

    def _act(self, actions):
        if actions is None:
            return None, None
        a = np.ascontiguousarray(actions, dtype=np.float64).reshape(self.N, self.D)
        return a, _dp(a)

    def step(self, actions, dt, substeps, iterations):
        a, p = self._act(actions)
        self._L.oracle_step(self._h, p, float(dt), int(substeps), int(iterations))

    def substep_phases(self, actions, h, iterations, phases=PH_ALL):
        a, p = self._act(actions)
        self._L.oracle_substep_phases(self._h, p, float(h), int(iterations), int(phases))

    def get_obs(self):
        obs = np.empty((self.N, self.obs_dim), np.float64)
        rew = np.empty(self.N, np.float64)
        done = np.empty(self.N, np.uint8)
        self._L.oracle_get_obs(self._h, _dp(obs), _dp(rew), done.ctypes.data)
        return obs, rew, done

    def get_contacts(self):
        rec = np.zeros((self.N, self.S), CONTACT_DTYPE)
        self._L.oracle_get_contacts(self._h, rec.ctypes.data)
        return rec

    def generate_contacts(self, brute=False):
        rec = np.zeros((self.N, self.S), CONTACT_DTYPE)
        self._L.oracle_generate_contacts(self._h, 1 if brute else 0, rec.ctypes.data)
        return rec

    def get_pair_contacts(self, cap=4096):
        """Capsule-capsule contacts of the last substep (all groups, in order)."""
        rec = np.zeros(cap, PAIR_CONTACT_DTYPE)
        n = self._L.oracle_get_pair_contacts(self._h, rec.ctypes.data, cap)
        return rec[:min(n, cap)].copy()

    def generate_pair_contacts(self, cap=4096):
        rec = np.zeros(cap, PAIR_CONTACT_DTYPE)
        n = self._L.oracle_generate_pair_contacts(self._h, rec.ctypes.data, cap)
        return rec[:min(n, cap)].copy()

    def start_trace(self, env=0, cap=4096):
        self._trace = np.zeros(cap, TRACE_DTYPE)
        self._L.oracle_set_trace(self._h, int(env), self._trace.ctypes.data, cap)

    def trace(self):
        n = self._L.oracle_trace_count(self._h)
        return self._trace[:n].copy()

    def joint_angles(self):
        th = np.empty((self.N, self.J, 3), np.float64)
        self._L.oracle_joint_angles(self._h, _dp(th))
        return th
