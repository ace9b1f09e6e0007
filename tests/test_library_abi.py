"""Host-only checks of the C-ABI shared library: it loads, exports every symbol
the header declares, and validates descriptions without touching a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import scenes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "sim.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sim_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_1810_05762_amd as P
    lib = P.load_library()
    names = _declared_symbols()
    assert len(names) >= 20 and "sim_step" in names and "sim_create" in names
    for n in names:
        assert hasattr(lib, n), n
    # the binding wraps the same set, name for name
    from paper_1810_05762_amd import binding
    assert sorted(binding._SYMBOLS) == names


def test_workspace_size_and_description_validation_need_no_gpu():
    import paper_1810_05762_amd as P
    sc, _ = scenes.config_scene(3, num_envs=100)
    d, keep = P.make_desc(sc)
    n100 = P.sim_workspace_bytes(d, 100)
    n200 = P.sim_workspace_bytes(d, 200)
    assert n200 > n100 > 256 * 256 * 4           # holds the heightfield at least
    for field, value in (("n_bodies", 0), ("n_bodies", 99), ("terrain_kind", 7), ("root_body", 50),
                         ("hf_cell", 0.0), ("n_feet", 9)):
        d2, keep2 = P.make_desc(sc)
        setattr(d2, field, value)
        with pytest.raises(P.SimError) as ei:
            P.sim_workspace_bytes(d2, 100)
        assert ei.value.code == -1 and P.sim_last_error()
    with pytest.raises(P.SimError):
        P.sim_workspace_bytes(d, 0)
    d3, keep3 = P.make_desc(sc)
    d3.joints[0].parent = d3.joints[0].child       # self-joint
    with pytest.raises(P.SimError):
        P.sim_workspace_bytes(d3, 10)


def test_collision_description_validation_needs_no_gpu():
    import ctypes as C
    import numpy as np
    import paper_1810_05762_amd as P
    rob = scenes.make_humanoid()
    sc = scenes.make_scene(rob, scenes.make_plane(), 64, params=scenes.SimParams(self_collide=1, group_size=4), spacing=1.0)
    d, keep = P.make_desc(sc)
    assert d.n_collide_pairs == len(rob.collide_pairs) > 0 and d.group_size == 4
    plain, _k = P.make_desc(scenes.make_scene(rob, scenes.make_plane(), 64))
    assert P.sim_workspace_bytes(d, 64) > P.sim_workspace_bytes(plain, 64)   # room for the contact records
    # the list never names two bodies that a joint connects
    joined = {(min(a, b), max(a, b)) for a, b in zip(rob.j_parent, rob.j_child)}
    assert not joined & {tuple(p) for p in rob.collide_pairs.tolist()}
    for field, value in (("group_size", 17), ("group_size", -1), ("n_collide_pairs", 500)):
        d2, keep2 = P.make_desc(sc)
        setattr(d2, field, value)
        with pytest.raises(P.SimError):
            P.sim_workspace_bytes(d2, 64)
    for bad in ((3, 3), (5, 2), (0, 13), (-1, 2)):
        d2, keep2 = P.make_desc(sc)
        arr = np.array([bad], np.int32)
        d2.n_collide_pairs, d2.collide_pairs = 1, arr.ctypes.data_as(C.POINTER(C.c_int32))
        with pytest.raises(P.SimError):
            P.sim_workspace_bytes(d2, 64)
    d2, keep2 = P.make_desc(sc)
    d2.collide_pairs = None
    with pytest.raises(P.SimError):
        P.sim_workspace_bytes(d2, 64)


def test_warm_start_description_validation_needs_no_gpu():
    import paper_1810_05762_amd as P
    rob = scenes.make_humanoid()
    plain, _k = P.make_desc(scenes.make_scene(rob, scenes.make_plane(), 64))
    warm, _k2 = P.make_desc(scenes.make_scene(rob, scenes.make_plane(), 64, params=scenes.SimParams(warm_start=0.8)))
    assert warm.warm_start == 0.8 and plain.warm_start == 0.0
    # room for the kept impulses: 6 per joint and 3 per slot, one float each, per env
    extra = P.sim_workspace_bytes(warm, 64) - P.sim_workspace_bytes(plain, 64)
    assert extra >= 64 * 4 * (6 * rob.n_joints + 3 * 2 * rob.n_bodies)
    for bad in (-0.1, 1.5, float("nan")):
        d, _k3 = P.make_desc(scenes.make_scene(rob, scenes.make_plane(), 64))
        d.warm_start = bad
        with pytest.raises(P.SimError):
            P.sim_workspace_bytes(d, 64)
    # together with collisions: accepted, the same room for the kept impulses on top
    both = scenes.make_scene(rob, scenes.make_plane(), 64, params=scenes.SimParams(self_collide=1, warm_start=0.5))
    coll = scenes.make_scene(rob, scenes.make_plane(), 64, params=scenes.SimParams(self_collide=1))
    assert P.sim_workspace_bytes(P.make_desc(both)[0], 64) - P.sim_workspace_bytes(P.make_desc(coll)[0], 64) == extra


def test_robots_beyond_the_size_limits_are_rejected_without_a_gpu():
    import paper_1810_05762_amd as P
    from scenes.robots import _Builder

    def chain(n, hinges):
        bld = _Builder("chain")
        prev = -1
        for k in range(n):
            b = bld.body(f"l{k}", 0.03, 0.1, 2, (0.0, 0.0, 3.0 - (k + 0.5) * 0.1), mass=0.3)
            bld.joint(prev, b, (0.0, 0.0, 3.0 - k * 0.1), [((0.0, 1.0, 0.0), -1.0, 1.0), ((1.0, 0.0, 0.0), -1.0, 1.0), ((0.0, 0.0, 1.0), -1.0, 1.0)][:hinges], 1.0)
            prev = b
        return bld.build(root_body=0, feet=(), term_height=-1e9, alive_bonus=0.0)

    ok = scenes.make_scene(chain(16, 2), scenes.make_plane(), 8)          # 16 bodies, 16 joints, 32 dofs: the limits
    assert P.sim_workspace_bytes(P.make_desc(ok)[0], 8) > 0
    for rob in (chain(17, 1), chain(12, 3)):                               # 17 bodies / joints; 36 dofs
        with pytest.raises(P.SimError):
            P.sim_workspace_bytes(P.make_desc(scenes.make_scene(rob, scenes.make_plane(), 8))[0], 8)


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_1810_05762_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f


def test_static_workspace_entry_point_rejects_oversize_descriptions_without_a_gpu():
    """sim_create_static checks the size before it touches the device."""
    import paper_1810_05762_amd as P
    sc, _ = scenes.config_scene(3, num_envs=16384)
    d, keep = P.make_desc(sc)
    assert P.sim_workspace_bytes(d, 16384) > 24 << 20
    with pytest.raises(P.SimError) as ei:
        P.sim_create_static(d, 16384)
    assert ei.value.code == -2 and "static workspace holds" in str(ei.value)


@pytest.mark.parametrize("kind,maker", [(1, "make_ant"), (2, "make_humanoid")])
def test_built_in_robot_tables_equal_the_shared_input_recipe(kind, maker):
    """The library's own ant and humanoid (sim_builtin_robot) are the robots of the benchmark
    configurations: every number of the tables equals the one the input module builds (host
    arithmetic in double on both sides; r ** 3 against r * r * r allows a last-digit difference),
    and the default parameters are the configurations'."""
    import paper_1810_05762_amd as P
    rob = getattr(scenes, maker)()
    ref, _keep = P.make_desc(scenes.make_scene(rob, scenes.make_plane(), 4))
    d = P.sim_builtin_robot(kind)
    assert (d.n_bodies, d.n_joints, d.root_body, d.n_feet) == (ref.n_bodies, ref.n_joints, ref.root_body, ref.n_feet)
    assert list(d.foot_bodies)[:d.n_feet] == list(ref.foot_bodies)[:ref.n_feet]
    assert (d.term_height, d.alive_bonus) == (ref.term_height, ref.alive_bonus)
    for b in range(d.n_bodies):
        x, y = d.bodies[b], ref.bodies[b]
        assert x.axis == y.axis
        got = [x.radius, x.half_len, x.mass, *x.inertia, *x.rest_pos]
        want = [y.radius, y.half_len, y.mass, *y.inertia, *y.rest_pos]
        np.testing.assert_allclose(got, want, rtol=1e-14, atol=0)
    n_act = 0
    for j in range(d.n_joints):
        x, y = d.joints[j], ref.joints[j]
        assert (x.parent, x.child, list(x.mode), list(x.act)) == (y.parent, y.child, list(y.mode), list(y.act))
        got = [*x.anchor, *[v for row in x.axes for v in row], *x.lo, *x.hi, *x.gear]
        want = [*y.anchor, *[v for row in y.axes for v in row], *y.lo, *y.hi, *y.gear]
        np.testing.assert_allclose(got, want, rtol=1e-14, atol=1e-300)
        n_act += sum(1 for m in x.mode if m == 1)
    assert n_act == rob.n_dofs
    for f in ("max_episode_steps", "mu", "contact_margin", "beta_joint", "beta_contact", "max_depen_vel", "lin_damping",
              "ang_damping", "max_ang_vel", "reset_noise", "gyroscopic", "contacts", "height_map", "group_size",
              "warm_start", "solver", "krylov_iterations"):
        assert getattr(d, f) == getattr(ref, f), f
    assert list(d.gravity) == list(ref.gravity) and d.terrain_kind == 0 and d.n_collide_pairs == 0
    with pytest.raises(P.SimError):
        P.sim_builtin_robot(3)
    # complete once the caller has added where the envs stand: the same workspace as the recipe's
    org = np.ascontiguousarray(scenes.make_scene(rob, scenes.make_plane(), 4).env_origins, np.float64)
    d.env_origins = org.ctypes.data_as(type(d.env_origins))
    assert P.sim_workspace_bytes(d, 4) == P.sim_workspace_bytes(ref, 4)


def test_header_is_a_plain_c_header():
    """include/sim.h compiles as C11 and as C++17 on its own (no HIP, no other header of the build)."""
    import subprocess
    hdr = os.path.join(ROOT, "include", "sim.h")
    for cmd in (["gcc", "-std=c11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr],
                ["g++", "-std=c++17", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c++", hdr]):
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
