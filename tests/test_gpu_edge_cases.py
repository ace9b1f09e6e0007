"""GPU parity on the degenerate shapes of the method: no joints, a joint to the world, a body
in more joints than the specialised kernel handles, more active contacts than contact threads,
reach boxes too large for the packed work units, one env, zero solver sweeps.  Same bar as the
main parity tests: contact sets bit-exact, states within 1e-4 after one step and 1e-3 after ten."""
import numpy as np
import pytest

import oracle
import scenes
from test_gpu_parity import rel_err, _same_sets

pytestmark = pytest.mark.gpu


def _pair(sc, state=None):
    import paper_1810_05762_amd as P
    sim = P.Sim(sc)
    st = scenes.rest_state(sc.robot, sc.num_envs) if state is None else state
    sim.set_state(st)
    ref = oracle.OracleSim(sc, threads=4)
    ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    return sim, ref


def _run(sim, ref, sc, seed, dt, sub, its, steps, check_at=(1, 10), record=True, warm=0):
    """Steps both sides with the same seeded actions; after `warm` steps the oracle is restarted
    from the GPU's fp32 state, then states are compared `check_at` steps later."""
    N, D = sc.num_envs, sc.robot.n_dofs
    if record:
        sim.record_contacts(True)
    act = lambda s: scenes.actions_for_step(seed, s, N, D) if D > 0 else None
    for s in range(warm):
        sim.step(act(s), dt, sub, its)
    ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    worst = {}
    for s in range(warm, warm + steps):
        # contact sets on identical states are only comparable at the restart step
        sim.step(act(s), dt, sub, its)
        ref.step(act(s), dt, sub, its)
        n = s - warm + 1
        if n in check_at:
            e = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
            worst[n] = e.max()
    sim.check()
    return worst


def test_world_anchored_chain_on_plane():
    sc = scenes.make_scene(scenes.make_chain(n_links=4, direction=(1.0, 0.0, 0.0), top=(0.0, 0.0, 1.5)),
                           scenes.make_plane(), 5)
    sim, ref = _pair(sc)
    w = _run(sim, ref, sc, 11, 1 / 60, 4, 20, 10)
    assert w[1] <= 1e-4 and w[10] <= 1e-3, w
    # the chain swings: it must have moved, and its first anchor must still be near the world point
    st = sim.get_state().cpu().numpy()
    assert np.abs(st[:, 3, 2] - 1.5).max() > 1e-3
    sim.close()


@pytest.mark.parametrize("terrain", ["plane", "heightfield"])
def test_single_sphere_one_env_drops_and_rests(terrain):
    ter = scenes.make_plane() if terrain == "plane" else scenes.make_heightfield(seed=1003)
    sc = scenes.make_scene(scenes.make_single(radius=0.1, pos=(0.0, 0.0, 0.25)), ter, 1, seed=3)
    if terrain == "heightfield":
        # start 0.15 m above the highest sample near the env origin
        sc.env_origins[0, 2] = scenes.terrain_height_max_near(ter, sc.env_origins[0, 0], sc.env_origins[0, 1], 0.5)
    sim, ref = _pair(sc)
    assert sim.act_dim == 0 and sim.obs_dim == 11 + 1
    w = _run(sim, ref, sc, 0, 1 / 60, 2, 8, 10)
    assert w[1] <= 1e-4 and w[10] <= 1e-3, w
    # let it land, then: contact active on both sides, sets identical on the identical state
    for s in range(40):
        sim.step(None, 1 / 60, 2, 8)
    ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    cg, co = sim.generate_contacts(), ref.generate_contacts()
    assert _same_sets(cg, co) and cg["active"].sum() >= 1
    sim.close()


def test_large_capsule_takes_the_direct_search_path():
    """Radius 0.8 m: the reach box spans more than 15 cells, so its slots cannot be cut into
    packed work units and are searched 8 lanes per slot."""
    ter = scenes.make_heightfield(seed=1003)
    rob = scenes.make_single(radius=0.8, seg_len=1.0, axis=0, pos=(0.0, 0.0, 1.0), mass=50.0)
    sc = scenes.make_scene(rob, ter, 7, seed=5)
    for e in range(7):
        sc.env_origins[e, 2] = scenes.terrain_height_max_near(ter, sc.env_origins[e, 0], sc.env_origins[e, 1], 1.5)
    sim, ref = _pair(sc)
    w = _run(sim, ref, sc, 0, 1 / 60, 4, 16, 10, warm=25)
    assert w[1] <= 1e-4 and w[10] <= 1e-3, w
    ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    cg, co = sim.generate_contacts(), ref.generate_contacts()
    assert _same_sets(cg, co) and cg["active"].sum() >= 7
    # the fused path records the same set as stand-alone generation
    sim2, _ = _pair(sc, state=ref.get_state())
    sim2.record_contacts(True)
    sim2.step(None, 1 / 60, 1, 0)
    assert _same_sets(sim2.get_contacts(), co)
    sim.close(); sim2.close()


def test_hub_with_six_joints_uses_the_general_kernel():
    sc = scenes.make_scene(scenes.make_star(n_legs=6), scenes.make_plane(), 37)
    sim, ref = _pair(sc)
    w = _run(sim, ref, sc, 21, 1 / 60, 4, 16, 10, warm=30)
    assert w[1] <= 1e-4 and w[10] <= 1e-3, w
    sim.close()


def test_more_active_contacts_than_contact_threads():
    """13 capsules lying on the ground in each of 16 envs of one workgroup: 416 active end-sphere
    contacts for the 384 contact threads of the 768-thread workgroup (12 joints x 2 sides x 16 envs
    take the other 384), the rest go through the LDS-resident impulse path."""
    sc = scenes.make_scene(scenes.make_raft(n_links=13), scenes.make_plane(), 16)
    sim, ref = _pair(sc)
    sim.set_envs_per_block(16)
    cg, co = sim.generate_contacts(), ref.generate_contacts()
    assert _same_sets(cg, co) and cg["active"].sum() == 16 * 26
    w = _run(sim, ref, sc, 4, 1 / 60, 4, 20, 10)
    assert w[1] <= 1e-4 and w[10] <= 1e-3, w
    sim.close()


def test_zero_sweeps_and_one_sweep_match_the_oracle():
    sc, cfg = scenes.config_scene(2, num_envs=33)
    import paper_1810_05762_amd as P
    for its in (0, 1):
        sim = P.Sim(sc); sim.reset(cfg["seed"])
        ref = oracle.OracleSim(sc, threads=4)
        ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
        act = scenes.actions_for_step(1, 0, 33, 21)
        sim.step(act, 1 / 60, 2, its); ref.step(act, 1 / 60, 2, its)
        e = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
        assert e.max() <= 1e-4, (its, e.max())
        sim.close()


def test_candidate_list_overflow_falls_back_to_the_direct_search():
    """13 capsules lying flat on a heightfield in each of 16 envs: about twice as many candidate
    triangles and edges as the candidate list of a workgroup holds, so part of the slots are
    searched by the fallback; the outcome must not depend on which."""
    ter = scenes.make_flat_heightfield(nx=160, ny=160, cell=0.1, height=0.0, origin=(-8.0, -8.0))
    sc = scenes.make_scene(scenes.make_raft(n_links=13), ter, 16, seed=2)
    sc.env_origins[:, 2] = 0.0
    sim, ref = _pair(sc)
    sim.set_envs_per_block(16)
    cg, co = sim.generate_contacts(), ref.generate_contacts()
    assert _same_sets(cg, co) and cg["active"].sum() >= 16 * 26
    sim2, _ = _pair(sc)
    sim2.set_envs_per_block(16)
    sim2.record_contacts(True)
    sim2.step(None, 1 / 60, 1, 0)
    assert _same_sets(sim2.get_contacts(), co)
    w = _run(sim, ref, sc, 4, 1 / 60, 4, 20, 10)
    assert w[1] <= 1e-4 and w[10] <= 1e-3, w
    sim.close(); sim2.close()


@pytest.mark.parametrize("with_task", [False, True])
def test_step_captured_in_a_graph_replays_like_eager_launches(with_task):
    """sim_step_obs allocates nothing, does not synchronise and launches on the caller's stream,
    so a caller can capture it in a HIP graph (here through torch) and replay it: every replay,
    with eager work of the same sim in between, must equal the eager step bit for bit."""
    import torch
    import paper_1810_05762_amd as P
    n = 300
    sc, cfg = scenes.config_scene(3, num_envs=n)
    dt = float(np.float32(cfg["dt"]))
    tp = scenes.TaskParams(fall_grace_frames=3, target_period=11, push_min_frames=5, push_max_frames=9, auto_reset=1, seed=4)

    def make():
        sim = P.Sim(sc); sim.reset(cfg["seed"])
        if with_task:
            sim.set_task(tp)
        return sim

    acts = [torch.as_tensor(scenes.actions_for_step(cfg["seed"], s, n, sc.robot.n_dofs)).cuda() for s in range(30)]
    eager, graphed = make(), make()
    abuf = acts[0].clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.step_obs(abuf, dt, cfg["substeps"], cfg["iterations"])
    # capturing runs nothing
    assert torch.equal(graphed.get_state(), eager.get_state())
    resets = 0
    for k in range(30):
        abuf.copy_(acts[k])
        g.replay()
        torch.cuda.synchronize()
        eo, er, ed = eager.step_obs(acts[k], dt, cfg["substeps"], cfg["iterations"])
        assert torch.equal(graphed.obs, eo) and torch.equal(graphed.reward, er) and torch.equal(graphed.done, ed)
        assert torch.equal(graphed.get_state(), eager.get_state())     # eager launches of the graphed sim between replays
        resets += int(ed.sum().item())
    if with_task:
        assert resets > 0
    graphed.check(); eager.check()
    graphed.close(); eager.close()


def _max_size_robot():
    """The largest robot the library takes: 16 capsules in a chain hung from the world, 16 joints
    with two hinge axes each (32 actuated degrees of freedom)."""
    from scenes.robots import _Builder
    bld = _Builder("max16")
    seg, r = 0.12, 0.03
    prev = -1
    for k in range(16):
        a = (0.0, 0.0, 1.75 - k * seg)
        b = bld.body(f"link{k}", r, seg, 2, (0.0, 0.0, 1.75 - (k + 0.5) * seg), mass=0.3)
        bld.joint(prev, b, a, [((0.0, 1.0, 0.0), -1.0, 1.0), ((1.0, 0.0, 0.0), -0.8, 0.8)], 1.5)
        prev = b
    return bld.build(root_body=0, feet=(15,), term_height=-1e9, alive_bonus=0.0)


@pytest.mark.parametrize("epb", [None, 14])
def test_largest_robot_the_library_takes(epb):
    rob = _max_size_robot()
    assert (rob.n_bodies, rob.n_joints, rob.n_dofs) == (16, 16, 32)
    sc = scenes.make_scene(rob, scenes.make_heightfield(seed=1003), 45)
    sim, ref = _pair(sc)
    if epb:
        sim.set_envs_per_block(epb)
    assert sim.obs_dim == 11 + 3 * 32 + 1 == ref.obs_dim
    w = _run(sim, ref, sc, 12, 1 / 60, 4, 20, 10, warm=50)     # the chain swings down onto the terrain first
    assert w[1] <= 1e-4 and w[10] <= 1e-3, w
    og, rg, dg = (t.cpu().numpy() for t in sim.get_obs())
    oo, ro, do = ref.get_obs()
    assert np.abs(og - oo).max() <= 1e-3 * max(1.0, np.abs(oo).max())     # ten free-running steps: the state's bar
    assert ref.get_contacts()["active"].sum() > 0
    sim.close()


@pytest.mark.parametrize("kind,maker", [(1, "make_ant"), (2, "make_humanoid")])
def test_sim_from_the_built_in_description_equals_the_sim_from_the_input_recipe(kind, maker):
    """A sim created through the C interface alone (default parameters, built-in robot tables,
    the caller adds only where the envs stand) steps bit for bit like the one whose description
    the input module builds."""
    import torch
    import paper_1810_05762_amd as P
    n = 40
    rob = getattr(scenes, maker)()
    sc = scenes.make_scene(rob, scenes.make_plane(), n)
    ref = P.Sim(sc)
    d = P.sim_builtin_robot(kind)
    org = np.ascontiguousarray(sc.env_origins, np.float64)
    d.env_origins = org.ctypes.data_as(type(d.env_origins))
    nbytes = P.sim_workspace_bytes(d, n)
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    h = P.sim_create(d, n, (ws.data_ptr() + 255) & ~255, nbytes)
    stream = torch.cuda.current_stream().cuda_stream
    P.sim_reset(h, None, 5, stream)
    ref.reset(5)
    st = torch.empty(n, rob.n_bodies, 13, dtype=torch.float32, device="cuda")
    for s in range(6):
        a = torch.as_tensor(scenes.actions_for_step(3, s, n, rob.n_dofs)).cuda()
        P.sim_step(h, a.data_ptr(), 1.0 / 60.0, 4, 20, stream)
        ref.step(a, 1.0 / 60.0, 4, 20)
    P.sim_get_state(h, st.data_ptr(), stream)
    assert torch.equal(st, ref.get_state())
    assert P.lib().sim_act_dim(h) == rob.n_dofs
    torch.cuda.synchronize()
    P.sim_destroy(h)
    ref.close()
