"""sim_create_static (the entry point for callers that cannot allocate device memory) against
sim_create: same description, same inputs, through the C ABI; the two run the same kernels, so
every output has to agree bit for bit.  Two static sims in a row, the second one smaller (it
reuses the array the first one left its contents in)."""
import numpy as np
import pytest

import scenes

pytestmark = pytest.mark.gpu


def _run(P, sc, cfg, static, steps):
    import torch
    N, D = sc.num_envs, sc.robot.n_dofs
    d, keep = P.make_desc(sc)
    st = torch.cuda.current_stream().cuda_stream
    ws = None
    if static:
        h = P.sim_create_static(d, N)
    else:
        nbytes = P.sim_workspace_bytes(d, N)
        ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
        h = P.sim_create(d, N, (ws.data_ptr() + 255) & ~255, nbytes)
    L = P.lib()
    B, od = L.sim_num_bodies(h), L.sim_obs_dim(h)
    obs = torch.zeros(N, od, device="cuda")
    rew = torch.zeros(N, device="cuda")
    done = torch.zeros(N, dtype=torch.uint8, device="cuda")
    state = torch.zeros(N, B, 13, device="cuda")
    P.sim_reset(h, None, cfg["seed"], st)
    dt = float(np.float32(cfg["dt"]))
    out = []
    for s in range(steps):
        a = torch.as_tensor(scenes.actions_for_step(cfg["seed"], s, N, D)).cuda()
        P.sim_step_obs(h, a.data_ptr(), dt, cfg["substeps"], cfg["iterations"], obs.data_ptr(), rew.data_ptr(),
                       done.data_ptr(), st)
        P.sim_get_state(h, state.data_ptr(), st)
        torch.cuda.synchronize()
        out.append((obs.cpu().numpy().copy(), rew.cpu().numpy().copy(), done.cpu().numpy().copy(),
                    state.cpu().numpy().copy()))
    P.sim_check(h, st)
    return h, out, ws


def test_static_workspace_sim_equals_sim_create_twice_in_a_row_second_one_smaller():
    import paper_1810_05762_amd as P
    for n_envs, steps in ((150, 35), (37, 35)):
        sc, cfg = scenes.config_scene(3, num_envs=n_envs)
        h_ref, ref, ws = _run(P, sc, cfg, False, steps)
        h_st, got, _ = _run(P, sc, cfg, True, steps)
        # a second static sim on the same GPU is refused while the first one lives
        d, keep = P.make_desc(sc)
        with pytest.raises(P.SimError) as ei:
            P.sim_create_static(d, n_envs)
        assert ei.value.code == -2 and "in use" in str(ei.value)
        for s, (r, g) in enumerate(zip(ref, got)):
            for x, y in zip(r, g):
                assert np.array_equal(x, y), (n_envs, s)
        assert np.isfinite(got[-1][3]).all() and np.abs(got[-1][0]).max() > 0.1
        P.sim_destroy(h_st)
        P.sim_destroy(h_ref)


def test_static_workspace_rejects_what_does_not_fit():
    import paper_1810_05762_amd as P
    sc, cfg = scenes.config_scene(3, num_envs=16384)
    d, keep = P.make_desc(sc)
    assert P.sim_workspace_bytes(d, 16384) > 24 << 20
    with pytest.raises(P.SimError) as ei:
        P.sim_create_static(d, 16384)
    assert ei.value.code == -2 and "static workspace holds" in str(ei.value)
    # and the refusal leaves the array free for a sim that fits
    sc2, _ = scenes.config_scene(0, num_envs=16)
    d2, keep2 = P.make_desc(sc2)
    h = P.sim_create_static(d2, 16)
    P.sim_destroy(h)
