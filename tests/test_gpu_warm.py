"""GPU parity of the warm start (rows start a substep from a share of the impulses they ended the
previous one with) against the oracle through the C ABI: free-running states to the tolerances
of the plain solver, the kept impulses themselves, what clears them, and the static closed form
(a hanging chain keeps its tension) on the GPU directly."""
import dataclasses

import numpy as np
import pytest

import oracle
import scenes
from helpers import free_params, single_scene
from helpers import TOL_1, TOL_10, gate_after_10_steps, rel_err4 as rel_err

pytestmark = pytest.mark.gpu
G = 9.81


def _P():
    import paper_1810_05762_amd as P
    return P


def _kept(sim):
    lj, ls = sim.get_kept_impulses()
    return lj.cpu().numpy().astype(np.float64), ls.cpu().numpy().astype(np.float64)


def _start(k, n_envs, settle, epb, share):
    P = _P()
    sc, cfg = scenes.config_scene(k, num_envs=n_envs)
    sc.params = dataclasses.replace(sc.params, warm_start=share)
    sim = P.Sim(sc)
    if epb:
        sim.set_envs_per_block(epb)
    sim.reset(cfg["seed"])
    dt = float(np.float32(cfg["dt"]))
    for s in range(settle):
        sim.step(scenes.actions_for_step(cfg["seed"], s, n_envs, sc.robot.n_dofs), dt, cfg["substeps"], cfg["iterations"])
    # both sides start from the same fp32 state and with nothing kept (set_state clears it)
    st = sim.get_state()
    sim.set_state(st)
    ref = oracle.OracleSim(sc, threads=8)
    ref.set_state(st.cpu().numpy().astype(np.float64))
    assert all(np.abs(x).max() == 0 for x in _kept(sim) if x.size)
    return sc, cfg, sim, ref, dt


# (config, envs, settle steps, envs per workgroup, one launch per substep)
CASES = [(3, 150, 40, 16, False), (3, 70, 40, 16, True), (2, 70, 40, 16, False), (1, 90, 40, None, True), (3, 37, 40, 8, False)]


@pytest.mark.parametrize("k,n_envs,settle,epb,split", CASES)
def test_states_and_kept_impulses_match_the_oracle(k, n_envs, settle, epb, split):
    """`split`: every substep is its own sim_step, so that what is kept goes through the workspace
    between two launches; otherwise it stays inside the workgroup from substep to substep."""
    sc, cfg, sim, ref, dt = _start(k, n_envs, settle, epb, 0.8)
    sub, its = cfg["substeps"], cfg["iterations"]
    errs, lam_err = {}, {}
    sim.record_contacts(True)
    forked = np.zeros(n_envs, bool)

    def compare_sets():
        cg, co = sim.get_contacts(), ref.get_contacts()
        return np.any([(cg[f] != co[f]).any(1) for f in ("active", "kind", "feat")], axis=0)

    for s in range(10):
        a = scenes.actions_for_step(cfg["seed"], settle + s, n_envs, sc.robot.n_dofs)
        if split:
            for _ in range(sub):
                sim.step(a, dt / sub, 1, its); ref.step(a, dt / sub, 1, its)
                forked |= compare_sets()
        else:
            sim.step(a, dt, sub, its); ref.step(a, dt, sub, its)
            forked |= compare_sets()            # (the sets of the step's last substep)
        if s in (0, 9):
            errs[s + 1] = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
            (gj, gs), (oj, os_) = _kept(sim), ref.get_warm()
            scale = max(1.0, np.abs(oj).max(), np.abs(os_).max())
            lam_err[s + 1] = np.array([np.abs(gj - oj).reshape(n_envs, -1).max(1), np.abs(gs - os_).reshape(n_envs, -1).max(1)]).max(0) / scale
            assert np.abs(oj).max() > 0.1 and np.abs(os_).max() > 0.01       # there is something to compare
    sim.check()
    e1, e10 = errs[1], errs[10]
    print(f"config {k} warm: 1 step {e1.max():.2e}; kept impulses 1 step {lam_err[1].max():.2e}, 10 steps median {np.median(lam_err[10]):.2e}")
    assert e1.max() <= TOL_1
    assert lam_err[1].max() <= 1e-4
    # ten steps: every env whose contact sets never differed within 1e-3, the others reported
    gate_after_10_steps(e10, forked, label=f"config {k} warm: ", sets_seen_every_substep=split)
    assert np.median(e10.max(1)) <= TOL_1
    assert np.median(lam_err[10]) <= 1e-3
    sim.close()


def test_share_zero_and_plain_library_paths_agree():
    # the warm-start variant of the kernel with nothing kept and the plain kernel compute the same step
    P = _P()
    n = 64
    out = []
    for share in (0.0, 1e-30):
        sc, cfg = scenes.config_scene(3, num_envs=n)
        sc.params = dataclasses.replace(sc.params, warm_start=share)
        sim = P.Sim(sc); sim.set_envs_per_block(16); sim.reset(cfg["seed"])
        for s in range(2):
            sim.step(scenes.actions_for_step(cfg["seed"], s, n, sc.robot.n_dofs), float(np.float32(cfg["dt"])), cfg["substeps"], cfg["iterations"])
        out.append(sim.get_state().cpu().numpy().astype(np.float64))
        sim.close()
    assert rel_err(out[1], out[0]).max() <= TOL_1


def test_reset_and_set_state_clear_what_is_kept():
    P = _P()
    n = 48
    sc, cfg = scenes.config_scene(3, num_envs=n)
    sc.params = dataclasses.replace(sc.params, warm_start=0.8)
    sim = P.Sim(sc); sim.set_envs_per_block(16); sim.reset(cfg["seed"])
    dt = float(np.float32(cfg["dt"]))
    for s in range(40):
        sim.step(scenes.actions_for_step(cfg["seed"], s, n, sc.robot.n_dofs), dt, cfg["substeps"], cfg["iterations"])
    gj, gs = _kept(sim)
    assert (np.abs(gj).reshape(n, -1).max(1) > 0).all() and (np.abs(gs).reshape(n, -1).max(1) > 0).mean() > 0.3
    mask = np.zeros(n, np.uint8); mask[::3] = 1
    sim.reset(7, mask=mask)
    rj, rs = _kept(sim)
    m = mask.astype(bool)
    assert np.abs(rj[m]).max() == 0 and np.abs(rs[m]).max() == 0
    assert np.array_equal(rj[~m], gj[~m]) and np.array_equal(rs[~m], gs[~m])
    sim.set_state(sim.get_state())
    assert all(np.abs(x).max() == 0 for x in _kept(sim))
    sim.close()


def test_auto_reset_starts_the_next_episode_with_nothing_kept():
    P = _P()
    n = 96
    sc, cfg = scenes.config_scene(3, num_envs=n)
    sc.params = dataclasses.replace(sc.params, warm_start=0.8)
    tp = scenes.TaskParams(fall_grace_frames=3, target_period=11, push_min_frames=5, push_max_frames=9, auto_reset=1, seed=21)
    sim = P.Sim(sc); sim.set_envs_per_block(16); sim.reset(cfg["seed"]); sim.set_task(tp)
    dt = float(np.float32(cfg["dt"]))
    ended = 0
    for f in range(70):
        _, _, done = sim.step_obs(scenes.actions_for_step(cfg["seed"], f, n, sc.robot.n_dofs), dt, cfg["substeps"], cfg["iterations"])
        d = done.cpu().numpy().astype(bool)
        gj, gs = _kept(sim)
        if d.any():
            assert np.abs(gj[d]).max() == 0 and np.abs(gs[d]).max() == 0
        if f > 5 and (~d).any():
            assert (np.abs(gj[~d]).reshape((~d).sum(), -1).max(1) > 0).all()
        ended += int(d.sum())
    assert ended > n // 2
    sim.check()
    sim.close()


def test_hanging_chain_keeps_its_static_tension_on_the_gpu():
    P = _P()
    nl, mass = 4, 0.5
    rob = scenes.make_chain(n_links=nl, mass=mass)
    dt, sub, its = float(np.float32(1 / 60)), 2, 4
    want = np.array([dt / sub * G * mass * (nl - k) for k in range(nl)])
    z_rest = scenes.rest_state(rob)[0][-1, 2]
    sag = {}
    for share in (0.0, 0.9):
        sc = single_scene(rob, params=free_params(contacts=0, warm_start=max(share, 1e-30)), num_envs=3)
        sim = P.Sim(sc)
        sim.set_state(scenes.rest_state(rob, 3))
        for _ in range(400):
            sim.step(None, dt, sub, its)
        gj, _ = _kept(sim)
        st = sim.get_state().cpu().numpy()
        np.testing.assert_allclose(gj[:, :, 2], np.tile(want, (3, 1)), rtol=2e-4)
        assert np.abs(gj[:, :, [0, 1, 3, 4, 5]]).max() < 1e-5
        assert np.abs(st[:, :, 7:13]).max() < 1e-4
        sag[share] = z_rest - st[0, -1, 2]
        sim.close()
    assert sag[0.9] == pytest.approx(0.1 * sag[0.0], rel=2e-2)


def test_contacts_beyond_one_per_thread_keep_their_impulses_in_place():
    """13 capsules lying on the ground in each of the 16 envs of one workgroup: 416 active contacts
    for 128 contact threads; the other 288 are relaxed through the per-slot array of kept impulses
    itself."""
    P = _P()
    sc = scenes.make_scene(scenes.make_raft(n_links=13), scenes.make_plane(), 16, params=scenes.SimParams(warm_start=0.8))
    sim = P.Sim(sc); sim.set_envs_per_block(16)
    st = scenes.rest_state(sc.robot, 16)
    sim.set_state(st)
    ref = oracle.OracleSim(sc, threads=4); ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    assert sim.launch_info()["threads_per_block"] == 512
    for s in range(10):
        a = scenes.actions_for_step(4, s, 16, sc.robot.n_dofs)
        sim.step(a, 1 / 60, 4, 20); ref.step(a, 1 / 60, 4, 20)
        if s in (0, 9):
            e = rel_err(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state()).max()
            (gj, gs), (oj, os_) = _kept(sim), ref.get_warm()
            assert ref.get_contacts()["active"].sum() > 200 and (np.abs(os_[:, :, 0]) > 0).sum() > 30   # far more active contacts than contact threads
            assert e <= (TOL_1 if s == 0 else TOL_10), (s, e)
            assert np.abs(gs - os_).max() <= 1e-4 * max(1.0, np.abs(os_).max())
            assert np.abs(gj - oj).max() <= 1e-4 * max(1.0, np.abs(oj).max())
    sim.check(); sim.close()
