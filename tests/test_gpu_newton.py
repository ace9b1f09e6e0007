"""GPU parity of the second solver (the paper's own, Section 3.1: non-smooth Newton iterations, each
solved by a fixed number of preconditioned conjugate-residual iterations) against the oracle's
implementation of the same algorithm, through the C ABI."""
import dataclasses

import numpy as np
import pytest

import oracle
import scenes
from helpers import TOL_1, TOL_10, free_params, gate_after_10_steps, rel_err4, single_scene

pytestmark = pytest.mark.gpu
NEWTON_ITS, KRYLOV = 3, 8


def _P():
    import paper_1810_05762_amd as P
    return P


def _newton_gate(e1, e10):
    """A Newton iterate that is cut off after three iterations depends on which branch every
    one-sided row took in each of them (lambda - s / D > 0 or not), and single and double precision
    take a different branch now and then: in such an env the two sides differ by a finite amount,
    not by rounding (tests/test_oracle_sensitivity.py shows the oracle doing the same against its own
    single-precision twin, in 0.4 % of the env-substeps).  So: the bulk at rounding level after one
    step (median 1e-5, 95 % within 1e-4) and nothing beyond 1e-2; after ten steps median within
    1e-4 and 85 % within 1e-3."""
    assert np.median(e1) <= 1e-5 and np.quantile(e1, 0.95) <= TOL_1 and e1.max() <= 1e-2
    assert np.median(e10) <= TOL_1 and np.quantile(e10, 0.85) <= TOL_10 and np.isfinite(e10).all()


def _newton_scene(k, n_envs, share=0.0):
    sc, cfg = scenes.config_scene(k, num_envs=n_envs)
    sc.params = dataclasses.replace(sc.params, solver=1, krylov_iters=KRYLOV, warm_start=share)
    return sc, cfg


@pytest.mark.parametrize("k,n_envs,warm,epb,share", [(1, 90, 40, None, 0.0), (2, 77, 40, 8, 0.0), (3, 77, 40, 8, 0.0), (3, 21, 40, 5, 0.0),
                                                     (3, 77, 40, 8, 0.8), (1, 45, 40, 5, 0.8)])
def test_newton_states_match_the_oracle_after_1_and_10_steps(k, n_envs, warm, epb, share):
    """`share` > 0: the rows' kept impulses are the first Newton iterate (warm start)."""
    P = _P()
    sc, cfg = _newton_scene(k, n_envs, share)
    sim = P.Sim(sc)
    if epb:
        sim.set_envs_per_block(epb)
    sim.reset(cfg["seed"])
    dt, sub = float(np.float32(cfg["dt"])), cfg["substeps"]
    for s in range(warm):
        sim.step(scenes.actions_for_step(cfg["seed"], s, n_envs, sc.robot.n_dofs), dt, sub, NEWTON_ITS)
    ref = oracle.OracleSim(sc, threads=8)
    if share > 0:
        sim.set_state(sim.get_state())        # both sides start with nothing kept
    ref.set_state(sim.get_state().cpu().numpy().astype(np.float64))
    sim.record_contacts(True)
    h = dt / sub
    forked = np.zeros(n_envs, bool)
    errs = {}
    for s in range(10):
        a = scenes.actions_for_step(cfg["seed"], warm + s, n_envs, sc.robot.n_dofs)
        for _ in range(sub):
            sim.step(a, h, 1, NEWTON_ITS); ref.step(a, h, 1, NEWTON_ITS)
            cg, co = sim.get_contacts(), ref.get_contacts()
            forked |= np.any([(cg[f] != co[f]).any(1) for f in ("active", "kind", "feat")], axis=0)
        if s in (0, 9):
            errs[s + 1] = rel_err4(sim.get_state().cpu().numpy().astype(np.float64), ref.get_state())
    sim.check()
    e1, e10 = errs[1].max(1), errs[10].max(1)
    print(f"newton config {k}: {sim.launch_info()} 1 step median {np.median(e1):.2e} p98 {np.quantile(e1, .98):.2e} max {e1.max():.2e}; "
          f"10 steps median {np.median(e10):.2e} p90 {np.quantile(e10, .9):.2e} max {e10.max():.2e} ({forked.sum()} forked)")
    assert ref.get_contacts()["active"].sum() > n_envs // 2
    _newton_gate(e1, e10)
    if share > 0:
        # the kept impulses themselves, after the last substep, relative to the largest
        lj, ls = sim.get_kept_impulses()
        oj, os_ = ref.get_warm()
        ej = np.abs(lj.cpu().numpy().astype(np.float64).reshape(oj.shape) - oj).reshape(n_envs, -1).max(1) / max(1.0, np.abs(oj).max())
        es = np.abs(ls.cpu().numpy().astype(np.float64).reshape(os_.shape) - os_).reshape(n_envs, -1).max(1) / max(1.0, np.abs(os_).max())
        assert np.abs(oj).max() > 0.1 and np.abs(os_).max() > 0.01
        assert np.median(ej) <= TOL_10 and np.median(es) <= TOL_10
    sim.close()


def test_hanging_chain_does_not_sag_on_the_gpu_either():
    """The closed form the oracle's solver is pinned with: eight links hanging at rest stay where
    they are (to fp32 rounding) under 2 x 16 Newton / Krylov iterations, while 20 Jacobi sweeps let
    the last link sink by millimetres."""
    P = _P()
    rob = scenes.make_chain(n_links=8, seg_len=0.3, mass=0.5)
    z_rest = scenes.rest_state(rob, 1)[0, -1, 2]
    sag = {}
    for name, solver, kry, its in (("jacobi", 0, 8, 20), ("newton", 1, 16, 2)):
        p = free_params(contacts=0)
        p.solver, p.krylov_iters, p.newton_reg = solver, kry, 0.0      # undamped Newton steps
        sim = P.Sim(single_scene(rob, params=p, num_envs=3))
        sim.set_state(scenes.rest_state(rob, 3))
        for _ in range(240):
            sim.step(None, 1 / 60, 4, its)
        st = sim.get_state().cpu().numpy()
        sag[name] = z_rest - st[:, -1, 2]
        sim.close()
    assert sag["jacobi"].min() > 2e-3
    assert np.abs(sag["newton"]).max() < 2e-5


def test_newton_solver_limits_are_reported():
    P = _P()
    sc, cfg = _newton_scene(3, 32)
    sim = P.Sim(sc)
    assert sim.launch_info()["envs_per_block"] <= 8
    with pytest.raises(P.SimError):
        sim.set_envs_per_block(16)
    sim.close()
    bad = dataclasses.replace(sc.params, krylov_iters=0)
    with pytest.raises(P.SimError):
        P.sim_workspace_bytes(P.make_desc(scenes.make_scene(sc.robot, sc.terrain, 8, params=bad))[0], 8)


def test_full_size_newton_sampled_envs_match_oracle():
    """4096 humanoids on the heightfield with the Newton solver in the launch shape
    `bench.py --solver newton` times; 32 sampled envs recomputed by the oracle."""
    P = _P()
    sc, cfg = _newton_scene(3, 4096)
    N = sc.num_envs
    sim = P.Sim(sc)
    sim.reset(cfg["seed"])
    dt = float(np.float32(cfg["dt"]))
    for s in range(40):
        sim.step(scenes.actions_for_step(cfg["seed"], s, N, 21), dt, cfg["substeps"], NEWTON_ITS)
    pick = np.random.default_rng(5).choice(N, 32, replace=False)
    pick[:2] = (0, N - 1)
    sub, _ = _newton_scene(3, 32)
    sub.env_origins = sc.env_origins[pick].copy()
    ref = oracle.OracleSim(sub, threads=8)
    ref.set_state(sim.get_state().cpu().numpy()[pick].astype(np.float64))
    sim.record_contacts(True)
    forked = np.zeros(32, bool)
    for s in range(40, 50):
        a = scenes.actions_for_step(cfg["seed"], s, N, 21)
        sim.step(a, dt, cfg["substeps"], NEWTON_ITS); ref.step(a[pick], dt, cfg["substeps"], NEWTON_ITS)
        cg, co = sim.get_contacts()[pick], ref.get_contacts()
        forked |= np.any([(cg[f] != co[f]).any(1) for f in ("active", "kind", "feat")], axis=0)
        if s == 40:
            e1 = rel_err4(sim.get_state().cpu().numpy()[pick].astype(np.float64), ref.get_state()).max(1)
    sim.check()
    e10 = rel_err4(sim.get_state().cpu().numpy()[pick].astype(np.float64), ref.get_state())
    e10 = e10.max(1)
    print(f"full size newton: {sim.launch_info()}, 1 step median {np.median(e1):.2e} max {e1.max():.2e}; 10 steps median {np.median(e10):.2e} max {e10.max():.2e}")
    _newton_gate(e1, e10)
    sim.close()
