"""How far does the fp64 oracle drift from a copy of itself whose state is rounded to
fp32 after every substep?  That copy differs from the oracle by nothing but the storage
precision the GPU path is required to use, so its drift is the floor any fp32
implementation sits on; the GPU parity gates are set with this spread in mind."""
import numpy as np
import pytest

import oracle
import scenes


def _rel_err(g, o):
    out = []
    for sl in (slice(0, 3), slice(3, 7), slice(7, 10), slice(10, 13)):
        d = np.abs(g[:, :, sl] - o[:, :, sl]).reshape(g.shape[0], -1).max(1)
        n = np.maximum(1.0, np.abs(o[:, :, sl]).reshape(g.shape[0], -1).max(1))
        out.append(d / n)
    return np.stack(out, 1).max(1)


@pytest.mark.parametrize("k,warm", [(2, 40), (4, 30)])
def test_fp32_state_storage_alone_spreads_trajectories(k, warm):
    N = 96
    sc, cfg = scenes.config_scene(k, num_envs=N)
    a, b = oracle.OracleSim(sc, threads=8), oracle.OracleSim(sc, threads=8)
    if cfg["fallen"]:
        a.set_state(scenes.fallen_states(sc, cfg["seed"]))
    else:
        a.reset(cfg["seed"])
    sub, its, h = cfg["substeps"], cfg["iterations"], cfg["dt"] / cfg["substeps"]
    for s in range(warm):
        a.step(scenes.actions_for_step(cfg["seed"], s, N, sc.robot.n_dofs), cfg["dt"], sub, its)
    s0 = a.get_state().astype(np.float32).astype(np.float64)
    a.set_state(s0); b.set_state(s0)
    for s in range(10):
        act = scenes.actions_for_step(cfg["seed"], warm + s, N, sc.robot.n_dofs)
        for _ in range(sub):
            a.step(act, h, 1, its)
            b.step(act, h, 1, its)
            b.set_state(b.get_state().astype(np.float32).astype(np.float64))
        if s == 0:
            e1 = _rel_err(b.get_state(), a.get_state())
    e10 = _rel_err(b.get_state(), a.get_state())
    print(f"config {k}: 1 step max {e1.max():.2e}; 10 steps median {np.median(e10):.2e} "
          f"p95 {np.quantile(e10, .95):.2e} max {e10.max():.2e}")
    # the floor is far below the 1-step tolerance, and grows by orders of magnitude in 10 steps
    assert e1.max() < 1e-4
    assert np.median(e10) < 1e-4
    assert e10.max() > 20 * np.median(e1)
