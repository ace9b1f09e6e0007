"""Where the step kernel's time goes: cycle counters around its phases.

    python3 paper_1810_05762_amd/phase_timing.py [--config 3] [--steps 20]
                                                 [--self-collide] [--group-size G --spacing S]

Builds the diagnostic variant of the library (-DSIM_PHASE_TIMING), runs the benchmark's workload
(60 settle steps, then `steps` measured ones) and prints, per env-step, the cycles thread 0 of one
workgroup spent between the kernel's phase marks.  The marks cost a few hundred cycles each; there
are none inside the sweep loop, so the sweeps' figure is a clean total.
"""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import numpy as np

MARKS = [(0, "load state, tables, heightfield patch"), (1, "A publish pose, inverse inertia"),
         (24, "B1a per-body reach pass (+ torques)"), (2, "B1b per-slot pass, own part"),
         (25, "B1b wait for the other wavefronts"), (10, "B2 stage 1, end spheres"),
         (11, "B2 stage 1, mid-segments"), (13, "B2 stage 2, exact distances"), (12, "B3 records"),
         (3, "clear search space"), (16, "P capsule-capsule contacts"), (4, "C weight sums"), (5, "D row constants"), (17, "D joint rows (thread 0's wavefront)"), (6, "S sweeps"),
         (7, "E integrate"), (8, "store state"), (9, "obs / reward / done")]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--self-collide", action="store_true")
    ap.add_argument("--group-size", type=int, default=1)
    ap.add_argument("--spacing", type=float, default=1.5)
    args = ap.parse_args()
    import torch
    import scenes
    from paper_1810_05762_amd import build
    build.LIB_PATH = build.build_timing()          # the binding loads whatever LIB_PATH names
    import paper_1810_05762_amd as P

    sc, cfg = scenes.config_scene(args.config)
    if args.self_collide or args.group_size > 1:
        sc.params.self_collide, sc.params.group_size = int(args.self_collide), args.group_size
        sc = scenes.make_scene(sc.robot, sc.terrain, sc.num_envs, seed=cfg["seed"], params=sc.params, name=cfg["name"],
                               spacing=args.spacing if args.group_size > 1 else None)
    N, D = sc.num_envs, sc.robot.n_dofs
    sim = P.Sim(sc)
    if cfg["fallen"]:
        sim.set_state(scenes.fallen_states(sc, cfg["seed"]))
    else:
        sim.reset(cfg["seed"])
    dt = float(np.float32(cfg["dt"]))
    acts = [torch.as_tensor(scenes.actions_for_step(cfg["seed"], s, N, D)).cuda() for s in range(16)]
    for k in range(80):
        sim.step(acts[k % 16], dt, cfg["substeps"], cfg["iterations"])
    # the counters live in the last 256 bytes of the workspace: a flag word, then 30 slots
    nbytes = P.sim_workspace_bytes(sim.desc, N)
    off = (sim._ws_ptr - sim.workspace.data_ptr()) + nbytes - 256 + 8
    dbg = sim.workspace[off:off + 30 * 8].view(torch.int64)
    torch.cuda.synchronize(); dbg.zero_(); torch.cuda.synchronize()
    for k in range(args.steps):
        sim.step(acts[k % 16], dt, cfg["substeps"], cfg["iterations"])
    torch.cuda.synchronize()
    d = dbg.cpu().numpy().astype(np.float64) / args.steps
    total = sum(d[i] for i, _ in MARKS)
    print(f"{cfg['name']}: {sim.launch_info()}")
    for i, name in MARKS:
        print(f"  {name:42s} {d[i]:10.0f} cycles per step  {100 * d[i] / total:5.1f} %")
    print(f"  {'total':42s} {total:10.0f}")
    print(f"  per substep: {d[14] / cfg['substeps']:.0f} work units, {d[15] / cfg['substeps']:.0f} candidates in this workgroup")
    sim.close()


if __name__ == "__main__":
    main()
