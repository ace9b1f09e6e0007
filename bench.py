"""Benchmark: env-steps/s of the whole hot path on one MI355X.

A step is one sim_step_obs (all substeps: contact generation, force integration,
block projected-Jacobi sweeps, position integration, obs/reward/done packing, with
obs/reward/done delivered into caller tensors), on the 4096-humanoid heightfield
workload (configuration 3).  Inputs are seeded and synthetic and already
resident in HBM when the timed region starts.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

# ---- algorithmic work per env-step (one FMA counts as 2 flops) ----
F_JOINT_SWEEP = 156.0     # 3 positional rows x 27 + 3 angular rows x 25
F_CONTACT_SWEEP = 95.0    # normal row 29 + friction pair 66
F_JOINT_SETUP = 420.0     # two rotation matrices, anchors, 6 effective masses and responses, joint angles
F_CONTACT_SETUP = 150.0
F_BODY_SUBSTEP = 240.0    # rotation + world inverse inertia, force/gyroscopic integration, pose integration
F_SLOT_REJECT = 30.0      # end points + reach test of a slot that is nowhere near the ground
F_SLOT_NARROW = 2000.0    # ~12 cells x 2 triangles (or 3 edges) x ~85 flops for a slot near the ground


def flops_per_env_step(B, J, S, substeps, iterations, active, blocks_per_body):
    sweep = J * F_JOINT_SWEEP + active * F_CONTACT_SWEEP + B * (6.0 * blocks_per_body + 6.0)
    setup = (J * F_JOINT_SETUP + active * F_CONTACT_SETUP + B * F_BODY_SUBSTEP
             + S * F_SLOT_REJECT + active * F_SLOT_NARROW)
    return substeps * (iterations * sweep + setup)


def bytes_per_env_step(B, J, S, D, obs_dim, substeps, iterations, active):
    """HBM byte accountings: A compulsory (state in+out, actions, obs, reward, done);
    B state and slot records streamed once per substep; C every sweep streams velocities
    and rows (what an unfused, one-kernel-per-sweep engine would move)."""
    state = B * 13 * 4
    a = 2 * state + D * 4 + obs_dim * 4 + 5
    b = substeps * (2 * state + S * 40) + D * 4 + obs_dim * 4 + 5
    rows = 6 * J + 3 * active
    c = substeps * iterations * (2 * B * 6 * 4 + rows * 52) + a
    return a, b, c


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="workload configuration (3 = headline)")
    ap.add_argument("--envs-per-block", type=int, default=0)
    ap.add_argument("--num-envs", type=int, default=0, help="override the number of envs (scaling runs)")
    ap.add_argument("--height-map", action="store_true", help="append the 15 x 11 height map to the observation")
    ap.add_argument("--self-collide", action="store_true", help="capsules of one robot collide with each other")
    ap.add_argument("--group-size", type=int, default=1, help="agents per interaction group (inter-agent collisions)")
    ap.add_argument("--spacing", type=float, default=1.5, help="distance between the agents of a group, metres")
    ap.add_argument("--task", action="store_true", help="task logic of Section 4.1: pushes, flagrun targets, grace period, auto-reset")
    ap.add_argument("--warm-start", type=float, default=0.0, help="share of the last substep's impulses the rows start from (0 = off)")
    ap.add_argument("--iterations", type=int, default=0, help="override the sweeps per substep (the workload is then named for it)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (envs would be sharded across GPUs with no "
              "exchange inside a step); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import scenes
    import paper_1810_05762_amd as P

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    scene, cfg = scenes.config_scene(args.config, num_envs=args.num_envs or None)
    if args.height_map:
        scene.params.height_map = 1
    if args.warm_start > 0:
        scene.params.warm_start = args.warm_start
    if args.iterations > 0:
        cfg["iterations"] = args.iterations
    collide = args.self_collide or args.group_size > 1
    if collide:
        # the same robots, terrain and stepping parameters with capsule-capsule collisions on
        scene.params.self_collide = 1 if args.self_collide else 0
        scene.params.group_size = args.group_size
        scene = scenes.make_scene(scene.robot, scene.terrain, scene.num_envs, seed=cfg["seed"], params=scene.params,
                                  name=cfg["name"], spacing=args.spacing if args.group_size > 1 else None)
    N, rob = scene.num_envs, scene.robot
    sim = P.Sim(scene, device=dev)
    if args.envs_per_block:
        sim.set_envs_per_block(args.envs_per_block)
    if cfg["fallen"]:
        sim.set_state(scenes.fallen_states(scene, cfg["seed"]))
    else:
        sim.reset(cfg["seed"])
    task = scenes.TaskParams(seed=cfg["seed"]) if args.task else None
    if task is not None:
        sim.set_task(task)
    dt, sub, its = float(np.float32(cfg["dt"])), cfg["substeps"], cfg["iterations"]
    ring = [torch.as_tensor(scenes.actions_for_step(cfg["seed"], s, N, rob.n_dofs)).to(dev) for s in range(16)]
    obs = torch.empty(N, sim.obs_dim, dtype=torch.float32, device=dev)
    rew = torch.empty(N, dtype=torch.float32, device=dev)
    done = torch.empty(N, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream

    def one_step(k):
        # sim_step + sim_get_obs in their one-launch form: the step kernel writes obs, reward and
        # done straight into the caller's tensors
        P.sim_step_obs(sim.h, ring[k % 16].data_ptr(), dt, sub, its, obs.data_ptr(), rew.data_ptr(), done.data_ptr(),
                       stream)

    settle = 60          # robots are dropped from their reset height; let them land first (untimed)
    for k in range(settle + args.warmup):
        one_step(k)
    torch.cuda.synchronize(dev)
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(settle + args.warmup + k)
    torch.cuda.synchronize(dev)
    elapsed = time.perf_counter() - t0
    sim.check()

    # dominant kernel: the fused step kernel, timed per launch with events on its stream
    n_ev = min(args.steps, 200)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
    for k, (e0, e1) in enumerate(evs):
        e0.record()
        one_step(k)
        e1.record()
    torch.cuda.synchronize(dev)
    kern_ms = float(np.mean([e0.elapsed_time(e1) for e0, e1 in evs]))
    con = sim.generate_contacts()
    active = float(con["active"].sum()) / N
    blocks_per_body = (2.0 * rob.n_joints + active) / rob.n_bodies

    fl = flops_per_env_step(rob.n_bodies, rob.n_joints, sim.S, sub, its, active, blocks_per_body)
    bA, bB, bC = bytes_per_env_step(rob.n_bodies, rob.n_joints, sim.S, rob.n_dofs, sim.obs_dim, sub, its, active)
    achieved_tflops = fl * N / (kern_ms * 1e-3) / 1e12
    # HBM bytes per launch of the step kernel at the headline size, from rocprofv3 FETCH_SIZE and
    # WRITE_SIZE scaled by what the same counters read for a 256 MiB copy (0.5 and 1.0): 8.6 MB
    # read + 6.9 MB written (summary under profiles/); other sizes were not measured
    # vector instructions per launch at the headline size (rocprofv3 SQ_INSTS_VALU, same summary):
    # times 64 lanes, over the kernel time, against what 256 CUs x 4 SIMDs x 16 lanes issue per
    # clock at 2.4 GHz without packed instructions
    valu_insts = 43.6e6 if (args.config == 3 and N == 4096 and not args.height_map and not collide and not args.task and not args.warm_start and not args.iterations) else None
    traffic = 15.5e6 if (args.config == 3 and N == 4096 and not args.height_map and not collide and not args.task and not args.warm_start and not args.iterations) else None
    pair_info = {}
    if collide:
        sim.record_contacts(True)
        one_step(0)
        pc, dropped = sim.get_pair_contacts(cap=64 * N)
        sim.record_contacts(False)
        pair_info = {"self_collide": int(args.self_collide), "group_size": args.group_size,
                     "spacing_m": args.spacing if args.group_size > 1 else None,
                     "capsule_contacts_per_env": round(len(pc) / N, 3),
                     "capsule_contacts_between_agents_per_env": round(float((pc["env_a"] != pc["env_b"]).sum()) / N, 3),
                     "capsule_contacts_dropped": dropped}
    peak_tflops = 157.3
    value = N * args.steps / elapsed
    out = {
        "metric": "env-steps/sec on 1 MI355X (4096 humanoids, heightfield); HBM roofline fraction",
        "value": value, "unit": "env-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": (cfg["name"] if not args.num_envs else f"{cfg['name']}_n{N}") + ("_heightmap" if args.height_map else "")
                               + ("_selfcollide" if args.self_collide else "") + (f"_group{args.group_size}" if args.group_size > 1 else "")
                               + ("_task" if args.task else "") + (f"_warm{args.warm_start:g}" if args.warm_start > 0 else "")
                               + (f"_its{args.iterations}" if args.iterations > 0 else ""),
                   "num_envs": N, "obs_dim": sim.obs_dim, "robot": rob.name, "bodies": rob.n_bodies,
                   "joints": rob.n_joints, "dofs": rob.n_dofs, "contact_slots": sim.S,
                   "terrain": "heightfield 256x256 x 0.1 m" if scene.terrain.kind else "plane",
                   "dt": cfg["dt"], "substeps": sub, "iterations": its, "settle_steps": settle,
                   "mean_active_contacts_per_env": round(active, 3), "kernel_launches_per_step": 1,
                   **sim.launch_info(), **pair_info},
        "roofline": {"bound": "alu", "kernel": "step_kernel", "achieved": achieved_tflops, "peak": peak_tflops,
                     "unit": "TFLOP/s", "frac": achieved_tflops / peak_tflops, "traffic": traffic,
                     "flops_per_env_step": fl, "kernel_ms": kern_ms,
                     "valu_issue_frac": (valu_insts * 64 / (kern_ms * 1e-3) / (256 * 4 * 16 * 2.4e9)) if valu_insts else None},
        "hbm_roofline": {
            "peak_GBps": 8000.0, "kernel_ms": kern_ms,
            "A_compulsory": {"bytes_per_env_step": bA, "GBps": bA * N / (kern_ms * 1e-3) / 1e9,
                             "frac": bA * N / (kern_ms * 1e-3) / 8e12},
            "B_per_substep": {"bytes_per_env_step": bB, "GBps": bB * N / (kern_ms * 1e-3) / 1e9,
                              "frac": bB * N / (kern_ms * 1e-3) / 8e12},
            "C_streaming_jacobi": {"bytes_per_env_step": bC, "GBps": bC * N / (kern_ms * 1e-3) / 1e9,
                                   "frac": bC * N / (kern_ms * 1e-3) / 8e12},
        },
    }

    if not args.no_cpu_baseline:
        import oracle
        n_s = min(N, 256)
        sub_scene, _ = scenes.config_scene(args.config, num_envs=n_s)
        sub_scene.params = scene.params
        sub_scene.env_origins = scene.env_origins[:n_s].copy()
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
        cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
        ref = oracle.OracleSim(sub_scene, threads=cores)
        ref.set_state(sim.get_state().cpu().numpy()[:n_s].astype(np.float64))
        if task is not None:
            ref.set_task(task)
        acts = [ring[k].cpu().numpy()[:n_s] for k in range(16)]
        ref.step(acts[0], dt, sub, its)
        t0 = time.perf_counter()
        n_steps = 0
        while True:
            ref.step(acts[n_steps % 16], dt, sub, its)
            n_steps += 1
            el = time.perf_counter() - t0
            if el > 12.0 or n_steps >= 400:
                break
        out["cpu_baseline"] = {"value": n_s * n_steps / el, "unit": "env-steps/s", "cores": cores, "kind": "oracle",
                               "sample": f"{n_s} envs x {n_steps} steps of the same workload "
                                         f"(plain fp64 C oracle, OpenMP over envs)"}
        # the same oracle on one thread (the paper's CPU comparison is single-core), 16 envs, about 3 s
        n_1 = min(N, 16)
        one_scene, _ = scenes.config_scene(args.config, num_envs=n_1)
        one_scene.params = scene.params
        one_scene.env_origins = scene.env_origins[:n_1].copy()
        ref1 = oracle.OracleSim(one_scene, threads=1)
        ref1.set_state(sim.get_state().cpu().numpy()[:n_1].astype(np.float64))
        if task is not None:
            ref1.set_task(task)
        t0 = time.perf_counter()
        n1_steps = 0
        while True:
            ref1.step(acts[n1_steps % 16][:n_1], dt, sub, its)
            n1_steps += 1
            el1 = time.perf_counter() - t0
            if el1 > 3.0 or n1_steps >= 200:
                break
        out["cpu_baseline"]["one_thread_value"] = n_1 * n1_steps / el1
        out["cpu_baseline"]["one_thread_sample"] = f"{n_1} envs x {n1_steps} steps"
    sim.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
