"""Benchmark: env-steps/s of the whole hot path on one MI355X.

A step is one sim_step_obs (all substeps: contact generation, force integration,
block projected-Jacobi sweeps, position integration, obs/reward/done packing, with
obs/reward/done delivered into caller tensors), on the 4096-humanoid heightfield
workload (configuration 3).  Inputs are seeded and synthetic and already
resident in HBM when the timed region starts.  Prints one JSON line.

The timed region (`--steps` env-steps between two synchronisations, with a pair of events on the
launch stream around it) is run `--repeats` times; the line reports the median repeat.
`--copy-probe` runs a plain device copy of known size instead (the calibration run of the HBM
traffic counters); `--print-csrc-hash` prints the hash that ties profiles/step_kernel_counters.json
to the kernel sources.
"""
import argparse
import hashlib
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


# Newton / Krylov solver: one application of J M^-1 J^T through the bodies
F_JOINT_APPLY = 162.0     # both sides: velocity change from 6 impulses (39 flops a side), 6 row products (42 a side)
F_CONTACT_APPLY = 80.0    # velocity change from 3 impulses, 3 row products
F_ROW_VECTOR = 14.0       # per row and inner iteration: the four vector updates and three partial dot products


def flops_per_env_step_newton(B, J, S, substeps, newton_its, krylov, active, blocks_per_body):
    apply_ = J * F_JOINT_APPLY + active * F_CONTACT_APPLY + B * 12.0 * blocks_per_body
    rows = 6 * J + 3 * active
    per_newton = (krylov + 2) * apply_ + krylov * rows * F_ROW_VECTOR + rows * 20.0
    setup = (J * F_JOINT_SETUP + active * F_CONTACT_SETUP + B * F_BODY_SUBSTEP
             + S * F_SLOT_REJECT + active * F_SLOT_NARROW)
    return substeps * (newton_its * per_newton + apply_ + setup)


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


def csrc_hash():
    """sha256 over the kernel sources: the counter figures under profiles/ are only quoted for the
    sources they were measured on."""
    d = os.path.join(ROOT, "paper_1810_05762_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".hpp")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()


def measured_counters(workload):
    """HBM bytes and vector instructions per launch of the step kernel from the tracked rocprofv3
    summary, or None when it was measured on other kernel sources or another workload."""
    path = os.path.join(ROOT, "profiles", "step_kernel_counters.json")
    try:
        rec = json.load(open(path))
    except (OSError, ValueError):
        return None
    if rec.get("csrc_sha256") != csrc_hash() or rec.get("workload") != workload:
        return None
    return rec


def copy_probe():
    """A plain device-to-device copy of 256 MiB, five times: under `rocprofv3 --pmc FETCH_SIZE` (or
    WRITE_SIZE) counter / size is the factor by which that counter over- or under-reports."""
    import torch
    if not torch.cuda.is_available():
        print("bench.py --copy-probe needs a GPU", file=sys.stderr)
        sys.exit(1)
    n = 256 * 1024 * 1024 // 4
    src = torch.arange(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    assert torch.equal(dst[:1000], src[:1000])
    print(json.dumps({"copy_probe_MiB": 256, "copies": 5}))


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
    ap.add_argument("--crowd", type=float, default=0.0,
                    help="with --group-size: all agents share one scene at this many agents per square metre, numbered "
                         "in no spatial order; the groups are then chosen from the positions (see --regroup-every)")
    ap.add_argument("--regroup-every", type=int, default=10, help="steps between two sim_regroup calls (--crowd)")
    ap.add_argument("--task", action="store_true", help="task logic of Section 4.1: pushes, flagrun targets, grace period, auto-reset")
    ap.add_argument("--warm-start", type=float, default=0.0, help="share of the last substep's impulses the rows start from (0 = off)")
    ap.add_argument("--iterations", type=int, default=0, help="override the sweeps per substep (the workload is then named for it)")
    ap.add_argument("--solver", choices=("jacobi", "newton"), default="jacobi",
                    help="newton: the paper's non-smooth Newton / Krylov solver, 3 Newton iterations of --krylov inner iterations per substep")
    ap.add_argument("--krylov", type=int, default=8, help="conjugate-residual iterations per Newton iteration (--solver newton)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--repeats", type=int, default=3, help="repeats of the timed region; the median is reported")
    ap.add_argument("--copy-probe", action="store_true", help="run the 256 MiB copy that calibrates the traffic counters, then exit")
    ap.add_argument("--print-csrc-hash", action="store_true")
    args = ap.parse_args()
    if args.print_csrc_hash:
        print(csrc_hash())
        return
    if args.copy_probe:
        copy_probe()
        return
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
    if args.solver == "newton":
        scene.params.solver, scene.params.krylov_iters = 1, args.krylov
        cfg["iterations"] = 3          # Newton iterations per substep
    if args.iterations > 0:
        cfg["iterations"] = args.iterations
    collide = args.self_collide or args.group_size > 1
    if collide:
        # the same robots, terrain and stepping parameters with capsule-capsule collisions on
        scene.params.self_collide = 1 if args.self_collide else 0
        scene.params.group_size = args.group_size
        scene = scenes.make_scene(scene.robot, scene.terrain, scene.num_envs, seed=cfg["seed"], params=scene.params,
                                  name=cfg["name"], spacing=args.spacing if args.group_size > 1 else None)
    crowd = args.crowd > 0 and args.group_size > 1
    if crowd:
        # one shared scene: on the heightfield the crowd stands in the middle of the field, every agent
        # lifted onto the terrain under it
        hf = scene.terrain.kind != 0
        side = float(np.sqrt(scene.num_envs / args.crowd))
        if hf and side > min(scene.terrain.extent) - 4.0:
            print(f"bench.py: a crowd of {scene.num_envs} at {args.crowd}/m2 needs {side:.0f} m, the heightfield has "
                  f"{min(scene.terrain.extent):.1f} m; use fewer agents (--num-envs) or a plane configuration", file=sys.stderr)
            sys.exit(2)
        base = tuple(np.asarray(scene.terrain.origin[:2]) + 0.5 * (np.asarray(scene.terrain.extent) - side)) if hf else (0.0, 0.0)
        org = scenes.crowd_origins(scene.num_envs, args.crowd, cfg["seed"], base=base)
        if hf:
            org[:, 2] = [scenes.terrain_height_max_near(scene.terrain, x, y, 0.5) for x, y in org[:, 0:2]]
        scene.env_origins = org.astype(np.float32).astype(np.float64)
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

    # configuration 4: a seeded per-env target direction that changes every 200 steps
    retarget = None
    if cfg.get("fallen") and task is None:
        retarget = [torch.as_tensor(scenes.targets_for_step(cfg["seed"], 200 * e, N)).to(dev) for e in range(8)]

    regroup_cell, regroup_reach = 2.4, 1.2     # metres: root bodies of two touching humanoids are at most about this far apart

    def one_step(k, may_retarget=True):
        if retarget is not None and may_retarget and k % 200 == 0:
            P.sim_set_targets(sim.h, retarget[(k // 200) % 8].data_ptr(), stream)
        if crowd and may_retarget and k % args.regroup_every == 0:
            P.sim_regroup(sim.h, regroup_cell, regroup_reach, stream)
        # sim_step + sim_get_obs in their one-launch form: the step kernel writes obs, reward and
        # done straight into the caller's tensors
        P.sim_step_obs(sim.h, ring[k % 16].data_ptr(), dt, sub, its, obs.data_ptr(), rew.data_ptr(), done.data_ptr(),
                       stream)

    settle = 60          # robots are dropped from their reset height; let them land first (untimed)
    for k in range(settle + args.warmup):
        one_step(k)
    # the timed region, `repeats` times: K steps between two synchronisations (host clock) with a
    # pair of events on the launch stream around them; the median repeat is reported
    host_s, event_ms = [], []
    k0 = settle + args.warmup
    for r in range(max(1, args.repeats)):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize(dev)
        t0 = time.perf_counter()
        ev0.record()
        for k in range(args.steps):
            one_step(k0 + k)
        ev1.record()
        torch.cuda.synchronize(dev)
        host_s.append(time.perf_counter() - t0)
        event_ms.append(ev0.elapsed_time(ev1))
        k0 += args.steps
    mid = int(np.argsort(host_s)[len(host_s) // 2])
    elapsed = host_s[mid]
    sim.check()

    # dominant kernel: the fused step kernel, timed per launch with events on its stream
    n_ev = min(args.steps, 200)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
    for k, (e0, e1) in enumerate(evs):
        e0.record()
        one_step(k, may_retarget=False)      # (the kernel alone between the two events)
        e1.record()
    torch.cuda.synchronize(dev)
    kern_ms = float(np.mean([e0.elapsed_time(e1) for e0, e1 in evs]))
    con = sim.generate_contacts()
    active = float(con["active"].sum()) / N
    blocks_per_body = (2.0 * rob.n_joints + active) / rob.n_bodies

    if args.solver == "newton":
        fl = flops_per_env_step_newton(rob.n_bodies, rob.n_joints, sim.S, sub, its, args.krylov, active, blocks_per_body)
    else:
        fl = flops_per_env_step(rob.n_bodies, rob.n_joints, sim.S, sub, its, active, blocks_per_body)
    bA, bB, bC = bytes_per_env_step(rob.n_bodies, rob.n_joints, sim.S, rob.n_dofs, sim.obs_dim, sub, its, active)
    achieved_tflops = fl * N / (kern_ms * 1e-3) / 1e12
    workload = ((cfg["name"] if not args.num_envs else f"{cfg['name']}_n{N}") + ("_heightmap" if args.height_map else "")
                + ("_selfcollide" if args.self_collide else "") + (f"_group{args.group_size}" if args.group_size > 1 else "")
                + (f"_crowd{args.crowd:g}" if crowd else "") + ("_task" if args.task else "") + (f"_warm{args.warm_start:g}" if args.warm_start > 0 else "")
                + (f"_its{args.iterations}" if args.iterations > 0 else "")
                + (f"_newton{cfg['iterations']}x{args.krylov}" if args.solver == "newton" else "")
                + (f"_epb{args.envs_per_block}" if args.envs_per_block else ""))
    # HBM bytes and vector instructions per launch come from the tracked rocprofv3 summary and are
    # quoted only for the kernel sources and the workload they were measured on (null otherwise)
    ctr = measured_counters(workload)
    valu_insts = ctr["valu_insts_per_launch"] if ctr else None
    traffic = (ctr["fetch_bytes_per_launch"] + ctr["write_bytes_per_launch"]) if ctr else None
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
        if crowd:
            # how well the groups chosen from the positions cover the agents that are close to each other
            near_now = sim.count_near_pairs(regroup_reach)
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            for _ in range(20):
                P.sim_regroup(sim.h, regroup_cell, regroup_reach, stream)
            ev1.record()
            torch.cuda.synchronize(dev)
            near_re = sim.count_near_pairs(regroup_reach)
            sim.set_groups(None)
            near_own = sim.count_near_pairs(regroup_reach)
            pair_info.update({"crowd_agents_per_m2": args.crowd, "regroup_every_steps": args.regroup_every,
                              "regroup_cell_m": regroup_cell, "regroup_reach_m": regroup_reach,
                              "regroup_ms": ev0.elapsed_time(ev1) / 20,
                              "agent_pairs_within_reach": near_now[0],
                              "of_them_in_different_groups": {"as_stepped": near_now[1], "just_regrouped": near_re[1],
                                                              "in_number_order": near_own[1]}})
    peak_tflops = 157.3
    value = N * args.steps / elapsed
    out = {
        "metric": "env-steps/sec on 1 MI355X (4096 humanoids, heightfield); HBM roofline fraction",
        "value": value, "unit": "env-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "repeats": {"n": len(host_s), "reported": "median", "host_ms_per_step": [t / args.steps * 1e3 for t in host_s],
                    "event_ms_per_step": [t / args.steps for t in event_ms]},
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload,
                   "num_envs": N, "obs_dim": sim.obs_dim, "robot": rob.name, "bodies": rob.n_bodies,
                   "joints": rob.n_joints, "dofs": rob.n_dofs, "contact_slots": sim.S,
                   "terrain": "heightfield 256x256 x 0.1 m" if scene.terrain.kind else "plane",
                   "dt": cfg["dt"], "substeps": sub, "iterations": its, "solver": args.solver, "settle_steps": settle,
                   "mean_active_contacts_per_env": round(active, 3), "kernel_launches_per_step": 1,
                   **sim.launch_info(), **pair_info},
        "roofline": {"bound": "alu", "kernel": "step_kernel", "achieved": achieved_tflops, "peak": peak_tflops,
                     "unit": "TFLOP/s", "frac": achieved_tflops / peak_tflops, "traffic": traffic,
                     "flops_per_env_step": fl, "kernel_ms": kern_ms,
                     "valu_issue_frac": (valu_insts * 64 / (kern_ms * 1e-3) / (256 * 4 * 16 * 2.4e9)) if valu_insts else None},
        # HBM is not what bounds this kernel (body state stays in LDS through all substeps and
        # sweeps); the byte accountings are printed for the record.  A and B are bytes the kernel has
        # to move, as fractions of 8 TB/s; C is what an engine with one kernel per sweep would stream
        # (velocities and rows through HBM every sweep): a hypothetical, not traffic of this kernel
        # and not a roofline fraction of it.
        "hbm_accountings": {
            "peak_GBps": 8000.0, "kernel_ms": kern_ms,
            "measured_GBps": (traffic / (kern_ms * 1e-3) / 1e9) if traffic else None,
            "measured_frac_of_peak": (traffic / (kern_ms * 1e-3) / 8e12) if traffic else None,
            "A_compulsory": {"bytes_per_env_step": bA, "GBps": bA * N / (kern_ms * 1e-3) / 1e9,
                             "frac_of_peak": bA * N / (kern_ms * 1e-3) / 8e12},
            "B_per_substep": {"bytes_per_env_step": bB, "GBps": bB * N / (kern_ms * 1e-3) / 1e9,
                              "frac_of_peak": bB * N / (kern_ms * 1e-3) / 8e12},
            "C_unfused_engine_hypothetical": {"bytes_per_env_step": bC,
                                              "equivalent_GBps": bC * N / (kern_ms * 1e-3) / 1e9},
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
