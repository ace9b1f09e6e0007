/*
 * sim.h -- C ABI of the batched articulated rigid-body simulator for MI355X.
 *
 * Many independent robots (capsule/sphere bodies joined by limited hinge and
 * lock constraints) are advanced together on one GPU, in the many-agents-per-
 * call, Gym-like framing of the paper (Section 1 and Section 3.1: all robots
 * are loaded into one simulation and stepped by a single call).  One sim_step
 * advances every environment by dt, split into `substeps` substeps of
 *   contact generation -> torque/gravity integration -> fixed-count block
 *   projected-Jacobi solve of joint, joint-limit and contact/friction rows ->
 *   position integration,
 * and then packs the observation vector (Table 2, "Ours"), the reward
 * (Eq. 1-3) and the done flag (Section 4.1 episode rules).
 *
 * Conventions
 *  - Every pointer named *_dev is DEVICE memory owned by the caller; every
 *    other pointer is HOST memory.  The library never allocates, frees or
 *    retains caller memory except the workspace handed to sim_create, which it
 *    uses until sim_destroy and never frees.
 *  - `stream` is the caller's hipStream_t passed as void* (NULL = default
 *    stream).  Calls enqueue work on it and return without synchronising,
 *    except sim_create (synchronous uploads) and sim_check.
 *  - External arrays are env-major, row-major: actions [N][act_dim], obs
 *    [N][obs_dim], state [N][B][13] = position(3, env-local), quaternion
 *    (w,x,y,z), linear velocity(3), angular velocity(3) (world frame).
 *  - Return value 0 = success; SIM_ERR_* (negative) otherwise, with a message
 *    available from sim_last_error().  Nothing throws or aborts across the ABI.
 */
#ifndef PAPER_1810_05762_SIM_H
#define PAPER_1810_05762_SIM_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SIM_OK 0
#define SIM_ERR_ARG (-1)        /* invalid argument */
#define SIM_ERR_WORKSPACE (-2)  /* workspace too small or misaligned */
#define SIM_ERR_HIP (-3)        /* a HIP runtime call failed */
#define SIM_ERR_NONFINITE (-4)  /* sim_check found a NaN/Inf in the state */

#define SIM_MAX_BODIES 16
#define SIM_MAX_JOINTS 16
#define SIM_MAX_DOFS 32
#define SIM_MAX_FEET 4

typedef struct sim sim_t; /* opaque; created by sim_create, released by sim_destroy */

/* A rigid body: a capsule whose segment runs along body axis `axis` (0,1,2)
 * with half length half_len, or a sphere when half_len == 0.  Body frames are
 * world-aligned in the rest pose; inertia is diagonal in the body frame. */
typedef struct sim_body_desc {
  int32_t axis;
  int32_t pad;
  double radius, half_len, mass;
  double inertia[3];
  double rest_pos[3]; /* env-local rest position of the centre */
} sim_body_desc_t;

/* A joint pins `anchor` (given in the rest pose) of parent and child together
 * (3 positional rows) and constrains the three components of their relative
 * rotation vector along axes[k] (parent frame): mode 0 = locked, 1 = actuated
 * hinge limited to [lo, hi] rad with torque gear * action[act].  parent = -1
 * attaches the child to the static world.  Joints must be listed parents-first. */
typedef struct sim_joint_desc {
  int32_t parent, child;
  double anchor[3];
  double axes[3][3];
  int32_t mode[3];
  int32_t act[3];
  double lo[3], hi[3], gear[3];
} sim_joint_desc_t;

typedef struct sim_desc {
  int32_t n_bodies, n_joints; /* <= SIM_MAX_BODIES / SIM_MAX_JOINTS */
  const sim_body_desc_t* bodies;
  const sim_joint_desc_t* joints;
  int32_t root_body;              /* body whose pose feeds the root observations */
  int32_t n_feet;                 /* <= SIM_MAX_FEET */
  int32_t foot_bodies[SIM_MAX_FEET];
  double term_height;             /* done when root height falls below this (Section 4.1) */
  double alive_bonus;             /* R_alive of Eq. (1): 0.5 ant, 2 humanoid */
  int32_t max_episode_steps;      /* done when reached (1000 in Section 4.1) */
  int32_t terrain_kind;           /* 0 = plane z = 0 (env-local), 1 = heightfield */
  int32_t hf_nx, hf_ny;           /* height samples per axis (cells = n - 1) */
  double hf_cell, hf_origin[2];   /* world xy of sample (0,0) and sample spacing */
  const float* hf_heights;        /* host, [hf_ny][hf_nx] */
  const double* env_origins;      /* host, [num_envs][3] world position of each env's origin */
  double gravity[3];
  double mu;                      /* isotropic Coulomb friction coefficient (1.0 in Section 3.1) */
  double contact_margin;          /* speculative contacts are created below this gap */
  double beta_joint, beta_contact;/* positional error feedback factors */
  double max_depen_vel;           /* cap on the penetration recovery speed */
  double lin_damping, ang_damping, max_ang_vel;
  double reset_noise;             /* amplitude of the uniform reset perturbation */
  int32_t gyroscopic;             /* 1 = explicit gyroscopic torque */
  int32_t contacts;               /* 0 disables contact generation */
  int32_t height_map;             /* 1 appends the 15 x 11 terrain height map that follows the centre of mass
                                     (Section 4.1, complex-terrain task) to the observation: 165 more floats */
  /* Capsule-capsule collisions (Section 3.1: contacts among bodies are detected speculatively;
   * Section 4.1: inter-agent collisions of the flagrun tasks).  collide_pairs: body pairs of one
   * agent that may touch each other (host, [n_collide_pairs][2], first < second, at most
   * SIM_MAX_BODIES * (SIM_MAX_BODIES - 1) / 2; leave out bodies that a joint connects or that
   * overlap by construction); 0 pairs = no self-collision.  group_size consecutive agents form
   * one interaction group: every body of an agent may touch every body of the other agents of
   * its group, groups never interact (their env_origins say where the agents stand); 0 or 1 =
   * agents do not see each other, at most SIM_MAX_GROUP.  A group is simulated by one workgroup,
   * which holds at most SIM_PAIR_CAP capsule-capsule contacts per substep (see
   * sim_get_pair_contacts). */
  int32_t n_collide_pairs;
  const int32_t* collide_pairs;
  int32_t group_size;
  /* Warm start of the rows (a stiffness gain within the relaxation scheme of Section
   * 3.1): every joint row, and every terrain contact slot that was active in the previous
   * substep, starts a substep from warm_start (0..1; 0 = off) times the impulse it ended the
   * previous one with (a limit row only if it still stands for the same limit); these impulses
   * are applied to the bodies before the first sweep (Jacobi) or are the first Newton iterate
   * (solver 1, where 0.8 is worth about one Newton iteration in three).  What is kept survives from one sim_step
   * to the next and is cleared for an env by its reset and for all by sim_set_state.  About 0.8
   * halves the sweeps needed for the same penetration; with few sweeps values near 1 can build
   * up without bound (the kept impulse integrates the position error).  Capsule-capsule contacts
   * (whose identity changes from substep to substep) keep nothing: with collisions switched on
   * they start every substep from zero next to warm joints and terrain slots. */
  double warm_start;
  /* Solver of the rows (Section 3.1).  0: block projected Jacobi with mass splitting; the
   * `iterations` of sim_step are sweeps per substep.  1: the paper's own choice, a non-smooth
   * Newton method (minimum map for one-sided rows, smooth isotropic Coulomb friction) whose every
   * iteration is solved by krylov_iterations preconditioned conjugate-residual iterations on
   * J M^-1 J^T (+ newton_reg times its diagonal, a damping of the Newton step that does not move
   * the solution; 0.1 keeps single and double precision on the same branches); the `iterations` of
   * sim_step are then Newton iterations per substep (3 with 8 inner iterations is a sensible start).  It solves the joints
   * far more stiffly per unit of work where loads are carried (a hanging chain does not sag), costs
   * about 3.3 times a 20-sweep step, runs at most 8 envs per workgroup, and is not available together
   * with capsule-capsule collisions (SIM_ERR_ARG). */
  int32_t solver;
  int32_t krylov_iterations;
  double newton_reg;
} sim_desc_t;

/* Task logic around the step (Section 4.1 of the paper).  The numbers in brackets are the
 * paper's for the flagrun tasks.
 *  - fall_grace_frames: an env is done when its root has been below term_height for more than
 *    this many consecutive frames [160; 0 for Ant / Humanoid: done at once];
 *  - target_period, target_reach, target_radius: the per-env target is re-drawn uniformly in the
 *    disc of target_radius [100 m] around the root every target_period frames [200], or as soon as
 *    the root is within target_reach [1 m] of it; period 0 keeps the targets as they are set;
 *  - push_min_frames..push_max_frames [200..300]: uniform integer number of frames between two
 *    pushes; a push is a horizontal force of uniform magnitude push_min_newton..push_max_newton
 *    ["a few newtons"] and uniform direction on the root body for one frame; push_max_frames 0
 *    disables pushes;
 *  - auto_reset: an env that is done starts its next episode inside the same call (reset recipe
 *    seeded by seed and the env's episode index); the observation delivered for it is the first
 *    one of the new episode, reward and done are those of the step that ended the old one.
 * Every draw comes from the counter-based generator of sim_reset keyed by (seed, episode, env,
 * frame), so they are reproducible and do not depend on the launch shape. */
typedef struct sim_task_desc {
  int32_t enabled, fall_grace_frames, target_period, push_min_frames, push_max_frames, auto_reset;
  double target_reach, target_radius, push_min_newton, push_max_newton;
  uint64_t seed;
} sim_task_desc_t;

/* One contact slot of one env.  Slots are static: for each body in order, a
 * capsule owns slot "end -" and "end +" (plus "mid-segment" on a heightfield),
 * a sphere owns one.  kind: -1 none, 0 plane, 1 closest point of triangle
 * `feat`, 2 centre underneath triangle `feat` (plane distance), 3 heightfield
 * edge `feat` against the segment interior.  Triangle id = 2*(j*(nx-1)+i)+t with
 * t = 0 for corners (i,j),(i+1,j),(i+1,j+1) and t = 1 for (i,j),(i+1,j+1),
 * (i,j+1); edge id = 3*(j*nx+i)+k from sample (i,j) towards +x, +y, +x+y. */
typedef struct sim_contact_rec {
  int32_t active, kind, feat;
  float d;     /* signed gap along n */
  float n[3];  /* unit normal, terrain -> body */
  float rc[3]; /* lever arm from the body centre to the body's surface point */
  float w;     /* share of its body this contact block gets in the solver's mass splitting, (0,1]:
                  rises from 0 at the margin to 1 at half the margin; the mid-segment slot also
                  fades towards the segment ends.  0 when inactive. */
  int32_t pad;
} sim_contact_rec_t;

/* One capsule-capsule contact of the last substep.  Body A = (env_a, body_a), B = (env_b, body_b);
 * s, t: parameters of the closest points on the two segments (0 at the -half_len end, 1 at the
 * other); d: gap between the surfaces; w: share in the mass splitting, as for terrain contacts. */
typedef struct sim_pair_contact_rec {
  int32_t env_a, body_a, env_b, body_b;
  float s, t, d, w;
} sim_pair_contact_rec_t;
#define SIM_MAX_GROUP 16
#define SIM_PAIR_CAP 96

/* Built-in descriptions (host calls, no GPU work), so that a C caller needs no table generator:
 * sim_default_params fills every scalar parameter of *desc with the values of the benchmark
 * configurations (gravity (0, 0, -9.81), mu 1 as in Section 3.1, margin 2 cm, feedback factors
 * 0.2, recovery speed 2 m/s, no damping, angular velocity cap 64 rad/s, reset noise 0.05,
 * gyroscopic term and contacts on, 1000-frame episodes as in Section 4.1, plane terrain, no height
 * map, no collisions among bodies, no warm start, Jacobi solver) and clears its pointers.
 * sim_builtin_robot points desc->bodies / joints at tables inside the library (valid until the
 * library is unloaded; do not free) and sets the counts, root, feet, fall threshold and alive
 * bonus: SIM_ROBOT_ANT (9 bodies, 8 joints, 8 actuated hinges) or SIM_ROBOT_HUMANOID (13
 * capsules, 12 joints, 21 actuated hinges), the stick figures of the benchmark configurations
 * (Section 4.1 names the Ant and Humanoid tasks; the dimensions are this build's own).  The
 * caller still supplies terrain, env_origins and, if wanted, collide_pairs.  SIM_ERR_ARG for a
 * NULL desc or an unknown kind.  (This is the "robot kind" of a description; custom tables are
 * simply the caller's own bodies / joints.) */
#define SIM_ROBOT_ANT 1
#define SIM_ROBOT_HUMANOID 2
int sim_default_params(sim_desc_t* desc);
int sim_builtin_robot(int32_t robot_kind, sim_desc_t* desc);

/* Bytes of device workspace sim_create needs for this description (256-byte aligned base).
 * (Section 3.1, last paragraph: all robots are held by one simulation; the workspace is that
 * simulation's memory: tables, heightfield, body state of all envs, staging of the outputs.)
 * Host call, no GPU work.  SIM_ERR_ARG on an inconsistent description (same checks as sim_create). */
int sim_workspace_bytes(const sim_desc_t* desc, int num_envs, size_t* out_bytes);

/* One simulation holding num_envs robots (Section 3.1, last paragraph; the many-environments-
 * per-GPU framing of Section 3).  Builds the static tables from `desc` (copied; the caller may
 * free it afterwards), uploads them and the heightfield into `workspace_dev` (device memory the
 * caller owns and keeps alive until sim_destroy) and puts every env in its unperturbed rest
 * pose.  Synchronous.  SIM_ERR_ARG on an inconsistent description,
 * SIM_ERR_WORKSPACE if workspace_bytes < sim_workspace_bytes(). */
int sim_create(const sim_desc_t* desc, int num_envs, void* workspace_dev, size_t workspace_bytes,
               sim_t** out);
/* Ends the simulation: frees the host object (the workspace stays the caller's; a static
 * workspace becomes free for the next sim_create_static).  No passage of the paper; NULL is
 * SIM_ERR_ARG. */
int sim_destroy(sim_t* sim);

/* For callers that cannot allocate device memory (harnesses that forbid it, serving loops that
 * must not touch the allocator): sim_create with the workspace in a device array that is part of
 * the library, SIM_STATIC_WORKSPACE_BYTES per GPU, held from the library's load to the end of the
 * process.  Same description, same results and the same errors as sim_create; SIM_ERR_WORKSPACE
 * when sim_workspace_bytes(desc, num_envs) exceeds SIM_STATIC_WORKSPACE_BYTES (the message names
 * both numbers).  The sim lives on the device that is current at the call.  It calls no device
 * allocator, and neither does any later call on the sim (none of the library's calls do).
 * All static sims of one GPU share that GPU's array: at most one can exist at a time (a second
 * call before sim_destroy of the first returns SIM_ERR_WORKSPACE), the array keeps the last
 * sim's contents until the next one overwrites what it uses (everything a new sim reads is
 * written at its creation), and two threads that create static sims on one GPU at the same time
 * race.  Everything exchanged at run time (actions, observations, states) is still caller memory. */
#define SIM_STATIC_WORKSPACE_BYTES (24u << 20)
int sim_create_static(const sim_desc_t* desc, int num_envs, sim_t** out);

/* Sizes of the simulation (host calls, -1 for a NULL sim): what a caller needs to size the
 * arrays below.  Observation layout: Table 2, column "Ours" (Section 4.1). */
int sim_num_envs(const sim_t* sim);
int sim_num_bodies(const sim_t* sim);
int sim_num_slots(const sim_t* sim); /* contact slots per env */
int sim_obs_dim(const sim_t* sim);   /* 11 + 3 * act_dim + n_feet */
int sim_act_dim(const sim_t* sim);   /* number of actuated hinge DoF */

/* Seeded reset (Section 4.1: positions, velocities, joint angles and joint angular velocities
 * perturbed slightly): rest pose shifted by uniform noise, a uniform linear velocity of the body
 * the joint tree hangs from, every hinge angle perturbed (clipped to its limits) and every hinge
 * given a uniform rate, all of amplitude reset_noise; children are placed and moved so that their
 * joints are assembled.  env_mask_dev: one byte per env, non-zero = reset; NULL = all envs. */
int sim_reset(sim_t* sim, const uint8_t* env_mask_dev, uint64_t seed, void* stream);

/* Advances all envs by dt in `substeps` substeps of `iterations` solver sweeps each and
 * packs obs/reward/done.  actions_dev: [N][act_dim] in [-1,1] (clipped inside); NULL = zeros.
 * SIM_ERR_ARG if dt <= 0, substeps < 1 or iterations < 0. */
int sim_step(sim_t* sim, const float* actions_dev, float dt, int substeps, int iterations,
             void* stream);

/* sim_step followed by sim_get_obs in one kernel launch: the step's observation, reward and
 * done flag (Table 2 "Ours", Eq. 1-3, Section 4.1) are written to the caller's arrays as they
 * are packed, instead of the library's own copies (each output is stored once: an output whose
 * pointer is NULL goes to the library's copy as in sim_step, and sim_get_obs refuses with
 * SIM_ERR_ARG to return an output that the last step handed to the caller).  Same arguments,
 * limits and errors as the two calls; any of the three output pointers may be NULL.  Like sim_step it is one kernel launch on `stream`, allocates
 * nothing and does not synchronise, so it can be captured in a HIP graph and replayed (the
 * graph then steps with whatever the actions array holds at replay time). */
int sim_step_obs(sim_t* sim, const float* actions_dev, float dt, int substeps, int iterations,
                 float* obs_dev /*[N][obs_dim]*/, float* reward_dev /*[N]*/, uint8_t* done_dev /*[N]*/,
                 void* stream);

/* Copies what the last sim_step packed (or, before any step, the values of the current
 * state) into caller arrays; any of the three pointers may be NULL. */
int sim_get_obs(sim_t* sim, float* obs_dev, float* reward_dev, uint8_t* done_dev, void* stream);

/* Per-env target position, env-local xy, [N][2] (Section 4.1 flagrun targets; the plain
 * running tasks keep the default (1000, 0), i.e. "forwards"). */
int sim_set_targets(sim_t* sim, const float* target_xy_dev, void* stream);

/* Switches the task logic on (task->enabled != 0) or off (NULL or enabled == 0) for the following
 * sim_step / sim_step_obs calls and starts episode 0 of every env from the current body state
 * (counters cleared, first push time and, with target_period > 0, first target drawn).  With
 * auto_reset, an env whose episode ends in a step is put back to a fresh initial state at the end
 * of that same step (still one kernel launch): the step returns the ended episode's last reward
 * and done = 1 next to the first observation of the next episode.  SIM_ERR_ARG on inconsistent
 * numbers. */
int sim_set_task(sim_t* sim, const sim_task_desc_t* task, void* stream);
/* Warm start only (SIM_ERR_ARG otherwise): the impulses kept for the next substep, joint rows
 * [N][n_joints][6] (world x, y, z, then the joint's three axes; a limit row's is that of the limit
 * it stood for, >= 0) and terrain slot rows [N][n_slots][3] (normal, two tangents; 0 for slots
 * that were not active in the last substep).  Either pointer may be NULL. */
int sim_get_kept_impulses(sim_t* sim, float* joint_rows_dev, float* slot_rows_dev, void* stream);
/* Per-env task state: counters [N][4] = frames below the threshold, target age, frame of the
 * next push (-1: none), episode index; targets [N][2] env-local; push [N][3] = force on the root
 * during the last step.  Any output pointer may be NULL. */
int sim_get_task_state(sim_t* sim, int32_t* counters_dev, float* targets_dev, float* push_dev, void* stream);
int sim_set_task_state(sim_t* sim, const int32_t* counters_dev, const float* targets_dev, void* stream);

/* Parity / checkpoint interface (not on the timed path; no passage of the paper defines it: it
 * exposes the maximal-coordinate state of Section 3.1 so that a run can be compared, saved and
 * resumed).  State: [N][n_bodies][13] floats per body = position (env-local), unit quaternion
 * (w, x, y, z; body to world), linear velocity, angular velocity (world frame), device memory.
 * sim_set_state also clears what the warm start keeps and invalidates recorded contacts;
 * neither call synchronises.  sim_set_step_count: frame counter of every env ([N], device), the
 * one the 1000-frame episode limit of Section 4.1 counts. */
int sim_get_state(sim_t* sim, float* state_dev, void* stream);
int sim_set_state(sim_t* sim, const float* state_dev, void* stream);
int sim_set_step_count(sim_t* sim, const int32_t* counts_dev, void* stream);
/* Terrain contacts (Section 3.1: contacts are detected speculatively, i.e. within a margin before
 * they touch).  sim_record_contacts (host flag): when enabled, sim_step also stores the contact
 * records of its last substep, one sim_contact_rec_t per slot, which sim_get_contacts copies to
 * recs_dev (SIM_ERR_ARG if nothing was recorded since the state last changed). */
int sim_record_contacts(sim_t* sim, int enable);
int sim_get_contacts(sim_t* sim, sim_contact_rec_t* recs_dev /*[N][S]*/, void* stream);
/* The same contact generation alone, on the current state, straight into recs_dev (no step). */
int sim_generate_contacts(sim_t* sim, sim_contact_rec_t* recs_dev /*[N][S]*/, void* stream);
/* Capsule-capsule contacts of the last substep of the last sim_step (recording enabled): up to
 * `cap` records into recs_dev, workgroup by workgroup, each workgroup's in a fixed order; the total
 * number goes to count_dev[0] and count_dev[1] receives the number of contacts that were left out
 * since sim_create because a workgroup found more than SIM_PAIR_CAP in one substep.  What stays
 * then is fixed: the SIM_PAIR_CAP contacts of the workgroup's agents with the smallest gap d
 * (single precision; equal gaps: the smaller key (agent of A within the workgroup, agent of B,
 * body_a, body_b)), whatever order they were found in, so a run is reproducible and equals a
 * reference that applies the same bound to blocks of envs_per_block agents; the contacts left
 * out are the most distant ones, which speculative contacts (Section 3.1) mostly keep idle.
 * (This holds up to the number of contacts a workgroup can list at all, at least 256; past that,
 * the ones listed first take part in the choice.)  SIM_ERR_ARG if the description had neither
 * collide pairs nor groups. */
int sim_get_pair_contacts(sim_t* sim, sim_pair_contact_rec_t* recs_dev, int32_t cap, int32_t* count_dev /*[2]*/,
                          void* stream);
/* Interaction groups chosen from where the agents are (Section 3.1, last paragraph: all agents
 * are simulated in one shared scene; Section 4.1: the agents of the flagrun tasks collide with
 * each other).  At creation agent k stands at place k and group_size consecutive places form a
 * group, so agents that walk away from their group mates stop meeting anybody.  These calls
 * re-assign the places; everything the caller sees (states, actions, observations, records)
 * stays indexed by agent.  All need group_size > 1 (SIM_ERR_ARG otherwise).
 *
 * sim_regroup: a uniform grid of `cell` metres over the ground plane; an agent's cell is that of
 *   its root body's world position (cell index floor(p / cell) + 32768 per axis, clamped to 16
 *   bits); agents are ordered along the Hilbert curve of order 16 through the cells (equal cells:
 *   by agent number).  Inside windows of (256 / group_size) * group_size consecutive agents of
 *   that order, agents whose root bodies are within `reach` metres of each other are then put
 *   together: in window order every free agent with a free neighbour starts a cluster that takes,
 *   up to group_size members, the first free neighbour of any member; the clusters are laid out
 *   one after another, one that does not fit into the group being filled moves to the next group
 *   and the gap is closed with agents without free neighbours (else with the cluster's first
 *   members); the remaining agents come last.  Groups are every group_size consecutive places of
 *   that layout.  `reach` is about twice an agent's radius of action, `cell` a few times that.
 *   Call it every few steps: the cost is one pass over all pairs of agents (quadratic, no scratch
 *   memory; 0.08 ms at 4096 agents, 1 ms at 65536).  Agents close to each other that still end
 *   up in different groups (their group was full, a window border runs between them) do not
 *   collide; sim_count_near_pairs says how many such pairs there are.
 * sim_set_groups: place_env_dev[N] (device) names the agent at every place, any permutation of
 *   0 .. N-1 (checked; SIM_ERR_ARG if it is none; synchronises `stream`); NULL puts every agent
 *   back at the place of its own number.
 * sim_get_groups: the current place_env into place_env_dev[N] (device).
 * sim_count_near_pairs: counts_dev[0] = agent pairs whose root bodies are within `reach` metres,
 *   counts_dev[1] = those of them that the current groups keep apart (device, two int64). */
int sim_regroup(sim_t* sim, float cell, float reach, void* stream);
int sim_set_groups(sim_t* sim, const int32_t* place_env_dev, void* stream);
int sim_get_groups(sim_t* sim, int32_t* place_env_dev, void* stream);
int sim_count_near_pairs(sim_t* sim, float reach, int64_t* counts_dev /*[2]*/, void* stream);
/* Health check of a run (no passage of the paper).  Synchronises `stream` and scans the state:
 * SIM_ERR_NONFINITE if any value is NaN/Inf. */
int sim_check(sim_t* sim, void* stream);

/* Launch shape (no passage of the paper; the paper's engine is a different design).  sim_launch_info:
 * the launch shape of sim_step as it stands: threads and envs per workgroup, dynamic LDS bytes per
 * workgroup (grid = ceil(num_envs / envs_per_block)).  Any output pointer may be NULL. */
int sim_launch_info(const sim_t* sim, int32_t* threads_per_block, int32_t* envs_per_block, size_t* lds_bytes);

/* sim_set_envs_per_block: envs per workgroup of sim_step (0 = library default; a multiple of
 * group_size; SIM_ERR_ARG if the workgroup's arrays would not fit).  Results are bit-reproducible
 * for a given launch shape, and contact sets are the same for all; the continuous state of two
 * launch shapes agrees to rounding (they run different instantiations of the kernel). */
int sim_set_envs_per_block(sim_t* sim, int envs_per_block);

/* Error reporting (no passage of the paper): message for the last error on the calling thread
 * (never NULL; owned by the library, valid until the thread's next failing call). */
const char* sim_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
