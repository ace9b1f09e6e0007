/*
 * CPU oracle for the batched rigid-body step -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar fp64 implementation of the per-substep physics step
 * (maximal coordinates, torque actuation, speculative unilateral contacts with
 * isotropic Coulomb friction mu, restitution 0, implicit-style velocity
 * stepping: Section 3.1 of the paper) with a fixed-count projected-Jacobi
 * solve (or the paper's non-smooth Newton / Krylov solver as the second
 * solver), followed by the observation vector of Table 2 ("Ours" column) and
 * the reward of Eq. (1)-(3).  It shares no code with the HIP library and must only
 * be used by tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * Every function of it is pinned by a closed form, an invariant, a brute-force
 * search or a value the paper prints (tests/test_oracle_*.py).  Parity unpinned:
 * the two odd multipliers that spread (env, index) over the generator's seeds
 * (any pair of odd constants would do; only the generator itself is pinned, to
 * its published outputs), and anything about gait quality or learning curves,
 * for which the paper gives no number.
 *
 * All arrays are host memory.  State interchange: state[N][B][13] =
 * position(3), quaternion(w,x,y,z), linear velocity(3), angular velocity(3),
 * positions env-local, velocities world-frame.
 */
#ifndef ORACLE_H
#define ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct oracle_desc {
  int32_t n_bodies, n_joints, n_dofs, n_feet;
  const double* radius;    /* [B] */
  const double* half_len;  /* [B] 0 = sphere */
  const int32_t* axis;     /* [B] body axis of the capsule segment */
  const double* mass;      /* [B] */
  const double* inertia;   /* [B][3] body-frame diagonal */
  const double* rest_pos;  /* [B][3] */
  const int32_t* j_parent; /* [J] -1 = world */
  const int32_t* j_child;  /* [J] */
  const double* j_anchor;  /* [J][3] rest-pose anchor */
  const double* j_axes;    /* [J][3][3] rows e_0,e_1,e_2 in the parent frame */
  const int32_t* j_mode;   /* [J][3] 0 lock, 1 limited actuated hinge */
  const double* j_lo;      /* [J][3] */
  const double* j_hi;      /* [J][3] */
  const double* j_gear;    /* [J][3] */
  const int32_t* j_act;    /* [J][3] action index or -1 */
  int32_t root_body;
  const int32_t* feet;     /* [n_feet] body indices */
  double term_height, alive_bonus;
  int32_t terrain_kind;    /* 0 plane z=0, 1 heightfield */
  int32_t hf_nx, hf_ny;
  double hf_cell, hf_origin[2];
  const float* hf_heights; /* [ny][nx] */
  const double* env_origins; /* [N][3] */
  double gravity[3], mu, margin, beta_joint, beta_contact, max_depen_vel;
  double lin_damping, ang_damping, max_ang_vel, reset_noise;
  int32_t gyroscopic, contacts, max_episode_steps;
  int32_t height_map;      /* 1: observation carries the 15 x 11 height map (Section 4.1, complex terrain) */
  /* Capsule-capsule collisions (Section 3.1: contacts among bodies; Section 4.1: inter-agent
   * collisions).  collide_pairs lists the body pairs of one agent that may touch (bodies joined
   * by a joint or overlapping in the rest pose are left out by whoever builds the list).
   * group_size consecutive agents form one interaction group: every body of an agent may touch
   * every body of another agent of its group; groups never interact.  0 or 1: no inter-agent
   * contacts. */
  int32_t n_collide_pairs;
  const int32_t* collide_pairs; /* [n_collide_pairs][2] */
  int32_t group_size;
} oracle_desc;

/* Task logic around the step (Section 4.1).  All off when `enabled` is 0.
 *  - fall_grace_frames: an env terminates when its root has been below term_height for more than
 *    this many consecutive frames (0: at once, as for Ant / Humanoid; 160 for the flagrun tasks);
 *  - target_period / target_reach / target_radius: the flagrun target is re-drawn uniformly in the
 *    disc of target_radius around the root every target_period frames, or as soon as the root is
 *    within target_reach of it (200 frames, 1 m, 100 m); period 0 keeps the targets as set;
 *  - push_*: every push_min..push_max frames (uniform integer; 200..300) a horizontal force of
 *    uniform magnitude push_min..push_max newton and uniform direction acts on the root body for
 *    one frame; push_max_frames 0 disables pushes;
 *  - auto_reset: an env that is done is reset at once (reset recipe, new episode seed); the
 *    observation returned for it is the first one of the new episode, reward and done are those
 *    of the step that ended the old one. */
typedef struct oracle_task {
  int32_t enabled, fall_grace_frames, target_period, push_min_frames, push_max_frames, auto_reset;
  double target_reach, target_radius, push_min_newton, push_max_newton;
  uint64_t seed;
} oracle_task;

typedef struct oracle_contact {
  int32_t active; /* 0/1 */
  int32_t kind;   /* -1 none, 0 plane, 1 triangle closest point, 2 triangle underneath, 3 edge (mid-segment) */
  int32_t feat;   /* -1, triangle id or edge id */
  int32_t pad;
  double d, n[3], rc[3];
  double w;       /* share of the body this contact block gets in the mass splitting, (0,1] */
} oracle_contact;

/* One capsule-capsule contact.  Body A = (env_a, body_a), body B = (env_b, body_b); s, t are the
 * single-precision parameters of the closest points on the two segments (0 at the -l end, 1 at
 * the +l end); n points from B to A; ra / rb are the contact point (midway between the closest
 * points of the two surfaces) relative to the respective body centre; d is the surface distance. */
typedef struct oracle_pair_contact {
  int32_t env_a, body_a, env_b, body_b;
  float s, t;
  double d, n[3], ra[3], rb[3];
  double w;       /* mass-splitting share on both bodies, as for terrain contacts */
  float gap32;    /* the surface distance as the single-precision decision sees it: (sqrt(d2) - r_a) - r_b */
  int32_t pad_;
} oracle_pair_contact;

/* per-sweep diagnostics of one env (used by the invariant pins) */
typedef struct oracle_sweep_trace {
  double bilateral_rms;   /* rms of (J v + bias) over bilateral rows, velocity snapshot of this sweep */
  double bilateral_max;
  double onesided_viol;   /* max over one-sided rows of max(0, -(J v + bias)) */
  double sum_lambda_n;    /* sum of accumulated normal impulses after the sweep */
  double cone_excess;     /* max over slots of |lambda_t| - mu*lambda_n_prev after the sweep */
  double pos_err_max;     /* max |C| over joints (constant within a substep) */
} oracle_sweep_trace;

typedef struct oracle_sim oracle_sim;

oracle_sim* oracle_create(const oracle_desc* desc, int32_t num_envs);
void oracle_destroy(oracle_sim*);
int32_t oracle_n_slots(const oracle_sim*);
int32_t oracle_obs_dim(const oracle_sim*);
void oracle_set_threads(oracle_sim*, int32_t n);       /* OpenMP threads over envs */
int32_t oracle_get_threads(const oracle_sim*);

void oracle_reset(oracle_sim*, const uint8_t* env_mask /*NULL=all*/, uint64_t seed);
void oracle_set_state(oracle_sim*, const double* state);
void oracle_get_state(const oracle_sim*, double* state);
/* Warm start (a stiffness gain within the Jacobi scheme, Section 3.1): every joint row and every
 * terrain contact slot that was active in the previous substep starts from `share` (0..1, 0 =
 * off, the default) times its impulse at the end of that substep; a limit row only if it stands
 * for the same limit as then.  These impulses are applied to the bodies before the first sweep.
 * Reset and oracle_set_state clear what is kept.  With few sweeps the kept impulse acts as an
 * integrator on the position error, and a share of 1 can then grow without bound (a hanging
 * chain at 4 sweeps does); 0.8 to 0.9 is the useful range. */
void oracle_set_warm_start(oracle_sim*, double share);
/* Solver of the rows.  kind 0 (default): block projected Jacobi, `iterations` of oracle_step are
 * sweeps.  kind 1: the paper's solver (Section 3.1), a non-smooth Newton method with a Krylov
 * inner solve: `iterations` of oracle_step are Newton iterations per substep, each solved by
 * `krylov_iters` preconditioned conjugate-residual iterations on J M^-1 J^T (+ reg times its
 * diagonal: a damping of the Newton step that leaves the fixed point where it is); same rows, biases and friction law as kind 0, no mass splitting. */
void oracle_set_solver(oracle_sim*, int32_t kind, int32_t krylov_iters, double reg);
/* What is kept for the next substep: joint row impulses [N][J][6] (world x, y, z, then the three
 * joint axes) and terrain slot impulses [N][S][3] (normal, two tangents; 0 for inactive slots). */
void oracle_get_warm(const oracle_sim*, double* lam_j, double* lam_s);
/* Overwrites what is kept (tests inject known impulses); a limit row's value then stands for
 * whichever limit is the nearer one in the next substep. */
void oracle_set_warm(oracle_sim*, const double* lam_j, const double* lam_s);
/* What the kept impulses stood for (after oracle_set_warm): limit_side [N][J][3], 0 = the lower
 * limit, 1 = the upper limit, -1 = whichever limit is nearer now; slot_was_active [N][S], 0 = the
 * slot was not active in the previous substep.  Sets bookkeeping only, no arithmetic. */
void oracle_set_warm_flags(oracle_sim*, const int32_t* limit_side, const int32_t* slot_was_active);
void oracle_set_targets(oracle_sim*, const double* target_xy /*[N][2] env-local*/);
void oracle_set_step_count(oracle_sim*, const int32_t* counts /*[N]*/);
/* Switches the task logic on (or off with NULL / enabled 0) and initialises the per-env task
 * state from the current body state: episode 0, counters 0, first push time and (period > 0)
 * first target drawn. */
void oracle_set_task(oracle_sim*, const oracle_task* task);
/* per-env task state: counters[N][4] = frames below threshold, target age, frame of the next
 * push (-1 none), episode index; targets[N][2] env-local */
void oracle_get_task_state(const oracle_sim*, int32_t* counters, double* targets);
void oracle_set_task_state(oracle_sim*, const int32_t* counters, const double* targets);
/* force (N) that acted on the root body during the last step, [N][3] */
void oracle_get_last_push(const oracle_sim*, double* push);

/* phase mask for oracle_step_phases */
#define ORACLE_PH_CONTACTS 1
#define ORACLE_PH_FORCES 2
#define ORACLE_PH_SOLVE 4
#define ORACLE_PH_INTEGRATE 8
#define ORACLE_PH_ALL 15

void oracle_step(oracle_sim*, const double* actions /*[N][D]*/, double dt, int32_t substeps,
                 int32_t iterations);
/* one substep of length h restricted to the given phases (no obs packing, no step count) */
void oracle_substep_phases(oracle_sim*, const double* actions, double h, int32_t iterations,
                           int32_t phase_mask);
void oracle_get_obs(const oracle_sim*, double* obs /*[N][obs_dim]*/, double* reward /*[N]*/,
                    uint8_t* done /*[N]*/);
/* contact records of the last substep, [N][S] */
void oracle_get_contacts(const oracle_sim*, oracle_contact* recs);
/* contact generation alone on the current state; brute != 0 scans every triangle/edge */
void oracle_generate_contacts(oracle_sim*, int32_t brute, oracle_contact* recs);
/* capsule-capsule contacts of the last substep, all groups in order; returns their number
 * (at most cap are written) */
int32_t oracle_get_pair_contacts(const oracle_sim*, oracle_pair_contact* out, int32_t cap);
/* the same from the current state, without stepping */
int32_t oracle_generate_pair_contacts(oracle_sim*, oracle_pair_contact* out, int32_t cap);
/* A bounded contact store (Section 3.1 fixes no size; a device that keeps a block of agents'
 * contacts in on-chip memory has one): consecutive blocks of `envs_per_unit` agents (a multiple of
 * the group size) keep at most `cap` capsule-capsule contacts per substep, those with the smallest
 * (gap32, key) in that order, key = (agent of A in the block << 20) | (agent of B in the block << 8)
 * | (body of A << 4) | body of B.  cap <= 0: no bound (the default).  Returns the number of
 * contacts removed since the last call. */
int64_t oracle_set_pair_cap(oracle_sim*, int32_t cap, int32_t envs_per_unit);
/* Interaction groups chosen from where the agents are (Section 3.1: all agents share one scene;
 * Section 4.1: the agents of the flagrun tasks collide with each other).  Groups are G consecutive
 * *places*; place p holds agent place_env[p] (at creation: agent p).  oracle_regroup orders the
 * agents along the Hilbert curve (order 16) through the cells of a uniform grid of `cell` metres
 * over the ground plane (an agent's cell is that of its root body's world position, cell index
 * floor(p / cell) + 32768 clamped to 16 bits per axis; ties by agent number); then, inside windows
 * of (256 / G) G consecutive agents of that order, agents whose root bodies are within `reach`
 * of each other are put together: in window order every free agent with a free neighbour starts
 * a cluster that takes, up to G members, the first free neighbour of any member; the clusters
 * are laid out one after another, one that does not fit into the group being filled moves on to
 * the next group and the gap is closed with agents that have no free neighbour (else with the
 * cluster's first members); the remaining agents come last.  The places
 * are handed out group by group.  oracle_set_groups takes any permutation (NULL: agents in their
 * own order; returns -1 if it is none).  oracle_count_near_pairs: counts[0] = agent pairs whose
 * root bodies are within `reach`, counts[1] = those of them in different groups.  All of these
 * decide in single precision (positions rounded to float before the origin is added). */
void oracle_regroup(oracle_sim*, double cell, double reach);
int32_t oracle_set_groups(oracle_sim*, const int32_t* place_env);
void oracle_get_groups(const oracle_sim*, int32_t* place_env);
void oracle_count_near_pairs(const oracle_sim*, double reach, int64_t* counts);
/* single-precision closest points of two segments P0P1, Q0Q1 (fixed operation order): writes the
 * parameters and returns the squared distance; exposed so it can be pinned */
float oracle_segment_segment_f32(const float* P0, const float* P1, const float* Q0, const float* Q1,
                                 float* s, float* t);
/* trace env `env`: buf receives one record per sweep of subsequent steps, up to cap */
void oracle_set_trace(oracle_sim*, int32_t env, oracle_sweep_trace* buf, int32_t cap);
int32_t oracle_trace_count(const oracle_sim*);
/* joint angles theta[N][J][3] of the current state (rotation-vector components) */
void oracle_joint_angles(const oracle_sim*, double* theta);
/* uniform [0,1) draw of the reset generator, exposed so it can be pinned */
double oracle_uniform(uint64_t seed, uint64_t env, uint64_t idx);

#ifdef __cplusplus
}
#endif
#endif
