// Device-resident static tables of one simulator instance (private layout).
//
// Built on the host by sim_create from the caller's description, uploaded once
// into the workspace and read by every kernel.  Plain data, fp32 / int32.
#pragma once
#include <stdint.h>

namespace sim355 {

constexpr int kMaxBodies = 16;
constexpr int kMaxJoints = 16;
constexpr int kMaxDofs = 32;
constexpr int kMaxFeet = 4;
constexpr int kMaxSlots = 3 * kMaxBodies;
constexpr int kMaxBodyJoints = 8;  // joint sides touching one body
constexpr int kHmRows = 15, kHmCols = 11;  // height-map observation
constexpr int kCoarse = 8;         // cells per side of a coarse max-height block
constexpr int kMaxPairs = kMaxBodies * (kMaxBodies - 1) / 2;  // body pairs of one agent
constexpr int kMaxGroup = 16;      // agents of one interaction group
constexpr int kMaxAgentPairs = kMaxGroup * (kMaxGroup - 1) / 2;
constexpr int kPairCap = 96;       // capsule-capsule contacts one workgroup holds per substep
constexpr int kPairWords = 6;      // queue entry: key, body refs, s, t, weight, distance

struct BodyTab {
  float radius, half_len, inv_mass;
  float inertia[3], inv_inertia[3];
  float rest_pos[3];
  int32_t axis;
  int32_t n_joint_sides;               // number of joints this body belongs to
  int32_t joint_sides[kMaxBodyJoints]; // 2*joint + side (0 parent, 1 child), ascending
  int32_t slot0, n_slots;              // its contact slots are slot0 .. slot0+n_slots-1
};

struct JointTab {
  int32_t parent, child;
  float la[3], lb[3];   // anchor in the parent / child frame
  float axes[3][3];     // rows e_0,e_1,e_2 in the parent frame
  int32_t mode[3], act[3];
  float lo[3], hi[3], gear[3];
};

struct SlotTab {
  int32_t body;
  int32_t kind;  // 0 end sphere at -half_len, 1 end sphere at +half_len (or the sphere), 2 mid-segment
};

struct Model {
  int32_t B, J, D, S, F;
  int32_t root, feet[kMaxFeet];
  int32_t terrain_kind, nx, ny;
  int32_t cnx, cny;  // coarse max-height grid: block (I,J) covers samples [8I, 8I+8] x [8J, 8J+8]
  float cell, inv_cell, hox, hoy;
  float g[3];
  float mu, margin, beta_j, beta_c, v_depen, c_lin, c_ang, w_max, reset_noise;
  float warm;   // warm start: share of the last substep's impulses the rows start from (0: none)
  // solver of the rows: 0 block projected Jacobi; 1 non-smooth Newton with `krylov` conjugate-residual
  // iterations per Newton iteration; newton_reg times the operator's diagonal damps the Newton step
  int32_t solver, krylov;
  float newton_reg;
  float term_height, alive_bonus;
  int32_t max_steps, gyro, contacts;
  int32_t max_joint_sides;  // largest n_joint_sides over the bodies
  // height-map observation: 0 = off; sample offsets along / across the heading, metres
  int32_t height_map;
  float hm_fwd[kHmRows], hm_lat[kHmCols];
  float body_mass_frac[kMaxBodies];  // mass of each body over the total (centre of mass)
  // Capsule-capsule collisions (Section 3.1: contacts among bodies; Section 4.1: inter-agent
  // collisions): body pairs of one agent that may touch, and the interaction groups (group
  // consecutive agents see each other; agent_pair_*[k] are the members of the k-th pair of a group).
  int32_t n_pairs, group, n_agent_pairs;
  uint8_t pair_a[kMaxPairs], pair_b[kMaxPairs];
  uint8_t agent_pair_a[kMaxAgentPairs], agent_pair_b[kMaxAgentPairs];
  BodyTab bodies[kMaxBodies];
  JointTab joints[kMaxJoints];
  SlotTab slots[kMaxSlots];
  // The tables above in the order and layout the step kernel keeps them in LDS (one contiguous
  // copy at kernel start): per body {joint-side count, slot0, slot count, joint sides[8]}, per
  // slot {body, kind}, per body {radius, half length, axis, 1/mass}, per body {inertia[3],
  // inverse inertia[3]}, then the joint table as it is.
  int32_t table_words;
  int32_t table_image[kMaxBodies * (kMaxBodyJoints + 3) + 2 * kMaxSlots + 10 * kMaxBodies + kMaxJoints * 32];
};
static_assert(sizeof(JointTab) == 32 * 4, "joint table entry is 32 words");

// Task logic around the step (Section 4.1), as set by sim_set_task; passed to the kernels by value.
struct TaskParams {
  int32_t enabled, grace, period, push_min_f, push_max_f, auto_reset;
  float reach, radius, push_min_n, push_max_n;
  uint64_t seed;
};
constexpr uint64_t kEpisodeStride = 0x9E3779B97F4A7C15ULL;  // seed of episode k = seed + k * this

// Contact record as kept in LDS / exported (matches sim_contact_rec_t: 12 words).
constexpr int kRecWords = 12;

}  // namespace sim355
