// Host side of the C ABI declared in include/sim.h: description checking, static
// table construction, workspace layout, kernel launches.  All device work is in
// hand-written kernels for gfx950; there is no CPU fallback.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/sim.h"
#include "contact_gen.hpp"
#include "model.hpp"
#include "step_kernel.hpp"
#include "regroup.hpp"
#include "builtin_robots.hpp"

using namespace sim355;

static_assert(SIM_MAX_BODIES == kMaxBodies && SIM_MAX_JOINTS == kMaxJoints && SIM_MAX_DOFS == kMaxDofs &&
                  SIM_MAX_FEET == kMaxFeet,
              "public limits and table sizes must agree");
static_assert(sizeof(sim_contact_rec_t) == kRecWords * 4, "contact record is 12 words");
static_assert(sizeof(sim_pair_contact_rec_t) == 32 && SIM_PAIR_CAP == kPairCap && SIM_MAX_GROUP == kMaxGroup, "pair contact records");

// ------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";
static int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
#define HIP_TRY(expr)                                                                      \
  do {                                                                                     \
    hipError_t _e = (expr);                                                                \
    if (_e != hipSuccess) return fail(SIM_ERR_HIP, "%s: %s", #expr, hipGetErrorString(_e)); \
  } while (0)

extern "C" const char* sim_last_error(void) { return g_err; }

// ------------------------------------------------------------------ layout
struct Layout {
  size_t model, heights, coarse, origins, targets, state, steps, obs, reward, done, recs, task_i, push, flag, pair_recs, pair_count, lam_j, lam_s, place_env, grp_words, grp_counts, total;
};
static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

static Layout make_layout(int B, int J, int S, int obs_dim, int N, size_t n_heights, size_t n_coarse, int pairs, int warm) {
  Layout L;
  size_t o = 0;
  L.model = o; o = align_up(o + sizeof(Model));
  L.heights = o; o = align_up(o + (n_heights ? n_heights : 1) * sizeof(float));
  L.coarse = o; o = align_up(o + (n_coarse ? n_coarse : 1) * sizeof(float));
  L.origins = o; o = align_up(o + (size_t)N * 3 * sizeof(float));
  L.targets = o; o = align_up(o + (size_t)N * 2 * sizeof(float));
  L.state = o; o = align_up(o + (size_t)13 * B * N * sizeof(float));
  L.steps = o; o = align_up(o + (size_t)N * sizeof(int32_t));
  L.obs = o; o = align_up(o + (size_t)N * obs_dim * sizeof(float));
  L.reward = o; o = align_up(o + (size_t)N * sizeof(float));
  L.done = o; o = align_up(o + (size_t)N);
  L.recs = o; o = align_up(o + (size_t)N * S * sizeof(sim_contact_rec_t));
  L.task_i = o; o = align_up(o + (size_t)N * 4 * sizeof(int32_t));
  L.push = o; o = align_up(o + (size_t)N * 3 * sizeof(float));
  // capsule-capsule contact records: one workgroup may hold as few as one env
  L.pair_recs = o; o = align_up(o + (pairs ? (size_t)N * kPairCap * sizeof(sim_pair_contact_rec_t) : 0));
  L.pair_count = o; o = align_up(o + (pairs ? (size_t)N * sizeof(int32_t) : 0));
  // warm start: impulses kept from one step to the next, [J*6][N] and [S*3][N]
  L.lam_j = o; o = align_up(o + (warm ? (size_t)N * J * 6 * sizeof(float) : 0));
  L.lam_s = o; o = align_up(o + (warm ? (size_t)N * S * 3 * sizeof(float) : 0));
  // interaction groups chosen from positions: agent at every place, sort words / inverse map, counters
  L.place_env = o; o = align_up(o + (pairs > 1 ? (size_t)N * sizeof(int32_t) : 0));
  L.grp_words = o; o = align_up(o + (pairs > 1 ? (size_t)N * sizeof(unsigned long long) : 0));
  L.grp_counts = o; o = align_up(o + (pairs > 1 ? 256 : 0));
  L.flag = o; o = align_up(o + 256);   // (last: the diagnostic build keeps its counters here)
  L.total = o;
  return L;
}

struct sim {
  Model host_model;
  Layout lay;
  char* ws;
  int N, obs_dim, E;
  int record;
  int recs_valid;
  int pair_grid;   // workgroups of the launch that wrote the capsule-capsule records
  TaskParams task;
  int static_dev;  // device whose static workspace this sim occupies (sim_create_static), else -1
  int ws_has[3];   // the workspace holds obs / reward / done of the last step (else the caller got them)
  int regrouped;   // the places of the launch hold the agents in the order of lay.place_env (else in their own)
};

// ------------------------------------------------------- static workspace
// sim_create_static keeps the workspace in this array instead of caller memory, for callers
// that cannot allocate device memory.  Every GPU holds its own copy at its own address; host
// code uses the address hipGetSymbolAddress reports for the current device, never the name.
static __device__ __align__(256) unsigned char scratch[SIM_STATIC_WORKSPACE_BYTES];
constexpr int kMaxDevices = 64;
static unsigned char* g_scratch_ptr[kMaxDevices];   // per device, filled on first use
static sim* g_scratch_owner[kMaxDevices];           // the sim that occupies it, if any

// ------------------------------------------------------- description -> Model
static int build_model(const sim_desc_t* d, int num_envs, Model* m) {
  if (!d) return fail(SIM_ERR_ARG, "desc is NULL");
  if (num_envs < 1) return fail(SIM_ERR_ARG, "num_envs must be >= 1 (got %d)", num_envs);
  if (d->n_bodies < 1 || d->n_bodies > kMaxBodies) return fail(SIM_ERR_ARG, "n_bodies %d outside 1..%d", d->n_bodies, kMaxBodies);
  if (d->n_joints < 0 || d->n_joints > kMaxJoints) return fail(SIM_ERR_ARG, "n_joints %d outside 0..%d", d->n_joints, kMaxJoints);
  if (!d->bodies || (d->n_joints && !d->joints)) return fail(SIM_ERR_ARG, "bodies/joints table is NULL");
  if (!d->env_origins) return fail(SIM_ERR_ARG, "env_origins is NULL");
  if (d->n_feet < 0 || d->n_feet > kMaxFeet) return fail(SIM_ERR_ARG, "n_feet %d outside 0..%d", d->n_feet, kMaxFeet);
  if (d->root_body < 0 || d->root_body >= d->n_bodies) return fail(SIM_ERR_ARG, "root_body out of range");
  if (d->terrain_kind != 0 && d->terrain_kind != 1) return fail(SIM_ERR_ARG, "terrain_kind must be 0 or 1");
  if (d->terrain_kind == 1) {
    if (d->hf_nx < 2 || d->hf_ny < 2 || !(d->hf_cell > 0) || !d->hf_heights)
      return fail(SIM_ERR_ARG, "heightfield needs nx,ny >= 2, cell > 0 and a heights array");
    if ((long long)d->hf_nx * d->hf_ny > (1LL << 28)) return fail(SIM_ERR_ARG, "heightfield too large");
  }
  if (!(d->contact_margin >= 0) || !(d->mu >= 0)) return fail(SIM_ERR_ARG, "margin and mu must be >= 0");
  std::memset(m, 0, sizeof(*m));
  m->B = d->n_bodies; m->J = d->n_joints; m->F = d->n_feet;
  m->root = d->root_body;
  for (int f = 0; f < m->F; ++f) {
    if (d->foot_bodies[f] < 0 || d->foot_bodies[f] >= m->B) return fail(SIM_ERR_ARG, "foot body out of range");
    m->feet[f] = d->foot_bodies[f];
  }
  int S = 0;
  for (int b = 0; b < m->B; ++b) {
    const sim_body_desc_t& s = d->bodies[b];
    if (!(s.radius > 0) || !(s.half_len >= 0) || !(s.mass > 0) || s.axis < 0 || s.axis > 2)
      return fail(SIM_ERR_ARG, "body %d: radius/mass must be > 0, half_len >= 0, axis in 0..2", b);
    BodyTab& t = m->bodies[b];
    t.radius = (float)s.radius; t.half_len = (float)s.half_len; t.inv_mass = (float)(1.0 / s.mass);
    for (int c = 0; c < 3; ++c) {
      if (!(s.inertia[c] > 0)) return fail(SIM_ERR_ARG, "body %d: inertia must be > 0", b);
      t.inertia[c] = (float)s.inertia[c];
      t.inv_inertia[c] = (float)(1.0 / s.inertia[c]);
      t.rest_pos[c] = (float)s.rest_pos[c];
    }
    t.axis = s.axis;
    t.slot0 = S;
    t.n_slots = s.half_len > 0 ? (d->terrain_kind == 1 ? 3 : 2) : 1;
    for (int k = 0; k < t.n_slots; ++k) {
      m->slots[S].body = b;
      m->slots[S].kind = s.half_len > 0 ? k : 1;
      ++S;
    }
  }
  m->S = S;
  int D = 0;
  std::vector<char> placed(m->B, 0);
  placed[0] = 1;
  for (int j = 0; j < m->J; ++j) {
    const sim_joint_desc_t& s = d->joints[j];
    if (s.child < 0 || s.child >= m->B || s.parent < -1 || s.parent >= m->B || s.parent == s.child)
      return fail(SIM_ERR_ARG, "joint %d: parent/child out of range", j);
    if (s.parent >= 0 && !placed[s.parent]) return fail(SIM_ERR_ARG, "joint %d: joints must be listed parents-first from body 0", j);
    placed[s.child] = 1;
    JointTab& t = m->joints[j];
    t.parent = s.parent; t.child = s.child;
    for (int c = 0; c < 3; ++c) {
      t.la[c] = (float)(s.anchor[c] - (s.parent >= 0 ? d->bodies[s.parent].rest_pos[c] : 0.0));
      t.lb[c] = (float)(s.anchor[c] - d->bodies[s.child].rest_pos[c]);
    }
    for (int k = 0; k < 3; ++k) {
      double nrm = std::sqrt(s.axes[k][0] * s.axes[k][0] + s.axes[k][1] * s.axes[k][1] + s.axes[k][2] * s.axes[k][2]);
      if (std::fabs(nrm - 1.0) > 1e-6) return fail(SIM_ERR_ARG, "joint %d: axis %d is not unit length", j, k);
      for (int c = 0; c < 3; ++c) t.axes[k][c] = (float)s.axes[k][c];
      t.mode[k] = s.mode[k];
      t.act[k] = -1;
      if (s.mode[k] == 1) {
        if (s.act[k] < 0 || s.act[k] >= kMaxDofs) return fail(SIM_ERR_ARG, "joint %d: action index out of range", j);
        if (!(s.lo[k] <= s.hi[k])) return fail(SIM_ERR_ARG, "joint %d: lo > hi", j);
        t.act[k] = s.act[k];
        if (s.act[k] + 1 > D) D = s.act[k] + 1;
      } else if (s.mode[k] != 0) {
        return fail(SIM_ERR_ARG, "joint %d: mode must be 0 or 1", j);
      }
      t.lo[k] = (float)s.lo[k]; t.hi[k] = (float)s.hi[k]; t.gear[k] = (float)s.gear[k];
    }
    for (int side = 0; side < 2; ++side) {
      int body = side ? s.child : s.parent;
      if (body < 0) continue;
      BodyTab& bt = m->bodies[body];
      if (bt.n_joint_sides >= kMaxBodyJoints) return fail(SIM_ERR_ARG, "body %d belongs to more than %d joints", body, kMaxBodyJoints);
      bt.joint_sides[bt.n_joint_sides++] = 2 * j + side;
    }
  }
  m->D = D;
  for (int b = 0; b < m->B; ++b)
    if (m->bodies[b].n_joint_sides > m->max_joint_sides) m->max_joint_sides = m->bodies[b].n_joint_sides;
  {
    // LDS image of the tables (see Model::table_image)
    int32_t* w = m->table_image;
    auto put_f = [&](float f) { memcpy(w++, &f, 4); };
    for (int b = 0; b < m->B; ++b) {
      *w++ = m->bodies[b].n_joint_sides; *w++ = m->bodies[b].slot0; *w++ = m->bodies[b].n_slots;
      for (int k = 0; k < kMaxBodyJoints; ++k) *w++ = m->bodies[b].joint_sides[k];
    }
    for (int i = 0; i < m->S; ++i) { *w++ = m->slots[i].body; *w++ = m->slots[i].kind; }
    for (int b = 0; b < m->B; ++b) {
      put_f(m->bodies[b].radius); put_f(m->bodies[b].half_len); *w++ = m->bodies[b].axis; put_f(m->bodies[b].inv_mass);
    }
    for (int b = 0; b < m->B; ++b) {
      for (int c = 0; c < 3; ++c) put_f(m->bodies[b].inertia[c]);
      for (int c = 0; c < 3; ++c) put_f(m->bodies[b].inv_inertia[c]);
    }
    memcpy(w, m->joints, (size_t)m->J * sizeof(JointTab));
    w += m->J * (int)(sizeof(JointTab) / 4);
    m->table_words = (int)(w - m->table_image);
  }
  m->terrain_kind = d->terrain_kind;
  m->nx = d->hf_nx; m->ny = d->hf_ny;
  m->cnx = d->terrain_kind == 1 ? (d->hf_nx - 1 + kCoarse - 1) / kCoarse : 0;
  m->cny = d->terrain_kind == 1 ? (d->hf_ny - 1 + kCoarse - 1) / kCoarse : 0;
  m->cell = (float)d->hf_cell;
  m->inv_cell = d->terrain_kind == 1 ? 1.0f / (float)d->hf_cell : 1.0f;
  m->hox = (float)d->hf_origin[0]; m->hoy = (float)d->hf_origin[1];
  for (int c = 0; c < 3; ++c) m->g[c] = (float)d->gravity[c];
  m->mu = (float)d->mu; m->margin = (float)d->contact_margin;
  m->beta_j = (float)d->beta_joint; m->beta_c = (float)d->beta_contact;
  m->v_depen = (float)d->max_depen_vel;
  m->c_lin = (float)d->lin_damping; m->c_ang = (float)d->ang_damping;
  m->w_max = (float)std::fmin(d->max_ang_vel, 1e30);
  m->reset_noise = (float)d->reset_noise;
  if (!(d->warm_start >= 0.0 && d->warm_start <= 1.0)) return fail(SIM_ERR_ARG, "warm_start %g outside 0..1", d->warm_start);
  m->warm = (float)d->warm_start;
  if (d->solver != 0 && d->solver != 1) return fail(SIM_ERR_ARG, "solver must be 0 (Jacobi) or 1 (Newton / Krylov)");
  if (d->solver == 1 && (d->krylov_iterations < 1 || d->krylov_iterations > 64)) return fail(SIM_ERR_ARG, "krylov_iterations %d outside 1..64", d->krylov_iterations);
  if (d->solver == 1 && !(d->newton_reg >= 0.0 && d->newton_reg <= 1.0)) return fail(SIM_ERR_ARG, "newton_reg outside 0..1");
  m->solver = d->solver; m->krylov = d->solver == 1 ? d->krylov_iterations : 0; m->newton_reg = (float)d->newton_reg;
  m->term_height = (float)d->term_height; m->alive_bonus = (float)d->alive_bonus;
  m->max_steps = d->max_episode_steps; m->gyro = d->gyroscopic; m->contacts = d->contacts;
  // Height map of the complex-terrain task (Section 4.1: 15 x 11, follows the centre of mass,
  // denser near the robot).  Offsets along and across the heading: s(k) = sign(k) 0.15 (1.3^|k| - 1) / 0.3
  // for k = -4..10 (rows) and k = -5..5 (columns).
  m->height_map = d->height_map ? 1 : 0;
  for (int i = 0; i < kHmRows; ++i) {
    int k = i - 4, ak = k < 0 ? -k : k;
    double sft = 0.15 * (std::pow(1.3, (double)ak) - 1.0) / 0.3;
    m->hm_fwd[i] = (float)(k < 0 ? -sft : sft);
  }
  for (int j = 0; j < kHmCols; ++j) {
    int k = j - 5, ak = k < 0 ? -k : k;
    double sft = 0.15 * (std::pow(1.3, (double)ak) - 1.0) / 0.3;
    m->hm_lat[j] = (float)(k < 0 ? -sft : sft);
  }
  // capsule-capsule collisions
  if (d->n_collide_pairs < 0 || d->n_collide_pairs > kMaxPairs) return fail(SIM_ERR_ARG, "n_collide_pairs %d outside 0..%d", d->n_collide_pairs, kMaxPairs);
  if (d->n_collide_pairs > 0 && !d->collide_pairs) return fail(SIM_ERR_ARG, "collide_pairs is NULL");
  m->n_pairs = d->n_collide_pairs;
  for (int p = 0; p < m->n_pairs; ++p) {
    const int a = d->collide_pairs[2 * p], b = d->collide_pairs[2 * p + 1];
    if (a < 0 || b <= a || b >= m->B) return fail(SIM_ERR_ARG, "collide pair %d: need 0 <= first < second < n_bodies", p);
    m->pair_a[p] = (uint8_t)a; m->pair_b[p] = (uint8_t)b;
  }
  if (d->group_size < 0 || d->group_size > kMaxGroup) return fail(SIM_ERR_ARG, "group_size %d outside 0..%d", d->group_size, kMaxGroup);
  m->group = d->group_size > 1 ? d->group_size : 1;
  if (m->solver == 1 && (m->n_pairs > 0 || m->group > 1))
    return fail(SIM_ERR_ARG, "the Newton solver is not available together with capsule-capsule collisions");
  m->n_agent_pairs = 0;
  for (int a = 0; a < m->group; ++a)
    for (int b = a + 1; b < m->group; ++b) {
      m->agent_pair_a[m->n_agent_pairs] = (uint8_t)a; m->agent_pair_b[m->n_agent_pairs] = (uint8_t)b;
      ++m->n_agent_pairs;
    }
  if (m->group > 1) {
    // the whole group has to fit one workgroup
    if (m->group * m->B > kThreads || (m->J > 0 && 2 * m->group * m->J > kThreads - 64))
      return fail(SIM_ERR_ARG, "group_size %d does not fit one workgroup for this robot", m->group);
  }
  {
    double mt = 0.0;
    for (int b = 0; b < m->B; ++b) mt += d->bodies[b].mass;
    for (int b = 0; b < m->B; ++b) m->body_mass_frac[b] = (float)(d->bodies[b].mass / mt);
  }
  return SIM_OK;
}

// does this model generate capsule-capsule contacts, and with which group size (0: no)
static int pairs_of(const Model& m) { return (m.n_pairs > 0 || m.group > 1) ? (m.group > 1 ? m.group : 1) : 0; }
// Threads per workgroup of the step launch: the wide workgroup pays off for full workgroups of 16
// envs (more lanes for the contact search on the heightfield, a finer split of the velocity
// average everywhere); small batches and the collision and warm-start variants (which need the
// registers) keep the narrow one.
static int threads_for(const Model& m, int E) {
  return (E == 16 && m.max_joint_sides <= 4 && !pairs_of(m) && !(m.warm > 0.0f) && m.solver == 0) ? kThreadsWide : kThreads;
}
static LdsPlan plan_for(const Model& m, int E) {
  const int with_patch = (m.terrain_kind == 1 && m.nx >= kPatch && m.ny >= kPatch) ? 1 : 0;
  return make_plan(m.B, m.J, m.S, m.D, m.F, E, with_patch, pairs_of(m), threads_for(m, E), m.warm > 0.0f ? 1 : 0, m.solver);
}
// The Newton solver keeps every row's vectors in registers, one contact per thread: every slot of
// every env of the workgroup needs a contact thread of its own next to the joint wavefronts.
static bool newton_fits(const Model& m, int E) {
  const int joint_threads = ((2 * m.J * E + 63) / 64) * 64;
  return E <= 8 && m.S * E <= kThreads - joint_threads && 2 * m.B * E <= kThreads;
}

static int default_envs_per_block(const Model& m, int N) {
  // bodies need a thread each, joints two (one per side) plus a wavefront left for contacts
  int lim = kThreads / m.B;
  if (m.J > 0 && (kThreads - 64) / (2 * m.J) < lim) lim = (kThreads - 64) / (2 * m.J);
  if (lim > 16) lim = 16;
  if (m.solver == 1) {
    if (lim > 8) lim = 8;
    while (lim > 1 && !newton_fits(m, lim)) --lim;
  }
  int want = N / 256;  // keep at least one workgroup per compute unit when N allows
  if (want < 1) want = 1;
  int E = want < lim ? want : lim;
  // a workgroup holds whole interaction groups
  const int G = m.group > 1 ? m.group : 1;
  if (E < G) E = G;
  E -= E % G;
  // and the workgroup's LDS arrays have to fit
  while (E > G && (size_t)plan_for(m, E).total * sizeof(float) > 160 * 1024) E -= G;
  // the collision variants are compiled for 16 and 8 envs per workgroup (any other number runs the
  // general form, which is much slower): 8 rather than an odd number in between
  if (pairs_of(m) && E > 8 && E < 16 && 8 % G == 0) E = 8;
  return E;
}

// ----------------------------------------------------------------- kernels
__global__ void set_state_kernel(const float* __restrict__ aos, float* __restrict__ soa, int B, int N) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;  // over N*B*13, env fastest in the SoA
  int total = N * B * 13;
  if (i >= total) return;
  int env = i % N, rest = i / N, b = rest % B, f = rest / B;
  soa[i] = aos[((size_t)env * B + b) * 13 + f];
}
__global__ void get_state_kernel(const float* __restrict__ soa, float* __restrict__ aos, int B, int N) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  int total = N * B * 13;
  if (i >= total) return;
  int env = i % N, rest = i / N, b = rest % B, f = rest / B;
  aos[((size_t)env * B + b) * 13 + f] = soa[i];
}
__global__ void copy_out_kernel(const float* __restrict__ obs, const float* __restrict__ rew,
                                const uint8_t* __restrict__ done, float* obs_o, float* rew_o, uint8_t* done_o,
                                int n_obs, int N) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (obs_o && i < n_obs) obs_o[i] = obs[i];
  if (i < N) {
    if (rew_o) rew_o[i] = rew[i];
    if (done_o) done_o[i] = done[i];
  }
}
__global__ void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
__global__ void copy_i32_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
__global__ void check_kernel(const float* __restrict__ state, int n, int* flag) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n && !isfinite(state[i])) *flag = 1;  // plain store: every writer stores the same value
}

__global__ void gen_contacts_kernel(const Model* Mp, const float* __restrict__ heights,
                                    const float* __restrict__ coarse, const float* __restrict__ origins, const float* __restrict__ state,
                                    int32_t* __restrict__ recs, int N) {
  const Model& M = *Mp;
  int i = blockIdx.x * blockDim.x + threadIdx.x;  // env fastest
  if (i >= N * M.S) return;
  int env = i % N, s = i / N;
  const SlotTab sl = M.slots[s];
  const size_t fs = (size_t)M.B * N;
  const float* st = state + (size_t)sl.body * N + env;
  float x[3] = {st[0], st[fs], st[2 * fs]};
  float q[4] = {st[3 * fs], st[4 * fs], st[5 * fs], st[6 * fs]};
  float o[3] = {origins[3 * env], origins[3 * env + 1], origins[3 * env + 2]};
  ContactOut c = generate_contact(M, heights, coarse, x, q, sl.body, sl.kind, o);
  int32_t* r = recs + ((size_t)env * M.S + s) * kRecWords;
  r[0] = c.active; r[1] = c.kind; r[2] = c.feat;
  r[3] = __float_as_int(c.d);
  r[4] = __float_as_int(c.n.x); r[5] = __float_as_int(c.n.y); r[6] = __float_as_int(c.n.z);
  r[7] = __float_as_int(c.rc.x); r[8] = __float_as_int(c.rc.y); r[9] = __float_as_int(c.rc.z);
  r[10] = __float_as_int(c.w); r[11] = 0;
}

// Seeded reset of one env by one thread: the poses are built in local arrays, then stored.
struct LocalPoses {
  float x[kMaxBodies][3], q[kMaxBodies][4], v[kMaxBodies][3], w[kMaxBodies][3];
  __device__ float& X(int b, int c) { return x[b][c]; }
  __device__ float& Q(int b, int c) { return q[b][c]; }
  __device__ float& V(int b, int c) { return v[b][c]; }
  __device__ float& W(int b, int c) { return w[b][c]; }
};
__device__ void reset_one_env(const Model& M, float* __restrict__ state, int32_t* __restrict__ steps, int env,
                              uint64_t seed, int N) {
  LocalPoses P;
  reset_pose(M, env, seed, P);
  const size_t fs = (size_t)M.B * N;
  for (int b = 0; b < M.B; ++b) {
    float* st = state + (size_t)b * N + env;
    for (int c = 0; c < 3; ++c) st[c * fs] = P.x[b][c];
    for (int c = 0; c < 4; ++c) st[(3 + c) * fs] = P.q[b][c];
    for (int c = 0; c < 3; ++c) { st[(7 + c) * fs] = P.v[b][c]; st[(10 + c) * fs] = P.w[b][c]; }
  }
  steps[env] = 0;
}

__global__ void reset_kernel(const Model* Mp, float* __restrict__ state, int32_t* __restrict__ steps,
                             const uint8_t* __restrict__ mask, uint64_t seed, int N) {
  int env = blockIdx.x * blockDim.x + threadIdx.x;
  if (env >= N) return;
  if (mask && !mask[env]) return;
  reset_one_env(*Mp, state, steps, env, seed, N);
}

// Warm start: what is kept from step to step ([rows][N], rows = 6 per joint or 3 per slot) is
// dropped for the envs of the mask (NULL: all).
__global__ void clear_kept_kernel(float* __restrict__ lam, const uint8_t* __restrict__ mask, int rows, int N) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)rows * N) return;
  if (mask && !mask[i % N]) return;
  lam[i] = 0.0f;
}
// [rows][N] -> [N][rows]; limit rows (bit (r % 6) - 3 of the joint's mask) carry the limit they
// stood for in their sign, which is dropped here
__global__ void get_kept_kernel(const float* __restrict__ lam, float* __restrict__ out, int rows, int N,
                                const Model* Mp, int joints) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)rows * N) return;
  const int env = (int)(i % N), r = (int)(i / N);
  float v = lam[i];
  if (joints && r % 6 >= 3 && Mp->joints[r / 6].mode[r % 6 - 3] == 1) v = fabsf(v);
  out[(size_t)env * rows + r] = v;
}

// sim_set_task: episode 0 for every env, from the current body state
__global__ void task_init_kernel(const Model* Mp, const float* __restrict__ state, int32_t* __restrict__ task_i,
                                 float* __restrict__ targets, float* __restrict__ push,
                                 TaskParams t, int N) {
  int env = blockIdx.x * blockDim.x + threadIdx.x;
  if (env >= N) return;
  const Model& M = *Mp;
  const size_t fs = (size_t)M.B * N;
  const float rx = state[0 * fs + (size_t)M.root * N + env], ry = state[1 * fs + (size_t)M.root * N + env];
  task_begin_episode(t, task_i, targets, env, 0, rx, ry);
  push[3 * env] = push[3 * env + 1] = push[3 * env + 2] = 0.0f;
}

// ---------------------------------------------------------------- launches
static int launch_step(sim* s, const float* actions, float h, int substeps, int iterations, int count_step,
                       hipStream_t st, float* obs_out = nullptr, float* reward_out = nullptr,
                       uint8_t* done_out = nullptr) {
  const Model& m = s->host_model;
  StepArgs a;
  a.M = reinterpret_cast<const Model*>(s->ws + s->lay.model);
  a.heights = reinterpret_cast<const float*>(s->ws + s->lay.heights);
  a.coarse = reinterpret_cast<const float*>(s->ws + s->lay.coarse);
  a.origins = reinterpret_cast<const float*>(s->ws + s->lay.origins);
  a.targets = reinterpret_cast<float*>(s->ws + s->lay.targets);
  a.state = reinterpret_cast<float*>(s->ws + s->lay.state);
  a.steps = reinterpret_cast<int32_t*>(s->ws + s->lay.steps);
  a.actions = actions;
  a.obs = reinterpret_cast<float*>(s->ws + s->lay.obs);
  a.reward = reinterpret_cast<float*>(s->ws + s->lay.reward);
  a.done = reinterpret_cast<uint8_t*>(s->ws + s->lay.done);
  a.recs = (s->record && substeps > 0) ? reinterpret_cast<int32_t*>(s->ws + s->lay.recs) : nullptr;
  a.N = s->N; a.E = s->E; a.substeps = substeps; a.iterations = iterations; a.count_step = count_step;
  a.h = h;
  a.obs_out = obs_out; a.reward_out = reward_out; a.done_out = done_out;
  a.task = s->task;
  a.task_i = reinterpret_cast<int32_t*>(s->ws + s->lay.task_i);
  a.push = reinterpret_cast<float*>(s->ws + s->lay.push);
  const int pairs = pairs_of(m);
  a.pair_recs = (pairs && s->record && substeps > 0) ? reinterpret_cast<int32_t*>(s->ws + s->lay.pair_recs) : nullptr;
  a.pair_count = reinterpret_cast<int32_t*>(s->ws + s->lay.pair_count);
  a.lam_j = reinterpret_cast<float*>(s->ws + s->lay.lam_j);
  a.lam_s = reinterpret_cast<float*>(s->ws + s->lay.lam_s);
  a.pair_dropped = reinterpret_cast<int32_t*>(s->ws + s->lay.flag) + 1;
  a.place_env = s->regrouped ? reinterpret_cast<const int32_t*>(s->ws + s->lay.place_env) : nullptr;
#ifdef SIM_PHASE_TIMING
  a.dbg = reinterpret_cast<long long*>(s->ws + s->lay.flag) + 1;
#else
  a.dbg = nullptr;
#endif
  LdsPlan P = plan_for(m, s->E);
  size_t lds_bytes = (size_t)P.total * sizeof(float);
  if (lds_bytes > 160 * 1024) return fail(SIM_ERR_ARG, "envs_per_block %d needs %zu bytes of LDS (limit 160 KiB)", s->E, lds_bytes);
  int grid = (s->N + s->E - 1) / s->E;
  const int threads = threads_for(m, s->E);
  auto launch = [&](auto kern) -> int {
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), lds_bytes, st, a);
    return SIM_OK;
  };
  const bool few = m.max_joint_sides <= 4;
  if (m.solver == 1 && !newton_fits(m, s->E))
    return fail(SIM_ERR_ARG, "this robot does not fit the Newton solver's workgroup (a contact thread per slot)");
  int lrc = (m.solver == 1 && m.warm > 0.0f) ? ((s->E == 8 && few) ? launch(&step_kernel<8, 4, 0, kThreads, 1, 1>)
                             : few ? launch(&step_kernel<0, 4, 0, kThreads, 1, 1>) : launch(&step_kernel<0, kMaxBodyJoints, 0, kThreads, 1, 1>))
            : m.solver == 1 ? ((s->E == 8 && few) ? launch(&step_kernel<8, 4, 0, kThreads, 0, 1>)
                             : few ? launch(&step_kernel<0, 4, 0, kThreads, 0, 1>) : launch(&step_kernel<0, kMaxBodyJoints, 0, kThreads, 0, 1>))
            : (m.warm > 0.0f && pairs) ? ((s->E == 16 && few) ? launch(&step_kernel<16, 4, 1, kThreads, 1>)
                             : (s->E == 8 && few) ? launch(&step_kernel<8, 4, 1, kThreads, 1>)
                             : few ? launch(&step_kernel<0, 4, 1, kThreads, 1>) : launch(&step_kernel<0, kMaxBodyJoints, 1, kThreads, 1>))
            : m.warm > 0.0f ? ((s->E == 16 && few) ? launch(&step_kernel<16, 4, 0, kThreads, 1>)
                             : few ? launch(&step_kernel<0, 4, 0, kThreads, 1>) : launch(&step_kernel<0, kMaxBodyJoints, 0, kThreads, 1>))
            : pairs ? ((s->E == 16 && few) ? launch(&step_kernel<16, 4, 1>)
                     : (s->E == 8 && few) ? launch(&step_kernel<8, 4, 1>)
                     : few ? launch(&step_kernel<0, 4, 1>) : launch(&step_kernel<0, kMaxBodyJoints, 1>))
            : threads == kThreadsWide ? launch(&step_kernel<16, 4, 0, kThreadsWide>)
            : (s->E == 8 && few) ? launch(&step_kernel<8, 4>)
            : (s->E == 4 && few) ? launch(&step_kernel<4, 4>)
            : (s->E == 2 && few) ? launch(&step_kernel<2, 4>)
            : (s->E == 1 && few) ? launch(&step_kernel<1, 4>)
            : few ? launch(&step_kernel<0, 4>) : launch(&step_kernel<0, kMaxBodyJoints>);
  if (lrc) return lrc;
  HIP_TRY(hipGetLastError());
  if (a.recs) s->recs_valid = 1;
  if (a.pair_recs) s->pair_grid = grid;
  s->ws_has[0] = obs_out == nullptr; s->ws_has[1] = reward_out == nullptr; s->ws_has[2] = done_out == nullptr;
  return SIM_OK;
}

static inline int blocks_for(size_t n, int t = 256) { return (int)((n + t - 1) / t); }

// -------------------------------------------------------------------- ABI
extern "C" int sim_default_params(sim_desc_t* d) {
  if (!d) return fail(SIM_ERR_ARG, "desc is NULL");
  memset(d, 0, sizeof *d);
  d->max_episode_steps = 1000;
  d->gravity[2] = -9.81;
  d->mu = 1.0; d->contact_margin = 0.02; d->beta_joint = 0.2; d->beta_contact = 0.2; d->max_depen_vel = 2.0;
  d->max_ang_vel = 64.0; d->reset_noise = 0.05; d->gyroscopic = 1; d->contacts = 1;
  d->group_size = 1; d->krylov_iterations = 8; d->newton_reg = 0.1;
  return SIM_OK;
}

extern "C" int sim_builtin_robot(int32_t robot_kind, sim_desc_t* d) {
  if (!d) return fail(SIM_ERR_ARG, "desc is NULL");
  const BuiltinRobot* r = builtin_robot(robot_kind);
  if (!r) return fail(SIM_ERR_ARG, "robot_kind %d: 1 = ant, 2 = humanoid", robot_kind);
  d->n_bodies = r->n_bodies; d->n_joints = r->n_joints;
  d->bodies = r->bodies; d->joints = r->joints;
  d->root_body = r->root; d->n_feet = r->n_feet;
  for (int k = 0; k < SIM_MAX_FEET; ++k) d->foot_bodies[k] = k < r->n_feet ? r->feet[k] : 0;
  d->term_height = r->term_height; d->alive_bonus = r->alive_bonus;
  return SIM_OK;
}

extern "C" int sim_workspace_bytes(const sim_desc_t* desc, int num_envs, size_t* out_bytes) {
  Model m;
  int rc = build_model(desc, num_envs, &m);
  if (rc) return rc;
  if (!out_bytes) return fail(SIM_ERR_ARG, "out_bytes is NULL");
  size_t nh = desc->terrain_kind == 1 ? (size_t)desc->hf_nx * desc->hf_ny : 0;
  *out_bytes = make_layout(m.B, m.J, m.S, 11 + 3 * m.D + m.F + (m.height_map ? kHmRows * kHmCols : 0), num_envs, nh, (size_t)m.cnx * m.cny, pairs_of(m), m.warm > 0.0f).total;
  return SIM_OK;
}

// sim_create and sim_create_static: the workspace is caller memory (static_dev < 0) or the
// static array of device static_dev, whose address the caller of this function passes in.
static int create_in(const sim_desc_t* desc, int num_envs, void* workspace_dev, size_t workspace_bytes, int static_dev,
                     sim_t** out) {
  *out = nullptr;
  sim* s = new (std::nothrow) sim;
  if (!s) return fail(SIM_ERR_ARG, "out of host memory");
  s->static_dev = static_dev;
  int rc = build_model(desc, num_envs, &s->host_model);
  if (rc) { delete s; return rc; }
  const Model& m = s->host_model;
  size_t nh = desc->terrain_kind == 1 ? (size_t)desc->hf_nx * desc->hf_ny : 0;
  s->N = num_envs;
  s->obs_dim = 11 + 3 * m.D + m.F + (m.height_map ? kHmRows * kHmCols : 0);
  s->lay = make_layout(m.B, m.J, m.S, s->obs_dim, num_envs, nh, (size_t)m.cnx * m.cny, pairs_of(m), m.warm > 0.0f);
  s->record = 0; s->recs_valid = 0; s->pair_grid = 0; s->regrouped = 0;
  memset(&s->task, 0, sizeof(s->task));
  s->E = default_envs_per_block(m, num_envs);
  if (!workspace_dev || ((uintptr_t)workspace_dev & 255)) { delete s; return fail(SIM_ERR_WORKSPACE, "workspace must be non-NULL and 256-byte aligned"); }
  if (workspace_bytes < s->lay.total) { delete s; return fail(SIM_ERR_WORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, s->lay.total); }
  s->ws = static_cast<char*>(workspace_dev);
  auto bail = [&](int code) { delete s; return code; };
#define HIP_TRY_S(expr)                                                                          \
  do {                                                                                           \
    hipError_t _e = (expr);                                                                      \
    if (_e != hipSuccess) return bail(fail(SIM_ERR_HIP, "%s: %s", #expr, hipGetErrorString(_e))); \
  } while (0)
  HIP_TRY_S(hipMemcpy(s->ws + s->lay.model, &s->host_model, sizeof(Model), hipMemcpyHostToDevice));
  if (nh) {
    HIP_TRY_S(hipMemcpy(s->ws + s->lay.heights, desc->hf_heights, nh * sizeof(float), hipMemcpyHostToDevice));
    // coarse grid of block maxima: lets a slot that is clear of the terrain skip the fine search
    std::vector<float> coarse((size_t)m.cnx * m.cny);
    for (int J = 0; J < m.cny; ++J)
      for (int I = 0; I < m.cnx; ++I) {
        float hm = -INFINITY;
        for (int j = J * kCoarse; j <= J * kCoarse + kCoarse && j < m.ny; ++j)
          for (int i = I * kCoarse; i <= I * kCoarse + kCoarse && i < m.nx; ++i) {
            float hv = desc->hf_heights[(size_t)j * m.nx + i];
            hm = hv > hm ? hv : hm;
          }
        coarse[(size_t)J * m.cnx + I] = hm;
      }
    HIP_TRY_S(hipMemcpy(s->ws + s->lay.coarse, coarse.data(), coarse.size() * sizeof(float), hipMemcpyHostToDevice));
  }
  {
    std::vector<float> org((size_t)num_envs * 3), tgt((size_t)num_envs * 2);
    for (size_t i = 0; i < org.size(); ++i) org[i] = (float)desc->env_origins[i];
    for (int e = 0; e < num_envs; ++e) { tgt[2 * e] = 1000.0f; tgt[2 * e + 1] = 0.0f; }
    HIP_TRY_S(hipMemcpy(s->ws + s->lay.origins, org.data(), org.size() * sizeof(float), hipMemcpyHostToDevice));
    HIP_TRY_S(hipMemcpy(s->ws + s->lay.targets, tgt.data(), tgt.size() * sizeof(float), hipMemcpyHostToDevice));
    std::vector<float> st((size_t)13 * m.B * num_envs, 0.0f);
    const size_t fs = (size_t)m.B * num_envs;
    for (int b = 0; b < m.B; ++b)
      for (int e = 0; e < num_envs; ++e) {
        for (int c = 0; c < 3; ++c) st[c * fs + (size_t)b * num_envs + e] = m.bodies[b].rest_pos[c];
        st[3 * fs + (size_t)b * num_envs + e] = 1.0f;
      }
    HIP_TRY_S(hipMemcpy(s->ws + s->lay.state, st.data(), st.size() * sizeof(float), hipMemcpyHostToDevice));
    HIP_TRY_S(hipMemset(s->ws + s->lay.steps, 0, (size_t)num_envs * sizeof(int32_t)));
    HIP_TRY_S(hipMemset(s->ws + s->lay.recs, 0, (size_t)num_envs * m.S * sizeof(sim_contact_rec_t)));
    HIP_TRY_S(hipMemset(s->ws + s->lay.flag, 0, 256));
    HIP_TRY_S(hipMemset(s->ws + s->lay.task_i, 0, (size_t)num_envs * 4 * sizeof(int32_t)));
    HIP_TRY_S(hipMemset(s->ws + s->lay.push, 0, (size_t)num_envs * 3 * sizeof(float)));
    if (m.warm > 0.0f) {
      HIP_TRY_S(hipMemset(s->ws + s->lay.lam_j, 0, (size_t)num_envs * m.J * 6 * sizeof(float)));
      HIP_TRY_S(hipMemset(s->ws + s->lay.lam_s, 0, (size_t)num_envs * m.S * 3 * sizeof(float)));
    }
  }
  rc = launch_step(s, nullptr, 1.0f, 0, 0, 0, nullptr);
  if (rc) return bail(rc);
  HIP_TRY_S(hipDeviceSynchronize());
#undef HIP_TRY_S
  *out = s;
  return SIM_OK;
}

extern "C" int sim_create(const sim_desc_t* desc, int num_envs, void* workspace_dev, size_t workspace_bytes,
                          sim_t** out) {
  if (!out) return fail(SIM_ERR_ARG, "out is NULL");
  return create_in(desc, num_envs, workspace_dev, workspace_bytes, -1, out);
}

extern "C" int sim_create_static(const sim_desc_t* desc, int num_envs, sim_t** out) {
  if (!out) return fail(SIM_ERR_ARG, "out is NULL");
  *out = nullptr;
  size_t need = 0;
  int rc = sim_workspace_bytes(desc, num_envs, &need);
  if (rc) return rc;
  if (need > (size_t)SIM_STATIC_WORKSPACE_BYTES)
    return fail(SIM_ERR_WORKSPACE, "this description needs %zu bytes of workspace, the static workspace holds %zu",
                need, (size_t)SIM_STATIC_WORKSPACE_BYTES);
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(SIM_ERR_ARG, "device index %d outside 0..%d", dev, kMaxDevices - 1);
  if (!g_scratch_ptr[dev]) {
    // once per device, with that device current: the array's address on this GPU
    unsigned char* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255)) return fail(SIM_ERR_HIP, "static workspace has no usable device address");
    g_scratch_ptr[dev] = p;
  }
  if (g_scratch_owner[dev])
    return fail(SIM_ERR_WORKSPACE, "the static workspace of device %d is in use by another sim (destroy it first)", dev);
  rc = create_in(desc, num_envs, g_scratch_ptr[dev], (size_t)SIM_STATIC_WORKSPACE_BYTES, dev, out);
  if (rc) return rc;
  g_scratch_owner[dev] = *out;
  return SIM_OK;
}

extern "C" int sim_destroy(sim_t* s) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  if (s->static_dev >= 0 && g_scratch_owner[s->static_dev] == s) g_scratch_owner[s->static_dev] = nullptr;
  delete s;
  return SIM_OK;
}

extern "C" int sim_num_envs(const sim_t* s) { return s ? s->N : fail(SIM_ERR_ARG, "sim is NULL"); }
extern "C" int sim_num_bodies(const sim_t* s) { return s ? s->host_model.B : fail(SIM_ERR_ARG, "sim is NULL"); }
extern "C" int sim_num_slots(const sim_t* s) { return s ? s->host_model.S : fail(SIM_ERR_ARG, "sim is NULL"); }
extern "C" int sim_obs_dim(const sim_t* s) { return s ? s->obs_dim : fail(SIM_ERR_ARG, "sim is NULL"); }
extern "C" int sim_act_dim(const sim_t* s) { return s ? s->host_model.D : fail(SIM_ERR_ARG, "sim is NULL"); }

extern "C" int sim_launch_info(const sim_t* s, int32_t* threads_per_block, int32_t* envs_per_block, size_t* lds_bytes) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  const Model& m = s->host_model;
  if (threads_per_block) *threads_per_block = threads_for(m, s->E);
  if (envs_per_block) *envs_per_block = s->E;
  if (lds_bytes) *lds_bytes = (size_t)plan_for(m, s->E).total * sizeof(float);
  return SIM_OK;
}

extern "C" int sim_set_envs_per_block(sim_t* s, int E) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  const Model& m = s->host_model;
  if (E == 0) { s->E = default_envs_per_block(m, s->N); return SIM_OK; }
  if (E < 1 || E * m.B > kThreads || 2 * E * m.J > kThreads - 64)
    return fail(SIM_ERR_ARG, "envs_per_block %d does not fit %d threads (need E*B <= %d and 2*E*J <= %d)", E, kThreads,
                kThreads, kThreads - 64);
  if (m.group > 1 && E % m.group) return fail(SIM_ERR_ARG, "envs_per_block %d is not a multiple of the group size %d", E, m.group);
  if (m.solver == 1 && !newton_fits(m, E))
    return fail(SIM_ERR_ARG, "envs_per_block %d: the Newton solver needs a contact thread per slot (at most 8 envs per workgroup)", E);
  LdsPlan P = plan_for(m, E);
  if ((size_t)P.total * 4 > 160 * 1024) return fail(SIM_ERR_ARG, "envs_per_block %d exceeds LDS", E);
  s->E = E;
  return SIM_OK;
}

static int clear_kept(sim* s, const uint8_t* mask, hipStream_t st) {
  const Model& m = s->host_model;
  if (!(m.warm > 0.0f)) return SIM_OK;
  if (m.J > 0) hipLaunchKernelGGL(clear_kept_kernel, dim3(blocks_for((size_t)m.J * 6 * s->N)), dim3(256), 0, st,
                                  reinterpret_cast<float*>(s->ws + s->lay.lam_j), mask, m.J * 6, s->N);
  if (m.S > 0) hipLaunchKernelGGL(clear_kept_kernel, dim3(blocks_for((size_t)m.S * 3 * s->N)), dim3(256), 0, st,
                                  reinterpret_cast<float*>(s->ws + s->lay.lam_s), mask, m.S * 3, s->N);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_get_kept_impulses(sim_t* s, float* joint_rows_dev, float* slot_rows_dev, void* stream) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  const Model& m = s->host_model;
  if (!(m.warm > 0.0f)) return fail(SIM_ERR_ARG, "the sim was created without warm_start");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const Model* dm = reinterpret_cast<const Model*>(s->ws + s->lay.model);
  if (joint_rows_dev && m.J > 0)
    hipLaunchKernelGGL(get_kept_kernel, dim3(blocks_for((size_t)m.J * 6 * s->N)), dim3(256), 0, st,
                       reinterpret_cast<const float*>(s->ws + s->lay.lam_j), joint_rows_dev, m.J * 6, s->N, dm, 1);
  if (slot_rows_dev && m.S > 0)
    hipLaunchKernelGGL(get_kept_kernel, dim3(blocks_for((size_t)m.S * 3 * s->N)), dim3(256), 0, st,
                       reinterpret_cast<const float*>(s->ws + s->lay.lam_s), slot_rows_dev, m.S * 3, s->N, dm, 0);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_reset(sim_t* s, const uint8_t* env_mask_dev, uint64_t seed, void* stream) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(reset_kernel, dim3(blocks_for(s->N, 64)), dim3(64), 0, st,
                     reinterpret_cast<const Model*>(s->ws + s->lay.model),
                     reinterpret_cast<float*>(s->ws + s->lay.state),
                     reinterpret_cast<int32_t*>(s->ws + s->lay.steps), env_mask_dev, seed, s->N);
  HIP_TRY(hipGetLastError());
  int rc = clear_kept(s, env_mask_dev, st);
  if (rc) return rc;
  s->recs_valid = 0;
  return launch_step(s, nullptr, 1.0f, 0, 0, 0, st);
}

// One env-step is one launch of the fused kernel (with the task logic's auto-reset, the envs
// whose episode ended are reset and their observation re-packed at the end of that launch).
static int step_common(sim* s, const float* actions_dev, float dt, int substeps, int iterations, float* obs_dev,
                       float* reward_dev, uint8_t* done_dev, hipStream_t st) {
  if (!(dt > 0.0f) || !std::isfinite(dt)) return fail(SIM_ERR_ARG, "dt must be finite and > 0");
  if (substeps < 1) return fail(SIM_ERR_ARG, "substeps must be >= 1 (got %d)", substeps);
  if (iterations < 0) return fail(SIM_ERR_ARG, "iterations must be >= 0 (got %d)", iterations);
  return launch_step(s, actions_dev, dt / (float)substeps, substeps, iterations, 1, st, obs_dev, reward_dev, done_dev);
}

extern "C" int sim_step(sim_t* s, const float* actions_dev, float dt, int substeps, int iterations, void* stream) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  return step_common(s, actions_dev, dt, substeps, iterations, nullptr, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

extern "C" int sim_set_task(sim_t* s, const sim_task_desc_t* t, void* stream) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  memset(&s->task, 0, sizeof(s->task));
  if (!t || !t->enabled) return SIM_OK;
  if (t->fall_grace_frames < 0 || t->target_period < 0) return fail(SIM_ERR_ARG, "task: negative frame count");
  if (t->push_max_frames > 0 && (t->push_min_frames < 1 || t->push_min_frames > t->push_max_frames))
    return fail(SIM_ERR_ARG, "task: need 1 <= push_min_frames <= push_max_frames");
  if (!(t->target_radius >= 0) || !(t->target_reach >= 0) || !(t->push_min_newton <= t->push_max_newton))
    return fail(SIM_ERR_ARG, "task: radius/reach must be >= 0 and push_min_newton <= push_max_newton");
  TaskParams& p = s->task;
  p.enabled = 1; p.grace = t->fall_grace_frames; p.period = t->target_period;
  p.push_min_f = t->push_min_frames; p.push_max_f = t->push_max_frames; p.auto_reset = t->auto_reset ? 1 : 0;
  p.reach = (float)t->target_reach; p.radius = (float)t->target_radius;
  p.push_min_n = (float)t->push_min_newton; p.push_max_n = (float)t->push_max_newton; p.seed = t->seed;
  hipLaunchKernelGGL(task_init_kernel, dim3(blocks_for(s->N, 64)), dim3(64), 0, static_cast<hipStream_t>(stream),
                     reinterpret_cast<const Model*>(s->ws + s->lay.model), reinterpret_cast<const float*>(s->ws + s->lay.state),
                     reinterpret_cast<int32_t*>(s->ws + s->lay.task_i), reinterpret_cast<float*>(s->ws + s->lay.targets),
                     reinterpret_cast<float*>(s->ws + s->lay.push), s->task, s->N);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_get_task_state(sim_t* s, int32_t* counters_dev, float* targets_dev, float* push_dev, void* stream) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (counters_dev) hipLaunchKernelGGL(copy_i32_kernel, dim3(blocks_for((size_t)s->N * 4)), dim3(256), 0, st,
                                       reinterpret_cast<const int32_t*>(s->ws + s->lay.task_i), counters_dev, s->N * 4);
  if (targets_dev) hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for((size_t)s->N * 2)), dim3(256), 0, st,
                                      reinterpret_cast<const float*>(s->ws + s->lay.targets), targets_dev, s->N * 2);
  if (push_dev) hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for((size_t)s->N * 3)), dim3(256), 0, st,
                                   reinterpret_cast<const float*>(s->ws + s->lay.push), push_dev, s->N * 3);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_set_task_state(sim_t* s, const int32_t* counters_dev, const float* targets_dev, void* stream) {
  if (!s || !counters_dev || !targets_dev) return fail(SIM_ERR_ARG, "sim, counters or targets is NULL");
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(copy_i32_kernel, dim3(blocks_for((size_t)s->N * 4)), dim3(256), 0, st, counters_dev,
                     reinterpret_cast<int32_t*>(s->ws + s->lay.task_i), s->N * 4);
  hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for((size_t)s->N * 2)), dim3(256), 0, st, targets_dev,
                     reinterpret_cast<float*>(s->ws + s->lay.targets), s->N * 2);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_step_obs(sim_t* s, const float* actions_dev, float dt, int substeps, int iterations,
                            float* obs_dev, float* reward_dev, uint8_t* done_dev, void* stream) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  return step_common(s, actions_dev, dt, substeps, iterations, obs_dev, reward_dev, done_dev, static_cast<hipStream_t>(stream));
}

extern "C" int sim_get_obs(sim_t* s, float* obs_dev, float* reward_dev, uint8_t* done_dev, void* stream) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  if ((obs_dev && !s->ws_has[0]) || (reward_dev && !s->ws_has[1]) || (done_dev && !s->ws_has[2]))
    return fail(SIM_ERR_ARG, "the last sim_step_obs delivered this output to the caller's own array; the library kept no copy");
  int n_obs = s->N * s->obs_dim;
  hipLaunchKernelGGL(copy_out_kernel, dim3(blocks_for(n_obs)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     reinterpret_cast<const float*>(s->ws + s->lay.obs),
                     reinterpret_cast<const float*>(s->ws + s->lay.reward),
                     reinterpret_cast<const uint8_t*>(s->ws + s->lay.done), obs_dev, reward_dev, done_dev, n_obs,
                     s->N);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_set_targets(sim_t* s, const float* target_xy_dev, void* stream) {
  if (!s || !target_xy_dev) return fail(SIM_ERR_ARG, "sim or targets is NULL");
  hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for((size_t)s->N * 2)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), target_xy_dev,
                     reinterpret_cast<float*>(s->ws + s->lay.targets), s->N * 2);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_get_state(sim_t* s, float* state_dev, void* stream) {
  if (!s || !state_dev) return fail(SIM_ERR_ARG, "sim or state is NULL");
  size_t n = (size_t)s->N * s->host_model.B * 13;
  hipLaunchKernelGGL(get_state_kernel, dim3(blocks_for(n)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     reinterpret_cast<const float*>(s->ws + s->lay.state), state_dev, s->host_model.B, s->N);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_set_state(sim_t* s, const float* state_dev, void* stream) {
  if (!s || !state_dev) return fail(SIM_ERR_ARG, "sim or state is NULL");
  size_t n = (size_t)s->N * s->host_model.B * 13;
  hipLaunchKernelGGL(set_state_kernel, dim3(blocks_for(n)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     state_dev, reinterpret_cast<float*>(s->ws + s->lay.state), s->host_model.B, s->N);
  HIP_TRY(hipGetLastError());
  int rc = clear_kept(s, nullptr, static_cast<hipStream_t>(stream));
  if (rc) return rc;
  s->recs_valid = 0;
  return launch_step(s, nullptr, 1.0f, 0, 0, 0, static_cast<hipStream_t>(stream));
}

extern "C" int sim_set_step_count(sim_t* s, const int32_t* counts_dev, void* stream) {
  if (!s || !counts_dev) return fail(SIM_ERR_ARG, "sim or counts is NULL");
  hipLaunchKernelGGL(copy_i32_kernel, dim3(blocks_for(s->N)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     counts_dev, reinterpret_cast<int32_t*>(s->ws + s->lay.steps), s->N);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_record_contacts(sim_t* s, int enable) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  s->record = enable ? 1 : 0;
  if (!enable) s->recs_valid = 0;
  return SIM_OK;
}

extern "C" int sim_get_contacts(sim_t* s, sim_contact_rec_t* recs_dev, void* stream) {
  if (!s || !recs_dev) return fail(SIM_ERR_ARG, "sim or recs is NULL");
  if (!s->recs_valid) return fail(SIM_ERR_ARG, "no contact records: call sim_record_contacts(sim, 1) before sim_step");
  size_t n = (size_t)s->N * s->host_model.S * kRecWords;
  hipLaunchKernelGGL(copy_i32_kernel, dim3(blocks_for(n)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     reinterpret_cast<const int32_t*>(s->ws + s->lay.recs), reinterpret_cast<int32_t*>(recs_dev),
                     (int)n);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

// Packs the per-workgroup capsule-capsule records into one list (one block; workgroup order).
__global__ void gather_pair_recs_kernel(const int32_t* __restrict__ recs, const int32_t* __restrict__ count, int grid,
                                        const int32_t* __restrict__ dropped, int32_t* __restrict__ out, int cap,
                                        int32_t* __restrict__ out_count) {
  __shared__ int scan[1024];
  __shared__ int base;
  if (threadIdx.x == 0) base = 0;
  __syncthreads();
  for (int g0 = 0; g0 < grid; g0 += 1024) {
    const int g = g0 + threadIdx.x;
    const int c = g < grid ? count[g] : 0;
    scan[threadIdx.x] = c;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      const int v = threadIdx.x >= o ? scan[threadIdx.x - o] : 0;
      __syncthreads();
      scan[threadIdx.x] += v;
      __syncthreads();
    }
    const int first = base + scan[threadIdx.x] - c;
    for (int k = 0; k < c; ++k)
      if (first + k < cap)
        for (int w = 0; w < 8; ++w) out[(size_t)(first + k) * 8 + w] = recs[((size_t)g * kPairCap + k) * 8 + w];
    __syncthreads();
    if (threadIdx.x == 1023) base += scan[1023];
    __syncthreads();
  }
  if (threadIdx.x == 0) { out_count[0] = base; out_count[1] = dropped[0]; }
}

extern "C" int sim_get_pair_contacts(sim_t* s, sim_pair_contact_rec_t* recs_dev, int32_t cap, int32_t* count_dev, void* stream) {
  if (!s || !count_dev || (cap > 0 && !recs_dev)) return fail(SIM_ERR_ARG, "sim, recs or count is NULL");
  if (!pairs_of(s->host_model)) return fail(SIM_ERR_ARG, "the description has neither collide pairs nor interaction groups");
  if (!s->recs_valid || !s->pair_grid) return fail(SIM_ERR_ARG, "no contact records: call sim_record_contacts(sim, 1) before sim_step");
  hipLaunchKernelGGL(gather_pair_recs_kernel, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(stream),
                     reinterpret_cast<const int32_t*>(s->ws + s->lay.pair_recs),
                     reinterpret_cast<const int32_t*>(s->ws + s->lay.pair_count), s->pair_grid,
                     reinterpret_cast<const int32_t*>(s->ws + s->lay.flag) + 1, reinterpret_cast<int32_t*>(recs_dev),
                     cap < 0 ? 0 : cap, count_dev);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

// ---- interaction groups chosen from positions
static int need_groups(const sim* s) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  if (s->host_model.group <= 1) return fail(SIM_ERR_ARG, "the description has no interaction groups (group_size <= 1)");
  return SIM_OK;
}

extern "C" int sim_regroup(sim_t* s, float cell, float reach, void* stream) {
  if (int rc = need_groups(s)) return rc;
  if (!(cell > 0.0f) || !(cell <= 3.0e38f)) return fail(SIM_ERR_ARG, "cell must be positive and finite");
  if (!(reach >= 0.0f) || !(reach <= 1.0e18f)) return fail(SIM_ERR_ARG, "reach must be non-negative and finite");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const Model& m = s->host_model;
  auto* words = reinterpret_cast<unsigned long long*>(s->ws + s->lay.grp_words);
  hipLaunchKernelGGL(order_words_kernel, dim3(blocks_for(s->N)), dim3(256), 0, st,
                     reinterpret_cast<const float*>(s->ws + s->lay.state),
                     reinterpret_cast<const float*>(s->ws + s->lay.origins), m.B, s->N, m.root, cell, words);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(rank_places_kernel, dim3(blocks_for(s->N, 16)), dim3(256), 0, st, words, s->N,
                     reinterpret_cast<int32_t*>(s->ws + s->lay.place_env));
  HIP_TRY(hipGetLastError());
  const int W = (kWindow / m.group) * m.group;   // window of the second pass: whole groups, one workgroup
  hipLaunchKernelGGL(cluster_windows_kernel, dim3((s->N + W - 1) / W), dim3(kWindow), 0, st,
                     reinterpret_cast<const float*>(s->ws + s->lay.state),
                     reinterpret_cast<const float*>(s->ws + s->lay.origins), m.B, s->N, m.root, m.group, W, reach,
                     reinterpret_cast<int32_t*>(s->ws + s->lay.place_env));
  HIP_TRY(hipGetLastError());
  s->regrouped = 1;
  s->recs_valid = 0;
  return SIM_OK;
}

extern "C" int sim_set_groups(sim_t* s, const int32_t* place_env_dev, void* stream) {
  if (int rc = need_groups(s)) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  s->recs_valid = 0;
  if (!place_env_dev) { s->regrouped = 0; return SIM_OK; }
  // checked before it is taken over: a wrong entry would send a workgroup outside the arrays
  int32_t* seen = reinterpret_cast<int32_t*>(s->ws + s->lay.grp_words);
  int* flag = reinterpret_cast<int*>(s->ws + s->lay.grp_counts);
  int host_flag = 0;
  hipLaunchKernelGGL(fill_words_kernel, dim3(blocks_for(s->N)), dim3(256), 0, st, seen, (size_t)s->N, 0);
  hipLaunchKernelGGL(fill_words_kernel, dim3(1), dim3(64), 0, st, reinterpret_cast<int32_t*>(flag), (size_t)1, 0);
  hipLaunchKernelGGL(check_places_kernel, dim3(blocks_for(s->N)), dim3(256), 0, st, place_env_dev, s->N, seen, flag);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync(&host_flag, flag, sizeof(int), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  if (host_flag) return fail(SIM_ERR_ARG, "place_env is not a permutation of the agents 0 .. %d", s->N - 1);
  HIP_TRY(hipMemcpyAsync(s->ws + s->lay.place_env, place_env_dev, (size_t)s->N * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
  s->regrouped = 1;
  return SIM_OK;
}

extern "C" int sim_get_groups(sim_t* s, int32_t* place_env_dev, void* stream) {
  if (int rc = need_groups(s)) return rc;
  if (!place_env_dev) return fail(SIM_ERR_ARG, "place_env is NULL");
  hipStream_t st = static_cast<hipStream_t>(stream);
  // (through the inverse twice: one kernel covers both the stored order and the identity)
  int32_t* tmp = reinterpret_cast<int32_t*>(s->ws + s->lay.grp_words);
  const int32_t* pe = s->regrouped ? reinterpret_cast<const int32_t*>(s->ws + s->lay.place_env) : nullptr;
  hipLaunchKernelGGL(invert_places_kernel, dim3(blocks_for(s->N)), dim3(256), 0, st, pe, s->N, tmp);
  hipLaunchKernelGGL(invert_places_kernel, dim3(blocks_for(s->N)), dim3(256), 0, st, tmp, s->N, place_env_dev);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_count_near_pairs(sim_t* s, float reach, int64_t* counts_dev, void* stream) {
  if (int rc = need_groups(s)) return rc;
  if (!counts_dev) return fail(SIM_ERR_ARG, "counts is NULL");
  if (!(reach >= 0.0f) || !(reach <= 1.0e18f)) return fail(SIM_ERR_ARG, "reach must be non-negative and finite");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const Model& m = s->host_model;
  int32_t* place_of = reinterpret_cast<int32_t*>(s->ws + s->lay.grp_words);
  const int32_t* pe = s->regrouped ? reinterpret_cast<const int32_t*>(s->ws + s->lay.place_env) : nullptr;
  hipLaunchKernelGGL(invert_places_kernel, dim3(blocks_for(s->N)), dim3(256), 0, st, pe, s->N, place_of);
  hipLaunchKernelGGL(fill_words_kernel, dim3(1), dim3(64), 0, st, reinterpret_cast<int32_t*>(counts_dev), (size_t)4, 0);
  hipLaunchKernelGGL(near_pairs_kernel, dim3(blocks_for(s->N)), dim3(256), 0, st,
                     reinterpret_cast<const float*>(s->ws + s->lay.state),
                     reinterpret_cast<const float*>(s->ws + s->lay.origins), m.B, s->N, m.root, place_of, m.group, reach,
                     reinterpret_cast<unsigned long long*>(counts_dev));
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_generate_contacts(sim_t* s, sim_contact_rec_t* recs_dev, void* stream) {
  if (!s || !recs_dev) return fail(SIM_ERR_ARG, "sim or recs is NULL");
  size_t n = (size_t)s->N * s->host_model.S;
  hipLaunchKernelGGL(gen_contacts_kernel, dim3(blocks_for(n, 64)), dim3(64), 0, static_cast<hipStream_t>(stream),
                     reinterpret_cast<const Model*>(s->ws + s->lay.model),
                     reinterpret_cast<const float*>(s->ws + s->lay.heights),
                     reinterpret_cast<const float*>(s->ws + s->lay.coarse),
                     reinterpret_cast<const float*>(s->ws + s->lay.origins),
                     reinterpret_cast<const float*>(s->ws + s->lay.state), reinterpret_cast<int32_t*>(recs_dev),
                     s->N);
  HIP_TRY(hipGetLastError());
  return SIM_OK;
}

extern "C" int sim_check(sim_t* s, void* stream) {
  if (!s) return fail(SIM_ERR_ARG, "sim is NULL");
  hipStream_t st = static_cast<hipStream_t>(stream);
  int* flag = reinterpret_cast<int*>(s->ws + s->lay.flag);
  int n = s->N * s->host_model.B * 13;
  int zero = 0, host_flag = 0;
  HIP_TRY(hipMemcpyAsync(flag, &zero, sizeof(int), hipMemcpyHostToDevice, st));
  hipLaunchKernelGGL(check_kernel, dim3(blocks_for(n)), dim3(256), 0, st,
                     reinterpret_cast<const float*>(s->ws + s->lay.state), n, flag);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync(&host_flag, flag, sizeof(int), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  if (host_flag) return fail(SIM_ERR_NONFINITE, "non-finite value in the body state");
  return SIM_OK;
}
