// Fused env-step kernel: every substep of one sim_step plus obs/reward packing
// in a single launch.
//
// Mapping.  One workgroup owns E consecutive environments for the whole step.
// All LDS arrays are laid out [item][component][E] with the env index fastest,
// and every thread role uses e = tid % E, so the lanes of a wavefront that work
// on the same item of neighbouring envs touch consecutive LDS banks and
// consecutive global addresses of the [field][body][env] state arrays.
// Roles (a thread can hold several):
//   body thread  (e, b): owns pose and velocity of one body in registers,
//   joint-side threads  : two neighbouring lanes own the six rows of one joint, one lane per
//                         body (parent, child); a row's J v is the sum of the two lanes' parts,
//   contact thread      : owns the three rows of one active contact slot (constants in
//                         registers); a workgroup's contacts beyond one per thread are
//                         rebuilt from their LDS record every sweep,
//   pair-side threads   : (collision variant) two lanes per capsule-capsule contact,
//   env thread   (e)    : packs root observations, reward and done, applies the task rules.
// The joint-side threads fill the low wavefronts, the contact threads the high ones, so that a
// wavefront runs either the joint or the contact branch of a sweep.
//
// Per substep (Section 3.1 of the paper: maximal coordinates, torque control,
// speculative unilateral contacts, isotropic Coulomb friction, restitution 0):
//   A  body threads publish pose and world inverse inertia
//   B  contact generation per slot; joint threads turn actions into torques
//   C  body threads count their blocks, integrate gravity/torque/gyroscopic term
//   P  (collision variant) capsule-capsule contacts within an agent and within a group
//   D  joint / contact threads build row constants
//   S  (warm-start variant: sweep -1 applies the impulses kept from the last substep)
//      `iterations` sweeps: every block relaxes its rows one after another on a
//      private copy of its bodies taken from the shared snapshot; a body is
//      shared out among its blocks by weight (joint 1, contact a ramp from 0 at
//      the margin to 1 at half the margin) and acts inside block c with inverse
//      mass scaled by W / w_c; then every body takes the weighted average of the
//      copies of its blocks in static order (no atomics)
//   E  damping, angular-velocity cap, position integration
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "contact_gen.hpp"
#include "model.hpp"

namespace sim355 {

constexpr int kThreads = 512;       // threads per workgroup every shape fits (host-side limits)
constexpr int kThreadsWide = 768;   // the wider workgroup the big heightfield batches are run with
constexpr int kGroup = 8;  // lanes that share the fine terrain search of one slot
constexpr int kPatch = 28; // samples per side of the per-env heightfield copy kept in LDS
constexpr int kPatchBlocks = (kPatch + kMip - 1) / kMip;

struct StepArgs {
  const Model* M;
  const float* heights;
  const float* coarse;   // block maxima of the heightfield
  const float* origins;  // [N][3]
  float* targets;  // [N][2]
  float* state;          // [13][B][N]
  int32_t* steps;        // [N]
  const float* actions;  // [N][D] or null
  float* obs;            // [N][obs_dim]
  float* reward;         // [N]
  uint8_t* done;         // [N]
  int32_t* recs;         // [N][S][12] or null
  int N, E, substeps, iterations, count_step;
  float h;
  float* obs_out;        // caller arrays for obs / reward / done (sim_step_obs) that replace the library's, or null
  float* reward_out;
  uint8_t* done_out;
  TaskParams task;       // task logic (enabled = 0: off)
  int32_t* task_i;       // [N][4]: frames below the threshold, target age, frame of the next push, episode
  float* push;           // [N][3]: force on the root body during this step
  long long* dbg;        // phase-timing slots (diagnostic build only)
  float* lam_j;          // warm start: [J*6][N] joint row impulses at the end of the last substep
  float* lam_s;          //             [S*3][N] terrain slot impulses (0 for slots that were inactive)
  int32_t* pair_recs;    // [grid][kPairCap][8] capsule-capsule contacts of the last substep, or null
  int32_t* pair_count;   // [grid] their number per workgroup
  int32_t* pair_dropped; // [1] contacts dropped because a workgroup found more than kPairCap
  const int32_t* place_env;  // [N] agent standing at every place of the launch, or null: agent = place
};

// Rows (E consecutive floats) per item of the velocity, inverse-inertia and copy arrays.  Odd
// counts, so that neighbouring items start in different LDS banks when E is 16.
constexpr int kVS = 7, kCS = 7, kJS = 13;
constexpr int kPairHitMin = 256;   // (gap, key) words a workgroup keeps at least

struct LdsPlan {
  int pos, vel, iw, nb, tq, push, outj, outc, tjs, rec, list, surv, lam, u, obs, lim, count, patch, mip, porg, org, tslot, tbody, tin, tjoint, total;
  int pq, po, pnear, pbs, pcount, pbcnt, pblist;  // capsule-capsule contacts (only with pairs != 0)
  int phit, hit_cap;                              // their (gap, key) words: offset (64-bit aligned) and capacity
  int wj, wc;                                     // kept impulses of joints and slots (only with warm != 0)
  int nu, nred, nsum;                             // Newton solver: body vectors, reduction entries, partial sums
};

// pairs: 0 = no capsule-capsule contacts, else the interaction group size (1 = self-collision only)
__host__ __device__ inline LdsPlan make_plan(int B, int J, int S, int D, int F, int E, int with_patch, int pairs = 0,
                                             int threads = kThreads, int warm = 0, int newton = 0) {
  LdsPlan p;
  int o = 0;
  p.pos = o; o += B * 7 * E;
  p.vel = o; o += B * kVS * E;
  p.iw = o; o += B * kVS * E;
  p.nb = o; o += B * E;
  p.tq = o; o += J * 3 * E;
  p.push = o; o += 3 * E;
  o += o & 1;  // the search results kept in the copy arrays are 64-bit words
  p.outj = o; o += J * kJS * E;
  p.outc = o; o += S * kCS * E;
  p.rec = o; o += S * kRecWords * E;
  p.list = o; o += S * E;
  p.surv = o; o += S * E;
  p.lam = o;   // (with the warm start these impulses live in the per-slot array below)
  o += warm ? 0 : 3 * (S * E > threads - ((2 * J * E + 63) / 64) * 64 ? S * E - (threads - ((2 * J * E + 63) / 64) * 64) : 0);
  p.u = o; o += (D > 0 ? D : 1) * E;
  p.obs = o; o += (11 + 3 * D + F) * E;
  p.lim = o; o += (D > 0 ? D : 1) * E;
  p.count = o; o += 8;
  p.porg = o; o += 2 * E;
  p.org = o; o += 3 * E;
  p.tjs = o; o += B * (kMaxBodyJoints + 3);  // tjs .. tjoint: one block, copied from Model::table_image
  p.tslot = o; o += 2 * S;
  p.tbody = o; o += 4 * B;
  p.tin = o; o += 6 * B;
  p.tjoint = o; o += J * (int)(sizeof(JointTab) / 4);
  p.patch = o; o += with_patch ? E * kPatch * kPatch : 0;
  p.mip = o; o += with_patch ? E * kPatchBlocks * kPatchBlocks : 0;
  p.pq = o; o += pairs ? kPairCap * kPairWords : 0;   // sorted queue of the substep's contacts
  p.po = o; o += pairs ? (kPairCap + 1) * 12 : 0;     // weighted velocity copies of their two bodies; the last entry stays zero
  p.pnear = o; o += pairs ? (E * pairs) / 2 + 1 : 0;  // agent pairs whose bounding spheres overlap
  p.pbs = o; o += pairs ? E : 0;                      // bounding radius of every agent about its root
  p.pcount = o; o += pairs ? 4 : 0;
  p.pbcnt = o; o += pairs ? B * E : 0;                  // per body: how many of them touch it
  p.pblist = o; o += pairs ? (B * E * 6 + 3) / 4 : 0;  // per body: up to six of them, one byte each
  // one 64-bit (gap, key) word per capsule-capsule contact found, for the choice of those that stay
  // when a workgroup finds more than it holds: in the space of the terrain search's candidate list
  // (idle by then) where that holds kPairHitMin words, else in a region of their own
  p.hit_cap = ((J * kJS + S * kCS) * E - 5 * S * E - 2) / 2;
  p.phit = p.outj + ((5 * S * E + 1) & ~1);
  if (pairs && p.hit_cap < kPairHitMin) {
    o += o & 1;
    p.phit = o; o += 2 * kPairHitMin;
    p.hit_cap = kPairHitMin;
  }
  p.wj = o; o += warm ? J * 6 * E : 0;
  p.wc = o; o += warm ? S * 3 * E : 0;
  p.nu = o; o += newton ? B * kVS * E : 0;
  p.nred = o; o += newton ? 3 * (J + S) * E : 0;
  p.nsum = o; o += newton ? 3 * 8 * E : 0;
  p.total = o;
  return p;
}

__device__ __forceinline__ void quat_to_mat(const float q[4], float R[9]) {
  // R[3*r + c]: row r, column c; column c is the image of body axis c
  float w = q[0], x = q[1], y = q[2], z = q[3];
  R[0] = 1.0f - 2.0f * (y * y + z * z); R[1] = 2.0f * (x * y - w * z); R[2] = 2.0f * (x * z + w * y);
  R[3] = 2.0f * (x * y + w * z); R[4] = 1.0f - 2.0f * (x * x + z * z); R[5] = 2.0f * (y * z - w * x);
  R[6] = 2.0f * (x * z - w * y); R[7] = 2.0f * (y * z + w * x); R[8] = 1.0f - 2.0f * (x * x + y * y);
}
__device__ __forceinline__ void mat_vec(const float R[9], const float a[3], float o[3]) {
  o[0] = R[0] * a[0] + R[1] * a[1] + R[2] * a[2];
  o[1] = R[3] * a[0] + R[4] * a[1] + R[5] * a[2];
  o[2] = R[6] * a[0] + R[7] * a[1] + R[8] * a[2];
}
__device__ __forceinline__ void mat_t_vec(const float R[9], const float a[3], float o[3]) {
  o[0] = R[0] * a[0] + R[3] * a[1] + R[6] * a[2];
  o[1] = R[1] * a[0] + R[4] * a[1] + R[7] * a[2];
  o[2] = R[2] * a[0] + R[5] * a[1] + R[8] * a[2];
}
// symmetric 3x3 (xx,xy,xz,yy,yz,zz) times vector
__device__ __forceinline__ void sym_vec(const float S[6], const float a[3], float o[3]) {
  o[0] = S[0] * a[0] + S[1] * a[1] + S[2] * a[2];
  o[1] = S[1] * a[0] + S[3] * a[1] + S[4] * a[2];
  o[2] = S[2] * a[0] + S[4] * a[1] + S[5] * a[2];
}
__device__ __forceinline__ void cross(const float a[3], const float b[3], float o[3]) {
  o[0] = a[1] * b[2] - a[2] * b[1];
  o[1] = a[2] * b[0] - a[0] * b[2];
  o[2] = a[0] * b[1] - a[1] * b[0];
}
__device__ __forceinline__ float dot(const float a[3], const float b[3]) {
  return a[0] * b[0] + a[1] * b[1] + a[2] * b[2];
}
// (r x e_k) . w for the unit vector e_k, zero terms left out
__device__ __forceinline__ float cross_unit_dot(const float r[3], int k, const float w[3]) {
  return k == 0 ? r[2] * w[1] - r[1] * w[2] : (k == 1 ? r[0] * w[2] - r[2] * w[0] : r[1] * w[0] - r[0] * w[1]);
}
// r x e_k
__device__ __forceinline__ void cross_unit(const float r[3], int k, float o[3]) {
  if (k == 0) { o[0] = 0.0f; o[1] = r[2]; o[2] = -r[1]; }
  else if (k == 1) { o[0] = -r[2]; o[1] = 0.0f; o[2] = r[0]; }
  else { o[0] = r[1]; o[1] = -r[0]; o[2] = 0.0f; }
}
// rotation vector of conj(qa) * qb, short way round
// atan2(y, x) for y >= 0, x >= 0 (not both zero), to about 2 ulp: the argument is brought into
// [0, tan(pi/8)] by the identities atan(t) = pi/2 - atan(1/t) and atan(t) = pi/4 + atan((t-1)/(t+1)),
// where an odd polynomial of degree 9 does (the classic single-precision arctangent of the Cephes
// library; coefficients as published there).  Runs once per joint side and substep, on the path
// everybody waits for, where the general library routine and two correctly rounded divisions
// cost several times as much.
__device__ __forceinline__ float atan2_first_quadrant(float y, float x) {
  const bool big = y > 2.414213562373095f * x, mid = y > 0.4142135623730950f * x;
  // t = y / x, or -x / y, or (y - x) / (y + x)
  const float num = big ? -x : (mid ? y - x : y), den = big ? y : (mid ? y + x : x);
  const float t = num * __builtin_amdgcn_rcpf(den);
  const float base = big ? 1.5707963267948966f : (mid ? 0.7853981633974483f : 0.0f);
  const float z = t * t;
  const float p = (((8.05374449538e-2f * z - 1.38776856032e-1f) * z + 1.99777106478e-1f) * z - 3.33329491539e-1f) * z * t + t;
  return base + p;
}

__device__ __forceinline__ void rel_rotvec(const float qa[4], const float qb[4], float phi[3]) {
  float w = qa[0] * qb[0] + qa[1] * qb[1] + qa[2] * qb[2] + qa[3] * qb[3];
  float x = qa[0] * qb[1] - qa[1] * qb[0] - qa[2] * qb[3] + qa[3] * qb[2];
  float y = qa[0] * qb[2] + qa[1] * qb[3] - qa[2] * qb[0] - qa[3] * qb[1];
  float z = qa[0] * qb[3] - qa[1] * qb[2] + qa[2] * qb[1] - qa[3] * qb[0];
  if (w < 0.0f) { w = -w; x = -x; y = -y; z = -z; }
  const float s2 = x * x + y * y + z * z;
  const float inv_s = __builtin_amdgcn_rsqf(fmaxf(s2, 1e-30f)), s = s2 * inv_s;
  float k = (s < 1e-12f) ? 2.0f : 2.0f * atan2_first_quadrant(s, w) * inv_s;
  phi[0] = k * x; phi[1] = k * y; phi[2] = k * z;
}

// Height of the heightfield surface under a world xy (plane of the containing triangle).
__device__ inline float terrain_height(const Model& M, const float* __restrict__ hts, float wx, float wy) {
  if (M.terrain_kind == 0) return 0.0f;
  float ux = (wx - M.hox) / M.cell, uy = (wy - M.hoy) / M.cell;
  float fi = floorf(ux), fj = floorf(uy);
  float mi = (float)(M.nx - 2), mj = (float)(M.ny - 2);
  fi = fminf(fmaxf(fi, 0.0f), mi); fj = fminf(fmaxf(fj, 0.0f), mj);
  int i = (int)fi, j = (int)fj;
  float fx = fminf(fmaxf(ux - fi, 0.0f), 1.0f), fy = fminf(fmaxf(uy - fj, 0.0f), 1.0f);
  float h00 = hts[j * M.nx + i], h10 = hts[j * M.nx + i + 1];
  float h11 = hts[(j + 1) * M.nx + i + 1], h01 = hts[(j + 1) * M.nx + i];
  if (fx >= fy) return h00 + fx * (h10 - h00) + fy * (h11 - h10);
  return h00 + fx * (h11 - h01) + fy * (h01 - h00);
}

__device__ __forceinline__ void store_record(float* Lrec, int* Lreci, int s, int ee, int E, const ContactOut& co) {
  Lreci[(s * kRecWords + 0) * E + ee] = co.active;
  Lreci[(s * kRecWords + 1) * E + ee] = co.kind;
  Lreci[(s * kRecWords + 2) * E + ee] = co.feat;
  Lrec[(s * kRecWords + 3) * E + ee] = co.d;
  Lrec[(s * kRecWords + 4) * E + ee] = co.n.x;
  Lrec[(s * kRecWords + 5) * E + ee] = co.n.y;
  Lrec[(s * kRecWords + 6) * E + ee] = co.n.z;
  Lrec[(s * kRecWords + 7) * E + ee] = co.rc.x;
  Lrec[(s * kRecWords + 8) * E + ee] = co.rc.y;
  Lrec[(s * kRecWords + 9) * E + ee] = co.rc.z;
  Lrec[(s * kRecWords + 10) * E + ee] = co.w;
}

// Rows of one joint as seen from ONE of its two bodies (a joint is relaxed by a pair of
// neighbouring lanes, one per side; a row's J v is the sum of the two lanes' parts, exchanged
// with a DPP lane swap, and each lane then updates its own body's copy).  sg = -1 for the
// parent side, +1 for the child side; all signs are folded into the stored vectors.
struct SideRows {
  float sr[3];             // sg * lever arm from the own centre to the shared impulse point
  float sv;                // sg * n_o / m_o: own linear response per unit impulse
  float sg;
  float Y[3][3];           // own angular response per unit impulse of positional row k
  float pme[3], pnb[3];    // -m_eff and -m_eff * bias of the positional rows (world x, y, z)
  float sax[3][3];         // sg * joint axis k (sign of an upper limit folded in)
  float Z[3][3];           // own angular response per unit impulse of angular row k
  float ame[3], anb[3];
  float nl[3];             // lower bound of the next increment of angular row k: minus the impulse so
                           // far for a limit row (impulse >= 0), -infinity for a locked axis
  float lam[3];            // impulses of the angular rows so far (only the warm start keeps them)
  float pD[3], pb[3];      // (Newton solver) diagonal of J M^-1 J^T and bias of the positional rows
  float aD[3], ab[3];      //                 and of the angular rows
  int onesided;            // bit k set: angular row k is a limit row (impulse >= 0)
  int upper;               // bit k set: that limit row stands for the upper limit
};
// value of the neighbouring lane (lane ^ 1), one DPP move
__device__ __forceinline__ float lane_swap1(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true));
}

struct ContactRows {
  float dir[3][3];   // n, t1, t2
  float ang[3][3];   // rc x dir
  float Y[3][3];     // angular response
  float ls;          // linear response n_b / m
  float meff[3], bias, lam[3];
  float D[3];        // (Newton solver) diagonal of J M^-1 J^T
  int slot_e;        // slot * E + e
  int body;
};

// Phase timing (diagnostic build, -DSIM_PHASE_TIMING): thread 0 of workgroup 7 adds the cycles
// since the previous mark to slot k of a small buffer in the workspace.
// Each mark costs a few hundred cycles itself, so marks are kept out of the sweep loop.
#ifdef SIM_PHASE_TIMING
#define TMARK(k) do { if (tid == 0 && blockIdx.x == 7) { long long _t = clock64(); a.dbg[k] += _t - t_last; t_last = _t; } } while (0)
#else
#define TMARK(k) do { } while (0)
#endif

// Row constants of one active contact slot from its LDS record (d, n, rc, weight), the
// body's world inverse inertia, weight sum and inverse mass.
__device__ __forceinline__ void build_contact_rows(ContactRows& c, const float* Lrec, const float* Liw,
                                                   const float* Lnb, int s, int ee, int E, int body, float imb,
                                                   float h, float beta_c, float v_depen, bool whole_body = false) {
  c.body = body;
  c.slot_e = s * E + ee;
  float d = Lrec[(s * kRecWords + 3) * E + ee];
  float n[3], rc[3], iwb[6];
  for (int k = 0; k < 3; ++k) { n[k] = Lrec[(s * kRecWords + 4 + k) * E + ee]; rc[k] = Lrec[(s * kRecWords + 7 + k) * E + ee]; }
  for (int k = 0; k < 6; ++k) iwb[k] = Liw[(body * kVS + k) * E + ee];
  float nbb = Lnb[body * E + ee] / Lrec[(s * kRecWords + 10) * E + ee];
  if (whole_body) nbb = 1.0f;   // (the Newton solver does not split the body among its blocks)
  float t1[3], t2[3];
  if (fabsf(n[0]) < 0.57735f) { t1[0] = 0.0f; t1[1] = n[2]; t1[2] = -n[1]; }
  else { t1[0] = -n[2]; t1[1] = 0.0f; t1[2] = n[0]; }
  float inv = 1.0f / sqrtf(dot(t1, t1));
  for (int k = 0; k < 3; ++k) t1[k] *= inv;
  cross(n, t1, t2);
  for (int k = 0; k < 3; ++k) { c.dir[0][k] = n[k]; c.dir[1][k] = t1[k]; c.dir[2][k] = t2[k]; }
  c.ls = nbb * imb;
  for (int r = 0; r < 3; ++r) {
    float y[3];
    cross(rc, c.dir[r], c.ang[r]);
    sym_vec(iwb, c.ang[r], y);
    float keff = nbb * (imb + dot(c.ang[r], y));
    c.meff[r] = keff > 0.0f ? 1.0f / keff : 0.0f;
    c.D[r] = keff;
    for (int k = 0; k < 3; ++k) c.Y[r][k] = nbb * y[k];
    c.lam[r] = 0.0f;
  }
  c.bias = d >= 0.0f ? d / h : fmaxf(beta_c * d / h, -v_depen);
}

// Friction pair (l1, l2) brought back onto the disc of radius lim >= 0 (Section 3.1: isotropic
// Coulomb friction).  Runs in every sweep of every contact, so the test compares squares and the
// scale lim / |l| comes from the hardware's reciprocal square root (1 ulp) instead of a correctly
// rounded square root and division; the floor keeps a denormal |l|^2 from turning into infinity.
__device__ __forceinline__ void project_on_disc(float& l1, float& l2, float lim) {
  const float n2 = l1 * l1 + l2 * l2;
  if (n2 > lim * lim) {
    const float sc = lim * __builtin_amdgcn_rsqf(fmaxf(n2, 1e-30f));
    l1 *= sc; l2 *= sc;
  }
}

// One sweep of a contact block on its private copy (vv, ww) of the body velocity:
// normal row (impulse >= 0), then the friction pair projected on the disc mu * lambda_n.
__device__ __forceinline__ void relax_contact(ContactRows& c, float mu, float vv[3], float ww[3]) {
  {
    float jv = dot(c.dir[0], vv) + dot(c.ang[0], ww);
    float dl = -c.meff[0] * (jv + c.bias);
    float ln = fmaxf(c.lam[0] + dl, 0.0f);
    dl = ln - c.lam[0];
    c.lam[0] = ln;
    for (int k = 0; k < 3; ++k) { vv[k] += c.ls * c.dir[0][k] * dl; ww[k] += c.Y[0][k] * dl; }
  }
  float jv1 = dot(c.dir[1], vv) + dot(c.ang[1], ww);
  float jv2 = dot(c.dir[2], vv) + dot(c.ang[2], ww);
  float l1 = c.lam[1] - c.meff[1] * jv1, l2 = c.lam[2] - c.meff[2] * jv2;
  const float lim = mu * c.lam[0];
  project_on_disc(l1, l2, lim);
  float d1 = l1 - c.lam[1], d2 = l2 - c.lam[2];
  c.lam[1] = l1; c.lam[2] = l2;
  for (int k = 0; k < 3; ++k) {
    vv[k] += c.ls * (c.dir[1][k] * d1 + c.dir[2][k] * d2);
    ww[k] += c.Y[1][k] * d1 + c.Y[2][k] * d2;
  }
}

// Warm start: the block's copy of its body after the impulses the rows start from.
__device__ __forceinline__ void apply_contact_impulses(const ContactRows& c, float vv[3], float ww[3]) {
  for (int r = 0; r < 3; ++r)
    for (int k = 0; k < 3; ++k) { vv[k] += c.ls * c.dir[r][k] * c.lam[r]; ww[k] += c.Y[r][k] * c.lam[r]; }
}

// Rows of one capsule-capsule contact (Section 3.1: contacts among bodies; Section 4.1:
// inter-agent collisions) as seen from ONE of its two bodies: normal and two tangents between
// body A (+J) and body B (-J), one contact point for both (midway between the closest surface
// points, so the pair of opposite impulses carries no net torque).  Like a joint, a contact is
// relaxed by two neighbouring lanes, one per body; a row's J v is the sum of the two lanes'
// parts, both lanes compute the same impulse and each updates its own body's copy.  All signs
// (+1 for A, -1 for B) are folded into the stored vectors.
struct PairSide {
  float sd[3][3];    // sg * (n, t1, t2); n points from B to A
  float sa[3][3];    // sg * (lever arm x direction)
  float Y[3][3];     // own angular response per unit impulse
  float ls;          // own linear response per unit impulse along sd
  float meff[3], bias, lam[3];
  float wk;          // the block's weight: copies are published multiplied by it
  int off;           // own body's velocity rows in LDS: body * kVS * E + env
};

// Builds side `side` (0: body A, 1: body B) of queue entry k from the poses, the segment
// parameters (s, t) the contact search found, the body's world inverse inertia and weight sum.
// Both lanes evaluate the same geometry with the same operations.
__device__ __forceinline__ void build_pair_side(PairSide& c, int side, const float* Lpq, const float* Lpos,
                                                const float* Liw, const float* Lnb, const float* Lorg,
                                                const float* Ltbody, int k, int E, float h, float beta_c,
                                                float v_depen) {
  const int refs = __float_as_int(Lpq[k * kPairWords + 1]);
  const int ra = refs & 0xffff, rb = (refs >> 16) & 0xffff;
  const int ba = ra / E, ea = ra - ba * E, bb = rb / E, eb = rb - bb * E;
  const float sp = Lpq[k * kPairWords + 2], tp = Lpq[k * kPairWords + 3], wk = Lpq[k * kPairWords + 4];
  float xa[3], xb[3], qa[4], qb[4];
  for (int i = 0; i < 3; ++i) {
    xa[i] = Lpos[(ba * 7 + i) * E + ea];
    xb[i] = Lpos[(bb * 7 + i) * E + eb] + (Lorg[i * E + eb] - Lorg[i * E + ea]);   // in A's env frame
  }
  for (int i = 0; i < 4; ++i) { qa[i] = Lpos[(ba * 7 + 3 + i) * E + ea]; qb[i] = Lpos[(bb * 7 + 3 + i) * E + eb]; }
  const float radA = Ltbody[4 * ba], hlA = Ltbody[4 * ba + 1];
  const float radB = Ltbody[4 * bb], hlB = Ltbody[4 * bb + 1];
  const int axA = __float_as_int(Ltbody[4 * ba + 2]), axB = __float_as_int(Ltbody[4 * bb + 2]);
  float Ra[9], Rb[9], cp[3], cq[3], df[3];
  quat_to_mat(qa, Ra);
  quat_to_mat(qb, Rb);
  for (int i = 0; i < 3; ++i) {
    const float ha = Ra[3 * i + axA] * hlA, hb = Rb[3 * i + axB] * hlB;
    cp[i] = xa[i] - ha + 2.0f * sp * ha;
    cq[i] = xb[i] - hb + 2.0f * tp * hb;
    df[i] = cp[i] - cq[i];
  }
  const float dist = sqrtf(dot(df, df));
  float n[3] = {0.0f, 0.0f, 1.0f};
  if (dist >= 1e-9f) { const float inv = 1.0f / dist; for (int i = 0; i < 3; ++i) n[i] = df[i] * inv; }
  const float d = dist - radA - radB;
  // own body
  const int bo = side ? bb : ba, eo = side ? eb : ea;
  const float sg = side ? -1.0f : 1.0f;
  float arm[3], iwo[6];
  for (int i = 0; i < 3; ++i) {
    const float pm = 0.5f * ((cp[i] - n[i] * radA) + (cq[i] + n[i] * radB));
    arm[i] = pm - (side ? xb[i] : xa[i]);
  }
  for (int i = 0; i < 6; ++i) iwo[i] = Liw[(bo * kVS + i) * E + eo];
  const float imo = Ltbody[4 * bo + 3];
  const float nbo = Lnb[bo * E + eo] / wk;
  float t1[3], t2[3];
  if (fabsf(n[0]) < 0.57735f) { t1[0] = 0.0f; t1[1] = n[2]; t1[2] = -n[1]; }
  else { t1[0] = -n[2]; t1[1] = 0.0f; t1[2] = n[0]; }
  const float inv = 1.0f / sqrtf(dot(t1, t1));
  for (int i = 0; i < 3; ++i) t1[i] *= inv;
  cross(n, t1, t2);
  for (int i = 0; i < 3; ++i) { c.sd[0][i] = sg * n[i]; c.sd[1][i] = sg * t1[i]; c.sd[2][i] = sg * t2[i]; }
  c.ls = nbo * imo;
  for (int r = 0; r < 3; ++r) {
    float y[3];
    cross(arm, c.sd[r], c.sa[r]);
    sym_vec(iwo, c.sa[r], y);
    const float kp = nbo * (imo + dot(c.sa[r], y));
    const float keff = kp + lane_swap1(kp);
    c.meff[r] = keff > 0.0f ? 1.0f / keff : 0.0f;
    for (int i = 0; i < 3; ++i) c.Y[r][i] = nbo * y[i];
    c.lam[r] = 0.0f;
  }
  c.bias = d >= 0.0f ? d / h : fmaxf(beta_c * d / h, -v_depen);
  c.wk = wk;
  c.off = bo * kVS * E + eo;
}

// One sweep of one side of a capsule-capsule block on its private copy of the own body's velocity.
__device__ __forceinline__ void relax_pair_side(PairSide& c, float mu, float v[3], float w[3]) {
  {
    const float part = dot(c.sd[0], v) + dot(c.sa[0], w);
    const float jv = part + lane_swap1(part);
    float dl = -c.meff[0] * (jv + c.bias);
    const float ln = fmaxf(c.lam[0] + dl, 0.0f);
    dl = ln - c.lam[0];
    c.lam[0] = ln;
    for (int k = 0; k < 3; ++k) { v[k] += c.ls * c.sd[0][k] * dl; w[k] += c.Y[0][k] * dl; }
  }
  const float p1 = dot(c.sd[1], v) + dot(c.sa[1], w), p2 = dot(c.sd[2], v) + dot(c.sa[2], w);
  const float jv1 = p1 + lane_swap1(p1), jv2 = p2 + lane_swap1(p2);
  float l1 = c.lam[1] - c.meff[1] * jv1, l2 = c.lam[2] - c.meff[2] * jv2;
  const float lim = mu * c.lam[0];
  project_on_disc(l1, l2, lim);
  const float d1 = l1 - c.lam[1], d2 = l2 - c.lam[2];
  c.lam[1] = l1; c.lam[2] = l2;
  for (int k = 0; k < 3; ++k) {
    v[k] += c.ls * (c.sd[1][k] * d1 + c.sd[2][k] * d2);
    w[k] += c.Y[1][k] * d1 + c.Y[2][k] * d2;
  }
}

// EC > 0: envs per workgroup fixed at compile time (LDS offsets become immediates);
// EC == 0: taken from the launch arguments.  NJ: compile-time bound on the joints one body
// belongs to (the per-body average reads NJ joint copies without branching).
// counter-based uniform draw: one 64-bit mixing finaliser per (seed, env, index)
__device__ inline float reset_uniform(uint64_t seed, uint64_t env, uint64_t idx) {
  uint64_t z = seed + env * 0x632BE59BD9B4E019ULL + idx * 0xD1B54A32D192ED03ULL;
  z += 0x9E3779B97F4A7C15ULL;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  z ^= z >> 31;
  return (float)(z >> 40) * (1.0f / 16777216.0f);
}
// draws of the task logic, keyed by (seed, episode, env, frame, k): k = 0 push magnitude,
// 1 push direction, 2 frames to the next push, 3 target distance, 4 target direction
__device__ inline float task_u(const TaskParams& t, int env, int episode, int frame, int k) {
  return reset_uniform(t.seed + (uint64_t)episode * kEpisodeStride, (uint64_t)env, (uint64_t)(1024 + 8 * frame + k));
}
__device__ inline int task_interval(const TaskParams& t, int env, int episode, int frame) {
  const int span = t.push_max_f - t.push_min_f + 1;
  const int d = t.push_min_f + (int)floorf(task_u(t, env, episode, frame, 2) * (float)span);
  return d > t.push_max_f ? t.push_max_f : d;
}
__device__ inline void task_draw_target(const TaskParams& t, int env, int episode, int frame, float rx, float ry,
                                        float* target_xy) {
  const float r = t.radius * sqrtf(task_u(t, env, episode, frame, 3));
  const float phi = 6.283185307179586f * task_u(t, env, episode, frame, 4);
  target_xy[0] = rx + r * cosf(phi);
  target_xy[1] = ry + r * sinf(phi);
}

// Seeded reset (Section 4.1: positions, velocities, joint angles and joint angular velocities
// perturbed slightly): the rest pose displaced by a uniform offset, every hinge angle and every
// hinge rate drawn uniformly (angles clamped to their limits), bodies placed parents-first
// through the joint list; the top of the tree gets one uniform linear velocity and no spin, a
// child turns with its parent plus its hinge rates and moves so that the two anchor points of its
// joint share one velocity (the world as a parent stands still).
// `P` holds the state while it is built: P.X(b, c), P.Q(b, c), P.V(b, c), P.W(b, c) are
// references to component c of position, quaternion, linear and angular velocity of body b (local
// arrays for the stand-alone reset kernels, the env's columns of the pose and velocity arrays in
// LDS for the reset at the end of a step).
template <class Poses>
__device__ inline void reset_pose(const Model& M, int env, uint64_t seed, Poses& P) {
  const float a = M.reset_noise;
  float off[3], vel[3];
  for (int c = 0; c < 3; ++c) {
    off[c] = a * (2.0f * reset_uniform(seed, env, c) - 1.0f);
    vel[c] = a * (2.0f * reset_uniform(seed, env, 3 + c) - 1.0f);
  }
  for (int b = 0; b < M.B; ++b) {
    for (int c = 0; c < 3; ++c) P.X(b, c) = M.bodies[b].rest_pos[c] + off[c];
    P.Q(b, 0) = 1.0f; P.Q(b, 1) = 0.0f; P.Q(b, 2) = 0.0f; P.Q(b, 3) = 0.0f;
    for (int c = 0; c < 3; ++c) { P.V(b, c) = vel[c]; P.W(b, c) = 0.0f; }
  }
  for (int j = 0; j < M.J; ++j) {
    const JointTab& jt = M.joints[j];
    float phi[3] = {0, 0, 0};
    for (int k = 0; k < 3; ++k) {
      if (jt.mode[k] != 1) continue;
      float th = a * (2.0f * reset_uniform(seed, env, 8 + 3 * j + k) - 1.0f);
      th = fminf(fmaxf(th, jt.lo[k]), jt.hi[k]);
      for (int c = 0; c < 3; ++c) phi[c] += th * jt.axes[k][c];
    }
    float ang = sqrtf(dot(phi, phi));
    float dq[4];
    if (ang < 1e-12f) { dq[0] = 1.0f; dq[1] = 0.5f * phi[0]; dq[2] = 0.5f * phi[1]; dq[3] = 0.5f * phi[2]; }
    else { float s = sinf(0.5f * ang) / ang; dq[0] = cosf(0.5f * ang); dq[1] = s * phi[0]; dq[2] = s * phi[1]; dq[3] = s * phi[2]; }
    float qa[4] = {1, 0, 0, 0}, xa[3] = {0, 0, 0}, va[3] = {0, 0, 0}, wa[3] = {0, 0, 0};
    if (jt.parent >= 0) {
      for (int c = 0; c < 4; ++c) qa[c] = P.Q(jt.parent, c);
      for (int c = 0; c < 3; ++c) { xa[c] = P.X(jt.parent, c); va[c] = P.V(jt.parent, c); wa[c] = P.W(jt.parent, c); }
    }
    float qb[4];
    qb[0] = qa[0] * dq[0] - qa[1] * dq[1] - qa[2] * dq[2] - qa[3] * dq[3];
    qb[1] = qa[0] * dq[1] + qa[1] * dq[0] + qa[2] * dq[3] - qa[3] * dq[2];
    qb[2] = qa[0] * dq[2] - qa[1] * dq[3] + qa[2] * dq[0] + qa[3] * dq[1];
    qb[3] = qa[0] * dq[3] + qa[1] * dq[2] - qa[2] * dq[1] + qa[3] * dq[0];
    float inv = 1.0f / sqrtf(qb[0] * qb[0] + qb[1] * qb[1] + qb[2] * qb[2] + qb[3] * qb[3]);
    for (int c = 0; c < 4; ++c) qb[c] *= inv;
    float Ra[9], Rb[9], t0[3], t1[3];
    quat_to_mat(qa, Ra);
    quat_to_mat(qb, Rb);
    mat_vec(Ra, jt.la, t0);
    mat_vec(Rb, jt.lb, t1);
    for (int c = 0; c < 4; ++c) P.Q(jt.child, c) = qb[c];
    for (int c = 0; c < 3; ++c) P.X(jt.child, c) = xa[c] + t0[c] - t1[c];
    float wb[3] = {wa[0], wa[1], wa[2]};
    for (int k = 0; k < 3; ++k) {
      if (jt.mode[k] != 1) continue;
      const float rate = a * (2.0f * reset_uniform(seed, env, 256 + 3 * j + k) - 1.0f);
      float ak[3];
      mat_vec(Ra, jt.axes[k], ak);
      for (int c = 0; c < 3; ++c) wb[c] += rate * ak[c];
    }
    float ca[3], cb[3];
    cross(wa, t0, ca);
    cross(wb, t1, cb);
    for (int c = 0; c < 3; ++c) { P.W(jt.child, c) = wb[c]; P.V(jt.child, c) = va[c] + ca[c] - cb[c]; }
  }
}
// Start of an episode for the task logic (Section 4.1): counters cleared, first push time and
// (flagrun) first target drawn around the root.
__device__ inline void task_begin_episode(const TaskParams& t, int32_t* __restrict__ task_i, float* __restrict__ targets,
                                          int env, int episode, float rx, float ry) {
  task_i[4 * env + 0] = 0; task_i[4 * env + 1] = 0;
  task_i[4 * env + 2] = t.push_max_f > 0 ? task_interval(t, env, episode, 0) : -1;
  task_i[4 * env + 3] = episode;
  if (t.period > 0) task_draw_target(t, env, episode, 0, rx, ry, targets + 2 * env);
}
// the env's column of the pose array in LDS ([body][7][E]) as the place reset_pose builds in
struct LdsPoses {
  float* Lpos; float* Lvel; int E, ee;
  __device__ float& X(int b, int c) { return Lpos[(b * 7 + c) * E + ee]; }
  __device__ float& Q(int b, int c) { return Lpos[(b * 7 + 3 + c) * E + ee]; }
  __device__ float& V(int b, int c) { return Lvel[(b * kVS + c) * E + ee]; }
  __device__ float& W(int b, int c) { return Lvel[(b * kVS + 3 + c) * E + ee]; }
};

// (squared distance, feature id) as one 64-bit word whose unsigned order is the lexicographic
// order of the pair (squared distances are non-negative, ids non-negative)
__device__ __forceinline__ unsigned long long pack_best(float d2, int id) {
  return ((unsigned long long)__float_as_uint(d2) << 32) | (unsigned)id;
}

// Number of set bits of a 64-bit lane mask below the calling lane.
__device__ __forceinline__ int lanes_below(unsigned long long m) {
  return (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
}
// Reserves n (0 .. 2^kBits - 1) consecutive entries of a list for each active lane with one
// atomic per wavefront; every active lane has to call it.  Returns the lane's first index.
template <int kBits>
__device__ __forceinline__ int wave_alloc(int n, int* counter) {
  int before = 0, total = 0;
#pragma unroll
  for (int bit = 0; bit < kBits; ++bit) {
    const unsigned long long bm = __ballot((n >> bit) & 1);
    before += lanes_below(bm) << bit;
    total += __popcll(bm) << bit;
  }
  int base = 0;
  if (total > 0) {
    if (lanes_below(__ballot(1)) == 0) base = atomicAdd(counter, total);
    base = __builtin_amdgcn_readfirstlane(base);
  }
  return base + before;
}

// PC != 0: capsule-capsule contacts (within an agent and between the agents of a group) compiled in.
// NT: threads per workgroup.
// NS != 0: the rows are solved by the non-smooth Newton / conjugate-residual solver instead of
// the Jacobi sweeps (at most 8 envs per workgroup, every slot has a contact thread of its own).
template <int EC, int NJ, int PC = 0, int NT = kThreads, int WS = 0, int NS = 0>
__global__ __launch_bounds__(NT) void step_kernel(StepArgs a) {
  constexpr int kThreads = NT;   // (shadows the namespace-scope default inside the kernel)
#ifdef SIM_PHASE_TIMING
  long long t_last = clock64();
#endif
  extern __shared__ float lds[];
  const Model& M = *a.M;
  const int B = M.B, J = M.J, S = M.S, D = M.D, F = M.F;
  const int E = EC > 0 ? EC : a.E, N = a.N;
  const int tid = threadIdx.x;
  const int e = tid % E, idx = tid / E;
  const int env = blockIdx.x * E + e;   // the thread's place in the launch: a workgroup holds E consecutive places
  const bool env_ok = env < N;
  // Which agent stands at a place: the agent of the same number, unless the interaction groups were
  // chosen from the agents' positions (capsule-capsule variants only).  Everything in global memory
  // is indexed by agent, everything in LDS by the place within the workgroup.
  auto agent_at = [&](int place) -> int {
    if constexpr (PC != 0) { if (a.place_env && place < N) return a.place_env[place]; }
    return place;
  };
  const int agent = agent_at(env);
  const bool is_body = idx < B && env_ok;
  const bool is_joint = idx < J && env_ok;
  const int obs_dim = 11 + 3 * D + F;                                      // staged in LDS
  const int obs_row = obs_dim + (M.height_map ? kHmRows * kHmCols : 0);   // row of the caller's array
  // model scalars the loops below use, read once (before the kernel's first store, so they come
  // through the scalar cache and stay in scalar registers)
  const int m_terrain = M.terrain_kind, m_contacts = M.contacts;
  const Field H0 = make_field(M, a.heights, a.coarse);
  const bool use_patch = m_terrain == 1 && H0.nx >= kPatch && H0.ny >= kPatch;
  const int m_group = PC ? (M.group > 1 ? M.group : 1) : 1, m_npairs = PC ? M.n_pairs : 0, m_nap = PC ? M.n_agent_pairs : 0;
  const LdsPlan P = make_plan(B, J, S, D, F, E, use_patch ? 1 : 0, PC ? m_group : 0, NT, WS, NS);
  float* Lpos = lds + P.pos;
  float* Lvel = lds + P.vel;
  float* Liw = lds + P.iw;
  float* Lnb = lds + P.nb;
  float* Loutj = lds + P.outj;
  float* Loutc = lds + P.outc;
  int* Ltjs = reinterpret_cast<int*>(lds + P.tjs);  // body table: joint-side count, slot0, slot count, joint sides
  float* Lrec = lds + P.rec;
  int* Lreci = reinterpret_cast<int*>(lds + P.rec);
  int* Llist = reinterpret_cast<int*>(lds + P.list);
  int* Lsurv = reinterpret_cast<int*>(lds + P.surv);
  float* Llam = lds + P.lam;                         // impulses of the contacts beyond one per thread
  // fine search: per slot (index s * E + env) the minimum of (squared distance, feature id) packed in 64 bits,
  // then the list of candidate edges; both live in the space of the copies the sweeps use
  unsigned long long* Lbest64 = reinterpret_cast<unsigned long long*>(lds + P.outj);
  float* Lgeo = lds + P.outj + 2 * S * E;           // per slot: reach, and R L, 1/L^2 of a segment
  unsigned* Lcand = reinterpret_cast<unsigned*>(lds + P.outj) + 5 * S * E;
  const int cand_cap = (J * kJS + S * kCS) * E - 5 * S * E;
  // work units of the fine search (8 cells of one queued slot each): end spheres in the first
  // third of the list, mid-segments in the rest.  The space holds the observations at the end.
  unsigned* Lunit = reinterpret_cast<unsigned*>(lds + P.obs);
  const int unit_cap = (11 + 3 * D + F) * E, unit_cap_e = unit_cap / 3;
  float* Ltq = lds + P.tq;                           // joint torques, [J][3][E]
  float* Lpush = lds + P.push;                       // external force on the root body, [3][E]
  float* Lu = lds + P.u;
  float* Lobs = lds + P.obs;
  int* Llim = reinterpret_cast<int*>(lds + P.lim);
  int* Lcount = reinterpret_cast<int*>(lds + P.count);
  int* Lporg = reinterpret_cast<int*>(lds + P.porg);
  float* Lpatch = lds + P.patch;
  float* Lmip = lds + P.mip;
  float* Lorg = lds + P.org;                          // env origins, [3][E]
  int* Ltslot = reinterpret_cast<int*>(lds + P.tslot);  // slot table: body, kind
  float* Ltbody = lds + P.tbody;                      // body table: radius, half length, axis, 1/mass
  float* Ltin = lds + P.tin;                          // body table: inertia(3), inverse inertia(3)
  const JointTab* Ltjoint = reinterpret_cast<const JointTab*>(lds + P.tjoint);  // joint table
  float* Lpq = lds + P.pq;                            // capsule-capsule contacts, kPairWords each, sorted by key
  float* Lpo = lds + P.po;                            // their copies times the block weight: A (v, w), B (v, w)
  int* Lnear = reinterpret_cast<int*>(lds + P.pnear);
  int* Lbs = reinterpret_cast<int*>(lds + P.pbs);     // bounding radii as float bits (ordered like ints)
  int* Lpcount = reinterpret_cast<int*>(lds + P.pcount);  // contacts found, near agent pairs
  int* Lpbcnt = reinterpret_cast<int*>(lds + P.pbcnt);
  uint8_t* Lpblist = reinterpret_cast<uint8_t*>(lds + P.pblist);
  // Warm start (WS != 0): the impulse every joint row ([J*6][E]; a limit row's carries the limit it
  // stood for in its sign, minus = upper) and every terrain slot row ([S*3][E]) ended the last
  // substep with.  Slots that were not active then hold zero.
  float* Lwj = lds + P.wj;
  float* Lwc = lds + P.wc;
  const float p_warm = WS ? M.warm : 0.0f;
  const float h = a.h;

  // ---- load: body state into registers, clipped actions into LDS
  float x[3] = {0, 0, 0}, q[4] = {1, 0, 0, 0}, v[3] = {0, 0, 0}, w[3] = {0, 0, 0};
  int my_slot0 = 0, my_nslots = 0, my_njs = 0;
  float root_ox = 0.0f, root_oy = 0.0f;
  const int b = idx;
  if (is_body) {
    const float* st = a.state + (size_t)b * N + agent;
    const size_t fs = (size_t)B * N;
    x[0] = st[0 * fs]; x[1] = st[1 * fs]; x[2] = st[2 * fs];
    q[0] = st[3 * fs]; q[1] = st[4 * fs]; q[2] = st[5 * fs]; q[3] = st[6 * fs];
    v[0] = st[7 * fs]; v[1] = st[8 * fs]; v[2] = st[9 * fs];
    w[0] = st[10 * fs]; w[1] = st[11 * fs]; w[2] = st[12 * fs];
    const BodyTab& bt = M.bodies[b];
    my_slot0 = bt.slot0; my_nslots = bt.n_slots; my_njs = bt.n_joint_sides;
    if (b == M.root) { root_ox = a.origins[3 * agent]; root_oy = a.origins[3 * agent + 1]; }   // for the heightfield copy
  }
  // uniform parameters and this thread's joint, read once
  const float g0 = M.g[0], g1 = M.g[1], g2 = M.g[2];
  const float p_mu = M.mu, p_margin = M.margin, p_beta_j = M.beta_j, p_beta_c = M.beta_c;
  const float p_vdepen = M.v_depen, p_clin = M.c_lin, p_cang = M.c_ang, p_wmax = M.w_max;
  const int p_gyro = M.gyro;
  for (int i = tid; i < E * D; i += kThreads) {
    int ee = i / D, d = i - ee * D;
    int env_i = blockIdx.x * E + ee;
    float uu = 0.0f;
    if (env_i < N && a.actions) uu = a.actions[(size_t)agent_at(env_i) * D + d];
    Lu[d * E + ee] = fminf(fmaxf(uu, -1.0f), 1.0f);
  }
  // small copies of what the per-slot code looks up all the time
  for (int i = tid; i < 3 * E; i += kThreads) {
    int c = i / E, ee = i - c * E, env_i = blockIdx.x * E + ee;
    Lorg[i] = env_i < N ? a.origins[3 * agent_at(env_i) + c] : 0.0f;
  }
  // external pushes (Section 4.1): is this frame the env's next push?
  if (tid < E) {
    const bool env_t_ok = blockIdx.x * E + tid < N;
    const int env_t = agent_at(blockIdx.x * E + tid);
    float fx = 0.0f, fy = 0.0f;
    if (a.task.enabled && a.task.push_max_f > 0 && a.count_step && env_t_ok) {
      const int f = a.steps[env_t], ep = a.task_i[4 * env_t + 3];
      if (f == a.task_i[4 * env_t + 2]) {
        const float mag = a.task.push_min_n + (a.task.push_max_n - a.task.push_min_n) * task_u(a.task, env_t, ep, f, 0);
        const float phi = 6.283185307179586f * task_u(a.task, env_t, ep, f, 1);
        fx = mag * cosf(phi); fy = mag * sinf(phi);
        a.task_i[4 * env_t + 2] = f + task_interval(a.task, env_t, ep, f);
      }
    }
    Lpush[0 * E + tid] = fx; Lpush[1 * E + tid] = fy; Lpush[2 * E + tid] = 0.0f;
    if (a.task.enabled && a.count_step && env_t_ok) { a.push[3 * env_t] = fx; a.push[3 * env_t + 1] = fy; a.push[3 * env_t + 2] = 0.0f; }
  }
  for (int i = tid; i < M.table_words; i += kThreads) reinterpret_cast<int*>(lds + P.tjs)[i] = M.table_image[i];
  for (int i = tid; i < (J * kJS + S * kCS) * E; i += kThreads) Loutj[i] = 0.0f;  // copies may be read (weight 0) before they are written
  if constexpr (WS != 0) {
    for (int i = tid; i < J * 6 * E; i += kThreads) {
      const int env_i = blockIdx.x * E + i % E;
      Lwj[i] = env_i < N ? a.lam_j[(size_t)(i / E) * N + agent_at(env_i)] : 0.0f;
    }
    for (int i = tid; i < S * 3 * E; i += kThreads) {
      const int env_i = blockIdx.x * E + i % E;
      Lwc[i] = env_i < N ? a.lam_s[(size_t)(i / E) * N + agent_at(env_i)] : 0.0f;
    }
  }
  if constexpr (PC != 0) {
    if (tid < 12) Lpo[kPairCap * 12 + tid] = 0.0f;   // the entry unused list slots point at
  }
  // contact records start cleared (a step with zero substeps packs "no contact")
  for (int i = tid; i < S * E; i += kThreads) {
    Lreci[(i / E * kRecWords + 0) * E + i % E] = 0;
    Lreci[(i / E * kRecWords + 1) * E + i % E] = -1;
    Lreci[(i / E * kRecWords + 2) * E + i % E] = -1;
    for (int c = 3; c < kRecWords; ++c) Lrec[(i / E * kRecWords + c) * E + i % E] = 0.0f;
  }

  // per-env copy of the heightfield samples around the root body (the whole robot stays
  // within it during one step; anything outside falls back to global memory)
  if (use_patch && a.substeps > 0) {   // (a launch without substeps never searches the terrain)
    // where the copy starts: from the root body's position, which its body thread has just loaded
    if (is_body && b == M.root) {
      const float rx = x[0] + root_ox, ry = x[1] + root_oy;
      float ci = floorf((rx - M.hox) * M.inv_cell), cj = floorf((ry - M.hoy) * M.inv_cell);
      ci = fminf(fmaxf(ci - (float)(kPatch / 2), 0.0f), (float)(M.nx - kPatch));
      cj = fminf(fmaxf(cj - (float)(kPatch / 2), 0.0f), (float)(M.ny - kPatch));
      Lporg[2 * e] = (int)ci; Lporg[2 * e + 1] = (int)cj;
    }
    if (tid < E && blockIdx.x * E + tid >= N) { Lporg[2 * tid] = 0; Lporg[2 * tid + 1] = 0; }
    __syncthreads();
    // many samples per thread in flight at a time (the reads come from L2, one at a time each
    // would cost its full latency): the wide workgroup fetches the copies of 16 envs in one round
    constexpr int kInFlight = NT >= 768 ? 17 : 13;
    for (int i0 = tid; i0 < E * kPatch * kPatch; i0 += kInFlight * kThreads) {
      float hv[kInFlight];
#pragma unroll
      for (int k = 0; k < kInFlight; ++k) {
        const int i = i0 + k * kThreads;
        hv[k] = 0.0f;
        if (i < E * kPatch * kPatch) {
          int ee = i / (kPatch * kPatch), r = i - ee * (kPatch * kPatch), pj = r / kPatch, pi = r - pj * kPatch;
          hv[k] = a.heights[(Lporg[2 * ee + 1] + pj) * H0.nx + Lporg[2 * ee] + pi];
        }
      }
#pragma unroll
      for (int k = 0; k < kInFlight; ++k)
        if (i0 + k * kThreads < E * kPatch * kPatch) Lpatch[i0 + k * kThreads] = hv[k];
    }
    __syncthreads();
    for (int i = tid; i < E * kPatchBlocks * kPatchBlocks; i += kThreads) {
      int ee = i / (kPatchBlocks * kPatchBlocks), r = i - ee * (kPatchBlocks * kPatchBlocks);
      int bj = r / kPatchBlocks, bi = r - bj * kPatchBlocks;
      // (kMip+1)^2 samples, indices clamped into the copy, all reads issued before the first use
      float hv[(kMip + 1) * (kMip + 1)];
#pragma unroll
      for (int dj = 0; dj <= kMip; ++dj)
#pragma unroll
        for (int di = 0; di <= kMip; ++di) {
          const int pj = bj * kMip + dj < kPatch ? bj * kMip + dj : kPatch - 1;
          const int pi = bi * kMip + di < kPatch ? bi * kMip + di : kPatch - 1;
          hv[dj * (kMip + 1) + di] = Lpatch[ee * (kPatch * kPatch) + pj * kPatch + pi];
        }
      __builtin_amdgcn_sched_group_barrier(0x100, (kMip + 1) * (kMip + 1), 0);
      float hm = -INFINITY;
#pragma unroll
      for (int k = 0; k < (kMip + 1) * (kMip + 1); ++k) hm = fmaxf(hm, hv[k]);
      Lmip[i] = hm;
    }
  }

  TMARK(0);
  // wavefronts [0, joint_threads/64) hold the joint-side threads; contact k of a workgroup goes
  // to thread kThreads-1-k as long as that thread is not in a joint wavefront (n_reg contacts)
  const int joint_threads = ((2 * J * E + 63) / 64) * 64;
  const int n_reg = kThreads - joint_threads;
  const bool joint_wave = __builtin_amdgcn_readfirstlane(tid) < joint_threads;
  // joint-side role: lanes 2p and 2p+1 are the parent and the child side of pair p = (joint, env)
  const int js_side = tid & 1, js_e = (tid >> 1) % E, js_j = (tid >> 1) / E;
  const bool js_on = js_j < J && blockIdx.x * E + js_e < N;

  const int tid_o = tid, e_o = e, idx_o = idx;
  const float h_o = h;
  for (int sub = 0; sub < a.substeps; ++sub) {
    // In the variants that are short of registers (capsule-capsule collisions, or the wide workgroup
    // with its 170 VGPRs per thread) the thread's indices and the time step are passed through empty
    // asm statements at the top of each substep: what is derived from them (LDS addresses, h-scaled
    // constants) is then recomputed per substep instead of being computed once before the loop and
    // kept alive across it.  The others have registers to spare and let the compiler hoist.
    // row constants of this substep (declared here: nothing of them is carried into the next one)
    SideRows jr;
    ContactRows cr;
    PairSide pr;
    bool has_contact = false;  // this thread owns an active contact this substep
    int tid = tid_o, e = e_o, idx = idx_o;
    float h = h_o;
    if constexpr (PC != 0 || NT > 512 || NS != 0) {
      asm volatile("" : "+v"(tid), "+v"(e), "+v"(idx));
      asm volatile("" : "+s"(h));
    }
    const int b = idx;
    // ---- A: publish pose and world inverse inertia
    if (tid == 0) { Lcount[0] = 0; Lcount[1] = 0; Lcount[2] = 0; Lcount[3] = 0; Lcount[4] = 0; Lcount[5] = 0; Lcount[6] = 0; Lcount[7] = 0; }
    if constexpr (PC != 0) {
      if (tid < 4) Lpcount[tid] = 0;
      if (tid < E) Lbs[tid] = 0;
      for (int i = tid; i < B * E; i += kThreads) Lpbcnt[i] = 0;
    }
    if (is_body) {
      for (int c = 0; c < 3; ++c) Lpos[(b * 7 + c) * E + e] = x[c];
      for (int c = 0; c < 4; ++c) Lpos[(b * 7 + 3 + c) * E + e] = q[c];
      // velocities are parked in LDS as well: nothing of the body stays in registers while the
      // contact phases run
      for (int c = 0; c < 3; ++c) { Lvel[(b * kVS + c) * E + e] = v[c]; Lvel[(b * kVS + 3 + c) * E + e] = w[c]; }
      float R[9], invIb[3];
      quat_to_mat(q, R);
      for (int c = 0; c < 3; ++c) invIb[c] = Ltin[6 * b + 3 + c];
      float iw[6];
      iw[0] = R[0] * R[0] * invIb[0] + R[1] * R[1] * invIb[1] + R[2] * R[2] * invIb[2];
      iw[1] = R[0] * R[3] * invIb[0] + R[1] * R[4] * invIb[1] + R[2] * R[5] * invIb[2];
      iw[2] = R[0] * R[6] * invIb[0] + R[1] * R[7] * invIb[1] + R[2] * R[8] * invIb[2];
      iw[3] = R[3] * R[3] * invIb[0] + R[4] * R[4] * invIb[1] + R[5] * R[5] * invIb[2];
      iw[4] = R[3] * R[6] * invIb[0] + R[4] * R[7] * invIb[1] + R[5] * R[8] * invIb[2];
      iw[5] = R[6] * R[6] * invIb[0] + R[7] * R[7] * invIb[1] + R[8] * R[8] * invIb[2];
      for (int c = 0; c < 6; ++c) Liw[(b * kVS + c) * E + e] = iw[c];
    }
    __syncthreads();

    TMARK(1);
    // ---- B: joint torques (stored once per joint; the body applies the sign).  They go through
    //         LDS only, so they are computed by the upper half of the workgroup when the joints fit
    //         there: the lower half runs the per-body pass below at the same time.
    {
      const int tq_base = J * E <= kThreads / 2 ? kThreads / 2 : 0;
      const int tj = (tid - tq_base) / E, te = (tid - tq_base) % E;
      if (tid >= tq_base && tj < J && blockIdx.x * E + te < N) {
        const JointTab& jt = Ltjoint[tj];
        float qa[4] = {1, 0, 0, 0};
        if (jt.parent >= 0)
          for (int c = 0; c < 4; ++c) qa[c] = Lpos[(jt.parent * 7 + 3 + c) * E + te];
        float Ra[9];
        quat_to_mat(qa, Ra);
        float tq[3] = {0, 0, 0};
        for (int k = 0; k < 3; ++k) {
          if (jt.mode[k] != 1) continue;
          float ak[3];
          mat_vec(Ra, jt.axes[k], ak);
          float t = jt.gear[k] * Lu[jt.act[k] * E + te];
          tq[0] += t * ak[0]; tq[1] += t * ak[1]; tq[2] += t * ak[2];
        }
        for (int c = 0; c < 3; ++c) Ltq[(tj * 3 + c) * E + te] = tq[c];
      }
    }
    // ---- B1: every slot: plane contact, or reach test against the heightfield copy.  A slot
    //          that may touch the heightfield (block maxima, then the exact maximum over its box)
    //          is queued (end spheres from the front of the queue, mid-segments from the back), its
    //          world-space geometry is left in its still unused record, and its box is cut into
    //          work units of 8 cells (samples for a mid-segment).
    //          Slots go to the threads from the top of the workgroup down: a second round, if any,
    //          then runs on the last wavefronts while the first ones hold the joint threads.
    // forces -> velocities (torques, gravity, push, explicit gyroscopic term): body threads, needs
    // the joint torques and nothing of the contacts
    auto forces = [&]() {
      if (!is_body) return;
      float tau[3] = {0, 0, 0};
      for (int k = 0; k < my_njs; ++k) {
        const int js = Ltjs[b * (kMaxBodyJoints + 3) + 3 + k];
        const float sg = (js & 1) ? 1.0f : -1.0f;
        for (int c = 0; c < 3; ++c) tau[c] += sg * Ltq[((js >> 1) * 3 + c) * E + e];
      }
      float R[9], qq[4], Ib[3], invIb[3];
      for (int c = 0; c < 4; ++c) qq[c] = Lpos[(b * 7 + 3 + c) * E + e];
      quat_to_mat(qq, R);
      for (int c = 0; c < 3; ++c) { Ib[c] = Ltin[6 * b + c]; invIb[c] = Ltin[6 * b + 3 + c]; }
      for (int c = 0; c < 3; ++c) { v[c] = Lvel[(b * kVS + c) * E + e]; w[c] = Lvel[(b * kVS + 3 + c) * E + e]; }
      if (a.task.enabled && b == M.root) {
        const float him = h * Ltbody[4 * b + 3];
        v[0] += him * Lpush[0 * E + e]; v[1] += him * Lpush[1 * E + e]; v[2] += him * Lpush[2 * E + e];
      }
      v[0] += h * g0; v[1] += h * g1; v[2] += h * g2;
      float wb[3], tb[3];
      mat_t_vec(R, w, wb);
      mat_t_vec(R, tau, tb);
      float Iw[3] = {Ib[0] * wb[0], Ib[1] * wb[1], Ib[2] * wb[2]};
      float gy[3];
      cross(wb, Iw, gy);
      if (!p_gyro) { gy[0] = gy[1] = gy[2] = 0.0f; }
      // only the increment goes back to the world frame (the velocity itself is not rotated
      // there and back, which would round it six times more)
      float dwb[3], dww[3];
      for (int c = 0; c < 3; ++c) dwb[c] = h * (tb[c] - gy[c]) * invIb[c];
      mat_vec(R, dwb, dww);
      for (int c = 0; c < 3; ++c) w[c] += dww[c];
      for (int c = 0; c < 3; ++c) { Lvel[(b * kVS + c) * E + e] = v[c]; Lvel[(b * kVS + 3 + c) * E + e] = w[c]; }
    };
    int n_b1 = S * E;            // slots the per-slot pass visits
    unsigned* Lslots = Lcand;    // heightfield: list of the slots of the bodies near the ground
    if (m_terrain == 1) {
      // ---- B1a: one thread per body: reach test of the whole capsule (box of its segment);
      //           the slots of a body that passes are listed for the per-slot pass, the others
      //           are inactive.  A slot can only pass its own test if its body passes this one.
      for (int i = tid; i < B * E; i += kThreads) {
        const int ee = i % E, bb = i / E;
        const int env_i = blockIdx.x * E + ee;
        const int s0 = Ltjs[bb * (kMaxBodyJoints + 3) + 1], ns = Ltjs[bb * (kMaxBodyJoints + 3) + 2];
        bool near = false;
        if (env_i < N && m_contacts) {
          float bx[3], bq[4], bo[3];
          for (int c = 0; c < 3; ++c) bx[c] = Lpos[(bb * 7 + c) * E + ee];
          for (int c = 0; c < 4; ++c) bq[c] = Lpos[(bb * 7 + 3 + c) * E + ee];
          for (int c = 0; c < 3; ++c) bo[c] = Lorg[c * E + ee];
          SlotGeom g = slot_geom(Ltbody[4 * bb], Ltbody[4 * bb + 1], __float_as_int(Ltbody[4 * bb + 2]), p_margin, bx, bq,
                                 2, bo);
          Field H = H0;
          if (use_patch) { H.patch = (const lds_float*)(Lpatch + ee * (kPatch * kPatch)); H.mip = (const lds_float*)(Lmip + ee * (kPatchBlocks * kPatchBlocks)); H.pi0 = Lporg[2 * ee]; H.pj0 = Lporg[2 * ee + 1]; H.ps = kPatch; }
          near = slot_reach(H, g, false);
        }
        const int pos = wave_alloc<2>(near ? ns : 0, &Lcount[7]);
        for (int k = 0; k < ns; ++k) {
          if (near) Lslots[pos + k] = (unsigned)((s0 + k) * E + ee);
          else {
            Lreci[((s0 + k) * kRecWords + 0) * E + ee] = 0;
            Lrec[((s0 + k) * kRecWords + 10) * E + ee] = 0.0f;
          }
        }
      }
      __syncthreads();
      TMARK(24);
      n_b1 = Lcount[7];
      // the lower wavefronts integrate the forces while the upper ones run the per-slot pass
      forces();
    }
    for (int x = kThreads - 1 - tid; x < n_b1; x += kThreads) {
      const int i = m_terrain == 1 ? (int)Lslots[x] : x;
      int ee = i % E, s = i / E;
      int env_i = blockIdx.x * E + ee;
      ContactOut co = no_contact();
      int nu_e = 0, nu_m = 0, qi = 0;
      if (env_i < N && m_contacts) {
        const SlotTab sl{Ltslot[2 * s], Ltslot[2 * s + 1]};
        float bx[3], bq[4], bo[3];
        for (int c = 0; c < 3; ++c) bx[c] = Lpos[(sl.body * 7 + c) * E + ee];
        for (int c = 0; c < 4; ++c) bq[c] = Lpos[(sl.body * 7 + 3 + c) * E + ee];
        for (int c = 0; c < 3; ++c) bo[c] = Lorg[c * E + ee];
        SlotGeom g = slot_geom(Ltbody[4 * sl.body], Ltbody[4 * sl.body + 1], __float_as_int(Ltbody[4 * sl.body + 2]),
                               p_margin, bx, bq, sl.kind, bo);
        if (m_terrain == 0) {
          co = plane_contact(g, p_margin);
        } else {
          Field H = H0;
          if (use_patch) { H.patch = (const lds_float*)(Lpatch + ee * (kPatch * kPatch)); H.mip = (const lds_float*)(Lmip + ee * (kPatchBlocks * kPatchBlocks)); H.pi0 = Lporg[2 * ee]; H.pj0 = Lporg[2 * ee + 1]; H.ps = kPatch; }
          if (slot_reach(H, g)) {
            const bool mid = sl.kind == 2;
            qi = mid ? S * E - 1 - atomicAdd(&Lcount[2], 1) : atomicAdd(&Lcount[1], 1);
            Lsurv[qi] = i;
            Lbest64[i] = ~0ull;
            const int ni = g.i1 - g.i0 + (mid ? 2 : 1), nj = g.j1 - g.j0 + (mid ? 2 : 1);
            const bool fits = ni <= 15 && nj <= 15 && g.i0 < 4096 && g.j0 < 4096;  // packed box below
            const f3 Pa = sl.kind == 1 ? g.P1 : g.P0;
            Lrec[(s * kRecWords + 1) * E + ee] = Pa.x; Lrec[(s * kRecWords + 2) * E + ee] = Pa.y;
            Lrec[(s * kRecWords + 3) * E + ee] = Pa.z;
            Lreci[(s * kRecWords + 7) * E + ee] = g.i0 | (g.j0 << 12) | (ni << 24) | (nj << 28);
            Lreci[(s * kRecWords + 8) * E + ee] = fits ? 0 : 1;   // 1: search this slot the slow way
            Lgeo[3 * i] = g.Rq;
            if (mid) {
              Lrec[(s * kRecWords + 4) * E + ee] = g.P1.x; Lrec[(s * kRecWords + 5) * E + ee] = g.P1.y;
              Lrec[(s * kRecWords + 6) * E + ee] = g.P1.z;
              float RL, inv_L2;
              seg_cull_consts(g, RL, inv_L2);
              Lgeo[3 * i + 1] = RL; Lgeo[3 * i + 2] = inv_L2;
            }
            if (!fits) Lcount[4] = 1;
            else if (mid) nu_m = (ni * nj + 7) >> 3;
            else nu_e = (ni * nj + 7) >> 3;
          }
        }
      }
      if (m_terrain == 1) {
        // list space for the units of the whole wavefront, one atomic per kind
        const int ue = wave_alloc<5>(nu_e, &Lcount[5]), um = wave_alloc<5>(nu_m, &Lcount[6]);
        const int nu = nu_e + nu_m, u0 = nu_e ? ue : um, cap = nu_e ? unit_cap_e : unit_cap - unit_cap_e;
        unsigned* U = Lunit + (nu_e ? 0 : unit_cap_e);
        for (int u = 0; u < nu; ++u)
          if (u0 + u < cap) U[u0 + u] = (unsigned)i | ((unsigned)u << 12);
        if (nu > 0 && u0 + nu > cap) { Lreci[(s * kRecWords + 8) * E + ee] = 1; Lcount[4] = 1; }
      }
      if (co.active) {
        store_record(Lrec, Lreci, s, ee, E, co);
        Llist[atomicAdd(&Lcount[0], 1)] = i;
      } else {
        Lreci[(s * kRecWords + 0) * E + ee] = 0;      // the other words of an inactive record are not read
        Lrec[(s * kRecWords + 10) * E + ee] = 0.0f;
      }
    }
    TMARK(2);
    if (m_terrain == 1) {
      __syncthreads();
      TMARK(25);
      // ---- B2: fine search in two stages.  Stage 1: kGroup lanes per work unit, one cell per
      //          lane: a cheap reach test decides which triangles (end sphere) or edges
      //          (mid-segment) of the cell become candidates.  Stage 2: one candidate per thread:
      //          exact distance, minimum of (d2, id) per slot with a 64-bit LDS atomic.
      const int grp = tid / kGroup, gl = tid % kGroup;
      Field H = H0;
      const int n_end = Lcount[1], n_mid = Lcount[2];
      for (int pass = 0; pass < 2; ++pass) {
        const int cap = pass == 0 ? unit_cap_e : unit_cap - unit_cap_e;
        const int n_u = Lcount[5 + pass] < cap ? Lcount[5 + pass] : cap;
        const unsigned* U = Lunit + (pass == 0 ? 0 : unit_cap_e);
        for (int x = grp; x < n_u; x += kThreads / kGroup) {
          const unsigned uw = U[x];
          const int i = uw & 4095, c = (int)(uw >> 12) * 8 + gl;   // slot index, cell within the box
          const int ee = i % E, s = i / E;
          const unsigned box = (unsigned)Lreci[(s * kRecWords + 7) * E + ee];
          const int i0 = box & 4095, j0 = (box >> 12) & 4095, ni = (box >> 24) & 15, nj = box >> 28;
          // c / ni for small non-negative integers: the quotient of (c + 0.5) / ni is at least
          // 0.5 / 15 away from an integer, far more than the error of the reciprocal
          const int dj = (int)(((float)c + 0.5f) * __builtin_amdgcn_rcpf((float)ni)), di = c - dj * ni;
          if (use_patch) { H.patch = (const lds_float*)(Lpatch + ee * (kPatch * kPatch)); H.mip = (const lds_float*)(Lmip + ee * (kPatchBlocks * kPatchBlocks)); H.pi0 = Lporg[2 * ee]; H.pj0 = Lporg[2 * ee + 1]; H.ps = kPatch; }
          const f3 Pa = f3{Lrec[(s * kRecWords + 1) * E + ee], Lrec[(s * kRecWords + 2) * E + ee], Lrec[(s * kRecWords + 3) * E + ee]};
          const float Rq = Lgeo[3 * i];
          int mask = 0;
          if (pass == 0) {
            if (c < ni * nj && sphere_cell_reach(H, Pa, Rq + kSelSlack, i0 + di, j0 + dj)) mask = 3;
          } else {
            const f3 Pb = f3{Lrec[(s * kRecWords + 4) * E + ee], Lrec[(s * kRecWords + 5) * E + ee], Lrec[(s * kRecWords + 6) * E + ee]};
            const SegCull sc = seg_cull_from(Pa, Pb, Rq, Lgeo[3 * i + 1], Lgeo[3 * i + 2], i0 + ni - 2, j0 + nj - 2);
            if (c < ni * nj) mask = segment_candidates(H, sc, i0 + di, j0 + dj);
          }
          int pos = wave_alloc<2>(__popc(mask), &Lcount[3]);
          const unsigned cw = (unsigned)i | ((unsigned)di << 14) | ((unsigned)dj << 18) | ((unsigned)pass << 22);
#pragma unroll
          for (int k = 0; k < 3; ++k)
            if ((mask >> k) & 1) {
              if (pos < cand_cap) Lcand[pos] = cw | ((unsigned)k << 12);
              ++pos;
            }
          if (mask != 0 && pos > cand_cap) {
            // candidate list full: the slot is searched again by the fallback below
            Lreci[(s * kRecWords + 8) * E + ee] = 1;
            Lcount[4] = 1;
          }
        }
        TMARK(10 + pass);
      }
      __syncthreads();
      {
        const int n_c = Lcount[3] < cand_cap ? Lcount[3] : cand_cap;
        for (int t = tid; t < n_c; t += kThreads) {
          const unsigned cw = Lcand[t];
          const int i = cw & 4095, k = (cw >> 12) & 3, di = (cw >> 14) & 15, dj = (cw >> 18) & 15;
          const int ee = i % E, s = i / E;
          const unsigned box = (unsigned)Lreci[(s * kRecWords + 7) * E + ee];
          const int ci = (int)(box & 4095) + di, cj = (int)((box >> 12) & 4095) + dj;
          if (use_patch) { H.patch = (const lds_float*)(Lpatch + ee * (kPatch * kPatch)); H.mip = (const lds_float*)(Lmip + ee * (kPatchBlocks * kPatchBlocks)); H.pi0 = Lporg[2 * ee]; H.pj0 = Lporg[2 * ee + 1]; H.ps = kPatch; }
          const f3 Pa = f3{Lrec[(s * kRecWords + 1) * E + ee], Lrec[(s * kRecWords + 2) * E + ee], Lrec[(s * kRecWords + 3) * E + ee]};
          float d2;
          if (((cw >> 22) & 1) == 0) {
            if (sphere_tri_d2(H, Pa, ci, cj, k, d2)) atomicMin(&Lbest64[i], pack_best(d2, 2 * (cj * (H.nx - 1) + ci) + k));
          } else {
            const f3 Pb = f3{Lrec[(s * kRecWords + 4) * E + ee], Lrec[(s * kRecWords + 5) * E + ee], Lrec[(s * kRecWords + 6) * E + ee]};
            if (segment_edge_d2(H, Pa, Pb, ci, cj, k, d2)) atomicMin(&Lbest64[i], pack_best(d2, 3 * (cj * H.nx + ci) + k));
          }
        }
        __syncthreads();
        TMARK(13);
        if (Lcount[4]) {
          // rare: a box too large for the packed indices, or a full list: those slots are searched
          // directly, kGroup lanes per slot
          for (int sv = grp; sv < n_end + n_mid; sv += kThreads / kGroup) {
            const int qi = sv < n_end ? sv : S * E - 1 - (sv - n_end);
            const int i = Lsurv[qi];
            const int ee = i % E, s = i / E;
            if (!Lreci[(s * kRecWords + 8) * E + ee]) continue;
            const SlotTab sl{Ltslot[2 * s], Ltslot[2 * s + 1]};
            float bx[3], bq[4], bo[3];
            for (int c = 0; c < 3; ++c) bx[c] = Lpos[(sl.body * 7 + c) * E + ee];
            for (int c = 0; c < 4; ++c) bq[c] = Lpos[(sl.body * 7 + 3 + c) * E + ee];
            for (int c = 0; c < 3; ++c) bo[c] = Lorg[c * E + ee];
            SlotGeom g = slot_geom(Ltbody[4 * sl.body], Ltbody[4 * sl.body + 1], __float_as_int(Ltbody[4 * sl.body + 2]),
                                   p_margin, bx, bq, sl.kind, bo);
            if (use_patch) { H.patch = (const lds_float*)(Lpatch + ee * (kPatch * kPatch)); H.mip = (const lds_float*)(Lmip + ee * (kPatchBlocks * kPatchBlocks)); H.pi0 = Lporg[2 * ee]; H.pj0 = Lporg[2 * ee + 1]; H.ps = kPatch; }
            slot_range(H, g);
            float best = INFINITY;
            int best_id = -1;
            if (sl.kind < 2) {
              const f3 Pc = sl.kind == 0 ? g.P0 : g.P1;
              const int ni = g.i1 - g.i0 + 1, nc = ni * (g.j1 - g.j0 + 1);
              for (int c = gl; c < nc; c += kGroup) sphere_cell(H, Pc, g.Rq, g.i0 + c % ni, g.j0 + c / ni, best, best_id);
            } else {
              const int ni = g.i1 - g.i0 + 2, nc = ni * (g.j1 - g.j0 + 2);
              const SegCull sc = seg_cull(g);
              for (int c = gl; c < nc; c += kGroup) segment_vertex(H, g, sc, g.i0 + c % ni, g.j0 + c / ni, best, best_id);
            }
            if (best_id >= 0) atomicMin(&Lbest64[i], pack_best(best, best_id));
          }
          __syncthreads();
        }
      }
#ifdef SIM_PHASE_TIMING
      if (tid == 0 && blockIdx.x == 7) { a.dbg[14] += Lcount[5] + Lcount[6]; a.dbg[15] += Lcount[3]; }
#endif
      // ---- B3: one thread per queued slot turns the selected feature into a contact record
      //          (end spheres on the lower half of the workgroup, mid-segments on the upper half,
      //          so that a wavefront follows one path)
      for (int sv = tid < kThreads / 2 ? tid : tid - kThreads / 2; sv < (tid < kThreads / 2 ? n_end : n_mid); sv += kThreads / 2) {
        const int qi = tid < kThreads / 2 ? sv : S * E - 1 - sv;
        const int i = Lsurv[qi];
        const int ee = i % E, s = i / E;
        const SlotTab sl{Ltslot[2 * s], Ltslot[2 * s + 1]};
        float bx[3], bq[4], bo[3];
        for (int c = 0; c < 3; ++c) bx[c] = Lpos[(sl.body * 7 + c) * E + ee];
        for (int c = 0; c < 4; ++c) bq[c] = Lpos[(sl.body * 7 + 3 + c) * E + ee];
        for (int c = 0; c < 3; ++c) bo[c] = Lorg[c * E + ee];
        SlotGeom g = slot_geom(Ltbody[4 * sl.body], Ltbody[4 * sl.body + 1], __float_as_int(Ltbody[4 * sl.body + 2]),
                               p_margin, bx, bq, sl.kind, bo);
        if (use_patch) { H.patch = (const lds_float*)(Lpatch + ee * (kPatch * kPatch)); H.mip = (const lds_float*)(Lmip + ee * (kPatchBlocks * kPatchBlocks)); H.pi0 = Lporg[2 * ee]; H.pj0 = Lporg[2 * ee + 1]; H.ps = kPatch; }
        ContactOut co = no_contact();
        const unsigned long long bw = Lbest64[i];
        const float bestd = __uint_as_float((unsigned)(bw >> 32));
        const int besti = (int)(unsigned)bw;
        if (sl.kind < 2) {
          // a centre underneath the surface overrides the nearest-triangle search
          if (!underneath_contact(H, g, p_margin, co)) co = finish_sphere(H, g, p_margin, bestd, besti);
        } else {
          co = finish_segment(H, g, p_margin, bestd, besti);
        }
        if (co.active) {
          store_record(Lrec, Lreci, s, ee, E, co);
          Llist[atomicAdd(&Lcount[0], 1)] = i;
        }
      }
      __syncthreads();
      TMARK(12);
      // the search results shared the space of the contact copies: leave finite numbers behind
      for (int i = tid; i < 5 * S * E; i += kThreads) Loutj[i] = 0.0f;
    }
    __syncthreads();
    TMARK(3);

    // ---- P: capsule-capsule contacts from the poses published in phase A (Section 3.1: contacts
    //         among bodies; Section 4.1: inter-agent collisions).  Candidates: the listed body pairs
    //         of every agent, and every body pair of two agents of one group whose bounding spheres
    //         overlap.  A candidate passes a bounding-sphere test (stage 1, which compacts the
    //         survivors into a list), then the segment-segment test in the fixed operation order
    //         (stage 2, one survivor per lane); hits are queued and the queue is sorted by key, so
    //         that the order in which the bodies later add up their contacts does not depend on which
    //         wavefront found what first.
    int n_pc = 0;
    if constexpr (PC != 0) {
      if (m_contacts && (m_npairs > 0 || m_group > 1)) {
        if (m_group > 1) {
          if (is_body) {
            float dx[3];
            for (int c = 0; c < 3; ++c) dx[c] = Lpos[(b * 7 + c) * E + e] - Lpos[(M.root * 7 + c) * E + e];
            const float rad = sqrtf(dot(dx, dx)) + Ltbody[4 * b + 1] + Ltbody[4 * b];
            atomicMax(&Lbs[e], __float_as_int(rad));
          }
          __syncthreads();
          const int n_ap = (E / m_group) * m_nap;
          for (int t = tid; t < n_ap; t += kThreads) {
            const int gi = t / m_nap, pi = t - gi * m_nap;
            const int ea = gi * m_group + M.agent_pair_a[pi], eb = gi * m_group + M.agent_pair_b[pi];
            bool near = false;
            if (blockIdx.x * E + eb < N) {   // (ea < eb)
              float dd = 0.0f;
              for (int c = 0; c < 3; ++c) {
                const float dc = (Lpos[(M.root * 7 + c) * E + eb] + Lorg[c * E + eb]) - (Lpos[(M.root * 7 + c) * E + ea] + Lorg[c * E + ea]);
                dd += dc * dc;
              }
              const float rr = __int_as_float(Lbs[ea]) + __int_as_float(Lbs[eb]) + p_margin + 2e-3f;
              near = dd <= rr * rr;
            }
            const int pos = wave_alloc<1>(near ? 1 : 0, &Lpcount[1]);
            if (near) Lnear[pos] = ea | (eb << 16);
          }
          __syncthreads();
        }
        float* Ltmp = Lpo;   // unsorted queue; the copies are not in use yet
        // Every hit also leaves (gap, key) as one 64-bit word whose unsigned order is that of the
        // pair: when a workgroup finds more than it can hold, the kPairCap contacts with the smallest
        // gap stay (ties: smaller key), whichever wavefront found what first.  Where they live:
        // see make_plan (cleared again below, since the sweeps' copies share the space).
        unsigned long long* Lhit = reinterpret_cast<unsigned long long*>(lds + P.phit);
        const int hit_cap = P.hit_cap;
        // the segment-segment test of one candidate pair from the poses of phase A
        auto eval_pair = [&](int ea, int ba, int eb, int bb, float& sp, float& tp, float& gap) -> bool {
          float xa[3], xb[3], off[3];
          for (int c = 0; c < 3; ++c) {
            off[c] = Lorg[c * E + eb] - Lorg[c * E + ea];
            xa[c] = Lpos[(ba * 7 + c) * E + ea];
            xb[c] = Lpos[(bb * 7 + c) * E + eb];
          }
          const float radA = Ltbody[4 * ba], hlA = Ltbody[4 * ba + 1], radB = Ltbody[4 * bb], hlB = Ltbody[4 * bb + 1];
          float dd = 0.0f;
          for (int c = 0; c < 3; ++c) { const float dc = (xb[c] + off[c]) - xa[c]; dd += dc * dc; }
          const float reach = (radA + hlA) + (radB + hlB) + p_margin + 2e-3f;
          if (!(dd <= reach * reach)) return false;
          float qa[4], qb[4];
          for (int c = 0; c < 4; ++c) { qa[c] = Lpos[(ba * 7 + 3 + c) * E + ea]; qb[c] = Lpos[(bb * 7 + 3 + c) * E + eb]; }
          f3 p0, p1, q0, q1;
          body_ends(xa, qa, hlA, __float_as_int(Ltbody[4 * ba + 2]), p0, p1);
          body_ends(xb, qb, hlB, __float_as_int(Ltbody[4 * bb + 2]), q0, q1);
          return pair_in_contact(p0, p1, q0, q1, off, radA, radB, p_margin, sp, tp, gap);
        };
        auto store_hit = [&](int pos, int ea, int ba, int eb, int bb, unsigned key, float sp, float tp, float gap) {
          Ltmp[pos * kPairWords + 0] = __uint_as_float(key);
          Ltmp[pos * kPairWords + 1] = __int_as_float((ba * E + ea) | ((bb * E + eb) << 16));
          Ltmp[pos * kPairWords + 2] = sp;
          Ltmp[pos * kPairWords + 3] = tp;
          Ltmp[pos * kPairWords + 4] = block_weight(p_margin, gap, 1.0f);
          Ltmp[pos * kPairWords + 5] = gap;
        };
        auto test_pair = [&](int ea, int ba, int eb, int bb, unsigned key, bool valid) {
          float sp = 0.0f, tp = 0.0f, gap = 0.0f;
          const bool hit = valid && eval_pair(ea, ba, eb, bb, sp, tp, gap);
          const int pos = wave_alloc<1>(hit ? 1 : 0, &Lpcount[0]);
          if (hit && pos < kPairCap) store_hit(pos, ea, ba, eb, bb, key, sp, tp, gap);
          if (hit && pos < hit_cap) {
            const unsigned gb = __float_as_uint(gap);
            const unsigned ordered = (gb & 0x80000000u) ? ~gb : (gb | 0x80000000u);   // unsigned order = float order
            Lhit[pos] = ((unsigned long long)ordered << 32) | key;
          }
        };
        // Stage 1: bounding spheres of the two capsules only; what passes is listed as a packed word
        // (env and body of A, env and body of B: also the sort key of a hit).  The list lives where
        // the observations are staged at the end of the step.
        unsigned* Lc2 = Lunit;
        auto cull_pair = [&](int ea, int ba, int eb, int bb, bool valid) {
          bool pass = false;
          if (valid) {
            float dd = 0.0f;
            for (int c = 0; c < 3; ++c) {
              const float dc = (Lpos[(bb * 7 + c) * E + eb] + (Lorg[c * E + eb] - Lorg[c * E + ea])) - Lpos[(ba * 7 + c) * E + ea];
              dd += dc * dc;
            }
            const float reach = (Ltbody[4 * ba] + Ltbody[4 * ba + 1]) + (Ltbody[4 * bb] + Ltbody[4 * bb + 1]) + p_margin + 2e-3f;
            pass = dd <= reach * reach;
          }
          const int pos = wave_alloc<1>(pass ? 1 : 0, &Lpcount[2]);
          if (pass) {
            if (pos < unit_cap) Lc2[pos] = ((unsigned)ea << 20) | ((unsigned)eb << 8) | (unsigned)(ba << 4) | (unsigned)bb;
            else Lpcount[3] = 1;   // list full: everything is tested the slow way below
          }
        };
        // the listed pairs of every agent: thread (idx, e) takes pairs idx, idx + stride, ...
        const int pair_stride = kThreads / E;
        if (idx < pair_stride)
          for (int pp = idx; pp < m_npairs; pp += pair_stride) cull_pair(e, M.pair_a[pp], e, M.pair_b[pp], env_ok);
        // agents of one group: 256 lanes per near agent pair, lane = (body of A) * 16 + (body of B)
        const int n_near = m_group > 1 ? Lpcount[1] : 0;
        for (int nn = tid >> 8; nn < n_near; nn += kThreads >> 8) {
          const int cb = tid & 255, ba = cb >> 4, bb = cb & 15;
          const int pr = Lnear[nn];
          cull_pair(pr & 0xffff, ba, pr >> 16, bb, ba < B && bb < B);
        }
        __syncthreads();
        // Stage 2: the segment-segment test, one listed candidate per lane
        if (!Lpcount[3]) {
          const int n_c2 = Lpcount[2];
          for (int c = tid; c < n_c2; c += kThreads) {
            const unsigned wd = Lc2[c];
            test_pair((int)(wd >> 20), (int)((wd >> 4) & 15u), (int)((wd >> 8) & 0xfffu), (int)(wd & 15u), wd, true);
          }
        } else {
          if (idx < pair_stride)
            for (int pp = idx; pp < m_npairs; pp += pair_stride)
              test_pair(e, M.pair_a[pp], e, M.pair_b[pp], ((unsigned)e << 20) | ((unsigned)e << 8) | (unsigned)(M.pair_a[pp] << 4) | (unsigned)M.pair_b[pp], env_ok);
          for (int nn = tid >> 8; nn < n_near; nn += kThreads >> 8) {
            const int cb = tid & 255, ba = cb >> 4, bb = cb & 15;
            const int pr = Lnear[nn], ea = pr & 0xffff, eb = pr >> 16;
            test_pair(ea, ba, eb, bb, ((unsigned)ea << 20) | ((unsigned)eb << 8) | (unsigned)(ba << 4) | (unsigned)bb, ba < B && bb < B);
          }
        }
        __syncthreads();
        const int n_raw = Lpcount[0];
        n_pc = n_raw < kPairCap ? n_raw : kPairCap;
        const int n_hit = n_raw < hit_cap ? n_raw : hit_cap;
        if (n_raw > kPairCap) {
          // more than the workgroup holds: the kPairCap smallest (gap, key) words stay; each is
          // found by its rank among all words and its contact worked out again from its key
          for (int i = tid; i < n_hit; i += kThreads) {
            const unsigned long long wi = Lhit[i];
            int rank = 0;
            for (int k = 0; k < n_hit; ++k) rank += Lhit[k] < wi ? 1 : 0;
            if (rank < kPairCap) {
              const unsigned key = (unsigned)wi;
              const int ea = (int)(key >> 20), eb = (int)((key >> 8) & 0xfffu), ba = (int)((key >> 4) & 15u), bb = (int)(key & 15u);
              float sp = 0.0f, tp = 0.0f, gap = 0.0f;
              eval_pair(ea, ba, eb, bb, sp, tp, gap);
              store_hit(rank, ea, ba, eb, bb, key, sp, tp, gap);
            }
          }
          __syncthreads();
        }
        for (int i = tid; i < 2 * n_hit; i += kThreads) reinterpret_cast<float*>(Lhit)[i] = 0.0f;   // finite numbers for the sweeps' copies
        if (tid < n_pc) {
          const unsigned key = __float_as_uint(Ltmp[tid * kPairWords]);
          int rank = 0;
          for (int k = 0; k < n_pc; ++k) rank += __float_as_uint(Ltmp[k * kPairWords]) < key ? 1 : 0;
          for (int wd = 0; wd < kPairWords; ++wd) Lpq[rank * kPairWords + wd] = Ltmp[tid * kPairWords + wd];
        }
        if (tid == 0 && n_raw > kPairCap) atomicAdd(a.pair_dropped, n_raw - kPairCap);
        __syncthreads();
        // every contact enters the lists of its two bodies (the order in which they arrive does not
        // matter: the averaging threads sort their list)
        if (tid < 2 * n_pc) {
          const int refs = __float_as_int(Lpq[(tid >> 1) * kPairWords + 1]);
          const int ref = (tid & 1) ? (refs >> 16) & 0xffff : refs & 0xffff;
          const int slot = atomicAdd(&Lpbcnt[ref], 1);
          if (slot < 6) Lpblist[ref * 6 + slot] = (uint8_t)tid;   // 2 * (queue index) + side
        }
        __syncthreads();
      }
    }
    TMARK(16);
    // The per-body average is split over several threads when the workgroup has room: thread (e, b)
    // takes the linear half of body b's velocity, thread (e, B + b) the angular half; in the wide
    // workgroup three threads take two components each (a wavefront issues one instruction every
    // five to six cycles however many others share its SIMD, so short threads beat a long one).
    // (the wide workgroup always has room for three threads per body: 3 * 16 bodies * 16 envs)
    constexpr bool g_three = NT >= 768 && EC == 16;
    const bool g_split = g_three || 2 * B * E <= kThreads;
    const int g_half = g_three ? (idx < B ? 0 : (idx < 2 * B ? 1 : 2)) : ((g_split && idx >= B) ? 1 : 0);
    const int g_b = idx - g_half * B;
    const bool g_on = env_ok && g_b < B && idx < (g_three ? 3 * B : (g_split ? 2 * B : B));
    const int g_ref = g_b * E + e;
    // capsule-capsule contacts of body g_b: where their (weighted) copies will be (up to kPairList
    // of them; a body with more walks the queue in every sweep), and the sum of their weights
    constexpr int kPairList = 6;   // (the list in LDS and the sorting network below are made for six)
    int gp_off[kPairList];
#pragma unroll
    for (int j = 0; j < kPairList; ++j) gp_off[j] = kPairCap * 12;
    bool gp_many = false;
    float gp_wsum = 0.0f;
    int gp_cnt = 0;
    if constexpr (PC != 0) {
      if (g_on) {
        const int cnt = n_pc > 0 ? Lpbcnt[g_ref] : 0;
        gp_cnt = cnt;
        if (cnt > 0 && cnt <= kPairList) {
          // the body's list (bytes 2 * queue index + side), sorted into queue order
          int v[kPairList];
#pragma unroll
          for (int j = 0; j < kPairList; ++j) v[j] = j < cnt ? (int)Lpblist[g_ref * 6 + j] : 255;
          auto cx = [&](int i, int j) { const int lo = min(v[i], v[j]), hi = max(v[i], v[j]); v[i] = lo; v[j] = hi; };
          cx(0, 5); cx(1, 3); cx(2, 4); cx(1, 2); cx(3, 4); cx(0, 3); cx(2, 5); cx(0, 1); cx(2, 3); cx(4, 5); cx(1, 2); cx(3, 4);
#pragma unroll
          for (int j = 0; j < kPairList; ++j) {
            const bool used = v[j] != 255;
            gp_off[j] = used ? v[j] * 6 : kPairCap * 12;
            const float wj = Lpq[(used ? v[j] >> 1 : 0) * kPairWords + 4];
            gp_wsum += used ? wj : 0.0f;
          }
        } else if (cnt > kPairList) {
          // more than the list holds: the weights by a walk over the queue (as in every sweep)
          for (int k = 0; k < n_pc; ++k) {
            const int refs = __float_as_int(Lpq[k * kPairWords + 1]);
            if ((refs & 0xffff) == g_ref || ((refs >> 16) & 0xffff) == g_ref) gp_wsum += Lpq[k * kPairWords + 4];
          }
        }
        gp_many = cnt > kPairList;
      }
    }
    // no body of this wavefront has more than two capsule-capsule contacts (the usual case): its
    // averages read two list entries instead of six
    // (only where a wavefront holds few bodies: with four envs per workgroup it holds sixteen, the
    // short forms are never taken and the choice itself costs 5 %)
    constexpr bool g_variants = EC >= 8;
    constexpr int kPairFew = 2;
    const bool gp_few = g_variants && PC != 0 && __ballot(gp_cnt > kPairFew) == 0ull;
    // ---- C: block weight sums (and, on the plane, forces -> velocities)
    float nbf = 0.0f;
    if (is_body) {
      nbf = (float)my_njs;
      for (int k = 0; k < my_nslots; ++k) nbf += Lrec[((my_slot0 + k) * kRecWords + 10) * E + e];
      nbf += gp_wsum;   // (a body thread is the first averaging thread of its own body)
      Lnb[b * E + e] = nbf;
    }
    if (m_terrain == 0) forces();   // plane: no per-body pass, the torques are complete only now
    if (a.recs && sub == a.substeps - 1) {
      // export the records of the last substep, [N][S][12] words
      for (int i = tid; i < S * E * kRecWords; i += kThreads) {
        int wd = i % kRecWords, rest = i / kRecWords, s = rest % S, ee = rest / S;
        int env_i = blockIdx.x * E + ee;
        if (env_i < N) {
          int word = Lreci[(s * kRecWords + wd) * E + ee];
          if (!Lreci[(s * kRecWords + 0) * E + ee]) word = (wd == 1 || wd == 2) ? -1 : 0;   // inactive: canonical record
          a.recs[((size_t)agent_at(env_i) * S + s) * kRecWords + wd] = word;
        }
      }
    }
    if constexpr (PC != 0) {
      if (a.pair_recs && sub == a.substeps - 1) {
        if (tid == 0) a.pair_count[blockIdx.x] = n_pc;
        if (tid < n_pc) {
          const int refs = __float_as_int(Lpq[tid * kPairWords + 1]);
          const int ra = refs & 0xffff, rb = (refs >> 16) & 0xffff;
          int32_t* o = a.pair_recs + ((size_t)blockIdx.x * kPairCap + tid) * 8;
          o[0] = agent_at(blockIdx.x * E + ra % E); o[1] = ra / E; o[2] = agent_at(blockIdx.x * E + rb % E); o[3] = rb / E;
          o[4] = __float_as_int(Lpq[tid * kPairWords + 2]); o[5] = __float_as_int(Lpq[tid * kPairWords + 3]);
          o[6] = __float_as_int(Lpq[tid * kPairWords + 5]); o[7] = __float_as_int(Lpq[tid * kPairWords + 4]);
        }
      }
    }
    __syncthreads();

    TMARK(4);
    // ---- D: row constants
    const int n_active = Lcount[0];
    // The joint rows and the contact rows are built inside the wavefront-uniform branches that use
    // them, so that the two sets of registers are never alive together.  Every lane of the
    // wavefronts concerned builds rows, the idle ones from a clamped index: a value assigned on
    // every path is not carried from one substep into the next in registers, as a conditionally
    // assigned one is.
    auto build_joint_side = [&]() {
     {
      const JointTab& jt = Ltjoint[js_j < J ? js_j : J - 1];
      const int e = js_e;
      const int ob = js_side ? jt.child : jt.parent;     // own body; -1: the static world
      const bool ghost = ob < 0;
      const int bo = ghost ? 0 : ob;                     // loads stay unconditional
      const float sg = js_side ? 1.0f : -1.0f;
      float xo[3], qo[4], iwo[6];
      for (int c = 0; c < 3; ++c) xo[c] = Lpos[(bo * 7 + c) * E + e];
      for (int c = 0; c < 4; ++c) qo[c] = Lpos[(bo * 7 + 3 + c) * E + e];
      for (int c = 0; c < 6; ++c) iwo[c] = Liw[(bo * kVS + c) * E + e];
      float no = NS ? 1.0f : Lnb[bo * E + e], imo = Ltbody[4 * bo + 3];   // (Newton: no mass splitting)
      if (ghost) {
        for (int c = 0; c < 3; ++c) xo[c] = 0.0f;
        qo[0] = 1.0f; qo[1] = qo[2] = qo[3] = 0.0f;
        for (int c = 0; c < 6; ++c) iwo[c] = 0.0f;
        no = 0.0f; imo = 0.0f;
      }
      // anchors: own one here, the other side's through the lane swap
      float Ro[9], lo[3], t0[3], pw[3], C[3], r[3];
      quat_to_mat(qo, Ro);
      for (int c = 0; c < 3; ++c) lo[c] = js_side ? jt.lb[c] : jt.la[c];
      mat_vec(Ro, lo, t0);
      for (int c = 0; c < 3; ++c) {
        pw[c] = xo[c] + t0[c];
        const float po = lane_swap1(pw[c]);
        C[c] = sg * (pw[c] - po);                        // child anchor minus parent anchor
        r[c] = 0.5f * (pw[c] + po) - xo[c];              // impulses act at the midpoint
      }
      // the world's side of a joint adds nothing to J v (whatever velocity its lane reads)
      const float sgl = ghost ? 0.0f : sg;
      for (int c = 0; c < 3; ++c) jr.sr[c] = sgl * r[c];
      jr.sg = sgl;
      jr.sv = sg * no * imo;
      const float inv_h = __builtin_amdgcn_rcpf(h), bh = p_beta_j * inv_h;
      for (int k = 0; k < 3; ++k) {
        float cr[3], y[3];
        cross_unit(r, k, cr);
        sym_vec(iwo, cr, y);
        const float kp = no * (imo + dot(cr, y));
        const float keff = kp + lane_swap1(kp);
        jr.pme[k] = keff > 0.0f ? -__builtin_amdgcn_rcpf(keff) : 0.0f;
        jr.pnb[k] = jr.pme[k] * (bh * C[k]);
        jr.pD[k] = keff; jr.pb[k] = bh * C[k];
        for (int c = 0; c < 3; ++c) jr.Y[k][c] = sg * no * y[c];
      }
      // joint angles from both orientations; axes live in the parent frame
      float qx[4], qa[4], qb[4], Ra[9], phi[3];
      for (int c = 0; c < 4; ++c) qx[c] = lane_swap1(qo[c]);
      for (int c = 0; c < 4; ++c) { qa[c] = js_side ? qx[c] : qo[c]; qb[c] = js_side ? qo[c] : qx[c]; }
      quat_to_mat(qa, Ra);
      rel_rotvec(qa, qb, phi);
      jr.onesided = 0;
      jr.upper = 0;
      for (int k = 0; k < 3; ++k) {
        float ak[3], z[3];
        mat_vec(Ra, jt.axes[k], ak);
        float th = dot(jt.axes[k], phi);
        float sgn = 1.0f, bias;
        if (jt.mode[k] == 0) {
          bias = bh * th;
        } else {
          float glo = th - jt.lo[k], ghi = jt.hi[k] - th, g;
          if (glo < ghi) { g = glo; } else { g = ghi; sgn = -1.0f; jr.upper |= 1 << k; }
          bias = g >= 0.0f ? g * inv_h : bh * g;
          jr.onesided |= 1 << k;
        }
        for (int c = 0; c < 3; ++c) ak[c] *= sgn;
        sym_vec(iwo, ak, z);
        const float kp = no * dot(ak, z);
        const float keff = kp + lane_swap1(kp);
        jr.ame[k] = keff > 0.0f ? -__builtin_amdgcn_rcpf(keff) : 0.0f;
        jr.anb[k] = jr.ame[k] * bias;
        jr.aD[k] = keff; jr.ab[k] = bias;
        jr.lam[k] = 0.0f;
        jr.nl[k] = jt.mode[k] == 0 ? -INFINITY : 0.0f;
        for (int c = 0; c < 3; ++c) { jr.sax[k][c] = sgl * ak[c]; jr.Z[k][c] = sg * no * z[c]; }
      }
     }
    };
    // contact k of the workgroup's list goes to thread kThreads-1-k (the joint threads sit at
    // the low end); contacts beyond one per thread start from zero impulse in LDS
    auto build_contact = [&]() {
      const int li = kThreads - 1 - tid;
      has_contact = li < n_active && li < n_reg;
      if (n_active > 0) {
        const int i = Llist[li < n_active ? li : n_active - 1];
        const int ee = i % E, sl = i / E, body = Ltslot[2 * sl];
        build_contact_rows(cr, Lrec, Liw, Lnb, sl, ee, E, body, Ltbody[4 * body + 3], h, p_beta_c, p_vdepen, NS != 0);
        if constexpr (WS != 0)
          for (int r = 0; r < 3; ++r) cr.lam[r] = p_warm * Lwc[(sl * 3 + r) * E + ee];
      } else {
        cr = ContactRows{};
      }
    };
    // capsule-capsule contact k of the sorted queue goes to two neighbouring lanes (body A, body B).
    // The contact lanes start right above the joint wavefronts (whose registers are busy with the
    // joint rows) and go up; what does not fit there goes below, into the joint wavefronts.
    const int pk_up = (kThreads - joint_threads) >> 1;
    const int pk = tid >= joint_threads ? (tid - joint_threads) >> 1 : pk_up + ((joint_threads - 1 - tid) >> 1);
    const bool has_pair = PC != 0 && pk < n_pc;
    auto build_pair = [&]() {
      if constexpr (PC != 0) {
        if (n_pc > 0) build_pair_side(pr, tid & 1, Lpq, Lpos, Liw, Lnb, Lorg, Ltbody, pk < n_pc ? pk : n_pc - 1, E, h, p_beta_c, p_vdepen);
        else pr = PairSide{};
      }
    };
    // impulses of the contacts beyond one per thread: slot k of a small array, or (warm start) the
    // contact's own place in the per-slot array, which already holds what was kept
    auto overflow_lam = [&](int k, int r) -> float& {
      if constexpr (WS != 0) { const int i = Llist[k]; return Lwc[(i / E * 3 + r) * E + i % E]; }
      else return Llam[3 * (k - n_reg) + r];
    };

    TMARK(5);
    // The copies a body averages: NJ joint sides (unused entries point at joint 0's copy with
    // weight 0) and its three contact slots (weight 0 when inactive).
    float g_inb = 0.0f;
    int gat_off[NJ], gat_slot[3];
    float gat_w[NJ + 3];
    {
      const int* tb = Ltjs + (g_on ? g_b : 0) * (kMaxBodyJoints + 3);
      const int g_njs = tb[0], g_slot0 = tb[1], g_nslots = tb[2];
      const float g_nbf = g_on ? Lnb[g_b * E + e] : 0.0f;
      g_inb = g_nbf > 0.0f ? 1.0f / g_nbf : 0.0f;
#pragma unroll
      for (int k = 0; k < NJ; ++k) {
        const bool used = g_on && k < g_njs;
        int js = used ? tb[3 + k] : 0;
        gat_off[k] = ((js >> 1) * kJS + (js & 1) * 6) * E + e;
        gat_w[k] = used ? 1.0f : 0.0f;
      }
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const bool used = g_on && k < g_nslots;
        gat_slot[k] = (g_slot0 + (used ? k : 0)) * kCS * E + e;
        gat_w[NJ + k] = used ? Lrec[((g_slot0 + k) * kRecWords + 10) * E + e] : 0.0f;
        if constexpr (NS != 0) gat_w[NJ + k] = (used && Lreci[((g_slot0 + k) * kRecWords + 0) * E + e]) ? 1.0f : 0.0f;
      }
    }
    // no body of this wavefront has more than two joint sides: its averages read two joint copies
    // instead of NJ (the same in all lanes, so the choice is a scalar branch)
    bool g_few = g_variants && NJ > 2;
#pragma unroll
    for (int k = 2; k < NJ; ++k) g_few = g_few && __ballot(gat_w[k] != 0.0f) == 0ull;
    // no slot of a body of this wavefront holds a contact in this substep: no slot copies are read
    const bool g_noc = g_variants && __ballot(gat_w[NJ] != 0.0f || gat_w[NJ + 1] != 0.0f || gat_w[NJ + 2] != 0.0f) == 0ull;
    // ---- S: sweeps
    // Wavefronts that hold joint threads run only the joint rows, the others only the contact
    // rows (a wave-uniform branch, so neither path carries the other's registers); both paths
    // execute the same two barriers per sweep.
    // components [c0, c0 + NC) of the average of body g_b (0..2 linear, 3..5 angular velocity)
    auto gather_part = [&](auto nc_tag, int c0) {
      constexpr int NC = decltype(nc_tag)::value;
      if (g_on && g_inb > 0.0f) {
        // every load is unconditional: unused entries read a valid location and enter the sum
        // with weight 0 (the copy arrays only ever hold finite numbers); all reads are issued
        // before the first use so their LDS latency is paid once
        // The average is taken over the copies' differences from the snapshot, (sum of w_k (copy_k -
        // v0)) / W added to v0: the differences are small next to the velocity itself, so the sum
        // rounds at their magnitude and the velocity is rounded once per sweep, where a weighted
        // sum of the copies themselves would round it once per copy.
        const int ho = c0 * E;
        float v0[NC], acc[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) v0[c] = Lvel[(g_b * kVS + c) * E + e + ho];
        // the first KJ joint copies and the three slots' copies
        auto sum_copies = [&](auto kj_tag, auto hc_tag) {
          constexpr int KJ = decltype(kj_tag)::value, HC = decltype(hc_tag)::value;
          float val[KJ + 3][NC];
#pragma unroll
          for (int k = 0; k < KJ; ++k)
#pragma unroll
            for (int c = 0; c < NC; ++c) val[k][c] = Loutj[gat_off[k] + ho + c * E];
          if constexpr (HC != 0) {
#pragma unroll
            for (int k = 0; k < 3; ++k)
#pragma unroll
              for (int c = 0; c < NC; ++c) val[KJ + k][c] = Loutc[gat_slot[k] + ho + c * E];
          }
          __builtin_amdgcn_sched_group_barrier(0x100, NC == 3 ? (KJ + 1 + 3 * HC) * 2 : KJ + 1 + 3 * HC, 0);  // the DS reads first
#pragma unroll
          for (int c = 0; c < NC; ++c) acc[c] = 0.0f;
#pragma unroll
          for (int k = 0; k < KJ; ++k)
#pragma unroll
            for (int c = 0; c < NC; ++c) acc[c] += gat_w[k] * (val[k][c] - v0[c]);
          if constexpr (HC != 0) {
#pragma unroll
            for (int k = 0; k < 3; ++k)
#pragma unroll
              for (int c = 0; c < NC; ++c) acc[c] += gat_w[NJ + k] * (val[KJ + k][c] - v0[c]);
          }
        };
        constexpr int kFew = NJ > 2 ? 2 : NJ;
        if constexpr (g_variants) {
          if (g_few && g_noc) sum_copies(std::integral_constant<int, kFew>{}, std::integral_constant<int, 0>{});
          else if (g_few) sum_copies(std::integral_constant<int, kFew>{}, std::integral_constant<int, 1>{});
          else sum_copies(std::integral_constant<int, NJ>{}, std::integral_constant<int, 1>{});
        } else {
          sum_copies(std::integral_constant<int, NJ>{}, std::integral_constant<int, 1>{});
        }
        if constexpr (PC != 0) {
          if (n_pc > 0) {
            if (gp_many) {
              // more contacts on this body than the list holds: walk the queue
              for (int k = 0; k < n_pc; ++k) {
                const int refs = __float_as_int(Lpq[k * kPairWords + 1]);
                if ((refs & 0xffff) == g_ref)
                  for (int c = 0; c < NC; ++c) acc[c] += Lpo[k * 12 + c0 + c];
                if (((refs >> 16) & 0xffff) == g_ref)
                  for (int c = 0; c < NC; ++c) acc[c] += Lpo[k * 12 + 6 + c0 + c];
              }
              for (int c = 0; c < NC; ++c) acc[c] -= gp_wsum * v0[c];   // (their copies come multiplied by the weights)
            } else {
              // the (weighted) copies of the listed contacts (the list holds the used entries first);
              // unused entries point at zeros
              auto sum_pairs = [&](auto kp_tag) {
                constexpr int KP = decltype(kp_tag)::value;
                float pv[KP][NC];
#pragma unroll
                for (int j = 0; j < KP; ++j)
#pragma unroll
                  for (int c = 0; c < NC; ++c) pv[j][c] = Lpo[gp_off[j] + c0 + c];
#pragma unroll
                for (int j = 0; j < KP; ++j)
#pragma unroll
                  for (int c = 0; c < NC; ++c) acc[c] += pv[j][c];
              };
              if constexpr (g_variants) {
                if (gp_few) sum_pairs(std::integral_constant<int, kPairFew>{});
                else sum_pairs(std::integral_constant<int, kPairList>{});
              } else {
                sum_pairs(std::integral_constant<int, kPairList>{});
              }
              // (the listed copies come multiplied by their weights: the snapshot's share goes off in one piece)
#pragma unroll
              for (int c = 0; c < NC; ++c) acc[c] -= gp_wsum * v0[c];
            }
          }
        }
        for (int c = 0; c < NC; ++c) Lvel[(g_b * kVS + c) * E + e + ho] = v0[c] + acc[c] * g_inb;
      }
    };
    // one sweep of this thread's side of a capsule-capsule contact, if it has one
    // (a capsule-capsule contact starts every substep without impulses: in the warm start's
    // sweep -1 its copies are the bodies' velocities as they are)
    auto pair_sweep = [&](bool relax) {
      if constexpr (PC != 0) {
        if (has_pair) {
          float vo[3], wo[3];
          for (int c = 0; c < 3; ++c) { vo[c] = Lvel[pr.off + c * E]; wo[c] = Lvel[pr.off + (3 + c) * E]; }
          if (relax) relax_pair_side(pr, p_mu, vo, wo);
          const int po = (2 * pk + (tid & 1)) * 6;
          for (int c = 0; c < 3; ++c) { Lpo[po + c] = pr.wk * vo[c]; Lpo[po + 3 + c] = pr.wk * wo[c]; }
        }
      }
    };
    auto gather = [&]() {
      if constexpr (g_three) {
        gather_part(std::integral_constant<int, 2>{}, 2 * g_half);   // two components per thread
      } else {
        gather_part(std::integral_constant<int, 3>{}, 3 * g_half);   // linear or angular half
        if (!g_split) gather_part(std::integral_constant<int, 3>{}, 3);
      }
    };
    // Warm start: sweep -1 relaxes nothing; every block applies the impulses it starts from (the
    // kept ones times the share) to its copies, and the average of the copies hands every body
    // the plain sum of them, as a sweep does with the increments.
    if constexpr (NS != 0) {
      // ---- S (Newton): the paper's solver (Section 3.1), a non-smooth Newton method whose every
      // iteration is solved by a fixed number of preconditioned conjugate-residual iterations.
      // Unknowns: the impulses lambda of all rows; u = v* + M^-1 J^T lambda; residual s = J u + bias.
      // Bilateral rows ask for s = 0; one-sided rows for min(lambda, s / D) = 0 (D the diagonal of
      // J M^-1 J^T); a friction pair follows the smooth isotropic Coulomb law lambda_t = -mu lambda_n
      // s_t / |s_t|_eps, which enters an iteration as a damper s_t + c lambda_t = 0 with the
      // compliance c = |s_t|_eps / (mu lambda_n) of the current iterate.  The operator is applied
      // through the bodies in the two phases of a Jacobi sweep: every block writes the velocity
      // change its rows' impulses give its bodies (scatter), a barrier, every body adds up its
      // blocks' contributions (gather), a barrier, every row takes J times the result.  Every row's
      // vectors stay in the registers of its lane (both lanes of a joint hold the same values).
      // Dot products over the rows of an env: every block leaves its partial sum in an LDS entry of
      // its own, one thread per env adds them up in block order, so the result does not depend on
      // which wavefront ran first.
      float* LU = lds + P.nu;        // [B][kVS][E]: M^-1 J^T x (plus v* when asked for)
      float* Lred = lds + P.nred;    // [3][J + S][E]: partial sums of the blocks
      float* Lsum = lds + P.nsum;    // [3][8][E]: sums over an eighth of the blocks each
      const int nblk = J + S;
      const float p_reg = M.newton_reg;
      const int n_kry = M.krylov;
      constexpr float kFrictionEps = 1e-3f;   // m/s
      constexpr int kRedParts = 4;            // (J + S <= 64 blocks: at most sixteen per part)
      const bool jrole = joint_wave;
      if constexpr (WS != 0) {
        // a slot that is not active in this substep hands nothing on to the next one
        for (int i = tid; i < S * E; i += kThreads)
          if (!Lreci[(i / E * kRecWords + 0) * E + i % E])
            for (int r = 0; r < 3; ++r) Lwc[(i / E * 3 + r) * E + i % E] = 0.0f;
      }
      if (jrole) build_joint_side(); else build_contact();
      for (int i = tid; i < 3 * nblk * E; i += kThreads) Lred[i] = 0.0f;   // inactive slots contribute nothing
      const int nr = jrole ? 6 : 3;
      const bool active = jrole ? js_on : has_contact;      // this lane holds rows
      // The row constants of either role in one array, so that the two roles share registers:
      //   joint side: K[0..2] lever arm, K[3] linear response, K[4] sign, K[5..13] angular response of
      //               the positional rows, K[14..22] the three axes, K[23..31] their angular response;
      //   contact:    K[0..8] directions n, t1, t2, K[9..17] lever x direction, K[18..26] angular
      //               response, K[27] linear response.
      float K[32], Dg[6], bs[6];
      int ones = 0, uppers = 0, c_body = 0, c_slot_e = 0;
      if (jrole) {
        for (int k = 0; k < 3; ++k) {
          K[k] = jr.sr[k];
          for (int c = 0; c < 3; ++c) { K[5 + 3 * k + c] = jr.Y[k][c]; K[14 + 3 * k + c] = jr.sax[k][c]; K[23 + 3 * k + c] = jr.Z[k][c]; }
          Dg[k] = jr.pD[k]; bs[k] = jr.pb[k]; Dg[3 + k] = jr.aD[k]; bs[3 + k] = jr.ab[k];
        }
        K[3] = jr.sv; K[4] = jr.sg;
        ones = jr.onesided;
        uppers = jr.upper;
      } else {
        for (int r = 0; r < 3; ++r) {
          for (int c = 0; c < 3; ++c) { K[3 * r + c] = cr.dir[r][c]; K[9 + 3 * r + c] = cr.ang[r][c]; K[18 + 3 * r + c] = cr.Y[r][c]; }
          Dg[r] = cr.D[r]; bs[r] = r == 0 ? cr.bias : 0.0f; Dg[3 + r] = 0.0f; bs[3 + r] = 0.0f;
        }
        K[27] = cr.ls; K[28] = K[29] = K[30] = K[31] = 0.0f;
        c_body = cr.body; c_slot_e = cr.slot_e;
      }
      const int my_e = jrole ? js_e : (c_slot_e % E);
      const int my_blk = jrole ? (js_j < J ? js_j : 0) : J + c_slot_e / E;
      const bool writes_partial = jrole ? (js_on && js_side == 0) : has_contact;
      const int j_ob = jrole ? (js_side ? Ltjoint[js_j < J ? js_j : 0].child : Ltjoint[js_j < J ? js_j : 0].parent) : 0;
      const int j_bo = j_ob < 0 ? 0 : j_ob;
      // the velocity change of the lane's own body from the impulses xv of its rows -> its copy
      auto scatter = [&](const float* xv) {
        if (jrole) {
          if (js_on && j_ob >= 0) {
            float dw[3] = {0.0f, 0.0f, 0.0f};
            for (int k = 0; k < 3; ++k)
              for (int c = 0; c < 3; ++c) dw[c] += K[5 + 3 * k + c] * xv[k] + K[23 + 3 * k + c] * xv[3 + k];
            for (int c = 0; c < 3; ++c) {
              Loutj[(js_j * kJS + js_side * 6 + c) * E + js_e] = K[3] * xv[c];
              Loutj[(js_j * kJS + js_side * 6 + 3 + c) * E + js_e] = dw[c];
            }
          }
        } else if (has_contact) {
          const int ee = c_slot_e % E, sl = c_slot_e / E;
          float dv[3] = {0.0f, 0.0f, 0.0f}, dw[3] = {0.0f, 0.0f, 0.0f};
          for (int r = 0; r < 3; ++r)
            for (int c = 0; c < 3; ++c) { dv[c] += K[27] * K[3 * r + c] * xv[r]; dw[c] += K[18 + 3 * r + c] * xv[r]; }
          for (int c = 0; c < 3; ++c) { Loutc[(sl * kCS + c) * E + ee] = dv[c]; Loutc[(sl * kCS + 3 + c) * E + ee] = dw[c]; }
        }
      };
      // every body: the plain sum of its blocks' contributions (in static order), on top of the
      // velocities the solve started from when `with_base`
      // (two threads per body, linear and angular half: the host only picks launch shapes where
      //  2 B E threads exist; all reads are issued before the first use)
      auto gather_sum = [&](bool with_base, float* dst) {
        if (!g_on) return;
        const int ho = 3 * g_half * E;
        float val[NJ + 3][3], base[3];
#pragma unroll
        for (int c = 0; c < 3; ++c) base[c] = with_base ? Lvel[(g_b * kVS + c) * E + e + ho] : 0.0f;
#pragma unroll
        for (int k = 0; k < NJ; ++k)
#pragma unroll
          for (int c = 0; c < 3; ++c) val[k][c] = Loutj[gat_off[k] + ho + c * E];
#pragma unroll
        for (int k = 0; k < 3; ++k)
#pragma unroll
          for (int c = 0; c < 3; ++c) val[NJ + k][c] = Loutc[gat_slot[k] + ho + c * E];
#pragma unroll
        for (int c = 0; c < 3; ++c) {
          float acc = 0.0f;
#pragma unroll
          for (int k = 0; k < NJ + 3; ++k) acc += gat_w[k] * val[k][c];
          dst[(g_b * kVS + c) * E + e + ho] = base[c] + acc;
        }
      };
      // y = J (body vectors in src) for the lane's rows
      auto rows_of = [&](const float* src, float* y) {
        const int bo = jrole ? j_bo : c_body, ee = my_e;
        float uv[3], uw[3];
        for (int c = 0; c < 3; ++c) { uv[c] = src[(bo * kVS + c) * E + ee]; uw[c] = src[(bo * kVS + 3 + c) * E + ee]; }
        if (jrole) {
#pragma unroll
          for (int k = 0; k < 3; ++k) {
            const float p0 = K[4] * uv[k] + cross_unit_dot(K, k, uw);
            y[k] = p0 + lane_swap1(p0);
            const float p1 = K[14 + 3 * k] * uw[0] + K[15 + 3 * k] * uw[1] + K[16 + 3 * k] * uw[2];
            y[3 + k] = p1 + lane_swap1(p1);
          }
        } else {
          for (int r = 0; r < 3; ++r) {
            y[r] = (K[3 * r] * uv[0] + K[3 * r + 1] * uv[1] + K[3 * r + 2] * uv[2]) +
                   (K[9 + 3 * r] * uw[0] + K[10 + 3 * r] * uw[1] + K[11 + 3 * r] * uw[2]);
            y[3 + r] = 0.0f;
          }
        }
      };
      // totals over the rows of the lane's env of up to three products
      // (indices of the adding threads, worked out once)
      const bool red_on = tid < 3 * kRedParts * E;
      const int red_q = tid / (kRedParts * E), red_r = tid - red_q * (kRedParts * E), red_part = red_r / E, red_e = red_r - red_part * E;
      const int red_per = (nblk + kRedParts - 1) / kRedParts;
      const int red_src = (red_q * nblk + red_part * red_per) * E + red_e, red_n = min(red_per, nblk - red_part * red_per);
      const int red_dst = (red_q * kRedParts + red_part) * E + red_e;
      auto reduce3 = [&](float pa, float pb, float pc, float& ta, float& tb, float& tc) {
        if (writes_partial) {
          Lred[(0 * nblk + my_blk) * E + my_e] = pa; Lred[(1 * nblk + my_blk) * E + my_e] = pb; Lred[(2 * nblk + my_blk) * E + my_e] = pc;
        }
        __syncthreads();
        // four threads per product and env add up a quarter of the blocks each (reads issued together)
        if (red_on) {
          float vals[16];
#pragma unroll
          for (int k = 0; k < 16; ++k) vals[k] = k < red_n ? Lred[red_src + k * E] : 0.0f;
          float sm = 0.0f;
#pragma unroll
          for (int k = 0; k < 16; ++k) sm += vals[k];
          Lsum[red_dst] = sm;
        }
        __syncthreads();
        // every lane adds the four partial sums of its env, in order
        float vals[3 * kRedParts];
#pragma unroll
        for (int k = 0; k < 3 * kRedParts; ++k) vals[k] = Lsum[k * E + my_e];
        ta = (vals[0] + vals[1]) + (vals[2] + vals[3]);
        tb = (vals[4] + vals[5]) + (vals[6] + vals[7]);
        tc = (vals[8] + vals[9]) + (vals[10] + vals[11]);
      };
      float lam[6] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
      if constexpr (WS != 0) {
        // Warm start: the first iterate is the share of what the rows ended the last substep with
        // (a limit row only if it stands for the same limit as then; a slot that was not active
        // then holds zero).
        if (jrole) {
          if (js_on) {
            for (int k = 0; k < 3; ++k) lam[k] = p_warm * Lwj[(js_j * 6 + k) * E + js_e];
            for (int k = 0; k < 3; ++k) {
              const float kept = Lwj[(js_j * 6 + 3 + k) * E + js_e];
              float l0 = p_warm * kept;
              if ((ones >> k) & 1) {
                const bool was_upper = __float_as_int(kept) < 0, is_upper = (uppers >> k) & 1;
                l0 = was_upper == is_upper ? fabsf(l0) : 0.0f;
              }
              lam[3 + k] = l0;
            }
          }
        } else if (has_contact) {
          for (int r = 0; r < 3; ++r) lam[r] = cr.lam[r];
        }
      }
      for (int it = 0; it < a.iterations; ++it) {
        float sres[6], known[6], cp[6], ipd[6], tmp[6];
        int on = 0;
        // residual of the current iterate
        scatter(lam);
        __syncthreads();
        gather_sum(true, LU);
        __syncthreads();
        rows_of(LU, sres);
        for (int k = 0; k < 6; ++k) { sres[k] += bs[k]; known[k] = 0.0f; cp[k] = 0.0f; }
        // the branch every row is on
        if (jrole) {
          on = 7;
          for (int k = 0; k < 3; ++k) {
            const bool one = (ones >> k) & 1;
            const bool s_branch = !one || (Dg[3 + k] > 0.0f && lam[3 + k] - sres[3 + k] / Dg[3 + k] > 0.0f);
            if (s_branch) on |= 8 << k; else known[3 + k] = -lam[3 + k];
          }
        } else {
          if (Dg[0] > 0.0f && lam[0] - sres[0] / Dg[0] > 0.0f) on |= 1; else known[0] = -lam[0];
          const float rad = p_mu * lam[0];
          if (rad > 0.0f) {
            on |= 6;
            cp[1] = cp[2] = sqrtf(sres[1] * sres[1] + sres[2] * sres[2] + kFrictionEps * kFrictionEps) / rad;
          } else { known[1] = -lam[1]; known[2] = -lam[2]; }
        }
        // (ipd: inverse of the preconditioner's diagonal on the rows of the "s" branch, 0 elsewhere)
        for (int k = 0; k < 6; ++k) {
          const float pdk = Dg[k] * (1.0f + p_reg) + cp[k];
          if (!(pdk > 0.0f) || k >= nr || !active) on &= ~(1 << k);
          ipd[k] = ((on >> k) & 1) ? 1.0f / pdk : 0.0f;
        }
        // right-hand side of the rows on the "s" branch: -s - c lambda - A known
        scatter(known);
        __syncthreads();
        gather_sum(false, LU);
        __syncthreads();
        rows_of(LU, tmp);
        float x[6], z[6], pv[6], q[6], az[6];
        for (int k = 0; k < 6; ++k) {
          const bool o = (on >> k) & 1;
          const float rhs = o ? -sres[k] - cp[k] * lam[k] - tmp[k] : 0.0f;
          x[k] = 0.0f; z[k] = rhs * ipd[k]; pv[k] = z[k];
        }
        // (A + reg D + c) z on the rows of the "s" branch
        auto apply_hat = [&](const float* xv, float* y) {
          scatter(xv);
          __syncthreads();
          gather_sum(false, LU);
          __syncthreads();
          rows_of(LU, y);
          for (int k = 0; k < 6; ++k) y[k] = ((on >> k) & 1) ? y[k] + (p_reg * Dg[k] + cp[k]) * xv[k] : 0.0f;
        };
        apply_hat(z, az);
        float gamma, den, unused;
        {
          float pa = 0.0f, pb = 0.0f;
          for (int k = 0; k < 6; ++k) { q[k] = az[k]; pa += z[k] * az[k]; pb += az[k] * az[k] * ipd[k]; }
          reduce3(pa, pb, 0.0f, gamma, den, unused);
        }
        const float gamma0 = gamma;
        bool done = false;
        for (int kk = 0; kk < n_kry; ++kk) {
          done = done || !(den > 0.0f) || !(gamma > 1e-12f * gamma0);
          const float alpha = done ? 0.0f : gamma / den;
          for (int k = 0; k < 6; ++k) { x[k] += alpha * pv[k]; z[k] -= alpha * q[k] * ipd[k]; }   // (all zero off the "s" branch)
          if (kk == n_kry - 1) break;       // (the last iteration's operator product would not be used)
          apply_hat(z, az);
          float pa = 0.0f, pb = 0.0f, pc = 0.0f, ta, tb, tc;
          for (int k = 0; k < 6; ++k) {
            pa += z[k] * az[k];
            pb += az[k] * az[k] * ipd[k]; pc += az[k] * q[k] * ipd[k];
          }
          reduce3(pa, pb, pc, ta, tb, tc);
          if (!done) {
            const float beta = ta / gamma;
            for (int k = 0; k < 6; ++k) { pv[k] = z[k] + beta * pv[k]; q[k] = az[k] + beta * q[k]; }
            den = tb + 2.0f * beta * tc + beta * beta * den;     // q . q / pd of the new q
            gamma = ta;
          }
        }
        // update, then back into the feasible set
        for (int k = 0; k < 6; ++k) lam[k] += ((on >> k) & 1) ? x[k] : known[k];
        if (jrole) {
          for (int k = 0; k < 3; ++k) if ((ones >> k) & 1) lam[3 + k] = fmaxf(lam[3 + k], 0.0f);
        } else {
          lam[0] = fmaxf(lam[0], 0.0f);
          const float rad = p_mu * lam[0], nrm = sqrtf(lam[1] * lam[1] + lam[2] * lam[2]);
          if (nrm > rad) { const float sc = nrm > 0.0f ? rad / nrm : 0.0f; lam[1] *= sc; lam[2] *= sc; }
        }
      }
      // the solved velocities: v* + M^-1 J^T lambda
      scatter(lam);
      __syncthreads();
      gather_sum(true, Lvel);
      __syncthreads();
      if constexpr (WS != 0) {
        // kept for the next substep (both lanes of a joint hold the same impulses; everybody has
        // read the old ones before the barriers above)
        if (jrole) {
          if (js_on && js_side == 0) {
            for (int k = 0; k < 3; ++k) Lwj[(js_j * 6 + k) * E + js_e] = lam[k];
            for (int k = 0; k < 3; ++k)
              Lwj[(js_j * 6 + 3 + k) * E + js_e] = ((ones & uppers) >> k) & 1 ? -lam[3 + k] : lam[3 + k];
          }
        } else if (has_contact) {
          const int ee = c_slot_e % E, sl = c_slot_e / E;
          for (int r = 0; r < 3; ++r) Lwc[(sl * 3 + r) * E + ee] = lam[r];
        }
      }
    } else
    if (joint_wave) {
      build_joint_side();
      build_pair();
      TMARK(17);
      float acc[3] = {0.0f, 0.0f, 0.0f};   // impulses of the positional rows so far (kept for the next substep)
      if constexpr (WS != 0) {
        const int jj = js_j < J ? js_j : J - 1;
        for (int k = 0; k < 3; ++k) acc[k] = p_warm * Lwj[(jj * 6 + k) * E + js_e];
        for (int k = 0; k < 3; ++k) {
          const float kept = Lwj[(jj * 6 + 3 + k) * E + js_e];
          float l0 = p_warm * kept;
          if (jr.onesided & (1 << k)) {
            // kept for the other limit: it would push the wrong way
            const bool was_upper = __float_as_int(kept) < 0, is_upper = (jr.upper >> k) & 1;
            l0 = was_upper == is_upper ? fabsf(l0) : 0.0f;
          }
          jr.lam[k] = l0;
          if (jr.onesided & (1 << k)) jr.nl[k] = -l0;
        }
      }
      // own body's velocity rows, found once (the world's side of a joint reads body 0's and writes
      // nothing): looked up inside the loop, the body index costs every sweep an LDS round trip
      // ahead of the reads that depend on it
      const int js_ob = js_side ? Ltjoint[js_j < J ? js_j : 0].child : Ltjoint[js_j < J ? js_j : 0].parent;
      const int js_voff = (js_ob < 0 ? 0 : js_ob) * kVS * E + js_e;
      for (int it = WS ? -1 : 0; it < a.iterations; ++it) {
        if (js_on) {
          const int e = js_e;
          const int ob = js_ob;
          float vo[3], wo[3];
          for (int c = 0; c < 3; ++c) { vo[c] = Lvel[js_voff + c * E]; wo[c] = Lvel[js_voff + (3 + c) * E]; }
  #pragma unroll
          for (int k = 0; k < 3; ++k) {
            float dl;
            if (WS != 0 && it < 0) {
              dl = acc[k];
            } else {
              const float part = jr.sg * vo[k] + cross_unit_dot(jr.sr, k, wo);
              const float jv = part + lane_swap1(part);
              dl = jv * jr.pme[k] + jr.pnb[k];
              if constexpr (WS != 0) acc[k] += dl;
            }
            vo[k] += jr.sv * dl;
            for (int c = 0; c < 3; ++c) wo[c] += jr.Y[k][c] * dl;
          }
  #pragma unroll
          for (int k = 0; k < 3; ++k) {
            float dl;
            if (WS != 0 && it < 0) {
              dl = jr.lam[k];
            } else {
              const float part = dot(jr.sax[k], wo);
              const float jv = part + lane_swap1(part);
              // a limit row's impulse stays >= 0: max(lam + dl, 0) - lam = max(dl, -lam)
              dl = fmaxf(jv * jr.ame[k] + jr.anb[k], jr.nl[k]);
              jr.nl[k] -= dl;
              if constexpr (WS != 0) jr.lam[k] += dl;
            }
            for (int c = 0; c < 3; ++c) wo[c] += jr.Z[k][c] * dl;
          }
          if (ob >= 0)
            for (int c = 0; c < 3; ++c) {
              Loutj[(js_j * kJS + js_side * 6 + c) * E + e] = vo[c];
              Loutj[(js_j * kJS + js_side * 6 + 3 + c) * E + e] = wo[c];
            }
        }
        pair_sweep(!(WS != 0 && it < 0));
        __syncthreads();
        gather();
        __syncthreads();
      }
      if constexpr (WS != 0) {
        // (both lanes of a joint hold the same impulses; the two sit in one wavefront, so the
        // parent side's stores follow both lanes' reads above)
        if (js_on && js_side == 0) {
          for (int k = 0; k < 3; ++k) Lwj[(js_j * 6 + k) * E + js_e] = acc[k];
          for (int k = 0; k < 3; ++k)
            Lwj[(js_j * 6 + 3 + k) * E + js_e] = ((jr.onesided & jr.upper) >> k) & 1 ? -jr.lam[k] : jr.lam[k];
        }
      }
    } else {
      if constexpr (WS != 0) {
        // a slot that is not active in this substep hands nothing on to the next one (nobody
        // reads its entries now; the records are final since the barrier after the contact search)
        for (int i = tid - joint_threads; i < S * E; i += n_reg)
          if (!Lreci[(i / E * kRecWords + 0) * E + i % E])
            for (int r = 0; r < 3; ++r) Lwc[(i / E * 3 + r) * E + i % E] = 0.0f;
      }
      build_contact();
      build_pair();
      // the starting impulses of the contacts beyond one per thread are set by the thread that
      // relaxes them in every sweep below (same index mapping), so no other thread's store is read
      for (int k = n_reg + (kThreads - 1 - tid); k < n_active; k += n_reg)
        for (int r = 0; r < 3; ++r) overflow_lam(k, r) = WS ? p_warm * overflow_lam(k, r) : 0.0f;
      for (int it = WS ? -1 : 0; it < a.iterations; ++it) {
        if (has_contact) {
          const int ee = cr.slot_e % E, sl = cr.slot_e / E;
          float vv[3], ww[3];
          for (int k = 0; k < 3; ++k) { vv[k] = Lvel[(cr.body * kVS + k) * E + ee]; ww[k] = Lvel[(cr.body * kVS + 3 + k) * E + ee]; }
          if (WS != 0 && it < 0) apply_contact_impulses(cr, vv, ww);
          else relax_contact(cr, p_mu, vv, ww);
          for (int k = 0; k < 3; ++k) { Loutc[(sl * kCS + k) * E + ee] = vv[k]; Loutc[(sl * kCS + 3 + k) * E + ee] = ww[k]; }
        }
        for (int k = n_reg + (kThreads - 1 - tid); k < n_active; k += n_reg) {
          // rare: more active contacts in the workgroup than threads; rows rebuilt from the record
          const int i = Llist[k];
          const int ee = i % E, sl = i / E, body = Ltslot[2 * sl];
          ContactRows c2;
          build_contact_rows(c2, Lrec, Liw, Lnb, sl, ee, E, body, Ltbody[4 * body + 3], h, p_beta_c, p_vdepen);
          for (int r = 0; r < 3; ++r) c2.lam[r] = overflow_lam(k, r);
          float vv[3], ww[3];
          for (int r = 0; r < 3; ++r) { vv[r] = Lvel[(body * kVS + r) * E + ee]; ww[r] = Lvel[(body * kVS + 3 + r) * E + ee]; }
          if (WS != 0 && it < 0) apply_contact_impulses(c2, vv, ww);
          else relax_contact(c2, p_mu, vv, ww);
          for (int r = 0; r < 3; ++r) overflow_lam(k, r) = c2.lam[r];
          for (int r = 0; r < 3; ++r) { Loutc[(sl * kCS + r) * E + ee] = vv[r]; Loutc[(sl * kCS + 3 + r) * E + ee] = ww[r]; }
        }
        pair_sweep(!(WS != 0 && it < 0));
        __syncthreads();
        gather();
        __syncthreads();
      }
      if constexpr (WS != 0) {
        if (has_contact) {
          const int ee = cr.slot_e % E, sl = cr.slot_e / E;
          for (int r = 0; r < 3; ++r) Lwc[(sl * 3 + r) * E + ee] = cr.lam[r];
        }
      }
    }

    TMARK(6);
    // ---- E: damping, angular-velocity cap, positions
    if (is_body) {
      // the pose was parked in LDS during the sweeps (unchanged since phase A)
      for (int c = 0; c < 3; ++c) x[c] = Lpos[(b * 7 + c) * E + e];
      for (int c = 0; c < 4; ++c) q[c] = Lpos[(b * 7 + 3 + c) * E + e];
      // the solved velocities were left in LDS by the threads that averaged them
      for (int c = 0; c < 3; ++c) { v[c] = Lvel[(b * kVS + c) * E + e]; w[c] = Lvel[(b * kVS + 3 + c) * E + e]; }
      float dl = __builtin_amdgcn_rcpf(1.0f + h * p_clin), da = __builtin_amdgcn_rcpf(1.0f + h * p_cang);
      for (int c = 0; c < 3; ++c) { v[c] *= dl; w[c] *= da; }
      const float w2 = dot(w, w);
      if (w2 > p_wmax * p_wmax) { float sc = p_wmax * __builtin_amdgcn_rsqf(w2); for (int c = 0; c < 3; ++c) w[c] *= sc; }
      for (int c = 0; c < 3; ++c) x[c] += h * v[c];
      float dq[4];
      dq[0] = -w[0] * q[1] - w[1] * q[2] - w[2] * q[3];
      dq[1] = w[0] * q[0] + w[1] * q[3] - w[2] * q[2];
      dq[2] = -w[0] * q[3] + w[1] * q[0] + w[2] * q[1];
      dq[3] = w[0] * q[2] - w[1] * q[1] + w[2] * q[0];
      float hh = 0.5f * h;
      for (int c = 0; c < 4; ++c) q[c] += hh * dq[c];
      float inv = __builtin_amdgcn_rsqf(q[0] * q[0] + q[1] * q[1] + q[2] * q[2] + q[3] * q[3]);
      for (int c = 0; c < 4; ++c) q[c] *= inv;
    }
    __syncthreads();  // the next substep overwrites pose, counters and lists read above
    TMARK(7);
  }

  // ---- store state, publish final pose/velocity for packing
  __syncthreads();
  TMARK(8);
  if (is_body) {
    float* st = a.state + (size_t)b * N + agent;
    const size_t fs = (size_t)B * N;
    if (a.substeps > 0) {
      st[0 * fs] = x[0]; st[1 * fs] = x[1]; st[2 * fs] = x[2];
      st[3 * fs] = q[0]; st[4 * fs] = q[1]; st[5 * fs] = q[2]; st[6 * fs] = q[3];
      st[7 * fs] = v[0]; st[8 * fs] = v[1]; st[9 * fs] = v[2];
      st[10 * fs] = w[0]; st[11 * fs] = w[1]; st[12 * fs] = w[2];
    }
    for (int c = 0; c < 3; ++c) Lpos[(b * 7 + c) * E + e] = x[c];
    for (int c = 0; c < 4; ++c) Lpos[(b * 7 + 3 + c) * E + e] = q[c];
    for (int c = 0; c < 3; ++c) { Lvel[(b * kVS + c) * E + e] = v[c]; Lvel[(b * kVS + 3 + c) * E + e] = w[c]; }
  }
  __syncthreads();

  // The observation is packed once for every env (pass 0).  With the task logic's auto-reset, an
  // env whose episode ends in pass 0 is put back to a fresh initial state right here, and pass 1
  // packs the observation of that state for it (no action, no contact), so the caller gets the
  // finished step's reward and done flag next to the first observation of the next episode.
  int* Lrst = reinterpret_cast<int*>(Lpush);   // [E]: env was reset in pass 0 (the pushes are no longer read)
  const bool may_reset = a.task.enabled && a.task.auto_reset && a.count_step;
  // ---- observation vector (Table 2 "Ours"), per joint part
  auto pack_joints = [&](auto pass_c) {
  constexpr int pass = decltype(pass_c)::value;
  if (is_joint && (pass == 0 || Lrst[e])) {
    const JointTab& jt = Ltjoint[idx];
    const int pa = jt.parent, pb = jt.child;
    float qa[4] = {1, 0, 0, 0}, wa[3] = {0, 0, 0}, qb[4], wb[3];
    if (pa >= 0) {
      for (int c = 0; c < 4; ++c) qa[c] = Lpos[(pa * 7 + 3 + c) * E + e];
      for (int c = 0; c < 3; ++c) wa[c] = Lvel[(pa * kVS + 3 + c) * E + e];
    }
    for (int c = 0; c < 4; ++c) qb[c] = Lpos[(pb * 7 + 3 + c) * E + e];
    for (int c = 0; c < 3; ++c) wb[c] = Lvel[(pb * kVS + 3 + c) * E + e];
    float Ra[9], phi[3];
    quat_to_mat(qa, Ra);
    rel_rotvec(qa, qb, phi);
    float dw[3] = {wb[0] - wa[0], wb[1] - wa[1], wb[2] - wa[2]};
    for (int k = 0; k < 3; ++k) {
      if (jt.mode[k] != 1) continue;
      int ai = jt.act[k];
      float ak[3];
      mat_vec(Ra, jt.axes[k], ak);
      float th = dot(jt.axes[k], phi);
      Lobs[e * obs_dim + 11 + ai] = th;
      Lobs[e * obs_dim + 11 + D + ai] = dot(ak, dw);
      Lobs[e * obs_dim + 11 + 2 * D + ai] = pass ? 0.0f : Lu[ai * E + e];
      float g = fminf(th - jt.lo[k], jt.hi[k] - th);
      Llim[ai * E + e] = g <= 0.0f ? 1 : 0;
    }
  }
  };
  // ---- root part, reward (Eq. 1-3), done (Section 4.1); returns whether the env was reset
  auto pack_root = [&](auto pass_c) -> bool {
  constexpr int pass = decltype(pass_c)::value;
  bool reset_now = false;
  if (tid < E && (blockIdx.x * E + tid) < N && (pass == 0 || Lrst[tid])) {
    const int ee = tid, env_e = agent_at(blockIdx.x * E + tid);
    const int rb = M.root;
    float rx[3], rq[4], rv[3], rw[3];
    for (int c = 0; c < 3; ++c) rx[c] = Lpos[(rb * 7 + c) * E + ee];
    for (int c = 0; c < 4; ++c) rq[c] = Lpos[(rb * 7 + 3 + c) * E + ee];
    for (int c = 0; c < 3; ++c) { rv[c] = Lvel[(rb * kVS + c) * E + ee]; rw[c] = Lvel[(rb * kVS + 3 + c) * E + ee]; }
    float ox = a.origins[3 * env_e], oy = a.origins[3 * env_e + 1], oz = a.origins[3 * env_e + 2];
    float height = rx[2];
    if (M.terrain_kind == 1) height = rx[2] + oz - terrain_height(M, a.heights, rx[0] + ox, rx[1] + oy);
    float qw = rq[0], qx = rq[1], qy = rq[2], qz = rq[3];
    float roll = atan2f(2.0f * (qw * qx + qy * qz), 1.0f - 2.0f * (qx * qx + qy * qy));
    float sp = fminf(fmaxf(2.0f * (qw * qy - qz * qx), -1.0f), 1.0f);
    float pitch = asinf(sp);
    float yaw = atan2f(2.0f * (qw * qz + qx * qy), 1.0f - 2.0f * (qy * qy + qz * qz));
    float tx = a.targets[2 * env_e] - rx[0], ty = a.targets[2 * env_e + 1] - rx[1];
    float psi = atan2f(ty, tx) - yaw;
    float sps = sinf(psi), cps = cosf(psi);
    float* o = Lobs + ee * obs_dim;
    o[0] = height; o[1] = roll; o[2] = pitch;
    o[3] = rv[0]; o[4] = rv[1]; o[5] = rv[2];
    o[6] = rw[0]; o[7] = rw[1]; o[8] = rw[2];
    o[9] = sps; o[10] = cps;
    int n_feet = 0;
    for (int f = 0; f < F; ++f) {
      const BodyTab& bt = M.bodies[M.feet[f]];
      int flag = 0;
      for (int k = 0; k < bt.n_slots; ++k) {
        int s = bt.slot0 + k;
        if (pass == 0 && Lreci[(s * kRecWords + 0) * E + ee] && Lrec[(s * kRecWords + 3) * E + ee] <= 0.005f) flag = 1;
      }
      o[11 + 3 * D + f] = (float)flag;
      n_feet += flag;
    }
    float l1 = 0.0f, l2 = 0.0f;
    int n_lim = 0;
    for (int d = 0; d < D; ++d) {
      float uu = Lu[d * E + ee];
      l1 += fabsf(uu); l2 += uu * uu;
      n_lim += Llim[d * E + ee];
    }
    float tn = sqrtf(tx * tx + ty * ty);
    float speed = tn > 0.0f ? (rv[0] * tx + rv[1] * ty) / tn : 0.0f;
    float r_head = cps > 0.8f ? 1.0f : cps / 0.8f;
    float cvert = 1.0f - 2.0f * (qx * qx + qy * qy);
    float r_stand = cvert > 0.93f ? 1.0f : 0.0f;
    int steps = a.steps[env_e] + (a.count_step ? 1 : 0);
    const bool only_obs = pass != 0;                 // re-packing a freshly reset env: obs only
    if (!only_obs) a.steps[env_e] = steps;
    const float rew = M.alive_bonus + speed + 0.5f * r_head + 0.05f * r_stand - 4.0f * l1 - 0.5f * l2 -
                      0.2f * (float)n_lim - (float)n_feet;
    uint8_t dn = (height < M.term_height || steps >= M.max_steps) ? 1 : 0;
    if (a.task.enabled && a.count_step && pass == 0) {
      // Section 4.1: termination only after `grace` consecutive frames below the threshold;
      // flagrun target re-drawn every `period` frames or when reached; finished envs start
      // their next episode below
      int fall = a.task_i[4 * env_e + 0], age = a.task_i[4 * env_e + 1];
      const int ep = a.task_i[4 * env_e + 3];
      fall = height < M.term_height ? fall + 1 : 0;
      dn = (fall > a.task.grace || steps >= M.max_steps) ? 1 : 0;
      if (a.task.period > 0) {
        age += 1;
        if (age >= a.task.period || tn < a.task.reach) {
          float txy[2];
          task_draw_target(a.task, env_e, ep, steps, rx[0], rx[1], txy);
          a.targets[2 * env_e] = txy[0]; a.targets[2 * env_e + 1] = txy[1];
          age = 0;
        }
      }
      a.task_i[4 * env_e + 0] = fall; a.task_i[4 * env_e + 1] = age;
      reset_now = dn && a.task.auto_reset;
    }
    if (!only_obs) {
      // (one copy each: the caller's array when there is one, else the library's)
      (a.reward_out ? a.reward_out : a.reward)[env_e] = rew;
      (a.done_out ? a.done_out : a.done)[env_e] = dn;
    }
    if (reset_now) {
      // next episode: the reset recipe with that episode's seed, built in this env's column of
      // the pose array (no other thread reads it before the barrier below)
      const int episode = a.task_i[4 * env_e + 3] + 1;
      LdsPoses poses{Lpos, Lvel, E, ee};
      reset_pose(M, env_e, a.task.seed + (uint64_t)episode * kEpisodeStride, poses);
      a.steps[env_e] = 0;
      task_begin_episode(a.task, a.task_i, a.targets, env_e, episode, Lpos[(rb * 7 + 0) * E + ee], Lpos[(rb * 7 + 1) * E + ee]);
    }
  }
  return reset_now;
  };
  pack_joints(std::integral_constant<int, 0>{});
  __syncthreads();
  const bool reset_now = pack_root(std::integral_constant<int, 0>{});
  if (may_reset) {
    if (tid < E) Lrst[tid] = reset_now ? 1 : 0;
    if (__syncthreads_or(reset_now)) {
      if (is_body && Lrst[e]) {
        float* st = a.state + (size_t)b * N + agent;
        const size_t fs = (size_t)B * N;
        for (int c = 0; c < 7; ++c) st[c * fs] = Lpos[(b * 7 + c) * E + e];
        for (int c = 0; c < 6; ++c) st[(7 + c) * fs] = Lvel[(b * kVS + c) * E + e];
      }
      pack_joints(std::integral_constant<int, 1>{});
      __syncthreads();
      pack_root(std::integral_constant<int, 1>{});
    }
  }
  __syncthreads();
  if constexpr (WS != 0) {
    // the kept impulses go back to the workspace for the next launch; an env that was just reset
    // starts its episode without any
    if (a.substeps > 0) {
      for (int i = tid; i < (J * 6 + S * 3) * E; i += kThreads) {
        const int ee = i % E, env_i = blockIdx.x * E + ee;
        if (env_i >= N) continue;
        const bool fresh = may_reset && Lrst[ee];
        const int ag = agent_at(env_i);
        if (i < J * 6 * E) a.lam_j[(size_t)(i / E) * N + ag] = fresh ? 0.0f : Lwj[i];
        else a.lam_s[(size_t)((i - J * 6 * E) / E) * N + ag] = fresh ? 0.0f : Lwc[i - J * 6 * E];
      }
    }
  }
  {
    const int env0 = blockIdx.x * E;
    const int n_here = min(E, N - env0);
    float* const obs_dst = a.obs_out ? a.obs_out : a.obs;   // one copy: the caller's array when there is one
    for (int i = tid; i < n_here * obs_dim; i += kThreads) {
      const float o = Lobs[i];
      const int ee = i / obs_dim, k = i - ee * obs_dim;
      obs_dst[(size_t)agent_at(env0 + ee) * obs_row + k] = o;
    }
    if (M.height_map) {
      // Height map (Section 4.1, complex-terrain task): terrain height under a 15 x 11 grid that
      // follows the centre of mass and is aligned with the root's heading, minus the height of
      // the centre of mass; written straight to the output rows (it is not staged in LDS).
      // Centre and heading per env first (in the space of the sweep copies, free by now).
      float* Lhm = Loutj;   // [5][E]: centre x,y,z (world), cos, sin of the yaw
      if (tid < n_here) {
        const int ee = tid;
        float cx = 0.0f, cy = 0.0f, cz = 0.0f;
        for (int bb = 0; bb < B; ++bb) {
          const float mf = M.body_mass_frac[bb];
          cx += mf * Lpos[(bb * 7 + 0) * E + ee]; cy += mf * Lpos[(bb * 7 + 1) * E + ee]; cz += mf * Lpos[(bb * 7 + 2) * E + ee];
        }
        const int rbb = M.root;
        const float qw = Lpos[(rbb * 7 + 3) * E + ee], qx = Lpos[(rbb * 7 + 4) * E + ee];
        const float qy = Lpos[(rbb * 7 + 5) * E + ee], qz = Lpos[(rbb * 7 + 6) * E + ee];
        const float yaw = atan2f(2.0f * (qw * qz + qx * qy), 1.0f - 2.0f * (qy * qy + qz * qz));
        const int ag = agent_at(env0 + ee);
        Lhm[0 * E + ee] = cx + a.origins[3 * ag];
        Lhm[1 * E + ee] = cy + a.origins[3 * ag + 1];
        Lhm[2 * E + ee] = cz + a.origins[3 * ag + 2];
        Lhm[3 * E + ee] = cosf(yaw); Lhm[4 * E + ee] = sinf(yaw);
      }
      __syncthreads();
      constexpr int kHm = kHmRows * kHmCols;
      for (int i = tid; i < n_here * kHm; i += kThreads) {
        const int ee = i / kHm, k = i - ee * kHm, hi = k / kHmCols, hj = k - hi * kHmCols;
          const float fw = M.hm_fwd[hi], lt = M.hm_lat[hj], c = Lhm[3 * E + ee], sn = Lhm[4 * E + ee];
        const float wx = Lhm[0 * E + ee] + (c * fw - sn * lt), wy = Lhm[1 * E + ee] + (sn * fw + c * lt);
        const float hz = terrain_height(M, a.heights, wx, wy) - Lhm[2 * E + ee];
        obs_dst[(size_t)agent_at(env0 + ee) * obs_row + obs_dim + k] = hz;
      }
    }
  }
  TMARK(9);
}

}  // namespace sim355
