/*
 * CPU oracle for the batched rigid-body step -- TEST INFRASTRUCTURE ONLY.
 * See oracle.h.  Plain scalar C, fp64 everywhere except the contact *selection*
 * predicate, which is evaluated in fp32 with a fixed operation order (no fused
 * multiply-add; compile with -ffp-contract=off) so that the integer outcome
 * (which slots are active and against which terrain feature) is a pure function
 * of the fp32-rounded state.
 *
 * Paper basis (Section 3.1): maximal coordinates, torque control, speculative
 * contacts as unilateral constraints, isotropic Coulomb friction, restitution
 * 0, implicit-style velocity-level time stepping.  Two solvers for the same
 * rows: a fixed-count block projected-Jacobi iteration (the default), and the
 * paper's own choice, a non-smooth Newton method with a conjugate-residual
 * inner solve; where the paper is silent a reading is taken and stated where
 * it is used.  Agents of one interaction group collide capsule against
 * capsule; the groups are consecutive places that any permutation of the
 * agents, or a grouping from their positions, can fill.
 * Observation: Table 2 ("Ours").  Reward: Eq. (1)-(3).  Episode rules: Section
 * 4.1 (fall threshold, 1000-frame cap).
 */
#include "oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MAXB 32
#define MAXJ 32
#define MAXS 96
#define MAXD 64
#define MAXOBS (11 + 3 * MAXD + 8 + 15 * 11)
#define MAXG 16                       /* agents of one interaction group */
#define MAXP (MAXB * (MAXB - 1) / 2)  /* body pairs of one agent that may collide */
#define MAXPC 512                     /* capsule-capsule contacts of one group */
#define FRICTION_EPS 1e-3             /* m/s: smoothing of the friction law in the Newton solver */

typedef struct { double x, y, z; } v3;
typedef struct { double w, x, y, z; } quat;

static v3 V(double x, double y, double z) { v3 r = {x, y, z}; return r; }
static v3 vadd(v3 a, v3 b) { return V(a.x + b.x, a.y + b.y, a.z + b.z); }
static v3 vsub(v3 a, v3 b) { return V(a.x - b.x, a.y - b.y, a.z - b.z); }
static v3 vscale(v3 a, double s) { return V(a.x * s, a.y * s, a.z * s); }
static double vdot(v3 a, v3 b) { return a.x * b.x + a.y * b.y + a.z * b.z; }
static v3 vcross(v3 a, v3 b) {
  return V(a.y * b.z - a.z * b.y, a.z * b.x - a.x * b.z, a.x * b.y - a.y * b.x);
}
static double vnorm(v3 a) { return sqrt(vdot(a, a)); }
static double vget(v3 a, int k) { return k == 0 ? a.x : (k == 1 ? a.y : a.z); }

static quat qmul(quat a, quat b) {
  quat r;
  r.w = a.w * b.w - a.x * b.x - a.y * b.y - a.z * b.z;
  r.x = a.w * b.x + a.x * b.w + a.y * b.z - a.z * b.y;
  r.y = a.w * b.y - a.x * b.z + a.y * b.w + a.z * b.x;
  r.z = a.w * b.z + a.x * b.y - a.y * b.x + a.z * b.w;
  return r;
}
static quat qconj(quat a) { quat r = {a.w, -a.x, -a.y, -a.z}; return r; }
static quat qnormalize(quat a) {
  double n = sqrt(a.w * a.w + a.x * a.x + a.y * a.y + a.z * a.z);
  quat r = {a.w / n, a.x / n, a.y / n, a.z / n};
  return r;
}
/* rotation matrix columns of a unit quaternion: m[c] is the image of body axis c */
static void qmat(quat q, v3 m[3]) {
  double w = q.w, x = q.x, y = q.y, z = q.z;
  m[0] = V(1 - 2 * (y * y + z * z), 2 * (x * y + w * z), 2 * (x * z - w * y));
  m[1] = V(2 * (x * y - w * z), 1 - 2 * (x * x + z * z), 2 * (y * z + w * x));
  m[2] = V(2 * (x * z + w * y), 2 * (y * z - w * x), 1 - 2 * (x * x + y * y));
}
static v3 mrot(const v3 m[3], v3 a) { /* R a */
  return vadd(vadd(vscale(m[0], a.x), vscale(m[1], a.y)), vscale(m[2], a.z));
}
static v3 mrot_t(const v3 m[3], v3 a) { /* R^T a */
  return V(vdot(m[0], a), vdot(m[1], a), vdot(m[2], a));
}
/* rotation vector of a unit quaternion, sign-fixed to the short way round */
static v3 qlog(quat q) {
  if (q.w < 0) { q.w = -q.w; q.x = -q.x; q.y = -q.y; q.z = -q.z; }
  v3 u = V(q.x, q.y, q.z);
  double s = vnorm(u);
  if (s < 1e-12) return vscale(u, 2.0);
  return vscale(u, 2.0 * atan2(s, q.w) / s);
}
static quat qexp(v3 phi) {
  double a = vnorm(phi);
  quat r;
  if (a < 1e-12) { r.w = 1; r.x = 0.5 * phi.x; r.y = 0.5 * phi.y; r.z = 0.5 * phi.z; return r; }
  double s = sin(0.5 * a) / a;
  r.w = cos(0.5 * a); r.x = s * phi.x; r.y = s * phi.y; r.z = s * phi.z;
  return r;
}

/* ------------------------------------------------------------------ model */

typedef struct {
  int body, kind; /* kind 0: end sphere at -l, 1: end sphere at +l (or the sphere itself), 2: mid-segment */
} slot_def;

typedef struct {
  int B, J, D, S, F;
  double radius[MAXB], half_len[MAXB], mass[MAXB];
  int axis[MAXB];
  v3 inertia[MAXB], rest_pos[MAXB];
  int jp[MAXJ], jc[MAXJ];
  v3 la[MAXJ], lb[MAXJ];       /* anchor in parent / child frame */
  v3 jaxes[MAXJ][3];
  int jmode[MAXJ][3], jact[MAXJ][3];
  double jlo[MAXJ][3], jhi[MAXJ][3], jgear[MAXJ][3];
  int root, feet[8];
  int body_joint_count[MAXB];
  slot_def slots[MAXS];
  double term_height, alive_bonus;
  int terrain_kind, nx, ny;
  double cell, hox, hoy;
  float* heights;
  v3 g;
  double mu, margin, beta_j, beta_c, v_depen, c_lin, c_ang, w_max, reset_noise;
  int gyro, contacts, max_steps, height_map;
  /* capsule-capsule collisions (Section 3.1: contacts among bodies; Section 4.1: inter-agent
   * collisions): body pairs of one agent that may touch, and the number of consecutive agents
   * that share one interaction group (1: agents do not see each other) */
  int NP, pair_a[MAXP], pair_b[MAXP], G;
  /* warm start: share of the previous substep's impulses the rows start from (0: none) */
  double warm;
  /* solver of the rows: 0 = block projected Jacobi with mass splitting (`iterations` sweeps);
   * 1 = non-smooth Newton with a conjugate-residual inner solve, the paper's own choice
   * (Section 3.1): `iterations` Newton iterations of `krylov_iters` inner iterations each;
   * newton_reg: damping of the Newton step, this share of the diagonal of J M^-1 J^T is added to the
   * operator that the increments are solved with (the fixed point does not depend on it) */
  int solver, krylov_iters;
  double newton_reg;
} model;

typedef struct {
  v3 x[MAXB], v[MAXB], w[MAXB];
  quat q[MAXB];
  v3 origin;
  double target[2];
  double u[MAXD]; /* clipped actions of the last step */
  int steps;
  oracle_contact con[MAXS];
  /* task logic (Section 4.1) */
  int fall_frames, target_age, next_push, episode;
  v3 push;                 /* external force on the root body during the current step */
  int has_store;           /* obs/reward/done of the last step kept (task mode packs at step end) */
  double obs_store[MAXOBS], rew_store;
  uint8_t done_store;
  /* warm start: impulses at the end of the previous substep; for a limit row also which limit
   * it stood for (0 lower, 1 upper), for a slot whether it was active */
  double lam_j[MAXJ][6], lam_s[MAXS][3];
  int side_j[MAXJ][3], lam_s_on[MAXS];
} env_state;

static void clear_warm(env_state* e) {
  memset(e->lam_j, 0, sizeof e->lam_j); memset(e->lam_s, 0, sizeof e->lam_s);
  memset(e->side_j, 0, sizeof e->side_j); memset(e->lam_s_on, 0, sizeof e->lam_s_on);
}

struct oracle_sim {
  model m;
  oracle_task task;
  int N, threads;
  env_state* env;
  oracle_pair_contact* pcon; /* [groups][MAXPC] capsule-capsule contacts of the last substep */
  int* pcon_n;               /* [groups] */
  int pair_cap, pair_unit;   /* bounded contact store: at most pair_cap per pair_unit agents (0: none) */
  long long pair_removed;
  /* interaction groups over places: place p holds agent place_env[p]; group gi = places
   * [gi G, gi G + G).  Identity until oracle_set_groups / oracle_regroup change it.  Inside a
   * substep agents are numbered by place (also in the contacts kept in pcon). */
  int* place_env;
  int regrouped;
  int trace_env, trace_cap, trace_n;
  oracle_sweep_trace* trace;
};

/* ------------------------------------------------- fp32 contact selection */
/* Everything in this block is single precision with the operation order
 * written out; it decides integers only (active, kind, feature id).           */

typedef struct { float x, y, z; } f3;
static f3 F3(float x, float y, float z) { f3 r = {x, y, z}; return r; }
static f3 fsub(f3 a, f3 b) { return F3(a.x - b.x, a.y - b.y, a.z - b.z); }
static float fdot(f3 a, f3 b) { float s = a.x * b.x; float t = a.y * b.y; s = s + t; t = a.z * b.z; return s + t; }
static f3 fcross(f3 a, f3 b) {
  float cx0 = a.y * b.z, cx1 = a.z * b.y;
  float cy0 = a.z * b.x, cy1 = a.x * b.z;
  float cz0 = a.x * b.y, cz1 = a.y * b.x;
  return F3(cx0 - cx1, cy0 - cy1, cz0 - cz1);
}

typedef struct {
  int nx, ny;
  float cell, inv_cell, ox, oy;
  const float* h;
} hf32;

static f3 hf_vertex(const hf32* H, int i, int j) {
  float fx = (float)i * H->cell, fy = (float)j * H->cell;
  return F3(H->ox + fx, H->oy + fy, H->h[(size_t)j * H->nx + i]);
}

/* squared distance from P to triangle (A,B,C); closest point through the six
 * projections of P onto the two edge directions at the three corners */
static float tri_dist2_f32(f3 P, f3 A, f3 B, f3 C) {
  f3 ab = fsub(B, A), ac = fsub(C, A), ap = fsub(P, A);
  float g11 = fdot(ab, ab), g12 = fdot(ab, ac), g22 = fdot(ac, ac);
  float d1 = fdot(ab, ap), d2 = fdot(ac, ap);
  float d3 = d1 - g11, d4 = d2 - g12, d5 = d1 - g12, d6 = d2 - g22;
  float v, w;
  if (d1 <= 0.0f && d2 <= 0.0f) { v = 0.0f; w = 0.0f; }
  else if (d3 >= 0.0f && d4 <= d3) { v = 1.0f; w = 0.0f; }
  else if (d6 >= 0.0f && d5 <= d6) { v = 0.0f; w = 1.0f; }
  else {
    float vc = d1 * d4 - d3 * d2;
    float vb = d5 * d2 - d1 * d6;
    float va = d3 * d6 - d5 * d4;
    float e43 = d4 - d3, e56 = d5 - d6;
    if (vc <= 0.0f && d1 >= 0.0f && d3 <= 0.0f) { v = d1 / g11; w = 0.0f; }
    else if (vb <= 0.0f && d2 >= 0.0f && d6 <= 0.0f) { v = 0.0f; w = d2 / g22; }
    else if (va <= 0.0f && e43 >= 0.0f && e56 >= 0.0f) { w = e43 / (e43 + e56); v = 1.0f - w; }
    else { float s = (va + vb) + vc; v = vb / s; w = vc / s; }
  }
  f3 c = F3(A.x + (ab.x * v + ac.x * w), A.y + (ab.y * v + ac.y * w), A.z + (ab.z * v + ac.z * w));
  f3 df = fsub(P, c);
  return fdot(df, df);
}

static void cell_range(const hf32* H, float lo, float hi, float origin, int ncell, int* c0, int* c1) {
  float a = floorf((lo - origin) * H->inv_cell), b = floorf((hi - origin) * H->inv_cell);
  /* compare in float first so huge values cannot overflow the int conversion */
  if (b < 0.0f || a > (float)(ncell - 1)) { *c0 = 0; *c1 = -1; return; }
  if (a < 0.0f) a = 0.0f;
  if (b > (float)(ncell - 1)) b = (float)(ncell - 1);
  *c0 = (int)a; *c1 = (int)b;
}

#define SEL_SLACK 1e-3f

/* sphere of radius r centred at world point P against the heightfield.
 * Returns 1 and (kind, feat) if the slot is active. */
static int select_sphere_hf(const hf32* H, f3 P, float r, float margin, int brute, int* kind, int* feat,
                            int range[4]) {
  int ncx = H->nx - 1, ncy = H->ny - 1;
  /* underneath rule: centre below the plane of the triangle that contains its xy */
  {
    float ux = (P.x - H->ox) * H->inv_cell, uy = (P.y - H->oy) * H->inv_cell;
    float fi = floorf(ux), fj = floorf(uy);
    if (fi >= 0.0f && fi <= (float)(ncx - 1) && fj >= 0.0f && fj <= (float)(ncy - 1)) {
      int i = (int)fi, j = (int)fj;
      float fx = ux - fi, fy = uy - fj;
      int t = (fx >= fy) ? 0 : 1;
      f3 A = hf_vertex(H, i, j);
      f3 Bv = t == 0 ? hf_vertex(H, i + 1, j) : hf_vertex(H, i + 1, j + 1);
      f3 Cv = t == 0 ? hf_vertex(H, i + 1, j + 1) : hf_vertex(H, i, j + 1);
      f3 nt = fcross(fsub(Bv, A), fsub(Cv, A));
      float face = fdot(fsub(P, A), nt);
      if (face < 0.0f) {
        *kind = 2; *feat = 2 * (j * ncx + i) + t;
        return 1; /* d < -r < margin always */
      }
    }
  }
  float Rq = (r + margin) + SEL_SLACK;
  int i0, i1, j0, j1;
  if (brute) { i0 = 0; i1 = ncx - 1; j0 = 0; j1 = ncy - 1; }
  else {
    cell_range(H, P.x - Rq, P.x + Rq, H->ox, ncx, &i0, &i1);
    cell_range(H, P.y - Rq, P.y + Rq, H->oy, ncy, &j0, &j1);
  }
  range[0] = i0; range[1] = i1; range[2] = j0; range[3] = j1;
  float best = INFINITY; int best_id = -1;
  for (int j = j0; j <= j1; ++j)
    for (int i = i0; i <= i1; ++i) {
      f3 A = hf_vertex(H, i, j), B1 = hf_vertex(H, i + 1, j), C1 = hf_vertex(H, i + 1, j + 1),
         D1 = hf_vertex(H, i, j + 1);
      for (int t = 0; t < 2; ++t) {
        f3 Bv = t == 0 ? B1 : C1, Cv = t == 0 ? C1 : D1;
        f3 nt = fcross(fsub(Bv, A), fsub(Cv, A));
        float face = fdot(fsub(P, A), nt);
        if (face < 0.0f) continue; /* back-facing */
        float d2 = tri_dist2_f32(P, A, Bv, Cv);
        if (d2 < best) { best = d2; best_id = 2 * (j * ncx + i) + t; }
      }
    }
  if (best_id < 0) return 0;
  float dist = sqrtf(best);
  float d = dist - r;
  if (d < margin) { *kind = 1; *feat = best_id; return 1; }
  return 0;
}

static float clamp01f(float s) { return s < 0.0f ? 0.0f : (s > 1.0f ? 1.0f : s); }

/* closest points between segment P0+s*(P1-P0) and edge Q0+t*(Q1-Q0); returns
 * squared distance, s and the sign of the vertical offset */
static float seg_edge_f32(f3 P0, f3 P1, f3 Q0, f3 Q1, float* s_out, float* dz_out) {
  f3 d1 = fsub(P1, P0), d2 = fsub(Q1, Q0), rr = fsub(P0, Q0);
  float a = fdot(d1, d1), e = fdot(d2, d2), f = fdot(d2, rr), c = fdot(d1, rr), b = fdot(d1, d2);
  float ae = a * e, bb = b * b;
  float denom = ae - bb;
  float s, t;
  if (denom > 1e-6f * ae) { float bf = b * f, ce = c * e; s = clamp01f((bf - ce) / denom); }
  else s = 0.5f;
  { float bs = b * s; t = (bs + f) / e; }
  if (t < 0.0f) { t = 0.0f; s = clamp01f((0.0f - c) / a); }
  else if (t > 1.0f) { t = 1.0f; s = clamp01f((b - c) / a); }
  f3 c1 = F3(P0.x + d1.x * s, P0.y + d1.y * s, P0.z + d1.z * s);
  f3 c2 = F3(Q0.x + d2.x * t, Q0.y + d2.y * t, Q0.z + d2.z * t);
  f3 df = fsub(c1, c2);
  *s_out = s; *dz_out = df.z;
  return fdot(df, df);
}

/* capsule segment [P0,P1] (interior only) against heightfield edges */
static int select_segment_hf(const hf32* H, f3 P0, f3 P1, float r, float margin, int brute, int* feat,
                             int range[4]) {
  int ncx = H->nx - 1, ncy = H->ny - 1;
  float Rq = (r + margin) + SEL_SLACK;
  int i0, i1, j0, j1;
  if (brute) { i0 = 0; i1 = ncx - 1; j0 = 0; j1 = ncy - 1; }
  else {
    float xl = P0.x < P1.x ? P0.x : P1.x, xh = P0.x < P1.x ? P1.x : P0.x;
    float yl = P0.y < P1.y ? P0.y : P1.y, yh = P0.y < P1.y ? P1.y : P0.y;
    cell_range(H, xl - Rq, xh + Rq, H->ox, ncx, &i0, &i1);
    cell_range(H, yl - Rq, yh + Rq, H->oy, ncy, &j0, &j1);
  }
  if (i1 < i0 || j1 < j0) return 0;
  range[0] = i0; range[1] = i1; range[2] = j0; range[3] = j1;
  float best = INFINITY; int best_id = -1;
  for (int j = j0; j <= j1 + 1; ++j)
    for (int i = i0; i <= i1 + 1; ++i) {
      f3 Q0 = hf_vertex(H, i, j);
      for (int k = 0; k < 3; ++k) {
        if ((k == 0 || k == 2) && i > i1) continue;
        if ((k == 1 || k == 2) && j > j1) continue;
        f3 Q1 = k == 0 ? hf_vertex(H, i + 1, j) : (k == 1 ? hf_vertex(H, i, j + 1) : hf_vertex(H, i + 1, j + 1));
        float s, dz;
        float d2 = seg_edge_f32(P0, P1, Q0, Q1, &s, &dz);
        if (!(s > 0.001f && s < 0.999f)) continue; /* the ends belong to the end-sphere slots */
        if (!(dz > 0.0f)) continue;                /* axis must be above the edge */
        if (d2 < best) { best = d2; best_id = 3 * (j * H->nx + i) + k; }
      }
    }
  if (best_id < 0) return 0;
  float dist = sqrtf(best);
  float d = dist - r;
  if (d < margin) { *feat = best_id; return 1; }
  return 0;
}

/* fp32 end points of a body's segment from the fp32-rounded state */
static void body_ends_f32(const model* m, const env_state* e, int b, int world, f3* p0, f3* p1) {
  float x = (float)e->x[b].x, y = (float)e->x[b].y, z = (float)e->x[b].z;
  float qw = (float)e->q[b].w, qx = (float)e->q[b].x, qy = (float)e->q[b].y, qz = (float)e->q[b].z;
  float l = (float)m->half_len[b];
  f3 c;
  if (m->axis[b] == 0) {
    float yy = qy * qy, zz = qz * qz, xy = qx * qy, wz = qw * qz, xz = qx * qz, wy = qw * qy;
    c = F3(1.0f - 2.0f * (yy + zz), 2.0f * (xy + wz), 2.0f * (xz - wy));
  } else if (m->axis[b] == 1) {
    float xx = qx * qx, zz = qz * qz, xy = qx * qy, wz = qw * qz, yz = qy * qz, wx = qw * qx;
    c = F3(2.0f * (xy - wz), 1.0f - 2.0f * (xx + zz), 2.0f * (yz + wx));
  } else {
    float xx = qx * qx, yy = qy * qy, xz = qx * qz, wy = qw * qy, yz = qy * qz, wx = qw * qx;
    c = F3(2.0f * (xz + wy), 2.0f * (yz - wx), 1.0f - 2.0f * (xx + yy));
  }
  f3 a = F3(l * c.x, l * c.y, l * c.z);
  *p0 = F3(x - a.x, y - a.y, z - a.z);
  *p1 = F3(x + a.x, y + a.y, z + a.z);
  if (world) {
    float ox = (float)e->origin.x, oy = (float)e->origin.y, oz = (float)e->origin.z;
    *p0 = F3(p0->x + ox, p0->y + oy, p0->z + oz);
    *p1 = F3(p1->x + ox, p1->y + oy, p1->z + oz);
  }
}

/* ----------------------------------- fp64 geometry of the selected feature */

static v3 hf_vertex64(const model* m, int i, int j) {
  /* vertex coordinates are the fp32 numbers the selection used */
  float fx = (float)i * (float)m->cell, fy = (float)j * (float)m->cell;
  float px = (float)m->hox + fx, py = (float)m->hoy + fy;
  return V((double)px, (double)py, (double)m->heights[(size_t)j * m->nx + i]);
}
static void tri_vertices64(const model* m, int tri, v3* A, v3* B, v3* C) {
  int ncx = m->nx - 1;
  int t = tri & 1, c = tri >> 1, i = c % ncx, j = c / ncx;
  *A = hf_vertex64(m, i, j);
  if (t == 0) { *B = hf_vertex64(m, i + 1, j); *C = hf_vertex64(m, i + 1, j + 1); }
  else { *B = hf_vertex64(m, i + 1, j + 1); *C = hf_vertex64(m, i, j + 1); }
}
static v3 closest_on_triangle64(v3 P, v3 A, v3 B, v3 C) {
  v3 ab = vsub(B, A), ac = vsub(C, A), ap = vsub(P, A);
  double g11 = vdot(ab, ab), g12 = vdot(ab, ac), g22 = vdot(ac, ac);
  double d1 = vdot(ab, ap), d2 = vdot(ac, ap);
  double d3 = d1 - g11, d4 = d2 - g12, d5 = d1 - g12, d6 = d2 - g22;
  double v, w;
  if (d1 <= 0 && d2 <= 0) { v = 0; w = 0; }
  else if (d3 >= 0 && d4 <= d3) { v = 1; w = 0; }
  else if (d6 >= 0 && d5 <= d6) { v = 0; w = 1; }
  else {
    double vc = d1 * d4 - d3 * d2, vb = d5 * d2 - d1 * d6, va = d3 * d6 - d5 * d4;
    if (vc <= 0 && d1 >= 0 && d3 <= 0) { v = d1 / g11; w = 0; }
    else if (vb <= 0 && d2 >= 0 && d6 <= 0) { v = 0; w = d2 / g22; }
    else if (va <= 0 && d4 - d3 >= 0 && d5 - d6 >= 0) { w = (d4 - d3) / ((d4 - d3) + (d5 - d6)); v = 1 - w; }
    else { double s = va + vb + vc; v = vb / s; w = vc / s; }
  }
  return vadd(A, vadd(vscale(ab, v), vscale(ac, w)));
}
static double clamp01(double s) { return s < 0 ? 0 : (s > 1 ? 1 : s); }
static double seg_edge64(v3 P0, v3 P1, v3 Q0, v3 Q1, v3* c1, v3* c2) {
  v3 d1 = vsub(P1, P0), d2 = vsub(Q1, Q0), rr = vsub(P0, Q0);
  double a = vdot(d1, d1), e = vdot(d2, d2), f = vdot(d2, rr), c = vdot(d1, rr), b = vdot(d1, d2);
  double denom = a * e - b * b, s, t;
  if (denom > 1e-6 * a * e) s = clamp01((b * f - c * e) / denom); else s = 0.5;
  t = (b * s + f) / e;
  if (t < 0) { t = 0; s = clamp01(-c / a); }
  else if (t > 1) { t = 1; s = clamp01((b - c) / a); }
  *c1 = vadd(P0, vscale(d1, s));
  *c2 = vadd(Q0, vscale(d2, t));
  return s;
}

static void clear_contact(oracle_contact* c) {
  memset(c, 0, sizeof(*c));
  c->kind = -1; c->feat = -1;
}

static double block_weight(const model* m, double d, double ramp_s) {
  /* share of its body a contact block gets in the mass splitting: rises from 0 at the margin
   * to 1 at half the margin, times a fade of the mid-segment slot towards the segment ends */
  double w = m->margin > 0 ? (m->margin - d) / (0.5 * m->margin) : 1.0;
  if (w > 1.0) w = 1.0;
  w *= ramp_s;
  return w < 1e-6 ? 1e-6 : w;
}

/* Speculative contact generation from positions (Section 3.1: contacts are
 * detected speculatively and enter as unilateral constraints). */
static void generate_contacts(const model* m, env_state* e, int brute, oracle_contact* out) {
  hf32 H;
  H.nx = m->nx; H.ny = m->ny; H.cell = (float)m->cell; H.inv_cell = 1.0f / (float)m->cell;
  H.ox = (float)m->hox; H.oy = (float)m->hoy; H.h = m->heights;
  float marginf = (float)m->margin;
  for (int s = 0; s < m->S; ++s) {
    oracle_contact* c = &out[s];
    clear_contact(c);
    if (!m->contacts) continue;
    int b = m->slots[s].body, kind = m->slots[s].kind;
    float rf = (float)m->radius[b];
    double r = m->radius[b];
    v3 R[3];
    qmat(e->q[b], R);
    v3 half = vscale(R[m->axis[b]], m->half_len[b]);
    v3 p0 = vsub(e->x[b], half), p1 = vadd(e->x[b], half); /* env-local fp64 */
    v3 p = kind == 0 ? p0 : p1;
    f3 f0, f1;
    body_ends_f32(m, e, b, m->terrain_kind == 1, &f0, &f1);
    if (m->terrain_kind == 0) {
      if (kind == 2) continue;
      f3 fp = kind == 0 ? f0 : f1;
      float df = fp.z - rf;
      if (!(df < marginf)) continue;
      c->active = 1; c->kind = 0; c->feat = -1;
      c->d = p.z - r; c->n[0] = 0; c->n[1] = 0; c->n[2] = 1;
      c->w = block_weight(m, c->d, 1.0);
      v3 rc = vsub(vsub(p, V(0, 0, r)), e->x[b]);
      c->rc[0] = rc.x; c->rc[1] = rc.y; c->rc[2] = rc.z;
      continue;
    }
    if (kind < 2) {
      int ck = -1, feat = -1, rg[4];
      if (!select_sphere_hf(&H, kind == 0 ? f0 : f1, rf, marginf, brute, &ck, &feat, rg)) continue;
      v3 Pw = vadd(p, e->origin), A, Bv, Cv, n;
      tri_vertices64(m, feat, &A, &Bv, &Cv);
      v3 nt = vcross(vsub(Bv, A), vsub(Cv, A));
      nt = vscale(nt, 1.0 / vnorm(nt));
      double d;
      if (ck == 2) { n = nt; d = vdot(vsub(Pw, A), nt) - r; }
      else {
        v3 cp = closest_on_triangle64(Pw, A, Bv, Cv);
        v3 df = vsub(Pw, cp);
        double dist = vnorm(df);
        n = dist < 1e-9 ? nt : vscale(df, 1.0 / dist);
        d = dist - r;
      }
      c->active = 1; c->kind = ck; c->feat = feat; c->d = d;
      c->n[0] = n.x; c->n[1] = n.y; c->n[2] = n.z;
      v3 rc = vsub(vsub(p, vscale(n, r)), e->x[b]);
      c->rc[0] = rc.x; c->rc[1] = rc.y; c->rc[2] = rc.z;
      c->w = block_weight(m, d, 1.0);
    } else {
      int feat = -1, rg[4];
      if (!select_segment_hf(&H, f0, f1, rf, marginf, brute, &feat, rg)) continue;
      int k = feat % 3, vtx = feat / 3, i = vtx % m->nx, j = vtx / m->nx;
      v3 Q0 = hf_vertex64(m, i, j);
      v3 Q1 = k == 0 ? hf_vertex64(m, i + 1, j) : (k == 1 ? hf_vertex64(m, i, j + 1) : hf_vertex64(m, i + 1, j + 1));
      v3 c1, c2;
      double sp = seg_edge64(vadd(p0, e->origin), vadd(p1, e->origin), Q0, Q1, &c1, &c2);
      v3 df = vsub(c1, c2);
      double dist = vnorm(df);
      v3 n = dist < 1e-9 ? V(0, 0, 1) : vscale(df, 1.0 / dist);
      c->active = 1; c->kind = 3; c->feat = feat; c->d = dist - r;
      c->n[0] = n.x; c->n[1] = n.y; c->n[2] = n.z;
      v3 rc = vsub(vsub(vsub(c1, e->origin), vscale(n, r)), e->x[b]);
      c->rc[0] = rc.x; c->rc[1] = rc.y; c->rc[2] = rc.z;
      /* the mid-segment block fades out towards the segment ends, where the end-sphere
       * slots take over the same contact point */
      double se = sp < 1 - sp ? sp : 1 - sp;
      double ramp_s = (se - 0.001) / 0.1;
      if (ramp_s > 1) ramp_s = 1;
      if (ramp_s < 0) ramp_s = 0;
      c->w = block_weight(m, c->d, ramp_s);
    }
  }
}

/* ------------------------------------------------------------ the substep */

/* world-frame inverse inertia applied to a vector: R I^-1 R^T a */
static v3 inv_inertia_apply(const v3 R[3], v3 inertia, v3 a) {
  v3 b = mrot_t(R, a);
  b = V(b.x / inertia.x, b.y / inertia.y, b.z / inertia.z);
  return mrot(R, b);
}

typedef struct {
  /* one scalar constraint row between body a (may be -1 = static) and body b */
  int a, b;
  v3 jla, jaa, jlb, jab; /* J blocks: linear/angular on a, linear/angular on b */
  double bias, meff, lambda;
  double sca, scb; /* inverse-mass scale of body a / b inside this row's block */
  int type;  /* 0 bilateral, 1 one-sided (lambda >= 0), 2 friction (paired with the next/prev row) */
  int slot;  /* contact rows: slot index, else -1 */
} row_t;

#define MAXROWS (6 * MAXJ + 3 * MAXS)

static double row_jv(const row_t* r, const v3* v, const v3* w) {
  double s = 0;
  if (r->a >= 0) s += vdot(r->jla, v[r->a]) + vdot(r->jaa, w[r->a]);
  if (r->b >= 0) s += vdot(r->jlb, v[r->b]) + vdot(r->jab, w[r->b]);
  return s;
}

static void joint_frames(const model* m, const env_state* e, int j, v3 Ra[3], v3* xa, quat* qa) {
  int a = m->jp[j];
  if (a >= 0) { qmat(e->q[a], Ra); *xa = e->x[a]; *qa = e->q[a]; }
  else { Ra[0] = V(1, 0, 0); Ra[1] = V(0, 1, 0); Ra[2] = V(0, 0, 1); *xa = V(0, 0, 0); qa->w = 1; qa->x = qa->y = qa->z = 0; }
}

/* joint angles: components of the rotation vector of q_a^-1 q_b along the joint axes */
static void joint_theta(const model* m, const env_state* e, int j, double th[3]) {
  v3 Ra[3], xa; quat qa;
  joint_frames(m, e, j, Ra, &xa, &qa);
  v3 phi = qlog(qmul(qconj(qa), e->q[m->jc[j]]));
  for (int k = 0; k < 3; ++k) th[k] = vdot(m->jaxes[j][k], phi);
}

/* closest points of two segments in single precision, one rounding per written operation */
static float segseg_f32(f3 P0, f3 P1, f3 Q0, f3 Q1, float* s_out, float* t_out) {
  const float tiny = 1e-12f;
  f3 d1 = fsub(P1, P0), d2 = fsub(Q1, Q0), r = fsub(P0, Q0);
  float a = fdot(d1, d1), e = fdot(d2, d2), f = fdot(d2, r), c = fdot(d1, r), b = fdot(d1, d2);
  float s, t;
  if (a <= tiny && e <= tiny) { s = 0.0f; t = 0.0f; }
  else if (a <= tiny) { s = 0.0f; t = clamp01f(f / e); }
  else if (e <= tiny) { t = 0.0f; s = clamp01f(-c / a); }
  else {
    float ae = a * e, bb = b * b;
    float den = ae - bb, floor_ = 1e-6f * ae;
    if (den > floor_) { float bf = b * f, ce = c * e; float num = bf - ce; s = clamp01f(num / den); }
    else s = 0.5f; /* parallel: any point of the overlap is closest; start from the middle */
    float bs = b * s;
    float tn = bs + f;
    t = tn / e;
    if (t < 0.0f) { t = 0.0f; s = clamp01f(-c / a); }
    else if (t > 1.0f) { t = 1.0f; float bc = b - c; s = clamp01f(bc / a); }
  }
  float ux = d1.x * s, uy = d1.y * s, uz = d1.z * s;
  float wx = d2.x * t, wy = d2.y * t, wz = d2.z * t;
  f3 cp = F3(P0.x + ux, P0.y + uy, P0.z + uz), cq = F3(Q0.x + wx, Q0.y + wy, Q0.z + wz);
  f3 df = fsub(cp, cq);
  *s_out = s; *t_out = t;
  return fdot(df, df);
}

float oracle_segment_segment_f32(const float* P0, const float* P1, const float* Q0, const float* Q1,
                                 float* s, float* t) {
  return segseg_f32(F3(P0[0], P0[1], P0[2]), F3(P1[0], P1[1], P1[2]), F3(Q0[0], Q0[1], Q0[2]),
                    F3(Q1[0], Q1[1], Q1[2]), s, t);
}

/* One candidate pair of capsules: body ba of agent A against body bb of agent B (the same agent
 * for self-collision).  The decision is taken in single precision in the frame of agent A; the
 * geometry of an accepted contact is then built in double precision from the segment parameters
 * the decision found. */
static int pair_contact(const model* m, const env_state* A, int ea, int ba, const env_state* Bv, int eb, int bb,
                        oracle_pair_contact* c) {
  f3 p0, p1, q0, q1;
  body_ends_f32(m, A, ba, 0, &p0, &p1);
  body_ends_f32(m, Bv, bb, 0, &q0, &q1);
  float ox = (float)Bv->origin.x - (float)A->origin.x, oy = (float)Bv->origin.y - (float)A->origin.y,
        oz = (float)Bv->origin.z - (float)A->origin.z;
  q0 = F3(q0.x + ox, q0.y + oy, q0.z + oz);
  q1 = F3(q1.x + ox, q1.y + oy, q1.z + oz);
  float s, t;
  float d2 = segseg_f32(p0, p1, q0, q1, &s, &t);
  float rr = (float)m->radius[ba] + (float)m->radius[bb];
  float lim = rr + (float)m->margin;
  if (!(d2 < lim * lim)) return 0;
  c->gap32 = (sqrtf(d2) - (float)m->radius[ba]) - (float)m->radius[bb];
  c->pad_ = 0;
  v3 RA[3], RB[3];
  qmat(A->q[ba], RA); qmat(Bv->q[bb], RB);
  v3 ha = vscale(RA[m->axis[ba]], m->half_len[ba]), hb = vscale(RB[m->axis[bb]], m->half_len[bb]);
  v3 xa = vadd(A->x[ba], A->origin), xb = vadd(Bv->x[bb], Bv->origin);
  v3 cp = vadd(vsub(xa, ha), vscale(ha, 2.0 * (double)s));
  v3 cq = vadd(vsub(xb, hb), vscale(hb, 2.0 * (double)t));
  v3 df = vsub(cp, cq);
  double dist = vnorm(df);
  v3 n = dist < 1e-9 ? V(0, 0, 1) : vscale(df, 1.0 / dist);
  c->env_a = ea; c->body_a = ba; c->env_b = eb; c->body_b = bb; c->s = s; c->t = t;
  c->d = dist - m->radius[ba] - m->radius[bb];
  c->n[0] = n.x; c->n[1] = n.y; c->n[2] = n.z;
  /* one contact point for both bodies, midway between the two surface points, so that the pair
   * of opposite impulses carries no net torque */
  v3 sa = vsub(cp, vscale(n, m->radius[ba])), sb = vadd(cq, vscale(n, m->radius[bb]));
  v3 pm = vscale(vadd(sa, sb), 0.5);
  v3 ra = vsub(pm, xa), rb = vsub(pm, xb);
  c->ra[0] = ra.x; c->ra[1] = ra.y; c->ra[2] = ra.z;
  c->rb[0] = rb.x; c->rb[1] = rb.y; c->rb[2] = rb.z;
  c->w = block_weight(m, c->d, 1.0);
  return 1;
}

/* capsule-capsule contacts of one interaction group from the positions at substep start:
 * agent by agent its own listed body pairs, then every body pair with each later agent */
static int generate_pair_contacts(const model* m, env_state* envs, int e0, int G, oracle_pair_contact* out) {
  int n = 0;
  if (!m->contacts) return 0;
  for (int ga = 0; ga < G; ++ga) {
    for (int p = 0; p < m->NP && n < MAXPC; ++p)
      n += pair_contact(m, &envs[ga], e0 + ga, m->pair_a[p], &envs[ga], e0 + ga, m->pair_b[p], &out[n]);
    for (int gb = ga + 1; gb < G; ++gb)
      for (int ba = 0; ba < m->B; ++ba)
        for (int bb = 0; bb < m->B && n < MAXPC; ++bb)
          n += pair_contact(m, &envs[ga], e0 + ga, ba, &envs[gb], e0 + gb, bb, &out[n]);
  }
  return n;
}

/* ------------------------------------------- non-smooth Newton / Krylov solve */

/* (dv, dw)[body] = M^-1 J^T x: every body receives the plain sum of its rows' impulses in
 * ascending row order, then its inverse mass and world inverse inertia */
static void rows_to_bodies(const model* m, const row_t* rows, int nrows, const double* x, v3 (*R)[3], int NB,
                           v3* dv, v3* dw) {
  const int B = m->B;
  for (int b = 0; b < NB; ++b) { dv[b] = V(0, 0, 0); dw[b] = V(0, 0, 0); }
  for (int i = 0; i < nrows; ++i) {
    const row_t* r = &rows[i];
    if (r->a >= 0) { dv[r->a] = vadd(dv[r->a], vscale(r->jla, x[i])); dw[r->a] = vadd(dw[r->a], vscale(r->jaa, x[i])); }
    dv[r->b] = vadd(dv[r->b], vscale(r->jlb, x[i])); dw[r->b] = vadd(dw[r->b], vscale(r->jab, x[i]));
  }
  for (int b = 0; b < NB; ++b) {
    dv[b] = vscale(dv[b], 1.0 / m->mass[b % B]);
    dw[b] = inv_inertia_apply(R[b], m->inertia[b % B], dw[b]);
  }
}

/* y = (J M^-1 J^T + reg D) x on the rows with on[i] != 0 (x is zero elsewhere), 0 on the others */
static void delassus_apply(const model* m, const row_t* rows, int nrows, const double* diag, const int* on,
                           const double* x, v3 (*R)[3], int NB, v3* dv, v3* dw, double* y) {
  rows_to_bodies(m, rows, nrows, x, R, NB, dv, dw);
  for (int i = 0; i < nrows; ++i)
    y[i] = (!on || on[i]) ? row_jv(&rows[i], dv, dw) + m->newton_reg * diag[i] * x[i] : 0.0;
}

/* The paper's solver (Section 3.1): a non-smooth Newton method on the complementarity form of
 * the rows, each Newton iteration solved by a Krylov method with a fixed number of iterations.
 * The paper gives no formulas; this reading:
 *   unknowns lambda; velocities u = v* + M^-1 J^T lambda; row residual s = J u + bias.
 *   bilateral rows:  s = 0.
 *   one-sided rows:  phi = min(lambda, s / D) = 0 (minimum map, D = diagonal of J M^-1 J^T).
 *   friction pair t of a contact with normal impulse lambda_n: the smooth isotropic Coulomb law
 *       lambda_t = -mu lambda_n s_t / sqrt(|s_t|^2 + eps^2)   (Section 3.1: "smooth isotropic").
 * A Newton iteration linearises with the branch every row is on: bilateral rows and one-sided
 * rows with lambda - s/D > 0 ask for s = 0 after the update, one-sided rows on the other branch
 * return to lambda = 0; a friction pair enters as a damper s_t + c lambda_t = 0 whose compliance
 * c = |s_t|_eps / (mu lambda_n) is taken from the current iterate (a pair without normal impulse
 * returns to zero), which keeps the linear system symmetric positive semi-definite.  It is solved
 * from zero by `krylov_iters` iterations of the conjugate-residual method with diagonal
 * preconditioning (matrix-free: J M^-1 J^T is applied through the bodies).  After the update
 * one-sided impulses are clipped at zero and friction pairs onto the disc mu lambda_n, so an
 * inexact inner solve never leaves the feasible set. */
static void newton_solve(const model* m, row_t* rows, int nrows, v3 (*R)[3], int NB, v3* vel, v3* om, int outer,
                         oracle_sweep_trace* trace, int* trace_n, int trace_cap, double pos_err_max) {
  static _Thread_local double *lam = NULL, *diag, *sres, *known, *rhs, *x, *z, *p, *q, *az, *tmp, *comp, *pd;
  static _Thread_local int* on;
  static _Thread_local v3 dv[MAXG * MAXB], dw[MAXG * MAXB], u[MAXG * MAXB], uw[MAXG * MAXB];
  const int cap = MAXG * MAXROWS + 3 * MAXPC;
  if (!lam) {
    lam = (double*)malloc(sizeof(double) * cap * 13);
    diag = lam + cap; sres = diag + cap; known = sres + cap; rhs = known + cap; x = rhs + cap; z = x + cap;
    p = z + cap; q = p + cap; az = q + cap; tmp = az + cap; comp = tmp + cap; pd = comp + cap;
    on = (int*)malloc(sizeof(int) * cap);
  }
  const int B = m->B;
  /* The scratch vectors are reused from solve to solve: every entry of this solve's range starts
   * as NaN, so that a value read before it is written cannot pass for a number (a friction pair
   * once left the compliance of its second row unset on the branch without normal impulse; what
   * lay in memory was then multiplied by zero, which only works as long as it is finite). */
  for (int i = 0; i < nrows; ++i) {
    lam[i] = diag[i] = sres[i] = known[i] = rhs[i] = x[i] = z[i] = p[i] = q[i] = az[i] = tmp[i] = comp[i] = pd[i] = NAN;
    on[i] = -1;
  }
  for (int i = 0; i < nrows; ++i) {
    const row_t* r = &rows[i];
    double k = 0;
    if (r->a >= 0) k += vdot(r->jla, r->jla) / m->mass[r->a % B] + vdot(r->jaa, inv_inertia_apply(R[r->a], m->inertia[r->a % B], r->jaa));
    k += vdot(r->jlb, r->jlb) / m->mass[r->b % B] + vdot(r->jab, inv_inertia_apply(R[r->b], m->inertia[r->b % B], r->jab));
    diag[i] = k;
    lam[i] = r->lambda;   /* 0, or the warm-start share of what was kept */
  }
  for (int it = 0; it <= outer; ++it) {
    /* velocities of the current iterate, from scratch */
    rows_to_bodies(m, rows, nrows, lam, R, NB, dv, dw);
    for (int b = 0; b < NB; ++b) { u[b] = vadd(vel[b], dv[b]); uw[b] = vadd(om[b], dw[b]); }
    if (it == outer) break;
    double sq = 0, mx = 0, viol = 0; int nbil = 0;
    for (int i = 0; i < nrows; ++i) {
      sres[i] = row_jv(&rows[i], u, uw) + rows[i].bias;
      if (rows[i].type == 0) { sq += sres[i] * sres[i]; nbil++; if (fabs(sres[i]) > mx) mx = fabs(sres[i]); }
      if (rows[i].type == 1 && -sres[i] > viol) viol = -sres[i];
    }
    if (trace && *trace_n < trace_cap) {
      oracle_sweep_trace* t = &trace[(*trace_n)++];
      t->bilateral_rms = nbil ? sqrt(sq / nbil) : 0; t->bilateral_max = mx; t->onesided_viol = viol;
      t->pos_err_max = pos_err_max; t->cone_excess = 0;
      double sl = 0;
      for (int r = 0; r < nrows; ++r) if (rows[r].slot >= 0 && rows[r].type == 1) sl += lam[r];
      t->sum_lambda_n = sl;
    }
    /* branch of every row */
    for (int i = 0; i < nrows; ++i) { known[i] = 0; comp[i] = 0; }
    for (int i = 0; i < nrows; ++i) {
      const row_t* r = &rows[i];
      if (r->type == 0) on[i] = 1;
      else if (r->type == 1) {
        on[i] = diag[i] > 0 && (lam[i] - sres[i] / diag[i] > 0);
        if (!on[i]) known[i] = -lam[i];
      } else {
        /* friction pair (i, i+1); its normal row is the one before the pair.  Smooth isotropic
         * Coulomb law: lambda_t = -mu lambda_n s_t / |s_t|_eps, i.e. the pair is a damper whose
         * compliance c = |s_t|_eps / (mu lambda_n) comes from the current iterate; with c known the
         * pair's two rows read s_t + c lambda_t = 0, which keeps the system symmetric.  Without
         * normal impulse there is no friction. */
        int n = i - 1;
        double rad = m->mu * lam[n];
        if (rad > 0) {
          double sn = sqrt(sres[i] * sres[i] + sres[i + 1] * sres[i + 1] + FRICTION_EPS * FRICTION_EPS);
          on[i] = on[i + 1] = 1;
          comp[i] = comp[i + 1] = sn / rad;
        } else {
          on[i] = on[i + 1] = 0;
          known[i] = -lam[i]; known[i + 1] = -lam[i + 1];
        }
        ++i;
      }
    }
    /* right-hand side of the rows on the "s" branch: -s - c lambda - (A known); the operator of
     * the inner solve is A + reg D + c on those rows, its preconditioner that operator's diagonal */
    delassus_apply(m, rows, nrows, diag, NULL, known, R, NB, dv, dw, tmp);
    for (int i = 0; i < nrows; ++i) {
      rhs[i] = on[i] ? -sres[i] - comp[i] * lam[i] - (tmp[i] - m->newton_reg * diag[i] * known[i]) : 0.0;
      pd[i] = diag[i] * (1.0 + m->newton_reg) + comp[i];
      if (!(pd[i] > 0)) on[i] = 0;
    }
    /* preconditioned conjugate residuals from x = 0 (stops early once the residual has dropped by
     * twelve orders of magnitude in this measure, where the recurrences would divide rounding noise) */
    double gamma = 0;
    for (int i = 0; i < nrows; ++i) { x[i] = 0; z[i] = on[i] ? rhs[i] / pd[i] : 0.0; p[i] = z[i]; }
    delassus_apply(m, rows, nrows, diag, on, z, R, NB, dv, dw, az);
    for (int i = 0; i < nrows; ++i) { az[i] += comp[i] * z[i]; q[i] = az[i]; gamma += z[i] * az[i]; }
    const double gamma0 = gamma;
    for (int k = 0; k < m->krylov_iters; ++k) {
      double den = 0;
      for (int i = 0; i < nrows; ++i) if (on[i]) den += q[i] * q[i] / pd[i];
      if (!(den > 0) || !(gamma > 1e-12 * gamma0)) break;
      double alpha = gamma / den;
      for (int i = 0; i < nrows; ++i) if (on[i]) { x[i] += alpha * p[i]; z[i] -= alpha * q[i] / pd[i]; }
      delassus_apply(m, rows, nrows, diag, on, z, R, NB, dv, dw, az);
      double gn = 0;
      for (int i = 0; i < nrows; ++i) { az[i] += comp[i] * z[i]; gn += z[i] * az[i]; }
      double beta = gn / gamma;
      for (int i = 0; i < nrows; ++i) { p[i] = z[i] + beta * p[i]; q[i] = az[i] + beta * q[i]; }
      gamma = gn;
    }
    /* update, then back into the feasible set */
    for (int i = 0; i < nrows; ++i) lam[i] += on[i] ? x[i] : known[i];
    for (int i = 0; i < nrows; ++i) {
      if (rows[i].type == 1 && lam[i] < 0) lam[i] = 0;
      if (rows[i].type == 2) {
        double rad = m->mu * lam[i - 1], nrm = sqrt(lam[i] * lam[i] + lam[i + 1] * lam[i + 1]);
        if (nrm > rad) { double sc = nrm > 0 ? rad / nrm : 0; lam[i] *= sc; lam[i + 1] *= sc; }
        ++i;
      }
    }
  }
  for (int b = 0; b < NB; ++b) { vel[b] = u[b]; om[b] = uw[b]; }
  for (int i = 0; i < nrows; ++i) rows[i].lambda = lam[i];
}

/* One substep of an interaction group of G agents (envs[0..G), global indices e0..).  Forces,
 * terrain contacts and integration are per agent; the solve couples the agents of the group
 * through the capsule-capsule contacts.  Bodies are numbered g*B + b inside the group. */
static void substep(const model* m, env_state* envs, int e0, int G, oracle_pair_contact* pcon, int* pcon_n,
                    double h, int iterations, int phases,
                    oracle_sweep_trace* trace, int* trace_n, int trace_cap) {
  const int B = m->B, J = m->J, S = m->S;
  static _Thread_local v3 R[MAXG * MAXB][3];
  /* 1. contacts from positions at substep start */
  if (phases & ORACLE_PH_CONTACTS) {
    for (int g = 0; g < G; ++g) generate_contacts(m, &envs[g], 0, envs[g].con);
    *pcon_n = (m->NP > 0 || G > 1) ? generate_pair_contacts(m, envs, e0, G, pcon) : 0;
  }
  for (int g = 0; g < G; ++g)
    for (int b = 0; b < B; ++b) qmat(envs[g].q[b], R[g * B + b]);

  /* 2. forces -> velocities: gravity, joint torques (+ on child, - on parent),
   *    explicit gyroscopic term in the body frame */
  if (phases & ORACLE_PH_FORCES) {
    for (int g = 0; g < G; ++g) {
      env_state* e = &envs[g];
      v3 tau[MAXB];
      for (int b = 0; b < B; ++b) tau[b] = V(0, 0, 0);
      for (int j = 0; j < J; ++j) {
        v3 Ra[3], xa; quat qa;
        joint_frames(m, e, j, Ra, &xa, &qa);
        for (int k = 0; k < 3; ++k) {
          if (m->jmode[j][k] != 1) continue;
          v3 ak = mrot(Ra, m->jaxes[j][k]);
          double t = m->jgear[j][k] * e->u[m->jact[j][k]];
          tau[m->jc[j]] = vadd(tau[m->jc[j]], vscale(ak, t));
          if (m->jp[j] >= 0) tau[m->jp[j]] = vsub(tau[m->jp[j]], vscale(ak, t));
        }
      }
      /* external push on the root body (Section 4.1, perturbations): constant over the step */
      e->v[m->root] = vadd(e->v[m->root], vscale(e->push, h / m->mass[m->root]));
      for (int b = 0; b < B; ++b) {
        const v3* Rb = R[g * B + b];
        e->v[b] = vadd(e->v[b], vscale(m->g, h));
        v3 wb = mrot_t(Rb, e->w[b]), tb = mrot_t(Rb, tau[b]), I = m->inertia[b];
        v3 Iw = V(I.x * wb.x, I.y * wb.y, I.z * wb.z);
        v3 rhs = m->gyro ? vsub(tb, vcross(wb, Iw)) : tb;
        wb = vadd(wb, V(h * rhs.x / I.x, h * rhs.y / I.y, h * rhs.z / I.z));
        e->w[b] = mrot(Rb, wb);
      }
    }
  }

  if (phases & ORACLE_PH_SOLVE) {
    /* 3. row setup.  A *block* is one joint (6 rows: 3 positional, 3 angular),
     * one active terrain contact slot or one capsule-capsule contact (3 rows:
     * normal, two tangents).  Mass splitting: body i is shared out among its
     * blocks in proportion to block weights (1 for a joint; for a contact the
     * record's weight, which rises from 0 at the margin, so a contact that has
     * just become active changes nothing).  W[i] is the weight sum; inside
     * block c body i acts with its inverse mass scaled by W[i] / w_c. */
    static _Thread_local row_t* rows = NULL;
    if (!rows) rows = (row_t*)malloc(sizeof(row_t) * (MAXG * MAXROWS + 3 * MAXPC));
    static _Thread_local v3 vel[MAXG * MAXB], om[MAXG * MAXB], v0[MAXG * MAXB], w0[MAXG * MAXB], pl[MAXG * MAXB],
        pa[MAXG * MAXB];
    static _Thread_local double W[MAXG * MAXB], wslot[MAXG * MAXS];
    int nrows = 0;
    const int npc = *pcon_n;
    for (int g = 0; g < G; ++g) {
      for (int b = 0; b < B; ++b) W[g * B + b] = m->body_joint_count[b];
      for (int s = 0; s < S; ++s) {
        wslot[g * S + s] = 0;
        if (!envs[g].con[s].active) continue;
        wslot[g * S + s] = envs[g].con[s].w;
        W[g * B + m->slots[s].body] += envs[g].con[s].w;
      }
    }
    for (int k = 0; k < npc; ++k) {
      W[(pcon[k].env_a - e0) * B + pcon[k].body_a] += pcon[k].w;
      W[(pcon[k].env_b - e0) * B + pcon[k].body_b] += pcon[k].w;
    }
    double pos_err_max = 0;
    for (int g = 0; g < G; ++g) {
      const env_state* e = &envs[g];
      const int f0 = g * B;
      for (int j = 0; j < J; ++j) {
        int a = m->jp[j], b = m->jc[j];
        v3 Ra[3], xa; quat qa;
        joint_frames(m, e, j, Ra, &xa, &qa);
        v3 pa_ = vadd(xa, mrot(Ra, m->la[j])), pb = vadd(e->x[b], mrot(R[f0 + b], m->lb[j]));
        v3 C = vsub(pb, pa_), mid = vscale(vadd(pa_, pb), 0.5);
        v3 ra = vsub(mid, xa), rb = vsub(mid, e->x[b]);
        double cn = vnorm(C);
        if (cn > pos_err_max) pos_err_max = cn;
        double th[3];
        joint_theta(m, e, j, th);
        for (int k = 0; k < 6; ++k) {
          row_t* r = &rows[nrows++];
          memset(r, 0xff, sizeof *r);   /* (every field is set below; a forgotten one reads as NaN / -1) */
          r->a = a >= 0 ? f0 + a : -1; r->b = f0 + b; r->slot = -1;
          r->lambda = m->warm * e->lam_j[j][k];
          r->sca = a >= 0 ? W[f0 + a] : 0.0; r->scb = W[f0 + b];
          if (k < 3) {
            v3 ex = V(k == 0, k == 1, k == 2);
            r->jla = vscale(ex, -1); r->jaa = vscale(vcross(ra, ex), -1);
            r->jlb = ex; r->jab = vcross(rb, ex);
            r->bias = m->beta_j / h * vget(C, k);
            r->type = 0;
          } else {
            int kk = k - 3;
            v3 ak = mrot(Ra, m->jaxes[j][kk]);
            r->jla = V(0, 0, 0); r->jlb = V(0, 0, 0);
            if (m->jmode[j][kk] == 0) {
              r->jaa = vscale(ak, -1); r->jab = ak;
              r->bias = m->beta_j / h * th[kk];
              r->type = 0;
            } else {
              double glo = th[kk] - m->jlo[j][kk], ghi = m->jhi[j][kk] - th[kk], gg;
              int side;
              if (glo < ghi) { gg = glo; r->jaa = vscale(ak, -1); r->jab = ak; side = 0; }
              else { gg = ghi; r->jaa = ak; r->jab = vscale(ak, -1); side = 1; }
              /* an impulse kept from the other limit would push the wrong way */
              if (e->side_j[j][kk] >= 0 && side != e->side_j[j][kk]) r->lambda = 0;
              envs[g].side_j[j][kk] = side;
              r->bias = gg >= 0 ? gg / h : m->beta_j * gg / h;
              r->type = 1;
            }
          }
        }
      }
      for (int s = 0; s < S; ++s) {
        const oracle_contact* c = &e->con[s];
        if (!c->active) continue;
        int b = m->slots[s].body;
        v3 n = V(c->n[0], c->n[1], c->n[2]), rc = V(c->rc[0], c->rc[1], c->rc[2]);
        /* tangent basis; the branch is decided in single precision like the contact selection */
        v3 t1 = (fabsf((float)n.x) < 0.57735f) ? vcross(n, V(1, 0, 0)) : vcross(n, V(0, 1, 0));
        t1 = vscale(t1, 1.0 / vnorm(t1));
        v3 t2 = vcross(n, t1);
        v3 dirs[3] = {n, t1, t2};
        for (int k = 0; k < 3; ++k) {
          row_t* r = &rows[nrows++];
          memset(r, 0xff, sizeof *r);   /* (every field is set below; a forgotten one reads as NaN / -1) */
          r->a = -1; r->b = f0 + b; r->slot = s;
          r->lambda = e->lam_s_on[s] ? m->warm * e->lam_s[s][k] : 0.0;
          r->sca = 0.0; r->scb = W[f0 + b] / wslot[g * S + s];
          r->jla = V(0, 0, 0); r->jaa = V(0, 0, 0);
          r->jlb = dirs[k]; r->jab = vcross(rc, dirs[k]);
          if (k == 0) {
            double bias = c->d >= 0 ? c->d / h : m->beta_c * c->d / h;
            if (c->d < 0 && bias < -m->v_depen) bias = -m->v_depen;
            r->bias = bias; r->type = 1;
          } else { r->bias = 0; r->type = 2; }
        }
      }
    }
    /* capsule-capsule contacts: the same three rows between two bodies, +J on body A, -J on B */
    for (int q = 0; q < npc; ++q) {
      const oracle_pair_contact* c = &pcon[q];
      int fa = (c->env_a - e0) * B + c->body_a, fb = (c->env_b - e0) * B + c->body_b;
      v3 n = V(c->n[0], c->n[1], c->n[2]), ra = V(c->ra[0], c->ra[1], c->ra[2]), rb = V(c->rb[0], c->rb[1], c->rb[2]);
      v3 t1 = (fabsf((float)n.x) < 0.57735f) ? vcross(n, V(1, 0, 0)) : vcross(n, V(0, 1, 0));
      t1 = vscale(t1, 1.0 / vnorm(t1));
      v3 t2 = vcross(n, t1);
      v3 dirs[3] = {n, t1, t2};
      for (int k = 0; k < 3; ++k) {
        row_t* r = &rows[nrows++];
        memset(r, 0xff, sizeof *r);   /* (every field is set below; a forgotten one reads as NaN / -1) */
        r->a = fb; r->b = fa; r->slot = S + q; r->lambda = 0;
        r->sca = W[fb] / c->w; r->scb = W[fa] / c->w;
        r->jlb = dirs[k]; r->jab = vcross(ra, dirs[k]);
        r->jla = vscale(dirs[k], -1); r->jaa = vscale(vcross(rb, dirs[k]), -1);
        if (k == 0) {
          double bias = c->d >= 0 ? c->d / h : m->beta_c * c->d / h;
          if (c->d < 0 && bias < -m->v_depen) bias = -m->v_depen;
          r->bias = bias; r->type = 1;
        } else { r->bias = 0; r->type = 2; }
      }
    }
    for (int i = 0; i < nrows; ++i) {
      row_t* r = &rows[i];
      double k = 0;
      if (r->a >= 0)
        k += r->sca * (vdot(r->jla, r->jla) / m->mass[r->a % B] +
                         vdot(r->jaa, inv_inertia_apply(R[r->a], m->inertia[r->a % B], r->jaa)));
      if (r->b >= 0)
        k += r->scb * (vdot(r->jlb, r->jlb) / m->mass[r->b % B] +
                         vdot(r->jab, inv_inertia_apply(R[r->b], m->inertia[r->b % B], r->jab)));
      r->meff = k > 0 ? 1.0 / k : 0.0;
    }
    for (int g = 0; g < G; ++g)
      for (int b = 0; b < B; ++b) { vel[g * B + b] = envs[g].v[b]; om[g * B + b] = envs[g].w[b]; }
    const int NB = G * B;
    if (m->solver == 1) {
      newton_solve(m, rows, nrows, R, NB, vel, om, iterations, trace, trace_n, trace_cap, pos_err_max);
    } else {
    /* warm start: the impulses the rows start from act on the bodies before the first sweep */
    if (m->warm > 0) {
      for (int i = 0; i < nrows; ++i) {
        const row_t* r = &rows[i];
        if (r->lambda == 0) continue;
        if (r->a >= 0) {
          vel[r->a] = vadd(vel[r->a], vscale(r->jla, r->lambda / m->mass[r->a % B]));
          om[r->a] = vadd(om[r->a], vscale(inv_inertia_apply(R[r->a], m->inertia[r->a % B], r->jaa), r->lambda));
        }
        vel[r->b] = vadd(vel[r->b], vscale(r->jlb, r->lambda / m->mass[r->b % B]));
        om[r->b] = vadd(om[r->b], vscale(inv_inertia_apply(R[r->b], m->inertia[r->b % B], r->jab), r->lambda));
      }
    }

    /* 4. projected-Jacobi sweeps over blocks: every block starts from the same
     * velocity snapshot; inside a block the rows are relaxed one after another
     * on the block's private copy of its bodies (inverse mass scaled as above). */
    for (int it = 0; it < iterations; ++it) {
      for (int b = 0; b < NB; ++b) { v0[b] = vel[b]; w0[b] = om[b]; pl[b] = V(0, 0, 0); pa[b] = V(0, 0, 0); }
      double sq = 0, mx = 0, viol = 0, cone = -INFINITY; int nbil = 0;
      /* diagnostics are taken on the snapshot, before any block is relaxed */
      for (int i = 0; i < nrows; ++i) {
        double res = row_jv(&rows[i], v0, w0) + rows[i].bias;
        if (rows[i].type == 0) { sq += res * res; nbil++; if (fabs(res) > mx) mx = fabs(res); }
        if (rows[i].type == 1 && -res > viol) viol = -res;
      }
      int i = 0;
      while (i < nrows) {
        int cnt = rows[i].slot < 0 ? 6 : 3;
        int a = rows[i].a, b = rows[i].b;
        v3 va = V(0, 0, 0), wa = V(0, 0, 0), vb = v0[b], wb = w0[b];
        if (a >= 0) { va = v0[a]; wa = w0[a]; }
        for (int k = 0; k < cnt; ++k) {
          row_t* r = &rows[i + k];
          int pair = (r->type == 2); /* friction rows come as a (t1,t2) pair solved together */
          int nr = pair ? 2 : 1;
          double dl[2];
          for (int t = 0; t < nr; ++t) {
            row_t* rr = &rows[i + k + t];
            double jv = vdot(rr->jlb, vb) + vdot(rr->jab, wb);
            if (a >= 0) jv += vdot(rr->jla, va) + vdot(rr->jaa, wa);
            dl[t] = -rr->meff * (jv + rr->bias);
          }
          if (r->type == 1) {
            double ln = r->lambda + dl[0];
            if (ln < 0) ln = 0;
            dl[0] = ln - r->lambda;
          } else if (pair) {
            row_t *rn = &rows[i], *r2 = &rows[i + k + 1];
            double l1 = r->lambda + dl[0], l2 = r2->lambda + dl[1];
            double lim = m->mu * rn->lambda, nrm = sqrt(l1 * l1 + l2 * l2);
            if (nrm > lim) { double sc = nrm > 0 ? lim / nrm : 0; l1 *= sc; l2 *= sc; }
            dl[0] = l1 - r->lambda; dl[1] = l2 - r2->lambda;
            double ex = sqrt(l1 * l1 + l2 * l2) - lim;
            if (ex > cone) cone = ex;
          }
          for (int t = 0; t < nr; ++t) {
            row_t* rr = &rows[i + k + t];
            rr->lambda += dl[t];
            if (a >= 0) {
              va = vadd(va, vscale(rr->jla, rr->sca * dl[t] / m->mass[a % B]));
              wa = vadd(wa, vscale(inv_inertia_apply(R[a], m->inertia[a % B], rr->jaa), rr->sca * dl[t]));
              pl[a] = vadd(pl[a], vscale(rr->jla, dl[t]));
              pa[a] = vadd(pa[a], vscale(rr->jaa, dl[t]));
            }
            vb = vadd(vb, vscale(rr->jlb, rr->scb * dl[t] / m->mass[b % B]));
            wb = vadd(wb, vscale(inv_inertia_apply(R[b], m->inertia[b % B], rr->jab), rr->scb * dl[t]));
            pl[b] = vadd(pl[b], vscale(rr->jlb, dl[t]));
            pa[b] = vadd(pa[b], vscale(rr->jab, dl[t]));
          }
          if (pair) ++k;
        }
        i += cnt;
      }
      /* every body receives the plain sum of the impulses of its blocks
       * (accumulated above in ascending block order) */
      for (int b = 0; b < NB; ++b) {
        vel[b] = vadd(vel[b], vscale(pl[b], 1.0 / m->mass[b % B]));
        om[b] = vadd(om[b], inv_inertia_apply(R[b], m->inertia[b % B], pa[b]));
      }
      if (trace && *trace_n < trace_cap) {
        oracle_sweep_trace* t = &trace[(*trace_n)++];
        t->bilateral_rms = nbil ? sqrt(sq / nbil) : 0;
        t->bilateral_max = mx;
        t->onesided_viol = viol;
        t->pos_err_max = pos_err_max;
        double sl = 0;
        for (int r = 0; r < nrows; ++r)
          if (rows[r].slot >= 0 && rows[r].type == 1) sl += rows[r].lambda;
        t->sum_lambda_n = sl;
        t->cone_excess = cone;
      }
    }
    }   /* solver */
    for (int g = 0; g < G; ++g)
      for (int b = 0; b < B; ++b) { envs[g].v[b] = vel[g * B + b]; envs[g].w[b] = om[g * B + b]; }
    /* impulses kept for the next substep's warm start (terrain slots and joints; a contact
     * between capsules always starts from zero) */
    {
      int i = 0;
      for (int g = 0; g < G; ++g) {
        env_state* e = &envs[g];
        for (int j = 0; j < J; ++j)
          for (int k = 0; k < 6; ++k) e->lam_j[j][k] = rows[i++].lambda;
        for (int s = 0; s < S; ++s) {
          e->lam_s_on[s] = e->con[s].active;
          if (!e->con[s].active) continue;
          for (int k = 0; k < 3; ++k) e->lam_s[s][k] = rows[i++].lambda;
        }
      }
    }
  }

  /* 5. damping, angular-velocity cap, position integration */
  if (phases & ORACLE_PH_INTEGRATE) {
    for (int g = 0; g < G; ++g) {
      env_state* e = &envs[g];
      for (int b = 0; b < B; ++b) {
        e->v[b] = vscale(e->v[b], 1.0 / (1.0 + h * m->c_lin));
        e->w[b] = vscale(e->w[b], 1.0 / (1.0 + h * m->c_ang));
        double wn = vnorm(e->w[b]);
        if (wn > m->w_max) e->w[b] = vscale(e->w[b], m->w_max / wn);
        e->x[b] = vadd(e->x[b], vscale(e->v[b], h));
        quat wq = {0, e->w[b].x, e->w[b].y, e->w[b].z};
        quat dq = qmul(wq, e->q[b]);
        quat qn = {e->q[b].w + 0.5 * h * dq.w, e->q[b].x + 0.5 * h * dq.x, e->q[b].y + 0.5 * h * dq.y,
                   e->q[b].z + 0.5 * h * dq.z};
        e->q[b] = qnormalize(qn);
      }
    }
  }
}

/* ------------------------------------------------------------ obs / reward */

static double terrain_height_at(const model* m, double wx, double wy) {
  if (m->terrain_kind == 0) return 0.0;
  double ux = (wx - (double)(float)m->hox) / m->cell, uy = (wy - (double)(float)m->hoy) / m->cell;
  int ncx = m->nx - 1, ncy = m->ny - 1;
  double fi = floor(ux), fj = floor(uy);
  if (fi < 0) fi = 0; if (fi > ncx - 1) fi = ncx - 1;
  if (fj < 0) fj = 0; if (fj > ncy - 1) fj = ncy - 1;
  int i = (int)fi, j = (int)fj;
  double fx = ux - fi, fy = uy - fj;
  if (fx < 0) fx = 0; if (fx > 1) fx = 1;
  if (fy < 0) fy = 0; if (fy > 1) fy = 1;
  double h00 = m->heights[(size_t)j * m->nx + i], h10 = m->heights[(size_t)j * m->nx + i + 1];
  double h11 = m->heights[(size_t)(j + 1) * m->nx + i + 1], h01 = m->heights[(size_t)(j + 1) * m->nx + i];
  /* plane of the triangle on this side of the (i,j)-(i+1,j+1) diagonal */
  if (fx >= fy) return h00 + fx * (h10 - h00) + fy * (h11 - h10);
  return h00 + fx * (h11 - h01) + fy * (h01 - h00);
}

/* Height map of the complex-terrain task (Section 4.1): a 15 x 11 rectangular grid of terrain
 * heights that follows the robot's centre of mass, denser near the robot.  The paper gives the
 * size only; this reading: the grid is aligned with the root body's heading (yaw), row i runs
 * along the heading at offset s(i - 4), column j across it at offset s(j - 5) (positive to the
 * left), with s(k) = sign(k) 0.15 (1.3^|k| - 1) / 0.3 metres (0, 0.15, 0.35, 0.60, ... : 0.93 m
 * behind to 6.4 m ahead, 1.36 m to either side); each entry is the terrain height under the
 * sample minus the height of the centre of mass (0 for the plane); samples beyond the field read
 * its nearest border cell.  Entries follow the other observations, row by row. */
#define HM_ROWS 15
#define HM_COLS 11
static double hm_offset(int k) {
  int a = k < 0 ? -k : k;
  double s = 0.15 * (pow(1.3, a) - 1.0) / 0.3;
  return k < 0 ? -s : s;
}
static void pack_height_map(const model* m, const env_state* e, double* out) {
  v3 com = V(0, 0, 0);
  double mt = 0;
  for (int b = 0; b < m->B; ++b) { com = vadd(com, vscale(e->x[b], m->mass[b])); mt += m->mass[b]; }
  com = vadd(vscale(com, 1.0 / mt), e->origin);
  quat q = e->q[m->root];
  double yaw = atan2(2 * (q.w * q.z + q.x * q.y), 1 - 2 * (q.y * q.y + q.z * q.z));
  double c = cos(yaw), s = sin(yaw);
  for (int i = 0; i < HM_ROWS; ++i)
    for (int j = 0; j < HM_COLS; ++j) {
      double f = hm_offset(i - 4), l = hm_offset(j - 5);
      double wx = com.x + c * f - s * l, wy = com.y + s * f + c * l;
      double hz = m->terrain_kind == 0 ? 0.0 : terrain_height_at(m, wx, wy);
      out[i * HM_COLS + j] = hz - com.z;
    }
}

static void pack_obs(const model* m, const env_state* e, double* obs, double* reward, uint8_t* done) {
  int D = m->D, rb = m->root, o = 0;
  quat q = e->q[rb];
  v3 x = e->x[rb];
  double height = x.z + e->origin.z - terrain_height_at(m, x.x + e->origin.x, x.y + e->origin.y);
  if (m->terrain_kind == 0) height = x.z;
  double roll = atan2(2 * (q.w * q.x + q.y * q.z), 1 - 2 * (q.x * q.x + q.y * q.y));
  double sp = 2 * (q.w * q.y - q.z * q.x);
  if (sp > 1) sp = 1; if (sp < -1) sp = -1;
  double pitch = asin(sp);
  double yaw = atan2(2 * (q.w * q.z + q.x * q.y), 1 - 2 * (q.y * q.y + q.z * q.z));
  double tx = e->target[0] - x.x, ty = e->target[1] - x.y;
  double psi = atan2(ty, tx) - yaw;
  obs[o++] = height; obs[o++] = roll; obs[o++] = pitch;
  obs[o++] = e->v[rb].x; obs[o++] = e->v[rb].y; obs[o++] = e->v[rb].z;
  obs[o++] = e->w[rb].x; obs[o++] = e->w[rb].y; obs[o++] = e->w[rb].z;
  obs[o++] = sin(psi); obs[o++] = cos(psi);
  int n_limit = 0;
  for (int j = 0; j < m->J; ++j) {
    double th[3];
    joint_theta(m, e, j, th);
    v3 Ra[3], xa; quat qa;
    joint_frames(m, e, j, Ra, &xa, &qa);
    v3 wrel = e->w[m->jc[j]];
    if (m->jp[j] >= 0) wrel = vsub(wrel, e->w[m->jp[j]]);
    for (int k = 0; k < 3; ++k) {
      if (m->jmode[j][k] != 1) continue;
      int a = m->jact[j][k];
      obs[11 + a] = th[k];
      obs[11 + D + a] = vdot(mrot(Ra, m->jaxes[j][k]), wrel);
      obs[11 + 2 * D + a] = e->u[a];
      double g = th[k] - m->jlo[j][k], g2 = m->jhi[j][k] - th[k];
      if (g2 < g) g = g2;
      if (g <= 0) n_limit++;
    }
  }
  int n_feet = 0;
  for (int f = 0; f < m->F; ++f) {
    int flag = 0;
    for (int s = 0; s < m->S; ++s)
      if (m->slots[s].body == m->feet[f] && e->con[s].active && e->con[s].d <= 0.005) flag = 1;
    obs[11 + 3 * D + f] = flag;
    n_feet += flag;
  }
  if (m->height_map) pack_height_map(m, e, obs + 11 + 3 * D + m->F);
  /* reward, Eq. (1)-(3) */
  double tn = sqrt(tx * tx + ty * ty);
  double S = tn > 0 ? (e->v[rb].x * tx + e->v[rb].y * ty) / tn : 0.0;
  double ct = cos(psi);
  double r_heading = ct > 0.8 ? 1.0 : ct / 0.8;
  double cvert = 1 - 2 * (q.x * q.x + q.y * q.y);
  double r_standing = cvert > 0.93 ? 1.0 : 0.0;
  double l1 = 0, l2 = 0;
  for (int a = 0; a < D; ++a) { l1 += fabs(e->u[a]); l2 += e->u[a] * e->u[a]; }
  *reward = m->alive_bonus + S + 0.5 * r_heading + 0.05 * r_standing - 4.0 * l1 - 0.5 * l2 -
            0.2 * n_limit - 1.0 * n_feet;
  *done = (height < m->term_height || e->steps >= m->max_steps) ? 1 : 0;
}

/* -------------------------------------------------------------- interface */

oracle_sim* oracle_create(const oracle_desc* d, int32_t N) {
  if (d->n_bodies > MAXB || d->n_joints > MAXJ || d->n_dofs > MAXD || d->n_feet > 8) return NULL;
  oracle_sim* o = (oracle_sim*)calloc(1, sizeof(oracle_sim));
  model* m = &o->m;
  m->B = d->n_bodies; m->J = d->n_joints; m->D = d->n_dofs; m->F = d->n_feet;
  for (int b = 0; b < m->B; ++b) {
    m->radius[b] = d->radius[b]; m->half_len[b] = d->half_len[b]; m->axis[b] = d->axis[b];
    m->mass[b] = d->mass[b];
    m->inertia[b] = V(d->inertia[3 * b], d->inertia[3 * b + 1], d->inertia[3 * b + 2]);
    m->rest_pos[b] = V(d->rest_pos[3 * b], d->rest_pos[3 * b + 1], d->rest_pos[3 * b + 2]);
  }
  for (int j = 0; j < m->J; ++j) {
    int a = d->j_parent[j], b = d->j_child[j];
    m->jp[j] = a; m->jc[j] = b;
    v3 anc = V(d->j_anchor[3 * j], d->j_anchor[3 * j + 1], d->j_anchor[3 * j + 2]);
    m->la[j] = a >= 0 ? vsub(anc, m->rest_pos[a]) : anc;
    m->lb[j] = vsub(anc, m->rest_pos[b]);
    for (int k = 0; k < 3; ++k) {
      const double* ax = &d->j_axes[9 * j + 3 * k];
      m->jaxes[j][k] = V(ax[0], ax[1], ax[2]);
      m->jmode[j][k] = d->j_mode[3 * j + k]; m->jact[j][k] = d->j_act[3 * j + k];
      m->jlo[j][k] = d->j_lo[3 * j + k]; m->jhi[j][k] = d->j_hi[3 * j + k];
      m->jgear[j][k] = d->j_gear[3 * j + k];
    }
    if (a >= 0) m->body_joint_count[a]++;
    m->body_joint_count[b]++;
  }
  m->root = d->root_body;
  for (int f = 0; f < m->F; ++f) m->feet[f] = d->feet[f];
  m->term_height = d->term_height; m->alive_bonus = d->alive_bonus;
  m->terrain_kind = d->terrain_kind; m->nx = d->hf_nx; m->ny = d->hf_ny;
  m->cell = d->hf_cell; m->hox = d->hf_origin[0]; m->hoy = d->hf_origin[1];
  if (m->terrain_kind == 1) {
    size_t n = (size_t)m->nx * m->ny;
    m->heights = (float*)malloc(n * sizeof(float));
    memcpy(m->heights, d->hf_heights, n * sizeof(float));
  }
  int S = 0;
  for (int b = 0; b < m->B; ++b) {
    if (m->half_len[b] > 0) {
      m->slots[S].body = b; m->slots[S++].kind = 0;
      m->slots[S].body = b; m->slots[S++].kind = 1;
      if (m->terrain_kind == 1) { m->slots[S].body = b; m->slots[S++].kind = 2; }
    } else { m->slots[S].body = b; m->slots[S++].kind = 1; }
  }
  m->S = S;
  m->g = V(d->gravity[0], d->gravity[1], d->gravity[2]);
  m->mu = d->mu; m->margin = d->margin; m->beta_j = d->beta_joint; m->beta_c = d->beta_contact;
  m->v_depen = d->max_depen_vel; m->c_lin = d->lin_damping; m->c_ang = d->ang_damping;
  m->w_max = d->max_ang_vel; m->reset_noise = d->reset_noise;
  m->gyro = d->gyroscopic; m->contacts = d->contacts; m->max_steps = d->max_episode_steps; m->height_map = d->height_map;
  m->NP = 0;
  for (int p = 0; p < d->n_collide_pairs && p < MAXP; ++p) {
    m->pair_a[m->NP] = d->collide_pairs[2 * p]; m->pair_b[m->NP] = d->collide_pairs[2 * p + 1]; m->NP++;
  }
  m->G = d->group_size < 1 ? 1 : (d->group_size > MAXG ? MAXG : d->group_size);
  o->N = N; o->threads = 1;
  o->env = (env_state*)calloc((size_t)N, sizeof(env_state));
  int groups = (N + m->G - 1) / m->G;
  o->pcon = (oracle_pair_contact*)calloc((size_t)groups * MAXPC, sizeof(oracle_pair_contact));
  o->pcon_n = (int*)calloc((size_t)groups, sizeof(int));
  o->place_env = (int*)malloc(sizeof(int) * (size_t)N);
  for (int p = 0; p < N; ++p) o->place_env[p] = p;
  o->regrouped = 0;
  for (int e = 0; e < N; ++e) {
    o->env[e].origin = V(d->env_origins[3 * e], d->env_origins[3 * e + 1], d->env_origins[3 * e + 2]);
    o->env[e].target[0] = 1000.0; o->env[e].target[1] = 0.0;
    for (int s = 0; s < MAXS; ++s) clear_contact(&o->env[e].con[s]);
  }
  o->trace_env = -1;
  oracle_reset(o, NULL, 0);
  return o;
}

void oracle_destroy(oracle_sim* o) {
  if (!o) return;
  free(o->m.heights); free(o->env); free(o->pcon); free(o->pcon_n); free(o->place_env); free(o);
}
int32_t oracle_n_slots(const oracle_sim* o) { return o->m.S; }
int32_t oracle_obs_dim(const oracle_sim* o) { return 11 + 3 * o->m.D + o->m.F + (o->m.height_map ? HM_ROWS * HM_COLS : 0); }
void oracle_set_threads(oracle_sim* o, int32_t n) { o->threads = n < 1 ? 1 : n; }
int32_t oracle_get_threads(const oracle_sim* o) { return o->threads; }

/* counter-based uniform generator: one splitmix64 finaliser per (seed, env, idx) */
static uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ULL;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}
double oracle_uniform(uint64_t seed, uint64_t env, uint64_t idx) {
  uint64_t z = mix64(seed + env * 0x632BE59BD9B4E019ULL + idx * 0xD1B54A32D192ED03ULL);
  return (double)(z >> 40) * (1.0 / 16777216.0);
}

/* Reset (Section 4.1, initial state perturbed slightly): rest pose translated by
 * uniform noise, common linear velocity noise, every hinge angle perturbed and
 * clipped to its limits; bodies placed parents-first through the joint list. */
static void reset_env(const model* m, env_state* e, int ei, uint64_t seed) {
  double a = m->reset_noise;
  {
    v3 off, vel;
    off = V(a * (2 * oracle_uniform(seed, ei, 0) - 1), a * (2 * oracle_uniform(seed, ei, 1) - 1),
            a * (2 * oracle_uniform(seed, ei, 2) - 1));
    vel = V(a * (2 * oracle_uniform(seed, ei, 3) - 1), a * (2 * oracle_uniform(seed, ei, 4) - 1),
            a * (2 * oracle_uniform(seed, ei, 5) - 1));
    for (int b = 0; b < m->B; ++b) {
      e->x[b] = vadd(m->rest_pos[b], off);
      e->q[b].w = 1; e->q[b].x = e->q[b].y = e->q[b].z = 0;
      e->v[b] = vel; e->w[b] = V(0, 0, 0);
    }
    for (int j = 0; j < m->J; ++j) {
      v3 phi = V(0, 0, 0);
      for (int k = 0; k < 3; ++k) {
        if (m->jmode[j][k] != 1) continue;
        double th = a * (2 * oracle_uniform(seed, ei, 8 + 3 * j + k) - 1);
        if (th < m->jlo[j][k]) th = m->jlo[j][k];
        if (th > m->jhi[j][k]) th = m->jhi[j][k];
        phi = vadd(phi, vscale(m->jaxes[j][k], th));
      }
      int pa = m->jp[j], b = m->jc[j];
      quat qa; v3 xa, Ra[3], Rb[3];
      joint_frames(m, e, j, Ra, &xa, &qa);
      e->q[b] = qnormalize(qmul(qa, qexp(phi)));
      qmat(e->q[b], Rb);
      e->x[b] = vsub(vadd(xa, mrot(Ra, m->la[j])), mrot(Rb, m->lb[j]));
      /* joint angular velocities (Section 4.1: perturbed slightly as well): a rate about every
       * hinge axis; the child turns with the parent plus these rates, and its centre moves so
       * that the two anchor points share one velocity (the world as a parent stands still) */
      v3 va = V(0, 0, 0), wa = V(0, 0, 0), wb;
      if (pa >= 0) { va = e->v[pa]; wa = e->w[pa]; }
      wb = wa;
      for (int k = 0; k < 3; ++k) {
        if (m->jmode[j][k] != 1) continue;
        double rate = a * (2 * oracle_uniform(seed, ei, 256 + 3 * j + k) - 1);
        wb = vadd(wb, vscale(mrot(Ra, m->jaxes[j][k]), rate));
      }
      e->w[b] = wb;
      e->v[b] = vsub(vadd(va, vcross(wa, mrot(Ra, m->la[j]))), vcross(wb, mrot(Rb, m->lb[j])));
    }
    e->steps = 0;
    for (int d = 0; d < m->D; ++d) e->u[d] = 0;
    for (int s = 0; s < MAXS; ++s) clear_contact(&e->con[s]);
    e->has_store = 0;
    clear_warm(e);
  }
}
void oracle_reset(oracle_sim* o, const uint8_t* mask, uint64_t seed) {
  for (int ei = 0; ei < o->N; ++ei) {
    if (mask && !mask[ei]) continue;
    reset_env(&o->m, &o->env[ei], ei, seed);
  }
}

/* ---- task logic (Section 4.1): draws are keyed by (seed, episode, env, frame, k) ---- */
static double task_u(const oracle_task* t, int env, int episode, int frame, int k) {
  return oracle_uniform(t->seed + (uint64_t)episode * 0x9E3779B97F4A7C15ULL, (uint64_t)env,
                        (uint64_t)(1024 + 8 * frame + k));
}
static int task_interval(const oracle_task* t, int env, int episode, int frame) {
  int span = t->push_max_frames - t->push_min_frames + 1;
  int d = t->push_min_frames + (int)floor(task_u(t, env, episode, frame, 2) * span);
  return d > t->push_max_frames ? t->push_max_frames : d;
}
static void task_draw_target(const oracle_task* t, const model* m, env_state* e, int env, int frame) {
  double r = t->target_radius * sqrt(task_u(t, env, e->episode, frame, 3));
  double phi = 2.0 * 3.14159265358979323846 * task_u(t, env, e->episode, frame, 4);
  e->target[0] = e->x[m->root].x + r * cos(phi);
  e->target[1] = e->x[m->root].y + r * sin(phi);
  e->target_age = 0;
}
static void task_begin_episode(const oracle_task* t, const model* m, env_state* e, int env) {
  e->fall_frames = 0; e->target_age = 0;
  e->next_push = t->push_max_frames > 0 ? task_interval(t, env, e->episode, 0) : -1;
  if (t->target_period > 0) task_draw_target(t, m, e, env, 0);
}
void oracle_set_task(oracle_sim* o, const oracle_task* task) {
  if (!task || !task->enabled) { memset(&o->task, 0, sizeof(o->task)); for (int e = 0; e < o->N; ++e) { o->env[e].push = V(0, 0, 0); o->env[e].has_store = 0; } return; }
  o->task = *task;
  for (int e = 0; e < o->N; ++e) {
    o->env[e].episode = 0;
    o->env[e].push = V(0, 0, 0);
    o->env[e].has_store = 0;
    task_begin_episode(&o->task, &o->m, &o->env[e], e);
  }
}
void oracle_get_task_state(const oracle_sim* o, int32_t* c, double* t) {
  for (int e = 0; e < o->N; ++e) {
    const env_state* E = &o->env[e];
    c[4 * e] = E->fall_frames; c[4 * e + 1] = E->target_age; c[4 * e + 2] = E->next_push; c[4 * e + 3] = E->episode;
    t[2 * e] = E->target[0]; t[2 * e + 1] = E->target[1];
  }
}
void oracle_set_task_state(oracle_sim* o, const int32_t* c, const double* t) {
  for (int e = 0; e < o->N; ++e) {
    env_state* E = &o->env[e];
    E->fall_frames = c[4 * e]; E->target_age = c[4 * e + 1]; E->next_push = c[4 * e + 2]; E->episode = c[4 * e + 3];
    E->target[0] = t[2 * e]; E->target[1] = t[2 * e + 1];
  }
}
void oracle_get_last_push(const oracle_sim* o, double* p) {
  for (int e = 0; e < o->N; ++e) { p[3 * e] = o->env[e].push.x; p[3 * e + 1] = o->env[e].push.y; p[3 * e + 2] = o->env[e].push.z; }
}
/* before the substeps of a frame: is this the frame of a push? */
static void task_before_step(const oracle_task* t, env_state* e, int env) {
  e->push = V(0, 0, 0);
  if (t->push_max_frames > 0 && e->steps == e->next_push) {
    int f = e->steps;
    double mag = t->push_min_newton + (t->push_max_newton - t->push_min_newton) * task_u(t, env, e->episode, f, 0);
    double phi = 2.0 * 3.14159265358979323846 * task_u(t, env, e->episode, f, 1);
    e->push = V(mag * cos(phi), mag * sin(phi), 0.0);
    e->next_push = f + task_interval(t, env, e->episode, f);
  }
}
/* after the substeps (steps already counted): pack, termination with grace, target, auto-reset */
static void task_after_step(const oracle_task* t, const model* m, env_state* e, int env) {
  uint8_t dn;
  pack_obs(m, e, e->obs_store, &e->rew_store, &dn);
  int below = e->obs_store[0] < m->term_height;
  e->fall_frames = below ? e->fall_frames + 1 : 0;
  e->done_store = (e->fall_frames > t->fall_grace_frames || e->steps >= m->max_steps) ? 1 : 0;
  e->has_store = 1;
  if (t->target_period > 0) {
    e->target_age += 1;
    double dx = e->target[0] - e->x[m->root].x, dy = e->target[1] - e->x[m->root].y;
    if (e->target_age >= t->target_period || sqrt(dx * dx + dy * dy) < t->target_reach)
      task_draw_target(t, m, e, env, e->steps);
  }
  if (e->done_store && t->auto_reset) {
    e->episode += 1;
    reset_env(m, e, env, t->seed + (uint64_t)e->episode * 0x9E3779B97F4A7C15ULL);
    task_begin_episode(t, m, e, env);
    double r; uint8_t d2;
    pack_obs(m, e, e->obs_store, &r, &d2);   /* first observation of the new episode */
    e->has_store = 1;
  }
}

void oracle_set_state(oracle_sim* o, const double* st) {
  int B = o->m.B;
  for (int e = 0; e < o->N; ++e)
    for (int b = 0; b < B; ++b) {
      const double* s = st + ((size_t)e * B + b) * 13;
      env_state* E = &o->env[e];
      E->x[b] = V(s[0], s[1], s[2]);
      E->q[b].w = s[3]; E->q[b].x = s[4]; E->q[b].y = s[5]; E->q[b].z = s[6];
      E->v[b] = V(s[7], s[8], s[9]); E->w[b] = V(s[10], s[11], s[12]);
      E->has_store = 0;
      clear_warm(E);
    }
}
void oracle_set_solver(oracle_sim* o, int32_t kind, int32_t krylov_iters, double reg) {
  o->m.solver = kind == 1 ? 1 : 0;
  o->m.krylov_iters = krylov_iters < 0 ? 0 : krylov_iters;
  o->m.newton_reg = reg < 0 ? 0 : reg;
}
void oracle_set_warm_start(oracle_sim* o, double share) { o->m.warm = share < 0 ? 0 : (share > 1 ? 1 : share); }
void oracle_set_warm(oracle_sim* o, const double* lam_j, const double* lam_s) {
  const int J = o->m.J, S = o->m.S;
  for (int e = 0; e < o->N; ++e) {
    env_state* E = &o->env[e];
    for (int j = 0; j < J; ++j) {
      for (int k = 0; k < 6; ++k) E->lam_j[j][k] = lam_j[((size_t)e * J + j) * 6 + k];
      for (int k = 0; k < 3; ++k) E->side_j[j][k] = -1;   /* stands for whichever limit is nearer */
    }
    for (int q = 0; q < S; ++q) {
      E->lam_s_on[q] = 1;
      for (int k = 0; k < 3; ++k) E->lam_s[q][k] = lam_s[((size_t)e * S + q) * 3 + k];
    }
  }
}
void oracle_set_warm_flags(oracle_sim* o, const int32_t* limit_side, const int32_t* slot_was_active) {
  const int J = o->m.J, S = o->m.S;
  for (int e = 0; e < o->N; ++e) {
    env_state* E = &o->env[e];
    for (int j = 0; j < J; ++j)
      for (int k = 0; k < 3; ++k) E->side_j[j][k] = limit_side[((size_t)e * J + j) * 3 + k];
    for (int q = 0; q < S; ++q) E->lam_s_on[q] = slot_was_active[(size_t)e * S + q] ? 1 : 0;
  }
}
void oracle_get_warm(const oracle_sim* o, double* lam_j, double* lam_s) {
  const int J = o->m.J, S = o->m.S;
  for (int e = 0; e < o->N; ++e) {
    const env_state* E = &o->env[e];
    for (int j = 0; j < J; ++j)
      for (int k = 0; k < 6; ++k) lam_j[((size_t)e * J + j) * 6 + k] = E->lam_j[j][k];
    for (int q = 0; q < S; ++q)
      for (int k = 0; k < 3; ++k) lam_s[((size_t)e * S + q) * 3 + k] = E->lam_s_on[q] ? E->lam_s[q][k] : 0.0;
  }
}
void oracle_get_state(const oracle_sim* o, double* st) {
  int B = o->m.B;
  for (int e = 0; e < o->N; ++e)
    for (int b = 0; b < B; ++b) {
      double* s = st + ((size_t)e * B + b) * 13;
      const env_state* E = &o->env[e];
      s[0] = E->x[b].x; s[1] = E->x[b].y; s[2] = E->x[b].z;
      s[3] = E->q[b].w; s[4] = E->q[b].x; s[5] = E->q[b].y; s[6] = E->q[b].z;
      s[7] = E->v[b].x; s[8] = E->v[b].y; s[9] = E->v[b].z;
      s[10] = E->w[b].x; s[11] = E->w[b].y; s[12] = E->w[b].z;
    }
}
void oracle_set_targets(oracle_sim* o, const double* t) {
  for (int e = 0; e < o->N; ++e) { o->env[e].target[0] = t[2 * e]; o->env[e].target[1] = t[2 * e + 1]; }
}
void oracle_set_step_count(oracle_sim* o, const int32_t* c) {
  for (int e = 0; e < o->N; ++e) o->env[e].steps = c[e];
}

static void load_actions(oracle_sim* o, const double* actions) {
  int D = o->m.D;
  for (int e = 0; e < o->N; ++e)
    for (int d = 0; d < D; ++d) {
      double u = actions ? actions[(size_t)e * D + d] : 0.0;
      o->env[e].u[d] = u < -1 ? -1 : (u > 1 ? 1 : u);
    }
}

/* agents [e0, e0 + G) of interaction group gi */
static int group_span(const oracle_sim* o, int gi, int* e0) {
  *e0 = gi * o->m.G;
  return *e0 + o->m.G <= o->N ? o->m.G : o->N - *e0;
}

/* ---- bounded contact store: the `cap` contacts with the smallest (gap32, key) of a block stay */
typedef struct { uint64_t word; int group, index; } cap_entry;
static int cap_entry_cmp(const void* a, const void* b) {
  uint64_t x = ((const cap_entry*)a)->word, y = ((const cap_entry*)b)->word;
  return x < y ? -1 : (x > y ? 1 : 0);
}
static uint64_t cap_word(const oracle_pair_contact* c, int unit_e0) {
  uint32_t gb;
  memcpy(&gb, &c->gap32, 4);
  uint32_t ordered = (gb & 0x80000000u) ? ~gb : (gb | 0x80000000u); /* unsigned order = order of the floats */
  uint32_t key = ((uint32_t)(c->env_a - unit_e0) << 20) | ((uint32_t)(c->env_b - unit_e0) << 8) |
                 ((uint32_t)c->body_a << 4) | (uint32_t)c->body_b;
  return ((uint64_t)ordered << 32) | key;
}
/* groups [g0, g1) form one block; their lists keep their order, minus what does not fit */
static int trim_pair_contacts(oracle_sim* o, int g0, int g1) {
  int total = 0;
  for (int gi = g0; gi < g1; ++gi) total += o->pcon_n[gi];
  if (total <= o->pair_cap) return 0;
  cap_entry* ent = (cap_entry*)malloc(sizeof(cap_entry) * (size_t)total);
  int n = 0, unit_e0 = g0 * o->m.G;
  for (int gi = g0; gi < g1; ++gi)
    for (int k = 0; k < o->pcon_n[gi]; ++k, ++n) {
      ent[n].word = cap_word(&o->pcon[(size_t)gi * MAXPC + k], unit_e0); ent[n].group = gi; ent[n].index = k;
    }
  qsort(ent, (size_t)total, sizeof(cap_entry), cap_entry_cmp);
  uint64_t last_kept = ent[o->pair_cap - 1].word;
  free(ent);
  for (int gi = g0; gi < g1; ++gi) {
    oracle_pair_contact* list = o->pcon + (size_t)gi * MAXPC;
    int kept = 0;
    for (int k = 0; k < o->pcon_n[gi]; ++k)
      if (cap_word(&list[k], unit_e0) <= last_kept) list[kept++] = list[k];
    o->pcon_n[gi] = kept;
  }
  return total - o->pair_cap;
}
static int groups_per_unit(const oracle_sim* o) {
  int groups = (o->N + o->m.G - 1) / o->m.G;
  if (o->pair_cap <= 0) return 1;
  int gpu = o->pair_unit / o->m.G;
  return gpu < 1 ? 1 : (gpu > groups ? groups : gpu);
}
/* one substep of the groups [g0, g1): with a bounded store all of them find their contacts
 * first, the block is trimmed, then each group goes on */
static long long substep_groups(oracle_sim* o, int g0, int g1, double h, int iterations, int phases) {
  long long removed = 0;
  for (int pass = 0; pass < 2; ++pass) {
    int ph = phases & (pass == 0 ? ORACLE_PH_CONTACTS : ~ORACLE_PH_CONTACTS);
    if (o->pair_cap <= 0) ph = pass == 0 ? phases : 0;   /* no bound: each group in one go */
    if (ph)
      for (int gi = g0; gi < g1; ++gi) {
        int e0, G = group_span(o, gi, &e0);
        int tr = 0;
        for (int g = 0; g < G; ++g) tr |= (o->place_env[e0 + g] == o->trace_env);
        env_state* members = &o->env[e0];
        if (o->regrouped) {
          /* the members of the group side by side for the substep, then back to their own places */
          members = (env_state*)malloc(sizeof(env_state) * (size_t)G);
          for (int g = 0; g < G; ++g) members[g] = o->env[o->place_env[e0 + g]];
        }
        substep(&o->m, members, e0, G, o->pcon + (size_t)gi * MAXPC, &o->pcon_n[gi], h, iterations, ph,
                tr ? o->trace : NULL, &o->trace_n, o->trace_cap);
        if (o->regrouped) {
          for (int g = 0; g < G; ++g) o->env[o->place_env[e0 + g]] = members[g];
          free(members);
        }
      }
    if (pass == 0 && (phases & ORACLE_PH_CONTACTS) && o->pair_cap > 0) removed += trim_pair_contacts(o, g0, g1);
  }
  return removed;
}

void oracle_substep_phases(oracle_sim* o, const double* actions, double h, int32_t iterations, int32_t phases) {
  load_actions(o, actions);
  int groups = (o->N + o->m.G - 1) / o->m.G, gpu = groups_per_unit(o);
  for (int g0 = 0; g0 < groups; g0 += gpu)
    o->pair_removed += substep_groups(o, g0, g0 + gpu < groups ? g0 + gpu : groups, h, iterations, phases);
}

void oracle_step(oracle_sim* o, const double* actions, double dt, int32_t substeps, int32_t iterations) {
  load_actions(o, actions);
  double h = dt / substeps;
  int groups = (o->N + o->m.G - 1) / o->m.G, gpu = groups_per_unit(o);
  int units = (groups + gpu - 1) / gpu;
  long long removed = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(o->threads) reduction(+ : removed)
#endif
  for (int u = 0; u < units; ++u) {
    int g0 = u * gpu, g1 = g0 + gpu < groups ? g0 + gpu : groups;
    int p_lo = g0 * o->m.G, p_hi = g1 * o->m.G < o->N ? g1 * o->m.G : o->N;
    if (o->task.enabled)
      for (int p = p_lo; p < p_hi; ++p) { int e = o->place_env[p]; task_before_step(&o->task, &o->env[e], e); }
    for (int s = 0; s < substeps; ++s) removed += substep_groups(o, g0, g1, h, iterations, ORACLE_PH_ALL);
    for (int p = p_lo; p < p_hi; ++p) {
      int e = o->place_env[p];
      o->env[e].steps++;
      if (o->task.enabled) task_after_step(&o->task, &o->m, &o->env[e], e);
    }
  }
  o->pair_removed += removed;
}

int64_t oracle_set_pair_cap(oracle_sim* o, int32_t cap, int32_t envs_per_unit) {
  long long r = o->pair_removed;
  o->pair_removed = 0;
  o->pair_cap = cap > 0 ? cap : 0;
  o->pair_unit = envs_per_unit > 0 ? envs_per_unit : o->m.G;
  return r;
}

/* a contact as the caller sees it: agents by their own numbers, not by place */
static oracle_pair_contact by_agent(const oracle_sim* o, oracle_pair_contact c) {
  c.env_a = o->place_env[c.env_a]; c.env_b = o->place_env[c.env_b];
  return c;
}
int32_t oracle_get_pair_contacts(const oracle_sim* o, oracle_pair_contact* out, int32_t cap) {
  int n = 0, groups = (o->N + o->m.G - 1) / o->m.G;
  for (int gi = 0; gi < groups; ++gi)
    for (int k = 0; k < o->pcon_n[gi]; ++k, ++n)
      if (n < cap) out[n] = by_agent(o, o->pcon[(size_t)gi * MAXPC + k]);
  return n;
}

int32_t oracle_generate_pair_contacts(oracle_sim* o, oracle_pair_contact* out, int32_t cap) {
  int n = 0, groups = (o->N + o->m.G - 1) / o->m.G;
  oracle_pair_contact* tmp = (oracle_pair_contact*)malloc(sizeof(oracle_pair_contact) * MAXPC);
  for (int gi = 0; gi < groups; ++gi) {
    int e0, G = group_span(o, gi, &e0);
    env_state* members = (env_state*)malloc(sizeof(env_state) * (size_t)G);
    for (int g = 0; g < G; ++g) members[g] = o->env[o->place_env[e0 + g]];
    int k = generate_pair_contacts(&o->m, members, e0, G, tmp);
    free(members);
    for (int i = 0; i < k; ++i, ++n)
      if (n < cap) out[n] = by_agent(o, tmp[i]);
  }
  free(tmp);
  return n;
}

/* ---- interaction groups chosen from where the agents are (Section 3.1: all agents share one
 * scene; Section 4.1: the agents of the flagrun tasks collide with each other).  A uniform grid
 * of `cell` metres over the ground plane; an agent's cell is that of its root body's world
 * position; agents are ordered along the Hilbert curve through the cells (ties: agent number);
 * inside windows of that order the groups are formed from agents within reach of each other
 * (oracle_regroup below).  All decisions in single precision. */
/* position of cell (x, y), 16 bits each, along the Hilbert curve of order 16: level by level
 * from the top bit, quadrant (rx, ry) contributes ((3 rx) xor ry) quadrant sizes; inside the
 * quadrant the coordinates are reflected (lower right quadrant) and exchanged (both lower
 * quadrants) so that the sub-curve starts where the curve enters the quadrant */
static uint32_t hilbert_index16(uint32_t x, uint32_t y) {
  uint32_t d = 0;
  for (int level = 15; level >= 0; --level) {
    uint32_t side = 1u << level, rx = (x >> level) & 1u, ry = (y >> level) & 1u;
    d += side * side * ((3u * rx) ^ ry);
    x &= side - 1u; y &= side - 1u;
    if (ry == 0u) {
      if (rx == 1u) { x = side - 1u - x; y = side - 1u - y; }
      uint32_t t = x; x = y; y = t;
    }
  }
  return d;
}
static uint32_t cell_coord(float p, float cell) {
  float c = floorf(p / cell);
  if (!(c >= -32768.0f)) c = -32768.0f;   /* (also catches NaN) */
  if (c > 32767.0f) c = 32767.0f;
  return (uint32_t)((int)c + 32768);
}
typedef struct { uint64_t word; } order_entry;
static int order_entry_cmp(const void* a, const void* b) {
  uint64_t x = ((const order_entry*)a)->word, y = ((const order_entry*)b)->word;
  return x < y ? -1 : (x > y ? 1 : 0);
}
static void root_world_f32(const oracle_sim* o, int e, float p[3]) {
  const env_state* E = &o->env[e];
  const v3 x = E->x[o->m.root];
  p[0] = (float)x.x + (float)E->origin.x; p[1] = (float)x.y + (float)E->origin.y; p[2] = (float)x.z + (float)E->origin.z;
}
/* counts[0]: agent pairs whose roots are within `reach`; counts[1]: those of them that the
 * current groups keep apart (they cannot collide) */
void oracle_count_near_pairs(const oracle_sim* o, double reach, int64_t* counts) {
  const int N = o->N, G = o->m.G;
  int* place_of = (int*)malloc(sizeof(int) * (size_t)N);
  float* P = (float*)malloc(sizeof(float) * 3 * (size_t)N);
  for (int p = 0; p < N; ++p) place_of[o->place_env[p]] = p;
  for (int e = 0; e < N; ++e) root_world_f32(o, e, P + 3 * e);
  const float r = (float)reach, r2 = r * r;
  counts[0] = counts[1] = 0;
  for (int i = 0; i < N; ++i)
    for (int j = i + 1; j < N; ++j) {
      float dx = P[3 * i] - P[3 * j], dy = P[3 * i + 1] - P[3 * j + 1], dz = P[3 * i + 2] - P[3 * j + 2];
      float d2 = (dx * dx + dy * dy) + dz * dz;
      if (d2 <= r2) { counts[0]++; if (place_of[i] / G != place_of[j] / G) counts[1]++; }
    }
  free(P); free(place_of);
}
#define GROUP_WINDOW 256
void oracle_regroup(oracle_sim* o, double cell, double reach) {
  const int N = o->N, G = o->m.G;
  const float cs = (float)cell, r = (float)reach, r2 = r * r;
  order_entry* ent = (order_entry*)malloc(sizeof(order_entry) * (size_t)N);
  for (int e = 0; e < N; ++e) {
    float p[3];
    root_world_f32(o, e, p);
    uint32_t key = hilbert_index16(cell_coord(p[0], cs), cell_coord(p[1], cs));
    ent[e].word = ((uint64_t)key << 32) | (uint32_t)e;
  }
  qsort(ent, (size_t)N, sizeof(order_entry), order_entry_cmp);
  /* second pass, inside windows of W consecutive agents of that order (whole groups, at most 256).
   * Neighbours: root bodies within reach.
   *  1. clusters: in window order every free agent with a free neighbour starts a cluster, which
   *     takes, while it has fewer than G members, the first free neighbour of any member;
   *  2. packing: clusters one after another; one that does not fit into the group being filled
   *     goes to the next group, the gap is closed with free agents in window order, or, when
   *     there are none left, with the first members of that cluster; the free agents that remain
   *     come last.  Groups are every G consecutive agents of the layout. */
  const int W = (GROUP_WINDOW / G) * G;
  for (int w0 = 0; w0 < N; w0 += W) {
    const int n = N - w0 < W ? N - w0 : W;
    static _Thread_local int agent[GROUP_WINDOW], taken[GROUP_WINDOW], layout[GROUP_WINDOW];
    static _Thread_local int cl_first[GROUP_WINDOW], cl_size[GROUP_WINDOW], cl_members[GROUP_WINDOW];
    static _Thread_local float P[GROUP_WINDOW][3];
    static _Thread_local uint8_t near[GROUP_WINDOW][GROUP_WINDOW];
    for (int k = 0; k < n; ++k) { agent[k] = (int)(uint32_t)ent[w0 + k].word; taken[k] = 0; root_world_f32(o, agent[k], P[k]); }
    for (int i = 0; i < n; ++i)
      for (int j = 0; j < n; ++j) {
        float dx = P[i][0] - P[j][0], dy = P[i][1] - P[j][1], dz = P[i][2] - P[j][2];
        float d2 = (dx * dx + dy * dy) + dz * dz;
        near[i][j] = (i != j && d2 <= r2) ? 1 : 0;
      }
    int n_cl = 0, n_mem = 0;
    for (int seed = 0; seed < n; ++seed) {
      if (taken[seed]) continue;
      int has = 0;
      for (int k = 0; k < n; ++k) has |= (near[seed][k] && !taken[k]);
      if (!has) continue;
      cl_first[n_cl] = n_mem; cl_members[n_mem++] = seed; taken[seed] = 1;
      int cnt = 1;
      while (cnt < G) {
        int nx = -1;
        for (int k = 0; k < n && nx < 0; ++k) {
          if (taken[k]) continue;
          for (int q = 0; q < cnt; ++q) if (near[k][cl_members[cl_first[n_cl] + q]]) { nx = k; break; }
        }
        if (nx < 0) break;
        cl_members[n_mem++] = nx; taken[nx] = 1; ++cnt;
      }
      cl_size[n_cl++] = cnt;
    }
    int out = 0, filled = 0, next_free = 0;
    for (int c = 0; c < n_cl; ++c) {
      int first = cl_first[c], sz = cl_size[c];
      if (filled + sz > G) {
        while (filled < G) {
          while (next_free < n && taken[next_free]) ++next_free;
          if (next_free >= n) break;
          layout[out++] = next_free; taken[next_free] = 1; ++filled;
        }
        while (filled < G) { layout[out++] = cl_members[first++]; --sz; ++filled; }
        filled = 0;
      }
      for (int t = 0; t < sz; ++t) layout[out++] = cl_members[first + t];
      filled += sz;
      if (filled == G) filled = 0;
    }
    for (int k = 0; k < n; ++k) if (!taken[k]) layout[out++] = k;
    for (int k = 0; k < n; ++k) o->place_env[w0 + k] = agent[layout[k]];
  }
  o->regrouped = 1;
  free(ent);
  memset(o->pcon_n, 0, sizeof(int) * (size_t)((N + G - 1) / G));
}
/* place_env[N]: a permutation of the agents (NULL: agents in their own order); returns 0, or -1
 * if it is none */
int32_t oracle_set_groups(oracle_sim* o, const int32_t* place_env) {
  const int N = o->N;
  if (place_env) {
    uint8_t* seen = (uint8_t*)calloc((size_t)N, 1);
    int ok = 1;
    for (int p = 0; p < N && ok; ++p) {
      if (place_env[p] < 0 || place_env[p] >= N || seen[place_env[p]]) ok = 0;
      else seen[place_env[p]] = 1;
    }
    free(seen);
    if (!ok) return -1;
  }
  o->regrouped = 0;
  for (int p = 0; p < N; ++p) {
    o->place_env[p] = place_env ? place_env[p] : p;
    if (o->place_env[p] != p) o->regrouped = 1;
  }
  memset(o->pcon_n, 0, sizeof(int) * (size_t)((N + o->m.G - 1) / o->m.G));
  return 0;
}
void oracle_get_groups(const oracle_sim* o, int32_t* place_env) {
  for (int p = 0; p < o->N; ++p) place_env[p] = o->place_env[p];
}

void oracle_get_obs(const oracle_sim* o, double* obs, double* reward, uint8_t* done) {
  int od = oracle_obs_dim(o);
  for (int e = 0; e < o->N; ++e) {
    const env_state* E = &o->env[e];
    if (o->task.enabled && E->has_store) {
      memcpy(obs + (size_t)e * od, E->obs_store, sizeof(double) * od);
      reward[e] = E->rew_store; done[e] = E->done_store;
    } else {
      pack_obs(&o->m, E, obs + (size_t)e * od, &reward[e], &done[e]);
    }
  }
}
void oracle_get_contacts(const oracle_sim* o, oracle_contact* recs) {
  for (int e = 0; e < o->N; ++e) memcpy(recs + (size_t)e * o->m.S, o->env[e].con, o->m.S * sizeof(oracle_contact));
}
void oracle_generate_contacts(oracle_sim* o, int32_t brute, oracle_contact* recs) {
  for (int e = 0; e < o->N; ++e) generate_contacts(&o->m, &o->env[e], brute, recs + (size_t)e * o->m.S);
}
void oracle_set_trace(oracle_sim* o, int32_t env, oracle_sweep_trace* buf, int32_t cap) {
  o->trace_env = buf ? env : -1; o->trace = buf; o->trace_cap = cap; o->trace_n = 0;
}
int32_t oracle_trace_count(const oracle_sim* o) { return o->trace_n; }
void oracle_joint_angles(const oracle_sim* o, double* theta) {
  for (int e = 0; e < o->N; ++e)
    for (int j = 0; j < o->m.J; ++j) joint_theta(&o->m, &o->env[e], j, theta + ((size_t)e * o->m.J + j) * 3);
}
