// Built-in robot tables (host code): the ant and the 13-capsule humanoid of the benchmark
// configurations (Section 4.1 names the tasks; the stick figures themselves are this build's own,
// inside the ranges the configurations give), so that a caller of the C interface needs no table
// generator of its own.  Filled once, on first use, into static storage that lives as long as the
// library.
#pragma once
#include <math.h>
#include <string.h>

#include <mutex>

#include "../../include/sim.h"

namespace sim355 {

struct BuiltinRobot {
  int n_bodies = 0, n_joints = 0, n_act = 0, root = 0, n_feet = 0;
  int feet[SIM_MAX_FEET] = {0, 0, 0, 0};
  double term_height = 0.0, alive_bonus = 0.0;
  sim_body_desc_t bodies[SIM_MAX_BODIES];
  sim_joint_desc_t joints[SIM_MAX_JOINTS];

  // solid capsule: cylinder of length seg_len plus two hemispherical caps; seg_len 0 = sphere;
  // density > 0 gives the mass, else `mass` is the total
  int body(double r, double seg_len, int axis, double cx, double cy, double cz, double density, double mass) {
    const double kPi = 3.14159265358979323846;
    const double vol_c = kPi * r * r * seg_len, vol_h = (2.0 / 3.0) * kPi * r * r * r;
    const double rho = density > 0.0 ? density : mass / (vol_c + 2.0 * vol_h);
    const double m_c = rho * vol_c, m_h = rho * vol_h;
    const double i_ax = m_c * r * r / 2.0 + 2.0 * m_h * (2.0 * r * r / 5.0);
    const double i_tr = m_c * (seg_len * seg_len / 12.0 + r * r / 4.0) +
                        2.0 * m_h * (2.0 * r * r / 5.0 + seg_len * seg_len / 4.0 + 3.0 * seg_len * r / 8.0);
    sim_body_desc_t& b = bodies[n_bodies];
    memset(&b, 0, sizeof b);
    b.axis = axis; b.radius = r; b.half_len = seg_len / 2.0; b.mass = m_c + 2.0 * m_h;
    for (int k = 0; k < 3; ++k) b.inertia[k] = (seg_len == 0.0 || k == axis) ? i_ax : i_tr;
    b.rest_pos[0] = cx; b.rest_pos[1] = cy; b.rest_pos[2] = cz;
    return n_bodies++;
  }

  // hinge axes first (each with its limits), the remaining axes locked: completed with the unit
  // vectors x, y, z (in this order) that are perpendicular to all axes chosen so far
  void joint(int parent, int child, double ax, double ay, double az, int n_hinges, const double hinge_axes[][3],
             const double lo[], const double hi[], double gear) {
    sim_joint_desc_t& j = joints[n_joints++];
    memset(&j, 0, sizeof j);
    j.parent = parent; j.child = child;
    j.anchor[0] = ax; j.anchor[1] = ay; j.anchor[2] = az;
    int n = 0;
    for (; n < n_hinges; ++n) {
      for (int c = 0; c < 3; ++c) j.axes[n][c] = hinge_axes[n][c];
      j.mode[n] = 1; j.act[n] = n_act++; j.lo[n] = lo[n]; j.hi[n] = hi[n]; j.gear[n] = gear;
    }
    for (int cand = 0; cand < 3 && n < 3; ++cand) {
      bool perpendicular = true;
      for (int k = 0; k < n; ++k) perpendicular = perpendicular && fabs(j.axes[k][cand]) < 1e-9;
      if (!perpendicular) continue;
      j.axes[n][0] = j.axes[n][1] = j.axes[n][2] = 0.0;
      j.axes[n][cand] = 1.0;
      j.mode[n] = 0; j.act[n] = -1;
      ++n;
    }
  }
};

// Torso sphere (r 0.25, 1 kg) and four legs of two capsules (segment 0.4, r 0.08, 0.2 kg each)
// along +x, +y, -x, -y; hip hinge about z, knee hinge about z x d; limits +-0.7 rad, gear 15.
inline void build_ant(BuiltinRobot& R) {
  const double z0 = 0.75, gear = 15.0;
  const int torso = R.body(0.25, 0.0, 2, 0.0, 0.0, z0, 0.0, 1.0);
  const double dirs[4][2] = {{1, 0}, {0, 1}, {-1, 0}, {0, -1}};
  const double lo[1] = {-0.7}, hi[1] = {0.7};
  for (int k = 0; k < 4; ++k) {
    const double dx = dirs[k][0], dy = dirs[k][1];
    const int axis = dx != 0.0 ? 0 : 1;
    const int up = R.body(0.08, 0.4, axis, 0.45 * dx, 0.45 * dy, z0, 0.0, 0.2);
    const int low = R.body(0.08, 0.4, axis, 0.85 * dx, 0.85 * dy, z0, 0.0, 0.2);
    const double hip[1][3] = {{0.0, 0.0, 1.0}};
    const double knee[1][3] = {{-dy, dx, 0.0}};   // z x d
    R.joint(torso, up, 0.25 * dx, 0.25 * dy, z0, 1, hip, lo, hi, gear);
    R.joint(up, low, 0.65 * dx, 0.65 * dy, z0, 1, knee, lo, hi, gear);
    R.feet[R.n_feet++] = low;
  }
  R.root = torso; R.term_height = 0.3; R.alive_bonus = 0.5;
}

// 13 capsules of density 1000 (45 kg), 12 joints, 21 limited hinges (abdomen 3, shoulders 2 x 2,
// elbows 1 x 2, hips 3 x 2, knees 1 x 2, ankles 2 x 2), neck locked; gear 100; pelvis at 1.4 m.
inline void build_humanoid(BuiltinRobot& R) {
  const double z0 = 1.4, gear = 100.0, rho = 1000.0;
  const double X[3] = {1, 0, 0}, Y[3] = {0, 1, 0}, Z[3] = {0, 0, 1};
  auto axes = [](const double* a, const double* b, const double* c, double out[][3]) {
    const double* src[3] = {a, b, c};
    for (int k = 0; k < 3; ++k)
      if (src[k]) for (int i = 0; i < 3; ++i) out[k][i] = src[k][i];
  };
  double ax[3][3];
  const int pelvis = R.body(0.09, 0.14, 1, 0, 0, z0, rho, 0);
  const int torso = R.body(0.09, 0.25, 2, 0, 0, z0 + 0.30, rho, 0);
  const int head = R.body(0.09, 0.10, 2, 0, 0, z0 + 0.66, rho, 0);
  { axes(X, Y, Z, ax); const double lo[3] = {-0.6, -1.0, -0.7}, hi[3] = {0.6, 0.5, 0.7};
    R.joint(pelvis, torso, 0, 0, z0 + 0.10, 3, ax, lo, hi, gear); }
  R.joint(torso, head, 0, 0, z0 + 0.52, 0, ax, nullptr, nullptr, gear);
  for (int side = 0; side < 2; ++side) {
    const double sy = side == 0 ? -1.0 : 1.0;
    const int ua = R.body(0.04, 0.24, 2, 0, 0.20 * sy, z0 + 0.33, rho, 0);
    const int la = R.body(0.04, 0.22, 2, 0, 0.20 * sy, z0 + 0.10, rho, 0);
    { axes(X, Y, nullptr, ax); const double lo[2] = {-1.2, -1.5}, hi[2] = {1.2, 1.5};
      R.joint(torso, ua, 0, 0.20 * sy, z0 + 0.45, 2, ax, lo, hi, gear); }
    { axes(Y, nullptr, nullptr, ax); const double lo[1] = {-2.0}, hi[1] = {0.0};
      R.joint(ua, la, 0, 0.20 * sy, z0 + 0.21, 1, ax, lo, hi, gear); }
  }
  for (int side = 0; side < 2; ++side) {
    const double sy = side == 0 ? -1.0 : 1.0;
    const int th = R.body(0.06, 0.35, 2, 0, 0.10 * sy, z0 - 0.225, rho, 0);
    const int sh = R.body(0.05, 0.30, 2, 0, 0.10 * sy, z0 - 0.55, rho, 0);
    const int ft = R.body(0.04, 0.16, 0, 0.04, 0.10 * sy, z0 - 0.75, rho, 0);
    { axes(X, Y, Z, ax); const double lo[3] = {-0.5, -1.6, -0.6}, hi[3] = {0.5, 0.6, 0.6};
      R.joint(pelvis, th, 0, 0.10 * sy, z0 - 0.05, 3, ax, lo, hi, gear); }
    { axes(Y, nullptr, nullptr, ax); const double lo[1] = {0.0}, hi[1] = {2.0};
      R.joint(th, sh, 0, 0.10 * sy, z0 - 0.40, 1, ax, lo, hi, gear); }
    { axes(Y, X, nullptr, ax); const double lo[2] = {-0.7, -0.4}, hi[2] = {0.7, 0.4};
      R.joint(sh, ft, 0, 0.10 * sy, z0 - 0.70, 2, ax, lo, hi, gear); }
    R.feet[R.n_feet++] = ft;
  }
  R.root = torso; R.term_height = 0.7; R.alive_bonus = 2.0;
}

inline const BuiltinRobot* builtin_robot(int kind) {
  static BuiltinRobot ant, humanoid;
  static std::once_flag once;
  std::call_once(once, [] { build_ant(ant); build_humanoid(humanoid); });
  return kind == SIM_ROBOT_ANT ? &ant : (kind == SIM_ROBOT_HUMANOID ? &humanoid : nullptr);
}

}  // namespace sim355
