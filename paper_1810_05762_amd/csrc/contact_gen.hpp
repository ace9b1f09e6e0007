// Speculative contact generation for one contact slot (device code).
//
// Section 3.1 of the paper: contacts are detected speculatively and enter the
// solve as unilateral constraints.  A slot becomes active when the gap between
// a capsule end sphere (or the capsule's segment interior) and the nearest
// terrain feature is below the contact margin.
//
// The integer outcome (active, kind, feature id) must be a pure function of the
// fp32 state, reproducible on any IEEE machine, so this whole file is compiled
// without fused multiply-add contraction and every expression is written as a
// sequence of single rounded operations in a fixed order:
//   dot(a,b)   = (a.x*b.x + a.y*b.y) + a.z*b.z
//   cross(a,b) = (a.y*b.z - a.z*b.y, a.z*b.x - a.x*b.z, a.x*b.y - a.y*b.x)
//   vertex(i,j) = (ox + float(i)*cell, oy + float(j)*cell, h[j][i])
// The nearest feature is the lexicographic minimum of (squared distance, id)
// over all admissible features, so candidates may be visited in any order and
// by any number of lanes.  Features that cannot reach the margin are skipped
// with conservative height tests (1 mm slack), which never changes the outcome.
#pragma once
#include <hip/hip_runtime.h>

#include "model.hpp"

namespace sim355 {

#pragma clang fp contract(off)

struct f3 {
  float x, y, z;
};
__device__ __forceinline__ f3 sub3(f3 a, f3 b) { return f3{a.x - b.x, a.y - b.y, a.z - b.z}; }
__device__ __forceinline__ float dot3(f3 a, f3 b) {
  float s = a.x * b.x;
  float t = a.y * b.y;
  s = s + t;
  t = a.z * b.z;
  return s + t;
}
__device__ __forceinline__ f3 cross3(f3 a, f3 b) {
  float x0 = a.y * b.z, x1 = a.z * b.y;
  float y0 = a.z * b.x, y1 = a.x * b.z;
  float z0 = a.x * b.y, z1 = a.y * b.x;
  return f3{x0 - x1, y0 - y1, z0 - z1};
}

typedef __attribute__((address_space(3))) float lds_float;  // LDS-resident data

struct Field {
  int nx, ny;
  float cell, inv_cell, ox, oy;
  const float* __restrict__ h;
  const float* __restrict__ coarse;  // max height over blocks of kCoarse x kCoarse cells
  int cnx;
  // optional copy of the samples [pi0, pi0+ps) x [pj0, pj0+ps) in LDS (ps = 0: none), and the
  // maxima of its blocks of kMip x kMip cells: block (I,J) covers samples [4I,4I+4] x [4J,4J+4]
  const lds_float* patch;
  const lds_float* mip;
  int pi0, pj0, ps;
};
constexpr int kMip = 4;

__device__ __forceinline__ float field_height(const Field& H, int i, int j) {
  unsigned di = (unsigned)(i - H.pi0), dj = (unsigned)(j - H.pj0);
  if (di < (unsigned)H.ps && dj < (unsigned)H.ps) return H.patch[dj * H.ps + di];
  return H.h[j * H.nx + i];
}

// Heights of the four corners of cell (i,j) with a single inside-the-copy test, so the four
// reads are issued together.
__device__ __forceinline__ void field_cell_heights(const Field& H, int i, int j, float& h00, float& h10,
                                                   float& h11, float& h01) {
  unsigned di = (unsigned)(i - H.pi0), dj = (unsigned)(j - H.pj0);
  if (di + 1u < (unsigned)H.ps && dj + 1u < (unsigned)H.ps) {
    const lds_float* p = H.patch + dj * H.ps + di;
    h00 = p[0]; h10 = p[1]; h01 = p[H.ps]; h11 = p[H.ps + 1];
  } else {
    const float* p = H.h + j * H.nx + i;
    h00 = p[0]; h10 = p[1]; h01 = p[H.nx]; h11 = p[H.nx + 1];
  }
}

// The same for a sample that may lie on the last row or column: the neighbours that do not exist
// are replaced by the sample itself (callers do not use them).
__device__ __forceinline__ void field_cell_heights_clamped(const Field& H, int i, int j, float& h00, float& h10,
                                                           float& h11, float& h01) {
  unsigned di = (unsigned)(i - H.pi0), dj = (unsigned)(j - H.pj0);
  if (di + 1u < (unsigned)H.ps && dj + 1u < (unsigned)H.ps) {
    const lds_float* p = H.patch + dj * H.ps + di;
    h00 = p[0]; h10 = p[1]; h01 = p[H.ps]; h11 = p[H.ps + 1];
  } else {
    const int ip = i + 1 < H.nx ? i + 1 : i, jp = j + 1 < H.ny ? j + 1 : j;
    h00 = H.h[j * H.nx + i]; h10 = H.h[j * H.nx + ip]; h01 = H.h[jp * H.nx + i]; h11 = H.h[jp * H.nx + ip];
  }
}
// world x / y of sample column i / row j
__device__ __forceinline__ float field_x(const Field& H, int i) { float fx = (float)i * H.cell; return H.ox + fx; }
__device__ __forceinline__ float field_y(const Field& H, int j) { float fy = (float)j * H.cell; return H.oy + fy; }

__device__ __forceinline__ f3 field_vertex(const Field& H, int i, int j) {
  float fx = (float)i * H.cell, fy = (float)j * H.cell;
  return f3{H.ox + fx, H.oy + fy, field_height(H, i, j)};
}

// Barycentric coordinates (v,w) of the point of triangle A,B,C closest to P,
// found from the projections of P on the two edge directions at each corner.
__device__ __forceinline__ void tri_closest_vw(f3 P, f3 A, f3 B, f3 C, float& v, float& w) {
  f3 ab = sub3(B, A), ac = sub3(C, A), ap = sub3(P, A);
  float g11 = dot3(ab, ab), g12 = dot3(ab, ac), g22 = dot3(ac, ac);
  float d1 = dot3(ab, ap), d2 = dot3(ac, ap);
  float d3 = d1 - g11, d4 = d2 - g12, d5 = d1 - g12, d6 = d2 - g22;
  if (d1 <= 0.0f && d2 <= 0.0f) {
    v = 0.0f; w = 0.0f;
  } else if (d3 >= 0.0f && d4 <= d3) {
    v = 1.0f; w = 0.0f;
  } else if (d6 >= 0.0f && d5 <= d6) {
    v = 0.0f; w = 1.0f;
  } else {
    float vc = d1 * d4 - d3 * d2;
    float vb = d5 * d2 - d1 * d6;
    float va = d3 * d6 - d5 * d4;
    float e43 = d4 - d3, e56 = d5 - d6;
    if (vc <= 0.0f && d1 >= 0.0f && d3 <= 0.0f) {
      v = d1 / g11; w = 0.0f;
    } else if (vb <= 0.0f && d2 >= 0.0f && d6 <= 0.0f) {
      v = 0.0f; w = d2 / g22;
    } else if (va <= 0.0f && e43 >= 0.0f && e56 >= 0.0f) {
      w = e43 / (e43 + e56); v = 1.0f - w;
    } else {
      float s = (va + vb) + vc;
      v = vb / s; w = vc / s;
    }
  }
}
__device__ __forceinline__ f3 tri_point(f3 A, f3 B, f3 C, float v, float w) {
  f3 ab = sub3(B, A), ac = sub3(C, A);
  return f3{A.x + (ab.x * v + ac.x * w), A.y + (ab.y * v + ac.y * w), A.z + (ab.z * v + ac.z * w)};
}

__device__ __forceinline__ bool cell_span(const Field& H, float lo, float hi, float origin, int ncell,
                                          int& c0, int& c1) {
  float a = floorf((lo - origin) * H.inv_cell), b = floorf((hi - origin) * H.inv_cell);
  if (b < 0.0f || a > (float)(ncell - 1)) return false;
  if (a < 0.0f) a = 0.0f;
  if (b > (float)(ncell - 1)) b = (float)(ncell - 1);
  c0 = (int)a; c1 = (int)b;
  return true;
}

constexpr float kSelSlack = 1e-3f;

struct ContactOut {
  int active, kind, feat;
  float d;
  f3 n, rc;
  float w;  // share of the body this block gets in the mass splitting
};

__device__ __forceinline__ ContactOut no_contact() {
  ContactOut o;
  o.active = 0; o.kind = -1; o.feat = -1; o.d = 0.0f;
  o.n = f3{0.0f, 0.0f, 0.0f}; o.rc = f3{0.0f, 0.0f, 0.0f}; o.w = 0.0f;
  return o;
}

// 0 at the margin, 1 from half the margin down, times the fade of the mid-segment slot
__device__ __forceinline__ float block_weight(float margin, float d, float ramp_s) {
  float w = margin > 0.0f ? fminf((margin - d) / (0.5f * margin), 1.0f) : 1.0f;
  return fmaxf(w * ramp_s, 1e-6f);
}

__device__ __forceinline__ float clamp01(float s) { return s < 0.0f ? 0.0f : (s > 1.0f ? 1.0f : s); }

// Closest points between segment P0->P1 and edge Q0->Q1 (parameters s, t).
__device__ __forceinline__ void seg_edge_st(f3 P0, f3 P1, f3 Q0, f3 Q1, float& s, float& t) {
  f3 d1 = sub3(P1, P0), d2 = sub3(Q1, Q0), rr = sub3(P0, Q0);
  float a = dot3(d1, d1), e = dot3(d2, d2), f = dot3(d2, rr), c = dot3(d1, rr), b = dot3(d1, d2);
  float ae = a * e, bb = b * b;
  float denom = ae - bb;
  if (denom > 1e-6f * ae) {
    float bf = b * f, ce = c * e;
    s = clamp01((bf - ce) / denom);
  } else {
    s = 0.5f;
  }
  {
    float bs = b * s;
    t = (bs + f) / e;
  }
  if (t < 0.0f) {
    t = 0.0f;
    s = clamp01((0.0f - c) / a);
  } else if (t > 1.0f) {
    t = 1.0f;
    s = clamp01((b - c) / a);
  }
}

// Closest points of two capsule segments P0->P1 and Q0->Q1 (either may have zero length):
// writes the parameters and returns the squared distance.  Decides which capsule pairs are
// in contact (Section 3.1: contacts among bodies; Section 4.1: inter-agent collisions), so
// it follows the fixed operation order of this file.  Parallel segments start from the
// middle of the first one.
__device__ __forceinline__ float segment_segment(f3 P0, f3 P1, f3 Q0, f3 Q1, float& s, float& t) {
  const float tiny = 1e-12f;
  f3 d1 = sub3(P1, P0), d2 = sub3(Q1, Q0), r = sub3(P0, Q0);
  float a = dot3(d1, d1), e = dot3(d2, d2), f = dot3(d2, r), c = dot3(d1, r), b = dot3(d1, d2);
  if (a <= tiny && e <= tiny) { s = 0.0f; t = 0.0f; }
  else if (a <= tiny) { s = 0.0f; t = clamp01(f / e); }
  else if (e <= tiny) { t = 0.0f; s = clamp01(-c / a); }
  else {
    float ae = a * e, bb = b * b;
    float den = ae - bb, floor_ = 1e-6f * ae;
    if (den > floor_) { float bf = b * f, ce = c * e; float num = bf - ce; s = clamp01(num / den); }
    else s = 0.5f;
    float bs = b * s;
    float tn = bs + f;
    t = tn / e;
    if (t < 0.0f) { t = 0.0f; s = clamp01(-c / a); }
    else if (t > 1.0f) { t = 1.0f; float bc = b - c; s = clamp01(bc / a); }
  }
  float ux = d1.x * s, uy = d1.y * s, uz = d1.z * s;
  float wx = d2.x * t, wy = d2.y * t, wz = d2.z * t;
  f3 cp = f3{P0.x + ux, P0.y + uy, P0.z + uz}, cq = f3{Q0.x + wx, Q0.y + wy, Q0.z + wz};
  f3 df = sub3(cp, cq);
  return dot3(df, df);
}

// Are two capsules within the contact margin?  Segment end points env-local, the second
// capsule's shifted by `off` (its env origin minus the first one's).  Returns the segment
// parameters of the closest points and the gap between the surfaces.
__device__ __forceinline__ bool pair_in_contact(f3 p0, f3 p1, f3 q0, f3 q1, const float off[3], float rad_a,
                                                float rad_b, float margin, float& s, float& t, float& gap) {
  q0 = f3{q0.x + off[0], q0.y + off[1], q0.z + off[2]};
  q1 = f3{q1.x + off[0], q1.y + off[1], q1.z + off[2]};
  const float d2 = segment_segment(p0, p1, q0, q1, s, t);
  const float rr = rad_a + rad_b;
  const float lim = rr + margin;
  if (!(d2 < lim * lim)) return false;
  gap = (sqrtf(d2) - rad_a) - rad_b;
  return true;
}

// End points of a body's segment: env-local (p0,p1) from the state, in the same
// operation order the selection is specified in.
__device__ __forceinline__ void body_ends(const float x[3], const float q[4], float half_len, int axis,
                                          f3& p0, f3& p1) {
  float qw = q[0], qx = q[1], qy = q[2], qz = q[3];
  f3 c;
  if (axis == 0) {
    float yy = qy * qy, zz = qz * qz, xy = qx * qy, wz = qw * qz, xz = qx * qz, wy = qw * qy;
    c = f3{1.0f - 2.0f * (yy + zz), 2.0f * (xy + wz), 2.0f * (xz - wy)};
  } else if (axis == 1) {
    float xx = qx * qx, zz = qz * qz, xy = qx * qy, wz = qw * qz, yz = qy * qz, wx = qw * qx;
    c = f3{2.0f * (xy - wz), 1.0f - 2.0f * (xx + zz), 2.0f * (yz + wx)};
  } else {
    float xx = qx * qx, yy = qy * qy, xz = qx * qz, wy = qw * qy, yz = qy * qz, wx = qw * qx;
    c = f3{2.0f * (xz + wy), 2.0f * (yz - wx), 1.0f - 2.0f * (xx + yy)};
  }
  f3 a = f3{half_len * c.x, half_len * c.y, half_len * c.z};
  p0 = f3{x[0] - a.x, x[1] - a.y, x[2] - a.z};
  p1 = f3{x[0] + a.x, x[1] + a.y, x[2] + a.z};
}

// Everything a slot needs to be tested against the terrain.
struct SlotGeom {
  f3 xc;          // body centre, env-local
  f3 p0, p1;      // segment end points, env-local
  f3 P0, P1;      // the same in world coordinates (env origin added)
  f3 org;
  float r, Rq;    // radius, reach = r + margin + slack
  int kind;       // 0 end -, 1 end +, 2 mid-segment
  int i0, i1, j0, j1;  // cells the reach box overlaps
};

__device__ __forceinline__ SlotGeom slot_geom(float radius, float half_len, int axis, float margin,
                                              const float x[3], const float q[4], int slot_kind,
                                              const float origin[3]) {
  SlotGeom g;
  g.kind = slot_kind;
  g.r = radius;
  g.Rq = (g.r + margin) + kSelSlack;
  body_ends(x, q, half_len, axis, g.p0, g.p1);
  g.xc = f3{x[0], x[1], x[2]};
  g.org = f3{origin[0], origin[1], origin[2]};
  g.P0 = f3{g.p0.x + g.org.x, g.p0.y + g.org.y, g.p0.z + g.org.z};
  g.P1 = f3{g.p1.x + g.org.x, g.p1.y + g.org.y, g.p1.z + g.org.z};
  g.i0 = 0; g.i1 = -1; g.j0 = 0; g.j1 = -1;
  return g;
}

__device__ __forceinline__ ContactOut plane_contact(const SlotGeom& g, float margin) {
  ContactOut out = no_contact();
  if (g.kind == 2) return out;
  f3 p = g.kind == 0 ? g.p0 : g.p1;
  float d = p.z - g.r;
  if (!(d < margin)) return out;
  out.active = 1; out.kind = 0; out.feat = -1; out.d = d;
  out.n = f3{0.0f, 0.0f, 1.0f};
  out.rc = f3{p.x - g.xc.x, p.y - g.xc.y, (p.z - g.r) - g.xc.z};
  out.w = block_weight(margin, d, 1.0f);
  return out;
}

// Cells overlapped by the reach box only (no height test).
__device__ __forceinline__ bool slot_range(const Field& H, SlotGeom& g) {
  const int ncx = H.nx - 1, ncy = H.ny - 1;
  float xl, xh, yl, yh;
  if (g.kind < 2) {
    f3 P = g.kind == 0 ? g.P0 : g.P1;
    xl = xh = P.x; yl = yh = P.y;
  } else {
    xl = g.P0.x < g.P1.x ? g.P0.x : g.P1.x; xh = g.P0.x < g.P1.x ? g.P1.x : g.P0.x;
    yl = g.P0.y < g.P1.y ? g.P0.y : g.P1.y; yh = g.P0.y < g.P1.y ? g.P1.y : g.P0.y;
  }
  if (!cell_span(H, xl - g.Rq, xh + g.Rq, H.ox, ncx, g.i0, g.i1)) return false;
  return cell_span(H, yl - g.Rq, yh + g.Rq, H.oy, ncy, g.j0, g.j1);
}

// Cells overlapped by the reach box; false when the slot cannot touch the field
// (box outside the field, or higher than every sample of the coarse blocks under it).
__device__ __forceinline__ bool slot_reach(const Field& H, SlotGeom& g, bool exact = true) {
  const int ncx = H.nx - 1, ncy = H.ny - 1;
  float xl, xh, yl, yh, zl;
  if (g.kind < 2) {
    f3 P = g.kind == 0 ? g.P0 : g.P1;
    xl = xh = P.x; yl = yh = P.y; zl = P.z;
  } else {
    xl = g.P0.x < g.P1.x ? g.P0.x : g.P1.x; xh = g.P0.x < g.P1.x ? g.P1.x : g.P0.x;
    yl = g.P0.y < g.P1.y ? g.P0.y : g.P1.y; yh = g.P0.y < g.P1.y ? g.P1.y : g.P0.y;
    zl = g.P0.z < g.P1.z ? g.P0.z : g.P1.z;
  }
  if (!cell_span(H, xl - g.Rq, xh + g.Rq, H.ox, ncx, g.i0, g.i1)) return false;
  if (!cell_span(H, yl - g.Rq, yh + g.Rq, H.oy, ncy, g.j0, g.j1)) return false;
  const float zcut = zl - g.Rq;
  float hmax = -INFINITY;
  if (H.ps > 0 && g.i0 >= H.pi0 && g.i1 + 1 < H.pi0 + H.ps && g.j0 >= H.pj0 && g.j1 + 1 < H.pj0 + H.ps) {
    // the whole reach box lies inside the LDS copy: maximum over the blocks it touches
    // (up to 3 x 3 of them read without a loop; larger boxes take the loop)
    const int nb = (H.ps + kMip - 1) / kMip;
    const int I0 = (g.i0 - H.pi0) / kMip, I1 = (g.i1 + 1 - H.pi0) / kMip;
    const int J0 = (g.j0 - H.pj0) / kMip, J1 = (g.j1 + 1 - H.pj0) / kMip;
    if (I1 - I0 <= 2 && J1 - J0 <= 2) {
      {
        float m[9];
#pragma unroll
        for (int dj = 0; dj < 3; ++dj)
#pragma unroll
          for (int di = 0; di < 3; ++di) {
            int I = I0 + di < I1 ? I0 + di : I1, J = J0 + dj < J1 ? J0 + dj : J1;
            m[dj * 3 + di] = H.mip[J * nb + I];
          }
        __builtin_amdgcn_sched_group_barrier(0x100, 9, 0);  // the nine reads first, one wait
#pragma unroll
        for (int k = 0; k < 9; ++k) hmax = fmaxf(hmax, m[k]);
      }
      // block maxima say "maybe": take the exact maximum over the samples of the box when it
      // is at most 6 x 6 (all 36 reads are issued together, indices clamped into the box)
      const int ni = g.i1 - g.i0 + 2, nj = g.j1 - g.j0 + 2;
      if (exact && !(zcut > hmax) && ni <= 6 && nj <= 6) {
        const int bi = g.i0 - H.pi0, bj = g.j0 - H.pj0;
        hmax = -INFINITY;
        float hv[36];
        int col[6], row[6];
#pragma unroll
        for (int d = 0; d < 6; ++d) { col[d] = bi + (d < ni ? d : ni - 1); row[d] = (bj + (d < nj ? d : nj - 1)) * H.ps; }
#pragma unroll
        for (int dj = 0; dj < 6; ++dj)
#pragma unroll
          for (int di = 0; di < 6; ++di) hv[dj * 6 + di] = H.patch[row[dj] + col[di]];
        __builtin_amdgcn_sched_group_barrier(0x100, 36, 0);  // all reads before the first use
#pragma unroll
        for (int k = 0; k < 36; ++k) hmax = fmaxf(hmax, hv[k]);
      }
    } else {
      for (int J = J0; J <= J1; ++J)
        for (int I = I0; I <= I1; ++I) hmax = fmaxf(hmax, H.mip[J * nb + I]);
    }
  } else {
    for (int J = g.j0 / kCoarse; J <= g.j1 / kCoarse; ++J)
      for (int I = g.i0 / kCoarse; I <= g.i1 / kCoarse; ++I) hmax = fmaxf(hmax, H.coarse[J * H.cnx + I]);
  }
  return !(zcut > hmax);
}

// Centre underneath the surface: triangle containing its xy, plane distance.
__device__ __forceinline__ bool underneath_contact(const Field& H, const SlotGeom& g, float margin,
                                                   ContactOut& out) {
  const int ncx = H.nx - 1, ncy = H.ny - 1;
  f3 P = g.kind == 0 ? g.P0 : g.P1;
  f3 pl = g.kind == 0 ? g.p0 : g.p1;
  float ux = (P.x - H.ox) * H.inv_cell, uy = (P.y - H.oy) * H.inv_cell;
  float fi = floorf(ux), fj = floorf(uy);
  if (!(fi >= 0.0f && fi <= (float)(ncx - 1) && fj >= 0.0f && fj <= (float)(ncy - 1))) return false;
  int i = (int)fi, j = (int)fj;
  float fx = ux - fi, fy = uy - fj;
  int t = (fx >= fy) ? 0 : 1;
  float h00, h10, h11, h01;
  field_cell_heights(H, i, j, h00, h10, h11, h01);   // the four corners in one go
  const float x0 = field_x(H, i), x1 = field_x(H, i + 1), y0 = field_y(H, j), y1 = field_y(H, j + 1);
  f3 A = f3{x0, y0, h00}, C1 = f3{x1, y1, h11};
  f3 Bv = t == 0 ? f3{x1, y0, h10} : C1;
  f3 Cv = t == 0 ? C1 : f3{x0, y1, h01};
  f3 nt = cross3(sub3(Bv, A), sub3(Cv, A));
  float face = dot3(sub3(P, A), nt);
  if (!(face < 0.0f)) return false;
  float inv = 1.0f / sqrtf(dot3(nt, nt));
  f3 n = f3{nt.x * inv, nt.y * inv, nt.z * inv};
  out.active = 1; out.kind = 2; out.feat = 2 * (j * ncx + i) + t;
  out.d = dot3(sub3(pl, sub3(A, g.org)), n) - g.r;  // gap measured in env-local coordinates
  out.n = n;
  out.rc = f3{(pl.x - g.r * n.x) - g.xc.x, (pl.y - g.r * n.y) - g.xc.y, (pl.z - g.r * n.z) - g.xc.z};
  out.w = block_weight(margin, out.d, 1.0f);
  return true;
}

__device__ __forceinline__ void keep_min(float d2, int id, float& best, int& best_id) {
  if (d2 < best || (d2 == best && id < best_id)) { best = d2; best_id = id; }
}

// Cheap part of the end-sphere search: can a triangle of cell (i,j) be within R of P?  Lower
// bound of the distance from the horizontal gap to the cell's square and the height of P above
// the cell's highest corner.
__device__ __forceinline__ bool sphere_cell_reach(const Field& H, f3 P, float R, int i, int j) {
  float h00, h10, h11, h01;
  field_cell_heights(H, i, j, h00, h10, h11, h01);
  const float zmax = fmaxf(fmaxf(h00, h10), fmaxf(h11, h01));
  const float x0 = H.ox + (float)i * H.cell, x1 = H.ox + (float)(i + 1) * H.cell;
  const float y0 = H.oy + (float)j * H.cell, y1 = H.oy + (float)(j + 1) * H.cell;
  const float gx = fmaxf(fmaxf(x0 - P.x, P.x - x1), 0.0f), gy = fmaxf(fmaxf(y0 - P.y, P.y - y1), 0.0f);
  const float gz = fmaxf(P.z - zmax, 0.0f);
  return !((gx * gx + gy * gy) + gz * gz > R * R);
}

// Exact part: triangle t of cell (i,j) against the sphere centre P.  False when back-facing.
__device__ __forceinline__ bool sphere_tri_d2(const Field& H, f3 P, int i, int j, int t, float& d2) {
  float h00, h10, h11, h01;
  field_cell_heights(H, i, j, h00, h10, h11, h01);
  float x0 = H.ox + (float)i * H.cell, x1 = H.ox + (float)(i + 1) * H.cell;
  float y0 = H.oy + (float)j * H.cell, y1 = H.oy + (float)(j + 1) * H.cell;
  f3 A = f3{x0, y0, h00}, C1 = f3{x1, y1, h11};
  f3 Bv = t == 0 ? f3{x1, y0, h10} : C1, Cv = t == 0 ? C1 : f3{x0, y1, h01};
  f3 nt = cross3(sub3(Bv, A), sub3(Cv, A));
  float face = dot3(sub3(P, A), nt);
  if (face < 0.0f) return false;  // back-facing
  float v, w;
  tri_closest_vw(P, A, Bv, Cv, v, w);
  f3 df = sub3(P, tri_point(A, Bv, Cv, v, w));
  d2 = dot3(df, df);
  return true;
}

// Both triangles of cell (i,j) against the end sphere centred at P (reach R = r + margin + slack).
__device__ __forceinline__ void sphere_cell(const Field& H, f3 P, float R, int i, int j, float& best,
                                            int& best_id) {
  const int ncx = H.nx - 1;
  if (!sphere_cell_reach(H, P, R + kSelSlack, i, j)) return;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    float d2;
    if (sphere_tri_d2(H, P, i, j, t, d2)) keep_min(d2, 2 * (j * ncx + i) + t, best, best_id);
  }
}

// Per-slot constants of the conservative edge culls of the mid-segment search.  In the xy
// plane, u = (dx,dy) is the segment's direction (length L): for a point p, cross = u x (p - P0)
// is L times its distance from the segment's line and along = u . (p - P0) is L times its
// coordinate along it.  Two points within the reach R of each other differ by at most R L in
// either, so an edge whose cross interval stays beyond R L, or whose along interval ends before
// -R L or starts after L^2 + R L, is out of reach; otherwise the part of the segment that can be
// within R of it has s = along / L^2 in [amin - R L, amax + R L] / L^2, and the edge is out of
// reach when that part stays more than R above both its ends.
struct SegCull {
  f3 P0;                                // first end point (world)
  float dx, dy, dz, L2, RL, R, inv_L2;  // inv_L2 = 0: segment (nearly) vertical, no s interval
  float zcut;                           // lower end minus the reach
  int i1, j1;                           // last cell of the box in x and y
};
__device__ __forceinline__ SegCull seg_cull_from(f3 P0, f3 P1, float Rq, float RL, float inv_L2, int i1, int j1) {
  SegCull c;
  c.P0 = P0;
  c.dx = P1.x - P0.x; c.dy = P1.y - P0.y; c.dz = P1.z - P0.z;
  c.L2 = c.dx * c.dx + c.dy * c.dy;
  c.R = Rq + kSelSlack;
  c.RL = RL; c.inv_L2 = inv_L2;
  c.zcut = (P0.z < P1.z ? P0.z : P1.z) - Rq;
  c.i1 = i1; c.j1 = j1;
  return c;
}
// the two per-slot constants worth keeping: R L and 1 / L^2
__device__ __forceinline__ void seg_cull_consts(const SlotGeom& g, float& RL, float& inv_L2) {
  const float dx = g.P1.x - g.P0.x, dy = g.P1.y - g.P0.y;
  const float L2 = dx * dx + dy * dy;
  RL = (g.Rq + kSelSlack) * sqrtf(L2);
  inv_L2 = L2 > 1e-8f ? 1.0f / L2 : 0.0f;
}
__device__ __forceinline__ SegCull seg_cull(const SlotGeom& g) {
  float RL, inv_L2;
  seg_cull_consts(g, RL, inv_L2);
  return seg_cull_from(g.P0, g.P1, g.Rq, RL, inv_L2, g.i1, g.j1);
}

// Cheap part of the mid-segment search at sample (i,j): bit k of the result is set when edge k
// of the up-to-three edges starting there belongs to the box and may be within reach of the
// segment.  The three edges lie in the square of cell (i,j), so one test of that square (cross
// and along intervals of its corners, height of the reachable part of the segment above its
// highest corner) serves all three.
__device__ __forceinline__ int segment_candidates(const Field& H, const SegCull& sc, int i, int j) {
  const float x0 = H.ox + (float)i * H.cell, y0 = H.oy + (float)j * H.cell;
  const float rx0 = x0 - sc.P0.x, ry0 = y0 - sc.P0.y;
  const float c0 = sc.dx * ry0 - sc.dy * rx0, a0 = sc.dx * rx0 + sc.dy * ry0;
  // a step of one cell along +x changes (cross, along) by (-se, ce), along +y by (ce, se)
  const float ce = sc.dx * H.cell, se = sc.dy * H.cell;
  const float cmin = c0 + fminf(ce, 0.0f) + fminf(-se, 0.0f), cmax = c0 + fmaxf(ce, 0.0f) + fmaxf(-se, 0.0f);
  const float amin = a0 + fminf(se, 0.0f) + fminf(ce, 0.0f), amax = a0 + fmaxf(se, 0.0f) + fmaxf(ce, 0.0f);
  // sample coordinates carry the rounding of ox + i * cell: 1 mm more on top of R
  const float lim = sc.RL + 1e-3f * (fabsf(sc.dx) + fabsf(sc.dy));
  if (cmin > lim || cmax < -lim) return 0;
  if (amax < -lim || amin > sc.L2 + lim) return 0;
  // corner heights; neighbours beyond the last sample are clamped (their edges are excluded below)
  const int ip = i + 1 < H.nx ? i + 1 : i, jp = j + 1 < H.ny ? j + 1 : j;
  float h00, h10, h11, h01;
  {
    unsigned di = (unsigned)(i - H.pi0), dj = (unsigned)(j - H.pj0);
    if (di + 1u < (unsigned)H.ps && dj + 1u < (unsigned)H.ps) {
      const lds_float* p = H.patch + dj * H.ps + di;
      h00 = p[0]; h10 = p[1]; h01 = p[H.ps]; h11 = p[H.ps + 1];
    } else {
      h00 = H.h[j * H.nx + i]; h10 = H.h[j * H.nx + ip]; h01 = H.h[jp * H.nx + i]; h11 = H.h[jp * H.nx + ip];
    }
  }
  const float zq = fmaxf(fmaxf(h00, h10), fmaxf(h01, h11));
  if (sc.zcut > zq) return 0;  // the whole square is out of reach below the capsule
  if (sc.inv_L2 > 0.0f) {
    const float s_lo = fmaxf((amin - lim) * sc.inv_L2 - 1e-4f, 0.0f);
    const float s_hi = fminf((amax + lim) * sc.inv_L2 + 1e-4f, 1.0f);
    const float zs = sc.P0.z + sc.dz * (sc.dz >= 0.0f ? s_lo : s_hi);
    if (zs - sc.R > zq) return 0;
  }
  int mask = 7;
  if (i > sc.i1) mask &= 2;   // edges 0 and 2 leave the box in x
  if (j > sc.j1) mask &= 1;   // edges 1 and 2 leave the box in y
  return mask;
}

// Exact part: edge k of sample (i,j) against the interior of segment P0->P1.  False when the
// edge is not admissible (closest point at an end of the segment, or the axis not above it).
__device__ __forceinline__ bool segment_edge_d2(const Field& H, f3 P0, f3 P1, int i, int j, int k, float& d2) {
  const int i1 = i + (k == 1 ? 0 : 1), j1 = j + (k == 0 ? 0 : 1);
  float h00, h10, h11, h01;
  field_cell_heights_clamped(H, i, j, h00, h10, h11, h01);
  f3 Q0 = f3{H.ox + (float)i * H.cell, H.oy + (float)j * H.cell, h00};
  f3 Q1 = f3{H.ox + (float)i1 * H.cell, H.oy + (float)j1 * H.cell, k == 0 ? h10 : (k == 1 ? h01 : h11)};
  float s, t;
  seg_edge_st(P0, P1, Q0, Q1, s, t);
  if (!(s > 0.001f && s < 0.999f)) return false;  // the ends belong to the end-sphere slots
  f3 d1 = sub3(P1, P0), d2v = sub3(Q1, Q0);
  f3 c1 = f3{P0.x + d1.x * s, P0.y + d1.y * s, P0.z + d1.z * s};
  f3 c2 = f3{Q0.x + d2v.x * t, Q0.y + d2v.y * t, Q0.z + d2v.z * t};
  f3 df = sub3(c1, c2);
  if (!(df.z > 0.0f)) return false;  // the axis must be above the edge
  d2 = dot3(df, df);
  return true;
}

// The up-to-three edges that start at sample (i,j) against the segment interior.
__device__ __forceinline__ void segment_vertex(const Field& H, const SlotGeom& g, const SegCull& sc, int i, int j,
                                               float& best, int& best_id) {
  const int mask = segment_candidates(H, sc, i, j);
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    float d2;
    if (((mask >> k) & 1) && segment_edge_d2(H, g.P0, g.P1, i, j, k, d2))
      keep_min(d2, 3 * (j * H.nx + i) + k, best, best_id);
  }
}

// Record of the selected triangle (end sphere).  The geometry is rebuilt in
// env-local coordinates (vertex minus env origin), where the sphere centre
// carries no rounding from the world offset.
__device__ __forceinline__ ContactOut finish_sphere(const Field& H, const SlotGeom& g, float margin, float best,
                                                    int best_id) {
  ContactOut out = no_contact();
  if (best_id < 0) return out;
  float dist = sqrtf(best);
  float d = dist - g.r;
  if (!(d < margin)) return out;
  const int ncx = H.nx - 1;
  f3 pl = g.kind == 0 ? g.p0 : g.p1;
  int t = best_id & 1, c = best_id >> 1, i = c % ncx, j = c / ncx;
  float h00, h10, h11, h01;
  field_cell_heights(H, i, j, h00, h10, h11, h01);
  const float x0 = field_x(H, i), x1 = field_x(H, i + 1), y0 = field_y(H, j), y1 = field_y(H, j + 1);
  const f3 C1 = f3{x1, y1, h11};
  f3 A = sub3(f3{x0, y0, h00}, g.org);
  f3 Bv = sub3(t == 0 ? f3{x1, y0, h10} : C1, g.org);
  f3 Cv = sub3(t == 0 ? C1 : f3{x0, y1, h01}, g.org);
  float v, w;
  tri_closest_vw(pl, A, Bv, Cv, v, w);
  f3 df = sub3(pl, tri_point(A, Bv, Cv, v, w));
  dist = sqrtf(dot3(df, df));
  d = dist - g.r;
  f3 n;
  if (dist < 1e-9f) {
    f3 nt = cross3(sub3(Bv, A), sub3(Cv, A));
    float inv = 1.0f / sqrtf(dot3(nt, nt));
    n = f3{nt.x * inv, nt.y * inv, nt.z * inv};
  } else {
    float inv = 1.0f / dist;
    n = f3{df.x * inv, df.y * inv, df.z * inv};
  }
  out.active = 1; out.kind = 1; out.feat = best_id; out.d = d; out.n = n;
  out.rc = f3{(pl.x - g.r * n.x) - g.xc.x, (pl.y - g.r * n.y) - g.xc.y, (pl.z - g.r * n.z) - g.xc.z};
  out.w = block_weight(margin, d, 1.0f);
  return out;
}

// Record of the selected edge (mid-segment slot), geometry in env-local coordinates.
__device__ __forceinline__ ContactOut finish_segment(const Field& H, const SlotGeom& g, float margin, float best,
                                                     int best_id) {
  ContactOut out = no_contact();
  if (best_id < 0) return out;
  float dist = sqrtf(best);
  float d = dist - g.r;
  if (!(d < margin)) return out;
  int k = best_id % 3, vtx = best_id / 3, i = vtx % H.nx, j = vtx / H.nx;
  float h00, h10, h11, h01;
  field_cell_heights_clamped(H, i, j, h00, h10, h11, h01);
  f3 Q0 = sub3(f3{field_x(H, i), field_y(H, j), h00}, g.org);
  f3 Q1 = sub3(f3{field_x(H, i + (k == 1 ? 0 : 1)), field_y(H, j + (k == 0 ? 0 : 1)), k == 0 ? h10 : (k == 1 ? h01 : h11)},
               g.org);
  float s, t;
  seg_edge_st(g.p0, g.p1, Q0, Q1, s, t);
  f3 d1 = sub3(g.p1, g.p0), d2 = sub3(Q1, Q0);
  f3 cl = f3{g.p0.x + d1.x * s, g.p0.y + d1.y * s, g.p0.z + d1.z * s};
  f3 c2 = f3{Q0.x + d2.x * t, Q0.y + d2.y * t, Q0.z + d2.z * t};
  f3 df = sub3(cl, c2);
  dist = sqrtf(dot3(df, df));
  d = dist - g.r;
  f3 n;
  if (dist < 1e-9f) n = f3{0.0f, 0.0f, 1.0f};
  else { float inv = 1.0f / dist; n = f3{df.x * inv, df.y * inv, df.z * inv}; }
  out.active = 1; out.kind = 3; out.feat = best_id; out.d = d; out.n = n;
  out.rc = f3{(cl.x - g.r * n.x) - g.xc.x, (cl.y - g.r * n.y) - g.xc.y, (cl.z - g.r * n.z) - g.xc.z};
  float se = s < 1.0f - s ? s : 1.0f - s;
  out.w = block_weight(margin, d, fminf(fmaxf((se - 0.001f) / 0.1f, 0.0f), 1.0f));
  return out;
}

__device__ __forceinline__ Field make_field(const Model& M, const float* heights, const float* coarse) {
  return Field{M.nx, M.ny, M.cell, M.inv_cell, M.hox, M.hoy, heights, coarse, M.cnx, nullptr, nullptr, 0, 0, 0};
}

// One slot handled by one thread (used by the stand-alone contact kernel).
__device__ inline ContactOut generate_contact(const Model& M, const float* __restrict__ heights,
                                              const float* __restrict__ coarse, const float x[3],
                                              const float q[4], int body, int slot_kind, const float origin[3]) {
  if (!M.contacts) return no_contact();
  SlotGeom g = slot_geom(M.bodies[body].radius, M.bodies[body].half_len, M.bodies[body].axis, M.margin, x, q, slot_kind,
                         origin);
  if (M.terrain_kind == 0) return plane_contact(g, M.margin);
  Field H = make_field(M, heights, coarse);
  if (!slot_reach(H, g)) return no_contact();
  float best = INFINITY;
  int best_id = -1;
  if (slot_kind < 2) {
    ContactOut out = no_contact();
    if (underneath_contact(H, g, M.margin, out)) return out;
    f3 P = slot_kind == 0 ? g.P0 : g.P1;
    for (int j = g.j0; j <= g.j1; ++j)
      for (int i = g.i0; i <= g.i1; ++i) sphere_cell(H, P, g.Rq, i, j, best, best_id);
    return finish_sphere(H, g, M.margin, best, best_id);
  }
  const SegCull sc = seg_cull(g);
  for (int j = g.j0; j <= g.j1 + 1; ++j)
    for (int i = g.i0; i <= g.i1 + 1; ++i) segment_vertex(H, g, sc, i, j, best, best_id);
  return finish_segment(H, g, M.margin, best, best_id);
}

#pragma clang fp contract(fast)

}  // namespace sim355
