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
// Triangles that cannot reach the margin are skipped with a conservative test
// (1 mm slack), which never changes the outcome.
#pragma once
#include <hip/hip_runtime.h>

#include "model.hpp"

namespace sim355 {

#pragma clang fp contract(off)

struct f3 {
  float x, y, z;
};
__device__ __forceinline__ f3 mk3(float x, float y, float z) { return f3{x, y, z}; }
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

struct Field {
  int nx, ny;
  float cell, inv_cell, ox, oy;
  const float* __restrict__ h;
};

__device__ __forceinline__ f3 field_vertex(const Field& H, int i, int j) {
  float fx = (float)i * H.cell, fy = (float)j * H.cell;
  return f3{H.ox + fx, H.oy + fy, H.h[j * H.nx + i]};
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

// One slot: body pose (x,q env-local), slot kind, env origin -> contact record.
__device__ inline ContactOut generate_contact(const Model& M, const float* __restrict__ heights,
                                              const float x[3], const float q[4], int body, int slot_kind,
                                              const float origin[3]) {
  ContactOut out;
  out.active = 0; out.kind = -1; out.feat = -1; out.d = 0.0f;
  out.n = f3{0.0f, 0.0f, 0.0f}; out.rc = f3{0.0f, 0.0f, 0.0f}; out.w = 0.0f;
  if (!M.contacts) return out;
  const float r = M.bodies[body].radius;
  const float margin = M.margin;
  f3 p0, p1;
  body_ends(x, q, M.bodies[body].half_len, M.bodies[body].axis, p0, p1);
  f3 xc = f3{x[0], x[1], x[2]};

  if (M.terrain_kind == 0) {
    if (slot_kind == 2) return out;
    f3 p = slot_kind == 0 ? p0 : p1;
    float d = p.z - r;
    if (!(d < margin)) return out;
    out.active = 1; out.kind = 0; out.feat = -1; out.d = d;
    out.n = f3{0.0f, 0.0f, 1.0f};
    out.rc = f3{p.x - xc.x, p.y - xc.y, (p.z - r) - xc.z};
    out.w = block_weight(margin, d, 1.0f);
    return out;
  }

  Field H{M.nx, M.ny, M.cell, M.inv_cell, M.hox, M.hoy, heights};
  const int ncx = H.nx - 1, ncy = H.ny - 1;
  f3 org = f3{origin[0], origin[1], origin[2]};
  f3 P0 = f3{p0.x + org.x, p0.y + org.y, p0.z + org.z};
  f3 P1 = f3{p1.x + org.x, p1.y + org.y, p1.z + org.z};
  const float Rq = (r + margin) + kSelSlack;

  if (slot_kind < 2) {
    f3 P = slot_kind == 0 ? P0 : P1;
    f3 pl = slot_kind == 0 ? p0 : p1;
    // centre underneath the surface: triangle containing its xy, plane distance
    {
      float ux = (P.x - H.ox) * H.inv_cell, uy = (P.y - H.oy) * H.inv_cell;
      float fi = floorf(ux), fj = floorf(uy);
      if (fi >= 0.0f && fi <= (float)(ncx - 1) && fj >= 0.0f && fj <= (float)(ncy - 1)) {
        int i = (int)fi, j = (int)fj;
        float fx = ux - fi, fy = uy - fj;
        int t = (fx >= fy) ? 0 : 1;
        f3 A = field_vertex(H, i, j);
        f3 Bv = t == 0 ? field_vertex(H, i + 1, j) : field_vertex(H, i + 1, j + 1);
        f3 Cv = t == 0 ? field_vertex(H, i + 1, j + 1) : field_vertex(H, i, j + 1);
        f3 nt = cross3(sub3(Bv, A), sub3(Cv, A));
        f3 pa = sub3(P, A);
        float face = dot3(pa, nt);
        if (face < 0.0f) {
          float inv = 1.0f / sqrtf(dot3(nt, nt));
          f3 n = f3{nt.x * inv, nt.y * inv, nt.z * inv};
          out.active = 1; out.kind = 2; out.feat = 2 * (j * ncx + i) + t;
          out.d = dot3(sub3(pl, sub3(A, org)), n) - r;  // gap measured in env-local coordinates
          out.n = n;
          out.rc = f3{(pl.x - r * n.x) - xc.x, (pl.y - r * n.y) - xc.y, (pl.z - r * n.z) - xc.z};
          out.w = block_weight(margin, out.d, 1.0f);
          return out;
        }
      }
    }
    int i0, i1, j0, j1;
    if (!cell_span(H, P.x - Rq, P.x + Rq, H.ox, ncx, i0, i1)) return out;
    if (!cell_span(H, P.y - Rq, P.y + Rq, H.oy, ncy, j0, j1)) return out;
    const float zcut = P.z - Rq;
    float best = INFINITY;
    int best_id = -1;
    for (int j = j0; j <= j1; ++j)
      for (int i = i0; i <= i1; ++i) {
        f3 A = field_vertex(H, i, j), B1 = field_vertex(H, i + 1, j), C1 = field_vertex(H, i + 1, j + 1),
           D1 = field_vertex(H, i, j + 1);
        float zmax = fmaxf(fmaxf(A.z, B1.z), fmaxf(C1.z, D1.z));
        if (zcut > zmax) continue;  // whole cell further than r + margin + slack below the sphere
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          f3 Bv = t == 0 ? B1 : C1, Cv = t == 0 ? C1 : D1;
          f3 nt = cross3(sub3(Bv, A), sub3(Cv, A));
          float face = dot3(sub3(P, A), nt);
          if (face < 0.0f) continue;
          float v, w;
          tri_closest_vw(P, A, Bv, Cv, v, w);
          f3 df = sub3(P, tri_point(A, Bv, Cv, v, w));
          float d2 = dot3(df, df);
          if (d2 < best) { best = d2; best_id = 2 * (j * ncx + i) + t; }
        }
      }
    if (best_id < 0) return out;
    float dist = sqrtf(best);
    float d = dist - r;
    if (!(d < margin)) return out;
    // geometry of the winner
    int t = best_id & 1, c = best_id >> 1, i = c % ncx, j = c / ncx;
    // The winner's geometry is rebuilt in env-local coordinates (vertex minus env
    // origin), where the sphere centre carries no rounding from the world offset.
    f3 A = sub3(field_vertex(H, i, j), org);
    f3 Bv = sub3(t == 0 ? field_vertex(H, i + 1, j) : field_vertex(H, i + 1, j + 1), org);
    f3 Cv = sub3(t == 0 ? field_vertex(H, i + 1, j + 1) : field_vertex(H, i, j + 1), org);
    float v, w;
    tri_closest_vw(pl, A, Bv, Cv, v, w);
    f3 df = sub3(pl, tri_point(A, Bv, Cv, v, w));
    dist = sqrtf(dot3(df, df));
    d = dist - r;
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
    out.rc = f3{(pl.x - r * n.x) - xc.x, (pl.y - r * n.y) - xc.y, (pl.z - r * n.z) - xc.z};
    out.w = block_weight(margin, d, 1.0f);
    return out;
  }

  // mid-segment slot: segment interior against heightfield edges
  {
    float xl = P0.x < P1.x ? P0.x : P1.x, xh = P0.x < P1.x ? P1.x : P0.x;
    float yl = P0.y < P1.y ? P0.y : P1.y, yh = P0.y < P1.y ? P1.y : P0.y;
    int i0, i1, j0, j1;
    if (!cell_span(H, xl - Rq, xh + Rq, H.ox, ncx, i0, i1)) return out;
    if (!cell_span(H, yl - Rq, yh + Rq, H.oy, ncy, j0, j1)) return out;
    const float zcut = (P0.z < P1.z ? P0.z : P1.z) - Rq;
    float best = INFINITY;
    int best_id = -1;
    for (int j = j0; j <= j1 + 1; ++j)
      for (int i = i0; i <= i1 + 1; ++i) {
        f3 Q0 = field_vertex(H, i, j);
#pragma unroll
        for (int k = 0; k < 3; ++k) {
          if ((k == 0 || k == 2) && i > i1) continue;
          if ((k == 1 || k == 2) && j > j1) continue;
          f3 Q1 = k == 0 ? field_vertex(H, i + 1, j)
                         : (k == 1 ? field_vertex(H, i, j + 1) : field_vertex(H, i + 1, j + 1));
          if (zcut > fmaxf(Q0.z, Q1.z)) continue;  // edge entirely out of reach below the capsule
          float s, t;
          seg_edge_st(P0, P1, Q0, Q1, s, t);
          if (!(s > 0.001f && s < 0.999f)) continue;
          f3 d1 = sub3(P1, P0), d2 = sub3(Q1, Q0);
          f3 c1 = f3{P0.x + d1.x * s, P0.y + d1.y * s, P0.z + d1.z * s};
          f3 c2 = f3{Q0.x + d2.x * t, Q0.y + d2.y * t, Q0.z + d2.z * t};
          f3 df = sub3(c1, c2);
          if (!(df.z > 0.0f)) continue;
          float dd = dot3(df, df);
          if (dd < best) { best = dd; best_id = 3 * (j * H.nx + i) + k; }
        }
      }
    if (best_id < 0) return out;
    float dist = sqrtf(best);
    float d = dist - r;
    if (!(d < margin)) return out;
    int k = best_id % 3, vtx = best_id / 3, i = vtx % H.nx, j = vtx / H.nx;
    // winner's geometry in env-local coordinates (see the end-sphere case)
    f3 Q0 = sub3(field_vertex(H, i, j), org);
    f3 Q1 = sub3(k == 0 ? field_vertex(H, i + 1, j)
                        : (k == 1 ? field_vertex(H, i, j + 1) : field_vertex(H, i + 1, j + 1)), org);
    float s, t;
    seg_edge_st(p0, p1, Q0, Q1, s, t);
    f3 d1 = sub3(p1, p0), d2 = sub3(Q1, Q0);
    f3 cl = f3{p0.x + d1.x * s, p0.y + d1.y * s, p0.z + d1.z * s};
    f3 c2 = f3{Q0.x + d2.x * t, Q0.y + d2.y * t, Q0.z + d2.z * t};
    f3 df = sub3(cl, c2);
    dist = sqrtf(dot3(df, df));
    d = dist - r;
    f3 n;
    if (dist < 1e-9f) n = f3{0.0f, 0.0f, 1.0f};
    else { float inv = 1.0f / dist; n = f3{df.x * inv, df.y * inv, df.z * inv}; }
    out.active = 1; out.kind = 3; out.feat = best_id; out.d = d; out.n = n;
    out.rc = f3{(cl.x - r * n.x) - xc.x, (cl.y - r * n.y) - xc.y, (cl.z - r * n.z) - xc.z};
    {
      float se = s < 1.0f - s ? s : 1.0f - s;
      out.w = block_weight(margin, d, fminf(fmaxf((se - 0.001f) / 0.1f, 0.0f), 1.0f));
    }
    return out;
  }
}

#pragma clang fp contract(fast)

}  // namespace sim355
