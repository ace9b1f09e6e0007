"""Pins for the oracle's contact generation (speculative contacts, Section 3.1):
brute force over every feature, plane/heightfield agreement, analytic distances,
independent closest-point routines, a symmetry of the triangulated field."""
import numpy as np
import pytest
from scipy.optimize import minimize

import oracle
import scenes
from helpers import free_params, single_scene


def _random_field(seed, n=12, cell=0.1, amp=0.15):
    rng = np.random.default_rng(seed)
    t = scenes.make_flat_heightfield(nx=n, ny=n, cell=cell)
    t.heights = rng.uniform(0.0, amp, (n, n)).astype(np.float32)
    return t


def _capsule_scene(terrain, n_envs, seed, seg_len=0.3, radius=0.05, zlo=0.0, zhi=0.35, margin=0.02):
    rob = scenes.make_single(radius=radius, seg_len=seg_len, axis=0, pos=(0, 0, 0), mass=1.0)
    sc = single_scene(rob, terrain, params=free_params(contact_margin=margin), num_envs=n_envs)
    rng = np.random.default_rng(seed)
    ex, ey = terrain.extent if terrain.kind == scenes.HEIGHTFIELD else (1.0, 1.0)
    st = np.zeros((n_envs, 1, 13))
    st[:, 0, 0] = rng.uniform(-0.1, ex + 0.1, n_envs)
    st[:, 0, 1] = rng.uniform(-0.1, ey + 0.1, n_envs)
    st[:, 0, 2] = rng.uniform(zlo, zhi, n_envs)
    q = rng.normal(size=(n_envs, 4))
    st[:, 0, 3:7] = q / np.linalg.norm(q, axis=1, keepdims=True)
    st = st.astype(np.float32).astype(np.float64)
    return rob, sc, st


def test_culled_search_equals_brute_force_over_all_features():
    terrain = _random_field(1)
    rob, sc, st = _capsule_scene(terrain, 400, 2)
    o = oracle.OracleSim(sc)
    o.set_state(st)
    fast, brute = o.generate_contacts(False), o.generate_contacts(True)
    for f in ("active", "kind", "feat"):
        assert np.array_equal(fast[f], brute[f])
    for f in ("d", "n", "rc"):
        assert np.array_equal(fast[f], brute[f])
    # the scene exercises every kind of record
    assert set(np.unique(fast["kind"])) == {-1, 1, 2, 3}
    assert 0.2 < fast["active"].mean() < 0.9


def test_flat_heightfield_reproduces_plane_contacts():
    flat = scenes.make_flat_heightfield(nx=16, ny=16, cell=0.1, height=0.0)
    rob, sc_h, st = _capsule_scene(flat, 200, 3, zlo=0.02, zhi=0.25)
    st[:, 0, 0] = np.clip(st[:, 0, 0], 0.3, 1.2)
    st[:, 0, 1] = np.clip(st[:, 0, 1], 0.3, 1.2)
    sc_p = single_scene(rob, scenes.make_plane(), params=sc_h.params, num_envs=200)
    oh, op = oracle.OracleSim(sc_h), oracle.OracleSim(sc_p)
    oh.set_state(st); op.set_state(st)
    ch, cp = oh.generate_contacts(), op.generate_contacts()
    ends_h = ch[:, :2]
    # a centre that starts below z = 0 is "underneath" on the field; both give the same geometry
    assert np.array_equal(ends_h["active"], cp["active"])
    act = cp["active"] == 1
    assert act.sum() > 50
    np.testing.assert_allclose(ends_h["d"][act], cp["d"][act], atol=1e-12)
    np.testing.assert_allclose(ends_h["n"][act], cp["n"][act], atol=1e-12)
    np.testing.assert_allclose(ends_h["rc"][act], cp["rc"][act], atol=1e-12)


def test_sphere_over_tilted_plane_field_has_analytic_distance():
    a, b, c = 0.3, -0.2, 0.1
    terrain = scenes.make_tilted_heightfield(nx=24, ny=24, cell=0.1, slope_x=a, slope_y=b, z0=c)
    rob = scenes.make_single(radius=0.08, seg_len=0.0, pos=(0, 0, 0))
    n_envs = 300
    sc = single_scene(rob, terrain, params=free_params(contact_margin=0.05), num_envs=n_envs)
    rng = np.random.default_rng(5)
    st = np.zeros((n_envs, 1, 13)); st[:, 0, 3] = 1
    st[:, 0, 0] = rng.uniform(0.5, 1.8, n_envs)
    st[:, 0, 1] = rng.uniform(0.5, 1.8, n_envs)
    plane_z = a * st[:, 0, 0] + b * st[:, 0, 1] + c
    st[:, 0, 2] = plane_z + rng.uniform(-0.05, 0.2, n_envs)
    st = st.astype(np.float32).astype(np.float64)
    o = oracle.OracleSim(sc)
    o.set_state(st)
    rec = o.generate_contacts()[:, 0]
    nrm = np.sqrt(1 + a * a + b * b)
    d_exact = (st[:, 0, 2] - (a * st[:, 0, 0] + b * st[:, 0, 1] + c)) / nrm - 0.08
    assert np.array_equal(rec["active"] == 1, d_exact < 0.05 - 1e-6) or \
        np.abs(d_exact[(rec["active"] == 1) != (d_exact < 0.05)] - 0.05).max() < 1e-5
    act = rec["active"] == 1
    assert act.sum() > 40 and (rec["kind"][act] == 2).any() and (rec["kind"][act] == 1).any()
    np.testing.assert_allclose(rec["d"][act], d_exact[act], atol=2e-6)   # heights are fp32 samples
    n_exact = np.array([-a, -b, 1.0]) / nrm
    np.testing.assert_allclose(rec["n"][act], np.broadcast_to(n_exact, (act.sum(), 3)), atol=2e-5)
    # lever arm reaches the sphere's surface point along -n
    np.testing.assert_allclose(rec["rc"][act], -0.08 * rec["n"][act], atol=1e-12)


def _tri_vertices(terrain, tri):
    ncx = terrain.nx - 1
    t, c = tri & 1, tri >> 1
    i, j = c % ncx, c // ncx
    def v(ii, jj):
        return np.array([np.float32(terrain.origin[0]) + np.float32(ii) * np.float32(terrain.cell),
                         np.float32(terrain.origin[1]) + np.float32(jj) * np.float32(terrain.cell),
                         terrain.heights[jj, ii]], np.float64)
    if t == 0:
        return v(i, j), v(i + 1, j), v(i + 1, j + 1)
    return v(i, j), v(i + 1, j + 1), v(i, j + 1)


def _dist_point_triangle_indep(P, A, B, C):
    """Different route from the oracle's: face projection if inside, else best of
    the three clamped edge projections."""
    n = np.cross(B - A, C - A)
    n /= np.linalg.norm(n)
    Q = P - n * ((P - A) @ n)
    inside = all(np.cross(b - a, Q - a) @ n >= 0 for a, b in ((A, B), (B, C), (C, A)))
    if inside:
        return np.linalg.norm(P - Q)
    best = np.inf
    for a, b in ((A, B), (B, C), (C, A)):
        t = np.clip((P - a) @ (b - a) / ((b - a) @ (b - a)), 0, 1)
        best = min(best, np.linalg.norm(P - (a + t * (b - a))))
    return best


def test_end_sphere_distance_is_the_minimum_over_front_facing_triangles():
    terrain = _random_field(7, n=6, amp=0.12)
    rob = scenes.make_single(radius=0.06, seg_len=0.0, pos=(0, 0, 0))
    n_envs = 300
    sc = single_scene(rob, terrain, params=free_params(contact_margin=0.04), num_envs=n_envs)
    rng = np.random.default_rng(8)
    st = np.zeros((n_envs, 1, 13)); st[:, 0, 3] = 1
    st[:, 0, 0:2] = rng.uniform(0.05, 0.45, (n_envs, 2))
    st[:, 0, 2] = rng.uniform(0.0, 0.25, n_envs)
    st = st.astype(np.float32).astype(np.float64)
    o = oracle.OracleSim(sc)
    o.set_state(st)
    rec = o.generate_contacts()[:, 0]
    n_tri = 2 * (terrain.nx - 1) * (terrain.ny - 1)
    checked = 0
    for e in range(n_envs):
        P = st[e, 0, 0:3]
        if rec["kind"][e] == 2:
            A, B, C = _tri_vertices(terrain, rec["feat"][e])
            n = np.cross(B - A, C - A); n /= np.linalg.norm(n)
            assert (P - A) @ n < 0
            assert rec["d"][e] == pytest.approx((P - A) @ n - 0.06, abs=1e-9)
            continue
        best = np.inf
        for tri in range(n_tri):
            A, B, C = _tri_vertices(terrain, tri)
            if (P - A) @ np.cross(B - A, C - A) < 0:
                continue
            best = min(best, _dist_point_triangle_indep(P, A, B, C))
        d = best - 0.06
        if abs(d - 0.04) < 1e-5:
            continue
        assert (rec["active"][e] == 1) == (d < 0.04)
        if rec["active"][e]:
            assert rec["d"][e] == pytest.approx(d, abs=1e-6)
            assert np.linalg.norm(rec["n"][e]) == pytest.approx(1.0, abs=1e-12)
            checked += 1
    assert checked > 50


def test_mid_segment_slot_matches_bounded_minimisation():
    terrain = _random_field(11, n=5, amp=0.2)
    rob, sc, st = _capsule_scene(terrain, 120, 12, seg_len=0.3, radius=0.04, zlo=0.1, zhi=0.3, margin=0.03)
    st[:, 0, 0:2] = np.random.default_rng(1).uniform(0.1, 0.3, (120, 2))
    st = st.astype(np.float32).astype(np.float64)
    o = oracle.OracleSim(sc)
    o.set_state(st)
    rec = o.generate_contacts(True)[:, 2]
    from helpers import rot_of
    nx = terrain.nx
    verts = lambda i, j: np.array([i * np.float32(0.1), j * np.float32(0.1), terrain.heights[j, i]], np.float64)
    checked = 0
    for e in range(120):
        if not rec["active"][e]:
            continue
        ax = rot_of(st[e, 0, 3:7]).apply([1.0, 0, 0]) * 0.15
        P0, P1 = st[e, 0, 0:3] - ax, st[e, 0, 0:3] + ax
        k, vtx = rec["feat"][e] % 3, rec["feat"][e] // 3
        i, j = vtx % nx, vtx // nx
        Q0 = verts(i, j)
        Q1 = verts(i + 1, j) if k == 0 else (verts(i, j + 1) if k == 1 else verts(i + 1, j + 1))
        f = lambda z: np.sum((P0 + z[0] * (P1 - P0) - Q0 - z[1] * (Q1 - Q0)) ** 2)
        best = min((minimize(f, z0, bounds=[(0, 1), (0, 1)], method="L-BFGS-B",
                             options=dict(ftol=1e-15, gtol=1e-12)) for z0 in
                    ([0.5, 0.5], [0.1, 0.1], [0.9, 0.9], [0.1, 0.9], [0.9, 0.1])), key=lambda r: r.fun)
        assert rec["d"][e] == pytest.approx(np.sqrt(best.fun) - 0.04, abs=2e-6)
        assert 0.001 < best.x[0] < 0.999 or abs(best.x[0] - 0.001) < 1e-3 or abs(best.x[0] - 0.999) < 1e-3
        assert rec["n"][e][2] > 0
        checked += 1
    assert checked > 10


def test_half_turn_about_field_centre_maps_records_onto_each_other():
    # the fixed diagonal of each cell is invariant under a 180 degree turn about z
    n, cell = 10, 0.125      # cell exactly representable: vertex coordinates carry no rounding
    rng = np.random.default_rng(21)
    t1 = scenes.make_flat_heightfield(nx=n, ny=n, cell=cell)
    t1.heights = rng.uniform(0, 0.15, (n, n)).astype(np.float32)
    t2 = scenes.make_flat_heightfield(nx=n, ny=n, cell=cell)
    t2.heights = np.ascontiguousarray(t1.heights[::-1, ::-1])
    ext = (n - 1) * cell
    rob, sc1, st1 = _capsule_scene(t1, 200, 22, seg_len=0.25, zlo=0.02, zhi=0.3)
    st1[:, 0, 0:2] = np.round(st1[:, 0, 0:2] * 1024) / 1024       # exact under x -> ext - x
    st2 = st1.copy()
    st2[:, 0, 0] = ext - st1[:, 0, 0]
    st2[:, 0, 1] = ext - st1[:, 0, 1]
    # rotate orientation by pi about z: q' = (0,0,0,1) * q
    w, x, y, z = (st1[:, 0, 3 + k] for k in range(4))
    st2[:, 0, 3], st2[:, 0, 4], st2[:, 0, 5], st2[:, 0, 6] = -z, -y, x, w
    sc2 = single_scene(rob, t2, params=sc1.params, num_envs=200)
    o1, o2 = oracle.OracleSim(sc1), oracle.OracleSim(sc2)
    o1.set_state(st1); o2.set_state(st2)
    c1, c2 = o1.generate_contacts(), o2.generate_contacts()
    same = c1["active"] == c2["active"]
    assert same.mean() > 0.99
    act = (c1["active"] == 1) & same
    assert act.sum() > 100
    np.testing.assert_allclose(c1["d"][act], c2["d"][act], atol=1e-6)
    flip = np.array([-1.0, -1.0, 1.0])
    np.testing.assert_allclose(c1["n"][act], c2["n"][act] * flip, atol=1e-5)
    np.testing.assert_allclose(c1["rc"][act], c2["rc"][act] * flip, atol=1e-6)


def test_plane_contact_record_closed_form():
    rob = scenes.make_single(radius=0.05, seg_len=0.4, axis=0, pos=(0, 0, 0))
    sc = single_scene(rob, params=free_params(contact_margin=0.02))
    o = oracle.OracleSim(sc)
    st = np.zeros((1, 1, 13))
    ang = 0.3                                   # pitched about y: +x end dips
    st[0, 0, 0:3] = (0.2, -0.1, 0.1)
    st[0, 0, 3:7] = (np.cos(ang / 2), 0, np.sin(ang / 2), 0)
    o.set_state(st)
    c = o.generate_contacts()[0]
    z_hi, z_lo = 0.1 + 0.2 * np.sin(ang), 0.1 - 0.2 * np.sin(ang)
    # rotation by +ang about y sends +x towards -z
    assert c[1]["d"] == pytest.approx(z_lo - 0.05, abs=1e-12)
    assert c[0]["d"] == pytest.approx(z_hi - 0.05, abs=1e-12) or c[0]["active"] == 0
    assert c[1]["active"] == 1 and c[0]["active"] == 0
    np.testing.assert_allclose(c[1]["n"], (0, 0, 1))
    np.testing.assert_allclose(c[1]["rc"], (0.2 * np.cos(ang), 0, -0.2 * np.sin(ang) - 0.05), atol=1e-12)


def test_outside_the_heightfield_there_is_no_terrain():
    """Reading of this build (the border is not extended outwards): a sphere 1 cm above a flat
    field of height 0.2 m touches it while its centre is over the field, touches the border edge
    / corner while it is within reach of it, and touches nothing beyond: it keeps falling."""
    t = scenes.make_flat_heightfield(nx=12, ny=12, cell=0.1)          # extent 1.1 x 1.1 m
    t.heights[:] = 0.2
    r = 0.05
    rob = scenes.make_single(radius=r, pos=(0.0, 0.0, 0.0), mass=1.0)
    xs = [0.5, 1.09, 1.1 + 0.03, 1.1 + r + 0.03, 3.0, -0.03, -(r + 0.03), -2.0]
    sc = single_scene(rob, t, params=free_params(), num_envs=len(xs))
    sc.env_origins[:] = 0.0
    st = np.zeros((len(xs), 1, 13))
    st[:, 0, 0], st[:, 0, 1], st[:, 0, 2], st[:, 0, 3] = xs, 0.55, 0.2 + r + 0.01, 1.0
    o = oracle.OracleSim(sc)
    o.set_state(st)
    con = o.generate_contacts(False)
    active = con["active"][:, 0].astype(bool)
    assert active.tolist() == [True, True, True, False, False, True, False, False]
    assert np.array_equal(active, o.generate_contacts(True)["active"][:, 0].astype(bool))
    # over the field: the face under it, 1 cm away; beyond the border but within reach: the border edge
    assert con["d"][0, 0] == pytest.approx(0.01, abs=1e-6) and con["n"][0, 0] == pytest.approx([0, 0, 1], abs=1e-6)
    assert con["d"][2, 0] == pytest.approx(np.hypot(0.03, r + 0.01) - r, abs=1e-6) and con["n"][2, 0, 0] > 0.3
    for _ in range(30):
        o.step(None, 1.0 / 60.0, 2, 8)
    z = o.get_state()[:, 0, 2]
    # over the field it rests; beyond the border it falls (also after rolling off the border edge)
    assert np.all(z[:2] > 0.2 + r - 2e-3) and np.all(z[2:] < 0.0)
