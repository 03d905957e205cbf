"""Pins of the oracle's collision manifolds (paper A.3.1-A.3.4) against things other than itself:
hand-evaluated cases, closed forms for axis-aligned boxes, and brute force (dense point sampling)."""
import numpy as np
import pytest

from oracle import k2d_oracle as ko

SQ = np.array([[0, 0], [1, 0], [1, 1], [0, 1]], dtype=float)   # unit square, CCW


# ---------------------------------------------------------------- circle-circle (A.3.2)
@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_cc_hand_numbers(dtype):
    m = ko.manifold_cc([0, 0], 1.0, [1.5, 0], 1.0, dtype)
    assert np.allclose(m["normal"], [1, 0]) and np.allclose(m["pos"][0], [1, 0]) and np.isclose(m["pen"][0], 0.5)
    # 3-4-5 triangle: centres 0.5 apart along (0.6, 0.8)
    m = ko.manifold_cc([1, 1], 0.25, [1.3, 1.4], 0.5, dtype)
    assert np.allclose(m["normal"], [0.6, 0.8], atol=1e-6)
    assert np.allclose(m["pos"][0], [1.15, 1.2], atol=1e-6)
    assert np.isclose(m["pen"][0], 0.25, atol=1e-6)
    # separated circles: negative penetration
    assert ko.manifold_cc([0, 0], 1.0, [3, 0], 1.0, dtype)["pen"][0] == pytest.approx(-1.0)


def test_cc_swap_symmetry():
    rng = np.random.default_rng(1)
    for _ in range(50):
        pa, pb = rng.uniform(-2, 2, 2), rng.uniform(-2, 2, 2)
        ra, rb = rng.uniform(0.1, 1, 2)
        m1, m2 = ko.manifold_cc(pa, ra, pb, rb), ko.manifold_cc(pb, rb, pa, ra)
        assert np.allclose(m1["normal"], -m2["normal"]) and np.isclose(m1["pen"][0], m2["pen"][0])
        # both contact points lie on the segment between the centres, pen apart
        assert np.allclose(m1["pos"][0] - m1["pen"][0] * m1["normal"], m2["pos"][0], atol=1e-12)


# ---------------------------------------------------------------- polygon-circle (A.3.3)
@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_pc_hand_numbers(dtype):
    tol = 1e-12 if dtype == "f64" else 1e-6
    m = ko.manifold_pc(SQ, [0.5, 1.2], 0.3, dtype)            # above the top edge
    assert np.allclose(m["normal"], [0, 1], atol=tol) and np.allclose(m["pos"][0], [0.5, 1.0], atol=tol)
    assert np.isclose(m["pen"][0], 0.1, atol=tol)
    m = ko.manifold_pc(SQ, [1.3, 1.4], 0.6, dtype)            # beyond the corner (1,1): clipped to it
    assert np.allclose(m["normal"], [0.6, 0.8], atol=tol) and np.allclose(m["pos"][0], [1, 1], atol=tol)
    assert np.isclose(m["pen"][0], 0.1, atol=tol)
    m = ko.manifold_pc(SQ, [0.5, 0.9], 0.2, dtype)            # centre inside: nearest face is the top one
    assert np.allclose(m["normal"], [0, 1], atol=tol) and np.allclose(m["pos"][0], [0.5, 1.0], atol=tol)
    assert np.isclose(m["pen"][0], 0.3, atol=tol)
    m = ko.manifold_pc(SQ, [0.5, 2.0], 0.3, dtype)            # far away
    assert m["pen"][0] == pytest.approx(-0.7, abs=tol)


def _boundary_samples(poly, step=2e-4):
    pts = []
    n = len(poly)
    for i in range(n):
        a, b = poly[i], poly[(i + 1) % n]
        k = int(np.ceil(np.linalg.norm(b - a) / step)) + 1
        t = np.linspace(0, 1, k)[:, None]
        pts.append(a + t * (b - a))
    return np.concatenate(pts)


def _inside(poly, pts):
    """Points strictly inside a CCW convex polygon (half-plane test)."""
    ok = np.ones(len(pts), dtype=bool)
    n = len(poly)
    for i in range(n):
        a, b = poly[i], poly[(i + 1) % n]
        ok &= ((b[0] - a[0]) * (pts[:, 1] - a[1]) - (b[1] - a[1]) * (pts[:, 0] - a[0])) > 0
    return ok


def _random_convex(rng, n, scale=1.0):
    while True:
        ang = np.sort(rng.uniform(0, 2 * np.pi, n))
        if np.min(np.diff(np.concatenate([ang, [ang[0] + 2 * np.pi]]))) < 0.5:
            continue
        r = rng.uniform(0.4, 1.0, n) * scale
        p = np.stack([r * np.cos(ang), r * np.sin(ang)], 1)
        # keep only convex ones
        e = np.roll(p, -1, 0) - p
        cr = e[:, 0] * np.roll(e, -1, 0)[:, 1] - e[:, 1] * np.roll(e, -1, 0)[:, 0]
        if (cr > 0.05).all():
            return p


def test_pc_brute_force_distance():
    """Outside the polygon, r - pen is the distance from the centre to the densely sampled boundary and
    pos is the nearest boundary point; inside, pen - r is the depth to the nearest face."""
    rng = np.random.default_rng(7)
    n_out = n_in = 0
    for _ in range(200):
        poly = _random_convex(rng, int(rng.integers(3, 5)))
        c = rng.uniform(-1.6, 1.6, 2) * (0.3 if rng.uniform() < 0.3 else 1.0)
        r = rng.uniform(0.05, 0.6)
        m = ko.manifold_pc(poly, c, r)
        bd = _boundary_samples(poly)
        d = np.linalg.norm(bd - c, axis=1)
        k = d.argmin()
        if _inside(poly, c[None])[0]:
            n_in += 1
            assert m["pen"][0] - r == pytest.approx(d[k], abs=3e-4)
            assert np.allclose(m["pos"][0], bd[k], atol=5e-4)
            # normal is the outward normal of the nearest face: moving along it leaves the polygon
            assert not _inside(poly, (c + (d[k] + 1e-3) * m["normal"])[None])[0]
        else:
            n_out += 1
            assert r - m["pen"][0] == pytest.approx(d[k], abs=3e-4)
            assert np.allclose(m["pos"][0], bd[k], atol=5e-4)
            assert np.allclose(m["normal"], (c - bd[k]) / d[k], atol=1e-3 + 4e-4 / d[k])
        assert np.isclose(np.linalg.norm(m["normal"]), 1.0)
    assert n_out > 50 and n_in > 20


# ---------------------------------------------------------------- polygon-polygon (A.3.4)
def _box(cx, cy, hx, hy):
    return np.array([[cx - hx, cy - hy], [cx + hx, cy - hy], [cx + hx, cy + hy], [cx - hx, cy + hy]], dtype=float)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_pp_box_on_floor_closed_form(dtype):
    """Axis-aligned box sunk 0.05 into a wide floor: two points, at the box's bottom corners, each with
    penetration 0.05, normal from the floor (a) up to the box (b)."""
    floor = _box(0, 0, 5, 0.1)
    box = _box(0.3, 0.1 + 0.5 - 0.05, 0.5, 0.5)
    m = ko.manifold_pp(floor, box, dtype=dtype)
    tol = 1e-12 if dtype == "f64" else 1e-6
    assert list(m["valid"]) == [1, 1]
    assert np.allclose(m["normal"], [0, 1], atol=tol)
    assert np.allclose(m["pen"], [0.05, 0.05], atol=tol)
    got = sorted(map(tuple, np.round(m["pos"], 6)))
    assert np.allclose(got, [(-0.2, 0.05), (0.8, 0.05)], atol=1e-5)


def test_pp_box_overhanging_edge_is_clipped():
    """A box overhanging the end of the floor: the incident face is clipped to the floor's side plane."""
    floor = _box(0, 0, 1, 0.1)                       # top face spans x in [-1, 1]
    box = _box(1.2, 0.1 + 0.5 - 0.02, 0.5, 0.5)      # bottom face spans x in [0.7, 1.7]
    m = ko.manifold_pp(floor, box)
    assert list(m["valid"]) == [1, 1] and np.allclose(m["pen"], [0.02, 0.02])
    xs = sorted(m["pos"][:, 0])
    assert np.allclose(xs, [0.7, 1.0])               # clipped at the floor's right end
    assert np.allclose(m["pos"][:, 1], 0.08)


def test_pp_triangle_vertex_into_face():
    """A triangle pointing down into the floor: only the tip penetrates -> one active point."""
    floor = _box(0, 0, 5, 0.1)
    tri = np.array([[0.0, 0.07], [0.6, 1.0], [-0.6, 1.0]])   # CCW, tip 0.03 below the floor top (y = 0.1)
    m = ko.manifold_pp(floor, tri)
    act = (m["valid"] == 1) & (m["pen"] > 0)
    assert act.sum() == 1
    k = int(np.argmax(act))
    assert np.allclose(m["pos"][k], [0.0, 0.07]) and np.isclose(m["pen"][k], 0.03)
    assert np.allclose(m["normal"], [0, 1])


def test_pp_separated_and_swapped():
    a, b = _box(0, 0, 0.5, 0.5), _box(1.2, 0, 0.5, 0.5)
    m = ko.manifold_pp(a, b)
    assert not ((m["valid"] == 1) & (m["pen"] > 0)).any()
    # overlapping by 0.1 along x; the normal always points from the first polygon to the second
    b = _box(0.9, 0.05, 0.5, 0.5)
    m1, m2 = ko.manifold_pp(a, b), ko.manifold_pp(b, a)
    assert np.allclose(m1["normal"], [1, 0]) and np.allclose(m2["normal"], [-1, 0])
    assert np.allclose(m1["pen"].max(), 0.1) and np.allclose(m2["pen"].max(), 0.1)


def test_pp_reference_face_hysteresis():
    """Parallel resting faces: the reference face stays with the first polygon unless the second one's
    face separation wins by more than tie_eps."""
    floor = _box(0, 0, 5, 0.1)
    box = _box(0, 0.1 + 0.5 - 0.01, 0.5, 0.5)
    m = ko.manifold_pp(floor, box)
    # reference = floor: contact points are the box's corners (y = 0.09), not points on the floor top (y = 0.1)
    assert np.allclose(m["pos"][:, 1], 0.09)
    m = ko.manifold_pp(box, floor)     # now the box is the first polygon: points are on the floor's top face
    assert np.allclose(m["pos"][:, 1], 0.1) and np.allclose(m["normal"], [0, -1])


def test_pp_brute_force_overlap_and_separation():
    """Dense point sampling: some manifold point is active <=> the interiors share a sampled point
    (cases closer to touching than the grid are skipped); moving b along the normal by the deepest
    penetration separates the polygons."""
    rng = np.random.default_rng(11)
    g = np.linspace(-2.2, 2.2, 1467)                 # grid pitch 3e-3
    gx, gy = np.meshgrid(g, g)
    grid = np.stack([gx.ravel(), gy.ravel()], 1)
    n_hit = n_miss = 0
    for _ in range(60):
        A = _random_convex(rng, int(rng.integers(3, 5)), 0.8)
        B = _random_convex(rng, int(rng.integers(3, 5)), 0.8) + rng.uniform(-1.3, 1.3, 2)
        m = ko.manifold_pp(A, B)
        active = (m["valid"] == 1) & (m["pen"] > 0)
        # local grid around A only
        inA = _inside(A, grid)
        both = _inside(B, grid[inA]).any()
        deepest = m["pen"][active].max() if active.any() else 0.0
        if active.any() and deepest < 8e-3:
            continue
        if not active.any():
            # separated by at least the margin the oracle reports?  (margin = |largest face separation|)
            if m["margin"] < 8e-3:
                continue
        assert both == bool(active.any())
        if active.any():
            n_hit += 1
            assert np.isclose(np.linalg.norm(m["normal"]), 1.0)
            B2 = B + (deepest + 4e-3) * m["normal"]
            inB2 = _inside(B2, grid[inA])
            assert not inB2.any(), "polygons still overlap after moving b out along the normal"
            # every active point is a (clipped) vertex of the incident face: it lies on the boundary of
            # one of the two polygons
            for k in np.nonzero(active)[0]:
                p = m["pos"][k]
                on = []
                for poly in (A, B):
                    e = np.roll(poly, -1, 0) - poly
                    nrm = np.stack([e[:, 1], -e[:, 0]], 1) / np.linalg.norm(e, axis=1)[:, None]
                    on.append(abs(((p - poly) * nrm).sum(1).max()) < 1e-9)
                assert any(on)
        else:
            n_miss += 1
    assert n_hit > 10 and n_miss > 10


def test_pp_float_and_double_agree():
    rng = np.random.default_rng(5)
    for _ in range(100):
        A = _random_convex(rng, 4, 0.8)
        B = _random_convex(rng, 3, 0.8) + rng.uniform(-1.0, 1.0, 2)
        m64, m32 = ko.manifold_pp(A, B, dtype="f64"), ko.manifold_pp(A, B, dtype="f32")
        if m64["margin"] < 1e-4:
            continue
        assert (m64["valid"] == m32["valid"]).all()
        if m64["valid"].any():
            assert np.allclose(m64["pen"], m32["pen"], atol=1e-5) and np.allclose(m64["pos"], m32["pos"], atol=1e-5)
