"""Degenerate input has a defined result (oracle side): coincident circle centres (A.3.2 prints a 0 / 0
normal), a polygon edge without length (its normal is 0 / 0), a joint with both ends on one shape, shape
indices outside the arrays, and a scene that blows up -- which the health check must flag."""
import numpy as np
import pytest

from helpers import degenerate_scene, same_bits_or_both_nan, DEGENERATE_TRI
from oracle import k2d_env
from oracle.k2d_oracle import Oracle, manifold_cc, manifold_pc, manifold_pp

KEYS = ("pos", "theta", "vel", "omega", "joint_acc", "joint_acc_ang", "lambda_n", "lambda_t", "pair_count")


def run(caps, prm, sc, steps):
    o = Oracle(caps, sc["pos"].shape[0], prm, "f32")
    o.load_scene(sc)
    o.step(np.zeros((steps, sc["pos"].shape[0], caps[2] + caps[3])))
    return o


def test_coincident_circle_centres_take_the_x_axis_as_normal():
    for dtype in ("f64", "f32"):
        m = manifold_cc((0.5, 1.0), 0.25, (0.5, 1.0), 0.4, dtype)
        assert m["normal"].tolist() == [1.0, 0.0]
        assert m["pen"][0] == pytest.approx(0.65) and m["pos"][0].tolist() == [0.75, 1.0] and m["valid"][0] == 1
    caps, prm, sc, _, steps = degenerate_scene("coincident_circles")
    o = run(caps, dict(prm, gravity_y=0.0), sc, 1)
    st = o.state()
    P = caps[0]
    pos = st["pos"].reshape(1, -1, 2)[0]
    a, b = pos[P], pos[P + 1]
    assert a[0] < 0.5 < b[0] and a[1] == 1.0 and b[1] == 1.0            # pushed apart along x, not along y
    ima, imb = sc["inv_mass"][0, P], sc["inv_mass"][0, P + 1]
    assert (0.5 - a[0]) / (b[0] - 0.5) == pytest.approx(ima / imb, rel=1e-5)     # shared by inverse mass
    assert np.isfinite(st["pos"]).all() and np.isfinite(st["vel"]).all()


def test_edge_without_length_is_ignored_by_the_manifolds():
    quad = np.vstack([DEGENERATE_TRI, DEGENERATE_TRI[2:3]]) + np.array([0.0, 0.6])
    tri = DEGENERATE_TRI + np.array([0.0, 0.6])
    rng = np.random.default_rng(2)
    for c in [(0.0, 0.95), (0.02, 0.81), (0.3, 0.7), (-0.4, 0.45), (0.0, 0.6)] + list(rng.uniform(-0.6, 1.0, (40, 2))):
        mq = manifold_pc(quad, c, 0.2, "f32")
        mt = manifold_pc(tri, c, 0.2, "f32")
        for k in ("normal", "pos", "pen", "valid"):
            assert np.array_equal(mq[k], mt[k]), (c, k)
    # against another polygon the face without length reports "separated": no manifold, nothing non-finite
    box = np.array([[-0.3, 0.5], [0.3, 0.5], [0.3, 0.9], [-0.3, 0.9]])
    m = manifold_pp(quad, box, 1e-3, "f32")
    assert m["valid"].tolist() == [0, 0]
    caps, prm, sc, twin, steps = degenerate_scene("zero_length_edge")
    st = run(caps, prm, sc, steps).state()
    for k in KEYS:
        assert np.isfinite(st[k]).all(), k
    assert st["pair_count"].sum() > 0                                    # it does collide with the circle on top of it
    bad, n_bad = k2d_env.health(st["pos"].reshape(1, -1, 2), st["theta"], st["vel"].reshape(1, -1, 2), st["omega"],
                                sc["active"])
    assert n_bad == 0


@pytest.mark.parametrize("kind", ["joint_on_itself", "indices_out_of_range"])
def test_malformed_joints_and_thrusters_count_as_inactive(kind):
    caps, prm, sc, twin, steps = degenerate_scene(kind)
    a, b = run(caps, prm, sc, steps), run(caps, prm, twin, steps)
    sa, sb_ = a.state(), b.state()
    for k in KEYS:
        assert np.array_equal(sa[k], sb_[k]), k
        assert np.isfinite(sa[k]).all()
    assert np.isfinite(a.obs()).all()
    if kind == "joint_on_itself":      # and the sound joint of the scene did its work
        assert np.abs(sa["joint_acc"]).max() > 0


def test_a_scene_that_blows_up_is_flagged_by_the_health_check():
    caps, prm, sc, _, steps = degenerate_scene("infinite_inverse_mass")
    st = run(caps, prm, sc, steps).state()
    N = caps[0] + caps[1]
    bad, n_bad = k2d_env.health(st["pos"].reshape(1, N, 2), st["theta"], st["vel"].reshape(1, N, 2), st["omega"],
                                sc["active"])
    assert n_bad == 1 and bad.tolist() == [1]
    assert not np.isfinite(st["pos"].reshape(1, N, 2)[0, 1]).all()       # the shape with no mass
    assert same_bits_or_both_nan(st["pos"], st["pos"])
