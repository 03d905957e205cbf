"""Pins of the oracle's dynamics (paper Algorithm 1, A.2, A.3.5-A.3.7, A.4-A.7) against closed forms and
invariants: free fall under semi-implicit Euler, head-on collisions with restitution, resting box,
energy, friction, pendulum, fixed joint, motor law, thruster impulse, warm-start bookkeeping, the order
of the sweep."""
import numpy as np
import pytest

import scenegen
from helpers import SceneBuilder, energy, pair_index, params, zeros_actions
from oracle import k2d_oracle as ko
from oracle.k2d_oracle import Oracle

CAPS = (3, 2, 2, 1)


def run(sb_or_scene, p, caps=CAPS, dtype="f64", f32_inputs=False):
    sc = sb_or_scene.scene(f32=f32_inputs) if isinstance(sb_or_scene, SceneBuilder) else sb_or_scene
    o = Oracle(caps, sc["pos"].shape[0], p, dtype)
    o.load_scene(sc)
    return o, sc


# ------------------------------------------------------------------ gravity + Euler step (Alg. 1)
@pytest.mark.parametrize("n_sub", [1, 3])
def test_free_fall_closed_form(n_sub):
    """Semi-implicit Euler: v_k = v_0 + k g h, y_k = y_0 + v_0 k h + g h^2 k(k+1)/2; x, theta linear."""
    sb = SceneBuilder(CAPS)
    i = sb.circle(0.3, (1.0, 50.0), vel=(0.7, 2.0), omega=1.5, theta=0.25)
    p = params(n_substeps=n_sub)
    o, sc = run(sb, p)
    n = 40
    o.step(zeros_actions(n, 1, CAPS))
    h, g, k = p["dt"] / n_sub, p["gravity_y"], n * n_sub
    st = o.state()
    pos = st["pos"].reshape(1, -1, 2)[0, i]
    assert pos[0] == pytest.approx(1.0 + 0.7 * k * h, rel=1e-13)
    assert pos[1] == pytest.approx(50.0 + 2.0 * k * h + g * h * h * k * (k + 1) / 2, rel=1e-13)
    assert st["vel"].reshape(1, -1, 2)[0, i, 1] == pytest.approx(2.0 + g * k * h, rel=1e-13)
    assert st["theta"][0, i] == pytest.approx(0.25 + 1.5 * k * h, rel=1e-13)
    # fp32 instance follows within rounding
    o32, _ = run(sb, p, dtype="f32", f32_inputs=True)
    o32.step(zeros_actions(n, 1, CAPS))
    assert np.allclose(o32.state()["pos"], st["pos"], rtol=2e-6, atol=1e-5)


def test_static_and_inactive_bodies_do_not_move():
    sb = SceneBuilder(CAPS)
    a = sb.box(1, 0.1, (0, 0), static=True)
    b = sb.circle(0.2, (0, 5))
    sb.sc["active"][0, b] = 0
    o, _ = run(sb, params())
    o.step(zeros_actions(10, 1, CAPS))
    st = o.state()
    assert np.all(st["pos"].reshape(-1, 2)[a] == 0) and np.all(st["pos"].reshape(-1, 2)[b] == (0, 5))
    assert np.all(st["vel"] == 0)


# ------------------------------------------------------------------ normal impulse (A.3.5)
@pytest.mark.parametrize("e", [0.0, 0.5, 1.0])
@pytest.mark.parametrize("mass_ratio", [1.0, 3.0])
def test_head_on_circles_restitution(e, mass_ratio):
    """Two circles meet head-on, no gravity, no corrections: momentum is conserved and the relative
    normal velocity becomes -e times what it was; e = 1 conserves kinetic energy; equal masses swap."""
    sb = SceneBuilder(CAPS)
    a = sb.circle(0.5, (-0.6, 0.0), vel=(2.0, 0.0), restitution=e, density=1.0, friction=0.0)
    b = sb.circle(0.5, (0.6, 0.0), vel=(-1.0, 0.0), restitution=e, density=mass_ratio, friction=0.0)
    p = params(gravity_y=0.0, alpha=0.0, beta=0.0, n_iters=4)
    o, sc = run(sb, p)
    ma, mb = 1 / sc["inv_mass"][0, a], 1 / sc["inv_mass"][0, b]
    n = 12
    o.step(zeros_actions(n, 1, CAPS))
    v = o.state()["vel"].reshape(-1, 2)
    assert ma * v[a, 0] + mb * v[b, 0] == pytest.approx(ma * 2.0 - mb * 1.0, rel=1e-12)
    assert v[a, 0] - v[b, 0] == pytest.approx(-e * 3.0, abs=1e-12)
    if e == 1.0:
        assert 0.5 * ma * v[a, 0] ** 2 + 0.5 * mb * v[b, 0] ** 2 == pytest.approx(0.5 * ma * 4 + 0.5 * mb * 1, rel=1e-12)
        if mass_ratio == 1.0:
            assert v[a, 0] == pytest.approx(-1.0) and v[b, 0] == pytest.approx(2.0)
    assert np.allclose(v[:, 1], 0) and np.allclose(o.state()["omega"], 0)


def test_positional_correction_uses_the_deepest_point_of_the_pair():
    """A.3.7 with a two-point manifold: a tilted box sunk into the floor, nothing moving, no sweeps.  One substep
    moves the box out along the normal by beta * (deepest penetration - slop), the floor not at all."""
    sb = SceneBuilder(CAPS)
    sb.box(5.0, 0.5, (0.0, -0.5), static=True)
    tilt = 0.05
    box = sb.box(0.5, 0.3, (0.0, 0.3 * np.cos(tilt) + 0.5 * np.sin(tilt) - 0.06), theta=tilt)
    p = params(gravity_y=0.0, n_iters=0, warm_start=0, beta=0.2, slop=0.005)
    o, sc = run(sb, p)
    o.step(zeros_actions(1, 1, CAPS))
    N = CAPS[0] + CAPS[1]
    pi = pair_index(0, box, N)
    pen = o.get("manifold_pen").reshape(1, -1, 2)[0, pi]
    act = o.get("pair_active").reshape(1, -1, 2)[0, pi]
    nrm = o.get("manifold_normal").reshape(1, -1, 2)[0, pi]
    assert act.all() and pen.max() == pytest.approx(0.06, abs=1e-9) and pen.max() - pen.min() > 0.04
    assert nrm == pytest.approx([0.0, 1.0], abs=1e-12)
    moved = o.state()["pos"].reshape(-1, 2)[box] - sc["pos"][0, box]
    assert moved == pytest.approx(0.2 * (pen.max() - 0.005) * nrm, abs=1e-12)
    assert np.array_equal(o.state()["pos"].reshape(-1, 2)[0], sc["pos"][0, 0])


def test_restitution_of_a_pair_is_the_smaller_of_the_two():
    """A.3.5: e = min(e_a, e_b).  A bouncy circle meets a dead one head-on: the relative normal velocity becomes
    -0.2 times what it was, not -0.9 times."""
    sb = SceneBuilder(CAPS)
    a = sb.circle(0.5, (-0.6, 0.0), vel=(2.0, 0.0), restitution=0.9, friction=0.0)
    b = sb.circle(0.5, (0.6, 0.0), vel=(-1.0, 0.0), restitution=0.2, friction=0.0)
    o, _ = run(sb, params(gravity_y=0.0, alpha=0.0, beta=0.0, n_iters=4))
    o.step(zeros_actions(12, 1, CAPS))
    v = o.state()["vel"].reshape(-1, 2)
    assert v[a, 0] - v[b, 0] == pytest.approx(-0.2 * 3.0, abs=1e-12)


def test_slow_approach_has_no_bounce():
    """Below the restitution threshold the collision is inelastic even for e = 1."""
    sb = SceneBuilder(CAPS)
    a = sb.circle(0.5, (-0.52, 0.0), vel=(0.3, 0.0), restitution=1.0)
    b = sb.circle(0.5, (0.52, 0.0), vel=(-0.3, 0.0), restitution=1.0)
    o, _ = run(sb, params(gravity_y=0.0, alpha=0.0, beta=0.0))
    o.step(zeros_actions(10, 1, CAPS))
    v = o.state()["vel"].reshape(-1, 2)
    assert v[a, 0] == pytest.approx(0.0, abs=1e-12) and v[b, 0] == pytest.approx(0.0, abs=1e-12)


def test_off_centre_hit_conserves_linear_and_angular_momentum():
    sb = SceneBuilder(CAPS)
    a = sb.box(0.5, 0.2, (0.0, 0.0), theta=0.3, vel=(0.0, 0.0), restitution=0.4)
    b = sb.circle(0.2, (0.3, 0.8), vel=(0.2, -3.0), restitution=0.6)
    o, sc = run(sb, params(gravity_y=0.0, alpha=0.0, beta=0.0))

    def momenta(st):
        m = 1 / sc["inv_mass"][0, [a, b]]
        I = 1 / sc["inv_inertia"][0, [a, b]]
        pos = st["pos"].reshape(-1, 2)[[a, b]]
        v = st["vel"].reshape(-1, 2)[[a, b]]
        w = st["omega"][0, [a, b]]
        L = (m * (pos[:, 0] * v[:, 1] - pos[:, 1] * v[:, 0]) + I * w).sum()
        return (m[:, None] * v).sum(0), L

    p0, L0 = momenta(o.state())
    o.step(zeros_actions(30, 1, CAPS))
    p1, L1 = momenta(o.state())
    assert abs(o.state()["omega"][0, a]) > 1e-3          # the box was set spinning: a contact happened
    assert np.allclose(p0, p1, atol=1e-12) and L1 == pytest.approx(L0, abs=1e-12)


# ------------------------------------------------------------------ resting contact (A.3.4, A.3.7, A.7)
@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_box_rests_on_floor(dtype):
    sb = SceneBuilder(CAPS)
    f = sb.box(5.0, 0.1, (0.0, 0.0), static=True)
    b = sb.box(0.4, 0.3, (0.5, 0.1 + 0.3 + 0.2), theta=0.0)
    p = params(n_substeps=2, n_iters=8)
    o, _ = run(sb, p, dtype=dtype, f32_inputs=True)
    o.step(zeros_actions(120, 1, CAPS))         # fall 0.2 and settle
    N = CAPS[0] + CAPS[1]
    ys = []
    for _ in range(200):
        o.step(zeros_actions(1, 1, CAPS))
        st = o.state()
        ys.append(st["pos"].reshape(-1, 2)[b, 1])
        assert np.abs(st["vel"].reshape(-1, 2)[b]).max() < 1e-3 and abs(st["omega"][0, b]) < 1e-3
        assert st["pair_count"][0, pair_index(f, b, N)] == 2
    assert np.abs(np.diff(ys)).max() < 1e-4
    # it rests on the floor top (y = 0.1) within the slop
    assert 0.1 + 0.3 - 2 * p["slop"] < ys[-1] < 0.1 + 0.3 + 1e-6


def test_stack_of_boxes_settles():
    """A.7's example: a stack needs several sweeps and warm starting, and then stays put."""
    caps = (4, 0, 0, 0)
    sb = SceneBuilder(caps)
    sb.box(5.0, 0.1, (0.0, 0.0), static=True)
    for k in range(3):
        sb.box(0.4, 0.2, (0.0, 0.1 + 0.2 + 0.4 * k + 0.01 * (k + 1)))
    o, _ = run(sb, params(n_substeps=3, n_iters=10), caps=caps, dtype="f32", f32_inputs=True)
    o.step(zeros_actions(300, 1, caps))
    y0 = o.state()["pos"].reshape(-1, 2)[:, 1].copy()
    o.step(zeros_actions(100, 1, caps))
    st = o.state()
    assert np.abs(st["pos"].reshape(-1, 2)[:, 1] - y0).max() < 2e-3
    assert np.abs(st["vel"]).max() < 5e-3 and np.abs(st["omega"]).max() < 5e-3


# ------------------------------------------------------------------ friction (A.3.6)
def test_sliding_box_decelerates_at_mu_g_and_stops():
    """mu = sqrt(mu_a^2 + mu_b^2); a box sliding on the floor loses speed at mu*g, stops, never reverses."""
    sb = SceneBuilder(CAPS)
    sb.box(50.0, 0.1, (0.0, 0.0), static=True, friction=0.3)
    b = sb.box(0.5, 0.1, (0.0, 0.1 + 0.1 - 0.004), vel=(3.0, 0.0), friction=0.4)
    p = params(n_substeps=2, n_iters=10)
    o, _ = run(sb, p)
    mu, g = np.hypot(0.3, 0.4), -p["gravity_y"]
    vx = [3.0]
    for _ in range(90):
        o.step(zeros_actions(1, 1, CAPS))
        vx.append(o.state()["vel"].reshape(-1, 2)[b, 0])
    vx = np.array(vx)
    sliding = vx > 0.3
    dec = -np.diff(vx)[sliding[1:]] / p["dt"]
    assert np.allclose(dec[3:], mu * g, rtol=0.02)
    assert vx.min() > -1e-6                     # never reverses
    assert abs(vx[-1]) < 1e-4                   # 3 / (0.5*9.81) = 0.61 s < 1.5 s


def test_box_on_slope_sticks_iff_tan_below_mu():
    for mu_each, angle, sticks in [(0.5, 0.45, True), (0.2, 0.45, False)]:
        sb = SceneBuilder(CAPS)
        c, s = np.cos(angle), np.sin(angle)
        sb.box(20.0, 0.1, (0.0, 0.0), theta=angle, static=True, friction=mu_each)
        # box centre sits 0.1 + 0.2 above the slope surface along its normal (-s, c)
        pos = np.array([-s, c]) * (0.1 + 0.2 - 0.004)
        b = sb.box(0.4, 0.2, pos, theta=angle, friction=mu_each)
        o, _ = run(sb, params(n_substeps=2, n_iters=10))
        o.step(zeros_actions(120, 1, CAPS))
        moved = np.linalg.norm(o.state()["pos"].reshape(-1, 2)[b] - pos)
        mu = np.hypot(mu_each, mu_each)
        assert (np.tan(angle) < mu) == sticks
        assert (moved < 0.02) if sticks else (moved > 0.5)


# ------------------------------------------------------------------ energy
def _energy_trace(o, sc, g, n):
    es = [energy(sc, o.state(), g)[0]]
    for _ in range(n):
        o.step(zeros_actions(1, o.n_envs, (o.P, o.C, o.J, o.T)))
        es.append(energy(sc, o.state(), g)[0])
    return np.array(es)


def _energy_run(warm_start, n_envs=32, n=150):
    caps, _, sc = scenegen.make_scene(0, n_envs=n_envs)
    sc["joint_motor_on"][:] = 0
    sc["thruster_active"][:] = 0
    p = params(n_iters=10, alpha=0.0, beta=0.0, gamma=0.0, joint_alpha=0.0, joint_beta=0.0, slop=0.0,
               warm_start=warm_start)
    o = Oracle(caps, n_envs, p, "f64")
    o.load_scene(sc)
    E = [energy(sc, o.state(), p["gravity_y"])]
    for _ in range(n):
        o.step(np.zeros((1, n_envs, caps[2] + caps[3])))
        E.append(energy(sc, o.state(), p["gravity_y"]))
    assert (o.state()["pair_count"].sum() > 0)      # something did collide
    return np.array(E)


def test_energy_never_increases_without_actuation_or_corrections():
    """No motors or thrusters, alpha = beta = gamma = 0, e <= 1, impulses solved from zero every step:
    kinetic + potential energy is non-increasing from step to step (the corrections add energy --
    A.3.7 -- hence switched off)."""
    E = _energy_run(warm_start=0)
    scale = np.abs(E).max(0) + 1.0
    assert (np.diff(E, axis=0) / scale < 1e-5).all()


def test_energy_with_warm_starting_stays_below_its_initial_value():
    """Warm starting re-applies last step's impulses at this step's manifold, which can hand back a
    little energy on single steps; it never exceeds what the scene started with and such steps are rare."""
    E = _energy_run(warm_start=1)
    scale = np.abs(E).max(0) + 1.0
    assert ((E - E[0]) / scale < 1e-9).all()
    d = np.diff(E, axis=0) / scale
    assert (d > 1e-5).mean() < 0.03 and d.max() < 0.05


# ------------------------------------------------------------------ joints (A.4)
def _pendulum(length, theta0, dtype="f64", **kw):
    caps = (2, 1, 1, 0)
    sb = SceneBuilder(caps)
    a = sb.box(0.2, 0.2, (0.0, 0.0), static=True)
    pos = (length * np.sin(theta0), -length * np.cos(theta0))
    b = sb.circle(0.1, pos)
    sb.joint(a, b, (0.0, 0.0))
    p = params(**kw)
    o, sc = run(sb, p, caps=caps, dtype=dtype, f32_inputs=(dtype == "f32"))
    return o, sc, a, b, caps, p


def test_pendulum_anchor_drift_bounded_and_period():
    L, th0 = 1.0, 0.1
    o, sc, a, b, caps, p = _pendulum(L, th0, n_substeps=2, n_iters=8)
    xs, drift = [], []
    for _ in range(1000):
        o.step(zeros_actions(1, 1, caps))
        st = o.state()
        pb, thb = st["pos"].reshape(-1, 2)[b], st["theta"][0, b]
        anc = sc["joint_anchor_b"][0, 0]
        world = pb + np.array([np.cos(thb) * anc[0] - np.sin(thb) * anc[1], np.sin(thb) * anc[0] + np.cos(thb) * anc[1]])
        drift.append(np.linalg.norm(world))
        xs.append(pb[0])
    assert max(drift) < 1e-2
    xs = np.array(xs)
    # period from zero crossings of x(t); physical pendulum: T = 2 pi sqrt(I_pivot / (m g d))
    up = np.nonzero((xs[:-1] < 0) & (xs[1:] >= 0))[0]
    T_meas = np.mean(np.diff(up)) * p["dt"]
    m, Icom = 1 / sc["inv_mass"][0, b], 1 / sc["inv_inertia"][0, b]
    T_true = 2 * np.pi * np.sqrt((Icom + m * L * L) / (m * 9.81 * L))
    assert T_meas == pytest.approx(T_true, rel=0.03)
    # the amplitude does not grow
    assert np.abs(xs[-200:]).max() <= np.abs(xs[:200]).max() * 1.02


def test_fixed_joint_pair_falls_like_one_body_and_keeps_angle():
    caps = (2, 1, 1, 0)
    sb = SceneBuilder(caps)
    a = sb.box(0.3, 0.2, (0.0, 10.0), theta=0.4, omega=0.0)
    b = sb.box(0.2, 0.2, (0.5, 10.0), theta=-0.2)
    sb.joint(a, b, (0.3, 10.0), fixed=True)
    p = params(n_substeps=2, n_iters=8)
    o, sc = run(sb, p, caps=caps)
    n = 60
    m = 1 / sc["inv_mass"][0, [a, b]]
    com0 = (m[:, None] * sc["pos"][0, [a, b]]).sum(0) / m.sum()
    o.step(zeros_actions(n, 1, caps))
    st = o.state()
    com = (m[:, None] * st["pos"].reshape(-1, 2)[[a, b]]).sum(0) / m.sum()
    h, k = p["dt"] / 2, n * 2
    assert com[0] == pytest.approx(com0[0], abs=1e-9)
    assert com[1] == pytest.approx(com0[1] + p["gravity_y"] * h * h * k * (k + 1) / 2, abs=1e-6)
    rel = st["theta"][0, a] - st["theta"][0, b]
    assert rel == pytest.approx(0.6, abs=1e-6)
    assert abs(st["omega"][0, a]) < 1e-6        # no net torque: the pair does not start to spin


def test_fixed_joint_holds_a_cantilever():
    """A box fixed to a static wall stays put under gravity; the relative angle error stays bounded."""
    caps = (2, 1, 1, 0)
    sb = SceneBuilder(caps)
    a = sb.box(0.2, 1.0, (0.0, 0.0), static=True)
    b = sb.box(0.5, 0.1, (0.7, 0.0))
    sb.joint(a, b, (0.2, 0.0), fixed=True)
    o, sc = run(sb, params(n_substeps=2, n_iters=8), caps=caps)
    worst = 0.0
    for _ in range(300):
        o.step(zeros_actions(1, 1, caps))
        worst = max(worst, abs(o.state()["theta"][0, b]))
    assert worst < 0.02
    assert np.linalg.norm(o.state()["pos"].reshape(-1, 2)[b] - (0.7, 0.0)) < 0.02


def test_joined_shapes_do_not_collide():
    caps = (2, 1, 1, 0)
    sb = SceneBuilder(caps)
    a = sb.box(0.5, 0.5, (0.0, 0.0))
    b = sb.box(0.5, 0.5, (0.3, 0.0))          # deeply overlapping
    sb.joint(a, b, (0.15, 0.0))
    o, _ = run(sb, params(gravity_y=0.0), caps=caps)
    o.step(zeros_actions(5, 1, caps))
    st = o.state()
    assert st["pair_count"].sum() == 0 and o.get("pair_eligible")[0, pair_index(a, b, 3)] == 0
    assert np.allclose(st["vel"], 0)
    # the same two boxes without the joint do collide
    sb.sc["joint_active"][:] = 0
    o, _ = run(sb, params(gravity_y=0.0), caps=caps)
    o.step(zeros_actions(1, 1, caps))
    assert o.state()["pair_count"][0, pair_index(a, b, 3)] > 0


# ------------------------------------------------------------------ motors (A.5), thrusters (A.6)
def test_motor_drives_relative_speed_to_target_and_conserves_angular_momentum():
    caps = (2, 1, 1, 0)
    sb = SceneBuilder(caps)
    a = sb.box(0.4, 0.4, (0.0, 0.0))
    b = sb.box(0.3, 0.3, (0.0, 0.0))
    sb.joint(a, b, (0.0, 0.0), motor_on=True, speed=3.0, power=0.05)
    p = params(gravity_y=0.0, rho=1.0)
    o, sc = run(sb, p, caps=caps)
    Ia, Ib = 1 / sc["inv_inertia"][0, a], 1 / sc["inv_inertia"][0, b]
    act = np.full((1, 1, 1), 0.5)
    target, gap = 3.0 * 0.5, []
    for _ in range(400):
        o.step(act)
        w = o.state()["omega"][0]
        gap.append(w[a] - w[b] - target)
        assert Ia * w[a] + Ib * w[b] == pytest.approx(0.0, abs=1e-12)
    gap = np.array(gap)
    assert gap[0] < 0 and (np.diff(np.abs(gap)) <= 1e-12).all() and abs(gap[-1]) < 1e-3
    # first step: the printed law, as a torque held for one substep, from rest
    o, _ = run(sb, p, caps=caps)
    o.step(act)
    jr = 0.05 * np.tanh((0.0 - 0.0 - 3.0 * 0.5) * 1.0) * p["dt"]
    w = o.state()["omega"][0]
    assert w[a] == pytest.approx(-jr / Ia, rel=1e-12) and w[b] == pytest.approx(jr / Ib, rel=1e-12)


def test_all_motors_see_the_velocities_from_before_any_motor():
    """A.8: motors are applied in parallel.  Three shapes in a chain, a motor in either joint, no sweeps (so that
    nothing but the motors acts): the middle shape receives both impulses, and each is the tanh law of the angular
    velocities the substep started with -- not of what the other motor left."""
    caps = (3, 1, 2, 0)
    sb = SceneBuilder(caps)
    a = sb.box(0.4, 0.4, (0.0, 0.0), omega=1.0)
    b = sb.box(0.3, 0.3, (0.0, 0.0), omega=0.25)
    c = sb.box(0.2, 0.5, (0.0, 0.0), omega=-2.0)
    sb.joint(a, b, (0.0, 0.0), motor_on=True, speed=3.0, power=0.05)
    sb.joint(b, c, (0.0, 0.0), motor_on=True, speed=2.0, power=0.08)
    p = params(gravity_y=0.0, rho=0.7, n_iters=0, warm_start=0, joint_beta=0.0)
    o, sc = run(sb, p, caps=caps)
    act = np.array([[[0.5, -0.25]]])
    o.step(act)
    ii = sc["inv_inertia"][0]
    m1 = 0.05 * np.tanh((1.0 - 0.25 - 3.0 * 0.5) * 0.7) * p["dt"]
    m2 = 0.08 * np.tanh((0.25 + 2.0 - 2.0 * -0.25) * 0.7) * p["dt"]
    w = o.state()["omega"][0]
    assert w[a] == pytest.approx(1.0 - ii[a] * m1, rel=1e-13)
    assert w[b] == pytest.approx(0.25 + ii[b] * m1 - ii[b] * m2, rel=1e-13)
    assert w[c] == pytest.approx(-2.0 + ii[c] * m2, rel=1e-13)
    m2_seq = 0.08 * np.tanh((0.25 + ii[b] * m1 + 2.0 - 2.0 * -0.25) * 0.7) * p["dt"]
    assert abs(m2_seq - m2) > 1e-6 * abs(m2)                 # the other reading would show


def test_motor_off_or_fixed_joint_ignores_action():
    caps = (2, 1, 1, 0)
    for kw in (dict(motor_on=False), dict(motor_on=True, fixed=True)):
        sb = SceneBuilder(caps)
        a = sb.box(0.4, 0.4, (0.0, 0.0))
        b = sb.box(0.3, 0.3, (0.0, 0.0))
        sb.joint(a, b, (0.0, 0.0), speed=3.0, power=1.0, **kw)
        o, _ = run(sb, params(gravity_y=0.0), caps=caps)
        o.step(np.ones((5, 1, 1)))
        assert np.allclose(o.state()["omega"], 0, atol=1e-14)


def test_thruster_closed_form():
    """Force p*A along the (rotated) thruster direction at its mount point, held for dt: from rest,
    dv = F/m * t and dw = (r x F)/I * t while the body has not yet rotated (one step)."""
    caps = (1, 1, 0, 1)
    sb = SceneBuilder(caps)
    b = sb.box(0.5, 0.25, (0.0, 0.0), theta=0.3)
    sb.thruster(b, (0.4, -0.1), angle=0.5, power=2.0)
    p = params(gravity_y=0.0)
    o, sc = run(sb, p, caps=caps)
    A = 0.7
    o.step(np.full((1, 1, 1), A))
    st = o.state()
    th = 0.3
    d = np.array([np.cos(th + 0.5), np.sin(th + 0.5)])
    r = np.array([np.cos(th) * 0.4 + np.sin(th) * 0.1, np.sin(th) * 0.4 - np.cos(th) * 0.1])
    J = 2.0 * A * p["dt"] * d
    assert np.allclose(st["vel"].reshape(-1, 2)[b], J * sc["inv_mass"][0, b], rtol=1e-12)
    assert st["omega"][0, b] == pytest.approx((r[0] * J[1] - r[1] * J[0]) * sc["inv_inertia"][0, b], rel=1e-12)
    # clip option: negative actions give nothing
    o, _ = run(sb, params(gravity_y=0.0, clip_thruster_01=1), caps=caps)
    o.step(np.full((1, 1, 1), -0.7))
    assert np.all(o.state()["vel"] == 0)
    # a thruster through the centre of mass pushes a free body along a straight line: v = F t / m
    sb = SceneBuilder(caps)
    b = sb.circle(0.3, (0.0, 0.0))
    sb.thruster(b, (0.0, 0.0), angle=0.0, power=3.0)
    o, sc = run(sb, p, caps=caps)
    o.step(np.ones((30, 1, 1)))
    assert o.state()["vel"].reshape(-1, 2)[b, 0] == pytest.approx(3.0 * 30 * p["dt"] * sc["inv_mass"][0, b], rel=1e-12)


# ------------------------------------------------------------------ warm starting (A.7)
def test_warm_start_bookkeeping():
    sb = SceneBuilder(CAPS)
    f = sb.box(5.0, 0.1, (0.0, 0.0), static=True)
    c = sb.circle(0.3, (0.0, 0.1 + 0.3 + 0.05))
    N = CAPS[0] + CAPS[1]
    q = pair_index(f, c, N)
    o, sc = run(sb, params(n_iters=6))
    lam_prev, touched = None, False
    for step in range(40):
        o.step(zeros_actions(1, 1, CAPS))
        st = o.state()
        lam = st["lambda_n"][0, 2 * q]
        if st["pair_count"][0, q] == 0:
            assert lam == 0 and st["prev_active"][0, 2 * q] == 0     # nothing accumulated while apart
        else:
            assert st["prev_active"][0, 2 * q] == 1 and lam > 0
            touched = True
        lam_prev = lam
    assert touched
    # resting: accumulated impulse per step ~ m g dt (the first guess carried from step to step)
    m = 1 / sc["inv_mass"][0, c]
    assert lam_prev == pytest.approx(m * 9.81 / 60.0, rel=0.05)
    # lift the circle off: the accumulators of the pair are wiped at the next step
    o.set("pos", np.where(np.arange(2 * N) == 2 * c + 1, 3.0, st["pos"]))
    o.step(zeros_actions(1, 1, CAPS))
    st = o.state()
    assert st["lambda_n"][0, 2 * q] == 0 and st["lambda_t"][0, 2 * q] == 0 and st["prev_active"][0, 2 * q] == 0


def test_a_collision_is_active_only_with_positive_penetration_and_adjacency_is_symmetric():
    """Table 2: a manifold point is an active collision iff its penetration is positive.  Two circles half a
    millimetre apart do not collide (no count, no adjacency, no impulse); half a millimetre into each other they
    do, and each shape's adjacency word names the other."""
    N = CAPS[0] + CAPS[1]
    for gap, touching in ((5e-4, False), (-5e-4, True)):
        sb = SceneBuilder(CAPS)
        a = sb.circle(0.5, (0.0, 0.0), vel=(0.5, 0.0))
        b = sb.circle(0.5, (1.0 + gap, 0.0), vel=(0.5, 0.0))
        o, _ = run(sb, params(gravity_y=0.0, alpha=0.0, beta=0.0, slop=0.0))
        o.step(zeros_actions(1, 1, CAPS))
        count = o.get("pair_count")[0, pair_index(a, b, N)]
        adj = o.get("shape_adj")[0].astype(np.int64)
        assert count == (1 if touching else 0)
        assert ((adj[a] >> b) & 1) == int(touching) and ((adj[b] >> a) & 1) == int(touching)
        assert [int(x) for x in adj if x] == ([1 << b, 1 << a] if touching else [])
        assert np.array_equal(o.state()["vel"].reshape(-1, 2)[[a, b]], [[0.5, 0.0], [0.5, 0.0]])


def test_joint_accumulators_without_warm_starting_hold_one_substep_only():
    """A.7 off: nothing is carried over, so after any number of steps the accumulated impulse of a joint that holds
    a hanging weight is the impulse of one substep, m g h -- not the sum over the substeps so far."""
    caps = (1, 1, 1, 0)
    sb = SceneBuilder(caps)
    top = sb.box(0.5, 0.1, (0.0, 2.0), static=True)
    bob = sb.circle(0.2, (0.0, 1.0))
    sb.joint(top, bob, (0.0, 2.0))
    p = params(n_substeps=2, n_iters=10, warm_start=0)
    o, sc = run(sb, p, caps=caps)
    o.step(zeros_actions(30, 1, caps))
    m = 1 / sc["inv_mass"][0, bob]
    acc = o.state()["joint_acc"][0, :2]
    assert abs(acc[1]) == pytest.approx(m * 9.81 * p["dt"] / 2, rel=0.05) and abs(acc[0]) < 1e-6


def test_warm_start_off_and_on_reach_the_same_rest_but_on_is_faster():
    res = {}
    for ws in (0, 1):
        caps = (4, 0, 0, 0)
        sb = SceneBuilder(caps)
        sb.box(5.0, 0.1, (0.0, 0.0), static=True)
        for k in range(3):
            sb.box(0.4, 0.2, (0.0, 0.1 + 0.2 + 0.4 * k))
        o, _ = run(sb, params(n_iters=3, warm_start=ws), caps=caps)
        o.step(zeros_actions(200, 1, caps))
        res[ws] = np.abs(o.state()["vel"]).max()
    assert res[1] < 1e-3 and res[1] <= res[0]


# ------------------------------------------------------------------ order of the sweep (A.8)
@pytest.mark.parametrize("N", [7, 9, 16])
def test_schedule_is_a_round_robin(N):
    a, b, r = ko.schedule(N)
    assert len(a) == N * (N - 1) // 2
    assert len({(int(x), int(y)) for x, y in zip(a, b)}) == len(a) and (a < b).all()
    for rr in np.unique(r):
        used = np.concatenate([a[r == rr], b[r == rr]])
        assert len(set(used.tolist())) == len(used)          # body-disjoint inside a round
    assert (np.diff(r) >= 0).all()


def _movable(st_or_sc, e, i):
    return st_or_sc["active"][e, i] > 0 and (st_or_sc["inv_mass"][e, i] != 0 or st_or_sc["inv_inertia"][e, i] != 0)


def _visiting_order(N, colliding, movable):
    """Written out here a second time, from the rule: walk the colliding pairs in tournament order, give each the
    lowest level no earlier colliding pair sharing a movable shape with it has taken.  Returns {(a, b): level} and
    {(a, b): dependency level} (one past the last earlier pair sharing a movable shape), for comparison."""
    a, b, r = ko.schedule(N)
    taken, last, level, dep = {}, {}, {}, {}
    for x, y, rr in zip(a.tolist(), b.tolist(), r.tolist()):
        if (x, y) not in colliding:
            continue
        ends = [s for s in (x, y) if movable(s)]
        busy = set().union(*[taken.get(s, set()) for s in ends]) if ends else set()
        lv = next(c for c in range(64) if c not in busy)
        d = max([last.get(s, 0) for s in ends], default=0)
        for s in ends:
            taken.setdefault(s, set()).add(lv)
            last[s] = d + 1
        level[(x, y)], dep[(x, y)] = lv, d
        assert lv <= d <= rr
    return level, dep


@pytest.mark.parametrize("workload", ["config 3", "dense pile", "towers"])
def test_visiting_order_is_the_lowest_free_level_walk_of_the_tournament_order(workload):
    """The level-after-level order of the sweep (sweep_order = 1; A.8 leaves the order to the engine): the oracle's
    levels equal the ones worked out here from the colliding set alone; pairs of one level share no movable shape; a
    level is never later than the place the pair would have one past its last conflicting predecessor, and on
    piles it is often earlier."""
    n = 16
    if workload == "config 3":
        caps, p, sc = scenegen.make_scene(3, n_envs=n)
        act = scenegen.make_actions(3, 60, n)
    elif workload == "dense pile":
        caps, p, sc = scenegen.make_dense_scene(n_envs=n)
        act = scenegen.make_actions(3, 120, n)
    else:
        caps, p, sc = scenegen.make_stack_scene(n_envs=n)
        act = np.zeros((20, n, caps[2] + caps[3]))
    N = caps[0] + caps[1]
    o = Oracle(caps, n, dict(p, sweep_order=1), "f32")
    o.load_scene(sc)
    o.step(act)
    colour = o.get("pair_level").reshape(n, -1)
    active = o.get("pair_active").reshape(n, -1, 2).any(-1)
    earlier = 0
    for e in range(n):
        colliding = {(i, j) for i in range(N) for j in range(i + 1, N) if active[e, pair_index(i, j, N)]}
        level, dep = _visiting_order(N, colliding, lambda i: _movable(sc, e, i))
        for i in range(N):
            for j in range(i + 1, N):
                assert colour[e, pair_index(i, j, N)] == level.get((i, j), -1), (e, i, j)
        for lv in set(level.values()):
            ends = [s for pr, l in level.items() if l == lv for s in pr if _movable(sc, e, s)]
            assert len(ends) == len(set(ends))
        earlier += sum(level[pr] < dep[pr] for pr in level)
    assert active.sum() > 3 * n
    if workload != "config 3":
        assert earlier > 0


def test_sweep_visits_the_levels_in_order_closed_form():
    """Four equal frictionless balls in a row, no gravity, no restitution, one sweep: a colliding pair that
    approaches ends at the mean of its two velocities.  The outcome depends on the order of the three contacts;
    under sweep_order = 1 the oracle's equals the one worked out here for the level-by-level order (the outer
    contacts, then the middle one), under sweep_order = 0 the one for the tournament order."""
    caps = (1, 4, 1, 1)
    N, r, pen = 5, 0.5, 1e-4
    a, b, _ = ko.schedule(N)
    place = None
    for perm in ((1, 2, 3, 4), (1, 3, 2, 4), (2, 1, 4, 3), (1, 2, 4, 3), (3, 1, 2, 4), (1, 4, 2, 3)):
        contacts = {tuple(sorted((perm[q], perm[q + 1]))) for q in range(3)}
        walk = [(x, y) for x, y in zip(a.tolist(), b.tolist()) if (x, y) in contacts]
        if set(walk[1]) & set(perm[1:3]) == set(perm[1:3]):    # the middle contact is walked second
            place = perm
            break
    assert place is not None
    v0 = {place[0]: 1.0, place[1]: 0.0, place[2]: 0.0, place[3]: -1.0}

    def expected(order):
        v = dict(v0)
        x_of = {s: q for q, s in enumerate(place)}
        for x, y in order:
            lo, hi = (x, y) if x_of[x] < x_of[y] else (y, x)
            if v[lo] > v[hi]:
                v[lo] = v[hi] = 0.5 * (v[lo] + v[hi])
        return v

    level, _ = _visiting_order(N, contacts, lambda i: True)
    by_level = sorted(walk, key=lambda pr: (level[pr], walk.index(pr)))
    assert by_level != walk and expected(by_level) != expected(walk)
    for sweep_order, order in ((1, by_level), (0, walk)):
        sb = SceneBuilder(caps)
        ids = {}
        for k in range(4):
            ids[k + 1] = sb.circle(r, (0.0, 0.0), friction=0.0)
        for q, s in enumerate(place):
            sb.sc["pos"][0, s] = (q * (2 * r - pen), 3.0)
            sb.sc["vel"][0, s] = (v0[s], 0.0)
        o, _ = run(sb, params(n_iters=1, gravity_y=0.0, warm_start=0, sweep_order=sweep_order), caps=caps)
        o.step(zeros_actions(1, 1, caps))
        vel = o.state()["vel"].reshape(-1, 2)
        want = expected(order)
        for s in place:
            assert vel[s, 0] == pytest.approx(want[s], abs=1e-12) and vel[s, 1] == 0.0


@pytest.mark.parametrize("sweep_order", [0, 1])
def test_group_at_once_equals_sequential_sweep(sweep_order):
    """Solving every pair of a round (tournament order) or of a level (level order) from the same snapshot
    gives bit-identical results to visiting them one after the other: the groups of both visiting orders are
    conflict-free."""
    caps, p, sc = scenegen.make_scene(3, n_envs=24)
    act = scenegen.make_actions(3, 40, 24)
    out = []
    for mode in (0, 1):
        o = Oracle(caps, 24, dict(p, order_mode=mode, sweep_order=sweep_order), "f32")
        o.load_scene(sc)
        o.step(act)
        out.append(o.state())
    assert out[0]["pair_count"].sum() > 24 * 3
    for k in ("pos", "theta", "vel", "omega", "lambda_n", "lambda_t", "joint_acc", "pair_count"):
        assert np.array_equal(out[0][k], out[1][k]), k


def test_the_two_visiting_orders_differ_in_bits_and_agree_in_behaviour():
    """Tournament order and level order are two sequential sweeps: different bits on a pile, the same physics --
    the towers of boxes stand under both (millimetres of drift, the same settling)."""
    caps, prm, sc = scenegen.make_stack_scene(n_envs=24)
    act = np.zeros((256, 24, caps[2] + caps[3]))
    p0 = np.asarray(sc["pos"])[:, 3:12]
    res = []
    for so in (0, 1):
        o = Oracle(caps, 24, dict(prm, sweep_order=so), "f32")
        o.load_scene(sc)
        o.step(act, n_threads=4)
        st = o.state()
        pos = st["pos"].reshape(24, -1, 2)[:, 3:12]
        res.append((st["pos"].copy(), np.abs(pos[..., 0] - p0[..., 0]).max(), (p0[..., 1] - pos[..., 1]).max(),
                    np.abs(st["vel"]).max(), o.get("levels_sum")[:, 0].mean() / (256 * prm["n_substeps"])))
    assert not np.array_equal(res[0][0], res[1][0])
    for _, dx, dy, v, _ in res:
        assert dx < 0.01 and 0.0 < dy < 0.03 and v < 0.02
    assert abs(res[0][2] - res[1][2]) < 2e-3
    assert res[1][4] <= 3.0          # a tower's contacts alternate between two levels, its foot takes a third


def test_deterministic_and_thread_count_invariant():
    caps, p, sc = scenegen.make_scene(2, n_envs=32)
    act = scenegen.make_actions(2, 8, 32)
    out = []
    for nt in (1, 1, 4):
        o = Oracle(caps, 32, p, "f32")
        o.load_scene(sc)
        o.step(act, n_threads=nt)
        out.append(o.state())
    for k in out[0]:
        assert np.array_equal(out[0][k], out[1][k]) and np.array_equal(out[0][k], out[2][k]), k


def test_table4_capacities_match_the_paper():
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table4_capacities.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, s, m, l = line.split()
                rows[k] = (int(s), int(m), int(l))
    for col, size in enumerate("SML"):
        assert scenegen.CAPS[size] == tuple(rows[k][col] for k in ("polygons", "circles", "joints", "thrusters"))


# ------------------------------------------------------------------ joint limits (A.4.3)
def _limited_pair(theta_a, omega_a, omega_b, limits, motor=None, gamma=None, n_iters=1):
    """Two free boxes hinged at their common centre of mass (the point constraint then carries no torque),
    no gravity: only the limit acts on the relative rotation theta_a - theta_b."""
    caps = (2, 1, 1, 0)
    sb = SceneBuilder(caps)
    a = sb.box(0.4, 0.4, (0.0, 0.0), theta=theta_a, omega=omega_a)
    b = sb.box(0.3, 0.3, (0.0, 0.0), omega=omega_b)
    kw = dict(motor_on=True, speed=motor[0], power=motor[1]) if motor else {}
    sb.joint(a, b, (0.0, 0.0), limits=limits, **kw)
    kw = dict(gravity_y=0.0, n_iters=n_iters)
    if gamma is not None:
        kw["gamma"] = gamma
    p = params(**kw)
    o, sc = run(sb, p, caps=caps)
    return o, sc, p, a, b


def test_joint_limit_closed_form_beyond_the_upper_limit():
    """Beyond the limit and still moving outwards: one visit leaves w_a - w_b = -gamma * excess (the fixed
    joint's angular impulse with the excess in the place of the angle error); angular momentum is kept."""
    o, sc, p, a, b = _limited_pair(0.6, 1.0, -0.5, (-0.5, 0.5))
    Ia, Ib = 1 / sc["inv_inertia"][0, a], 1 / sc["inv_inertia"][0, b]
    o.step(np.zeros((1, 1, 1)))
    w = o.state()["omega"][0]
    assert w[a] - w[b] == pytest.approx(-p["gamma"] * 0.1, rel=1e-9)
    assert Ia * w[a] + Ib * w[b] == pytest.approx(Ia * 1.0 - Ib * 0.5, rel=1e-12)
    # the impulse itself: j_r = (w_rel + gamma*excess) / (1/I_a + 1/I_b), taken from a, given to b
    jr = (1.5 + p["gamma"] * 0.1) / (1 / Ia + 1 / Ib)
    assert w[a] == pytest.approx(1.0 - jr / Ia, rel=1e-9) and w[b] == pytest.approx(-0.5 + jr / Ib, rel=1e-9)


def test_joint_limit_mirror_symmetry_lower_limit():
    o1, _, _, a, b = _limited_pair(0.6, 1.0, -0.5, (-0.5, 0.5))
    o2, _, _, _, _ = _limited_pair(-0.6, -1.0, 0.5, (-0.5, 0.5))
    o1.step(np.zeros((3, 1, 1))); o2.step(np.zeros((3, 1, 1)))
    s1, s2 = o1.state(), o2.state()
    assert np.allclose(s1["omega"], -s2["omega"], rtol=1e-12, atol=0)
    assert np.allclose(s1["theta"], -s2["theta"], rtol=1e-12, atol=0)


def test_joint_limit_leaves_restoring_motion_and_in_range_motion_alone():
    # beyond the limit but already coming back: nothing is applied, however slowly it returns
    o, _, _, a, b = _limited_pair(0.6, -0.01, 0.0, (-0.5, 0.5))
    o.step(np.zeros((1, 1, 1)))
    w = o.state()["omega"][0]
    assert w[a] == -0.01 and w[b] == 0.0
    # within the limits: free rotation whatever the speed
    o, _, _, a, b = _limited_pair(0.2, 3.0, -1.0, (-0.5, 0.5))
    o.step(np.zeros((1, 1, 1)))
    w = o.state()["omega"][0]
    assert w[a] == 3.0 and w[b] == -1.0
    # a fixed joint ignores the limit fields, an unlimited joint too
    caps = (2, 1, 1, 0)
    sb = SceneBuilder(caps)
    a = sb.box(0.4, 0.4, (0.0, 0.0), theta=0.6, omega=1.0)
    b = sb.box(0.3, 0.3, (0.0, 0.0))
    sb.joint(a, b, (0.0, 0.0))
    o, _ = run(sb, params(gravity_y=0.0), caps=caps)
    o.step(np.zeros((1, 1, 1)))
    assert o.state()["omega"][0, a] == 1.0


def test_joint_limit_motor_returns_faster_than_the_correction():
    """A.4.3: the correction is withheld while the shapes are already returning, so a motor may bring them
    back faster than gamma * excess would."""
    g = 2.0
    o, sc, p, a, b = _limited_pair(0.6, 0.0, 0.0, (-0.5, 0.5), motor=(4.0, 0.2), gamma=g, n_iters=4)
    act = np.full((1, 1, 1), -1.0)          # motor target w_a - w_b = -4: back towards the range
    o.step(act)
    w = o.state()["omega"][0]
    rel1 = w[a] - w[b]
    assert rel1 < -g * 0.1                  # faster than the correction speed, and not slowed down to it
    # without the motor the same start gives exactly the correction speed
    o2, _, _, _, _ = _limited_pair(0.6, 0.0, 0.0, (-0.5, 0.5), gamma=g, n_iters=4)
    o2.step(np.zeros((1, 1, 1)))
    w2 = o2.state()["omega"][0]
    assert w2[a] - w2[b] == pytest.approx(-g * 0.1, rel=1e-9)


def test_limited_pendulum_stays_within_its_range():
    """A bar hinged to a static block swings under gravity against a limit: the relative rotation never
    leaves [lo, hi] by more than a small overshoot, and comes to rest at the limit."""
    caps = (2, 1, 1, 0)
    sb = SceneBuilder(caps)
    top = sb.box(0.2, 0.2, (0.0, 2.0), static=True)
    bar = sb.box(0.5, 0.05, (0.5, 2.0))                     # horizontal, hinged at its left end
    sb.joint(top, bar, (0.0, 2.0), limits=(-0.1, 0.6))       # theta_top - theta_bar: the bar may drop 0.6 rad
    p = params(n_substeps=2, n_iters=8)
    o, sc = run(sb, p, caps=caps)
    rel = []
    for _ in range(600):
        o.step(np.zeros((1, 1, 1)))
        th = o.state()["theta"][0]
        rel.append(th[top] - th[bar])
    rel = np.array(rel)
    assert rel.max() < 0.6 + 0.05 and rel.min() > -0.1 - 0.05     # at most one substep of travel at impact speed
    assert rel.max() > 0.55                                  # it did reach the limit
    assert abs(rel[-1] - 0.6) < 0.02 and abs(o.state()["omega"][0, bar]) < 0.05
    # without the limit the same bar swings far past it
    sb2 = SceneBuilder(caps)
    top = sb2.box(0.2, 0.2, (0.0, 2.0), static=True)
    bar = sb2.box(0.5, 0.05, (0.5, 2.0))
    sb2.joint(top, bar, (0.0, 2.0))
    o2, _ = run(sb2, p, caps=caps)
    o2.step(np.zeros((60, 1, 1)))
    th = o2.state()["theta"][0]
    assert th[top] - th[bar] > 1.0


# ------------------------------------------------------------------ stacking (A.7)
def test_towers_of_boxes_stand_and_warm_starting_is_what_holds_them():
    """The stacking workload: up to nine boxes on top of each other.  With warm starting (A.7) the towers
    stand for 256 steps -- millimetres of sideways drift, a settling of the order of the slop per contact,
    velocities of millimetres per second; without it the same sweeps leave them sagging and jittering."""
    import scenegen
    caps, prm, sc = scenegen.make_stack_scene(n_envs=48)
    act = np.zeros((256, 48, caps[2] + caps[3]))
    p0 = np.asarray(sc["pos"])[:, 3:12]

    def settle(p):
        o, _ = run(sc, p, caps=caps, dtype="f32")
        o.step(act, n_threads=4)
        st = o.state()
        pos = st["pos"].reshape(48, -1, 2)[:, 3:12]
        return (np.abs(pos[..., 0] - p0[..., 0]).max(), (p0[..., 1] - pos[..., 1]).max(),
                np.abs(st["vel"]).max(), (st["pair_count"] > 0).sum(1))

    dx, dy, v, pairs = settle(prm)
    assert dx < 0.01 and 0.0 < dy < 0.03 and v < 0.02
    assert (pairs == 13).all()                       # 9 box contacts in the towers + 4 balls on the floor
    dx0, dy0, v0, _ = settle(dict(prm, warm_start=0))
    assert dy0 > 2 * dy and v0 > 5 * v


# ------------------------------------------------------------------ batched impulse resolution (A.8)
def _wedge(batch_size):
    """A frictionless ball touching both faces of a V of two static slabs, moving into the corner."""
    sb = SceneBuilder(CAPS)
    r, pen, hy, c = 0.5, 0.002, 0.3, np.array([0.2, 1.0])
    normals = []
    for phi in (np.deg2rad(30.0), np.deg2rad(-30.0)):
        n = np.array([-np.sin(phi), np.cos(phi)])
        sb.box(3.0, hy, tuple(c - (r - pen + hy) * n), theta=phi, static=True, friction=0.0)
        normals.append(n)
    ball = sb.circle(r, tuple(c), vel=(0.3, -0.4), friction=0.0)
    p = params(n_iters=1, gravity_y=-9.81, warm_start=0, batch_size=batch_size)
    o, sc = run(sb, p, f32_inputs=False)
    o.step(zeros_actions(1, 1, CAPS))
    st = o.state()
    v0 = np.array([0.3, -0.4 - 9.81 * p["dt"]])
    return st["vel"].reshape(-1, 2)[ball], v0, normals


def test_batched_resolution_closed_form_in_a_wedge():
    """Two active constraints on one body.  Solved one after the other (batch size 1) the second sees the
    velocity the first left; solved in one batch both see the starting velocity and their impulses add."""
    def project(v, n):
        return v - min(v @ n, 0.0) * n

    v_seq, v0, (n1, n2) = _wedge(1)
    v_ref, _, _ = _wedge(0)
    assert np.array_equal(v_seq, v_ref)
    orders = [project(project(v0, n1), n2), project(project(v0, n2), n1)]
    assert min(np.abs(v_seq - w).max() for w in orders) < 1e-12
    v_par, _, _ = _wedge(1000)
    jacobi = v0 - min(v0 @ n1, 0.0) * n1 - min(v0 @ n2, 0.0) * n2
    assert np.abs(v_par - jacobi).max() < 1e-12
    assert min(np.abs(jacobi - w).max() for w in orders) > 0.05     # the two answers are far apart


def test_batch_size_one_is_the_sequential_sweep():
    caps, p, sc = scenegen.make_scene(3, n_envs=16)
    act = scenegen.make_actions(3, 30, 16)
    out = []
    for B in (0, 1, 16):
        o = Oracle(caps, 16, dict(p, batch_size=B), "f32")
        o.load_scene(sc)
        o.step(act)
        out.append(o.state())
    assert out[0]["pair_count"].sum() > 16 * 3
    for k in ("pos", "theta", "vel", "omega", "lambda_n", "lambda_t", "joint_acc", "pair_count"):
        assert np.array_equal(out[0][k], out[1][k]), k
    assert not np.array_equal(out[0]["vel"], out[2]["vel"])


def test_batched_resolution_conserves_momentum():
    """Every impulse of a batch is applied to a and, reversed, to b: three bodies hitting each other at once,
    all points in one batch, keep their total linear and angular momentum."""
    sb = SceneBuilder(CAPS)
    ids = [sb.box(0.5, 0.2, (0.0, 0.0), theta=0.3, restitution=0.4),
           sb.circle(0.2, (0.3, 0.8), vel=(0.2, -3.0), restitution=0.6),
           sb.circle(0.25, (-0.35, -0.75), vel=(0.5, 2.5), restitution=0.2)]
    o, sc = run(sb, params(gravity_y=0.0, alpha=0.0, beta=0.0, batch_size=1000))

    def momenta(st):
        m = 1 / sc["inv_mass"][0, ids]
        I = 1 / sc["inv_inertia"][0, ids]
        pos = st["pos"].reshape(-1, 2)[ids]
        v = st["vel"].reshape(-1, 2)[ids]
        w = st["omega"][0, ids]
        return (m[:, None] * v).sum(0), (m * (pos[:, 0] * v[:, 1] - pos[:, 1] * v[:, 0]) + I * w).sum()

    p0, L0 = momenta(o.state())
    o.step(zeros_actions(30, 1, CAPS))
    p1, L1 = momenta(o.state())
    assert abs(o.state()["omega"][0, ids[0]]) > 1e-3
    assert np.allclose(p0, p1, atol=1e-12) and L1 == pytest.approx(L0, abs=1e-12)


def test_towers_show_the_stability_trade_off_of_the_batch_size():
    """A.8: solving every collision constraint in parallel noticeably reduces stability, batches of 16
    keep the speed-up without that cost.  On the towers of boxes: batches of up to 16 points stand like the
    sequential sweep, larger batches jitter, one batch of everything blows the towers apart."""
    caps, prm, sc = scenegen.make_stack_scene(n_envs=48)
    act = np.zeros((256, 48, caps[2] + caps[3]))
    p0 = np.asarray(sc["pos"])[:, 3:12]

    def settle(B):
        o, _ = run(sc, dict(prm, batch_size=B), caps=caps, dtype="f32")
        o.step(act, n_threads=4)
        st = o.state()
        pos = st["pos"].reshape(48, -1, 2)[:, 3:12]
        return (p0[..., 1] - pos[..., 1]).max(), np.abs(st["vel"]).max()

    dy1, v1 = settle(0)
    dy16, v16 = settle(16)
    dy32, v32 = settle(32)
    dyall, vall = settle(2 * 120)
    assert dy16 < 1.1 * dy1 and v16 < 0.02
    assert dy32 > 1.5 * dy1 and v32 > 10 * max(v1, v16)
    assert vall > 100.0
