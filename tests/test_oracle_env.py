"""Pins of the environment-outcome oracle (Sec. 3.2, "Reward") on hand-built scenes with known answers."""
import numpy as np
import pytest

from helpers import SceneBuilder, params, pair_index
from oracle.k2d_oracle import Oracle
from oracle import k2d_env

CAPS = (2, 2, 1, 1)
GREEN, BLUE, RED = 1, 2, 3


def _run(sb, p, steps, kappa=0.5):
    sc = sb.scene(f32=True)
    o = Oracle(CAPS, 1, p, "f32")
    o.load_scene(sc)
    N = CAPS[0] + CAPS[1]
    d = np.full(1, -1.0, dtype=np.float32)
    out = []
    for _ in range(steps):
        o.step(np.zeros((1, 1, 2)))
        st = o.state()
        r, done, d = k2d_env.outcome(st["pos"].reshape(1, N, 2), sc["role"], sc["active"], st["pair_count"], d, kappa,
                                     GREEN, BLUE, RED)
        out.append((float(r[0]), int(done[0]), float(d[0])))
    return out


def test_dense_term_closed_form_in_free_flight():
    """No gravity, a green ball flying at constant speed towards a resting blue ball: d shrinks by v*dt per
    step, so every step after the first pays kappa * v * dt; the first step has no d_t and pays nothing."""
    sb = SceneBuilder(CAPS)
    sb.circle(0.2, (0.0, 0.0), vel=(1.5, 0.0), role=GREEN)
    sb.circle(0.2, (4.0, 0.0), role=BLUE)
    p = params(gravity_y=0.0)
    out = _run(sb, p, 20, kappa=0.5)
    assert out[0][0] == 0.0 and out[0][1] == 0
    assert out[0][2] == pytest.approx(4.0 - 1.5 * p["dt"], rel=1e-6)
    for r, done, _ in out[1:]:
        assert done == 0 and r == pytest.approx(0.5 * 1.5 * p["dt"], rel=1e-4)


@pytest.mark.parametrize("role,sign", [(BLUE, 1.0), (RED, -1.0)])
def test_green_reaching_blue_or_red_ends_the_episode(role, sign):
    sb = SceneBuilder(CAPS)
    sb.box(2.0, 0.2, (0.0, 0.0), static=True, role=role)
    sb.circle(0.25, (0.0, 1.0), role=GREEN)
    out = _run(sb, params(), 40, kappa=0.0)
    done = [d for _, d, _ in out]
    first = done.index(1)
    assert 5 < first < 30                       # it has to fall 0.55 first: 0.5 g t^2 -> t = 0.33 s = 20 steps
    assert all(d == 0 for d in done[:first])
    assert out[first][0] == sign and all(r == 0.0 for r, _, _ in out[:first])


def test_goal_wins_over_red_and_bystanders_do_not_count():
    sb = SceneBuilder(CAPS)
    sb.box(1.0, 0.2, (-1.0, 0.0), static=True, role=BLUE)
    sb.box(1.0, 0.2, (1.0, 0.0), static=True, role=RED)
    sb.circle(0.3, (0.0, 0.45), role=GREEN)                    # straddles both boxes
    sb.circle(0.2, (1.5, 0.35), role=0)                        # a neutral ball on the red box
    out = _run(sb, params(), 3, kappa=0.0)
    assert out[0][1] == 1 and out[0][0] == 1.0
    sb = SceneBuilder(CAPS)                                    # neutral on red, green in the air: nothing
    sb.box(1.0, 0.2, (1.0, 0.0), static=True, role=RED)
    sb.circle(0.2, (1.5, 0.35), role=0)
    sb.circle(0.2, (-3.0, 5.0), role=GREEN)
    out = _run(sb, params(), 3, kappa=0.0)
    assert all(d == 0 and r == 0.0 for r, d, _ in out)


def test_distance_is_the_smallest_over_pairs_and_zero_without_a_pair():
    N = 4
    pos = np.array([[[0.0, 0.0], [3.0, 4.0], [1.0, 0.0], [9.0, 9.0]]])
    role = np.array([[GREEN, BLUE, BLUE, GREEN]])
    active = np.ones((1, N), dtype=int)
    pc = np.zeros((1, N * (N - 1) // 2))
    r, done, d = k2d_env.outcome(pos, role, active, pc, np.array([2.0], dtype=np.float32), 1.0, GREEN, BLUE, RED)
    assert d[0] == 1.0 and r[0] == 1.0 and done[0] == 0        # 2.0 -> 1.0, kappa = 1
    active[0, 2] = 0                                           # the near blue shape switched off
    r, done, d = k2d_env.outcome(pos, role, active, pc, np.array([2.0], dtype=np.float32), 1.0, GREEN, BLUE, RED)
    assert d[0] == 5.0 and r[0] == -3.0
    role[0, 1] = 0                                             # no blue shape left
    r, done, d = k2d_env.outcome(pos, role, active, pc, np.array([2.0], dtype=np.float32), 1.0, GREEN, BLUE, RED)
    assert d[0] == 0.0 and r[0] == 0.0
    pc[0, pair_index(0, 1, N)] = 2                             # touching something that is not blue or red
    r, done, d = k2d_env.outcome(pos, role, active, pc, np.array([2.0], dtype=np.float32), 1.0, GREEN, BLUE, RED)
    assert done[0] == 0


# ------------------------------------------------------------------ entity observation, action decoding
def test_entity_observation_on_a_hand_built_chain():
    """Three shapes in a chain a - b - c (two joints), a loose fourth and an inactive fifth with a joint of its
    own: one-hots, the two views of a joint, and the masks (direct neighbours vs. everything reachable over
    joints; inactive shapes neither attend nor are attended to)."""
    caps = (2, 3, 3, 1)
    sb = SceneBuilder(caps)
    a = sb.box(0.3, 0.2, (0.0, 1.0), role=1, theta=0.4)
    tri = sb.polygon(np.array([[-0.3, -0.1], [0.3, -0.1], [0.0, 0.2]]), (0.5, 1.0), role=3)   # centred on its centroid
    c = sb.circle(0.15, (1.0, 1.0), role=2)
    loose = sb.circle(0.1, (3.0, 3.0))
    ghost = sb.circle(0.1, (1.2, 1.0))
    sb.joint(a, tri, (0.25, 1.0), motor_on=True, speed=2.0, power=0.5)
    sb.joint(tri, c, (0.75, 1.0), fixed=True)
    sb.joint(c, ghost, (1.1, 1.0))
    sb.sc["active"][0, ghost] = 0
    sb.thruster(c, (0.05, 0.0), angle=0.3, power=1.5)
    sc = sb.scene(f32=True)
    o = Oracle(caps, 1, params(gravity_y=0.0), "f32")
    o.load_scene(sc)
    ent = k2d_env.entities(o.obs(), sc, o.get("shape_adj"), caps)
    S = ent["shapes"][0]
    assert S.shape == (5, 30)
    assert list(S[a, 8:12]) == [0, 1, 0, 0] and list(S[tri, 8:12]) == [0, 0, 0, 1] and list(S[c, 8:12]) == [0, 0, 1, 0]
    assert list(S[a, 16:18]) == [0, 1] and list(S[c, 16:18]) == [1, 0]           # circle, polygon
    assert list(S[a, 27:29]) == [0, 1] and list(S[tri, 27:29]) == [1, 0]         # triangle, rectangle
    assert S[c, 18] == np.float32(0.15) and S[a, 18] == 0 and (S[c, 19:29] == 0).all()
    assert S[a, 0] == 0.0 and S[a, 1] == 1.0 and list(S[:, 29]) == [1, 1, 1, 1, 0]
    J = ent["joints"][0]
    assert list(ent["joint_idx"][0, 0]) == [a, tri] and list(ent["joint_idx"][0, 1]) == [tri, a]
    assert np.array_equal(J[0, 2:4], J[1, 4:6]) and np.array_equal(J[0, 4:6], J[1, 2:4])
    assert J[0, 9] == pytest.approx(np.sin(0.4), abs=2e-7) and J[0, 10] == pytest.approx(np.cos(0.4), abs=2e-7)
    assert J[1, 9] == -J[0, 9] and J[1, 10] == J[0, 10] and J[0, 8] == 1 and J[2, 1] == 1
    assert list(ent["thruster_idx"][0]) == [c] and ent["thrusters"][0, 0, 3] == np.float32(1.5)
    M = ent["masks"][0]
    bit = lambda *idx: sum(1 << i for i in idx)
    assert list(M[0]) == [bit(a, tri, c, loose)] * 4 + [0]
    assert list(M[1]) == [bit(a, tri), bit(a, tri, c), bit(tri, c), bit(loose), 0]
    assert list(M[2]) == [bit(a, tri, c)] * 3 + [bit(loose), 0]
    assert list(M[3]) == [0, 0, 0, 0, 0]


def test_multi_discrete_actions():
    d = np.array([[[0, 1, 2, 0, 1], [2, 2, 1, 1, 0]]])
    out = k2d_env.decode_actions(d, 3, 2)
    assert out.dtype == np.float32
    assert out.tolist() == [[[0.0, 1.0, -1.0, 0.0, 1.0], [-1.0, -1.0, 1.0, 1.0, 0.0]]]


def test_observation_widths_match_the_papers_tables():
    """Tables 5-7 fix which fields an entity carries and how wide each is."""
    import os
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "tables5to7_observation_fields.txt"))
            if l.strip() and not l.startswith("#")]
    sym = {"n_roles": k2d_env.N_ROLES, "n_types": 2, "n_colours": 0}     # joint colours are not engine state
    width = {}
    for table, _, dims in rows:
        width[table] = width.get(table, 0) + (sym[dims] if dims in sym else int(dims))
    assert k2d_env.SHAPE_DIM == width["shape"] + 1                       # + the active flag (the set's mask)
    assert k2d_env.JOINT_DIM == width["joint"] and k2d_env.THRUSTER_DIM == width["thruster"]
    # the engine's flat observation: the same fields without one-hots (role passed through, n_verts for the
    # polygon kind, an active flag per shape)
    for caps in ((5, 2, 1, 1), (12, 4, 6, 2)):
        P, C, J, T = caps
        o = Oracle(caps, 1, params(), "f32")
        per_poly = width["shape"] - sym["n_roles"] - sym["n_types"] - 1 - 2 + 1 + 1 + 1   # no radius, n_verts, active, role
        per_circ = width["shape"] - sym["n_roles"] - sym["n_types"] - 8 - 2 + 1 + 1        # no vertices, active, role
        assert o.obs().shape[1] == P * per_poly + C * per_circ + J * width["joint"] + T * width["thruster"]


# ------------------------------------------------------------------ health of the batch
def test_health_flags_non_finite_active_shapes_only():
    n, N = 7, 4
    pos, vel = np.zeros((n, N, 2)), np.ones((n, N, 2))
    theta, omega = np.zeros((n, N)), np.zeros((n, N))
    active = np.ones((n, N), dtype=np.int64)
    active[:, 3] = 0
    pos[1, 0, 1] = np.nan           # active shape: flagged
    vel[2, 2, 0] = -np.inf          # active shape: flagged
    omega[3, 3] = np.nan            # inactive shape: ignored
    theta[4, 1] = np.inf            # active: flagged
    vel[5, 0] = 3.0e38              # huge but finite: fine
    pos[6, 1, 0] = np.inf           # an infinite position is as bad as a NaN
    bad, count = k2d_env.health(pos, theta, vel, omega, active)
    assert bad.tolist() == [0, 1, 1, 0, 1, 0, 1] and count == 4


# ------------------------------------------------------------------ values of the flat observation
def test_flat_observation_values_written_out_from_tables_5_to_7():
    """Every slot of the engine's flat observation on a hand-built scene, against numbers typed in here from
    the scene's definition and Tables 5-7: position 2, velocity 2, inverse mass, inverse inertia, density,
    tanh(angular velocity / 10), sin and cos of the rotation, friction, restitution, then radius (circle) or
    the 8 vertex coordinates and the vertex count (polygon), active, role; joints and thrusters as tabled.
    The transcendental slots are checked against double-precision libm (the engine's fp32 routines are within
    1.5e-7 of it), so swapping the sin / cos slots, or dropping the "/ 10", fails here."""
    caps = (2, 1, 1, 1)
    sb = SceneBuilder(caps)
    tri_v = np.array([[-0.3, -0.1], [0.3, -0.1], [0.0, 0.2]])          # centred on its centroid, area 0.09
    tri = sb.polygon(tri_v, (1.25, 2.5), theta=0.3, vel=(0.5, -0.75), omega=5.0, density=2.0, friction=0.7,
                     restitution=0.15, role=2)
    box = sb.box(0.4, 0.1, (-1.0, 0.5), theta=-1.2, vel=(0.0, 0.25), omega=-20.0, density=0.5, friction=0.3,
                 restitution=0.05, role=1)
    cir = sb.circle(0.25, (3.0, 1.5), theta=2.0, vel=(-1.5, 0.0), omega=0.5, density=4.0, friction=0.9,
                    restitution=0.45, role=3)
    sb.joint(tri, cir, (1.5, 2.5), motor_on=True, speed=2.5, power=0.75)
    sb.thruster(box, (0.125, -0.05), angle=-0.6, power=1.75)
    sc = sb.scene(f32=True)
    o = Oracle(caps, 1, params(gravity_y=0.0), "f32")
    o.load_scene(sc)
    obs = o.obs()[0]
    assert obs.shape == (23 * 2 + 15 + 11 + 6,)
    f = np.float32

    def close(x, want):
        assert abs(float(x) - want) < 3e-7, (float(x), want)

    # ---- the triangle: mass = density * area = 2 * 0.09; polar moment about the centroid of a triangle with
    # vertices r_i: (m / 6) * (|r0|^2 + |r1|^2 + |r2|^2 + r0.r1 + r1.r2 + r2.r0)
    t = obs[0:23]
    assert [t[0], t[1], t[2], t[3]] == [f(1.25), f(2.5), f(0.5), f(-0.75)]
    m_tri = 2.0 * 0.09
    r = tri_v
    i_tri = m_tri / 6.0 * (sum(r[i] @ r[i] for i in range(3)) + r[0] @ r[1] + r[1] @ r[2] + r[2] @ r[0])
    close(t[4], 1.0 / m_tri)
    assert abs(t[5] * i_tri - 1.0) < 1e-6
    assert t[6] == f(2.0)
    close(t[7], np.tanh(5.0 / 10.0))                                    # 0.46211715726
    close(t[8], np.sin(0.3)); close(t[9], np.cos(0.3))                  # 0.29552020666, 0.95533648912
    assert abs(float(t[7]) - 0.46211715726) < 3e-7 and abs(float(t[8]) - 0.29552020666) < 3e-7
    assert abs(float(t[9]) - 0.95533648912) < 3e-7
    assert [t[10], t[11]] == [f(0.7), f(0.15)]
    assert list(t[12:20]) == [f(-0.3), f(-0.1), f(0.3), f(-0.1), f(0.0), f(0.2), f(0.0), f(0.0)]
    assert [t[20], t[21], t[22]] == [3.0, 1.0, 2.0]                     # vertex count, active, role
    # ---- the box 0.8 x 0.2: mass = 0.5 * 0.16, inertia = m (w^2 + h^2) / 12
    b = obs[23:46]
    assert [b[0], b[1], b[2], b[3]] == [f(-1.0), f(0.5), f(0.0), f(0.25)]
    m_box = 0.5 * 0.16
    close(b[4], 1.0 / m_box)
    assert abs(b[5] * (m_box * (0.8 ** 2 + 0.2 ** 2) / 12.0) - 1.0) < 1e-6
    assert b[6] == f(0.5)
    close(b[7], np.tanh(-2.0))                                          # -0.96402758007
    close(b[8], np.sin(-1.2)); close(b[9], np.cos(-1.2))                # -0.93203908597, 0.36235775448
    assert abs(float(b[8]) + 0.93203908597) < 3e-7 and abs(float(b[9]) - 0.36235775448) < 3e-7
    assert [b[10], b[11]] == [f(0.3), f(0.05)]
    assert list(b[12:20]) == [f(-0.4), f(-0.1), f(0.4), f(-0.1), f(0.4), f(0.1), f(-0.4), f(0.1)]
    assert [b[20], b[21], b[22]] == [4.0, 1.0, 1.0]
    # ---- the circle: mass = density * pi r^2, inertia = m r^2 / 2
    c = obs[46:61]
    assert [c[0], c[1], c[2], c[3]] == [f(3.0), f(1.5), f(-1.5), f(0.0)]
    m_c = 4.0 * np.pi * 0.25 ** 2
    assert abs(c[4] * m_c - 1.0) < 1e-6 and abs(c[5] * (0.5 * m_c * 0.25 ** 2) - 1.0) < 1e-6
    assert c[6] == f(4.0)
    close(c[7], np.tanh(0.05)); close(c[8], np.sin(2.0)); close(c[9], np.cos(2.0))   # 0.04995837, 0.90929743, -0.41614684
    assert abs(float(c[9]) + 0.41614683655) < 3e-7
    assert [c[10], c[11], c[12], c[13], c[14]] == [f(0.9), f(0.45), f(0.25), 1.0, 3.0]
    # ---- the joint: active, fixed, anchor on a (local frame of the triangle: world offset (0.25, 0) turned by
    # -0.3), anchor on b (world offset (-1.5, 1.0) turned by -2.0), motor power, motor speed, motor on,
    # sin / cos of rotation(a) - rotation(b) = 0.3 - 2.0
    j = obs[61:72]
    assert [j[0], j[1]] == [1.0, 0.0]
    close(j[2], 0.25 * np.cos(0.3)); close(j[3], -0.25 * np.sin(0.3))
    close(j[4], -1.5 * np.cos(2.0) + 1.0 * np.sin(2.0)); close(j[5], 1.5 * np.sin(2.0) + 1.0 * np.cos(2.0))
    assert [j[6], j[7], j[8]] == [f(0.75), f(2.5), 1.0]
    close(j[9], np.sin(-1.7)); close(j[10], np.cos(-1.7))               # -0.99166481045, -0.12884449430
    assert abs(float(j[9]) + 0.99166481045) < 3e-7 and abs(float(j[10]) + 0.12884449430) < 3e-7
    # ---- the thruster: active, mount point (local), power, sin / cos of its local angle
    th = obs[72:78]
    assert [th[0], th[1], th[2], th[3]] == [1.0, f(0.125), f(-0.05), f(1.75)]
    close(th[4], np.sin(-0.6)); close(th[5], np.cos(-0.6))              # -0.56464247340, 0.82533561491
    assert abs(float(th[4]) + 0.56464247340) < 3e-7 and abs(float(th[5]) - 0.82533561491) < 3e-7
    # an inactive shape keeps its slots and reports active = 0
    sc2 = {k: v.copy() for k, v in sc.items()}
    sc2["active"][0, box] = 0
    o.load_scene(sc2)
    assert o.obs()[0][23 + 21] == 0.0 and o.obs()[0][21] == 1.0
