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
    """Three shapes in a chain a - b - c (two joints) and a loose fourth: one-hots, the two views of a joint,
    and the masks (direct neighbours vs. everything reachable over joints)."""
    caps = (2, 2, 2, 1)
    sb = SceneBuilder(caps)
    a = sb.box(0.3, 0.2, (0.0, 1.0), role=1)
    tri = sb.polygon(np.array([[-0.3, -0.1], [0.3, -0.1], [0.0, 0.2]]), (0.5, 1.0), role=3)   # centred on its centroid
    c = sb.circle(0.15, (1.0, 1.0), role=2)
    loose = sb.circle(0.1, (3.0, 3.0))
    sb.joint(a, tri, (0.25, 1.0), motor_on=True, speed=2.0, power=0.5)
    sb.joint(tri, c, (0.75, 1.0), fixed=True)
    sb.thruster(c, (0.05, 0.0), angle=0.3, power=1.5)
    sc = sb.scene(f32=True)
    o = Oracle(caps, 1, params(gravity_y=0.0), "f32")
    o.load_scene(sc)
    ent = k2d_env.entities(o.obs(), sc, o.get("shape_adj"), caps)
    S = ent["shapes"][0]
    assert S.shape == (4, 30)
    assert list(S[a, 8:12]) == [0, 1, 0, 0] and list(S[tri, 8:12]) == [0, 0, 0, 1] and list(S[c, 8:12]) == [0, 0, 1, 0]
    assert list(S[a, 16:18]) == [0, 1] and list(S[c, 16:18]) == [1, 0]           # circle, polygon
    assert list(S[a, 27:29]) == [0, 1] and list(S[tri, 27:29]) == [1, 0]         # triangle, rectangle
    assert S[c, 18] == np.float32(0.15) and S[a, 18] == 0 and (S[c, 19:29] == 0).all()
    assert S[a, 0] == 0.0 and S[a, 1] == 1.0 and (S[:, 29] == 1).all()
    J = ent["joints"][0]
    assert list(ent["joint_idx"][0, 0]) == [a, tri] and list(ent["joint_idx"][0, 1]) == [tri, a]
    assert np.array_equal(J[0, 2:4], J[1, 4:6]) and np.array_equal(J[0, 4:6], J[1, 2:4])
    assert J[0, 9] == -J[1, 9] and J[0, 10] == J[1, 10] and J[0, 8] == 1 and J[2, 1] == 1
    assert list(ent["thruster_idx"][0]) == [c] and ent["thrusters"][0, 0, 3] == np.float32(1.5)
    M = ent["masks"][0]
    bit = lambda *idx: sum(1 << i for i in idx)
    assert list(M[0]) == [bit(a, tri, c, loose)] * 4
    assert list(M[1]) == [bit(a, tri), bit(a, tri, c), bit(tri, c), bit(loose)]
    assert list(M[2]) == [bit(a, tri, c)] * 3 + [bit(loose)]
    assert list(M[3]) == [0, 0, 0, 0]


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
    n, N = 6, 4
    pos, vel = np.zeros((n, N, 2)), np.ones((n, N, 2))
    theta, omega = np.zeros((n, N)), np.zeros((n, N))
    active = np.ones((n, N), dtype=np.int64)
    active[:, 3] = 0
    pos[1, 0, 1] = np.nan           # active shape: flagged
    vel[2, 2, 0] = -np.inf          # active shape: flagged
    omega[3, 3] = np.nan            # inactive shape: ignored
    theta[4, 1] = np.inf            # active: flagged
    vel[5, 0] = 3.0e38              # huge but finite: fine
    bad, count = k2d_env.health(pos, theta, vel, omega, active)
    assert bad.tolist() == [0, 1, 1, 0, 1, 0] and count == 3
