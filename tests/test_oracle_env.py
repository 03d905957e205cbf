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
