"""CPU oracle of the environment outcome (Sec. 3.2, "Reward"): TEST INFRASTRUCTURE, not part of the product.

Plain numpy loops over the result of the engine oracle (oracle/k2d_oracle.py).  Only tests/, the smoke check
and the benchmark's CPU leg may use this module; it shares no code with the HIP path.

What is computed, per environment, after an engine step:
  * the episode ends with reward +1 if a green shape collides with a blue shape, with reward -1 if a green
    shape collides with a red shape (a collision = an active manifold point between the two shapes at the
    last substep, Table 2: penetration > 0);
  * the dense term kappa * (d_t - d_{t+1}), d = distance between the green and the blue object.

Readings of what the section leaves open: roles are small integers carried by every shape (which integer
means green / blue / red is a parameter); with several green or blue shapes d is the smallest centre
distance over the active (green, blue) pairs, 0 if there is none; a green shape touching blue and red in
the same step counts as reaching the goal; at the first step of an episode (no d_t yet, marked by a
negative stored distance) the dense term is 0.  Arithmetic in fp32, one rounding per operation.
"""
import numpy as np


def pair_index(i, j, N):
    return i * (2 * N - i - 1) // 2 + (j - i - 1)


def outcome(pos, role, active, pair_count, d_prev, kappa, green=1, blue=2, red=3):
    """pos [n, N, 2], role [n, N], active [n, N], pair_count [n, NP] (lexicographic pairs), d_prev [n]
    -> reward [n] float32, done [n] uint8, d_new [n] float32."""
    pos = np.asarray(pos, dtype=np.float32)
    n, N = role.shape
    f = np.float32
    reward = np.zeros(n, dtype=np.float32)
    done = np.zeros(n, dtype=np.uint8)
    d_new = np.zeros(n, dtype=np.float32)
    for e in range(n):
        goal = bad = False
        best = None
        for i in range(N):
            if not active[e, i] or role[e, i] != green:
                continue
            for j in range(N):
                if j == i or not active[e, j]:
                    continue
                a, b = min(i, j), max(i, j)
                touching = pair_count[e, pair_index(a, b, N)] > 0
                if role[e, j] == blue:
                    goal |= bool(touching)
                    dx = f(pos[e, j, 0] - pos[e, i, 0])
                    dy = f(pos[e, j, 1] - pos[e, i, 1])
                    d = np.sqrt(f(f(dx * dx) + f(dy * dy)))
                    best = d if best is None or d < best else best
                elif role[e, j] == red:
                    bad |= bool(touching)
        d_new[e] = f(0) if best is None else best
        dense = f(0)
        if d_prev[e] >= 0 and best is not None:
            dense = f(f(kappa) * f(f(d_prev[e]) - d_new[e]))
        sparse = f(1) if goal else (f(-1) if bad else f(0))
        reward[e] = f(sparse + dense)
        done[e] = 1 if (goal or bad) else 0
    return reward, done, d_new
