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


# ----------------------------------------------------------------------------------------------------------
# Symbolic-Entity observation (Sec. 3.2 "Observation Space", Sec. 4, Appendix C Tables 5-7) and the
# multi-discrete action space (Sec. 3.2 "Action Space").
# ----------------------------------------------------------------------------------------------------------
N_ROLES = 4
SHAPE_DIM, JOINT_DIM, THRUSTER_DIM = 30, 11, 6


def decode_actions(discrete, J, T):
    """Multi-discrete actions: a motor is off (0), run forwards (1) or backwards (2) at full power; a
    thruster is off (0) or on (1).  discrete int [..., J+T] -> float32 [..., J+T]."""
    d = np.asarray(discrete)
    out = np.zeros(d.shape, dtype=np.float32)
    m = d[..., :J]
    out[..., :J] = np.where(m == 1, 1.0, np.where(m == 2, -1.0, 0.0))
    out[..., J:] = np.where(d[..., J:] == 1, 1.0, 0.0)
    return out


def entities(flat_obs, scene, shape_adj, caps):
    """From the engine oracle's flat observation [n, obs_dim] (Tables 5-7, entity after entity), the scene
    description and the collision adjacency words [n, N]:
      shapes    float32 [n, N, 30]: position 2, velocity 2, inverse mass, inverse inertia, density,
                tanh(angular velocity / 10), one-hot role (4), sin, cos of the rotation, friction, restitution,
                one-hot type (circle, polygon), radius (circles), vertices 8 and one-hot (triangle, rectangle)
                (polygons), active                                                       (Table 5 + mask)
      joints    float32 [n, 2J, 11]: active, fixed, anchor on `from` 2, anchor on `to` 2, motor power, motor
                speed, motor on, sin, cos of rotation(from) - rotation(to); entity 2q is joint q seen from its
                shape a, entity 2q+1 the same joint with from and to swapped                  (Table 7)
      joint_idx int32 [n, 2J, 2]: (from, to) shape of every joint entity
      thrusters float32 [n, T, 6] (Table 6), thruster_idx int32 [n, T]
      masks     uint32 [n, 4, N]: bit j of word i set iff shape i may attend to shape j -- all active shapes;
                shapes joined to it by an active joint; shapes reachable over any number of joints; shapes
                it is colliding with (Sec. 4).  A shape attends to itself in the first three.
    """
    P, C, J, T = caps
    N = P + C
    flat = np.asarray(flat_obs, dtype=np.float64)
    n = flat.shape[0]
    shapes = np.zeros((n, N, SHAPE_DIM), dtype=np.float32)
    joints = np.zeros((n, 2 * J, JOINT_DIM), dtype=np.float32)
    jidx = np.zeros((n, 2 * J, 2), dtype=np.int32)
    thr = np.zeros((n, T, THRUSTER_DIM), dtype=np.float32)
    tidx = np.zeros((n, T), dtype=np.int32)
    masks = np.zeros((n, 4, N), dtype=np.uint32)
    for e in range(n):
        o = flat[e]
        for i in range(N):
            f = o[i * 23:(i + 1) * 23] if i < P else o[P * 23 + (i - P) * 15:P * 23 + (i - P + 1) * 15]
            s = shapes[e, i]
            s[0:8] = f[0:8]
            role = int(f[22] if i < P else f[14])
            if 0 <= role < N_ROLES:
                s[8 + role] = 1.0
            s[12:16] = f[8:12]                          # sin, cos, friction, restitution
            s[16 if i >= P else 17] = 1.0               # type: circle, polygon
            if i < P:
                s[19:27] = f[12:20]
                s[27 if int(f[20]) == 3 else 28] = 1.0
                s[29] = f[21]
            else:
                s[18] = f[12]
                s[29] = f[13]
        act = np.asarray(scene["active"][e]) > 0
        full = 0
        for i in range(N):
            if act[i]:
                full |= 1 << i
        direct = [(1 << i) if act[i] else 0 for i in range(N)]
        base = P * 23 + C * 15
        for q in range(J):
            f = o[base + q * 11:base + (q + 1) * 11]
            a, b = int(scene["joint_a"][e, q]), int(scene["joint_b"][e, q])
            a, b = min(max(a, 0), N - 1), min(max(b, 0), N - 1)
            joints[e, 2 * q] = f
            g = f.copy()
            g[2:4], g[4:6] = f[4:6], f[2:4]
            g[9] = -f[9]                                # sin of the opposite rotation; cos is even
            joints[e, 2 * q + 1] = g
            jidx[e, 2 * q] = (a, b)
            jidx[e, 2 * q + 1] = (b, a)
            if f[0] != 0 and act[a] and act[b] and a != b:
                direct[a] |= 1 << b
                direct[b] |= 1 << a
        reach = list(direct)
        for k in range(N):                              # transitive closure
            for i in range(N):
                if (reach[i] >> k) & 1:
                    reach[i] |= reach[k]
        tb = base + J * 11
        for t in range(T):
            thr[e, t] = o[tb + t * 6:tb + (t + 1) * 6]
            tidx[e, t] = min(max(int(scene["thruster_body"][e, t]), 0), N - 1)
        for i in range(N):
            masks[e, 0, i] = full if act[i] else 0
            masks[e, 1, i] = direct[i]
            masks[e, 2, i] = reach[i]
            masks[e, 3, i] = int(shape_adj[e, i])
    return dict(shapes=shapes, joints=joints, joint_idx=jidx, thrusters=thr, thruster_idx=tidx, masks=masks)


def health(pos, theta, vel, omega, active):
    """Which environments have blown up: position (n, N, 2), rotation (n, N), velocity (n, N, 2) or angular
    velocity (n, N) of an active shape (active: n, N) is infinite or NaN.  Returns (bad uint8 [n], count)."""
    finite = (np.isfinite(pos).all(-1) & np.isfinite(theta) & np.isfinite(vel).all(-1) & np.isfinite(omega))
    bad = ((~finite) & (np.asarray(active) != 0)).any(-1)
    return bad.astype(np.uint8), int(bad.sum())
