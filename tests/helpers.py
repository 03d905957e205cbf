"""Hand-built scenes and small utilities shared by the tests (no step arithmetic here)."""
import numpy as np

import scenegen


def params(**kw):
    p = scenegen.default_params(kw.pop("n_substeps", 1), kw.pop("n_iters", 5), kw.pop("dt", 1.0 / 60.0))
    p.update(kw)
    return p


class SceneBuilder:
    """One environment at a time; polygons occupy shape indices 0..P-1, circles P..P+C-1."""

    def __init__(self, caps, n_envs=1):
        self.caps = caps
        self.P, self.C, self.J, self.T = caps
        self.sc = scenegen.empty_scene(caps, n_envs)
        self.n_poly = [0] * n_envs
        self.n_circ = [0] * n_envs
        self.n_joint = [0] * n_envs
        self.n_thr = [0] * n_envs

    def _body(self, e, i, pos, theta, vel, omega, inv_m, inv_i, friction, restitution, density, role):
        s = self.sc
        s["pos"][e, i] = pos
        s["theta"][e, i] = theta
        s["vel"][e, i] = vel
        s["omega"][e, i] = omega
        s["inv_mass"][e, i] = inv_m
        s["inv_inertia"][e, i] = inv_i
        s["friction"][e, i] = friction
        s["restitution"][e, i] = restitution
        s["density"][e, i] = density
        s["role"][e, i] = role
        s["active"][e, i] = 1

    def polygon(self, verts, pos, theta=0.0, vel=(0, 0), omega=0.0, density=1.0, static=False, friction=0.5,
                restitution=0.0, role=0, e=0):
        i = self.n_poly[e]
        assert i < self.P
        self.n_poly[e] += 1
        v = np.zeros((4, 2))
        n = len(verts)
        v[:n] = verts
        v2, im, ii = scenegen.polygon_mass_props(v[None], np.array([n]), np.array([density]))
        # the caller's frame must already be centred on the centroid
        assert np.allclose(v2[0, :n], v[:n], atol=1e-12), "polygon vertices must be centred on the centroid"
        self.sc["verts"][e, i] = v
        self.sc["n_verts"][e, i] = n
        if static:
            im, ii = np.zeros(1), np.zeros(1)
        self._body(e, i, pos, theta, vel, omega, im[0], ii[0], friction, restitution, density, role)
        return i

    def box(self, hx, hy, pos, **kw):
        return self.polygon(scenegen.box_verts(hx, hy), pos, **kw)

    def circle(self, r, pos, theta=0.0, vel=(0, 0), omega=0.0, density=1.0, static=False, friction=0.5,
               restitution=0.0, role=0, e=0):
        k = self.n_circ[e]
        assert k < self.C
        self.n_circ[e] += 1
        i = self.P + k
        im, ii = scenegen.circle_mass_props(np.array([r]), np.array([density]))
        if static:
            im, ii = np.zeros(1), np.zeros(1)
        self.sc["radius"][e, k] = r
        self._body(e, i, pos, theta, vel, omega, im[0], ii[0], friction, restitution, density, role)
        return i

    def joint(self, a, b, world_anchor, fixed=False, motor_on=False, speed=0.0, power=0.0, limits=None, e=0):
        q = self.n_joint[e]
        assert q < self.J
        self.n_joint[e] += 1
        s = self.sc
        wa = np.asarray(world_anchor, dtype=np.float64)

        def local(i):
            d = wa - s["pos"][e, i]
            c, sn = np.cos(-s["theta"][e, i]), np.sin(-s["theta"][e, i])
            return np.array([c * d[0] - sn * d[1], sn * d[0] + c * d[1]])

        s["joint_active"][e, q] = 1
        s["joint_a"][e, q], s["joint_b"][e, q] = a, b
        s["joint_anchor_a"][e, q] = local(a)
        s["joint_anchor_b"][e, q] = local(b)
        s["joint_fixed"][e, q] = int(fixed)
        s["joint_theta_f"][e, q] = s["theta"][e, a] - s["theta"][e, b]
        s["joint_motor_on"][e, q] = int(motor_on)
        s["joint_motor_speed"][e, q] = speed
        s["joint_motor_power"][e, q] = power
        if limits is not None:               # (lo, hi) of theta_a - theta_b
            s["joint_limited"][e, q] = 1
            s["joint_limit_lo"][e, q], s["joint_limit_hi"][e, q] = limits
        return q

    def thruster(self, body, local_pos, angle, power, e=0):
        k = self.n_thr[e]
        assert k < self.T
        self.n_thr[e] += 1
        s = self.sc
        s["thruster_active"][e, k] = 1
        s["thruster_body"][e, k] = body
        s["thruster_pos"][e, k] = local_pos
        s["thruster_angle"][e, k] = angle
        s["thruster_power"][e, k] = power
        return k

    def scene(self, f32=True):
        return scenegen.to_f32(self.sc) if f32 else {k: v.copy() for k, v in self.sc.items()}


def pair_index(i, j, N):
    return i * (2 * N - i - 1) // 2 + (j - i - 1)


def zeros_actions(n_steps, n_envs, caps):
    return np.zeros((n_steps, n_envs, caps[2] + caps[3]))


def energy(sc, state, g):
    """Kinetic + potential energy of the dynamic bodies."""
    im, ii = sc["inv_mass"], sc["inv_inertia"]
    dyn = (im > 0) & (sc["active"] > 0)
    m = np.where(dyn, 1.0 / np.where(im > 0, im, 1.0), 0.0)
    I = np.where(dyn & (ii > 0), 1.0 / np.where(ii > 0, ii, 1.0), 0.0)
    v2 = (state["vel"].reshape(im.shape + (2,)) ** 2).sum(-1)
    ke = 0.5 * m * v2 + 0.5 * I * state["omega"] ** 2
    pe = m * (-g) * state["pos"].reshape(im.shape + (2,))[..., 1]
    return (ke + pe).sum(-1)


# ---------------------------------------------------------------------------------------------------
# Degenerate scenes (input that the engine must give a defined result for): the CPU pins and the GPU
# parity tests run the same ones.
# ---------------------------------------------------------------------------------------------------
DEGENERATE_TRI = np.array([[-0.3, -0.1], [0.3, -0.1], [0.0, 0.2]])      # centred on its centroid


def degenerate_scene(kind):
    """(caps, params, scene, sane twin or None, steps): `kind` in coincident_circles, zero_length_edge,
    joint_on_itself, indices_out_of_range, infinite_inverse_mass.  The twin is the well-formed scene that the
    degenerate one must behave like, where there is one."""
    caps = scenegen.CAPS["M"]                      # 6 polygons, 3 circles, 2 joints, 2 thrusters
    prm = params(n_substeps=2, n_iters=6)
    twin = None
    sb = SceneBuilder(caps)
    floor = sb.box(5.0, 0.1, (0.0, 0.0), static=True)
    if kind == "coincident_circles":
        sb.circle(0.25, (0.5, 1.0))
        sb.circle(0.25, (0.5, 1.0), density=2.0)   # same centre: the printed normal is 0 / 0
        sb.box(0.3, 0.2, (-1.0, 0.4))
        sc = sb.scene()
    elif kind == "zero_length_edge":
        # a "quadrilateral" whose last two vertices coincide: one edge has no length, its normal is 0 / 0
        quad = np.vstack([DEGENERATE_TRI, DEGENERATE_TRI[2:3]])
        p = sb.polygon(DEGENERATE_TRI, (0.0, 0.6), theta=0.4)
        sb.circle(0.2, (0.05, 1.05))
        sb.circle(0.15, (-0.6, 0.3))
        sb.box(0.3, 0.2, (1.5, 0.35))
        twin = sb.scene()
        sc = {k: v.copy() for k, v in twin.items()}
        sc["n_verts"][0, p] = 4
        sc["verts"][0, p] = scenegen.to_f32(dict(v=quad))["v"]
    elif kind == "joint_on_itself":
        a = sb.box(0.3, 0.2, (0.0, 0.5), theta=0.2)
        b = sb.box(0.25, 0.25, (1.0, 0.8))
        sb.circle(0.2, (0.1, 1.1))
        sb.joint(a, b, (0.5, 0.6), motor_on=True, speed=2.0, power=0.4)
        sb.joint(a, b, (0.2, 0.5), fixed=True)
        sc = sb.scene()
        twin = {k: v.copy() for k, v in sc.items()}
        sc["joint_b"][0, 1] = sc["joint_a"][0, 1]          # both ends on shape a
        twin["joint_active"][0, 1] = 0
    elif kind == "indices_out_of_range":
        a = sb.box(0.3, 0.2, (0.0, 0.5), theta=0.2)
        b = sb.box(0.25, 0.25, (1.0, 0.8))
        c = sb.circle(0.2, (0.1, 1.1))
        sb.joint(a, b, (0.5, 0.6), motor_on=True, speed=2.0, power=0.4)
        sb.joint(b, c, (0.6, 0.9))
        sb.thruster(a, (0.1, 0.0), 0.5, 2.0)
        sb.thruster(b, (0.0, 0.1), -1.0, 3.0)
        sc = sb.scene()
        twin = {k: v.copy() for k, v in sc.items()}
        sc["joint_a"][0, 0] = 99
        sc["joint_b"][0, 1] = -3
        sc["thruster_body"][0, 1] = 77
        twin["joint_active"][0, :] = 0
        twin["thruster_active"][0, 1] = 0
    elif kind == "infinite_inverse_mass":
        bad = sb.box(0.3, 0.2, (0.0, 0.25))               # touches the floor: the first impulse is infinite
        sb.circle(0.2, (2.0, 1.0))
        sc = sb.scene()
        sc["inv_mass"][0, bad] = np.inf
    else:
        raise KeyError(kind)
    return caps, prm, sc, twin, 20


def same_bits_or_both_nan(x, y):
    x, y = np.asarray(x), np.asarray(y)
    return x.shape == y.shape and bool(np.all((x == y) | (np.isnan(x) & np.isnan(y))))
