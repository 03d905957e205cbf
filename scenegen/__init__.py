"""Seeded synthetic inputs for the batched 2D rigid-body step: scenes, actions, step parameters.

This module serves both the GPU path and the CPU oracle and therefore holds none of the step's
arithmetic: it only draws numbers and prepares scene descriptions (shape geometry, mass properties,
joint anchors), which are *inputs* of the step.  Random numbers come from a counter-based generator
(splitmix64 of seed, config, episode, env id, draw index), so any environment of any config can be
regenerated alone -- which is what the reset-heavy heterogeneous workload needs.

The workloads stand in for the paper's S / M / L random levels (Table 4 gives the capacities; the
level generator itself and its levels are not available) under the engine-only, many-environments
protocol of its speed test (Appendix B).
"""
import numpy as np

SEED = 20241030

# Table 4: polygons, circles, joints, thrusters
CAPS = {"S": (5, 2, 1, 1), "M": (6, 3, 2, 2), "L": (12, 4, 6, 2)}

# name, capacity class, n_envs, n_steps, n_substeps, n_iters
CONFIGS = [
    dict(name="S", size="S", n_envs=64, n_steps=200, n_substeps=1, n_iters=5),
    dict(name="M", size="M", n_envs=1024, n_steps=256, n_substeps=2, n_iters=8),
    dict(name="L", size="L", n_envs=8192, n_steps=256, n_substeps=3, n_iters=10),
    dict(name="L-stress", size="L", n_envs=32768, n_steps=512, n_substeps=3, n_iters=10),
    dict(name="hetero", size="L", n_envs=16384, n_steps=256, n_substeps=3, n_iters=10),
]

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix(x):
    """splitmix64 finaliser on a uint64 array."""
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


class Draws:
    """Counter-based uniform draws, one independent stream per environment id."""

    def __init__(self, seed, config, episode, env_ids):
        env_ids = np.asarray(env_ids, dtype=np.uint64)
        episode = np.broadcast_to(np.asarray(episode, dtype=np.uint64), env_ids.shape)
        k = _mix(np.full(env_ids.shape, np.uint64(seed), dtype=np.uint64))
        k = _mix(k ^ np.uint64(config + 1))
        k = _mix(k ^ episode)
        self.key = _mix(k ^ env_ids)
        self.counter = 0
        self.n = env_ids.shape[0]

    def u(self, *shape, lo=0.0, hi=1.0):
        """Uniform [lo, hi) of shape [n_envs, *shape] (float64)."""
        cnt = int(np.prod(shape)) if shape else 1
        idx = np.arange(cnt, dtype=np.uint64) + np.uint64(self.counter)
        self.counter += cnt
        with np.errstate(over="ignore"):
            bits = _mix(self.key[:, None] + idx[None, :] * np.uint64(0xD1342543DE82EF95))
        r = (bits >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
        return (lo + (hi - lo) * r).reshape((self.n,) + tuple(shape))

    def integers(self, n, *shape):
        return np.minimum((self.u(*shape) * n).astype(np.int64), n - 1)


def default_params(n_substeps=1, n_iters=5, dt=1.0 / 60.0):
    """Step parameters.  The paper names alpha, beta, gamma, rho but prints no values: the correction
    speeds are set so that a fixed fraction of the error is removed per substep."""
    h = dt / n_substeps
    return dict(dt=dt, gravity_y=-9.81, n_substeps=n_substeps, n_iters=n_iters, warm_start=1,
                alpha=0.1 / h, beta=0.2, gamma=0.1 / h, rho=1.0, slop=0.005, restitution_threshold=1.0,
                clip_thruster_01=0, joint_alpha=0.1 / h, joint_beta=0.2, tie_eps=1e-3)


def empty_scene(caps, n_envs):
    """All-inactive scene of the given capacities (float64 / int64 arrays, one row per env)."""
    P, C, J, T = caps
    N = P + C
    z = lambda *s: np.zeros((n_envs,) + s)
    zi = lambda *s: np.zeros((n_envs,) + s, dtype=np.int64)
    sc = dict(pos=z(N, 2), theta=z(N), vel=z(N, 2), omega=z(N), inv_mass=z(N), inv_inertia=z(N),
              friction=z(N), restitution=z(N), density=z(N), role=zi(N), active=zi(N),
              n_verts=zi(P) + 4, verts=z(P, 4, 2), radius=z(C),
              joint_active=zi(J), joint_a=zi(J), joint_b=zi(J), joint_fixed=zi(J), joint_motor_on=zi(J),
              joint_anchor_a=z(J, 2), joint_anchor_b=z(J, 2), joint_theta_f=z(J), joint_motor_speed=z(J),
              joint_motor_power=z(J), joint_limited=zi(J), joint_limit_lo=z(J), joint_limit_hi=z(J),
              thruster_active=zi(T), thruster_body=zi(T), thruster_pos=z(T, 2), thruster_angle=z(T),
              thruster_power=z(T))
    if J:
        sc["joint_b"][:] = min(1, N - 1)
    return sc


def to_f32(scene):
    """Round every real-valued entry to fp32 (what both implementations are fed)."""
    out = {}
    for k, v in scene.items():
        out[k] = v.astype(np.float32).astype(np.float64) if v.dtype.kind == "f" else v.copy()
    return out


def add_joint_limits(scene, seed=SEED, width=(0.05, 0.5)):
    """Variant of a generated scene in which every revolute joint is limited (A.4.3): the relative rotation
    theta_a - theta_b may leave its initial value by U[width] radians either way.  Returns a new dict."""
    sc = {k: v.copy() for k, v in scene.items()}
    rng = np.random.default_rng(seed)
    shape = sc["joint_theta_f"].shape
    sc["joint_limited"] = (np.asarray(sc["joint_fixed"]) == 0).astype(np.int64)
    sc["joint_limit_lo"] = sc["joint_theta_f"] - rng.uniform(width[0], width[1], shape)
    sc["joint_limit_hi"] = sc["joint_theta_f"] + rng.uniform(width[0], width[1], shape)
    return to_f32(sc)


def select_envs(scene, ids):
    return {k: v[ids] for k, v in scene.items()}


# ------------------------------------------------------------------------------------------------
# Shape preparation (inputs of the step: geometry about the centre of mass, inverse mass / inertia)
# ------------------------------------------------------------------------------------------------
def polygon_mass_props(verts, n_verts, density):
    """verts [...,4,2] CCW (entry 3 unused for triangles), n_verts [...] -> recentred verts, inv_mass,
    inv_inertia.  Uniform density; area, centroid and polar second moment of a simple polygon."""
    v = np.array(verts, dtype=np.float64)
    tri = (np.asarray(n_verts) == 3)
    v[tri, 3, :] = v[tri, 0, :]          # closes the triangle with a zero-length edge (adds nothing)
    w = np.roll(v, -1, axis=-2)
    cr = v[..., 0] * w[..., 1] - v[..., 1] * w[..., 0]
    area = 0.5 * cr.sum(-1)
    cx = ((v[..., 0] + w[..., 0]) * cr).sum(-1) / (6.0 * area)
    cy = ((v[..., 1] + w[..., 1]) * cr).sum(-1) / (6.0 * area)
    v = v - np.stack([cx, cy], -1)[..., None, :]
    w = np.roll(v, -1, axis=-2)
    cr = v[..., 0] * w[..., 1] - v[..., 1] * w[..., 0]
    quad = (v * v).sum(-1) + (v * w).sum(-1) + (w * w).sum(-1)
    inertia = density * (cr * quad).sum(-1) / 12.0
    mass = density * area
    v[tri, 3, :] = 0.0
    return v, 1.0 / mass, 1.0 / inertia


def circle_mass_props(radius, density):
    mass = density * np.pi * radius ** 2
    return 1.0 / mass, 1.0 / (0.5 * mass * radius ** 2)


def box_verts(hx, hy):
    hx = np.asarray(hx, dtype=np.float64)
    hy = np.asarray(hy, dtype=np.float64)
    return np.stack([np.stack([-hx, -hy], -1), np.stack([hx, -hy], -1), np.stack([hx, hy], -1),
                     np.stack([-hx, hy], -1)], -2)


def _hull4(pts):
    """Convex hull of 4 points per row: [M,4,2] -> (verts [M,4,2] CCW, n_verts [M])."""
    M = pts.shape[0]

    def cross(o, a, b):
        return (a[:, 0] - o[:, 0]) * (b[:, 1] - o[:, 1]) - (a[:, 1] - o[:, 1]) * (b[:, 0] - o[:, 0])

    inside = np.zeros((M, 4), dtype=bool)
    for i in range(4):
        o = [j for j in range(4) if j != i]
        a, b, c, p = pts[:, o[0]], pts[:, o[1]], pts[:, o[2]], pts[:, i]
        d1, d2, d3 = cross(a, b, p), cross(b, c, p), cross(c, a, p)
        neg = (d1 < 0) | (d2 < 0) | (d3 < 0)
        posi = (d1 > 0) | (d2 > 0) | (d3 > 0)
        inside[:, i] = ~(neg & posi)
    n_in = inside.sum(1)
    # drop (at most) the first interior point
    drop = np.where(n_in > 0, inside.argmax(1), -1)
    keep = np.ones((M, 4), dtype=bool)
    keep[np.arange(M)[drop >= 0], drop[drop >= 0]] = False
    nv = keep.sum(1)
    cnt = keep.sum(1, keepdims=True)
    mean = (pts * keep[..., None]).sum(1) / cnt
    ang = np.arctan2(pts[..., 1] - mean[:, None, 1], pts[..., 0] - mean[:, None, 0])
    ang = np.where(keep, ang, 1e9)       # dropped point sorts last
    order = np.argsort(ang, axis=1, kind="stable")
    verts = np.take_along_axis(pts, order[..., None], axis=1)
    verts[nv == 3, 3, :] = 0.0
    return verts, nv


def _random_hulls(d, n_poly, extent_lo, extent_hi):
    """n_poly random convex 3-4-gons per env: hull of 4 points U[-s/2,s/2]^2, s ~ U[extent_lo, extent_hi]."""
    E = d.n
    verts = np.zeros((E, n_poly, 4, 2))
    nv = np.full((E, n_poly), 4, dtype=np.int64)
    todo = np.ones((E, n_poly), dtype=bool)
    for _ in range(12):
        s = d.u(n_poly, lo=extent_lo, hi=extent_hi)
        pts = (d.u(n_poly, 4, 2) - 0.5) * s[..., None, None]
        hv, hn = _hull4(pts.reshape(-1, 4, 2))
        hv = hv.reshape(E, n_poly, 4, 2)
        hn = hn.reshape(E, n_poly)
        closed = hv.copy()
        t = hn == 3
        closed[t, 3, :] = closed[t, 0, :]
        w = np.roll(closed, -1, axis=-2)
        area = 0.5 * (closed[..., 0] * w[..., 1] - closed[..., 1] * w[..., 0]).sum(-1)
        ok = todo & (area >= 0.01 * (extent_hi ** 2))
        verts[ok] = hv[ok]
        nv[ok] = hn[ok]
        todo &= ~ok
        if not todo.any():
            break
    if todo.any():                       # fallback: a small square
        verts[todo] = box_verts(0.15, 0.15)
        nv[todo] = 4
    return verts, nv


def _place(d, radii, region, static_boxes, retries, fixed_mask):
    """Centres for the shapes (bounding-circle rejection against earlier shapes and the static boxes).
    radii [E,N]; fixed_mask [N] marks shapes whose position is already final (pos ignored here)."""
    E, N = radii.shape
    (x0, x1), (y0, y1) = region
    pos = np.zeros((E, N, 2))
    for i in range(N):
        if fixed_mask[i]:
            continue
        need = np.ones(E, dtype=bool)
        for _ in range(max(1, retries + 1)):
            cand = np.stack([d.u(lo=x0, hi=x1), d.u(lo=y0, hi=y1)], -1)
            pos[need, i] = cand[need]
            if retries == 0:
                break
            bad = np.zeros(E, dtype=bool)
            for j in range(i):
                if fixed_mask[j]:
                    continue
                dist = np.linalg.norm(pos[:, i] - pos[:, j], axis=-1)
                bad |= dist < radii[:, i] + radii[:, j]
            for (bx0, bx1, by0, by1) in static_boxes:
                cx = np.clip(pos[:, i, 0], bx0, bx1)
                cy = np.clip(pos[:, i, 1], by0, by1)
                bad |= np.hypot(pos[:, i, 0] - cx, pos[:, i, 1] - cy) < radii[:, i]
            need &= bad
            if not need.any():
                break
    return pos


def _rot(theta, v):
    c, s = np.cos(theta), np.sin(theta)
    return np.stack([c * v[..., 0] - s * v[..., 1], s * v[..., 0] + c * v[..., 1]], -1)


def _generate(cfg_id, caps, env_ids, episode, seed, *, statics, poly_kind, extent, circle_r, region, retries,
              joint_fixed_pattern, mask_mode, restitution_hi, friction_range, chains=False):
    P, C, J, T = caps
    N = P + C
    d = Draws(seed, cfg_id, episode, env_ids)
    E = d.n
    sc = empty_scene(caps, E)
    n_static = len(statics)
    # --- shapes ---------------------------------------------------------------------------------
    verts = np.zeros((E, P, 4, 2))
    nv = np.full((E, P), 4, dtype=np.int64)
    for i, (cx, cy, hx, hy) in enumerate(statics):
        verts[:, i] = box_verts(hx, hy)
        sc["pos"][:, i] = (cx, cy)
    nd = P - n_static
    if poly_kind == "box":
        hx = d.u(nd, lo=extent[0], hi=extent[1])
        hy = d.u(nd, lo=extent[0], hi=extent[1])
        verts[:, n_static:] = box_verts(hx, hy)
    else:
        verts[:, n_static:], nv[:, n_static:] = _random_hulls(d, nd, extent[0], extent[1])
    density = np.ones((E, N))
    v2, im, ii = polygon_mass_props(verts, nv, density[:, :P])
    radius = d.u(C, lo=circle_r[0], hi=circle_r[1])
    cim, cii = circle_mass_props(radius, density[:, P:])
    sc["verts"], sc["n_verts"], sc["radius"] = v2, nv, radius
    sc["inv_mass"] = np.concatenate([im, cim], 1)
    sc["inv_inertia"] = np.concatenate([ii, cii], 1)
    sc["inv_mass"][:, :n_static] = 0.0
    sc["inv_inertia"][:, :n_static] = 0.0
    sc["density"] = density
    sc["friction"] = d.u(N, lo=friction_range[0], hi=friction_range[1])
    sc["restitution"] = d.u(N, lo=0.0, hi=restitution_hi) if restitution_hi > 0 else np.zeros((E, N))
    sc["restitution"][:, :n_static] = 0.0
    sc["role"] = d.integers(4, N)
    sc["theta"] = d.u(N, lo=-np.pi, hi=np.pi)
    sc["theta"][:, :n_static] = 0.0
    bound = np.concatenate([np.linalg.norm(v2, axis=-1).max(-1), radius], 1)
    fixed_mask = np.zeros(N, dtype=bool)
    fixed_mask[:n_static] = True
    boxes = [(cx - hx, cx + hx, cy - hy, cy + hy) for (cx, cy, hx, hy) in statics]
    pos = _place(d, bound, region, boxes, retries, fixed_mask)
    sc["pos"][:, n_static:] = pos[:, n_static:]
    # --- activity masks ---------------------------------------------------------------------------
    act = np.ones((E, N), dtype=np.int64)
    jact = np.ones((E, J), dtype=np.int64)
    tact = np.ones((E, T), dtype=np.int64)
    if mask_mode == "p15":           # every non-static entity inactive with probability 0.15
        act[:, n_static:] = d.u(N - n_static) >= 0.15
        jact[:] = d.u(J) >= 0.15
        tact[:] = d.u(T) >= 0.15
    elif mask_mode == "keep":        # per-env keep fraction U[0.6, 1.0]
        keep = d.u(lo=0.6, hi=1.0)[:, None]
        act[:, n_static:] = d.u(N - n_static) < keep
        jact[:] = d.u(J) < keep
        tact[:] = d.u(T) < keep
    elif mask_mode == "size":        # heterogeneous batch: S : M : L content = 1 : 1 : 2, padded with masks
        cls = d.integers(4)
        cls = np.where(cls >= 2, 2, cls)
        sizes = np.array([CAPS["S"], CAPS["M"], CAPS["L"]])
        nP, nC, nJ, nT = [sizes[cls, k] for k in range(4)]
        idx = np.arange(N)[None, :]
        # polygons: the floor always; walls only in L content; then the first dynamic polygons
        n_dyn = np.where(cls == 2, nP - 3, nP - 1)
        pa = (idx < P) & (((idx >= n_static) & (idx < n_static + n_dyn[:, None])) | (idx == 0) |
                          ((idx < n_static) & (cls[:, None] == 2)))
        ca = (idx >= P) & (idx < P + nC[:, None])
        act[:] = pa | ca
        jact[:] = np.arange(J)[None, :] < nJ[:, None]
        tact[:] = np.arange(T)[None, :] < nT[:, None]
        sc["size_class"] = cls
    sc["active"] = act
    # --- joints ---------------------------------------------------------------------------------
    n_dynamic = N - n_static
    if J:
        # half extents of every shape in its own frame (anchors are drawn inside them)
        ext = np.concatenate([np.abs(v2).max(-2), np.repeat(radius[..., None], 2, -1) / np.sqrt(2.0)], 1)
        e_all = np.arange(E)
        if chains:
            # articulated chains: joint q links dynamic shape q to dynamic shape q+1 (a new chain starts
            # after at most 4 links)
            ja = n_static + (np.arange(J)[None, :] + np.zeros((E, 1), dtype=np.int64))
            jb = ja + 1
            chain_break = (np.arange(J) % 5 == 4)
        else:
            # shape b of joint q: distinct dynamic shapes (a random permutation); shape a: any shape whose
            # position is already final (static, never a "b", or the b of an earlier joint) -- the way the
            # paper's generator connects a new shape to an existing one
            perm = np.argsort(d.u(n_dynamic), axis=1, kind="stable")
            jb = n_static + perm[:, :J]
            ja = np.zeros((E, J), dtype=np.int64)
            for q in range(J):
                cand = np.ones((E, N), dtype=bool)
                for q2 in range(q, J):
                    cand[e_all, jb[:, q2]] = False
                r = d.integers(N - (J - q))
                ja[:, q] = (np.cumsum(cand, 1) == (r + 1)[:, None]).argmax(1)
        sc["joint_a"], sc["joint_b"] = ja, jb
        fixed = np.broadcast_to(np.asarray(joint_fixed_pattern, dtype=np.int64)[None, :J], (E, J)).copy()
        sc["joint_fixed"] = fixed
        sc["joint_motor_on"] = 1 - fixed
        sc["joint_motor_speed"] = d.u(J, lo=1.0, hi=4.0)
        motor_accel = d.u(J, lo=2.0, hi=10.0)     # rad/s^2 of relative spin at full torque; scaled below
        # Shape b is moved so that its anchor meets a's (joined shapes overlap and do not collide).  As in
        # the paper's generator (Sec. 3.3) a proposed attachment is rejected if it would start in collision
        # (bounding circles against the other placed shapes, bounding circle against the static boxes);
        # after `retries` failed proposals the joint is left inactive and b stays where it was.
        placed = np.ones((E, N), dtype=bool)
        if not chains:
            for q in range(J):
                placed[e_all, jb[:, q]] = False
        joint_ok = np.ones((E, J), dtype=bool)
        for q in range(J):
            a, b = ja[:, q], jb[:, q]
            need = np.ones(E, dtype=bool)
            pos_b = sc["pos"][e_all, b].copy()
            anchor_a = np.zeros((E, 2))
            anchor_b = np.zeros((E, 2))
            for _ in range(max(1, retries)):
                ca = d.u(2, lo=-0.8, hi=0.8) * ext[e_all, a]
                cb = d.u(2, lo=-0.8, hi=0.8) * ext[e_all, b]
                wa = sc["pos"][e_all, a] + _rot(sc["theta"][e_all, a], ca)
                cand = wa - _rot(sc["theta"][e_all, b], cb)
                bad = np.zeros(E, dtype=bool)
                for k, (bx0, bx1, by0, by1) in enumerate(boxes):
                    cx = np.clip(cand[:, 0], bx0, bx1)
                    cy = np.clip(cand[:, 1], by0, by1)
                    bad |= (np.hypot(cand[:, 0] - cx, cand[:, 1] - cy) < bound[e_all, b]) & (a != k)
                if retries > 0:
                    for j in range(n_static, N):
                        hit = np.linalg.norm(cand - sc["pos"][:, j], axis=-1) < bound[e_all, b] + bound[:, j]
                        bad |= hit & placed[:, j] & (a != j) & (b != j) & (act[:, j] > 0)
                take = need & ~bad
                pos_b[take] = cand[take]
                anchor_a[take] = ca[take]
                anchor_b[take] = cb[take]
                need &= bad
                if not need.any():
                    break
            joint_ok[:, q] = ~need
            # a rejected joint still gets consistent anchors (it is inactive, but a caller may switch it on)
            wa = sc["pos"][e_all, a] + _rot(sc["theta"][e_all, a], anchor_a)
            anchor_b[need] = _rot(-sc["theta"][e_all, b], wa - pos_b)[need]
            sc["pos"][e_all, b] = pos_b
            placed[e_all, b] = True
            sc["joint_anchor_a"][:, q] = anchor_a
            sc["joint_anchor_b"][:, q] = anchor_b
            sc["joint_theta_f"][:, q] = sc["theta"][e_all, a] - sc["theta"][e_all, b]
        jact = jact & joint_ok
        # motor power (a torque) in proportion to the reduced inertia of the joined pair, so that light
        # and heavy pairs see the same range of angular accelerations
        ia = np.take_along_axis(sc["inv_inertia"], ja, 1)
        ib = np.take_along_axis(sc["inv_inertia"], jb, 1)
        sc["joint_motor_power"] = motor_accel / np.maximum(ia + ib, 1e-6)
        if chains:
            jact = jact & ~np.broadcast_to(chain_break[None, :], (E, J))
        sc["joint_active"] = jact
    # --- thrusters ------------------------------------------------------------------------------
    if T:
        sc["thruster_body"] = n_static + d.integers(n_dynamic, T)
        text = np.take_along_axis(ext, sc["thruster_body"][..., None], 1) if J else None
        if text is None:
            ext = np.concatenate([np.abs(v2).max(-2), np.repeat(radius[..., None], 2, -1) / np.sqrt(2.0)], 1)
            text = np.take_along_axis(ext, sc["thruster_body"][..., None], 1)
        sc["thruster_pos"] = d.u(T, 2, lo=-0.8, hi=0.8) * text      # mounted inside the shape
        sc["thruster_angle"] = d.u(T, lo=-np.pi, hi=np.pi)
        # thruster power (a force) in proportion to the mass it pushes: 2..15 m/s^2 at full action
        tm = np.take_along_axis(sc["inv_mass"], sc["thruster_body"], 1)
        sc["thruster_power"] = d.u(T, lo=2.0, hi=15.0) / np.maximum(tm, 1e-6)
        sc["thruster_active"] = tact
    return sc


_FLOOR = (2.5, 0.0, 5.0, 0.1)
_WALLS = [(-2.6, 5.0, 0.1, 5.0), (7.6, 5.0, 0.1, 5.0)]


def make_scene(cfg_id, n_envs=None, env_ids=None, episode=0, seed=SEED):
    """Scene description (dict of per-env float64 / int64 arrays, reals already rounded to fp32) for
    BASELINE config `cfg_id` (0..4).  Returns (caps, params, scene)."""
    cfg = CONFIGS[cfg_id]
    caps = CAPS[cfg["size"]]
    if env_ids is None:
        env_ids = np.arange(cfg["n_envs"] if n_envs is None else n_envs)
    params = default_params(cfg["n_substeps"], cfg["n_iters"])
    if cfg_id == 0:
        sc = _generate(0, caps, env_ids, episode, seed, statics=[_FLOOR], poly_kind="box", extent=(0.1, 0.5),
                       circle_r=(0.1, 0.4), region=((1.0, 4.0), (1.0, 4.0)), retries=8,
                       joint_fixed_pattern=[0], mask_mode="none", restitution_hi=0.3,
                       friction_range=(0.5, 0.5))
    elif cfg_id == 1:
        sc = _generate(1, caps, env_ids, episode, seed, statics=[_FLOOR], poly_kind="hull", extent=(1.0, 1.0),
                       circle_r=(0.05, 0.5), region=((1.0, 4.0), (1.0, 4.0)), retries=8,
                       joint_fixed_pattern=[0, 1], mask_mode="p15", restitution_hi=0.3,
                       friction_range=(0.5, 0.5))
    elif cfg_id == 2:
        sc = _generate(2, caps, env_ids, episode, seed, statics=[_FLOOR] + _WALLS, poly_kind="hull",
                       extent=(0.3, 1.0), circle_r=(0.05, 0.5), region=((-1.0, 6.0), (1.2, 5.0)), retries=8,
                       joint_fixed_pattern=[0, 0, 1, 0, 0, 1], mask_mode="keep", restitution_hi=0.3,
                       friction_range=(0.5, 0.5))
    elif cfg_id == 3:
        sc = _generate(3, caps, env_ids, episode, seed, statics=[_FLOOR] + _WALLS, poly_kind="hull",
                       extent=(0.3, 1.0), circle_r=(0.05, 0.5), region=((1.0, 4.0), (1.0, 4.0)), retries=0,
                       joint_fixed_pattern=[0, 0, 1, 0, 0, 1], mask_mode="none", restitution_hi=0.0,
                       friction_range=(0.2, 1.0))
    elif cfg_id == 4:
        sc = _generate(4, caps, env_ids, episode, seed, statics=[_FLOOR] + _WALLS, poly_kind="hull",
                       extent=(0.3, 1.0), circle_r=(0.05, 0.5), region=((-1.0, 6.0), (1.2, 5.0)), retries=8,
                       joint_fixed_pattern=[0, 0, 0, 0, 0, 0], mask_mode="size", restitution_hi=0.3,
                       friction_range=(0.5, 0.5), chains=True)
    else:
        raise ValueError("config id 0..4")
    sc.pop("size_class", None)
    return caps, params, to_f32(sc)


def make_dense_scene(n_envs=None, env_ids=None, episode=0, seed=SEED, pen=(1.6, 3.4)):
    """The contact-heavy variant of workload 3: the same generator (all 16 shapes active, no rejection,
    restitution 0, friction U[0.2, 1]), but the two static walls stand at the edges of a pen only
    `pen[1] - pen[0]` wide, so that the heap cannot spread over the floor and piles up in layers.  What it
    yields (oracle counters): about 14 colliding pairs per environment once settled, up to 21, more than 16
    in a tenth of the environment-steps -- thirteen movable convex shapes in the plane do not touch more
    neighbours than that once they rest.  Returns (caps, params, scene) like make_scene."""
    cfg = CONFIGS[3]
    caps = CAPS[cfg["size"]]
    if env_ids is None:
        env_ids = np.arange(8192 if n_envs is None else n_envs)
    xl, xr = pen
    walls = [(xl - 0.1, 5.0, 0.1, 5.0), (xr + 0.1, 5.0, 0.1, 5.0)]
    sc = _generate(3, caps, np.asarray(env_ids), episode, seed ^ 0x00D0E05E, statics=[_FLOOR] + walls, poly_kind="hull",
                   extent=(0.3, 1.0), circle_r=(0.05, 0.5), region=((xl + 0.3, xr - 0.3), (1.0, 4.0)), retries=0,
                   joint_fixed_pattern=[0, 0, 1, 0, 0, 1], mask_mode="none", restitution_hi=0.0,
                   friction_range=(0.2, 1.0))
    sc.pop("size_class", None)
    return caps, default_params(cfg["n_substeps"], cfg["n_iters"]), to_f32(sc)


def make_stack_scene(n_envs=None, env_ids=None, episode=0, seed=SEED, n_substeps=3, n_iters=10):
    """A stacking workload (the case Appendix A.7 describes: rectangles resting on top of each other, where
    solving one contact disturbs its neighbours): L capacities, the floor and two walls, nine boxes piled
    into one, two or three towers with a little sideways jitter, four balls resting on the floor.  No joint,
    no thruster.  Long dependency chains are the worst case of a level-by-level constraint sweep.
    Returns (caps, params, scene) like make_scene."""
    caps = CAPS["L"]
    P, C, J, T = caps
    N = P + C
    if env_ids is None:
        env_ids = np.arange(1024 if n_envs is None else n_envs)
    env_ids = np.asarray(env_ids)
    E = len(env_ids)
    d = Draws(seed, 5, episode, env_ids)
    sc = empty_scene(caps, E)
    sc["friction"][:] = 0.6
    sc["density"][:] = 1.0
    half = np.zeros((E, P, 2))
    half[:, 0] = (5.0, 0.1)
    half[:, 1] = half[:, 2] = (0.1, 5.0)
    sc["pos"][:, 0] = (2.5, 0.0)
    sc["pos"][:, 1] = (-2.6, 5.0)
    sc["pos"][:, 2] = (7.6, 5.0)
    n_towers = 1 + d.integers(3)                                  # 1..3 towers
    tower = np.minimum((d.u(9) * n_towers[:, None]).astype(np.int64), n_towers[:, None] - 1)
    tower[:, 0] = 0
    hx = d.u(9, lo=0.3, hi=0.5)
    hy = d.u(9, lo=0.1, hi=0.25)
    jitter = d.u(9, lo=-0.05, hi=0.05)
    top = np.full((E, 3), 0.1)                                    # the floor's upper face
    for q in range(9):
        i = 3 + q
        t = tower[:, q]
        half[:, i, 0], half[:, i, 1] = hx[:, q], hy[:, q]
        y = top[np.arange(E), t] + hy[:, q] + 0.001
        sc["pos"][:, i, 0] = 0.5 + 1.6 * t + jitter[:, q]
        sc["pos"][:, i, 1] = y
        top[np.arange(E), t] = y + hy[:, q]
    for i in range(P):
        sc["verts"][:, i] = np.stack([-half[:, i, 0], -half[:, i, 1], half[:, i, 0], -half[:, i, 1],
                                      half[:, i, 0], half[:, i, 1], -half[:, i, 0], half[:, i, 1]], -1).reshape(E, 4, 2)
    sc["n_verts"][:] = 4
    area = 4.0 * half[..., 0] * half[..., 1]
    inertia = area * (4.0 * half[..., 0] ** 2 + 4.0 * half[..., 1] ** 2) / 12.0
    sc["inv_mass"][:, 3:P] = 1.0 / area[:, 3:]
    sc["inv_inertia"][:, 3:P] = 1.0 / inertia[:, 3:]
    r = d.u(C, lo=0.15, hi=0.3)
    sc["radius"][:] = r
    sc["pos"][:, P:, 0] = 5.2 + 0.65 * np.arange(C)[None, :]
    sc["pos"][:, P:, 1] = 0.1 + r + 0.001
    im, ii = circle_mass_props(r, np.ones_like(r))
    sc["inv_mass"][:, P:] = im
    sc["inv_inertia"][:, P:] = ii
    sc["active"][:] = 1
    sc["role"] = d.integers(4, N)
    return caps, default_params(n_substeps, n_iters), to_f32(sc)


def make_actions(cfg_id, n_steps, n_envs, seed=SEED, step0=0):
    """Actions U[-1,1], fp32 values, shape [n_steps, n_envs, J+T]; independent per (step, env)."""
    caps = CAPS[CONFIGS[cfg_id]["size"]]
    A = caps[2] + caps[3]
    out = np.empty((n_steps, n_envs, A), dtype=np.float32)
    ids = np.arange(n_envs)
    for s in range(n_steps):
        d = Draws(seed ^ 0x5A5A5A5A, cfg_id, step0 + s, ids)
        out[s] = d.u(A, lo=-1.0, hi=1.0).astype(np.float32)
    return out


def reset_ids(cfg_id, step, n_envs, frac=0.05, seed=SEED):
    """Environments reset after `step` in the heterogeneous workload: a seeded random 5 %."""
    d = Draws(seed ^ 0x0C0FFEE0, cfg_id, step, np.arange(n_envs))
    return np.nonzero(d.u() < frac)[0].astype(np.int32)
