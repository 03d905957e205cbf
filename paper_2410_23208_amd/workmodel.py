"""Algorithmic work of one environment-step: the arithmetic the method itself asks for.

Counting rule: add / sub / mul / div / sqrt / sin / cos / tanh = 1 each; min, max, compare, select, negate = 0.
What is counted is what Algorithm 1 (Appendix A) must evaluate for the scene at hand: world transforms
of the active polygons, the manifold of every *eligible* pair (both shapes active, not joined, not both
static), and constraint work only for *active* manifold points and *live* joints.  Padding, masked-off
lanes, culling tests and the paper's own solve-every-pair-every-sweep (A.8) are not counted.  The per-unit
figures below were counted by hand from the formulas as the CPU oracle writes them out.
"""
import numpy as np

# per-unit operation counts
F_GRAVITY = 2                     # per active dynamic shape
F_WORLD = lambda n: 2 + 16 * n    # per active polygon: sin, cos; 8 per vertex; 8 per edge normal
F_CC = 14                         # circle-circle manifold (A.3.2)
F_PC = lambda n: 23 * n + 6       # polygon-circle manifold, n edges (A.3.3)
F_PP_SAT = lambda na, nb: 10 * na * nb   # both face queries of the separating-axis search (A.3.4)
F_PP_CLIP = 50                    # reference/incident choice, clipping, two penetrations (overlapping pairs)
F_PRESOLVE_SLOT = 48              # r_a, r_b, both effective masses, bias, restitution sample
F_PRESOLVE_PAIR = 8               # mu, positional-correction length
F_WARM_SLOT = 24
F_SOLVE_SLOT = 75                 # normal (38) + friction (37) impulse of one point in one sweep
F_JOINT_PRE = 51
F_JOINT_WARM = 18
F_JOINT_WARM_FIXED = 4
F_JOINT_SOLVE = 40
F_JOINT_SOLVE_FIXED = 8
F_MOTOR = 11
F_THRUSTER = 29
F_INTEGRATE = 6                   # per active shape
F_POSCORR_PAIR = 10
F_POSCORR_JOINT = 34


def static_counts(caps, scene):
    """Per-environment counts that are fixed by the scene description (numpy, vectorised)."""
    P, C, J, T = caps
    N = P + C
    act = np.asarray(scene["active"]) != 0
    im = np.asarray(scene["inv_mass"])
    E = act.shape[0]
    e_idx = np.arange(E)
    ja = np.clip(np.asarray(scene["joint_a"]), 0, N - 1)
    jb = np.clip(np.asarray(scene["joint_b"]), 0, N - 1)
    jlive = ((np.asarray(scene["joint_active"]) != 0) & (ja != jb) & act[e_idx[:, None], ja] &
             act[e_idx[:, None], jb] & ((im[e_idx[:, None], ja] + im[e_idx[:, None], jb]) > 0))
    joined = np.zeros((E, N, N), dtype=bool)
    for q in range(J):
        m = jlive[:, q]
        joined[e_idx[m], ja[m, q], jb[m, q]] = True
        joined[e_idx[m], jb[m, q], ja[m, q]] = True
    elig = act[:, :, None] & act[:, None, :] & ~joined & ((im[:, :, None] + im[:, None, :]) > 0)
    iu = np.triu(np.ones((N, N), dtype=bool), 1)
    elig &= iu[None]
    nv = np.asarray(scene["n_verts"]).astype(np.int64)
    nvN = np.concatenate([nv, np.zeros((E, C), dtype=np.int64)], 1)
    f_pairs = np.zeros(E)
    pp = elig[:, :P, :P]
    f_pairs += (pp * (10 * nv[:, :, None] * nv[:, None, :])).sum((1, 2))
    pc = elig[:, :P, P:]
    f_pairs += (pc * (23 * nv[:, :, None] + 6)).sum((1, 2))
    f_pairs += F_CC * elig[:, P:, P:].sum((1, 2))
    fixed = np.asarray(scene["joint_fixed"]) != 0
    motor = jlive & ~fixed & (np.asarray(scene["joint_motor_on"]) != 0)
    tb = np.clip(np.asarray(scene["thruster_body"]), 0, N - 1)
    thr = (np.asarray(scene["thruster_active"]) != 0) & act[e_idx[:, None], tb]
    return dict(
        n_active=act.sum(1), n_dynamic=(act & (im > 0)).sum(1),
        f_world=(act[:, :P] * (2 + 16 * nv)).sum(1), f_manifolds=f_pairs, n_eligible=elig.sum((1, 2)),
        n_joint_live=jlive.sum(1), n_joint_fixed=(jlive & fixed).sum(1), n_motor=motor.sum(1), n_thruster=thr.sum(1))


def flops_per_env_step(caps, scene, params, slots_per_substep, pairs_per_substep, pp_overlap_per_substep):
    """Mean algorithmic flops of one environment-step of this workload.  The three dynamic figures are
    means per environment-substep (active manifold points, pairs with an active point, overlapping
    polygon pairs), measured on a CPU run of the same scenes."""
    st = static_counts(caps, scene)
    n_it = params["n_iters"]
    ws = 1 if params["warm_start"] else 0
    per_sub = (F_GRAVITY * st["n_dynamic"] + st["f_world"] + st["f_manifolds"]
               + st["n_joint_live"] * (F_JOINT_PRE + ws * F_JOINT_WARM + n_it * F_JOINT_SOLVE + F_POSCORR_JOINT)
               + st["n_joint_fixed"] * (ws * F_JOINT_WARM_FIXED + n_it * F_JOINT_SOLVE_FIXED)
               + F_MOTOR * st["n_motor"] + F_THRUSTER * st["n_thruster"] + F_INTEGRATE * st["n_active"]).mean()
    per_sub += F_PP_CLIP * pp_overlap_per_substep
    per_sub += slots_per_substep * (F_PRESOLVE_SLOT + ws * F_WARM_SLOT + n_it * F_SOLVE_SLOT)
    per_sub += pairs_per_substep * (F_PRESOLVE_PAIR + F_POSCORR_PAIR)
    return float(per_sub * params["n_substeps"]), {k: float(np.mean(v)) for k, v in st.items()}


# ---------------------------------------------------------------------------------------------------
# Two more figures for the benchmark line, both from states of a CPU run sampled along the rollout.
# ---------------------------------------------------------------------------------------------------
CULL_MARGIN = 1e-3   # the step kernel grows every bounding box by this much before its overlap test


def _eligible(caps, scene):
    P, C, J, T = caps
    N = P + C
    act = np.asarray(scene["active"]) != 0
    im = np.asarray(scene["inv_mass"])
    E = act.shape[0]
    e_idx = np.arange(E)
    ja = np.clip(np.asarray(scene["joint_a"]), 0, N - 1)
    jb = np.clip(np.asarray(scene["joint_b"]), 0, N - 1)
    jlive = ((np.asarray(scene["joint_active"]) != 0) & (ja != jb) & act[e_idx[:, None], ja] &
             act[e_idx[:, None], jb] & ((im[e_idx[:, None], ja] + im[e_idx[:, None], jb]) > 0))
    joined = np.zeros((E, N, N), dtype=bool)
    for q in range(J):
        m = jlive[:, q]
        joined[e_idx[m], ja[m, q], jb[m, q]] = True
        joined[e_idx[m], jb[m, q], ja[m, q]] = True
    elig = act[:, :, None] & act[:, None, :] & ~joined & ((im[:, :, None] + im[:, None, :]) > 0)
    return elig & np.triu(np.ones((N, N), dtype=bool), 1)[None], jlive, ja, jb


def executed_manifold_flops(caps, scene, pos, theta):
    """Arithmetic of the manifolds the step kernel really evaluates in one substep: those of the eligible
    pairs whose bounding boxes (grown by CULL_MARGIN) overlap -- the kernel's cull, re-stated in numpy on a
    sampled state (pos [E, N, 2], theta [E, N]).  Returns (mean flops per environment, mean survivors)."""
    P, C, J, T = caps
    N = P + C
    E = pos.shape[0]
    elig, _, _, _ = _eligible(caps, scene)
    verts = np.asarray(scene["verts"]).reshape(E, P, 4, 2)
    nv = np.asarray(scene["n_verts"]).astype(np.int64)
    c, s = np.cos(theta[:, :P]), np.sin(theta[:, :P])
    wx = pos[:, :P, None, 0] + c[..., None] * verts[..., 0] - s[..., None] * verts[..., 1]
    wy = pos[:, :P, None, 1] + s[..., None] * verts[..., 0] + c[..., None] * verts[..., 1]
    tri = nv == 3
    wx[tri, 3] = wx[tri, 0]
    wy[tri, 3] = wy[tri, 0]
    lo = np.zeros((E, N, 2))
    hi = np.zeros((E, N, 2))
    lo[:, :P, 0], hi[:, :P, 0], lo[:, :P, 1], hi[:, :P, 1] = wx.min(-1), wx.max(-1), wy.min(-1), wy.max(-1)
    r = np.asarray(scene["radius"])
    lo[:, P:], hi[:, P:] = pos[:, P:] - r[..., None], pos[:, P:] + r[..., None]
    lo -= CULL_MARGIN
    hi += CULL_MARGIN
    ov = ((lo[:, :, None, 0] <= hi[:, None, :, 0]) & (lo[:, None, :, 0] <= hi[:, :, None, 0]) &
          (lo[:, :, None, 1] <= hi[:, None, :, 1]) & (lo[:, None, :, 1] <= hi[:, :, None, 1])) & elig
    f = (ov[:, :P, :P] * (10 * nv[:, :, None] * nv[:, None, :])).sum((1, 2)).astype(np.float64)
    f += (ov[:, :P, P:] * (23 * nv[:, :, None] + 6)).sum((1, 2))
    f += F_CC * ov[:, P:, P:].sum((1, 2))
    return float(f.mean()), float(ov.sum((1, 2)).mean())


# Instructions one wavefront must issue one after the other for a constraint visit (counted from the
# formulas: one instruction per add, multiply or fused multiply-add), whatever the number of lanes it uses.
I_POINT_VISIT = 54        # normal row then friction row of one manifold point (A.3.5, A.3.6)
I_JOINT_VISIT = 31        # point row of a joint (A.4.1)
I_JOINT_FIXED = 8         # angular row of a fixed joint (A.4.2)
I_POINT_WARM = 12         # re-applying the accumulated impulses of one manifold point (A.7)
I_JOINT_WARM = 12


def sequential_chain_instructions(caps, scene, params, pair_points, schedule):
    """Length, in instructions, of the chain of constraint visits that the sweep order forces to run one
    after the other in one substep of every environment: constraints that share a movable shape keep their
    order (joints in index order; collisions in tournament order, or -- params["sweep_order"] = 1 -- level
    after level, a pair taking the lowest level that no earlier colliding pair of the tournament order sharing
    a movable shape with it has; Algorithm 1 and A.8), the others may run side by side.  pair_points [E, n_pairs] = active manifold points per pair
    (lexicographic pair order) of a sampled substep; schedule = (a[], b[]) tournament order.  A visit of a pair costs its points one
    after the other; a level costs its longest visit.  Returns an array [E]: instructions per substep for
    warm starting plus `n_iters` sweeps -- at best one instruction every four clocks on one wavefront."""
    P, C, J, T = caps
    N = P + C
    E = pair_points.shape[0]
    _, jlive, ja, jb = _eligible(caps, scene)
    act = np.asarray(scene["active"]) != 0
    movable = act & ((np.asarray(scene["inv_mass"]) != 0) | (np.asarray(scene["inv_inertia"]) != 0))
    fixed = np.asarray(scene["joint_fixed"]) != 0
    sa, sb = schedule
    pidx = [a * (2 * N - a - 1) // 2 + (b - a - 1) for a, b in zip(sa, sb)]
    out = np.zeros(E)
    for e in range(E):
        nxt = np.zeros(N, dtype=np.int64)        # joints: next free level of every shape
        jl_cost = {}
        for q in range(J):
            if not jlive[e, q]:
                continue
            a, b = ja[e, q], jb[e, q]
            lv = max(nxt[a] if movable[e, a] else 0, nxt[b] if movable[e, b] else 0)
            jl_cost[lv] = max(jl_cost.get(lv, 0), I_JOINT_VISIT + (I_JOINT_FIXED if fixed[e, q] else 0))
            if movable[e, a]:
                nxt[a] = lv + 1
            if movable[e, b]:
                nxt[b] = lv + 1
        taken = [0] * N                          # collisions: levels already taken at every shape
        pl_pts = {}
        for a, b, pi in zip(sa, sb, pidx):
            npt = int(pair_points[e, pi])
            if npt == 0:
                continue
            busy = (taken[a] if movable[e, a] else 0) | (taken[b] if movable[e, b] else 0)
            if params.get("sweep_order", 0) == 1:      # level order: the lowest free level
                lv = 0
                while (busy >> lv) & 1:
                    lv += 1
            else:                                      # tournament order: one past the last pair it must wait for
                lv = busy.bit_length()
            pl_pts[lv] = max(pl_pts.get(lv, 0), npt)
            if movable[e, a]:
                taken[a] |= 1 << lv
            if movable[e, b]:
                taken[b] |= 1 << lv
        sweep = sum(jl_cost.values()) + I_POINT_VISIT * sum(pl_pts.values())
        warm = (I_JOINT_WARM * len(jl_cost) + I_POINT_WARM * sum(pl_pts.values())) if params["warm_start"] else 0
        out[e] = params["n_iters"] * sweep + warm
    return out
