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
