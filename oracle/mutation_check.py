#!/usr/bin/env python3
"""How much the pins pin: plants one mistake at a time in a copy of the oracle (a dropped term, a wrong sign,
a swapped operand, a wrong index, a transposed order) and runs the CPU test suite against the copy.  A mistake
that no test notices is a gap in the pins.  CPU only; nothing here touches the GPU library.

  python oracle/mutation_check.py [-j 4] [-k name-substring]

Every entry: (name, text in k2d_oracle.cpp that must occur exactly once, replacement)."""
import argparse
import concurrent.futures as cf
import os
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "k2d_oracle.cpp")

MUTANTS = [
    ("gravity sign", "b.vel.y = b.vel.y + R(P.gravity_y) * h;", "b.vel.y = b.vel.y - R(P.gravity_y) * h;"),
    ("gravity on static shapes", "if (b.active && b.inv_mass > R(0)) b.vel.y", "if (b.active) b.vel.y"),
    ("Euler step before the velocities", "    b.pos = b.pos + h * b.vel;\n", "    b.pos = b.pos + (h * R(0.5)) * b.vel;\n"),
    ("Euler step forgets the rotation", "    b.theta = b.theta + h * b.omega;\n", "    b.theta = b.theta;\n"),
    ("edge normal points inward", "wp.nrm[i] = {e.y / len, -e.x / len};", "wp.nrm[i] = {-e.y / len, e.x / len};"),
    ("CC normal from b to a", "V2<R> d = pb - pa;\n  R L = std::sqrt(dot(d, d));", "V2<R> d = pa - pb;\n  R L = std::sqrt(dot(d, d));"),
    ("CC penetration forgets a radius", "m.pen[0] = ra + rb - L;", "m.pen[0] = rb - L;"),
    ("CC contact point on the wrong circle", "m.pos[0] = pa + ra * n;", "m.pos[0] = pb + ra * n;"),
    ("PC projection not clipped to the segment", "t = std::min(std::max(t, R(0)), R(1));", "t = t;"),
    ("PC penetration printed form r_b - |p| of the point", "m.pen[0] = rb - dist;", "m.pen[0] = rb - std::sqrt(dot(q, q));"),
    ("PC inside case takes the wrong face", "if (s > smax) { ssecond = smax; smax = s; imax = i; }", "if (s > smax) { ssecond = smax; smax = s; imax = 0; }"),
    ("PP face query takes the largest distance", "smin = std::min(smin, dot(X.nrm[i], Y.w[k] - X.w[i]));", "smin = std::max(smin == std::numeric_limits<R>::infinity() ? -smin : smin, dot(X.nrm[i], Y.w[k] - X.w[i]));"),
    ("PP separating axis ignored", "if (std::max(sa, sb) >= R(0)) return;  // a separating axis exists: no collision", ""),
    ("PP reference face always a", "bool ref_b = sb > sa + tie_eps;", "bool ref_b = false;"),
    ("PP incident face most parallel", "if (d < dmin) { dsecond = dmin; dmin = d; jinc = j; }", "if (-d < dmin) { dsecond = dmin; dmin = -d; jinc = j; }"),
    ("PP no clipping", "R uc = std::min(std::max(u[k], R(0)), len);", "R uc = u[k];"),
    ("PP normal not flipped for reference b", "m.normal = ref_b ? V2<R>{-nref.x, -nref.y} : nref;", "m.normal = nref;"),
    ("PP penetration sign", "m.pen[k] = -dot(nref, x - r1);", "m.pen[k] = dot(nref, x - r1);"),
    ("impulse forgets the rotation", "b.omega = std::fma(b.inv_inertia, cross(r, j), b.omega);", "b.omega = b.omega;"),
    ("relative velocity forgets w_b x r_b", "return {std::fma(b.omega, rb.y, std::fma(-a.omega, ra.y, a.vel.x) - b.vel.x),", "return {(std::fma(-a.omega, ra.y, a.vel.x) - b.vel.x),"),
    ("normal impulse not clamped", "R ln = std::max(acc.lambda_n[k] + dl, R(0));", "R ln = acc.lambda_n[k] + dl;"),
    ("restitution term dropped", "R dl = row.mass_n * (vn + row.rest + row.bias);", "R dl = row.mass_n * (vn + row.bias);"),
    ("velocity correction dropped", "R dl = row.mass_n * (vn + row.rest + row.bias);", "R dl = row.mass_n * (vn + row.rest);"),
    ("normal impulse on one body only", "  apply_impulse(b, V2<R>{-j.x, -j.y}, row.rb);\n  // friction impulse", "  // friction impulse"),
    ("friction unclipped", "R lt = std::min(std::max(acc.lambda_t[k] + dt_, -lim), lim);", "R lt = acc.lambda_t[k] + dt_;"),
    ("friction clip by the increment", "R lim = cp.mu * ln;", "R lim = cp.mu * dl;"),
    ("friction along the normal", "R vt = dot(cp.t, rel_vel(a, row.ra, b, row.rb));", "R vt = dot(cp.n, rel_vel(a, row.ra, b, row.rb));"),
    ("second manifold point never solved", "  for (int k = 0; k < 2; ++k)\n    if (cp.row[k].active) solve_contact_point(", "  for (int k = 0; k < 1; ++k)\n    if (cp.row[k].active) solve_contact_point("),
    ("friction coefficient: mean instead of root of squares", "cp.mu = std::sqrt(a.friction * a.friction + b.friction * b.friction);", "cp.mu = (a.friction + b.friction) / R(2);"),
    ("restitution: max instead of min", "cp.e = std::min(a.restitution, b.restitution);", "cp.e = std::max(a.restitution, b.restitution);"),
    ("effective mass forgets the inertia of b", "R kn = a.inv_mass + b.inv_mass + ran * ran * a.inv_inertia + rbn * rbn * b.inv_inertia;", "R kn = a.inv_mass + b.inv_mass + ran * ran * a.inv_inertia;"),
    ("lever arm of b from a's centre", "row.rb = m.pos[k] - b.pos;", "row.rb = m.pos[k] - a.pos;"),
    ("slop ignored in the bias", "row.bias = R(P.alpha) * std::max(m.pen[k] - R(P.slop), R(0));", "row.bias = R(P.alpha) * std::max(m.pen[k], R(0));"),
    ("accumulated impulses never wiped", "if (!(P.warm_start && row.active && acc.prev_active[k])) {", "if (!P.warm_start) {"),
    ("restitution below the threshold", "row.rest = (vn0 > R(P.restitution_threshold)) ? cp.e * vn0 : R(0);", "row.rest = cp.e * vn0;"),
    ("warm start applies the normal impulse with the wrong sign", "V2<R> j = (-acc.lambda_n[k]) * cp.n + acc.lambda_t[k] * cp.t;", "V2<R> j = (acc.lambda_n[k]) * cp.n + acc.lambda_t[k] * cp.t;"),
    ("joined shapes collide", "joined[j.a * N + j.b] = joined[j.b * N + j.a] = 1;", "joined[j.a * N + j.b] = 0;"),
    ("joint matrix off-diagonal sign", "jr.k12 = -a.inv_inertia * jr.ra.x * jr.ra.y - b.inv_inertia * jr.rb.x * jr.rb.y;", "jr.k12 = a.inv_inertia * jr.ra.x * jr.ra.y + b.inv_inertia * jr.rb.x * jr.rb.y;"),
    ("joint solve transposed", "V2<R> j{(jr.k22 * rhs.x - jr.k12 * rhs.y) * jr.inv_det, (jr.k11 * rhs.y - jr.k12 * rhs.x) * jr.inv_det};", "V2<R> j{(jr.k11 * rhs.x - jr.k12 * rhs.y) * jr.inv_det, (jr.k22 * rhs.y - jr.k12 * rhs.x) * jr.inv_det};"),
    ("joint anchors not rotated", "jr.ra = turn(a.theta, jt.anchor_a);", "jr.ra = jt.anchor_a;"),
    ("joint velocity correction dropped", "jr.bias = R(P.joint_alpha) * sep;", "jr.bias = R(0) * sep;"),
    ("fixed joint angular sign", "R d = -(a.omega - b.omega + jr.ang_bias) * jr.ang_mass;", "R d = (a.omega - b.omega + jr.ang_bias) * jr.ang_mass;"),
    ("fixed joint forgets its rest angle", "jr.ang_bias = R(P.gamma) * (a.theta - b.theta - jt.theta_f);", "jr.ang_bias = R(P.gamma) * (a.theta - b.theta);"),
    ("joint limit pushes while restoring", "if (!restoring) {", "if (true) {"),
    ("joint limit: lower limit ignored", "else if (rel < jt.limit_lo) jr.lim_excess = rel - jt.limit_lo;", ""),
    ("motor sign", "a.omega = a.omega - a.inv_inertia * motor[q];\n    b.omega = b.omega + b.inv_inertia * motor[q];", "a.omega = a.omega + a.inv_inertia * motor[q];\n    b.omega = b.omega - b.inv_inertia * motor[q];"),
    ("motor without tanh", "motor[q] = jt.motor_power * Fn<R>::tanh(arg) * h;", "motor[q] = jt.motor_power * arg * h;"),
    ("motors applied one after the other", "    motor[q] = jt.motor_power * Fn<R>::tanh(arg) * h;\n  }", "    motor[q] = jt.motor_power * Fn<R>::tanh(arg) * h;\n    E.bodies[jt.a].omega -= E.bodies[jt.a].inv_inertia * motor[q]; E.bodies[jt.b].omega += E.bodies[jt.b].inv_inertia * motor[q]; motor[q] = 0;\n  }"),
    ("thruster at the centre of mass", "apply_impulse(b, imp, r);", "apply_impulse(b, imp, V2<R>{0, 0});"),
    ("thruster direction not rotated with the body", "V2<R> dir = rotate(u.x, u.y, unit(th.angle));", "V2<R> dir = unit(th.angle);"),
    ("positional correction shared equally", "a.pos = a.pos - (a.inv_mass * c) * cp.n;", "a.pos = a.pos - (b.inv_mass * c) * cp.n;"),
    ("positional correction from the shallowest point", "for (int k = 0; k < 2; ++k) if (m.active[k]) pen = std::max(pen, m.pen[k]);", "pen = std::numeric_limits<R>::infinity(); for (int k = 0; k < 2; ++k) if (m.active[k]) pen = std::min(pen, m.pen[k]);"),
    ("joint positional correction dropped", "V2<R> c = (R(P.joint_beta) / (a.inv_mass + b.inv_mass)) * (xa - xb);", "V2<R> c = R(0) * (xa - xb);"),
    ("sweeps: collisions before joints", "    for (int q = 0; q < nJ; ++q)\n      if (jrs[q].live) solve_joint(E, E.joints[q], jrs[q]);\n    if (P.batch_size > 0) {", "    if (P.batch_size > 0) {"),
    ("level order: one past the last predecessor", "      while ((busy >> lv) & 1u) ++lv;\n      if (movable(cps[q].a)) taken[cps[q].a] |= 1u << lv;", "      while ((busy >> lv) != 0u) ++lv;\n      if (movable(cps[q].a)) taken[cps[q].a] |= 1u << lv;"),
    ("level order: static shapes tie pairs together", "unsigned busy = (movable(cps[q].a) ? taken[cps[q].a] : 0u) | (movable(cps[q].b) ? taken[cps[q].b] : 0u);", "unsigned busy = taken[cps[q].a] | taken[cps[q].b]; taken[cps[q].a] |= 1u << 0; "),
    ("tournament order: last round first", "      else { x = (r + k) % (m - 1); y = ((r - k) % (m - 1) + (m - 1)) % (m - 1); }", "      else { x = (r + k) % (m - 1); y = ((r - k) % (m - 1) + (m - 1)) % (m - 1); std::swap(x, y); x = (x + 1) % (m - 1); y = (y + 1) % (m - 1); }"),
    ("batches: impulses applied in reverse point order", "    for (const Pending& p : pend) {", "    std::reverse(pend.begin(), pend.end());\n    for (const Pending& p : pend) {"),
    ("batches: solved on the bodies themselves, not on private copies", "Body<R> a = E.bodies[cp.a], bb = E.bodies[cp.b];   // private copies: the batch's starting velocities", "Body<R>& a = E.bodies[cp.a]; Body<R>& bb = E.bodies[cp.b];"),
    ("batches: consecutive points share a batch", "    for (int s = b; s < n_points; s += n_b) {", "    for (int s = b * B; s < std::min(n_points, (b + 1) * B); ++s) {"),
    ("substep length ignores the number of substeps", "const R h = R(P.dt) / R(P.n_substeps);", "const R h = R(P.dt);"),
    ("joint accumulators kept without warm starting", "if (!P.warm_start) { jt.acc = {0, 0}; jt.acc_ang = 0; }", ""),
    ("joint warm start with the wrong sign on b", "      apply_impulse(b, V2<R>{-jt.acc.x, -jt.acc.y}, jrs[q].rb);\n    }\n  }", "      apply_impulse(b, V2<R>{jt.acc.x, jt.acc.y}, jrs[q].rb);\n    }\n  }"),
    ("thruster clip clamps to [-1, 1]", "if (P.clip_thruster_01) A = std::min(std::max(A, R(0)), R(1));", "if (P.clip_thruster_01) A = std::min(std::max(A, R(-1)), R(1));"),
    ("pair count counts pairs, not points", "out[(long)e * NP + p] = envs[e].manifolds[p].active[0] + envs[e].manifolds[p].active[1];", "out[(long)e * NP + p] = envs[e].manifolds[p].active[0] || envs[e].manifolds[p].active[1];"),
    ("adjacency one-sided", "if (m.active[0] || m.active[1]) { adj[i] |= 1u << j; adj[j] |= 1u << i; }", "if (m.active[0] || m.active[1]) { adj[i] |= 1u << j; }"),
    ("collision active at zero penetration", "m.active[k] = m.valid[k] && m.pen[k] > R(0);", "m.active[k] = m.valid[k] && m.pen[k] >= R(-1e-3);"),
    ("static-static pairs eligible", "m.eligible = a.active && b.active && !joined[i * N + j] && (a.inv_mass + b.inv_mass) > R(0);", "m.eligible = a.active && b.active && !joined[i * N + j];"),
    ("observation: sin and cos of the rotation swapped", "        { V2<R> u = unit(b.theta); *o++ = u.y; *o++ = u.x; }", "        { V2<R> u = unit(b.theta); *o++ = u.x; *o++ = u.y; }"),
    ("observation: joint rotation b - a", "R rel = E.bodies[ja].theta - E.bodies[jb].theta;\n        *o++ = j.active;", "R rel = E.bodies[jb].theta - E.bodies[ja].theta;\n        *o++ = j.active;"),
    ("observation: thruster power and position swapped", "*o++ = t.active; *o++ = t.pos.x; *o++ = t.pos.y; *o++ = t.power;", "*o++ = t.active; *o++ = t.power; *o++ = t.pos.x; *o++ = t.pos.y;"),
    ("observation: restitution before friction", "*o++ = b.friction; *o++ = b.restitution;", "*o++ = b.restitution; *o++ = b.friction;"),
    ("observation: angular velocity not scaled", "*o++ = Fn<R>::tanh(b.omega / R(10));", "*o++ = Fn<R>::tanh(b.omega);"),
]


# Mistakes that change nothing but the order in which fp32 roundings happen: no closed form or invariant sees
# them; they are held only by the bit-for-bit comparison of the two implementations (the GPU tests).
ROUNDING_ORDER_ONLY = {"batches: impulses applied in reverse point order"}


# The same for the numpy statement of the environment layer (oracle/k2d_env.py: reward and termination, entity
# observation and masks, multi-discrete actions, health).
ENV_SRC = os.path.join(HERE, "k2d_env.py")
ENV_MUTANTS = [
    ("reward: red counts as the goal", "sparse = f(1) if goal else (f(-1) if bad else f(0))", "sparse = f(1) if (goal or bad) else f(0)"),
    ("reward: red wins over blue", "sparse = f(1) if goal else (f(-1) if bad else f(0))", "sparse = f(-1) if bad else (f(1) if goal else f(0))"),
    ("reward: dense term with the wrong sign", "dense = f(f(kappa) * f(f(d_prev[e]) - d_new[e]))", "dense = f(f(kappa) * f(d_new[e] - f(d_prev[e])))"),
    ("reward: dense term on the first step", "if d_prev[e] >= 0 and best is not None:", "if best is not None:"),
    ("reward: largest distance over the pairs", "best = d if best is None or d < best else best", "best = d if best is None or d > best else best"),
    ("reward: inactive shapes count", "if j == i or not active[e, j]:", "if j == i:"),
    ("reward: any shape may reach the goal", "if not active[e, i] or role[e, i] != green:", "if not active[e, i]:"),
    ("reward: episode does not end on red", "done[e] = 1 if (goal or bad) else 0", "done[e] = 1 if goal else 0"),
    ("actions: motor directions swapped", "np.where(m == 1, 1.0, np.where(m == 2, -1.0, 0.0))", "np.where(m == 1, -1.0, np.where(m == 2, 1.0, 0.0))"),
    ("actions: thruster on at 2", "np.where(d[..., J:] == 1, 1.0, 0.0)", "np.where(d[..., J:] == 2, 1.0, 0.0)"),
    ("entities: role one-hot shifted", "s[8 + role] = 1.0", "s[8 + (role + 1) % N_ROLES] = 1.0"),
    ("entities: type one-hot swapped", "s[16 if i >= P else 17] = 1.0", "s[17 if i >= P else 16] = 1.0"),
    ("entities: triangle and rectangle swapped", "s[27 if int(f[20]) == 3 else 28] = 1.0", "s[28 if int(f[20]) == 3 else 27] = 1.0"),
    ("entities: reversed joint keeps its anchors", "g[2:4], g[4:6] = f[4:6], f[2:4]", "g[2:4], g[4:6] = f[2:4], f[4:6]"),
    ("entities: reversed joint keeps its rotation", "g[9] = -f[9]", "g[9] = f[9]"),
    ("entities: reversed joint's shapes not swapped", "jidx[e, 2 * q + 1] = (b, a)", "jidx[e, 2 * q + 1] = (a, b)"),
    ("masks: joints on inactive shapes count", "if f[0] != 0 and act[a] and act[b] and a != b:", "if f[0] != 0 and a != b:"),
    ("masks: joint mask one-sided", "                direct[b] |= 1 << a\n", "                pass\n"),
    ("masks: no transitive closure", "                    reach[i] |= reach[k]", "                    reach[i] |= 0"),
    ("masks: collision mask is the joint mask", "masks[e, 3, i] = int(shape_adj[e, i])", "masks[e, 3, i] = direct[i]"),
    ("masks: inactive shapes attend", "masks[e, 0, i] = full if act[i] else 0", "masks[e, 0, i] = full"),
    ("health: inactive shapes count", "bad = ((~finite) & (np.asarray(active) != 0)).any(-1)", "bad = (~finite).any(-1)"),
    ("health: infinities pass", "np.isfinite(pos).all(-1) & np.isfinite(theta)", "(~np.isnan(pos)).all(-1) & np.isfinite(theta)"),
]

_ENV_RUNNER = """
import sys, importlib.util
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import oracle, pytest
spec = importlib.util.spec_from_file_location("oracle.k2d_env", {mut!r})
m = importlib.util.module_from_spec(spec)
sys.modules["oracle.k2d_env"] = m
spec.loader.exec_module(m)
oracle.k2d_env = m
sys.exit(pytest.main([{tests!r}, "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"]))
"""


def run_env_one(entry):
    name, old, new = entry
    text = open(ENV_SRC).read()
    if text.count(old) != 1:
        return name, "SKIPPED (text occurs %d times)" % text.count(old), ""
    with tempfile.TemporaryDirectory(prefix="k2d_mut_") as tmp:
        mut = os.path.join(tmp, "k2d_env.py")
        open(mut, "w").write(text.replace(old, new))
        code = _ENV_RUNNER.format(root=ROOT, tests=os.path.join(ROOT, "tests"), mut=mut)
        r = subprocess.run([sys.executable, "-c", code], cwd=tmp, capture_output=True, text=True)
        tail = [l for l in r.stdout.splitlines() if l.startswith(("FAILED", "ERROR"))]
        if r.returncode == 0:
            return name, "SURVIVED", ""
        return name, "noticed", tail[0] if tail else (r.stdout + r.stderr)[-200:]


def run_one(entry, pytest_args):
    name, old, new = entry
    text = open(SRC).read()
    if text.count(old) != 1:
        return name, "SKIPPED (text occurs %d times)" % text.count(old), ""
    with tempfile.TemporaryDirectory(prefix="k2d_mut_") as tmp:
        src = os.path.join(tmp, "k2d_oracle.cpp")
        open(src, "w").write(text.replace(old, new))
        env = dict(os.environ, K2D_ORACLE_SOURCE=src)
        r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests"), "-x", "-q", "-m", "not gpu",
                            "-p", "no:cacheprovider"] + pytest_args, cwd=tmp, env=env, capture_output=True, text=True)
        tail = [l for l in r.stdout.splitlines() if l.startswith(("FAILED", "ERROR"))]
        if r.returncode == 0:
            return name, "SURVIVED", ""
        if "error:" in r.stdout + r.stderr and not tail:
            return name, "DID NOT COMPILE", (r.stdout + r.stderr)[-400:]
        return name, "noticed", tail[0] if tail else r.stdout[-200:]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("-j", type=int, default=4)
    ap.add_argument("-k", default="")
    args = ap.parse_args()
    todo = [m for m in MUTANTS if args.k in m[0]]
    todo_env = [m for m in ENV_MUTANTS if args.k in m[0]]
    survived = 0
    with cf.ThreadPoolExecutor(args.j) as ex:
        results = list(ex.map(lambda m: run_one(m, []), todo)) + list(ex.map(run_env_one, todo_env))
        for name, verdict, detail in results:
            if verdict == "SURVIVED" and name in ROUNDING_ORDER_ONLY:
                verdict = "survived (rounding order only; held by the bit-identity tests)"
            else:
                survived += verdict != "noticed"
            print("%-58s %s  %s" % (name, verdict, detail.replace(ROOT + "/", "")[:120]), flush=True)
    print("%d planted mistakes, %d not noticed" % (len(todo) + len(todo_env), survived))
    return 1 if survived else 0


if __name__ == "__main__":
    sys.exit(main())
