// k2d_oracle.cpp -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
//
// A plain, slow, one-environment-at-a-time CPU statement of the batched 2D rigid-body step that the
// paper's physics engine runs for every environment (Appendix A, Algorithm 1): gravity, collision
// manifolds for every pair of shapes, motors, thrusters, warm starting, `n_iters` sweeps of
// (joint constraints, then collision constraints), an Euler step of position and rotation, and the
// positional corrections.  Only tests, the smoke check and the CPU-baseline leg of the benchmark may
// call this library; the GPU library never does and shares no source, header, table or constant with it.
//
// Every routine names the passage of the paper it follows.  Where the paper is silent the reading taken
// is stated in the comment beside the code (the full list lives in the repository's design notes).
//
// The arithmetic type is a template parameter: `float` is the precision the engine computes in (and the
// precision in which every discrete decision -- contact active or not, reference face, incident face --
// is taken when results are compared with the GPU); `double` exists to measure how much of any
// difference is plain fp32 rounding.
//
// Pins (tests/test_oracle_*.py): closed-form free fall under semi-implicit Euler, head-on circle
// collisions with restitution, box resting on a floor, energy non-increase without actuation,
// pendulum drift and period, motor tanh law, thruster closed form, warm-start bookkeeping, brute-force
// point-sampled overlap for the narrowphase, hand-evaluated manifolds, the visiting order of the sweep
// (levels recomputed from the colliding set, four balls in a row in closed form, level-at-once == sequential),
// joint limits (closed form of one visit, symmetry, restoring motion untouched), towers of boxes standing,
// batched impulse resolution (closed form of two constraints on one body solved in one batch, batch size 1
// == sequential, momentum, the stability trade-off of A.8 on the towers).
// Unpinned by the paper (no values printed there): the coefficients alpha, beta, gamma, rho, the
// penetration slop, the restitution threshold and the reference-face tie margin; they are pinned only
// through the invariants above ("parity unpinned" for their numeric values).
//
// Rounding: the paper gives formulas, not the rounding of their evaluation.  Here two-term products (dot
// and cross products, rotations, "v + j/m", the relative velocity of A.3.5) are evaluated with one fused
// multiply-add, everything else one operation at a time (built with -ffp-contract=off); sin, cos and
// tanh in fp32 are fixed operation sequences of their own.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <string>
#include <thread>
#include <vector>

namespace {

// ----------------------------------------------------------------------------------------------
// Parameters of the step.  The paper names the coefficients (A.3.7: alpha, beta; A.4.2: gamma;
// A.5: rho; Algorithm 1: num_solver_steps, warm starting) but prints no values.
// ----------------------------------------------------------------------------------------------
struct Params {
  double dt = 1.0 / 60.0;
  double gravity_y = -9.81;
  int n_substeps = 1;
  int n_iters = 5;
  int warm_start = 1;
  double alpha = 6.0;                  // contact velocity-correction coefficient, 1/s   (A.3.7)
  double beta = 0.2;                   // contact positional-correction coefficient       (A.3.7)
  double gamma = 6.0;                  // fixed-joint angular correction, 1/s             (A.4.2)
  double rho = 1.0;                    // motor tanh sharpness                            (A.5)
  double slop = 0.005;                 // penetration left uncorrected (0 = literal paper)
  double restitution_threshold = 1.0;  // approach speed below which e is taken as 0
  int clip_thruster_01 = 0;            // clamp thruster actions to [0,1] (env-level range, Sec. 3.2)
  double joint_alpha = 6.0;            // joint point-constraint velocity correction, 1/s (A.4.1)
  double joint_beta = 0.2;             // joint positional correction                     (A.4.1)
  double tie_eps = 1e-3;               // reference face goes to b only if sep_b > sep_a + tie_eps
  int order_mode = 0;                  // 0: one pair after the other; 1 (test): every group of the visiting order
                                       // (a round, or a level) from one snapshot of the bodies
  int batch_size = 0;                  // 0: sequential sweep; B >= 1: batched impulse resolution (A.8)
  int sweep_order = 0;                 // visiting order of the colliding pairs: 0 = tournament order,
                                       // 1 = level after level (lowest free level), see substep()
};
constexpr int kNumParams = 18;

template <class R>
struct V2 {
  R x, y;
};
template <class R> inline V2<R> operator+(V2<R> a, V2<R> b) { return {a.x + b.x, a.y + b.y}; }
template <class R> inline V2<R> operator-(V2<R> a, V2<R> b) { return {a.x - b.x, a.y - b.y}; }
template <class R> inline V2<R> operator*(R s, V2<R> a) { return {s * a.x, s * a.y}; }
// The two-term products below (dot, cross, rotation, "v + s*j") round once: they are written with the
// fused multiply-add every current CPU and GPU has, p*q + r*s = fma(p, q, r*s).  Everything else in this
// file is plain one-operation-one-rounding arithmetic (the build switches contraction off).
template <class R> inline R dot(V2<R> a, V2<R> b) { return std::fma(a.x, b.x, a.y * b.y); }
// vector x vector -> scalar, scalar x vector -> vector (A.2: "the choice should be inferable")
template <class R> inline R cross(V2<R> a, V2<R> b) { return std::fma(a.x, b.y, -(a.y * b.x)); }
template <class R> inline V2<R> cross(R w, V2<R> r) { return {-w * r.y, w * r.x}; }
template <class R> inline V2<R> rotate(R c, R s, V2<R> l) { return {std::fma(c, l.x, -(s * l.y)), std::fma(s, l.x, c * l.y)}; }
// v + s*j
template <class R> inline V2<R> madd(V2<R> v, R s, V2<R> j) { return {std::fma(s, j.x, v.x), std::fma(s, j.y, v.y)}; }

// ----------------------------------------------------------------------------------------------
// sin, cos and tanh.  In double they are libm's.  In fp32 -- the engine's precision -- they are fixed
// sequences of IEEE fp32 operations (round-to-nearest, no fused multiply-add), so that every
// implementation of the engine that performs the same sequence gets the same bits whatever maths
// library it links: quadrant reduction with a three-term split of pi/2 followed by polynomials in r^2
// for sin and cos; tanh from a polynomial below 0.55 and from 1 - 2/(e^{2|x|} + 1) above, e^t by
// reduction with a two-term split of ln 2 and a polynomial.  The coefficients are least-squares fits
// on Chebyshev nodes.  Pinned against libm in double: |error| < 1.5e-7 (tests/test_oracle_math.py).
// ----------------------------------------------------------------------------------------------
template <class R>
struct Fn {
  static void sincos(R x, R& s, R& c) { s = std::sin(x); c = std::cos(x); }
  static R tanh(R x) { return std::tanh(x); }
};
template <>
struct Fn<float> {
  static void sincos(float x, float& sn, float& cs) {
    const float k = std::nearbyint(x * 0x1.45f306p-1f);                       // x * 2/pi, to nearest even
    float r = x - k * 0x1.92p+0f;                                             // pi/2 = 1.5703125
    r = r - k * 0x1.fb4p-12f;                                                 //      + 4.8375130e-4
    r = r - k * 0x1.4442d2p-24f;                                              //      + 7.5497901e-8
    const float z = r * r;
    const float ps = (-0x1.9b021cp-13f * z + 0x1.110ccap-7f) * z + -0x1.555554p-3f;
    const float pc = (0x1.9c05c8p-16f * z + -0x1.6c1354p-10f) * z + 0x1.555554p-5f;
    const float s = r + (r * z) * ps;
    const float c = (1.0f - 0.5f * z) + (z * z) * pc;
    switch (static_cast<int>(k) & 3) {
      case 0: sn = s; cs = c; break;
      case 1: sn = c; cs = -s; break;
      case 2: sn = -s; cs = -c; break;
      default: sn = -c; cs = s; break;
    }
  }
  static float tanh(float x) {
    const float a = std::fabs(x);
    float y;
    if (a < 0.55f) {
      const float z = a * a;
      const float p = (((-0x1.b3b502p-8f * z + 0x1.5d873cp-6f) * z + -0x1.b9aa82p-5f) * z + 0x1.111018p-3f) * z +
                      -0x1.555554p-2f;
      y = a + (a * z) * p;
    } else {
      const float t2 = 2.0f * a;
      const float t = (t2 < 40.0f) ? t2 : 40.0f;
      const float n = std::nearbyint(t * 0x1.715476p+0f);                      // t * log2(e)
      float r = t - n * 0x1.62cp-1f;                                           // ln 2 = 0.69287109375
      r = r - n * 0x1.217f7ep-12f;                                             //      + 2.7608682e-4
      const float p = (((0x1.6d435ap-10f * r + 0x1.120b66p-7f) * r + 0x1.5554e8p-5f) * r + 0x1.5554dcp-3f) * r + 0.5f;
      float e = (1.0f + r) + (r * r) * p;
      e = std::ldexp(e, static_cast<int>(n));
      y = 1.0f - 2.0f / (e + 1.0f);
    }
    return x < 0.0f ? -y : y;
  }
};

// (cos, sin) of an angle, and a vector turned by an angle
template <class R> inline V2<R> unit(R angle) { R s, c; Fn<R>::sincos(angle, s, c); return {c, s}; }
template <class R> inline V2<R> turn(R angle, V2<R> l) { V2<R> u = unit(angle); return rotate(u.x, u.y, l); }

// ----------------------------------------------------------------------------------------------
// Scene: fixed-capacity arrays with active masks (Sec. 3.1; capacities of Table 4).
// Shapes share one index space: polygons 0..P-1, circles P..P+C-1.  Body position = centre of mass.
// ----------------------------------------------------------------------------------------------
template <class R>
struct Body {
  V2<R> pos{0, 0};
  R theta = 0;
  V2<R> vel{0, 0};
  R omega = 0;
  R inv_mass = 0, inv_inertia = 0, friction = 0, restitution = 0, density = 0;
  int role = 0, active = 0;
  int n_verts = 4;          // polygons: 3 or 4 vertices, counter-clockwise, local frame
  V2<R> verts[4] = {{0, 0}, {0, 0}, {0, 0}, {0, 0}};
  R radius = 0;             // circles
};

template <class R>
struct Joint {
  int active = 0, a = 0, b = 0, fixed = 0, motor_on = 0;
  int limited = 0;          // revolute only: the relative rotation theta_a - theta_b is kept in [limit_lo, limit_hi] (A.4.3)
  V2<R> anchor_a{0, 0}, anchor_b{0, 0};   // local frames of a and b
  R theta_f = 0, motor_speed = 0, motor_power = 0;
  R limit_lo = 0, limit_hi = 0;
  V2<R> acc{0, 0};          // accumulated point impulse (on a)        (A.7)
  R acc_ang = 0;            // accumulated angular impulse, fixed only (A.7)
};

template <class R>
struct Thruster {
  int active = 0, body = 0;
  V2<R> pos{0, 0};          // mount point, local frame of the body
  R angle = 0, power = 0;   // direction = body rotation + angle
};

// Collision manifold (Table 2): position, unit normal (always from a to b, a = lower index),
// penetration; a point is an active collision iff penetration > 0.  Polygon-polygon pairs have
// two points (A.3.4), the other pair types one.
template <class R>
struct Manifold {
  int eligible = 0;
  V2<R> normal{0, 0};
  V2<R> pos[2] = {{0, 0}, {0, 0}};
  R pen[2] = {0, 0};
  int valid[2] = {0, 0};
  int active[2] = {0, 0};
  int overlap = 0;          // polygon pairs: no separating axis was found (work counter only)
  double margin = std::numeric_limits<double>::infinity();  // distance of the nearest discrete decision
};

template <class R>
struct ContactAcc {
  R lambda_n[2] = {0, 0};
  R lambda_t[2] = {0, 0};
  int prev_active[2] = {0, 0};
};

template <class R>
struct Env {
  std::vector<Body<R>> bodies;
  std::vector<Joint<R>> joints;
  std::vector<Thruster<R>> thrusters;
  std::vector<Manifold<R>> manifolds;  // lexicographic pair order
  std::vector<int> pair_level;         // lexicographic pair order: lowest free level of the pair at the last substep, -1 = not colliding
  std::vector<ContactAcc<R>> acc;      // lexicographic pair order
  double min_margin = std::numeric_limits<double>::infinity();
  // work counters, summed over substeps (they feed the benchmark's count of arithmetic, nothing else)
  int n_active_slots_sum = 0;          // active manifold points
  int n_active_pairs_sum = 0;          // pairs with at least one active point
  int n_pp_overlap_sum = 0;            // polygon pairs that went past the separating-axis test
  int n_levels_sum = 0;                // levels (independent sets) of the colliding pairs, summed over substeps
  int n_substeps_done = 0;
};

inline int pair_index(int i, int j, int N) { return i * (2 * N - i - 1) / 2 + (j - i - 1); }

// The order in which shape pairs are walked: a round-robin tournament over the shape indices (all
// pairs of one round touch disjoint shapes).  The batched schedule of A.8 deals the manifold points
// over its batches in this order; the sequential sweep derives its visiting order from it (see
// "Visiting order of the colliding pairs" in substep()).
struct Schedule {
  int n_rounds = 0, per_round = 0;
  std::vector<int> a, b, round;   // in tournament order
};
Schedule make_schedule(int N) {
  Schedule s;
  int m = (N % 2 == 0) ? N : N + 1;
  s.n_rounds = m - 1;
  s.per_round = m / 2;
  for (int r = 0; r < m - 1; ++r) {
    for (int k = 0; k < m / 2; ++k) {
      int x, y;
      if (k == 0) { x = m - 1; y = r; }
      else { x = (r + k) % (m - 1); y = ((r - k) % (m - 1) + (m - 1)) % (m - 1); }
      if (x >= N || y >= N) continue;  // the phantom index of an odd N sits out
      s.a.push_back(std::min(x, y));
      s.b.push_back(std::max(x, y));
      s.round.push_back(r);
    }
  }
  return s;
}

// ----------------------------------------------------------------------------------------------
// World-frame polygon: vertices and outward unit edge normals (edge i runs from vertex i to i+1).
// ----------------------------------------------------------------------------------------------
template <class R>
struct WorldPoly {
  int n = 0;
  V2<R> w[4];
  V2<R> nrm[4];
};

template <class R>
WorldPoly<R> world_polygon(const Body<R>& b) {
  WorldPoly<R> wp;
  wp.n = b.n_verts;
  R c, s;
  Fn<R>::sincos(b.theta, s, c);
  for (int i = 0; i < wp.n; ++i) wp.w[i] = b.pos + rotate(c, s, b.verts[i]);
  for (int i = 0; i < wp.n; ++i) {
    V2<R> e = wp.w[(i + 1) % wp.n] - wp.w[i];
    R len = std::sqrt(dot(e, e));
    wp.nrm[i] = {e.y / len, -e.x / len};
  }
  return wp;
}

inline void note(double& margin, double m) { margin = std::min(margin, std::fabs(m)); }

// A.3.2 -- circle a, circle b.
template <class R>
void manifold_cc(V2<R> pa, R ra, V2<R> pb, R rb, Manifold<R>& m) {
  V2<R> d = pb - pa;
  R L = std::sqrt(dot(d, d));
  // coincident centres: the paper's normal is 0/0; take +x
  V2<R> n = (L > R(1e-9)) ? V2<R>{d.x / L, d.y / L} : V2<R>{1, 0};
  m.normal = n;
  m.pos[0] = pa + ra * n;
  m.pen[0] = ra + rb - L;
  m.valid[0] = 1;
  note(m.margin, m.pen[0]);
}

// A.3.3 -- polygon a, circle b.  For every edge the centre is clipped to the segment and projected;
// the closest of those points gives the manifold.  The printed penetration `r_b - |p|` is read as
// r_b minus the distance from the centre to that closest point.  A centre inside the polygon (the
// printed normal would point inward) takes the face of largest signed distance instead.
template <class R>
void manifold_pc(const WorldPoly<R>& A, V2<R> c, R rb, Manifold<R>& m) {
  R best_d2 = std::numeric_limits<R>::infinity();
  V2<R> q{0, 0};
  R smax = -std::numeric_limits<R>::infinity(), ssecond = smax;
  int imax = 0;
  for (int i = 0; i < A.n; ++i) {
    V2<R> v = A.w[i];
    V2<R> e = A.w[(i + 1) % A.n] - v;
    R t = dot(c - v, e) / dot(e, e);
    t = std::min(std::max(t, R(0)), R(1));
    V2<R> qi = v + t * e;
    V2<R> dq = c - qi;
    R d2 = dot(dq, dq);
    if (d2 < best_d2) { best_d2 = d2; q = qi; }
    R s = dot(A.nrm[i], c - v);
    if (s > smax) { ssecond = smax; smax = s; imax = i; }
    else if (s > ssecond) { ssecond = s; }
  }
  if (smax <= R(0)) {
    V2<R> n = A.nrm[imax];
    m.normal = n;
    m.pen[0] = rb - smax;
    m.pos[0] = c - smax * n;
    note(m.margin, double(smax) - double(ssecond));   // which face: discontinuous on the medial axis
  } else {
    R dist = std::sqrt(best_d2);
    V2<R> dq = c - q;
    m.normal = {dq.x / dist, dq.y / dist};
    m.pen[0] = rb - dist;
    m.pos[0] = q;
  }
  m.valid[0] = 1;
  note(m.margin, m.pen[0]);
}

// Largest over X's faces of the smallest signed distance of Y's vertices to that face (A.3.4: the
// separating-axis search; the face attaining it is the axis of least penetration of X).
template <class R>
void face_query(const WorldPoly<R>& X, const WorldPoly<R>& Y, R& best, int& idx, R& second) {
  best = -std::numeric_limits<R>::infinity();
  second = best;
  idx = 0;
  for (int i = 0; i < X.n; ++i) {
    R smin = std::numeric_limits<R>::infinity();
    for (int k = 0; k < Y.n; ++k) smin = std::min(smin, dot(X.nrm[i], Y.w[k] - X.w[i]));
    if (smin > best) { second = best; best = smin; idx = i; }
    else if (smin > second) { second = smin; }
  }
}

// A.3.4 -- polygon a, polygon b.  Separating-axis test; reference face = face of least penetration
// (b's only if it beats a's by tie_eps, so that parallel resting faces do not flip-flop); incident
// face = the face of the other polygon most anti-parallel to the reference normal; the incident
// segment is clipped to the side planes of the reference face; each clipped end point is a manifold
// point whose penetration is its depth below the reference face.
template <class R>
void manifold_pp(const WorldPoly<R>& A, const WorldPoly<R>& B, R tie_eps, Manifold<R>& m) {
  R sa, sb, sa2, sb2;
  int ia, ib;
  face_query(A, B, sa, ia, sa2);
  face_query(B, A, sb, ib, sb2);
  note(m.margin, std::max(sa, sb));
  if (std::max(sa, sb) >= R(0)) return;  // a separating axis exists: no collision
  m.overlap = 1;
  bool ref_b = sb > sa + tie_eps;
  note(m.margin, double(sb) - (double(sa) + double(tie_eps)));
  note(m.margin, ref_b ? double(sb) - double(sb2) : double(sa) - double(sa2));
  const WorldPoly<R>& Rf = ref_b ? B : A;
  const WorldPoly<R>& In = ref_b ? A : B;
  int ir = ref_b ? ib : ia;
  V2<R> nref = Rf.nrm[ir];
  V2<R> r1 = Rf.w[ir], r2 = Rf.w[(ir + 1) % Rf.n];
  int jinc = 0;
  R dmin = std::numeric_limits<R>::infinity(), dsecond = dmin;
  for (int j = 0; j < In.n; ++j) {
    R d = dot(In.nrm[j], nref);
    if (d < dmin) { dsecond = dmin; dmin = d; jinc = j; }
    else if (d < dsecond) { dsecond = d; }
  }
  note(m.margin, double(dsecond) - double(dmin));
  V2<R> v[2] = {In.w[jinc], In.w[(jinc + 1) % In.n]};
  V2<R> t{-nref.y, nref.x};  // along the reference face, from r1 to r2
  R u[2] = {dot(t, v[0] - r1), dot(t, v[1] - r1)};
  R len = dot(t, r2 - r1);
  if ((u[0] < R(0) && u[1] < R(0)) || (u[0] > len && u[1] > len)) return;  // nothing left after clipping
  m.normal = ref_b ? V2<R>{-nref.x, -nref.y} : nref;
  for (int k = 0; k < 2; ++k) {
    R uc = std::min(std::max(u[k], R(0)), len);
    V2<R> x = v[k];
    if (uc != u[k]) {
      R s = (uc - u[0]) / (u[1] - u[0]);
      x = v[0] + s * (v[1] - v[0]);
    }
    m.pos[k] = x;
    m.pen[k] = -dot(nref, x - r1);
    m.valid[k] = 1;
    note(m.margin, m.pen[k]);
  }
}

// ----------------------------------------------------------------------------------------------
// A.2 -- an impulse j applied at offset r from the centre of mass.
// ----------------------------------------------------------------------------------------------
template <class R>
inline void apply_impulse(Body<R>& b, V2<R> j, V2<R> r) {
  b.vel = madd(b.vel, b.inv_mass, j);
  b.omega = std::fma(b.inv_inertia, cross(r, j), b.omega);
}

// Relative velocity of the contact points: v_a + w_a x r_a - v_b - w_b x r_b (A.3.5).
template <class R>
inline V2<R> rel_vel(const Body<R>& a, V2<R> ra, const Body<R>& b, V2<R> rb) {
  // with w x r = (-w r_y, w r_x), one fused multiply-add per cross term
  return {std::fma(b.omega, rb.y, std::fma(-a.omega, ra.y, a.vel.x) - b.vel.x),
          std::fma(-b.omega, rb.x, std::fma(a.omega, ra.x, a.vel.y) - b.vel.y)};
}

template <class R>
struct ContactRow {   // per manifold point, fixed for one substep
  int active = 0;
  V2<R> ra, rb;
  R mass_n = 0, mass_t = 0;   // 1 / denominators of the normal and friction impulse (A.3.5, A.3.6)
  R bias = 0, rest = 0;
};
template <class R>
struct ContactPair {
  int a = 0, b = 0, any = 0;
  V2<R> n, t;
  R mu = 0, e = 0;
  ContactRow<R> row[2];
};
template <class R>
struct JointRow {   // fixed for one substep
  int live = 0;
  V2<R> ra, rb;
  R k11 = 0, k12 = 0, k22 = 0;   // 2x2 effective-mass matrix of the point constraint
  R inv_det = 0;                 // 1 / its determinant
  V2<R> bias{0, 0};
  R ang_mass = 0, ang_bias = 0;
  R lim_excess = 0;              // rotation beyond the upper (> 0) or the lower (< 0) limit; 0 = within limits
  R lim_bias = 0;                // gamma * lim_excess
};

// A joint takes part only if it is active and joins two different, active shapes of which at least one can
// move; a joint (or a thruster) that names a shape index outside the scene's arrays counts as inactive.
template <class R>
inline bool joint_live(const Env<R>& E, const Joint<R>& j) {
  if (!j.active) return false;
  const int N = (int)E.bodies.size();
  if (j.a < 0 || j.a >= N || j.b < 0 || j.b >= N) return false;
  const Body<R>& a = E.bodies[j.a];
  const Body<R>& b = E.bodies[j.b];
  return j.a != j.b && a.active && b.active && (a.inv_mass + b.inv_mass) > R(0);
}

// One manifold point of a colliding pair: normal impulse then friction impulse (A.3.5, A.3.6), each
// accumulated and clamped (A.7), applied to the bodies a and b that the caller hands in.  `j` and `jf`
// return the two impulses that a received (b received the opposite ones).
template <class R>
void solve_contact_point(Body<R>& a, Body<R>& b, const ContactPair<R>& cp, int k, ContactAcc<R>& acc, V2<R>& j,
                         V2<R>& jf) {
  const ContactRow<R>& row = cp.row[k];
  // normal impulse (A.3.5) with the velocity correction added to the numerator (A.3.7),
  // accumulated and kept non-negative (A.7)
  R vn = dot(cp.n, rel_vel(a, row.ra, b, row.rb));
  R dl = row.mass_n * (vn + row.rest + row.bias);
  R ln = std::max(acc.lambda_n[k] + dl, R(0));
  dl = ln - acc.lambda_n[k];
  acc.lambda_n[k] = ln;
  j = (-dl) * cp.n;   // impulse on a; b receives the opposite
  apply_impulse(a, j, row.ra);
  apply_impulse(b, V2<R>{-j.x, -j.y}, row.rb);
  // friction impulse (A.3.6), clipped to +-mu * accumulated normal impulse
  R vt = dot(cp.t, rel_vel(a, row.ra, b, row.rb));
  R dt_ = -row.mass_t * vt;
  R lim = cp.mu * ln;
  R lt = std::min(std::max(acc.lambda_t[k] + dt_, -lim), lim);
  dt_ = lt - acc.lambda_t[k];
  acc.lambda_t[k] = lt;
  jf = dt_ * cp.t;
  apply_impulse(a, jf, row.ra);
  apply_impulse(b, V2<R>{-jf.x, -jf.y}, row.rb);
}

template <class R>
void solve_contact_pair(Env<R>& E, ContactPair<R>& cp, ContactAcc<R>& acc) {
  V2<R> j, jf;
  for (int k = 0; k < 2; ++k)
    if (cp.row[k].active) solve_contact_point(E.bodies[cp.a], E.bodies[cp.b], cp, k, acc, j, jf);
}

// Batched impulse resolution (A.8): the manifold points -- two per shape pair, pairs in tournament order --
// are dealt in turn over n_b = ceil(points / B) batches, so that neighbouring points (which tend to be
// active together) land in different batches and a batch holds at most B points.  The batches are
// solved one after the other; the active points of one batch are all solved from the velocities the
// batch started with, each on its own copy of its two bodies, and their impulses are then applied
// to the bodies in point order.  B = 1 is the sequential sweep; B >= points solves every point in
// parallel.
template <class R>
void solve_contacts_batched(Env<R>& E, std::vector<ContactPair<R>>& cps, int N, int B) {
  struct Pending { int z, k; V2<R> j, jf; };
  const int n_points = 2 * (int)cps.size();
  const int n_b = (n_points + B - 1) / B;
  std::vector<Pending> pend;
  for (int b = 0; b < n_b; ++b) {
    pend.clear();
    for (int s = b; s < n_points; s += n_b) {
      const int z = s / 2, k = s % 2;
      ContactPair<R>& cp = cps[z];
      if (!cp.row[k].active) continue;
      Body<R> a = E.bodies[cp.a], bb = E.bodies[cp.b];   // private copies: the batch's starting velocities
      Pending p{z, k, {0, 0}, {0, 0}};
      solve_contact_point(a, bb, cp, k, E.acc[pair_index(cp.a, cp.b, N)], p.j, p.jf);
      pend.push_back(p);
    }
    for (const Pending& p : pend) {
      const ContactPair<R>& cp = cps[p.z];
      const ContactRow<R>& row = cp.row[p.k];
      apply_impulse(E.bodies[cp.a], p.j, row.ra);
      apply_impulse(E.bodies[cp.b], V2<R>{-p.j.x, -p.j.y}, row.rb);
      apply_impulse(E.bodies[cp.a], p.jf, row.ra);
      apply_impulse(E.bodies[cp.b], V2<R>{-p.jf.x, -p.jf.y}, row.rb);
    }
  }
}

template <class R>
void solve_joint(Env<R>& E, Joint<R>& jt, const JointRow<R>& jr) {
  Body<R>& a = E.bodies[jt.a];
  Body<R>& b = E.bodies[jt.b];
  if (jt.fixed && jr.ang_mass > R(0)) {
    // A.4.2: j_r = (w_a - w_b)/(1/I_a + 1/I_b), plus the correction gamma*(th_a - th_b - th_f)
    R d = -(a.omega - b.omega + jr.ang_bias) * jr.ang_mass;
    a.omega = a.omega + a.inv_inertia * d;
    b.omega = b.omega - b.inv_inertia * d;
    jt.acc_ang = jt.acc_ang + d;
  }
  if (!jt.fixed && jr.lim_excess != R(0) && jr.ang_mass > R(0)) {
    // A.4.3: beyond a limit the angular impulse of a fixed joint (with the correction gamma * excess) is
    // applied -- unless the relative angular velocity already brings the shapes back within the limits
    // (so that a motor may return them faster than the correction would).  Not accumulated (A.7: warm
    // starting joint limits is unstable).
    R w = a.omega - b.omega;
    bool restoring = (jr.lim_excess > R(0)) ? (w < R(0)) : (w > R(0));
    if (!restoring) {
      R d = -(w + jr.lim_bias) * jr.ang_mass;
      a.omega = a.omega + a.inv_inertia * d;
      b.omega = b.omega - b.inv_inertia * d;
    }
    E.min_margin = std::min(E.min_margin, std::fabs(double(w)));
  }
  // A.4.1: the two anchor points must have zero relative velocity; the velocity correction pulls
  // them back together.  Solved as a 2-D point constraint (the printed 1-D "collision along the
  // separation" is singular at zero separation and cannot remove tangential relative velocity).
  V2<R> cdot = rel_vel(a, jr.ra, b, jr.rb);
  V2<R> rhs{-(cdot.x + jr.bias.x), -(cdot.y + jr.bias.y)};
  V2<R> j{(jr.k22 * rhs.x - jr.k12 * rhs.y) * jr.inv_det, (jr.k11 * rhs.y - jr.k12 * rhs.x) * jr.inv_det};
  apply_impulse(a, j, jr.ra);
  apply_impulse(b, V2<R>{-j.x, -j.y}, jr.rb);
  jt.acc = jt.acc + j;
}

// One pass of the body of Algorithm 1 with time step h.
template <class R>
void substep(Env<R>& E, const Params& P, const Schedule& S, int nP, const double* actions) {
  const int N = (int)E.bodies.size();
  const int nJ = (int)E.joints.size();
  const int nT = (int)E.thrusters.size();
  const R h = R(P.dt) / R(P.n_substeps);

  // -- Apply gravity (Alg. 1) ------------------------------------------------------------------
  for (Body<R>& b : E.bodies)
    if (b.active && b.inv_mass > R(0)) b.vel.y = b.vel.y + R(P.gravity_y) * h;

  // -- Calculate collision manifolds (Alg. 1; A.3.1-A.3.4) for every pair of shapes --------------
  std::vector<WorldPoly<R>> wp(nP);
  for (int i = 0; i < nP; ++i) wp[i] = world_polygon(E.bodies[i]);
  std::vector<char> joined(N * N, 0);   // A.4: joined shapes do not collide
  for (const Joint<R>& j : E.joints)
    if (joint_live(E, j)) joined[j.a * N + j.b] = joined[j.b * N + j.a] = 1;
  for (int i = 0; i < N; ++i) {
    for (int j = i + 1; j < N; ++j) {
      Manifold<R> m;
      const Body<R>& a = E.bodies[i];
      const Body<R>& b = E.bodies[j];
      m.eligible = a.active && b.active && !joined[i * N + j] && (a.inv_mass + b.inv_mass) > R(0);
      if (m.eligible) {
        if (j < nP) manifold_pp(wp[i], wp[j], R(P.tie_eps), m);
        else if (i < nP) manifold_pc(wp[i], b.pos, b.radius, m);
        else manifold_cc(a.pos, a.radius, b.pos, b.radius, m);
        for (int k = 0; k < 2; ++k) m.active[k] = m.valid[k] && m.pen[k] > R(0);
        E.min_margin = std::min(E.min_margin, m.margin);
        E.n_pp_overlap_sum += m.overlap;
        E.n_active_pairs_sum += (m.active[0] || m.active[1]);
      }
      E.manifolds[pair_index(i, j, N)] = m;
    }
  }

  // -- Per-substep constants of every active manifold point --------------------------------------
  std::vector<ContactPair<R>> cps(S.a.size());
  for (size_t q = 0; q < S.a.size(); ++q) {
    ContactPair<R>& cp = cps[q];
    cp.a = S.a[q];
    cp.b = S.b[q];
    int pi = pair_index(cp.a, cp.b, N);
    const Manifold<R>& m = E.manifolds[pi];
    ContactAcc<R>& acc = E.acc[pi];
    const Body<R>& a = E.bodies[cp.a];
    const Body<R>& b = E.bodies[cp.b];
    cp.n = m.normal;
    cp.t = {-m.normal.y, m.normal.x};                                        // A.3.6: perpendicular to n
    cp.e = std::min(a.restitution, b.restitution);                           // A.3.5
    cp.mu = std::sqrt(a.friction * a.friction + b.friction * b.friction);    // A.3.6
    for (int k = 0; k < 2; ++k) {
      ContactRow<R>& row = cp.row[k];
      row.active = m.active[k];
      if (row.active) {
        cp.any = 1;
        row.ra = m.pos[k] - a.pos;
        row.rb = m.pos[k] - b.pos;
        R ran = cross(row.ra, cp.n), rbn = cross(row.rb, cp.n);
        R rat = cross(row.ra, cp.t), rbt = cross(row.rb, cp.t);
        R kn = a.inv_mass + b.inv_mass + ran * ran * a.inv_inertia + rbn * rbn * b.inv_inertia;
        R kt = a.inv_mass + b.inv_mass + rat * rat * a.inv_inertia + rbt * rbt * b.inv_inertia;
        row.mass_n = R(1) / kn;
        row.mass_t = R(1) / kt;
        row.bias = R(P.alpha) * std::max(m.pen[k] - R(P.slop), R(0));         // A.3.7
        E.n_active_slots_sum += 1;
      }
      // A.7: a manifold point keeps its accumulated impulses only if it was also colliding
      // at the previous substep
      if (!(P.warm_start && row.active && acc.prev_active[k])) {
        acc.lambda_n[k] = 0;
        acc.lambda_t[k] = 0;
      }
      acc.prev_active[k] = row.active;
    }
  }
  E.n_substeps_done += 1;

  // -- Joint constants: anchors, effective masses, correction speeds ------------------------------
  std::vector<JointRow<R>> jrs(nJ);
  for (int q = 0; q < nJ; ++q) {
    Joint<R>& jt = E.joints[q];
    JointRow<R>& jr = jrs[q];
    jr.live = joint_live(E, jt);
    if (!jr.live) { jt.acc = {0, 0}; jt.acc_ang = 0; continue; }
    if (!P.warm_start) { jt.acc = {0, 0}; jt.acc_ang = 0; }
    const Body<R>& a = E.bodies[jt.a];
    const Body<R>& b = E.bodies[jt.b];
    jr.ra = turn(a.theta, jt.anchor_a);
    jr.rb = turn(b.theta, jt.anchor_b);
    R ms = a.inv_mass + b.inv_mass;
    jr.k11 = ms + a.inv_inertia * jr.ra.y * jr.ra.y + b.inv_inertia * jr.rb.y * jr.rb.y;
    jr.k22 = ms + a.inv_inertia * jr.ra.x * jr.ra.x + b.inv_inertia * jr.rb.x * jr.rb.x;
    jr.k12 = -a.inv_inertia * jr.ra.x * jr.ra.y - b.inv_inertia * jr.rb.x * jr.rb.y;
    jr.inv_det = R(1) / (jr.k11 * jr.k22 - jr.k12 * jr.k12);
    V2<R> sep = (a.pos + jr.ra) - (b.pos + jr.rb);
    jr.bias = R(P.joint_alpha) * sep;
    R is = a.inv_inertia + b.inv_inertia;
    jr.ang_mass = (is > R(0)) ? R(1) / is : R(0);
    jr.ang_bias = R(P.gamma) * (a.theta - b.theta - jt.theta_f);
    if (!jt.fixed) jt.acc_ang = 0;
    if (!jt.fixed && jt.limited) {   // A.4.3, decided once per substep like the collision manifolds
      R rel = a.theta - b.theta;
      if (rel > jt.limit_hi) jr.lim_excess = rel - jt.limit_hi;
      else if (rel < jt.limit_lo) jr.lim_excess = rel - jt.limit_lo;
      jr.lim_bias = R(P.gamma) * jr.lim_excess;
      E.min_margin = std::min(E.min_margin, std::min(std::fabs(double(rel) - double(jt.limit_hi)),
                                                     std::fabs(double(rel) - double(jt.limit_lo))));
    }
  }

  // -- Apply motors (A.5): angular impulse p*tanh((w_a - w_b - s*A)*rho), read as a torque held
  //    for h.  All motors are evaluated on the same velocities ("parallelised", A.8), then applied
  //    in index order; a positive impulse slows a and speeds b, driving w_a - w_b towards s*A.
  std::vector<R> motor(nJ, R(0));
  for (int q = 0; q < nJ; ++q) {
    const Joint<R>& jt = E.joints[q];
    if (!jrs[q].live || jt.fixed || !jt.motor_on) continue;
    R A = R(actions[q]);
    R arg = (E.bodies[jt.a].omega - E.bodies[jt.b].omega - jt.motor_speed * A) * R(P.rho);
    motor[q] = jt.motor_power * Fn<R>::tanh(arg) * h;
  }
  for (int q = 0; q < nJ; ++q) {
    if (motor[q] == R(0)) continue;
    Body<R>& a = E.bodies[E.joints[q].a];
    Body<R>& b = E.bodies[E.joints[q].b];
    a.omega = a.omega - a.inv_inertia * motor[q];
    b.omega = b.omega + b.inv_inertia * motor[q];
  }

  // -- Apply thrusters (A.6): force p*A along the thruster direction at its mount point, held for h.
  for (int q = 0; q < nT; ++q) {
    const Thruster<R>& th = E.thrusters[q];
    if (!th.active || th.body < 0 || th.body >= N) continue;
    Body<R>& b = E.bodies[th.body];
    if (!b.active) continue;
    R A = R(actions[nJ + q]);
    if (P.clip_thruster_01) A = std::min(std::max(A, R(0)), R(1));
    V2<R> u = unit(b.theta);
    V2<R> dir = rotate(u.x, u.y, unit(th.angle));
    V2<R> r = rotate(u.x, u.y, th.pos);
    V2<R> imp = (th.power * A * h) * dir;
    apply_impulse(b, imp, r);
  }

  // -- Restitution target -e*v_r (A.3.5), v_r sampled once here: after the external impulses,
  //    before any constraint impulse.  Slow approaches (resting contact) take e = 0.
  for (ContactPair<R>& cp : cps) {
    for (int k = 0; k < 2; ++k) {
      ContactRow<R>& row = cp.row[k];
      if (!row.active) continue;
      R vn0 = dot(cp.n, rel_vel(E.bodies[cp.a], row.ra, E.bodies[cp.b], row.rb));
      row.rest = (vn0 > R(P.restitution_threshold)) ? cp.e * vn0 : R(0);
      if (cp.e > R(0)) E.min_margin = std::min(E.min_margin, std::fabs(double(vn0) - P.restitution_threshold));
    }
  }

  // -- Visiting order of the colliding pairs (A.8).  The paper solves constraints one after the other
  //    where it can afford to, and leaves the order of the active manifolds to the engine (its own
  //    spreads them over its batches).  Two orders are built here, both sequential (Gauss-Seidel):
  //    sweep_order 0: the tournament order itself.  Its groups are the rounds (disjoint shapes).
  //    sweep_order 1: walk the colliding pairs in tournament order and give each the lowest level that
  //      no earlier colliding pair sharing a movable shape with it has taken; visit level 0 first, then
  //      level 1, ..., tournament order inside a level.  Pairs of one level share no shape that an
  //      impulse can move, so a level is a set of independent constraints, and the sweep is as short as
  //      the busiest shape's contacts allow.  Shapes that no impulse moves (inactive, or neither inverse
  //      mass nor inverse inertia) tie nothing together.
  std::vector<int> visit;            // indices into cps, in visiting order
  std::vector<int> group_end;        // visit[group_end[g-1] .. group_end[g]) is group g (a round, or a level)
  {
    auto movable = [&](int i) {
      const Body<R>& s = E.bodies[i];
      return s.active && (s.inv_mass != R(0) || s.inv_inertia != R(0));
    };
    std::vector<unsigned> taken(N, 0u);   // levels already used at each movable shape
    std::vector<int> group(cps.size(), -1);
    int n_groups = 0, n_levels = 0;
    for (size_t q = 0; q < cps.size(); ++q) {
      E.pair_level[pair_index(cps[q].a, cps[q].b, N)] = -1;
      if (!cps[q].any) continue;
      unsigned busy = (movable(cps[q].a) ? taken[cps[q].a] : 0u) | (movable(cps[q].b) ? taken[cps[q].b] : 0u);
      int lv = 0;
      while ((busy >> lv) & 1u) ++lv;
      if (movable(cps[q].a)) taken[cps[q].a] |= 1u << lv;
      if (movable(cps[q].b)) taken[cps[q].b] |= 1u << lv;
      E.pair_level[pair_index(cps[q].a, cps[q].b, N)] = lv;
      n_levels = std::max(n_levels, lv + 1);
      group[q] = P.sweep_order == 1 ? lv : S.round[q];
      n_groups = std::max(n_groups, group[q] + 1);
    }
    for (int g = 0; g < n_groups; ++g) {
      for (size_t q = 0; q < cps.size(); ++q)
        if (group[q] == g) visit.push_back((int)q);
      group_end.push_back((int)visit.size());
    }
    E.n_levels_sum += n_levels;
  }

  // -- Warm starting (Alg. 1; A.7): collisions in visiting order, then joints in index order -------
  if (P.warm_start) {
    for (int q : visit) {
      const ContactPair<R>& cp = cps[q];
      const ContactAcc<R>& acc = E.acc[pair_index(cp.a, cp.b, N)];
      for (int k = 0; k < 2; ++k) {
        if (!cp.row[k].active) continue;
        V2<R> j = (-acc.lambda_n[k]) * cp.n + acc.lambda_t[k] * cp.t;
        apply_impulse(E.bodies[cp.a], j, cp.row[k].ra);
        apply_impulse(E.bodies[cp.b], V2<R>{-j.x, -j.y}, cp.row[k].rb);
      }
    }
    for (int q = 0; q < nJ; ++q) {
      if (!jrs[q].live) continue;
      Joint<R>& jt = E.joints[q];
      Body<R>& a = E.bodies[jt.a];
      Body<R>& b = E.bodies[jt.b];
      if (jt.fixed) {
        a.omega = a.omega + a.inv_inertia * jt.acc_ang;
        b.omega = b.omega - b.inv_inertia * jt.acc_ang;
      }
      apply_impulse(a, jt.acc, jrs[q].ra);
      apply_impulse(b, V2<R>{-jt.acc.x, -jt.acc.y}, jrs[q].rb);
    }
  }

  // -- Solver sweeps (Alg. 1): joints sequentially (A.8), then collisions in visiting order --------
  for (int it = 0; it < P.n_iters; ++it) {
    for (int q = 0; q < nJ; ++q)
      if (jrs[q].live) solve_joint(E, E.joints[q], jrs[q]);
    if (P.batch_size > 0) {
      solve_contacts_batched(E, cps, N, P.batch_size);
    } else if (P.order_mode != 1) {
      for (int q : visit) solve_contact_pair(E, cps[q], E.acc[pair_index(cps[q].a, cps[q].b, N)]);
    } else {
      // test mode: every pair of a group (round or level) starts from the same snapshot of the bodies and
      // only what it did to its own two bodies is kept -- equal to the sequential sweep iff the pairs of a
      // group share no shape that an impulse moves
      int z0 = 0;
      for (int z1 : group_end) {
        std::vector<Body<R>> snap = E.bodies, out = E.bodies;
        for (int z = z0; z < z1; ++z) {
          ContactPair<R>& cp = cps[visit[z]];
          E.bodies = snap;
          solve_contact_pair(E, cp, E.acc[pair_index(cp.a, cp.b, N)]);
          out[cp.a] = E.bodies[cp.a];
          out[cp.b] = E.bodies[cp.b];
        }
        E.bodies = out;
        z0 = z1;
      }
    }
  }

  // -- Euler step position and rotation (Alg. 1), with the already updated velocities --------------
  for (Body<R>& b : E.bodies) {
    if (!b.active) continue;
    b.pos = b.pos + h * b.vel;
    b.theta = b.theta + h * b.omega;
  }

  // -- Positional corrections (A.3.7, A.4.1): colliding pairs in visiting order are moved apart by
  //    beta * (deepest penetration of the pair at the start of the substep, less the slop), shared
  //    in proportion to inverse mass; then joints in index order pull their anchors together.
  for (int q : visit) {
    const ContactPair<R>& cp = cps[q];
    const Manifold<R>& m = E.manifolds[pair_index(cp.a, cp.b, N)];
    R pen = R(0);
    for (int k = 0; k < 2; ++k) if (m.active[k]) pen = std::max(pen, m.pen[k]);
    Body<R>& a = E.bodies[cp.a];
    Body<R>& b = E.bodies[cp.b];
    R c = R(P.beta) * std::max(pen - R(P.slop), R(0)) / (a.inv_mass + b.inv_mass);
    a.pos = a.pos - (a.inv_mass * c) * cp.n;
    b.pos = b.pos + (b.inv_mass * c) * cp.n;
  }
  for (int q = 0; q < nJ; ++q) {
    if (!jrs[q].live) continue;
    const Joint<R>& jt = E.joints[q];
    Body<R>& a = E.bodies[jt.a];
    Body<R>& b = E.bodies[jt.b];
    V2<R> xa = a.pos + turn(a.theta, jt.anchor_a);
    V2<R> xb = b.pos + turn(b.theta, jt.anchor_b);
    V2<R> c = (R(P.joint_beta) / (a.inv_mass + b.inv_mass)) * (xa - xb);
    a.pos = a.pos - a.inv_mass * c;
    b.pos = b.pos + b.inv_mass * c;
  }
}

// ----------------------------------------------------------------------------------------------
// Batch container behind the C interface
// ----------------------------------------------------------------------------------------------
struct BatchBase {
  virtual ~BatchBase() {}
  virtual int set(const std::string& f, const int* ids, long n_ids, const double* data, long count) = 0;
  virtual int get(const std::string& f, double* out, long count) = 0;
  virtual long field_size(const std::string& f) = 0;
  virtual int step(const double* actions, int n_steps, int n_threads) = 0;
  virtual int obs(double* out) = 0;
  virtual int obs_dim() = 0;
  Params params;
};

template <class R>
struct Batch : BatchBase {
  int P, C, J, T, N, NP, n_envs;
  Schedule sched;
  std::vector<Env<R>> envs;

  Batch(int P_, int C_, int J_, int T_, int n) : P(P_), C(C_), J(J_), T(T_), N(P_ + C_), n_envs(n) {
    NP = N * (N - 1) / 2;
    sched = make_schedule(N);
    envs.resize(n);
    for (Env<R>& e : envs) {
      e.bodies.resize(N);
      e.joints.resize(J);
      e.thrusters.resize(T);
      e.manifolds.resize(NP);
      e.pair_level.assign(NP, -1);
      e.acc.resize(NP);
    }
  }

  // A field is (name, elements per environment, accessor).  All traffic is in double; every float is
  // exactly representable, integers are rounded.
  struct Acc { long n; double (*get)(Batch&, Env<R>&, long); void (*set)(Batch&, Env<R>&, long, double); };

  bool find(const std::string& f, Acc& a) {
#define FIELD(NAME, COUNT, LVALUE, CAST)                                                   \
  if (f == NAME) {                                                                         \
    a.n = (COUNT);                                                                         \
    a.get = [](Batch& B, Env<R>& e, long i) -> double { (void)B; (void)i; return double(LVALUE); }; \
    a.set = [](Batch& B, Env<R>& e, long i, double v) { (void)B; (void)i; LVALUE = CAST(v); };      \
    return true;                                                                           \
  }
#define RR(v) R(v)
#define II(v) int(std::lround(v))
    FIELD("pos", N * 2, (i % 2 ? e.bodies[i / 2].pos.y : e.bodies[i / 2].pos.x), RR)
    FIELD("theta", N, e.bodies[i].theta, RR)
    FIELD("vel", N * 2, (i % 2 ? e.bodies[i / 2].vel.y : e.bodies[i / 2].vel.x), RR)
    FIELD("omega", N, e.bodies[i].omega, RR)
    FIELD("inv_mass", N, e.bodies[i].inv_mass, RR)
    FIELD("inv_inertia", N, e.bodies[i].inv_inertia, RR)
    FIELD("friction", N, e.bodies[i].friction, RR)
    FIELD("restitution", N, e.bodies[i].restitution, RR)
    FIELD("density", N, e.bodies[i].density, RR)
    FIELD("role", N, e.bodies[i].role, II)
    FIELD("active", N, e.bodies[i].active, II)
    FIELD("n_verts", P, e.bodies[i].n_verts, II)
    FIELD("verts", P * 8, (i % 2 ? e.bodies[i / 8].verts[(i / 2) % 4].y : e.bodies[i / 8].verts[(i / 2) % 4].x), RR)
    FIELD("radius", C, e.bodies[B.P + i].radius, RR)
    FIELD("joint_active", J, e.joints[i].active, II)
    FIELD("joint_a", J, e.joints[i].a, II)
    FIELD("joint_b", J, e.joints[i].b, II)
    FIELD("joint_fixed", J, e.joints[i].fixed, II)
    FIELD("joint_motor_on", J, e.joints[i].motor_on, II)
    FIELD("joint_anchor_a", J * 2, (i % 2 ? e.joints[i / 2].anchor_a.y : e.joints[i / 2].anchor_a.x), RR)
    FIELD("joint_anchor_b", J * 2, (i % 2 ? e.joints[i / 2].anchor_b.y : e.joints[i / 2].anchor_b.x), RR)
    FIELD("joint_theta_f", J, e.joints[i].theta_f, RR)
    FIELD("joint_motor_speed", J, e.joints[i].motor_speed, RR)
    FIELD("joint_motor_power", J, e.joints[i].motor_power, RR)
    FIELD("joint_limited", J, e.joints[i].limited, II)
    FIELD("joint_limit_lo", J, e.joints[i].limit_lo, RR)
    FIELD("joint_limit_hi", J, e.joints[i].limit_hi, RR)
    FIELD("joint_acc", J * 2, (i % 2 ? e.joints[i / 2].acc.y : e.joints[i / 2].acc.x), RR)
    FIELD("joint_acc_ang", J, e.joints[i].acc_ang, RR)
    FIELD("thruster_active", T, e.thrusters[i].active, II)
    FIELD("thruster_body", T, e.thrusters[i].body, II)
    FIELD("thruster_pos", T * 2, (i % 2 ? e.thrusters[i / 2].pos.y : e.thrusters[i / 2].pos.x), RR)
    FIELD("thruster_angle", T, e.thrusters[i].angle, RR)
    FIELD("thruster_power", T, e.thrusters[i].power, RR)
    FIELD("lambda_n", NP * 2, e.acc[i / 2].lambda_n[i % 2], RR)
    FIELD("lambda_t", NP * 2, e.acc[i / 2].lambda_t[i % 2], RR)
    FIELD("prev_active", NP * 2, e.acc[i / 2].prev_active[i % 2], II)
    // results of the last substep's narrowphase (set() on these is accepted and meaningless)
    FIELD("pair_eligible", NP, e.manifolds[i].eligible, II)
    FIELD("pair_active", NP * 2, e.manifolds[i / 2].active[i % 2], II)
    FIELD("manifold_pen", NP * 2, e.manifolds[i / 2].pen[i % 2], RR)
    FIELD("manifold_normal", NP * 2, (i % 2 ? e.manifolds[i / 2].normal.y : e.manifolds[i / 2].normal.x), RR)
    FIELD("manifold_pos", NP * 4, (i % 2 ? e.manifolds[i / 4].pos[(i / 2) % 2].y : e.manifolds[i / 4].pos[(i / 2) % 2].x), RR)
    FIELD("pair_level", NP, e.pair_level[i], II)
    FIELD("pair_margin", NP, e.manifolds[i].margin, double)
    FIELD("min_margin", 1, e.min_margin, double)
    FIELD("active_slots_sum", 1, e.n_active_slots_sum, II)
    FIELD("active_pairs_sum", 1, e.n_active_pairs_sum, II)
    FIELD("pp_overlap_sum", 1, e.n_pp_overlap_sum, II)
    FIELD("levels_sum", 1, e.n_levels_sum, II)
    FIELD("substeps_done", 1, e.n_substeps_done, II)
#undef FIELD
#undef RR
#undef II
    return false;
  }

  long field_size(const std::string& f) override {
    Acc a;
    if (f == "pair_count" || f == "shape_adj") return f == "pair_count" ? NP : N;
    return find(f, a) ? a.n : -1;
  }

  int set(const std::string& f, const int* ids, long n_ids, const double* data, long count) override {
    Acc a;
    if (!find(f, a)) return -1;
    long rows = ids ? n_ids : n_envs;
    if (count != rows * a.n) return -2;
    for (long r = 0; r < rows; ++r) {
      long e = ids ? ids[r] : r;
      if (e < 0 || e >= n_envs) return -3;
      for (long i = 0; i < a.n; ++i) a.set(*this, envs[e], i, data[r * a.n + i]);
    }
    return 0;
  }

  int get(const std::string& f, double* out, long count) override {
    if (f == "pair_count") {   // number of active manifold points per pair: 0, 1 or 2
      if (count != (long)n_envs * NP) return -2;
      for (int e = 0; e < n_envs; ++e)
        for (int p = 0; p < NP; ++p)
          out[(long)e * NP + p] = envs[e].manifolds[p].active[0] + envs[e].manifolds[p].active[1];
      return 0;
    }
    if (f == "shape_adj") {    // bit j of word i: shapes i and j are in active collision
      if (count != (long)n_envs * N) return -2;
      for (int e = 0; e < n_envs; ++e) {
        std::vector<uint32_t> adj(N, 0);
        for (int i = 0; i < N; ++i)
          for (int j = i + 1; j < N; ++j) {
            const Manifold<R>& m = envs[e].manifolds[pair_index(i, j, N)];
            if (m.active[0] || m.active[1]) { adj[i] |= 1u << j; adj[j] |= 1u << i; }
          }
        for (int i = 0; i < N; ++i) out[(long)e * N + i] = double(adj[i]);
      }
      return 0;
    }
    Acc a;
    if (!find(f, a)) return -1;
    if (count != (long)n_envs * a.n) return -2;
    for (long e = 0; e < n_envs; ++e)
      for (long i = 0; i < a.n; ++i) out[e * a.n + i] = a.get(*this, envs[e], i);
    return 0;
  }

  int step(const double* actions, int n_steps, int n_threads) override {
    const int A = J + T;
    auto run = [&](int e0, int e1) {
      for (int e = e0; e < e1; ++e)
        for (int s = 0; s < n_steps; ++s) {
          const double* act = actions + ((long)s * n_envs + e) * A;   // the same action for every substep
          for (int u = 0; u < params.n_substeps; ++u) substep(envs[e], params, sched, P, act);
        }
    };
    if (n_threads <= 1) { run(0, n_envs); return 0; }
    std::vector<std::thread> th;
    int per = (n_envs + n_threads - 1) / n_threads;
    for (int t = 0; t < n_threads; ++t) {
      int e0 = t * per, e1 = std::min(n_envs, e0 + per);
      if (e0 < e1) th.emplace_back(run, e0, e1);
    }
    for (auto& t : th) t.join();
    return 0;
  }

  // Flat symbolic observation: the physical entries of the paper's Tables 5-7, per entity, in entity
  // order polygons, circles, joints, thrusters (role / type / colour one-hots are left to the caller;
  // the role is passed through as a number).
  int obs_dim() override { return P * 23 + C * 15 + J * 11 + T * 6; }
  int obs(double* out) override {
    const int D = obs_dim();
    for (int e = 0; e < n_envs; ++e) {
      double* o = out + (long)e * D;
      const Env<R>& E = envs[e];
      for (int i = 0; i < N; ++i) {
        const Body<R>& b = E.bodies[i];
        *o++ = b.pos.x; *o++ = b.pos.y; *o++ = b.vel.x; *o++ = b.vel.y;
        *o++ = b.inv_mass; *o++ = b.inv_inertia; *o++ = b.density;
        *o++ = Fn<R>::tanh(b.omega / R(10));
        { V2<R> u = unit(b.theta); *o++ = u.y; *o++ = u.x; }
        *o++ = b.friction; *o++ = b.restitution;
        if (i < P) {
          for (int k = 0; k < 4; ++k) { *o++ = b.verts[k].x; *o++ = b.verts[k].y; }
          *o++ = b.n_verts;
        } else {
          *o++ = b.radius;
        }
        *o++ = b.active; *o++ = b.role;
      }
      for (const Joint<R>& j : E.joints) {
        // (shape indices outside the arrays -- such a joint is inactive in the step -- are clamped here)
        const int ja = std::min(std::max(j.a, 0), N - 1), jb = std::min(std::max(j.b, 0), N - 1);
        R rel = E.bodies[ja].theta - E.bodies[jb].theta;
        *o++ = j.active; *o++ = j.fixed;
        *o++ = j.anchor_a.x; *o++ = j.anchor_a.y; *o++ = j.anchor_b.x; *o++ = j.anchor_b.y;
        *o++ = j.motor_power; *o++ = j.motor_speed; *o++ = j.motor_on;
        { V2<R> u = unit(rel); *o++ = u.y; *o++ = u.x; }
      }
      for (const Thruster<R>& t : E.thrusters) {
        *o++ = t.active; *o++ = t.pos.x; *o++ = t.pos.y; *o++ = t.power;
        { V2<R> u = unit(t.angle); *o++ = u.y; *o++ = u.x; }
      }
    }
    return 0;
  }
};

// Stand-alone manifolds for unit tests.  Polygons are given in world coordinates (n, xy[2n], CCW).
// out = [normal.x, normal.y, pos0.x, pos0.y, pen0, valid0, pos1.x, pos1.y, pen1, valid1, margin]
void pack(const Manifold<double>& m, double* out) {
  out[0] = m.normal.x; out[1] = m.normal.y;
  for (int k = 0; k < 2; ++k) {
    out[2 + 4 * k] = m.pos[k].x; out[3 + 4 * k] = m.pos[k].y; out[4 + 4 * k] = m.pen[k]; out[5 + 4 * k] = m.valid[k];
  }
  out[10] = m.margin;
}
template <class R>
WorldPoly<R> poly_from(int n, const double* xy) {
  Body<R> b;
  b.n_verts = n;
  for (int i = 0; i < n; ++i) b.verts[i] = {R(xy[2 * i]), R(xy[2 * i + 1])};
  return world_polygon(b);   // theta = 0, pos = 0: local frame == world frame
}
template <class R>
void pack_r(const Manifold<R>& m, double* out) {
  Manifold<double> d;
  d.normal = {m.normal.x, m.normal.y};
  for (int k = 0; k < 2; ++k) { d.pos[k] = {m.pos[k].x, m.pos[k].y}; d.pen[k] = m.pen[k]; d.valid[k] = m.valid[k]; }
  d.margin = m.margin;
  pack(d, out);
}
}  // namespace

// ----------------------------------------------------------------------------------------------
// C interface (ctypes).  Pointers are host memory; nothing is retained after a call returns.
// ----------------------------------------------------------------------------------------------
extern "C" {

void* ko_create(int P, int C, int J, int T, int n_envs, int use_double) {
  if (P < 0 || C < 0 || J < 0 || T < 0 || P + C < 1 || P + C > 32 || n_envs < 1) return nullptr;
  if (use_double) return static_cast<BatchBase*>(new Batch<double>(P, C, J, T, n_envs));
  return static_cast<BatchBase*>(new Batch<float>(P, C, J, T, n_envs));
}
void ko_destroy(void* h) { delete static_cast<BatchBase*>(h); }

// params: [dt, gravity_y, n_substeps, n_iters, warm_start, alpha, beta, gamma, rho, slop,
//          restitution_threshold, clip_thruster_01, joint_alpha, joint_beta, tie_eps, order_mode,
//          batch_size, sweep_order]
int ko_set_params(void* h, const double* p, int n) {
  if (!h || !p || n != kNumParams) return -1;
  Params& q = static_cast<BatchBase*>(h)->params;
  q.dt = p[0]; q.gravity_y = p[1]; q.n_substeps = (int)p[2]; q.n_iters = (int)p[3]; q.warm_start = (int)p[4];
  q.alpha = p[5]; q.beta = p[6]; q.gamma = p[7]; q.rho = p[8]; q.slop = p[9];
  q.restitution_threshold = p[10]; q.clip_thruster_01 = (int)p[11];
  q.joint_alpha = p[12]; q.joint_beta = p[13]; q.tie_eps = p[14]; q.order_mode = (int)p[15];
  q.batch_size = (int)p[16]; q.sweep_order = (int)p[17];
  if (q.n_substeps < 1 || q.n_iters < 0 || q.batch_size < 0 || q.sweep_order < 0 || q.sweep_order > 1) return -2;
  return 0;
}
long ko_field_size(void* h, const char* f) { return static_cast<BatchBase*>(h)->field_size(f); }
int ko_set(void* h, const char* f, const double* data, long count) {
  return static_cast<BatchBase*>(h)->set(f, nullptr, 0, data, count);
}
int ko_set_rows(void* h, const char* f, const int* env_ids, long n_ids, const double* data, long count) {
  return static_cast<BatchBase*>(h)->set(f, env_ids, n_ids, data, count);
}
int ko_get(void* h, const char* f, double* out, long count) { return static_cast<BatchBase*>(h)->get(f, out, count); }
int ko_step(void* h, const double* actions, int n_steps, int n_threads) {
  if (!h || !actions || n_steps < 1) return -1;
  return static_cast<BatchBase*>(h)->step(actions, n_steps, n_threads);
}
int ko_obs_dim(void* h) { return static_cast<BatchBase*>(h)->obs_dim(); }
int ko_obs(void* h, double* out) { return static_cast<BatchBase*>(h)->obs(out); }

// The engine's sin, cos, tanh for unit tests: out[i] = {sin, cos, tanh}(x[i]) in fp32 or double.
void ko_math(int use_double, const double* x, long n, double* sn, double* cs, double* th) {
  for (long i = 0; i < n; ++i) {
    if (use_double) { double s, c; Fn<double>::sincos(x[i], s, c); sn[i] = s; cs[i] = c; th[i] = Fn<double>::tanh(x[i]); }
    else { float s, c; Fn<float>::sincos((float)x[i], s, c); sn[i] = s; cs[i] = c; th[i] = Fn<float>::tanh((float)x[i]); }
  }
}

// Canonical visiting order of the shape pairs: writes a[], b[], round[]; returns the number of pairs.
int ko_schedule(int N, int* a, int* b, int* round) {
  Schedule s = make_schedule(N);
  for (size_t i = 0; i < s.a.size(); ++i) { a[i] = s.a[i]; b[i] = s.b[i]; round[i] = s.round[i]; }
  return (int)s.a.size();
}

void ko_manifold_cc(int use_double, const double* pa, double ra, const double* pb, double rb, double* out) {
  if (use_double) { Manifold<double> m; manifold_cc<double>({pa[0], pa[1]}, ra, {pb[0], pb[1]}, rb, m); pack_r(m, out); }
  else { Manifold<float> m; manifold_cc<float>({(float)pa[0], (float)pa[1]}, (float)ra, {(float)pb[0], (float)pb[1]}, (float)rb, m); pack_r(m, out); }
}
void ko_manifold_pc(int use_double, int n, const double* xy, const double* c, double r, double* out) {
  if (use_double) { Manifold<double> m; manifold_pc<double>(poly_from<double>(n, xy), {c[0], c[1]}, r, m); pack_r(m, out); }
  else { Manifold<float> m; manifold_pc<float>(poly_from<float>(n, xy), {(float)c[0], (float)c[1]}, (float)r, m); pack_r(m, out); }
}
void ko_manifold_pp(int use_double, int na, const double* xya, int nb, const double* xyb, double tie_eps, double* out) {
  if (use_double) { Manifold<double> m; manifold_pp<double>(poly_from<double>(na, xya), poly_from<double>(nb, xyb), tie_eps, m); pack_r(m, out); }
  else { Manifold<float> m; manifold_pp<float>(poly_from<float>(na, xya), poly_from<float>(nb, xyb), (float)tie_eps, m); pack_r(m, out); }
}

}  // extern "C"
