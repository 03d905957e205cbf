// k2d.hip -- MI355X (gfx950) implementation of the batched 2D rigid-body step behind include/k2d.h.
//
// What is computed: the main loop of the paper's physics engine (Appendix A, Algorithm 1) for every
// environment of a batch: gravity, collision manifolds for all shape pairs (A.3.1-A.3.4), motors (A.5),
// thrusters (A.6), warm starting (A.7), `n_iters` sweeps of joint constraints (A.4) then collision
// constraints (A.3.5-A.3.7), the Euler step, and the positional corrections (A.3.7, A.4.1).
//
// How it is mapped onto CDNA4:
//   * One environment is owned by a group of G consecutive lanes: G = 16, so that a 64-wide wavefront
//     steps four environments, or G = 8 and eight environments (chosen per launch: faster for the small
//     capacity class in large batches).  A workgroup is exactly one wavefront, which makes every
//     synchronisation point a wavefront-scope fence and lets the hardware place wavefronts on CUs freely.
//   * The whole scene of an environment lives in LDS for the entire launch (all steps, substeps and
//     solver sweeps).  HBM is touched when the launch begins (one coalesced read of the record), once per
//     step for the actions, when it ends -- and in between only for the accumulated impulses (A.7) of
//     pairs that change lanes because the set of colliding pairs changed, for the pair records of piles
//     deeper than registers and LDS hold, and for the new scenes of restarted episodes.  Lanes of a group
//     exchange body velocities through LDS.
//   * The sweep order of the collision constraints (A.8 leaves it to the engine) is built from a
//     round-robin tournament over the shapes, whose rounds touch disjoint shapes.  Walking the colliding
//     pairs in that order, a pair is placed on a level that none of the earlier colliding pairs sharing a
//     movable shape with it is on: one past the last of them (the sweep then has the bits of visiting the
//     pairs one after the other in tournament order), or, as an option, the lowest free one (the sweep
//     then visits level after level, in about as many trips as the busiest shape has contacts).  The
//     pairs of a level are independent, all of them are solved at once, and the result is bit-identical
//     to a sequential Gauss-Seidel sweep (the sequential end of the speed/stability trade-off of A.8,
//     reached without the paper's batch-of-16 compromise).
//   * Active manifolds of a substep become records that live in registers: lane k of the environment
//     keeps active pairs k and G + k for the whole substep (warm start, all sweeps, corrections), so a
//     visit costs one LDS round trip for the two bodies' velocities and nothing else; the accumulated
//     impulses of pair k stay in the lane's registers from substep to substep while the set of colliding
//     pairs is unchanged.  Pairs beyond 2G stay in a small LDS pool, the rare excess beyond that spills
//     to the environment's HBM record.
//   * Joints are solved in index order per shape (A.8: sequential); joints that share no shape are
//     independent, so they are grouped into dependency levels once per episode and lane j solves joint j.
//   * A launch of many steps first sorts the environments by expected work, so that the environments
//     of a wavefront are alike: what a wavefront skips when none of its environments changed its set of
//     colliding pairs (candidate list, dependency levels) it then skips more often.
//
// Nothing here is a dense contraction: no MFMA.  Arithmetic is fp32; the kernel is compiled without
// automatic contraction of a*b+c; the fused multiply-adds are the ones written out (dot and cross
// products, rotations, impulse application), so the rounding of every formula is fixed by the source.

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <mutex>
#include <new>

#include "k2d.h"

// Phase clocks (builds with -DK2D_PHASE_TIMERS only; the product library has none of this): every
// wavefront adds up the shader clocks it spends in each phase of a substep and leaves the sums, followed
// by its totals of collision and joint dependency levels, in a caller-owned device buffer
// (k2d_debug_set_phase_buffer), kPhaseSlots 64-bit words per wavefront.
#ifdef K2D_PHASE_TIMERS
#define K2D_T(i) { const long long t_now_ = clock64(); t_acc[i] += t_now_ - t_last; t_last = t_now_; }
#else
#define K2D_T(i)
#endif
enum {   // phases of one substep, in the order they run
  kT_Actions = 0, kT_Shapes, kT_JointConstants, kT_External, kT_Cull, kT_Manifolds, kT_Presolve, kT_Levels,
  kT_WarmStart, kT_SweepJoints, kT_SweepPairs, kT_Euler, kT_CorrectPairs, kT_CorrectJoints, kT_Restart, kT_Count
};
constexpr int kPhaseSlots = kT_Count + 2;

namespace {

constexpr int kRecW = 25;  // words of one active-pair record (see PairRec)
constexpr float kCullMargin = 1e-3f;   // by how much every bounding box is grown before the overlap test

constexpr int align_up(int x, int a) { return (x + a - 1) / a * a; }

// Word offsets of one environment record (documented in k2d.h).
constexpr k2d_layout make_layout(int P, int C, int J, int T) {
  k2d_layout L{};
  const int N = P + C;
  L.n_shapes = N;
  L.n_pairs = N * (N - 1) / 2;
  int o = 0;
  L.pos_x = o; o += N;
  L.pos_y = o; o += N;
  L.theta = o; o += N;
  L.vel_x = o; o += N;
  L.vel_y = o; o += N;
  L.omega = o; o += N;
  L.inv_mass = o; o += N;
  L.inv_inertia = o; o += N;
  L.friction = o; o += N;
  L.restitution = o; o += N;
  L.density = o; o += N;
  L.shape_flags = o; o += N;
  L.n_verts = o; o += P;
  L.verts = o; o += 8 * P;
  L.radius = o; o += C;
  L.joint_flags = o; o += J;
  L.joint_a = o; o += J;
  L.joint_b = o; o += J;
  L.anchor_a_x = o; o += J;
  L.anchor_a_y = o; o += J;
  L.anchor_b_x = o; o += J;
  L.anchor_b_y = o; o += J;
  L.theta_f = o; o += J;
  L.motor_speed = o; o += J;
  L.motor_power = o; o += J;
  L.limit_lo = o; o += J;
  L.limit_hi = o; o += J;
  L.acc_x = o; o += J;
  L.acc_y = o; o += J;
  L.acc_ang = o; o += J;
  L.thr_flags = o; o += T;
  L.thr_body = o; o += T;
  L.thr_pos_x = o; o += T;
  L.thr_pos_y = o; o += T;
  L.thr_angle = o; o += T;
  L.thr_power = o; o += T;
  L.scene_words = o;
  o = align_up(o, 4);
  L.lambda = o; o += 4 * L.n_pairs;
  L.pair_state = o; o += (L.n_pairs + 3) / 4;
  L.state_words = o;
  L.obs_dim = P * 23 + C * 15 + J * 11 + T * 6;
  return L;
}

// Compile-time description of one capacity class and of its LDS image.
template <int P_, int C_, int J_, int T_, int H_>
struct Cfg {
  static constexpr int P = P_, C = C_, J = J_, T = T_, H = H_;
  static constexpr int N = P + C, NP = N * (N - 1) / 2, A = J + T;
  static constexpr int M = N + (N & 1);   // tournament size (an odd N gets a phantom that sits out)
  static constexpr int R = M - 1;         // rounds
  static constexpr int PPR = M / 2;       // pairs per round
  static constexpr int GP = PPR <= 4 ? 4 : 8;  // lanes that share the pairs of one round
  static constexpr int G = GP * H;             // lanes per environment: lane k tests pair k % GP of the rounds
                                               // r with r % H == k / GP
  static constexpr int EPW = 64 / G;           // environments per wavefront
  static_assert(PPR <= 8 && J <= G && T <= G && R <= 15 && (G == 8 || G == 16) && (H & (H - 1)) == 0 &&
                    (R + H - 1) / H <= 16,
                "capacity class does not fit the lane mapping");
  // Active pairs are numbered 0, 1, ... as the narrowphase finds them.  Pairs below NREG live in
  // registers (lane k holds pairs k and G + k): the lane that found the manifold leaves it in an LDS
  // staging slot, the lane that keeps the pair derives the substep constants from it.  Pairs beyond them
  // live as full records in a small LDS pool (POOL records, as many as the LDS budget of the class has
  // room for, eight at most) or, past that, in the HBM record.
  static constexpr int NREG = 2 * G, kManW = 9;
  static constexpr k2d_layout L = make_layout(P, C, J, T);
  // HBM record: state words, then room for the pair records that neither registers nor the LDS pool hold
  // (sized for the lane mapping that holds fewest, so that every mapping of a class shares one record)
  static constexpr int SPILL = NP > 16 ? NP - 16 : 0;
  static constexpr int G_SPILL = align_up(L.state_words, 4);
  static constexpr int REC_WORDS = align_up(G_SPILL + SPILL * kRecW, 32);
  // LDS image of one environment: scene words, then derived data
  static constexpr int X_COS = align_up(L.scene_words, 2);
  static constexpr int X_SIN = X_COS + N;
  static constexpr int X_BOX = align_up(X_SIN + N, 4);     // bounding box of every shape, float4 (min x, min y, max x, max y),
                                                           // grown by kCullMargin on every side
  static constexpr int X_WV = X_BOX + 4 * N;               // world vertices, float2 [4][P]
  static constexpr int X_WN = X_WV + 8 * P;                // outward unit edge normals, float2 [4][P]
  static constexpr int NID = R * GP;                       // pair ids: id = r * GP + k (tournament order)
  static constexpr int X_TABLE = align_up(X_WN + 8 * P, 4);        // bytes [NID]: number of the active pair with this id (set for the pairs not held in registers)
  static constexpr int TABLE_W = align_up((NID + 3) / 4, 4);       // read back four words at a time
  static constexpr int X_LIST = X_TABLE + TABLE_W;         // bytes [NID]: candidate ids, one shape-type mix after the other
  static constexpr int X_JOINED = X_LIST;                  // (launch set-up only) bit j of word i: shapes i, j joined
  static constexpr int LIST_W = (NID + 3) / 4 > N ? (NID + 3) / 4 : N;
  static constexpr int LCAP = 16;                          // a level holds at most one pair per movable shape
  static constexpr int X_SCHED = X_LIST + LIST_W;          // bytes [R][LCAP]: numbers of the active pairs not held in registers, level by level
  static constexpr int X_PSTATE = align_up(X_SCHED + R * LCAP / 4, 4);   // bytes [G][16]: active-point bits of pair (r, k) at [k][r]
  static constexpr int X_BITMAP = X_PSTATE + GP * 4;       // 4 words: bit id set = pair id is active and not held in registers
  static constexpr int X_TAKEN = X_BITMAP + 4;             // 16-bit words [N]: bit l set = a colliding pair of the shape has level l
  static constexpr int X_LVL = X_TAKEN + (N + 1) / 2;      // bytes [NID]: level of pair id
  static constexpr int X_STAGE = X_LVL + (NID + 3) / 4;    // staged manifolds, kManW words each
  static constexpr int X_DUMP = X_STAGE;                   // (once the staged manifolds are taken) 2N+1 words that swallow the
                                                           // velocity stores of shapes no impulse moves (offsets 0, N, 2N)
  static constexpr int X_POOL = X_STAGE + NREG * kManW;
  static_assert(NREG * kManW >= 2 * N + 1 && L.pos_x == 0 && L.pos_y == N, "dump slots do not fit the staging area");
  // LDS budget of one environment: a CU's 160 KiB shared by the lanes of eight wavefronts' worth of
  // 16-lane environments (or four wavefronts' worth of 8-lane ones): 1280 words.  The stride is an odd
  // multiple of G words, so that the same word of different environments falls into different banks.
  static constexpr int MAX_STRIDE = (1280 / G - ((1280 / G) % 2 == 0 ? 1 : 0)) * G;
  static constexpr int POOL_WANT = NP > NREG ? (NP - NREG < 8 ? NP - NREG : 8) : 0;
  static constexpr int POOL_FIT = MAX_STRIDE > X_POOL ? (MAX_STRIDE - X_POOL) / kRecW : 0;
  static constexpr int POOL = POOL_WANT < POOL_FIT ? POOL_WANT : POOL_FIT;
  static_assert(NREG + POOL >= 16 && NP - NREG - POOL <= SPILL, "spill room of the record");
  static constexpr int LDS_WORDS = X_POOL + POOL * kRecW;
  static constexpr int LDS_STRIDE = align_up(LDS_WORDS - G, 2 * G) + G;
  static_assert(LDS_STRIDE >= LDS_WORDS && (LDS_STRIDE / G) % 2 == 1 && LDS_STRIDE <= MAX_STRIDE, "stride rule");
  static constexpr int LDS_BYTES = LDS_STRIDE * EPW * 4;
};

struct Params {   // device copy of k2d_params with the substep precomputed
  float h, gravity_y;
  int n_substeps, n_iters, warm_start;
  float alpha, beta, gamma, rho, slop, rest_thr;
  int clip_thr;
  float joint_alpha, joint_beta, tie_eps;
  int n_batches;   // batched schedule (A.8): batches per sweep of the collision constraints, 0 = not used
  int lowest_free_level;   // visiting order of the colliding pairs: 0 = tournament order, 1 = level after level
};

__device__ __forceinline__ int f2i(float f) { return __float_as_int(f); }

// Inclusive prefix sum, sum and OR over the G lanes of an environment's group.  A group of 16 is one DPP
// row (shifts within the row read zero where there is no source lane; rotations reach every lane); a
// group of 8 is half a row: shifts are masked at the group's edge, sums and ORs use the exchanges within
// a quad and the mirror of the half row.
#define K2D_DPP(v, ctrl, bc) __builtin_amdgcn_update_dpp(0, (int)(v), ctrl, 0xf, 0xf, bc)
template <int G>
__device__ __forceinline__ unsigned group_prefix_sum(unsigned v, int k) {
  if constexpr (G == 16) {
    v += (unsigned)K2D_DPP(v, 0x111, true);
    v += (unsigned)K2D_DPP(v, 0x112, true);
    v += (unsigned)K2D_DPP(v, 0x114, true);
    v += (unsigned)K2D_DPP(v, 0x118, true);
  } else {
    unsigned t = (unsigned)K2D_DPP(v, 0x111, true); v += (k >= 1) ? t : 0u;
    t = (unsigned)K2D_DPP(v, 0x112, true); v += (k >= 2) ? t : 0u;
    t = (unsigned)K2D_DPP(v, 0x114, true); v += (k >= 4) ? t : 0u;
  }
  return v;
}
template <int G>
__device__ __forceinline__ unsigned group_sum(unsigned v) {
  if constexpr (G == 16) {
    v += (unsigned)K2D_DPP(v, 0x121, false);
    v += (unsigned)K2D_DPP(v, 0x122, false);
    v += (unsigned)K2D_DPP(v, 0x124, false);
    v += (unsigned)K2D_DPP(v, 0x128, false);
  } else {
    v += (unsigned)K2D_DPP(v, 0xB1, false);    // lanes 0<->1, 2<->3 of every quad
    v += (unsigned)K2D_DPP(v, 0x4E, false);    // lanes 0<->2, 1<->3
    v += (unsigned)K2D_DPP(v, 0x141, false);   // mirror of the half row: the other quad's sum
  }
  return v;
}
template <int G>
__device__ __forceinline__ unsigned group_or(unsigned v) {
  if constexpr (G == 16) {
    v |= (unsigned)K2D_DPP(v, 0x121, false);
    v |= (unsigned)K2D_DPP(v, 0x122, false);
    v |= (unsigned)K2D_DPP(v, 0x124, false);
    v |= (unsigned)K2D_DPP(v, 0x128, false);
  } else {
    v |= (unsigned)K2D_DPP(v, 0xB1, false);
    v |= (unsigned)K2D_DPP(v, 0x4E, false);
    v |= (unsigned)K2D_DPP(v, 0x141, false);
  }
  return v;
}

// A workgroup of the step kernel is one wavefront, and the memory operations of one wavefront are
// performed in the order they are issued: lanes that exchange data through LDS need no hardware barrier
// and no wait, only a point that the compiler does not move memory accesses across.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// sin, cos and tanh as fixed sequences of IEEE fp32 operations (no maths-library call, no fused
// multiply-add): quadrant reduction against a three-term split of pi/2, then polynomials in r*r; tanh
// by polynomial below 0.55 and through e^{2|x|} above.  Any implementation that performs the same
// operations in the same order produces the same bits, which is what lets a CPU run of the same step be
// compared with this one exactly.  Absolute error below 1.5e-7.
__device__ __forceinline__ void k2d_sincos(float x, float& sn, float& cs) {
  const float q = rintf(x * 0x1.45f306p-1f);
  float r = x - q * 0x1.92p+0f;
  r = r - q * 0x1.fb4p-12f;
  r = r - q * 0x1.4442d2p-24f;
  const float z = r * r;
  const float s = r + (r * z) * ((-0x1.9b021cp-13f * z + 0x1.110ccap-7f) * z + -0x1.555554p-3f);
  const float c = (1.0f - 0.5f * z) + (z * z) * ((0x1.9c05c8p-16f * z + -0x1.6c1354p-10f) * z + 0x1.555554p-5f);
  const int quad = (int)q & 3;
  const float a = (quad & 1) ? c : s;      // value that lands in the sine slot before the sign
  const float b = (quad & 1) ? s : c;
  sn = (quad & 2) ? -a : a;
  cs = ((quad + 1) & 2) ? -b : b;
}
__device__ __forceinline__ float k2d_tanh(float x) {
  const float a = fabsf(x);
  float y;
  if (a < 0.55f) {
    const float z = a * a;
    y = a + (a * z) * ((((-0x1.b3b502p-8f * z + 0x1.5d873cp-6f) * z + -0x1.b9aa82p-5f) * z + 0x1.111018p-3f) * z +
                       -0x1.555554p-2f);
  } else {
    const float t2 = 2.0f * a;
    const float t = (t2 < 40.0f) ? t2 : 40.0f;
    const float n = rintf(t * 0x1.715476p+0f);
    float r = t - n * 0x1.62cp-1f;
    r = r - n * 0x1.217f7ep-12f;
    float e = (1.0f + r) + (r * r) * ((((0x1.6d435ap-10f * r + 0x1.120b66p-7f) * r + 0x1.5554e8p-5f) * r +
                                       0x1.5554dcp-3f) * r + 0.5f);
    e = ldexpf(e, (int)n);
    y = 1.0f - 2.0f / (e + 1.0f);
  }
  return x < 0.0f ? -y : y;
}
__device__ __forceinline__ float i2f(int i) { return __int_as_float(i); }

// Two-term products round once: a.b = fma(ax, bx, ay*by), a x b = fma(ax, by, -(ay*bx)); an impulse is
// applied as v = fma(1/m, j, v).  Everything else is one operation, one rounding (contraction is off).
__device__ __forceinline__ float dot2(float ax, float ay, float bx, float by) { return fmaf(ax, bx, ay * by); }
__device__ __forceinline__ float cross2(float ax, float ay, float bx, float by) { return fmaf(ax, by, -(ay * bx)); }
// an impulse (jx, jy) at offset (rx, ry) from the centre of mass (A.2)
__device__ __forceinline__ void apply_impulse(float& vx, float& vy, float& w, float im, float ii, float jx, float jy,
                                              float rx, float ry) {
  vx = fmaf(im, jx, vx);
  vy = fmaf(im, jy, vy);
  w = fmaf(ii, cross2(rx, ry, jx, jy), w);
}

// One active pair of the current substep.  Body indices and per-point activity are packed in `ab`.
struct PairRec {
  float nx, ny, mu, corr;        // unit normal a->b; friction coefficient; positional-correction length
  int ab;                        // a | b<<8 | active0<<16 | active1<<17 | pair id<<18
  float rax[2], ray[2], rbx[2], rby[2], mass_n[2], mass_t[2], bias[2], rest[2], lam_n[2], lam_t[2];
};

// LDS pointers are passed with their address space spelled out, so that a record access can never
// degrade into a flat access when the LDS and the HBM (spill) variants of a code path are merged.
using LdsF = __attribute__((address_space(3))) float*;
using LdsCF = const __attribute__((address_space(3))) float*;
__device__ __forceinline__ LdsF to_lds(float* p) { return (LdsF)p; }

template <class Ptr>
__device__ __forceinline__ void rec_store(Ptr p, const PairRec& r) {
  p[0] = r.nx; p[1] = r.ny; p[2] = r.mu; p[3] = r.corr; p[4] = i2f(r.ab);
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    auto q = p + 5 + 10 * k;
    q[0] = r.rax[k]; q[1] = r.ray[k]; q[2] = r.rbx[k]; q[3] = r.rby[k]; q[4] = r.mass_n[k];
    q[5] = r.mass_t[k]; q[6] = r.bias[k]; q[7] = r.rest[k]; q[8] = r.lam_n[k]; q[9] = r.lam_t[k];
  }
}
template <class Ptr>
__device__ __forceinline__ void rec_load(Ptr p, PairRec& r) {
  r.nx = p[0]; r.ny = p[1]; r.mu = p[2]; r.corr = p[3]; r.ab = f2i(p[4]);
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    auto q = p + 5 + 10 * k;
    r.rax[k] = q[0]; r.ray[k] = q[1]; r.rbx[k] = q[2]; r.rby[k] = q[3]; r.mass_n[k] = q[4];
    r.mass_t[k] = q[5]; r.bias[k] = q[6]; r.rest[k] = q[7]; r.lam_n[k] = q[8]; r.lam_t[k] = q[9];
  }
}

// Collision manifold (Table 2) of one pair: unit normal from a to b, up to two points.
struct Manifold {
  float nx = 0.f, ny = 0.f;
  float px[2] = {0.f, 0.f}, py[2] = {0.f, 0.f}, pen[2] = {0.f, 0.f};
  bool valid[2] = {false, false};
};

template <class K>
struct Step {
  static constexpr k2d_layout L = K::L;
  static constexpr int N = K::N, P = K::P, G = K::G;

  // ---- LDS accessors (E = base of this environment's image) ----
  static __device__ __forceinline__ float2 wv(const float* E, int i, int p) {
    return *reinterpret_cast<const float2*>(E + K::X_WV + 2 * (i * P + p));
  }
  static __device__ __forceinline__ float2 wn(const float* E, int i, int p) {
    return *reinterpret_cast<const float2*>(E + K::X_WN + 2 * (i * P + p));
  }

  // Pair k of round r of the round-robin tournament; returns false for the phantom's pair.
  static __device__ __forceinline__ bool sched_pair(int r, int k, int& a, int& b) {
    int x, y;
    if (k == 0) {
      x = K::M - 1;
      y = r;
    } else {
      x = r + k;
      if (x >= K::M - 1) x -= K::M - 1;
      y = r - k;
      if (y < 0) y += K::M - 1;
    }
    a = min(x, y);
    b = max(x, y);
    return k < K::PPR && b < N;
  }
  static __device__ __forceinline__ int pair_index(int a, int b) { return a * (2 * N - a - 1) / 2 + (b - a - 1); }

  // ---- A.3.2: circle a, circle b ----
  static __device__ __forceinline__ void manifold_cc(float pax, float pay, float ra, float pbx, float pby, float rb,
                                                     Manifold& m) {
    float dx = pbx - pax, dy = pby - pay;
    float len = sqrtf(dot2(dx, dy, dx, dy));
    bool ok = len > 1e-9f;
    m.nx = ok ? dx / len : 1.f;
    m.ny = ok ? dy / len : 0.f;
    m.px[0] = pax + ra * m.nx;
    m.py[0] = pay + ra * m.ny;
    m.pen[0] = ra + rb - len;
    m.valid[0] = true;
  }

  // ---- A.3.3: polygon a (index pa in the world arrays), circle b ----
  static __device__ __forceinline__ void manifold_pc(const float* E, int pa, int na, float cx, float cy, float rb,
                                                     Manifold& m) {
    float best_d2 = INFINITY, qx = 0.f, qy = 0.f;
    float smax = -INFINITY, snx = 0.f, sny = 0.f;
    float2 v = wv(E, 0, pa);
    // (vertex slot 3 of a triangle repeats vertex 0; its fourth "edge" is computed and thrown away, so
    // that the loop has no branch)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool real = i < 3 || na == 4;
      float2 v1 = wv(E, (i + 1) & 3, pa);
      float2 nr = wn(E, i, pa);
      float ex = v1.x - v.x, ey = v1.y - v.y;
      float rx = cx - v.x, ry = cy - v.y;
      float t = dot2(rx, ry, ex, ey) / dot2(ex, ey, ex, ey);
      t = fminf(fmaxf(t, 0.f), 1.f);
      float qix = v.x + t * ex, qiy = v.y + t * ey;
      float dqx = cx - qix, dqy = cy - qiy;
      float d2 = dot2(dqx, dqy, dqx, dqy);
      if (real && d2 < best_d2) { best_d2 = d2; qx = qix; qy = qiy; }
      float s = dot2(nr.x, nr.y, rx, ry);
      if (real && s > smax) { smax = s; snx = nr.x; sny = nr.y; }
      v = v1;
    }
    if (smax <= 0.f) {   // centre inside the polygon: the face of largest signed distance
      m.nx = snx; m.ny = sny;
      m.pen[0] = rb - smax;
      m.px[0] = cx - smax * snx;
      m.py[0] = cy - smax * sny;
    } else {
      float dist = sqrtf(best_d2);
      float dqx = cx - qx, dqy = cy - qy;
      m.nx = dqx / dist; m.ny = dqy / dist;
      m.pen[0] = rb - dist;
      m.px[0] = qx; m.py[0] = qy;
    }
    m.valid[0] = true;
  }

  // Largest over X's faces of the smallest signed distance of Y's vertices to the face (A.3.4).
  static __device__ __forceinline__ void face_query(const float* E, int px, int nx_, const float2 (&yw)[4], int ny_,
                                                    float& best, int& idx) {
    best = -INFINITY;
    idx = 0;
    // (vertex slot 3 of a triangle repeats vertex 0, which leaves the minimum over Y's vertices as it is;
    // the fourth "face" of a triangle X is computed and thrown away: no branch in the loops)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float2 nr = wn(E, i, px);
      float2 w = wv(E, i, px);
      float smin = INFINITY;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float s = dot2(nr.x, nr.y, yw[k].x - w.x, yw[k].y - w.y);
        smin = (s < smin) ? s : smin;
      }
      if ((i < 3 || nx_ == 4) && smin > best) { best = smin; idx = i; }
    }
  }

  // ---- A.3.4: polygon a, polygon b (indices in the world arrays) ----
  static __device__ __forceinline__ void manifold_pp(const float* E, int pa, int na, int pb, int nb, float tie_eps,
                                                     Manifold& m) {
    float2 aw[4], bw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { aw[i] = wv(E, i, pa); bw[i] = wv(E, i, pb); }
    float sa, sb;
    int ia, ib;
    face_query(E, pa, na, bw, nb, sa, ia);
    face_query(E, pb, nb, aw, na, sb, ib);
    if (fmaxf(sa, sb) >= 0.f) return;   // a separating axis exists
    bool ref_b = sb > sa + tie_eps;
    int pr = ref_b ? pb : pa, nr_ = ref_b ? nb : na, ir = ref_b ? ib : ia;
    int pi = ref_b ? pa : pb, ni = ref_b ? na : nb;
    float2 nref = wn(E, ir, pr);
    float2 r1 = wv(E, ir, pr);
    float2 r2 = wv(E, (ir + 1 == nr_) ? 0 : ir + 1, pr);
    int jinc = 0;
    float dmin = INFINITY;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float2 nj = wn(E, j, pi);
      float d = dot2(nj.x, nj.y, nref.x, nref.y);
      if ((j < 3 || ni == 4) && d < dmin) { dmin = d; jinc = j; }
    }
    float2 v0 = wv(E, jinc, pi);
    float2 v1 = wv(E, (jinc + 1 == ni) ? 0 : jinc + 1, pi);
    float tx = -nref.y, ty = nref.x;
    float u0 = dot2(tx, ty, v0.x - r1.x, v0.y - r1.y);
    float u1 = dot2(tx, ty, v1.x - r1.x, v1.y - r1.y);
    float len = dot2(tx, ty, r2.x - r1.x, r2.y - r1.y);
    if ((u0 < 0.f && u1 < 0.f) || (u0 > len && u1 > len)) return;
    m.nx = ref_b ? -nref.x : nref.x;
    m.ny = ref_b ? -nref.y : nref.y;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      float uk = k ? u1 : u0;
      float uc = fminf(fmaxf(uk, 0.f), len);
      float x = k ? v1.x : v0.x, y = k ? v1.y : v0.y;
      if (uc != uk) {
        float s = (uc - u0) / (u1 - u0);
        x = v0.x + s * (v1.x - v0.x);
        y = v0.y + s * (v1.y - v0.y);
      }
      m.px[k] = x; m.py[k] = y;
      m.pen[k] = -dot2(nref.x, nref.y, x - r1.x, y - r1.y);
      m.valid[k] = true;
    }
  }

  // Relative velocity of the contact points, v_a + w_a x r_a - v_b - w_b x r_b (A.3.5).
  static __device__ __forceinline__ void rel_vel(float vax, float vay, float wa, float rax, float ray, float vbx,
                                                 float vby, float wb, float rbx, float rby, float& x, float& y) {
    x = fmaf(wb, rby, fmaf(-wa, ray, vax) - vbx);
    y = fmaf(-wb, rbx, fmaf(wa, rax, vay) - vby);
  }

  // One visit of an active pair in a solver sweep: per point, normal impulse then friction impulse,
  // accumulated and clamped (A.3.5, A.3.6, A.7), on the velocities of its two bodies.
  static __device__ __forceinline__ void solve_points(PairRec& rc, float ima, float iia, float imb, float iib,
                                                      float& vax, float& vay, float& wa, float& vbx, float& vby,
                                                      float& wb) {
    const float tx = -rc.ny, ty = rc.nx;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      if ((rc.ab >> (16 + k)) & 1) {
        float rx, ry;
        rel_vel(vax, vay, wa, rc.rax[k], rc.ray[k], vbx, vby, wb, rc.rbx[k], rc.rby[k], rx, ry);
        float vn = dot2(rc.nx, rc.ny, rx, ry);
        float dl = rc.mass_n[k] * (vn + rc.rest[k] + rc.bias[k]);
        float ln = fmaxf(rc.lam_n[k] + dl, 0.f);
        dl = ln - rc.lam_n[k];
        rc.lam_n[k] = ln;
        float jx = (-dl) * rc.nx, jy = (-dl) * rc.ny;
        apply_impulse(vax, vay, wa, ima, iia, jx, jy, rc.rax[k], rc.ray[k]);
        apply_impulse(vbx, vby, wb, imb, iib, -jx, -jy, rc.rbx[k], rc.rby[k]);
        rel_vel(vax, vay, wa, rc.rax[k], rc.ray[k], vbx, vby, wb, rc.rbx[k], rc.rby[k], rx, ry);
        float vt = dot2(tx, ty, rx, ry);
        float dt_ = -rc.mass_t[k] * vt;
        float lim = rc.mu * ln;
        float lt = fminf(fmaxf(rc.lam_t[k] + dt_, -lim), lim);
        dt_ = lt - rc.lam_t[k];
        rc.lam_t[k] = lt;
        float fx = dt_ * tx, fy = dt_ * ty;
        apply_impulse(vax, vay, wa, ima, iia, fx, fy, rc.rax[k], rc.ray[k]);
        apply_impulse(vbx, vby, wb, imb, iib, -fx, -fy, rc.rbx[k], rc.rby[k]);
      }
    }
  }
  // Batched schedule (A.8): point q of a pair solved on private copies of the two bodies' velocities (the
  // arithmetic of solve_points); returns the normal impulse (jx, jy) and the friction impulse (fx, fy)
  // that a receives, for the batch to apply afterwards, and the contact arms.  (With more than one batch
  // the two points of a pair never share a batch, so one visit handles at most one of them: its
  // constants are picked by q, which keeps the record in registers.)
  static __device__ __forceinline__ void point_impulses(PairRec& rc, bool q, float ima, float iia, float imb, float iib,
                                                        float vax, float vay, float wa, float vbx, float vby, float wb,
                                                        float& jx, float& jy, float& fx, float& fy, float& rax,
                                                        float& ray, float& rbx, float& rby) {
    const float tx = -rc.ny, ty = rc.nx;
    rax = q ? rc.rax[1] : rc.rax[0]; ray = q ? rc.ray[1] : rc.ray[0];
    rbx = q ? rc.rbx[1] : rc.rbx[0]; rby = q ? rc.rby[1] : rc.rby[0];
    const float mass_n = q ? rc.mass_n[1] : rc.mass_n[0], mass_t = q ? rc.mass_t[1] : rc.mass_t[0];
    const float rest = q ? rc.rest[1] : rc.rest[0], bias = q ? rc.bias[1] : rc.bias[0];
    const float lam_n = q ? rc.lam_n[1] : rc.lam_n[0], lam_t = q ? rc.lam_t[1] : rc.lam_t[0];
    float rx, ry;
    rel_vel(vax, vay, wa, rax, ray, vbx, vby, wb, rbx, rby, rx, ry);
    float vn = dot2(rc.nx, rc.ny, rx, ry);
    float dl = mass_n * (vn + rest + bias);
    float ln = fmaxf(lam_n + dl, 0.f);
    dl = ln - lam_n;
    jx = (-dl) * rc.nx; jy = (-dl) * rc.ny;
    apply_impulse(vax, vay, wa, ima, iia, jx, jy, rax, ray);
    apply_impulse(vbx, vby, wb, imb, iib, -jx, -jy, rbx, rby);
    rel_vel(vax, vay, wa, rax, ray, vbx, vby, wb, rbx, rby, rx, ry);
    float vt = dot2(tx, ty, rx, ry);
    float dt_ = -mass_t * vt;
    float lim = rc.mu * ln;
    float lt = fminf(fmaxf(lam_t + dt_, -lim), lim);
    dt_ = lt - lam_t;
    fx = dt_ * tx; fy = dt_ * ty;
    if (q) { rc.lam_n[1] = ln; rc.lam_t[1] = lt; }
    else { rc.lam_n[0] = ln; rc.lam_t[0] = lt; }
  }
  // Where the two points of pair `id` (tournament order) fall in the batched schedule: the points, two per
  // pair, are dealt in turn over n_b batches.  Returns batch | place<<8 of point 0, the same <<16 of point 1.
  static __device__ __forceinline__ int batch_places(int id, int n_b) {
    constexpr int odd = N & 1;   // the phantom's pair (slot 0 of every round) is not a pair
    const int dense = (id / K::GP) * (K::PPR - odd) + (id % K::GP) - odd;
    const int s0 = 2 * dense;
    const int j0 = s0 / n_b, b0 = s0 - j0 * n_b;
    int b1 = b0 + 1, j1 = j0;
    if (b1 == n_b) { b1 = 0; j1 = j0 + 1; }
    return b0 | (j0 << 8) | (b1 << 16) | (j1 << 24);
  }
  // Warm starting of one pair (A.7): re-apply the kept accumulated impulses.
  static __device__ __forceinline__ void warm_points(const PairRec& rc, float ima, float iia, float imb, float iib,
                                                     float& vax, float& vay, float& wa, float& vbx, float& vby,
                                                     float& wb) {
    const float tx = -rc.ny, ty = rc.nx;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      if ((rc.ab >> (16 + k)) & 1) {
        float jx = (-rc.lam_n[k]) * rc.nx + rc.lam_t[k] * tx;
        float jy = (-rc.lam_n[k]) * rc.ny + rc.lam_t[k] * ty;
        apply_impulse(vax, vay, wa, ima, iia, jx, jy, rc.rax[k], rc.ray[k]);
        apply_impulse(vbx, vby, wb, imb, iib, -jx, -jy, rc.rbx[k], rc.rby[k]);
      }
    }
  }

  // A pair whose record is not held in registers (LDS pool or HBM): velocities through LDS, the bodies'
  // constants looked up per visit.  WARM selects warm starting instead of a solver visit.
  template <bool WARM>
  static __device__ __forceinline__ void visit_pair(float* E, PairRec& rc, unsigned fixed) {
    const int a = rc.ab & 0xff, b = (rc.ab >> 8) & 0xff;
    float vax = E[L.vel_x + a], vay = E[L.vel_y + a], wa = E[L.omega + a];
    float vbx = E[L.vel_x + b], vby = E[L.vel_y + b], wb = E[L.omega + b];
    const float ima = E[L.inv_mass + a], iia = E[L.inv_inertia + a];
    const float imb = E[L.inv_mass + b], iib = E[L.inv_inertia + b];
    if (WARM) warm_points(rc, ima, iia, imb, iib, vax, vay, wa, vbx, vby, wb);
    else solve_points(rc, ima, iia, imb, iib, vax, vay, wa, vbx, vby, wb);
    if (!((fixed >> a) & 1u)) { E[L.vel_x + a] = vax; E[L.vel_y + a] = vay; E[L.omega + a] = wa; }
    if (!((fixed >> b) & 1u)) { E[L.vel_x + b] = vbx; E[L.vel_y + b] = vby; E[L.omega + b] = wb; }
  }

  // An active pair that a lane keeps in registers for one substep.
  struct Own {
    PairRec rc;
    float ima, iia, imb, iib;
    int pa, pb;   // shape indices
    int sa, sb;   // where the velocities go back: the shape itself, or the dump slot if no impulse moves it
    int id;       // pair id in tournament order, -1 = nothing held
    int lv;       // dependency level of this substep
  };
  // Substep constants of an active pair from its manifold (A.3.5-A.3.7) and the accumulated impulses it
  // keeps (A.7).  `w` packs a | b<<8 | active0<<16 | active1<<17 | pair id<<18 | active bits of the
  // previous substep<<25; `lam` holds the stored impulses (n0, t0, n1, t1).
  static __device__ __forceinline__ void presolve(const float* E, const Params& prm, const Manifold& m, int w,
                                                  float4 lam, PairRec& rc, float& ima, float& iia, float& imb,
                                                  float& iib) {
    const int a = w & 0xff, b = (w >> 8) & 0xff;
    const bool act0 = (w >> 16) & 1, act1 = (w >> 17) & 1;
    const unsigned prev = (unsigned)(w >> 25) & 3u;
    rc.nx = m.nx; rc.ny = m.ny;
    rc.ab = w & 0x1ffffff;
    ima = E[L.inv_mass + a]; iia = E[L.inv_inertia + a];
    imb = E[L.inv_mass + b]; iib = E[L.inv_inertia + b];
    const float fa = E[L.friction + a], fb = E[L.friction + b];
    const float e = fminf(E[L.restitution + a], E[L.restitution + b]);   // A.3.5
    rc.mu = sqrtf(fa * fa + fb * fb);                                        // A.3.6
    const float pax = E[L.pos_x + a], pay = E[L.pos_y + a], pbx = E[L.pos_x + b], pby = E[L.pos_y + b];
    const float vax = E[L.vel_x + a], vay = E[L.vel_y + a], wa = E[L.omega + a];
    const float vbx = E[L.vel_x + b], vby = E[L.vel_y + b], wb = E[L.omega + b];
    const float tx = -m.ny, ty = m.nx;
    float pen = 0.f;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const bool on = q ? act1 : act0;
      rc.rax[q] = m.px[q] - pax; rc.ray[q] = m.py[q] - pay;
      rc.rbx[q] = m.px[q] - pbx; rc.rby[q] = m.py[q] - pby;
      float ran = cross2(rc.rax[q], rc.ray[q], m.nx, m.ny), rbn = cross2(rc.rbx[q], rc.rby[q], m.nx, m.ny);
      float rat = cross2(rc.rax[q], rc.ray[q], tx, ty), rbt = cross2(rc.rbx[q], rc.rby[q], tx, ty);
      float kn = ima + imb + ran * ran * iia + rbn * rbn * iib;
      float kt = ima + imb + rat * rat * iia + rbt * rbt * iib;
      rc.mass_n[q] = on ? 1.f / kn : 0.f;
      rc.mass_t[q] = on ? 1.f / kt : 0.f;
      rc.bias[q] = prm.alpha * fmaxf(m.pen[q] - prm.slop, 0.f);            // A.3.7
      // restitution target -e*v_r (A.3.5), v_r sampled here: after motors and thrusters,
      // before any constraint impulse; slow approaches take e = 0
      float rx, ry;
      rel_vel(vax, vay, wa, rc.rax[q], rc.ray[q], vbx, vby, wb, rc.rbx[q], rc.rby[q], rx, ry);
      float vn0 = dot2(m.nx, m.ny, rx, ry);
      rc.rest[q] = (vn0 > prm.rest_thr) ? e * vn0 : 0.f;
      bool keep = prm.warm_start && on && ((prev >> q) & 1u);                 // A.7
      rc.lam_n[q] = keep ? (q ? lam.z : lam.x) : 0.f;
      rc.lam_t[q] = keep ? (q ? lam.w : lam.y) : 0.f;
      if (on) pen = fmaxf(pen, m.pen[q]);
    }
    rc.corr = prm.beta * fmaxf(pen - prm.slop, 0.f) / (ima + imb);          // A.3.7
  }
  // The lane that keeps pair idx picks its staged manifold up and derives the record in its own registers.
  static __device__ __forceinline__ void take_own(const float* E, const float* Rg, const Params& prm, int idx,
                                                  unsigned fixed, int kept_id, float4 kept_lam, Own& o) {
    LdsCF p = (LdsCF)(E + K::X_STAGE + idx * K::kManW);
    Manifold m;
    m.nx = p[0]; m.ny = p[1];
    m.px[0] = p[2]; m.py[0] = p[3]; m.pen[0] = p[4];
    m.px[1] = p[5]; m.py[1] = p[6]; m.pen[1] = p[7];
    const int w = f2i(p[8]);
    const int a = w & 0xff, b = (w >> 8) & 0xff;
    float4 lam = make_float4(0.f, 0.f, 0.f, 0.f);
    if (prm.warm_start && ((w >> 25) & 3)) {   // the impulses it accumulated: still in this lane, or in the HBM record
      if (((w >> 18) & 127) == kept_id) lam = kept_lam;
      else lam = *reinterpret_cast<const float4*>(Rg + L.lambda + 4 * pair_index(a, b));
    }
    presolve(E, prm, m, w, lam, o.rc, o.ima, o.iia, o.imb, o.iib);
    o.pa = a; o.pb = b;
    o.sa = ((fixed >> a) & 1u) ? K::X_DUMP - L.vel_x : a;
    o.sb = ((fixed >> b) & 1u) ? K::X_DUMP - L.vel_x : b;
    o.id = (w >> 18) & 127;
    o.lv = -1;
  }
  template <bool WARM>
  static __device__ __forceinline__ void visit_own(float* E, Own& o) {
    float vax = E[L.vel_x + o.pa], vay = E[L.vel_y + o.pa], wa = E[L.omega + o.pa];
    float vbx = E[L.vel_x + o.pb], vby = E[L.vel_y + o.pb], wb = E[L.omega + o.pb];
    if (WARM) warm_points(o.rc, o.ima, o.iia, o.imb, o.iib, vax, vay, wa, vbx, vby, wb);
    else solve_points(o.rc, o.ima, o.iia, o.imb, o.iib, vax, vay, wa, vbx, vby, wb);
    E[L.vel_x + o.sa] = vax; E[L.vel_y + o.sa] = vay; E[L.omega + o.sa] = wa;
    E[L.vel_x + o.sb] = vbx; E[L.vel_y + o.sb] = vby; E[L.omega + o.sb] = wb;
  }
};

// RESET: after step s an environment e with reset_level[s * n_envs + e] = l >= 0 starts a new episode from
// record l of `levels` (what k2d_reset does between launches, without leaving the kernel).
// BATCHED: the collision constraints of a sweep are solved in the batches of A.8 instead of level by level.
template <class K, bool RESET, bool BATCHED>
__global__ void __launch_bounds__(64, K::EPW == 4 ? 2 : 1) k2d_step_kernel(float* __restrict__ state, const float* __restrict__ actions,
                                                      int n_envs, int n_steps, Params prm,
                                                      const float* __restrict__ levels, int n_level_records,
                                                      const int32_t* __restrict__ reset_level,
                                                      const int32_t* __restrict__ order
#ifdef K2D_PHASE_TIMERS
                                                      , unsigned long long* __restrict__ phase_clocks
#endif
                                                      ) {
  using S = Step<K>;
  constexpr k2d_layout L = K::L;
  constexpr int N = K::N, P = K::P, J = K::J, T = K::T, G = K::G, R = K::R, GP = K::GP, H = K::H;
  extern __shared__ __align__(16) float lds[];

  const int lane = threadIdx.x;
  const int g = lane / G, k = lane % G;
  const int kp = k % GP, rpar = k / GP;   // this lane's pair slot within a round, and which rounds it takes
  // which environments this wavefront steps: a launch may come with an ordering of the environments
  // (slot -> environment, -1 = none) that puts similar ones together; without one, slot s is environment s
  const int slot0 = blockIdx.x * K::EPW;
  auto env_of = [&](int slot) { return order ? order[slot] : (slot < n_envs ? slot : -1); };
  const int env = env_of(slot0 + g);
  const bool env_ok = env >= 0;
  float* E = lds + g * K::LDS_STRIDE;
  float* Rg = state + (size_t)(env_ok ? env : 0) * K::REC_WORDS;   // this environment's HBM record

  // ---- load the scene description into LDS, one environment after the other, 64 words at a time ----
  for (int e = 0; e < K::EPW; ++e) {
    float* dst = lds + e * K::LDS_STRIDE;
    const int env_e = env_of(slot0 + e);
    if (env_e >= 0) {
      const float* src = state + (size_t)env_e * K::REC_WORDS;
      for (int w = lane; w < L.scene_words; w += 64) dst[w] = src[w];
    } else {
      for (int w = lane; w < L.scene_words; w += 64) dst[w] = 0.f;   // all-inactive padding environment
    }
  }
  wave_sync();
  unsigned my_r = 0u;   // the rounds this lane takes
  for (int r = 0; r < R; ++r)
    if (r % H == rpar) my_r |= 1u << r;

#ifdef K2D_PHASE_TIMERS
  long long t_acc[kT_Count] = {};
  long long t_last = clock64();
  unsigned long long t_pair_levels = 0, t_joint_levels = 0;
#endif
  int step = 0;
  bool first = true;
  do {   // (one pass, unless environments are re-initialised on the way)
  // ---- derived data: per launch, and again after environments of the wavefront started a new episode ----
  for (int i = k; i < N; i += G) {
    float sn, cs;
    k2d_sincos(E[L.theta + i], sn, cs);
    E[K::X_COS + i] = cs;
    E[K::X_SIN + i] = sn;
    E[K::X_JOINED + i] = i2f(0);
  }
  wave_sync();
  // joints: lane j of the group owns joint j for the whole episode
  bool j_live = false, j_fixed = false, j_motor = false, j_limited = false;
  int ja = 0, jb = 0;
  float j_aax = 0.f, j_aay = 0.f, j_abx = 0.f, j_aby = 0.f, j_thf = 0.f, j_speed = 0.f, j_power = 0.f;
  float j_accx = 0.f, j_accy = 0.f, j_acca = 0.f;
  if (k < J) {
    int fl = f2i(E[L.joint_flags + k]);
    ja = f2i(E[L.joint_a + k]);
    jb = f2i(E[L.joint_b + k]);
    bool idx_ok = ja >= 0 && ja < N && jb >= 0 && jb < N && ja != jb;
    if (!idx_ok) { ja = 0; jb = 0; }
    j_fixed = (fl >> 1) & 1;
    j_motor = (fl >> 2) & 1;
    j_limited = ((fl >> 4) & 1) && !j_fixed;
    j_live = (fl & 1) && idx_ok && (f2i(E[L.shape_flags + ja]) & 1) && (f2i(E[L.shape_flags + jb]) & 1) &&
             (E[L.inv_mass + ja] + E[L.inv_mass + jb]) > 0.f;
    j_aax = E[L.anchor_a_x + k]; j_aay = E[L.anchor_a_y + k];
    j_abx = E[L.anchor_b_x + k]; j_aby = E[L.anchor_b_y + k];
    j_thf = E[L.theta_f + k]; j_speed = E[L.motor_speed + k]; j_power = E[L.motor_power + k];
    j_accx = E[L.acc_x + k]; j_accy = E[L.acc_y + k]; j_acca = E[L.acc_ang + k];
    if (!j_live) { j_accx = 0.f; j_accy = 0.f; j_acca = 0.f; }
    if (!j_fixed) j_acca = 0.f;
    if (j_live) {   // A.4: joined shapes do not collide
      atomicOr(reinterpret_cast<unsigned*>(E + K::X_JOINED + ja), 1u << jb);
      atomicOr(reinterpret_cast<unsigned*>(E + K::X_JOINED + jb), 1u << ja);
    }
    E[L.joint_flags + k] = i2f((fl & 23) | (j_live ? 8 : 0));
  }
  wave_sync();
  // Shapes that no impulse can move (no inverse mass, no inverse inertia; inactive ones too).  An
  // impulse leaves their velocity and position exactly as they are, so constraints that share only
  // such a shape do not depend on each other, and nothing is ever written back for them.
  unsigned static_mask = 0u;
  for (int i = 0; i < N; ++i)
    if (!(f2i(E[L.shape_flags + i]) & 1) || (E[L.inv_mass + i] == 0.f && E[L.inv_inertia + i] == 0.f))
      static_mask |= 1u << i;
  const bool ja_fix = (static_mask >> ja) & 1u, jb_fix = (static_mask >> jb) & 1u;
  // where a joint's velocity results go: the shape, or the dump slot if no impulse moves it
  const int jsa = ja_fix ? K::X_DUMP - L.vel_x : ja, jsb = jb_fix ? K::X_DUMP - L.vel_x : jb;
  // dependency levels of the joints: a joint runs one level after the last earlier joint that shares a
  // movable shape with it, so joints sharing a shape keep their index order, the others run side by side
  int j_level = 0, n_levels = 0;
  {
    unsigned long long last = 0ull;   // 4 bits per shape: next free level
    for (int q = 0; q < J; ++q) {
      int fl = f2i(E[L.joint_flags + q]);
      if (fl & 8) {
        int a = f2i(E[L.joint_a + q]), b = f2i(E[L.joint_b + q]);
        const bool da = !((static_mask >> a) & 1u), db = !((static_mask >> b) & 1u);
        int la = da ? (int)((last >> (4 * a)) & 15ull) : 0, lb = db ? (int)((last >> (4 * b)) & 15ull) : 0;
        int lv = max(la, lb);
        if (q == k) j_level = lv;
        n_levels = max(n_levels, lv + 1);
        if (da) last = (last & ~(15ull << (4 * a))) | ((unsigned long long)(lv + 1) << (4 * a));
        if (db) last = (last & ~(15ull << (4 * b))) | ((unsigned long long)(lv + 1) << (4 * b));
      }
    }
  }
  // levels are per environment; the wavefront walks as many as its deepest environment has
  int wave_levels = 0;
  for (int lv = 1; lv <= J; ++lv)
    if (__any(n_levels >= lv)) wave_levels = lv;
  // thrusters: lane t of the group owns thruster t
  bool t_live = false;
  int t_body = 0;
  float t_px = 0.f, t_py = 0.f, t_dx = 0.f, t_dy = 0.f, t_power = 0.f;
  if (k < T) {
    int fl = f2i(E[L.thr_flags + k]);
    t_body = f2i(E[L.thr_body + k]);
    bool idx_ok = t_body >= 0 && t_body < N;
    if (!idx_ok) t_body = 0;
    t_live = (fl & 1) && idx_ok && (f2i(E[L.shape_flags + t_body]) & 1);
    t_px = E[L.thr_pos_x + k]; t_py = E[L.thr_pos_y + k];
    k2d_sincos(E[L.thr_angle + k], t_dy, t_dx);
    t_power = E[L.thr_power + k];
  }
  // pairs: the lane tests pair k % GP of the rounds r with r % H == k / GP; eligibility is fixed for the episode
  unsigned char* table = reinterpret_cast<unsigned char*>(E + K::X_TABLE);
  unsigned char* cand_list = reinterpret_cast<unsigned char*>(E + K::X_LIST);
  unsigned char* sched = reinterpret_cast<unsigned char*>(E + K::X_SCHED);
  unsigned char* pstate = reinterpret_cast<unsigned char*>(E + K::X_PSTATE);
  unsigned* bitmap = reinterpret_cast<unsigned*>(E + K::X_BITMAP);
  unsigned elig = 0u, pp_mask = 0u, pc_mask = 0u;
  if (k < GP && first)
    for (int r = 0; r < 16; ++r) pstate[k * 16 + r] = 0;
  wave_sync();
  unsigned my_ab4[4] = {0u, 0u, 0u, 0u};   // this lane's pairs, a | b << 4, eight bits for each of its rounds
  for (int r = 0; r < R; ++r) {
    int a, b;
    if (((my_r >> r) & 1u) && S::sched_pair(r, kp, a, b)) {
      my_ab4[(r / H) >> 2] |= (unsigned)(a | (b << 4)) << (8 * ((r / H) & 3));
      if (b < P) pp_mask |= 1u << r;
      else if (a < P) pc_mask |= 1u << r;
      bool ok = (f2i(E[L.shape_flags + a]) & 1) && (f2i(E[L.shape_flags + b]) & 1) &&
                !((f2i(E[K::X_JOINED + a]) >> b) & 1) && (E[L.inv_mass + a] + E[L.inv_mass + b]) > 0.f;
      if (ok) {
        elig |= 1u << r;
        if (first && env_ok) {
          const unsigned char* ps = reinterpret_cast<const unsigned char*>(Rg + L.pair_state);
          pstate[kp * 16 + r] = ps[S::pair_index(a, b)] & 3;
        }
      }
    }
  }
  wave_sync();   // the joined-shape words share their LDS with the candidate list
  // Dependency levels of the collision constraints are kept from one substep to the next: they depend
  // only on which pairs collide, and that set is the same in most consecutive substeps.
  int wave_clevels = 0;       // levels of the wavefront's deepest environment
  bool levels_valid = false;  // false until the levels of the current set of colliding pairs are worked out
  // Likewise the list of candidate pairs (it stays in LDS) while no lane's candidates change, and the
  // accumulated impulses of the pairs a lane kept in registers (A.7): if the lane keeps the same pair in the
  // next substep they are taken from here, not from the HBM record.
  unsigned prev_cand = 0u, kind_tot = 0u;
  bool list_valid = false;
  int kept_id = -1;           // (the first of the lane's two pairs only: a second one is rare)
  float4 kept_lam = make_float4(0.f, 0.f, 0.f, 0.f);
  auto flush_kept = [&]() {   // the kept impulses into the HBM record (A.7 state of the environment)
    if (kept_id >= 0 && env_ok) {
      int a, b;
      S::sched_pair(kept_id / GP, kept_id % GP, a, b);
      *reinterpret_cast<float4*>(Rg + L.lambda + 4 * S::pair_index(a, b)) = kept_lam;
    }
  };
  unsigned short* taken = reinterpret_cast<unsigned short*>(E + K::X_TAKEN);
  unsigned char* lvl = reinterpret_cast<unsigned char*>(E + K::X_LVL);
  float* pool = E + K::X_POOL;
  float* spill = Rg + K::G_SPILL;
  const float h = prm.h;
  const int A = J + T;

  for (; step < n_steps; ++step) {
    float act_m = 0.f, act_t = 0.f;
    if (!order) {
      // the wavefront's environments are neighbours: their action rows are one contiguous run, read by the
      // first lanes of the wavefront as whole lines (one request instead of one per environment) and
      // handed out through LDS (the staging area is free between steps)
      const long first = ((long)step * n_envs + slot0) * A;
      if (lane < K::EPW * A && slot0 + lane / A < n_envs) lds[(lane / A) * K::LDS_STRIDE + K::X_STAGE + lane % A] = actions[first + lane];
      wave_sync();
      if (env_ok) {
        if (k < J) act_m = E[K::X_STAGE + k];
        if (k < T) act_t = E[K::X_STAGE + J + k];
      }
      wave_sync();
    } else if (env_ok) {
      const float* ap = actions + ((size_t)step * n_envs + env) * A;
      if (k < J) act_m = ap[k];
      if (k < T) act_t = ap[J + k];
    }
    if (prm.clip_thr) act_t = fminf(fmaxf(act_t, 0.f), 1.f);

    K2D_T(kT_Actions);
    for (int sub = 0; sub < prm.n_substeps; ++sub) {
      // ---- gravity (Alg. 1) and world-frame polygons ----
      for (int i = k; i < N; i += G) {
        bool act = f2i(E[L.shape_flags + i]) & 1;
        if (act && E[L.inv_mass + i] > 0.f) E[L.vel_y + i] = E[L.vel_y + i] + prm.gravity_y * h;
        if (i < P) {
          float cs = E[K::X_COS + i], sn = E[K::X_SIN + i], px = E[L.pos_x + i], py = E[L.pos_y + i];
          int nv = f2i(E[L.n_verts + i]);
          float wx[4], wy[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            float lx = E[L.verts + (2 * v) * P + i], ly = E[L.verts + (2 * v + 1) * P + i];
            wx[v] = px + fmaf(cs, lx, -(sn * ly));
            wy[v] = py + fmaf(sn, lx, cs * ly);
          }
          if (nv == 3) { wx[3] = wx[0]; wy[3] = wy[0]; }   // a triangle's spare slot repeats vertex 0: the
                                                           // manifold code can then run over four vertices
          *reinterpret_cast<float4*>(E + K::X_BOX + 4 * i) =
              make_float4(fminf(fminf(wx[0], wx[1]), fminf(wx[2], wx[3])) - kCullMargin,
                          fminf(fminf(wy[0], wy[1]), fminf(wy[2], wy[3])) - kCullMargin,
                          fmaxf(fmaxf(wx[0], wx[1]), fmaxf(wx[2], wx[3])) + kCullMargin,
                          fmaxf(fmaxf(wy[0], wy[1]), fmaxf(wy[2], wy[3])) + kCullMargin);
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            int v1 = (v + 1 == nv) ? 0 : ((v + 1) & 3);
            float ex = wx[v1] - wx[v], ey = wy[v1] - wy[v];
            float len = sqrtf(dot2(ex, ey, ex, ey));
            *reinterpret_cast<float2*>(E + K::X_WV + 2 * (v * P + i)) = make_float2(wx[v], wy[v]);
            *reinterpret_cast<float2*>(E + K::X_WN + 2 * (v * P + i)) = make_float2(ey / len, -ex / len);
          }
        } else {
          const float px = E[L.pos_x + i], py = E[L.pos_y + i], r = E[L.radius + (i - P)] + kCullMargin;
          *reinterpret_cast<float4*>(E + K::X_BOX + 4 * i) = make_float4(px - r, py - r, px + r, py + r);
        }
      }
      wave_sync();

      K2D_T(kT_Shapes);
      // ---- joint constants of this substep; motor and thruster impulses from the same velocities ----
      float j_rax = 0.f, j_ray = 0.f, j_rbx = 0.f, j_rby = 0.f, j_k11 = 0.f, j_k12 = 0.f, j_k22 = 0.f;
      float j_idet = 0.f, j_bx = 0.f, j_by = 0.f, j_angm = 0.f, j_angb = 0.f, j_exc = 0.f, motor = 0.f;
      float j_ima = 0.f, j_iia = 0.f, j_imb = 0.f, j_iib = 0.f;
      if (k < J && j_live) {
        if (!prm.warm_start) { j_accx = 0.f; j_accy = 0.f; j_acca = 0.f; }
        j_ima = E[L.inv_mass + ja]; j_iia = E[L.inv_inertia + ja];
        j_imb = E[L.inv_mass + jb]; j_iib = E[L.inv_inertia + jb];
        float ca = E[K::X_COS + ja], sa = E[K::X_SIN + ja], cb = E[K::X_COS + jb], sb = E[K::X_SIN + jb];
        j_rax = fmaf(ca, j_aax, -(sa * j_aay)); j_ray = fmaf(sa, j_aax, ca * j_aay);
        j_rbx = fmaf(cb, j_abx, -(sb * j_aby)); j_rby = fmaf(sb, j_abx, cb * j_aby);
        float ms = j_ima + j_imb;
        j_k11 = ms + j_iia * j_ray * j_ray + j_iib * j_rby * j_rby;
        j_k22 = ms + j_iia * j_rax * j_rax + j_iib * j_rbx * j_rbx;
        j_k12 = -j_iia * j_rax * j_ray - j_iib * j_rbx * j_rby;
        j_idet = 1.f / (j_k11 * j_k22 - j_k12 * j_k12);
        float sx = (E[L.pos_x + ja] + j_rax) - (E[L.pos_x + jb] + j_rbx);
        float sy = (E[L.pos_y + ja] + j_ray) - (E[L.pos_y + jb] + j_rby);
        j_bx = prm.joint_alpha * sx; j_by = prm.joint_alpha * sy;
        float is = j_iia + j_iib;
        j_angm = (is > 0.f) ? 1.f / is : 0.f;
        j_angb = prm.gamma * (E[L.theta + ja] - E[L.theta + jb] - j_thf);
        if (j_limited) {   // A.4.3: rotation beyond a limit, decided once per substep
          const float rel = E[L.theta + ja] - E[L.theta + jb];
          const float lo = E[L.limit_lo + k], hi = E[L.limit_hi + k];
          if (rel > hi) j_exc = rel - hi;
          else if (rel < lo) j_exc = rel - lo;
          j_angb = prm.gamma * j_exc;
        }
        if (!j_fixed && j_motor) {   // A.5
          float arg = (E[L.omega + ja] - E[L.omega + jb] - j_speed * act_m) * prm.rho;
          motor = j_power * k2d_tanh(arg) * h;
        }
      }
      float t_ix = 0.f, t_iy = 0.f, t_rx = 0.f, t_ry = 0.f;
      if (k < T && t_live) {   // A.6
        float cs = E[K::X_COS + t_body], sn = E[K::X_SIN + t_body];
        float dx = fmaf(cs, t_dx, -(sn * t_dy)), dy = fmaf(sn, t_dx, cs * t_dy);
        t_rx = fmaf(cs, t_px, -(sn * t_py)); t_ry = fmaf(sn, t_px, cs * t_py);
        float f = t_power * act_t * h;
        t_ix = f * dx; t_iy = f * dy;
      }
      K2D_T(kT_JointConstants);
      wave_sync();
      for (int lv = 0; lv < wave_levels; ++lv) {
        if (k < J && j_live && j_level == lv && motor != 0.f) {
          if (!ja_fix) E[L.omega + ja] = E[L.omega + ja] - j_iia * motor;
          if (!jb_fix) E[L.omega + jb] = E[L.omega + jb] + j_iib * motor;
        }
        wave_sync();
      }
      for (int t = 0; t < T; ++t) {
        if (k == t && t_live) {
          float im = E[L.inv_mass + t_body], ii = E[L.inv_inertia + t_body];
          E[L.vel_x + t_body] = fmaf(im, t_ix, E[L.vel_x + t_body]);
          E[L.vel_y + t_body] = fmaf(im, t_iy, E[L.vel_y + t_body]);
          E[L.omega + t_body] = fmaf(ii, cross2(t_rx, t_ry, t_ix, t_iy), E[L.omega + t_body]);
        }
        wave_sync();
      }

      K2D_T(kT_External);
      // ---- collision manifolds of all eligible pairs (A.3.1-A.3.4) and their substep constants ----
      // 1. the cheap test for all of this lane's pairs: bounding boxes (of the very world vertices and
      //    centres the manifolds use, grown by a margin a thousand times the rounding error of a
      //    coordinate) that do not overlap mean no manifold point can have positive penetration;
      // 2. the surviving pair ids of the environment are gathered into one list, one shape-type mix
      //    after the other, so that the group's lanes share them evenly and a wavefront runs one kind
      //    of manifold code per trip;
      // 3. the manifold of every active pair is staged in LDS for the lane that keeps the pair in
      //    registers for the rest of the substep (pairs beyond two per lane become records in LDS / HBM).
      unsigned cand = 0u;
      bool set_changed = false;   // a pair of this lane collides now and did not one substep ago, or the reverse
      {
#pragma unroll
        for (int j = 0; j < (R + H - 1) / H; ++j) {   // round j * H + rpar: every lane is busy in every trip
          const unsigned pk = (my_ab4[j >> 2] >> (8 * (j & 3))) & 0xffu;
          const int a = pk & 15, b = pk >> 4;
          const float4 ba = *reinterpret_cast<const float4*>(E + K::X_BOX + 4 * a);
          const float4 bb = *reinterpret_cast<const float4*>(E + K::X_BOX + 4 * b);
          if (ba.x <= bb.z && bb.x <= ba.z && ba.y <= bb.w && bb.y <= ba.w) cand |= 1u << (j * H + rpar);
        }
        cand &= elig;
      }
      {   // pairs that were colliding and are not even candidates now: their points are no longer active
        uint4 ps = *reinterpret_cast<const uint4*>(pstate + kp * 16);
        unsigned nz = 0u;
#pragma unroll
        for (int r = 0; r < R; ++r) {
          unsigned w = r < 4 ? ps.x : r < 8 ? ps.y : r < 12 ? ps.z : ps.w;
          if ((w >> (8 * (r & 3))) & 0xffu) nz |= 1u << r;
        }
        const unsigned gone = nz & ~cand & my_r;
        set_changed = gone != 0u;
        for (unsigned st = gone; st != 0u; st &= st - 1u) pstate[kp * 16 + (__ffs(st) - 1)] = 0;
      }
      if (k < 4) bitmap[k] = 0u;
      int kind_n[3], kind_off[3];
      const bool same_list = list_valid && !__any(cand != prev_cand);
      prev_cand = cand;
      list_valid = true;
      if (!same_list) {
        const unsigned m0 = cand & pp_mask, m1 = cand & pc_mask, m2 = cand & ~(pp_mask | pc_mask);
        const unsigned mine = (unsigned)__popc(m0) | ((unsigned)__popc(m1) << 8) | ((unsigned)__popc(m2) << 16);
        const unsigned incl = group_prefix_sum<G>(mine, k), excl = incl - mine;
        kind_tot = group_sum<G>(mine);
        int w0 = (int)(excl & 255), w1 = (int)(kind_tot & 255) + (int)((excl >> 8) & 255);
        int w2 = (int)(kind_tot & 255) + (int)((kind_tot >> 8) & 255) + (int)((excl >> 16) & 255);
        for (unsigned mm = m0; mm != 0u; mm &= mm - 1u) cand_list[w0++] = (unsigned char)((__ffs(mm) - 1) * GP + kp);
        for (unsigned mm = m1; mm != 0u; mm &= mm - 1u) cand_list[w1++] = (unsigned char)((__ffs(mm) - 1) * GP + kp);
        for (unsigned mm = m2; mm != 0u; mm &= mm - 1u) cand_list[w2++] = (unsigned char)((__ffs(mm) - 1) * GP + kp);
      }
      kind_n[0] = kind_tot & 255; kind_n[1] = (kind_tot >> 8) & 255; kind_n[2] = (kind_tot >> 16) & 255;
      kind_off[0] = 0; kind_off[1] = kind_n[0]; kind_off[2] = kind_n[0] + kind_n[1];
      wave_sync();
      K2D_T(kT_Cull);
      int pool_base = 0;
      for (int kind = 0; kind < 3; ++kind) {
       const int n_kind = kind_n[kind], off_kind = kind_off[kind];
       for (int base = 0; __any(base < n_kind); base += G) {
        Manifold m;
        int a = 0, b = 0, r = 0, kk = 0, id = 0;
        const bool have = base + k < n_kind;
        if (have) {
          id = cand_list[off_kind + base + k];
          r = id / GP;
          kk = id % GP;
          S::sched_pair(r, kk, a, b);
          if (kind == 0) {
            S::manifold_pp(E, a, f2i(E[L.n_verts + a]), b, f2i(E[L.n_verts + b]), prm.tie_eps, m);
          } else if (kind == 1) {
            S::manifold_pc(E, a, f2i(E[L.n_verts + a]), E[L.pos_x + b], E[L.pos_y + b], E[L.radius + (b - P)], m);
          } else {
            S::manifold_cc(E[L.pos_x + a], E[L.pos_y + a], E[L.radius + (a - P)], E[L.pos_x + b], E[L.pos_y + b],
                           E[L.radius + (b - P)], m);
          }
        }
        const bool act0 = m.valid[0] && m.pen[0] > 0.f, act1 = m.valid[1] && m.pen[1] > 0.f;
        const bool active = act0 || act1;
        const int prev_bits = have ? (int)pstate[kk * 16 + r] : 0;   // which points collided one substep ago
        set_changed |= have && ((prev_bits != 0) != active);
        unsigned long long bal = __ballot(active);
        unsigned envbits = (unsigned)(bal >> (g * G)) & (G >= 32 ? 0xffffffffu : ((1u << (G & 31)) - 1u));
        const int idx = pool_base + __popc(envbits & ((1u << k) - 1u));
        pool_base += __popc(envbits);
        if (active) {
          const int w = a | (b << 8) | ((int)act0 << 16) | ((int)act1 << 17) | (id << 18) | (prev_bits << 25);
          if (idx < K::NREG) {   // staged for the lane that keeps it
            LdsF p = to_lds(E + K::X_STAGE + idx * K::kManW);
            p[0] = m.nx; p[1] = m.ny;
            p[2] = m.px[0]; p[3] = m.py[0]; p[4] = m.pen[0];
            p[5] = m.px[1]; p[6] = m.py[1]; p[7] = m.pen[1];
            p[8] = i2f(w);
          } else {               // beyond the register-held pairs: a full record in the LDS pool or in HBM
            float4 lam = make_float4(0.f, 0.f, 0.f, 0.f);
            if (prm.warm_start && ((w >> 25) & 3))
              lam = *reinterpret_cast<const float4*>(Rg + L.lambda + 4 * S::pair_index(a, b));
            PairRec rc;
            float ima, iia, imb, iib;
            S::presolve(E, prm, m, w, lam, rc, ima, iia, imb, iib);
            if (idx < K::NREG + K::POOL) rec_store(to_lds(pool + (idx - K::NREG) * kRecW), rc);
            else rec_store(spill + (idx - K::NREG - K::POOL) * kRecW, rc);
            atomicOr(&bitmap[id >> 5], 1u << (id & 31));
            table[id] = (unsigned char)idx;
          }
        }
        if (have) pstate[kk * 16 + r] = (unsigned char)((unsigned)act0 | ((unsigned)act1 << 1));
       }
      }
      wave_sync();
      K2D_T(kT_Manifolds);
      // lane k keeps active pairs k and G + k of its environment in registers
      typename S::Own oa, ob;
      oa.id = -1; ob.id = -1; oa.lv = -1; ob.lv = -1;
      oa.rc.ab = 0; ob.rc.ab = 0;
      // The pairs change lanes only when the set of colliding pairs changes: then the impulses kept in
      // registers go to the HBM record first, from where the lanes that take the pairs over read them.
      if (__any(set_changed)) {
        flush_kept();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      }
      if (k < pool_base) S::take_own(E, Rg, prm, k, static_mask, kept_id, kept_lam, oa);
      if (__any(pool_base > G)) {
        if (k + G < pool_base && k + G < K::NREG) S::take_own(E, Rg, prm, k + G, static_mask, -1, kept_lam, ob);
      }
      wave_sync();
      K2D_T(kT_Presolve);
      // Levels of the active pairs.  The colliding pairs are walked in tournament order (round by round).
      // k2d_params.sweep_order = K2D_SWEEP_TOURNAMENT: the sweep visits them in that order, and a pair is
      // placed one level after the last earlier colliding pair that shares a movable shape with it --
      // pairs that share one keep their order, so sweeping the levels in turn, each level at once, gives
      // the same bits as the one-after-the-other sweep in tournament order.
      // K2D_SWEEP_LEVELS: a pair takes the lowest level that no earlier colliding pair sharing a movable
      // shape with it has taken, and the sweep's order *is* level 0, then level 1, ...: as few trips as
      // the busiest shape has contacts (or one more).
      // Either way the pairs of a level touch disjoint movable shapes, everything resting on the static
      // floor is one level, and a level never exceeds the round.  The lane that tests a pair also places
      // it: the pairs of a round touch disjoint shapes, so the lanes of a round read and extend the sets
      // of levels taken at their two shapes (16-bit words in LDS) without getting in each other's way,
      // and the rounds follow one another.
      if (!levels_valid || __any(set_changed)) {
        if (k < (N + 1) / 2) reinterpret_cast<unsigned*>(taken)[k] = 0u;
        wave_sync();
        const uint4 ps = *reinterpret_cast<const uint4*>(pstate + kp * 16);
        int my_levels = 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const unsigned w = r < 4 ? ps.x : r < 8 ? ps.y : r < 12 ? ps.z : ps.w;
          const bool act = ((my_r >> r) & 1u) && ((w >> (8 * (r & 3))) & 0xffu) != 0u;
          if (__any(act)) {
            if (act) {
              const unsigned pk = (my_ab4[(r / H) >> 2] >> (8 * ((r / H) & 3))) & 0xffu;
              const int a = pk & 15, b = pk >> 4;
              const bool ma = !((static_mask >> a) & 1u), mb = !((static_mask >> b) & 1u);
              const unsigned ta = ma ? (unsigned)taken[a] : 0u, tb = mb ? (unsigned)taken[b] : 0u;
              const int lv = prm.lowest_free_level ? __ffs((int)~(ta | tb)) - 1 : 32 - __clz((int)(ta | tb));
              if (ma) taken[a] = (unsigned short)(ta | (1u << lv));
              if (mb) taken[b] = (unsigned short)(tb | (1u << lv));
              lvl[r * GP + kp] = (unsigned char)lv;
              my_levels = max(my_levels, lv + 1);
            }
            wave_sync();
          }
        }
        wave_clevels = 0;
        for (int lv = 1; lv <= R; ++lv)
          if (__any(my_levels >= lv)) wave_clevels = lv;
        levels_valid = true;
      }
      wave_sync();
      if (oa.id >= 0) oa.lv = lvl[oa.id];
      if (ob.id >= 0) ob.lv = lvl[ob.id];
      // the pairs that are not held in registers are listed level by level (lane s mod G writes entry s)
      unsigned long long level_cnt = 0ull;   // listed pairs per level, 4 bits each (a level holds fewer than 16)
      const uint4 bl = *reinterpret_cast<const uint4*>(bitmap);
      const bool any_listed = __any((bl.x | bl.y | bl.z | bl.w) != 0u);
      if (any_listed) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          for (unsigned bits = w == 0 ? bl.x : w == 1 ? bl.y : w == 2 ? bl.z : bl.w; bits != 0u; bits &= bits - 1u) {
            const int id = 32 * w + __ffs(bits) - 1;
            const int lv = lvl[id];
            const int slot = (int)((level_cnt >> (4 * lv)) & 15ull);
            level_cnt += 1ull << (4 * lv);
            if ((slot & (G - 1)) == k) sched[lv * K::LCAP + slot] = table[id];
          }
        }
        wave_sync();
      }
      auto cnt_of = [&](int lv) { return (int)((level_cnt >> (4 * lv)) & 15ull); };
      // one level at a time: the pairs held in registers (first and second of the lane), then the listed ones
      const bool any_b = __any(ob.id >= 0);
      auto for_each_level = [&](auto&& f_own, auto&& f_listed) {
        if (!any_b && !any_listed) {   // the common case, as a loop of its own: one pair per lane, all in registers
          for (int lv = 0; lv < wave_clevels; ++lv) {
            if (oa.lv == lv) f_own(oa);
            wave_sync();
          }
          return;
        }
        for (int lv = 0; lv < wave_clevels; ++lv) {
          if (oa.lv == lv) f_own(oa);
          if (any_b) {
            if (ob.lv == lv) f_own(ob);
          }
          if (any_listed) {
            const int c = cnt_of(lv);
            for (int base = 0; __any(base < c); base += G)
              if (base + k < c) f_listed((int)sched[lv * K::LCAP + base + k] - K::NREG);
          }
          wave_sync();
        }
      };

      K2D_T(kT_Levels);
#ifdef K2D_PHASE_TIMERS
      t_pair_levels += wave_clevels; t_joint_levels += wave_levels;
#endif
      // ---- warm starting (Alg. 1, A.7): collisions level after level, then joints ----
      if (prm.warm_start) {
        for_each_level([&](typename S::Own& o) { S::template visit_own<true>(E, o); },
                       [&](int q) {
                         PairRec rc;
                         if (q < K::POOL) rec_load(to_lds(pool + q * kRecW), rc);
                         else rec_load(spill + (q - K::POOL) * kRecW, rc);
                         S::template visit_pair<true>(E, rc, static_mask);
                       });
        for (int lv = 0; lv < wave_levels; ++lv) {
          if (k < J && j_live && j_level == lv) {
            float wa = E[L.omega + ja], wb = E[L.omega + jb];
            if (j_fixed) {
              wa = wa + j_iia * j_acca;
              wb = wb - j_iib * j_acca;
            }
            E[L.vel_x + jsa] = fmaf(j_ima, j_accx, E[L.vel_x + ja]);
            E[L.vel_y + jsa] = fmaf(j_ima, j_accy, E[L.vel_y + ja]);
            E[L.omega + jsa] = fmaf(j_iia, cross2(j_rax, j_ray, j_accx, j_accy), wa);
            E[L.vel_x + jsb] = fmaf(j_imb, -j_accx, E[L.vel_x + jb]);
            E[L.vel_y + jsb] = fmaf(j_imb, -j_accy, E[L.vel_y + jb]);
            E[L.omega + jsb] = fmaf(j_iib, cross2(j_rbx, j_rby, -j_accx, -j_accy), wb);
          }
          wave_sync();
        }
      }

      K2D_T(kT_WarmStart);
      // ---- solver sweeps (Alg. 1): joints, then collisions ----
      const int n_b = BATCHED ? prm.n_batches : 1;
      int oa_bj = 0, ob_bj = 0;   // batched schedule: batch and place of the two points of the held pairs
      if constexpr (BATCHED) {
        if (oa.id >= 0) oa_bj = S::batch_places(oa.id, n_b);
        if (ob.id >= 0) ob_bj = S::batch_places(ob.id, n_b);
      }
      for (int it = 0; it < prm.n_iters; ++it) {
        for (int lv = 0; lv < wave_levels; ++lv) {
          if (k < J && j_live && j_level == lv) {
            float vax = E[L.vel_x + ja], vay = E[L.vel_y + ja], wa = E[L.omega + ja];
            float vbx = E[L.vel_x + jb], vby = E[L.vel_y + jb], wb = E[L.omega + jb];
            if (j_fixed && j_angm > 0.f) {   // A.4.2
              float d = -(wa - wb + j_angb) * j_angm;
              wa = wa + j_iia * d;
              wb = wb - j_iib * d;
              j_acca = j_acca + d;
            }
            if (!j_fixed && j_exc != 0.f && j_angm > 0.f) {   // A.4.3: not while already coming back, never accumulated
              const float w = wa - wb;
              const bool restoring = (j_exc > 0.f) ? (w < 0.f) : (w > 0.f);
              if (!restoring) {
                float d = -(w + j_angb) * j_angm;
                wa = wa + j_iia * d;
                wb = wb - j_iib * d;
              }
            }
            float cx, cy;   // A.4.1: point constraint, 2x2 solve
            S::rel_vel(vax, vay, wa, j_rax, j_ray, vbx, vby, wb, j_rbx, j_rby, cx, cy);
            float rx = -(cx + j_bx), ry = -(cy + j_by);
            float jx = (j_k22 * rx - j_k12 * ry) * j_idet, jy = (j_k11 * ry - j_k12 * rx) * j_idet;
            apply_impulse(vax, vay, wa, j_ima, j_iia, jx, jy, j_rax, j_ray);
            apply_impulse(vbx, vby, wb, j_imb, j_iib, -jx, -jy, j_rbx, j_rby);
            j_accx = j_accx + jx; j_accy = j_accy + jy;
            E[L.vel_x + jsa] = vax; E[L.vel_y + jsa] = vay; E[L.omega + jsa] = wa;
            E[L.vel_x + jsb] = vbx; E[L.vel_y + jsb] = vby; E[L.omega + jsb] = wb;
          }
          wave_sync();
        }
        K2D_T(kT_SweepJoints);
        if constexpr (BATCHED) {
          // A.8: the points of batch b are solved from the velocities the batch starts with, their impulses
          // staged by their place in the batch; then lane s applies to shape s, in place order, the
          // impulses of the points that touch it (so every body sees them in point order).
          for (int b = 0; b < n_b; ++b) {
            unsigned pm = 0u;   // places of the batch taken by this lane's points
            auto stage_point = [&](int j, int ab, float jx, float jy, float fx, float fy, float rax, float ray,
                                   float rbx, float rby) {
              LdsF p = to_lds(E + K::X_STAGE + j * K::kManW);
              p[0] = jx; p[1] = jy; p[2] = fx; p[3] = fy;
              p[4] = rax; p[5] = ray; p[6] = rbx; p[7] = rby;
              p[8] = i2f(ab & 0xffff);
              pm |= 1u << j;
            };
            auto own_points = [&](typename S::Own& o, int bj) {
              if (o.id < 0) return;
              const bool hit0 = ((o.rc.ab >> 16) & 1) && (bj & 0xff) == b;
              const bool hit1 = ((o.rc.ab >> 17) & 1) && ((bj >> 16) & 0xff) == b;
              if (hit0 || hit1) {
                const float vax = E[L.vel_x + o.pa], vay = E[L.vel_y + o.pa], wa = E[L.omega + o.pa];
                const float vbx = E[L.vel_x + o.pb], vby = E[L.vel_y + o.pb], wb = E[L.omega + o.pb];
                float jx, jy, fx, fy, rax, ray, rbx, rby;
                S::point_impulses(o.rc, hit1, o.ima, o.iia, o.imb, o.iib, vax, vay, wa, vbx, vby, wb, jx, jy, fx, fy,
                                  rax, ray, rbx, rby);
                stage_point((bj >> (hit1 ? 24 : 8)) & 0xff, o.rc.ab, jx, jy, fx, fy, rax, ray, rbx, rby);
              }
            };
            own_points(oa, oa_bj);
            if (any_b) own_points(ob, ob_bj);
            if (any_listed) {
              auto listed_points = [&](auto rp) {
                PairRec rc;
                rec_load(rp, rc);
                const int bj = S::batch_places((rc.ab >> 18) & 127, n_b);
                const bool hit0 = ((rc.ab >> 16) & 1) && (bj & 0xff) == b;
                const bool hit1 = ((rc.ab >> 17) & 1) && ((bj >> 16) & 0xff) == b;
                if (hit0 || hit1) {
                  const int a = rc.ab & 0xff, bb = (rc.ab >> 8) & 0xff;
                  const float vax = E[L.vel_x + a], vay = E[L.vel_y + a], wa = E[L.omega + a];
                  const float vbx = E[L.vel_x + bb], vby = E[L.vel_y + bb], wb = E[L.omega + bb];
                  const float ima = E[L.inv_mass + a], iia = E[L.inv_inertia + a];
                  const float imb = E[L.inv_mass + bb], iib = E[L.inv_inertia + bb];
                  float jx, jy, fx, fy, rax, ray, rbx, rby;
                  S::point_impulses(rc, hit1, ima, iia, imb, iib, vax, vay, wa, vbx, vby, wb, jx, jy, fx, fy, rax, ray,
                                    rbx, rby);
                  stage_point((bj >> (hit1 ? 24 : 8)) & 0xff, rc.ab, jx, jy, fx, fy, rax, ray, rbx, rby);
                  if (hit1) { rp[15 + 8] = rc.lam_n[1]; rp[15 + 9] = rc.lam_t[1]; }
                  else { rp[5 + 8] = rc.lam_n[0]; rp[5 + 9] = rc.lam_t[0]; }
                }
              };
              for (int lv = 0; lv < wave_clevels; ++lv) {
                const int c = cnt_of(lv);
                for (int base = 0; __any(base < c); base += G) {
                  if (base + k < c) {
                    const int q = (int)sched[lv * K::LCAP + base + k] - K::NREG;
                    if (q < K::POOL) listed_points(to_lds(pool + q * kRecW));
                    else listed_points(spill + (q - K::POOL) * kRecW);
                  }
                }
              }
            }
            pm = group_or<G>(pm);
            wave_sync();
            if (__any(pm != 0u)) {
              for (int i = k; i < N; i += G) {   // lane k applies to shapes k, k + G, ...
                if (!((static_mask >> i) & 1u) && pm != 0u) {
                  float vx = E[L.vel_x + i], vy = E[L.vel_y + i], w = E[L.omega + i];
                  const float im = E[L.inv_mass + i], ii = E[L.inv_inertia + i];
                  for (unsigned m = pm; m != 0u; m &= m - 1u) {
                    LdsCF p = (LdsCF)(E + K::X_STAGE + (__ffs(m) - 1) * K::kManW);
                    const int ab = f2i(p[8]);
                    if ((ab & 0xff) == i) {
                      apply_impulse(vx, vy, w, im, ii, p[0], p[1], p[4], p[5]);
                      apply_impulse(vx, vy, w, im, ii, p[2], p[3], p[4], p[5]);
                    } else if ((ab >> 8) == i) {
                      apply_impulse(vx, vy, w, im, ii, -p[0], -p[1], p[6], p[7]);
                      apply_impulse(vx, vy, w, im, ii, -p[2], -p[3], p[6], p[7]);
                    }
                  }
                  E[L.vel_x + i] = vx; E[L.vel_y + i] = vy; E[L.omega + i] = w;
                }
              }
              wave_sync();
            }
          }
        } else
        for_each_level([&](typename S::Own& o) { S::template visit_own<false>(E, o); },
                       [&](int q) {
                         // (the two branches keep LDS and HBM accesses apart: a merged pointer would turn
                         // every access into a slow flat one)
                         PairRec rc;
                         if (q < K::POOL) {
                           LdsF rp = to_lds(pool + q * kRecW);
                           rec_load(rp, rc);
                           S::template visit_pair<false>(E, rc, static_mask);
#pragma unroll
                           for (int z = 0; z < 2; ++z) { rp[5 + 10 * z + 8] = rc.lam_n[z]; rp[5 + 10 * z + 9] = rc.lam_t[z]; }
                         } else {
                           float* rp = spill + (q - K::POOL) * kRecW;
                           rec_load(rp, rc);
                           S::template visit_pair<false>(E, rc, static_mask);
#pragma unroll
                           for (int z = 0; z < 2; ++z) { rp[5 + 10 * z + 8] = rc.lam_n[z]; rp[5 + 10 * z + 9] = rc.lam_t[z]; }
                         }
                       });
        K2D_T(kT_SweepPairs);
      }

      // ---- Euler step of position and rotation (Alg. 1) ----
      for (int i = k; i < N; i += G) {
        if (f2i(E[L.shape_flags + i]) & 1) {
          E[L.pos_x + i] = E[L.pos_x + i] + h * E[L.vel_x + i];
          E[L.pos_y + i] = E[L.pos_y + i] + h * E[L.vel_y + i];
          float th = E[L.theta + i] + h * E[L.omega + i];
          E[L.theta + i] = th;
          float sn, cs;
          k2d_sincos(th, sn, cs);
          E[K::X_COS + i] = cs;
          E[K::X_SIN + i] = sn;
        }
      }
      wave_sync();

      K2D_T(kT_Euler);
      // ---- positional corrections (A.3.7, A.4.1); the pair's accumulated impulses go to HBM ----
      auto correct = [&](float nx, float ny, float corr, int ab, float4 lam, bool to_hbm) {
        const int a = ab & 0xff, b = (ab >> 8) & 0xff;
        // the pair's accumulated impulses wait for the next substep (A.7): the first pair of a lane in the
        // lane's registers (see kept_lam), every other pair in the HBM record
        if (to_hbm && env_ok) *reinterpret_cast<float4*>(Rg + L.lambda + 4 * S::pair_index(a, b)) = lam;
        const float ima = E[L.inv_mass + a], imb = E[L.inv_mass + b];
        // (the positions of shapes no impulse moves go to the dump slot: L.pos_x is word 0 of the image)
        const int da = ((static_mask >> a) & 1u) ? K::X_DUMP : a, db = ((static_mask >> b) & 1u) ? K::X_DUMP : b;
        E[L.pos_x + da] = E[L.pos_x + a] - (ima * corr) * nx;
        E[L.pos_y + da] = E[L.pos_y + a] - (ima * corr) * ny;
        E[L.pos_x + db] = E[L.pos_x + b] + (imb * corr) * nx;
        E[L.pos_y + db] = E[L.pos_y + b] + (imb * corr) * ny;
      };
      for_each_level([&](typename S::Own& o) {
                       correct(o.rc.nx, o.rc.ny, o.rc.corr, o.rc.ab,
                               make_float4(o.rc.lam_n[0], o.rc.lam_t[0], o.rc.lam_n[1], o.rc.lam_t[1]), &o == &ob);
                     },
                     [&](int q) {
                       if (q < K::POOL) {
                         LdsCF rp = to_lds(pool + q * kRecW);
                         correct(rp[0], rp[1], rp[3], f2i(rp[4]), make_float4(rp[13], rp[14], rp[23], rp[24]), true);
                       } else {
                         const float* rp = spill + (q - K::POOL) * kRecW;
                         correct(rp[0], rp[1], rp[3], f2i(rp[4]), make_float4(rp[13], rp[14], rp[23], rp[24]), true);
                       }
                     });
      kept_id = oa.id;
      kept_lam = make_float4(oa.rc.lam_n[0], oa.rc.lam_t[0], oa.rc.lam_n[1], oa.rc.lam_t[1]);
      K2D_T(kT_CorrectPairs);
      for (int lv = 0; lv < wave_levels; ++lv) {
        if (k < J && j_live && j_level == lv) {
          float ca = E[K::X_COS + ja], sa = E[K::X_SIN + ja], cb = E[K::X_COS + jb], sb = E[K::X_SIN + jb];
          float xax = E[L.pos_x + ja] + fmaf(ca, j_aax, -(sa * j_aay)), xay = E[L.pos_y + ja] + fmaf(sa, j_aax, ca * j_aay);
          float xbx = E[L.pos_x + jb] + fmaf(cb, j_abx, -(sb * j_aby)), xby = E[L.pos_y + jb] + fmaf(sb, j_abx, cb * j_aby);
          float cf = prm.joint_beta / (j_ima + j_imb);
          float cx = cf * (xax - xbx), cy = cf * (xay - xby);
          const int da = ja_fix ? K::X_DUMP : ja, db = jb_fix ? K::X_DUMP : jb;
          E[L.pos_x + da] = E[L.pos_x + ja] - j_ima * cx;
          E[L.pos_y + da] = E[L.pos_y + ja] - j_ima * cy;
          E[L.pos_x + db] = E[L.pos_x + jb] + j_imb * cx;
          E[L.pos_y + db] = E[L.pos_y + jb] + j_imb * cy;
        }
        wave_sync();
      }
      K2D_T(kT_CorrectJoints);
    }
    if (RESET) {   // new episodes (wave-uniform branch: the wavefront leaves the step loop together)
      int rl = env_ok ? reset_level[(size_t)step * n_envs + env] : -1;
      if (rl >= n_level_records) rl = -1;
      if (__any(rl >= 0)) {
        if (rl >= 0) {
          const float* src = levels + (size_t)rl * L.scene_words;
          for (int w = k; w < L.scene_words; w += G) {
            float v = src[w];
            if (w >= L.acc_x && w < L.thr_flags) v = 0.f;   // accumulated joint impulses start at zero
            E[w] = v;
            Rg[w] = v;
          }
          j_accx = 0.f; j_accy = 0.f; j_acca = 0.f;
          if (k < GP)   // no collision is carried into the new episode
            for (int r = 0; r < 16; ++r) pstate[k * 16 + r] = 0;
        }
        ++step;
        break;
      }
    }
  }
  flush_kept();
  // the joint accumulators return to the LDS image (from where a new pass, or the write-back, takes them)
  if (k < J) {
    E[L.acc_x + k] = j_accx;
    E[L.acc_y + k] = j_accy;
    E[L.acc_ang + k] = j_acca;
  }
  wave_sync();
  first = false;
  } while (RESET && step < n_steps);

#ifdef K2D_PHASE_TIMERS
  K2D_T(kT_Restart);
  if (phase_clocks && lane == 0) {
    unsigned long long* out = phase_clocks + (size_t)blockIdx.x * kPhaseSlots;
    for (int i = 0; i < kT_Count; ++i) out[i] = (unsigned long long)t_acc[i];
    out[kT_Count] = t_pair_levels;
    out[kT_Count + 1] = t_joint_levels;
  }
#endif
  // ---- write back: dynamic shape state, joint accumulators, pair states ----
  for (int e = 0; e < K::EPW; ++e) {
    const int env_e = env_of(slot0 + e);
    if (env_e >= 0) {
      const float* src = lds + e * K::LDS_STRIDE;
      float* dst = state + (size_t)env_e * K::REC_WORDS;
      for (int w = lane; w < 6 * N; w += 64) dst[w] = src[w];
      for (int w = lane; w < 3 * J; w += 64) dst[L.acc_x + w] = src[L.acc_x + w];
    }
  }
  if (env_ok) {
    unsigned char* ps = reinterpret_cast<unsigned char*>(Rg + L.pair_state);
    const unsigned char* pstate = reinterpret_cast<const unsigned char*>(E + K::X_PSTATE);
    for (int r = 0; r < R; ++r) {
      int a, b;
      if (((my_r >> r) & 1u) && S::sched_pair(r, kp, a, b)) ps[S::pair_index(a, b)] = pstate[kp * 16 + r];
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Small data-movement kernels
// ---------------------------------------------------------------------------------------------------
// Scene records -> state records (k2d_reset); zeroes the accumulators and the pair states.
__global__ void k2d_reset_kernel(float* state, const float* scenes, const int32_t* ids, int n, int n_envs,
                                 int rec_words, k2d_layout L) {
  int r = blockIdx.x;
  if (r >= n) return;
  int env = ids ? ids[r] : r;
  if (env < 0 || env >= n_envs) return;
  float* dst = state + (size_t)env * rec_words;
  const float* src = scenes + (size_t)r * L.scene_words;
  for (int w = threadIdx.x; w < L.state_words; w += blockDim.x) {
    float v = 0.f;
    if (w < L.scene_words) {
      v = src[w];
      if (w >= L.acc_x && w < L.thr_flags) v = 0.f;   // acc_x, acc_y, acc_ang are contiguous
    }
    dst[w] = v;
  }
}

// Full records out of (dir = 0) or into (dir = 1) the batch.
__global__ void k2d_copy_state_kernel(float* state, float* records, int n_envs, int rec_words, k2d_layout L,
                                      int dir) {
  const int state_words = L.state_words;
  int env = blockIdx.x;
  if (env >= n_envs) return;
  float* a = state + (size_t)env * rec_words;
  float* b = records + (size_t)env * state_words;
  const unsigned char* ps = reinterpret_cast<const unsigned char*>(a + L.pair_state);
  for (int w = threadIdx.x; w < state_words; w += blockDim.x) {
    if (dir == 0) {
      float v = a[w];
      // accumulated impulses of manifold points that are not in collision are zero by definition (A.7)
      if (w >= L.lambda && w < L.lambda + 4 * L.n_pairs) {
        int q = w - L.lambda;
        if (!((ps[q >> 2] >> ((q >> 1) & 1)) & 1)) v = 0.f;
      }
      b[w] = v;
    } else {
      a[w] = b[w];
    }
  }
}

// Flat symbolic observation (Tables 5-7): one thread per entity.
__global__ void k2d_obs_kernel(const float* state, float* obs, int n_envs, int rec_words, k2d_layout L, int P, int C,
                               int J, int T) {
  const int n_ent = P + C + J + T;
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)n_envs * n_ent) return;
  int env = (int)(gid / n_ent), ent = (int)(gid % n_ent);
  const float* S = state + (size_t)env * rec_words;
  float* o = obs + (size_t)env * L.obs_dim;
  if (ent < P + C) {
    int i = ent;
    o += (i < P) ? i * 23 : P * 23 + (i - P) * 15;
    int fl = __float_as_int(S[L.shape_flags + i]);
    float sn, cs;
    k2d_sincos(S[L.theta + i], sn, cs);
    o[0] = S[L.pos_x + i]; o[1] = S[L.pos_y + i]; o[2] = S[L.vel_x + i]; o[3] = S[L.vel_y + i];
    o[4] = S[L.inv_mass + i]; o[5] = S[L.inv_inertia + i]; o[6] = S[L.density + i];
    o[7] = k2d_tanh(S[L.omega + i] / 10.f);
    o[8] = sn; o[9] = cs; o[10] = S[L.friction + i]; o[11] = S[L.restitution + i];
    int q = 12;
    if (i < P) {
      for (int v = 0; v < 8; ++v) o[q++] = S[L.verts + v * P + i];
      o[q++] = (float)__float_as_int(S[L.n_verts + i]);
    } else {
      o[q++] = S[L.radius + (i - P)];
    }
    o[q++] = (float)(fl & 1);
    o[q++] = (float)(fl >> 8);
  } else if (ent < P + C + J) {
    int j = ent - P - C;
    o += P * 23 + C * 15 + j * 11;
    int fl = __float_as_int(S[L.joint_flags + j]);
    int a = __float_as_int(S[L.joint_a + j]), b = __float_as_int(S[L.joint_b + j]);
    a = min(max(a, 0), P + C - 1); b = min(max(b, 0), P + C - 1);
    float sn, cs;
    k2d_sincos(S[L.theta + a] - S[L.theta + b], sn, cs);
    o[0] = (float)(fl & 1); o[1] = (float)((fl >> 1) & 1);
    o[2] = S[L.anchor_a_x + j]; o[3] = S[L.anchor_a_y + j]; o[4] = S[L.anchor_b_x + j]; o[5] = S[L.anchor_b_y + j];
    o[6] = S[L.motor_power + j]; o[7] = S[L.motor_speed + j]; o[8] = (float)((fl >> 2) & 1);
    o[9] = sn; o[10] = cs;
  } else {
    int t = ent - P - C - J;
    o += P * 23 + C * 15 + J * 11 + t * 6;
    int fl = __float_as_int(S[L.thr_flags + t]);
    float sn, cs;
    k2d_sincos(S[L.thr_angle + t], sn, cs);
    o[0] = (float)(fl & 1); o[1] = S[L.thr_pos_x + t]; o[2] = S[L.thr_pos_y + t]; o[3] = S[L.thr_power + t];
    o[4] = sn; o[5] = cs;
  }
}

// Symbolic-Entity observation (Sec. 3.2, Sec. 4, Tables 5-7): one thread per entity.  Entities of an
// environment: N shapes, then two per joint (the joint seen from either of its shapes), then T thrusters.
__global__ void k2d_entities_kernel(const float* state, float* shapes, float* joints, int32_t* joint_idx,
                                    float* thrusters, int32_t* thruster_idx, int n_envs, int rec_words, k2d_layout L,
                                    int P, int C, int J, int T) {
  const int N = P + C, n_ent = N + 2 * J + T;
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)n_envs * n_ent) return;
  const int env = (int)(gid / n_ent), ent = (int)(gid % n_ent);
  const float* S = state + (size_t)env * rec_words;
  if (ent < N) {
    const int i = ent;
    float* o = shapes + ((size_t)env * N + i) * 30;
    const int fl = __float_as_int(S[L.shape_flags + i]);
    float sn, cs;
    k2d_sincos(S[L.theta + i], sn, cs);
    o[0] = S[L.pos_x + i]; o[1] = S[L.pos_y + i]; o[2] = S[L.vel_x + i]; o[3] = S[L.vel_y + i];
    o[4] = S[L.inv_mass + i]; o[5] = S[L.inv_inertia + i]; o[6] = S[L.density + i];
    o[7] = k2d_tanh(S[L.omega + i] / 10.f);
    const int role = fl >> 8;
    for (int r = 0; r < 4; ++r) o[8 + r] = (role == r) ? 1.f : 0.f;
    o[12] = sn; o[13] = cs; o[14] = S[L.friction + i]; o[15] = S[L.restitution + i];
    o[16] = (i >= P) ? 1.f : 0.f; o[17] = (i < P) ? 1.f : 0.f;
    o[18] = (i >= P) ? S[L.radius + (i - P)] : 0.f;
    const int nv = (i < P) ? __float_as_int(S[L.n_verts + i]) : 0;
    for (int v = 0; v < 8; ++v) o[19 + v] = (i < P) ? S[L.verts + v * P + i] : 0.f;
    o[27] = (i < P && nv == 3) ? 1.f : 0.f;
    o[28] = (i < P && nv != 3) ? 1.f : 0.f;
    o[29] = (float)(fl & 1);
  } else if (ent < N + 2 * J) {
    const int q = (ent - N) >> 1, swapped = (ent - N) & 1;
    float* o = joints + ((size_t)env * 2 * J + (ent - N)) * 11;
    const int fl = __float_as_int(S[L.joint_flags + q]);
    int a = __float_as_int(S[L.joint_a + q]), b = __float_as_int(S[L.joint_b + q]);
    a = min(max(a, 0), N - 1); b = min(max(b, 0), N - 1);
    float sn, cs;
    k2d_sincos(S[L.theta + a] - S[L.theta + b], sn, cs);
    const float aax = S[L.anchor_a_x + q], aay = S[L.anchor_a_y + q], abx = S[L.anchor_b_x + q], aby = S[L.anchor_b_y + q];
    o[0] = (float)(fl & 1); o[1] = (float)((fl >> 1) & 1);
    o[2] = swapped ? abx : aax; o[3] = swapped ? aby : aay;
    o[4] = swapped ? aax : abx; o[5] = swapped ? aay : aby;
    o[6] = S[L.motor_power + q]; o[7] = S[L.motor_speed + q]; o[8] = (float)((fl >> 2) & 1);
    o[9] = swapped ? -sn : sn; o[10] = cs;
    int32_t* ix = joint_idx + ((size_t)env * 2 * J + (ent - N)) * 2;
    ix[0] = swapped ? b : a; ix[1] = swapped ? a : b;
  } else {
    const int t = ent - N - 2 * J;
    float* o = thrusters + ((size_t)env * T + t) * 6;
    const int fl = __float_as_int(S[L.thr_flags + t]);
    float sn, cs;
    k2d_sincos(S[L.thr_angle + t], sn, cs);
    o[0] = (float)(fl & 1); o[1] = S[L.thr_pos_x + t]; o[2] = S[L.thr_pos_y + t]; o[3] = S[L.thr_power + t];
    o[4] = sn; o[5] = cs;
    thruster_idx[(size_t)env * T + t] = min(max(__float_as_int(S[L.thr_body + t]), 0), N - 1);
  }
}

// The four attention masks of the entity model (Sec. 4): bit j of word i set iff shape i may attend to
// shape j.  16 lanes per environment, lane i holds the words of shape i.
__global__ void __launch_bounds__(64) k2d_masks_kernel(const float* state, uint32_t* masks, int n_envs, int rec_words,
                                                       k2d_layout L, int J) {
  const int lane = threadIdx.x, i = lane & 15;
  const int env = blockIdx.x * 4 + (lane >> 4);
  const bool ok = env < n_envs;
  const float* S = state + (size_t)(ok ? env : 0) * rec_words;
  const unsigned char* ps = reinterpret_cast<const unsigned char*>(S + L.pair_state);
  const int N = L.n_shapes;
  const bool act = ok && i < N && (__float_as_int(S[L.shape_flags + i]) & 1);
  unsigned full = 0u;
  for (int j = 0; j < N; ++j) full |= (unsigned)__shfl((int)act, j, 16) << j;
  unsigned direct = act ? (1u << i) : 0u;
  for (int q = 0; q < J; ++q) {
    const int fl = __float_as_int(S[L.joint_flags + q]);
    int a = __float_as_int(S[L.joint_a + q]), b = __float_as_int(S[L.joint_b + q]);
    a = min(max(a, 0), N - 1); b = min(max(b, 0), N - 1);
    if ((fl & 1) && a != b && ((full >> a) & 1u) && ((full >> b) & 1u)) {
      if (i == a) direct |= 1u << b;
      if (i == b) direct |= 1u << a;
    }
  }
  unsigned reach = direct;
  for (int k = 0; k < N; ++k) {   // transitive closure
    const unsigned rk = (unsigned)__shfl((int)reach, k, 16);
    if ((reach >> k) & 1u) reach |= rk;
  }
  unsigned touch = 0u;
  if (ok && i < N)
    for (int j = 0; j < N; ++j) {
      if (j == i) continue;
      const int a = min(i, j), b = max(i, j);
      if (ps[a * (2 * N - a - 1) / 2 + (b - a - 1)] & 3) touch |= 1u << j;
    }
  if (ok && i < N) {
    uint32_t* m = masks + (size_t)env * 4 * N;
    m[i] = act ? full : 0u;
    m[N + i] = direct;
    m[2 * N + i] = reach;
    m[3 * N + i] = touch;
  }
}

// Multi-discrete actions (Sec. 3.2): a motor is off (0), forwards (1) or backwards (2) at full power, a
// thruster off (0) or on (1).
__global__ void k2d_decode_actions_kernel(const int32_t* discrete, float* actions, size_t n, int J, int A) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n) return;
  const int c = (int)(idx % A), d = discrete[idx];
  actions[idx] = (c < J) ? (d == 1 ? 1.f : d == 2 ? -1.f : 0.f) : (d == 1 ? 1.f : 0.f);
}

// Active manifold points per pair and the shape adjacency words, from the pair-state bytes.
__global__ void k2d_contacts_kernel(const float* state, uint8_t* pair_count, uint32_t* shape_adj, int n_envs,
                                    int rec_words, k2d_layout L) {
  int env = blockIdx.x;
  if (env >= n_envs) return;
  const unsigned char* ps = reinterpret_cast<const unsigned char*>(state + (size_t)env * rec_words + L.pair_state);
  const int N = L.n_shapes;
  if (pair_count)
    for (int p = threadIdx.x; p < L.n_pairs; p += blockDim.x)
      pair_count[(size_t)env * L.n_pairs + p] = (uint8_t)((ps[p] & 1) + ((ps[p] >> 1) & 1));
  if (shape_adj)
    for (int i = threadIdx.x; i < N; i += blockDim.x) {
      uint32_t w = 0;
      for (int j = 0; j < N; ++j) {
        if (j == i) continue;
        int a = min(i, j), b = max(i, j);
        if (ps[a * (2 * N - a - 1) / 2 + (b - a - 1)] & 3) w |= 1u << j;
      }
      shape_adj[(size_t)env * N + i] = w;
    }
}

// Ordering of the environments for one launch of the step kernel (slot -> environment).  Environments are
// sorted by how much work they are expected to be (active pairs of the last substep, then movable shapes, then
// the depth of the joints' dependency levels), busiest first, so that a wavefront steps similar ones instead
// of paying for the most pairs, the most shapes and the deepest joint chain of a random few.  The result of
// the step does not depend on the ordering.
// Two kernels: the keys (one lane per environment), then a counting sort over the key values in one workgroup.
constexpr int kOrderKeys = 1024;
__global__ void k2d_order_keys_kernel(const float* state, int32_t* keys, int n_envs, int rec_words, k2d_layout L,
                                      int n_joints) {
  const int env = blockIdx.x * blockDim.x + threadIdx.x;
  if (env >= n_envs) return;
  const float* S = state + (size_t)env * rec_words;
  const unsigned* ps = reinterpret_cast<const unsigned*>(S + L.pair_state);
  const int N = L.n_shapes;
  int pairs = 0, movable = 0;
  for (int w = 0; w < (L.n_pairs + 3) / 4; ++w) {   // four pair-state bytes per word (the padding bytes are zero)
    const unsigned v = ps[w] & 0x03030303u;
    pairs += ((v & 0xffu) != 0) + ((v & 0xff00u) != 0) + ((v & 0xff0000u) != 0) + ((v & 0xff000000u) != 0);
  }
  unsigned active = 0u, moves = 0u;
  for (int i = 0; i < N; ++i) {
    const bool on = __float_as_int(S[L.shape_flags + i]) & 1;
    const bool mv = on && (S[L.inv_mass + i] != 0.f || S[L.inv_inertia + i] != 0.f);
    active |= (unsigned)on << i;
    moves |= (unsigned)mv << i;
    movable += mv;
  }
  // joints that share a movable shape run one after the other (the step kernel's rule): depth of that chain
  unsigned long long next = 0ull;   // 4 bits per shape
  int depth = 0;
  for (int q = 0; q < n_joints; ++q) {
    const int a = __float_as_int(S[L.joint_a + q]), b = __float_as_int(S[L.joint_b + q]);
    if (!(__float_as_int(S[L.joint_flags + q]) & 1) || a < 0 || a >= N || b < 0 || b >= N || a == b) continue;
    if (!((active >> a) & (active >> b) & 1u) || !(S[L.inv_mass + a] + S[L.inv_mass + b] > 0.f)) continue;
    const bool da = (moves >> a) & 1u, db = (moves >> b) & 1u;
    const int lv = max(da ? (int)((next >> (4 * a)) & 15ull) : 0, db ? (int)((next >> (4 * b)) & 15ull) : 0);
    if (da) next = (next & ~(15ull << (4 * a))) | ((unsigned long long)(lv + 1) << (4 * a));
    if (db) next = (next & ~(15ull << (4 * b))) | ((unsigned long long)(lv + 1) << (4 * b));
    depth = max(depth, lv + 1);
  }
  static_assert(14 * 68 + 16 * 4 + 3 < kOrderKeys, "key range");
  keys[env] = kOrderKeys - 1 - (min(pairs, 14) * 68 + min(movable, 16) * 4 + min(depth, 3));   // busiest first
}
// The counting sort.  Slots are handed out in key order (slot s belongs to wavefront s / envs_per_wave), so the
// environments of a wavefront have the same or neighbouring keys.  Inside a key the environments are free to
// trade places, and that freedom is used for the L2: wavefront w of the step kernel runs on XCD w % 8
// (workgroups go to the eight XCDs in turn) and every XCD has an L2 of its own, so the environments whose action
// rows share a 128-byte line (`envs_per_line` neighbours; class c = (env / envs_per_line) % 8) look for a slot
// on XCD c among the slots of their key: the line that one of them fetches is then in the L2 that the others
// ask.  The environments of a key that find the slots of their class taken (the classes of a key are not equally
// large) take what the other classes of the key leave free.
constexpr int kOrderClasses = 8;
__global__ void __launch_bounds__(1024) k2d_order_kernel(int32_t* keys, int32_t* order, int n_envs, int n_waves,
                                                         int envs_per_wave, int envs_per_line) {
  __shared__ int count[kOrderKeys * kOrderClasses];   // histogram over (key, class); then ranks
  __shared__ int part[1024];
  const int t = threadIdx.x;
  auto class_of = [&](int env) { return (env / envs_per_line) % kOrderClasses; };
  for (int q = t; q < kOrderKeys * kOrderClasses; q += blockDim.x) count[q] = 0;
  __syncthreads();
  for (int env = t; env < n_envs; env += blockDim.x) atomicAdd(&count[keys[env] * kOrderClasses + class_of(env)], 1);
  __syncthreads();
  // exclusive prefix sum over the bins: thread t owns the bins of key t
  static_assert(kOrderKeys == 1024, "one thread per key");
  int mine = 0;
  for (int c = 0; c < kOrderClasses; ++c) mine += count[t * kOrderClasses + c];
  part[t] = mine;
  __syncthreads();
  for (int d = 1; d < 1024; d <<= 1) {
    const int v = t >= d ? part[t - d] : 0;
    __syncthreads();
    part[t] += v;
    __syncthreads();
  }
  int acc = part[t] - mine;
  for (int c = 0; c < kOrderClasses; ++c) { const int n = count[t * kOrderClasses + c]; count[t * kOrderClasses + c] = acc; acc += n; }
  for (int sl = t; sl < n_waves * envs_per_wave; sl += blockDim.x) order[sl] = -1;
  __syncthreads();
  // every environment draws its rank (key-major, class-minor); the rank is kept beside the key
  for (int env = t; env < n_envs; env += blockDim.x) {
    const int key = keys[env];
    const int r = atomicAdd(&count[key * kOrderClasses + class_of(env)], 1);
    keys[env] = key | (r << 10);
  }
  __syncthreads();
  // now count[x] is the first rank of bin x + 1: the bins' boundaries can be read off again
  auto first_rank = [&](int x) { return x > 0 ? count[x - 1] : 0; };
  const int wave_slots = envs_per_wave, period = kOrderClasses * envs_per_wave;
  // slots below s that lie on XCD c, and the j-th slot of XCD c
  auto slots_before = [&](int c, int s) {
    const int full = s / period, rem = s % period;
    return full * wave_slots + min(max(rem - c * wave_slots, 0), wave_slots);
  };
  auto slot_of = [&](int c, int j) { return ((j / wave_slots) * kOrderClasses + c) * wave_slots + j % wave_slots; };
  for (int env = t; env < n_envs; env += blockDim.x) {
    const int key = keys[env] & 1023, r = keys[env] >> 10, c = class_of(env);
    const int r0 = first_rank(key * kOrderClasses), r1 = count[key * kOrderClasses + kOrderClasses - 1];   // the key's slots
    const int i = r - first_rank(key * kOrderClasses + c);                                               // place within (key, class)
    const int have = slots_before(c, r1) - slots_before(c, r0);
    if (i < have) {
      order[slot_of(c, slots_before(c, r0) + i)] = env;
    } else {   // the o-th environment of the key without a slot on its XCD takes the o-th slot the key has left
      int o = i - have;
      for (int c2 = 0; c2 < c; ++c2) {
        const int n2 = count[key * kOrderClasses + c2] - first_rank(key * kOrderClasses + c2);
        o += max(0, n2 - (slots_before(c2, r1) - slots_before(c2, r0)));
      }
      for (int c2 = 0; c2 < kOrderClasses; ++c2) {
        const int n2 = count[key * kOrderClasses + c2] - first_rank(key * kOrderClasses + c2);
        const int fre = max(0, (slots_before(c2, r1) - slots_before(c2, r0)) - n2);
        if (o < fre) { order[slot_of(c2, slots_before(c2, r0) + n2 + o)] = env; break; }
        o -= fre;
      }
    }
  }
}

// Reward and termination (Sec. 3.2): 16 lanes per environment, lane i looks at shape i.  A green shape in
// active collision with a blue one ends the episode with +1, with a red one with -1; the dense term is
// kappa * (d_t - d_{t+1}), d = smallest centre distance over the active (green, blue) pairs.
__global__ void __launch_bounds__(64) k2d_outcome_kernel(const float* state, float* dist, float* reward,
                                                         uint8_t* done, int n_envs, int rec_words, k2d_layout L,
                                                         float kappa, int green, int blue, int red) {
  const int lane = threadIdx.x, i = lane & 15;
  const int env = blockIdx.x * 4 + (lane >> 4);
  const bool ok = env < n_envs;
  const float* S = state + (size_t)(ok ? env : 0) * rec_words;
  const unsigned char* ps = reinterpret_cast<const unsigned char*>(S + L.pair_state);
  const int N = L.n_shapes;
  const bool mine = ok && i < N;
  const int fl = mine ? __float_as_int(S[L.shape_flags + i]) : 0;
  const bool act = fl & 1;
  const int role = act ? (fl >> 8) : -1;
  const float px = mine ? S[L.pos_x + i] : 0.f, py = mine ? S[L.pos_y + i] : 0.f;
  bool goal = false, bad = false;
  float best = INFINITY;
  for (int j = 0; j < N; ++j) {   // (every lane takes part in the exchange; only green lanes use it)
    const int rj = __shfl(role, j, 16);
    const float qx = __shfl(px, j, 16), qy = __shfl(py, j, 16);
    if (role == green && j != i && rj >= 0) {
      const int a = min(i, j), b = max(i, j);
      const bool touching = (ps[a * (2 * N - a - 1) / 2 + (b - a - 1)] & 3) != 0;
      if (rj == blue) {
        goal |= touching;
        const float dx = qx - px, dy = qy - py;
        best = fminf(best, sqrtf(dx * dx + dy * dy));
      } else if (rj == red) {
        bad |= touching;
      }
    }
  }
  for (int d = 8; d >= 1; d >>= 1) {
    best = fminf(best, __shfl_xor(best, d, 16));
    goal |= (bool)__shfl_xor((int)goal, d, 16);
    bad |= (bool)__shfl_xor((int)bad, d, 16);
  }
  if (ok && i == 0) {
    const bool have = best < INFINITY;
    const float d_new = have ? best : 0.f;
    const float d_prev = dist[env];
    const float dense = (d_prev >= 0.f && have) ? kappa * (d_prev - d_new) : 0.f;
    const float sparse = goal ? 1.f : (bad ? -1.f : 0.f);
    reward[env] = sparse + dense;
    done[env] = (goal || bad) ? 1 : 0;
    dist[env] = d_new;
  }
}

// Health of the batch: an environment is flagged when position, rotation or velocity of one of its active
// shapes is not finite (a simulation that blew up).  16 lanes per environment, lane i looks at shape i.
__global__ void k2d_zero_word_kernel(int32_t* w) { *w = 0; }
__global__ void __launch_bounds__(64) k2d_health_kernel(const float* state, uint8_t* bad, int32_t* count, int n_envs,
                                                        int rec_words, k2d_layout L) {
  const int lane = threadIdx.x, i = lane & 15;
  const int env = blockIdx.x * 4 + (lane >> 4);
  const bool ok = env < n_envs;
  const float* S = state + (size_t)(ok ? env : 0) * rec_words;
  int mine = 0;
  if (ok && i < L.n_shapes && (__float_as_int(S[L.shape_flags + i]) & 1)) {
    const int words[6] = {L.pos_x, L.pos_y, L.theta, L.vel_x, L.vel_y, L.omega};
    for (int w = 0; w < 6; ++w) {
      const unsigned u = (unsigned)__float_as_int(S[words[w] + i]);
      if ((u & 0x7f800000u) == 0x7f800000u) mine = 1;   // exponent all ones: infinity or NaN
    }
  }
  for (int d = 8; d >= 1; d >>= 1) mine |= __shfl_xor(mine, d, 16);
  if (ok && i == 0) {
    bad[env] = (uint8_t)mine;
    if (mine) atomicAdd(count, 1);
  }
}

// ---------------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------------
// Two lane mappings per capacity class: 16 lanes per environment (four environments per wavefront) and 8
// lanes per environment (eight per wavefront: half the instructions per environment, but an LDS image twice
// as large per wavefront).
using CfgS = Cfg<5, 2, 1, 1, 4>;
using CfgM = Cfg<6, 3, 2, 2, 2>;
using CfgL = Cfg<12, 4, 6, 2, 2>;
using CfgS8 = Cfg<5, 2, 1, 1, 2>;
using CfgM8 = Cfg<6, 3, 2, 2, 1>;
using CfgL8 = Cfg<12, 4, 6, 2, 1>;
static_assert(CfgS::G == 16 && CfgM::G == 16 && CfgL::G == 16 && CfgS8::G == 8 && CfgM8::G == 8 && CfgL8::G == 8, "lane mappings");
static_assert(CfgS::REC_WORDS == CfgS8::REC_WORDS && CfgM::REC_WORDS == CfgM8::REC_WORDS &&
                  CfgL::REC_WORDS == CfgL8::REC_WORDS, "the mappings of a class share one record");
// the LDS images of a CU's resident wavefronts must fit its 160 KiB: eight (16 lanes) or four (8 lanes) per CU
static_assert(CfgL::LDS_BYTES * 8 <= 160 * 1024 && CfgL8::LDS_BYTES * 4 <= 160 * 1024, "L image too large");
// environments beyond which the 8-lane mapping is chosen: what the 16-lane mapping keeps resident at once
constexpr int kResidentEnvs16 = 256 * 8 * 4;

int caps_class(const k2d_caps* c) {
  if (!c) return -1;
  if (c->n_polygons == 5 && c->n_circles == 2 && c->n_joints == 1 && c->n_thrusters == 1) return 0;
  if (c->n_polygons == 6 && c->n_circles == 3 && c->n_joints == 2 && c->n_thrusters == 2) return 1;
  if (c->n_polygons == 12 && c->n_circles == 4 && c->n_joints == 6 && c->n_thrusters == 2) return 2;
  return -1;
}
int rec_words_of(int cls) { return cls == 0 ? CfgS::REC_WORDS : cls == 1 ? CfgM::REC_WORDS : CfgL::REC_WORDS; }

// Per-device host bookkeeping (a process may drive several GPUs from several threads).
constexpr int kMaxDevices = 64;
std::mutex g_host_mutex;

// Ordering scratch of k2d_step_noalloc: slot -> environment for one launch, then the sort keys.  One copy
// per GPU, inside the code object, held until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress; kernels get the address that call returns.
constexpr int kNoAllocSlots = (K2D_NOALLOC_MAX_ENVS + 7) / 8 * 8;
__device__ __align__(256) int32_t scratch[2 * kNoAllocSlots];
int32_t* g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch` (looked up once per device).
int scratch_of_current_device(int32_t** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return K2D_E_HIP;
  std::lock_guard<std::mutex> lock(g_host_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return K2D_E_HIP;
    g_scratch_ptr[dev] = static_cast<int32_t*>(p);
  }
  *out = g_scratch_ptr[dev];
  return K2D_OK;
}

// A kernel launch that records its own failure in `ok`: an error that an earlier, unrelated runtime call
// of this thread left behind is read off first, so that it is not taken for this launch's.
#define K2D_LAUNCH(ok, ...) \
  do { (void)hipGetLastError(); hipLaunchKernelGGL(__VA_ARGS__); ok = (hipGetLastError() == hipSuccess) && ok; } while (0)

#ifdef K2D_PHASE_TIMERS
unsigned long long* g_phase_clocks = nullptr;   // caller-owned device buffer, kPhaseSlots words per wavefront
long g_phase_waves = 0;
bool g_phase_keep_order = false;                // launches take the environments as they are numbered
#endif

template <class K, bool RESET, bool BATCHED>
int launch_step(float* state, const float* actions, int n_envs, int n_steps, const Params& prm, const float* levels,
                int n_levels, const int32_t* reset_level, int32_t* order, int rec_words, const k2d_layout& layout,
                hipStream_t st) {
  {   // the kernel's LDS image is larger than the default limit: raise it once per device
    static bool attr_done[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return K2D_E_HIP;
    std::lock_guard<std::mutex> lock(g_host_mutex);
    if (!attr_done[dev]) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k2d_step_kernel<K, RESET, BATCHED>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, K::LDS_BYTES) != hipSuccess)
        return K2D_E_HIP;
      attr_done[dev] = true;
    }
  }
  int grid = (n_envs + K::EPW - 1) / K::EPW;
  bool ok = true;
  if (order) {   // (a launch of a few steps is not worth the ordering pass)
    int32_t* keys = order + grid * K::EPW;
    K2D_LAUNCH(ok, k2d_order_keys_kernel, dim3((n_envs + 255) / 256), dim3(256), 0, st, state, keys, n_envs, rec_words,
                       layout, K::J);
    // action rows that share a 128-byte line (rows of K::A floats; at least one environment per line)
    const int envs_per_line = K::A > 0 && 32 / K::A > 0 ? 32 / K::A : 1;
    K2D_LAUNCH(ok, k2d_order_kernel, dim3(1), dim3(1024), 0, st, keys, order, n_envs, grid, K::EPW, envs_per_line);
  }
#ifdef K2D_PHASE_TIMERS
  K2D_LAUNCH(ok, (k2d_step_kernel<K, RESET, BATCHED>), dim3(grid), dim3(64), K::LDS_BYTES, st, state, actions, n_envs,
                     n_steps, prm, levels, n_levels, reset_level, order, grid <= g_phase_waves ? g_phase_clocks : nullptr);
#else
  K2D_LAUNCH(ok, (k2d_step_kernel<K, RESET, BATCHED>), dim3(grid), dim3(64), K::LDS_BYTES, st, state, actions, n_envs,
                     n_steps, prm, levels, n_levels, reset_level, order);
#endif
  return ok ? K2D_OK : K2D_E_HIP;
}

}  // namespace

struct k2d_batch {
  int cls;
  k2d_caps caps;
  k2d_params params;
  k2d_layout layout;
  int n_envs;
  int rec_words;
  float* state;
  int32_t* order;   // behind the records in the caller's buffer: slot -> environment for one launch
  int lanes;        // lanes per environment of the step kernel: 8, 16, or 0 = chosen by the batch size
};

// launches of fewer steps than this keep the identity ordering (the ordering pass would cost more than it could save)
constexpr int kOrderMinSteps = 8;
// the counting sort keeps an environment's rank in 21 bits beside its key
constexpr int kOrderMaxEnvs = 1 << 21;
static size_t records_bytes(int cls, int n_envs) {
  return ((size_t)n_envs * rec_words_of(cls) * sizeof(float) + 255) / 256 * 256;
}

static Params device_params(const k2d_params& p) {
  Params prm;
  prm.h = p.dt / (float)p.n_substeps;
  prm.gravity_y = p.gravity_y;
  prm.n_substeps = p.n_substeps;
  prm.n_iters = p.n_iters;
  prm.warm_start = p.warm_start;
  prm.alpha = p.alpha; prm.beta = p.beta; prm.gamma = p.gamma; prm.rho = p.rho; prm.slop = p.slop;
  prm.rest_thr = p.restitution_threshold;
  prm.clip_thr = p.clip_thruster_01;
  prm.joint_alpha = p.joint_alpha; prm.joint_beta = p.joint_beta; prm.tie_eps = p.tie_eps;
  prm.n_batches = 0;
  prm.lowest_free_level = p.sweep_order == K2D_SWEEP_LEVELS;
  return prm;
}

template <bool RESET, bool BATCHED>
static int step_launch_as(k2d_batch* b, const float* actions_dev, int n_envs, int n_steps, const float* lv, int n_levels,
                          const int32_t* reset_level_dev, int32_t* order_buf, hipStream_t st) {
  Params prm = device_params(b->params);
  if (BATCHED) {
    prm.n_batches = (2 * b->layout.n_pairs + b->params.batch_size - 1) / b->params.batch_size;
    if (prm.n_batches < 2) return K2D_E_ARG;   // (the kernel relies on the two points of a pair being in different batches)
  }
  // A launch of many steps takes its environments in the order of their expected work: the four of a
  // wavefront are then alike, and what a wavefront skips when none of its environments changed (candidate
  // list, dependency levels) it skips more often (7 % of the launch time on the Large workload).
  int32_t* ord = (n_steps >= kOrderMinSteps && n_envs < kOrderMaxEnvs) ? order_buf : nullptr;
#ifdef K2D_PHASE_TIMERS
  if (g_phase_keep_order) ord = nullptr;
#endif
  // lane mapping: as set on the batch; else 16 lanes per environment, except for Small environments in
  // batches larger than that mapping keeps resident at once.  (Measured on MI355X: with 8 lanes the Small
  // class steps 16384 and more environments 1.5 to 1.7 times faster; the Medium and Large classes are
  // slower with 8 lanes at every batch size -- their LDS images allow one wavefront of eight environments per
  // SIMD, whose dependent instructions then have no second wavefront to overlap with.)
  int lanes = b->lanes;
  if (lanes == 0) lanes = (b->cls == 0 && n_envs > kResidentEnvs16 && !(BATCHED && b->params.batch_size > 16)) ? 8 : 16;
  if (lanes == 8 && BATCHED && b->params.batch_size > 16) return K2D_E_ARG;
#define K2D_STEP_AS(CFG) \
  launch_step<CFG, RESET, BATCHED>(b->state, actions_dev, n_envs, n_steps, prm, lv, n_levels, reset_level_dev, ord, \
                                   b->rec_words, b->layout, st)
  if (lanes == 8) {
    switch (b->cls) {
      case 0: return K2D_STEP_AS(CfgS8);
      case 1: return K2D_STEP_AS(CfgM8);
      default: return K2D_STEP_AS(CfgL8);
    }
  }
  switch (b->cls) {
    case 0: return K2D_STEP_AS(CfgS);
    case 1: return K2D_STEP_AS(CfgM);
    default: return K2D_STEP_AS(CfgL);
  }
#undef K2D_STEP_AS
}
template <bool RESET>
static int step_launch(k2d_batch* b, const float* actions_dev, int n_envs, int n_steps, const float* lv, int n_levels,
                       const int32_t* reset_level_dev, int32_t* order_buf, hipStream_t st) {
  if (b->params.batch_size > 0)
    return step_launch_as<RESET, true>(b, actions_dev, n_envs, n_steps, lv, n_levels, reset_level_dev, order_buf, st);
  return step_launch_as<RESET, false>(b, actions_dev, n_envs, n_steps, lv, n_levels, reset_level_dev, order_buf, st);
}

extern "C" {

#ifdef K2D_PHASE_TIMERS
// Instrumented build only: where the step kernel leaves its phase clocks (device memory, kPhaseSlots
// 64-bit words for each of n_waves wavefronts; a launch with more wavefronts than that records nothing).
// Returns the number of words per wavefront.
int k2d_debug_set_phase_buffer(void* clocks_dev, long n_waves) {
  g_phase_clocks = static_cast<unsigned long long*>(clocks_dev);
  g_phase_waves = clocks_dev ? n_waves : 0;
  return kPhaseSlots;
}
// Instrumented build only: launches keep the environments in the order of their numbers (no sorting by
// expected work), so that a measurement can decide which environments share a wavefront.
int k2d_debug_keep_order(int on) {
  g_phase_keep_order = on != 0;
  return K2D_OK;
}
#endif

int k2d_get_layout(const k2d_caps* caps, k2d_layout* out) {
  if (!caps || !out) return K2D_E_ARG;
  if (caps_class(caps) < 0) return K2D_E_CAP;
  *out = make_layout(caps->n_polygons, caps->n_circles, caps->n_joints, caps->n_thrusters);
  return K2D_OK;
}

int k2d_obs_dim(const k2d_caps* caps) {
  if (caps_class(caps) < 0) return -1;
  return make_layout(caps->n_polygons, caps->n_circles, caps->n_joints, caps->n_thrusters).obs_dim;
}

size_t k2d_state_bytes(const k2d_caps* caps, int n_envs) {
  int cls = caps_class(caps);
  if (cls < 0 || n_envs < 1) return 0;
  return records_bytes(cls, n_envs) + 2 * (size_t)((n_envs + 7) / 8 * 8) * sizeof(int32_t);   // + ordering, keys
}

int k2d_alloc_batch(const k2d_caps* caps, const k2d_params* params, int n_envs, void* state_dev, size_t state_bytes,
                    k2d_batch** out) {
  if (!caps || !params || !state_dev || !out || n_envs < 1) return K2D_E_ARG;
  if ((reinterpret_cast<uintptr_t>(state_dev) & 255u) != 0) return K2D_E_ARG;
  int cls = caps_class(caps);
  if (cls < 0) return K2D_E_CAP;
  if (params->n_substeps < 1 || params->n_iters < 0 || !(params->dt > 0.f)) return K2D_E_ARG;
  if (params->batch_size < 0 || params->batch_size > K2D_MAX_BATCH_SIZE) return K2D_E_ARG;
  if (params->sweep_order != K2D_SWEEP_TOURNAMENT && params->sweep_order != K2D_SWEEP_LEVELS) return K2D_E_ARG;
  if (state_bytes < k2d_state_bytes(caps, n_envs)) return K2D_E_SIZE;
  k2d_batch* b = new (std::nothrow) k2d_batch;
  if (!b) return K2D_E_ARG;
  b->cls = cls;
  b->caps = *caps;
  b->params = *params;
  b->layout = make_layout(caps->n_polygons, caps->n_circles, caps->n_joints, caps->n_thrusters);
  b->n_envs = n_envs;
  b->rec_words = rec_words_of(cls);
  b->state = static_cast<float*>(state_dev);
  b->order = reinterpret_cast<int32_t*>(static_cast<char*>(state_dev) + records_bytes(cls, n_envs));
  b->lanes = 0;
  {   // set-up for k2d_step_noalloc on this device (nothing to do, and no error, where no GPU is visible)
    int32_t* unused = nullptr;
    (void)scratch_of_current_device(&unused);
  }
  *out = b;
  return K2D_OK;
}

int k2d_set_lanes_per_env(k2d_batch* b, int lanes) {
  if (!b || (lanes != 0 && lanes != 8 && lanes != 16)) return K2D_E_ARG;
  if (lanes == 8 && b->params.batch_size > 16) return K2D_E_ARG;
  b->lanes = lanes;
  return K2D_OK;
}

int k2d_free_batch(k2d_batch* batch) {
  delete batch;
  return K2D_OK;
}

int k2d_reset(k2d_batch* b, const void* scenes_dev, const int32_t* env_ids_dev, int n, void* stream) {
  if (!b || !scenes_dev || n < 1) return K2D_E_ARG;
  if (!env_ids_dev && n > b->n_envs) return K2D_E_SIZE;
  bool ok = true;
  K2D_LAUNCH(ok, k2d_reset_kernel, dim3(n), dim3(256), 0, static_cast<hipStream_t>(stream), b->state,
                     static_cast<const float*>(scenes_dev), env_ids_dev, n, b->n_envs, b->rec_words, b->layout);
  return ok ? K2D_OK : K2D_E_HIP;
}

int k2d_step(k2d_batch* b, const float* actions_dev, int n_envs, int n_steps, void* stream) {
  if (!b || !actions_dev || n_steps < 1) return K2D_E_ARG;
  if (n_envs != b->n_envs) return K2D_E_SIZE;
  return step_launch<false>(b, actions_dev, n_envs, n_steps, nullptr, 0, nullptr, b->order,
                            static_cast<hipStream_t>(stream));
}

int k2d_step_noalloc(k2d_batch* b, const float* actions_dev, int n_envs, int n_steps, void* stream) {
  if (!b || !actions_dev || n_steps < 1) return K2D_E_ARG;
  if (n_envs != b->n_envs) return K2D_E_SIZE;
  if (n_envs > K2D_NOALLOC_MAX_ENVS) return K2D_E_SIZE;   // the built-in scratch holds no more
  int32_t* order_buf = nullptr;
  if (int rc = scratch_of_current_device(&order_buf)) return rc;
  return step_launch<false>(b, actions_dev, n_envs, n_steps, nullptr, 0, nullptr, order_buf,
                            static_cast<hipStream_t>(stream));
}

int k2d_step_reset(k2d_batch* b, const float* actions_dev, int n_envs, int n_steps, const void* levels_dev,
                   int n_levels, const int32_t* reset_level_dev, void* stream) {
  if (!b || !actions_dev || n_steps < 1 || !levels_dev || n_levels < 1 || !reset_level_dev) return K2D_E_ARG;
  if (n_envs != b->n_envs) return K2D_E_SIZE;
  return step_launch<true>(b, actions_dev, n_envs, n_steps, static_cast<const float*>(levels_dev), n_levels,
                           reset_level_dev, b->order, static_cast<hipStream_t>(stream));
}

int k2d_read_obs(k2d_batch* b, float* obs_dev, void* stream) {
  if (!b || !obs_dev) return K2D_E_ARG;
  const k2d_caps& c = b->caps;
  long n = (long)b->n_envs * (c.n_polygons + c.n_circles + c.n_joints + c.n_thrusters);
  bool ok = true;
  K2D_LAUNCH(ok, k2d_obs_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     b->state, obs_dev, b->n_envs, b->rec_words, b->layout, c.n_polygons, c.n_circles, c.n_joints,
                     c.n_thrusters);
  return ok ? K2D_OK : K2D_E_HIP;
}

int k2d_read_contacts(k2d_batch* b, uint8_t* pair_count_dev, uint32_t* shape_adj_dev, void* stream) {
  if (!b) return K2D_E_ARG;
  if (!pair_count_dev && !shape_adj_dev) return K2D_OK;
  bool ok = true;
  K2D_LAUNCH(ok, k2d_contacts_kernel, dim3(b->n_envs), dim3(128), 0, static_cast<hipStream_t>(stream), b->state,
                     pair_count_dev, shape_adj_dev, b->n_envs, b->rec_words, b->layout);
  return ok ? K2D_OK : K2D_E_HIP;
}

int k2d_read_entities(k2d_batch* b, float* shapes_dev, float* joints_dev, int32_t* joint_idx_dev, float* thrusters_dev,
                      int32_t* thruster_idx_dev, uint32_t* masks_dev, void* stream) {
  if (!b || !shapes_dev || !masks_dev) return K2D_E_ARG;
  const k2d_caps& c = b->caps;
  if ((c.n_joints > 0 && (!joints_dev || !joint_idx_dev)) || (c.n_thrusters > 0 && (!thrusters_dev || !thruster_idx_dev)))
    return K2D_E_ARG;
  if (b->layout.n_shapes > 16) return K2D_E_CAP;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long n = (long)b->n_envs * (c.n_polygons + c.n_circles + 2 * c.n_joints + c.n_thrusters);
  bool ok = true;
  K2D_LAUNCH(ok, k2d_entities_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, b->state, shapes_dev,
                     joints_dev, joint_idx_dev, thrusters_dev, thruster_idx_dev, b->n_envs, b->rec_words, b->layout,
                     c.n_polygons, c.n_circles, c.n_joints, c.n_thrusters);
  K2D_LAUNCH(ok, k2d_masks_kernel, dim3((b->n_envs + 3) / 4), dim3(64), 0, st, b->state, masks_dev, b->n_envs,
                     b->rec_words, b->layout, c.n_joints);
  return ok ? K2D_OK : K2D_E_HIP;
}

int k2d_decode_actions(const k2d_caps* caps, const int32_t* discrete_dev, float* actions_dev, size_t n_rows,
                       void* stream) {
  if (!caps || !discrete_dev || !actions_dev) return K2D_E_ARG;
  if (caps_class(caps) < 0) return K2D_E_CAP;
  const int A = caps->n_joints + caps->n_thrusters;
  const size_t n = n_rows * (size_t)A;
  if (n == 0) return K2D_OK;
  bool ok = true;
  K2D_LAUNCH(ok, k2d_decode_actions_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), discrete_dev, actions_dev, n, caps->n_joints, A);
  return ok ? K2D_OK : K2D_E_HIP;
}

int k2d_read_outcome(k2d_batch* b, const k2d_reward_params* rp, float* dist_dev, float* reward_dev, uint8_t* done_dev,
                     void* stream) {
  if (!b || !rp || !dist_dev || !reward_dev || !done_dev) return K2D_E_ARG;
  if (b->layout.n_shapes > 16) return K2D_E_CAP;
  bool ok = true;
  K2D_LAUNCH(ok, k2d_outcome_kernel, dim3((b->n_envs + 3) / 4), dim3(64), 0, static_cast<hipStream_t>(stream),
                     b->state, dist_dev, reward_dev, done_dev, b->n_envs, b->rec_words, b->layout, rp->kappa,
                     rp->role_green, rp->role_blue, rp->role_red);
  return ok ? K2D_OK : K2D_E_HIP;
}

int k2d_read_health(k2d_batch* b, uint8_t* bad_dev, int32_t* count_dev, void* stream) {
  if (!b || !bad_dev || !count_dev) return K2D_E_ARG;
  if (b->layout.n_shapes > 16) return K2D_E_CAP;
  hipStream_t st = static_cast<hipStream_t>(stream);
  bool ok = true;
  K2D_LAUNCH(ok, k2d_zero_word_kernel, dim3(1), dim3(1), 0, st, count_dev);
  K2D_LAUNCH(ok, k2d_health_kernel, dim3((b->n_envs + 3) / 4), dim3(64), 0, st, b->state, bad_dev, count_dev,
                     b->n_envs, b->rec_words, b->layout);
  return ok ? K2D_OK : K2D_E_HIP;
}

int k2d_read_state(k2d_batch* b, void* records_dev, void* stream) {
  if (!b || !records_dev) return K2D_E_ARG;
  bool ok = true;
  K2D_LAUNCH(ok, k2d_copy_state_kernel, dim3(b->n_envs), dim3(256), 0, static_cast<hipStream_t>(stream), b->state,
                     static_cast<float*>(records_dev), b->n_envs, b->rec_words, b->layout, 0);
  return ok ? K2D_OK : K2D_E_HIP;
}

int k2d_write_state(k2d_batch* b, const void* records_dev, void* stream) {
  if (!b || !records_dev) return K2D_E_ARG;
  bool ok = true;
  K2D_LAUNCH(ok, k2d_copy_state_kernel, dim3(b->n_envs), dim3(256), 0, static_cast<hipStream_t>(stream), b->state,
                     const_cast<float*>(static_cast<const float*>(records_dev)), b->n_envs, b->rec_words,
                     b->layout, 1);
  return ok ? K2D_OK : K2D_E_HIP;
}

}  // extern "C"
