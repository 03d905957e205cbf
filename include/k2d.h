/* k2d.h -- C boundary of the MI355X-native batched 2D rigid-body step.
 *
 * The library steps thousands of independent scenes ("environments") of the paper's physics engine
 * (Sec. 3.1; Appendix A, Algorithm 1): every scene is a set of fixed-capacity arrays of convex polygons,
 * circles, joints and thrusters with active masks (capacities per environment class: Table 4).
 *
 * Conventions
 *   - every function returns 0 (K2D_OK) or a negative K2D_E_* code; nothing throws, exits or prints;
 *   - pointers named *_dev are DEVICE pointers owned by the caller (e.g. torch tensors); the library never
 *     allocates or frees device memory; `k2d_batch` is a small HOST descriptor owned by the library;
 *   - all device work is enqueued on the caller's stream (`void* stream` is a hipStream_t, NULL = the null
 *     stream) and no call synchronises with the host;
 *   - calls on the same batch must be ordered by the caller (same stream, or events between streams).
 */
#ifndef K2D_H_
#define K2D_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define K2D_OK 0
#define K2D_E_ARG (-1)   /* NULL pointer, non-positive count, misaligned buffer          */
#define K2D_E_CAP (-2)   /* capacities not one of the supported classes (Table 4 sizes) */
#define K2D_E_SIZE (-3)  /* buffer too small, n_envs does not match the batch          */
#define K2D_E_HIP (-4)   /* a HIP call or kernel launch failed                          */

/* Capacities of one environment (Table 4): polygons, circles, joints, thrusters.
 * Supported: {5,2,1,1} (Small), {6,3,2,2} (Medium), {12,4,6,2} (Large).
 * Shapes share one index space: polygons 0..P-1, then circles P..P+C-1. */
typedef struct {
  int32_t n_polygons, n_circles, n_joints, n_thrusters;
} k2d_caps;

/* Parameters of the step, fixed when the batch is created.  The paper names the coefficients but prints no
 * values (A.3.7: alpha, beta; A.4.2: gamma; A.5: rho; Algorithm 1: num_solver_steps, warm starting). */
typedef struct {
  float dt;                    /* time of one step; a substep lasts dt / n_substeps                    */
  float gravity_y;             /* added to v.y of every active dynamic shape, times the substep        */
  int32_t n_substeps;          /* passes of the body of Algorithm 1 per step (same action for all)     */
  int32_t n_iters;             /* num_solver_steps of Algorithm 1                                      */
  int32_t warm_start;          /* A.7: start from last substep's accumulated impulses                  */
  float alpha;                 /* A.3.7 velocity correction: bias speed = alpha * max(pen - slop, 0)   */
  float beta;                  /* A.3.7 positional correction: move apart by beta * max(pen - slop, 0) */
  float gamma;                 /* A.4.2 fixed-joint angular correction speed per radian of error       */
  float rho;                   /* A.5 motor: impulse = power * tanh((w_a - w_b - speed*A) * rho) * dt  */
  float slop;                  /* penetration left uncorrected (0 = literal A.3.7)                     */
  float restitution_threshold; /* approach speeds at or below it take e = 0 (resting contact)          */
  int32_t clip_thruster_01;    /* clamp thruster actions to [0,1] (Sec. 3.2 continuous action range)   */
  float joint_alpha;           /* A.4.1 velocity correction of the joint point constraint, 1/s         */
  float joint_beta;            /* A.4.1 positional correction of the joint point constraint            */
  float tie_eps;               /* A.3.4: b's face is the reference face only if it wins by tie_eps     */
  int32_t batch_size;          /* A.8: 0 = collision constraints one after the other (sweep_order);     */
                               /* B in 1..K2D_MAX_BATCH_SIZE = the manifold points, two per pair in     */
                               /* tournament order, dealt in turn over ceil(points / B) batches; a      */
                               /* batch is solved from the velocities it starts with and its impulses   */
                               /* applied in point order (16 in the paper)                              */
  int32_t sweep_order;         /* A.8 leaves the order of the active collision constraints to the       */
                               /* engine.  K2D_SWEEP_TOURNAMENT (0): the order of a round-robin         */
                               /* tournament over the shapes (round r pairs (m-1, r) and ((r+k) mod     */
                               /* (m-1), (r-k) mod (m-1)), m = N rounded up to even).                   */
                               /* K2D_SWEEP_LEVELS (1): the colliding pairs are walked in that order,   */
                               /* each takes the lowest level that no earlier colliding pair sharing a  */
                               /* movable shape with it has taken, and the sweep visits level 0, then   */
                               /* level 1, ...: fewer dependent steps on piles and stacks.  Both are    */
                               /* sequential sweeps; pairs without a common movable shape are solved    */
                               /* side by side, which changes no bit.  Warm start and positional        */
                               /* corrections follow the same order.                                    */
} k2d_params;
#define K2D_MAX_BATCH_SIZE 32
#define K2D_SWEEP_TOURNAMENT 0
#define K2D_SWEEP_LEVELS 1

/* Word (4-byte) offsets inside one environment record.  A record is an array of 32-bit words, floats
 * unless marked (i) = int32.  Arrays are stored component-major ("structure of arrays" inside the
 * environment): entry i of array X is word X + i.  The first `scene_words` words are the scene
 * description (what k2d_reset consumes); the full `state_words` record adds the contact accumulators.
 *
 *   per shape (N = P + C entries each):
 *     pos_x pos_y theta vel_x vel_y omega inv_mass inv_inertia friction restitution density
 *     shape_flags(i): bit0 = active, bits 8.. = role (passed through to the observation)
 *   per polygon (P entries each):  n_verts(i) in {3,4};  verts: 8 arrays [P], array 2*v+c holds
 *     coordinate c of local vertex v (counter-clockwise, centred on the centre of mass)
 *   per circle (C): radius
 *   per joint (J): joint_flags(i): bit0 active, bit1 fixed, bit2 motor on, bit4 limited (revolute joints
 *     only, A.4.3);  joint_a(i) joint_b(i) shape indices;
 *     anchor_a_x anchor_a_y anchor_b_x anchor_b_y (local frames); theta_f; motor_speed; motor_power;
 *     limit_lo limit_hi (range of theta_a - theta_b of a limited joint);
 *     acc_x acc_y (accumulated point impulse, A.7); acc_ang (accumulated angular impulse of a fixed joint)
 *   per thruster (T): thr_flags(i): bit0 active; thr_body(i); pos_x pos_y (local); angle; power
 *   -- end of scene description --
 *   lambda: [n_pairs][4] = accumulated (normal, friction) impulse of manifold point 0 and of point 1 (A.7);
 *     pairs in lexicographic order of (i < j): index = i*(2N-i-1)/2 + (j-i-1)
 *   pair_state: n_pairs BYTES (padded to a word): bit k = manifold point k was an active collision at the
 *     last substep (Table 2: penetration > 0)
 */
typedef struct {
  int32_t n_shapes, n_pairs;
  int32_t pos_x, pos_y, theta, vel_x, vel_y, omega, inv_mass, inv_inertia, friction, restitution, density,
      shape_flags;
  int32_t n_verts, verts, radius;
  int32_t joint_flags, joint_a, joint_b, anchor_a_x, anchor_a_y, anchor_b_x, anchor_b_y, theta_f, motor_speed,
      motor_power, limit_lo, limit_hi, acc_x, acc_y, acc_ang;
  int32_t thr_flags, thr_body, thr_pos_x, thr_pos_y, thr_angle, thr_power;
  int32_t scene_words;
  int32_t lambda, pair_state;
  int32_t state_words;   /* words of one record as exchanged through k2d_read_state / k2d_write_state */
  int32_t obs_dim;       /* floats per environment written by k2d_read_obs                            */
} k2d_layout;

typedef struct k2d_batch k2d_batch; /* opaque host descriptor */

/* Fills `out` for the given capacities.  K2D_E_CAP if unsupported. */
int k2d_get_layout(const k2d_caps* caps, k2d_layout* out);

/* Bytes of device memory the caller must provide for `n_envs` environments (0 on bad arguments): the records
 * and, behind them, eight bytes per environment in which a launch sorts the environments by expected work. */
size_t k2d_state_bytes(const k2d_caps* caps, int n_envs);

/* Binds a caller-owned device buffer (>= k2d_state_bytes, 256-byte aligned) as the state of a new batch.
 * The buffer's contents are undefined until k2d_reset or k2d_write_state has covered every environment. */
int k2d_alloc_batch(const k2d_caps* caps, const k2d_params* params, int n_envs, void* state_dev,
                    size_t state_bytes, k2d_batch** out);

/* How the step kernel maps environments onto the 64 lanes of a wavefront: `lanes` = 16 (four environments
 * per wavefront), 8 (eight per wavefront: half the instructions per environment, twice the on-chip memory
 * per wavefront), or 0 = chosen per launch (the default: 8 lanes for Small environments in batches of more
 * than 8192, where that is faster, 16 otherwise).  The mapping changes no result (the pairs of a level of
 * the sweep touch disjoint movable shapes, A.8, whichever lanes hold them).  With 8 lanes the batched
 * schedule takes batch sizes up to 16 (the paper's).  K2D_E_ARG otherwise. */
int k2d_set_lanes_per_env(k2d_batch* batch, int lanes);

/* Frees the host descriptor only. */
int k2d_free_batch(k2d_batch* batch);

/* Starts new episodes (Sec. 3.1: a scene is a set of polygons, circles, joints and thrusters in
 * fixed-capacity arrays with active masks; Table 4 gives the capacities).  scenes_dev holds n records of
 * `scene_words` words (layout above), record r goes to environment env_ids_dev[r] (NULL: environment r).
 * A new episode has nothing to warm-start from (A.7): the accumulated joint and collision impulses and the
 * pair states of those environments are zeroed.  Environment indices out of range are skipped.
 * Entities that refer to a shape index outside 0..N-1 (a joint's joint_a / joint_b, a thruster's body), and
 * joints with joint_a == joint_b, are treated as inactive by every entry point. */
int k2d_reset(k2d_batch* batch, const void* scenes_dev, const int32_t* env_ids_dev, int n, void* stream);

/* Advances every environment by n_steps steps of the engine's main loop (Algorithm 1: gravity, collision
 * manifolds of all shape pairs (A.3.1-A.3.4), motors (A.5), thrusters (A.6), warm starting (A.7), n_iters
 * sweeps of joint (A.4) then collision (A.3.5-A.3.7) constraints, Euler step, positional corrections),
 * each step being n_substeps passes with the same action.  The collision constraints of a sweep run in the
 * schedule that k2d_params.batch_size selects (A.8).
 * actions_dev: float [n_steps][n_envs][J+T]: first the J motor actions, then the T thruster actions.
 * n_envs must equal the batch's. */
int k2d_step(k2d_batch* batch, const float* actions_dev, int n_envs, int n_steps, void* stream);

/* k2d_step for callers that cannot allocate device memory or size a workspace for the library: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and
 * results as k2d_step; the one difference is where the launch keeps its ordering of the environments (the
 * eight bytes per environment that k2d_step takes from the tail of the caller's state buffer): here it is
 * a fixed array inside the library's code object, one copy per GPU, 2 * K2D_NOALLOC_MAX_ENVS * 4 bytes,
 * held until the process ends.  Calls hipMalloc / hipFree or any allocating routine never; the array's
 * device address is looked up once per device (k2d_alloc_batch does it when a device is current, else the
 * first call here).  K2D_E_SIZE if n_envs > K2D_NOALLOC_MAX_ENVS.  All calls on one GPU share that GPU's
 * array: calls that may overlap in time on one GPU (different streams) race on it and must be ordered by
 * the caller; every call rewrites the part it uses, nothing has to be cleared between calls. */
#define K2D_NOALLOC_MAX_ENVS 65536
int k2d_step_noalloc(k2d_batch* batch, const float* actions_dev, int n_envs, int n_steps, void* stream);

/* k2d_step with new episodes started inside the launch (training runs every environment on levels sampled
 * anew whenever an episode ends, Sec. 4; Appendix B times the engine over whole rollouts): after step s
 * (0-based) every environment e with reset_level_dev[s * n_envs + e] = l, 0 <= l < n_levels, is
 * re-initialised from record l of levels_dev exactly as k2d_reset would do it (scene description copied,
 * joint and contact accumulators and pair states zeroed); other values (-1) leave the environment alone.
 * levels_dev: n_levels records of `scene_words` words (the layout k2d_reset consumes), device memory;
 * reset_level_dev: int32 [n_steps][n_envs], device memory.  Both must stay valid until the launch has run. */
int k2d_step_reset(k2d_batch* batch, const float* actions_dev, int n_envs, int n_steps, const void* levels_dev,
                   int n_levels, const int32_t* reset_level_dev, void* stream);

/* Floats per environment of the flat symbolic observation that k2d_read_obs writes (Tables 5-7:
 * 23 per polygon, 15 per circle, 11 per joint, 6 per thruster); -1 on a null pointer or unsupported capacities. */
int k2d_obs_dim(const k2d_caps* caps);

/* Flat symbolic observation (the physical entries of Tables 5-7), float [n_envs][obs_dim]; per polygon:
 * pos 2, vel 2, inv_mass, inv_inertia, density, tanh(omega/10), sin theta, cos theta, friction, restitution,
 * vertices 8, n_verts, active, role (23); per circle the same 12 then radius, active, role (15); per joint:
 * active, fixed, anchor_a 2, anchor_b 2, motor power, motor speed, motor on, sin/cos(theta_a - theta_b) (11);
 * per thruster: active, pos 2, power, sin/cos(angle) (6). */
int k2d_read_obs(k2d_batch* batch, float* obs_dev, void* stream);

/* Collisions of the last substep (A.3.1, Table 2: a manifold point is an active collision iff its
 * penetration is positive; polygon pairs have two points, A.3.4).  pair_count_dev uint8 [n_envs][n_pairs] =
 * active manifold points of the pair (0, 1 or 2; lexicographic pair order); shape_adj_dev uint32
 * [n_envs][N]: bit j of word i set iff shapes i and j are in active collision.  Either pointer may be NULL. */
int k2d_read_contacts(k2d_batch* batch, uint8_t* pair_count_dev, uint32_t* shape_adj_dev, void* stream);

/* Symbolic-Entity observation (Sec. 3.2 "Observation Space", Sec. 4, Appendix C Tables 5-7): the set of
 * entities of every environment, and the four attention masks of the entity model.  Device memory, caller-owned.
 *   shapes_dev    float [n_envs][N][30]: position 2, velocity 2, inverse mass, inverse inertia, density,
 *                 tanh(angular velocity / 10), one-hot role (roles 0..3), sin and cos of the rotation, friction,
 *                 restitution, one-hot type (circle, polygon), radius (circles), vertices 8 and one-hot
 *                 (triangle, rectangle) (polygons), active
 *   joints_dev    float [n_envs][2J][11]: active, fixed, anchor on `from` 2, anchor on `to` 2, motor power,
 *                 motor speed, motor on, sin and cos of rotation(from) - rotation(to).  Entity 2q is joint q seen
 *                 from its shape a, entity 2q+1 the same joint with from and to swapped (Appendix C)
 *   joint_idx_dev int32 [n_envs][2J][2]: the (from, to) shapes of every joint entity
 *   thrusters_dev float [n_envs][T][6]: active, position 2 (local), power, sin and cos of the local angle;
 *   thruster_idx_dev int32 [n_envs][T]: the shape a thruster sits on
 *   masks_dev     uint32 [n_envs][4][N]: bit j of word i set iff shape i may attend to shape j -- (0) every
 *                 active shape, (1) itself and the shapes an active joint connects it to, (2) itself and the
 *                 shapes reachable over any number of joints, (3) the shapes it is in active collision with
 * joints_dev / joint_idx_dev may be NULL if J = 0, thrusters_dev / thruster_idx_dev if T = 0. */
int k2d_read_entities(k2d_batch* batch, float* shapes_dev, float* joints_dev, int32_t* joint_idx_dev,
                      float* thrusters_dev, int32_t* thruster_idx_dev, uint32_t* masks_dev, void* stream);

/* Multi-discrete action space (Sec. 3.2 "Action Space"): every motor is off (0), run forwards (1) or backwards
 * (2) at full power, every thruster off (0) or on (1).  discrete_dev: int32 [n_rows][J+T] -> actions_dev:
 * float [n_rows][J+T] (+1, -1, 0), the actions k2d_step consumes; n_rows = n_steps * n_envs. */
int k2d_decode_actions(const k2d_caps* caps, const int32_t* discrete_dev, float* actions_dev, size_t n_rows,
                       void* stream);

/* Reward and termination of the environment built on the engine (Sec. 3.2, "Reward"): the episode of an
 * environment ends with reward +1 if an active green shape is in active collision (a manifold point with
 * penetration > 0 at the last substep) with an active blue shape, else with reward -1 if it is with a red
 * shape; to this the dense term kappa * (d_t - d_{t+1}) is added, d = smallest centre distance over the
 * active (green, blue) pairs.  A shape's role is the integer in bits 8.. of its shape_flags.
 * dist_dev: float [n_envs], in: d_t (negative = no previous step, dense term 0), out: d_{t+1} (0 if the
 * environment has no green or no blue shape; the dense term is then 0 too);
 * reward_dev: float [n_envs]; done_dev: uint8 [n_envs] (1 = episode ended).  Device memory, caller-owned. */
typedef struct {
  float kappa;                               /* weight of the dense term */
  int32_t role_green, role_blue, role_red;   /* which role integers mean green, blue, red */
} k2d_reward_params;
int k2d_read_outcome(k2d_batch* batch, const k2d_reward_params* params, float* dist_dev, float* reward_dev,
                     uint8_t* done_dev, void* stream);

/* Health check of the batch (a solver of this kind can blow up: A.8 names the stability cost of parallel
 * constraint solving): bad_dev[e] = 1 if position, rotation or velocity of an active shape of environment e
 * is infinite or NaN, else 0; *count_dev = number of such environments.  bad_dev: device, n_envs bytes;
 * count_dev: device, one int32 (overwritten).  Enqueued on `stream`; the caller owns both buffers.
 * K2D_E_ARG on a null pointer. */
int k2d_read_health(k2d_batch* batch, uint8_t* bad_dev, int32_t* count_dev, void* stream);

/* Copies full records ([n_envs][state_words] words, layout above) out of / into the batch
 * (checkpoint and resume; k2d_write_state keeps the accumulators it is given). */
int k2d_read_state(k2d_batch* batch, void* records_dev, void* stream);
int k2d_write_state(k2d_batch* batch, const void* records_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* K2D_H_ */
