"""GPU parity tests: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars: integer outputs (active-contact masks, manifold point counts) bit-exact; floating-point state within
1e-4 absolute + 1e-4 relative after one step and 1e-3 after 16 steps, environments whose nearest discrete
decision came within 1e-5 of its threshold compared separately.  The kernel is built without contraction
and with the same fixed-sequence sin/cos/tanh as the oracle, so the stronger statement -- identical bits --
is asserted too.
"""
import numpy as np
import pytest

import scenegen
import parity
from helpers import SceneBuilder, params as mkparams

pytestmark = pytest.mark.gpu

SMALL = {0: 67, 1: 131, 2: 259, 3: 131, 4: 195}     # several wavefronts and a ragged tail each


def _both(cfg, n, steps, chunk=None):
    caps, prm, sc = scenegen.make_scene(cfg, n_envs=n)
    act = scenegen.make_actions(cfg, steps, n)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act, chunk=chunk)
    return b, o, caps


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_one_step_within_1e4(cfg):
    b, o, _ = _both(cfg, SMALL[cfg], 1)
    res = parity.compare(b.state_dict(), o.state(), atol=1e-4, rtol=1e-4)
    parity.assert_parity(res, "config %d, 1 step" % cfg, min_clean_frac=0.9)


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_sixteen_steps_within_1e3(cfg):
    b, o, _ = _both(cfg, SMALL[cfg], 16)
    res = parity.compare(b.state_dict(), o.state(), atol=1e-3, rtol=1e-3)
    parity.assert_parity(res, "config %d, 16 steps" % cfg, min_clean_frac=0.6)
    assert len(res["bad_flagged"]) == 0      # even near-threshold environments agree in practice


@pytest.mark.parametrize("cfg,steps", [(0, 200), (1, 64), (2, 64), (3, 96), (4, 64)])
def test_bit_identical_rollouts(cfg, steps):
    b, o, _ = _both(cfg, SMALL[cfg], steps)
    gs, os_ = b.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    assert (os_["pair_count"] > 0).sum() > 0


@pytest.mark.parametrize("cfg,episode,n,steps", [(3, 1, 259, 40), (3, 2, 131, 80), (2, 3, 387, 48), (1, 4, 259, 64),
                                                 (4, 5, 259, 48), (0, 6, 131, 120)])
def test_bit_identical_other_episodes(cfg, episode, n, steps):
    """Other draws of the same workloads (the generator's episode counter), other batch sizes."""
    caps, prm, sc = scenegen.make_scene(cfg, n_envs=n, episode=episode)
    act = scenegen.make_actions(cfg, steps, n)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act)
    gs, os_ = b.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    assert (os_["pair_count"] > 0).sum() > n


@pytest.mark.parametrize("cfg,n,steps,B", [(0, 131, 120, 0), (1, 259, 64, 0), (2, 259, 64, 0), (3, 195, 64, 0),
                                           (4, 259, 48, 0), (2, 131, 32, 16), (0, 67, 40, 5), (1, 131, 32, 1)])
def test_eight_lanes_per_environment_bit_identical(cfg, n, steps, B):
    """The other lane mapping of the step kernel (eight environments per wavefront), forced through
    k2d_set_lanes_per_env: same bits as the oracle on every workload, under both schedules, and the same
    records as the 16-lane mapping."""
    caps, prm, sc = scenegen.make_scene(cfg, n_envs=n)
    prm = dict(prm, batch_size=B)
    act = scenegen.make_actions(cfg, steps, n)
    o = parity.run_oracle(caps, prm, sc, act)
    b8 = parity.run_gpu(caps, prm, sc, act, lanes=8)
    gs, os_ = b8.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    b16 = parity.run_gpu(caps, prm, sc, act, lanes=16)
    assert np.array_equal(b8.read_state().cpu().numpy(), b16.read_state().cpu().numpy())


def test_eight_lanes_dense_pile_and_pool_overflow():
    """Many colliding pairs per environment on eight lanes: two register-held pairs per lane, the LDS pool and
    the records in HBM all take part."""
    caps, prm, sc = scenegen.make_dense_scene(n_envs=131)
    act = scenegen.make_actions(3, 64, 131)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act, lanes=8)
    gs, os_ = b.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    assert ((os_["pair_count"] > 0).sum(1) > 16).any()


@pytest.mark.parametrize("cfg,n,steps,lanes", [(0, 67, 120, 0), (1, 131, 64, 0), (2, 259, 64, 0), (3, 131, 96, 0),
                                               (4, 195, 64, 0), (3, 131, 48, 8), (0, 131, 64, 8)])
def test_level_order_of_the_sweep_bit_identical(cfg, n, steps, lanes):
    """k2d_params.sweep_order = K2D_SWEEP_LEVELS (the colliding pairs visited level after level, each on the
    lowest level free at its movable shapes) against the oracle sweeping in the same order -- and the result
    differs from the tournament order's wherever a shape has several contacts."""
    caps, prm, sc = scenegen.make_scene(cfg, n_envs=n)
    prm = dict(prm, sweep_order=1)
    act = scenegen.make_actions(cfg, steps, n)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act, lanes=lanes)
    gs, os_ = b.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    if cfg in (2, 3):
        other = parity.run_oracle(caps, dict(prm, sweep_order=0), sc, act).state()
        assert not np.array_equal(other["vel"], os_["vel"])


@pytest.mark.parametrize("sweep_order", [0, 1])
def test_stacking_workload_bit_identical(sweep_order):
    """Towers of up to nine boxes: chains of contacts, which the tournament order walks in as many dependent
    steps as a tower is high and the level order in three."""
    caps, prm, sc = scenegen.make_stack_scene(n_envs=131)
    prm = dict(prm, sweep_order=sweep_order)
    act = np.zeros((96, 131, caps[2] + caps[3]), dtype=np.float32)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act)
    gs, os_ = b.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    assert ((os_["pair_count"] > 0).sum(1) == 13).all()


@pytest.mark.parametrize("sweep_order", [0, 1])
def test_dense_pile_workload_bit_identical(sweep_order):
    """Workload 3's heap in a narrow pen: many environments keep more colliding pairs than one per lane, so the
    second register-held pair of a lane is exercised over several wavefronts."""
    caps, prm, sc = scenegen.make_dense_scene(n_envs=195)
    prm = dict(prm, sweep_order=sweep_order)
    act = scenegen.make_actions(3, 96, 195)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act)
    gs, os_ = b.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    n_pairs = (os_["pair_count"] > 0).sum(1)
    assert (n_pairs > 16).sum() >= 8 and n_pairs.mean() > 10


@pytest.mark.parametrize("cfg,B,n,steps", [(0, 16, 67, 120), (0, 1, 67, 60), (0, 32, 131, 60), (1, 16, 131, 64),
                                           (1, 5, 67, 48), (2, 16, 259, 64), (2, 1, 131, 32), (2, 32, 131, 48),
                                           (3, 16, 131, 64), (3, 7, 67, 48), (4, 16, 195, 48)])
def test_batched_schedule_bit_identical(cfg, B, n, steps):
    """The batched impulse resolution of A.8 (16 is the paper's batch size; 1 is a sequential sweep in the plain
    tournament order, 32 the largest the library takes), odd and even numbers of shapes, against the oracle running the same schedule."""
    caps, prm, sc = scenegen.make_scene(cfg, n_envs=n)
    prm = dict(prm, batch_size=B)
    act = scenegen.make_actions(cfg, steps, n)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act)
    gs, os_ = b.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    assert (os_["pair_count"] > 0).sum() > n


def test_batched_schedule_on_the_towers_and_with_restarts():
    import torch
    import paper_2410_23208_amd as k2d
    caps, prm, sc = scenegen.make_stack_scene(n_envs=131)
    prm = dict(prm, batch_size=16)
    act = np.zeros((96, 131, caps[2] + caps[3]), dtype=np.float32)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act)
    gs, os_ = b.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    assert ((os_["pair_count"] > 0).sum(1) == 13).all()
    # the launch that restarts episodes runs the same schedule: no restarts scheduled == plain launch
    caps, prm, sc = scenegen.make_scene(2, n_envs=67)
    prm = dict(prm, batch_size=16)
    act = torch.from_numpy(scenegen.make_actions(2, 24, 67)).cuda()
    words = k2d.pack_scenes(caps, sc)
    x, y = k2d.Batch(caps, 67, prm), k2d.Batch(caps, 67, prm)
    x.reset(words)
    y.reset(words)
    x.step(act)
    y.step_reset(act, torch.from_numpy(words.view(np.int32)).cuda(), torch.full((24, 67), -1, dtype=torch.int32).cuda())
    assert np.array_equal(x.read_state().cpu().numpy(), y.read_state().cpu().numpy())


def test_contacts_and_observation_outputs():
    b, o, caps = _both(3, 131, 40)
    pc, adj = b.read_contacts()
    assert np.array_equal(pc.cpu().numpy().astype(np.float64), o.get("pair_count"))
    assert np.array_equal(adj.cpu().numpy().astype(np.int64) & 0xFFFFFFFF, o.get("shape_adj").astype(np.int64))
    assert pc.sum().item() > 100
    obs = b.read_obs().cpu().numpy().astype(np.float64)
    ref = o.obs()
    assert obs.shape == ref.shape
    assert np.array_equal(obs, ref)


def test_chunking_and_determinism():
    """n_steps in one launch == the same steps in launches of 1, 3, ...; a rerun gives identical bytes."""
    caps, prm, sc = scenegen.make_scene(2, n_envs=100)
    act = scenegen.make_actions(2, 12, 100)
    recs = []
    for chunk in (12, 1, 3, 12):
        b = parity.run_gpu(caps, prm, sc, act, chunk=chunk)
        recs.append(b.read_state().cpu().numpy())
    for r in recs[1:]:
        assert np.array_equal(recs[0], r)


def test_state_roundtrip_checkpoint_resume():
    import torch
    import paper_2410_23208_amd as k2d
    caps, prm, sc = scenegen.make_scene(3, n_envs=64)
    act = torch.from_numpy(scenegen.make_actions(3, 30, 64)).cuda()
    a = k2d.Batch(caps, 64, prm)
    a.reset(k2d.pack_scenes(caps, sc))
    a.step(act[:20].contiguous())
    snap = a.read_state()
    a.step(act[20:].contiguous())
    b = k2d.Batch(caps, 64, prm)
    b.write_state(snap)
    b.step(act[20:].contiguous())
    assert torch.equal(a.read_state(), b.read_state())


def test_heterogeneous_batch_with_resets():
    """Config 4 protocol: one step, then a seeded 5 % of the environments restart from new scenes."""
    import torch
    import paper_2410_23208_amd as k2d
    from oracle.k2d_oracle import Oracle
    n, steps = 195, 24
    caps, prm, sc = scenegen.make_scene(4, n_envs=n)
    act = scenegen.make_actions(4, steps, n)
    o = Oracle(caps, n, prm, "f32")
    o.load_scene(sc)
    b = k2d.Batch(caps, n, prm)
    b.reset(k2d.pack_scenes(caps, sc))
    act_d = torch.from_numpy(act).cuda()
    n_reset = 0
    for s in range(steps):
        o.step(act[s:s + 1])
        b.step(act_d[s:s + 1].contiguous())
        ids = scenegen.reset_ids(4, s, n)
        if len(ids):
            _, _, fresh = scenegen.make_scene(4, env_ids=ids, episode=s + 1)
            o.load_scene(fresh, env_ids=ids)
            o.set("min_margin", np.full((len(ids), 1), np.inf), ids)
            b.reset(k2d.pack_scenes(caps, fresh), env_ids=ids)
            n_reset += len(ids)
    assert n_reset > steps
    gs, os_ = b.state_dict(), o.state()
    res = parity.compare(gs, os_, atol=1e-3, rtol=1e-3)
    parity.assert_parity(res, "hetero with resets")
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k


@pytest.mark.parametrize("cfg,n,steps,sweep_order", [(4, 195, 24, 0), (1, 131, 30, 0), (0, 67, 20, 0), (4, 195, 24, 1),
                                                     (3, 131, 20, 1)])
def test_resets_inside_one_launch(cfg, n, steps, sweep_order):
    """k2d_step_reset: the protocol of the heterogeneous workload (a seeded 5 % of the environments restart
    from new scenes after every step) in ONE launch, against the oracle stepped and reloaded from the host,
    and against the GPU path that alternates k2d_step(1) and k2d_reset."""
    import torch
    import paper_2410_23208_amd as k2d
    from oracle.k2d_oracle import Oracle
    caps, prm, sc = scenegen.make_scene(cfg, n_envs=n)
    prm = dict(prm, sweep_order=sweep_order)
    act = scenegen.make_actions(cfg, steps, n)
    o = Oracle(caps, n, prm, "f32")
    o.load_scene(sc)
    alt = k2d.Batch(caps, n, prm)
    alt.reset(k2d.pack_scenes(caps, sc))
    act_d = torch.from_numpy(act).cuda()
    levels, sched = [], np.full((steps, n), -1, dtype=np.int32)
    for s in range(steps):
        o.step(act[s:s + 1])
        alt.step(act_d[s:s + 1].contiguous())
        ids = scenegen.reset_ids(cfg, s, n, frac=0.08)
        if len(ids):
            _, _, fresh = scenegen.make_scene(cfg, env_ids=ids, episode=s + 1)
            o.load_scene(fresh, env_ids=ids)
            alt.reset(k2d.pack_scenes(caps, fresh), env_ids=ids)
            words = k2d.pack_scenes(caps, fresh)
            sched[s, ids] = np.arange(len(levels), len(levels) + len(ids))
            levels.extend(list(words))
    assert len(levels) > steps
    one = k2d.Batch(caps, n, prm)
    one.reset(k2d.pack_scenes(caps, sc))
    lv = torch.from_numpy(np.stack(levels).view(np.int32)).cuda()
    one.step_reset(act_d, lv, torch.from_numpy(sched).cuda())
    torch.cuda.synchronize()
    assert torch.equal(one.read_state(), alt.read_state())
    gs, os_ = one.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    # the static description of a restarted environment is the new level's (next launch starts from it)
    more = scenegen.make_actions(cfg, 4, n)
    o.step(more)
    one.step(torch.from_numpy(more).cuda())
    gs, os_ = one.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k


@pytest.mark.parametrize("cfg,n,steps", [(3, 131, 12), (2, 259, 40), (0, 67, 30)])
def test_reward_and_termination(cfg, n, steps):
    """k2d_read_outcome after every step against the outcome oracle (Sec. 3.2): flags and floats bit for bit."""
    import torch
    import paper_2410_23208_amd as k2d
    from oracle.k2d_oracle import Oracle
    from oracle import k2d_env
    caps, prm, sc = scenegen.make_scene(cfg, n_envs=n)
    N = caps[0] + caps[1]
    act = scenegen.make_actions(cfg, steps, n)
    o = Oracle(caps, n, prm, "f32")
    o.load_scene(sc)
    b = k2d.Batch(caps, n, prm)
    b.reset(k2d.pack_scenes(caps, sc))
    act_d = torch.from_numpy(act).cuda()
    d_ref = np.full(n, -1.0, dtype=np.float32)
    d_gpu = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
    n_done = n_dense = 0
    for s in range(steps):
        o.step(act[s:s + 1])
        b.step(act_d[s:s + 1].contiguous())
        st = o.state()
        r_ref, done_ref, d_ref = k2d_env.outcome(st["pos"].reshape(n, N, 2), sc["role"], sc["active"], st["pair_count"],
                                                 d_ref, 0.25)
        r, done = b.read_outcome(d_gpu, kappa=0.25)
        assert np.array_equal(done.cpu().numpy(), done_ref), s
        assert np.array_equal(r.cpu().numpy(), r_ref), s
        assert np.array_equal(d_gpu.cpu().numpy(), d_ref), s
        n_done += int(done_ref.sum())
        n_dense += int(((r_ref != 0) & (done_ref == 0)).sum())
    assert n_done > 0 and n_dense > n


@pytest.mark.parametrize("cfg,n,steps", [(4, 131, 30), (1, 67, 20), (3, 67, 10)])
def test_entity_observation_and_masks(cfg, n, steps):
    """k2d_read_entities against the numpy oracle built on the engine oracle's flat observation: exact."""
    from oracle import k2d_env
    b, o, caps = _both(cfg, n, steps)
    _, _, sc = scenegen.make_scene(cfg, n_envs=n)
    ref = k2d_env.entities(o.obs(), sc, o.get("shape_adj"), caps)
    got = b.read_entities()
    for k, v in ref.items():
        g = got[k].cpu().numpy()
        if k == "masks":
            g = g.view(np.uint32)
        assert g.shape == v.shape, k
        assert np.array_equal(g, v), k
    assert (ref["masks"][:, 3] != 0).any() and (ref["masks"][:, 2] != ref["masks"][:, 1]).any() or cfg != 4


def test_multi_discrete_action_decoding():
    import torch
    import paper_2410_23208_amd as k2d
    from oracle import k2d_env
    caps = scenegen.CAPS["L"]
    _, prm, sc = scenegen.make_scene(2, n_envs=5)
    b = k2d.Batch(caps, 5, prm)
    rng = np.random.default_rng(3)
    d = rng.integers(0, 3, size=(7, 5, caps[2] + caps[3])).astype(np.int32)
    out = b.decode_actions(torch.from_numpy(d).cuda()).cpu().numpy()
    assert np.array_equal(out, k2d_env.decode_actions(d, caps[2], caps[3]))


# ------------------------------------------------------------------------------------------ edge cases
def _hand_scene_parity(sb, prm, steps, n_envs=1):
    sc = sb.scene()
    caps = sb.caps
    act = np.zeros((steps, n_envs, caps[2] + caps[3]), dtype=np.float32)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act)
    gs, os_ = b.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    return gs, os_


@pytest.mark.parametrize("cfg,lanes", [(2, 0), (0, 8), (1, 0)])
def test_ordered_launch_of_small_ragged_batches(cfg, lanes):
    """Launches long enough to be ordered (8 steps and more), with so few environments that the classes of the
    ordering (environments sharing an action line, one class per XCD) do not fill their wavefronts evenly: every
    environment must still be stepped exactly once."""
    for n in (2, 3, 5, 9, 17, 31, 33, 47, 65):
        caps, prm, sc = scenegen.make_scene(cfg, n_envs=n)
        act = scenegen.make_actions(cfg, 10, n)
        o = parity.run_oracle(caps, prm, sc, act)
        b = parity.run_gpu(caps, prm, sc, act, lanes=lanes)
        gs, os_ = b.state_dict(), o.state()
        for k in parity.FLOAT_KEYS + parity.INT_KEYS:
            assert np.array_equal(gs[k], os_[k]), (n, k)


def test_single_environment_and_empty_scene():
    caps = scenegen.CAPS["S"]
    sb = SceneBuilder(caps)                      # nothing active at all
    gs, _ = _hand_scene_parity(sb, mkparams(), 3)
    assert np.all(gs["pos"] == 0) and np.all(gs["pair_count"] == 0)
    sb = SceneBuilder(caps)
    sb.box(5.0, 0.1, (0, 0), static=True)
    sb.box(0.3, 0.3, (0.2, 0.45), theta=0.3)
    sb.circle(0.2, (-1.0, 0.35))
    gs, os_ = _hand_scene_parity(sb, mkparams(n_substeps=2, n_iters=6), 50)
    assert os_["pair_count"].sum() >= 2


@pytest.mark.parametrize("B,lanes,sweep_order", [(0, 0, 0), (16, 0, 0), (32, 0, 0), (3, 0, 0), (0, 8, 0), (16, 8, 0),
                                                 (0, 0, 1), (16, 0, 1), (0, 8, 1)])
def test_pile_deeper_than_the_lds_pool(B, lanes, sweep_order):
    """All 16 shapes of an L scene dumped onto one spot: far more active pairs than the per-environment
    LDS pool holds, so the overflow path through the HBM record is exercised (under both schedules)."""
    caps = scenegen.CAPS["L"]
    sb = SceneBuilder(caps, n_envs=3)
    rng = np.random.default_rng(5)
    for e in range(3):
        sb.box(6.0, 0.1, (0, 0), static=True, e=e)
        for k in range(11):
            sb.box(0.3 + 0.02 * k, 0.25, (0.05 * k + 0.01 * e, 0.5 + 0.04 * k), theta=0.1 * k, friction=0.4, e=e)
        for k in range(4):
            sb.circle(0.3, (0.1 * k, 0.6 + 0.05 * k), e=e)
    prm = mkparams(n_substeps=3, n_iters=10, alpha=0.5, beta=0.02, batch_size=B,    # gentle corrections: the pile persists
                   sweep_order=sweep_order)
    sc = sb.scene()
    act = np.zeros((6, 3, caps[2] + caps[3]), dtype=np.float32)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act, lanes=lanes)
    gs, os_ = b.state_dict(), o.state()
    assert (os_["pair_count"] > 0).sum(1).max() > 40
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k


def test_triangles_circles_inside_polygons_and_static_joints():
    caps = scenegen.CAPS["M"]
    sb = SceneBuilder(caps)
    f = sb.box(5.0, 0.1, (0, 0), static=True)
    tri = np.array([[-0.4, -0.2], [0.4, -0.2], [0.0, 0.4]])
    t = sb.polygon(tri, (0.0, 0.5), theta=2.0)
    big = sb.box(0.6, 0.6, (2.0, 0.8))
    c_in = sb.circle(0.1, (2.05, 0.85))              # centre inside the box
    c2 = sb.circle(0.25, (0.1, 1.2))
    sb.joint(f, t, (0.0, 0.5), motor_on=True, speed=2.0, power=0.5)   # hinge on a static shape
    sb.joint(big, c2, (1.5, 1.0), fixed=True)
    _hand_scene_parity(sb, mkparams(n_substeps=2, n_iters=8), 40)


def test_joint_limits_hand_scene():
    """A.4.3: a bar hinged to a static block drops against its limit; a motorised limited hinge in free space."""
    caps = scenegen.CAPS["M"]
    sb = SceneBuilder(caps)
    top = sb.box(0.2, 0.2, (0.0, 2.0), static=True)
    bar = sb.box(0.5, 0.05, (0.5, 2.0))
    a = sb.box(0.4, 0.3, (3.0, 3.0), omega=2.0)
    b = sb.box(0.3, 0.2, (3.3, 3.0))
    sb.box(5.0, 0.1, (0, 0), static=True)
    sb.joint(top, bar, (0.0, 2.0), limits=(-0.1, 0.6))
    sb.joint(a, b, (3.2, 3.0), motor_on=True, speed=2.0, power=0.3, limits=(-0.3, 0.2))
    prm = mkparams(n_substeps=2, n_iters=8)
    sc = sb.scene()
    act = scenegen.make_actions(1, 90, 1)
    o = parity.run_oracle(caps, prm, sc, act)
    b_ = parity.run_gpu(caps, prm, sc, act)
    gs, os_ = b_.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    th = os_["theta"][0]
    assert -0.15 < th[top] - th[bar] < 0.65               # the bar stays within its range


@pytest.mark.parametrize("cfg,steps", [(2, 48), (4, 64)])
def test_joint_limits_generated_scenes(cfg, steps):
    """The generated workloads with every revolute joint limited: bit-identical, and the limits matter."""
    n = SMALL[cfg]
    caps, prm, sc0 = scenegen.make_scene(cfg, n_envs=n)
    sc = scenegen.add_joint_limits(sc0)
    act = scenegen.make_actions(cfg, steps, n)
    o = parity.run_oracle(caps, prm, sc, act)
    b = parity.run_gpu(caps, prm, sc, act)
    gs, os_ = b.state_dict(), o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    free = parity.run_oracle(caps, prm, sc0, act).state()
    assert (np.abs(free["theta"] - os_["theta"]).max(1) > 1e-3).mean() > 0.2


# ------------------------------------------------------------------------- full sizes, sampled outputs
@pytest.mark.parametrize("cfg,steps,n_sample", [(0, 200, 64), (1, 256, 128), (2, 256, 192), (3, 512, 96),
                                                (4, 256, 128)])
def test_full_size_launch_sampled_against_oracle(cfg, steps, n_sample):
    """The launch configuration the benchmark times (full environment count, all steps in one launch);
    environments are independent, so the oracle recomputes a seeded sample of them one by one."""
    import torch
    import paper_2410_23208_amd as k2d
    from oracle import k2d_env
    c = scenegen.CONFIGS[cfg]
    n = c["n_envs"]
    caps, prm, sc = scenegen.make_scene(cfg)
    act = scenegen.make_actions(cfg, steps, n)
    b = k2d.Batch(caps, n, prm)
    b.reset(k2d.pack_scenes(caps, sc))
    b.step(torch.from_numpy(act).cuda(), steps)
    # The generated heaps start from overlapping shapes, and in a few environments in ten thousand the method's
    # own iteration runs away (velocities grow without bound under either side's arithmetic and any order of the
    # sweep).  Which ones do must not differ between the two sides: the environments that the library flags
    # join the sample, and the oracle must blow up in exactly those.
    bad, count = b.read_health()
    bad_ids = np.nonzero(bad.cpu().numpy())[0]
    assert len(bad_ids) == int(count.item()) and len(bad_ids) <= n // 4096
    ids = np.random.default_rng(cfg).choice(n, size=min(n, n_sample), replace=False)
    ids = np.union1d(ids, np.concatenate([bad_ids[:8], [n - 1]]))    # and always the last environment (ragged tail)
    gs = k2d.unpack_state(caps, b.read_state()[torch.from_numpy(ids).cuda()].cpu().numpy())
    o = parity.run_oracle(caps, prm, scenegen.select_envs(sc, ids), act[:, ids])
    os_ = o.state()
    fine = ~np.isin(ids, bad_ids)      # (a blown-up environment holds no meaningful numbers: the flag is what is compared)
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k][fine], os_[k][fine]), k
    N = caps[0] + caps[1]
    want, _ = k2d_env.health(os_["pos"].reshape(len(ids), N, 2), os_["theta"], os_["vel"].reshape(len(ids), N, 2),
                             os_["omega"], np.asarray(sc["active"])[ids])
    assert np.array_equal(want.astype(bool), np.isin(ids, bad_ids))
    # properties that hold at any size, over the whole batch
    full = k2d.unpack_state(caps, b.read_state().cpu().numpy())
    static = np.repeat((sc["inv_mass"] == 0), 2, axis=1)
    assert np.array_equal(full["pos"][static], np.asarray(sc["pos"]).reshape(n, -1)[static])


def test_full_size_heterogeneous_launch_with_restarts_sampled_against_oracle():
    """Workload 4 as the benchmark times it: 16384 environments x 256 steps in ONE k2d_step_reset launch, a
    seeded 5 % of the environments restarting from fresh scenes after every step; a seeded sample of the
    environments is recomputed by the oracle, reloaded from the host at the same steps."""
    import torch
    import paper_2410_23208_amd as k2d
    from oracle.k2d_oracle import Oracle
    cfg = 4
    c = scenegen.CONFIGS[cfg]
    n, steps = c["n_envs"], c["n_steps"]
    caps, prm, sc = scenegen.make_scene(cfg)
    _, _, fresh = scenegen.make_scene(cfg, episode=1)
    act = scenegen.make_actions(cfg, steps, n)
    sched = np.full((steps, n), -1, dtype=np.int32)
    for s in range(steps):
        ids = scenegen.reset_ids(cfg, s, n)
        sched[s, ids] = ids
    b = k2d.Batch(caps, n, prm)
    b.reset(k2d.pack_scenes(caps, sc))
    pool = torch.from_numpy(k2d.pack_scenes(caps, fresh).view(np.int32)).cuda()
    b.step_reset(torch.from_numpy(act).cuda(), pool, torch.from_numpy(sched).cuda(), steps)
    ids = np.sort(np.random.default_rng(44).choice(n, size=128, replace=False))
    ids[0], ids[-1] = 0, n - 1
    gs = k2d.unpack_state(caps, b.read_state()[torch.from_numpy(ids).cuda()].cpu().numpy())
    o = Oracle(caps, len(ids), prm, "f32")
    o.load_scene(scenegen.select_envs(sc, ids))
    n_restarts = 0
    for s in range(steps):
        o.step(act[s:s + 1, ids], n_threads=8)
        rows = np.nonzero(sched[s, ids] >= 0)[0]
        if len(rows):
            o.load_scene(scenegen.select_envs(fresh, ids[rows]), env_ids=rows)
            n_restarts += len(rows)
    assert n_restarts > 1000
    os_ = o.state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    bad, count = b.read_health()
    assert int(count.item()) == 0


def test_very_many_environments_sampled_against_oracle():
    """300 000 small environments in one launch (record and action offsets beyond 2^31 bytes are not reached
    here, beyond 2^27 words are): a seeded sample, the first and the last environment against the oracle."""
    import torch
    import paper_2410_23208_amd as k2d
    n, steps = 300000, 12
    caps, prm, sc = scenegen.make_scene(0, n_envs=n)
    act = scenegen.make_actions(0, steps, n)
    b = k2d.Batch(caps, n, prm)
    b.reset(k2d.pack_scenes(caps, sc))
    b.step(torch.from_numpy(act).cuda(), steps)
    ids = np.sort(np.random.default_rng(3).choice(n, size=96, replace=False))
    ids[0], ids[-1] = 0, n - 1
    gs = k2d.unpack_state(caps, b.read_state()[torch.from_numpy(ids).cuda()].cpu().numpy())
    os_ = parity.run_oracle(caps, prm, scenegen.select_envs(sc, ids), act[:, ids]).state()
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert np.array_equal(gs[k], os_[k]), k
    bad, count = b.read_health()
    assert int(count.item()) == 0


def test_long_rollout_statistics():
    """Beyond the element-wise horizon: distribution statistics of a 256-step rollout agree."""
    b, o, caps = _both(2, 515, 256)
    gs, os_ = b.state_dict(), o.state()
    for stat in (np.nanmean, np.nanstd):
        for k in ("vel", "omega"):
            assert abs(stat(gs[k]) - stat(os_[k])) <= 1e-3 * (abs(stat(os_[k])) + 1.0)
    hg = np.bincount((gs["pair_count"] > 0).sum(1).astype(int), minlength=40)
    ho = np.bincount((os_["pair_count"] > 0).sum(1).astype(int), minlength=40)
    assert np.abs(hg - ho).sum() <= 0.02 * len(gs["pos"])
    assert not np.isnan(gs["pos"]).any()


def test_health_check_flags_the_environments_with_non_finite_state():
    """k2d_read_health against the numpy definition: values planted through k2d_write_state (NaN, infinities,
    in active and in inactive shapes), and a clean batch."""
    import torch
    import paper_2410_23208_amd as k2d
    from oracle import k2d_env
    caps, prm, sc = scenegen.make_scene(1, n_envs=133)      # M scenes: some shapes inactive
    b = k2d.Batch(caps, 133, prm)
    b.reset(k2d.pack_scenes(caps, sc))
    b.step(torch.from_numpy(scenegen.make_actions(1, 8, 133)).cuda())
    bad, count = b.read_health()
    assert int(count.item()) == 0 and not bad.any().item()
    L = k2d.get_layout(caps)
    rec = b.read_state().cpu().numpy().view(np.float32).copy()
    rng = np.random.default_rng(11)
    N = L["n_shapes"]
    for e in rng.choice(133, size=40, replace=False):
        field = ["pos_x", "pos_y", "theta", "vel_x", "vel_y", "omega"][int(rng.integers(6))]
        rec[e, L[field] + int(rng.integers(N))] = [np.nan, np.inf, -np.inf][int(rng.integers(3))]
    b.write_state(torch.from_numpy(rec.view(np.int32)).cuda())
    st = k2d.unpack_state(caps, rec.view(np.uint32))
    want, n_want = k2d_env.health(st["pos"].reshape(133, N, 2), st["theta"], st["vel"].reshape(133, N, 2),
                                  st["omega"], st["active"])
    bad, count = b.read_health()
    assert np.array_equal(bad.cpu().numpy(), want) and int(count.item()) == n_want
    assert 0 < n_want < 40                                  # some of the planted values sit in inactive shapes


# --------------------------------------------------------------------------------- degenerate input
@pytest.mark.parametrize("kind", ["coincident_circles", "zero_length_edge", "joint_on_itself", "indices_out_of_range",
                                  "infinite_inverse_mass"])
def test_degenerate_scenes_have_the_oracles_defined_result(kind):
    """Through k2d_reset and k2d_step: coincident circle centres, a polygon edge without length, a joint with
    both ends on one shape, shape indices outside the arrays, an infinite inverse mass.  The state and the
    observation equal the oracle's bit for bit, and k2d_read_health flags exactly the environments whose
    oracle state is not finite (the one with the infinite inverse mass, which blows up on its first contact)."""
    from helpers import degenerate_scene, same_bits_or_both_nan
    from oracle import k2d_env
    caps, prm, sc, twin, steps = degenerate_scene(kind)
    # three environments: the degenerate one between two copies of a sound scene
    _, _, sound, _, _ = degenerate_scene("coincident_circles") if twin is None else (caps, prm, twin, None, steps)
    batch = {k: np.concatenate([sound[k], sc[k], sound[k]], 0) for k in sc}
    act = np.zeros((steps, 3, caps[2] + caps[3]), dtype=np.float32)
    o = parity.run_oracle(caps, prm, batch, act)
    b = parity.run_gpu(caps, prm, batch, act)
    gs, os_ = b.state_dict(), o.state()
    # an environment that has blown up holds no meaningful numbers: there the two sides must agree that it
    # has (next assertion block), not on which of its entries are NaN and which infinite (the kernel never
    # writes to shapes that no impulse can move, the oracle multiplies their zero inverse mass by the
    # non-finite impulse); everywhere else every bit must agree
    rows = [0, 2] if kind == "infinite_inverse_mass" else [0, 1, 2]
    for k in parity.FLOAT_KEYS + parity.INT_KEYS:
        assert same_bits_or_both_nan(gs[k][rows], os_[k][rows]), k
    assert same_bits_or_both_nan(b.read_obs().cpu().numpy().astype(np.float64)[rows], o.obs()[rows])
    N = caps[0] + caps[1]
    want, n_want = k2d_env.health(os_["pos"].reshape(3, N, 2), os_["theta"], os_["vel"].reshape(3, N, 2),
                                  os_["omega"], batch["active"])
    bad, count = b.read_health()
    assert np.array_equal(bad.cpu().numpy(), want) and int(count.item()) == n_want
    assert n_want == (1 if kind == "infinite_inverse_mass" else 0)
    assert np.isfinite(gs["pos"][[0, 2]]).all()               # the neighbours of a blown-up environment are untouched


def test_device_sin_cos_tanh_against_libm_through_the_observation():
    """The kernel's own sin / cos / tanh (k2d_read_obs evaluates them on the device) against double-precision
    libm at 1.5e-7, over sweeps of the rotation, the angular velocity, the joint's relative rotation and the
    thruster angle -- independent of the oracle's copy of those routines."""
    import torch
    import paper_2410_23208_amd as k2d
    caps = scenegen.CAPS["M"]
    P, C, J, T = caps
    N = P + C
    n = 4096
    rng = np.random.default_rng(17)
    sc = scenegen.empty_scene(caps, n)
    sc["active"][:] = 1
    sc["theta"][:] = np.concatenate([np.linspace(-3.0 * np.pi, 3.0 * np.pi, n * N // 2), rng.uniform(-50, 50, n * N - n * N // 2)]).reshape(n, N)
    sc["omega"][:] = np.concatenate([np.linspace(-120.0, 120.0, n * N // 2), rng.uniform(-6, 6, n * N - n * N // 2)]).reshape(n, N)
    sc["joint_a"][:] = rng.integers(0, N, (n, J))
    sc["joint_b"][:] = (sc["joint_a"] + 1 + rng.integers(0, N - 1, (n, J))) % N
    sc["thruster_angle"][:] = rng.uniform(-2.0 * np.pi, 2.0 * np.pi, (n, T))
    sc = scenegen.to_f32(sc)
    b = k2d.Batch(caps, n, scenegen.default_params())
    b.reset(k2d.pack_scenes(caps, sc))
    obs = b.read_obs().cpu().numpy().astype(np.float64)
    th, om = sc["theta"], sc["omega"]
    worst = 0.0
    for i in range(N):
        base = i * 23 if i < P else P * 23 + (i - P) * 15
        arg = (om[:, i].astype(np.float32) / np.float32(10.0)).astype(np.float64)     # the quotient is an fp32 value
        worst = max(worst, np.abs(obs[:, base + 7] - np.tanh(arg)).max(),
                    np.abs(obs[:, base + 8] - np.sin(th[:, i])).max(), np.abs(obs[:, base + 9] - np.cos(th[:, i])).max())
    for q in range(J):
        base = P * 23 + C * 15 + q * 11
        rel = (th[np.arange(n), sc["joint_a"][:, q]].astype(np.float32) - th[np.arange(n), sc["joint_b"][:, q]].astype(np.float32)).astype(np.float64)
        worst = max(worst, np.abs(obs[:, base + 9] - np.sin(rel)).max(), np.abs(obs[:, base + 10] - np.cos(rel)).max())
    for t in range(T):
        base = P * 23 + C * 15 + J * 11 + t * 6
        worst = max(worst, np.abs(obs[:, base + 4] - np.sin(sc["thruster_angle"][:, t])).max(),
                    np.abs(obs[:, base + 5] - np.cos(sc["thruster_angle"][:, t])).max())
    assert 0.0 < worst < 1.5e-7, worst
