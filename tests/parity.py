"""GPU-vs-oracle comparison helpers (used by the GPU tests, the smoke check and the benchmark)."""
import numpy as np

import scenegen
from oracle.k2d_oracle import Oracle

FLOAT_KEYS = ("pos", "theta", "vel", "omega", "joint_acc", "joint_acc_ang", "lambda_n", "lambda_t")
INT_KEYS = ("pair_count", "prev_active")
BAND = 1e-5      # environments whose nearest discrete decision (penetration sign, reference face, ...) came
                 # closer than this are compared separately: both outcomes are valid there


def run_oracle(caps, params, scene, actions, dtype="f32", n_threads=8):
    o = Oracle(caps, scene["pos"].shape[0], params, dtype)
    o.load_scene(scene)
    o.step(actions, n_threads=n_threads)
    return o


def run_gpu(caps, params, scene, actions, chunk=None, lanes=0):
    import torch
    import paper_2410_23208_amd as k2d
    n = scene["pos"].shape[0]
    b = k2d.Batch(caps, n, params)
    if lanes:
        b.set_lanes_per_env(lanes)        # 8 or 16 lanes per environment instead of the library's own choice
    b.reset(k2d.pack_scenes(caps, scene))
    act = torch.from_numpy(np.ascontiguousarray(actions, dtype=np.float32)).cuda()
    n_steps = act.shape[0]
    chunk = n_steps if chunk is None else chunk
    for s in range(0, n_steps, chunk):
        b.step(act[s:s + chunk].contiguous())
    torch.cuda.synchronize()
    return b


def compare(gpu_state, ora_state, atol, rtol, band=BAND):
    """Per-environment comparison.  Returns a dict with the worst errors over the environments whose
    decisions all stayed outside the band, and the lists of mismatching environments."""
    margin = ora_state["min_margin"][:, 0]
    clean = margin >= band
    bad = np.zeros(margin.shape[0], dtype=bool)
    worst = {}
    for k in INT_KEYS:
        neq = (gpu_state[k] != ora_state[k]).any(1)
        bad |= neq
        worst[k] = int((neq & clean).sum())
    for k in FLOAT_KEYS:
        g, o = gpu_state[k], ora_state[k]
        err = np.abs(g - o) - rtol * np.abs(o)
        err = np.where(np.isnan(g) | np.isnan(o), np.where(np.isnan(g) & np.isnan(o), 0.0, np.inf), err)
        e = err.max(1) if err.shape[1] else np.zeros(err.shape[0])
        bad |= e > atol
        worst[k] = float(e[clean].max()) if clean.any() else 0.0
    return dict(worst=worst, n=len(margin), n_clean=int(clean.sum()), bad_clean=np.nonzero(bad & clean)[0],
                bad_flagged=np.nonzero(bad & ~clean)[0], atol=atol)


def assert_parity(res, what, min_clean_frac=0.5):
    w = res["worst"]
    assert len(res["bad_clean"]) == 0, "%s: environments %s differ (worst %s)" % (what, res["bad_clean"][:10], w)
    assert res["n_clean"] >= min_clean_frac * res["n"], "%s: only %d of %d environments comparable" % (
        what, res["n_clean"], res["n"])
