"""k2d_step_noalloc (the entry point for callers that cannot allocate) against k2d_step, through the C ABI:
same scenes and actions, full state records compared bit for bit, on two calls in a row, the second with
a smaller batch -- the two calls share the GPU's built-in scratch array."""
import numpy as np
import pytest

import scenegen

pytestmark = pytest.mark.gpu


def _records(cfg, n, steps, noalloc):
    import torch
    import paper_2410_23208_amd as k2d
    caps, prm, sc = scenegen.make_scene(cfg, n_envs=n)
    act = torch.from_numpy(scenegen.make_actions(cfg, steps, n)).cuda()
    b = k2d.Batch(caps, n, prm)
    b.reset(k2d.pack_scenes(caps, sc))
    if noalloc:
        b.step_noalloc(act, steps)
    else:
        b.step(act, steps)
    rec = b.read_state().cpu().numpy()
    torch.cuda.synchronize()
    return rec


def test_noalloc_step_equals_step_twice_second_smaller():
    # (launches long enough to use the ordering scratch; the first batch is larger than one round of wavefronts)
    for cfg, n, steps in ((0, 8451, 24), (0, 8259, 16)):
        want = _records(cfg, n, steps, noalloc=False)
        got = _records(cfg, n, steps, noalloc=True)
        assert want.shape == got.shape
        assert np.array_equal(want, got), "cfg %d, %d envs: k2d_step_noalloc differs from k2d_step" % (cfg, n)
        assert (want != 0).any()


def test_noalloc_step_other_capacity_class_after_it():
    for cfg, n in ((1, 8323), (2, 131)):
        want = _records(cfg, n, 16, noalloc=False)
        got = _records(cfg, n, 16, noalloc=True)
        assert np.array_equal(want, got)
