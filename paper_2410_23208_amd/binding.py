"""Thin ctypes binding of libk2d.so (include/k2d.h).  Argument marshalling only: every step of the path
runs in the HIP kernels.  torch is used for device memory and streams; numpy for packing host-side scene
descriptions into the record layout the header documents.

There is no CPU fallback: without the built library (or without a GPU for the calls that launch
kernels) this module raises.
"""
import ctypes
import os

import numpy as np

from . import build as _build

K2D_OK = 0
_ERR = {-1: "K2D_E_ARG", -2: "K2D_E_CAP", -3: "K2D_E_SIZE", -4: "K2D_E_HIP"}


class k2d_caps(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_polygons", "n_circles", "n_joints", "n_thrusters")]


class k2d_params(ctypes.Structure):
    _fields_ = [("dt", ctypes.c_float), ("gravity_y", ctypes.c_float), ("n_substeps", ctypes.c_int32),
                ("n_iters", ctypes.c_int32), ("warm_start", ctypes.c_int32), ("alpha", ctypes.c_float),
                ("beta", ctypes.c_float), ("gamma", ctypes.c_float), ("rho", ctypes.c_float),
                ("slop", ctypes.c_float), ("restitution_threshold", ctypes.c_float),
                ("clip_thruster_01", ctypes.c_int32), ("joint_alpha", ctypes.c_float),
                ("joint_beta", ctypes.c_float), ("tie_eps", ctypes.c_float), ("batch_size", ctypes.c_int32),
                ("sweep_order", ctypes.c_int32)]


_LAYOUT_FIELDS = ["n_shapes", "n_pairs", "pos_x", "pos_y", "theta", "vel_x", "vel_y", "omega", "inv_mass",
                  "inv_inertia", "friction", "restitution", "density", "shape_flags", "n_verts", "verts", "radius",
                  "joint_flags", "joint_a", "joint_b", "anchor_a_x", "anchor_a_y", "anchor_b_x", "anchor_b_y",
                  "theta_f", "motor_speed", "motor_power", "limit_lo", "limit_hi", "acc_x", "acc_y", "acc_ang", "thr_flags", "thr_body",
                  "thr_pos_x", "thr_pos_y", "thr_angle", "thr_power", "scene_words", "lambda", "pair_state",
                  "state_words", "obs_dim"]


class k2d_reward_params(ctypes.Structure):
    _fields_ = [("kappa", ctypes.c_float), ("role_green", ctypes.c_int32), ("role_blue", ctypes.c_int32),
                ("role_red", ctypes.c_int32)]


class k2d_layout(ctypes.Structure):
    _fields_ = [(n if n != "lambda" else "lambda_", ctypes.c_int32) for n in _LAYOUT_FIELDS]


_lib = None


def _declare(L):
    vp, i32 = ctypes.c_void_p, ctypes.c_int
    L.k2d_get_layout.argtypes = [ctypes.POINTER(k2d_caps), ctypes.POINTER(k2d_layout)]
    L.k2d_obs_dim.argtypes = [ctypes.POINTER(k2d_caps)]
    L.k2d_state_bytes.restype = ctypes.c_size_t
    L.k2d_state_bytes.argtypes = [ctypes.POINTER(k2d_caps), i32]
    L.k2d_alloc_batch.argtypes = [ctypes.POINTER(k2d_caps), ctypes.POINTER(k2d_params), i32, vp, ctypes.c_size_t,
                                  ctypes.POINTER(vp)]
    L.k2d_free_batch.argtypes = [vp]
    L.k2d_set_lanes_per_env.argtypes = [vp, i32]
    L.k2d_reset.argtypes = [vp, vp, vp, i32, vp]
    L.k2d_step.argtypes = [vp, vp, i32, i32, vp]
    L.k2d_step_noalloc.argtypes = [vp, vp, i32, i32, vp]
    L.k2d_step_reset.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp]
    L.k2d_read_obs.argtypes = [vp, vp, vp]
    L.k2d_read_contacts.argtypes = [vp, vp, vp, vp]
    L.k2d_read_entities.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    L.k2d_decode_actions.argtypes = [ctypes.POINTER(k2d_caps), vp, vp, ctypes.c_size_t, vp]
    L.k2d_read_outcome.argtypes = [vp, ctypes.POINTER(k2d_reward_params), vp, vp, vp, vp]
    L.k2d_read_health.argtypes = [vp, vp, vp, vp]
    L.k2d_read_state.argtypes = [vp, vp, vp]
    L.k2d_write_state.argtypes = [vp, vp, vp]
    return L


def lib():
    """The loaded C-ABI library (built beforehand, in-tree)."""
    global _lib
    if _lib is None:
        _lib = _declare(ctypes.CDLL(_build.ensure_built()))
    return _lib


def use_library(path):
    """Bind this module to another build of the same library (the instrumented build of phase_timers.py).
    Call before any batch exists."""
    global _lib
    _lib = _declare(ctypes.CDLL(path))
    return _lib


EXPORTS = ["k2d_get_layout", "k2d_obs_dim", "k2d_state_bytes", "k2d_alloc_batch", "k2d_set_lanes_per_env", "k2d_free_batch", "k2d_reset", "k2d_step",
           "k2d_step_noalloc", "k2d_step_reset", "k2d_read_outcome", "k2d_read_entities", "k2d_decode_actions",
           "k2d_read_obs", "k2d_read_contacts", "k2d_read_health", "k2d_read_state", "k2d_write_state"]


def _check(rc, what):
    if rc != K2D_OK:
        raise RuntimeError("%s failed: %s" % (what, _ERR.get(rc, rc)))


def make_caps(caps):
    return k2d_caps(*[int(x) for x in caps])


def make_params(p):
    p = dict(p)
    p.setdefault("batch_size", 0)
    p.setdefault("sweep_order", 0)
    return k2d_params(**{k: (int(p[k]) if k in ("n_substeps", "n_iters", "warm_start", "clip_thruster_01", "batch_size",
                                                "sweep_order")
                             else float(p[k])) for k, _ in k2d_params._fields_})


def get_layout(caps):
    out = k2d_layout()
    c = make_caps(caps)
    _check(lib().k2d_get_layout(ctypes.byref(c), ctypes.byref(out)), "k2d_get_layout")
    d = {n: getattr(out, n if n != "lambda" else "lambda_") for n in _LAYOUT_FIELDS}
    return d


def obs_dim(caps):
    c = make_caps(caps)
    return lib().k2d_obs_dim(ctypes.byref(c))


def state_bytes(caps, n_envs):
    c = make_caps(caps)
    return lib().k2d_state_bytes(ctypes.byref(c), int(n_envs))


# ---------------------------------------------------------------------------------------------------
# Host-side packing of scene descriptions (dict of per-env arrays) into record words, and back.
# ---------------------------------------------------------------------------------------------------
def pack_scenes(caps, scene):
    """dict of arrays [n, ...] -> uint32 words [n, scene_words] in the layout of k2d.h."""
    L = get_layout(caps)
    P, C, J, T = caps
    N = P + C
    n = scene["pos"].shape[0]
    W = np.zeros((n, L["scene_words"]), dtype=np.uint32)

    def putf(off, arr):
        a = np.ascontiguousarray(np.asarray(arr, dtype=np.float32)).reshape(n, -1)
        W[:, off:off + a.shape[1]] = a.view(np.uint32)

    def puti(off, arr):
        a = np.ascontiguousarray(np.asarray(arr, dtype=np.int32)).reshape(n, -1)
        W[:, off:off + a.shape[1]] = a.view(np.uint32)

    pos = np.asarray(scene["pos"]).reshape(n, N, 2)
    vel = np.asarray(scene["vel"]).reshape(n, N, 2)
    putf(L["pos_x"], pos[..., 0]); putf(L["pos_y"], pos[..., 1]); putf(L["theta"], scene["theta"])
    putf(L["vel_x"], vel[..., 0]); putf(L["vel_y"], vel[..., 1]); putf(L["omega"], scene["omega"])
    for k in ("inv_mass", "inv_inertia", "friction", "restitution", "density"):
        putf(L[k], scene[k])
    puti(L["shape_flags"], (np.asarray(scene["active"]) != 0).astype(np.int32) | (np.asarray(scene["role"]).astype(np.int32) << 8))
    puti(L["n_verts"], scene["n_verts"])
    verts = np.asarray(scene["verts"]).reshape(n, P, 8)            # [n][P][2*v+c]
    putf(L["verts"], np.transpose(verts, (0, 2, 1)))                # -> [n][2*v+c][P]
    putf(L["radius"], scene["radius"])
    jf = ((np.asarray(scene["joint_active"]) != 0).astype(np.int32) |
          ((np.asarray(scene["joint_fixed"]) != 0).astype(np.int32) << 1) |
          ((np.asarray(scene["joint_motor_on"]) != 0).astype(np.int32) << 2))
    if "joint_limited" in scene:
        jf = jf | ((np.asarray(scene["joint_limited"]) != 0).astype(np.int32) << 4)
        putf(L["limit_lo"], scene["joint_limit_lo"]); putf(L["limit_hi"], scene["joint_limit_hi"])
    puti(L["joint_flags"], jf); puti(L["joint_a"], scene["joint_a"]); puti(L["joint_b"], scene["joint_b"])
    aa = np.asarray(scene["joint_anchor_a"]).reshape(n, J, 2)
    ab = np.asarray(scene["joint_anchor_b"]).reshape(n, J, 2)
    putf(L["anchor_a_x"], aa[..., 0]); putf(L["anchor_a_y"], aa[..., 1])
    putf(L["anchor_b_x"], ab[..., 0]); putf(L["anchor_b_y"], ab[..., 1])
    putf(L["theta_f"], scene["joint_theta_f"]); putf(L["motor_speed"], scene["joint_motor_speed"])
    putf(L["motor_power"], scene["joint_motor_power"])
    if "joint_acc" in scene:
        acc = np.asarray(scene["joint_acc"]).reshape(n, J, 2)
        putf(L["acc_x"], acc[..., 0]); putf(L["acc_y"], acc[..., 1]); putf(L["acc_ang"], scene["joint_acc_ang"])
    puti(L["thr_flags"], (np.asarray(scene["thruster_active"]) != 0).astype(np.int32))
    puti(L["thr_body"], scene["thruster_body"])
    tp = np.asarray(scene["thruster_pos"]).reshape(n, T, 2)
    putf(L["thr_pos_x"], tp[..., 0]); putf(L["thr_pos_y"], tp[..., 1])
    putf(L["thr_angle"], scene["thruster_angle"]); putf(L["thr_power"], scene["thruster_power"])
    return W


def unpack_state(caps, words):
    """uint32 words [n, state_words] (k2d_read_state) -> dict of float64 / int arrays shaped like the
    scene description plus accumulators (lambda_n, lambda_t, prev_active as [n, n_pairs*2])."""
    L = get_layout(caps)
    P, C, J, T = caps
    N = P + C
    NP = L["n_pairs"]
    W = np.ascontiguousarray(words).view(np.uint32)
    n = W.shape[0]
    F = W.view(np.float32)
    I = W.view(np.int32)

    def f(off, cnt):
        return F[:, off:off + cnt].astype(np.float64)

    out = {}
    out["pos"] = np.stack([f(L["pos_x"], N), f(L["pos_y"], N)], -1).reshape(n, 2 * N)
    out["theta"] = f(L["theta"], N)
    out["vel"] = np.stack([f(L["vel_x"], N), f(L["vel_y"], N)], -1).reshape(n, 2 * N)
    out["omega"] = f(L["omega"], N)
    out["joint_acc"] = np.stack([f(L["acc_x"], J), f(L["acc_y"], J)], -1).reshape(n, 2 * J)
    out["joint_acc_ang"] = f(L["acc_ang"], J)
    lam = f(L["lambda"], 4 * NP).reshape(n, NP, 2, 2)       # [pair][point][normal, friction]
    out["lambda_n"] = lam[..., 0].reshape(n, 2 * NP)
    out["lambda_t"] = lam[..., 1].reshape(n, 2 * NP)
    ps = np.ascontiguousarray(W[:, L["pair_state"]:L["pair_state"] + (NP + 3) // 4]).view(np.uint8)[:, :NP]
    out["prev_active"] = np.stack([ps & 1, (ps >> 1) & 1], -1).reshape(n, 2 * NP).astype(np.float64)
    out["pair_count"] = ((ps & 1) + ((ps >> 1) & 1)).astype(np.float64)
    out["active"] = (I[:, L["shape_flags"]:L["shape_flags"] + N] & 1).astype(np.int64)
    return out


class Batch:
    """A batch of environments on the current torch device, stepped by the HIP library."""

    def __init__(self, caps, n_envs, params, device="cuda"):
        import torch
        self.torch = torch
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2410_23208_amd needs a GPU: there is no CPU fallback")
        self.caps = tuple(int(x) for x in caps)
        self.P, self.C, self.J, self.T = self.caps
        self.n_envs = int(n_envs)
        self.layout = get_layout(self.caps)
        self.device = torch.device(device)
        nbytes = state_bytes(self.caps, self.n_envs)
        if nbytes == 0:
            raise ValueError("unsupported capacities %r" % (self.caps,))
        self.state = torch.zeros(nbytes // 4, dtype=torch.float32, device=self.device)
        self._h = ctypes.c_void_p()
        c, p = make_caps(self.caps), make_params(params)
        _check(lib().k2d_alloc_batch(ctypes.byref(c), ctypes.byref(p), self.n_envs, self.state.data_ptr(), nbytes,
                                     ctypes.byref(self._h)), "k2d_alloc_batch")

    def set_lanes_per_env(self, lanes):
        """Lane mapping of the step kernel: 8 or 16 lanes per environment, 0 = chosen by the batch size."""
        _check(lib().k2d_set_lanes_per_env(self._h, int(lanes)), "k2d_set_lanes_per_env")

    def __del__(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().k2d_free_batch(self._h)
            self._h = None

    def _stream(self):
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def reset(self, scene_words, env_ids=None):
        """scene_words: host uint32 [n, scene_words] (pack_scenes) or a device int32/float32 tensor."""
        torch = self.torch
        if isinstance(scene_words, np.ndarray):
            scene_words = torch.from_numpy(np.ascontiguousarray(scene_words).view(np.int32)).to(self.device)
        n = scene_words.shape[0]
        ids_ptr = None
        if env_ids is not None:
            if isinstance(env_ids, np.ndarray):
                env_ids = torch.from_numpy(np.ascontiguousarray(env_ids, dtype=np.int32)).to(self.device)
            ids_ptr = env_ids.data_ptr()
        _check(lib().k2d_reset(self._h, scene_words.data_ptr(), ids_ptr, int(n), self._stream()), "k2d_reset")
        self._keep = (scene_words, env_ids)     # alive until the stream has consumed them

    def step(self, actions, n_steps=None):
        """actions: device float32 tensor [n_steps, n_envs, J+T]."""
        if n_steps is None:
            n_steps = actions.shape[0]
        assert actions.is_cuda and actions.dtype == self.torch.float32 and actions.is_contiguous()
        assert actions.numel() >= n_steps * self.n_envs * (self.J + self.T)
        _check(lib().k2d_step(self._h, actions.data_ptr(), self.n_envs, int(n_steps), self._stream()), "k2d_step")

    def step_noalloc(self, actions, n_steps=None):
        """k2d_step_noalloc: the same step, with the launch's ordering scratch inside the library."""
        if n_steps is None:
            n_steps = actions.shape[0]
        assert actions.is_cuda and actions.dtype == self.torch.float32 and actions.is_contiguous()
        assert actions.numel() >= n_steps * self.n_envs * (self.J + self.T)
        _check(lib().k2d_step_noalloc(self._h, actions.data_ptr(), self.n_envs, int(n_steps), self._stream()),
               "k2d_step_noalloc")

    def step_reset(self, actions, levels, reset_level, n_steps=None):
        """k2d_step with episodes restarted inside the launch.  levels: device int32/float32 words
        [n_levels, scene_words] (pack_scenes); reset_level: device int32 [n_steps, n_envs], -1 = no reset."""
        torch = self.torch
        if n_steps is None:
            n_steps = actions.shape[0]
        assert actions.is_cuda and actions.dtype == torch.float32 and actions.is_contiguous()
        assert actions.numel() >= n_steps * self.n_envs * (self.J + self.T)
        assert levels.is_cuda and levels.is_contiguous() and levels.element_size() == 4
        assert levels.dim() == 2 and levels.shape[1] == self.layout["scene_words"]
        assert reset_level.is_cuda and reset_level.dtype == torch.int32 and reset_level.is_contiguous()
        assert reset_level.numel() >= n_steps * self.n_envs
        _check(lib().k2d_step_reset(self._h, actions.data_ptr(), self.n_envs, int(n_steps), levels.data_ptr(),
                                    int(levels.shape[0]), reset_level.data_ptr(), self._stream()), "k2d_step_reset")
        self._keep = (levels, reset_level, actions)

    def read_obs(self):
        obs = self.torch.empty((self.n_envs, self.layout["obs_dim"]), dtype=self.torch.float32, device=self.device)
        _check(lib().k2d_read_obs(self._h, obs.data_ptr(), self._stream()), "k2d_read_obs")
        return obs

    def read_entities(self):
        """Symbolic-Entity observation: dict of device tensors (shapes, joints, joint_idx, thrusters,
        thruster_idx, masks), see k2d_read_entities in include/k2d.h."""
        torch = self.torch
        n, N, J, T = self.n_envs, self.layout["n_shapes"], self.J, self.T
        f = lambda *s: torch.empty(s, dtype=torch.float32, device=self.device)
        i = lambda *s: torch.empty(s, dtype=torch.int32, device=self.device)
        out = dict(shapes=f(n, N, 30), joints=f(n, 2 * J, 11), joint_idx=i(n, 2 * J, 2), thrusters=f(n, T, 6),
                   thruster_idx=i(n, T), masks=i(n, 4, N))
        ptr = lambda t: t.data_ptr() if t.numel() else None
        _check(lib().k2d_read_entities(self._h, out["shapes"].data_ptr(), ptr(out["joints"]), ptr(out["joint_idx"]),
                                       ptr(out["thrusters"]), ptr(out["thruster_idx"]), out["masks"].data_ptr(),
                                       self._stream()), "k2d_read_entities")
        return out

    def decode_actions(self, discrete):
        """Multi-discrete device int32 [..., J+T] -> device float32 actions of the same shape."""
        torch = self.torch
        assert discrete.is_cuda and discrete.dtype == torch.int32 and discrete.is_contiguous()
        assert discrete.shape[-1] == self.J + self.T
        out = torch.empty(discrete.shape, dtype=torch.float32, device=self.device)
        c = make_caps(self.caps)
        _check(lib().k2d_decode_actions(ctypes.byref(c), discrete.data_ptr(), out.data_ptr(),
                                        discrete.numel() // (self.J + self.T), self._stream()), "k2d_decode_actions")
        return out

    def read_outcome(self, dist, kappa=1.0, green=1, blue=2, red=3):
        """Reward and termination (Sec. 3.2).  dist: device float32 [n_envs], d_t in, d_{t+1} out (negative =
        first step of an episode).  Returns (reward float32 [n_envs], done uint8 [n_envs])."""
        torch = self.torch
        assert dist.is_cuda and dist.dtype == torch.float32 and dist.numel() == self.n_envs and dist.is_contiguous()
        reward = torch.empty(self.n_envs, dtype=torch.float32, device=self.device)
        done = torch.empty(self.n_envs, dtype=torch.uint8, device=self.device)
        rp = k2d_reward_params(float(kappa), int(green), int(blue), int(red))
        _check(lib().k2d_read_outcome(self._h, ctypes.byref(rp), dist.data_ptr(), reward.data_ptr(), done.data_ptr(),
                                      self._stream()), "k2d_read_outcome")
        return reward, done

    def read_health(self):
        """(bad uint8 [n_envs], count int32 [1]): environments whose active shapes hold a non-finite value."""
        torch = self.torch
        bad = torch.empty(self.n_envs, dtype=torch.uint8, device=self.device)
        count = torch.empty(1, dtype=torch.int32, device=self.device)
        _check(lib().k2d_read_health(self._h, bad.data_ptr(), count.data_ptr(), self._stream()), "k2d_read_health")
        return bad, count

    def read_contacts(self):
        torch = self.torch
        pc = torch.empty((self.n_envs, self.layout["n_pairs"]), dtype=torch.uint8, device=self.device)
        adj = torch.empty((self.n_envs, self.layout["n_shapes"]), dtype=torch.int32, device=self.device)
        _check(lib().k2d_read_contacts(self._h, pc.data_ptr(), adj.data_ptr(), self._stream()), "k2d_read_contacts")
        return pc, adj

    def read_state(self):
        rec = self.torch.empty((self.n_envs, self.layout["state_words"]), dtype=self.torch.int32, device=self.device)
        _check(lib().k2d_read_state(self._h, rec.data_ptr(), self._stream()), "k2d_read_state")
        return rec

    def write_state(self, rec):
        assert rec.is_cuda and rec.is_contiguous() and rec.shape == (self.n_envs, self.layout["state_words"])
        _check(lib().k2d_write_state(self._h, rec.data_ptr(), self._stream()), "k2d_write_state")

    def state_dict(self):
        """Host copy of the state as a dict of arrays (synchronises)."""
        return unpack_state(self.caps, self.read_state().cpu().numpy())
