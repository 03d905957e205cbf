"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE, not the product).

Only tests, the smoke check and the CPU-baseline leg of the benchmark import this module.  It builds
`libk2d_oracle.so` from `k2d_oracle.cpp` with g++ on demand and exposes the batch object, the stand-alone
manifold routines and the tournament order of the shape pairs.  It imports nothing from the GPU package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "k2d_oracle.cpp")
_LIB = os.path.join(_HERE, "libk2d_oracle.so")

PARAM_ORDER = ["dt", "gravity_y", "n_substeps", "n_iters", "warm_start", "alpha", "beta", "gamma", "rho",
               "slop", "restitution_threshold", "clip_thruster_01", "joint_alpha", "joint_beta", "tie_eps",
               "order_mode", "batch_size", "sweep_order"]

# Fields a scene description may carry (see k2d_oracle.cpp, Batch::find).
SCENE_FIELDS = ["pos", "theta", "vel", "omega", "inv_mass", "inv_inertia", "friction", "restitution", "density",
                "role", "active", "n_verts", "verts", "radius",
                "joint_active", "joint_a", "joint_b", "joint_fixed", "joint_motor_on", "joint_anchor_a",
                "joint_anchor_b", "joint_theta_f", "joint_motor_speed", "joint_motor_power",
                "thruster_active", "thruster_body", "thruster_pos", "thruster_angle", "thruster_power"]
OPTIONAL_FIELDS = ["joint_limited", "joint_limit_lo", "joint_limit_hi"]     # absent = no joint is limited
ACC_FIELDS = ["joint_acc", "joint_acc_ang", "lambda_n", "lambda_t", "prev_active"]


# K2D_ORACLE_SANITIZE=1 builds and loads a second library, compiled with AddressSanitizer and
# UndefinedBehaviorSanitizer (host code only), to run the CPU test suite under:
#   LD_PRELOAD="$(g++ -print-file-name=libasan.so):$LD_PRELOAD" ASAN_OPTIONS=detect_leaks=0 \
#   K2D_ORACLE_SANITIZE=1 python -m pytest tests -q -m "not gpu"
SANITIZE = os.environ.get("K2D_ORACLE_SANITIZE", "") not in ("", "0")
if SANITIZE:
    _LIB = os.path.join(_HERE, "libk2d_oracle_san.so")
# K2D_ORACLE_SOURCE=<file> builds and loads that source instead (the library is put beside it): how
# oracle/mutation_check.py runs the pins against copies of the oracle with a mistake planted in each.
if os.environ.get("K2D_ORACLE_SOURCE"):
    _SRC = os.environ["K2D_ORACLE_SOURCE"]
    _LIB = _SRC + ".so"


def build(force=False):
    """Compile the oracle with plain g++ (-O2, no contraction of a*b+c into fma)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
               "-o", _LIB, _SRC]
        if SANITIZE:
            cmd[1:2] = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                        "-fno-omit-frame-pointer"]
        try:   # std::fma as one instruction where the host has it (a libm call gives the same bits, slowly)
            if " fma " in open("/proc/cpuinfo").read():
                cmd.insert(1, "-mfma")
        except OSError:
            pass
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        L.ko_create.restype = ctypes.c_void_p
        L.ko_create.argtypes = [ctypes.c_int] * 6
        L.ko_destroy.argtypes = [ctypes.c_void_p]
        L.ko_set_params.argtypes = [ctypes.c_void_p, dp, ctypes.c_int]
        L.ko_field_size.restype = ctypes.c_long
        L.ko_field_size.argtypes = [ctypes.c_void_p, ctypes.c_char_p]
        L.ko_set.argtypes = [ctypes.c_void_p, ctypes.c_char_p, dp, ctypes.c_long]
        L.ko_set_rows.argtypes = [ctypes.c_void_p, ctypes.c_char_p, ip, ctypes.c_long, dp, ctypes.c_long]
        L.ko_get.argtypes = [ctypes.c_void_p, ctypes.c_char_p, dp, ctypes.c_long]
        L.ko_step.argtypes = [ctypes.c_void_p, dp, ctypes.c_int, ctypes.c_int]
        L.ko_obs_dim.argtypes = [ctypes.c_void_p]
        L.ko_obs.argtypes = [ctypes.c_void_p, dp]
        L.ko_schedule.argtypes = [ctypes.c_int, ip, ip, ip]
        L.ko_math.argtypes = [ctypes.c_int, dp, ctypes.c_long, dp, dp, dp]
        L.ko_manifold_cc.argtypes = [ctypes.c_int, dp, ctypes.c_double, dp, ctypes.c_double, dp]
        L.ko_manifold_pc.argtypes = [ctypes.c_int, ctypes.c_int, dp, dp, ctypes.c_double, dp]
        L.ko_manifold_pp.argtypes = [ctypes.c_int, ctypes.c_int, dp, ctypes.c_int, dp, ctypes.c_double, dp]
        _lib = L
    return _lib


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


class Oracle:
    """A batch of `n_envs` scenes of capacity (P polygons, C circles, J joints, T thrusters)."""

    def __init__(self, caps, n_envs, params, dtype="f32"):
        self.P, self.C, self.J, self.T = [int(x) for x in caps]
        self.N = self.P + self.C
        self.NP = self.N * (self.N - 1) // 2
        self.n_envs = int(n_envs)
        self.dtype = dtype
        self._h = lib().ko_create(self.P, self.C, self.J, self.T, self.n_envs, 1 if dtype == "f64" else 0)
        if not self._h:
            raise ValueError("ko_create refused the capacities")
        self.set_params(params)

    def __del__(self):
        if getattr(self, "_h", None):
            lib().ko_destroy(self._h)
            self._h = None

    def set_params(self, params):
        p = dict(params)
        p.setdefault("order_mode", 0)
        p.setdefault("batch_size", 0)
        p.setdefault("sweep_order", 0)
        v = _f64([p[k] for k in PARAM_ORDER])
        rc = lib().ko_set_params(self._h, _dptr(v), len(v))
        if rc:
            raise ValueError("ko_set_params rc=%d" % rc)
        self.params = p

    def field_size(self, name):
        n = lib().ko_field_size(self._h, name.encode())
        if n < 0:
            raise KeyError(name)
        return n

    def set(self, name, value, env_ids=None):
        n = self.field_size(name)
        v = _f64(value).reshape(-1)
        if env_ids is None:
            rc = lib().ko_set(self._h, name.encode(), _dptr(v), v.size)
        else:
            ids = np.ascontiguousarray(np.asarray(env_ids, dtype=np.int32))
            rc = lib().ko_set_rows(self._h, name.encode(), ids.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                                   ids.size, _dptr(v), v.size)
        if rc:
            raise ValueError("ko_set(%s) rc=%d (expected %d per env)" % (name, rc, n))

    def get(self, name):
        n = self.field_size(name)
        out = np.empty((self.n_envs, n), dtype=np.float64)
        rc = lib().ko_get(self._h, name.encode(), _dptr(out), out.size)
        if rc:
            raise ValueError("ko_get(%s) rc=%d" % (name, rc))
        return out

    def load_scene(self, scene, env_ids=None, zero_acc=True):
        """Write a scene description (dict of per-env arrays); accumulators start at zero."""
        rows = self.n_envs if env_ids is None else len(env_ids)
        for f in SCENE_FIELDS:
            self.set(f, scene[f], env_ids)
        for f in OPTIONAL_FIELDS:
            self.set(f, scene[f] if f in scene else np.zeros((rows, self.field_size(f))), env_ids)
        for f in ACC_FIELDS:
            if f in scene and not zero_acc:
                self.set(f, scene[f], env_ids)
            else:
                self.set(f, np.zeros((rows, self.field_size(f))), env_ids)
        # a fresh episode has had no substep yet: no collisions to report
        self.set("pair_active", np.zeros((rows, self.field_size("pair_active"))), env_ids)

    def step(self, actions, n_steps=None, n_threads=1):
        """actions: [n_steps, n_envs, J+T]."""
        a = _f64(actions)
        if a.ndim == 2:
            a = a[None]
        if n_steps is None:
            n_steps = a.shape[0]
        assert a.shape == (n_steps, self.n_envs, self.J + self.T), a.shape
        rc = lib().ko_step(self._h, _dptr(a), int(n_steps), int(n_threads))
        if rc:
            raise ValueError("ko_step rc=%d" % rc)

    def obs(self):
        d = lib().ko_obs_dim(self._h)
        out = np.empty((self.n_envs, d), dtype=np.float64)
        lib().ko_obs(self._h, _dptr(out))
        return out

    def state(self):
        """Dynamic state + accumulators + last narrowphase result, as a dict of arrays."""
        names = ["pos", "theta", "vel", "omega", "joint_acc", "joint_acc_ang", "lambda_n", "lambda_t",
                 "prev_active", "pair_count", "shape_adj", "min_margin"]
        return {k: self.get(k) for k in names}


def schedule(N):
    """Canonical visiting order of the shape pairs: arrays a, b, round."""
    cap = N * (N - 1) // 2
    a = np.zeros(cap, dtype=np.int32)
    b = np.zeros(cap, dtype=np.int32)
    r = np.zeros(cap, dtype=np.int32)
    ip = ctypes.POINTER(ctypes.c_int)
    n = lib().ko_schedule(N, a.ctypes.data_as(ip), b.ctypes.data_as(ip), r.ctypes.data_as(ip))
    return a[:n], b[:n], r[:n]


def _unpack(out):
    return {"normal": out[0:2].copy(), "pos": np.array([out[2:4], out[6:8]]), "pen": np.array([out[4], out[8]]),
            "valid": np.array([int(out[5]), int(out[9])]), "margin": out[10]}


def manifold_cc(pa, ra, pb, rb, dtype="f64"):
    out = np.zeros(11)
    lib().ko_manifold_cc(int(dtype == "f64"), _dptr(_f64(pa)), float(ra), _dptr(_f64(pb)), float(rb), _dptr(out))
    return _unpack(out)


def manifold_pc(poly_xy, c, r, dtype="f64"):
    xy = _f64(poly_xy).reshape(-1, 2)
    out = np.zeros(11)
    lib().ko_manifold_pc(int(dtype == "f64"), xy.shape[0], _dptr(xy), _dptr(_f64(c)), float(r), _dptr(out))
    return _unpack(out)


def manifold_pp(poly_a, poly_b, tie_eps=1e-3, dtype="f64"):
    a = _f64(poly_a).reshape(-1, 2)
    b = _f64(poly_b).reshape(-1, 2)
    out = np.zeros(11)
    lib().ko_manifold_pp(int(dtype == "f64"), a.shape[0], _dptr(a), b.shape[0], _dptr(b), float(tie_eps), _dptr(out))
    return _unpack(out)


def math_fns(x, dtype="f32"):
    """The engine's (sin, cos, tanh) evaluated elementwise in the given precision."""
    x = _f64(x).reshape(-1)
    sn, cs, th = np.empty_like(x), np.empty_like(x), np.empty_like(x)
    lib().ko_math(int(dtype == "f64"), _dptr(x), x.size, _dptr(sn), _dptr(cs), _dptr(th))
    return sn, cs, th
