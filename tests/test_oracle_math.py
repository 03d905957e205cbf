"""Pin of the oracle's fp32 sin / cos / tanh (fixed operation sequences) against libm in double."""
import numpy as np

from oracle import k2d_oracle as ko


def test_sincos_against_libm():
    for lo, hi in ((-7.0, 7.0), (-400.0, 400.0), (-3000.0, 3000.0)):
        x = np.linspace(lo, hi, 400001).astype(np.float32).astype(np.float64)
        sn, cs, _ = ko.math_fns(x, "f32")
        assert np.abs(sn - np.sin(x)).max() < 1.5e-7
        assert np.abs(cs - np.cos(x)).max() < 1.5e-7
        assert np.abs(sn * sn + cs * cs - 1).max() < 4e-7
    sn, cs, _ = ko.math_fns([0.0], "f32")
    assert sn[0] == 0.0 and cs[0] == 1.0


def test_tanh_against_libm():
    x = np.concatenate([np.linspace(-12, 12, 400001), np.linspace(-0.6, 0.6, 100001), [50.0, -50.0, 1e6]])
    x = x.astype(np.float32).astype(np.float64)
    _, _, th = ko.math_fns(x, "f32")
    ref = np.tanh(x)
    assert np.abs(th - ref).max() < 1.5e-7
    nz = ref != 0
    assert np.abs((th[nz] - ref[nz]) / ref[nz]).max() < 3e-7
    assert (np.abs(th) <= 1.0).all() and (np.sign(th) == np.sign(x)).all()
    # odd, monotone non-decreasing
    xs = np.sort(x)
    assert (np.diff(ko.math_fns(xs, "f32")[2]) >= -1.2e-7).all()


def test_double_instance_is_a_double_precision_library_routine():
    x = np.linspace(-5, 5, 1001)
    sn, cs, th = ko.math_fns(x, "f64")
    for got, ref in ((sn, np.sin(x)), (cs, np.cos(x)), (th, np.tanh(x))):
        assert np.abs(got - ref).max() < 1e-15
