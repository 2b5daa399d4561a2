"""The library's angle-bin rule (csrc/pq_angle.hpp), built for the CPU, against the oracle:
random pairs, every axis / diagonal tie, signed zeros, subnormals, fp16-grid values."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from oracle import polar

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def host_lib(tmp_path_factory):
    out = tmp_path_factory.mktemp("anglehost") / "libangle_host.so"
    src = os.path.join(ROOT, "tests", "host", "angle_bin_host.cpp")
    inc = os.path.join(ROOT, "paper_2502_00527_amd", "csrc")
    subprocess.run(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-shared", "-fPIC", "-I", inc, src,
                    "-o", str(out)], check=True)
    lib = ctypes.CDLL(str(out))
    lib.angle_bins_host.restype = ctypes.c_int
    lib.angle_bins_host.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]
    lib.angle_bins_interior_host.restype = ctypes.c_int
    lib.angle_bins_interior_host.argtypes = lib.angle_bins_host.argtypes
    lib.round_to_half_host.restype = None
    lib.round_to_half_host.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    return lib


def _host_bins(lib, x, y, t):
    x = np.ascontiguousarray(x, np.float32)
    y = np.ascontiguousarray(y, np.float32)
    out = np.empty(x.size, np.int32)
    assert lib.angle_bins_host(x.ctypes.data, y.ctypes.data, x.size, t, out.ctypes.data) == 0
    return out


def _inputs():
    rng = np.random.default_rng(77)
    xs, ys = [], []
    # random float32 and fp16-grid pairs (fp16 pairs hit |x| == |y| about 5e-4 of the time)
    xs.append(rng.standard_normal(200000).astype(np.float32)); ys.append(rng.standard_normal(200000).astype(np.float32))
    h = rng.standard_normal((2, 400000)).astype(np.float16).astype(np.float32)
    xs.append(h[0]); ys.append(h[1])
    # exact ties at many magnitudes, with both signs of zero
    mags = np.array([2.0 ** e for e in range(-24, 16, 3)] + [3.0, 0.1, 65504.0, 5.9604645e-08], np.float32)
    dirs = [(1, 0), (1, 1), (0, 1), (-1, 1), (-1, 0), (-1, -1), (0, -1), (1, -1), (0, 0),
            (-1, -0.0), (1, -0.0), (-0.0, 1), (-0.0, -1), (-0.0, -0.0), (-0.0, 0.0), (0.0, -0.0)]
    for dx, dy in dirs:
        xs.append(np.float32(dx) * mags); ys.append(np.float32(dy) * mags)
    # coarse integer lattice: many near-edge and on-edge directions
    g = np.arange(-12, 13, dtype=np.float32)
    gx, gy = np.meshgrid(g, g)
    xs.append(gx.ravel()); ys.append(gy.ravel())
    return np.concatenate(xs), np.concatenate(ys)


@pytest.mark.parametrize("t", [2, 3, 4, 5])
def test_angle_rule_matches_oracle(host_lib, t):
    x, y = _inputs()
    want, edge = polar.angle_bin(x, y, t)
    got = _host_bins(host_lib, x, y, t)
    bad = got != want
    # the two float64 evaluations may differ only within ~1e-15 rad of an irrational edge
    assert not np.any(bad & (edge > 1e-12)), (x[bad][:5], y[bad][:5], got[bad][:5], want[bad][:5])
    assert bad.sum() <= 2


@pytest.mark.parametrize("t", [2, 3, 4, 5])
def test_interior_rule_agrees_with_the_full_rule(host_lib, t):
    """The encoder's short rule for pairs strictly inside an octant gives the full rule's bin, and
    declines exactly the pairs on an axis, a diagonal or the origin."""
    x, y = _inputs()
    x = np.ascontiguousarray(x, np.float32)
    y = np.ascontiguousarray(y, np.float32)
    full = _host_bins(host_lib, x, y, t)
    got = np.empty(x.size, np.int32)
    assert host_lib.angle_bins_interior_host(x.ctypes.data, y.ctypes.data, x.size, t, got.ctypes.data) == 0
    on_boundary = (x == 0) | (y == 0) | (np.abs(x) == np.abs(y))
    assert np.array_equal(got == -1, on_boundary)
    assert on_boundary.sum() > 300 and (~on_boundary).sum() > 500000
    want, edge = polar.angle_bin(x, y, t)
    inside = ~on_boundary
    bad = inside & (got != full)
    assert not np.any(bad & (edge > 1e-12))
    assert bad.sum() <= 2
    bad = inside & (got != want)
    assert not np.any(bad & (edge > 1e-12)) and bad.sum() <= 2


def test_round_to_half_is_one_nearest_even_rounding(host_lib):
    """float64 -> fp16 in one step: NumPy's float64 -> float16 cast is the reference (a detour
    through float32 would round twice and differ on some of these inputs)."""
    rng = np.random.default_rng(78)
    v = np.concatenate([
        rng.uniform(-np.pi, np.pi, 200000), rng.uniform(-0.5, 0.5, 100000), rng.standard_normal(100000) * 1e-3,
        rng.standard_normal(50000) * 1e-6, rng.standard_normal(20000) * 1e-8, [0.0, -0.0, 6.0e-8, 2.0 ** -25, 3 * 2.0 ** -25],
        # exact ties between neighbouring fp16 values, and values a float32 detour gets wrong
        (np.arange(2048, 4096)[::7] + 0.5) * 2.0 ** -10, (np.arange(2048, 4096)[::7] + 0.5) * 2.0 ** -10 * (1 + 2.0 ** -40),
        (np.arange(1, 1024)[::5] + 0.5) * 2.0 ** -24])
    out = np.empty_like(v)
    host_lib.round_to_half_host(v.ctypes.data, v.size, out.ctypes.data)
    want = v.astype(np.float16).astype(np.float64)
    assert np.array_equal(out, want)
    twice = v.astype(np.float32).astype(np.float16).astype(np.float64)
    assert (twice != want).any()
