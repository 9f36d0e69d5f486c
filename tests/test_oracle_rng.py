"""Pins for the oracle's random stream: Philox4x32-10 against published
known-answer vectors, the uniform maps by exact integer inversion, and
Box-Muller by inverting it with independent library routines plus
distribution tests against scipy's normal law."""
import os

import numpy as np
import pytest
from scipy import stats

from oracle import perturbation as P
from oracle.philox import philox4x32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox_kat.txt")


def _read_kat():
    vec, nth = [], []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "nth":
            nth.append(tuple(int(x) for x in f[1:]))
        else:
            v = [int(x, 16) for x in f]
            vec.append((v[0:4], v[4:6], v[6:10]))
    return vec, nth


def test_philox_known_answers():
    vec, _ = _read_kat()
    assert len(vec) == 3
    for ctr, key, out in vec:
        assert philox4x32(ctr, key).tolist() == out


def test_philox_cxx26_10000th_value():
    _, nth = _read_kat()
    (n, k0, k1, val), = nth
    calls = (n + 3) // 4
    ctr = np.zeros((calls, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(calls)
    out = philox4x32(ctr, [k0, k1]).reshape(-1)
    assert int(out[n - 1]) == val


def test_philox_vectorised_equals_scalar_calls():
    rng = np.random.default_rng(0)
    ctr = rng.integers(0, 2 ** 32, size=(64, 4), dtype=np.uint64)
    key = rng.integers(0, 2 ** 32, size=(2,), dtype=np.uint64)
    out = philox4x32(ctr, key)
    for i in range(64):
        assert np.array_equal(out[i], philox4x32(ctr[i], key))
    # a one-bit change of the counter or key changes about half of the 128 output bits
    flips = []
    for word in range(4):
        c2 = ctr.copy()
        c2[:, word] ^= np.uint64(1)
        x = philox4x32(c2, key) ^ out
        flips.append(np.unpackbits(x.view(np.uint8)).mean())
    assert all(0.45 < f < 0.55 for f in flips)


def test_counter_layout():
    c = P.counters(np.array([5, (7 << 32) | 9], dtype=np.uint64), tensor_id=11, stream=1, step=3)
    assert c[0].tolist() == [5, 0, 11 | (1 << 31), 3]
    assert c[1].tolist() == [9, 7, 11 | (1 << 31), 3]
    assert P.key_of((2 << 32) | 42).tolist() == [42, 2]
    # the two streams, different tensors, steps and seeds are different streams
    e = np.arange(64)
    base = P.gauss_at(42, 0, 1, 0, e)
    for other in (P.gauss_at(42, 0, 1, 1, e), P.gauss_at(42, 1, 1, 0, e), P.gauss_at(42, 0, 2, 0, e),
                  P.gauss_at(43, 0, 1, 0, e)):
        assert not np.any(other == base)


def test_uniform_maps_are_exact_and_invertible():
    rng = np.random.default_rng(1)
    w = rng.integers(0, 2 ** 32, size=100000, dtype=np.uint64)
    w[:4] = [0, 2 ** 32 - 1, 511, 512]
    u, v = P.uniforms32(w, w)
    # exactly representable in fp32, strictly inside (0,1) / [0,1)
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)
    assert np.array_equal(v.astype(np.float32).astype(np.float64), v)
    assert u.min() > 0 and u.max() < 1 and v.min() >= 0 and v.max() < 1
    assert np.array_equal((u * 2 ** 23 - 0.5).astype(np.uint64), w >> np.uint64(9))
    assert np.array_equal((v * 2 ** 24).astype(np.uint64), w >> np.uint64(8))
    h = np.arange(65536, dtype=np.uint64)
    u16, v16 = P.uniforms16(h, h)
    assert u16.min() == 2.0 ** -17 and u16.max() == 1 - 2.0 ** -17 and v16.max() == 1 - 2.0 ** -16
    assert np.array_equal((u16 * 65536 - 0.5).astype(np.uint64), h)


@pytest.mark.parametrize("bits", [32, 16])
def test_box_muller_inverts_to_its_uniforms(bits):
    """rho^2 = -2 ln u and the polar angle is 2 pi v: recover both uniforms of
    every pair from the Gaussians with hypot/arctan2/exp."""
    n = 1 << 16
    e = np.arange(n, dtype=np.uint64)
    g = P.gauss_at(7, 3, 5, 0, e, bits).astype(np.float64)
    per = 4 if bits == 32 else 8
    w = philox4x32(P.counters(np.arange(n // per, dtype=np.uint64), 5, 0, 3), P.key_of(7)).astype(np.uint64)
    if bits == 32:
        u, v = P.uniforms32(w[:, [0, 2]].reshape(-1), w[:, [1, 3]].reshape(-1))
    else:
        w = w.reshape(-1)
        u, v = P.uniforms16(w & np.uint64(0xFFFF), w >> np.uint64(16))
    x, y = g[0::2], g[1::2]
    u_back = np.exp(-0.5 * (x * x + y * y))
    v_back = np.mod(np.arctan2(y, x) / (2 * np.pi), 1.0)
    assert np.allclose(u_back, u, rtol=2e-6, atol=0)
    dv = np.abs(v_back - v)
    dv = np.minimum(dv, 1 - dv)
    # the angle is only resolved to ~ulp(g)/rho; pairs with tiny rho are excluded
    big = np.hypot(x, y) > 0.05
    assert np.all(dv[big] < 2e-6)


def test_exact_quadrant_values():
    c, s = P.cos_sin_2pi(np.array([0.0, 0.25, 0.5, 0.75, 0.125]))
    assert c[:4].tolist() == [1.0, 0.0, -1.0, 0.0] and s[:4].tolist() == [0.0, 1.0, 0.0, -1.0]
    assert np.isclose(c[4], np.sqrt(0.5), rtol=1e-15) and np.isclose(s[4], np.sqrt(0.5), rtol=1e-15)
    v = np.arange(0, 1 << 12) / float(1 << 12)
    c, s = P.cos_sin_2pi(v)
    assert np.allclose(c, np.cos(2 * np.pi * v), atol=1e-15) and np.allclose(s, np.sin(2 * np.pi * v), atol=1e-15)


@pytest.mark.parametrize("bits,bound", [(32, 5.7682), (16, 4.8551)])
def test_gaussian_distribution(bits, bound):
    n = 1 << 22
    g = P.gauss_field(1234, 0, 9, 0, 1, n, bits).reshape(-1).astype(np.float64)
    assert np.all(np.isfinite(g)) and np.abs(g).max() <= bound
    assert abs(g.mean()) < 2e-3
    assert abs(g.var() - 1) < 3e-3
    assert abs(stats.kurtosis(g, fisher=False) - 3) < 0.02
    assert abs(stats.skew(g)) < 0.01
    ks = stats.kstest(g[: 1 << 18], "norm")
    assert ks.pvalue > 1e-3
    # even (cos) and odd (sin) lanes are uncorrelated standard normals
    assert abs(np.mean(g[0::2] * g[1::2])) < 3e-3


def test_largest_possible_values():
    # u at its minimum gives the largest radius: sqrt(-2 ln 2^-24) resp. sqrt(-2 ln 2^-17)
    x, _ = P.box_muller(*P.uniforms32(np.uint64(0), np.uint64(0)))
    assert np.isclose(x, np.sqrt(2 * 24 * np.log(2)), rtol=1e-7)
    x, _ = P.box_muller(*P.uniforms16(np.uint64(0), np.uint64(0)))
    assert np.isclose(x, np.sqrt(2 * 17 * np.log(2)), rtol=1e-7)


def test_gauss_field_matches_gauss_at():
    f = P.gauss_field(5, 2, 3, 1, 37, 53, 32)
    idx = np.array([0, 1, 2, 3, 4, 52, 53, 1000, 37 * 53 - 1])
    assert np.array_equal(f.reshape(-1)[idx], P.gauss_at(5, 2, 3, 1, idx, 32))
    f16 = P.gauss_field(5, 2, 3, 1, 37, 53, 16)
    assert np.array_equal(f16.reshape(-1)[idx], P.gauss_at(5, 2, 3, 1, idx, 16))
