"""Pins for the oracle's decode-and-update (Section 4.1: Adam SGD with beta1 = 0.9, beta2 = 0.999, eps = 1e-8,
applied at the decoded keys): closed forms of the two moving averages and of the step, written out with
Python's exact rationals, and the invariants that follow from the equations."""
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import ref
from paper_2112_04291_amd import workloads as W


def one_stream(dim, nnz, keep, seed, tau=128):
    rng = np.random.default_rng(seed)
    keys = np.sort(rng.choice(dim, nnz, replace=False)).astype(np.uint32)
    vals = rng.laplace(0.0, 1e-3, nnz).astype(np.float32)
    if tau > 128:                          # a wider range of magnitudes, so that the codes past 128 are in use
        vals = (vals * np.exp(rng.uniform(-10, 0, nnz))).astype(np.float32)
    rc, st = ref.compress(keys, vals, ref.params(W.solve_base(vals, keep, tau), tau, 2, 256))
    assert rc == ref.OK
    rc, k, g = ref.decompress(st)
    assert rc == ref.OK and k.size > 0
    return st, k, g


def test_first_step_from_zero_state_closed_form():
    # m0 = v0 = 0:  m1 = (1-b1) g,  v1 = (1-b2) g^2,  theta1 = theta0 - eta (1-b1) g / sqrt((1-b2) g^2 + eps)
    dim = 60_000
    st, k, g = one_stream(dim, 9_000, 0.4, 1)
    theta = np.linspace(-1, 1, dim).astype(np.float32)
    theta0 = theta.copy()
    m, v = np.zeros(dim, np.float32), np.zeros(dim, np.float32)
    rc, cnt = ref.decompress_adam(st, theta, m, v, 0.01)
    assert rc == ref.OK and cnt == k.size
    g64 = g.astype(np.float64)
    assert np.array_equal(m[k], (0.1 * g64).astype(np.float32)) or np.allclose(m[k], 0.1 * g64, rtol=2e-7, atol=0)
    assert np.allclose(v[k], 0.001 * g64 * g64, rtol=2e-7, atol=1e-45)
    # rationals on a few coordinates (exact up to the final roundings to binary32)
    for j in (0, k.size // 2, k.size - 1):
        gj = Fr(float(g[j]))
        m1 = Fr(float(np.float32(float((1 - Fr(0.9)) * gj))))
        v1 = Fr(float(np.float32(float((1 - Fr(0.999)) * gj * gj))))
        assert Fr(float(m[k[j]])) == m1 and Fr(float(v[k[j]])) == v1
        step = 0.01 * float(m1) / float(v1 + Fr(1e-8)) ** 0.5
        assert abs(float(theta[k[j]]) - (float(theta0[k[j]]) - step)) <= 1.2e-7 * max(abs(float(theta0[k[j]])), abs(step))
    untouched = np.ones(dim, bool)
    untouched[k] = False
    assert np.array_equal(theta[untouched], theta0[untouched])
    assert not m[untouched].any() and not v[untouched].any()


def test_sign_step_when_eps_is_zero():
    # eps = 0 and zero state: the step is eta (1-b1)/sqrt(1-b2) * sign(g), whatever |g|
    dim = 20_000
    st, k, g = one_stream(dim, 5_000, 0.5, 2)
    theta, m, v = (np.zeros(dim, np.float32) for _ in range(3))
    rc, _ = ref.decompress_adam(st, theta, m, v, 1e-3, 0.9, 0.999, 0.0)
    assert rc == ref.OK
    size = 1e-3 * (1 - 0.9) / (1 - 0.999) ** 0.5
    assert np.allclose(theta[k], -np.sign(g) * size, rtol=3e-7, atol=0)


def test_betas_are_not_swapped_and_second_moment_uses_the_square():
    # beta1 = 0 : m = g exactly;  beta2 = 0 : v = g^2;  then theta -= eta g / sqrt(g^2 + eps)
    dim = 20_000
    st, k, g = one_stream(dim, 5_000, 0.5, 3)
    theta = np.zeros(dim, np.float32)
    m = np.full(dim, 7.0, np.float32)
    v = np.full(dim, 9.0, np.float32)
    rc, _ = ref.decompress_adam(st, theta, m, v, 0.5, 0.0, 0.0, 1e-8)
    assert rc == ref.OK
    g64 = g.astype(np.float64)
    assert np.array_equal(m[k], g)
    assert np.array_equal(v[k], (g64 * g64).astype(np.float32))
    assert np.allclose(theta[k], -0.5 * g64 / np.sqrt((g64 * g64).astype(np.float32).astype(np.float64) + 1e-8), rtol=2e-7)
    # beta1 = 1, beta2 = 1: the averages keep their old values and the step uses them
    theta = np.zeros(dim, np.float32)
    m = np.full(dim, 0.25, np.float32)
    v = np.full(dim, 4.0, np.float32)
    rc, _ = ref.decompress_adam(st, theta, m, v, 1.0, 1.0, 1.0, 0.0)
    assert rc == ref.OK
    assert np.all(m == np.float32(0.25)) and np.all(v == np.float32(4.0))
    assert np.array_equal(theta[k], np.full(k.size, -0.125, np.float32))
    assert np.count_nonzero(theta) == k.size


def test_repeated_steps_follow_the_geometric_closed_form():
    # the same gradient t times from zero state: m_t = (1 - b1^t) g, v_t = (1 - b2^t) g^2
    dim = 5_000
    st, k, g = one_stream(dim, 2_000, 0.5, 4)
    theta, m, v = (np.zeros(dim, np.float32) for _ in range(3))
    g64 = g.astype(np.float64)
    walked = np.zeros(k.size)
    for t in range(1, 13):
        rc, _ = ref.decompress_adam(st, theta, m, v, 1e-2)
        assert rc == ref.OK
        assert np.allclose(m[k], (1 - 0.9 ** t) * g64, rtol=2e-6)
        assert np.allclose(v[k], (1 - 0.999 ** t) * g64 * g64, rtol=2e-6)
        walked += 1e-2 * (1 - 0.9 ** t) * g64 / np.sqrt((1 - 0.999 ** t) * g64 * g64 + 1e-8)
    assert np.allclose(theta[k], -walked, rtol=1e-5)


def test_adam_rejects_keys_beyond_the_arrays_and_corrupt_streams():
    st, k, g = one_stream(10_000, 2_000, 0.5, 5)
    top = int(k.max())
    a = [np.zeros(top, np.float32) for _ in range(3)]
    assert ref.decompress_adam(st, *a, 0.1)[0] == ref.ERR_BUFFER_TOO_SMALL
    a = [np.zeros(top + 1, np.float32) for _ in range(3)]
    assert ref.decompress_adam(st, *a, 0.1)[0] == ref.OK
    bad = st.copy()
    bad[4] ^= 0x7
    a = [np.zeros(top + 1, np.float32) for _ in range(3)]
    assert ref.decompress_adam(bad, *a, 0.1) == (ref.ERR_CORRUPT_STREAM, 0)
    assert not any(x.any() for x in a)
