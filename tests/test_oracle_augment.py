"""Pins for the oracle's random augmentation and inverse transform (Transformations
section: a random rotation and a random translation of at most a given distance per example).

The paper names neither generator nor distribution; the oracle's reading is Philox4x32-10
counters, a Haar-uniform rotation (Shoemake) and a per-axis uniform translation.  These tests
pin the generator to its published known answers and the draws to what the distributions fix."""
import os

import numpy as np
import pytest
from scipy import stats

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden",
                      "philox4x32_10_known_answers.txt")


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(v, 16) for v in r]
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(v) for v in out] == w[6:10]


def test_philox_is_a_bijection_of_the_counter_on_a_sample():
    # distinct counters give distinct blocks; one flipped input bit changes about half the bits
    key = [123, 456]
    seen = set()
    for c in range(2000):
        seen.add(tuple(int(v) for v in oracle.philox4x32_10([c, 0, 0, 0], key)))
    assert len(seen) == 2000
    a = oracle.philox4x32_10([7, 0, 0, 0], key)
    flips = []
    for word in range(4):
        for bit in (0, 13, 31):
            c = [7, 0, 0, 0]
            c[word] ^= 1 << bit
            b = oracle.philox4x32_10(c, key)
            flips.append(sum(bin(int(x) ^ int(y)).count("1") for x, y in zip(a, b)))
    assert 50 < np.mean(flips) < 78          # 64 of 128 expected


def test_switches_and_unit_norm():
    q, t = oracle.draw_transforms(1, 0, 64, random_rotation=False, max_translation=0.0)
    assert np.array_equal(q, np.tile(np.array([1, 0, 0, 0], np.float32), (64, 1)))
    assert np.array_equal(t, np.zeros((64, 3), np.float32))
    q, t = oracle.draw_transforms(1, 0, 4096, True, 2.0)
    assert np.allclose((q.astype(np.float64) ** 2).sum(1), 1.0, atol=3e-7)
    assert np.all(np.abs(t) <= 2.0)
    # the rotation does not depend on the translation switch, and the other way round
    q2, t2 = oracle.draw_transforms(1, 0, 4096, True, 0.0)
    q3, t3 = oracle.draw_transforms(1, 0, 4096, False, 2.0)
    assert np.array_equal(q, q2) and np.array_equal(t, t3)
    # translation scales with the maximum distance
    _, t4 = oracle.draw_transforms(1, 0, 4096, True, 1.0)
    assert np.allclose(t4 * 2.0, t, atol=3e-7)


def test_draw_depends_on_seed_draw_and_example_only():
    q, t = oracle.draw_transforms(99, 5, 50, True, 2.0)
    q1, t1 = oracle.draw_transforms(99, 5, 7, True, 2.0)
    assert np.array_equal(q[:7], q1) and np.array_equal(t[:7], t1)      # not on B
    for seed, draw in [(98, 5), (99, 6), (99 + 2 ** 32, 5), (99, 5 + 2 ** 32)]:
        q2, t2 = oracle.draw_transforms(seed, draw, 50, True, 2.0)
        assert not np.any(np.all(q2 == q, axis=1))
        assert not np.any(np.all(t2 == t, axis=1))
    assert len({tuple(r) for r in q}) == 50 and len({tuple(r) for r in t}) == 50


def _matrices(q):
    return np.stack([oracle.quat_to_matrix(r) for r in q])


def test_rotations_are_haar_uniform():
    n = 40000
    q, _ = oracle.draw_transforms(2024, 3, n, True, 0.0)
    R = _matrices(q)
    # (a) every entry of a Haar rotation has mean 0 and variance 1/3
    assert np.all(np.abs(R.mean(0)) < 5 * np.sqrt(1 / 3 / n))
    assert np.allclose((R ** 2).mean(0), 1 / 3, atol=0.01)
    # (b) the image of each basis vector is uniform on the sphere: every coordinate U(-1,1)
    for col in range(3):
        for row in range(3):
            assert stats.kstest(R[:, row, col], stats.uniform(-1, 2).cdf).pvalue > 1e-4
    # (c) rotation angle: density (1 - cos a)/pi on [0, pi], CDF (a - sin a)/pi
    ang = np.arccos(np.clip((np.trace(R, axis1=1, axis2=2) - 1) / 2, -1, 1))
    assert stats.kstest(ang, lambda a: (a - np.sin(a)) / np.pi).pvalue > 1e-4
    # (d) the character of the 3-d representation is orthonormal: E[tr] = 0, E[tr^2] = 1
    tr = np.trace(R, axis1=1, axis2=2)
    assert abs(tr.mean()) < 5 / np.sqrt(n)
    assert abs((tr ** 2).mean() - 1.0) < 0.03
    # (e) a uniform unit quaternion: each component has E[q_i^2] = 1/4 and q ~ -q
    assert np.allclose((q.astype(np.float64) ** 2).mean(0), 0.25, atol=0.005)
    assert np.all(np.abs(q.mean(0)) < 5 * 0.5 / np.sqrt(n))
    # (f) invariance: composing with a fixed rotation leaves the angle law unchanged
    F = oracle.quat_to_matrix(np.array([0.3, -0.5, 0.7, 0.2], np.float32))
    tr2 = np.trace(F @ R, axis1=1, axis2=2)
    ang2 = np.arccos(np.clip((tr2 - 1) / 2, -1, 1))
    assert stats.kstest(ang2, lambda a: (a - np.sin(a)) / np.pi).pvalue > 1e-4


def test_translations_are_uniform_in_the_box_and_axes_independent():
    n = 40000
    T = 2.0
    _, t = oracle.draw_transforms(7, 11, n, False, T)
    for m in range(3):
        assert stats.kstest(t[:, m], stats.uniform(-T, 2 * T).cdf).pvalue > 1e-4
    assert np.all(np.abs(t.mean(0)) < 5 * T / np.sqrt(3 * n))
    assert np.allclose(t.var(0), T * T / 3, rtol=0.03)
    c = np.corrcoef(t.T)
    assert np.all(np.abs(c - np.eye(3)) < 5 / np.sqrt(n))
    assert np.abs(t).max() > 0.999 * T and np.all(np.abs(t) <= T)       # reaches the faces
    # successive examples are uncorrelated too
    assert abs(np.corrcoef(t[:-1, 0], t[1:, 0])[0, 1]) < 5 / np.sqrt(n)


def test_first_draw_by_hand():
    """One example recomputed here from the generator's words (checks the word-to-angle wiring)."""
    seed, draw, b = 0x123456789ABCDEF, 0x1_0000_0002, 3
    key = [seed & 0xFFFFFFFF, seed >> 32]
    w = [int(v) for v in oracle.philox4x32_10([b, draw & 0xFFFFFFFF, draw >> 32, 0], key)]
    u = [(x + 0.5) / 2 ** 32 for x in w]
    s1, s2 = np.sqrt(1 - u[0]), np.sqrt(u[0])
    want_q = np.array([s2 * np.cos(2 * np.pi * u[2]), s1 * np.sin(2 * np.pi * u[1]),
                       s1 * np.cos(2 * np.pi * u[1]), s2 * np.sin(2 * np.pi * u[2])])
    w = [int(v) for v in oracle.philox4x32_10([b, draw & 0xFFFFFFFF, draw >> 32, 1], key)]
    want_t = np.array([1.5 * (2 * (x + 0.5) / 2 ** 32 - 1) for x in w[:3]])
    q, t = oracle.draw_transforms(seed, draw, b + 1, True, 1.5)
    assert np.allclose(q[b], want_q, atol=6e-8) and np.allclose(t[b], want_t, atol=1.2e-7)


def test_inverse_transform_undoes_forward():
    rng = np.random.default_rng(3)
    B, N = 5, 40
    x = rng.uniform(-20, 20, (B, N, 3)).astype(np.float32)
    c = rng.uniform(-5, 5, (B, 3)).astype(np.float32)
    q, t = oracle.draw_transforms(5, 0, B, True, 2.0)
    y = oracle.transform(x, c, q, t, as_float=False)
    # feed the float-rounded forward result back: the inverse returns x within rounding of y
    back = oracle.transform_inverse(y.astype(np.float32), c, q, t, as_float=False)
    assert np.abs(back - x).max() < 4e-6
    # distances and the centre are preserved, and the inverse matches the transposed matrix
    for b in range(B):
        R = oracle.quat_to_matrix(q[b])
        want = (y[b] - t[b].astype(float) - c[b].astype(float)) @ R + c[b].astype(float)
        got = oracle.transform_inverse(y[b:b + 1].astype(np.float32), c[b:b + 1], q[b:b + 1],
                                       t[b:b + 1], as_float=False)[0]
        assert np.abs(got - want).max() < 4e-6
    # vectors (gradients): with no centre and no translation the inverse is R^T v
    v = rng.standard_normal((B, N, 3)).astype(np.float32)
    gv = oracle.transform_inverse(v, None, q, None, as_float=False)
    for b in range(B):
        assert np.allclose(gv[b], v[b].astype(float) @ oracle.quat_to_matrix(q[b]), atol=1e-14)
    # all-NULL arguments: identity
    assert np.array_equal(oracle.transform_inverse(x), x)
