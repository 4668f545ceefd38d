"""Pins for the oracle's transform: x' = R(q)(x - c) + c + t (Transformations section)."""
import os

import numpy as np
import pytest
from scipy.spatial.transform import Rotation

import oracle

from test_oracle_density import read_golden


def test_identity_quaternion_from_paper_is_a_no_op():
    q = np.array([float(v) for v in read_golden()["identity_quaternion"].split()], np.float32)
    assert np.array_equal(oracle.quat_to_matrix(q), np.eye(3))
    rng = np.random.default_rng(0)
    x = rng.uniform(-20, 20, (2, 11, 3)).astype(np.float32)
    c = rng.uniform(-3, 3, (2, 3)).astype(np.float32)
    out = oracle.transform(x, centers=c, quats=np.tile(q, (2, 1)),
                           translations=np.zeros((2, 3), np.float32))
    # (x - c) + c in double, rounded to float, gives x back
    assert np.array_equal(out, x)
    assert np.array_equal(oracle.transform(x), x)           # all-NULL arguments


def test_quarter_turn_about_z():
    # w = cos(45 deg), z = sin(45 deg); (1,0,0,1) normalises to exactly that rotation
    R = oracle.quat_to_matrix(np.array([1, 0, 0, 1], np.float32))
    assert np.array_equal(R, np.array([[0, -1, 0], [1, 0, 0], [0, 0, 1]], float))
    x = np.array([[[1, 0, 0], [0, 1, 0], [0, 0, 1]]], np.float32)
    out = oracle.transform(x, quats=np.array([[1, 0, 0, 1]], np.float32))
    assert np.array_equal(out[0], np.array([[0, 1, 0], [-1, 0, 0], [0, 0, 1]], np.float32))
    # quarter turns about x and y: right-handed, active
    Rx = oracle.quat_to_matrix(np.array([1, 1, 0, 0], np.float32))
    assert np.array_equal(Rx @ [0, 1, 0], [0, 0, 1])
    Ry = oracle.quat_to_matrix(np.array([1, 0, 1, 0], np.float32))
    assert np.array_equal(Ry @ [0, 0, 1], [1, 0, 0])


def test_matrix_matches_scipy_rotation_and_is_orthonormal():
    rng = np.random.default_rng(1)
    for _ in range(200):
        q = rng.standard_normal(4).astype(np.float32) * np.float32(rng.uniform(0.3, 3.0))
        R = oracle.quat_to_matrix(q)
        w, x, y, z = (float(v) for v in q)
        ref = Rotation.from_quat([x, y, z, w]).as_matrix()       # scipy: scalar last
        assert np.allclose(R, ref, atol=1e-14)
        assert np.allclose(R @ R.T, np.eye(3), atol=1e-14)
        assert np.linalg.det(R) == pytest.approx(1.0, abs=1e-14)


def test_zero_quaternion_means_no_rotation():
    assert np.array_equal(oracle.quat_to_matrix(np.zeros(4, np.float32)), np.eye(3))


def test_rotation_is_about_the_center_then_translated():
    rng = np.random.default_rng(2)
    B, N = 4, 9
    x = rng.uniform(-10, 10, (B, N, 3)).astype(np.float32)
    c = rng.uniform(-5, 5, (B, 3)).astype(np.float32)
    t = rng.uniform(-2, 2, (B, 3)).astype(np.float32)
    q = rng.standard_normal((B, 4)).astype(np.float32)
    out = oracle.transform(x, centers=c, quats=q, translations=t, as_float=False)
    for b in range(B):
        w, qx, qy, qz = (float(v) for v in q[b])
        rot = Rotation.from_quat([qx, qy, qz, w])
        ref = rot.apply(x[b].astype(float) - c[b].astype(float)) + c[b].astype(float) \
            + t[b].astype(float)
        assert np.allclose(out[b], ref, atol=1e-13)
        # the center itself is a fixed point of the rotation: it only translates
        cc = oracle.transform(c[b].reshape(1, 1, 3), centers=c[b:b + 1], quats=q[b:b + 1],
                              translations=t[b:b + 1], as_float=False)
        assert np.allclose(cc[0, 0], c[b].astype(float) + t[b].astype(float), atol=1e-14)
    # the float result is the double result rounded once
    out32 = oracle.transform(x, centers=c, quats=q, translations=t, as_float=True)
    assert np.array_equal(out32, out.astype(np.float32))
