"""Seeded synthetic inputs shaped like the paper's protein-ligand workloads.

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: it only draws random arrays (numpy, host
memory).  The protein-ligand structures the paper trains on are not available
here; these inputs stand in for them (receptor atoms filling a box around a
pocket, a small ligand near the center, one type channel per atom, a random
rotation and a small random translation per example as in the data
augmentation the GridMaker and Transformations sections describe).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

SEED_BASE = 19120482200


@dataclass
class Workload:
    name: str
    B: int
    N: int
    T: int
    resolution: float
    dimension: float
    D: int
    coords: np.ndarray                      # [B,N,3] float32
    types: np.ndarray                       # [B,N]   int32
    radii: np.ndarray                       # [T]     float32, per type
    centers: np.ndarray                     # [B,3]   float32
    quats: Optional[np.ndarray] = None      # [B,4]   float32 (w,x,y,z), not normalised exactly
    translations: Optional[np.ndarray] = None   # [B,3] float32
    weights: Optional[np.ndarray] = None    # [B,N,T] float32 (vector types)
    grad_out: Optional[np.ndarray] = None   # [B,T,D,D,D] float32 (upstream gradient)
    extra: dict = field(default_factory=dict)

    @property
    def out_shape(self):
        return (self.B, self.T, self.D, self.D, self.D)

    @property
    def out_bytes(self):
        return 4 * self.B * self.T * self.D ** 3


def _random_quats(rng, B):
    q = rng.standard_normal((B, 4))
    q /= np.linalg.norm(q, axis=1, keepdims=True)
    return q.astype(np.float32)


def tiny(seed: int = SEED_BASE + 0) -> Workload:
    """B=1, 100 atoms uniform in a 10 A cube, 4 types, 24^3 points at 0.5 A, no transform."""
    rng = np.random.default_rng(seed)
    B, N, T = 1, 100, 4
    coords = rng.uniform(-5.0, 5.0, (B, N, 3)).astype(np.float32)
    types = rng.integers(0, T, (B, N)).astype(np.int32)
    radii = np.array([1.6, 1.9, 1.8, 1.5], np.float32)
    return Workload("tiny", B, N, T, 0.5, 11.5, 24, coords, types, radii,
                    np.zeros((B, 3), np.float32))


def protein_ligand(B: int = 50, seed: int = SEED_BASE + 1, *, n_receptor: int = 2000,
                   n_ligand: int = 40, cube: float = 30.0, ligand_sigma: float = 3.0,
                   resolution: float = 0.5, dimension: float = 23.5, D: int = 48,
                   with_grad: bool = False, with_weights: bool = False) -> Workload:
    """Per example: receptor atoms uniform in a cube (14 receptor types), ligand atoms
    Gaussian about the center (14 ligand types), radii[28] ~ U(1.2, 2.0), a random unit
    quaternion and a +-2 A translation."""
    rng = np.random.default_rng(seed)
    N, T = n_receptor + n_ligand, 28
    rec = rng.uniform(-cube / 2, cube / 2, (B, n_receptor, 3))
    lig = rng.normal(0.0, ligand_sigma, (B, n_ligand, 3))
    coords = np.concatenate([rec, lig], axis=1).astype(np.float32)
    types = np.concatenate([rng.integers(0, 14, (B, n_receptor)),
                            rng.integers(14, 28, (B, n_ligand))], axis=1).astype(np.int32)
    radii = rng.uniform(1.2, 2.0, T).astype(np.float32)
    quats = _random_quats(rng, B)
    translations = rng.uniform(-2.0, 2.0, (B, 3)).astype(np.float32)
    w = Workload("protein_ligand", B, N, T, resolution, dimension, D, coords, types, radii,
                 np.zeros((B, 3), np.float32), quats, translations)
    if with_weights:
        wrng = np.random.default_rng(seed + 1000003)
        w.weights = wrng.dirichlet(np.full(T, 0.3), size=(B, N)).astype(np.float32)
    if with_grad:
        grng = np.random.default_rng(seed + 2000003)
        w.grad_out = grng.standard_normal(w.out_shape, dtype=np.float32)
    return w


def large_chunk(chunk: int, B: int = 16, seed: int = SEED_BASE + 4, *, N: int = 8000,
                cube: float = 40.0) -> Workload:
    """One chunk of the high-resolution case: 8000 atoms uniform in a 40 A cube, 28 types,
    96^3 points at 0.25 A, random rotation and +-2 A translation."""
    rng = np.random.default_rng([seed, chunk])
    T = 28
    coords = rng.uniform(-cube / 2, cube / 2, (B, N, 3)).astype(np.float32)
    types = rng.integers(0, T, (B, N)).astype(np.int32)
    radii = np.random.default_rng(seed).uniform(1.2, 2.0, T).astype(np.float32)
    quats = _random_quats(rng, B)
    translations = rng.uniform(-2.0, 2.0, (B, 3)).astype(np.float32)
    return Workload("large_chunk%d" % chunk, B, N, T, 0.25, 23.75, 96, coords, types, radii,
                    np.zeros((B, 3), np.float32), quats, translations)


def ragged_small(seed: int = 7, B: int = 3, N: int = 37, T: int = 5, D: int = 13,
                 resolution: float = 0.75) -> Workload:
    """A small awkward case: D not a multiple of 4, off-origin centers, atoms outside,
    straddling and inside the box, padded atoms (type -1) and a ragged natoms."""
    rng = np.random.default_rng(seed)
    dimension = (D - 1) * resolution
    centers = rng.uniform(-3.0, 3.0, (B, 3)).astype(np.float32)
    span = dimension / 2 + 4.0
    coords = (centers[:, None, :] + rng.uniform(-span, span, (B, N, 3))).astype(np.float32)
    types = rng.integers(-1, T + 1, (B, N)).astype(np.int32)   # includes -1 and T: skipped
    radii = rng.uniform(0.8, 2.2, T).astype(np.float32)
    quats = (_random_quats(rng, B) * rng.uniform(0.5, 2.0, (B, 1))).astype(np.float32)
    translations = rng.uniform(-1.0, 1.0, (B, 3)).astype(np.float32)
    w = Workload("ragged_small", B, N, T, resolution, dimension, D, coords, types, radii,
                 centers, quats, translations)
    w.extra["natoms"] = np.array([N, N // 2, 0][:B] + [N] * max(0, B - 3), np.int32)
    w.weights = rng.dirichlet(np.full(T, 0.3), size=(B, N)).astype(np.float32)
    w.grad_out = rng.standard_normal(w.out_shape).astype(np.float32)
    return w
