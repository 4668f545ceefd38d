"""``torch.autograd`` glue over the C-ABI binding (GridMaker section: the grid is generated
in place on a Torch tensor, and ``backward`` turns a gradient on the grid into atomic gradients,
so coordinates -- and, with vector types, type weights -- can be optimised through the grid).

No arithmetic of the method happens here: ``forward`` calls ``mg_forward_*`` and ``backward``
calls ``mg_backward_*``; this module only tells autograd which call belongs to which.  When a
gradient will be asked for, forward builds the tables once (``mg_prepare``) in a workspace of its
own and both passes run on them (the ``*_prepared`` calls): the backward pass then starts without
a prep kernel.
A binary GridMaker has no gradient (the indicator is piecewise constant); asking for one raises.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import molgrid


class _IndexGrid(torch.autograd.Function):
    @staticmethod
    def forward(ctx, coords, gm, types, radii, T, natoms, centers, quats, translations):
        ctx.gm, ctx.T, ctx.ws = gm, T, None
        ctx.save_for_backward(coords, types, radii, natoms, centers, quats, translations)
        if ctx.needs_input_grad[0] and not gm.binary:
            B, N, _ = coords.shape
            ctx.ws = gm.mg_prepare(coords.detach(), types, radii, T, natoms=natoms, centers=centers,
                                   quats=quats, translations=translations)
            return gm.mg_forward_index_prepared(B, N, T, ctx.ws)
        return gm.mg_forward_index(coords.detach(), types, radii, T, natoms=natoms, centers=centers,
                                   quats=quats, translations=translations)

    @staticmethod
    def backward(ctx, grad_out):
        if ctx.gm.binary:
            raise RuntimeError("a binary GridMaker has no gradient")
        coords, types, radii, natoms, centers, quats, translations = ctx.saved_tensors
        if ctx.ws is not None and grad_out.dtype == torch.float32:
            B, N, _ = coords.shape
            g = ctx.gm.mg_backward_index_prepared(B, N, ctx.T, grad_out.contiguous(), ctx.ws)
            return (g,) + (None,) * 8
        g = ctx.gm.mg_backward_index(coords.detach(), types, radii, ctx.T, grad_out.contiguous(),
                                     natoms=natoms, centers=centers, quats=quats,
                                     translations=translations)
        return (g,) + (None,) * 8


class _VectorGrid(torch.autograd.Function):
    @staticmethod
    def forward(ctx, coords, weights, gm, radii, natoms, centers, quats, translations):
        ctx.gm, ctx.ws = gm, None
        ctx.save_for_backward(coords, weights, radii, natoms, centers, quats, translations)
        if (ctx.needs_input_grad[0] or ctx.needs_input_grad[1]) and not gm.binary:
            ctx.ws = gm.mg_prepare(coords.detach(), None, radii, weights.shape[2], natoms=natoms,
                                   centers=centers, quats=quats, translations=translations)
            return gm.mg_forward_vector_prepared(weights.detach(), radii, ctx.ws)
        return gm.mg_forward_vector(coords.detach(), weights.detach(), radii, natoms=natoms,
                                    centers=centers, quats=quats, translations=translations)

    @staticmethod
    def backward(ctx, grad_out):
        if ctx.gm.binary:
            raise RuntimeError("a binary GridMaker has no gradient")
        coords, weights, radii, natoms, centers, quats, translations = ctx.saved_tensors
        want_c, want_w = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        if ctx.ws is not None and grad_out.dtype == torch.float32:
            gc, gw = ctx.gm.mg_backward_vector_prepared(
                weights.detach(), radii, grad_out.contiguous(), ctx.ws, want_coords=True,
                want_weights=bool(want_w))
            return (gc if want_c else None, gw if want_w else None) + (None,) * 6
        gc, gw = ctx.gm.mg_backward_vector(
            coords.detach(), weights.detach(), radii, grad_out.contiguous(), natoms=natoms,
            centers=centers, quats=quats, translations=translations,
            want_coords=True, want_weights=bool(want_w))
        return (gc if want_c else None, gw if want_w else None) + (None,) * 6


class GridLayer(torch.nn.Module):
    """A GridMaker as a differentiable layer: ``layer(coords, types=... | weights=..., ...)``
    returns the ``[B,T,D,D,D]`` grid (``[B,S,S,S,T,D,D,D]`` with ``subgrids_per_side`` = S > 1);
    gradients flow to ``coords`` (and ``weights``).

    ``random_rotation`` / ``random_translation`` (GridMaker.forward's optional augmentation): a
    fresh per-example rotation and a translation of at most that many Angstrom per axis are
    drawn on the device for every call (``mg_draw_transforms``, counter-based: ``seed`` and the
    number of the call fix them) and kept in ``last_quats`` / ``last_translations``, so the
    applied transformation can be retained; gradients come back in the caller's frame."""

    def __init__(self, resolution=0.5, dimension=23.5, binary=False, radius_type_indexed=True,
                 radius_scale=1.0, gaussian_radius_multiple=1.0, subgrids_per_side=1):
        super().__init__()
        self.gm = molgrid.GridMaker(resolution, dimension, binary=binary,
                                    radius_type_indexed=radius_type_indexed,
                                    radius_scale=radius_scale,
                                    gaussian_radius_multiple=gaussian_radius_multiple,
                                    subgrids_per_side=subgrids_per_side)
        self.seed, self.draws = 0, 0
        self.last_quats = self.last_translations = None

    def forward(self, coords, radii, *, types: Optional[torch.Tensor] = None,
                weights: Optional[torch.Tensor] = None, T: Optional[int] = None, natoms=None,
                centers=None, quats=None, translations=None, random_rotation=False,
                random_translation=0.0):
        if (types is None) == (weights is None):
            raise ValueError("give exactly one of types (index) or weights (vector)")
        if random_rotation or random_translation > 0.0:
            if quats is not None or translations is not None:
                raise ValueError("give explicit transforms or ask for random ones, not both")
            quats, translations = molgrid.mg_draw_transforms(
                self.seed, self.draws, coords.shape[0], random_rotation=bool(random_rotation),
                max_translation=float(random_translation), device=coords.device)
            self.draws += 1
            self.last_quats, self.last_translations = quats, translations
        if types is not None:
            if T is None:
                raise ValueError("index types need the number of channels T")
            return _IndexGrid.apply(coords, self.gm, types, radii, T, natoms, centers, quats,
                                    translations)
        return _VectorGrid.apply(coords, weights, self.gm, radii, natoms, centers, quats,
                                 translations)
