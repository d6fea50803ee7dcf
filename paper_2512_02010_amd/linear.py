"""The NVFP4 linear layer of Fig. 3 as a sequence of library calls.

Nothing is computed here: every function strings together ``nvfp4_46_tensor_scale``,
``nvfp4_46_quantize`` and ``nvfp4_46_gemm`` the way the figure wires them.

    FPROP   y  = x W^T          x [T][K] BF16 rowwise, RTN          W [N][K] FP32 rowwise
    DGRAD   dx = dy W           dy [T][N] BF16 rowwise, SR          W columnwise (= W^T rowwise)
    WGRAD   dW = dy^T x         dy columnwise, Hadamard + SR        x columnwise, Hadamard

Every operand is quantized along the contraction axis of the product it enters.  The weight
matrix is quantized once per step, by default in 16x16 tiles (Section 4.1), which yields the
packing for W and for W^T with identical codes and scales.  Stochastic rounding is used on
the gradient operands, the random Hadamard transform on both operands of WGRAD (same sign
vector along the contraction axis, so it cancels in the product).

Every function takes an optional ``workspace`` (``binding.new_workspace()``): with it the five
tensor scales of a step are one launch each (``nvfp4_46_tensor_scale_ws``) instead of three.
One workspace serves all calls issued on one stream.
"""
from __future__ import annotations

import torch

from . import binding as B


def _tensor_scale(t, stream, workspace, **kw):
    if workspace is None:
        return B.nvfp4_46_tensor_scale(t, stream=stream, **kw)
    return B.nvfp4_46_tensor_scale_ws(t, workspace, stream=stream, **kw)


def quantize_weight(w: torch.Tensor, select: int = B.SEL_46_MSE, block2d: bool = True,
                    stream=None, workspace: torch.Tensor | None = None) -> dict:
    """W [N][K] (FP32 master copy or BF16) -> both packings and the tensor scale."""
    alpha = _tensor_scale(w, stream, workspace)
    q = B.nvfp4_46_quantize(w, alpha, layout=B.BOTH, select=select, want_choice=False,
                            block2d=int(block2d), stream=stream)
    q.update(alpha=alpha, block2d=bool(block2d), shape=tuple(w.shape))
    return q


def _rowwise(t, stream, workspace, **kw):
    alpha = _tensor_scale(t, stream, workspace)
    q = B.nvfp4_46_quantize(t, alpha, want_choice=False, stream=stream, **kw)
    return q["codes_row"], q["scales_row"], alpha


def _columnwise(t, stream, workspace, rht_seed, **kw):
    alpha = _tensor_scale(t, stream, workspace, layout=B.COLWISE, rht=1, rht_seed=rht_seed)
    q = B.nvfp4_46_quantize(t, alpha, layout=B.COLWISE, rht=1, rht_seed=rht_seed,
                            want_choice=False, stream=stream, **kw)
    return q["codes_col"], q["scales_col"], alpha


def fprop(x: torch.Tensor, qw: dict, select: int = B.SEL_46_MSE, stream=None,
          workspace: torch.Tensor | None = None) -> torch.Tensor:
    """y [T][N] BF16 = x W^T."""
    cx, sx, ax = _rowwise(x, stream, workspace, select=select)
    flags = B.GEMM_B_TILE_SCALES if qw["block2d"] else 0
    return B.nvfp4_46_gemm(cx, sx, ax, qw["codes_row"], qw["scales_row"], qw["alpha"],
                           out_dtype=B.OUT_BF16, flags=flags, stream=stream)


def dgrad(dy: torch.Tensor, qw: dict, sr_seed: int, select: int = B.SEL_46_MSE,
          stream=None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """dx [T][K] BF16 = dy W, the gradient rounded stochastically."""
    cg, sg, ag = _rowwise(dy, stream, workspace, select=select, rounding=B.SR, sr_seed=sr_seed)
    flags = B.GEMM_B_TILE_SCALES if qw["block2d"] else 0
    return B.nvfp4_46_gemm(cg, sg, ag, qw["codes_col"], qw["scales_col"], qw["alpha"],
                           out_dtype=B.OUT_BF16, flags=flags, stream=stream)


def wgrad(dy: torch.Tensor, x: torch.Tensor, sr_seed: int, rht_seed: int,
          select: int = B.SEL_46_MSE, stream=None,
          workspace: torch.Tensor | None = None) -> torch.Tensor:
    """dW [N][K] FP32 = dy^T x, both operands Hadamard-transformed along the token axis."""
    cg, sg, ag = _columnwise(dy, stream, workspace, rht_seed, select=select, rounding=B.SR,
                             sr_seed=sr_seed)
    cx, sx, ax = _columnwise(x, stream, workspace, rht_seed, select=select)
    return B.nvfp4_46_gemm(cg, sg, ag, cx, sx, ax, out_dtype=B.OUT_F32, stream=stream)
