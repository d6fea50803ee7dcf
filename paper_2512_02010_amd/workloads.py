"""Seeded synthetic input tensors for the five benchmark workloads.

This module only *draws numbers*: it holds none of the quantization method's
arithmetic and is the one piece shared by the CPU oracle's tests and the HIP
path's tests / benchmark.  Every tensor is generated on the host in fp32 with a
``torch.Generator`` and then cast to BF16 with round-to-nearest-even; the BF16
bit patterns (``uint16``) are what both sides consume.

The five recipes stand in for the weight, activation and gradient tensors the
paper quantizes (Section 4; Figure 3), which need model checkpoints that are
not available here:

====  ==============  =========================================================
name  full shape      values
====  ==============  =========================================================
c1    256 x 1024      i.i.d. N(0,1)
c2    8192 x 8192     0.02 * Student-t(nu=3); 1 % of the columns (seeded
                      choice) multiplied by 50 -- "outlier channels" of a
                      weight matrix
c3    16384 x 4096    N(0,1) * per-row lognormal(0,1); 0.1 % of the elements
                      (seeded positions) replaced by +-U(100,1000) -- an
                      activation batch with massive activations
c4    8192 x 8192     i.i.d. N(0,1) (both block orientations are produced)
c5    32768 x 8192    N(0,(1e-3)^2) * per-row lognormal(0,2) -- a gradient
                      tensor with a very wide per-row dynamic range
====  ==============  =========================================================

Any (rows, cols) may be requested so that the parity tests can run the same
recipes at sizes the CPU oracle finishes quickly.
"""
from __future__ import annotations

import numpy as np
import torch

SEEDS = {"c1": 4601, "c2": 4602, "c3": 4603, "c4": 4604, "c5": 4605}

FULL_SHAPES = {
    "c1": (256, 1024),
    "c2": (8192, 8192),
    "c3": (16384, 4096),
    "c4": (8192, 8192),
    "c5": (32768, 8192),
}

# Fixed seeds for the random numbers the method itself draws in workload c5
# (stochastic rounding uniforms and Hadamard sign vectors).
C5_SR_SEED = 0x46F5EED00000C5
C5_RHT_SEED = 0x4AD0000000C5


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def _chunked_rows(rows: int, cols: int, budget_elems: int = 1 << 24):
    step = max(1, budget_elems // max(cols, 1))
    r = 0
    while r < rows:
        n = min(step, rows - r)
        yield r, n
        r += n


def _normal(shape, g):
    return torch.randn(shape, generator=g, dtype=torch.float32)


def make_c1(rows=256, cols=1024, seed=SEEDS["c1"], dtype=torch.bfloat16) -> torch.Tensor:
    g = _gen(seed)
    return _normal((rows, cols), g).to(dtype)


def make_c2(rows=8192, cols=8192, seed=SEEDS["c2"], dtype=torch.bfloat16) -> torch.Tensor:
    g = _gen(seed)
    n_out = max(1, round(0.01 * cols))
    perm = torch.randperm(cols, generator=g)
    col_gain = torch.ones(cols, dtype=torch.float32)
    col_gain[perm[:n_out]] = 50.0
    out = torch.empty((rows, cols), dtype=dtype)
    for r0, n in _chunked_rows(rows, cols, 1 << 22):
        z = _normal((n, cols), g)
        chi = _normal((n, cols), g).square_()
        chi += _normal((n, cols), g).square_()
        chi += _normal((n, cols), g).square_()
        t = z / torch.sqrt(chi / 3.0)
        out[r0:r0 + n] = (0.02 * t * col_gain).to(dtype)
    return out


def make_c3(rows=16384, cols=4096, seed=SEEDS["c3"], dtype=torch.bfloat16) -> torch.Tensor:
    g = _gen(seed)
    row_mag = torch.exp(_normal((rows, 1), g))
    out = torch.empty((rows, cols), dtype=dtype)
    for r0, n in _chunked_rows(rows, cols):
        x = _normal((n, cols), g) * row_mag[r0:r0 + n]
        hit = torch.rand((n, cols), generator=g) < 1.0e-3
        mag = 100.0 + 900.0 * torch.rand((n, cols), generator=g)
        sgn = torch.where(torch.rand((n, cols), generator=g) < 0.5, -1.0, 1.0)
        x = torch.where(hit, mag * sgn, x)
        out[r0:r0 + n] = x.to(dtype)
    return out


def make_c4(rows=8192, cols=8192, seed=SEEDS["c4"], dtype=torch.bfloat16) -> torch.Tensor:
    g = _gen(seed)
    out = torch.empty((rows, cols), dtype=dtype)
    for r0, n in _chunked_rows(rows, cols):
        out[r0:r0 + n] = _normal((n, cols), g).to(dtype)
    return out


def make_c5(rows=32768, cols=8192, seed=SEEDS["c5"], dtype=torch.bfloat16) -> torch.Tensor:
    g = _gen(seed)
    row_mag = torch.exp(2.0 * _normal((rows, 1), g))
    out = torch.empty((rows, cols), dtype=dtype)
    for r0, n in _chunked_rows(rows, cols):
        x = 1.0e-3 * _normal((n, cols), g) * row_mag[r0:r0 + n]
        out[r0:r0 + n] = x.to(dtype)
    return out


_MAKERS = {"c1": make_c1, "c2": make_c2, "c3": make_c3, "c4": make_c4, "c5": make_c5}


def make(name: str, rows: int | None = None, cols: int | None = None,
         seed: int | None = None, dtype: torch.dtype = torch.bfloat16) -> torch.Tensor:
    """CPU tensor for workload `name`, at its full shape unless overridden.  BF16 by default;
    ``dtype=torch.float32`` keeps the fp32 draws unrounded (FP32 master weights, Fig. 3)."""
    fr, fc = FULL_SHAPES[name]
    return _MAKERS[name](rows or fr, cols or fc, SEEDS[name] if seed is None else seed, dtype)


def bf16_bits(x: torch.Tensor) -> np.ndarray:
    """View a BF16 tensor as a C-contiguous uint16 numpy array (no copy)."""
    assert x.dtype == torch.bfloat16 and x.is_contiguous() and x.device.type == "cpu"
    return x.view(torch.int16).numpy().view(np.uint16)


def host_array(x: torch.Tensor) -> np.ndarray:
    """What the CPU side consumes: BF16 tensors as uint16 bit patterns, fp32 tensors as
    float32 arrays (no copy)."""
    if x.dtype == torch.float32:
        assert x.is_contiguous() and x.device.type == "cpu"
        return x.numpy()
    return bf16_bits(x)


def bits_to_bf16(bits: np.ndarray) -> torch.Tensor:
    """Inverse of :func:`bf16_bits`."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return torch.from_numpy(b.view(np.int16)).view(torch.bfloat16)


def adversarial(kind: str, rows: int = 32, cols: int = 64,
                dtype: torch.dtype = torch.bfloat16) -> torch.Tensor:
    """Small edge-case tensors (shapes are multiples of 16 both ways)."""
    g = _gen(977)
    if kind == "zeros":
        x = torch.zeros((rows, cols))
    elif kind == "neg_zeros":
        x = -torch.zeros((rows, cols))
    elif kind == "constant":
        x = torch.full((rows, cols), 0.3125)
    elif kind == "neg_constant":
        x = torch.full((rows, cols), -7.0)
    elif kind == "one_hot":
        x = torch.zeros((rows, cols))
        x[rows // 2, cols // 3] = 5.0
    elif kind == "one_hot_per_block":
        x = torch.zeros((rows, cols))
        x[:, ::16] = _normal((rows, cols // 16), g)
    elif kind == "tiny":
        # far below the tensor maximum: block scales fall into the E4M3
        # subnormal range or to zero
        x = _normal((rows, cols), g) * 1.0e-4
        x[0, 0] = 300.0
    elif kind == "wide_range":
        e = torch.randint(-20, 8, (rows, cols), generator=g).float()
        x = _normal((rows, cols), g) * torch.exp2(e)
    elif kind == "grid_exact":
        # already NVFP4-representable: grid values times a power-of-two scale
        grid = torch.tensor([0, .5, 1, 1.5, 2, 3, 4, 6, -0.5, -1, -1.5, -2, -3, -4, -6, 6.0])
        idx = torch.randint(0, 16, (rows, cols), generator=g)
        x = grid[idx]
        x[:, ::16] = 6.0
        x = x * 0.25
    elif kind == "ties":
        # many values on E2M1 rounding midpoints once scaled (max 6 per block)
        mids = torch.tensor([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, -0.25, -2.5, -5.0, 6.0, 4.0])
        idx = torch.randint(0, len(mids), (rows, cols), generator=g)
        x = mids[idx]
        x[:, ::16] = 6.0
    elif kind == "decision_stress":
        # blocks on which the two scalings give equal or nearly equal errors: a lone
        # outlier (everything else rounds to zero both ways), an outlier over faint noise,
        # two equal peaks, constants, plain noise -- at many magnitudes
        nb = cols // 16
        x = torch.zeros((rows, nb, 16))
        pat = torch.randint(0, 6, (rows, nb), generator=g)
        mag = torch.exp2(torch.randint(-12, 6, (rows, nb), generator=g).float())
        mag = mag * (1.0 + torch.rand((rows, nb), generator=g))
        noise = _normal((rows, nb, 16), g)
        pos = torch.randint(0, 16, (rows, nb), generator=g)
        peak = torch.zeros((rows, nb, 16)).scatter_(2, pos.unsqueeze(-1), 1.0)
        pos2 = (pos + 1 + torch.randint(0, 15, (rows, nb), generator=g)) % 16
        peak2 = torch.zeros((rows, nb, 16)).scatter_(2, pos2.unsqueeze(-1), 1.0)
        x = torch.where((pat == 0).unsqueeze(-1), peak, x)
        x = torch.where((pat == 1).unsqueeze(-1), peak + 1e-3 * noise, x)
        x = torch.where((pat == 2).unsqueeze(-1), peak + 0.03 * noise, x)
        x = torch.where((pat == 3).unsqueeze(-1), peak - peak2, x)
        x = torch.where((pat == 4).unsqueeze(-1), torch.ones(16) * 0.75, x)
        x = torch.where((pat == 5).unsqueeze(-1), 0.3 * noise, x)
        x = (x * mag.unsqueeze(-1)).reshape(rows, cols)
    elif kind == "sq_underflow_stress":
        # the near-tie patterns of "decision_stress" at those magnitudes
        return (adversarial("decision_stress", rows, cols, torch.float32) * 2.0 ** -62).to(dtype).contiguous()
    elif kind.startswith("sq_underflow_"):
        # magnitudes at which the squared errors of a block fall into the fp32 subnormal
        # range (max|x| around 2^-58 ... 2^-72) without all of them underflowing to zero
        e = int(kind.rsplit("_", 1)[1])
        x = _normal((rows, cols), g) * 2.0 ** -e
    elif kind == "bf16_small":
        x = _normal((rows, cols), g) * 1.0e-24
    elif kind == "bf16_large":
        x = _normal((rows, cols), g) * 1.0e30
    else:
        raise ValueError(kind)
    return x.to(dtype).contiguous()


ADVERSARIAL_KINDS = ("zeros", "neg_zeros", "constant", "neg_constant", "one_hot",
                     "one_hot_per_block", "tiny", "wide_range", "grid_exact", "ties",
                     "bf16_small", "bf16_large", "sq_underflow_60", "sq_underflow_66",
                     "sq_underflow_70", "sq_underflow_72", "sq_underflow_74",
                     "sq_underflow_stress")
