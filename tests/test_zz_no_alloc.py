"""GPU: the tensor-scale entry point that allocates nothing (its scratch is a static device
array inside the library) against the entry points it is a variant of, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2512_02010_amd import binding as B
from paper_2512_02010_amd import workloads as wl

pytestmark = pytest.mark.gpu

RHT_SEED = wl.C5_RHT_SEED


def _bits(t):
    return int(t.cpu().view(torch.int32).item()) & 0xFFFFFFFF


def _three_ways(x, **kw):
    """alpha by the static-scratch call, the workspace call and the three-launch call."""
    rows, cols = x.shape
    xd = x.cuda()
    p = B.make_params(rows, cols, x_dtype=B.x_dtype_of(x), **kw)
    st = torch.cuda.current_stream()
    a_static = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    a_ws = torch.full((1,), -2.0, dtype=torch.float32, device="cuda")
    a_plain = torch.full((1,), -3.0, dtype=torch.float32, device="cuda")
    ws = B.new_workspace()
    assert B.tensor_scale_static_raw(xd, p, a_static, st) == 0
    assert B.tensor_scale_ws_raw(xd, p, a_ws, ws, ws.numel(), st) == 0
    assert B.tensor_scale_raw(xd, p, a_plain, st) == 0
    torch.cuda.synchronize()
    return _bits(a_static), _bits(a_ws), _bits(a_plain)


def test_static_scratch_tensor_scale_twice_in_a_row_second_call_smaller():
    big = wl.make("c2", 2048, 4096)
    small = wl.make("c1", 64, 256)
    for x in (big, small, big, small):            # each call finds what the last one left
        s, w, p = _three_ways(x)
        want = np.array([ref.tensor_scale(wl.bf16_bits(x))], np.float32).view(np.uint32)[0]
        assert s == w == p == int(want), (tuple(x.shape), hex(s), hex(w), hex(p), hex(int(want)))


@pytest.mark.parametrize("kw", [dict(rht=1, rht_seed=RHT_SEED, layout=B.ROWWISE),
                                dict(rht=1, rht_seed=RHT_SEED, layout=B.COLWISE),
                                dict(fp8_max=448.0)])
def test_static_scratch_tensor_scale_options(kw):
    for x in (wl.make("c5", 1024, 2048), wl.make("c3", 48, 176),
              wl.make("c2", 512, 1024, dtype=torch.float32), wl.make("c1", 16, 16, dtype=torch.float32)):
        s, w, p = _three_ways(x, **kw)
        assert s == w == p, (tuple(x.shape), kw, hex(s), hex(w), hex(p))


def test_static_scratch_tensor_scale_edge_cases_and_errors():
    z = torch.zeros((32, 64), dtype=torch.bfloat16)
    s, w, p = _three_ways(z)
    assert s == w == p == 0x3F800000              # an all-zero tensor: alpha = 1
    s, w, p = _three_ways(wl.make("c1", 1, 16))   # the smallest tensor
    assert s == w == p
    xd = wl.make("c1", 32, 64).cuda()
    a = torch.empty(1, dtype=torch.float32, device="cuda")
    assert B.tensor_scale_static_raw(None, B.make_params(32, 64), a) == 1
    assert B.tensor_scale_static_raw(xd, B.make_params(32, 64), None) == 1
    assert B.tensor_scale_static_raw(xd, B.make_params(32, 40), a) == 2
    assert B.tensor_scale_static_raw(xd, B.make_params(1 << 32, 16), a) == 2      # beyond the maximum size
    assert B.tensor_scale_static_raw(xd, B.make_params(32, 64, rht=1, layout=B.BOTH), a) == 5
    # a rejected call leaves the scratch usable
    s, w, p = _three_ways(wl.make("c4", 128, 256))
    assert s == w == p
