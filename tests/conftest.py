import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

GOLDEN = Path(__file__).resolve().parent / "golden"


def pytest_configure(config):
    # Tests marked `gpu` call the HIP library on cuda:0 and fail (they do not
    # skip) where no GPU is visible; CPU-only runs deselect them with -m "not gpu".
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return GOLDEN


# ---- guard zones around every output of a GPU test -------------------------------------
# The library writes through raw pointers; an out-of-range store on a ragged shape would land
# in a neighbouring allocation and go unseen.  For tests marked `gpu`, every output tensor that
# the binding allocates is a view into the middle of a larger buffer filled with a sentinel
# byte, and after the test both margins of every such buffer must still hold the sentinel.
_GUARD_BYTES = 4096        # each side; a multiple of 256, so the view keeps its alignment
_SENTINEL = 0xA5


class _GuardedAllocator:
    def __init__(self):
        self.buffers = []

    def __call__(self, shape, dtype, device):
        import torch
        shape = tuple(int(d) for d in (shape if isinstance(shape, (tuple, list)) else (shape,)))
        n = 1
        for d in shape:
            n *= d
        nbytes = n * torch.empty((), dtype=dtype).element_size()
        raw = torch.full((nbytes + 2 * _GUARD_BYTES,), _SENTINEL, dtype=torch.uint8, device=device)
        self.buffers.append((raw, nbytes))
        return raw[_GUARD_BYTES:_GUARD_BYTES + nbytes].view(dtype).view(shape)

    def check(self):
        import torch
        torch.cuda.synchronize()
        for raw, nbytes in self.buffers:
            lo, hi = raw[:_GUARD_BYTES], raw[_GUARD_BYTES + nbytes:]
            assert bool((lo == _SENTINEL).all()) and bool((hi == _SENTINEL).all()), (
                f"a kernel wrote outside an output of {nbytes} bytes")
        self.buffers.clear()


@pytest.fixture(autouse=True)
def guarded_outputs(request):
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    from paper_2512_02010_amd import binding
    guard = _GuardedAllocator()
    saved = binding.OUTPUT_ALLOCATOR
    binding.OUTPUT_ALLOCATOR = guard
    try:
        yield
        guard.check()
    finally:
        binding.OUTPUT_ALLOCATOR = saved
