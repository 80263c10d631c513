"""The entry point that allocates nothing (tm_sq_sum_static: block partials in a buffer built into the
library) against the entry point it is a variant of (tm_sq_sum with caller scratch): same kernels, same
order, so the same bits; two calls in a row, the second on a smaller input, so that stale partials of
the first call would show; the size limit is an error code."""
import numpy as np
import pytest

from tests.gpu_util import require_gpu, stream_ptr

pytestmark = pytest.mark.gpu


def test_static_scratch_squared_sum_equals_the_scratch_form():
    torch = require_gpu()
    import paper_2412_12636_amd as tm
    s = stream_ptr(torch)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    big = torch.empty(50_000_003, dtype=torch.float32, device="cuda").normal_(0, 1e-2, generator=gen)
    for n in (50_000_000, 4096 * 3 + 5, 7, 0):            # second and later calls are smaller than the first
        print(f"tm_sq_sum_static n={n}", flush=True)
        g = big[:n] if n else big[:4]
        want = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
        got = torch.full((1,), -2.0, dtype=torch.float64, device="cuda")
        scratch = torch.empty(max(8, tm.tm_sq_sum_scratch_bytes(n)), dtype=torch.uint8, device="cuda")
        tm.tm_sq_sum(n, g, scratch, want, s)
        tm.tm_sq_sum_static(n, g, got, s)
        torch.cuda.synchronize()
        assert got.item() == want.item(), (n, got.item(), want.item())
        ref = float((g[:n].double() ** 2).sum().item()) if n else 0.0
        assert abs(got.item() - ref) <= 1e-5 * ref, (n, got.item(), ref)     # fp32 inside a thread's 16 elements
    # beyond the built-in buffer: a clear error, nothing launched
    limit = tm.tm_sq_sum_static_max_elems()
    assert limit == 4096 * (1 << 20)
    out = torch.zeros(1, dtype=torch.float64, device="cuda")
    with pytest.raises(tm.TmError) as e:
        tm.tm_sq_sum_static(limit + 1, big, out, s)
    assert e.value.code == tm.TM_ESIZE and "built-in scratch" in e.value.message
    torch.cuda.synchronize()
    assert out.item() == 0.0
