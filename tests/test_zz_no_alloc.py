"""The entry point that allocates nothing (partial sums in a static device array of the library):
same result as nnt_tile_bias_grad with caller scratch, and the oracle's column sums, on two calls in
a row, the second with a smaller input; sizes beyond the static array are refused."""
import numpy as np
import pytest
import torch

from gpu_util import TOL, code, from_dev, quant, relerr, stream_ptr, to_dev
from oracle import definition as D

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def capi():
    from paper_2504_13236_amd import capi
    return capi


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_bias_grad_static_matches_bias_grad_on_two_calls(capi, dtype):
    r = np.random.default_rng(77)
    st = stream_ptr()
    for m, n in ((768, 8192), (200, 300)):            # the second call is smaller: stale partial sums of the first lie behind it
        dY = quant(r.standard_normal((m, n)), dtype)
        d_dy = to_dev(dY, dtype)
        want = torch.full((m,), 7.0, dtype=torch.float32, device="cuda")
        got = torch.full((m,), 7.0, dtype=torch.float32, device="cuda")
        scratch = torch.empty(capi.nnt_tile_bias_grad_scratch(m, n), dtype=torch.float32, device="cuda")
        for accumulate in (0, 1):
            capi.nnt_tile_bias_grad(st, code(dtype), m, n, d_dy.data_ptr(), want.data_ptr(), accumulate, scratch.data_ptr())
            capi.nnt_tile_bias_grad_static(st, code(dtype), m, n, d_dy.data_ptr(), got.data_ptr(), accumulate)
            torch.cuda.synchronize()
            assert torch.equal(got, want), (m, n, accumulate)                     # same kernels, same order of sums
            assert relerr(from_dev(got, (m,)), (1 + accumulate) * D.bias_grad(dY)) <= TOL["f32"]


def test_bias_grad_static_refuses_what_does_not_fit(capi):
    cap = capi.nnt_tile_bias_grad_static_max()
    assert cap == 1 << 20
    m, n = 4096, 128 * 257                                                       # 257 partial rows of 4096 > 2^20
    assert capi.nnt_tile_bias_grad_scratch(m, n) > cap
    x = torch.zeros(8, device="cuda")
    rc = capi.nnt_tile_bias_grad_static.raw(stream_ptr(), 0, m, n, x.data_ptr(), x.data_ptr(), 0)
    assert rc == capi.NNT_EINVAL
    torch.cuda.synchronize()
    m, n = 4096, 128 * 256                                                       # exactly the limit
    assert capi.nnt_tile_bias_grad_scratch(m, n) == cap
    dY = torch.ones(m * n, device="cuda")
    db = torch.empty(m, device="cuda")
    capi.nnt_tile_bias_grad_static(stream_ptr(), 0, m, n, dY.data_ptr(), db.data_ptr(), 0)
    torch.cuda.synchronize()
    assert torch.all(db == float(n))
