"""The allocation-free BatchNorm statistics entry point (partial results in an array inside the library) against the
entry point that takes a scratch buffer, through the C ABI: identical bits for the same scratch size, and the oracle's
statistics within the activation tolerance; two calls in a row, the second on a smaller input, so that whatever the
first call left in the shared array must not matter."""
import numpy as np
import pytest

from oracle import numerics as nm
from paper_2010_14501_amd import monet
from parity_util import ACT_TOL, check_close

pytestmark = pytest.mark.gpu

STATIC_BYTES = 4 << 20


def both_forms(torch, x, eps=1e-5):
    rows, C = x.shape
    dx = torch.from_numpy(x).cuda()
    scratch = torch.full((STATIC_BYTES // 4,), float("nan"), dtype=torch.float32, device="cuda")
    want = torch.full((2 * C,), float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full((2 * C,), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_bn_stats", None, dx.data_ptr(), want.data_ptr(), rows, C, eps, scratch.data_ptr(), STATIC_BYTES)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    monet.call("monet_bn_stats_static", None, dx.data_ptr(), got.data_ptr(), rows, C, eps)
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy(), free_before - torch.cuda.mem_get_info()[0]


@pytest.mark.parametrize("first,second", [((50000, 256), (3000, 64)),          # partial results per 64 rows
                                          ((300000, 512), (777, 12)),          # too many groups for 4 MiB: row slabs
                                          ((4100, 8192), (64, 8192))])         # the widest tensor the entry point takes
def test_static_scratch_statistics_match_the_scratch_form_twice_in_a_row(first, second):
    import torch
    rng = np.random.default_rng(5)
    grown = []
    for rows, C in (first, second):
        x = (rng.standard_normal((rows, C), dtype=np.float32) * np.float32(3.0) + np.float32(10.0))
        got, want, g = both_forms(torch, x)
        grown.append(g)
        assert np.array_equal(got, want), (rows, C)
        mean, invstd = nm.bn_stats(np.ascontiguousarray(x.T.astype(np.float64))[None, :, :, None], 1e-5)
        check_close(got[:C], mean, ACT_TOL, what=("mean", rows, C))
        check_close(got[C:], invstd, ACT_TOL, what=("invstd", rows, C))
    assert grown[1] <= 0, grown          # the second call took no device memory


def test_static_scratch_statistics_refuse_what_does_not_fit():
    import torch
    x = torch.zeros((8, 8200), dtype=torch.float32, device="cuda")
    out = torch.zeros((2 * 8200,), dtype=torch.float32, device="cuda")
    for rows, C in ((8, 8196), (8, 6), (0, 64)):
        with pytest.raises(monet.MonetError):
            monet.call("monet_bn_stats_static", None, x.data_ptr(), out.data_ptr(), rows, C, 1e-5)
    assert float(out.abs().sum().item()) == 0.0       # nothing was enqueued
