"""The measurement aids behind bench.py's yardsticks do what their declarations say (ds_bench_copy, ds_bench_stream):
the figures they give are only worth quoting if the kernels move the bytes they are credited with."""
import pytest
import torch

from paper_1907_07346_amd import binding as b

pytestmark = pytest.mark.gpu


def test_bench_copy_and_streams_results():
    n = 256 * 1024 + 4                                   # 16-byte multiples, not a multiple of the workgroup
    g = torch.randn(n, device="cuda")
    x = torch.randn(n, device="cuda")
    d = torch.randn(n, device="cuda")
    x0, d0 = x.clone(), d.clone()
    out = torch.zeros_like(g)
    b.ds_bench_copy(out, g)
    assert torch.equal(out, g)
    b.ds_bench_stream(x, d, g)                           # three loads, two stores: x += g, d += g
    assert torch.equal(x, x0 + g) and torch.equal(d, d0 + g)
    b.ds_bench_stream(x, None, g)                        # two loads, one store: x += g, the second array untouched
    assert torch.equal(x, (x0 + g) + g) and torch.equal(d, d0 + g)


def test_bench_stream_refusals():
    g = torch.zeros(1024, device="cuda")
    x = torch.zeros(1024, device="cuda")
    st = b.lib().ds_bench_stream(x.data_ptr() + 4, None, g.data_ptr(), 1024, None)     # misaligned
    assert st == b.DS_EINVAL
    st = b.lib().ds_bench_stream(x.data_ptr(), None, g.data_ptr(), 1000, None)         # not a multiple of 16
    assert st == b.DS_EINVAL
    st = b.lib().ds_bench_stream(None, None, g.data_ptr(), 1024, None)
    assert st == b.DS_EINVAL
