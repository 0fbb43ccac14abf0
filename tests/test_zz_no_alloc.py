"""The fixed-order sum without a scratch argument (gnntrain_sum_static: for callers that cannot allocate)
against gnntrain_sum, which takes the scratch buffer from the caller.  Same kernels, same order of additions:
the results must agree bit for bit.  Two calls in a row share the library's array, the second on a smaller
input, so stale block sums of the first call would show."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_sum_without_scratch_argument_matches_the_one_with():
    import paper_2308_10087_amd as g
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(2308100899)
    scratch = torch.zeros(1024, device=dev)
    for n in (5_000_003, 70_001, 4096, 1, 0):       # 1024 blocks first, then fewer and fewer
        x = torch.randn(max(n, 1), generator=gen, device=dev)[:n]
        want = torch.full((1,), float("nan"), device=dev)
        got = torch.full((1,), float("nan"), device=dev)
        g.gnntrain_sum(x, 0.25, scratch, want)
        g.gnntrain_sum_static(x, 0.25, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (n, got.item(), want.item())
        # and both are the sum: against fp64 on the host, at fp32 summation accuracy
        ref = 0.25 * float(x.double().sum().item())
        assert abs(got.item() - ref) <= 1e-5 * max(1.0, float(x.double().abs().sum().item()) * 0.25)


def test_sum_without_scratch_argument_rejects_what_it_cannot_do():
    import paper_2308_10087_amd as g
    dev = "cuda:0"
    x = torch.ones(16, device=dev)
    out = torch.zeros(1, device=dev)
    with pytest.raises(g.GnnStageError) as e:
        g.gnntrain_sum_static(x, 1.0, out, n=2**31)      # beyond the stated maximum: refused before any launch
    assert e.value.code == -6 and "GNNTRAIN_SUM_STATIC_MAX_N" in str(e.value)
    with pytest.raises(g.GnnStageError) as e:
        g.gnntrain_sum_static(x, 1.0, out, n=-1)
    assert e.value.code == -1
    g.gnntrain_sum_static(x, 2.0, out)                   # the entry point still works afterwards
    torch.cuda.synchronize()
    assert out.item() == 32.0
