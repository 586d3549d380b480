"""cmpq_act_stats_static - the variant of cmpq_act_stats for callers that cannot allocate (its
row-split partial sums go to a fixed device array inside the library) - against cmpq_act_stats
itself, through the C ABI: two calls in a row, the second on a smaller input, then chunked
accumulation and the status flag.  The same kernels run in the same launch shape, so the bar is
the strictest one: every fp64 accumulator and every fp32 statistic identical."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

DEV = "cuda"


def test_act_stats_static_matches_act_stats_on_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2410_13056_amd import binding as B
    B.lib()
    ws = B.Workspace(DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    st_a = torch.zeros(1, dtype=torch.int32, device=DEV)
    st_b = torch.zeros(1, dtype=torch.int32, device=DEV)
    # a large input first (many row splits: most of the fixed array is written), then smaller
    # ones: the second call must not see anything the first one left behind
    for n, d_in, dtype in ((6000, 8192, torch.float16), (300, 1000, torch.float16), (77, 264, torch.float32),
                           (33, 100, torch.float16)):
        X = (torch.randn((n, d_in), generator=g, device=DEV) * 3).to(dtype)
        if d_in == 100:
            X = torch.cat([X, X], 1)[:, 3:103]                 # unaligned start: the other streaming kernel
        acc_a = torch.empty(d_in, dtype=torch.float64, device=DEV)
        acc_b = torch.full((d_in,), -1.0, dtype=torch.float64, device=DEV)
        s_a = torch.empty(d_in, dtype=torch.float32, device=DEV)
        s_b = torch.full((d_in,), -1.0, dtype=torch.float32, device=DEV)
        B.act_stats(X, acc_a, s_a, False, ws, st_a)
        B.act_stats_static(X, acc_b, s_b, False, st_b)
        torch.cuda.synchronize()
        assert torch.equal(acc_a, acc_b) and torch.equal(s_a, s_b), (n, d_in)
        ref = (X.double() ** 2).sum(0)
        assert torch.allclose(acc_b, ref, rtol=1e-12, atol=0)
        # more tokens into the same accumulators
        B.act_stats(X[: n // 2], acc_a, s_a, True, ws, st_a)
        B.act_stats_static(X[: n // 2], acc_b, s_b, True, st_b)
        torch.cuda.synchronize()
        assert torch.equal(acc_a, acc_b) and torch.equal(s_a, s_b), (n, d_in)
    assert st_a.item() == 0 and st_b.item() == 0
    bad = torch.randn((50, 64), generator=g, device=DEV).half()
    bad[7, 9] = float("nan")
    acc = torch.empty(64, dtype=torch.float64, device=DEV)
    B.act_stats_static(bad, acc, None, False, st_b)
    torch.cuda.synchronize()
    assert st_b.item() & B.STATUS_NONFINITE
    # beyond the fixed array: refused on the host, nothing enqueued
    with pytest.raises(B.CmpqError) as e:
        B.act_stats_static(torch.empty((1, 262152), dtype=torch.float16, device=DEV),
                           torch.empty(262152, dtype=torch.float64, device=DEV), None, False)
    assert e.value.code == -2
