"""The entry point that allocates nothing (ds_colsum_static) against the entry point it is a variant of (ds_colsum),
through the C ABI: two calls in a row on the same GPU, the second with a smaller input, so that the second call runs
over whatever the first left in the shared device array.  Collected last on purpose (file name)."""
import numpy as np
import pytest
import torch

from paper_2311_10418_amd import binding as ds
from helpers import DEV, both_err, to_np

pytestmark = pytest.mark.gpu


def _pair(rows, n, dt, seed, accumulate):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.randn((rows, n), generator=g, device=DEV, dtype=torch.float32).to(dt)
    base = torch.randn((n,), generator=g, device=DEV, dtype=torch.float32)
    ref, got = base.clone(), base.clone()
    partial = torch.empty(int(ds.ds_norm_bwd_scratch_floats(rows, n)), dtype=torch.float32, device=DEV)
    ds.ds_colsum(x, ref, partial, accumulate=accumulate)
    ds.ds_colsum_static(x, got, accumulate=accumulate)
    torch.cuda.synchronize()
    return x, base, ref, got


@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float32])
def test_two_calls_in_a_row_second_one_smaller(dt):
    for rows, n, acc in ((70001, 2048, False), (333, 264, True), (5000, 8192, False), (7, 8, True)):
        x, base, ref, got = _pair(rows, n, dt, rows + n, acc)
        # same kernels, same partial-row count: the two entry points agree to the last bit ...
        assert torch.equal(ref, got), (rows, n)
        # ... and with the plain definition
        plain = to_np(x).sum(axis=0) + (to_np(base) if acc else 0.0)
        assert both_err(to_np(got), plain) <= 1e-5, (rows, n)


def test_sizes_beyond_the_fixed_capacity_are_rejected():
    x = torch.zeros((2, 65536 + 8), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((65536 + 8,), dtype=torch.float32, device=DEV)
    with pytest.raises(ds.DsError) as e:
        ds.ds_colsum_static(x, out)
    assert e.value.code == ds.DS_ELIMIT
    ds.ds_colsum_static(x[:, :65536].contiguous(), out[:65536])           # the largest width it takes
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0


def test_no_allocation_happens_inside_the_call():
    x = torch.randn((4096, 1024), device=DEV, dtype=torch.float32).to(torch.bfloat16)
    out = torch.zeros((1024,), dtype=torch.float32, device=DEV)
    ds.ds_colsum_static(x, out)                                           # first use on this device: address lookup
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(20):
        ds.ds_colsum_static(x, out)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
