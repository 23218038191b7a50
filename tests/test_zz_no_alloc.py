"""The entry point that allocates nothing (sampler_step_noalloc) against sampler_step, through the C ABI.

Two calls in a row on one GPU, the second on a smaller input: both share the library's file-scope
scratch array, so the second call must not be disturbed by what the first left there.  The two entry
points run the same kernels, so the comparison is bit for bit (the integer bar of the parity tests).
"""
import numpy as np
import pytest
import torch

from paper_2505_14741_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_sampler_step_noalloc_equals_sampler_step_on_two_calls_in_a_row():
    a, b = 0.9931, 0.0517
    g = torch.Generator(device=DEV); g.manual_seed(5)
    sizes = [3 * (1 << 20) + 7, 4099]                # 769 workgroups of partial sums, then 2
    bufs = []
    for n in sizes:
        x, e, p = (torch.randn(n, generator=g, device=DEV) for _ in range(3))
        bufs.append((x, e, p, torch.empty_like(x), torch.full((4,), -1.0, device=DEV)))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for (x, e, p, out, sums), n in zip(bufs, sizes):  # back to back on one stream, nothing allocated in between
        print(f"sampler_step_noalloc n={n}", flush=True)
        B.sampler_step_noalloc(x, e, p, a, b, out, sums)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for (x, e, p, out, sums), n in zip(bufs, sizes):
        ref_x, ref_s = B.sampler_step(x, e, p, a, b)
        torch.cuda.synchronize()
        assert torch.equal(out, ref_x), n
        assert torch.equal(sums, ref_s), n
        assert bool((sums >= 0).all())
    # without eps_prev and in place; without sums (the scratch array is then not touched)
    x, e, p, out, sums = bufs[1]
    ref_x, ref_s = B.sampler_step(x, e, None, a, b)
    xc = x.clone()
    B.sampler_step_noalloc(xc, e, None, a, b, xc, sums)
    torch.cuda.synchronize()
    assert torch.equal(xc, ref_x) and torch.equal(sums, ref_s)
    xc = x.clone()
    B.sampler_step_noalloc(xc, e, None, a, b, xc, None)
    torch.cuda.synchronize()
    assert torch.equal(xc, ref_x)


def test_sampler_step_noalloc_rejects_what_it_cannot_do():
    x = torch.zeros(8, device=DEV)
    L = B.lib()
    too_many = (1 << 31) + 4
    assert L.sampler_step_noalloc(x.data_ptr(), x.data_ptr(), None, x.data_ptr(), 1.0, 0.0, too_many, None, None) == -2
    assert L.sampler_step_noalloc(None, x.data_ptr(), None, x.data_ptr(), 1.0, 0.0, 8, None, None) == -1
    e = torch.ones(8, device=DEV)
    assert L.sampler_step_noalloc(x.data_ptr(), e.data_ptr(), None, e.data_ptr(), 1.0, 0.0, 8, None, None) == -2
