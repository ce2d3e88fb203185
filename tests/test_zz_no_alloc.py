"""The allocation-free sampling entry point against hss_kernel_sample (GPU only): two calls in a row, the second
on a smaller input, through the C ABI; results must be bit-identical (same kernels on the same padded inputs) and
within the sampling tolerance of the oracle.  Sizes beyond the fixed scratch array are rejected."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_noalloc_sampling_matches_the_allocating_entry_point():
    import torch
    from oracle import hss as ohss
    from paper_2108_04167_amd import binding
    ctx = binding.Context()
    rng = np.random.default_rng(21)
    dev = lambda a: torch.tensor(np.ascontiguousarray(a), device="cuda:0")
    for (n, r, s, h) in [(4096, 54, 128, 3.0), (777, 8, 100, 1.5), (4096, 96, 1, 4.0), (300, 3, 128, 0.7)]:
        F = rng.standard_normal((n, r))
        Om = rng.standard_normal((n, s))
        Fd, Od = dev(F), dev(Om)
        out = torch.full((n, s), float("nan"), dtype=torch.float64, device="cuda:0")
        # the binding allocates nothing through torch either: the count of allocation events stands still (the
        # bytes in use are no measure: the garbage collector may free earlier tests' tensors at any moment)
        events = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]
        before = events()
        assert ctx.hss_kernel_sample_noalloc(Fd, h, Od, out) == 0
        torch.cuda.synchronize()
        assert events() == before
        ref = ctx.hss_kernel_sample(Fd, h, Od)
        assert torch.equal(out, ref), (n, r, s)
        orc = ohss.sample(F, Om, h)
        assert np.abs(out.cpu().numpy() - orc).max() <= 1e-12 * np.abs(orc).max()
    # beyond the fixed array: rejected, nothing written
    for (n, r, s) in [(4097, 8, 16), (256, 8, 129)]:
        Fd, Od = dev(rng.standard_normal((n, r))), dev(rng.standard_normal((n, s)))
        out = torch.full((n, s), 7.0, dtype=torch.float64, device="cuda:0")
        with pytest.raises(binding.HssError) as e:
            ctx.hss_kernel_sample_noalloc(Fd, 1.0, Od, out)
        assert e.value.code == binding.HSS_EUNSUPPORTED
        assert bool((out == 7.0).all())
    ctx.close()
