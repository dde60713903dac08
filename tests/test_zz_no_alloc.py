"""The sampler entry point that allocates nothing (``rsd_sample_static``) against the context-based
``rsd_sample``: two calls in a row on the same workspace, the second with a smaller input."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_static_sampler_matches_context_sampler():
    import torch
    from rsd_inputs import workload
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import Session

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    s = Session(workload("cfg0"))
    rng = np.random.default_rng(31)
    cases = [(64, 151936), (5, 1024)]          # the second call is smaller in both dimensions
    for it, (T, top_p) in enumerate(((0.7, 0.95), (0.0, 1.0), (1.3, 0.3))):
        for n, V in cases:
            lg = torch.from_numpy((rng.normal(size=(n, V)) * 0.8).astype(np.float32)).cuda()
            u = torch.from_numpy(rng.random(n).astype(np.float32)).cuda()
            ref = R.rsd_sample(s.ctx, lg, u, T, top_p).cpu().numpy()
            out = torch.full((n,), -7, dtype=torch.int32, device="cuda")
            free0 = torch.cuda.mem_get_info()[0]
            R.rsd_sample_static(lg, u, T, top_p, out=out)
            torch.cuda.synchronize()
            if it > 0:      # (the very first call may still load code or grow a runtime pool)
                assert torch.cuda.mem_get_info()[0] == free0, "the call changed the amount of free device memory"
            got = out.cpu().numpy()
            assert np.array_equal(got, ref), (T, top_p, n, V, int((got != ref).sum()))
    # sizes beyond the static workspace are refused, as are missing uniforms
    big = torch.zeros((65, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(R.RsdError):
        R.rsd_sample_static(big, torch.zeros(65, device="cuda"), 0.7, 0.9)
    with pytest.raises(R.RsdError):
        R.rsd_sample_static(big[:4].contiguous(), None, 0.7, 0.9)
    s.close()
