"""The sampler entry point that allocates nothing (its tables live in the library's own
fixed device array) against the workspace form, through the C ABI: bit-exact indices and
info on two calls in a row, the second on a smaller problem, so that whatever the first
call left in the shared array would show."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2509_13232_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def spo():
    from paper_2509_13232_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _pair(spo, alpha, beta, B, seed, iteration, replace):
    want, winfo = spo.spo_sample_prompts(alpha, beta, B, 0.05, seed, iteration, replace, return_info=True)
    got, ginfo = spo.spo_sample_prompts_static(alpha, beta, B, 0.05, seed, iteration, replace)
    torch.cuda.synchronize()
    return want.cpu().numpy(), winfo.cpu().numpy(), got.cpu().numpy(), ginfo.cpu().numpy()


def test_static_scratch_sampler_matches_workspace_form(spo, oracle):
    c5 = wl.CONFIGS["C5"]
    a5, b5 = wl.tracker_state(c5)
    big = (torch.as_tensor(a5).cuda(), torch.as_tensor(b5).cuda())
    rng = np.random.default_rng(5)
    small = (torch.as_tensor(rng.uniform(0.5, 50, 5000).astype(np.float32)).cuda(),
             torch.as_tensor(rng.uniform(0.5, 50, 5000).astype(np.float32)).cuda())
    assert a5.shape[0] == spo.SPO_SAMPLE_STATIC_MAX_N
    print("[case] static sampler: 4096 of 2^20 without replacement, then 300 of 5000", flush=True)
    # call 1: the largest problem the array holds; call 2: a smaller one right after it
    for (al, be), B, replace in ((big, c5.B, False), (small, 300, False), (big, 1000, True), (small, 4999, False)):
        want, winfo, got, ginfo = _pair(spo, al, be, B, c5.sample_seed, 3, replace)
        assert np.array_equal(got, want) and np.array_equal(ginfo, winfo)
        assert (got >= 0).all() and (got < al.numel()).all()
        if not replace:
            assert len(np.unique(got)) == B
    # the small problem once more against the oracle (the workspace form is checked against it elsewhere)
    got, _ = spo.spo_sample_prompts_static(small[0], small[1], 300, 0.05, c5.sample_seed, 3, False)
    ref = oracle.sample_prompts(small[0].cpu().numpy(), small[1].cpu().numpy(), 300, 0.05, c5.sample_seed, 3)
    assert np.array_equal(got.cpu().numpy(), ref)


def test_static_scratch_sampler_rejects_what_does_not_fit(spo):
    n = spo.SPO_SAMPLE_STATIC_MAX_N + 1
    a = torch.ones(n, device="cuda")
    idx = torch.full((8,), -7, dtype=torch.int32, device="cuda")
    rc = spo.lib().spo_sample_prompts_static(C.c_void_p(a.data_ptr()), C.c_void_p(a.data_ptr()), n, 8, 0.05, 0, 0, 0, 0,
                                             C.c_void_p(idx.data_ptr()), None, None)
    assert rc == -3 and "size" in spo.status_string(rc)
    torch.cuda.synchronize()
    assert (idx == -7).all()          # outputs untouched on error
