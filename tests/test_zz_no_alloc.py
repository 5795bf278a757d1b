"""srft_kv_scores_static (the entry point that allocates nothing) against srft_kv_scores, through the C ABI."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2605_05699_amd import workloads as W

pytestmark = pytest.mark.gpu


def _ptr(t):
    return C.c_void_p(t.data_ptr())


@pytest.mark.parametrize("d", [128, 256])
def test_static_workspace_scores_equal_the_workspace_entry_point_on_two_calls_in_a_row(d):
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2605_05699_amd import binding as B
    L = B.lib()
    g = 32
    plan = B.Plan(d, g, 77 + d, W.lognormal_lambda(d, seed=d))
    stream = C.c_void_p(int(torch.cuda.current_stream().cuda_stream))
    ws = torch.empty(L.srft_scores_workspace_bytes(plan.handle), dtype=torch.uint8, device="cuda")
    # the second call is smaller in both the keys and the queries: nothing of the first call may leak into it
    for n_q, n_keys in ((32, 40_001), (5, 1_203)):
        keys = torch.from_numpy(W.gaussian_with_outliers(n_keys, d, seed=n_keys, outliers=1, gain=15.0)).cuda()
        q = torch.from_numpy(W.gaussian_with_outliers(n_q, d, seed=n_q, outliers=1, gain=4.0)).cuda()
        codes, scales = plan.quantize(keys)
        want = torch.full((n_q, n_keys), float("nan"), dtype=torch.float32, device="cuda")
        got = torch.full((n_q, n_keys), float("nan"), dtype=torch.float32, device="cuda")
        rc = L.srft_kv_scores(plan.handle, _ptr(q), n_q, _ptr(codes), _ptr(scales), n_keys, _ptr(want), _ptr(ws), stream)
        assert rc == 0, rc
        rc = L.srft_kv_scores_static(plan.handle, _ptr(q), n_q, _ptr(codes), _ptr(scales), n_keys, _ptr(got), stream)
        assert rc == 0, rc
        torch.cuda.synchronize()
        w, gt = want.cpu().numpy(), got.cpu().numpy()
        assert np.isfinite(w).all() and np.isfinite(gt).all()
        # the same kernels on the same inputs: the scores are bit-identical (the bar for the workspace entry point
        # itself, against the oracle, is in test_gpu_scores.py)
        assert np.array_equal(w.view(np.uint32), gt.view(np.uint32)), float(np.abs(w - gt).max())
    # argument checks as for srft_kv_scores, before any HIP call
    assert L.srft_kv_scores_static(None, None, 1, None, None, 1, None, None) == -1
    assert L.srft_kv_scores_static(plan.handle, None, 0, None, None, 1, None, None) == -7
    assert L.srft_kv_scores_static(plan.handle, None, 1, None, None, 0, None, None) == 0
    assert L.srft_kv_scores_static(plan.handle, None, 1, None, None, 1, None, None) == -1
    plan.close()
