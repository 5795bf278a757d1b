"""GPU parity of the lambda calibration statistic: per-channel abs-max of the transform over a batch."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import srft_oracle as O
from paper_2605_05699_amd import workloads as W

pytestmark = pytest.mark.gpu

# The kernel's w carries the fp32 accumulation error of a d-term sum, about 1e-6 of lambda_k ||x||; a channel
# maximum is one such w, so it is held to 2e-6 of lambda_k max||x|| (the bar used for scales in the parity tests).
AMAX_ERR = 2e-6


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_05699_amd import binding
    binding.lib()
    return binding


def _check(amax_gpu, x, s, lam, running=None):
    ref = O.channel_absmax(x, s, lam, running=running)
    lam64 = np.ones(x.shape[1]) if lam is None else np.asarray(lam, dtype=np.float64)
    tol = AMAX_ERR * lam64 * np.linalg.norm(x.astype(np.float64), axis=1).max(initial=0.0) + 1e-30
    assert np.all(np.abs(amax_gpu.astype(np.float64) - ref) <= tol + 2.0 ** -23 * ref), \
        f"max excess {np.max(np.abs(amax_gpu - ref) - tol)}"
    return ref


@pytest.mark.parametrize("d", [32, 64, 96, 128, 160, 192, 224, 256])
@pytest.mark.parametrize("n", [1, 33, 2531])
def test_channel_absmax_matches_oracle(B, d, n):
    x = W.gaussian_with_outliers(n, d, seed=7 * d + n, outliers=max(1, d // 64), gain=20.0)
    plan = B.Plan(d, 32, 1000 + d)                       # lambda = 1: the plain SRFT output
    amax = plan.channel_absmax(torch.from_numpy(x).cuda()).cpu().numpy()
    _check(amax, x, plan.signs, None)
    plan.close()


def test_running_maximum_over_batches_and_with_lambda(B):
    d = 128
    lam = W.lognormal_lambda(d, seed=3)
    plan = B.Plan(d, 32, 5, lam)
    s = plan.signs
    amax = torch.zeros(d, dtype=torch.float32, device="cuda")
    running = None
    for i, n in enumerate((700, 1, 4096, 31)):
        x = W.gaussian_with_outliers(n, d, seed=50 + i, outliers=1, gain=5.0 * (i + 1))
        plan.channel_absmax(torch.from_numpy(x).cuda(), amax)
        running = _check(amax.cpu().numpy(), x, s, lam, running=running)
    # a batch of smaller vectors changes nothing; an empty batch neither
    before = amax.clone()
    small = (W.gaussian_with_outliers(500, d, seed=99) * np.float16(1e-3)).astype(np.float16)
    plan.channel_absmax(torch.from_numpy(small).cuda(), amax)
    plan.channel_absmax(torch.empty(0, d, dtype=torch.float16, device="cuda"), amax)
    assert torch.equal(before, amax)
    plan.close()


def test_result_does_not_depend_on_the_grid(B):
    d, n = 96, 50000
    x = torch.from_numpy(W.gaussian_with_outliers(n, d, seed=8)).cuda()
    plan = B.Plan(d, 32, 21)
    a = plan.channel_absmax(x)
    for cap in (1, 7, 300):
        B.srft_plan_set_max_workgroups(plan.handle, cap)
        assert torch.equal(a, plan.channel_absmax(x))        # a maximum has no rounding: bitwise equal
    plan.close()


def test_closed_form_and_calibrated_plan_round_trip(B):
    """Constant vectors move only the DC channel; lambda from the statistic makes every channel of the
    calibration batch peak at 1, and the plan built from it quantizes to the oracle's codes."""
    from tests import parity_util as P
    d, n = 128, 3000
    plan1 = B.Plan(d, 32, 77)
    s = plan1.signs
    c = np.array([0.5, -3.0, 2.0], dtype=np.float64)
    amax = plan1.channel_absmax(torch.from_numpy(np.outer(c, s).astype(np.float16)).cuda()).cpu().numpy()
    assert abs(amax[0] - 3.0 * np.sqrt(d)) < 1e-4 and np.all(amax[1:] < 1e-4)

    w = W.WORKLOADS["qwen2.5-1.5b-4k"]
    x = W.make_kv(w, 0, n_vec=n, device="cuda")
    amax = plan1.channel_absmax(x).cpu().numpy()
    lam = B.srft_lambda_from_absmax(amax)
    assert np.allclose(lam, O.lambda_from_absmax(amax), rtol=1e-6)
    plan2 = B.Plan(d, 32, 77, lam)
    peak = plan2.channel_absmax(x).cpu().numpy()
    assert np.allclose(peak, 1.0, atol=2e-5)
    codes, scales = plan2.quantize(x)
    P.check_quantize(x.cpu().numpy(), s, lam, 32, codes.cpu().numpy(), scales.cpu().numpy())
    plan1.close()
    plan2.close()


def test_argument_errors(B):
    L = B.lib()
    plan = B.Plan(64, 32, 1)
    x = torch.zeros(8, 64, dtype=torch.float16, device="cuda")
    a = torch.zeros(64, dtype=torch.float32, device="cuda")
    assert L.srft_kv_channel_absmax(None, x.data_ptr(), 8, a.data_ptr(), None) == -1
    assert L.srft_kv_channel_absmax(plan.handle, None, 8, a.data_ptr(), None) == -1
    assert L.srft_kv_channel_absmax(plan.handle, x.data_ptr(), 8, None, None) == -1
    assert L.srft_kv_channel_absmax(plan.handle, x.data_ptr(), -1, a.data_ptr(), None) == -7
    assert L.srft_kv_channel_absmax(plan.handle, x.data_ptr() + 2, 4, a.data_ptr(), None) == -5
    assert L.srft_kv_channel_absmax(plan.handle, x.data_ptr(), 0, None, None) == 0
    with pytest.raises(ValueError):
        B.srft_kv_channel_absmax(plan.handle, x, torch.zeros(32, dtype=torch.float32, device="cuda"))
    plan.close()
