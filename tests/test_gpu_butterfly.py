"""The butterfly form of the write path (srft_kv_quantize_butterfly: fp32 FFT on the vector ALU, Sec. 3.2 / Sec. 7.1)
against the oracle, to the same bar as the matrix-core form, and against that form."""
import numpy as np
import pytest
import torch

from paper_2605_05699_amd import workloads as W
from tests import parity_util as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_05699_amd import binding
    binding.lib()
    return binding


def _butterfly(B, plan, x):
    n, d = x.shape
    codes = torch.empty(n, d // 2, dtype=torch.uint8, device="cuda")
    scales = torch.empty(n, d // 32, dtype=torch.float32, device="cuda")
    B.srft_kv_quantize_butterfly(plan.handle, x, codes, scales)
    torch.cuda.synchronize()
    return codes, scales


@pytest.mark.parametrize("d,n", [(128, 1), (128, 63), (128, 64), (128, 65), (128, 1003), (128, 70_001),
                                 (256, 1), (256, 31), (256, 32), (256, 33), (256, 1003), (256, 70_001)])
def test_butterfly_form_matches_the_oracle(B, d, n):
    # d = 128: a vector per lane, 64 per step; d = 256: a vector on two lanes, 32 per step
    g = 32
    lam = W.lognormal_lambda(d, seed=n + d)
    plan = B.Plan(d, g, 900 + n + d, lam)
    xh = W.gaussian_with_outliers(n, d, seed=n + d, outliers=d // 128, gain=20.0)
    x = torch.from_numpy(xh).cuda()
    codes, scales = _butterfly(B, plan, x)
    q = P.check_quantize(xh, plan.signs, lam, g, codes.cpu().numpy(), scales.cpu().numpy())
    assert q["ill_conditioned_groups"] == 0
    if n > 1000:
        assert q["mismatch_rate"] < 1e-3
    # the read path decodes its record like any other
    out = plan.dequantize(codes, scales)
    P.check_dequantize(codes.cpu().numpy(), scales.cpu().numpy(), plan.signs, lam, g, out.cpu().numpy())
    # against the matrix-core form: the same scales to fp32 rounding, the same codes except at rounding boundaries
    c2, s2 = plan.quantize(x)
    assert torch.allclose(scales, s2, rtol=4e-6, atol=0)
    differ = (codes != c2).float().mean().item()
    assert differ < 1e-3, differ
    plan.close()


def test_butterfly_form_on_the_llama_shaped_workload_and_its_argument_checks(B):
    w = W.WORKLOADS["llama3-70b-128k"]
    seed, lam, _ = W.plan_constants(w, 0)
    plan = B.Plan(w.d, w.g, seed, lam)
    n = 262_144
    x = W.make_kv(w, 0, n_vec=n, device="cuda")
    codes, scales = _butterfly(B, plan, x)
    idx = np.unique(np.concatenate([np.arange(64), np.arange(n - 64, n), np.random.RandomState(0).randint(0, n, 4096)]))
    it = torch.from_numpy(idx).cuda()
    q = P.check_quantize(x[it].cpu().numpy(), plan.signs, lam, w.g, codes[it].cpu().numpy(), scales[it].cpu().numpy())
    assert q["ill_conditioned_groups"] == 0 and q["mismatch_rate"] < 1e-3
    L = B.lib()
    assert L.srft_kv_quantize_butterfly(None, None, 1, None, None, None) == -1
    assert L.srft_kv_quantize_butterfly(plan.handle, None, -1, None, None, None) == -7
    assert L.srft_kv_quantize_butterfly(plan.handle, None, 0, None, None, None) == 0
    assert L.srft_kv_quantize_butterfly(plan.handle, None, 1, None, None, None) == -1
    other = B.Plan(96, 32, 1)
    assert L.srft_kv_quantize_butterfly(other.handle, x.data_ptr(), 1, codes.data_ptr(), scales.data_ptr(), None) == -2
    other.close()
    wide = B.Plan(128, 64, 1)
    assert L.srft_kv_quantize_butterfly(wide.handle, x.data_ptr(), 1, codes.data_ptr(), scales.data_ptr(), None) == -3
    wide.close()
    plan.close()
