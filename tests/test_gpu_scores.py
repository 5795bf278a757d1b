"""GPU parity of the scores-in-the-rotated-domain entry point against the oracle's plain definition."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import srft_oracle as O
from paper_2605_05699_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_05699_amd import binding
    binding.lib()
    return binding


def _tolerance(q, keys_ref64):
    # fp32 accumulation of d terms in the transform of q and in the contraction: about 1e-6 of ||q|| ||k||; the
    # oracle is fp64.  4e-6 leaves room for the two-term fp16 split of q' (about 2^-21 relative per element).
    return 4e-6 * np.linalg.norm(q.astype(np.float64), axis=1)[:, None] * np.linalg.norm(keys_ref64, axis=1)[None, :] + 1e-30


@pytest.mark.parametrize("d", [64, 128, 192, 256])
@pytest.mark.parametrize("n_q,n_keys", [(1, 1), (8, 33), (32, 1000), (5, 4097)])
def test_scores_match_the_definition(B, d, n_q, n_keys):
    g = 32
    keys = W.gaussian_with_outliers(n_keys, d, seed=d + n_keys, outliers=1, gain=15.0)
    q = W.gaussian_with_outliers(n_q, d, seed=7 * d + n_q, outliers=1, gain=4.0)
    lam = W.lognormal_lambda(d, seed=d + 3)
    plan = B.Plan(d, g, 500 + d, lam)
    s = plan.signs
    codes, scales = plan.quantize(torch.from_numpy(keys).cuda())
    got = plan.scores(torch.from_numpy(q).cuda(), codes, scales).cpu().numpy().astype(np.float64)
    c, sc = codes.cpu().numpy(), scales.cpu().numpy()
    ref = O.attention_scores(q, c, sc, s, lam, g)
    back = O.dequantize_f64(c, sc, s, lam, g)
    assert got.shape == (n_q, n_keys)
    assert np.all(np.abs(got - ref) <= _tolerance(q, back)), float((np.abs(got - ref) / _tolerance(q, back)).max())
    # and they are what attention over the dequantized prefix would see, up to that prefix's fp16 rounding
    out = plan.dequantize(codes, scales).cpu().numpy().astype(np.float64)
    via_prefix = q.astype(np.float64) @ out.T
    assert np.all(np.abs(got - via_prefix) <= 2.0 ** -10 * np.abs(q.astype(np.float64)) @ np.abs(out).T + _tolerance(q, back))
    plan.close()


def test_scores_with_wide_groups_hadamard_and_a_grid_cap(B):
    d, n_keys, n_q = 128, 3001, 8
    keys = W.gaussian_with_outliers(n_keys, d, seed=1)
    q = W.gaussian_with_outliers(n_q, d, seed=2)
    for g, transform, form in ((64, "dft", "dense"), (128, "dft", "dense"), (32, "hadamard", "hadamard")):
        lam = W.lognormal_lambda(d, seed=g)
        plan = B.Plan(d, g, 9, lam, transform=transform)
        codes, scales = plan.quantize(torch.from_numpy(keys).cuda())
        qd = torch.from_numpy(q).cuda()
        a = plan.scores(qd, codes, scales)
        B.srft_plan_set_max_workgroups(plan.handle, 3)
        assert torch.equal(a, plan.scores(qd, codes, scales))          # independent of the launch shape
        c, sc = codes.cpu().numpy(), scales.cpu().numpy()
        ref = O.attention_scores(q, c, sc, plan.signs, lam, g, form=form)
        back = O.dequantize_f64(c, sc, plan.signs, lam, g, form=form)
        assert np.all(np.abs(a.cpu().numpy() - ref) <= _tolerance(q, back))
        plan.close()


@pytest.mark.parametrize("d", [64, 128])
def test_every_query_count_and_nothing_written_outside(B, d):
    # n_q = 1..32 walks every kernel instance (16 and 32 rows of queries, every store count) and every partly
    # filled last store; the output sits between two guard zones that must come back untouched.
    g, n_keys, guard = 32, 77, 4096
    keys = W.gaussian_with_outliers(n_keys, d, seed=21, outliers=1, gain=10.0)
    lam = W.lognormal_lambda(d, seed=22)
    plan = B.Plan(d, g, 23, lam)
    codes, scales = plan.quantize(torch.from_numpy(keys).cuda())
    c, sc = codes.cpu().numpy(), scales.cpu().numpy()
    back = O.dequantize_f64(c, sc, plan.signs, lam, g)
    ws = torch.empty(B.lib().srft_scores_workspace_bytes(plan.handle), dtype=torch.uint8, device="cuda")
    for n_q in range(1, 33):
        q = W.gaussian_with_outliers(n_q, d, seed=100 + n_q)
        buf = torch.full((guard + n_q * n_keys + guard,), -12345.0, dtype=torch.float32, device="cuda")
        out = buf[guard:guard + n_q * n_keys].view(n_q, n_keys)
        B.srft_kv_scores(plan.handle, torch.from_numpy(q).cuda(), codes, scales, out, ws)
        torch.cuda.synchronize()
        host = buf.cpu().numpy()
        assert np.all(host[:guard] == -12345.0) and np.all(host[-guard:] == -12345.0), n_q
        got = host[guard:-guard].reshape(n_q, n_keys).astype(np.float64)
        ref = O.attention_scores(q, c, sc, plan.signs, lam, g)
        assert np.all(np.abs(got - ref) <= _tolerance(q, back)), n_q
    plan.close()


def test_scores_argument_errors(B):
    L = B.lib()
    plan = B.Plan(128, 32, 1)
    q = torch.zeros(4, 128, dtype=torch.float16, device="cuda")
    c = torch.zeros(64, 64, dtype=torch.uint8, device="cuda")
    s = torch.zeros(64, 4, dtype=torch.float32, device="cuda")
    o = torch.zeros(4, 64, dtype=torch.float32, device="cuda")
    ws = torch.zeros(L.srft_scores_workspace_bytes(plan.handle), dtype=torch.uint8, device="cuda")
    args = (q.data_ptr(), 4, c.data_ptr(), s.data_ptr(), 64, o.data_ptr(), ws.data_ptr(), None)
    assert L.srft_kv_scores(plan.handle, *args) == 0
    assert L.srft_kv_scores(None, *args) == -1
    assert L.srft_kv_scores(plan.handle, q.data_ptr(), 0, *args[2:]) == -7
    assert L.srft_kv_scores(plan.handle, q.data_ptr(), 33, *args[2:]) == -7
    assert L.srft_kv_scores(plan.handle, q.data_ptr(), 4, c.data_ptr(), s.data_ptr(), 64, o.data_ptr(), None, None) == -1
    assert L.srft_kv_scores(plan.handle, q.data_ptr(), 4, c.data_ptr(), s.data_ptr(), 0, None, None, None) == 0
    for bad in (B.Plan(96, 32, 1), B.Plan(128, 16, 1), B.Plan(128, 32, 1, bits=8)):
        assert L.srft_kv_scores(bad.handle, *args) in (-2, -3, -9)
        bad.close()
    torch.cuda.synchronize()
    plan.close()
