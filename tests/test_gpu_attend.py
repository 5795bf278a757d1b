"""GPU parity of the value side of attention over the stored cache (srft_kv_attend, srft_kv_decode_attention) against
the oracle's plain definitions."""
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


def _attend(B, plan, w, codes, scales):
    out = torch.full((w.shape[0], plan.d), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(B.lib().srft_attend_workspace_bytes(plan.handle), dtype=torch.uint8, device="cuda")
    B.srft_kv_attend(plan.handle, w, codes, scales, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def _tolerance(w64, vals64):
    # the products w * scale are carried as fp16 hi + lo (2^-21 relative each), the sums are fp32 over at most a few
    # hundred tiles per workgroup and a few hundred workgroups, the inverse transform is fp32 over d terms: a few
    # 1e-6 of sum_t |w_t| max|v| covers all of it; the oracle is fp64
    return 6e-6 * np.abs(w64).sum(axis=1)[:, None] * np.abs(vals64).max() + 1e-30


@pytest.mark.parametrize("d", [64, 128, 192, 256])
@pytest.mark.parametrize("n_q,n_keys", [(1, 1), (8, 33), (32, 1000), (5, 4097), (3, 64), (12, 300), (16, 129), (17, 100)])
def test_attend_matches_the_definition(B, d, n_q, n_keys):
    g = 32
    vals = W.gaussian_with_outliers(n_keys, d, seed=3 * d + n_keys, outliers=1, gain=10.0)
    lam = W.lognormal_lambda(d, seed=d + 5)
    plan = B.Plan(d, g, 700 + d, lam)
    codes, scales = plan.quantize(torch.from_numpy(vals).cuda())
    rng = np.random.RandomState(n_q + n_keys)
    w = rng.rand(n_q, n_keys).astype(np.float32)
    w[0] = 0.0
    w[0, n_keys // 2] = 1.0                       # a one-hot row: that value's reconstruction
    if n_q > 1:
        w[1] = rng.standard_normal(n_keys).astype(np.float32)      # weights need not be probabilities
    got = _attend(B, plan, torch.from_numpy(w).cuda(), codes, scales)
    c, sc = codes.cpu().numpy(), scales.cpu().numpy()
    ref = O.attention_output(w, c, sc, plan.signs, lam, g)
    back = O.dequantize_f64(c, sc, plan.signs, lam, g)
    assert got.shape == (n_q, d) and np.isfinite(got).all()
    tol = _tolerance(w.astype(np.float64), back)
    assert np.all(np.abs(got - ref) <= tol), float((np.abs(got - ref) / tol).max())
    assert np.all(np.abs(got[0] - back[n_keys // 2]) <= tol[0])
    plan.close()


def test_attend_over_many_tiles_wide_groups_a_grid_cap_and_argument_checks(B):
    d, n_keys, n_q = 128, 200_003, 8
    vals = W.gaussian_with_outliers(n_keys, d, seed=4, outliers=1, gain=20.0)
    rng = np.random.RandomState(1)
    logits = rng.standard_normal((n_q, n_keys)) * 3.0
    w = O.softmax_rows(logits).astype(np.float32)
    wd = torch.from_numpy(w).cuda()
    for g in (32, 64, 128):
        lam = W.lognormal_lambda(d, seed=g)
        plan = B.Plan(d, g, 11, lam)
        codes, scales = plan.quantize(torch.from_numpy(vals).cuda())
        got = _attend(B, plan, wd, codes, scales)
        c, sc = codes.cpu().numpy(), scales.cpu().numpy()
        ref = O.attention_output(w, c, sc, plan.signs, lam, g)
        tol = _tolerance(w.astype(np.float64), O.dequantize_f64(c[:4096], sc[:4096], plan.signs, lam, g) * 1.5)
        assert np.all(np.abs(got - ref) <= tol), (g, float((np.abs(got - ref) / tol).max()))
        if g == 32:
            # fewer workgroups: another split of the keys, the same sums to rounding
            B.srft_plan_set_max_workgroups(plan.handle, 3)
            again = _attend(B, plan, wd, codes, scales)
            assert np.all(np.abs(again - ref) <= tol)
            B.srft_plan_set_max_workgroups(plan.handle, 0)
            twice = _attend(B, plan, wd, codes, scales)
            assert np.array_equal(twice, got)                     # fixed summation order: bitwise repeatable
            L = B.lib()
            ws = torch.empty(L.srft_attend_workspace_bytes(plan.handle), dtype=torch.uint8, device="cuda")
            out = torch.empty(n_q, d, dtype=torch.float32, device="cuda")
            args = (wd.data_ptr(), n_q, codes.data_ptr(), scales.data_ptr(), n_keys, out.data_ptr(), ws.data_ptr(), None)
            assert L.srft_kv_attend(None, *args) == -1
            assert L.srft_kv_attend(plan.handle, wd.data_ptr(), 33, *args[2:]) == -7
            assert L.srft_kv_attend(plan.handle, wd.data_ptr(), n_q, codes.data_ptr(), scales.data_ptr(), 0, out.data_ptr(), ws.data_ptr(), None) == -7
            assert L.srft_kv_attend(plan.handle, None, *args[1:]) == -1
            assert L.srft_kv_attend(plan.handle, wd.data_ptr(), n_q, codes.data_ptr() + 1, *args[3:]) == -5
        plan.close()
    p96 = B.Plan(96, 32, 1)
    assert B.lib().srft_attend_workspace_bytes(p96.handle) > 0
    assert B.lib().srft_kv_attend(p96.handle, wd.data_ptr(), 1, wd.data_ptr(), wd.data_ptr(), 1, wd.data_ptr(), wd.data_ptr(), None) == -2
    p96.close()


@pytest.mark.parametrize("d,n_q,n_keys", [(128, 8, 5000), (256, 4, 1234), (64, 32, 777), (128, 16, 70001), (192, 9, 40)])
def test_decode_attention_matches_the_definition(B, d, n_q, n_keys):
    g = 32
    k = W.gaussian_with_outliers(n_keys, d, seed=d + 1, outliers=1, gain=15.0)
    v = W.gaussian_with_outliers(n_keys, d, seed=d + 2, outliers=0)
    q = W.gaussian_with_outliers(n_q, d, seed=d + 3, outliers=1, gain=4.0)
    lam_k, lam_v = W.lognormal_lambda(d, seed=1), W.lognormal_lambda(d, seed=2)
    pk, pv = B.Plan(d, g, 21, lam_k), B.Plan(d, g, 22, lam_v)
    kc, ks = pk.quantize(torch.from_numpy(k).cuda())
    vc, vs = pv.quantize(torch.from_numpy(v).cuda())
    scale = d ** -0.5
    out = torch.full((n_q, d), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(B.lib().srft_decode_attention_workspace_bytes(pk.handle, pv.handle, n_q, n_keys), dtype=torch.uint8,
                     device="cuda")
    B.srft_kv_decode_attention(pk.handle, pv.handle, torch.from_numpy(q).cuda(), kc, ks, vc, vs, scale, out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref = O.decode_attention(q, kc.cpu().numpy(), ks.cpu().numpy(), pk.signs, lam_k, vc.cpu().numpy(), vs.cpu().numpy(),
                             pv.signs, lam_v, g, scale)
    vb = O.dequantize_f64(vc.cpu().numpy(), vs.cpu().numpy(), pv.signs, lam_v, g)
    # the scores carry an absolute error of about 4e-6 |q| |k| (test_gpu_scores.py); times softmax_scale it moves every
    # probability by that relative amount, and the output by at most twice that times max |v|; plus the weighted sum's own
    kb = O.dequantize_f64(kc.cpu().numpy(), ks.cpu().numpy(), pk.signs, lam_k, g)
    ds = 4e-6 * scale * np.linalg.norm(q.astype(np.float64), axis=1).max() * np.linalg.norm(kb, axis=1).max() + 2e-7
    tol = (2 * ds + 6e-6) * np.abs(vb).max() + 1e-30
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= tol, float(np.abs(got - ref).max() / tol)
    pk.close()
    pv.close()


def test_decode_attention_replayed_from_a_hip_graph_equals_the_eager_calls(B):
    """The entry point only enqueues kernels on the caller's stream (no allocation, no memset), so a caller may record
    it into a HIP graph.  Three replays, each after new queries were written into the captured buffer by ordinary eager
    work, must equal the eager call on the same inputs bit for bit (the summation order is fixed)."""
    d, g, n_q, n_keys = 128, 32, 8, 20_000
    k = W.gaussian_with_outliers(n_keys, d, seed=31, outliers=1, gain=15.0)
    v = W.gaussian_with_outliers(n_keys, d, seed=32, outliers=0)
    pk, pv = B.Plan(d, g, 41, W.lognormal_lambda(d, seed=3)), B.Plan(d, g, 42, W.lognormal_lambda(d, seed=4))
    kc, ks = pk.quantize(torch.from_numpy(k).cuda())
    vc, vs = pv.quantize(torch.from_numpy(v).cuda())
    scale = d ** -0.5
    q = torch.zeros(n_q, d, dtype=torch.float16, device="cuda")
    out = torch.zeros(n_q, d, dtype=torch.float32, device="cuda")
    nbytes = B.lib().srft_decode_attention_workspace_bytes(pk.handle, pv.handle, n_q, n_keys)
    ws, ws_eager = (torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2))
    q.copy_(torch.from_numpy(W.gaussian_with_outliers(n_q, d, seed=50, outliers=0)))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):              # one eager call on the capture stream first
        B.srft_kv_decode_attention(pk.handle, pv.handle, q, kc, ks, vc, vs, scale, out, ws, side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        B.srft_kv_decode_attention(pk.handle, pv.handle, q, kc, ks, vc, vs, scale, out, ws, torch.cuda.current_stream())
    for rep in range(3):
        q.copy_(torch.from_numpy(W.gaussian_with_outliers(n_q, d, seed=60 + rep, outliers=1, gain=3.0)))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        eager = torch.empty_like(out)
        B.srft_kv_decode_attention(pk.handle, pv.handle, q, kc, ks, vc, vs, scale, eager, ws_eager)
        torch.cuda.synchronize()
        assert torch.equal(got, eager), rep
        assert torch.isfinite(got).all() and got.abs().max() > 0
    pk.close()
    pv.close()
